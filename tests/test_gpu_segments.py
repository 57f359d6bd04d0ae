"""Segment-descriptor engine on the GPU against the oracle: pack, unpack, scatter to scatter, slice
fill counters, invalid descriptors."""
import numpy as np
import pytest
import torch

from definitions import random_topk
from test_oracle_segments import _random_layout

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def fusco():
    import paper_2512_22036_amd as f
    f.load_library()
    assert torch.cuda.is_available()
    return f


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def desc_dev(off, size):
    return dev(np.stack([np.asarray(off, dtype=np.int64), np.asarray(size, dtype=np.int64)], axis=1))


def scan(fusco, desc):
    n = desc.shape[0]
    cum = torch.full((n + 1,), -1, dtype=torch.int64, device="cuda")
    status = torch.full((1,), -1, dtype=torch.int32, device="cuda")
    fusco.fusco_segments_scan(desc, cum, status)
    return cum, status


@pytest.mark.parametrize("n,max_units", [(0, 4), (1, 4), (7, 40), (300, 40), (5000, 9), (2000, 1200), (70000, 3)])
def test_pack_and_unpack_match_oracle(fusco, oracle, n, max_units):
    rng = np.random.default_rng(n + max_units)
    size, off, span = _random_layout(rng, n, max_units=max_units)
    src = rng.integers(0, 256, size=max(span, 16), dtype=np.uint8)
    total = int(size.sum())
    cap = total + 4096
    want, fill_want = oracle.segments_copy(src, size, src_off=off, slice_bytes=16384) if n else (np.zeros(0, np.uint8), np.zeros(0, np.uint32))
    d_desc = desc_dev(off, size) if n else torch.zeros((0, 2), dtype=torch.int64, device="cuda")
    cum, status = scan(fusco, d_desc)
    assert np.array_equal(cum.cpu().numpy(), np.concatenate([[0], np.cumsum(size.astype(np.int64))]))
    packed = torch.full((cap,), 0xCD, dtype=torch.uint8, device="cuda")
    fill = torch.full(((cap + 16383) // 16384,), 77, dtype=torch.int32, device="cuda")
    fusco.fusco_segments_copy(dev(src), d_desc, packed, None, cum, cap, status, slice_bytes=16384, slice_fill=fill)
    torch.cuda.synchronize()
    assert int(status.item()) == 0
    assert np.array_equal(packed[:total].cpu().numpy(), want)
    assert bool((packed[total:] == 0xCD).all())
    got_fill = fill.cpu().numpy()
    assert np.array_equal(got_fill[:len(fill_want)], fill_want.astype(np.int32)) and np.all(got_fill[len(fill_want):] == 0)
    # receiver side: scatter the packed stream back
    back = torch.full((max(span, 16),), 0xAB, dtype=torch.uint8, device="cuda")
    fusco.fusco_segments_copy(packed, None, back, d_desc, cum, cap, status)
    torch.cuda.synchronize()
    assert int(status.item()) == 0
    if n:
        want_back = oracle.segments_copy(want, size, dst_off=off, dst_bytes=len(src), fill_value=0xAB)
        assert np.array_equal(back.cpu().numpy(), want_back)


def test_scatter_to_scatter_and_token_rows(fusco, oracle):
    # the shuffle's level 2 written as a descriptor list: one 14336-byte segment per slot
    rng = np.random.default_rng(3)
    N, k, E, D, row = 300, 8, 64, 8, 14336
    A = random_topk(rng, N, k, E)
    x = rng.integers(0, 256, size=(N, row), dtype=np.uint8)
    pl = oracle.plan(A, E, D)
    _, expert_want = oracle.dispatch(pl, x)
    size = np.full(pl.P, row, dtype=np.int64)
    src_desc = desc_dev(pl.slot_token.astype(np.int64) * row, size)
    dst_desc = desc_dev(np.arange(pl.P, dtype=np.int64) * row, size)
    cum, status = scan(fusco, src_desc)
    out = torch.zeros((pl.P, row), dtype=torch.uint8, device="cuda")
    fusco.fusco_segments_copy(dev(x), src_desc, out, dst_desc, cum, pl.P * row, status)
    torch.cuda.synchronize()
    assert int(status.item()) == 0 and np.array_equal(out.cpu().numpy(), expert_want)


def test_invalid_descriptors_are_counted_and_skipped(fusco):
    size = np.array([64, 40, 32, 64], dtype=np.int64)       # 40 is not a multiple of 16
    off = np.array([0, 64, 136, 4096], dtype=np.int64)      # 136 is not a multiple of 16; 4096 lies outside src
    d = desc_dev(off, size)
    cum, status = scan(fusco, d)
    assert int(status.item()) == 2
    assert cum.cpu().tolist() == [0, 64, 64, 64, 128]
    src = torch.arange(256, dtype=torch.uint8, device="cuda")
    dst = torch.full((256,), 0xEE, dtype=torch.uint8, device="cuda")
    fusco.fusco_segments_copy(src, d, dst, None, cum, 256, status)
    torch.cuda.synchronize()
    assert int(status.item()) == 2 + 4                      # four 16-byte units of the out-of-range segment
    assert torch.equal(dst[:64], src[:64]) and bool((dst[64:] == 0xEE).all())


def test_offsets_that_wrap_are_counted_and_touch_nothing(fusco):
    """Offsets whose sum with the position inside the segment leaves the buffer, or wraps around 2^64 (a negative
    int64, a huge value), are skipped unit by unit: nothing is read or written through them, the rows next to the
    buffer stay as they were, and a slice with such holes does not reach its size."""
    seg = 64
    good = np.array([0, 128], dtype=np.int64)
    bad = np.array([-16, -64, np.iinfo(np.int64).min, np.iinfo(np.int64).max - 15, 1 << 40], dtype=np.int64)
    off = np.concatenate([good[:1], bad, good[1:]])             # 7 segments of 64 bytes, 5 of them wild
    size = np.full(len(off), seg, dtype=np.int64)
    d = desc_dev(off, size)
    cum, status = scan(fusco, d)
    assert int(status.item()) == 0                               # aligned offsets and sizes: the scan accepts them
    total = seg * len(off)
    # the buffers are windows in the middle of larger allocations, so that a write or a read just outside
    # would hit memory we own and can inspect
    room = torch.full((3, 4096), 0x5A, dtype=torch.uint8, device="cuda")
    src = room[1, :256]
    src.copy_(torch.arange(256, dtype=torch.uint8, device="cuda"))
    out_room = torch.full((3, 16384), 0xEE, dtype=torch.uint8, device="cuda")
    packed = out_room[1]
    fill = torch.full((1,), 77, dtype=torch.int32, device="cuda")
    fusco.fusco_segments_copy(src, d, packed, None, cum, 16384, status, slice_bytes=16384, slice_fill=fill)
    torch.cuda.synchronize()
    units_bad = len(bad) * seg // 16
    assert int(status.item()) == units_bad
    got = packed.cpu().numpy()
    want = np.full(16384, 0xEE, dtype=np.uint8)
    want[0:64] = np.arange(0, 64)
    want[6 * seg:7 * seg] = np.arange(128, 192)
    assert np.array_equal(got, want)
    assert bool((out_room[0] == 0xEE).all()) and bool((out_room[2] == 0xEE).all())
    assert int(fill.item()) == total - 16 * units_bad           # holes are not counted: the slice is not ready
    # receiver side: the same wild offsets as destinations
    status.zero_()
    dst = out_room[1, :256]
    out_room.fill_(0xEE)
    stream_in = torch.arange(total, dtype=torch.int32, device="cuda").to(torch.uint8)
    fusco.fusco_segments_copy(stream_in, None, dst, d, cum, total, status)
    torch.cuda.synchronize()
    assert int(status.item()) == units_bad
    want = np.full(256, 0xEE, dtype=np.uint8)
    want[0:64] = np.arange(0, 64)
    want[128:192] = (np.arange(6 * seg, 7 * seg) % 256).astype(np.uint8)
    assert np.array_equal(dst.cpu().numpy(), want)
    assert bool((out_room[0] == 0xEE).all()) and bool((out_room[2] == 0xEE).all()) and bool((out_room[1, 256:] == 0xEE).all())
    assert bool((room[0] == 0x5A).all()) and bool((room[2] == 0x5A).all())


def test_consumer_on_another_stream_sees_complete_slices_only(fusco, oracle):
    """The slice protocol under concurrency (section 3.2, pipelined workflow: the consumer takes a slice as soon
    as it is ready).  A consumer workgroup on a second stream polls the per-slice byte counters while
    fusco_segments_copy packs the stream, and adds up the words of every slice it sees complete: each such sum
    must be the sum of that slice of the oracle's packed stream, i.e. a complete counter implies visible bytes.
    The consumer's polling is bounded, so the test ends whatever the scheduling."""
    rng = np.random.default_rng(99)
    n = 12000
    size, off, span = _random_layout(rng, n, max_units=1200)      # segments of 16 B .. 19 KB, about 115 MB in all
    src = rng.integers(0, 256, size=span, dtype=np.uint8)
    slice_bytes = 1 << 20
    want, fill_want = oracle.segments_copy(src, size, src_off=off, slice_bytes=slice_bytes)
    total = int(size.sum())
    slices = len(fill_want)
    words = np.zeros(slices * (slice_bytes // 4), dtype=np.uint32)
    words[:total // 4] = want.view(np.uint32)
    sums_want = words.reshape(slices, -1).astype(np.uint64).sum(axis=1)

    d_src, d_desc = dev(src), desc_dev(off, size)
    cum, status = scan(fusco, d_desc)
    produce, consume = torch.cuda.Stream(), torch.cuda.Stream()
    waited_total = 0
    for attempt in range(3):
        packed = torch.zeros(total + 4096, dtype=torch.uint8, device="cuda")
        fill = torch.zeros(slices, dtype=torch.int32, device="cuda")
        report = torch.full((slices, 4), -1, dtype=torch.int32, device="cuda")
        torch.cuda.synchronize()
        with torch.cuda.stream(consume):
            fusco.fusco_probe_consume_slices(packed, total, slice_bytes, fill, 1 << 20, report)
        with torch.cuda.stream(produce):
            fusco.fusco_segments_copy(d_src, d_desc, packed, None, cum, total + 4096, status, slice_bytes=slice_bytes,
                                      slice_fill=fill)
        torch.cuda.synchronize()
        assert int(status.item()) == 0
        assert np.array_equal(fill.cpu().numpy().astype(np.uint32), fill_want)
        assert np.array_equal(packed[:total].cpu().numpy(), want)
        rep = report.cpu().numpy().view(np.uint32).astype(np.uint64)
        ready, polls = rep[:, 0], rep[:, 1]
        sums = rep[:, 2] | (rep[:, 3] << np.uint64(32))
        assert set(ready.tolist()) <= {0, 1}
        # the one thing the protocol promises: a slice seen complete had all its bytes visible
        assert np.array_equal(sums[ready == 1], sums_want[ready == 1]), attempt
        # the consumer's poll budget is far beyond the producer's run time, so it sees every slice
        assert int(ready.sum()) == slices, (attempt, int(ready.sum()), slices)
        waited_total += int((polls > 0).sum())
        print("attempt %d: consumer had to wait for %d of %d slices" % (attempt, int((polls > 0).sum()), slices), flush=True)
    # over three runs the consumer was at least once ahead of the producer (it starts first): the two did overlap
    assert waited_total > 0
