"""Measurement-aid kernels on the GPU: they move exactly the rows their shape says, so the bandwidth
figures taken with them count the right bytes.  Expected values come from numpy index arithmetic on
the host (a permutation i -> i * m mod n), not from the shuffle kernels."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def fusco():
    import paper_2512_22036_amd as f
    f.load_library()
    assert torch.cuda.is_available()
    return f


def _rows(n, units, seed):
    rng = np.random.default_rng(seed)
    return rng.integers(0, 2**32, size=(n, units * 4), dtype=np.uint32)


def _sorted_rows(a):
    return a[np.lexsort(a.T[::-1])]


@pytest.mark.parametrize("n,units", [(1, 1), (5, 3), (64, 300), (1000, 17)])
@pytest.mark.parametrize("through", [False, True])
def test_copy_shape_is_a_row_permutation(fusco, n, units, through):
    src = _rows(n, units, n + units)
    d_src = torch.from_numpy(src.view(np.int32)).cuda()
    # in launch order: a plain copy
    d_dst = torch.zeros_like(d_src)
    fusco.fusco_probe_rows(d_src, d_dst, 1, 1, scatter=False, write_through=through)
    assert np.array_equal(d_dst.cpu().numpy().view(np.uint32), src)
    # scattered: every row arrives exactly once, somewhere
    d_dst = torch.zeros_like(d_src)
    fusco.fusco_probe_rows(d_src, d_dst, 1, 1, scatter=True, write_through=through)
    got = d_dst.cpu().numpy().view(np.uint32)
    assert np.array_equal(_sorted_rows(got), _sorted_rows(src))
    if n >= 64:
        assert not np.array_equal(got, src)


def test_dispatch_and_combine_shapes(fusco):
    n, units = 96, 40
    src = _rows(n, units, 7)
    d_src = torch.from_numpy(src.view(np.int32)).cuda()
    # one row read, eight rows written: every source row shows up exactly 8 times
    d_dst = torch.zeros((n * 8, units * 4), dtype=torch.int32, device="cuda")
    for scatter in (False, True):
        d_dst.zero_()
        fusco.fusco_probe_rows(d_src, d_dst, 1, 8, scatter=scatter)
        got = d_dst.cpu().numpy().view(np.uint32)
        assert np.array_equal(_sorted_rows(got), _sorted_rows(np.repeat(src, 8, axis=0)))
    # eight rows read, one written: the XOR of each group of 8, in launch order
    d_out = torch.zeros((n // 8, units * 4), dtype=torch.int32, device="cuda")
    fusco.fusco_probe_rows(d_src, d_out, 8, 1, scatter=False)
    want = np.bitwise_xor.reduce(src.reshape(n // 8, 8, -1), axis=1)
    assert np.array_equal(d_out.cpu().numpy().view(np.uint32), want)
    d_out.zero_()
    fusco.fusco_probe_rows(d_src, d_out, 8, 1, scatter=True)
    assert np.array_equal(np.bitwise_xor.reduce(d_out.cpu().numpy().view(np.uint32), axis=0),
                          np.bitwise_xor.reduce(src, axis=0))


def test_fill_and_read_shapes(fusco):
    n, units = 50, 9
    d_dst = torch.full((n, units * 4), -1, dtype=torch.int32, device="cuda")
    fusco.fusco_probe_rows(None, d_dst, 0, 1, scatter=True)
    got = d_dst.cpu().numpy().view(np.uint32).reshape(n, units, 4)
    # a filled unit holds (workgroup, unit index, 0, 0): each workgroup number once, all units of a row alike
    assert sorted(got[:, 0, 0].tolist()) == list(range(n))
    assert np.array_equal(got[:, :, 1], np.broadcast_to(np.arange(units, dtype=np.uint32), (n, units)))
    assert not got[:, :, 2:].any()
    sink = torch.full((1,), 123, dtype=torch.int32, device="cuda")
    d_src = torch.from_numpy(_rows(n, units, 3).view(np.int32)).cuda()
    fusco.fusco_probe_rows(d_src, None, 1, 0, scatter=True, sink=sink)
    torch.cuda.synchronize()
    assert sink.item() == 123


def test_probe_rejects_bad_shapes(fusco):
    a = torch.zeros((8, 16), dtype=torch.int32, device="cuda")
    b = torch.zeros((12, 16), dtype=torch.int32, device="cuda")
    with pytest.raises(fusco.FuscoError):
        fusco.fusco_probe_rows(a, b, 1, 8, scatter=False)          # 12 rows are not groups of 8
    with pytest.raises(fusco.FuscoError):
        fusco.fusco_probe_rows(a, a, 3, 1, scatter=False)          # shape not offered
    with pytest.raises(fusco.FuscoError):
        fusco.fusco_probe_rows(a, None, 1, 0, scatter=False)       # read-only shape without a sink


def test_call_timing_events(fusco):
    """Armed events are recorded by the call's own kernels, are used up by one call, and change no result."""
    rng = np.random.default_rng(5)
    N, k, E, D, H = 3000, 4, 32, 4, 512
    A = np.stack([rng.permutation(E)[:k] for _ in range(N)]).astype(np.int32)
    d_A = torch.from_numpy(A).cuda()
    L = fusco.Layout(N, k, E, D)
    x = torch.randn((N, H), device="cuda").to(torch.bfloat16)
    w = torch.full((N, k), 1.0 / k, device="cuda")
    eb0 = torch.empty((N * k, H), dtype=torch.bfloat16, device="cuda")
    out0 = torch.empty((N, H), dtype=torch.bfloat16, device="cuda")
    fusco.fusco_plan(L, d_A)
    ref_layout = L.mem.clone()
    fusco.fusco_dispatch(L, x, eb0)
    fusco.fusco_combine(L, eb0, w, out0)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(6)]
    fresh = torch.cuda.Event(enable_timing=True)
    with pytest.raises(fusco.FuscoError):
        fusco.fusco_probe_time_next_call(fresh, ev[0])      # never recorded: no HIP event behind it yet
    for e in ev:
        e.record()
    torch.cuda.synchronize()
    eb = torch.zeros_like(eb0)
    out = torch.zeros_like(out0)
    fusco.fusco_probe_time_next_call(ev[0], ev[1])
    fusco.fusco_plan(L, d_A)                                # three kernels (12 tiles): first start, last end
    fusco.fusco_probe_time_next_call(ev[2], ev[3])
    fusco.fusco_dispatch(L, x, eb)
    fusco.fusco_probe_time_next_call(ev[4], ev[5])
    fusco.fusco_combine(L, eb, w, out)
    fusco.fusco_combine(L, eb, w, out)                      # not armed any more: ordinary launch
    torch.cuda.synchronize()
    assert torch.equal(L.mem, ref_layout) and torch.equal(eb, eb0) and torch.equal(out, out0)
    for i in range(0, 6, 2):
        ms = ev[i].elapsed_time(ev[i + 1])
        assert 0.0005 < ms < 5.0, (i, ms)
    # the calls ran in stream order: plan ends before dispatch starts, dispatch before combine
    assert ev[1].elapsed_time(ev[2]) >= 0.0 and ev[3].elapsed_time(ev[4]) >= 0.0


@pytest.mark.parametrize("pieces,run", [(8, 1), (64, 1), (64, 2), (64, 8), (56, 7), (4096, 16), (4096, 512), (229376, 7)])
def test_pieces_probe_writes_every_piece_exactly_once(fusco, pieces, run):
    buf = torch.full((pieces, 1024), -1, dtype=torch.int32, device="cuda")          # 4 KiB per row
    fusco.fusco_probe_pieces(buf, write=True, run_pieces=run)
    got = buf.cpu().numpy().view(np.uint32).reshape(pieces, 256, 4)
    assert np.array_equal(got[:, :, 0], np.repeat(np.arange(pieces, dtype=np.uint32)[:, None], 256, axis=1))
    assert np.array_equal(got[:, :, 1], np.repeat(np.arange(256, dtype=np.uint32)[None, :], pieces, axis=0))
    # the workgroup that wrote piece p: XCD (b mod 8) owns runs of `run` pieces, 8 runs to a round
    b = got[:, 0, 2].astype(np.int64)
    p = np.arange(pieces)
    assert np.array_equal(np.sort(b), p)
    assert np.array_equal(b % 8, (p // run) % 8)
    # scattered: still every piece once; reads touch nothing
    buf.fill_(-1)
    fusco.fusco_probe_pieces(buf, write=True, scatter=True)
    got = buf.cpu().numpy().view(np.uint32).reshape(pieces, 256, 4)
    assert np.array_equal(got[:, 0, 0], np.arange(pieces, dtype=np.uint32))
    assert np.array_equal(np.sort(got[:, 0, 2]), np.arange(pieces, dtype=np.uint32))
    before = buf.clone()
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    fusco.fusco_probe_pieces(buf, write=False, run_pieces=run, sink=sink)
    fusco.fusco_probe_pieces(buf, write=False, scatter=True, sink=sink)
    torch.cuda.synchronize()
    assert torch.equal(buf, before) and int(sink.item()) == 0
