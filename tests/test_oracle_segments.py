"""Pins for the oracle's segment-descriptor transfer: byte-level brute force, round trips, and the
reduction to the fixed-row dispatch."""
import numpy as np
import pytest

from definitions import random_topk


def _random_layout(rng, n, max_units=40, pad_units=3):
    """n segments of random sizes (multiples of 16) at disjoint, shuffled places of a buffer."""
    size = rng.integers(0, max_units + 1, size=n).astype(np.uint64) * 16
    order = rng.permutation(n)
    off = np.zeros(n, dtype=np.uint64)
    pos = 0
    for i in order:
        pos += int(rng.integers(0, pad_units + 1)) * 16
        off[i] = pos
        pos += int(size[i])
    return size, off, pos + 16 * pad_units


@pytest.mark.parametrize("n", [0, 1, 7, 100])
def test_pack_unpack_against_byte_loops(oracle, n):
    rng = np.random.default_rng(n)
    size, off, span = _random_layout(rng, n)
    src = rng.integers(0, 256, size=span, dtype=np.uint8)
    packed, fill = oracle.segments_copy(src, size, src_off=off, slice_bytes=256)
    want = bytearray()
    for i in range(n):
        for b in range(int(size[i])):
            want.append(int(src[int(off[i]) + b]))
    assert packed.tobytes() == bytes(want)
    total = len(want)
    assert fill.tolist() == [min(256, total - s * 256) for s in range((total + 255) // 256)]
    # unpack puts every segment back where it came from and touches nothing else
    back = oracle.segments_copy(packed, size, dst_off=off, dst_bytes=span, fill_value=0xAB)
    mask = np.zeros(span, dtype=bool)
    for i in range(n):
        mask[int(off[i]):int(off[i]) + int(size[i])] = True
    assert np.array_equal(back[mask], src[mask]) and np.all(back[~mask] == 0xAB)


def test_scatter_to_scatter_is_pack_then_unpack(oracle):
    rng = np.random.default_rng(5)
    n = 60
    size, soff, sspan = _random_layout(rng, n)
    _, doff, dspan = _random_layout(np.random.default_rng(6), n)
    # destination layout must use the same sizes: rebuild offsets for them
    order = rng.permutation(n)
    doff = np.zeros(n, dtype=np.uint64)
    pos = 0
    for i in order:
        doff[i] = pos
        pos += int(size[i]) + 32
    src = rng.integers(0, 256, size=sspan, dtype=np.uint8)
    direct = oracle.segments_copy(src, size, src_off=soff, dst_off=doff, dst_bytes=pos, fill_value=7)
    via = oracle.segments_copy(oracle.segments_copy(src, size, src_off=soff), size, dst_off=doff, dst_bytes=pos, fill_value=7)
    assert np.array_equal(direct, via)


def test_fixed_rows_reduce_to_the_token_dispatch(oracle):
    # one segment per send row, all of one size: packing them is the level-1 transfer of the shuffle
    rng = np.random.default_rng(7)
    N, k, E, D, row = 50, 4, 16, 4, 48
    A = random_topk(rng, N, k, E)
    x = rng.integers(0, 256, size=(N, row), dtype=np.uint8)
    pl = oracle.plan(A, E, D)
    send_buf, expert_buf = oracle.dispatch(pl, x)
    size = np.full(pl.U, row, dtype=np.uint64)
    packed = oracle.segments_copy(x.reshape(-1), size, src_off=pl.send_src.astype(np.uint64) * row)
    assert np.array_equal(packed.reshape(pl.U, row), send_buf)
    # level 2 as a scatter-to-scatter list: one segment per slot
    size2 = np.full(pl.P, row, dtype=np.uint64)
    exp = oracle.segments_copy(send_buf.reshape(-1), size2, src_off=pl.slot_send_row.astype(np.uint64) * row,
                               dst_off=np.arange(pl.P, dtype=np.uint64) * row, dst_bytes=pl.P * row)
    assert np.array_equal(exp.reshape(pl.P, row), expert_buf)
