"""Pins for the oracle's data movement and weighted sum: library gathers, closed forms, special
cases and the accumulate error bound."""
import numpy as np
import pytest
import torch

import workloads as W
from definitions import random_topk


def _rand_bf16(rng, shape):
    return W.bf16_bits(rng.standard_normal(shape).astype(np.float32))


@pytest.mark.parametrize("N,k,E,D,H", [(37, 2, 8, 4, 24), (64, 4, 16, 2, 40), (19, 8, 32, 8, 8), (50, 3, 6, 6, 16)])
def test_dispatch_is_index_select(oracle, N, k, E, D, H):
    rng = np.random.default_rng(N * H)
    A = random_topk(rng, N, k, E)
    x = _rand_bf16(rng, (N, H))
    pl = oracle.plan(A, E, D)
    send_buf, expert_buf = oracle.dispatch(pl, x)
    # the rearrangement operator the paper measures (section 2.3) is index_select
    xt = torch.from_numpy(x.astype(np.int32))
    assert np.array_equal(expert_buf, torch.index_select(xt, 0, torch.from_numpy(pl.slot_token).long()).numpy())
    assert np.array_equal(send_buf, torch.index_select(xt, 0, torch.from_numpy(pl.send_src).long()).numpy())
    # row s of the expert tensor holds the row of the token whose expert id opens segment s
    seg_expert = np.repeat(np.arange(E), pl.exp_count)
    for s in range(pl.P):
        t = pl.slot_token[s]
        assert seg_expert[s] in A[t]
        assert np.array_equal(expert_buf[s], x[t])


def test_dispatch_rows_equals_full_dispatch(oracle):
    rng = np.random.default_rng(13)
    A = random_topk(rng, 60, 4, 16)
    x = _rand_bf16(rng, (60, 24))
    pl = oracle.plan(A, 16, 4)
    _, expert_buf = oracle.dispatch(pl, x)
    slots = np.array([0, 239, 17, 17, 100], dtype=np.int32)
    assert np.array_equal(oracle.dispatch_rows(pl, x, slots), expert_buf[slots])
    assert np.array_equal(oracle.dispatch_rows(pl, x, slots), x[pl.slot_token[slots]])
    with pytest.raises(ValueError):
        oracle.dispatch_rows(pl, x, [240])


def test_dispatch_aux_plane_follows_payload(oracle):
    rng = np.random.default_rng(11)
    A = random_topk(rng, 20, 4, 16)
    x = rng.integers(0, 256, size=(20, 256), dtype=np.uint8)
    sc = rng.standard_normal((20, 2)).astype(np.float32)
    pl = oracle.plan(A, 16, 8)
    send_buf, expert_buf, send_aux, expert_aux = oracle.dispatch(pl, x, sc)
    assert np.array_equal(expert_buf, x[pl.slot_token]) and np.array_equal(expert_aux, sc[pl.slot_token])
    assert np.array_equal(send_buf, x[pl.send_src]) and np.array_equal(send_aux, sc[pl.send_src])


def test_dispatch_k1_is_row_permutation(oracle):
    rng = np.random.default_rng(12)
    A = random_topk(rng, 33, 1, 4)
    x = _rand_bf16(rng, (33, 16))
    pl = oracle.plan(A, 4, 2)
    _, expert_buf = oracle.dispatch(pl, x)
    assert np.array_equal(np.sort(expert_buf.view(np.uint16), axis=0), np.sort(x, axis=0))
    assert np.array_equal(expert_buf[pl.pair_slot], x)


@pytest.mark.parametrize("k", [1, 2, 4, 8])
def test_combine_dyadic_weights_return_x_exactly(oracle, k):
    # dispatch, identity experts, combine with w = 1/k: every product and partial sum is exact in
    # single precision and the result is the bfloat16 input itself
    rng = np.random.default_rng(20 + k)
    N, E, D, H = 45, 16, 4, 32
    A = random_topk(rng, N, k, E)
    x = _rand_bf16(rng, (N, H))
    pl = oracle.plan(A, E, D)
    _, y = oracle.dispatch(pl, x)
    w = np.full((N, k), 1.0 / k, dtype=np.float32)
    o32, o16 = oracle.combine_f32(y, w, pl.pair_slot)
    assert np.array_equal(o16, x)
    assert np.array_equal(o32, W.bf16_bits_to_f32(x))
    assert np.array_equal(oracle.combine_f64(y, w, pl.pair_slot), W.bf16_bits_to_f32(x).astype(np.float64))


def test_combine_one_hot_selects_one_row(oracle):
    rng = np.random.default_rng(30)
    N, k, E, D, H = 31, 4, 8, 2, 16
    A = random_topk(rng, N, k, E)
    pl = oracle.plan(A, E, D)
    y = _rand_bf16(rng, (pl.P, H))
    pick = rng.integers(0, k, size=N)
    w = np.zeros((N, k), dtype=np.float32)
    w[np.arange(N), pick] = 1.0
    o32, o16 = oracle.combine_f32(y, w, pl.pair_slot)
    want = y[pl.pair_slot.reshape(N, k)[np.arange(N), pick]]
    assert np.array_equal(o16, want)
    assert np.array_equal(oracle.combine_f64(y, w, pl.pair_slot), W.bf16_bits_to_f32(want).astype(np.float64))


def test_combine_distinguishes_weight_order(oracle):
    # a transposed or j-reversed weight lookup changes the result
    N, k, E, D, H = 3, 2, 4, 2, 4
    A = np.array([[0, 3], [2, 1], [1, 0]], dtype=np.int32)
    pl = oracle.plan(A, E, D)
    y = W.bf16_bits(np.arange(pl.P * H, dtype=np.float32).reshape(pl.P, H))
    w = np.array([[0.25, 0.75], [0.5, 0.5], [1.0, 0.0]], dtype=np.float32)
    yf = W.bf16_bits_to_f32(y).astype(np.float64)
    want = np.zeros((N, H))
    for t in range(N):
        for j in range(k):
            e = A[t, j]
            # slot by definition: pairs with a smaller expert, then earlier pairs of the same expert
            s = int(np.sum(A < e) + sum(1 for t2 in range(N) for j2 in range(k)
                                        if A[t2, j2] == e and (t2, j2) < (t, j)))
            want[t] += float(w[t, j]) * yf[s]
    assert np.array_equal(oracle.combine_f64(y, w, pl.pair_slot), want)


@pytest.mark.parametrize("ydt", ["bf16", "f32"])
def test_combine_matches_fp64_library_sum_and_error_bound(oracle, ydt):
    rng = np.random.default_rng(40)
    N, k, E, D, H = 120, 8, 64, 8, 96
    A = random_topk(rng, N, k, E)
    pl = oracle.plan(A, E, D)
    if ydt == "bf16":
        y = _rand_bf16(rng, (pl.P, H))
        yf = W.bf16_bits_to_f32(y)
    else:
        y = rng.standard_normal((pl.P, H)).astype(np.float32)
        yf = y
    w = rng.random((N, k)).astype(np.float32)
    w /= w.sum(1, keepdims=True)
    # library cross-check: gather + einsum in double precision
    yt = torch.from_numpy(yf.astype(np.float64))[torch.from_numpy(pl.pair_slot).long()].reshape(N, k, H)
    want = torch.einsum("nk,nkh->nh", torch.from_numpy(w.astype(np.float64)), yt).numpy()
    got64 = oracle.combine_f64(y, w, pl.pair_slot)
    scale = oracle.combine_abs_f64(y, w, pl.pair_slot)
    assert np.all(np.abs(got64 - want) <= 1e-15 * scale + 1e-300)
    wantabs = torch.einsum("nk,nkh->nh", torch.from_numpy(w.astype(np.float64)), yt.abs()).numpy()
    assert np.allclose(scale, wantabs, rtol=1e-14, atol=0)
    # single-precision variant stays within k ulp(float32) of the scale: far inside the 1e-5 bar
    o32, o16 = oracle.combine_f32(y, w, pl.pair_slot)
    assert np.all(np.abs(o32.astype(np.float64) - got64) <= k * 2.0 ** -24 * scale)
    # bfloat16 output is the nearest-even rounding of the float32 sum
    assert np.array_equal(o16, W.bf16_bits(o32))
    tb = torch.from_numpy(o32).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(o16, tb)


def test_combine_token_subset(oracle):
    rng = np.random.default_rng(50)
    N, k, E, D, H = 40, 4, 16, 4, 8
    A = random_topk(rng, N, k, E)
    pl = oracle.plan(A, E, D)
    y = _rand_bf16(rng, (pl.P, H))
    w = rng.random((N, k)).astype(np.float32)
    full = oracle.combine_f64(y, w, pl.pair_slot)
    toks = np.array([39, 0, 7, 7, 21], dtype=np.int32)
    assert np.array_equal(oracle.combine_f64(y, w, pl.pair_slot, tokens=toks), full[toks])
    f32_full, b16_full = oracle.combine_f32(y, w, pl.pair_slot)
    f32_sub, b16_sub = oracle.combine_f32(y, w, pl.pair_slot, tokens=toks)
    assert np.array_equal(f32_sub, f32_full[toks]) and np.array_equal(b16_sub, b16_full[toks])


def test_bf16_rounding_ties_to_even(oracle):
    # 1 + 2^-8 is halfway between bfloat16 1.0 and 1 + 2^-7: ties go to the even mantissa (1.0);
    # 1 + 3*2^-8 is halfway between 1 + 2^-7 and 1 + 2^-6: goes to 1 + 2^-6 (even)
    y = np.array([[1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20, -1.0 - 2.0 ** -8]],
                 dtype=np.float32)
    w = np.ones((1, 1), dtype=np.float32)
    _, o16 = oracle.combine_f32(y, w, np.zeros(1, dtype=np.int32))
    assert o16.tolist() == [[0x3F80, 0x3F82, 0x3F81, 0xBF80]]


def test_bf16_rounding_is_nearest_representable_over_the_range(oracle):
    """Definition, not bit tricks: the result is the bfloat16 value nearest to the float (both neighbours are
    built by truncation and compared in float64), ties go to the even mantissa, values past the largest finite
    bfloat16 by half a step or more become infinity."""
    rng = np.random.default_rng(8)
    bits = rng.integers(0, 1 << 32, size=20000, dtype=np.uint64).astype(np.uint32)
    # (-0.0 is left out: the chain starts from +0 and w * (-0) + (+0) is +0)
    edge = np.array([0x00000000, 0x00000001, 0x00007FFF, 0x00008000, 0x00008001, 0x00018000, 0x007F8000,
                     0x7F7F7FFF, 0x7F7F8000, 0x7F7FFFFF, 0xFF7F8000, 0x7F800000, 0xFF800000, 0x3F808000, 0x3F818000],
                    dtype=np.uint32)
    bits = np.concatenate([bits, edge])
    f = bits.view(np.float32)
    keep = ~np.isnan(f)
    bits, f = bits[keep], f[keep]
    w = np.ones((1, 1), dtype=np.float32)
    _, o16 = oracle.combine_f32(f.reshape(1, -1), w, np.zeros(1, dtype=np.int32))
    got = o16.reshape(-1)
    lo = (bits & 0xFFFF0000).astype(np.uint32)                       # neighbour towards zero
    hi = lo + np.uint32(0x10000)                                     # next bfloat16 away from zero (may be inf)
    x = f.astype(np.float64)
    flo = lo.view(np.float32).astype(np.float64)
    with np.errstate(all="ignore"):
        fhi = hi.view(np.float32).astype(np.float64)
        # an infinite upper neighbour stands for the next power of two in the distance test
        fhi = np.where(np.isinf(fhi), np.sign(fhi) * 2.0 ** 128, fhi)
        dlo, dhi = np.abs(x - flo), np.abs(fhi - x)
    even_lo = ((lo >> 16) & 1) == 0
    want = np.where(np.isinf(f), lo, np.where((dlo < dhi) | ((dlo == dhi) & even_lo), lo, hi)) >> 16
    assert np.array_equal(got, want.astype(np.uint16))


def test_combine_special_values_follow_ieee(oracle):
    inf, nan = np.float32(np.inf), np.float32(np.nan)
    y = np.array([[1.0, -0.0, inf, 1e-45, 3.0e38, nan, 0.0]], dtype=np.float32)
    one = np.ones((1, 1), dtype=np.float32)
    z = np.zeros(1, dtype=np.int32)
    f32, _ = oracle.combine_f32(y, one, z)
    keep = [0, 2, 3, 4]
    assert np.array_equal(f32.view(np.uint32)[0, keep], y.view(np.uint32)[0, keep]) and np.isnan(f32[0, 5])
    # the chain starts from +0: 1 * (-0) + (+0) is +0, as IEEE addition of opposite zeros says
    assert f32.view(np.uint32)[0, 1] == 0
    f32, b16 = oracle.combine_f32(y, np.full((1, 1), 2.0, dtype=np.float32), z)
    assert f32[0, 4] == inf and b16[0, 4] == 0x7F80            # overflow in the product
    assert f32[0, 3] == np.float32(2.8e-45)                    # a subnormal stays a subnormal (no flush to zero)
    f32, _ = oracle.combine_f32(y, np.zeros((1, 1), dtype=np.float32), z)
    assert np.isnan(f32[0, 2]) and f32[0, 0] == 0.0            # 0 * inf is a NaN
    # inf - inf over two terms
    y2 = np.array([[inf], [inf]], dtype=np.float32)
    f32, b16 = oracle.combine_f32(y2, np.array([[1.0, -1.0]], dtype=np.float32), np.array([0, 1], dtype=np.int32))
    assert np.isnan(f32[0, 0]) and (b16[0, 0] & 0x7FFF) > 0x7F80


# ---- combine along the two levels in reverse (per-device partial sums) ----

def test_two_hop_combine_single_device_equals_flat_sum(oracle):
    # D = 1: one partial per token holds the whole chain, so both associations coincide bit for bit
    rng = np.random.default_rng(60)
    N, k, E, H = 40, 8, 32, 24
    A = random_topk(rng, N, k, E)
    pl = oracle.plan(A, E, 1)
    y = _rand_bf16(rng, (pl.P, H))
    w = rng.random((N, k)).astype(np.float32)
    f32, b16 = oracle.combine_f32(y, w, pl.pair_slot)
    h32, h16 = oracle.combine_two_hop_f32(pl, y, w)
    assert np.array_equal(f32.view(np.uint32), h32.view(np.uint32)) and np.array_equal(b16, h16)


def test_two_hop_combine_one_expert_per_device_is_products_then_ordered_adds(oracle):
    # D = E: every partial is one correctly rounded product; the result is their float32 sum in j order
    rng = np.random.default_rng(61)
    N, k, E, H = 30, 5, 8, 16
    A = random_topk(rng, N, k, E)
    pl = oracle.plan(A, E, E)
    y = rng.standard_normal((pl.P, H)).astype(np.float32)
    w = rng.standard_normal((N, k)).astype(np.float32)
    h32, _, part = oracle.combine_two_hop_f32(pl, y, w, want_partial=True)
    prod = w.reshape(N, k, 1) * y[pl.pair_slot].reshape(N, k, H)            # float32 multiply, rounded once
    assert np.array_equal(part[pl.pair_send_row].reshape(N, k, H).view(np.uint32), prod.view(np.uint32))
    acc = np.zeros((N, H), dtype=np.float32)
    for j in range(k):
        acc = acc + prod[:, j]
    assert np.array_equal(h32.view(np.uint32), acc.view(np.uint32))


def test_two_hop_combine_groups_by_device_in_first_appearance_order(oracle):
    # hand case: devices of the entries are [1, 0, 1]; partials are (e0 + e2) and (e1); out = p(dev1) + p(dev0)
    A = np.array([[2, 0, 3]], dtype=np.int32)
    pl = oracle.plan(A, 4, 2)
    assert pl.pair_first.tolist() == [1, 1, 0]
    big, tiny = np.float32(2.0 ** 24), np.float32(1.0)
    y = np.zeros((3, 1), dtype=np.float32)
    y[pl.pair_slot[0]], y[pl.pair_slot[1]], y[pl.pair_slot[2]] = big, tiny, -big
    w = np.ones((1, 3), dtype=np.float32)
    h32, _, part = oracle.combine_two_hop_f32(pl, y, w, want_partial=True)
    f32, _ = oracle.combine_f32(y, w, pl.pair_slot)
    assert part[pl.pair_send_row[0], 0] == 0.0 and part[pl.pair_send_row[1], 0] == 1.0
    assert h32[0, 0] == 1.0          # (2^24 - 2^24) + 1
    assert f32[0, 0] == 0.0          # ((2^24 + 1) - 2^24) loses the 1 in single precision


@pytest.mark.parametrize("k", [1, 2, 4, 8])
def test_two_hop_combine_dyadic_weights_return_x_exactly(oracle, k):
    rng = np.random.default_rng(62 + k)
    N, E, D, H = 45, 16, 4, 32
    A = random_topk(rng, N, k, E)
    x = _rand_bf16(rng, (N, H))
    pl = oracle.plan(A, E, D)
    _, y = oracle.dispatch(pl, x)
    w = np.full((N, k), 1.0 / k, dtype=np.float32)
    h32, h16 = oracle.combine_two_hop_f32(pl, y, w)
    assert np.array_equal(h16, x) and np.array_equal(h32, W.bf16_bits_to_f32(x))


def test_two_hop_combine_error_bound_and_subset(oracle):
    rng = np.random.default_rng(63)
    N, k, E, D, H = 100, 8, 64, 8, 48
    A = random_topk(rng, N, k, E)
    pl = oracle.plan(A, E, D)
    y = _rand_bf16(rng, (pl.P, H))
    w = (rng.standard_normal((N, k)) * 2).astype(np.float32)
    h32, h16, part = oracle.combine_two_hop_f32(pl, y, w, want_partial=True)
    ref = oracle.combine_f64(y, w, pl.pair_slot)
    scale = oracle.combine_abs_f64(y, w, pl.pair_slot)
    assert np.all(np.abs(h32.astype(np.float64) - ref) <= (k + D) * 2.0 ** -24 * scale)
    assert not np.isnan(part).any()
    # every partial row is the flat sum of the token's entries on that device
    for r in rng.integers(0, pl.U, size=40):
        t = pl.send_src[r]
        js = [j for j in range(k) if pl.pair_send_row[t * k + j] == r]
        sub32, _ = oracle.combine_f32(y[pl.pair_slot[t * k + np.array(js)]], w[t:t + 1, js], np.arange(len(js), dtype=np.int32))
        assert np.array_equal(part[r].view(np.uint32), sub32[0].view(np.uint32))
    toks = np.array([99, 0, 5], dtype=np.int32)
    s32, s16 = oracle.combine_two_hop_f32(pl, y, w, tokens=toks)
    assert np.array_equal(s32, h32[toks]) and np.array_equal(s16, h16[toks])


# ---- one rounding per term: the fused multiply-add of the single-precision chain ----
# Hand-worked.  Term 0 puts acc = -y0 exactly (w = 1).  Term 1 has an exact product w1 * y1 that needs one
# bit more than single precision holds, and that bit survives only if the product is not rounded before
# the addition:
#   float32 y:  w1 = y1 = 1 + 2^-12      product = 1 + 2^-11 + 2^-24   (2^-24 is half an ulp of 1: a tie that
#               rounds to the even neighbour 1 + 2^-11)   y0 = -1
#               fused:   -1 + (1 + 2^-11 + 2^-24) = 2^-11 + 2^-24     multiply, round, add: 2^-11
#   bfloat16 y: y1 = 1 + 2^-7 (8 significant bits), w1 = 1 + 2^-17   product = 1 + 2^-7 + 2^-17 + 2^-24
#               y0 = -(1 + 2^-7)   fused: 2^-17 + 2^-24               multiply, round, add: 2^-17
# Rounded to bfloat16 (8 significant bits): 2^-11 (1 + 2^-13) -> 2^-11;  2^-17 (1 + 2^-7) is exact.
FMA_F32 = dict(y0=-1.0, y1=1.0 + 2.0 ** -12, w1=1.0 + 2.0 ** -12, fused=2.0 ** -11 + 2.0 ** -24, unfused=2.0 ** -11,
               bf16_out=2.0 ** -11)
FMA_BF16 = dict(y0=-(1.0 + 2.0 ** -7), y1=1.0 + 2.0 ** -7, w1=1.0 + 2.0 ** -17, fused=2.0 ** -17 + 2.0 ** -24,
                unfused=2.0 ** -17, bf16_out=2.0 ** -17 + 2.0 ** -24)


def _fma_case(case, as_bf16):
    y = np.array([[case["y0"]], [case["y1"]]], dtype=np.float32)
    if as_bf16:
        bits = W.bf16_bits(y)
        assert np.array_equal(W.bf16_bits_to_f32(bits), y)          # both values are exact in bfloat16
        y = bits
    w = np.array([[1.0, case["w1"]]], dtype=np.float32)
    assert float(w[0, 1]) == case["w1"]                             # and the weight is exact in float32
    return y, w


@pytest.mark.parametrize("case,as_bf16", [(FMA_F32, False), (FMA_BF16, True)])
def test_combine_f32_rounds_once_per_term(oracle, case, as_bf16):
    y, w = _fma_case(case, as_bf16)
    f32, b16 = oracle.combine_f32(y, w, np.array([0, 1], dtype=np.int32))
    assert float(f32[0, 0]) == case["fused"] and float(f32[0, 0]) != case["unfused"]
    # the bfloat16 output is the nearest bfloat16 of that sum
    assert np.array_equal(W.bf16_bits_to_f32(b16), np.array([[case["bf16_out"]]], dtype=np.float32))
    # the double-precision sum is exact here and agrees with the fused result
    assert float(oracle.combine_f64(y, w, np.array([0, 1], dtype=np.int32))[0, 0]) == case["fused"]


@pytest.mark.parametrize("case,as_bf16", [(FMA_F32, False), (FMA_BF16, True)])
def test_two_hop_partials_round_once_per_term(oracle, case, as_bf16):
    y, w = _fma_case(case, as_bf16)
    # both entries on one device: the partial row is the fused chain, the output adds it to +0
    A = np.array([[0, 1]], dtype=np.int32)
    same = oracle.plan(A, 2, 1)
    h32, _, part = oracle.combine_two_hop_f32(same, y[same.slot_pair], w, want_partial=True)
    assert float(part[0, 0]) == case["fused"] and float(h32[0, 0]) == case["fused"]
    # one entry per device: each partial is one rounded product, and their sum has lost the last bit
    split = oracle.plan(A, 2, 2)
    h32, _, part = oracle.combine_two_hop_f32(split, y[split.slot_pair], w, want_partial=True)
    assert float(part[split.pair_send_row[0], 0]) == case["y0"]
    assert float(part[split.pair_send_row[1], 0]) == float(np.float32(case["w1"]) * np.float32(case["y1"]))
    assert float(h32[0, 0]) == case["unfused"]
