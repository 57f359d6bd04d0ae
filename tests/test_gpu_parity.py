"""Parity of the HIP path against the CPU oracle, element by element, through the C boundary.

Integer descriptors and moved bytes must be bit-exact.  The weighted sum must be (i) bit-exact
against the oracle's single-precision fused-multiply-add sum in j order (the precision the method
is specified in, both for float32 and bfloat16 outputs) and (ii) within 1e-5 * sum_j |w_j y_j| of
the oracle's double-precision sum.
"""
import numpy as np
import pytest
import torch

import workloads as W
from definitions import PLAN_FIELDS, check_plan_invariants, random_topk

pytestmark = pytest.mark.gpu

REL_TOL = 1e-5


@pytest.fixture(scope="module")
def fusco():
    import paper_2512_22036_amd as f
    f.load_library()
    assert torch.cuda.is_available()
    return f


def dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a)).cuda()
    return t.view(dtype) if dtype is not None else t


def bf16_dev(bits):
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)


def bits_host(t):
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


def gpu_plan(fusco, A, E, D):
    N, k = A.shape
    L = fusco.Layout(N, k, E, D)
    L.mem.fill_(0x7B)   # stale contents must not leak into the result
    fusco.fusco_plan(L, dev(A.astype(np.int32)).reshape(N, k))
    torch.cuda.synchronize()
    return L, L.to_host()


def assert_plan_equal(got, want):
    assert int(got.status[0]) == 0
    for f in PLAN_FIELDS:
        assert np.array_equal(getattr(got, f), getattr(want, f)), f


def assert_tile_order(oracle, L, got, want, tag=""):
    """The transfer order the planner lists for dispatch: per tile of L.tile_tokens tokens, the tile's slots ascending."""
    ts = oracle.tile_order(want.pair_slot, L.N, L.k, L.tile_tokens)
    assert L.tile_count == (L.N + L.tile_tokens - 1) // L.tile_tokens or (L.N == 0 and L.tile_count == 1), tag
    assert np.array_equal(got.tile_slots[:len(ts)], ts), tag


PLAN_SHAPES = [
    # N, k, E, D, distinct experts per token
    # (a planner tile holds 1024 pairs for inputs of up to 1024 pairs, 2048 pairs otherwise)
    (1, 1, 1, 1, True), (1, 8, 256, 8, True), (5, 2, 4, 2, True), (64, 2, 16, 4, True),
    (128, 8, 256, 8, True),        # exactly one tile of 1024 pairs
    (129, 8, 256, 8, True),        # one tile of 2048 pairs
    (256, 8, 256, 8, True),        # exactly one tile of 2048 pairs
    (257, 8, 256, 8, True),        # two tiles of 2048 pairs, the second holding one token
    (1000, 8, 256, 8, True),       # several tiles, ragged tail
    (4096, 2, 16, 4, True), (3000, 8, 128, 16, True), (777, 6, 96, 12, True),
    (300, 64, 1024, 64, True),     # largest k and E
    (500, 3, 1024, 1024, True),    # one expert per device
    (900, 4, 64, 1, True),         # single device
    (1300, 5, 10, 5, False),       # repeated experts inside a token
    (2100, 7, 7, 7, False), (129, 33, 66, 2, True),
    (8192, 8, 256, 8, True),       # 32 tiles: the counts of all other tiles come from the loads issued up front
    (17000, 8, 256, 8, True),      # 67 tiles: more tiles than those loads cover
    # many tiles: per-tile counts are first summed over chunks of tiles (from 96 tiles on)
    (24320, 8, 256, 8, False),     # 95 tiles: the last size read tile by tile
    (24321, 8, 256, 8, False),     # 96 tiles, the last one holding one token
    (30011, 8, 64, 16, True),      # 118 tiles, ragged
    (3300, 64, 1024, 1024, True),  # 104 tiles, more count columns than threads
    (49153, 8, 256, 8, False),     # 193 tiles in chunks of 16
    (50011, 8, 64, 16, True),      # 196 tiles, ragged
    (600000, 8, 32, 4, False),     # 2344 tiles, chunks of 64, last chunk ragged
]


@pytest.mark.parametrize("N,k,E,D,distinct", PLAN_SHAPES)
def test_plan_matches_oracle(fusco, oracle, N, k, E, D, distinct):
    A = random_topk(np.random.default_rng(N * 31 + k), N, k, E, distinct)
    L, got = gpu_plan(fusco, A, E, D)
    want = oracle.plan(A, E, D)
    assert_plan_equal(got, want)
    assert got.U == want.U
    assert_tile_order(oracle, L, got, want)


def _random_shape(rng):
    k = int(rng.choice([1, 2, 3, 4, 6, 8, 12, 16, 31, 64]))
    D = int(rng.choice([1, 2, 3, 4, 8, 16, 64]))
    eloc = int(rng.choice([1, 2, 3, 8, 16]))
    E = min(D * eloc, 1024)
    D = E // eloc
    distinct = bool(rng.integers(0, 2)) and k <= E
    # around the planner's tile boundaries (1024 and 2048 pairs) as well as anywhere
    tpt1 = 1024 // k
    N = int(rng.choice([rng.integers(1, 4000), tpt1 * int(rng.integers(1, 6)) + int(rng.integers(-1, 2)),
                        2 * tpt1 + int(rng.integers(-1, 2))]))
    return max(N, 1), k, E, D, distinct


def test_random_shapes_whole_path(fusco, oracle):
    """300 random shapes (sizes, k, E, D, repeated or distinct experts, tile-boundary token counts, rows from 16
    bytes to 18 KiB so that every chunks-per-thread variant of the movers is drawn, an optional second plane):
    plan, dispatch (expert and wire tensors, both planes) and combine against the oracle, element by element."""
    rng = np.random.default_rng(20251127)
    seen_chunks = set()
    seen_tiled = 0
    for case in range(300):
        N, k, E, D, distinct = _random_shape(rng)
        # 16-byte units per row: up to 64 for any shape, up to 1152 (18 KiB) where the expert tensor stays small
        budget = max(1, (48 << 20) // (16 * N * k))
        C = int(rng.choice([1, 2, 5, 16, 33, 64, 127, 128, 200, 511, 512, 896, 1152]))
        C = min(C, budget) if C > 64 else C
        Ca = int(rng.choice([0, 0, 1, 3, 14])) if C + 14 <= max(budget, 64) else 0      # second plane, 16-byte units
        seen_chunks.add(4 if C + Ca >= 512 else (2 if C + Ca >= 128 else 1))
        A = random_topk(rng, N, k, E, distinct)
        want = oracle.plan(A, E, D)
        L, got = gpu_plan(fusco, A, E, D)
        tag = "case %d: N=%d k=%d E=%d D=%d distinct=%s C=%d Ca=%d" % (case, N, k, E, D, distinct, C, Ca)
        for f in PLAN_FIELDS:
            assert np.array_equal(getattr(got, f), getattr(want, f)), (tag, f)
        assert_tile_order(oracle, L, got, want, tag)
        H = C * 8
        xb = W.bf16_bits(rng.standard_normal((N, H)).astype(np.float32))
        eb = torch.zeros((L.P, H), dtype=torch.bfloat16, device="cuda")
        sb = torch.zeros((L.send_cap, H), dtype=torch.bfloat16, device="cuda")
        if Ca:
            xa = rng.integers(0, 2 ** 32, size=(N, Ca * 4), dtype=np.uint32)
            send_want, expert_want, send_aux_want, expert_aux_want = oracle.dispatch(want, xb, xa)
            ea = torch.zeros((L.P, Ca * 4), dtype=torch.int32, device="cuda")
            sa = torch.zeros((L.send_cap, Ca * 4), dtype=torch.int32, device="cuda")
            fusco.fusco_dispatch(L, bf16_dev(xb), eb, x_aux=dev(xa.view(np.int32)), expert_aux=ea, send_buf=sb,
                                 send_aux=sa, flags=3)
        else:
            send_want, expert_want = oracle.dispatch(want, xb)
            fusco.fusco_dispatch(L, bf16_dev(xb), eb, send_buf=sb, flags=3)
        w = rng.random((N, k)).astype(np.float32)
        out = torch.zeros((N, H), dtype=torch.bfloat16, device="cuda")
        fusco.fusco_combine(L, eb, dev(w), out)
        torch.cuda.synchronize()
        assert np.array_equal(bits_host(eb), expert_want), tag
        assert np.array_equal(bits_host(sb[:want.U]), send_want), tag
        if Ca:
            assert np.array_equal(ea.cpu().numpy().view(np.uint32), expert_aux_want), tag
            assert np.array_equal(sa[:want.U].cpu().numpy().view(np.uint32), send_aux_want), tag
        _, o16 = oracle.combine_f32(expert_want, w, want.pair_slot)
        assert np.array_equal(bits_host(out), o16), tag
        # the expert tensor alone, in transfer order wherever the shape allows it (16 tiles and more)
        eb3 = torch.zeros_like(eb)
        ea3 = torch.zeros_like(ea) if Ca else None
        fusco.fusco_probe_dispatch_kernel(2)
        try:
            seen_tiled += bool(fusco.fusco_dispatch_in_transfer_order(L, H * 2, Ca * 16))
            fusco.fusco_dispatch(L, bf16_dev(xb), eb3, x_aux=dev(xa.view(np.int32)) if Ca else None, expert_aux=ea3)
            torch.cuda.synchronize()
        finally:
            fusco.fusco_probe_dispatch_kernel(0)
        assert torch.equal(eb3, eb) and (not Ca or torch.equal(ea3, ea)), tag
        if N <= 2048 // k:                                      # the single-launch path gives the same
            L2 = fusco.Layout(N, k, E, D)
            eb2 = torch.zeros_like(eb)
            if Ca:
                ea2 = torch.zeros_like(ea)
                fusco.fusco_plan_dispatch(L2, dev(A), bf16_dev(xb), eb2, x_aux=dev(xa.view(np.int32)), expert_aux=ea2)
            else:
                fusco.fusco_plan_dispatch(L2, dev(A), bf16_dev(xb), eb2)
            torch.cuda.synchronize()
            got2 = L2.to_host()
            for f in PLAN_FIELDS:
                assert np.array_equal(getattr(got2, f), getattr(want, f)), (tag, "fused", f)
            assert_tile_order(oracle, L2, got2, want, tag)
            assert torch.equal(eb2, eb), tag
            if Ca:
                assert torch.equal(ea2, ea), tag
    assert seen_chunks == {1, 2, 4}          # one, two and four 16-byte chunks per thread were all exercised
    assert seen_tiled >= 15                  # and the tiled dispatch took its share of the shapes (21 of these 300)


def test_plan_empty_input(fusco, oracle):
    L, got = gpu_plan(fusco, np.zeros((0, 4), dtype=np.int32), 8, 2)
    assert got.exp_off.tolist() == [0] * 9 and got.send_off.tolist() == [0] * 3
    assert got.exp_count.tolist() == [0] * 8 and got.send_count.tolist() == [0] * 2 and int(got.status[0]) == 0


def test_movers_accept_an_empty_layout(fusco):
    L, _ = gpu_plan(fusco, np.zeros((0, 4), dtype=np.int32), 8, 2)
    x = torch.empty((0, 64), dtype=torch.bfloat16, device="cuda")
    eb = torch.empty((0, 64), dtype=torch.bfloat16, device="cuda")
    sb = torch.empty((0, 64), dtype=torch.bfloat16, device="cuda")
    for flags in (0, 2, 3, 4):
        fusco.fusco_dispatch(L, x, eb, send_buf=sb, flags=flags)
    out = torch.empty((0, 64), dtype=torch.bfloat16, device="cuda")
    w = torch.empty((0, 4), dtype=torch.float32, device="cuda")
    fusco.fusco_combine(L, eb, w, out)
    fusco.fusco_combine_two_hop(L, eb, w, torch.empty((0, 64), dtype=torch.float32, device="cuda"), out)
    torch.cuda.synchronize()
    with pytest.raises(fusco.FuscoError):
        fusco.fusco_dispatch(L, torch.empty((0, 24), dtype=torch.uint8, device="cuda"), eb)   # row size still checked


def test_plan_skewed_all_to_one_expert(fusco, oracle):
    A = np.zeros((5000, 1), dtype=np.int32) + 3
    L, got = gpu_plan(fusco, A, 8, 4)
    assert_plan_equal(got, oracle.plan(A, 8, 4))


@pytest.mark.parametrize("name,n", [("tiny", 4096), ("dsv3", 8192), ("qwen3", 16384), ("skewed", 32768),
                                    ("decode_fp8", 128)])
def test_plan_on_full_configs(fusco, oracle, name, n):
    cfg = W.get_config(name).with_tokens(n)
    A, _ = W.make_routing(cfg)
    L, got = gpu_plan(fusco, A, cfg.E, cfg.D)
    want = oracle.plan(A, cfg.E, cfg.D)
    assert_plan_equal(got, want)
    assert_tile_order(oracle, L, got, want)
    check_plan_invariants(got, A)


def test_plan_is_deterministic(fusco):
    cfg = W.get_config("dsv3").with_tokens(3000)
    A, _ = W.make_routing(cfg)
    L, first = gpu_plan(fusco, A, cfg.E, cfg.D)
    ref = L.mem.clone()
    At = dev(A)
    for _ in range(20):
        fusco.fusco_plan(L, At)
        torch.cuda.synchronize()
        assert torch.equal(L.mem, ref)


def test_movers_are_deterministic(fusco):
    """Dispatch and combine (flat and along the two levels) give the same bytes on each of 20 runs: neither uses
    atomics, every output element has one writer and a fixed order of operations."""
    cfg = W.get_config("dsv3").with_tokens(2000)
    A, w = W.make_routing(cfg)
    x = bf16_dev(W.make_activations(cfg))
    L, _ = gpu_plan(fusco, A, cfg.E, cfg.D)
    d_w = dev(w)
    eb = torch.empty((cfg.P, cfg.H), dtype=torch.bfloat16, device="cuda")
    sb = torch.empty((L.send_cap, cfg.H), dtype=torch.bfloat16, device="cuda")
    out = torch.empty((cfg.N, cfg.H), dtype=torch.bfloat16, device="cuda")
    out2 = torch.empty((cfg.N, cfg.H), dtype=torch.float32, device="cuda")
    part = torch.zeros((L.send_cap, cfg.H), dtype=torch.float32, device="cuda")
    U = int(L.array("send_off")[cfg.D].item())
    ref = None
    for _ in range(20):
        eb.fill_(0); sb.fill_(0); out.fill_(0); out2.fill_(0)
        fusco.fusco_dispatch(L, x, eb, send_buf=sb, flags=3)
        fusco.fusco_combine(L, eb, d_w, out)
        fusco.fusco_combine_two_hop(L, eb, d_w, part, out2)
        torch.cuda.synchronize()
        got = (eb.clone(), sb[:U].clone(), out.clone(), out2.clone(), part[:U].clone())
        if ref is None:
            ref = got
        else:
            assert all(torch.equal(a.view(torch.uint8), b.view(torch.uint8)) for a, b in zip(got, ref))


@pytest.mark.parametrize("N", [700, 30000, 150000])          # 2 tiles; 59 tiles read one by one; 293 tiles in chunks
def test_plan_counts_invalid_ids(fusco, oracle, N):
    rng = np.random.default_rng(77)
    k, E, D = 4, 32, 4
    A = random_topk(rng, N, k, E)
    bad = rng.choice(N * k, size=9, replace=False)
    Ab = A.copy().reshape(-1)
    Ab[bad[:5]] = E + 3
    Ab[bad[5:]] = -2
    Ab = Ab.reshape(N, k)
    L, got = gpu_plan(fusco, Ab, E, D)
    assert int(got.status[0]) == 9
    assert np.all(got.pair_slot[bad] == -1) and np.all(got.pair_send_row[bad] == -1)
    assert np.all(got.pair_first[bad] == 0)
    ok = np.ones(N * k, dtype=bool)
    ok[bad] = False
    assert int(got.exp_count.sum()) == N * k - 9
    # valid pairs still form a stable expert-major order among themselves
    order = np.argsort(Ab.reshape(-1)[ok], kind="stable")
    assert np.array_equal(got.slot_pair[:N * k - 9], np.flatnonzero(ok)[order])
    # the transfer order lists the valid pairs' rows only (expected slots built here from the stable order above)
    slot_of = np.full(N * k, -1, dtype=np.int32)
    slot_of[np.flatnonzero(ok)[order]] = np.arange(N * k - 9, dtype=np.int32)
    assert np.array_equal(got.tile_slots, oracle.tile_order(slot_of, N, k, L.tile_tokens))
    # the movers skip invalid pairs instead of faulting
    x = bf16_dev(W.bf16_bits(rng.standard_normal((N, 64)).astype(np.float32)))
    eb = torch.zeros((N * k, 64), dtype=torch.bfloat16, device="cuda")
    fusco.fusco_dispatch(L, x, eb)
    out = torch.empty((N, 64), dtype=torch.bfloat16, device="cuda")
    fusco.fusco_combine(L, eb, torch.full((N, k), 0.25, device="cuda"), out)
    torch.cuda.synchronize()
    # and a later valid plan on the same layout clears the status word
    fusco.fusco_plan(L, dev(A))
    torch.cuda.synchronize()
    assert_plan_equal(L.to_host(), oracle.plan(A, E, D))


DISPATCH_SHAPES = [
    # N, k, E, D, row_bytes
    (33, 2, 8, 4, 16), (100, 4, 16, 4, 48), (257, 8, 64, 8, 2048), (300, 8, 256, 8, 14336),
    (513, 2, 16, 4, 16 * 37), (64, 3, 6, 3, 16 * 129), (40, 8, 32, 32, 16 * 1025), (1, 1, 1, 1, 4096),
    (5, 2, 4, 2, 1 << 20),         # the largest row the movers take (1 MiB)
    (7, 3, 6, 3, (1 << 20) - 16),
]


@pytest.mark.parametrize("N,k,E,D,row_bytes", DISPATCH_SHAPES)
@pytest.mark.parametrize("flags", [0, 2, 3, 8, 8 + 2, 8 + 3])      # 8: the same rows written with streaming stores
def test_dispatch_matches_oracle(fusco, oracle, N, k, E, D, row_bytes, flags):
    streaming, flags = flags & 8, flags & 7
    rng = np.random.default_rng(N + row_bytes)
    A = random_topk(rng, N, k, E)
    x = rng.integers(0, 256, size=(N, row_bytes), dtype=np.uint8)
    want = oracle.plan(A, E, D)
    send_want, expert_want = oracle.dispatch(want, x)
    L, got = gpu_plan(fusco, A, E, D)
    eb = torch.full((L.P, row_bytes), 0xEE, dtype=torch.uint8, device="cuda")
    sb = torch.full((L.send_cap, row_bytes), 0xEE, dtype=torch.uint8, device="cuda")
    fusco.fusco_dispatch(L, dev(x), eb if flags != 2 else None, send_buf=sb if flags & 2 else None,
                         flags=flags | streaming)
    torch.cuda.synchronize()
    if flags != 2:
        assert np.array_equal(eb.cpu().numpy(), expert_want)
    else:
        assert bool((eb == 0xEE).all())
    if flags & 2:
        assert np.array_equal(sb[:want.U].cpu().numpy(), send_want)
        assert bool((sb[want.U:] == 0xEE).all())       # rows past U stay untouched
        if flags == 3:   # two-level identity: the expert tensor is the send tensor expanded by the dedup map
            assert torch.equal(sb[dev(want.slot_send_row).long()], eb)
    else:
        assert bool((sb == 0xEE).all())


@pytest.mark.parametrize("N,k,E,D,H", [(128, 8, 256, 64, 7168), (77, 4, 16, 8, 256)])
def test_dispatch_with_aux_plane(fusco, oracle, N, k, E, D, H):
    rng = np.random.default_rng(H)
    A = random_topk(rng, N, k, E)
    q = rng.integers(0, 256, size=(N, H), dtype=np.uint8)
    sc = rng.standard_normal((N, H // 128 if H >= 512 else 4)).astype(np.float32)
    want = oracle.plan(A, E, D)
    send_want, expert_want, saux_want, eaux_want = oracle.dispatch(want, q, sc)
    L, _ = gpu_plan(fusco, A, E, D)
    eb = torch.zeros((L.P, H), dtype=torch.uint8, device="cuda")
    ea = torch.zeros((L.P, sc.shape[1]), dtype=torch.float32, device="cuda")
    sb = torch.zeros((L.send_cap, H), dtype=torch.uint8, device="cuda")
    sa = torch.zeros((L.send_cap, sc.shape[1]), dtype=torch.float32, device="cuda")
    fusco.fusco_dispatch(L, dev(q), eb, x_aux=dev(sc), expert_aux=ea, send_buf=sb, send_aux=sa, flags=3)
    torch.cuda.synchronize()
    assert np.array_equal(eb.cpu().numpy(), expert_want) and np.array_equal(ea.cpu().numpy(), eaux_want)
    assert np.array_equal(sb[:want.U].cpu().numpy(), send_want)
    assert np.array_equal(sa[:want.U].cpu().numpy(), saux_want)


def _combine_case(fusco, oracle, A, E, D, y_bits_or_f32, w, out_dtype):
    N, k = A.shape
    L, _ = gpu_plan(fusco, A, E, D)
    want_plan = oracle.plan(A, E, D)
    if y_bits_or_f32.dtype == np.uint16:
        y = bf16_dev(y_bits_or_f32)
    else:
        y = dev(y_bits_or_f32)
    H = y.shape[1]
    out = torch.full((N, H), float("nan"), dtype=out_dtype, device="cuda")
    fusco.fusco_combine(L, y, dev(w), out)
    torch.cuda.synchronize()
    o32, o16 = oracle.combine_f32(y_bits_or_f32, w, want_plan.pair_slot)
    if out_dtype == torch.float32:
        got = out.cpu().numpy()
        assert np.array_equal(got.view(np.uint32), o32.view(np.uint32))
        ref = oracle.combine_f64(y_bits_or_f32, w, want_plan.pair_slot)
        scale = oracle.combine_abs_f64(y_bits_or_f32, w, want_plan.pair_slot)
        assert np.all(np.abs(got.astype(np.float64) - ref) <= REL_TOL * scale)
    else:
        assert np.array_equal(bits_host(out), o16)


COMBINE_SHAPES = [
    # N, k, E, D, H
    (50, 2, 8, 4, 8), (129, 8, 64, 8, 1024), (300, 8, 256, 8, 7168), (65, 4, 16, 4, 8 * 37),
    (40, 1, 4, 2, 512), (33, 9, 18, 6, 8 * 129), (20, 17, 34, 2, 2056), (10, 64, 128, 8, 4096),
    (3, 2, 4, 2, 1 << 19),         # the largest row (1 MiB of bf16)
    (4, 3, 6, 2, 8 * 8191 + 8),
    (70, 8, 32, 4, 8 * 1285),      # 1285 chunks: two column segments of 643 and 642
]


@pytest.mark.parametrize("N,k,E,D,H", COMBINE_SHAPES)
@pytest.mark.parametrize("out_dtype", [torch.bfloat16, torch.float32])
def test_combine_bf16_input_matches_oracle(fusco, oracle, N, k, E, D, H, out_dtype):
    rng = np.random.default_rng(N * H + k)
    A = random_topk(rng, N, k, E)
    y = W.bf16_bits(rng.standard_normal((N * k, H)).astype(np.float32))
    w = rng.random((N, k)).astype(np.float32)
    w /= w.sum(1, keepdims=True)
    _combine_case(fusco, oracle, A, E, D, y, w, out_dtype)


@pytest.mark.parametrize("N,k,E,D,H", [(70, 8, 32, 4, 1024), (31, 3, 6, 3, 4 * 37), (16, 2, 4, 2, 4)])
@pytest.mark.parametrize("out_dtype", [torch.bfloat16, torch.float32])
def test_combine_f32_input_matches_oracle(fusco, oracle, N, k, E, D, H, out_dtype):
    rng = np.random.default_rng(N * H + k + 1)
    A = random_topk(rng, N, k, E)
    y = rng.standard_normal((N * k, H)).astype(np.float32)
    w = (rng.standard_normal((N, k)) * 3).astype(np.float32)     # mixed signs: cancellation
    _combine_case(fusco, oracle, A, E, D, y, w, out_dtype)


# inputs of 64 MiB and more take the token's rows two at a time instead of all at once: odd k, a k that is not a
# multiple of the group, the largest k, two column segments, fp32 input
COMBINE_SHAPES_TWO_ROWS_IN_FLIGHT = [
    # N, k, E, D, H, y is fp32
    (3000, 5, 20, 4, 2304, False), (6000, 3, 6, 3, 2304, False), (600, 64, 128, 8, 1024, False),
    (1200, 8, 32, 4, 8 * 1285, False), (2500, 7, 14, 2, 1024, True), (9000, 1, 4, 2, 4096, False),
]


@pytest.mark.parametrize("N,k,E,D,H,y_f32", COMBINE_SHAPES_TWO_ROWS_IN_FLIGHT)
@pytest.mark.parametrize("out_dtype", [torch.bfloat16, torch.float32])
def test_combine_of_memory_bound_sizes_matches_oracle(fusco, oracle, N, k, E, D, H, y_f32, out_dtype):
    assert N * k * H * (4 if y_f32 else 2) >= 64 << 20
    rng = np.random.default_rng(N * H + k + 2)
    A = random_topk(rng, N, k, E)
    y = rng.standard_normal((N * k, H)).astype(np.float32)
    if not y_f32:
        y = W.bf16_bits(y)
    w = (rng.standard_normal((N, k)) * 2).astype(np.float32)
    _combine_case(fusco, oracle, A, E, D, y, w, out_dtype)


@pytest.mark.parametrize("out_dtype", [torch.bfloat16, torch.float32])
def test_combine_special_values(fusco, oracle, out_dtype):
    """Zeros of both signs, subnormals, the largest finite values, infinities and NaNs in y, and weights that
    overflow, underflow and cancel: every finite or infinite result is bit-identical to the oracle's fp32 chain;
    where the result is a NaN both sides give a NaN (IEEE 754 fixes neither its sign nor its payload)."""
    rng = np.random.default_rng(99)
    N, k, E, D, H = 257, 8, 32, 4, 256
    A = random_topk(rng, N, k, E)
    special = np.array([0x0000, 0x8000, 0x0001, 0x8001, 0x007F, 0x807F, 0x0080, 0x8080, 0x7F7F, 0xFF7F, 0x7F80,
                        0xFF80, 0x7FC0, 0xFFC1, 0x3F80, 0xBF80, 0x3F81, 0x3F7F, 0x4049, 0x0300], dtype=np.uint16)
    y = W.bf16_bits(rng.standard_normal((N * k, H)).astype(np.float32))
    pick = rng.random((N * k, H)) < 0.3
    y[pick] = special[rng.integers(0, len(special), size=int(pick.sum()))]
    wv = np.array([0.0, -0.0, 1.0, -1.0, 0.5, 1e-30, -1e-38, 1e30, 3.0e38, 1.0 / 3.0], dtype=np.float32)
    w = wv[rng.integers(0, len(wv), size=(N, k))]
    w[:40] = rng.random((40, k)).astype(np.float32)          # ordinary weights on special rows too
    L, _ = gpu_plan(fusco, A, E, D)
    want = oracle.plan(A, E, D)
    out = torch.zeros((N, H), dtype=out_dtype, device="cuda")
    fusco.fusco_combine(L, bf16_dev(y), dev(w), out)
    torch.cuda.synchronize()
    o32, o16 = oracle.combine_f32(y, w, want.pair_slot)
    nan = np.isnan(o32)
    assert nan.any() and np.isinf(o32).any() and (np.abs(o32[~nan]) < 1e-38).any()     # the cases are there
    if out_dtype == torch.float32:
        got = out.cpu().numpy()
        assert np.array_equal(np.isnan(got), nan)
        assert np.array_equal(got.view(np.uint32)[~nan], o32.view(np.uint32)[~nan])
    else:
        got = bits_host(out)
        got_nan = (got & 0x7FFF) > 0x7F80
        assert np.array_equal(got_nan, nan)
        assert np.array_equal(got[~nan], o16[~nan])


@pytest.mark.parametrize("k", [1, 2, 4, 8])
def test_dispatch_identity_combine_returns_input_exactly(fusco, k):
    # w = 1/k is dyadic: dispatch -> identity experts -> combine reproduces x bit for bit
    rng = np.random.default_rng(k)
    N, E, D, H = 600, 64, 8, 2048
    A = random_topk(rng, N, k, E)
    xb = W.bf16_bits(rng.standard_normal((N, H)).astype(np.float32))
    L, _ = gpu_plan(fusco, A, E, D)
    x = bf16_dev(xb)
    eb = torch.empty((L.P, H), dtype=torch.bfloat16, device="cuda")
    out = torch.empty((N, H), dtype=torch.bfloat16, device="cuda")
    fusco.fusco_dispatch(L, x, eb)
    fusco.fusco_combine(L, eb, torch.full((N, k), 1.0 / k, device="cuda"), out)
    torch.cuda.synchronize()
    assert np.array_equal(bits_host(out), xb)


@pytest.mark.parametrize("name,n", [("tiny", 1500), ("dsv3", 700), ("qwen3", 900), ("skewed", 800)])
def test_whole_path_on_configs_reduced(fusco, oracle, name, n):
    """plan -> dispatch -> combine at the configurations' real row sizes, a few planner tiles."""
    cfg = W.get_config(name).with_tokens(n)
    A, w = W.make_routing(cfg)
    xb = W.make_activations(cfg)
    want = oracle.plan(A, cfg.E, cfg.D)
    send_want, expert_want = oracle.dispatch(want, xb)
    L, got = gpu_plan(fusco, A, cfg.E, cfg.D)
    assert_plan_equal(got, want)
    eb = torch.empty((L.P, cfg.H), dtype=torch.bfloat16, device="cuda")
    sb = torch.empty((L.send_cap, cfg.H), dtype=torch.bfloat16, device="cuda")
    fusco.fusco_dispatch(L, bf16_dev(xb), eb, send_buf=sb, flags=3)
    torch.cuda.synchronize()
    assert np.array_equal(bits_host(eb), expert_want)
    assert np.array_equal(bits_host(sb[:want.U]), send_want)
    yb = W.make_expert_output(cfg)
    for out_dtype in (torch.bfloat16, torch.float32):
        _combine_case(fusco, oracle, A, cfg.E, cfg.D, yb, w, out_dtype)


def test_decode_fp8_config(fusco, oracle):
    cfg = W.get_config("decode_fp8")
    A, w = W.make_routing(cfg)
    q, sc = W.make_fp8_activations(cfg)
    want = oracle.plan(A, cfg.E, cfg.D)
    send_want, expert_want, saux_want, eaux_want = oracle.dispatch(want, q, sc)
    L, got = gpu_plan(fusco, A, cfg.E, cfg.D)
    assert_plan_equal(got, want)
    eb = torch.zeros((L.P, cfg.H), dtype=torch.uint8, device="cuda")
    ea = torch.zeros((L.P, cfg.H // 128), dtype=torch.float32, device="cuda")
    sb = torch.zeros((L.send_cap, cfg.H), dtype=torch.uint8, device="cuda")
    sa = torch.zeros((L.send_cap, cfg.H // 128), dtype=torch.float32, device="cuda")
    fusco.fusco_dispatch(L, dev(q), eb, x_aux=dev(sc), expert_aux=ea, send_buf=sb, send_aux=sa, flags=3)
    torch.cuda.synchronize()
    assert np.array_equal(eb.cpu().numpy(), expert_want) and np.array_equal(ea.cpu().numpy(), eaux_want)
    assert np.array_equal(sb[:want.U].cpu().numpy(), send_want) and np.array_equal(sa[:want.U].cpu().numpy(), saux_want)
    yb = W.make_expert_output(cfg)
    _combine_case(fusco, oracle, A, cfg.E, cfg.D, yb, w, torch.bfloat16)
    _combine_case(fusco, oracle, A, cfg.E, cfg.D, yb, w, torch.float32)


FUSED_SHAPES = [
    # N, k, E, D, row_bytes, aux_row_bytes, distinct       (one planner tile: N <= 2048 // k)
    (1, 1, 1, 1, 16, 0, True), (128, 8, 256, 64, 7168, 224, True), (128, 8, 256, 8, 14336, 0, True),
    (1024, 1, 8, 4, 48, 16, True), (16, 64, 1024, 64, 4096, 0, True), (31, 33, 66, 2, 16 * 129, 0, True),
    (100, 5, 10, 5, 16 * 37, 0, False),                       # repeated experts inside a token
    (3, 2, 4, 2, 16 * 5000, 16 * 9, True),                    # row longer than the part held in registers
    (2, 2, 4, 2, 1 << 20, 0, True),                           # the largest row
    # tiles of 2048 pairs
    (129, 8, 256, 8, 2048, 0, True), (256, 8, 256, 64, 7168, 224, True), (2048, 1, 16, 4, 32, 0, True),
    (32, 64, 1024, 64, 1024, 16, True), (62, 33, 66, 2, 16 * 7, 0, True), (400, 5, 10, 5, 64, 0, False),
]


@pytest.mark.parametrize("N,k,E,D,row_bytes,aux_bytes,distinct", FUSED_SHAPES)
def test_fused_plan_dispatch_matches_oracle(fusco, oracle, N, k, E, D, row_bytes, aux_bytes, distinct):
    rng = np.random.default_rng(N * 7 + k + row_bytes)
    A = random_topk(rng, N, k, E, distinct)
    x = rng.integers(0, 256, size=(N, row_bytes), dtype=np.uint8)
    xa = rng.integers(0, 256, size=(N, aux_bytes), dtype=np.uint8) if aux_bytes else None
    want = oracle.plan(A, E, D)
    L = fusco.Layout(N, k, E, D)
    L.mem.fill_(0x7B)
    eb = torch.full((L.P, row_bytes), 0xEE, dtype=torch.uint8, device="cuda")
    ea = torch.full((L.P, aux_bytes), 0xEE, dtype=torch.uint8, device="cuda") if aux_bytes else None
    fusco.fusco_plan_dispatch(L, dev(A), dev(x), eb, x_aux=dev(xa) if aux_bytes else None, expert_aux=ea)
    torch.cuda.synchronize()
    assert_plan_equal(L.to_host(), want)
    if aux_bytes:
        _, expert_want, _, eaux_want = oracle.dispatch(want, x, xa)
        assert np.array_equal(ea.cpu().numpy(), eaux_want)
    else:
        _, expert_want = oracle.dispatch(want, x)
    assert np.array_equal(eb.cpu().numpy(), expert_want)


def test_fused_plan_dispatch_edge_cases(fusco, oracle):
    # empty input: the plan of nothing is still written
    L = fusco.Layout(0, 4, 8, 2)
    L.mem.fill_(0x7B)
    fusco.fusco_plan_dispatch(L, torch.empty((0, 4), dtype=torch.int32, device="cuda"),
                              torch.empty((0, 64), dtype=torch.uint8, device="cuda"),
                              torch.empty((0, 64), dtype=torch.uint8, device="cuda"))
    torch.cuda.synchronize()
    got = L.to_host()
    assert got.exp_off.tolist() == [0] * 9 and got.send_off.tolist() == [0] * 3 and int(got.status[0]) == 0
    # invalid ids are counted and their rows skipped, as by the two separate calls
    rng = np.random.default_rng(3)
    N, k, E, D = 60, 4, 32, 4
    A = random_topk(rng, N, k, E).reshape(-1)
    A[[5, 77, 200]] = [E, -1, 1000]
    A = A.reshape(N, k)
    x = rng.integers(0, 256, size=(N, 256), dtype=np.uint8)
    L1, L2 = fusco.Layout(N, k, E, D), fusco.Layout(N, k, E, D)
    L1.mem.fill_(0x7B)          # same stale bytes wherever neither path writes (unassigned slots, rows past U)
    L2.mem.fill_(0x7B)
    e1 = torch.full((N * k, 256), 0xEE, dtype=torch.uint8, device="cuda")
    e2 = torch.full((N * k, 256), 0xEE, dtype=torch.uint8, device="cuda")
    fusco.fusco_plan_dispatch(L1, dev(A), dev(x), e1)
    fusco.fusco_plan(L2, dev(A))
    fusco.fusco_dispatch(L2, dev(x), e2)
    torch.cuda.synchronize()
    assert int(L1.array("status").item()) == 3
    assert torch.equal(L1.mem, L2.mem) and torch.equal(e1, e2)
    # more than 2048 pairs: refused, nothing launched
    Lb = fusco.Layout(257, 8, 256, 8)
    with pytest.raises(fusco.FuscoError):
        fusco.fusco_plan_dispatch(Lb, torch.zeros((257, 8), dtype=torch.int32, device="cuda"),
                                  torch.zeros((257, 64), dtype=torch.uint8, device="cuda"),
                                  torch.zeros((257 * 8, 64), dtype=torch.uint8, device="cuda"))


def test_binding_rejects_wrong_shapes(fusco):
    L = fusco.Layout(16, 2, 4, 2)
    x = torch.zeros((16, 64), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(fusco.FuscoError):
        fusco.fusco_dispatch(L, x, torch.zeros((31, 64), dtype=torch.bfloat16, device="cuda"))
    with pytest.raises(fusco.FuscoError):
        fusco.fusco_dispatch(L, x[:8], torch.zeros((32, 64), dtype=torch.bfloat16, device="cuda"))
    with pytest.raises(fusco.FuscoError):
        fusco.fusco_plan(L, torch.zeros((16, 3), dtype=torch.int32, device="cuda"))
    with pytest.raises(fusco.FuscoError):
        fusco.fusco_combine(L, torch.zeros((32, 64), dtype=torch.bfloat16, device="cuda"),
                            torch.zeros((16, 2), device="cuda"), torch.zeros((16, 32), dtype=torch.bfloat16, device="cuda"))
    with pytest.raises(fusco.FuscoError):
        fusco.Layout(16, 2, 4, 3)


@pytest.fixture
def transfer_order_everywhere(fusco):
    """The tests of the tiled dispatch run it on small inputs, where fusco_dispatch would walk the tokens: the study
    knob takes the transfer order wherever its workgroup shape allows."""
    assert fusco.fusco_probe_dispatch_kernel(2) == 0
    yield
    assert fusco.fusco_probe_dispatch_kernel(0) == 2


TILED_SHAPES = [
    # N, k, E, D, row_bytes, aux_row_bytes, distinct: inputs of at least 16 tiles of 2048 pairs whose tile of source
    # rows fits an XCD's L2, so that dispatch moves the rows in transfer order
    (4100, 8, 64, 8, 2048, 0, True),          # 17 tiles, the last one ragged; one XCD gets three tiles, the others two
    (3000, 16, 128, 16, 20480, 0, True),      # rows longer than one workgroup column (1280 chunks): two columns
    (20000, 2, 16, 4, 48, 16, True),          # tiny rows and a second plane, 1024 tokens per tile
    (1100, 64, 1024, 64, 512, 0, True),       # 35 tiles of 32 tokens, largest k
    (5000, 8, 256, 8, 14336, 224, True),      # the benchmark's rows plus a plane of scales: 3.7 MB of source per tile
    (6000, 6, 10, 5, 256, 0, False),          # repeated experts inside a token
    (8192, 8, 256, 8, 4096, 0, True),         # exactly 32 full tiles
    # rows of 4 KiB and more that are not multiples of 4 KiB
    (4100, 8, 32, 8, 6144, 0, True),          # one and a half pieces per row, long runs (32 experts)
    (4200, 8, 256, 8, 5008, 48, True),        # an odd number of 16-byte units per row, short runs, a second plane
    (2100, 16, 64, 8, 18448, 0, True),        # 1153 units: two workgroup columns; 128 tokens per tile
    (1100, 32, 64, 8, 28688, 16, True),       # 1794 chunks with the second plane: two segments; 64 tokens per tile
    (6000, 6, 10, 5, 4112, 0, False),         # repeated experts inside a token: neighbouring slots from one token
    # rows that are moved in column segments (the source rows of a tile would not fit the L2 whole)
    (4200, 8, 64, 8, 16384, 0, True),         # two segments of 8 KiB
    (4200, 8, 64, 8, 20496, 64, True),        # two uneven planes over two segments: 1285 chunks
    (8300, 4, 32, 8, 14336, 0, True),         # 512 tokens per tile: two segments of 7 KiB
    (2100, 16, 64, 8, 30736, 0, True),        # 128 tokens per tile: two segments of 1024 and 897 chunks
    (1100, 32, 64, 8, 41008, 16, True),       # 64 tokens per tile: three segments
    (2100, 16, 64, 8, 65536 + 48, 0, True),   # five segments of 832 chunks, the last one shorter
]


@pytest.mark.parametrize("N,k,E,D,row_bytes,aux_bytes,distinct", TILED_SHAPES)
def test_dispatch_in_transfer_order_matches_oracle(fusco, oracle, transfer_order_everywhere, N, k, E, D, row_bytes, aux_bytes,
                                                   distinct):
    rng = np.random.default_rng(N + row_bytes)
    A = random_topk(rng, N, k, E, distinct)
    x = rng.integers(0, 256, size=(N, row_bytes), dtype=np.uint8)
    xa = rng.integers(0, 256, size=(N, aux_bytes), dtype=np.uint8) if aux_bytes else None
    want = oracle.plan(A, E, D)
    L, got = gpu_plan(fusco, A, E, D)
    assert_plan_equal(got, want)
    assert_tile_order(oracle, L, got, want)
    assert fusco.fusco_dispatch_in_transfer_order(L, row_bytes, aux_bytes)           # the path under test
    assert not fusco.fusco_dispatch_in_transfer_order(L, row_bytes, aux_bytes, 3)    # with the wire tensor: token walk
    eb = torch.full((L.P, row_bytes), 0xEE, dtype=torch.uint8, device="cuda")
    ea = torch.full((L.P, aux_bytes), 0xEE, dtype=torch.uint8, device="cuda") if aux_bytes else None
    fusco.fusco_dispatch(L, dev(x), eb, x_aux=dev(xa) if aux_bytes else None, expert_aux=ea)
    torch.cuda.synchronize()
    if aux_bytes:
        _, expert_want, _, eaux_want = oracle.dispatch(want, x, xa)
        assert np.array_equal(ea.cpu().numpy(), eaux_want)
    else:
        _, expert_want = oracle.dispatch(want, x)
    assert np.array_equal(eb.cpu().numpy(), expert_want)
    # the token walk (chosen here by asking for the wire tensor as well) writes the same expert tensor
    eb2 = torch.full_like(eb, 0x11)
    sb = torch.empty((L.send_cap, row_bytes), dtype=torch.uint8, device="cuda")
    sa = torch.empty((L.send_cap, aux_bytes), dtype=torch.uint8, device="cuda") if aux_bytes else None
    ea2 = torch.full_like(ea, 0x11) if aux_bytes else None
    fusco.fusco_dispatch(L, dev(x), eb2, x_aux=dev(xa) if aux_bytes else None, expert_aux=ea2, send_buf=sb, send_aux=sa,
                         flags=3)
    torch.cuda.synchronize()
    assert torch.equal(eb2, eb) and (not aux_bytes or torch.equal(ea2, ea))


@pytest.mark.parametrize("chunk_tiles", [8, 16])
@pytest.mark.parametrize("N,k,E,D,row_bytes,aux_bytes,distinct", TILED_SHAPES)
def test_dispatch_in_source_chunks_matches_oracle(fusco, oracle, transfer_order_everywhere, chunk_tiles, N, k, E, D, row_bytes,
                                                  aux_bytes, distinct):
    """Source tensors larger than the memory-side cache are moved in chunks of tiles, every chunk starting with a read
    of its source rows.  The chunk size is lowered here so that small inputs take that path: 8 tiles (the smallest,
    a last chunk with fewer tiles than XCDs for the 17- and 35-tile inputs) and 16 tiles."""
    rng = np.random.default_rng(N + row_bytes + chunk_tiles)
    A = random_topk(rng, N, k, E, distinct)
    x = rng.integers(0, 256, size=(N, row_bytes), dtype=np.uint8)
    xa = rng.integers(0, 256, size=(N, aux_bytes), dtype=np.uint8) if aux_bytes else None
    want = oracle.plan(A, E, D)
    L, got = gpu_plan(fusco, A, E, D)
    assert fusco.fusco_dispatch_in_transfer_order(L, row_bytes, aux_bytes)
    eb = torch.full((L.P, row_bytes), 0xEE, dtype=torch.uint8, device="cuda")
    ea = torch.full((L.P, aux_bytes), 0xEE, dtype=torch.uint8, device="cuda") if aux_bytes else None
    limit = chunk_tiles * L.tile_tokens * (row_bytes + aux_bytes)
    assert N * (row_bytes + aux_bytes) > limit                      # several chunks
    before = fusco.fusco_probe_source_chunk_bytes(limit)
    try:
        assert fusco.fusco_probe_source_chunk_bytes() == limit
        fusco.fusco_dispatch(L, dev(x), eb, x_aux=dev(xa) if aux_bytes else None, expert_aux=ea)
        torch.cuda.synchronize()
    finally:
        fusco.fusco_probe_source_chunk_bytes(before)
    assert fusco.fusco_probe_source_chunk_bytes() == before == 128 << 20
    if aux_bytes:
        _, expert_want, _, eaux_want = oracle.dispatch(want, x, xa)
        assert np.array_equal(ea.cpu().numpy(), eaux_want)
    else:
        _, expert_want = oracle.dispatch(want, x)
    assert np.array_equal(eb.cpu().numpy(), expert_want)


@pytest.mark.parametrize("N,k,E,D,row_bytes,aux_bytes,distinct", [TILED_SHAPES[i] for i in (0, 4, 13, 16)])
def test_tiled_dispatch_study_knobs_do_not_change_the_result(fusco, oracle, transfer_order_everywhere, N, k, E, D, row_bytes,
                                                             aux_bytes, distinct):
    """Workgroups per compute unit (a launch with unused dynamic LDS) and the pull of a tile's source rows at the start
    of the tile are choices of speed: every setting gives the oracle's expert tensor.  Shapes: a ragged last tile, a
    second plane, two and three column segments."""
    rng = np.random.default_rng(N + row_bytes + 7)
    A = random_topk(rng, N, k, E, distinct)
    x = rng.integers(0, 256, size=(N, row_bytes), dtype=np.uint8)
    xa = rng.integers(0, 256, size=(N, aux_bytes), dtype=np.uint8) if aux_bytes else None
    want = oracle.plan(A, E, D)
    L, _ = gpu_plan(fusco, A, E, D)
    assert fusco.fusco_dispatch_in_transfer_order(L, row_bytes, aux_bytes)
    if aux_bytes:
        _, expert_want, _, eaux_want = oracle.dispatch(want, x, xa)
    else:
        _, expert_want = oracle.dispatch(want, x)
    assert fusco.fusco_probe_dispatch_occupancy() == 0 and fusco.fusco_probe_dispatch_pull() == 0
    try:
        for occupancy in (3, 5, 7, 12, 16):
            for pull in (1, 2):
                fusco.fusco_probe_dispatch_occupancy(occupancy)
                fusco.fusco_probe_dispatch_pull(pull)
                eb = torch.full((L.P, row_bytes), 0xEE, dtype=torch.uint8, device="cuda")
                ea = torch.full((L.P, aux_bytes), 0xEE, dtype=torch.uint8, device="cuda") if aux_bytes else None
                fusco.fusco_dispatch(L, dev(x), eb, x_aux=dev(xa) if aux_bytes else None, expert_aux=ea)
                torch.cuda.synchronize()
                assert np.array_equal(eb.cpu().numpy(), expert_want), (occupancy, pull)
                assert not aux_bytes or np.array_equal(ea.cpu().numpy(), eaux_want), (occupancy, pull)
    finally:
        fusco.fusco_probe_dispatch_occupancy(0)
        fusco.fusco_probe_dispatch_pull(0)
    with pytest.raises(fusco.FuscoError):
        fusco.fusco_probe_dispatch_occupancy(2)
    with pytest.raises(fusco.FuscoError):
        fusco.fusco_probe_dispatch_pull(3)
    assert fusco.fusco_probe_dispatch_occupancy() == 0 and fusco.fusco_probe_dispatch_pull() == 0


def test_dispatch_in_transfer_order_skips_invalid_ids(fusco, oracle, transfer_order_everywhere):
    rng = np.random.default_rng(5)
    N, k, E, D, row_bytes = 5000, 8, 64, 8, 1024
    A = random_topk(rng, N, k, E).reshape(-1)
    bad = rng.choice(N * k, size=40, replace=False)
    A[bad[:20]] = E
    A[bad[20:]] = -5
    A = A.reshape(N, k)
    L, got = gpu_plan(fusco, A, E, D)
    assert int(got.status[0]) == 40 and fusco.fusco_dispatch_in_transfer_order(L, row_bytes)
    x = rng.integers(0, 256, size=(N, row_bytes), dtype=np.uint8)
    eb = torch.full((L.P, row_bytes), 0xEE, dtype=torch.uint8, device="cuda")
    fusco.fusco_dispatch(L, dev(x), eb)
    torch.cuda.synchronize()
    ebh = eb.cpu().numpy()
    ok = np.ones(N * k, dtype=bool)
    ok[bad] = False
    order = np.flatnonzero(ok)[np.argsort(A.reshape(-1)[ok], kind="stable")]      # pairs in expert-major order
    assert np.array_equal(ebh[:len(order)], x[order // k])
    assert np.all(ebh[len(order):] == 0xEE)                                      # rows nobody owns stay untouched


def test_dispatch_chooses_the_token_walk_where_the_transfer_order_does_not_pay(fusco):
    tiled = fusco.fusco_dispatch_in_transfer_order
    small = fusco.Layout(1000, 8, 64, 8)             # 4 tiles: too few for the eight XCDs
    many = fusco.Layout(8192, 8, 256, 8)             # 32 tiles of 256 tokens
    top1 = fusco.Layout(65536, 1, 64, 8)             # k = 1: a row is used once, nothing to keep in the L2
    wide = fusco.Layout(40000, 2, 64, 8)             # 1024 tokens per tile: a segment may hold 3840 B of a row
    long = fusco.Layout(65536, 8, 256, 8)
    # sizes: an expert tensor that fits the memory-side cache is left to the token walk, and so are rows shorter
    # than 8 KiB when the source tensor has 128 MiB or more
    assert tiled(many, 14336) and tiled(many, 14336, 224) and tiled(many, 4112)
    assert not tiled(many, 4096) and not tiled(many, 2048)              # 256 MiB and 128 MiB of expert rows
    assert tiled(long, 2032) and not tiled(long, 2048) and not tiled(long, 4096) and tiled(long, 8192)
    half = fusco.Layout(32768, 8, 256, 8)
    assert tiled(half, 4096) and not tiled(half, 4112) and tiled(half, 2048)       # 128 MiB of source rows, just more, half
    # a source tensor of more than 128 MiB: only with 8 rows per token, or 5 and more when the rows need no segments
    four, six = fusco.Layout(32768, 4, 128, 8), fusco.Layout(32768, 6, 128, 8)
    assert not tiled(four, 8192) and not tiled(four, 12288) and tiled(fusco.Layout(8192, 4, 128, 8), 12288)
    assert tiled(six, 8192) and tiled(six, 10240) and not tiled(six, 14336)       # 341 tokens per tile: 14 KiB rows take two segments
    assert tiled(long, 16384) and tiled(fusco.Layout(16384, 6, 128, 8), 7168)     # k = 8 with segments; 112 MiB of source rows
    assert fusco.fusco_probe_dispatch_kernel(2) == 0
    try:
        # workgroup shapes: the whole tile's source rows, or two column segments of them, must fit an XCD's L2
        assert not tiled(small, 2048) and not tiled(top1, 2048)
        assert tiled(many, 2048) and tiled(long, 4096)
        assert tiled(many, 15360) and tiled(many, 15376)                # one segment, two segments
        assert tiled(many, 30736) and tiled(many, 8 * 15360) and not tiled(many, 8 * 15360 + 16)   # up to eight segments
        assert tiled(wide, 3840) and not tiled(wide, 4096)              # segments would be narrower than 4 KiB
        assert not tiled(wide, 16384)
        assert not tiled(many, 14336, 0, fusco.DISPATCH_WIRE) and not tiled(many, 14336, 0, fusco.DISPATCH_TWO_HOP)
        assert tiled(many, 14336, 0, fusco.DISPATCH_STREAMING)
    finally:
        assert fusco.fusco_probe_dispatch_kernel(0) == 2


@pytest.mark.parametrize("which", [1, 2, 3, 4])
def test_token_walk_loads_and_stores_do_not_change_the_result(fusco, oracle, which):
    """Non-temporal or cached loads, plain or non-temporal stores of the token walk (the library picks by the sizes of
    the tensors): the expert tensor, the wire tensor and their second planes are the oracle's with every pairing.
    Rows of 1153 chunks with the second plane: two column segments per token."""
    rng = np.random.default_rng(500 + which)
    N, k, E, D, row_bytes, aux_bytes = 700, 6, 48, 8, 18416, 32
    A = random_topk(rng, N, k, E)
    x = rng.integers(0, 256, size=(N, row_bytes), dtype=np.uint8)
    xa = rng.integers(0, 256, size=(N, aux_bytes), dtype=np.uint8)
    want = oracle.plan(A, E, D)
    L, _ = gpu_plan(fusco, A, E, D)
    eb = torch.full((L.P, row_bytes), 0xEE, dtype=torch.uint8, device="cuda")
    ea = torch.full((L.P, aux_bytes), 0xEE, dtype=torch.uint8, device="cuda")
    sb = torch.full((L.send_cap, row_bytes), 0xEE, dtype=torch.uint8, device="cuda")
    sa = torch.full((L.send_cap, aux_bytes), 0xEE, dtype=torch.uint8, device="cuda")
    assert fusco.fusco_probe_dispatch_walk(which) == 0
    try:
        fusco.fusco_dispatch(L, dev(x), eb, x_aux=dev(xa), expert_aux=ea, send_buf=sb, send_aux=sa, flags=3)
        torch.cuda.synchronize()
    finally:
        assert fusco.fusco_probe_dispatch_walk(0) == which
    send_want, expert_want, saux_want, eaux_want = oracle.dispatch(want, x, xa)
    U = want.U
    assert np.array_equal(eb.cpu().numpy(), expert_want) and np.array_equal(ea.cpu().numpy(), eaux_want)
    assert np.array_equal(sb.cpu().numpy()[:U], send_want) and np.array_equal(sa.cpu().numpy()[:U], saux_want)
    assert np.all(sb.cpu().numpy()[U:] == 0xEE)
    with pytest.raises(fusco.FuscoError):
        fusco.fusco_probe_dispatch_walk(5)


def test_dispatch_kept_on_the_token_walk_gives_the_same_rows(fusco, oracle):
    """The study knob that keeps fusco_dispatch on the token walk changes the kernel, not the result."""
    rng = np.random.default_rng(77)
    N, k, E, D, row_bytes = 4500, 8, 64, 8, 1024
    A = random_topk(rng, N, k, E)
    x = rng.integers(0, 256, size=(N, row_bytes), dtype=np.uint8)
    want = oracle.plan(A, E, D)
    L, got = gpu_plan(fusco, A, E, D)
    eb = torch.full((L.P, row_bytes), 0xEE, dtype=torch.uint8, device="cuda")
    assert fusco.fusco_probe_dispatch_kernel(2) == 0 and fusco.fusco_dispatch_in_transfer_order(L, row_bytes)
    assert fusco.fusco_probe_dispatch_kernel(1) == 2
    try:
        assert not fusco.fusco_dispatch_in_transfer_order(L, row_bytes)
        fusco.fusco_dispatch(L, dev(x), eb)
        torch.cuda.synchronize()
    finally:
        fusco.fusco_probe_dispatch_kernel(0)
    assert fusco.fusco_probe_dispatch_kernel() == 0
    _, expert_want = oracle.dispatch(want, x)
    assert np.array_equal(eb.cpu().numpy(), expert_want)
