"""Two-hop dispatch (the two descriptor levels executed one after the other) and the disaggregated
multi-stage baseline must produce the same bytes as the oracle and as the fused path."""
import numpy as np
import pytest
import torch

import workloads as W
from definitions import random_topk

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def fusco():
    import paper_2512_22036_amd as f
    f.load_library()
    assert torch.cuda.is_available()
    return f


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def bf16_dev(bits):
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)


def bits_host(t):
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


SHAPES = [(33, 2, 8, 4, 16), (257, 8, 64, 8, 2048), (300, 8, 256, 8, 14336), (513, 2, 16, 4, 16 * 37),
          (64, 3, 6, 3, 16 * 129), (40, 8, 32, 32, 16 * 1025), (1, 1, 1, 1, 4096), (700, 4, 16, 1, 256)]


@pytest.mark.parametrize("N,k,E,D,row_bytes", SHAPES)
def test_two_hop_dispatch_matches_oracle(fusco, oracle, N, k, E, D, row_bytes):
    rng = np.random.default_rng(N + row_bytes + 1)
    A = random_topk(rng, N, k, E)
    x = rng.integers(0, 256, size=(N, row_bytes), dtype=np.uint8)
    want = oracle.plan(A, E, D)
    send_want, expert_want = oracle.dispatch(want, x)     # the oracle itself goes hop by hop
    L = fusco.Layout(N, k, E, D)
    fusco.fusco_plan(L, dev(A))
    eb = torch.full((L.P, row_bytes), 0xEE, dtype=torch.uint8, device="cuda")
    sb = torch.full((L.send_cap, row_bytes), 0xEE, dtype=torch.uint8, device="cuda")
    fusco.fusco_dispatch(L, dev(x), eb, send_buf=sb, flags=fusco.DISPATCH_TWO_HOP)
    torch.cuda.synchronize()
    assert np.array_equal(eb.cpu().numpy(), expert_want)
    assert np.array_equal(sb[:want.U].cpu().numpy(), send_want)
    assert bool((sb[want.U:] == 0xEE).all())


def test_two_hop_with_aux_plane_on_decode_config(fusco, oracle):
    cfg = W.get_config("decode_fp8")
    A, _ = W.make_routing(cfg)
    q, sc = W.make_fp8_activations(cfg)
    want = oracle.plan(A, cfg.E, cfg.D)
    send_want, expert_want, saux_want, eaux_want = oracle.dispatch(want, q, sc)
    L = fusco.Layout(cfg.N, cfg.k, cfg.E, cfg.D)
    fusco.fusco_plan(L, dev(A))
    eb = torch.zeros((L.P, cfg.H), dtype=torch.uint8, device="cuda")
    ea = torch.zeros((L.P, cfg.H // 128), dtype=torch.float32, device="cuda")
    sb = torch.zeros((L.send_cap, cfg.H), dtype=torch.uint8, device="cuda")
    sa = torch.zeros((L.send_cap, cfg.H // 128), dtype=torch.float32, device="cuda")
    fusco.fusco_dispatch(L, dev(q), eb, x_aux=dev(sc), expert_aux=ea, send_buf=sb, send_aux=sa,
                         flags=fusco.DISPATCH_TWO_HOP)
    torch.cuda.synchronize()
    assert np.array_equal(eb.cpu().numpy(), expert_want) and np.array_equal(ea.cpu().numpy(), eaux_want)
    assert np.array_equal(sb[:want.U].cpu().numpy(), send_want) and np.array_equal(sa[:want.U].cpu().numpy(), saux_want)


def test_two_hop_skips_invalid_pairs(fusco):
    rng = np.random.default_rng(5)
    N, k, E, D = 300, 4, 16, 4
    A = random_topk(rng, N, k, E)
    A[7, 2] = 99
    A[200, 0] = -1
    L = fusco.Layout(N, k, E, D)
    fusco.fusco_plan(L, dev(A))
    x = dev(rng.integers(0, 256, size=(N, 64), dtype=np.uint8))
    eb = torch.full((L.P, 64), 0xEE, dtype=torch.uint8, device="cuda")
    sb = torch.full((L.send_cap, 64), 0xEE, dtype=torch.uint8, device="cuda")
    fusco.fusco_dispatch(L, x, eb, send_buf=sb, flags=fusco.DISPATCH_TWO_HOP)
    torch.cuda.synchronize()
    got = L.to_host()
    assert int(got.status[0]) == 2
    assigned = int(got.exp_off[E])
    assert assigned == N * k - 2
    assert torch.equal(eb[:assigned], x[dev(got.slot_token[:assigned]).long()])
    assert bool((eb[assigned:] == 0xEE).all())


@pytest.mark.parametrize("N,k,E,D,H", [(50, 2, 8, 4, 8), (300, 8, 256, 8, 7168), (513, 4, 16, 4, 296),
                                       (129, 8, 64, 64, 1024), (90, 3, 6, 1, 512)])
def test_disaggregated_baseline_matches_oracle(fusco, oracle, N, k, E, D, H):
    rng = np.random.default_rng(N * H + 3)
    A = random_topk(rng, N, k, E)
    xb = W.bf16_bits(rng.standard_normal((N, H)).astype(np.float32))
    w = rng.random((N, k)).astype(np.float32)
    w /= w.sum(1, keepdims=True)
    want = oracle.plan(A, E, D)
    _, expert_want = oracle.dispatch(want, xb)
    L = fusco.Layout(N, k, E, D)
    Lr = fusco.Layout(N, k, D, D)
    d_A = dev(A)
    fusco.fusco_plan(L, d_A)
    fusco.fusco_disaggregated_plan(Lr, L, d_A, torch.empty_like(d_A))
    P = N * k
    sa = torch.zeros((P, H), dtype=torch.bfloat16, device="cuda")
    sb = torch.zeros((P, H), dtype=torch.bfloat16, device="cuda")
    eb = torch.zeros((P, H), dtype=torch.bfloat16, device="cuda")
    fusco.fusco_disaggregated_dispatch(L, Lr, bf16_dev(xb), sa, sb, eb)
    torch.cuda.synchronize()
    assert np.array_equal(bits_host(eb), expert_want)
    # stage 1 of the paper's baseline: tokens rearranged by destination device (stable in (t, j))
    dev_of_pair = (A // (E // D)).reshape(-1)
    order = np.argsort(dev_of_pair, kind="stable")
    assert np.array_equal(bits_host(sa), xb[order // k])
    assert np.array_equal(bits_host(sb), xb[order // k])
    # the rank-major plan is the oracle's plan of the device ids
    rank_want = oracle.plan(A // (E // D), D, D)
    got = Lr.to_host()
    assert np.array_equal(got.pair_slot, rank_want.pair_slot) and np.array_equal(got.slot_token, rank_want.slot_token)

    yb = W.bf16_bits(rng.standard_normal((P, H)).astype(np.float32))
    o32, o16 = oracle.combine_f32(yb, w, want.pair_slot)
    for out_dtype in (torch.bfloat16, torch.float32):
        out = torch.full((N, H), float("nan"), dtype=out_dtype, device="cuda")
        fusco.fusco_disaggregated_combine(L, Lr, bf16_dev(yb), dev(w), sa, sb, out)
        torch.cuda.synchronize()
        if out_dtype == torch.bfloat16:
            assert np.array_equal(bits_host(out), o16)
        else:
            assert np.array_equal(out.cpu().numpy().view(np.uint32), o32.view(np.uint32))
        # stage 3' put every expert row at its rank row
        assert np.array_equal(bits_host(sa), yb[want.pair_slot[order]])


TWO_HOP_COMBINE_SHAPES = [(50, 2, 8, 4, 8), (300, 8, 256, 8, 7168), (65, 4, 16, 4, 296), (129, 8, 64, 64, 1024),
                          (90, 3, 6, 1, 512), (20, 17, 34, 2, 2056), (10, 64, 128, 8, 4096),
                          (12, 9, 18, 3, 8 * 1285)]       # rows of two and three uneven column segments, general k


@pytest.mark.parametrize("N,k,E,D,H", TWO_HOP_COMBINE_SHAPES)
@pytest.mark.parametrize("y_f32", [False, True])
def test_two_hop_combine_matches_oracle(fusco, oracle, N, k, E, D, H, y_f32):
    rng = np.random.default_rng(N * H + k + 7)
    A = random_topk(rng, N, k, E)
    want = oracle.plan(A, E, D)
    if y_f32:
        y = rng.standard_normal((N * k, H)).astype(np.float32)
        d_y = dev(y)
    else:
        y = W.bf16_bits(rng.standard_normal((N * k, H)).astype(np.float32))
        d_y = bf16_dev(y)
    w = (rng.standard_normal((N, k)) * 2).astype(np.float32)
    o32, o16, part = oracle.combine_two_hop_f32(want, y, w, want_partial=True)
    ref = oracle.combine_f64(y, w, want.pair_slot)
    scale = oracle.combine_abs_f64(y, w, want.pair_slot)
    L = fusco.Layout(N, k, E, D)
    fusco.fusco_plan(L, dev(A))
    for out_dtype in (torch.float32, torch.bfloat16):
        d_p = torch.full((L.send_cap, H), float("nan"), dtype=torch.float32, device="cuda")
        out = torch.full((N, H), float("nan"), dtype=out_dtype, device="cuda")
        fusco.fusco_combine_two_hop(L, d_y, dev(w), d_p, out)
        torch.cuda.synchronize()
        assert np.array_equal(d_p[:want.U].cpu().numpy().view(np.uint32), part.view(np.uint32))
        assert bool(torch.isnan(d_p[want.U:]).all())        # rows past U stay untouched
        if out_dtype == torch.float32:
            g = out.cpu().numpy()
            assert np.array_equal(g.view(np.uint32), o32.view(np.uint32))
            assert np.all(np.abs(g.astype(np.float64) - ref) <= 1e-5 * scale)
        else:
            assert np.array_equal(bits_host(out), o16)


def test_two_hop_round_trip_returns_input_exactly(fusco):
    rng = np.random.default_rng(9)
    N, k, E, D, H = 600, 8, 64, 8, 2048
    A = random_topk(rng, N, k, E)
    xb = W.bf16_bits(rng.standard_normal((N, H)).astype(np.float32))
    L = fusco.Layout(N, k, E, D)
    fusco.fusco_plan(L, dev(A))
    eb = torch.empty((L.P, H), dtype=torch.bfloat16, device="cuda")
    sb = torch.empty((L.send_cap, H), dtype=torch.bfloat16, device="cuda")
    part = torch.empty((L.send_cap, H), dtype=torch.float32, device="cuda")
    out = torch.empty((N, H), dtype=torch.bfloat16, device="cuda")
    fusco.fusco_dispatch(L, bf16_dev(xb), eb, send_buf=sb, flags=fusco.DISPATCH_TWO_HOP)
    fusco.fusco_combine_two_hop(L, eb, torch.full((N, k), 1.0 / k, device="cuda"), part, out)
    torch.cuda.synchronize()
    assert np.array_equal(bits_host(out), xb)


def test_calls_follow_the_given_stream_and_can_be_captured_in_a_graph(fusco, oracle):
    """The library only enqueues on the caller's stream: a step issued on a side stream, and a step
    captured into a HIP graph and replayed several times with eager work in between, give the eager
    result bit for bit."""
    rng = np.random.default_rng(21)
    N, k, E, D, H = 700, 8, 64, 8, 1024
    A = random_topk(rng, N, k, E)
    xb = W.bf16_bits(rng.standard_normal((N, H)).astype(np.float32))
    w = rng.random((N, k)).astype(np.float32)
    want = oracle.plan(A, E, D)
    _, expert_want = oracle.dispatch(want, xb)
    _, out_want = oracle.combine_f32(expert_want, w, want.pair_slot)
    d_A, d_x, d_w = dev(A), bf16_dev(xb), dev(w)
    L = fusco.Layout(N, k, E, D)
    eb = torch.zeros((N * k, H), dtype=torch.bfloat16, device="cuda")
    out = torch.zeros((N, H), dtype=torch.bfloat16, device="cuda")

    def step():
        fusco.fusco_plan(L, d_A)
        fusco.fusco_dispatch(L, d_x, eb)
        fusco.fusco_combine(L, eb, d_w, out)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    side.synchronize()
    assert np.array_equal(bits_host(eb), expert_want) and np.array_equal(bits_host(out), out_want)

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()
    for i in range(4):
        eb.zero_()
        out.zero_()
        L.mem.fill_(0x5A)                  # eager work between the replays; the plan must be rebuilt by the graph
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert np.array_equal(bits_host(eb), expert_want), i
        assert np.array_equal(bits_host(out), out_want), i
        got = L.to_host()
        assert np.array_equal(got.pair_slot, want.pair_slot) and np.array_equal(got.send_src, want.send_src)


def test_plain_c_program_uses_the_boundary_without_python(fusco):
    """examples/c_abi_usage.c: HIP runtime + the C boundary only; it checks its own results and prints ok."""
    import os
    import subprocess
    from paper_2512_22036_amd import build
    if not os.path.exists(build.EXAMPLE_BIN):
        build.build_c_example()          # host compiler only, a second or two
    res = subprocess.run([build.EXAMPLE_BIN], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=100)
    assert res.returncode == 0 and "c_abi_usage ok" in res.stdout, res.stdout


def test_cross_node_load_matrix_feeds_the_balancer(fusco, oracle):
    """Section 3.4 end to end: every GPU of a 2-node x 4-GPU cluster plans its own (skewed) routing, writes its
    cross-node load into its cell of the device-resident load matrix, and Algorithm 1 groups the GPUs."""
    import dataclasses
    import workloads as W
    nodes, gpus, row_bytes = 2, 4, 14336
    base = W.get_config("skewed").with_tokens(1500)
    matrix = torch.full((nodes, gpus), -1, dtype=torch.int64, device="cuda")
    want = np.zeros((nodes, gpus), dtype=np.int64)
    for n in range(nodes):
        for g in range(gpus):
            cfg = dataclasses.replace(base, seed=base.seed + 17 * (n * gpus + g))
            A, _ = W.make_routing(cfg)
            L = fusco.Layout(cfg.N, cfg.k, cfg.E, cfg.D)
            fusco.fusco_plan(L, torch.from_numpy(A).cuda())
            fusco.fusco_cross_node_load(L, cfg.D // nodes, n, row_bytes, matrix[n, g:g + 1])
            want[n, g] = oracle.cross_node_load(A, cfg.E, cfg.D, cfg.D // nodes, n, row_bytes)
    torch.cuda.synchronize()
    got = matrix.cpu().numpy()
    assert np.array_equal(got, want)
    assert len(set(want.ravel().tolist())) > 1                 # the skewed routing does load the GPUs unevenly
    assert np.array_equal(fusco.fusco_balance_groups(got), oracle.balance_groups(want))
    # one device per node: the load is everything but the GPU's own device
    cfg = base
    A, _ = W.make_routing(cfg)
    L = fusco.Layout(cfg.N, cfg.k, cfg.E, cfg.D)
    fusco.fusco_plan(L, torch.from_numpy(A).cuda())
    cell = torch.zeros(1, dtype=torch.int64, device="cuda")
    for home in (0, cfg.D - 1):
        fusco.fusco_cross_node_load(L, 1, home, 16, cell)
        torch.cuda.synchronize()
        assert int(cell.item()) == oracle.cross_node_load(A, cfg.E, cfg.D, 1, home, 16)
    fusco.fusco_cross_node_load(L, cfg.D, 0, 16, cell)        # a single node: nothing crosses
    torch.cuda.synchronize()
    assert int(cell.item()) == 0
