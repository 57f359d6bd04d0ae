"""The hot path at the benchmark's full sizes, in the launch configuration bench.py times.

The descriptor and the combined output are compared whole with the oracle (the output in chunks of
tokens, so that the host never holds more than a chunk's rows).  Moved rows are compared whole where
the tensor fits the host comfortably, else on sampled rows plus a property checked on every row
(every slot holds its token's row).
"""
import numpy as np
import pytest
import torch

import workloads as W
from definitions import PLAN_FIELDS

pytestmark = pytest.mark.gpu

REL_TOL = 1e-5


@pytest.fixture(scope="module")
def fusco():
    import paper_2512_22036_amd as f
    f.load_library()
    assert torch.cuda.is_available()
    return f


def _bf16_dev(bits):
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)


def _bits(t):
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


@pytest.mark.timeout(600)
@pytest.mark.parametrize("name,compare_all", [("tiny", True), ("dsv3", True), ("qwen3", False), ("skewed", False)])
def test_full_size_path(fusco, oracle, name, compare_all):
    cfg = W.get_config(name)
    print("config", name, "N", cfg.N, "H", cfg.H, flush=True)
    A, w = W.make_routing(cfg)
    xb = W.make_activations(cfg)
    want = oracle.plan(A, cfg.E, cfg.D)

    L = fusco.Layout(cfg.N, cfg.k, cfg.E, cfg.D)
    d_x = _bf16_dev(xb)
    d_w = torch.from_numpy(w).cuda()
    fusco.fusco_plan(L, torch.from_numpy(A).cuda())
    torch.cuda.synchronize()
    got = L.to_host()
    assert int(got.status[0]) == 0
    for f in PLAN_FIELDS:
        assert np.array_equal(getattr(got, f), getattr(want, f)), f
    assert np.array_equal(got.tile_slots, oracle.tile_order(want.pair_slot, cfg.N, cfg.k, L.tile_tokens))

    # dispatch, expert tensor and wire tensor
    d_e = torch.empty((cfg.P, cfg.H), dtype=torch.bfloat16, device="cuda")
    d_s = torch.empty((L.send_cap, cfg.H), dtype=torch.bfloat16, device="cuda")
    fusco.fusco_dispatch(L, d_x, d_e, send_buf=d_s, flags=3)
    torch.cuda.synchronize()
    rng = np.random.default_rng(cfg.seed)
    if compare_all:
        send_want, expert_want = oracle.dispatch(want, xb)
        assert np.array_equal(_bits(d_e), expert_want)
        assert np.array_equal(_bits(d_s[:want.U]), send_want)
        del send_want, expert_want
    slots = np.unique(np.concatenate([rng.integers(0, cfg.P, size=4096), [0, cfg.P - 1], want.exp_off[:-1],
                                      np.maximum(want.exp_off[1:] - 1, 0)])).astype(np.int32)
    rows_want = oracle.dispatch_rows(want, xb, slots)
    assert np.array_equal(_bits(d_e[torch.from_numpy(slots).long().cuda()]), rows_want)
    # property at any size: every slot holds the row of its token, every send row the row of its source
    d_tok = torch.from_numpy(want.slot_token).long().cuda()
    step = 1 << 15
    for s0 in range(0, cfg.P, step):
        assert torch.equal(d_e[s0:s0 + step], d_x[d_tok[s0:s0 + step]])
    d_src = torch.from_numpy(want.send_src).long().cuda()
    for s0 in range(0, want.U, step):
        assert torch.equal(d_s[s0:min(s0 + step, want.U)], d_x[d_src[s0:s0 + step]])
    del d_s

    # combine over the expert tensor (identity experts): the WHOLE output against the oracle's single-precision
    # chain, bit for bit, for both output types.  The oracle works through the tokens in chunks (it rebuilds the
    # chunk's k rows per token from the descriptors), so host memory stays bounded at any size.
    d_o16 = torch.full((cfg.N, cfg.H), float("nan"), dtype=torch.bfloat16, device="cuda")
    d_o32 = torch.full((cfg.N, cfg.H), float("nan"), dtype=torch.float32, device="cuda")
    fusco.fusco_combine(L, d_e, d_w, d_o16)
    fusco.fusco_combine(L, d_e, d_w, d_o32)
    torch.cuda.synchronize()
    chunk = 2048
    for t0 in range(0, cfg.N, chunk):
        t1 = min(t0 + chunk, cfg.N)
        print("combine tokens", t0, t1, flush=True)
        y_sub = oracle.dispatch_rows(want, xb, want.pair_slot[t0 * cfg.k:t1 * cfg.k])
        w_sub = w[t0:t1]
        ps_sub = np.arange((t1 - t0) * cfg.k, dtype=np.int32)
        o32, o16 = oracle.combine_f32(y_sub, w_sub, ps_sub)
        assert np.array_equal(_bits(d_o16[t0:t1]), o16), (t0, t1)
        g = d_o32[t0:t1].cpu().numpy()
        assert np.array_equal(g.view(np.uint32), o32.view(np.uint32)), (t0, t1)
        # the 1e-5 bound against the double-precision sum, on a sample of every chunk
        pick = np.unique(rng.integers(0, t1 - t0, size=48)).astype(np.int32)
        ref = oracle.combine_f64(y_sub, w_sub, ps_sub, tokens=pick)
        scale = oracle.combine_abs_f64(y_sub, w_sub, ps_sub, tokens=pick)
        assert np.all(np.abs(g[pick].astype(np.float64) - ref) <= REL_TOL * scale)
        del y_sub, o32, o16, g
