"""fusco_plan_static, the planner entry point that allocates nothing (its scratch is a static array inside the
library), against fusco_plan on the same inputs: every descriptor array must agree bit for bit, on two calls in
a row of which the second is the smaller input (the shared array still holds the first call's counts)."""
import ctypes

import numpy as np
import pytest
import torch

from definitions import random_topk

pytestmark = pytest.mark.gpu

FIELDS = ("exp_count", "exp_off", "send_count", "send_off", "pair_slot", "slot_pair", "slot_token", "send_src",
          "pair_send_row", "slot_send_row", "pair_first", "tile_slots", "status")


def _plan_both_ways(f, lib, A, E, D):
    N, k = A.shape
    d_A = torch.from_numpy(A).cuda()
    ref = f.Layout(N, k, E, D)
    ref.mem.fill_(0xA5)
    f.fusco_plan(ref, d_A)
    got = f.Layout(N, k, E, D)
    got.mem.fill_(0xA5)                        # same background: slots left unassigned by invalid ids stay as they were
    stream = torch.cuda.current_stream().cuda_stream
    rc = lib.fusco_plan_static(ctypes.byref(got.c), ctypes.c_void_p(d_A.data_ptr()), ctypes.c_void_p(stream))
    assert rc == 0, lib.fusco_status_string(rc)
    torch.cuda.synchronize()
    U = int(ref.array("send_off")[D].item())
    for name in FIELDS:
        a, b = ref.array(name), got.array(name)
        if name == "send_src":
            a, b = a[:U], b[:U]                   # rows >= U are not written by either call
        assert torch.equal(a, b), name
    return ref


def test_static_scratch_plan_matches_fusco_plan_twice_in_a_row():
    import paper_2512_22036_amd as f
    lib = f.load_library()
    assert torch.cuda.is_available()
    rng = np.random.default_rng(77)
    # first call: 27 tiles of 2048 pairs
    big = random_topk(rng, 6700, 8, 256)
    first = _plan_both_ways(f, lib, big, 256, 8)
    assert int(first.array("status").item()) == 0
    # second call, smaller and with other sizes: a single tile each, on the array the first call used
    _plan_both_ways(f, lib, random_topk(rng, 300, 6, 48), 48, 16)
    _plan_both_ways(f, lib, random_topk(rng, 100, 8, 256), 256, 64)
    # and a large one again: 196 tiles, with a chunk level
    _plan_both_ways(f, lib, random_topk(rng, 50000, 8, 256), 256, 8)
    # invalid expert ids are counted the same way
    bad = random_topk(rng, 900, 4, 32)
    bad[5, 1], bad[700, 3] = -1, 32
    layout = _plan_both_ways(f, lib, bad, 32, 4)
    assert int(layout.array("status").item()) == 2


def test_static_scratch_plan_result_feeds_dispatch_and_combine(oracle):
    import paper_2512_22036_amd as f
    import workloads as W
    f.load_library()
    cfg = W.get_config("dsv3").with_tokens(700)
    A, w = W.make_routing(cfg)
    xb = W.make_activations(cfg)
    want = oracle.plan(A, cfg.E, cfg.D)
    _, expert_want = oracle.dispatch(want, xb)
    _, out_want = oracle.combine_f32(expert_want, w, want.pair_slot)
    L = f.Layout(cfg.N, cfg.k, cfg.E, cfg.D)
    x = torch.from_numpy(xb.view(np.int16)).cuda().view(torch.bfloat16)
    eb = torch.empty((cfg.P, cfg.H), dtype=torch.bfloat16, device="cuda")
    out = torch.empty((cfg.N, cfg.H), dtype=torch.bfloat16, device="cuda")
    f.fusco_plan_static(L, torch.from_numpy(A).cuda())
    f.fusco_dispatch(L, x, eb)
    f.fusco_combine(L, eb, torch.from_numpy(w).cuda(), out)
    torch.cuda.synchronize()
    got = L.to_host()
    for name in FIELDS[:-1]:
        if name != "tile_slots":
            assert np.array_equal(getattr(got, name), getattr(want, name)), name
    assert np.array_equal(got.tile_slots, oracle.tile_order(want.pair_slot, cfg.N, cfg.k, L.tile_tokens))
    assert np.array_equal(eb.view(torch.int16).cpu().numpy().view(np.uint16), expert_want)
    assert np.array_equal(out.view(torch.int16).cpu().numpy().view(np.uint16), out_want)
