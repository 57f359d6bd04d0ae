"""Pins for the oracle's planner: hand-worked examples, brute force from the definitions,
stable argsort, invariants, special cases and the closed-form expected send-row count."""
import os

import numpy as np
import pytest

import workloads as W
from definitions import (PLAN_FIELDS, brute_force_plan, check_plan_invariants,
                         expected_send_rows_per_token, random_topk)

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "plan_hand_examples.txt")


def _read_examples():
    examples, cur = [], {}
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        if line == "---":
            examples.append(cur)
            cur = {}
            continue
        key, vals = line.split(":")
        cur[key.strip()] = np.array([int(v) for v in vals.split()], dtype=np.int64)
    examples.append(cur)
    return examples


@pytest.mark.parametrize("ex", _read_examples(), ids=lambda e: "N%dk%dE%dD%d" % (e["N"][0], e["k"][0], e["E"][0], e["D"][0]))
def test_hand_worked_examples(oracle, ex):
    N, k, E, D = (int(ex[c][0]) for c in "NkED")
    pl = oracle.plan(ex["A"].reshape(N, k), E, D)
    for f in PLAN_FIELDS:
        assert np.array_equal(getattr(pl, f), ex[f]), f


CASES = [(1, 1, 1, 1), (1, 4, 8, 2), (7, 2, 4, 2), (9, 3, 6, 3), (12, 2, 16, 4), (16, 4, 8, 8),
         (10, 8, 32, 4), (13, 3, 12, 1), (11, 5, 5, 5), (24, 2, 6, 6), (5, 6, 64, 64), (20, 1, 4, 2)]


@pytest.mark.parametrize("N,k,E,D", CASES)
@pytest.mark.parametrize("distinct", [True, False])
def test_brute_force_definitions(oracle, N, k, E, D, distinct):
    rng = np.random.default_rng(1000 * N + 10 * k + E + D + int(distinct))
    for _ in range(6):
        A = random_topk(rng, N, k, E, distinct)
        pl = oracle.plan(A, E, D)
        ref = brute_force_plan(A, E, D)
        for f in PLAN_FIELDS:
            assert np.array_equal(getattr(pl, f), ref[f]), (f, A.tolist())


def test_many_tiny_random_cases(oracle):
    rng = np.random.default_rng(7)
    for _ in range(400):
        D = int(rng.choice([1, 2, 3, 4, 8]))
        E = D * int(rng.integers(1, 5))
        k = int(rng.integers(1, min(E, 6) + 1))
        N = int(rng.integers(1, 9))
        A = random_topk(rng, N, k, E, bool(rng.integers(0, 2)))
        pl = oracle.plan(A, E, D)
        ref = brute_force_plan(A, E, D)
        for f in PLAN_FIELDS:
            assert np.array_equal(getattr(pl, f), ref[f]), (f, A.tolist(), E, D)


@pytest.mark.parametrize("N,k,E,D", [(300, 4, 32, 8), (1000, 8, 256, 8), (513, 2, 16, 4), (257, 6, 128, 16)])
def test_expert_major_order_is_stable_argsort(oracle, N, k, E, D):
    A = random_topk(np.random.default_rng(N + k), N, k, E)
    pl = oracle.plan(A, E, D)
    assert np.array_equal(pl.slot_pair, np.argsort(A.reshape(-1), kind="stable"))
    check_plan_invariants(pl, A)


@pytest.mark.parametrize("name", ["tiny", "dsv3", "qwen3", "skewed", "decode_fp8"])
def test_invariants_and_dedup_statistics_on_configs(oracle, name):
    cfg = W.get_config(name)
    if cfg.N > 8192:
        cfg = cfg.with_tokens(8192)
    A, _ = W.make_routing(cfg)
    pl = oracle.plan(A, cfg.E, cfg.D)
    check_plan_invariants(pl, A)
    assert np.array_equal(pl.slot_pair, np.argsort(A.reshape(-1), kind="stable"))
    ratio = pl.U / cfg.N
    if cfg.routing == "zipf_limited":
        assert ratio <= cfg.max_devices
        d = A // (cfg.E // cfg.D)
        assert max(len(set(r)) for r in d.tolist()) <= cfg.max_devices
    else:
        # k distinct experts drawn uniformly: E[U]/N = D (1 - C(E - E/D, k) / C(E, k))
        want = expected_send_rows_per_token(cfg.E, cfg.k, cfg.D)
        # per-token count lies in [1, min(k, D)], so its standard deviation is below min(k, D) / 2
        tol = 5.0 * (min(cfg.k, cfg.D) / 2.0) / np.sqrt(cfg.N)
        assert abs(ratio - want) < tol, (ratio, want)


def test_special_case_single_device(oracle):
    A = random_topk(np.random.default_rng(3), 50, 4, 16)
    pl = oracle.plan(A, 16, 1)
    assert pl.U == 50
    assert np.array_equal(pl.send_src, np.arange(50))
    assert np.array_equal(pl.pair_send_row, np.repeat(np.arange(50), 4))
    assert np.array_equal(pl.pair_first.reshape(50, 4), np.tile([1, 0, 0, 0], (50, 1)))


def test_special_case_one_expert_per_device(oracle):
    A = random_topk(np.random.default_rng(4), 40, 3, 8)
    pl = oracle.plan(A, 8, 8)
    assert pl.U == pl.P
    assert np.all(pl.pair_first == 1)
    assert np.array_equal(pl.send_count, pl.exp_count)
    assert np.array_equal(pl.pair_send_row, pl.pair_slot)   # both levels coincide
    assert np.array_equal(pl.send_src, pl.slot_token)


def test_special_case_all_tokens_to_one_device(oracle):
    rng = np.random.default_rng(5)
    A = np.stack([4 + rng.permutation(4)[:3] for _ in range(30)]).astype(np.int32)   # experts 4..7 = device 1 of 4
    pl = oracle.plan(A, 16, 4)
    assert pl.U == 30
    assert pl.send_count.tolist() == [0, 30, 0, 0]
    assert np.array_equal(pl.send_src, np.arange(30))


def test_k1_is_a_permutation(oracle):
    A = random_topk(np.random.default_rng(6), 64, 1, 8)
    pl = oracle.plan(A, 8, 2)
    assert np.array_equal(np.sort(pl.slot_token), np.arange(64))
    assert pl.U == 64 and np.all(pl.pair_first == 1)


def test_empty_input(oracle):
    pl = oracle.plan(np.zeros((0, 4), dtype=np.int32), 8, 2)
    assert pl.U == 0 and pl.exp_off.tolist() == [0] * 9 and pl.send_off.tolist() == [0] * 3


def test_rejects_bad_arguments(oracle):
    with pytest.raises(ValueError):
        oracle.plan(np.array([[0, 9]], dtype=np.int32), 8, 2)      # id out of range
    with pytest.raises(ValueError):
        oracle.plan(np.array([[0, -1]], dtype=np.int32), 8, 2)
    with pytest.raises(ValueError):
        oracle.plan(np.array([[0, 1]], dtype=np.int32), 8, 3)      # E % D != 0


# ---- transfer order of the expert-tensor rows (tiles of tokens, rows ascending inside a tile) ----

def _tile_order_by_definition(pair_slot, N, k, tile_tokens):
    out = []
    for t0 in range(0, N, tile_tokens):
        mine = sorted(int(s) for s in pair_slot[t0 * k:min(t0 + tile_tokens, N) * k] if s >= 0)
        out += mine + [-1] * (tile_tokens * k - len(mine))
    return np.array(out, dtype=np.int32)


@pytest.mark.parametrize("N,k,E,D,tile_tokens", [(1, 1, 1, 1, 1), (10, 2, 4, 2, 4), (37, 3, 9, 3, 8), (64, 8, 32, 4, 16),
                                                 (100, 4, 16, 4, 100), (100, 4, 16, 4, 1000), (33, 5, 5, 5, 7)])
def test_tile_order_matches_its_definition(oracle, N, k, E, D, tile_tokens):
    rng = np.random.default_rng(N * 7 + tile_tokens)
    A = random_topk(rng, N, k, E, distinct=k <= E)
    pl = oracle.plan(A, E, D)
    got = oracle.tile_order(pl.pair_slot, N, k, tile_tokens)
    assert np.array_equal(got, _tile_order_by_definition(pl.pair_slot, N, k, tile_tokens))
    # every row of the expert tensor is listed exactly once, by the tile of its token, experts ascending inside a tile
    listed = got[got >= 0]
    assert np.array_equal(np.sort(listed), np.arange(pl.P))
    cap = tile_tokens * k
    for i in range(len(got) // cap):
        rows = got[i * cap:(i + 1) * cap]
        rows = rows[rows >= 0]
        assert np.all(np.diff(rows) > 0)
        assert np.all(pl.slot_token[rows] // tile_tokens == i)
        experts = A.reshape(-1)[pl.slot_pair[rows]]
        assert np.all(np.diff(experts) >= 0)


def test_tile_order_skips_pairs_without_a_row_and_handles_one_tile(oracle):
    ps = np.array([5, -1, 0, 3, -1, -1, 2, 1], dtype=np.int32)             # 4 tokens x 2, three pairs without a row
    assert oracle.tile_order(ps, 4, 2, 2).tolist() == [0, 3, 5, -1, 1, 2, -1, -1]
    assert oracle.tile_order(ps, 4, 2, 4).tolist() == [0, 1, 2, 3, 5, -1, -1, -1]
    assert oracle.tile_order(ps, 4, 2, 3).tolist() == [0, 3, 5, -1, -1, -1, 1, 2, -1, -1, -1, -1]
    assert oracle.tile_order(np.zeros(0, dtype=np.int32), 0, 2, 4).tolist() == []
