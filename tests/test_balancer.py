"""Algorithm 1 (Online Group-Balanced Assignment): the oracle against a hand-worked example and the
algorithm's own invariants, and the library's host function against the oracle."""
import itertools
import os

import numpy as np
import pytest

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "balancer_hand_example.txt")


def _golden():
    load, groups = [], []
    for line in open(GOLDEN):
        if line.startswith("load:"):
            load.append([int(v) for v in line.split(":")[1].split()])
        if line.startswith("group:"):
            groups.append([int(v) for v in line.split(":")[1].split()])
    return np.array(load, dtype=np.int64), np.array(groups, dtype=np.int32)


def _check_invariants(load, G):
    nodes, gpus = load.shape
    assert G.shape == (gpus, nodes)
    # every group holds exactly one GPU of every node, and every GPU is in exactly one group
    for n in range(nodes):
        assert sorted(G[:, n].tolist()) == list(range(gpus))
    # the heaviest GPU of each node lands in a different group when there are at least as many GPUs as nodes
    if gpus >= nodes:
        heavy_group = []
        for n in range(nodes):
            top = min(range(gpus), key=lambda g: (-int(load[n][g]), g))
            heavy_group.append(int(np.flatnonzero(G[:, n] == top)[0]))
        assert len(set(heavy_group)) == nodes


def test_oracle_hand_worked_example(oracle):
    load, groups = _golden()
    assert np.array_equal(oracle.balance_groups(load), groups)


@pytest.mark.parametrize("nodes,gpus", [(1, 1), (1, 8), (2, 2), (4, 4), (8, 8), (3, 4), (8, 4), (5, 7)])
def test_oracle_invariants(oracle, nodes, gpus):
    rng = np.random.default_rng(nodes * 10 + gpus)
    for trial in range(20):
        load = rng.integers(0, 6 if trial % 2 else 10 ** 9, size=(nodes, gpus))     # with and without ties
        _check_invariants(load, oracle.balance_groups(load))


def test_oracle_sorted_nodes_reduce_to_plain_rotation(oracle):
    # loads already descending in GPU index: P_n is the identity, so group i of node n is GPU (i + n) mod M
    nodes, gpus = 4, 4
    load = np.tile(np.arange(gpus, 0, -1), (nodes, 1))
    G = oracle.balance_groups(load)
    for i in range(gpus):
        for n in range(nodes):
            assert G[i][n] == (i + n) % gpus


def test_greedy_is_never_better_than_the_exhaustive_optimum_and_beats_same_index_on_skew(oracle):
    rng = np.random.default_rng(3)
    nodes, gpus = 3, 3
    worse_than_static = 0
    for _ in range(30):
        load = rng.integers(0, 100, size=(nodes, gpus))
        G = oracle.balance_groups(load)
        greedy = max(sum(load[n][G[i][n]] for n in range(nodes)) for i in range(gpus))
        best = min(max(sum(load[n][perm[n][i]] for n in range(nodes)) for i in range(gpus))
                   for perm in itertools.product(itertools.permutations(range(gpus)), repeat=nodes))
        assert greedy >= best
    # every node has one hot GPU at the same local index: same-index grouping stacks them, the greedy spreads them
    load = np.full((4, 4), 10)
    load[:, 2] = 1000
    G = oracle.balance_groups(load)
    greedy = max(sum(load[n][G[i][n]] for n in range(4)) for i in range(4))
    static = max(load[:, i].sum() for i in range(4))
    assert greedy == 1030 and static == 4000


def test_library_matches_oracle(oracle):
    import paper_2512_22036_amd as fusco
    load, groups = _golden()
    assert np.array_equal(fusco.fusco_balance_groups(load), groups)
    rng = np.random.default_rng(8)
    for nodes, gpus in [(1, 1), (2, 8), (8, 8), (8, 4), (3, 5), (16, 8), (64, 8)]:
        for trial in range(10):
            load = rng.integers(0, 5 if trial % 2 else 10 ** 12, size=(nodes, gpus))
            got = fusco.fusco_balance_groups(load)
            assert np.array_equal(got, oracle.balance_groups(load)), (nodes, gpus)
            _check_invariants(load, got)


def test_library_rejects_bad_arguments():
    import ctypes
    import paper_2512_22036_amd as fusco
    lib = fusco.load_library()
    buf = (ctypes.c_int64 * 4)()
    out = (ctypes.c_int32 * 4)()
    assert lib.fusco_balance_groups(None, 2, 2, out) == -1
    assert lib.fusco_balance_groups(buf, 2, 2, None) == -1
    assert lib.fusco_balance_groups(buf, 0, 2, out) == -1
    assert lib.fusco_balance_groups(buf, 2, 0, out) == -1
    assert lib.fusco_balance_groups(buf, 1 << 20, 1 << 10, out) == -1


# ---- the balancer's input: cross-node traffic load of a GPU, from its routing (section 3.4) ----

def _load_golden():
    path = os.path.join(os.path.dirname(__file__), "golden", "cross_node_load_hand_example.txt")
    kv, tokens, loads = {}, [], {}
    for line in open(path):
        if line.startswith("#") or ":" not in line:
            continue
        key, val = line.split(":")
        if key == "token":
            tokens.append([int(v) for v in val.split()])
        elif key == "load_from_node":
            n, b = val.split()
            loads[int(n)] = int(b)
        else:
            kv[key] = int(val)
    return kv, np.array(tokens, dtype=np.int32), loads


def test_cross_node_load_hand_worked_example(oracle):
    kv, A, loads = _load_golden()
    for node, want in loads.items():
        assert oracle.cross_node_load(A, kv["E"], kv["D"], kv["devices_per_node"], node, kv["row_bytes"]) == want


def test_cross_node_load_special_cases_and_plan_relation(oracle):
    from definitions import random_topk
    rng = np.random.default_rng(21)
    for N, k, E, D, dpn in [(50, 4, 16, 8, 2), (33, 8, 64, 8, 4), (20, 2, 6, 6, 1), (40, 3, 12, 4, 4), (10, 5, 10, 1, 1)]:
        A = random_topk(rng, N, k, E)
        pl = oracle.plan(A, E, D)
        nodes = D // dpn
        total = 0
        for home in range(nodes):
            got = oracle.cross_node_load(A, E, D, dpn, home, 16)
            # the same count read off the planner's per-device send rows (built by list appends, not by sets)
            remote = sum(int(pl.send_count[d]) for d in range(D) if d // dpn != home)
            assert got == 16 * remote
            total += got
        # over all home nodes every send row is remote for all nodes but its own
        assert total == 16 * pl.U * (nodes - 1)
        if nodes == 1:
            assert total == 0                      # a single node has no cross-node traffic
