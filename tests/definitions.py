"""Definition-level restatements used to pin the oracle.

Each function counts straight from the defining sentence with nested loops (no sort, no scan, no
cursor), so it shares no mechanism with the oracle's list-append construction.  Tiny inputs only.
"""
from math import comb

import numpy as np


def brute_force_plan(A, E, D):
    """All descriptor arrays from their definitions, O((N k)^2)."""
    A = np.asarray(A)
    N, k = A.shape
    P = N * k
    eloc = E // D
    pairs = [(t, j) for t in range(N) for j in range(k)]
    dev = lambda t, j: int(A[t, j]) // eloc
    B = [set(dev(t, j) for j in range(k)) for t in range(N)]

    pair_slot = np.zeros(P, dtype=np.int32)
    for (t, j) in pairs:
        e = int(A[t, j])
        lower = sum(1 for (t2, j2) in pairs if int(A[t2, j2]) < e)
        before = sum(1 for (t2, j2) in pairs if int(A[t2, j2]) == e and (t2, j2) < (t, j))
        pair_slot[t * k + j] = lower + before
    slot_pair = np.zeros(P, dtype=np.int32)
    slot_token = np.zeros(P, dtype=np.int32)
    for p in range(P):
        slot_pair[pair_slot[p]] = p
        slot_token[pair_slot[p]] = p // k

    pair_first = np.zeros(P, dtype=np.uint8)
    for (t, j) in pairs:
        pair_first[t * k + j] = 0 if any(dev(t, j2) == dev(t, j) for j2 in range(j)) else 1

    def send_row(t, d):
        lower = sum(1 for t2 in range(N) for d2 in B[t2] if d2 < d)
        before = sum(1 for t2 in range(t) if d in B[t2])
        return lower + before

    U = sum(len(b) for b in B)
    send_src = np.zeros(U, dtype=np.int32)
    pair_send_row = np.zeros(P, dtype=np.int32)
    slot_send_row = np.zeros(P, dtype=np.int32)
    for (t, j) in pairs:
        r = send_row(t, dev(t, j))
        send_src[r] = t
        pair_send_row[t * k + j] = r
        slot_send_row[pair_slot[t * k + j]] = r
    exp_count = np.array([sum(1 for (t, j) in pairs if int(A[t, j]) == e) for e in range(E)], dtype=np.int32)
    send_count = np.array([sum(1 for t in range(N) if d in B[t]) for d in range(D)], dtype=np.int32)
    exp_off = np.array([sum(exp_count[:e]) for e in range(E + 1)], dtype=np.int32)
    send_off = np.array([sum(send_count[:d]) for d in range(D + 1)], dtype=np.int32)
    return dict(exp_count=exp_count, exp_off=exp_off, send_count=send_count, send_off=send_off,
                pair_slot=pair_slot, slot_pair=slot_pair, slot_token=slot_token, send_src=send_src,
                pair_send_row=pair_send_row, slot_send_row=slot_send_row, pair_first=pair_first)


PLAN_FIELDS = ("exp_count", "exp_off", "send_count", "send_off", "pair_slot", "slot_pair", "slot_token",
               "send_src", "pair_send_row", "slot_send_row", "pair_first")


def expected_send_rows_per_token(E, k, D):
    """E[U]/N for k distinct experts drawn uniformly at random: D (1 - C(E - E/D, k) / C(E, k))."""
    return D * (1.0 - comb(E - E // D, k) / comb(E, k))


def random_topk(rng, N, k, E, distinct=True):
    if distinct:
        return np.stack([rng.permutation(E)[:k] for _ in range(N)]).astype(np.int32).reshape(N, k)
    return rng.integers(0, E, size=(N, k)).astype(np.int32)


def check_plan_invariants(pl, A):
    """Structural properties every valid plan has (any size)."""
    A = np.asarray(A)
    N, k = A.shape
    P, E, D = N * k, pl.E, pl.D
    eloc = E // D
    flat = A.reshape(-1)
    # counts sum to N k, offsets are the running sums
    assert int(pl.exp_count.sum()) == P
    assert pl.exp_off[0] == 0 and pl.exp_off[E] == P
    assert np.array_equal(np.diff(pl.exp_off), pl.exp_count)
    assert np.array_equal(pl.exp_count, np.bincount(flat, minlength=E))
    # slot maps are inverse permutations
    assert np.array_equal(np.sort(pl.slot_pair), np.arange(P))
    assert np.array_equal(pl.pair_slot[pl.slot_pair], np.arange(P))
    assert np.array_equal(pl.slot_token, pl.slot_pair // k)
    # each expert segment holds exactly that expert's pairs, tokens ascending (pairs ascending)
    seg_expert = np.repeat(np.arange(E), pl.exp_count)
    assert np.array_equal(flat[pl.slot_pair], seg_expert)
    if P > 1:
        same = seg_expert[1:] == seg_expert[:-1]
        assert np.all(pl.slot_pair[1:][same] > pl.slot_pair[:-1][same])
    # level 1
    U = pl.U
    assert int(pl.send_count.sum()) == U and pl.send_off[0] == 0
    assert np.array_equal(np.diff(pl.send_off), pl.send_count)
    if N > 0:
        assert N <= U <= min(P, N * min(k, D))
    dev = flat // eloc
    tok = np.repeat(np.arange(N), k)
    distinct_td = np.unique(tok.astype(np.int64) * D + dev)
    assert U == len(distinct_td)
    assert int(pl.pair_first.sum()) == U
    first_td = (tok.astype(np.int64) * D + dev)[pl.pair_first.astype(bool)]
    assert len(np.unique(first_td)) == U          # exactly one first per distinct (token, device)
    row_dev = np.repeat(np.arange(D), pl.send_count)
    # every send row is a distinct (token, device) the token really targets, tokens ascending per device
    assert np.array_equal(np.sort(pl.send_src.astype(np.int64) * D + row_dev), distinct_td)
    if U > 1:
        same = row_dev[1:] == row_dev[:-1]
        assert np.all(pl.send_src[1:][same] > pl.send_src[:-1][same])
    # dedup keeps every (token, expert) pair reachable: the send row of a slot holds the slot's token
    # and lies in the receive tensor of the slot's device
    assert np.array_equal(pl.send_src[pl.slot_send_row], pl.slot_token)
    assert np.array_equal(row_dev[pl.slot_send_row], seg_expert // eloc)
    assert np.array_equal(pl.slot_send_row, pl.pair_send_row[pl.slot_pair])
    got = np.stack([pl.send_src[pl.slot_send_row], seg_expert], axis=1)
    want = np.stack([tok, flat], axis=1)
    assert np.array_equal(got[np.lexsort((got[:, 1], got[:, 0]))], want[np.lexsort((want[:, 1], want[:, 0]))])
