"""numpy front end of the C oracle in fusco_oracle.c.

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the benchmark's
CPU-baseline leg.  The product package never imports this module, and this module never
imports the product package.  It marshals numpy arrays into the C functions and does no
arithmetic of its own.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "fusco_oracle.c")
_LIB = os.path.join(_HERE, "libfusco_oracle.so")

BF16, F32 = 0, 1


_LIB_SANITIZED = os.path.join(_HERE, "libfusco_oracle_sanitized.so")
# set in the environment of a process that has the AddressSanitizer runtime preloaded: the oracle is then the
# instrumented build (tests/test_oracle_sanitized.py runs the pins that way)
SANITIZED_ENV = "FUSCO_ORACLE_SANITIZED"


def build(force: bool = False, sanitized: bool = False) -> str:
    """Compile the oracle with gcc (plain -O2, no contraction so that only the explicit fmaf fuses).
    sanitized: the same source with AddressSanitizer and UndefinedBehaviorSanitizer, as a library of its own."""
    lib = _LIB_SANITIZED if sanitized else _LIB
    if force or not os.path.exists(lib) or os.path.getmtime(lib) < os.path.getmtime(_SRC):
        tmp = lib + ".tmp%d" % os.getpid()
        extra = ["-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
                 "-fno-sanitize-recover=all"] if sanitized else ["-O2"]
        subprocess.check_call(["gcc", "-std=c11", "-ffp-contract=off", "-fPIC", "-shared", "-Wall", "-Wextra"]
                              + extra + ["-o", tmp, _SRC, "-lm"])
        os.replace(tmp, lib)
    return lib


_lib = None


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build(sanitized=os.environ.get(SANITIZED_ENV) == "1"))
        for name in ("fusco_oracle_plan", "fusco_oracle_dispatch", "fusco_oracle_dispatch_rows",
                     "fusco_oracle_combine_f64",
                     "fusco_oracle_combine_f32", "fusco_oracle_combine_abs_f64",
                     "fusco_oracle_combine_two_hop_f32", "fusco_oracle_segments_copy", "fusco_oracle_tile_order"):
            getattr(_lib, name).restype = ctypes.c_int
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


@dataclass
class Plan:
    """Layout descriptor as the oracle computes it (all int32 unless noted)."""
    N: int
    k: int
    E: int
    D: int
    exp_count: np.ndarray
    exp_off: np.ndarray
    send_count: np.ndarray
    send_off: np.ndarray
    pair_slot: np.ndarray
    slot_pair: np.ndarray
    slot_token: np.ndarray
    send_src: np.ndarray        # [U]
    pair_send_row: np.ndarray
    slot_send_row: np.ndarray
    pair_first: np.ndarray      # uint8

    @property
    def P(self) -> int:
        return self.N * self.k

    @property
    def U(self) -> int:
        return int(self.send_off[self.D])


def plan(topk_idx: np.ndarray, E: int, D: int) -> Plan:
    A = np.ascontiguousarray(topk_idx, dtype=np.int32)
    N, k = A.shape
    P = N * k
    i32 = lambda n: np.full(max(n, 1), -1, dtype=np.int32)[:n]
    out = dict(exp_count=i32(E), exp_off=i32(E + 1), send_count=i32(D), send_off=i32(D + 1),
               pair_slot=i32(P), slot_pair=i32(P), slot_token=i32(P), send_src=i32(N * min(k, D)),
               pair_send_row=i32(P), slot_send_row=i32(P))
    first = np.zeros(P, dtype=np.uint8)
    rc = _load().fusco_oracle_plan(_p(A), N, k, E, D, _p(out["exp_count"]), _p(out["exp_off"]),
                                   _p(out["send_count"]), _p(out["send_off"]), _p(out["pair_slot"]),
                                   _p(out["slot_pair"]), _p(out["slot_token"]), _p(out["send_src"]),
                                   _p(out["pair_send_row"]), _p(out["slot_send_row"]), _p(first))
    if rc != 0:
        raise ValueError("fusco_oracle_plan failed with code %d" % rc)
    U = int(out["send_off"][D])
    out["send_src"] = out["send_src"][:U]
    return Plan(N=N, k=k, E=E, D=D, pair_first=first, **out)


def tile_order(pair_slot: np.ndarray, N: int, k: int, tile_tokens: int) -> np.ndarray:
    """Transfer order of the expert-tensor rows: per tile of tile_tokens tokens, the slots of its pairs ascending,
    padded with -1 to tile_tokens * k entries.  int32 [ceil(N / tile_tokens) * tile_tokens * k]."""
    ps = np.ascontiguousarray(pair_slot, dtype=np.int32)
    tiles = (N + tile_tokens - 1) // tile_tokens
    out = np.full(max(tiles * tile_tokens * k, 1), -7, dtype=np.int32)[:tiles * tile_tokens * k]
    rc = _load().fusco_oracle_tile_order(_p(ps), N, k, tile_tokens, _p(out))
    if rc != 0:
        raise ValueError("fusco_oracle_tile_order failed with code %d" % rc)
    return out


def dispatch(pl: Plan, x: np.ndarray, x_aux: Optional[np.ndarray] = None):
    """Returns (send_buf [U,row], expert_buf [P,row]) and, with an aux plane, also (send_aux, expert_aux).

    x is any 2-D array with N rows; rows are moved as opaque bytes and come back in x's dtype."""
    x = np.ascontiguousarray(x)
    row_bytes = x.shape[1] * x.itemsize
    send_buf = np.empty((pl.U, x.shape[1]), dtype=x.dtype)
    expert_buf = np.empty((pl.P, x.shape[1]), dtype=x.dtype)
    if x_aux is not None:
        x_aux = np.ascontiguousarray(x_aux)
        aux_bytes = x_aux.shape[1] * x_aux.itemsize
        send_aux = np.empty((pl.U, x_aux.shape[1]), dtype=x_aux.dtype)
        expert_aux = np.empty((pl.P, x_aux.shape[1]), dtype=x_aux.dtype)
    else:
        aux_bytes, send_aux, expert_aux = 0, None, None
    rc = _load().fusco_oracle_dispatch(_p(x), ctypes.c_int64(row_bytes), _p(x_aux), ctypes.c_int64(aux_bytes),
                                       pl.U, pl.P, _p(pl.send_src), _p(pl.slot_send_row),
                                       _p(send_buf), _p(send_aux), _p(expert_buf), _p(expert_aux))
    if rc != 0:
        raise ValueError("fusco_oracle_dispatch failed with code %d" % rc)
    if x_aux is None:
        return send_buf, expert_buf
    return send_buf, expert_buf, send_aux, expert_aux


def dispatch_rows(pl: Plan, x: np.ndarray, slots) -> np.ndarray:
    """Rows `slots` of the expert-activation tensor, without building the whole tensor."""
    x = np.ascontiguousarray(x)
    slots = np.ascontiguousarray(slots, dtype=np.int32)
    out = np.empty((len(slots), x.shape[1]), dtype=x.dtype)
    rc = _load().fusco_oracle_dispatch_rows(_p(x), ctypes.c_int64(x.shape[1] * x.itemsize), pl.P, _p(pl.send_src),
                                            _p(pl.slot_send_row), _p(slots), len(slots), _p(out))
    if rc != 0:
        raise ValueError("fusco_oracle_dispatch_rows failed with code %d" % rc)
    return out


def _y_args(y: np.ndarray):
    y = np.ascontiguousarray(y)
    if y.dtype == np.uint16:
        return y, BF16
    if y.dtype == np.float32:
        return y, F32
    raise TypeError("y must be uint16 (bfloat16 bit patterns) or float32")


def _tok_args(tokens, N):
    if tokens is None:
        return None, 0, N
    tokens = np.ascontiguousarray(tokens, dtype=np.int32)
    return tokens, len(tokens), len(tokens)


def combine_f64(y: np.ndarray, w: np.ndarray, pair_slot: np.ndarray, tokens=None) -> np.ndarray:
    """Weighted sum in double precision, [rows, H] float64."""
    y, dt = _y_args(y)
    w = np.ascontiguousarray(w, dtype=np.float32)
    N, k = w.shape
    tok, nt, rows = _tok_args(tokens, N)
    out = np.empty((rows, y.shape[1]), dtype=np.float64)
    rc = _load().fusco_oracle_combine_f64(_p(y), dt, _p(w), _p(np.ascontiguousarray(pair_slot, dtype=np.int32)),
                                          N, k, y.shape[1], _p(tok), nt, _p(out))
    if rc != 0:
        raise ValueError("fusco_oracle_combine_f64 failed with code %d" % rc)
    return out


def combine_abs_f64(y: np.ndarray, w: np.ndarray, pair_slot: np.ndarray, tokens=None) -> np.ndarray:
    """sum_j |w_j * y_j| in double precision: the scale of the combine tolerance."""
    y, dt = _y_args(y)
    w = np.ascontiguousarray(w, dtype=np.float32)
    N, k = w.shape
    tok, nt, rows = _tok_args(tokens, N)
    out = np.empty((rows, y.shape[1]), dtype=np.float64)
    rc = _load().fusco_oracle_combine_abs_f64(_p(y), dt, _p(w),
                                              _p(np.ascontiguousarray(pair_slot, dtype=np.int32)),
                                              N, k, y.shape[1], _p(tok), nt, _p(out))
    if rc != 0:
        raise ValueError("fusco_oracle_combine_abs_f64 failed with code %d" % rc)
    return out


def combine_f32(y: np.ndarray, w: np.ndarray, pair_slot: np.ndarray, tokens=None):
    """Single-precision fused-multiply-add sum in j order: (float32 [rows,H], bfloat16 bits uint16 [rows,H])."""
    y, dt = _y_args(y)
    w = np.ascontiguousarray(w, dtype=np.float32)
    N, k = w.shape
    tok, nt, rows = _tok_args(tokens, N)
    o32 = np.empty((rows, y.shape[1]), dtype=np.float32)
    o16 = np.empty((rows, y.shape[1]), dtype=np.uint16)
    rc = _load().fusco_oracle_combine_f32(_p(y), dt, _p(w), _p(np.ascontiguousarray(pair_slot, dtype=np.int32)),
                                          N, k, y.shape[1], _p(tok), nt, _p(o32), _p(o16))
    if rc != 0:
        raise ValueError("fusco_oracle_combine_f32 failed with code %d" % rc)
    return o32, o16


def combine_two_hop_f32(pl: Plan, y: np.ndarray, w: np.ndarray, tokens=None, want_partial: bool = False):
    """Combine along the two levels in reverse (per-device partial sums, then their sum).
    Returns (float32 [rows,H], bfloat16 bits [rows,H]) and, with want_partial, also the [U,H] partial rows."""
    y, dt = _y_args(y)
    w = np.ascontiguousarray(w, dtype=np.float32)
    N, k = w.shape
    tok, nt, rows = _tok_args(tokens, N)
    H = y.shape[1]
    o32 = np.empty((rows, H), dtype=np.float32)
    o16 = np.empty((rows, H), dtype=np.uint16)
    part = np.full((pl.U, H), np.nan, dtype=np.float32) if want_partial else None
    rc = _load().fusco_oracle_combine_two_hop_f32(_p(y), dt, _p(w), _p(pl.pair_slot), _p(pl.pair_send_row),
                                                  _p(pl.pair_first), N, k, H, _p(tok), nt, _p(part), _p(o32), _p(o16))
    if rc != 0:
        raise ValueError("fusco_oracle_combine_two_hop_f32 failed with code %d" % rc)
    return (o32, o16, part) if want_partial else (o32, o16)


def cross_node_load(topk_idx: np.ndarray, E: int, D: int, devices_per_node: int, home_node: int, row_bytes: int) -> int:
    """Cross-node traffic load of one GPU (paper section 3.4: the volume it must transmit to remote nodes),
    counted from the routing itself: every token sends one row of row_bytes to each distinct destination
    device (experts placed in contiguous blocks of E / D), and only devices on another node than the GPU's
    own count.  Plain loops over the token-expert matrix; no use of the planner's arrays."""
    A = np.asarray(topk_idx)
    eloc = E // D
    total = 0
    for t in range(A.shape[0]):
        devices = set(int(e) // eloc for e in A[t])
        total += sum(1 for d in devices if d // devices_per_node != home_node)
    return total * int(row_bytes)


def balance_groups(load) -> np.ndarray:
    """Online Group-Balanced Assignment (Algorithm 1 of the paper), step by step in its notation.

    load[n][g] is the cross-node traffic load of GPU g of node n.  Returns G with G[i][n] = the GPU of
    node n that belongs to communication group g_i.  Readings where the algorithm is silent: equal
    loads keep ascending GPU index; "circular shift by n" moves position n of P_n to the front."""
    load = np.asarray(load)
    nodes, gpus = load.shape
    P = [sorted(range(gpus), key=lambda g, n=n: (-int(load[n][g]), g)) for n in range(nodes)]   # sort by descending load
    S = [P[n][n % gpus:] + P[n][:n % gpus] for n in range(nodes)]                              # circular shift by n
    G = np.empty((gpus, nodes), dtype=np.int32)
    for i in range(gpus):                                                                       # form groups
        for n in range(nodes):
            G[i][n] = S[n][i]
    return G


def segments_copy(src: np.ndarray, size, src_off=None, dst_off=None, dst_bytes: Optional[int] = None,
                  slice_bytes: int = 0, fill_value: int = 0):
    """Move n segments from src (uint8) into a new uint8 buffer of dst_bytes (default: total size).
    src_off / dst_off None means that side is the contiguous stream.  Returns dst, or (dst, slice_fill)
    when slice_bytes > 0."""
    src = np.ascontiguousarray(src, dtype=np.uint8)
    size = np.ascontiguousarray(size, dtype=np.uint64)
    so = None if src_off is None else np.ascontiguousarray(src_off, dtype=np.uint64)
    do = None if dst_off is None else np.ascontiguousarray(dst_off, dtype=np.uint64)
    total = int(size.sum())
    dst = np.full(total if dst_bytes is None else dst_bytes, fill_value, dtype=np.uint8)
    fill = np.zeros((total + slice_bytes - 1) // slice_bytes, dtype=np.uint32) if slice_bytes > 0 else None
    rc = _load().fusco_oracle_segments_copy(_p(src), _p(so), _p(dst), _p(do), _p(size), ctypes.c_int64(len(size)),
                                            ctypes.c_uint64(slice_bytes), _p(fill))
    if rc != 0:
        raise ValueError("fusco_oracle_segments_copy failed with code %d" % rc)
    return (dst, fill) if slice_bytes > 0 else dst
