"""Seeded synthetic MoE-shaped inputs shared by the CPU oracle's tests and the HIP path's tests.

This module only draws numbers and shapes them into router outputs and activation
rows.  It contains none of the shuffle's arithmetic (no histogram, scan, slot, dedup,
gather or combine code): both the oracle and the GPU library receive what is made here
as plain input buffers.

Every value is a pure function of (seed, stream, element index) through a counter-based
generator, so the first n tokens of a configuration are the same whether n tokens or the
whole configuration are generated, on any machine.

The five named configurations take their shapes from the paper's benchmark setup
(Table 2: hidden 7168, top-8, 256 experts) and from public model shapes; the routing
itself is synthetic because the paper's captured routing trace is not available.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Optional, Tuple

import numpy as np

__all__ = [
    "MoEConfig", "CONFIGS", "get_config", "make_routing", "make_activations",
    "make_fp8_activations", "make_expert_output", "uniform", "normal", "bf16_bits",
    "bf16_bits_to_f32",
]

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)

# stream ids: one independent sequence per kind of input
STREAM_X, STREAM_LOGITS, STREAM_NOISE, STREAM_PERM, STREAM_Y, STREAM_AUX = 1, 2, 3, 4, 5, 6


def _mix(z: np.ndarray) -> np.ndarray:
    """splitmix64 finaliser on uint64 arrays (wrap-around arithmetic)."""
    with np.errstate(over="ignore"):
        z = (z ^ (z >> np.uint64(30))) * _M1
        z = (z ^ (z >> np.uint64(27))) * _M2
        return z ^ (z >> np.uint64(31))


def _key(seed: int, stream: int) -> np.uint64:
    s = np.array([seed & 0xFFFFFFFFFFFFFFFF], dtype=np.uint64)
    t = np.array([stream & 0xFFFFFFFFFFFFFFFF], dtype=np.uint64)
    with np.errstate(over="ignore"):
        return _mix(s + _GOLDEN * (_mix(t + _GOLDEN) | np.uint64(1)))[0]


def _bits(seed: int, stream: int, start: int, count: int) -> np.ndarray:
    """uint64 word number start..start+count-1 of the (seed, stream) sequence."""
    idx = np.arange(start + 1, start + 1 + count, dtype=np.uint64)
    with np.errstate(over="ignore"):
        return _mix(_key(seed, stream) + idx * _GOLDEN)


def uniform(seed: int, stream: int, start: int, count: int) -> np.ndarray:
    """float64 uniforms strictly inside (0, 1)."""
    b = _bits(seed, stream, start, count)
    return ((b >> np.uint64(11)).astype(np.float64) + 0.5) * (1.0 / 9007199254740992.0)


def normal(seed: int, stream: int, start: int, count: int) -> np.ndarray:
    """float64 standard normals; elements 2m and 2m+1 are the cosine and sine branch of one
    Box-Muller pair drawn from words 2m and 2m+1."""
    m0, m1 = start // 2, (start + count + 1) // 2
    u = uniform(seed, stream, 2 * m0, 2 * (m1 - m0))
    r = np.sqrt(-2.0 * np.log(u[0::2]))
    a = (2.0 * np.pi) * u[1::2]
    z = np.empty(2 * (m1 - m0), dtype=np.float64)
    z[0::2] = r * np.cos(a)
    z[1::2] = r * np.sin(a)
    return z[start - 2 * m0: start - 2 * m0 + count]


def bf16_bits(f: np.ndarray) -> np.ndarray:
    """Round finite float32 values to bfloat16 (nearest even) and return the uint16 patterns."""
    u = np.ascontiguousarray(f, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


@dataclass(frozen=True)
class MoEConfig:
    name: str
    N: int            # tokens
    H: int            # hidden size (elements per row)
    payload: str      # "bf16" or "fp8" (e4m3 bytes + one fp32 scale per 128 elements)
    E: int            # experts
    k: int            # experts per token
    D: int            # virtual expert-parallel devices, E % D == 0
    routing: str      # "uniform" | "normal" | "zipf_limited"
    weights: str      # "softmax" | "sigmoid"
    seed: int
    max_devices: int = 0   # zipf_limited: a token's experts come from at most this many devices
    zipf_s: float = 0.0

    @property
    def P(self) -> int:
        return self.N * self.k

    @property
    def row_bytes(self) -> int:
        return self.H * (2 if self.payload == "bf16" else 1)

    @property
    def aux_row_bytes(self) -> int:
        return (self.H // 128) * 4 if self.payload == "fp8" else 0

    def with_tokens(self, n: int) -> "MoEConfig":
        """Same configuration on its first n tokens."""
        return replace(self, N=int(n))


_SEED0 = 0xF05C0000

CONFIGS = {
    "tiny": MoEConfig("tiny", 4096, 1024, "bf16", 16, 2, 4, "uniform", "softmax", _SEED0 + 1),
    "dsv3": MoEConfig("dsv3", 8192, 7168, "bf16", 256, 8, 8, "normal", "sigmoid", _SEED0 + 2),
    "qwen3": MoEConfig("qwen3", 16384, 4096, "bf16", 128, 8, 16, "normal", "softmax", _SEED0 + 3),
    "skewed": MoEConfig("skewed", 32768, 7168, "bf16", 256, 8, 8, "zipf_limited", "softmax",
                        _SEED0 + 4, max_devices=4, zipf_s=1.2),
    "decode_fp8": MoEConfig("decode_fp8", 128, 7168, "fp8", 256, 8, 64, "normal", "softmax", _SEED0 + 5),
}


def get_config(name: str) -> MoEConfig:
    return CONFIGS[name]


def _topk_desc(score: np.ndarray, k: int) -> np.ndarray:
    """Indices of the k largest entries per row, descending; equal scores go to the lower index."""
    order = np.argsort(-score, axis=1, kind="stable")
    return order[:, :k]


def make_routing(cfg: MoEConfig) -> Tuple[np.ndarray, np.ndarray]:
    """Router output for cfg: (topk_idx int32 [N,k], gate weights float32 [N,k]).

    The j order of a token's k entries is descending score and is part of the input."""
    N, E, k, D = cfg.N, cfg.E, cfg.k, cfg.D
    if cfg.routing == "uniform":
        score = uniform(cfg.seed, STREAM_LOGITS, 0, N * E).reshape(N, E)
        idx = _topk_desc(score, k)
    elif cfg.routing == "normal":
        score = normal(cfg.seed, STREAM_LOGITS, 0, N * E).reshape(N, E)
        idx = _topk_desc(score, k)
    elif cfg.routing == "zipf_limited":
        # popularity rank of each expert: a seeded permutation (argsort of uniforms)
        rank = np.argsort(np.argsort(uniform(cfg.seed, STREAM_PERM, 0, E), kind="stable"), kind="stable") + 1
        logp = -cfg.zipf_s * np.log(rank.astype(np.float64))
        logp -= np.log(np.sum(np.exp(logp)))
        g = -np.log(-np.log(uniform(cfg.seed, STREAM_NOISE, 0, N * E))).reshape(N, E)
        score = logp[None, :] + g
        eloc = E // D
        per_dev = np.sort(score.reshape(N, D, eloc), axis=2)
        dev_score = per_dev[:, :, -1] + per_dev[:, :, -2] if eloc >= 2 else per_dev[:, :, -1]
        keep = _topk_desc(dev_score, min(cfg.max_devices, D))
        allowed = np.zeros((N, D), dtype=bool)
        np.put_along_axis(allowed, keep, True, axis=1)
        masked = np.where(np.repeat(allowed, eloc, axis=1), score, -np.inf)
        idx = _topk_desc(masked, k)
    else:
        raise ValueError(cfg.routing)
    chosen = np.take_along_axis(score, idx, axis=1)
    if cfg.weights == "softmax":
        z = np.exp(chosen - chosen.max(axis=1, keepdims=True))
    elif cfg.weights == "sigmoid":
        z = 1.0 / (1.0 + np.exp(-chosen))
    else:
        raise ValueError(cfg.weights)
    w = z / z.sum(axis=1, keepdims=True)
    return np.ascontiguousarray(idx, dtype=np.int32), np.ascontiguousarray(w, dtype=np.float32)


def _normal_bf16_rows(seed: int, stream: int, row0: int, rows: int, H: int) -> np.ndarray:
    out = np.empty((rows, H), dtype=np.uint16)
    step = max(1, (1 << 22) // H)
    for r in range(0, rows, step):
        n = min(step, rows - r)
        z = normal(seed, stream, (row0 + r) * H, n * H).astype(np.float32)
        out[r:r + n] = bf16_bits(z).reshape(n, H)
    return out


def make_activations(cfg: MoEConfig, row0: int = 0, rows: Optional[int] = None) -> np.ndarray:
    """Token rows x ~ N(0,1) rounded to bfloat16, as uint16 bit patterns [rows, H]."""
    rows = cfg.N - row0 if rows is None else rows
    return _normal_bf16_rows(cfg.seed, STREAM_X, row0, rows, cfg.H)


def make_expert_output(cfg: MoEConfig, row0: int = 0, rows: Optional[int] = None) -> np.ndarray:
    """Stand-in expert outputs y ~ N(0,1) in bfloat16 bit patterns, one row per (token, expert) slot."""
    rows = cfg.P - row0 if rows is None else rows
    return _normal_bf16_rows(cfg.seed, STREAM_Y, row0, rows, cfg.H)


def _e4m3_table() -> np.ndarray:
    code = np.arange(0x7F)                      # 0x7F is NaN in e4m3fn; largest finite is 0x7E = 448
    exp, man = code >> 3, code & 7
    return np.where(exp == 0, man / 8.0 * 2.0 ** -6, (1.0 + man / 8.0) * 2.0 ** (exp - 7.0))


def make_fp8_activations(cfg: MoEConfig) -> Tuple[np.ndarray, np.ndarray]:
    """fp8 payload for cfg: (e4m3 bytes uint8 [N,H], float32 scales [N,H/128]).

    x ~ N(0,1) in float32; each block of 128 elements gets scale = amax/448 and is stored as
    round-to-nearest-even e4m3 of x/scale.  The shuffle treats both planes as opaque bytes."""
    N, H = cfg.N, cfg.H
    x = normal(cfg.seed, STREAM_X, 0, N * H).astype(np.float32).reshape(N, H // 128, 128)
    amax = np.abs(x).max(axis=2)
    scale = (amax / np.float32(448.0)).astype(np.float32)
    q = (x / scale[:, :, None]).astype(np.float64)
    tab = _e4m3_table()
    a = np.minimum(np.abs(q), 448.0)
    hi = np.clip(np.searchsorted(tab, a, side="left"), 1, len(tab) - 1)
    lo = hi - 1
    dlo, dhi = a - tab[lo], tab[hi] - a
    pick_hi = (dhi < dlo) | ((dhi == dlo) & ((hi & 1) == 0))
    code = np.where(pick_hi, hi, lo).astype(np.uint8)
    code |= (np.signbit(q).astype(np.uint8) << 7)
    return code.reshape(N, H), np.ascontiguousarray(scale)
