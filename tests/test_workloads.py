"""The seeded input generator: reproducible, prefix-stable, and shaped as the recipe says."""
import numpy as np
import pytest

import workloads as W


def test_streams_are_reproducible_and_prefix_stable():
    a = W.normal(123, W.STREAM_X, 0, 1000)
    assert np.array_equal(a, W.normal(123, W.STREAM_X, 0, 1000))
    assert np.array_equal(a[333:777], W.normal(123, W.STREAM_X, 333, 444))
    assert not np.array_equal(a, W.normal(124, W.STREAM_X, 0, 1000))
    assert not np.array_equal(a, W.normal(123, W.STREAM_Y, 0, 1000))
    u = W.uniform(9, 1, 0, 200000)
    assert 0.0 < u.min() and u.max() < 1.0 and abs(u.mean() - 0.5) < 0.005
    z = W.normal(9, 2, 0, 400000)
    assert abs(z.mean()) < 0.01 and abs(z.std() - 1.0) < 0.01 and abs(np.mean(z ** 4) - 3.0) < 0.1


def test_known_first_words():
    # fixed values guard against silent changes of the generator (all seeded inputs depend on it)
    assert W._bits(1, 1, 0, 2).tolist() == [0xE5CCA583BB90F8BA, 0x1F659629E8B001C1]
    assert np.allclose(W.normal(1, 1, 0, 2), [0.33341724640337866, 0.3236886081787438], rtol=1e-12)
    assert W.bf16_bits(np.array([1.0, -2.0, 0.1], dtype=np.float32)).tolist() == [0x3F80, 0xC000, 0x3DCD]


@pytest.mark.parametrize("name", list(W.CONFIGS))
def test_routing_shape_and_contract(name):
    cfg = W.get_config(name).with_tokens(min(W.get_config(name).N, 2048))
    idx, w = W.make_routing(cfg)
    assert idx.shape == (cfg.N, cfg.k) and idx.dtype == np.int32
    assert w.shape == (cfg.N, cfg.k) and w.dtype == np.float32
    assert idx.min() >= 0 and idx.max() < cfg.E
    assert all(len(set(r)) == cfg.k for r in idx.tolist())       # experts of a token are distinct
    assert np.allclose(w.sum(1), 1.0, atol=1e-6) and w.min() > 0
    assert np.all(np.diff(w, axis=1) <= 1e-7)                   # descending score order
    full_idx, full_w = W.make_routing(W.get_config(name).with_tokens(cfg.N + 5))
    assert np.array_equal(full_idx[:cfg.N], idx) and np.array_equal(full_w[:cfg.N], w)


def test_skewed_config_is_skewed_and_device_limited():
    cfg = W.get_config("skewed").with_tokens(4096)
    idx, _ = W.make_routing(cfg)
    d = idx // (cfg.E // cfg.D)
    assert max(len(set(r)) for r in d.tolist()) <= 4
    counts = np.bincount(idx.reshape(-1), minlength=cfg.E)
    assert counts.max() > 8 * np.median(counts)


def test_activations():
    cfg = W.get_config("tiny")
    x = W.make_activations(cfg, rows=64)
    assert x.shape == (64, cfg.H) and x.dtype == np.uint16
    assert np.array_equal(x[10:20], W.make_activations(cfg, row0=10, rows=10))
    f = W.bf16_bits_to_f32(x)
    assert abs(f.mean()) < 0.02 and abs(f.std() - 1.0) < 0.02


def test_fp8_payload():
    cfg = W.get_config("decode_fp8")
    q, s = W.make_fp8_activations(cfg)
    assert q.shape == (128, 7168) and q.dtype == np.uint8 and s.shape == (128, 56) and s.dtype == np.float32
    assert cfg.row_bytes == 7168 and cfg.aux_row_bytes == 224
    assert np.all((q & 0x7F) != 0x7F)                 # no NaN codes
    assert np.all((q.reshape(128, 56, 128) & 0x7F).max(axis=2) == 0x7E)   # each block reaches +-448
    import torch
    deq = torch.from_numpy(q).view(torch.float8_e4m3fn).float().numpy().reshape(128, 56, 128) * s[:, :, None]
    x = W.normal(cfg.seed, W.STREAM_X, 0, 128 * 7168).reshape(128, 56, 128)
    assert np.max(np.abs(deq - x) / np.abs(x).max(axis=2, keepdims=True)) < 1.0 / 16
