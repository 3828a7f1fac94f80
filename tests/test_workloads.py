"""Checks of the synthetic-input generators (CPU only)."""
import math

import numpy as np
import pytest
import torch

import workloads as W


def test_bf16_round_matches_torch_round_to_nearest_even():
    g = np.random.default_rng(0)
    x = np.concatenate([
        g.standard_normal(20000).astype(np.float32) * 3,
        np.array([0.0, -0.0, 1.0, 1.00390625, 1.001953125, 1.005859375, 255.5, 3.0e-40, 65504.0, -7.999], np.float32),
    ])
    ref = torch.from_numpy(x).to(torch.bfloat16)
    assert np.array_equal(W.bf16_round(x), ref.float().numpy())
    assert np.array_equal(W.bf16_bits(x), ref.view(torch.int16).numpy().view(np.uint16))
    assert np.array_equal(W.bits_to_f32(W.bf16_bits(x)), W.bf16_round(x))
    # ties go to even: 1 + 2^-8 is halfway between 1 and 1 + 2^-7
    assert W.bf16_round(np.array([1.00390625], np.float32))[0] == 1.0
    assert W.bf16_round(np.array([1.01171875], np.float32))[0] == 1.015625


def test_rope_depends_on_relative_position_only():
    g = np.random.default_rng(1)
    a, b = g.standard_normal(32), g.standard_normal(32)
    ref = W.rope_rotate(a, 17) @ W.rope_rotate(b, 5)
    for shift in (0, 3, 1000):
        assert W.rope_rotate(a, 17 + shift) @ W.rope_rotate(b, 5 + shift) == pytest.approx(ref, abs=1e-9)
    assert np.allclose(W.rope_rotate(a, 0), a)
    assert np.linalg.norm(W.rope_rotate(a, 123)) == pytest.approx(np.linalg.norm(a))
    # first pair turns by exactly `pos` radians
    v = np.zeros(8); v[0] = 1.0
    out = W.rope_rotate(v, 0.5)
    assert out[0] == pytest.approx(math.cos(0.5)) and out[1] == pytest.approx(math.sin(0.5))


def test_sinusoidal_pe_values():
    pe = W.sinusoidal_pe(np.arange(0, 4), 6)
    assert np.allclose(pe[0], [0, 1, 0, 1, 0, 1])
    assert pe[3, 0] == pytest.approx(math.sin(3.0)) and pe[3, 1] == pytest.approx(math.cos(3.0))
    assert pe[2, 4] == pytest.approx(math.sin(2.0 / 10000 ** (4 / 6)))


def test_layer_norm_moments():
    x = np.random.default_rng(2).standard_normal((7, 64)) * 5 + 3
    y = W.layer_norm(x)
    assert np.allclose(y.mean(axis=1), 0, atol=1e-12)
    assert np.allclose(y.var(axis=1), 1, atol=1e-4)


def test_workload_table_matches_the_benchmark_configs():
    w = W.WORKLOADS
    s = w["speech_bf16"]
    assert (s.batch, s.d_model, s.n_heads, s.d_head, s.r, s.d_rope, s.stride, s.prefix, s.steps, s.dtype) == \
        (16, 512, 8, 64, 256, 32, 2, 1024, 256, "bf16")
    t = w["tiny_f32"]
    assert (t.batch, t.d_model, t.n_heads, t.d_head, t.r, t.d_rope, t.stride, t.prefix, t.steps, t.dtype) == \
        (1, 256, 4, 64, 64, 32, 2, 256, 64, "f32")
    l = w["long_bf16"]
    assert (l.batch, l.n_heads, l.d_head, l.r, l.d_rope, l.stride, l.prefix, l.steps) == (8, 32, 128, 512, 64, 4, 32768, 128)
    r = w["ragged_bf16"]
    assert (r.batch, r.n_heads, r.d_head, r.r, r.d_rope, r.stride, r.prefix, r.steps) == (256, 16, 128, 512, 64, 2, (512, 4096), 64)
    L = W.prefix_lengths(r)
    assert L.shape == (256,) and L.min() >= 512 and L.max() <= 4096 and len(set(L.tolist())) > 100
    assert np.array_equal(L, W.prefix_lengths(r))
    assert s.max_slots == (1024 + 256) // 2 and l.max_slots == (32768 + 128) // 4
    for k in ("prefill_s2", "prefill_s4"):
        assert (w[k].batch, w[k].prefix, w[k].n_heads, w[k].d_head, w[k].r) == (8, 4096, 16, 128, 512)


def test_tokens_are_reproducible_storage_exact_and_range_independent():
    wl = W.WORKLOADS["speech_bf16"].scaled(d_model=64, prefix=40, steps=8)
    wts = W.make_weights(wl)
    full = W.make_tokens(wl, wts, 3, 0, 48)
    part = W.make_tokens(wl, wts, 3, 1020, 1030)       # straddles an RNG block edge
    again = W.make_tokens(wl, wts, 3, 1020, 1030)
    sub = W.make_tokens(wl, wts, 3, 10, 20)
    assert np.array_equal(full.c[10:20], sub.c) and np.array_equal(full.q_rope[10:20], sub.q_rope)
    assert np.array_equal(part.c, again.c) and part.c.shape == (10, wl.r)
    for a in (full.c, full.kr, full.q, full.q_rope, wts.w_uk, wts.w_uv, wts.hyp_A, wts.hyp_G):
        assert a.dtype == np.float32 and np.array_equal(W.bf16_round(a), a)
    # different sequences differ; latents are LayerNorm outputs
    other = W.make_tokens(wl, wts, 4, 0, 48)
    assert not np.array_equal(other.c, full.c)
    assert abs(full.c.mean()) < 0.05 and abs(full.c.std() - 1) < 0.05
    # library-layout weights are views of the same W_K / W_V
    h, k, n = 5, 7, 11
    assert wts.w_uk[h, k, n] == wts.W_K[n, h * wl.d_head + k]
    assert wts.w_uv[h, n, k] == wts.W_V[n, h * wl.d_head + k]
    assert wts.hyp_G.shape == (wl.max_slots, wl.d_hyper)
