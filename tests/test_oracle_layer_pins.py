"""Pins for the oracle's layer functions (projections, LayerNorm, decoupled RoPE, W_O): closed
forms, invariants, loops written here, and a second route through the paper's equations (the
absorbed form of Eq. (obsorb) / (with-rope) against the two-stage form the oracle follows).
CPU only."""
import math

import numpy as np
import pytest

from oracle import mtla_oracle as O


def layer_problem(seed, T=7, d=12, n_h=3, d_h=4, r=8, d_rope=4, d_y=5, s=2):
    g = np.random.default_rng(seed)
    return dict(
        x=g.standard_normal((T, d)),
        w_q=g.standard_normal((n_h * d_h, d)) / math.sqrt(d), w_qr=g.standard_normal((n_h * d_rope, d)) / math.sqrt(d),
        w_r=g.standard_normal((r, d)) / math.sqrt(d), w_kr=g.standard_normal((d_rope, d)) / math.sqrt(d),
        w_o=g.standard_normal((d, n_h * d_h)) / math.sqrt(n_h * d_h),
        hyp_A=g.standard_normal((d_y, r)) / math.sqrt(r), hyp_G=g.standard_normal((-(-T // s), d_y)),
        w_uk=g.standard_normal((n_h, d_h, r)) / math.sqrt(r), w_uv=g.standard_normal((n_h, r, d_h)) / math.sqrt(r),
        n_h=n_h, d_h=d_h, r=r, d_rope=d_rope, s=s, scale=1.0 / math.sqrt(d_h))


# ------------------------------------------------------------------ LayerNorm
def test_layer_norm_closed_forms():
    v = np.array([1.0, 2.0, 3.0, 4.0])                       # mean 2.5, variance 1.25
    y = O.layer_norm(v, eps=0.0)
    assert np.allclose(y, (v - 2.5) / math.sqrt(1.25), rtol=0, atol=1e-15)
    g = np.random.default_rng(0)
    v = g.standard_normal(256) * 3.0 + 5.0
    y = O.layer_norm(v, eps=1e-5)
    assert abs(y.mean()) < 1e-14
    var = v.var()
    assert abs(y.var() - var / (var + 1e-5)) < 1e-12          # exact effect of eps
    # invariant under a shift of the input; a scale only enters through eps
    assert np.allclose(O.layer_norm(v + 17.0), y, atol=1e-12)
    assert np.allclose(O.layer_norm(4.0 * v, eps=16.0 * 1e-5), y, atol=1e-12)
    # affine part
    gamma, beta = g.standard_normal(256), g.standard_normal(256)
    assert np.allclose(O.layer_norm(v, 1e-5, gamma, beta), y * gamma + beta, atol=1e-14)


def test_layer_norm_constant_vector_is_zero():
    assert np.all(O.layer_norm(np.full(8, 3.25)) == 0.0)


# ------------------------------------------------------------------ RoPE
def test_rope_is_a_plane_rotation_per_pair():
    # d = 2: one pair, angle = pos (base^0 = 1): textbook 2-D rotation
    for pos in (0, 1, 5):
        out = O.rope(np.array([1.0, 0.0]), pos)
        assert np.allclose(out, [math.cos(pos), math.sin(pos)], atol=1e-15)
    # d = 4, base 100: second pair turns by pos * 100^(-2/4) = pos / 10
    out = O.rope(np.array([0.0, 0.0, 0.0, 2.0]), 3, base=100.0)
    assert np.allclose(out, [0.0, 0.0, -2.0 * math.sin(0.3), 2.0 * math.cos(0.3)], atol=1e-15)


def test_rope_identity_norm_and_relative_position():
    g = np.random.default_rng(1)
    a, b = g.standard_normal(32), g.standard_normal(32)
    assert np.array_equal(O.rope(a, 0), a)
    assert abs(np.linalg.norm(O.rope(a, 37)) - np.linalg.norm(a)) < 1e-13
    # <R_m a, R_n b> depends on m - n only
    for m, n in ((5, 3), (40, 38), (2, 0)):
        assert abs(O.rope(a, m) @ O.rope(b, n) - O.rope(a, m - n) @ b) < 1e-12
    # composition of rotations
    assert np.allclose(O.rope(O.rope(a, 3), 4), O.rope(a, 7), atol=1e-13)
    # heads are rotated independently with the same angles
    A = g.standard_normal((3, 8))
    R = O.rope(A, 9)
    for h in range(3):
        assert np.allclose(R[h], O.rope(A[h], 9), atol=0)


# ------------------------------------------------------------------ projections and the whole layer
def test_layer_front_against_loops():
    P = layer_problem(2)
    x, pos = P["x"][4], 4
    q, qr, c, kr = O.layer_front(x, pos, P["w_q"], P["w_qr"], P["w_r"], P["w_kr"], P["n_h"])
    d = len(x)
    for h in range(P["n_h"]):
        for k in range(P["d_h"]):
            assert abs(q[h, k] - sum(x[i] * P["w_q"][h * P["d_h"] + k, i] for i in range(d))) < 1e-13
    raw_qr = np.array([[sum(x[i] * P["w_qr"][h * P["d_rope"] + k, i] for i in range(d)) for k in range(P["d_rope"])]
                       for h in range(P["n_h"])])
    for h in range(P["n_h"]):
        for k in range(P["d_rope"] // 2):
            ang = pos * 10000.0 ** (-2.0 * k / P["d_rope"])
            re = raw_qr[h, 2 * k] * math.cos(ang) - raw_qr[h, 2 * k + 1] * math.sin(ang)
            im = raw_qr[h, 2 * k] * math.sin(ang) + raw_qr[h, 2 * k + 1] * math.cos(ang)
            assert abs(qr[h, 2 * k] - re) < 1e-13 and abs(qr[h, 2 * k + 1] - im) < 1e-13
    raw_c = np.array([sum(x[i] * P["w_r"][n, i] for i in range(d)) for n in range(P["r"])])
    mu = sum(raw_c) / len(raw_c)
    sd = math.sqrt(sum((t - mu) ** 2 for t in raw_c) / len(raw_c) + 1e-5)
    assert np.allclose(c, (raw_c - mu) / sd, atol=1e-13)
    assert kr.shape == (P["d_rope"],)
    assert abs(np.linalg.norm(kr) - np.linalg.norm(P["w_kr"] @ x)) < 1e-13


def test_layer_decode_step_is_front_then_path_then_w_o():
    # the layer function equals the path functions (pinned elsewhere) fed with projections made here
    P = layer_problem(3)
    T = len(P["x"])
    cache_a = O.LatentCache(P["r"], P["d_rope"], P["s"])
    cache_b = O.LatentCache(P["r"], P["d_rope"], P["s"])
    for t in range(T):
        y, out, w, slot = O.layer_decode_step(cache_a, P["x"][t], P["w_q"], P["w_qr"], P["w_r"], P["w_kr"], P["w_o"],
                                              P["hyp_A"], None, P["hyp_G"], P["w_uk"], P["w_uv"], P["scale"])
        x = P["x"][t]
        raw_c = P["w_r"] @ x
        c = (raw_c - raw_c.mean()) / np.sqrt(raw_c.var() + 1e-5)
        k = np.arange(P["d_rope"] // 2)
        ang = t * 10000.0 ** (-2.0 * k / P["d_rope"])
        rot = lambda v: np.stack([v[..., 0::2] * np.cos(ang) - v[..., 1::2] * np.sin(ang),
                                  v[..., 0::2] * np.sin(ang) + v[..., 1::2] * np.cos(ang)], axis=-1).reshape(v.shape)
        q = (P["w_q"] @ x).reshape(P["n_h"], P["d_h"])
        qr = rot((P["w_qr"] @ x).reshape(P["n_h"], P["d_rope"]))
        kr = rot(P["w_kr"] @ x)
        w_b, slot_b, _ = O.append_token(cache_b, c, kr, P["hyp_A"], None, P["hyp_G"])
        out_b, _, _, _ = O.decode_attn(cache_b, q, qr, P["w_uk"], P["w_uv"], P["scale"])
        assert slot == slot_b == t // P["s"] and abs(w - w_b) < 1e-13
        assert np.allclose(out, out_b, atol=1e-12)
        assert np.allclose(y, P["w_o"] @ out_b.reshape(-1), atol=1e-12)


def test_layer_equals_the_absorbed_form():
    # Eq. (obsorb) / (with-rope): W_K absorbed into W_Q and W_V into W_O give the same layer output
    P = layer_problem(4, T=9, s=3)
    n_h, d_h, r, d = P["n_h"], P["d_h"], P["r"], P["x"].shape[1]
    # per head: W_QK^(h) [r, d] = W_K^(h) W_Q^(h),  W_VO^(h) [d, r] = W_O^(h) W_V^(h)T
    w_qk = [P["w_uk"][h].T @ P["w_q"][h * d_h:(h + 1) * d_h] for h in range(n_h)]
    w_vo = [P["w_o"][:, h * d_h:(h + 1) * d_h] @ P["w_uv"][h].T for h in range(n_h)]
    cache = O.LatentCache(r, P["d_rope"], P["s"])
    for t in range(len(P["x"])):
        y, _, _, _ = O.layer_decode_step(cache, P["x"][t], P["w_q"], P["w_qr"], P["w_r"], P["w_kr"], P["w_o"],
                                         P["hyp_A"], None, P["hyp_G"], P["w_uk"], P["w_uv"], P["scale"])
        C_hat, KR_hat = cache.arrays()
        x = P["x"][t]
        qr = O.rope((P["w_qr"] @ x).reshape(n_h, -1), t)
        y_abs = np.zeros(d)
        for h in range(n_h):
            e = (C_hat @ (w_qk[h] @ x) + KR_hat @ qr[h]) * P["scale"]
            p = np.exp(e - e.max())
            p /= p.sum()
            y_abs += w_vo[h] @ (p @ C_hat)
        assert np.allclose(y, y_abs, atol=1e-12)


@pytest.mark.parametrize("s", [1, 2, 4])
def test_layer_positions_follow_the_token_count(s):
    # the rotation uses the 0-based token position i - 1, whatever the stride; the slot key is the
    # key of the newest token folded into the slot
    P = layer_problem(5, T=8, s=s)
    cache = O.LatentCache(P["r"], P["d_rope"], s)
    for t in range(8):
        O.layer_decode_step(cache, P["x"][t], P["w_q"], P["w_qr"], P["w_r"], P["w_kr"], P["w_o"],
                            P["hyp_A"], None, np.tile(P["hyp_G"], (s, 1)), P["w_uk"], P["w_uv"], P["scale"])
        _, KR_hat = cache.arrays()
        assert np.allclose(KR_hat[-1], O.rope(P["w_kr"] @ P["x"][t], t), atol=1e-13)


@pytest.mark.parametrize("s,T", [(1, 6), (2, 9), (3, 10), (4, 8)])
def test_layer_prefill_equals_the_incremental_layer(s, T):
    # the parallel form of the whole layer gives, row by row, what one layer_decode_step per token gives
    P = layer_problem(6 + s, T=T, s=s)
    y_par, out_par = O.layer_prefill(P["x"], P["w_q"], P["w_qr"], P["w_r"], P["w_kr"], P["w_o"], P["hyp_A"], None,
                                     P["hyp_G"], P["w_uk"], P["w_uv"], s, P["scale"])
    cache = O.LatentCache(P["r"], P["d_rope"], s)
    for t in range(T):
        y, out, _, _ = O.layer_decode_step(cache, P["x"][t], P["w_q"], P["w_qr"], P["w_r"], P["w_kr"], P["w_o"],
                                           P["hyp_A"], None, P["hyp_G"], P["w_uk"], P["w_uv"], P["scale"])
        assert np.allclose(y_par[t], y, atol=1e-12) and np.allclose(out_par[t], out, atol=1e-12)
    # a subset of rows is the same rows
    y_sub, _ = O.layer_prefill(P["x"], P["w_q"], P["w_qr"], P["w_r"], P["w_kr"], P["w_o"], P["hyp_A"], None,
                               P["hyp_G"], P["w_uk"], P["w_uv"], s, P["scale"], rows=[0, T - 1])
    assert np.array_equal(y_sub, y_par[[0, T - 1]])


def test_layer_prefill_first_row_is_the_value_path_of_one_token():
    # row 0 sees only itself: y_0 = W_O concat_h(w_0 c_0 W_V^(h)), whatever the queries are
    P = layer_problem(12, T=5, s=2)
    y, _ = O.layer_prefill(P["x"], P["w_q"], P["w_qr"], P["w_r"], P["w_kr"], P["w_o"], P["hyp_A"], None, P["hyp_G"],
                           P["w_uk"], P["w_uv"], 2, P["scale"], rows=[0])
    raw = P["w_r"] @ P["x"][0]
    c0 = (raw - raw.mean()) / math.sqrt(raw.var() + 1e-5)
    w0 = 1.0 / (1.0 + math.exp(-float((P["hyp_A"] @ c0) @ P["hyp_G"][0])))
    o = np.concatenate([(w0 * c0) @ P["w_uv"][h] for h in range(P["n_h"])])
    assert np.allclose(y[0], P["w_o"] @ o, atol=1e-12)
