"""GPU parity of mtla_layer_decode_step (projections, LayerNorm, decoupled RoPE, the decode step, W_O)
against the float64 oracle's layer functions, through the C-ABI.  Both sides start from the same
rounded token stream x and the same rounded weights; every sequence is built token by token from an
empty cache, so the rotation positions, the LayerNorm'ed latents in the cache and the merge weights
all come from the library's own projections.  Integers exact; floating point within 2e-2 (bf16)."""
import numpy as np
import pytest
import torch

import workloads as W
from oracle import mtla_oracle as O
from tests import harness as H

pytestmark = pytest.mark.gpu


def _run(wl, n_tokens, check_steps, seqs, affine=False, ln_eps=0.0, rope_base=0.0):
    wts = W.make_weights(wl)
    lw = W.make_layer_weights(wl, wts)
    sess = H.make_session(wl)
    H.upload_weights(sess, wts)
    gamma = beta = None
    if affine:  # LayerNorm scale and shift, values exactly representable in the storage type
        g = np.random.default_rng(wl.seed + 5)
        gamma = W.storage_round(1.0 + 0.25 * g.standard_normal(wl.r), wl.dtype)
        beta = W.storage_round(0.25 * g.standard_normal(wl.r), wl.dtype)
    sess.set_layer_weights(w_q=lw.w_q, w_qr=lw.w_qr, w_r=lw.w_r, w_kr=lw.w_kr, w_o=lw.w_o, ln_gamma=gamma, ln_beta=beta,
                           ln_eps=ln_eps, rope_base=rope_base)
    okw = dict(ln_eps=ln_eps or 1e-5, rope_base=rope_base or 10000.0, ln_gamma=gamma, ln_beta=beta)
    B = wl.batch
    xs = np.stack([W.make_x(wl, b, 0, n_tokens) for b in range(B)])           # [B, T, d]
    x_dev = H.to_device(xs, wl.dtype)
    y = torch.empty(B, wl.d_model, dtype=torch.float32, device="cuda")
    out = torch.empty(B, wl.n_heads, wl.d_head, dtype=torch.float32, device="cuda")
    ob = H.OracleBatch.new(wl, wts)
    scale = O.softmax_scale(wl.d_head)
    worst = dict(y=0.0, out=0.0)
    for t in range(n_tokens):
        sess.layer_step(x_dev[:, t].contiguous(), y=y, out=out)
        refs = {}
        for b in seqs:
            refs[b] = O.layer_decode_step(ob.caches[b], xs[b, t], lw.w_q, lw.w_qr, lw.w_r, lw.w_kr, lw.w_o, wts.hyp_A,
                                          None, wts.hyp_G, wts.w_uk, wts.w_uv, scale, **okw)
        if t in check_steps:
            y_gpu, o_gpu = y.cpu().numpy().astype(np.float64), out.cpu().numpy().astype(np.float64)
            for b in seqs:
                y_ref, o_ref, _, slot = refs[b]
                assert slot == t // wl.stride
                worst["y"] = max(worst["y"], float(np.abs(y_gpu[b] - y_ref).max()))
                worst["out"] = max(worst["out"], float(np.abs(o_gpu[b] - o_ref).max()))
            assert worst["y"] <= H.TOL[wl.dtype] and worst["out"] <= H.TOL[wl.dtype], (t, worst)
            H.check_cache(sess, ob, seqs=seqs, what=f"token {t}", kr_exact=False)
    assert sess.device_status() == 0
    assert sess.seq_len.cpu().tolist() == [n_tokens] * B
    return worst


@pytest.mark.parametrize("stride,batch,d_model,n_heads,d_head,r,d_rope", [(2, 5, 128, 8, 64, 256, 32),
                                                                           (3, 18, 96, 4, 64, 128, 64),
                                                                           (1, 3, 256, 16, 128, 512, 64)])
def test_layer_step_every_token(stride, batch, d_model, n_heads, d_head, r, d_rope):
    # ragged token tiles (5 and 18 sequences), three strides, both RoPE widths, every token checked
    T = 26
    wl = W.WORKLOADS["speech_bf16"].scaled(name="layer", batch=batch, d_model=d_model, n_heads=n_heads, d_head=d_head,
                                           r=r, d_rope=d_rope, stride=stride, prefix=T, steps=0, seed=51 + stride)
    _run(wl, T, set(range(T)), list(range(batch)))


def test_layer_step_affine_layer_norm_and_other_constants():
    # LayerNorm with scale and shift, a larger epsilon, another RoPE base
    T = 15
    wl = W.WORKLOADS["speech_bf16"].scaled(name="layer_affine", batch=4, d_model=64, prefix=T, steps=0, stride=2, seed=91)
    _run(wl, T, set(range(T)), list(range(4)), affine=True, ln_eps=1e-3, rope_base=500.0)


def test_layer_step_headline_shape():
    # the paper's decoder shape (d = 512, 8 x 64 heads, r = 256, d_R = 32, s = 2), batch 16, 300 tokens from an
    # empty cache; every tenth step and the last one are compared, on four sequences
    T = 300
    wl = W.WORKLOADS["speech_bf16"].scaled(name="layer_speech", prefix=T, steps=0)
    worst = _run(wl, T, set(range(0, T, 10)) | {T - 1}, [0, 5, 10, 15])
    print("layer step, headline shape: max abs err", worst)


def test_layer_rope_positions_far_out():
    # rotation angles at positions in the tens of thousands: the sequences are declared 40000 tokens long
    # (stride 4: slot 10000 onwards), so that the next tokens are rotated at p = 40000, 40001, ...
    wl = W.WORKLOADS["speech_bf16"].scaled(name="layer_far", batch=2, d_model=64, prefix=40016, steps=0, stride=4, seed=77)
    wts = W.make_weights(wl)
    lw = W.make_layer_weights(wl, wts)
    sess = H.make_session(wl)
    H.upload_weights(sess, wts)
    sess.set_layer_weights(w_q=lw.w_q, w_qr=lw.w_qr, w_r=lw.w_r, w_kr=lw.w_kr, w_o=lw.w_o)
    p0 = 40000
    sess.cache_c.zero_()
    sess.cache_kr.zero_()
    sess.tail_c.zero_()
    sess.seq_len.fill_(p0)
    xs = np.stack([W.make_x(wl, b, p0, p0 + 6) for b in range(2)])
    x_dev = H.to_device(xs, wl.dtype)
    y = torch.empty(2, wl.d_model, dtype=torch.float32, device="cuda")
    for t in range(6):
        sess.layer_step(x_dev[:, t].contiguous(), y=y)
        kr_gpu = sess.cache_kr[:, (p0 + t) // 4].float().cpu().numpy().astype(np.float64)
        for b in range(2):
            kr_ref = O.rope(lw.w_kr.astype(np.float64) @ xs[b, t].astype(np.float64), p0 + t)
            assert np.abs(kr_gpu[b] - kr_ref).max() <= 2.0 ** -8 * np.abs(kr_ref).max() + 1e-6
