"""GPU parity of mtla_layer_prefill (the whole attention layer in the parallel form: projections as
matrix products, LayerNorm, decoupled RoPE, cache append, attention under the stride-aware mask, W_O)
against the float64 oracle's layer_prefill, through the C-ABI.  Both sides start from the same rounded
token stream and weights.  Sequences are fed whole, in ragged pieces, and mixed with single-token
layer steps; the cache the call leaves is compared with the oracle's.  Integers exact; floating point
within 2e-2 (bf16)."""
import numpy as np
import pytest
import torch

import workloads as W
from oracle import mtla_oracle as O
from tests import harness as H

pytestmark = pytest.mark.gpu


def _setup(wl, affine=False, ln_eps=0.0, rope_base=0.0):
    wts = W.make_weights(wl)
    lw = W.make_layer_weights(wl, wts)
    sess = H.make_session(wl)
    H.upload_weights(sess, wts)
    gamma = beta = None
    if affine:
        g = np.random.default_rng(wl.seed + 5)
        gamma = W.storage_round(1.0 + 0.25 * g.standard_normal(wl.r), wl.dtype)
        beta = W.storage_round(0.25 * g.standard_normal(wl.r), wl.dtype)
    sess.set_layer_weights(w_q=lw.w_q, w_qr=lw.w_qr, w_r=lw.w_r, w_kr=lw.w_kr, w_o=lw.w_o, ln_gamma=gamma, ln_beta=beta,
                           ln_eps=ln_eps, rope_base=rope_base)
    okw = dict(ln_eps=ln_eps or 1e-5, rope_base=rope_base or 10000.0, ln_gamma=gamma, ln_beta=beta)
    return wts, lw, sess, okw


def _oracle_rows(wl, wts, lw, okw, x, rows=None):
    y, _ = O.layer_prefill(x, lw.w_q, lw.w_qr, lw.w_r, lw.w_kr, lw.w_o, wts.hyp_A, None, wts.hyp_G, wts.w_uk, wts.w_uv,
                           wl.stride, O.softmax_scale(wl.d_head), rows=rows, **okw)
    return y


def _oracle_cache(wl, wts, lw, okw, ob, b, x):
    for p in range(len(x)):
        _, _, c, kr = O.layer_front(x[p], p, lw.w_q, lw.w_qr, lw.w_r, lw.w_kr, wl.n_heads, **okw)
        O.append_token(ob.caches[b], c, kr, wts.hyp_A, None, wts.hyp_G)


def _feed(wl, lens, pieces, step_at=(), **kw):
    """Sequence b (lens[b] tokens) goes through the layer in pieces of at most pieces[i] tokens; piece i in
    `step_at` is one token per sequence through mtla_layer_decode_step.  Returns the worst error of y."""
    wts, lw, sess, okw = _setup(wl, **kw)
    B, T_all = wl.batch, int(max(lens))
    xs = [W.make_x(wl, b, 0, T_all) for b in range(B)]
    refs = [_oracle_rows(wl, wts, lw, okw, xs[b][:lens[b]]) for b in range(B)]
    worst, start = 0.0, 0
    for i, Tn in enumerate(pieces):
        n_new = np.clip(np.asarray(lens) - start, 0, Tn).astype(np.int32)
        x = np.full((B, Tn, wl.d_model), np.nan)  # padding rows may hold anything
        for b in range(B):
            x[b, :n_new[b]] = xs[b][start:start + n_new[b]]
        x_dev = H.to_device(x, wl.dtype)
        if i in step_at:
            assert Tn == 1 and n_new.min() == 1
            y = torch.empty(B, wl.d_model, dtype=torch.float32, device="cuda")
            sess.layer_step(x_dev[:, 0].contiguous(), y=y)
            y = y[:, None]
        else:
            y = torch.full((B, Tn, wl.d_model), 9.0, dtype=torch.float32, device="cuda")
            keep = sess.layer_prefill(x_dev, y=y, max_past_slots=start // wl.stride, n_new=torch.from_numpy(n_new).cuda())
            torch.cuda.synchronize()
            del keep
        for b in range(B):
            n = int(n_new[b])
            if n:
                worst = max(worst, H.max_err(y[b, :n], refs[b][start:start + n]))
            assert torch.all(y[b, n:] == 0), (i, b)
        start += Tn
        print(f"  piece {i} ({Tn} tokens): worst so far {worst:.2e}")
        assert worst <= H.TOL["bf16"], (i, worst)
    assert sess.device_status() == 0
    assert sess.seq_len.cpu().tolist() == [int(n) for n in lens]
    ob = H.OracleBatch.new(wl, wts)
    for b in range(B):
        _oracle_cache(wl, wts, lw, okw, ob, b, xs[b][:lens[b]])
    H.check_cache(sess, ob, what="after the last piece", kr_exact=False)
    return worst


@pytest.mark.parametrize("stride,n_heads,d_head,r,d_rope,d_model", [(2, 8, 64, 256, 32, 128), (3, 4, 128, 128, 64, 96),
                                                                     (1, 6, 64, 512, 64, 256), (4, 16, 64, 64, 32, 64),
                                                                     (2, 3, 64, 128, 32, 64), (3, 2, 128, 64, 64, 32)])
def test_layer_prefill_whole_prompt(stride, n_heads, d_head, r, d_rope, d_model):
    # sequences of different lengths in one call (several row blocks, a ragged last one, one sequence of 2 tokens);
    # the fifth shape has n_h d_R = 96 columns of RoPE queries: the shared key is then a product of its own;
    # the last one has d_model = 32, a contraction of a single step
    wl = W.WORKLOADS["speech_bf16"].scaled(name="lp", batch=3, d_model=d_model, n_heads=n_heads, d_head=d_head, r=r,
                                           d_rope=d_rope, stride=stride, prefix=300, steps=0, seed=81 + stride)
    worst = _feed(wl, [300, 171, 2], [300])
    print(f"layer prefill, stride {stride}: max abs err {worst:.2e}")


@pytest.mark.parametrize("stride", [2, 3])
def test_layer_prefill_in_pieces_with_layer_steps_between(stride):
    # pieces that end inside a slot, single-token layer steps in between, sequences running out in different pieces
    wl = W.WORKLOADS["speech_bf16"].scaled(name="lp_pieces", batch=4, d_model=128, stride=stride, prefix=260, steps=0,
                                           seed=91 + stride)
    worst = _feed(wl, [260, 260, 200, 259], [45, 1, 1, 83, 130], step_at=(1, 2))
    print(f"layer prefill in pieces, stride {stride}: max abs err {worst:.2e}")


def test_layer_prefill_pieces_of_one_and_two_tokens():
    # the call itself with T = 1 and T = 2 (the append then takes its single-token path) between longer pieces
    wl = W.WORKLOADS["speech_bf16"].scaled(name="lp_tiny_pieces", batch=3, d_model=64, stride=3, prefix=100, steps=0, seed=97)
    worst = _feed(wl, [100, 100, 61], [31, 1, 2, 1, 65])
    print(f"layer prefill with one- and two-token pieces: max abs err {worst:.2e}")


def test_layer_prefill_affine_layer_norm_and_other_constants():
    wl = W.WORKLOADS["speech_bf16"].scaled(name="lp_affine", batch=2, d_model=64, stride=2, prefix=150, steps=0, seed=93)
    _feed(wl, [150, 77], [100, 50], affine=True, ln_eps=1e-3, rope_base=500.0)


def test_layer_prefill_full_size_sampled_rows():
    # the prefill workload's shape (d = 2048, 16 heads x 128, r = 512, d_R = 64, s = 2), 4 sequences of 2048 tokens
    # in two pieces of 1024; the oracle evaluates sampled rows of two sequences
    base = W.WORKLOADS["prefill_s2"]
    T_all, Tn, B = 2048, 1024, 4
    wl = base.scaled(name="lp_full", batch=B, prefix=T_all, steps=0)
    wts, lw, sess, okw = _setup(wl)
    xs = [W.make_x(wl, b, 0, T_all) for b in range(B)]
    rows = [0, 1, 2, 3, 64, 1000, 1023, 1024, 1025, 2046, 2047]
    refs = {b: _oracle_rows(wl, wts, lw, okw, xs[b], rows=rows) for b in (0, 3)}
    worst = 0.0
    for start in range(0, T_all, Tn):
        x_dev = H.to_device(np.stack([x[start:start + Tn] for x in xs]), wl.dtype)
        y = torch.empty(B, Tn, wl.d_model, dtype=torch.float32, device="cuda")
        keep = sess.layer_prefill(x_dev, y=y, max_past_slots=start // wl.stride)
        torch.cuda.synchronize()
        del keep
        for b in (0, 3):
            for k, m in enumerate(rows):
                if start <= m < start + Tn:
                    worst = max(worst, H.max_err(y[b, m - start], refs[b][k]))
    print(f"layer prefill, full size: max abs err {worst:.2e}")
    assert worst <= H.TOL["bf16"]
    assert sess.device_status() == 0


def test_layer_prefill_and_chunk_attn_replay_from_a_hip_graph():
    # the calls enqueue kernels only (no allocation, no synchronisation, no memset): captured once into a
    # HIP graph they can be replayed on new inputs; three replays with eager work in between, every replay
    # compared with an eager call on a second session
    wl = W.WORKLOADS["speech_bf16"].scaled(name="lp_graph", batch=3, d_model=64, stride=2, prefix=120, steps=0, seed=99)
    wts, lw, sess, okw = _setup(wl)
    _, _, ref_sess, _ = _setup(wl)
    B, Tn, past_max = 3, 40, 40
    xs = [W.make_x(wl, b, 0, 120) for b in range(B)]
    x_static = torch.zeros(B, Tn, wl.d_model, dtype=sess.tdt, device="cuda")
    y_static = torch.zeros(B, Tn, wl.d_model, dtype=torch.float32, device="cuda")
    scratch = torch.empty(sess.ctx.layer_prefill_scratch_bytes(wl.d_model, B, Tn, past_max), dtype=torch.uint8, device="cuda")

    def call(s, x, y, scr):
        s.ctx.layer_prefill(s.layer_w, s.cache_c, s.cache_kr, s.tail_c, s.seq_len, x, None, s.hyp_A, s.hyp_a, s.hyp_G,
                            s.w_uk, s.w_uv, B, Tn, past_max, y, scr, s.workspace, s.stream)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):          # warm-up on the capture stream, then rewind the state
        call(sess, x_static, y_static, scratch)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    sess.seq_len.zero_()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        call(sess, x_static, y_static, scratch)
    sess.seq_len.zero_()                   # capture does not run the kernels
    ref_scratch = torch.empty_like(scratch)
    y_ref = torch.empty_like(y_static)
    for i in range(3):                     # pieces 0..39, 40..79, 80..119 of every sequence
        x_piece = H.to_device(np.stack([x[40 * i:40 * i + 40] for x in xs]), wl.dtype)
        x_static.copy_(x_piece)
        graph.replay()
        call(ref_sess, x_piece, y_ref, ref_scratch)   # eager work between the replays
        torch.cuda.synchronize()
        assert torch.equal(y_static, y_ref), f"replay {i} differs from the eager call"
    assert sess.seq_len.cpu().tolist() == [120] * B and sess.device_status() == 0
    assert torch.equal(sess.cache_c, ref_sess.cache_c) and torch.equal(sess.cache_kr, ref_sess.cache_kr)
