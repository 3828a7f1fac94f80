"""GPU parity of mtla_prefill_chunk_attn (the parallel form for sequences that continue from a cache)
against the float64 oracle: a sequence fed in pieces must give, row by row, what the oracle's masked
parallel form gives for the whole sequence (which the oracle's pins tie to incremental inference).
The pieces are ragged, start inside a slot as well as on a slot boundary, and are mixed with single
decode steps.  Integers exact; floating point within 2e-2 (bf16)."""
import numpy as np
import pytest
import torch

import workloads as W
from oracle import mtla_oracle as O
from tests import harness as H

pytestmark = pytest.mark.gpu


def _reference(wl, wts, toks, lens):
    refs = []
    for b, n in enumerate(lens):
        o_ref, _, _, _ = O.prefill_attn(toks[b].q[:n], toks[b].q_rope[:n], toks[b].c[:n], toks[b].kr[:n], wts.w_uk,
                                        wts.w_uv, wl.stride, O.softmax_scale(wl.d_head), hyp_A=wts.hyp_A, hyp_a=None,
                                        hyp_G=wts.hyp_G)
        refs.append(o_ref)
    return refs


def _feed(wl, lens, pieces, decode_at=(), tol=None):
    """Feeds sequence b (lens[b] tokens) in pieces of at most pieces[i] tokens; piece i in `decode_at` is
    one token per sequence through mtla_decode_step.  Returns the worst error against the oracle."""
    wts = W.make_weights(wl)
    B, T_all = wl.batch, int(max(lens))
    assert sum(pieces) >= T_all
    toks = [W.make_tokens(wl, wts, b, 0, T_all) for b in range(B)]
    refs = _reference(wl, wts, toks, lens)
    sess = H.make_session(wl, max_slots=-(-T_all // wl.stride) + 1)
    H.upload_weights(sess, wts)
    def st(f, a, n):  # tokens a .. a+n-1 of every sequence; padding rows may hold anything: NaN here
        rows = [getattr(t, f)[a:min(a + n, lens[b])] for b, t in enumerate(toks)]
        return H.to_device(np.stack([np.concatenate([x, np.full((n - len(x),) + x.shape[1:], np.nan, x.dtype)])
                                     for x in rows]), wl.dtype)
    done = np.zeros(B, np.int64)
    worst = 0.0
    start = 0
    for i, Tn in enumerate(pieces):
        n_new = np.clip(np.asarray(lens) - start, 0, Tn).astype(np.int32)
        d = {f: st(f, start, Tn) for f in ("q", "q_rope", "c", "kr")}
        if i in decode_at:
            assert Tn == 1 and n_new.min() == 1
            out = torch.empty(B, wl.n_heads, wl.d_head, dtype=torch.float32, device="cuda")
            sess.step(d["c"][:, 0].contiguous(), d["kr"][:, 0].contiguous(), d["q"][:, 0].contiguous(),
                      d["q_rope"][:, 0].contiguous(), out=out)
            out = out[:, None]
        else:
            out = torch.full((B, Tn, wl.n_heads, wl.d_head), 9.0, dtype=torch.float32, device="cuda")
            keep = sess.prefill_chunk(d["q"], d["q_rope"], d["c"], d["kr"], out=out, max_past_slots=start // wl.stride,
                                      n_new=torch.from_numpy(n_new).cuda())
            torch.cuda.synchronize()
            del keep
        for b in range(B):
            n = int(n_new[b])
            if n:
                worst = max(worst, H.max_err(out[b, :n], refs[b][start:start + n]))
            assert torch.all(out[b, n:] == 0), (i, b)
        done += n_new
        start += Tn
        assert worst <= (H.TOL["bf16"] if tol is None else tol), (i, worst)
    assert sess.device_status() == 0
    assert sess.seq_len.cpu().tolist() == [int(x) for x in lens]
    return worst


@pytest.mark.parametrize("stride", [1, 2, 3, 4])
def test_chunked_prefill_matches_whole_sequence(stride):
    # pieces that end inside a slot and on slot boundaries, a one-token piece, a piece of several row blocks;
    # sequences of different lengths run out inside different pieces (and one is shorter than the first piece)
    wl = W.WORKLOADS["speech_bf16"].scaled(name="pf_chunk", batch=4, d_model=64, n_heads=6, d_head=64, r=128, d_rope=32,
                                           stride=stride, prefix=333, steps=0, seed=61 + stride)
    lens = [333, 190, 23, 332]
    worst = _feed(wl, lens, [37, 1, 90, 140, 65])
    print(f"chunked prefill stride {stride}: max abs err {worst:.2e}")


@pytest.mark.parametrize("n_heads,d_head,r,d_rope,stride", [(3, 128, 256, 64, 3), (20, 64, 64, 64, 2), (4, 128, 512, 32, 4)])
def test_chunked_prefill_other_shapes_with_decode_steps_between(n_heads, d_head, r, d_rope, stride):
    # a prompt, some single-token decode steps, then more prompt: the chunk call continues from a cache that
    # mtla_decode_step has extended (tail slot in progress)
    wl = W.WORKLOADS["speech_bf16"].scaled(name="pf_chunk_mix", batch=2, d_model=64, n_heads=n_heads, d_head=d_head, r=r,
                                           d_rope=d_rope, stride=stride, prefix=150, steps=0, seed=71 + stride)
    lens = [150, 150]
    worst = _feed(wl, lens, [70, 1, 1, 1, 77], decode_at=(1, 2, 3))
    print(f"chunk / decode / chunk, stride {stride}: max abs err {worst:.2e}")


def test_chunked_prefill_full_size_sampled_rows():
    # the prefill workload (batch 8, T = 4096, 16 heads x 128, r = 512, s = 2) in pieces of 1024, one sequence
    # shorter; the oracle evaluates sampled rows of two sequences, among them the first and last of every piece
    wl = W.WORKLOADS["prefill_s2"]
    T_all, Tn, B = wl.prefix, 1024, wl.batch
    lens = np.full(B, T_all)
    lens[5] = 2500
    wts = W.make_weights(wl)
    toks = [W.make_tokens(wl, wts, b, 0, T_all) for b in range(B)]
    rows = {0: [0, 1, 2, 3, 63, 64, 1000, 1023, 1024, 1025, 2047, 2048, 3071, 3072, 4094, 4095],
            5: [0, 5, 1023, 1024, 2047, 2048, 2400, 2498, 2499]}
    refs = {}
    for b, rr in rows.items():
        n = int(lens[b])
        refs[b], _, _, _ = O.prefill_attn(toks[b].q[:n], toks[b].q_rope[:n], toks[b].c[:n], toks[b].kr[:n], wts.w_uk,
                                          wts.w_uv, wl.stride, O.softmax_scale(wl.d_head), hyp_A=wts.hyp_A, hyp_a=None,
                                          hyp_G=wts.hyp_G, rows=rr)
    sess = H.make_session(wl, max_slots=T_all // wl.stride)
    H.upload_weights(sess, wts)
    worst = 0.0
    for start in range(0, T_all, Tn):
        d = {f: H.to_device(np.stack([getattr(t, f)[start:start + Tn] for t in toks]), wl.dtype)
             for f in ("q", "q_rope", "c", "kr")}
        n_new = np.clip(lens - start, 0, Tn).astype(np.int32)
        out = torch.empty(B, Tn, wl.n_heads, wl.d_head, dtype=torch.float32, device="cuda")
        keep = sess.prefill_chunk(d["q"], d["q_rope"], d["c"], d["kr"], out=out, max_past_slots=start // wl.stride,
                                  n_new=torch.from_numpy(n_new).cuda())
        torch.cuda.synchronize()
        del keep
        for b, rr in rows.items():
            for k, m in enumerate(rr):
                if start <= m < start + Tn:
                    worst = max(worst, H.max_err(out[b, m - start], refs[b][k]))
            assert torch.all(out[b, int(n_new[b]):] == 0)
    print(f"chunked prefill, full size: max abs err {worst:.2e}")
    assert worst <= H.TOL["bf16"]
    assert sess.device_status() == 0
    assert sess.seq_len.cpu().tolist() == [int(x) for x in lens]


def test_chunk_start_outside_the_declared_past_is_reported():
    # pos0 / s above max_past_slots: the kernels stay inside their arrays and the status word says so
    wl = W.WORKLOADS["speech_bf16"].scaled(name="pf_chunk_bad", batch=2, d_model=64, n_heads=4, d_head=64, r=128,
                                           d_rope=32, stride=2, prefix=80, steps=0, seed=5)
    wts = W.make_weights(wl)
    toks = [W.make_tokens(wl, wts, b, 0, 80) for b in range(2)]
    sess = H.make_session(wl, max_slots=64)
    H.upload_weights(sess, wts)
    d = {f: H.to_device(np.stack([getattr(t, f)[:40] for t in toks]), wl.dtype) for f in ("q", "q_rope", "c", "kr")}
    out = torch.empty(2, 40, wl.n_heads, wl.d_head, dtype=torch.float32, device="cuda")
    keep = sess.prefill_chunk(d["q"], d["q_rope"], d["c"], d["kr"], out=out, max_past_slots=0)
    d2 = {f: H.to_device(np.stack([getattr(t, f)[40:80] for t in toks]), wl.dtype) for f in ("q", "q_rope", "c", "kr")}
    keep2 = sess.prefill_chunk(d2["q"], d2["q_rope"], d2["c"], d2["kr"], out=out, max_past_slots=10)  # 20 needed
    torch.cuda.synchronize()
    assert sess.device_status() == 1
    assert torch.isfinite(out).all()
    del keep, keep2


@pytest.mark.parametrize("case", range(6))
def test_chunked_prefill_seeded_random_shapes(case):
    # shapes, lengths and piece sizes drawn from a seeded generator over what the call supports
    g = np.random.default_rng(1000 + case)
    d_head = int(g.choice([64, 128]))
    r = int(g.choice([64, 128, 256, 512]))
    d_rope = int(g.choice([32, 64]))
    n_heads = int(g.integers(1, 21))
    # strides 1 .. 4 (the paper's are 2, 3, 4): a bf16 cache row holds the sum of s weighted latents, so its
    # rounding grows with s, and at s = 5 the past columns alone reach the 2e-2 bound (measured: 2.02e-2)
    stride = int(g.integers(1, 5))
    batch = int(g.integers(1, 5))
    T_all = int(g.integers(40, 400))
    lens = [T_all] + [int(g.integers(1, T_all + 1)) for _ in range(batch - 1)]
    pieces, left = [], T_all
    while left > 0:
        n = int(min(left, g.integers(1, 160)))
        pieces.append(n)
        left -= n
    wl = W.WORKLOADS["speech_bf16"].scaled(name=f"pf_chunk_rand{case}", batch=batch, d_model=64, n_heads=n_heads,
                                           d_head=d_head, r=r, d_rope=d_rope, stride=stride, prefix=T_all, steps=0,
                                           seed=2000 + case)
    worst = _feed(wl, lens, pieces)
    print(f"case {case}: heads {n_heads} x {d_head}, r {r}, d_R {d_rope}, s {stride}, lens {lens}, pieces {pieces}: {worst:.2e}")


@pytest.mark.parametrize("stride", [5, 8])
def test_chunked_prefill_beyond_stride_4_keeps_the_documented_bound(stride):
    # the header gives 2e-2 up to s = 4 and 2e-2 * s / 4 beyond (a cache row is the bf16 rounding of a sum of s
    # weighted latents): the shapes of the stride tests above, at strides the random shapes leave out
    wl = W.WORKLOADS["speech_bf16"].scaled(name=f"pf_chunk_s{stride}", batch=3, d_model=96, n_heads=6, d_head=64, r=128,
                                           d_rope=32, stride=stride, prefix=230, steps=0, seed=41 + stride)
    worst = _feed(wl, [230, 171, 20], [37, 1, 64, 128], tol=H.TOL["bf16"] * stride / 4)
    print(f"stride {stride}: worst error {worst:.3e} against {H.TOL['bf16'] * stride / 4:.3e}")


def test_prefill_step_equals_append_then_chunk_attn():
    # the one-call form against its two halves driven by hand (copies of the state taken before the append):
    # same kernels, so the outputs, merge weights and states agree bit for bit
    wl = W.WORKLOADS["speech_bf16"].scaled(name="pf_step", batch=3, d_model=64, n_heads=5, d_head=64, r=128, d_rope=32,
                                           stride=3, prefix=140, steps=0, seed=17)
    wts = W.make_weights(wl)
    toks = [W.make_tokens(wl, wts, b, 0, 140) for b in range(3)]
    one, two = H.make_session(wl), H.make_session(wl)
    for s in (one, two):
        H.upload_weights(s, wts)
    for a, n in ((0, 50), (50, 90)):       # the second piece starts inside a slot (50 % 3 != 0)
        d = {f: H.to_device(np.stack([getattr(t, f)[a:a + n] for t in toks]), wl.dtype) for f in ("q", "q_rope", "c", "kr")}
        n_new = torch.tensor([n, n - 7, 1], dtype=torch.int32, device="cuda")
        o1 = torch.empty(3, n, wl.n_heads, wl.d_head, dtype=torch.float32, device="cuda")
        o2 = torch.empty_like(o1)
        w1 = torch.zeros(3, n, dtype=torch.float32, device="cuda")
        w2 = torch.zeros_like(w1)
        keep = one.prefill_chunk(d["q"], d["q_rope"], d["c"], d["kr"], out=o1, max_past_slots=a // 3, n_new=n_new, w_out=w1)
        tail_prev, pos0 = two.tail_c.clone(), two.seq_len.clone()
        two.append(d["c"], d["kr"], n_new=n_new, w_out=w2)
        ws = torch.empty(two.ctx.prefill_chunk_workspace_bytes(3, n, a // 3), dtype=torch.uint8, device="cuda")
        two.ctx.prefill_chunk_attn(two.cache_c, two.cache_kr, tail_prev, pos0, d["q"], d["q_rope"], d["c"], d["kr"], w2,
                                   n_new, 3, n, a // 3, two.w_uk, two.w_uv, o2, ws, two.workspace, two.stream)
        torch.cuda.synchronize()
        del keep
        assert torch.equal(o1, o2) and torch.equal(w1, w2)
    for f in ("cache_c", "cache_kr", "tail_c", "seq_len"):
        assert torch.equal(getattr(one, f), getattr(two, f)), f
    assert one.device_status() == 0 and two.device_status() == 0
