"""GPU tests of paged slot storage (the *_paged calls and mtla_cache_fork_paged) through the C-ABI: the same
seeded inputs through a contiguous session and through a paged one whose pages are handed out in a scrambled
order must leave the same state row for row and give the same outputs bit for bit; both are checked against the
float64 oracle; beams that fork and drop share complete pages and stay equal to the oracle's copies."""
import copy

import numpy as np
import pytest
import torch

import workloads as W
from oracle import mtla_oracle as O
from paper_2505_13544_amd.session import PagedSession
from tests import harness as H

pytestmark = pytest.mark.gpu


def make_paged(wl, *, page_slots, n_pages, max_slots=None, decode_schedule=0, decode_chunk=None, seed=0):
    order = np.random.default_rng(seed).permutation(n_pages)
    return PagedSession(n_heads=wl.n_heads, d_head=wl.d_head, r=wl.r, d_rope=wl.d_rope, d_hyper=wl.d_hyper,
                        stride=wl.stride, max_batch=wl.batch, max_slots=max_slots or wl.max_slots, page_slots=page_slots,
                        n_pages=n_pages, dtype=wl.dtype, decode_schedule=decode_schedule, decode_chunk=decode_chunk,
                        page_order=order)


def assert_same_state(paged, flat, lens, what):
    assert torch.equal(paged.seq_len[:len(lens)], flat.seq_len[:len(lens)]), what
    assert torch.equal(paged.tail_c[:len(lens)], flat.tail_c[:len(lens)]), what
    for b, n in enumerate(lens):
        live = -(-int(n) // paged.stride)
        if live:
            c, kr = paged.rows(b, live)
            assert torch.equal(c, flat.cache_c[b, :live]), f"{what}: latent rows of sequence {b}"
            assert torch.equal(kr, flat.cache_kr[b, :live]), f"{what}: RoPE keys of sequence {b}"


@pytest.mark.parametrize("schedule,stride,n_heads,r,d_rope,page_slots", [(1, 2, 8, 256, 32, 16), (2, 2, 8, 256, 32, 32),
                                                                        (2, 3, 20, 512, 64, 64), (1, 4, 5, 128, 32, 16),
                                                                        (0, 1, 3, 64, 64, 16)])
def test_paged_decode_equals_contiguous_and_the_oracle(schedule, stride, n_heads, r, d_rope, page_slots):
    # ragged prefixes (one empty, one that ends exactly on a page boundary, one inside a slot), a bulk append and
    # decode steps that cross page boundaries; static and balanced schedules, one and two head tiles, r = 64
    B, steps = 6, 2 * page_slots * stride // 4 + 5
    wl = W.WORKLOADS["speech_bf16"].scaled(name=f"paged_s{stride}", batch=B, d_model=96, n_heads=n_heads, d_head=64, r=r,
                                           d_rope=d_rope, stride=stride, prefix=(0, 5 * page_slots * stride), steps=steps,
                                           seed=300 + stride)
    plen = np.array([0, 1, page_slots * stride, 3 * page_slots * stride - 1, 5 * page_slots * stride - stride, 37], np.int32)
    wts = W.make_weights(wl)
    toks = [W.make_tokens(wl, wts, b, 0, int(plen[b]) + steps) for b in range(B)]
    max_slots = -(-(int(plen.max()) + steps) // stride)
    flat = H.make_session(wl, max_slots=max_slots, decode_schedule=schedule, decode_chunk=32)
    paged = make_paged(wl, page_slots=page_slots, n_pages=B * (-(-max_slots // page_slots)) + 3, max_slots=max_slots,
                       decode_schedule=schedule, decode_chunk=32, seed=stride)
    for s in (flat, paged):
        H.upload_weights(s, wts)
    ob = H.OracleBatch.new(wl, wts)
    n_max = int(plen.max())
    pre = {f: H.to_device(H.pad_stack([getattr(t, f)[:plen[b]] for b, t in enumerate(toks)], n_max), wl.dtype) for f in ("c", "kr")}
    w_f = torch.zeros(B, n_max, device="cuda")
    w_p = torch.zeros(B, n_max, device="cuda")
    flat.append(pre["c"], pre["kr"], n_new=torch.from_numpy(plen).cuda(), w_out=w_f)
    paged.append(pre["c"], pre["kr"], n_new=plen, w_out=w_p)
    torch.cuda.synchronize()
    assert torch.equal(w_f, w_p)
    assert_same_state(paged, flat, plen, "after the prefix")
    for b in range(B):
        ob.append(b, toks[b].c[:plen[b]], toks[b].kr[:plen[b]])
    H.check_cache(flat, ob, what="prefix:")
    worst = 0.0
    for t in range(steps):
        pick = lambda f: H.to_device(np.stack([getattr(toks[b], f)[plen[b] + t] for b in range(B)]), wl.dtype)
        c, kr, q, qr = pick("c").unsqueeze(1), pick("kr").unsqueeze(1), pick("q"), pick("q_rope")
        outs = []
        for s in (flat, paged):
            o = torch.empty(B, n_heads, 64, dtype=torch.float32, device="cuda")
            ol = torch.empty(B, n_heads, r, dtype=torch.float32, device="cuda")
            ls = torch.empty(B, n_heads, dtype=torch.float32, device="cuda")
            if t % 3 == 2:      # the two-call form now and then
                s.append(c, kr)
                s.decode(q, qr, out=o, out_latent=ol, lse=ls)
            else:
                s.step(c, kr, q, qr, out=o, out_latent=ol, lse=ls)
            outs.append((o, ol, ls))
        torch.cuda.synchronize()
        for x, y in zip(*outs):
            assert torch.equal(x, y), f"step {t}: paged and contiguous storage disagree"
        for b in range(B):
            ob.append(b, toks[b].c[plen[b] + t][None], toks[b].kr[plen[b] + t][None])
            o_ref, _, lse_ref, _ = ob.decode(b, toks[b].q[plen[b] + t], toks[b].q_rope[plen[b] + t])
            worst = max(worst, H.max_err(outs[1][0][b], o_ref), H.max_err(outs[1][2][b], lse_ref))
    assert worst <= H.TOL["bf16"], worst
    assert_same_state(paged, flat, plen + steps, "after the steps")
    assert flat.device_status() == 0 and paged.device_status() == 0
    used = sum(-(-(-(-(int(plen[b]) + steps) // stride)) // page_slots) for b in range(B))
    assert paged.pages_in_use() == used
    print(f"paged decode, schedule {schedule}, stride {stride}, {n_heads} heads, r {r}, pages of {page_slots}: {worst:.2e}")


@pytest.mark.parametrize("stride,page_slots,schedule", [(2, 16, 0), (3, 32, 2), (1, 16, 1)])
def test_paged_beams_fork_drop_and_share_the_prompt(stride, page_slots, schedule):
    # one prompt, prefilled once; every beam then refers to its complete pages (a fork of sequence 0 into all beams);
    # each step the beams decode one token and are reordered by a seeded draw with forks (a source continued twice
    # or more) and drops; the oracle keeps one cache copy per beam
    B, prompt, steps = 8, 5 * page_slots * stride // 2 + 3, 3 * page_slots * stride // 2 + 2
    wl = W.WORKLOADS["speech_bf16"].scaled(name=f"beams_s{stride}", batch=B, d_model=96, n_heads=8, d_head=64, r=256,
                                           d_rope=32, stride=stride, prefix=prompt, steps=steps, seed=400 + stride)
    wts = W.make_weights(wl)
    rng = np.random.default_rng(500 + stride)
    stream = W.make_tokens(wl, wts, 0, 0, prompt + steps * B + 8)   # a pool of tokens to draw the beams' tokens from
    max_slots = -(-(prompt + steps) // stride)
    sess = make_paged(wl, page_slots=page_slots, n_pages=3 * B * (-(-max_slots // page_slots)), max_slots=max_slots,
                      decode_schedule=schedule, seed=9)
    H.upload_weights(sess, wts)
    n_new = [prompt] + [0] * (B - 1)
    zeros = lambda f: H.to_device(np.concatenate([getattr(stream, f)[None, :prompt]] + [np.zeros_like(getattr(stream, f)[None, :prompt])] * (B - 1)), wl.dtype)
    sess.append(zeros("c"), zeros("kr"), n_new=n_new)
    cache0 = O.LatentCache(wl.r, wl.d_rope, stride)
    for t in range(prompt):
        O.append_token(cache0, stream.c[t], stream.kr[t], wts.hyp_A, None, wts.hyp_G)
    prompt_pages = sess.pages_in_use()
    sess.fork([0] * B)
    caches = [copy.deepcopy(cache0) for _ in range(B)]
    # the prompt is stored once: its complete pages, plus one page per beam for what comes next
    full = (prompt // stride) // page_slots
    assert sess.pages_in_use() == full + B, (sess.pages_in_use(), full, B, prompt_pages)
    scale = O.softmax_scale(wl.d_head)
    worst, cursor = 0.0, prompt
    out = torch.empty(B, wl.n_heads, wl.d_head, dtype=torch.float32, device="cuda")
    for t in range(steps):
        ids = [cursor + b for b in range(B)]          # every beam its own token
        cursor += B
        pick = lambda f: H.to_device(np.stack([getattr(stream, f)[i] for i in ids]), wl.dtype)
        sess.step(pick("c").unsqueeze(1), pick("kr").unsqueeze(1), pick("q"), pick("q_rope"), out=out)
        torch.cuda.synchronize()
        for b in range(B):
            O.append_token(caches[b], stream.c[ids[b]], stream.kr[ids[b]], wts.hyp_A, None, wts.hyp_G)
            o_ref = O.decode_attn(caches[b], stream.q[ids[b]], stream.q_rope[ids[b]], wts.w_uk, wts.w_uv, scale)[0]
            worst = max(worst, H.max_err(out[b], o_ref))
        assert worst <= H.TOL["bf16"], (t, worst)
        src = rng.integers(0, B, size=B) if t % 2 == 0 else rng.permutation(B)   # forks and drops / a pure permutation
        sess.fork(src)
        caches = [copy.deepcopy(caches[int(s)]) for s in src]
        # state of every beam, gathered out of the pool, against its oracle copy
        torch.cuda.synchronize()
        assert sess.seq_len.cpu().tolist() == [c.i for c in caches]
        for b in range(B):
            C_ref, KR_ref = caches[b].arrays()
            c, kr = sess.rows(b, caches[b].n_slots)
            err = np.abs(c.float().cpu().numpy() - C_ref)
            assert np.all(err <= H.cache_tolerance(C_ref, "bf16")), (t, b, err.max())
            assert np.array_equal(kr.float().cpu().numpy(), KR_ref)
        # the device table agrees with the host's view wherever a page is assigned
        dev_table = sess.table.cpu().numpy()
        for b in range(B):
            k = int((sess.h_table[b] >= 0).sum())
            assert np.array_equal(dev_table[b, :k], sess.h_table[b, :k]), (t, b)
        # page accounting: no leak, and sharing really happens
        refs = np.zeros(sess.n_pages, np.int32)
        for b in range(B):
            for p in sess.h_table[b]:
                if p >= 0:
                    refs[p] += 1
        assert np.array_equal(refs, sess.refs)
        assert sess.pages_in_use() + len(sess.free) == sess.n_pages
    live = -(-(prompt + steps) // stride)
    assert sess.pages_in_use() < B * (-(-live // page_slots)), "beams share no page"
    assert sess.device_status() == 0
    print(f"paged beams, stride {stride}, pages of {page_slots}: max abs err {worst:.2e}, "
          f"{sess.pages_in_use()} pages in use against {B * (-(-live // page_slots))} without sharing")


@pytest.mark.parametrize("stride", [2, 3])
def test_paged_chunked_prefill_equals_contiguous(stride):
    # a prompt fed in ragged pieces through mtla_prefill_step_paged: rows and state as the contiguous call leaves them
    B, T_all, page_slots = 3, 150, 16
    wl = W.WORKLOADS["speech_bf16"].scaled(name="paged_pf", batch=B, d_model=64, n_heads=6, d_head=64, r=128, d_rope=32,
                                           stride=stride, prefix=T_all, steps=0, seed=600 + stride)
    wts = W.make_weights(wl)
    toks = [W.make_tokens(wl, wts, b, 0, T_all) for b in range(B)]
    lens = [150, 97, 20]
    max_slots = -(-T_all // stride) + 1
    flat = H.make_session(wl, max_slots=max_slots)
    paged = make_paged(wl, page_slots=page_slots, n_pages=B * (-(-max_slots // page_slots)), max_slots=max_slots, seed=4)
    for s in (flat, paged):
        H.upload_weights(s, wts)
    start, worst = 0, 0.0
    for Tn in (37, 1, 64, 48):
        n_new = np.clip(np.asarray(lens) - start, 0, Tn).astype(np.int32)
        d = {f: H.to_device(np.stack([np.concatenate([getattr(t, f)[start:min(start + Tn, lens[b])],
                                                      np.zeros((Tn - max(0, min(start + Tn, lens[b]) - start),) + getattr(t, f).shape[1:], np.float32)])
                                      for b, t in enumerate(toks)]), wl.dtype) for f in ("q", "q_rope", "c", "kr")}
        o_f = torch.full((B, Tn, wl.n_heads, wl.d_head), 9.0, dtype=torch.float32, device="cuda")
        o_p = torch.full_like(o_f, 7.0)
        k1 = flat.prefill_chunk(d["q"], d["q_rope"], d["c"], d["kr"], out=o_f, max_past_slots=start // stride,
                                n_new=torch.from_numpy(n_new).cuda())
        k2 = paged.prefill_chunk(d["q"], d["q_rope"], d["c"], d["kr"], out=o_p, max_past_slots=start // stride, n_new=n_new)
        torch.cuda.synchronize()
        del k1, k2
        assert torch.equal(o_f, o_p)
        for b in range(B):
            n = int(n_new[b])
            if n:
                ref = O.prefill_attn(toks[b].q[:lens[b]], toks[b].q_rope[:lens[b]], toks[b].c[:lens[b]], toks[b].kr[:lens[b]],
                                     wts.w_uk, wts.w_uv, stride, O.softmax_scale(wl.d_head), hyp_A=wts.hyp_A, hyp_a=None,
                                     hyp_G=wts.hyp_G, rows=list(range(start, start + n)))[0]
                worst = max(worst, H.max_err(o_p[b, :n], ref))
        start += Tn
    assert worst <= H.TOL["bf16"], worst
    assert_same_state(paged, flat, lens, "after the pieces")
    assert flat.device_status() == 0 and paged.device_status() == 0
