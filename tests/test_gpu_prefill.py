"""GPU parity of mtla_prefill_attn (parallel form under the stride-aware causal
mask) against the float64 oracle's masked parallel form, and against the
library's own incremental decode of the same sequence."""
import numpy as np
import pytest
import torch

import workloads as W
from oracle import mtla_oracle as O
from tests import harness as H

pytestmark = pytest.mark.gpu


def _prefill_inputs(wl, wts, T):
    toks = [W.make_tokens(wl, wts, b, 0, T) for b in range(wl.batch)]
    st = lambda f: np.stack([getattr(t, f) for t in toks])
    return toks, {f: H.to_device(st(f), wl.dtype) for f in ("q", "q_rope", "c", "kr")}


def _gpu_prefill(wl, wts, d, T, seq_lens=None, want_latent=True):
    sess = H.make_session(wl, max_slots=-(-T // wl.stride))
    H.upload_weights(sess, wts)
    # merge weights come from the append call that builds the prefix cache
    w = torch.zeros(wl.batch, T, dtype=torch.float32, device="cuda")
    n_new = None if seq_lens is None else torch.from_numpy(seq_lens).cuda()
    sess.append(d["c"], d["kr"], n_new=n_new, w_out=w)
    out = torch.full((wl.batch, T, wl.n_heads, wl.d_head), 9.0, dtype=torch.float32, device="cuda")
    lat = torch.full((wl.batch, T, wl.n_heads, wl.r), 9.0, dtype=torch.float32, device="cuda") if want_latent else None
    ws = sess.prefill(d["q"], d["q_rope"], d["c"], d["kr"], w, out=out, out_latent=lat, seq_lens=n_new)
    torch.cuda.synchronize()
    del ws
    return sess, w, out, lat


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("stride", [1, 2, 3, 4])
def test_prefill_matches_oracle_all_rows(dtype, stride):
    T = 75                                                   # not a multiple of 2, 4: ragged last chunk
    wl = W.WORKLOADS["speech_bf16"].scaled(name="pf", dtype=dtype, batch=3, d_model=96, n_heads=6, d_head=32,
                                           r=128, d_rope=32, stride=stride, prefix=T, steps=0, seed=31 + stride)
    wts = W.make_weights(wl)
    toks, d = _prefill_inputs(wl, wts, T)
    seq_lens = np.array([T, T - 7, 1], np.int32)             # rows past seq_lens[b] are padding
    sess, w, out, lat = _gpu_prefill(wl, wts, d, T, seq_lens)
    tol = H.TOL[dtype]
    for b in range(wl.batch):
        n = int(seq_lens[b])
        o_ref, ol_ref, _, Cp = O.prefill_attn(toks[b].q[:n], toks[b].q_rope[:n], toks[b].c[:n], toks[b].kr[:n],
                                             wts.w_uk, wts.w_uv, stride, O.softmax_scale(wl.d_head),
                                             hyp_A=wts.hyp_A, hyp_a=None, hyp_G=wts.hyp_G)
        assert H.max_err(out[b, :n], o_ref) <= tol
        lat_err = np.abs(lat[b, :n].cpu().numpy().astype(np.float64) - ol_ref)
        H.check_latent(lat_err, Cp, dtype, "prefill rows", strict=False)
        assert torch.all(out[b, n:] == 0) and torch.all(lat[b, n:] == 0)


@pytest.mark.parametrize("n_heads,r,d_rope,stride", [(20, 256, 64, 2), (32, 128, 32, 3), (5, 64, 32, 2), (16, 512, 64, 4)])
def test_prefill_other_shapes(n_heads, r, d_rope, stride):
    # more than 16 heads (one query row per workgroup), r = 64 (slot-split rows kernel), r = 512;
    # T not a multiple of the stride or of the rows per workgroup
    T = 45
    wl = W.WORKLOADS["speech_bf16"].scaled(name="pf_shapes", batch=2, d_model=64, n_heads=n_heads, d_head=64, r=r,
                                           d_rope=d_rope, stride=stride, prefix=T, steps=0, seed=11)
    wts = W.make_weights(wl)
    toks, d = _prefill_inputs(wl, wts, T)
    seq_lens = np.array([T, 22], np.int32)
    _, w, out, lat = _gpu_prefill(wl, wts, d, T, seq_lens)
    for b in range(wl.batch):
        n = int(seq_lens[b])
        o_ref, ol_ref, _, Cp = O.prefill_attn(toks[b].q[:n], toks[b].q_rope[:n], toks[b].c[:n], toks[b].kr[:n],
                                             wts.w_uk, wts.w_uv, stride, O.softmax_scale(wl.d_head),
                                             hyp_A=wts.hyp_A, hyp_a=None, hyp_G=wts.hyp_G)
        assert H.max_err(out[b, :n], o_ref) <= H.TOL["bf16"]
        lat_err = np.abs(lat[b, :n].cpu().numpy().astype(np.float64) - ol_ref)
        H.check_latent(lat_err, Cp, "bf16", "prefill rows")  # the explicit form's second pass: the strict bound holds
        assert torch.all(out[b, n:] == 0) and torch.all(lat[b, n:] == 0)


@pytest.mark.parametrize("n_heads,d_head,r,d_rope,stride,T", [(11, 128, 64, 32, 4, 130), (3, 128, 64, 64, 2, 300)])
def test_prefill_latent_where_r_is_no_multiple_of_d_head(n_heads, d_head, r, d_rope, stride, T):
    # the latent-space output cannot come from the explicit form here (its second pass cuts r into slices of
    # d_head columns): `out` still does (the strict bound; the absorbed form's bf16 operands measured 2.008e-2 on
    # `out` at the first of these shapes), out_latent comes from the absorbed form alone (storage term on every column)
    wl = W.WORKLOADS["speech_bf16"].scaled(name="pf_rdh", batch=3, d_model=64, n_heads=n_heads, d_head=d_head, r=r,
                                           d_rope=d_rope, stride=stride, prefix=T, steps=0, seed=7038)
    wts = W.make_weights(wl)
    toks, d = _prefill_inputs(wl, wts, T)
    seq_lens = np.array([T, T - 41, 3], np.int32)
    _, w, out, lat = _gpu_prefill(wl, wts, d, T, seq_lens)
    for b in range(wl.batch):
        n = int(seq_lens[b])
        o_ref, ol_ref, _, Cp = O.prefill_attn(toks[b].q[:n], toks[b].q_rope[:n], toks[b].c[:n], toks[b].kr[:n],
                                             wts.w_uk, wts.w_uv, stride, O.softmax_scale(wl.d_head),
                                             hyp_A=wts.hyp_A, hyp_a=None, hyp_G=wts.hyp_G)
        assert H.max_err(out[b, :n], o_ref) <= H.TOL["bf16"]
        lat_err = np.abs(lat[b, :n].cpu().numpy().astype(np.float64) - ol_ref)
        H.check_latent(lat_err, Cp, "bf16", "prefill rows", strict=False)
        assert torch.all(out[b, n:] == 0) and torch.all(lat[b, n:] == 0)


@pytest.mark.parametrize("seed", range(8))
def test_prefill_seeded_random_shapes(seed):
    # shapes, lengths and strides drawn from a seed; both outputs on every live row against the oracle.  With
    # d_head 64 or 128 (and r a multiple of it) the explicit form runs, latent output by its second pass (strict
    # bound); other shapes take the absorbed form (storage term on every column)
    rng = np.random.default_rng(7000 + seed)
    d_head = int(rng.choice([32, 64, 128]))
    r = int(rng.choice([64, 128, 256, 512]))
    n_heads = int(rng.integers(1, 25))
    d_rope = int(rng.choice([32, 64]))
    stride = int(rng.integers(1, 5))
    B = int(rng.integers(1, 5))
    T = int(rng.choice([1, 7, 130, 259, 400]))
    wl = W.WORKLOADS["speech_bf16"].scaled(name=f"pf_rand_{seed}", batch=B, d_model=64, n_heads=n_heads, d_head=d_head, r=r,
                                           d_rope=d_rope, stride=stride, prefix=T, steps=0, seed=7000 + seed)
    wts = W.make_weights(wl)
    toks, d = _prefill_inputs(wl, wts, T)
    seq_lens = rng.integers(1, T + 1, size=B).astype(np.int32)
    seq_lens[0] = T
    _, w, out, lat = _gpu_prefill(wl, wts, d, T, seq_lens)
    explicit = d_head in (64, 128) and r % d_head == 0
    for b in range(B):
        n = int(seq_lens[b])
        o_ref, ol_ref, _, Cp = O.prefill_attn(toks[b].q[:n], toks[b].q_rope[:n], toks[b].c[:n], toks[b].kr[:n],
                                             wts.w_uk, wts.w_uv, stride, O.softmax_scale(wl.d_head),
                                             hyp_A=wts.hyp_A, hyp_a=None, hyp_G=wts.hyp_G)
        assert H.max_err(out[b, :n], o_ref) <= H.TOL["bf16"], (seed, b)
        lat_err = np.abs(lat[b, :n].cpu().numpy().astype(np.float64) - ol_ref)
        H.check_latent(lat_err, Cp, "bf16", f"prefill rows, seed {seed}", strict=explicit)
        assert torch.all(out[b, n:] == 0) and torch.all(lat[b, n:] == 0)


@pytest.mark.parametrize("n_heads,d_head,r,d_rope,stride,T", [(6, 64, 128, 32, 2, 75), (3, 128, 256, 64, 3, 200),
                                                              (20, 64, 64, 64, 1, 140), (4, 128, 512, 32, 4, 333)])
def test_prefill_explicit_form_all_rows(n_heads, d_head, r, d_rope, stride, T):
    # without the latent output the library takes the explicit key / value form: several 128-row
    # blocks with a ragged last one, lengths that end inside a block, a sequence of one token
    wl = W.WORKLOADS["speech_bf16"].scaled(name="pf_explicit", batch=3, d_model=64, n_heads=n_heads, d_head=d_head,
                                           r=r, d_rope=d_rope, stride=stride, prefix=T, steps=0, seed=21 + stride)
    wts = W.make_weights(wl)
    toks, d = _prefill_inputs(wl, wts, T)
    seq_lens = np.array([T, T - 70, 1], np.int32)
    _, w, out, _ = _gpu_prefill(wl, wts, d, T, seq_lens, want_latent=False)
    for b in range(wl.batch):
        n = int(seq_lens[b])
        o_ref, _, _, _ = O.prefill_attn(toks[b].q[:n], toks[b].q_rope[:n], toks[b].c[:n], toks[b].kr[:n],
                                        wts.w_uk, wts.w_uv, stride, O.softmax_scale(wl.d_head),
                                        hyp_A=wts.hyp_A, hyp_a=None, hyp_G=wts.hyp_G)
        assert H.max_err(out[b, :n], o_ref) <= H.TOL["bf16"]
        assert torch.all(out[b, n:] == 0)


@pytest.mark.parametrize("batch,n_heads,d_head,r,d_rope,stride,T", [(16, 16, 128, 256, 64, 2, 600),
                                                                    (8, 32, 64, 128, 32, 3, 777)])
def test_prefill_explicit_form_many_jobs(batch, n_heads, d_head, r, d_rope, stride, T):
    # several hundred (sequence, head, row block pair) jobs, numbered across the XCDs: ragged last block,
    # lengths ending inside a block and inside a chunk; four sequences checked on all rows
    wl = W.WORKLOADS["speech_bf16"].scaled(name="pf_jobs", batch=batch, d_model=64, n_heads=n_heads, d_head=d_head,
                                           r=r, d_rope=d_rope, stride=stride, prefix=T, steps=0, seed=41 + stride)
    wts = W.make_weights(wl)
    toks, d = _prefill_inputs(wl, wts, T)
    seq_lens = np.full(batch, T, np.int32)
    seq_lens[1], seq_lens[2], seq_lens[batch - 1] = T - 301, 257, T - 1
    _, w, out, _ = _gpu_prefill(wl, wts, d, T, seq_lens, want_latent=False)
    for b in (0, 1, 2, batch - 1):
        n = int(seq_lens[b])
        o_ref, _, _, _ = O.prefill_attn(toks[b].q[:n], toks[b].q_rope[:n], toks[b].c[:n], toks[b].kr[:n],
                                        wts.w_uk, wts.w_uv, stride, O.softmax_scale(wl.d_head),
                                        hyp_A=wts.hyp_A, hyp_a=None, hyp_G=wts.hyp_G)
        assert H.max_err(out[b, :n], o_ref) <= H.TOL["bf16"]
        assert torch.all(out[b, n:] == 0)


def test_prefill_equals_incremental_decode_on_gpu():
    T, stride = 50, 3
    wl = W.WORKLOADS["speech_bf16"].scaled(name="pf_inc", batch=2, d_model=64, stride=stride, prefix=T, steps=0)
    wts = W.make_weights(wl)
    toks, d = _prefill_inputs(wl, wts, T)
    _, w, out, lat = _gpu_prefill(wl, wts, d, T)
    sess = H.make_session(wl, max_slots=-(-T // stride))
    H.upload_weights(sess, wts)
    o1 = torch.empty(2, wl.n_heads, wl.d_head, dtype=torch.float32, device="cuda")
    l1 = torch.empty(2, wl.n_heads, wl.r, dtype=torch.float32, device="cuda")
    for t in range(T):
        sess.append(d["c"][:, t:t + 1].contiguous(), d["kr"][:, t:t + 1].contiguous())
        sess.decode(d["q"][:, t].contiguous(), d["q_rope"][:, t].contiguous(), out=o1, out_latent=l1)
        assert (l1 - lat[:, t]).abs().max().item() <= 2e-2
        assert (o1.float() - out[:, t].float()).abs().max().item() <= 2e-2


@pytest.mark.parametrize("name,want_latent", [("prefill_s2", False), ("prefill_s4", False), ("prefill_s2", True)])
def test_prefill_full_size_sampled_rows(name, want_latent):
    # batch 8, T = 4096, 16 heads x 128, r = 512: the oracle evaluates sampled rows of two sequences.
    # The explicit key / value form runs (what the benchmark times); the latent-space output, when asked
    # for, comes from its second pass over the partial states.
    wl = W.WORKLOADS[name]
    T = wl.prefix
    wts = W.make_weights(wl)
    toks, d = _prefill_inputs(wl, wts, T)
    _, w, out, lat = _gpu_prefill(wl, wts, d, T, want_latent=want_latent)
    rows = [0, 1, 2, 3, 4, 5, 63, 64, 127, 128, 1000, 2047, 2048, 4093, 4094, 4095]
    w_cpu = w.cpu().numpy()
    for b in (0, 5):
        o_ref, ol_ref, _, Cp = O.prefill_attn(toks[b].q, toks[b].q_rope, toks[b].c, toks[b].kr, wts.w_uk, wts.w_uv,
                                              wl.stride, O.softmax_scale(wl.d_head), hyp_A=wts.hyp_A, hyp_a=None,
                                              hyp_G=wts.hyp_G, rows=rows)
        assert H.max_err(out[b, rows], o_ref) <= H.TOL["bf16"]
        if want_latent:
            lat_err = np.abs(lat[b, rows].cpu().numpy().astype(np.float64) - ol_ref)
            H.check_latent(lat_err, Cp, "bf16", "prefill rows, full size")
        # the merge weights handed to the kernel are the hyper-network's
        w_ref = np.array([O.merge_weight(toks[b].c[n], wts.hyp_A, None, wts.hyp_G[n // wl.stride]) for n in rows])
        assert np.abs(w_cpu[b, rows] - w_ref).max() <= H.TOL_W


def test_prefill_more_than_65535_rows():
    # batch * T above the 16-bit grid limit of the vector kernels: matrix-core paths only
    T, B = 4100, 17
    wl = W.WORKLOADS["speech_bf16"].scaled(name="pf_rows", batch=B, d_model=32, n_heads=2, d_head=64, r=128, d_rope=32,
                                           stride=3, prefix=T, steps=0, seed=3)
    wts = W.make_weights(wl)
    toks, d = _prefill_inputs(wl, wts, T)
    rows = [0, 1, 2, 3, 127, 128, 129, 2050, T - 2, T - 1]
    for want_latent in (False, True):
        _, w, out, lat = _gpu_prefill(wl, wts, d, T, want_latent=want_latent)
        for b in (0, B - 1):
            o_ref, _, _, _ = O.prefill_attn(toks[b].q, toks[b].q_rope, toks[b].c, toks[b].kr, wts.w_uk, wts.w_uv,
                                            wl.stride, O.softmax_scale(wl.d_head), hyp_A=wts.hyp_A, hyp_a=None,
                                            hyp_G=wts.hyp_G, rows=rows)
            assert H.max_err(out[b, rows], o_ref) <= H.TOL["bf16"]
    f32 = H.make_session(wl.scaled(dtype="f32"), max_slots=-(-T // wl.stride))
    nb = f32.ctx.prefill_workspace_bytes(B, T)
    assert f32.ctx.prefill_attn_status(d["q"], d["q_rope"], d["c"], d["kr"], w, None, B, T, d["q"], d["q"], out, None,
                                       torch.empty(16, dtype=torch.uint8, device="cuda") if nb > (1 << 33) else
                                       torch.empty(nb, dtype=torch.uint8, device="cuda"), f32.stream) == 4  # UNSUPPORTED
