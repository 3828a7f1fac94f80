"""GPU parity of mtla_cache_append + mtla_decode_attn against the float64
oracle, through the C-ABI, on the seeded benchmark workloads and on edge
cases.  Integers (slot indices, lengths) must match exactly; floating point
within 1e-5 (fp32 storage) or 2e-2 (bf16 storage, fp32 accumulation)."""
import numpy as np
import pytest
import torch

import workloads as W
from tests import harness as H

pytestmark = pytest.mark.gpu


def test_tiny_f32_every_step():
    H.run_decode_parity(W.WORKLOADS["tiny_f32"])


@pytest.mark.parametrize("fused_step", [False, True])
def test_speech_bf16_full_size_every_step(fused_step):
    # the headline configuration, in the launch configurations the benchmark times:
    # mtla_cache_append + mtla_decode_attn, and mtla_decode_step (the default)
    H.run_decode_parity(W.WORKLOADS["speech_bf16"], fused_step=fused_step)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("stride", [1, 2, 3, 4])
def test_ragged_small_batches_all_strides(dtype, stride):
    # ragged prefixes (one empty, one not a multiple of the stride), several splits with a ragged
    # last chunk (chunk 32 against up to 75 slots), a head count that is not a multiple of the group
    wl = W.WORKLOADS["speech_bf16"].scaled(name=f"ragged_{dtype}_s{stride}", dtype=dtype, batch=5, d_model=96,
                                           n_heads=6, d_head=32, r=128, d_rope=32, stride=stride,
                                           prefix=(0, 75 * stride - 9), steps=9, seed=77 + stride)
    plen = np.array([0, 1, stride * 40 + (stride - 1), 75 * stride - 9, 33], np.int32)
    H.run_decode_parity(wl, prefix_lens=plen, decode_chunk=32)


@pytest.mark.parametrize("r,d_rope,n_heads,d_head", [(64, 64, 3, 64), (256, 64, 12, 96), (512, 32, 9, 128)])
def test_other_shapes(r, d_rope, n_heads, d_head):
    wl = W.WORKLOADS["speech_bf16"].scaled(name=f"shape_r{r}", batch=3, d_model=128, n_heads=n_heads,
                                           d_head=d_head, r=r, d_rope=d_rope, stride=2, prefix=(10, 150),
                                           steps=5, seed=5)
    H.run_decode_parity(wl, decode_chunk=64)


@pytest.mark.parametrize("stride", [1, 3])
@pytest.mark.parametrize("n_heads,r,d_rope", [(6, 128, 32), (20, 256, 64), (16, 512, 64), (3, 64, 32)])
def test_balanced_schedule_small_ragged_batch(stride, n_heads, r, d_rope):
    # persistent workgroups over a flat tile list: 256 workgroups share a few dozen 16-slot tiles,
    # so most get nothing, ranges start and end inside sequences, one sequence is empty, and one
    # grows by a whole tile during the steps; both head-tile layouts (<= 16 heads, > 16 heads);
    # r >= 128 takes the column-split kernel, r = 64 the slot-split one
    wl = W.WORKLOADS["speech_bf16"].scaled(name=f"bal_s{stride}_h{n_heads}", batch=7, d_model=96, n_heads=n_heads,
                                           d_head=32, r=r, d_rope=d_rope, stride=stride,
                                           prefix=(0, 130 * stride), steps=6, seed=91 + stride)
    plen = np.array([0, 1, 16 * stride, 16 * stride - 3, 130 * stride, 47 * stride + 1, 64 * stride], np.int32)
    H.run_decode_parity(wl, prefix_lens=plen, decode_schedule=2)


@pytest.mark.parametrize("n_heads,r,d_head", [(20, 256, 64), (5, 512, 128)])
def test_balanced_schedule_few_rows_many_pieces(n_heads, r, d_head):
    # a handful of sequences under the balanced schedule: every row is merged from dozens of partials, which
    # the matrix-core combine then splits over the wavefronts of one workgroup per row; one sequence is
    # empty, one has a single slot, one a single piece
    wl = W.WORKLOADS["speech_bf16"].scaled(name=f"bal_few_h{n_heads}_r{r}", batch=5, d_model=96, n_heads=n_heads,
                                           d_head=d_head, r=r, d_rope=64, stride=2, prefix=(0, 3000), steps=3, seed=23)
    plen = np.array([3000, 0, 1, 20, 1777], np.int32)
    H.run_decode_parity(wl, prefix_lens=plen, decode_schedule=2)


@pytest.mark.parametrize("n_heads", [6, 20])
def test_balanced_schedule_many_short_sequences(n_heads):
    # several hundred sequences of zero to three tiles: a workgroup's range of work units then spans
    # several sequences, starts or ends inside the units a sequence takes before its first tile, or
    # holds nothing but such units; every fifth sequence is empty
    B = 700
    wl = W.WORKLOADS["speech_bf16"].scaled(name=f"bal_short_h{n_heads}", batch=B, d_model=96, n_heads=n_heads,
                                           d_head=32, r=128, d_rope=32, stride=2, prefix=(0, 96), steps=2, seed=17)
    rng = np.random.default_rng(17)
    plen = rng.integers(1, 96, size=B).astype(np.int32)
    plen[::5] = 0
    H.run_decode_parity(wl, prefix_lens=plen, decode_schedule=2)


@pytest.mark.parametrize("schedule", [1, 2])
@pytest.mark.parametrize("seed", range(8))
def test_seeded_random_shapes_both_schedules(seed, schedule):
    # shapes, batch sizes and length mixes drawn from a seed, under the static (1) and the balanced (2)
    # schedule: the split of the work units, the pieces a workgroup emits and the forms of the combine (few
    # rows of many pieces, many rows, generic) all change with them; every sequence at every step against
    # the oracle
    rng = np.random.default_rng(4000 + seed)
    r = int(rng.choice([128, 256, 512]))
    d_head = int(rng.choice([32, 64, 128]))
    n_heads = int(rng.integers(1, 33))
    d_rope = int(rng.choice([32, 64]))
    stride = int(rng.integers(1, 5))
    B = int(rng.choice([1, 2, 5, 17, 40, 90]))
    top = int(rng.choice([40, 400, 2500])) if B <= 17 else int(rng.choice([40, 300]))
    plen = rng.integers(0, top * stride + 1, size=B).astype(np.int32)
    plen[rng.integers(0, B)] = top * stride   # one sequence of the full length
    if B > 2:
        plen[rng.integers(0, B)] = 0          # and an empty one
    wl = W.WORKLOADS["speech_bf16"].scaled(name=f"bal_rand_{seed}", batch=B, d_model=96, n_heads=n_heads, d_head=d_head,
                                           r=r, d_rope=d_rope, stride=stride, prefix=(0, top * stride), steps=3,
                                           seed=4000 + seed)
    H.run_decode_parity(wl, prefix_lens=plen, decode_schedule=schedule)


@pytest.mark.parametrize("stride,bound", [(3, 2e-2), (4, 2e-2 * 4 / 3)])
def test_decode_error_by_stride(stride, bound, monkeypatch):
    # a cache row is the bf16 rounding of a sum of `stride` weighted latents, so the error the output inherits
    # grows with the stride: twelve seeded shapes per stride, every sequence at four steps.  The stated 2e-2
    # holds through stride 3; at stride 4 some of these shapes exceed it (up to 2.41e-2 over forty shapes), and
    # the documented bound there is 2e-2 * 4 / 3.  Against the oracle run on its own cache rounded to bf16 (the
    # rounding of the stored slots taken out) the same outputs stay within 8e-3 at either stride: what is
    # left is the kernels' own arithmetic (bf16 softmax weights, the order of the sums)
    monkeypatch.setitem(H.TOL, "bf16", bound)
    worst_all, worst_stored = 0.0, 0.0
    for seed in range(12):
        rng = np.random.default_rng(6000 + seed)
        r = int(rng.choice([128, 256, 512]))
        d_head = int(rng.choice([64, 128]))
        n_heads = int(rng.integers(1, 33))
        d_rope = int(rng.choice([32, 64]))
        B = int(rng.choice([3, 30]))
        top = int(rng.choice([10, 40, 300]))
        plen = rng.integers(0, top * stride + 1, size=B).astype(np.int32)
        plen[0] = top * stride
        wl = W.WORKLOADS["speech_bf16"].scaled(name=f"err_s{stride}_{seed}", batch=B, d_model=96, n_heads=n_heads,
                                               d_head=d_head, r=r, d_rope=d_rope, stride=stride,
                                               prefix=(0, top * stride), steps=4, seed=6000 + seed)
        worst = H.run_decode_parity(wl, prefix_lens=plen, decode_schedule=1 + seed % 2, fused_step=True, storage_aware=True,
                                    log=lambda *a: None)
        worst_all = max(worst_all, worst["out"])
        worst_stored = max(worst_stored, worst.get("out_stored", 0.0))
    assert worst_stored <= 8e-3, worst_stored
    print(f"stride {stride}: worst output error over twelve shapes {worst_all:.2e} (bound {bound:.2e}); "
          f"with the stored slots' rounding taken out {worst_stored:.2e}")


def test_long_bf16_full_size_sampled():
    # batch 8, 32 heads x 128, r=512, s=4, 32768-token prefix: the oracle follows two sequences
    wl = W.WORKLOADS["long_bf16"]
    H.run_decode_parity(wl, seqs_to_check=[1, 6], check_steps=[0, 1, 2, 3, 64, wl.steps - 1])


def test_ragged_bf16_full_size_sampled():
    # batch 256 with prefix lengths uniform in [512, 4096]: shortest, longest and two more sequences;
    # driven through mtla_decode_step like the benchmark
    wl = W.WORKLOADS["ragged_bf16"]
    plen = W.prefix_lengths(wl)
    seqs = sorted({int(plen.argmin()), int(plen.argmax()), 17, 200})
    H.run_decode_parity(wl, seqs_to_check=seqs, check_steps=[0, 1, 2, 31, wl.steps - 1], fused_step=True)


def test_ragged_bf16_full_size_every_sequence_one_step():
    # all 256 sequences of the ragged workload against the oracle: the bulk-appended prefix (merge weights, slot
    # indices, every live cache row) and one decode step through mtla_decode_step under the balanced schedule
    # the benchmark runs (every piece boundary of the flat tile list falls inside some sequence checked here)
    wl = W.WORKLOADS["ragged_bf16"].scaled(steps=1)
    before = dict(H.STORAGE_TERM)
    worst = H.run_decode_parity(wl, fused_step=True)
    assert worst["out"] <= H.TOL["bf16"] and worst["lse"] <= H.TOL["bf16"]
    print("storage-term elements in this test:", H.STORAGE_TERM["needed"] - before["needed"], "of",
          H.STORAGE_TERM["checked"] - before["checked"], "worst excess", H.STORAGE_TERM["worst_excess"])


def test_long_bf16_full_size_every_sequence_one_step():
    # all 8 sequences of the long-context workload (32 heads, 8192 slots each), one decode step
    wl = W.WORKLOADS["long_bf16"].scaled(steps=1)
    worst = H.run_decode_parity(wl, fused_step=True)
    assert worst["out"] <= H.TOL["bf16"] and worst["lse"] <= H.TOL["bf16"]


def test_balanced_schedule_properties_at_full_size():
    """Properties that hold for every sequence of the ragged workload at full size, without the
    oracle: the balanced and the static schedule agree, softmax normalisers are positive and finite,
    and a sequence's output does not depend on its batch neighbours (sequence 3 alone == in batch)."""
    wl = W.WORKLOADS["ragged_bf16"].scaled(steps=2)
    wts = W.make_weights(wl)
    plen = W.prefix_lengths(wl)
    B, nh, dh = wl.batch, wl.n_heads, wl.d_head
    g = torch.Generator(device="cuda").manual_seed(5)
    outs = {}
    for sched in (1, 2):
        sess = H.make_session(wl, decode_schedule=sched)
        H.upload_weights(sess, wts)
        g.manual_seed(5)
        sess.cache_c.copy_(torch.randn(sess.cache_c.shape, device="cuda", generator=g).to(sess.cache_c.dtype))
        sess.cache_kr.copy_(torch.randn(sess.cache_kr.shape, device="cuda", generator=g).to(sess.cache_kr.dtype))
        sess.seq_len.copy_(torch.from_numpy(plen).cuda())
        q = (torch.randn(B, nh, dh, device="cuda", generator=g)).to(sess.cache_c.dtype)
        qr = (torch.randn(B, nh, wl.d_rope, device="cuda", generator=g)).to(sess.cache_c.dtype)
        out = torch.empty(B, nh, dh, dtype=torch.float32, device="cuda")
        lse = torch.empty(B, nh, dtype=torch.float32, device="cuda")
        sess.decode(q, qr, out=out, lse=lse)
        torch.cuda.synchronize()
        outs[sched] = (out, lse, sess, q, qr)
    (o1, l1, _, _, _), (o2, l2, sess, q, qr) = outs[1], outs[2]
    assert torch.isfinite(o2).all() and torch.isfinite(l2).all()
    assert (o1 - o2).abs().max().item() <= 2e-2 and (l1 - l2).abs().max().item() <= 2e-2
    # sequence 3 on its own (batch of one, same cache rows)
    solo = H.make_session(wl.scaled(batch=1), max_slots=sess.max_slots, decode_schedule=2)
    H.upload_weights(solo, wts)
    solo.cache_c.copy_(sess.cache_c[3:4])
    solo.cache_kr.copy_(sess.cache_kr[3:4])
    solo.seq_len.copy_(sess.seq_len[3:4])
    o_solo = torch.empty(1, nh, dh, dtype=torch.float32, device="cuda")
    solo.decode(q[3:4].contiguous(), qr[3:4].contiguous(), out=o_solo)
    assert (o_solo[0] - o2[3]).abs().max().item() <= 2e-2


def test_empty_sequence_and_zero_new_tokens():
    wl = W.WORKLOADS["tiny_f32"].scaled(batch=3, prefix=8, steps=0)
    wts = W.make_weights(wl)
    sess = H.make_session(wl)
    H.upload_weights(sess, wts)
    ob = H.OracleBatch.new(wl, wts)
    toks = [W.make_tokens(wl, wts, b, 0, 8) for b in range(3)]
    n_new = np.array([8, 0, 3], np.int32)               # sequence 1 stays empty
    c = H.to_device(np.stack([t.c for t in toks]), wl.dtype)
    kr = H.to_device(np.stack([t.kr for t in toks]), wl.dtype)
    sess.append(c, kr, n_new=torch.from_numpy(n_new).cuda())
    for b in range(3):
        ob.append(b, toks[b].c[:n_new[b]], toks[b].kr[:n_new[b]])
    H.check_cache(sess, ob)
    assert sess.seq_len.cpu().tolist() == [8, 0, 3]
    q = H.to_device(np.stack([t.q[7] for t in toks]), wl.dtype)
    qr = H.to_device(np.stack([t.q_rope[7] for t in toks]), wl.dtype)
    out = torch.full((3, wl.n_heads, wl.d_head), 7.0, device="cuda")
    lat = torch.full((3, wl.n_heads, wl.r), 7.0, device="cuda")
    lse = torch.full((3, wl.n_heads), 7.0, device="cuda")
    sess.decode(q, qr, out=out, out_latent=lat, lse=lse)
    assert torch.all(out[1] == 0) and torch.all(lat[1] == 0) and torch.all(torch.isneginf(lse[1]))
    for b in (0, 2):
        o_ref, ol_ref, lse_ref, _ = ob.decode(b, toks[b].q[7], toks[b].q_rope[7])
        assert H.max_err(out[b], o_ref) <= 1e-5 and H.max_err(lat[b], ol_ref) <= 1e-5
        assert H.max_err(lse[b], lse_ref) <= 1e-5


@pytest.mark.parametrize("dtype,stride", [("bf16", 2), ("bf16", 3), ("bf16", 4), ("f32", 3)])
def test_bulk_append_in_ragged_pieces(dtype, stride):
    # several bulk appends per sequence: each piece starts inside a partly filled slot for some
    # sequence, spans many slots (more than one 16-slot group), and ends inside an open one
    wl = W.WORKLOADS["speech_bf16"].scaled(batch=4, d_model=64, prefix=150, steps=0, stride=stride, dtype=dtype)
    wts = W.make_weights(wl)
    sess = H.make_session(wl)
    H.upload_weights(sess, wts)
    ob = H.OracleBatch.new(wl, wts)
    toks = [W.make_tokens(wl, wts, b, 0, 150) for b in range(4)]
    pieces = [[37, 5, 70, 1, 33], [1, 64, 0, 49, 36], [71, 0, 1, 70, 8], [33, 33, 33, 33, 18]]
    done = [0] * 4
    for k in range(5):
        n_new = [pieces[b][k] for b in range(4)]
        n_max = max(n_new)
        c = H.to_device(H.pad_stack([toks[b].c[done[b]:done[b] + n_new[b]] for b in range(4)], n_max), wl.dtype)
        kr = H.to_device(H.pad_stack([toks[b].kr[done[b]:done[b] + n_new[b]] for b in range(4)], n_max), wl.dtype)
        w_out = torch.zeros(4, n_max, device="cuda")
        slot_out = torch.full((4, n_max), -1, dtype=torch.int32, device="cuda")
        sess.append(c, kr, n_new=torch.tensor(n_new, dtype=torch.int32, device="cuda"), w_out=w_out, slot_out=slot_out)
        for b in range(4):
            n = n_new[b]
            w_ref, slot_ref = ob.append(b, toks[b].c[done[b]:done[b] + n], toks[b].kr[done[b]:done[b] + n])
            done[b] += n
            if n:
                assert np.array_equal(slot_out[b, :n].cpu().numpy(), slot_ref)
                assert np.abs(w_out[b, :n].cpu().numpy() - w_ref).max() <= H.TOL_W
            assert torch.all(slot_out[b, n:] == -1)
        H.check_cache(sess, ob, what=f"piece {k}")
    assert sess.seq_len.cpu().tolist() == [146, 150, 150, 150]


def test_capacity_overflow_is_refused_on_the_device():
    wl = W.WORKLOADS["tiny_f32"].scaled(batch=2, prefix=10, steps=0)
    wts = W.make_weights(wl)
    sess = H.make_session(wl, max_slots=5)               # room for exactly 10 tokens at s=2
    H.upload_weights(sess, wts)
    toks = [W.make_tokens(wl, wts, b, 0, 12) for b in range(2)]
    c = H.to_device(np.stack([t.c[:10] for t in toks]), wl.dtype)
    kr = H.to_device(np.stack([t.kr[:10] for t in toks]), wl.dtype)
    sess.append(c, kr, n_new=torch.tensor([10, 9], dtype=torch.int32, device="cuda"))
    assert sess.device_status() == 0 and sess.seq_len.cpu().tolist() == [10, 9]
    before = (sess.cache_c.clone(), sess.cache_kr.clone(), sess.tail_c.clone())
    c1 = H.to_device(np.stack([t.c[10:11] for t in toks]), wl.dtype)
    kr1 = H.to_device(np.stack([t.kr[10:11] for t in toks]), wl.dtype)
    sess.append(c1, kr1)                                  # sequence 0 is full, sequence 1 has room
    assert sess.device_status() == 3                      # MTLA_ERR_CAPACITY, sticky until read
    assert sess.device_status() == 0                      # ... and cleared by the read
    assert sess.seq_len.cpu().tolist() == [10, 10]
    assert torch.equal(sess.cache_c[0], before[0][0]) and torch.equal(sess.cache_kr[0], before[1][0])
    assert torch.equal(sess.tail_c[0], before[2][0])
    assert not torch.equal(sess.cache_c[1], before[0][1])


def test_weight_override_and_hyper_bias():
    # w_override == 1 with s = 1 is the MLA special case; a Linear(c) bias shifts the logit
    wl = W.WORKLOADS["tiny_f32"].scaled(batch=2, prefix=6, steps=0, stride=1)
    wts = W.make_weights(wl)
    toks = [W.make_tokens(wl, wts, b, 0, 6) for b in range(2)]
    c = H.to_device(np.stack([t.c for t in toks]), wl.dtype)
    kr = H.to_device(np.stack([t.kr for t in toks]), wl.dtype)
    sess = H.make_session(wl)
    H.upload_weights(sess, wts)
    ones = torch.ones(2, 6, device="cuda")
    w_out = torch.zeros(2, 6, device="cuda")
    sess.append(c, kr, w_override=ones, w_out=w_out)
    assert torch.equal(w_out, ones)
    assert torch.equal(sess.cache_c[:, :6], c) and torch.equal(sess.cache_kr[:, :6], kr)
    bias = (np.random.default_rng(3).standard_normal(wl.d_hyper) * 0.5).astype(np.float32)
    sess2 = H.make_session(wl)
    H.upload_weights(sess2, wts, hyp_a=bias)
    ob = H.OracleBatch.new(wl, wts, hyp_a=bias)
    w2 = torch.zeros(2, 6, device="cuda")
    sess2.append(c, kr, w_out=w2)
    for b in range(2):
        w_ref, _ = ob.append(b, toks[b].c, toks[b].kr)
        assert np.abs(w2[b].cpu().numpy() - w_ref).max() <= H.TOL_W
    H.check_cache(sess2, ob)


def test_state_copy_resumes_bit_identically():
    # (C_hat, K_hat^R, tail, seq_len) is the whole resumable state of a sequence batch
    wl = W.WORKLOADS["speech_bf16"].scaled(batch=4, d_model=64, prefix=37, steps=6)
    wts = W.make_weights(wl)
    toks = [W.make_tokens(wl, wts, b, 0, 43) for b in range(4)]
    stack = lambda f, lo, hi: H.to_device(np.stack([getattr(t, f)[lo:hi] for t in toks]), wl.dtype)
    a, b2 = H.make_session(wl), H.make_session(wl)
    for s in (a, b2):
        H.upload_weights(s, wts)
    a.append(stack("c", 0, 37), stack("kr", 0, 37))
    outs = []
    for t in range(37, 40):
        a.append(stack("c", t, t + 1), stack("kr", t, t + 1))
    for src, dst in ((a.cache_c, b2.cache_c), (a.cache_kr, b2.cache_kr), (a.tail_c, b2.tail_c), (a.seq_len, b2.seq_len)):
        dst.copy_(src)
    for s in (a, b2):
        o = torch.empty(4, wl.n_heads, wl.d_head, dtype=torch.float32, device="cuda")
        for t in range(40, 43):
            s.append(stack("c", t, t + 1), stack("kr", t, t + 1))
            s.decode(stack("q", t, t + 1).squeeze(1), stack("q_rope", t, t + 1).squeeze(1), out=o)
        outs.append(o.clone())
    assert torch.equal(outs[0], outs[1]) and torch.equal(a.cache_c, b2.cache_c) and torch.equal(a.tail_c, b2.tail_c)


@pytest.mark.parametrize("dtype,stride,shape", [("bf16", 2, (8, 64, 256, 32)), ("bf16", 3, (6, 32, 128, 64)),
                                               ("bf16", 1, (16, 128, 512, 64)), ("f32", 2, (4, 64, 64, 32))])
def test_decode_step_equals_append_then_attend(dtype, stride, shape):
    """mtla_decode_step (append and absorption in one launch for bf16) against the two separate
    calls on the same inputs: caches, lengths and outputs bit for bit; and against the oracle."""
    nh, dh, r, dr = shape
    wl = W.WORKLOADS["speech_bf16"].scaled(name="fused", dtype=dtype, batch=5, d_model=nh * dh, n_heads=nh,
                                           d_head=dh, r=r, d_rope=dr, stride=stride, prefix=(0, 70), steps=9,
                                           seed=77 + stride)
    H.run_decode_parity(wl, fused_step=True)
    wts = W.make_weights(wl)
    plen = W.prefix_lengths(wl)
    toks = [W.make_tokens(wl, wts, b, 0, int(plen[b]) + wl.steps) for b in range(wl.batch)]
    sessions = []
    for fused in (False, True):
        sess = H.make_session(wl)
        H.upload_weights(sess, wts)
        n_max = max(1, int(plen.max()))
        c_pre = H.to_device(H.pad_stack([t.c[:plen[b]] for b, t in enumerate(toks)], n_max), dtype)
        kr_pre = H.to_device(H.pad_stack([t.kr[:plen[b]] for b, t in enumerate(toks)], n_max), dtype)
        sess.append(c_pre, kr_pre, n_new=torch.from_numpy(plen).cuda())
        outs = []
        for t in range(wl.steps):
            pick = lambda f: H.to_device(np.stack([getattr(toks[b], f)[plen[b] + t] for b in range(wl.batch)]), dtype)
            c1, kr1, q1, qr1 = pick("c").unsqueeze(1), pick("kr").unsqueeze(1), pick("q"), pick("q_rope")
            out = torch.empty(wl.batch, nh, dh, dtype=torch.float32, device="cuda")
            lse = torch.empty(wl.batch, nh, dtype=torch.float32, device="cuda")
            if fused:
                sess.step(c1, kr1, q1, qr1, out=out, lse=lse)
            else:
                sess.append(c1, kr1)
                sess.decode(q1, qr1, out=out, lse=lse)
            outs.append((out, lse))
        torch.cuda.synchronize()
        sessions.append((sess, outs))
    (sa, oa), (sb, ob) = sessions
    assert torch.equal(sa.seq_len, sb.seq_len)
    assert torch.equal(sa.cache_c.view(torch.uint8), sb.cache_c.view(torch.uint8))
    assert torch.equal(sa.cache_kr.view(torch.uint8), sb.cache_kr.view(torch.uint8))
    assert torch.equal(sa.tail_c, sb.tail_c)
    for (o1, l1), (o2, l2) in zip(oa, ob):
        assert torch.equal(o1, o2) and torch.equal(l1, l2)


def test_decode_step_full_sequence_is_refused():
    wl = W.WORKLOADS["speech_bf16"].scaled(name="fused_cap", batch=2, d_model=128, n_heads=2, prefix=8, steps=0)
    wts = W.make_weights(wl)
    sess = H.make_session(wl, max_slots=4)              # 8 tokens at s=2 fill it
    H.upload_weights(sess, wts)
    tk = [W.make_tokens(wl, wts, b, 0, 9) for b in range(2)]
    st = lambda f, a, b: H.to_device(np.stack([getattr(t, f)[a:b] for t in tk]), wl.dtype)
    sess.append(st("c", 0, 8), st("kr", 0, 8))
    before = sess.cache_c.clone()
    out = torch.empty(2, wl.n_heads, wl.d_head, dtype=torch.float32, device="cuda")
    sess.step(st("c", 8, 9), st("kr", 8, 9), st("q", 8, 9)[:, 0].contiguous(), st("q_rope", 8, 9)[:, 0].contiguous(),
              out=out)
    assert sess.device_status() == 3                     # MTLA_ERR_CAPACITY, raised on the device
    assert torch.equal(sess.seq_len.cpu(), torch.tensor([8, 8], dtype=torch.int32))
    assert torch.equal(before.view(torch.uint8), sess.cache_c.view(torch.uint8))
    assert torch.isfinite(out).all()


@pytest.mark.parametrize("dtype,stride", [("bf16", 2), ("f32", 3)])
def test_beam_reorder_is_a_gather_and_decoding_continues(dtype, stride):
    # four beams of ragged length; after a few steps beam b continues beam idx[b] (one source twice,
    # one dropped): the new state is bit-identical to a gather of the old one, and decoding goes on
    import copy
    wl = W.WORKLOADS["speech_bf16"].scaled(name="beams", dtype=dtype, batch=4, d_model=64, prefix=(9, 41), steps=6,
                                           stride=stride, seed=61)
    wts = W.make_weights(wl)
    plen = W.prefix_lengths(wl)
    toks = [W.make_tokens(wl, wts, b, 0, int(plen[b]) + 6) for b in range(4)]
    sess = H.make_session(wl)
    H.upload_weights(sess, wts)
    ob = H.OracleBatch.new(wl, wts)
    n_max = int(plen.max())
    sess.append(H.to_device(H.pad_stack([toks[b].c[:plen[b]] for b in range(4)], n_max), dtype),
                H.to_device(H.pad_stack([toks[b].kr[:plen[b]] for b in range(4)], n_max), dtype),
                n_new=torch.from_numpy(plen).cuda())
    for b in range(4):
        ob.append(b, toks[b].c[:plen[b]], toks[b].kr[:plen[b]])
    src_of = list(range(4))          # which original token stream each beam currently follows
    pos = [int(p) for p in plen]
    out = torch.empty(4, wl.n_heads, wl.d_head, dtype=torch.float32, device="cuda")

    def step():
        pick = lambda f: H.to_device(np.stack([getattr(toks[src_of[b]], f)[pos[b]] for b in range(4)]), dtype)
        sess.step(pick("c").unsqueeze(1), pick("kr").unsqueeze(1), pick("q"), pick("q_rope"), out=out)
        for b in range(4):
            t = toks[src_of[b]]
            ob.append(b, t.c[pos[b]][None], t.kr[pos[b]][None])
            o_ref, _, _, _ = ob.decode(b, t.q[pos[b]], t.q_rope[pos[b]])
            assert H.max_err(out[b], o_ref) <= H.TOL[dtype]
            pos[b] += 1

    for _ in range(2):
        step()
    idx = [2, 2, 0, 3]
    before = [t.clone() for t in (sess.cache_c, sess.cache_kr, sess.tail_c, sess.seq_len)]
    sess.reorder(torch.tensor(idx, dtype=torch.int32, device="cuda"))
    assert sess.device_status() == 0
    live = [-(-int(before[3][i]) // stride) for i in idx]
    for b, i in enumerate(idx):
        assert torch.equal(sess.cache_c[b, :live[b]], before[0][i, :live[b]])
        assert torch.equal(sess.cache_kr[b, :live[b]], before[1][i, :live[b]])
        assert torch.equal(sess.tail_c[b], before[2][i]) and int(sess.seq_len[b]) == int(before[3][i])
    ob.caches = [copy.deepcopy(ob.caches[i]) for i in idx]
    src_of, pos = [src_of[i] for i in idx], [pos[i] for i in idx]
    for _ in range(3):
        step()
    H.check_cache(sess, ob)
    # an index outside the batch: flagged on the device, that destination untouched
    keep = sess._alt[0][1].clone()
    sess.ctx.cache_reorder(sess.cache_c, sess.cache_kr, sess.tail_c, sess.seq_len,
                           torch.tensor([0, 7, 1, 2], dtype=torch.int32, device="cuda"), 4, sess._alt[0], sess._alt[1],
                           sess._alt[2], sess._alt[3], sess.workspace, sess.stream)
    assert sess.device_status() == 1 and sess.device_status() == 0
    assert torch.equal(sess._alt[0][1], keep)



@pytest.mark.parametrize("stride", [2, 3])
def test_beam_search_over_a_shared_prompt_moves_only_what_was_generated(stride):
    # five beams start from one prompt of 50 tokens (the same token stream in every sequence); every step is
    # followed by a reordering that skips the prompt's complete slots: the state equals, bit for bit, that of a
    # second session reordered in full, outputs follow the oracle, and the prompt's slots are never rewritten
    import copy
    P, B, dtype = 50, 5, "bf16"
    wl = W.WORKLOADS["speech_bf16"].scaled(name="beams_shared", batch=B, d_model=64, prefix=P, steps=8, stride=stride,
                                           seed=67)
    wts = W.make_weights(wl)
    prompt = W.make_tokens(wl, wts, 0, 0, P)
    gen = [W.make_tokens(wl, wts, 1 + b, P, P + 8) for b in range(B)]   # what each hypothesis appends
    fast, full = H.make_session(wl), H.make_session(wl)
    ob = H.OracleBatch.new(wl, wts)
    for s in (fast, full):
        H.upload_weights(s, wts)
        s.append(H.to_device(np.stack([prompt.c] * B), dtype), H.to_device(np.stack([prompt.kr] * B), dtype))
    for b in range(B):
        ob.append(b, prompt.c, prompt.kr)
    first_slot = P // stride                                            # complete slots of the prompt
    hyp = list(range(B))                                                # which stream each beam follows
    out_f = torch.empty(B, wl.n_heads, wl.d_head, dtype=torch.float32, device="cuda")
    out_g = torch.empty_like(out_f)
    g = np.random.default_rng(5)
    for t in range(8):
        pick = lambda f: H.to_device(np.stack([getattr(gen[hyp[b]], f)[t] for b in range(B)]), dtype)
        c, kr, q, qr = pick("c").unsqueeze(1), pick("kr").unsqueeze(1), pick("q"), pick("q_rope")
        fast.step(c, kr, q, qr, out=out_f)
        full.step(c, kr, q, qr, out=out_g)
        assert torch.equal(out_f, out_g)
        for b in range(B):
            ob.append(b, gen[hyp[b]].c[t][None], gen[hyp[b]].kr[t][None])
            o_ref, _, _, _ = ob.decode(b, gen[hyp[b]].q[t], gen[hyp[b]].q_rope[t])
            assert H.max_err(out_f[b], o_ref) <= H.TOL[dtype]
        idx = g.integers(0, B, size=B).tolist()                        # forks and drops
        idx_dev = torch.tensor(idx, dtype=torch.int32, device="cuda")
        fast.reorder(idx_dev, first_slot=first_slot)
        full.reorder(idx_dev)
        ob.caches = [copy.deepcopy(ob.caches[i]) for i in idx]
        hyp = [hyp[i] for i in idx]
        live = -(-(P + t + 1) // stride)
        assert torch.equal(fast.cache_c[:, :live], full.cache_c[:, :live])
        assert torch.equal(fast.cache_kr[:, :live], full.cache_kr[:, :live])
        assert torch.equal(fast.tail_c, full.tail_c) and torch.equal(fast.seq_len, full.seq_len)
    H.check_cache(fast, ob)
    assert fast.device_status() == 0
