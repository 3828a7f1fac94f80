"""GPU test of mtla_set_shared_prefix: beams that read the slots of a common prompt from one stored copy.
Two sessions decode the same streams.  In the first every sequence holds its own copy of its group's prompt;
in the second only the group's first sequence does, the other sequences' rows of those slots are overwritten
with NaN, and the decode calls are told where to read them instead.  The kernels do the same arithmetic in the
same order on the same values, so the outputs are compared bit for bit; the first session is also compared
with the float64 oracle (2e-2, bf16 storage)."""
import numpy as np
import pytest
import torch

import workloads as W
from paper_2505_13544_amd.binding import MtlaError
from tests import harness as H

pytestmark = pytest.mark.gpu


def _groups(wl, wts, prompts, steps):
    """Token streams: sequence b of group k = the group's prompt, then tokens of its own."""
    streams = []
    for k, (members, P) in enumerate(prompts):
        prompt = W.make_tokens(wl, wts, 100 + k, 0, P)
        for b in members:
            own = W.make_tokens(wl, wts, b, P, P + steps)
            streams.append((prompt, own))
    return streams


@pytest.mark.parametrize("schedule,n_heads,d_head,r,d_rope,stride",
                         [(1, 8, 64, 256, 32, 2), (2, 8, 64, 256, 32, 3), (2, 16, 128, 512, 64, 2),
                          (2, 32, 64, 512, 64, 2), (1, 32, 64, 128, 64, 3), (2, 4, 64, 128, 32, 4)])
def test_decode_over_one_stored_copy_of_a_prompt_equals_own_copies(schedule, n_heads, d_head, r, d_rope, stride):
    # groups (sequences, prompt tokens): prompts that end inside a slot, a group of one, both schedules, one and
    # two head tiles, all three latent widths of the column-split kernel
    prompts, steps, dtype = [((0, 1, 2), 50), ((3, 4, 5, 6), 33), ((7,), 20)], 7, "bf16"
    B = 8
    wl = W.WORKLOADS["speech_bf16"].scaled(name="shared_prefix", batch=B, d_model=64, n_heads=n_heads, d_head=d_head, r=r,
                                           d_rope=d_rope, stride=stride, prefix=50, steps=steps, seed=71 + stride)
    wts = W.make_weights(wl)
    streams = _groups(wl, wts, prompts, steps)
    own, shared = (H.make_session(wl, decode_schedule=schedule) for _ in range(2))
    ob = H.OracleBatch.new(wl, wts)
    P_of = [P for members, P in prompts for _ in members]
    owner = [members[0] for members, P in prompts for _ in members]
    n_pre = [0 if owner[b] == b else P_of[b] // stride for b in range(B)]   # complete slots of the prompt
    P_max = max(P_of)
    n_new = torch.tensor(P_of, dtype=torch.int32, device="cuda")
    for s in (own, shared):
        H.upload_weights(s, wts)
        s.append(H.to_device(H.pad_stack([st[0].c for st in streams], P_max), dtype),
                 H.to_device(H.pad_stack([st[0].kr for st in streams], P_max), dtype), n_new=n_new)
    for b in range(B):
        ob.append(b, streams[b][0].c, streams[b][0].kr)
    for b in range(B):                       # the copies that are not needed any more
        shared.cache_c[b, :n_pre[b]] = float("nan")
        shared.cache_kr[b, :n_pre[b]] = float("nan")
    shared.share_prefix(torch.tensor(owner, dtype=torch.int32, device="cuda"),
                        torch.tensor(n_pre, dtype=torch.int32, device="cuda"))
    out_o = torch.empty(B, n_heads, d_head, dtype=torch.float32, device="cuda")
    out_s = torch.empty_like(out_o)
    worst = 0.0
    for t in range(steps):
        pick = lambda f: H.to_device(np.stack([getattr(streams[b][1], f)[t] for b in range(B)]), dtype)
        c, kr, q, qr = pick("c").unsqueeze(1), pick("kr").unsqueeze(1), pick("q"), pick("q_rope")
        own.step(c, kr, q, qr, out=out_o)
        shared.step(c, kr, q, qr, out=out_s)
        torch.cuda.synchronize()
        assert torch.equal(out_s, out_o), f"step {t}: reading the prompt from its owner changed the output"
        for b in range(B):
            ob.append(b, streams[b][1].c[t][None], streams[b][1].kr[t][None])
            o_ref, _, _, _ = ob.decode(b, streams[b][1].q[t], streams[b][1].q_rope[t])
            worst = max(worst, H.max_err(out_o[b], o_ref))
    print(f"shared prefix, schedule {schedule}, {n_heads} heads, r {r}, stride {stride}: max abs err {worst:.2e}")
    assert worst <= H.TOL[dtype]
    assert own.device_status() == 0 and shared.device_status() == 0
    for b in range(B):                       # nothing wrote into the rows that were given up
        assert torch.isnan(shared.cache_c[b, :n_pre[b]].float()).all()
    # owners and slot counts outside their ranges are clamped: the call still reads inside the caches only
    shared.share_prefix(torch.tensor([-3, 99, 2, 3, 4, 5, 6, 7], dtype=torch.int32, device="cuda"),
                        torch.tensor([10 ** 6, -5, 0, 0, 0, 0, 0, 0], dtype=torch.int32, device="cuda"))
    shared.decode(q, qr, out=out_s)
    torch.cuda.synchronize()
    assert shared.device_status() == 0
    shared.share_prefix()                    # back to own rows: sequences 2.. hold NaN there, 7 is whole
    shared.decode(q, qr, out=out_s)
    torch.cuda.synchronize()
    assert torch.equal(out_s[7], out_o[7]) and torch.isnan(out_s[1]).any()


def test_shared_prefix_is_refused_where_no_kernel_follows_it():
    wl = W.WORKLOADS["tiny_f32"]
    sess = H.make_session(wl)
    idx = torch.zeros(wl.batch, dtype=torch.int32, device="cuda")
    with pytest.raises(MtlaError):           # fp32 storage
        sess.share_prefix(idx, idx)
    with pytest.raises(MtlaError):           # one array without the other
        sess.ctx.set_shared_prefix(idx, None, wl.batch)


def test_whole_layer_step_follows_the_shared_prefix():
    # four beams over one prompt, fed through the whole-layer calls: mtla_layer_prefill writes every beam's own
    # copy, three of them are then given up, and mtla_layer_decode_step reads the first beam's rows instead
    B, P, steps, stride = 4, 40, 4, 2
    wl = W.WORKLOADS["speech_bf16"].scaled(name="shared_prefix_layer", batch=B, d_model=64, stride=stride, prefix=P,
                                           steps=steps, seed=83)
    wts = W.make_weights(wl)
    lw = W.make_layer_weights(wl, wts)
    prompt = W.make_x(wl, 50, 0, P)
    own_x = [W.make_x(wl, b, P, P + steps) for b in range(B)]
    sessions = []
    for _ in range(2):
        s = H.make_session(wl)
        H.upload_weights(s, wts)
        s.set_layer_weights(w_q=lw.w_q, w_qr=lw.w_qr, w_r=lw.w_r, w_kr=lw.w_kr, w_o=lw.w_o)
        y = torch.empty(B, P, wl.d_model, dtype=torch.float32, device="cuda")
        keep = s.layer_prefill(H.to_device(np.stack([prompt] * B), wl.dtype), y=y)
        torch.cuda.synchronize()
        del keep
        sessions.append(s)
    own, shared = sessions
    n_pre = [0] + [P // stride] * (B - 1)
    for b in range(1, B):
        shared.cache_c[b, :n_pre[b]] = float("nan")
        shared.cache_kr[b, :n_pre[b]] = float("nan")
    shared.share_prefix(torch.zeros(B, dtype=torch.int32, device="cuda"), torch.tensor(n_pre, dtype=torch.int32, device="cuda"))
    y_o = torch.empty(B, wl.d_model, dtype=torch.float32, device="cuda")
    y_s = torch.empty_like(y_o)
    for t in range(steps):
        x = H.to_device(np.stack([own_x[b][t] for b in range(B)]), wl.dtype)
        own.layer_step(x, y=y_o)
        shared.layer_step(x, y=y_s)
        torch.cuda.synchronize()
        assert torch.equal(y_s, y_o) and not torch.isnan(y_s).any(), f"step {t}"
    assert shared.device_status() == 0


@pytest.mark.parametrize("stride", [2, 3])
def test_beam_search_that_never_copies_the_prompt(stride):
    # two utterances of three beams.  Only the first beam of each is prefilled; the others are expanded from it by
    # a reordering that moves the slots from `first` on (the open slot, the tail value, the length), and read the
    # slots before `first` from the first beam's rows for good.  Every step is followed by a reordering inside
    # the groups (forks and drops, the first beam's own hypothesis included) that leaves those slots alone.
    # Outputs follow the oracle; the rows the beams never received stay NaN to the end.
    import copy
    B, steps, dtype = 6, 8, "bf16"
    P_of, owner = [50, 50, 50, 33, 33, 33], [0, 0, 0, 3, 3, 3]
    wl = W.WORKLOADS["speech_bf16"].scaled(name="beams_no_copy", batch=B, d_model=64, prefix=50, steps=steps, stride=stride,
                                           seed=59 + stride)
    wts = W.make_weights(wl)
    prompts = {0: W.make_tokens(wl, wts, 100, 0, 50), 3: W.make_tokens(wl, wts, 101, 0, 33)}
    gen = [W.make_tokens(wl, wts, b, P_of[b], P_of[b] + steps) for b in range(B)]      # what each hypothesis appends
    sess = H.make_session(wl)
    H.upload_weights(sess, wts)
    ob = H.OracleBatch.new(wl, wts)
    first = min(P_of) // stride                                                        # slots no reordering touches
    c0 = H.pad_stack([prompts[owner[b]].c if owner[b] == b else prompts[owner[b]].c[:0] for b in range(B)], 50)
    kr0 = H.pad_stack([prompts[owner[b]].kr if owner[b] == b else prompts[owner[b]].kr[:0] for b in range(B)], 50)
    sess.append(H.to_device(c0, dtype), H.to_device(kr0, dtype),
                n_new=torch.tensor([P_of[b] if owner[b] == b else 0 for b in range(B)], dtype=torch.int32, device="cuda"))
    for b in range(B):
        ob.append(b, prompts[owner[b]].c, prompts[owner[b]].kr)
    sess.reorder(torch.tensor(owner, dtype=torch.int32, device="cuda"), first_slot=first)   # the expansion
    n_pre = [0 if owner[b] == b else first for b in range(B)]
    for bufs in ((sess.cache_c, sess.cache_kr), tuple(sess._alt[:2])):                 # both sets of buffers
        for b in range(B):
            bufs[0][b, :n_pre[b]] = float("nan")
            bufs[1][b, :n_pre[b]] = float("nan")
    sess.share_prefix(torch.tensor(owner, dtype=torch.int32, device="cuda"), torch.tensor(n_pre, dtype=torch.int32, device="cuda"))
    hyp = list(range(B))
    out = torch.empty(B, wl.n_heads, wl.d_head, dtype=torch.float32, device="cuda")
    g = np.random.default_rng(11)
    worst = 0.0
    for t in range(steps):
        pick = lambda f: H.to_device(np.stack([getattr(gen[hyp[b]], f)[t] for b in range(B)]), dtype)
        sess.step(pick("c").unsqueeze(1), pick("kr").unsqueeze(1), pick("q"), pick("q_rope"), out=out)
        for b in range(B):
            ob.append(b, gen[hyp[b]].c[t][None], gen[hyp[b]].kr[t][None])
            o_ref, _, _, _ = ob.decode(b, gen[hyp[b]].q[t], gen[hyp[b]].q_rope[t])
            worst = max(worst, H.max_err(out[b], o_ref))
        idx = [3 * (b // 3) + int(g.integers(0, 3)) for b in range(B)]                 # inside the group
        sess.reorder(torch.tensor(idx, dtype=torch.int32, device="cuda"), first_slot=first)
        ob.caches = [copy.deepcopy(ob.caches[i]) for i in idx]
        hyp = [hyp[i] for i in idx]
    print(f"beam search without prompt copies, stride {stride}: max abs err {worst:.2e}")
    assert worst <= H.TOL[dtype] and sess.device_status() == 0
    for b in range(B):
        assert torch.isnan(sess.cache_c[b, :n_pre[b]].float()).all()


@pytest.mark.parametrize("stride", [2, 3])
def test_chunked_prefill_reads_the_cached_prompt_from_its_owner(stride):
    # three beams continue one prompt of 41 tokens with 24 tokens of their own in one parallel-form call: the
    # prompt's complete slots are staged from the first beam's rows, the open slot and the new tokens are their own
    B, P, T, dtype = 3, 41, 24, "bf16"
    wl = W.WORKLOADS["speech_bf16"].scaled(name="shared_prefix_chunk", batch=B, d_model=64, stride=stride, prefix=P + T,
                                           steps=0, seed=87 + stride)
    wts = W.make_weights(wl)
    prompt = W.make_tokens(wl, wts, 60, 0, P)
    own_t = [W.make_tokens(wl, wts, b, P, P + T) for b in range(B)]
    n_pre = [0] + [P // stride] * (B - 1)
    outs = []
    for share in (False, True):
        s = H.make_session(wl)
        H.upload_weights(s, wts)
        s.append(H.to_device(np.stack([prompt.c] * B), dtype), H.to_device(np.stack([prompt.kr] * B), dtype))
        if share:
            for b in range(1, B):
                s.cache_c[b, :n_pre[b]] = float("nan")
                s.cache_kr[b, :n_pre[b]] = float("nan")
            s.share_prefix(torch.zeros(B, dtype=torch.int32, device="cuda"), torch.tensor(n_pre, dtype=torch.int32, device="cuda"))
        out = torch.empty(B, T, wl.n_heads, wl.d_head, dtype=torch.float32, device="cuda")
        pick = lambda f: H.to_device(np.stack([getattr(own_t[b], f) for b in range(B)]), dtype)
        keep = s.prefill_chunk(pick("q"), pick("q_rope"), pick("c"), pick("kr"), out=out, max_past_slots=-(-P // stride))
        torch.cuda.synchronize()
        del keep
        assert s.device_status() == 0 and s.seq_len.cpu().tolist() == [P + T] * B
        outs.append(out)
    assert torch.equal(outs[0], outs[1]) and not torch.isnan(outs[1]).any()
    ob = H.OracleBatch.new(wl, wts)          # and the first session follows the oracle
    worst = 0.0
    for b in range(B):
        ob.append(b, prompt.c, prompt.kr)
        for t in range(T):
            ob.append(b, own_t[b].c[t][None], own_t[b].kr[t][None])
            o_ref, _, _, _ = ob.decode(b, own_t[b].q[t], own_t[b].q_rope[t])
            worst = max(worst, H.max_err(outs[0][b, t], o_ref))
    print(f"chunked prefill over a shared prompt, stride {stride}: max abs err {worst:.2e}")
    assert worst <= H.TOL[dtype]
