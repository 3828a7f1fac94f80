"""mtla_decode_step_static (the decode step for callers that cannot bring a workspace: its scratch
is a static device array of the library) against mtla_decode_step, through the C-ABI: two calls in
a row on the same GPU, the second with a smaller batch, so the second finds the first one's
leftovers in the shared array."""
import numpy as np
import pytest
import torch

import workloads as W
from paper_2505_13544_amd import binding as B
from tests import harness as H

pytestmark = pytest.mark.gpu


def _prefix_and_steps(wl, wts, plen, steps, dev="cuda:0"):
    toks = [W.make_tokens(wl, wts, b, 0, int(plen[b]) + steps) for b in range(wl.batch)]
    n_max = int(plen.max())
    pre = {f: H.to_device(H.pad_stack([getattr(t, f)[:plen[b]] for b, t in enumerate(toks)], n_max), wl.dtype, dev)
           for f in ("c", "kr")}
    step = {f: [H.to_device(np.stack([getattr(toks[b], f)[plen[b] + t] for b in range(wl.batch)]), wl.dtype, dev)
                for t in range(steps)] for f in ("c", "kr", "q", "q_rope")}
    return toks, pre, step


@pytest.mark.parametrize("schedule", [1, 2])
def test_static_scratch_step_matches_the_workspace_step(schedule):
    wl = W.WORKLOADS["speech_bf16"].scaled(batch=6, prefix=150, steps=2, d_model=128)
    wts = W.make_weights(wl)
    plen = np.array([150, 33, 97, 1, 64, 129], np.int32)
    toks, pre, step = _prefix_and_steps(wl, wts, plen, wl.steps)
    sessions = []
    for _ in range(2):  # [0] brings its own workspace, [1] uses the library's static scratch
        s = H.make_session(wl, max_slots=(150 + wl.steps + wl.stride - 1) // wl.stride, decode_schedule=schedule)
        H.upload_weights(s, wts)
        s.append(pre["c"], pre["kr"], n_new=torch.from_numpy(plen).cuda())
        sessions.append(s)
    ref, sta = sessions
    assert ref.ctx.workspace_bytes() <= B.MTLA_STATIC_SCRATCH_BYTES
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    ob = H.OracleBatch.new(wl, wts)
    for b in range(wl.batch):
        ob.append(b, toks[b].c[:plen[b]], toks[b].kr[:plen[b]])
    # call 1: the whole batch; call 2: the first three sequences only (the other rows of the
    # scratch keep what call 1 left there)
    for t, batch in enumerate((wl.batch, 3)):
        outs = []
        for s, static in ((ref, False), (sta, True)):
            o = torch.full((batch, wl.n_heads, wl.d_head), 7.0, dtype=torch.float32, device="cuda")
            ol = torch.full((batch, wl.n_heads, wl.r), 7.0, dtype=torch.float32, device="cuda")
            ls = torch.full((batch, wl.n_heads), 7.0, dtype=torch.float32, device="cuda")
            a = [step[f][t][:batch].contiguous() for f in ("c", "kr", "q", "q_rope")]
            if static:
                s.step_static(a[0].unsqueeze(1), a[1].unsqueeze(1), a[2], a[3], status=status, out=o, out_latent=ol,
                              lse=ls)
            else:
                s.step(a[0].unsqueeze(1), a[1].unsqueeze(1), a[2], a[3], out=o, out_latent=ol, lse=ls)
            outs.append((o, ol, ls))
        torch.cuda.synchronize()
        for x, y in zip(*outs):  # the same kernels on the same inputs
            assert torch.equal(x, y), f"call {t + 1}: static-scratch step differs from the workspace step"
        for name in ("cache_c", "cache_kr", "tail_c", "seq_len"):
            assert torch.equal(getattr(ref, name), getattr(sta, name)), f"call {t + 1}: {name} differs"
        for b in range(batch):  # and both are right
            ob.append(b, toks[b].c[plen[b] + t][None], toks[b].kr[plen[b] + t][None])
            o_ref, _, lse_ref, _ = ob.decode(b, toks[b].q[plen[b] + t], toks[b].q_rope[plen[b] + t])
            assert H.max_err(outs[1][0][b], o_ref) <= H.TOL["bf16"]
            assert H.max_err(outs[1][2][b], lse_ref) <= H.TOL["bf16"]
    assert int(status.item()) == 0 and ref.device_status() == 0


def test_static_scratch_step_reports_a_full_sequence_in_the_callers_word():
    wl = W.WORKLOADS["speech_bf16"].scaled(batch=2, prefix=8, steps=1, d_model=128)
    wts = W.make_weights(wl)
    plen = np.array([8, 5], np.int32)
    toks, pre, step = _prefix_and_steps(wl, wts, plen, 1)
    s = H.make_session(wl, max_slots=4)  # 8 tokens at stride 2: sequence 0 is full
    H.upload_weights(s, wts)
    s.append(pre["c"], pre["kr"], n_new=torch.from_numpy(plen).cuda())
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    o = torch.empty(2, wl.n_heads, wl.d_head, dtype=torch.float32, device="cuda")
    s.step_static(step["c"][0].unsqueeze(1), step["kr"][0].unsqueeze(1), step["q"][0], step["q_rope"][0], status=status,
                  out=o)
    torch.cuda.synchronize()
    assert int(status.item()) == B.MTLA_ERR_CAPACITY
    assert s.seq_len.cpu().tolist() == [8, 6]
    assert s.device_status() == 0  # the session's own workspace was not involved


def test_static_scratch_step_refuses_a_context_that_does_not_fit():
    big = B.Context(n_heads=32, d_head=128, r=512, d_rope=64, d_hyper=64, stride=4, max_batch=8, max_slots=8224,
                    dtype="bf16")
    assert big.workspace_bytes() > B.MTLA_STATIC_SCRATCH_BYTES
    one = torch.zeros(64, dtype=torch.int32, device="cuda")
    st = big.decode_step_static_status(*([one] * 13), 1, one, None, None, one)
    assert st == B.MTLA_ERR_SCRATCH
