#!/usr/bin/env python3
"""MTLA decode benchmark on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic input:
mtla_decode_step = mtla_cache_append (one new token per sequence: hyper-network
weight + temporal merge) followed by mtla_decode_attn (absorption, attention
over the live slots, split combine, value up-projection).  The default workload is the
paper's decoder shape: batch 16, 8 heads x 64, r=256, RoPE dim 32, s=2, a
1024-token prefix and 256 decode steps, bf16 storage with fp32 accumulation.

Other modes: --workload prefill_s2 / prefill_s4 (the parallel form; --pieces N feeds the sequences in N
pieces through mtla_prefill_step), --layer (mtla_layer_decode_step, or mtla_layer_prefill with a prefill workload), --reorder (mtla_cache_reorder).

Prints ONE JSON line.  `value` is
tokens/s with all inputs resident in HBM, the K steps replayed as one HIP
graph; the eager (one ctypes call per library entry) rate is reported beside
it.  `roofline` refers to the dominant kernel (the pass over the cache slots),
timed with HIP event pairs recorded by the library around each launch.
"""
from __future__ import annotations

import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X HBM3E, published
# HBM bytes per launch of the decode attention kernel, from rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE
# runs of this script, each counter scaled by its reading for a plain 256 MiB device copy
# (profiles/decode_attention_hbm_traffic.md), as a line in the launch's algorithmic bytes (the live cache
# rows): traffic = fixed + slope * algorithmic.  The headline workload was measured at two step counts
# (20 and 256 steps: 7.288 MB for 4.772 MB, 7.908 MB for 5.307 MB), which fixes both numbers -- the fixed
# part is the split partials, the query operand and first tiles requested before the length is known;
# the other workloads were measured once, so their line goes through the origin.
MEASURED_TRAFFIC_LINE = {"speech_bf16": (1.776e6, 1.155),
                         "ragged_bf16": (0.0, (357175.6 + 11556.9) * 1024 / 339.5e6),
                         "long_bf16": (0.0, (78746.6 + 8062.6) * 1024 / 75.5e6),
                         "speech_b1024_bf16": (0.0, (306855.4 + 4164.1) * 1024 / 304.6e6)}
# the same for the prefill attention kernel (profiles/prefill_hbm_traffic.md); every launch of a workload
# is the same work, so the step count does not matter
MEASURED_PREFILL_TRAFFIC_BYTES = {"prefill_s2": 2.0 * 277890.8 * 1024 + 262147.9 * 1024,
                                  "prefill_s4": 2.0 * 261745.8 * 1024 + 262151.1 * 1024}
MFMA_BF16_PEAK_TFLOPS = 2500.0   # MI355X dense bf16 matrix rate, published


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=256)
    ap.add_argument("--warmup", type=int, default=32)
    ap.add_argument("--workload", default="speech_bf16",
                    help="decode: speech_bf16 (headline), long_bf16, ragged_bf16, tiny_f32, speech_b1024_bf16 "
                         "(supplement: headline shape at batch 1024); "
                         "parallel form: prefill_s2, prefill_s4 (a step is one forward over batch x T tokens)")
    ap.add_argument("--reps", type=int, default=5, help="timed repetitions of the K steps (median is reported)")
    ap.add_argument("--chunk", type=int, default=0, help="decode slots per workgroup (0 = library default)")
    ap.add_argument("--schedule", type=int, default=0, help="decode schedule: 0 auto, 1 static, 2 balanced")
    ap.add_argument("--two-calls", action="store_true",
                    help="drive a step as mtla_cache_append + mtla_decode_attn instead of mtla_decode_step")
    ap.add_argument("--layer", action="store_true",
                    help="decode workloads: a step is mtla_layer_decode_step (projections from the token stream x, "
                         "LayerNorm, RoPE, the decode step, W_O) instead of mtla_decode_step")
    ap.add_argument("--reorder", action="store_true",
                    help="decode workloads: time mtla_cache_reorder (beam reordering of the whole sequence state) "
                         "instead of decode steps")
    ap.add_argument("--stride", type=int, default=0,
                    help="run the workload's shape at another temporal stride s (s = 1 is the uncompressed, MLA-shaped "
                         "latent cache); the name in config.workload says so")
    ap.add_argument("--latent", action="store_true",
                    help="prefill workloads: also ask for the latent-space output (a second pass of the attention kernel, the timed one)")
    ap.add_argument("--pieces", type=int, default=1,
                    help="prefill workloads: feed every sequence in this many equal pieces, each continuing from the "
                         "cache the earlier ones left (mtla_prefill_step)")
    ap.add_argument("--first-slot", type=int, default=0,
                    help="--reorder: leave the first SLOTS slots of every sequence alone (a prompt all beams share: "
                         "mtla_cache_reorder_from)")
    ap.add_argument("--beams", type=int, default=1,
                    help="decode workloads: groups of this many consecutive sequences are beams over one prompt (the "
                         "first sequence's); the others read its slots instead of their own copies "
                         "(mtla_set_shared_prefix)")
    ap.add_argument("--paged", type=int, default=0,
                    help="paged slot storage with this many slots per page (decode workloads: mtla_decode_step_paged over "
                         "pages handed out in a scrambled order; with --reorder: mtla_cache_fork_paged)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 256 MiB device copy, the known-size kernel that rocprofv3 "
                         "FETCH_SIZE / WRITE_SIZE readings are scaled by")
    return ap.parse_args()


_BLOCKER = None


def queue_ahead(torch, dev, fills=6):
    """Enqueue a few ms of plain fills on the current stream (no result is used), so the host
    runs ahead and the event-timed launches that follow execute back to back, as they do in the
    graph replay that `value` is measured on."""
    global _BLOCKER
    if _BLOCKER is None:
        _BLOCKER = torch.empty(4 << 30, dtype=torch.uint8, device=dev)
    for i in range(fills):
        _BLOCKER.fill_(i)


def stream_probe_gbs(torch, sess, dev, nbytes=2 << 30, reps=3):
    """HBM read rate of a plain streaming kernel over a 2 GiB buffer (far beyond the last-level
    cache), timed with events on the current stream: the practical ceiling on the device at hand."""
    buf = torch.ones(nbytes, dtype=torch.uint8, device=dev)
    sess.ctx.probe_stream_read(buf, nbytes, sess.workspace, sess.stream)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        sess.ctx.probe_stream_read(buf, nbytes, sess.workspace, sess.stream)
    e1.record()
    torch.cuda.synchronize()
    del buf
    return nbytes * reps / (e0.elapsed_time(e1) * 1e-3) / 1e9


def _oracle_worker(conn):
    """One process of the all-cores oracle leg: builds the prefix caches of its sequences, reports ready,
    waits for the start signal, runs the decode steps and sends back the seconds it took and its last outputs."""
    import numpy as np  # noqa: F401
    from threadpoolctl import threadpool_limits
    from oracle import mtla_oracle as O
    import copy
    cfg, seqs, n_steps, n_rep = conn.recv()
    with threadpool_limits(limits=1):
        caches = []
        for sq in seqs:
            cache = O.LatentCache(cfg["r"], cfg["dr"], cfg["s"])
            for t in range(len(sq["pre_c"])):
                O.append_token(cache, sq["pre_c"][t], sq["pre_kr"][t], cfg["hyp_A"], None, cfg["hyp_G"])
            caches.append(cache)
        conn.send("ready")
        conn.recv()
        scale = O.softmax_scale(cfg["dh"])
        t0 = time.perf_counter()
        last = [None] * len(seqs)
        for _ in range(n_rep):
            run = copy.deepcopy(caches)
            for t in range(n_steps):
                for i, sq in enumerate(seqs):
                    O.append_token(run[i], sq["c"][t], sq["kr"][t], cfg["hyp_A"], None, cfg["hyp_G"])
                    last[i] = O.decode_attn(run[i], sq["q"][t], sq["qr"][t], cfg["w_uk"], cfg["w_uv"], scale)[0]
        conn.send((time.perf_counter() - t0, last))


def oracle_all_cores(cfg, seqs, n_proc, n_steps, expect, n_rep):
    """The same oracle work spread over n_proc processes (sequence i goes to process i mod n_proc); the clock
    runs from the start signal to the last answer.  The answers must equal the one-core leg's."""
    import multiprocessing as mp
    import numpy as np
    ctx = mp.get_context("spawn")   # fresh interpreters: nothing of this process's GPU state is inherited
    procs = []
    for p in range(n_proc):
        parent, child = ctx.Pipe()
        pr = ctx.Process(target=_oracle_worker, args=(child,), daemon=True)
        pr.start()
        parent.send((cfg, seqs[p::n_proc], n_steps, n_rep))
        procs.append((pr, parent))
    for _, conn in procs:
        assert conn.recv() == "ready"
    t0 = time.perf_counter()
    for _, conn in procs:
        conn.send("go")
    outs = [conn.recv() for _, conn in procs]
    wall = time.perf_counter() - t0
    for pr, _ in procs:
        pr.join(timeout=30)
    for p, (_, last) in enumerate(outs):
        for i, o in enumerate(last):
            assert np.array_equal(o, expect[p + i * n_proc]), "all-cores oracle leg disagrees with the one-core leg"
    return {"value": n_rep * len(seqs) * n_steps / wall, "unit": "tokens/s", "cores": n_proc, "kind": "oracle",
            "sample": f"the same {n_rep} x {n_steps} decode steps x {len(seqs)} sequences over {n_proc} processes, one per host core "
                      f"(sequences dealt round-robin, numerical library held to one thread each), {wall:.1f} s wall"}


def main():
    args = parse_args()
    if args.gpus != 1:
        print(f"bench.py: this build runs on one GPU only (got --gpus {args.gpus}); "
              "sequences shard across GPUs with no communication", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import workloads as W
    from paper_2505_13544_amd.session import Session, to_device

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    dev = "cuda:0"
    wl = W.WORKLOADS[args.workload]
    if args.stride > 0 and args.stride != wl.stride:
        wl = wl.scaled(name=f"{wl.name} at stride {args.stride}", stride=args.stride)
    if wl.steps == 0:
        return bench_prefill(args, wl)
    if args.reorder:
        return bench_reorder(args, wl)
    K, Wm = args.steps, args.warmup
    if wl.name == "speech_b1024_bf16" and K == 256:
        K, Wm = wl.steps, 2
    B, nh, dh, r, dr, s = wl.batch, wl.n_heads, wl.d_head, wl.r, wl.d_rope, wl.stride
    esz = 2 if wl.dtype == "bf16" else 4
    plen = W.prefix_lengths(wl)
    max_slots = -(-(int(plen.max()) + K) // s)

    # ---------------- inputs (seeded, synthetic), uploaded before any timing
    t_gen = time.time()
    wts = W.make_weights(wl, max_slots=max_slots)
    toks = [W.make_tokens(wl, wts, b, 0, int(plen[b]) + K) for b in range(B)]
    G = max(1, args.beams)
    owner = np.array([b - b % G for b in range(B)], np.int32)
    n_pre = np.array([0 if owner[b] == b else min(int(plen[owner[b]]), int(plen[b])) // s for b in range(B)], np.int32)
    for b in range(B):  # the beams of a group carry the group's prompt: the same tokens at the same positions
        for f in ("c", "kr"):
            getattr(toks[b], f)[:n_pre[b] * s] = getattr(toks[owner[b]], f)[:n_pre[b] * s]
    n_max = int(plen.max())
    pre_c = np.zeros((B, n_max, r), np.float32)
    pre_kr = np.zeros((B, n_max, dr), np.float32)
    for b in range(B):
        pre_c[b, :plen[b]] = toks[b].c[:plen[b]]
        pre_kr[b, :plen[b]] = toks[b].kr[:plen[b]]
    pick = lambda f: np.stack([np.stack([getattr(toks[b], f)[plen[b] + t] for b in range(B)]) for t in range(K)])
    step_c, step_kr, step_q, step_qr = pick("c"), pick("kr"), pick("q"), pick("q_rope")
    if args.paged:
        from paper_2505_13544_amd.session import PagedSession
        n_pages = int(sum(-(-(-(-(int(plen[b]) + K) // s)) // args.paged) for b in range(B))) + 8
        sess = PagedSession(n_heads=nh, d_head=dh, r=r, d_rope=dr, d_hyper=wl.d_hyper, stride=s, max_batch=B,
                            max_slots=max_slots, page_slots=args.paged, n_pages=n_pages, dtype=wl.dtype,
                            decode_chunk=args.chunk or None, decode_schedule=args.schedule,
                            page_order=np.random.default_rng(wl.seed).permutation(n_pages))
    else:
        sess = Session(n_heads=nh, d_head=dh, r=r, d_rope=dr, d_hyper=wl.d_hyper, stride=s, max_batch=B,
                       max_slots=max_slots, dtype=wl.dtype, decode_chunk=args.chunk or None,
                       decode_schedule=args.schedule)
    sess.set_weights(hyp_A=wts.hyp_A, hyp_G=wts.hyp_G, w_uk=wts.w_uk_lib, w_uv=wts.w_uv_lib)
    d_c = to_device(step_c, wl.dtype, dev).unsqueeze(2)      # [K, B, 1, r]
    d_kr = to_device(step_kr, wl.dtype, dev).unsqueeze(2)
    d_q, d_qr = to_device(step_q, wl.dtype, dev), to_device(step_qr, wl.dtype, dev)
    out = torch.empty(K, B, nh, dh, dtype=torch.float32, device=dev)
    if args.layer:  # the step's own inputs: the token stream and the projection weights
        lw = W.make_layer_weights(wl, wts)
        step_x = np.stack([np.stack([W.make_x(wl, b, int(plen[b]) + t, int(plen[b]) + t + 1)[0] for b in range(B)])
                           for t in range(K)])
        d_x = to_device(step_x, wl.dtype, dev)                   # [K, B, d_model]
        y = torch.empty(K, B, wl.d_model, dtype=torch.float32, device=dev)
        sess.set_layer_weights(w_q=lw.w_q, w_qr=lw.w_qr, w_r=lw.w_r, w_kr=lw.w_kr, w_o=lw.w_o)
    if args.paged:
        assert not (args.layer or args.two_calls or G > 1), "--paged runs mtla_decode_step_paged"
        sess.append(to_device(pre_c, wl.dtype, dev), to_device(pre_kr, wl.dtype, dev), n_new=plen)
        sess.reserve([K] * B)      # every page the K steps will reach: the steps below do not touch the table
    else:
        sess.append(to_device(pre_c, wl.dtype, dev), to_device(pre_kr, wl.dtype, dev),
                    n_new=torch.from_numpy(plen).to(dev))
    if G > 1:  # every cache still holds its own copy of the prompt's slots; the decode calls no longer read it
        sess.share_prefix(torch.from_numpy(owner).to(dev), torch.from_numpy(n_pre).to(dev))
    torch.cuda.synchronize()
    state = (sess.pool_c, sess.pool_kr, sess.tail_c, sess.seq_len) if args.paged else (sess.cache_c, sess.cache_kr, sess.tail_c, sess.seq_len)
    snap = [t.clone() for t in state]
    t_gen = time.time() - t_gen

    def restore():
        for dst, src in zip(state, snap):
            dst.copy_(src)
        torch.cuda.synchronize()

    def run_steps(n):
        for t in range(n):
            if args.layer:
                sess.layer_step(d_x[t], y=y[t], out=out[t])
            elif args.two_calls:
                sess.append(d_c[t], d_kr[t])
                sess.decode(d_q[t], d_qr[t], out=out[t])
            elif args.paged:
                sess.step(d_c[t], d_kr[t], d_q[t], d_qr[t], out=out[t], reserve=False)
            else:
                sess.step(d_c[t], d_kr[t], d_q[t], d_qr[t], out=out[t])

    # ---------------- warm-up (untimed), eager timing
    run_steps(min(Wm, K))
    restore()
    eager_ms = []
    for _ in range(args.reps):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        run_steps(K)
        torch.cuda.synchronize()
        eager_ms.append((time.perf_counter() - t0) * 1e3 / K)
        restore()

    # ---------------- the K steps as one HIP graph
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run_steps(K)
    restore()
    graph.replay()            # untimed replay
    restore()
    graph_ms = []
    for _ in range(args.reps):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        graph.replay()
        torch.cuda.synchronize()
        graph_ms.append((time.perf_counter() - t0) * 1e3 / K)
        out_graph = out.clone()
        restore()
    ms_per_step = statistics.median(graph_ms)
    tokens_per_s = B / (ms_per_step * 1e-3)

    # ---------------- dominant kernel: HIP event pair around every launch (eager pass)
    # (the library attaches the two events to the kernel's own dispatch, so the interval is the
    # kernel's execution time whatever the host does between calls)
    sess.ctx.profile_start(K)
    queue_ahead(torch, dev)
    run_steps(K)
    torch.cuda.synchronize()
    kern_ms = sess.ctx.profile_read()
    out_eager = out.clone()
    y_eager = y.clone() if args.layer else None
    assert sess.device_status() == 0
    restore()
    assert torch.equal(out_eager, out_graph), "graph replay and eager launches disagree"
    probe_gbs = stream_probe_gbs(torch, sess, dev)
    live = np.stack([-(-(plen + t + 1) // s) for t in range(K)])          # [K, B] live slots per step
    cache_bytes = live.sum(axis=1).astype(np.float64) * (r + dr) * esz     # algorithmic bytes per launch
    alg_bytes = float(cache_bytes.mean())
    kern_avg_ms = float(np.mean(kern_ms))
    achieved = alg_bytes / (kern_avg_ms * 1e-3) / 1e9
    line = MEASURED_TRAFFIC_LINE.get(wl.name) if (args.stride == 0 and G == 1 and not args.schedule and not args.chunk and not args.paged) else None
    traffic = line[0] + line[1] * alg_bytes if line else None
    step_bytes = alg_bytes + 2 * nh * dh * r * esz + wl.d_hyper * r * esz  # + absorbed weights + hyper-network
    if args.layer:  # + W_Q, W_QR, W_r, W_KR, W_O
        step_bytes += (2 * nh * dh + nh * dr + r + dr) * wl.d_model * esz

    res = {
        "metric": (f"MTLA whole-layer decode tokens/s ({wl.name}, d_model {wl.d_model}; the projections around the "
                   "headline path included)") if args.layer
                  else "MTLA decode tokens/s + achieved HBM GB/s vs peak (B=16,T=1024,s=2)" if wl.name == "speech_bf16"
                  else f"MTLA decode tokens/s + achieved HBM GB/s vs peak ({wl.name}; not the headline configuration)",
        "value": tokens_per_s, "unit": "tokens/s", "n_gpus": 1, "steps": K, "warmup": Wm,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if wl.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": f"{wl.name}: batch {B}, {nh} heads x {dh}, r={r}, d_rope={dr}, s={s}, "
                               f"prefix {wl.prefix}, {K} decode steps, one attention layer",
                   "launch": "HIP graph replay of K steps",
                   "entry": "mtla_layer_decode_step" if args.layer
                            else "mtla_cache_append + mtla_decode_attn" if args.two_calls
                            else f"mtla_decode_step_paged (pages of {args.paged} slots, handed out in a scrambled order)" if args.paged
                            else "mtla_decode_step",
                   "decode_chunk": sess.ctx.get_decode_chunk(),
                   "reps": args.reps},
        **({"beams": {"group": G, "slots_read_from_the_group_owner": float(n_pre.sum() / live[0].sum()),
                      "distinct_cache_bytes_per_launch": float((live[0].sum() - n_pre.sum()) * (r + dr) * esz)}}
           if G > 1 else {}),
        "eager_ms_per_step": statistics.median(eager_ms),
        "eager_tokens_per_s": B / (statistics.median(eager_ms) * 1e-3),
        "step_effective_GBps": step_bytes / (ms_per_step * 1e-3) / 1e9,
        "roofline": {"bound": "hbm", "kernel": "decode attention over cache slots (split pass)",
                     "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "streaming_probe_GBps": probe_gbs,
                     "frac_of_streaming_probe": achieved / probe_gbs,
                     "traffic": traffic,
                     "traffic_source": ("profiles/decode_attention_hbm_traffic.md: counters of the same command at "
                                        f"other step counts, as {line[0]:.4g} B + {line[1]:.4g} x algorithmic bytes")
                                       if traffic is not None else None,
                     "algorithmic_bytes_per_launch": alg_bytes,
                     "algorithmic_bytes_first_and_last_launch": [float(cache_bytes[0]), float(cache_bytes[-1])], "avg_launch_ms": kern_avg_ms,
                     "launches_timed": len(kern_ms)},
        "input_gen_s": t_gen,
    }

    # ---------------- CPU baseline: the float64 oracle on the host cores, same inputs.  Two legs: one core
    # (the numerical library held to one thread), then every host core (one process per core, each with its
    # share of the sequences and the numerical library held to one thread).
    if not args.no_cpu_baseline:
        from oracle import mtla_oracle as O
        from threadpoolctl import threadpool_limits
        host_cpus = len(os.sched_getaffinity(0))
        # bounded sample: all sequences when cheap, else the first few; prefix build is excluded
        per_pair_flop = nh * float(live.mean()) * (4 * r + 2 * dr)
        n_seq = B if per_pair_flop * B * K < 5e10 else max(1, min(B, int(5e10 / (per_pair_flop * K))))
        n_steps = K if per_pair_flop * n_seq * K < 1e11 else max(1, int(1e11 / (per_pair_flop * n_seq)))
        scale = O.softmax_scale(dh)
        last, last_y = {}, {}
        with threadpool_limits(limits=1):
            caches = []
            for b in range(n_seq):
                cache = O.LatentCache(r, dr, s)
                for t in range(int(plen[b])):
                    O.append_token(cache, toks[b].c[t], toks[b].kr[t], wts.hyp_A, None, wts.hyp_G)
                caches.append(cache)
            import copy
            wall = cpu = 0.0
            n_rep = 0
            while n_rep == 0 or (wall < 8.0 and n_rep < 400):   # about ten seconds of work: the same steps again
                run = copy.deepcopy(caches)                      # from the state the prefix left
                w0, c0 = time.perf_counter(), time.process_time()
                for t in range(n_steps):
                    for b in range(n_seq):
                        if args.layer:
                            last_y[b], last[b] = O.layer_decode_step(run[b], step_x[t, b], lw.w_q, lw.w_qr, lw.w_r, lw.w_kr,
                                                                     lw.w_o, wts.hyp_A, None, wts.hyp_G, wts.w_uk, wts.w_uv,
                                                                     scale)[:2]
                            continue
                        O.append_token(run[b], step_c[t, b], step_kr[t, b], wts.hyp_A, None, wts.hyp_G)
                        last[b] = O.decode_attn(run[b], step_q[t, b], step_qr[t, b], wts.w_uk, wts.w_uv, scale)[0]
                wall, cpu = wall + time.perf_counter() - w0, cpu + time.process_time() - c0
                n_rep += 1
        err = max(float(np.abs(out_eager[n_steps - 1, b].float().cpu().numpy() - last[b]).max()) for b in range(n_seq))
        res["cpu_baseline"] = {"value": n_rep * n_seq * n_steps / wall, "unit": "tokens/s", "cores": 1, "kind": "oracle",
                               "sample": f"{n_rep} x {n_steps} decode steps x {n_seq} sequences of the same workload "
                                         f"(numpy float64, its numerical library held to one thread; prefix build "
                                         f"excluded), {wall:.1f} s wall, {cpu:.1f} s of processor time",
                               "host_cpus": host_cpus}
        res["parity_max_abs_err_vs_oracle"] = err
        if args.layer:
            res["parity_max_abs_err_y_vs_oracle"] = max(
                float(np.abs(y_eager[n_steps - 1, b].cpu().numpy() - last_y[b]).max()) for b in range(n_seq))
        else:
            res["cpu_baseline_all_cores"] = oracle_all_cores(
                dict(r=r, dr=dr, s=s, dh=dh, hyp_A=wts.hyp_A, hyp_G=wts.hyp_G, w_uk=wts.w_uk, w_uv=wts.w_uv),
                [dict(pre_c=toks[b].c[:plen[b]], pre_kr=toks[b].kr[:plen[b]], c=step_c[:n_steps, b], kr=step_kr[:n_steps, b],
                      q=step_q[:n_steps, b], qr=step_qr[:n_steps, b]) for b in range(n_seq)],
                min(host_cpus, n_seq), n_steps, {b: last[b] for b in range(n_seq)}, n_rep)
    if args.calibrate_copy:
        src = torch.ones(256 << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)      # reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
    print(json.dumps(res))


def bench_reorder(args, wl):
    """Beam reordering: a step is one mtla_cache_reorder of the whole batch (a random assignment of
    source sequences, some continued twice, some dropped) from one set of state buffers into another.
    Bytes = live cache rows + tail shadows, read once and written once."""
    import numpy as np
    import torch

    import workloads as W
    from paper_2505_13544_amd.session import Session, to_device

    dev = "cuda:0"
    K = args.steps if args.steps != 256 else 20
    B, r, dr, s = wl.batch, wl.r, wl.d_rope, wl.stride
    esz = 2 if wl.dtype == "bf16" else 4
    plen = W.prefix_lengths(wl)
    max_slots = -(-int(plen.max()) // s)
    t_gen = time.time()
    rng = np.random.default_rng([wl.seed, 0xBEA3])
    if args.paged:
        return bench_fork_paged(args, wl, rng, K)
    sess = Session(n_heads=wl.n_heads, d_head=wl.d_head, r=r, d_rope=dr, d_hyper=wl.d_hyper, stride=s, max_batch=B,
                   max_slots=max_slots, dtype=wl.dtype)
    # the reorder moves bytes whatever they are: seeded random rows stand in for a built cache
    sess.cache_c.copy_(to_device(rng.standard_normal((B, max_slots, r), dtype=np.float32), wl.dtype, dev))
    sess.cache_kr.copy_(to_device(rng.standard_normal((B, max_slots, dr), dtype=np.float32), wl.dtype, dev))
    sess.tail_c.copy_(torch.from_numpy(rng.standard_normal((B, r), dtype=np.float32)).to(dev))
    sess.seq_len.copy_(torch.from_numpy(plen).to(dev))
    idx_np = rng.integers(0, B, size=B).astype(np.int32)
    idx = torch.from_numpy(idx_np).to(dev)
    dst = [torch.empty_like(t) for t in (sess.cache_c, sess.cache_kr, sess.tail_c, sess.seq_len)]
    t_gen = time.time() - t_gen
    F = max(0, args.first_slot)
    if F:  # the shared prefix is in both sets of buffers already
        dst[0][:, :F].copy_(sess.cache_c[:, :F])
        dst[1][:, :F].copy_(sess.cache_kr[:, :F])
    call = lambda: sess.ctx.cache_reorder_from(sess.cache_c, sess.cache_kr, sess.tail_c, sess.seq_len, idx, B, F, dst[0],
                                               dst[1], dst[2], dst[3], sess.workspace, sess.stream)
    for _ in range(max(1, args.warmup if args.warmup != 32 else 3)):
        call()
    torch.cuda.synchronize()
    ms = []
    for _ in range(args.reps):
        queue_ahead(torch, dev, fills=2)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(K):
            call()
        e1.record()
        torch.cuda.synchronize()
        ms.append(e0.elapsed_time(e1) / K)
    ms_per_step = statistics.median(ms)
    assert sess.device_status() == 0
    live = -(-plen[idx_np] // s)
    moved = np.maximum(live - F, 0)
    nbytes = float(2 * (moved.sum() * (r + dr) * esz + B * r * 4))      # read + written
    # bit-exact against the definition (a gather of whole sequences), all sequences
    for b in range(B):
        n = int(live[b])
        assert torch.equal(dst[0][b, F:n], sess.cache_c[idx_np[b], F:n]) and torch.equal(dst[1][b, F:n], sess.cache_kr[idx_np[b], F:n])
    assert torch.equal(dst[2], sess.tail_c[idx.long()]) and torch.equal(dst[3], sess.seq_len[idx.long()])
    achieved = nbytes / (ms_per_step * 1e-3) / 1e9
    res = {
        "metric": f"MTLA beam reorder of the sequence state, GB/s read + written ({wl.name}; not the headline metric)",
        "value": achieved, "unit": "GB/s", "n_gpus": 1, "steps": K, "warmup": 3, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "u8", "data": "synthetic",
        "config": {"workload": f"{wl.name}: batch {B}, r={r}, d_rope={dr}, s={s}, prefix {wl.prefix}: one "
                               "mtla_cache_reorder of all sequences per step"
                               + (f", the first {F} slots of every sequence left alone (shared prompt)" if F else ""),
                   "launch": "eager", "reps": args.reps},
        "roofline": {"bound": "hbm", "kernel": "reorder_kernel (gather of whole sequences)", "achieved": achieved,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": None,
                     "algorithmic_bytes_per_launch": nbytes, "avg_launch_ms": ms_per_step, "launches_timed": K * args.reps},
        "input_gen_s": t_gen,
    }
    if not args.no_cpu_baseline:  # the definition itself on the host: numpy fancy indexing of the same state
        c_h, k_h = sess.cache_c.view(torch.int16).cpu().numpy() if esz == 2 else sess.cache_c.cpu().numpy(), \
            sess.cache_kr.view(torch.int16).cpu().numpy() if esz == 2 else sess.cache_kr.cpu().numpy()
        t_h = sess.tail_c.cpu().numpy()
        w0 = time.perf_counter()
        n_rep = 0
        while time.perf_counter() - w0 < 5.0:
            out_c, out_k = np.empty_like(c_h), np.empty_like(k_h)
            for b in range(B):
                n = int(live[b])
                out_c[b, F:n] = c_h[idx_np[b], F:n]
                out_k[b, F:n] = k_h[idx_np[b], F:n]
            out_t = t_h[idx_np]
            n_rep += 1
        wall = time.perf_counter() - w0
        res["cpu_baseline"] = {"value": nbytes * n_rep / wall / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
                               "sample": f"the gather written with numpy row copies, {n_rep} repetitions in {wall:.1f} s"}
    print(json.dumps(res))


def bench_fork_paged(args, wl, rng, K):
    """The same beam reordering over paged storage: a step is one mtla_cache_fork_paged of the whole batch (the same
    seeded draw of sources): table rows, one open page per beam and the tail shadows move, the caches do not."""
    import numpy as np
    import torch

    from paper_2505_13544_amd.session import PagedSession
    dev = "cuda:0"
    B, r, dr, s, P = wl.batch, wl.r, wl.d_rope, wl.stride, args.paged
    plen = W_prefix = None
    import workloads as W
    plen = W.prefix_lengths(wl)
    max_slots = -(-int(plen.max()) // s) + 1
    n_seq_pages = [-(-(-(-int(n) // s)) // P) for n in plen]
    n_pages = int(sum(n_seq_pages)) + 2 * B + 8
    t_gen = time.time()
    sess = PagedSession(n_heads=wl.n_heads, d_head=wl.d_head, r=r, d_rope=dr, d_hyper=wl.d_hyper, stride=s, max_batch=B,
                        max_slots=max_slots, page_slots=P, n_pages=n_pages, dtype=wl.dtype,
                        page_order=rng.permutation(n_pages))
    # the fork moves bytes whatever they are: seeded random rows stand in for a built cache
    sess.pool_c.copy_(torch.randn(sess.pool_c.shape, device=dev, generator=torch.Generator(device=dev).manual_seed(1)).to(sess.pool_c.dtype))
    sess.pool_kr.copy_(torch.randn(sess.pool_kr.shape, device=dev, generator=torch.Generator(device=dev).manual_seed(2)).to(sess.pool_kr.dtype))
    sess.reserve([int(n) for n in plen])
    sess.h_len[:] = plen
    sess.seq_len.copy_(torch.from_numpy(plen).to(dev))
    sess.tail_c.copy_(torch.from_numpy(rng.standard_normal((B, r), dtype=np.float32)).to(dev))
    idx_np = rng.integers(0, B, size=B).astype(np.int32)
    fresh_np = np.array([sess._alloc() for _ in range(B)], np.int32)
    idx, fresh = torch.from_numpy(idx_np).to(dev), torch.from_numpy(fresh_np).to(dev)
    dst = [torch.zeros_like(sess.table), torch.empty_like(sess.tail_c), torch.zeros_like(sess.seq_len)]
    t_gen = time.time() - t_gen
    call = lambda: sess.ctx.cache_fork_paged(sess.pool_c, sess.pool_kr, sess.table, sess.tail_c, sess.seq_len, idx, fresh, B,
                                             dst[0], dst[1], dst[2], sess.workspace, sess.stream)
    for _ in range(3):
        call()
    torch.cuda.synchronize()
    ms = []
    for _ in range(args.reps):
        queue_ahead(torch, dev, fills=2)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(K):
            call()
        e1.record()
        torch.cuda.synchronize()
        ms.append(e0.elapsed_time(e1) / K)
    ms_per_step = statistics.median(ms)
    assert sess.device_status() == 0
    # against the definition: destination b holds the source's rows, complete pages by reference
    live = -(-plen[idx_np] // s)
    pw = np.minimum(plen[idx_np] // s, max_slots - 1) // P
    tab = dst[0].cpu().numpy()
    open_rows = 0
    for b in range(B):
        src = int(idx_np[b])
        assert np.array_equal(tab[b, :pw[b]], sess.h_table[src, :pw[b]]) and tab[b, pw[b]] == fresh_np[b]
        n = int(live[b]) - int(pw[b]) * P
        if n > 0:
            open_rows += n
            sp = int(sess.h_table[src, pw[b]])
            assert torch.equal(sess.pool_c[fresh_np[b], :n], sess.pool_c[sp, :n]) and torch.equal(sess.pool_kr[fresh_np[b], :n], sess.pool_kr[sp, :n])
    assert torch.equal(dst[1], sess.tail_c[idx.long()]) and torch.equal(dst[2], sess.seq_len[idx.long()])
    nbytes = float(2 * (open_rows * (r + dr) * 2 + B * r * 4) + 2 * int(pw.sum()) * 4)   # read + written
    achieved = nbytes / (ms_per_step * 1e-3) / 1e9
    res = {
        "metric": f"MTLA beam reorder over paged storage, ms per reordering of all beams ({wl.name}; not the headline metric)",
        "value": ms_per_step, "unit": "ms", "n_gpus": 1, "steps": K, "warmup": 3, "ms_per_step": ms_per_step,
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "u8", "data": "synthetic",
        "config": {"workload": f"{wl.name}: batch {B}, r={r}, d_rope={dr}, s={s}, prefix {wl.prefix}, pages of {P} slots: one "
                               "mtla_cache_fork_paged of all sequences per step", "launch": "eager", "reps": args.reps},
        "roofline": {"bound": "hbm", "kernel": "fork_paged_kernel (table rows, open pages, tail shadows)", "achieved": achieved,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": None,
                     "algorithmic_bytes_per_launch": nbytes, "avg_launch_ms": ms_per_step, "launches_timed": K * args.reps},
        "bytes_the_contiguous_reorder_moves": float(2 * (live.sum() * (r + dr) * 2 + B * r * 4)),
        "input_gen_s": t_gen,
    }
    print(json.dumps(res))


def bench_prefill(args, wl):
    """Parallel (prefill / training forward) form: a step is mtla_cache_append over all T tokens of
    every sequence (hyper-network weights + the decode-ready cache) followed by mtla_prefill_attn
    (running chunk states, absorption, attention under the stride-aware mask, up-projection)."""
    import numpy as np
    import torch

    import workloads as W
    from paper_2505_13544_amd.session import Session, to_device

    dev = "cuda:0"
    K = args.steps if args.steps != 256 else 10
    Wm = args.warmup if args.warmup != 32 else 2
    B, T, nh, dh, r, dr, s = wl.batch, wl.prefix, wl.n_heads, wl.d_head, wl.r, wl.d_rope, wl.stride
    t_gen = time.time()
    wts = W.make_weights(wl)
    toks = [W.make_tokens(wl, wts, b, 0, T) for b in range(B)]
    st = lambda f: to_device(np.stack([getattr(t, f) for t in toks]), wl.dtype, dev)
    d_q, d_qr, d_c, d_kr = st("q"), st("q_rope"), st("c"), st("kr")
    sess = Session(n_heads=nh, d_head=dh, r=r, d_rope=dr, d_hyper=wl.d_hyper, stride=s, max_batch=B,
                   max_slots=-(-T // s), dtype=wl.dtype)
    sess.set_weights(hyp_A=wts.hyp_A, hyp_G=wts.hyp_G, w_uk=wts.w_uk_lib, w_uv=wts.w_uv_lib)
    w = torch.zeros(B, T, dtype=torch.float32, device=dev)
    out = torch.empty(B, T, nh, dh, dtype=torch.float32, device=dev)
    ws = torch.empty(sess.ctx.prefill_workspace_bytes(B, T), dtype=torch.uint8, device=dev)
    out_lat = torch.empty(B, T, nh, r, dtype=torch.float32, device=dev) if args.latent else None
    t_gen = time.time() - t_gen

    P = max(1, args.pieces)
    if P > 1:  # every piece is a call of its own on contiguous inputs, continuing from the cache
        assert T % P == 0, "--pieces must divide T"
        Tn = T // P
        cut = lambda t: [t[:, i * Tn:(i + 1) * Tn].contiguous() for i in range(P)]
        p_q, p_qr, p_c, p_kr = cut(d_q), cut(d_qr), cut(d_c), cut(d_kr)
        p_w = [torch.zeros(B, Tn, dtype=torch.float32, device=dev) for _ in range(P)]
        p_out = [torch.empty(B, Tn, nh, dh, dtype=torch.float32, device=dev) for _ in range(P)]
        past = [i * Tn // s for i in range(P)]
        ws_c = torch.empty(sess.ctx.prefill_step_scratch_bytes(B, Tn, past[-1]), dtype=torch.uint8, device=dev)

    if args.layer:  # the whole layer: the step's inputs are the token stream and the projection weights
        lw = W.make_layer_weights(wl, wts)
        sess.set_layer_weights(w_q=lw.w_q, w_qr=lw.w_qr, w_r=lw.w_r, w_kr=lw.w_kr, w_o=lw.w_o)
        xs = [W.make_x(wl, b, 0, T) for b in range(B)]
        d_x = to_device(np.stack(xs), wl.dtype, dev)
        Tn = T // P
        p_x = [d_x[:, i * Tn:(i + 1) * Tn].contiguous() for i in range(P)]
        p_y = [torch.empty(B, Tn, wl.d_model, dtype=torch.float32, device=dev) for _ in range(P)]
        past = [i * Tn // s for i in range(P)]
        scratch = torch.empty(sess.ctx.layer_prefill_scratch_bytes(wl.d_model, B, Tn, past[-1]), dtype=torch.uint8,
                              device=dev)

    def step():
        sess.seq_len.zero_()          # the sequences start empty again
        if args.layer:
            for i in range(P):
                sess.ctx.layer_prefill(sess.layer_w, sess.cache_c, sess.cache_kr, sess.tail_c, sess.seq_len, p_x[i], None,
                                       sess.hyp_A, sess.hyp_a, sess.hyp_G, sess.w_uk, sess.w_uv, B, Tn, past[i], p_y[i],
                                       scratch, sess.workspace, sess.stream)
            return
        if P == 1:
            sess.append(d_c, d_kr, w_out=w)
            sess.ctx.prefill_attn(d_q, d_qr, d_c, d_kr, w, None, B, T, sess.w_uk, sess.w_uv, out, out_lat, ws,
                                  sess.stream)
            return
        for i in range(P):   # mtla_prefill_step: append + attention of the piece, continuing from the cache
            sess.ctx.prefill_step(sess.cache_c, sess.cache_kr, sess.tail_c, sess.seq_len, p_q[i], p_qr[i], p_c[i], p_kr[i],
                                  None, sess.hyp_A, sess.hyp_a, sess.hyp_G, sess.w_uk, sess.w_uv, B, Tn, past[i],
                                  p_out[i], p_w[i], ws_c, sess.workspace, sess.stream)

    for _ in range(Wm):
        step()
    times = []
    for _ in range(args.reps):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(K):
            step()
        torch.cuda.synchronize()
        times.append((time.perf_counter() - t0) * 1e3 / K)
    ms_per_step = statistics.median(times)
    sess.ctx.profile_start(K * P)
    queue_ahead(torch, dev)
    for _ in range(K):
        step()
    torch.cuda.synchronize()
    kern_ms = sess.ctx.profile_read()
    if P > 1:  # one launch per piece: the step's attention time is their sum
        kern_ms = [sum(kern_ms[k * P:(k + 1) * P]) for k in range(K)]
        if not args.layer:
            out = torch.cat(p_out, dim=1)
    assert sess.device_status() == 0
    cols = np.arange(T) // s + 1                                  # unmasked columns of each row
    # The library takes the explicit key / value form (bf16 storage, d_head 64 or 128): QK^T over
    # [k | kR] (d_h + d_R), then PV over d_h, per open (row, column) pair and head; the absorbed form would
    # be 2 (r + d_R) + 2 r per pair.  The latent-space output (--latent) is a second, timed pass of the
    # same kernel over the partial states as values: softmax . C_hat' needs the logits once and r columns
    # of values per pair; the pass forms the logits again for each of its r / d_h column slices
    # (executed_flop_per_open_pair).
    explicit = wl.dtype == "bf16" and dh in (64, 128) and (not args.latent or r % dh == 0)
    latent_pass = explicit and args.latent
    per_pair = (2 * (dh + dr) + 2 * r) if latent_pass else (2 * (dh + dr) + 2 * dh) if explicit else (2 * (r + dr) + 2 * r)
    executed_per_pair = (r // dh) * (2 * (dh + dr) + 2 * dh) if latent_pass else per_pair
    flops = float(B) * nh * float(cols.sum()) * per_pair
    kern_avg_ms = float(np.mean(kern_ms))
    achieved = flops / (kern_avg_ms * 1e-3) / 1e12
    d = wl.d_model
    # the layer's matrix products around the path: x W_Q, x W_QR, x W_KR, x W_r, o W_O, and K, V = C_hat' W_K, C_hat' W_V
    layer_flops = 2.0 * B * T * (d * (nh * dh + nh * dr + dr + r) + nh * dh * d) if args.layer else 0.0
    res = {
        "metric": "MTLA prefill tokens/s + achieved MFMA TFLOP/s vs peak (parallel form, stride-aware mask)",
        "value": B * T / (ms_per_step * 1e-3), "unit": "tokens/s", "n_gpus": 1, "steps": K, "warmup": Wm,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if wl.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": f"{wl.name}: batch {B}, T={T}, {nh} heads x {dh}, r={r}, d_rope={dr}, s={s}, "
                               "one attention layer, forward"
                               + (f", through mtla_layer_prefill (d_model {d}: projections, LayerNorm, RoPE and W_O included)"
                                  if args.layer else "")
                               + (f", every sequence fed in {P} pieces of {T // P} tokens (each continues from the cache)"
                                  if P > 1 else ""), "launch": "eager", "reps": args.reps},
        "roofline": {"bound": "mfma", "kernel": "prefill attention over the unmasked columns ("
                               + ("latent-space output: explicit keys, the partial states as values, fp16 MFMA" if latent_pass
                                  else "explicit keys/values, fp16 MFMA" if explicit else "absorbed form, bf16 MFMA") + ")",
                     "flop_per_open_pair": per_pair, "executed_flop_per_open_pair": executed_per_pair,
                     "achieved": achieved, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / MFMA_BF16_PEAK_TFLOPS,
                     "traffic": MEASURED_PREFILL_TRAFFIC_BYTES.get(wl.name) if explicit and P == 1 and not args.layer and not args.latent else None,
                     "launches_per_step": P, "algorithmic_flops_per_launch": flops / P, "avg_launch_ms": kern_avg_ms / P,
                     "launches_timed": len(kern_ms)},
        "input_gen_s": t_gen,
    }
    if args.layer:
        res["layer_matrix_product_flops_per_step"] = layer_flops
        res["step_TFLOPs_all_products"] = (layer_flops + flops + 2.0 * 2 * B * T * r * nh * dh) / (ms_per_step * 1e-3) / 1e12
    if not args.no_cpu_baseline:
        from oracle import mtla_oracle as O

        def oracle_rows(rows):
            if args.layer:
                return O.layer_prefill(xs[0], lw.w_q, lw.w_qr, lw.w_r, lw.w_kr, lw.w_o, wts.hyp_A, None, wts.hyp_G, wts.w_uk,
                                       wts.w_uv, s, O.softmax_scale(dh), rows=rows)[0]
            return O.prefill_attn(toks[0].q, toks[0].q_rope, toks[0].c, toks[0].kr, wts.w_uk, wts.w_uv, s,
                                  O.softmax_scale(dh), hyp_A=wts.hyp_A, hyp_a=None, hyp_G=wts.hyp_G, rows=rows)[0]

        def timed(n_rows):
            rows = sorted(set(np.linspace(0, T - 1, n_rows).astype(int).tolist()))
            from threadpoolctl import threadpool_limits
            with threadpool_limits(limits=1):   # one core: the numerical library held to one thread
                w0, c0 = time.perf_counter(), time.process_time()
                ref = oracle_rows(rows)
                return rows, ref, time.perf_counter() - w0, time.process_time() - c0

        rows, ref, wall, cpu = timed(64)
        if wall < 5.0:  # a sample of about ten seconds, sized from the first
            rows, ref, wall, cpu = timed(min(T, max(64, int(64 * 10.0 / max(wall, 0.02)))))
        res["cpu_baseline"] = {"value": len(rows) / wall, "unit": "tokens/s", "cores": 1, "kind": "oracle",
                               "sample": f"{len(rows)} evenly spaced rows of sequence 0 ("
                                         + ("projections, " if args.layer else "")
                                         + "hyper-network weights and running states of the whole sequence included), "
                                         f"numerical library held to one thread, {wall:.1f} s wall, {cpu:.1f} s of processor time",
                               "host_cpus": len(os.sched_getaffinity(0))}
        got = torch.cat(p_y, dim=1)[0, rows] if args.layer else out[0, rows]
        res["parity_max_abs_err_vs_oracle"] = float(np.abs(got.cpu().numpy() - ref).max())
    print(json.dumps(res))


if __name__ == "__main__":
    main()
