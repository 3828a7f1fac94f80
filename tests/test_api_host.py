"""Host-side behaviour of the C-ABI library, no GPU needed: the library loads,
exports every symbol the header declares, sizes follow the documented layouts
and invalid calls are rejected before anything is enqueued."""
import ctypes
import os
import re

import pytest

from paper_2505_13544_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
GOOD = dict(n_heads=8, d_head=64, r=256, d_rope=32, d_hyper=64, stride=2, max_batch=16, max_slots=640, dtype="bf16")


def declared_functions():
    text = open(os.path.join(ROOT, "include", "mtla.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(mtla_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert {"mtla_cache_append", "mtla_decode_attn", "mtla_prefill_attn", "mtla_create"} <= set(names)
    raw = ctypes.CDLL(B.LIB_PATH)
    for n in names:
        assert hasattr(raw, n), f"libmtla.so does not export {n}"
    assert set(names) == set(B.SIGNATURES), "binding and header disagree on the entry points"


def test_sizes_follow_the_cache_accounting():
    ctx = B.Context(**GOOD)
    assert ctx.cache_c_bytes() == 16 * 640 * 256 * 2
    assert ctx.cache_kr_bytes() == 16 * 640 * 32 * 2
    assert ctx.tail_bytes() == 16 * 256 * 4
    # (r + d_R) / s elements per token (9 d_h / (2 s) with the paper's ratios)
    per_token = (ctx.cache_c_bytes() + ctx.cache_kr_bytes()) / 2 / (16 * 640 * 2)
    assert per_token == (256 + 32) / 2 == 9 * 64 / (2 * 2)
    f32 = B.Context(**{**GOOD, "dtype": "f32"})
    assert f32.cache_c_bytes() == 2 * ctx.cache_c_bytes()
    assert ctx.workspace_bytes() > 256 and ctx.workspace_bytes() % 256 == 0
    assert ctx.prefill_workspace_bytes(2, 128) > 0 and ctx.prefill_workspace_bytes(0, 128) == 0


def test_decode_chunk_knob():
    ctx = B.Context(**GOOD)
    d = ctx.get_decode_chunk()
    assert d >= 32 and d % 32 == 0
    small = ctx.workspace_bytes()
    ctx.set_decode_chunk(d * 2)
    assert ctx.get_decode_chunk() == d * 2 and ctx.workspace_bytes() <= small
    ctx.set_decode_chunk(0)
    assert ctx.get_decode_chunk() == d
    for bad in (-32, 16, 48):
        with pytest.raises(B.MtlaError) as e:
            ctx.set_decode_chunk(bad)
        assert e.value.status == B.MTLA_ERR_INVALID_ARG


def test_shared_prefix_setter_checks_its_arguments():
    # the setter only records two device addresses and their length: no GPU is touched
    ctx = B.Context(**GOOD)
    ctx.set_shared_prefix(None, None)
    ctx.set_shared_prefix(0x1000, 0x2000, GOOD["max_batch"])
    ctx.set_shared_prefix(None, None)
    for owner, slots, n in ((0x1000, None, 4), (None, 0x2000, 4), (0x1000, 0x2000, 0), (0x1000, 0x2000, GOOD["max_batch"] + 1)):
        with pytest.raises(B.MtlaError) as e:
            ctx.set_shared_prefix(owner, slots, n)
        assert e.value.status == B.MTLA_ERR_INVALID_ARG
    f32 = B.Context(**{**GOOD, "dtype": "f32"})
    f32.set_shared_prefix(None, None)
    with pytest.raises(B.MtlaError) as e:
        f32.set_shared_prefix(0x1000, 0x2000, 4)
    assert e.value.status == B.MTLA_ERR_UNSUPPORTED
    # arrays of 4 entries: a decode call for 5 sequences is refused before anything is enqueued
    ctx.set_shared_prefix(0x1000, 0x2000, 4)
    P = 0x1000
    assert ctx.decode_attn_status(P, P, P, P, P, P, P, 5, P, None, None, P) == B.MTLA_ERR_INVALID_ARG
    assert ctx.prefill_chunk_attn_status(P, P, P, P, P, P, P, P, P, None, 5, 8, 0, P, P, P, P, P) == B.MTLA_ERR_INVALID_ARG


@pytest.mark.parametrize("field,value,status", [
    ("n_heads", 0, B.MTLA_ERR_SHAPE), ("n_heads", 65, B.MTLA_ERR_SHAPE),
    ("d_head", 48, B.MTLA_ERR_SHAPE), ("d_head", 512, B.MTLA_ERR_SHAPE),
    ("r", 96, B.MTLA_ERR_SHAPE), ("r", 1024, B.MTLA_ERR_SHAPE),
    ("d_rope", 16, B.MTLA_ERR_SHAPE), ("d_hyper", 0, B.MTLA_ERR_SHAPE),
    ("stride", 0, B.MTLA_ERR_SHAPE), ("max_batch", 0, B.MTLA_ERR_SHAPE),
    ("max_slots", 0, B.MTLA_ERR_SHAPE), ("dtype", 7, B.MTLA_ERR_UNSUPPORTED),
    ("softmax_scale", -1.0, B.MTLA_ERR_INVALID_ARG),
])
def test_create_rejects_bad_configs(field, value, status):
    with pytest.raises(B.MtlaError) as e:
        B.Context(**{**GOOD, field: value})
    assert e.value.status == status


def test_create_null_arguments():
    assert B.lib.mtla_create(None, None) == B.MTLA_ERR_INVALID_ARG
    assert B.status_str(B.MTLA_ERR_CAPACITY) == "sequence exceeds max_slots"
    assert B.status_str(0) == "ok" and B.status_str(99) == "unknown status"
    B.lib.mtla_destroy(None)                                 # destroying NULL is a no-op


def test_compute_calls_validate_before_enqueueing():
    ctx = B.Context(**GOOD)
    P = 0x1000                                               # a non-NULL, 16-byte aligned stand-in address
    ok_append = [P, P, P, P, P, P, None, 1, 16, P, None, P, None, None, None, P]
    assert ctx.cache_append_status(*[None] * 6, None, 1, 16, *[None] * 7) == B.MTLA_ERR_INVALID_ARG
    for i in (0, 1, 3, 4, 5, 15):                            # each required pointer in turn
        a = list(ok_append)
        a[i] = None
        assert ctx.cache_append_status(*a) == B.MTLA_ERR_INVALID_ARG
    a = list(ok_append); a[2] = None                         # bf16 storage needs the fp32 tail
    assert ctx.cache_append_status(*a) == B.MTLA_ERR_INVALID_ARG
    a = list(ok_append); a[8] = 17                           # batch > max_batch
    assert ctx.cache_append_status(*a) == B.MTLA_ERR_INVALID_ARG
    a = list(ok_append); a[7] = 0                            # n_new_max < 1
    assert ctx.cache_append_status(*a) == B.MTLA_ERR_INVALID_ARG
    a = list(ok_append); a[9] = None                         # no hyper-network and no override
    assert ctx.cache_append_status(*a) == B.MTLA_ERR_INVALID_ARG
    a = list(ok_append); a[0] = P + 2                        # misaligned cache
    assert ctx.cache_append_status(*a) == B.MTLA_ERR_INVALID_ARG
    a = list(ok_append); a[7] = 640 * 2 + 1                  # longer than the whole capacity
    assert ctx.cache_append_status(*a) == B.MTLA_ERR_CAPACITY

    ok_dec = [P, P, P, P, P, P, P, 16, P, None, None, P]
    for i in (0, 1, 2, 4, 5, 6, 11):
        a = list(ok_dec)
        a[i] = None
        assert ctx.decode_attn_status(*a) == B.MTLA_ERR_INVALID_ARG
    a = list(ok_dec); a[3] = None                            # out without W_V
    assert ctx.decode_attn_status(*a) == B.MTLA_ERR_INVALID_ARG
    a = list(ok_dec); a[8] = None                            # W_V without out
    assert ctx.decode_attn_status(*a) == B.MTLA_ERR_INVALID_ARG
    a = list(ok_dec); a[3] = None; a[8] = None               # nothing requested
    assert ctx.decode_attn_status(*a) == B.MTLA_ERR_INVALID_ARG
    a = list(ok_dec); a[7] = 0
    assert ctx.decode_attn_status(*a) == B.MTLA_ERR_INVALID_ARG

    ok_pre = [P, P, P, P, P, None, 2, 64, P, P, P, None, P]
    for i in (0, 1, 2, 3, 4, 8, 9, 10, 12):
        a = list(ok_pre)
        a[i] = None
        assert ctx.prefill_attn_status(*a) == B.MTLA_ERR_INVALID_ARG
    a = list(ok_pre); a[7] = 0
    assert ctx.prefill_attn_status(*a) == B.MTLA_ERR_INVALID_ARG
    a = list(ok_pre); a[6] = 17
    assert ctx.prefill_attn_status(*a) == B.MTLA_ERR_INVALID_ARG
    assert B.lib.mtla_workspace_init(None, None, None) == B.MTLA_ERR_INVALID_ARG


def test_cache_reorder_validates_before_enqueueing():
    ctx = B.Context(**GOOD)
    P, Q = 0x1000, 0x2000
    ok = [P, P, P, P, P, 16, Q, Q, Q, Q, P]
    for i in (0, 1, 3, 4, 6, 7, 9, 10):
        a = list(ok)
        a[i] = None
        assert ctx.cache_reorder_status(*a) == B.MTLA_ERR_INVALID_ARG
    a = list(ok); a[2] = None                                # bf16 storage carries the fp32 tail
    assert ctx.cache_reorder_status(*a) == B.MTLA_ERR_INVALID_ARG
    a = list(ok); a[5] = 17
    assert ctx.cache_reorder_status(*a) == B.MTLA_ERR_INVALID_ARG
    a = list(ok); a[6] = P                                   # in place
    assert ctx.cache_reorder_status(*a) == B.MTLA_ERR_INVALID_ARG
    a = list(ok); a[7] = Q + 8                               # misaligned
    assert ctx.cache_reorder_status(*a) == B.MTLA_ERR_INVALID_ARG
    # the prefix-skipping form: same checks, and a first slot below zero is refused
    ok_from = ok[:6] + [3] + ok[6:]
    a = list(ok_from); a[6] = -1
    assert ctx.cache_reorder_from_status(*a) == B.MTLA_ERR_INVALID_ARG
    a = list(ok_from); a[0] = None
    assert ctx.cache_reorder_from_status(*a) == B.MTLA_ERR_INVALID_ARG


def test_prefill_chunk_validates_before_enqueueing():
    ctx = B.Context(**GOOD)
    P = 0x1000
    # cache_c, cache_kr, tail_prev, pos0, q, q_rope, c, kr, w, n_new, batch, T, max_past_slots, w_uk, w_uv, out, chunk_ws, ws
    ok = [P, P, P, P, P, P, P, P, P, None, 4, 100, 50, P, P, P, P, P]
    for i in (0, 1, 2, 3, 4, 5, 6, 7, 8, 13, 14, 15, 16, 17):
        a = list(ok)
        a[i] = None
        assert ctx.prefill_chunk_attn_status(*a) == B.MTLA_ERR_INVALID_ARG, i
    for i, v in ((10, 0), (10, GOOD["max_batch"] + 1), (11, 0), (12, -1), (12, GOOD["max_slots"] + 1)):
        a = list(ok)
        a[i] = v
        assert ctx.prefill_chunk_attn_status(*a) == B.MTLA_ERR_INVALID_ARG, (i, v)
    a = list(ok); a[4] = P + 8                               # misaligned queries
    assert ctx.prefill_chunk_attn_status(*a) == B.MTLA_ERR_INVALID_ARG
    f32 = B.Context(**{**GOOD, "dtype": "f32"})              # explicit form: bf16 storage only
    assert f32.prefill_chunk_attn_status(*ok) == B.MTLA_ERR_UNSUPPORTED
    # scratch: fp16 states, RoPE keys, keys and values for batch * (max_past_slots + T) rows, two weight copies
    g = GOOD
    rows = 4 * (50 + 100)
    need = rows * 2 * (g["r"] + g["d_rope"] + 2 * g["n_heads"] * g["d_head"]) + 2 * 2 * g["n_heads"] * g["d_head"] * g["r"]
    got = ctx.prefill_chunk_workspace_bytes(4, 100, 50)
    assert need <= got <= need + 6 * 256
    assert ctx.prefill_chunk_workspace_bytes(0, 100, 50) == 0


def test_prefill_step_validates_before_enqueueing():
    ctx = B.Context(**GOOD)
    P = 0x1000
    # cache_c, cache_kr, tail_c, seq_len, q, q_rope, c, kr, n_new, hyp_A, hyp_a, hyp_G, w_uk, w_uv, batch, T,
    # max_past_slots, out, w_out, scratch, workspace
    ok = [P, P, P, P, P, P, P, P, None, P, None, P, P, P, 4, 100, 0, P, None, P, P]
    for i in (0, 1, 2, 3, 4, 5, 6, 7, 9, 11, 12, 13, 17, 19, 20):
        a = list(ok)
        a[i] = None
        assert ctx.prefill_step_status(*a) == B.MTLA_ERR_INVALID_ARG, i
    for i, v in ((14, 0), (14, GOOD["max_batch"] + 1), (15, 0), (16, -1), (16, GOOD["max_slots"] + 1)):
        a = list(ok)
        a[i] = v
        assert ctx.prefill_step_status(*a) == B.MTLA_ERR_INVALID_ARG, (i, v)
    a = list(ok); a[18] = P + 4                              # misaligned merge-weight output
    assert ctx.prefill_step_status(*a) == B.MTLA_ERR_INVALID_ARG
    f32 = B.Context(**{**GOOD, "dtype": "f32"})
    assert f32.prefill_step_status(*ok) == B.MTLA_ERR_UNSUPPORTED
    assert ctx.prefill_step_scratch_bytes(4, 100, 9) > ctx.prefill_chunk_workspace_bytes(4, 100, 9) + 4 * 100 * 4
    assert ctx.prefill_step_scratch_bytes(4, 0, 9) == 0


def test_layer_prefill_validates_before_enqueueing():
    ctx = B.Context(**GOOD)
    P = 0x1000
    lw = dict(w_q=P, w_qr=P, w_r=P, w_kr=P, w_o=P, d_model=512)
    # lw, cache_c, cache_kr, tail_c, seq_len, x, n_new, hyp_A, hyp_a, hyp_G, w_uk, w_uv, batch, T, max_past_slots, y, scratch, ws
    ok = [lw, P, P, P, P, P, None, P, None, P, P, P, 4, 100, 0, P, P, P]
    for i in (1, 2, 3, 4, 5, 7, 9, 10, 11, 15, 16, 17):
        a = list(ok)
        a[i] = None
        assert ctx.layer_prefill_status(*a) == B.MTLA_ERR_INVALID_ARG, i
    for k in ("w_q", "w_qr", "w_r", "w_kr", "w_o"):
        a = list(ok)
        a[0] = {**lw, k: None}
        assert ctx.layer_prefill_status(*a) == B.MTLA_ERR_INVALID_ARG, k
    for i, v in ((12, 0), (12, GOOD["max_batch"] + 1), (13, 0), (14, -1), (14, GOOD["max_slots"] + 1)):
        a = list(ok)
        a[i] = v
        assert ctx.layer_prefill_status(*a) == B.MTLA_ERR_INVALID_ARG, (i, v)
    a = list(ok); a[0] = {**lw, "d_model": 100}              # not a multiple of 32
    assert ctx.layer_prefill_status(*a) == B.MTLA_ERR_UNSUPPORTED
    a = list(ok); a[0] = {**lw, "ln_eps": -1.0}
    assert ctx.layer_prefill_status(*a) == B.MTLA_ERR_INVALID_ARG
    a = list(ok); a[5] = P + 8                               # misaligned token stream
    assert ctx.layer_prefill_status(*a) == B.MTLA_ERR_INVALID_ARG
    f32 = B.Context(**{**GOOD, "dtype": "f32"})
    assert f32.layer_prefill_status(*ok) == B.MTLA_ERR_UNSUPPORTED
    # hyper-network widths or strides the matrix-core bulk append does not take: the other append kernel would merge
    # the rounded latents while the attention works from the unrounded ones, so the call is refused
    for odd in ({"d_hyper": 40}, {"d_hyper": 96}, {"stride": 17}):
        assert B.Context(**{**GOOD, **odd}).layer_prefill_status(*ok) == B.MTLA_ERR_UNSUPPORTED, odd
    # the scratch holds at least the projections' outputs and the scratch of the continuing prefill
    g = GOOD
    M = 4 * 100
    least = M * 2 * (2 * g["n_heads"] * g["d_head"] + g["n_heads"] * g["d_rope"]) + ctx.prefill_chunk_workspace_bytes(4, 100, 7)
    assert ctx.layer_prefill_scratch_bytes(512, 4, 100, 7) > least
    assert ctx.layer_prefill_scratch_bytes(512, 0, 100, 7) == 0


def test_layer_step_validates_before_enqueueing():
    ctx = B.Context(**GOOD)
    P = 0x1000
    lw = dict(w_q=P, w_qr=P, w_r=P, w_kr=P, w_o=P, d_model=512)
    ok = [lw, P, P, P, P, P, P, None, P, P, P, 16, P, None, P, P]
    assert ctx.layer_scratch_bytes(16) > 0 and ctx.layer_scratch_bytes(0) == 0
    for i in (4, 5, 9, 10, 12, 14):                          # seq_len, x, w_uk, w_uv, y, scratch
        a = list(ok)
        a[i] = None
        assert ctx.layer_decode_step_status(*a) == B.MTLA_ERR_INVALID_ARG
    for k in ("w_q", "w_qr", "w_r", "w_kr", "w_o"):
        a = list(ok)
        a[0] = dict(lw, **{k: None})
        assert ctx.layer_decode_step_status(*a) == B.MTLA_ERR_INVALID_ARG
    a = list(ok); a[11] = 17                                 # batch > max_batch
    assert ctx.layer_decode_step_status(*a) == B.MTLA_ERR_INVALID_ARG
    a = list(ok); a[5] = P + 4                               # misaligned x
    assert ctx.layer_decode_step_status(*a) == B.MTLA_ERR_INVALID_ARG
    a = list(ok); a[0] = dict(lw, ln_eps=-1.0)
    assert ctx.layer_decode_step_status(*a) == B.MTLA_ERR_INVALID_ARG
    a = list(ok); a[0] = dict(lw, d_model=100)               # not a multiple of 32
    assert ctx.layer_decode_step_status(*a) == B.MTLA_ERR_UNSUPPORTED
    a = list(ok); a[1] = None                                # caught by the step's own argument check
    assert ctx.layer_decode_step_status(*a) == B.MTLA_ERR_INVALID_ARG
    f32 = B.Context(**dict(GOOD, dtype="f32"))
    assert f32.layer_decode_step_status(*ok) == B.MTLA_ERR_UNSUPPORTED


def test_paged_contexts_validate_their_geometry_and_take_paged_calls_only():
    paged = dict(GOOD, page_slots=64, n_pages=200)
    ctx = B.Context(**paged)
    assert ctx.cache_c_bytes() == 200 * 64 * 256 * 2 and ctx.cache_kr_bytes() == 200 * 64 * 32 * 2
    assert ctx.page_table_bytes() == 16 * 10 * 4            # ceil(640 / 64) entries per sequence
    assert B.Context(**GOOD).page_table_bytes() == 0
    for bad, status in ((dict(page_slots=48), B.MTLA_ERR_SHAPE), (dict(page_slots=8), B.MTLA_ERR_SHAPE),
                        (dict(page_slots=64, n_pages=0), B.MTLA_ERR_SHAPE), (dict(page_slots=0, n_pages=5), B.MTLA_ERR_SHAPE),
                        (dict(dtype="f32"), B.MTLA_ERR_UNSUPPORTED)):
        with pytest.raises(B.MtlaError) as e:
            B.Context(**{**paged, **bad})
        assert e.value.status == status, bad
    P = 0x1000
    # a paged context refuses the contiguous calls, a contiguous one the paged calls, before anything is enqueued
    flat = B.Context(**GOOD)
    assert ctx.decode_attn_status(P, P, P, P, P, P, P, 4, P, None, None, P) == B.MTLA_ERR_INVALID_ARG
    assert flat.decode_attn_paged_status(P, P, P, P, P, P, P, P, 4, P, None, None, P) == B.MTLA_ERR_INVALID_ARG
    assert ctx.cache_append_status(P, P, P, P, P, P, None, 1, 4, P, None, P, None, None, None, P) == B.MTLA_ERR_INVALID_ARG
    assert flat.cache_append_paged_status(P, P, P, P, P, P, P, None, 1, 4, P, None, P, None, None, None, P) == B.MTLA_ERR_INVALID_ARG
    assert ctx.cache_reorder_status(P, P, P, P, P, 4, 0x2000, 0x3000, 0x4000, 0x5000, P) == B.MTLA_ERR_INVALID_ARG
    assert flat.cache_fork_paged_status(P, P, P, P, P, P, P, 4, 0x2000, 0x3000, 0x4000, P) == B.MTLA_ERR_INVALID_ARG
    # the fork's own checks: NULL, batch, source and destination the same arrays
    ok = [P, P, P, P, P, P, P, 4, 0x2000, 0x3000, 0x4000, P]
    for i in (0, 1, 2, 3, 4, 5, 6, 8, 9, 10, 11):
        a = list(ok); a[i] = None
        assert ctx.cache_fork_paged_status(*a) == B.MTLA_ERR_INVALID_ARG, i
    for i, v in ((7, 0), (7, 17), (8, P), (9, P), (10, P)):
        a = list(ok); a[i] = v
        assert ctx.cache_fork_paged_status(*a) == B.MTLA_ERR_INVALID_ARG, (i, v)


def test_single_hip_runtime_in_process():
    """The library must share the HIP runtime of the process that owns the buffers: importing the
    binding (before or after torch) may never leave two copies of the runtime loaded."""
    import torch  # noqa: F401
    loaded = {line.split()[-1] for line in open("/proc/self/maps") if "libamdhip64" in line}
    assert len(loaded) == 1, loaded


def test_header_is_plain_c_and_cpp(tmp_path):
    """The boundary is a C ABI: the header must compile on its own as C99 and as C++17."""
    import shutil
    import subprocess
    hdr = os.path.join(ROOT, "include", "mtla.h")
    for cc, std, lang in (("gcc", "-std=c99", "c"), ("g++", "-std=c++17", "c++")):
        if shutil.which(cc) is None:
            pytest.skip(f"{cc} not available")
        src = tmp_path / f"use_header.{'c' if lang == 'c' else 'cpp'}"
        src.write_text('#include "mtla.h"\nint main(void) { mtla_config c; (void)c; return (int)MTLA_OK; }\n')
        subprocess.run([cc, std, "-Wall", "-Wextra", "-Werror", "-pedantic", "-fsyntax-only", "-I",
                        os.path.dirname(hdr), str(src)], check=True)


def test_bench_refuses_more_than_one_gpu():
    # every box has one GPU: --gpus above 1 ends with a message and a non-zero status, before anything is loaded
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=60)
    assert r.returncode == 2 and "one GPU" in r.stderr and r.stdout.strip() == ""
