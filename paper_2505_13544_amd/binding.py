"""ctypes binding of libmtla: the same names and arguments as include/mtla.h.

Argument marshalling only -- every step of the path runs in the HIP kernels.
Device buffers are passed as integer addresses (e.g. ``tensor.data_ptr()``)
or objects exposing ``data_ptr()``; ``None`` is a NULL pointer.  Importing this
module loads the in-tree ``libmtla.so`` and fails loudly if it is missing:
there is no fallback implementation.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libmtla.so")

MTLA_OK, MTLA_ERR_INVALID_ARG, MTLA_ERR_SHAPE, MTLA_ERR_CAPACITY, MTLA_ERR_UNSUPPORTED, MTLA_ERR_HIP, MTLA_ERR_SCRATCH = range(7)
MTLA_STATIC_SCRATCH_BYTES = 16 << 20
MTLA_F32, MTLA_BF16 = 0, 1
DTYPES = {"f32": MTLA_F32, "bf16": MTLA_BF16}


class mtla_config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in
                ("n_heads", "d_head", "r", "d_rope", "d_hyper", "stride", "max_batch", "max_slots", "dtype")]
    _fields_.append(("softmax_scale", C.c_float))
    _fields_ += [("page_slots", C.c_int32), ("n_pages", C.c_int32)]


class mtla_layer_weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("w_q", "w_qr", "w_r", "w_kr", "w_o", "ln_gamma", "ln_beta")]
    _fields_ += [("d_model", C.c_int32), ("ln_eps", C.c_float), ("rope_base", C.c_float)]


class MtlaError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        detail = f" [{lib.mtla_last_hip_error().decode()}]" if status == MTLA_ERR_HIP else ""
        super().__init__(f"{where}: {status_str(status)} (status {status}){detail}")


def _load() -> C.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2505_13544_amd.build` "
            "(there is no non-HIP fallback)")
    # The buffers this binding passes come from torch, so the library has to talk to the HIP
    # runtime torch brought along.  torch is loaded first: the dynamic loader then resolves
    # libmtla's dependency against that copy instead of opening a second runtime beside it
    # (two runtimes in one process do not share devices, streams or allocations).
    import torch  # noqa: F401
    return C.CDLL(LIB_PATH)


lib = _load()
_vp, _i32, _sz = C.c_void_p, C.c_int32, C.c_size_t
_ctx = C.c_void_p

# name -> (restype, argtypes); one entry per declaration in include/mtla.h
SIGNATURES = {
    "mtla_create": (C.c_int, [C.POINTER(mtla_config), C.POINTER(_ctx)]),
    "mtla_destroy": (None, [_ctx]),
    "mtla_status_str": (C.c_char_p, [C.c_int]),
    "mtla_last_hip_error": (C.c_char_p, []),
    "mtla_cache_c_bytes": (_sz, [_ctx]),
    "mtla_cache_kr_bytes": (_sz, [_ctx]),
    "mtla_tail_bytes": (_sz, [_ctx]),
    "mtla_page_table_bytes": (_sz, [_ctx]),
    "mtla_cache_append_paged": (C.c_int, [_ctx, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _i32,
                                          _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp]),
    "mtla_decode_attn_paged": (C.c_int, [_ctx, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _vp, _vp, _vp, _vp, _vp]),
    "mtla_decode_step_paged": (C.c_int, [_ctx] + [_vp] * 14 + [_i32] + [_vp] * 5),
    "mtla_prefill_chunk_attn_paged": (C.c_int, [_ctx, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _i32, _i32,
                                                _vp, _vp, _vp, _vp, _vp, _vp]),
    "mtla_prefill_step_paged": (C.c_int, [_ctx] + [_vp] * 15 + [_i32] * 3 + [_vp] * 5),
    "mtla_cache_fork_paged": (C.c_int, [_ctx] + [_vp] * 7 + [_i32] + [_vp] * 5),
    "mtla_workspace_bytes": (_sz, [_ctx]),
    "mtla_prefill_workspace_bytes": (_sz, [_ctx, _i32, _i32]),
    "mtla_workspace_init": (C.c_int, [_ctx, _vp, _vp]),
    "mtla_device_status": (C.c_int, [_ctx, _vp, _vp, C.POINTER(_i32)]),
    "mtla_set_decode_chunk": (C.c_int, [_ctx, _i32]),
    "mtla_get_decode_chunk": (_i32, [_ctx]),
    "mtla_set_decode_schedule": (C.c_int, [_ctx, _i32]),
    "mtla_set_shared_prefix": (C.c_int, [_ctx, _vp, _vp, _i32]),
    "mtla_profile_start": (C.c_int, [_ctx, _i32]),
    "mtla_profile_read": (C.c_int, [_ctx, C.POINTER(C.c_float), C.POINTER(_i32)]),
    "mtla_probe_stream_read": (C.c_int, [_ctx, _vp, _sz, _vp, _vp]),
    "mtla_cache_append": (C.c_int, [_ctx, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _i32,
                                    _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp]),
    "mtla_decode_attn": (C.c_int, [_ctx, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _vp, _vp, _vp, _vp, _vp]),
    "mtla_decode_step": (C.c_int, [_ctx] + [_vp] * 13 + [_i32] + [_vp] * 5),
    "mtla_decode_step_static": (C.c_int, [_ctx] + [_vp] * 13 + [_i32] + [_vp] * 5),
    "mtla_prefill_chunk_workspace_bytes": (_sz, [_ctx, _i32, _i32, _i32]),
    "mtla_prefill_chunk_attn": (C.c_int, [_ctx, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _i32, _i32,
                                          _vp, _vp, _vp, _vp, _vp, _vp]),
    "mtla_prefill_step_scratch_bytes": (_sz, [_ctx, _i32, _i32, _i32]),
    "mtla_prefill_step": (C.c_int, [_ctx] + [_vp] * 14 + [_i32] * 3 + [_vp] * 5),
    "mtla_prefill_attn": (C.c_int, [_ctx, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _i32, _vp, _vp, _vp, _vp, _vp, _vp]),
    "mtla_cache_reorder": (C.c_int, [_ctx] + [_vp] * 5 + [_i32] + [_vp] * 6),
    "mtla_cache_reorder_from": (C.c_int, [_ctx] + [_vp] * 5 + [_i32, _i32] + [_vp] * 6),
    "mtla_layer_scratch_bytes": (_sz, [_ctx, _i32]),
    "mtla_layer_prefill_scratch_bytes": (_sz, [_ctx, _i32, _i32, _i32, _i32]),
    "mtla_layer_prefill": (C.c_int, [_ctx, C.POINTER(mtla_layer_weights)] + [_vp] * 11 + [_i32] * 3 + [_vp] * 4),
    "mtla_layer_decode_step": (C.c_int, [_ctx, C.POINTER(mtla_layer_weights)] + [_vp] * 10 + [_i32] + [_vp] * 5),
}
for _name, (_res, _args) in SIGNATURES.items():
    _fn = getattr(lib, _name)          # AttributeError here = the library does not export the symbol
    _fn.restype, _fn.argtypes = _res, _args


def _p(x) -> Optional[int]:
    """Address of a device/host buffer: None, int, or anything with data_ptr()."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return x.data_ptr()


def status_str(status: int) -> str:
    return lib.mtla_status_str(status).decode()


def _check(status: int, where: str) -> None:
    if status != MTLA_OK:
        raise MtlaError(status, where)


class Context:
    """Owns an mtla_ctx*; methods mirror the C entry points one to one."""

    def __init__(self, *, n_heads, d_head, r, d_rope, d_hyper, stride, max_batch, max_slots,
                 dtype, softmax_scale: float = 0.0, page_slots: int = 0, n_pages: int = 0):
        self.cfg = mtla_config(n_heads, d_head, r, d_rope, d_hyper, stride, max_batch, max_slots,
                               DTYPES[dtype] if isinstance(dtype, str) else dtype, softmax_scale, page_slots, n_pages)
        self._h = _ctx()
        _check(lib.mtla_create(C.byref(self.cfg), C.byref(self._h)), "mtla_create")

    def close(self):
        if getattr(self, "_h", None):
            lib.mtla_destroy(self._h)
            self._h = None

    __del__ = close

    # sizes
    def cache_c_bytes(self): return lib.mtla_cache_c_bytes(self._h)
    def cache_kr_bytes(self): return lib.mtla_cache_kr_bytes(self._h)
    def tail_bytes(self): return lib.mtla_tail_bytes(self._h)
    def page_table_bytes(self): return lib.mtla_page_table_bytes(self._h)
    def workspace_bytes(self): return lib.mtla_workspace_bytes(self._h)
    def prefill_workspace_bytes(self, batch, T): return lib.mtla_prefill_workspace_bytes(self._h, batch, T)

    def prefill_chunk_workspace_bytes(self, batch, T, max_past_slots):
        return lib.mtla_prefill_chunk_workspace_bytes(self._h, batch, T, max_past_slots)

    def set_decode_chunk(self, chunk: int):
        _check(lib.mtla_set_decode_chunk(self._h, chunk), "mtla_set_decode_chunk")

    def set_decode_schedule(self, schedule: int):
        _check(lib.mtla_set_decode_schedule(self._h, schedule), "mtla_set_decode_schedule")

    def set_shared_prefix(self, prefix_owner, prefix_slots, n: int = 0):
        """The context keeps the two device addresses: the arrays are held here until they are replaced."""
        _check(lib.mtla_set_shared_prefix(self._h, _p(prefix_owner), _p(prefix_slots), n), "mtla_set_shared_prefix")
        self._prefix_arrays = (prefix_owner, prefix_slots)

    def get_decode_chunk(self) -> int:
        return lib.mtla_get_decode_chunk(self._h)

    def workspace_init(self, workspace, stream=None):
        _check(lib.mtla_workspace_init(self._h, _p(workspace), _p(stream)), "mtla_workspace_init")

    def device_status(self, workspace, stream=None) -> int:
        out = _i32(0)
        _check(lib.mtla_device_status(self._h, _p(workspace), _p(stream), C.byref(out)), "mtla_device_status")
        return out.value

    def profile_start(self, capacity: int):
        self._prof_cap = capacity
        _check(lib.mtla_profile_start(self._h, capacity), "mtla_profile_start")

    def profile_read(self):
        """Elapsed milliseconds of each bracketed dominant-kernel launch."""
        ms = (C.c_float * self._prof_cap)()
        n = _i32(0)
        _check(lib.mtla_profile_read(self._h, ms, C.byref(n)), "mtla_profile_read")
        return [ms[i] for i in range(n.value)]

    # raw status-returning calls (used by the error-path tests)
    def cache_append_status(self, cache_c, cache_kr, tail_c, seq_len, c_new, kr_new, n_new, n_new_max,
                            batch, hyp_A, hyp_a, hyp_G, w_override, w_out, slot_out, workspace,
                            stream=None) -> int:
        return lib.mtla_cache_append(self._h, _p(cache_c), _p(cache_kr), _p(tail_c), _p(seq_len), _p(c_new),
                                     _p(kr_new), _p(n_new), n_new_max, batch, _p(hyp_A), _p(hyp_a),
                                     _p(hyp_G), _p(w_override), _p(w_out), _p(slot_out), _p(workspace),
                                     _p(stream))

    def decode_attn_status(self, q, q_rope, w_uk, w_uv, cache_c, cache_kr, seq_len, batch, out,
                           out_latent, lse, workspace, stream=None) -> int:
        return lib.mtla_decode_attn(self._h, _p(q), _p(q_rope), _p(w_uk), _p(w_uv), _p(cache_c),
                                    _p(cache_kr), _p(seq_len), batch, _p(out), _p(out_latent), _p(lse),
                                    _p(workspace), _p(stream))

    def probe_stream_read(self, buf, nbytes: int, workspace, stream=None):
        _check(lib.mtla_probe_stream_read(self._h, _p(buf), nbytes, _p(workspace), _p(stream)), "mtla_probe_stream_read")

    def decode_step_status(self, cache_c, cache_kr, tail_c, seq_len, c_new, kr_new, hyp_A, hyp_a, hyp_G, q,
                           q_rope, w_uk, w_uv, batch, out, out_latent, lse, workspace, stream=None) -> int:
        return lib.mtla_decode_step(self._h, _p(cache_c), _p(cache_kr), _p(tail_c), _p(seq_len), _p(c_new),
                                    _p(kr_new), _p(hyp_A), _p(hyp_a), _p(hyp_G), _p(q), _p(q_rope), _p(w_uk),
                                    _p(w_uv), batch, _p(out), _p(out_latent), _p(lse), _p(workspace),
                                    _p(stream))

    def decode_step_static_status(self, cache_c, cache_kr, tail_c, seq_len, c_new, kr_new, hyp_A, hyp_a, hyp_G, q,
                                  q_rope, w_uk, w_uv, batch, out, out_latent, lse, device_status, stream=None) -> int:
        return lib.mtla_decode_step_static(self._h, _p(cache_c), _p(cache_kr), _p(tail_c), _p(seq_len), _p(c_new),
                                           _p(kr_new), _p(hyp_A), _p(hyp_a), _p(hyp_G), _p(q), _p(q_rope), _p(w_uk),
                                           _p(w_uv), batch, _p(out), _p(out_latent), _p(lse), _p(device_status),
                                           _p(stream))

    def decode_step_static(self, *a, **k):
        _check(self.decode_step_static_status(*a, **k), "mtla_decode_step_static")

    # paged storage: the same calls with the page table behind the state arguments
    def cache_append_paged_status(self, cache_c, cache_kr, tail_c, seq_len, page_table, c_new, kr_new, n_new, n_new_max,
                                  batch, hyp_A, hyp_a, hyp_G, w_override, w_out, slot_out, workspace, stream=None) -> int:
        return lib.mtla_cache_append_paged(self._h, _p(cache_c), _p(cache_kr), _p(tail_c), _p(seq_len), _p(page_table),
                                           _p(c_new), _p(kr_new), _p(n_new), n_new_max, batch, _p(hyp_A), _p(hyp_a),
                                           _p(hyp_G), _p(w_override), _p(w_out), _p(slot_out), _p(workspace), _p(stream))

    def decode_attn_paged_status(self, q, q_rope, w_uk, w_uv, cache_c, cache_kr, seq_len, page_table, batch, out,
                                 out_latent, lse, workspace, stream=None) -> int:
        return lib.mtla_decode_attn_paged(self._h, _p(q), _p(q_rope), _p(w_uk), _p(w_uv), _p(cache_c), _p(cache_kr),
                                          _p(seq_len), _p(page_table), batch, _p(out), _p(out_latent), _p(lse),
                                          _p(workspace), _p(stream))

    def decode_step_paged_status(self, cache_c, cache_kr, tail_c, seq_len, page_table, c_new, kr_new, hyp_A, hyp_a, hyp_G,
                                 q, q_rope, w_uk, w_uv, batch, out, out_latent, lse, workspace, stream=None) -> int:
        return lib.mtla_decode_step_paged(self._h, _p(cache_c), _p(cache_kr), _p(tail_c), _p(seq_len), _p(page_table),
                                          _p(c_new), _p(kr_new), _p(hyp_A), _p(hyp_a), _p(hyp_G), _p(q), _p(q_rope),
                                          _p(w_uk), _p(w_uv), batch, _p(out), _p(out_latent), _p(lse), _p(workspace),
                                          _p(stream))

    def prefill_chunk_attn_paged_status(self, cache_c, cache_kr, tail_prev, pos0, page_table, q, q_rope, c, kr, w, n_new,
                                        batch, T, max_past_slots, w_uk, w_uv, out, chunk_workspace, workspace,
                                        stream=None) -> int:
        return lib.mtla_prefill_chunk_attn_paged(self._h, _p(cache_c), _p(cache_kr), _p(tail_prev), _p(pos0), _p(page_table),
                                                 _p(q), _p(q_rope), _p(c), _p(kr), _p(w), _p(n_new), batch, T,
                                                 max_past_slots, _p(w_uk), _p(w_uv), _p(out), _p(chunk_workspace),
                                                 _p(workspace), _p(stream))

    def prefill_step_paged_status(self, cache_c, cache_kr, tail_c, seq_len, page_table, q, q_rope, c, kr, n_new, hyp_A,
                                  hyp_a, hyp_G, w_uk, w_uv, batch, T, max_past_slots, out, w_out, scratch, workspace,
                                  stream=None) -> int:
        return lib.mtla_prefill_step_paged(self._h, _p(cache_c), _p(cache_kr), _p(tail_c), _p(seq_len), _p(page_table),
                                           _p(q), _p(q_rope), _p(c), _p(kr), _p(n_new), _p(hyp_A), _p(hyp_a), _p(hyp_G),
                                           _p(w_uk), _p(w_uv), batch, T, max_past_slots, _p(out), _p(w_out), _p(scratch),
                                           _p(workspace), _p(stream))

    def cache_fork_paged_status(self, cache_c, cache_kr, src_table, src_tail_c, src_seq_len, src_index, fresh_pages, batch,
                                dst_table, dst_tail_c, dst_seq_len, workspace, stream=None) -> int:
        return lib.mtla_cache_fork_paged(self._h, _p(cache_c), _p(cache_kr), _p(src_table), _p(src_tail_c), _p(src_seq_len),
                                         _p(src_index), _p(fresh_pages), batch, _p(dst_table), _p(dst_tail_c),
                                         _p(dst_seq_len), _p(workspace), _p(stream))

    def cache_append_paged(self, *a, **k): _check(self.cache_append_paged_status(*a, **k), "mtla_cache_append_paged")
    def decode_attn_paged(self, *a, **k): _check(self.decode_attn_paged_status(*a, **k), "mtla_decode_attn_paged")
    def decode_step_paged(self, *a, **k): _check(self.decode_step_paged_status(*a, **k), "mtla_decode_step_paged")
    def prefill_step_paged(self, *a, **k): _check(self.prefill_step_paged_status(*a, **k), "mtla_prefill_step_paged")
    def cache_fork_paged(self, *a, **k): _check(self.cache_fork_paged_status(*a, **k), "mtla_cache_fork_paged")

    def cache_reorder_status(self, src_cache_c, src_cache_kr, src_tail_c, src_seq_len, src_index, batch, dst_cache_c,
                             dst_cache_kr, dst_tail_c, dst_seq_len, workspace, stream=None) -> int:
        return lib.mtla_cache_reorder(self._h, _p(src_cache_c), _p(src_cache_kr), _p(src_tail_c), _p(src_seq_len),
                                      _p(src_index), batch, _p(dst_cache_c), _p(dst_cache_kr), _p(dst_tail_c),
                                      _p(dst_seq_len), _p(workspace), _p(stream))

    def cache_reorder(self, *a, **k):
        _check(self.cache_reorder_status(*a, **k), "mtla_cache_reorder")

    def cache_reorder_from_status(self, src_cache_c, src_cache_kr, src_tail_c, src_seq_len, src_index, batch, first_slot,
                                  dst_cache_c, dst_cache_kr, dst_tail_c, dst_seq_len, workspace, stream=None) -> int:
        return lib.mtla_cache_reorder_from(self._h, _p(src_cache_c), _p(src_cache_kr), _p(src_tail_c), _p(src_seq_len),
                                           _p(src_index), batch, first_slot, _p(dst_cache_c), _p(dst_cache_kr),
                                           _p(dst_tail_c), _p(dst_seq_len), _p(workspace), _p(stream))

    def cache_reorder_from(self, *a, **k):
        _check(self.cache_reorder_from_status(*a, **k), "mtla_cache_reorder_from")

    def layer_scratch_bytes(self, batch: int) -> int:
        return lib.mtla_layer_scratch_bytes(self._h, batch)

    def layer_decode_step_status(self, lw, cache_c, cache_kr, tail_c, seq_len, x, hyp_A, hyp_a, hyp_G, w_uk, w_uv,
                                 batch, y, out, scratch, workspace, stream=None) -> int:
        """lw: dict with w_q, w_qr, w_r, w_kr, w_o, d_model and optionally ln_gamma, ln_beta, ln_eps, rope_base."""
        st = mtla_layer_weights(_p(lw["w_q"]), _p(lw["w_qr"]), _p(lw["w_r"]), _p(lw["w_kr"]), _p(lw["w_o"]),
                                _p(lw.get("ln_gamma")), _p(lw.get("ln_beta")), lw["d_model"],
                                lw.get("ln_eps", 0.0), lw.get("rope_base", 0.0))
        return lib.mtla_layer_decode_step(self._h, C.byref(st), _p(cache_c), _p(cache_kr), _p(tail_c), _p(seq_len),
                                          _p(x), _p(hyp_A), _p(hyp_a), _p(hyp_G), _p(w_uk), _p(w_uv), batch, _p(y),
                                          _p(out), _p(scratch), _p(workspace), _p(stream))

    def layer_prefill_scratch_bytes(self, d_model: int, batch: int, T: int, max_past_slots: int) -> int:
        return lib.mtla_layer_prefill_scratch_bytes(self._h, d_model, batch, T, max_past_slots)

    def layer_prefill_status(self, lw, cache_c, cache_kr, tail_c, seq_len, x, n_new, hyp_A, hyp_a, hyp_G, w_uk, w_uv,
                             batch, T, max_past_slots, y, scratch, workspace, stream=None) -> int:
        st = mtla_layer_weights(_p(lw["w_q"]), _p(lw["w_qr"]), _p(lw["w_r"]), _p(lw["w_kr"]), _p(lw["w_o"]),
                                _p(lw.get("ln_gamma")), _p(lw.get("ln_beta")), lw["d_model"],
                                lw.get("ln_eps", 0.0), lw.get("rope_base", 0.0))
        return lib.mtla_layer_prefill(self._h, C.byref(st), _p(cache_c), _p(cache_kr), _p(tail_c), _p(seq_len), _p(x),
                                      _p(n_new), _p(hyp_A), _p(hyp_a), _p(hyp_G), _p(w_uk), _p(w_uv), batch, T,
                                      max_past_slots, _p(y), _p(scratch), _p(workspace), _p(stream))

    def layer_prefill(self, *a, **k):
        _check(self.layer_prefill_status(*a, **k), "mtla_layer_prefill")

    def prefill_attn_status(self, q, q_rope, c, kr, w, seq_lens, batch, T, w_uk, w_uv, out, out_latent,
                            prefill_workspace, stream=None) -> int:
        return lib.mtla_prefill_attn(self._h, _p(q), _p(q_rope), _p(c), _p(kr), _p(w), _p(seq_lens),
                                     batch, T, _p(w_uk), _p(w_uv), _p(out), _p(out_latent),
                                     _p(prefill_workspace), _p(stream))

    def cache_append(self, *a, **k):
        _check(self.cache_append_status(*a, **k), "mtla_cache_append")

    def decode_attn(self, *a, **k):
        _check(self.decode_attn_status(*a, **k), "mtla_decode_attn")

    def decode_step(self, *a, **k):
        _check(self.decode_step_status(*a, **k), "mtla_decode_step")

    def prefill_step_scratch_bytes(self, batch, T, max_past_slots):
        return lib.mtla_prefill_step_scratch_bytes(self._h, batch, T, max_past_slots)

    def prefill_step_status(self, cache_c, cache_kr, tail_c, seq_len, q, q_rope, c, kr, n_new, hyp_A, hyp_a, hyp_G,
                            w_uk, w_uv, batch, T, max_past_slots, out, w_out, scratch, workspace, stream=None) -> int:
        return lib.mtla_prefill_step(self._h, _p(cache_c), _p(cache_kr), _p(tail_c), _p(seq_len), _p(q), _p(q_rope),
                                     _p(c), _p(kr), _p(n_new), _p(hyp_A), _p(hyp_a), _p(hyp_G), _p(w_uk), _p(w_uv),
                                     batch, T, max_past_slots, _p(out), _p(w_out), _p(scratch), _p(workspace),
                                     _p(stream))

    def prefill_step(self, *a, **k):
        _check(self.prefill_step_status(*a, **k), "mtla_prefill_step")

    def prefill_chunk_attn_status(self, cache_c, cache_kr, tail_prev, pos0, q, q_rope, c, kr, w, n_new, batch, T,
                                  max_past_slots, w_uk, w_uv, out, chunk_workspace, workspace, stream=None) -> int:
        return lib.mtla_prefill_chunk_attn(self._h, _p(cache_c), _p(cache_kr), _p(tail_prev), _p(pos0), _p(q),
                                           _p(q_rope), _p(c), _p(kr), _p(w), _p(n_new), batch, T, max_past_slots,
                                           _p(w_uk), _p(w_uv), _p(out), _p(chunk_workspace), _p(workspace), _p(stream))

    def prefill_chunk_attn(self, *a, **k):
        _check(self.prefill_chunk_attn_status(*a, **k), "mtla_prefill_chunk_attn")

    def prefill_attn(self, *a, **k):
        _check(self.prefill_attn_status(*a, **k), "mtla_prefill_attn")

    def layer_decode_step(self, *a, **k):
        _check(self.layer_decode_step_status(*a, **k), "mtla_layer_decode_step")
