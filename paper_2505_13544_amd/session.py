"""Device-memory plumbing around the C-ABI: torch allocates the buffers and
supplies the stream; every computation happens inside libmtla."""
from __future__ import annotations

from typing import Optional

import numpy as np
import torch

from . import binding as B


def torch_dtype(dtype: str) -> torch.dtype:
    return {"f32": torch.float32, "bf16": torch.bfloat16}[dtype]


def to_device(a: np.ndarray, dtype: str, device="cuda:0") -> torch.Tensor:
    """Upload a float32 array whose values are exact in `dtype` (no rounding happens)."""
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(device)
    return t if dtype == "f32" else t.to(torch.bfloat16)


class Session:
    """One MTLA attention layer's device state plus the library calls."""

    def __init__(self, *, n_heads, d_head, r, d_rope, d_hyper, stride, max_batch, max_slots, dtype,
                 softmax_scale: float = 0.0, device="cuda:0", decode_chunk: Optional[int] = None,
                 decode_schedule: int = 0):
        if not torch.cuda.is_available():
            raise RuntimeError("libmtla needs a GPU: no HIP device is visible")
        self.dtype, self.device = dtype, torch.device(device)
        self.tdt = torch_dtype(dtype)
        self.ctx = B.Context(n_heads=n_heads, d_head=d_head, r=r, d_rope=d_rope, d_hyper=d_hyper,
                             stride=stride, max_batch=max_batch, max_slots=max_slots, dtype=dtype,
                             softmax_scale=softmax_scale)
        if decode_chunk:
            self.ctx.set_decode_chunk(decode_chunk)
        if decode_schedule:
            self.ctx.set_decode_schedule(decode_schedule)
        self.n_heads, self.d_head, self.r, self.d_rope, self.d_hyper = n_heads, d_head, r, d_rope, d_hyper
        self.stride, self.max_batch, self.max_slots = stride, max_batch, max_slots
        dev = self.device
        self.cache_c = torch.zeros(max_batch, max_slots, r, dtype=self.tdt, device=dev)
        self.cache_kr = torch.zeros(max_batch, max_slots, d_rope, dtype=self.tdt, device=dev)
        self.tail_c = torch.zeros(max_batch, r, dtype=torch.float32, device=dev)
        self.seq_len = torch.zeros(max_batch, dtype=torch.int32, device=dev)
        assert self.cache_c.numel() * self.cache_c.element_size() == self.ctx.cache_c_bytes()
        assert self.cache_kr.numel() * self.cache_kr.element_size() == self.ctx.cache_kr_bytes()
        assert self.tail_c.numel() * 4 == self.ctx.tail_bytes()
        self.workspace = torch.empty(self.ctx.workspace_bytes(), dtype=torch.uint8, device=dev)
        self.ctx.workspace_init(self.workspace, self.stream)
        self.hyp_A = self.hyp_a = self.hyp_G = self.w_uk = self.w_uv = None

    @property
    def stream(self) -> int:
        return torch.cuda.current_stream(self.device).cuda_stream

    def set_weights(self, *, hyp_A, hyp_G, w_uk, w_uv, hyp_a=None):
        up = lambda a: None if a is None else to_device(a, self.dtype, self.device)
        self.hyp_A, self.hyp_a, self.hyp_G, self.w_uk, self.w_uv = up(hyp_A), up(hyp_a), up(hyp_G), up(w_uk), up(w_uv)

    def append(self, c_new: torch.Tensor, kr_new: torch.Tensor, *, n_new: Optional[torch.Tensor] = None,
               w_override: Optional[torch.Tensor] = None, w_out: Optional[torch.Tensor] = None,
               slot_out: Optional[torch.Tensor] = None):
        batch, n_new_max = c_new.shape[0], c_new.shape[1]
        self.ctx.cache_append(self.cache_c, self.cache_kr, self.tail_c, self.seq_len, c_new, kr_new, n_new,
                              n_new_max, batch, self.hyp_A, self.hyp_a, self.hyp_G, w_override, w_out,
                              slot_out, self.workspace, self.stream)

    def decode(self, q: torch.Tensor, q_rope: torch.Tensor, *, out=None, out_latent=None, lse=None):
        batch = q.shape[0]
        self.ctx.decode_attn(q, q_rope, self.w_uk, self.w_uv if out is not None else None, self.cache_c,
                             self.cache_kr, self.seq_len, batch, out, out_latent, lse, self.workspace,
                             self.stream)

    def step(self, c_new: torch.Tensor, kr_new: torch.Tensor, q: torch.Tensor, q_rope: torch.Tensor, *,
             out=None, out_latent=None, lse=None):
        """One step of incremental inference: append the token of every sequence, then attend."""
        batch = q.shape[0]
        self.ctx.decode_step(self.cache_c, self.cache_kr, self.tail_c, self.seq_len, c_new, kr_new, self.hyp_A,
                             self.hyp_a, self.hyp_G, q, q_rope, self.w_uk, self.w_uv if out is not None else None,
                             batch, out, out_latent, lse, self.workspace, self.stream)

    def step_static(self, c_new, kr_new, q, q_rope, *, status: torch.Tensor, out=None, out_latent=None, lse=None):
        """The same step with the library's static scratch instead of this session's workspace;
        `status` is the caller's sticky int32 status word on the device."""
        batch = q.shape[0]
        self.ctx.decode_step_static(self.cache_c, self.cache_kr, self.tail_c, self.seq_len, c_new, kr_new, self.hyp_A,
                                    self.hyp_a, self.hyp_G, q, q_rope, self.w_uk, self.w_uv if out is not None else None,
                                    batch, out, out_latent, lse, status, self.stream)

    def reorder(self, src_index: torch.Tensor, first_slot: int = 0):
        """Beam reordering: sequence b continues what was sequence src_index[b] (int32 device tensor).
        The state is gathered into a second set of buffers, which then becomes the session's state.
        `first_slot` > 0: all sequences hold the same first slots (a shared prompt) in both sets of buffers
        (the first such call copies them over), and only the slots from there on are moved."""
        batch = src_index.shape[0]
        if getattr(self, "_alt", None) is None:
            self._alt = [torch.empty_like(t) for t in (self.cache_c, self.cache_kr, self.tail_c, self.seq_len)]
            if first_slot > 0:
                self._alt[0][:, :first_slot].copy_(self.cache_c[:, :first_slot])
                self._alt[1][:, :first_slot].copy_(self.cache_kr[:, :first_slot])
        self.ctx.cache_reorder_from(self.cache_c, self.cache_kr, self.tail_c, self.seq_len, src_index, batch, first_slot,
                                    self._alt[0], self._alt[1], self._alt[2], self._alt[3], self.workspace, self.stream)
        cur = [self.cache_c, self.cache_kr, self.tail_c, self.seq_len]
        self.cache_c, self.cache_kr, self.tail_c, self.seq_len = self._alt
        self._alt = cur

    def share_prefix(self, prefix_owner=None, prefix_slots=None):
        """Decode calls read slots j < prefix_slots[b] of sequence b from sequence prefix_owner[b]'s rows (int32
        device tensors, kept alive here); no arguments: every sequence reads its own rows again."""
        n = 0 if prefix_owner is None else int(prefix_owner.numel())
        self.ctx.set_shared_prefix(prefix_owner, prefix_slots, n)

    def set_layer_weights(self, *, w_q, w_qr, w_r, w_kr, w_o, ln_gamma=None, ln_beta=None, ln_eps=0.0,
                          rope_base=0.0):
        """Weights of the projections around the path, output-major ([out_features, d_model])."""
        up = lambda a: None if a is None else to_device(a, self.dtype, self.device)
        self.layer_w = dict(w_q=up(w_q), w_qr=up(w_qr), w_r=up(w_r), w_kr=up(w_kr), w_o=up(w_o), ln_gamma=up(ln_gamma),
                            ln_beta=up(ln_beta), d_model=int(w_q.shape[1]), ln_eps=ln_eps, rope_base=rope_base)
        self.layer_scratch = None

    def layer_step(self, x: torch.Tensor, *, y: torch.Tensor, out=None):
        """One token per sequence through the whole attention layer: projections, step, W_O."""
        batch = x.shape[0]
        if self.layer_scratch is None or self.layer_scratch.numel() < self.ctx.layer_scratch_bytes(batch):
            self.layer_scratch = torch.empty(self.ctx.layer_scratch_bytes(batch), dtype=torch.uint8, device=self.device)
        self.ctx.layer_decode_step(self.layer_w, self.cache_c, self.cache_kr, self.tail_c, self.seq_len, x, self.hyp_A,
                                   self.hyp_a, self.hyp_G, self.w_uk, self.w_uv, batch, y, out, self.layer_scratch,
                                   self.workspace, self.stream)

    def layer_prefill(self, x: torch.Tensor, *, y: torch.Tensor, max_past_slots: int = 0, n_new=None):
        """T tokens per sequence through the whole attention layer in the parallel form, continuing from
        whatever the cache holds (`max_past_slots` bounds seq_len // stride before the call)."""
        batch, T = x.shape[0], x.shape[1]
        nbytes = self.ctx.layer_prefill_scratch_bytes(self.layer_w["d_model"], batch, T, max_past_slots)
        scratch = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        self.ctx.layer_prefill(self.layer_w, self.cache_c, self.cache_kr, self.tail_c, self.seq_len, x, n_new,
                               self.hyp_A, self.hyp_a, self.hyp_G, self.w_uk, self.w_uv, batch, T, max_past_slots, y,
                               scratch, self.workspace, self.stream)
        return scratch  # keep alive until the stream has consumed it

    def prefill(self, q, q_rope, c, kr, w, *, out, out_latent=None, seq_lens=None):
        batch, T = c.shape[0], c.shape[1]
        nbytes = self.ctx.prefill_workspace_bytes(batch, T)
        ws = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        self.ctx.prefill_attn(q, q_rope, c, kr, w, seq_lens, batch, T, self.w_uk, self.w_uv, out, out_latent,
                              ws, self.stream)
        return ws  # keep alive until the stream has consumed it

    def prefill_chunk(self, q, q_rope, c, kr, *, out, max_past_slots: int, n_new=None, w_out=None):
        """T more tokens for every sequence, behind what the cache already holds: appends them (the cache then
        covers the chunk) and gives the attention output of every one of them, as incremental inference
        would step by step.  `max_past_slots` bounds seq_len // stride before the call (the caller keeps
        the lengths on the host)."""
        batch, T = c.shape[0], c.shape[1]
        scratch = torch.empty(self.ctx.prefill_step_scratch_bytes(batch, T, max_past_slots), dtype=torch.uint8,
                              device=self.device)
        self.ctx.prefill_step(self.cache_c, self.cache_kr, self.tail_c, self.seq_len, q, q_rope, c, kr, n_new,
                              self.hyp_A, self.hyp_a, self.hyp_G, self.w_uk, self.w_uv, batch, T, max_past_slots, out,
                              w_out, scratch, self.workspace, self.stream)
        return scratch  # keep alive until the stream has consumed it

    def device_status(self) -> int:
        return self.ctx.device_status(self.workspace, self.stream)


class PagedSession:
    """Session over paged slot storage: one pool of pages, a page table per sequence, and the bookkeeping of
    who refers to which page.  That bookkeeping is memory management, done here on the host (the lengths are
    mirrored on the host: every append is issued from here); everything the method computes happens in libmtla."""

    def __init__(self, *, n_heads, d_head, r, d_rope, d_hyper, stride, max_batch, max_slots, page_slots, n_pages,
                 dtype="bf16", softmax_scale: float = 0.0, device="cuda:0", decode_chunk: Optional[int] = None,
                 decode_schedule: int = 0, page_order=None):
        if not torch.cuda.is_available():
            raise RuntimeError("libmtla needs a GPU: no HIP device is visible")
        self.dtype, self.device, self.tdt = dtype, torch.device(device), torch_dtype(dtype)
        self.ctx = B.Context(n_heads=n_heads, d_head=d_head, r=r, d_rope=d_rope, d_hyper=d_hyper, stride=stride,
                             max_batch=max_batch, max_slots=max_slots, dtype=dtype, softmax_scale=softmax_scale,
                             page_slots=page_slots, n_pages=n_pages)
        if decode_chunk:
            self.ctx.set_decode_chunk(decode_chunk)
        if decode_schedule:
            self.ctx.set_decode_schedule(decode_schedule)
        self.n_heads, self.d_head, self.r, self.d_rope = n_heads, d_head, r, d_rope
        self.stride, self.max_batch, self.max_slots = stride, max_batch, max_slots
        self.page_slots, self.n_pages = page_slots, n_pages
        self.max_pages = -(-max_slots // page_slots)
        dev = self.device
        self.pool_c = torch.zeros(n_pages, page_slots, r, dtype=self.tdt, device=dev)
        self.pool_kr = torch.zeros(n_pages, page_slots, d_rope, dtype=self.tdt, device=dev)
        assert self.pool_c.numel() * 2 == self.ctx.cache_c_bytes() and self.pool_kr.numel() * 2 == self.ctx.cache_kr_bytes()
        assert max_batch * self.max_pages * 4 == self.ctx.page_table_bytes()
        self.tail_c = torch.zeros(max_batch, r, dtype=torch.float32, device=dev)
        self.seq_len = torch.zeros(max_batch, dtype=torch.int32, device=dev)
        self.table = torch.zeros(max_batch, self.max_pages, dtype=torch.int32, device=dev)
        self.workspace = torch.empty(self.ctx.workspace_bytes(), dtype=torch.uint8, device=dev)
        self.ctx.workspace_init(self.workspace, self.stream)
        self.hyp_A = self.hyp_a = self.hyp_G = self.w_uk = self.w_uv = None
        # host side: table (-1 = no page yet), lengths, reference counts, free pages (handed out in `page_order`)
        self.h_table = np.full((max_batch, self.max_pages), -1, np.int32)
        self.h_len = np.zeros(max_batch, np.int64)
        self.refs = np.zeros(n_pages, np.int32)
        self.free = list(range(n_pages)) if page_order is None else [int(p) for p in page_order]
        self._alt = None

    @property
    def stream(self) -> int:
        return torch.cuda.current_stream(self.device).cuda_stream

    set_weights = Session.set_weights

    # ---- pages
    def _alloc(self) -> int:
        if not self.free:
            raise RuntimeError("page pool exhausted")
        p = self.free.pop(0)
        self.refs[p] = 1
        return p

    def _release(self, p: int):
        self.refs[p] -= 1
        assert self.refs[p] >= 0
        if self.refs[p] == 0:
            self.free.append(int(p))

    def reserve(self, n_new):
        """Pages for n_new[b] more tokens of every sequence, ahead of time (a caller that replays steps as a graph
        reserves once and then steps with reserve=False)."""
        self._reserve(n_new)

    def _reserve(self, n_new):
        """Pages for n_new[b] more tokens of every sequence; uploads the table if it changed."""
        changed = False
        for b, n in enumerate(n_new):
            need = -(-(-(-(int(self.h_len[b]) + int(n)) // self.stride)) // self.page_slots)
            for k in range(min(need, self.max_pages)):
                if self.h_table[b, k] < 0:
                    self.h_table[b, k] = self._alloc()
                    changed = True
        if changed:
            self.table.copy_(torch.from_numpy(self.h_table).to(self.device))

    def pages_in_use(self) -> int:
        return int((self.refs > 0).sum())

    def rows(self, b: int, n_slots: int):
        """Slots 0 .. n_slots-1 of sequence b gathered out of the pool: (C_hat, K_hat^R) as the contiguous layout holds them."""
        pages = torch.from_numpy(self.h_table[b, :-(-n_slots // self.page_slots)].astype(np.int64)).to(self.device)
        c = self.pool_c[pages].reshape(-1, self.r)[:n_slots]
        kr = self.pool_kr[pages].reshape(-1, self.d_rope)[:n_slots]
        return c, kr

    # ---- calls
    def append(self, c_new, kr_new, *, n_new=None, w_out=None, slot_out=None):
        """n_new: host integers (list / array) or None for c_new.shape[1] tokens everywhere."""
        batch, n_max = c_new.shape[0], c_new.shape[1]
        n_host = [n_max] * batch if n_new is None else [int(x) for x in n_new]
        self._reserve(n_host)
        n_dev = None if n_new is None else torch.tensor(n_host, dtype=torch.int32, device=self.device)
        self.ctx.cache_append_paged(self.pool_c, self.pool_kr, self.tail_c, self.seq_len, self.table, c_new, kr_new, n_dev,
                                    n_max, batch, self.hyp_A, self.hyp_a, self.hyp_G, None, w_out, slot_out, self.workspace,
                                    self.stream)
        self.h_len[:batch] += np.asarray(n_host)

    def decode(self, q, q_rope, *, out=None, out_latent=None, lse=None):
        self.ctx.decode_attn_paged(q, q_rope, self.w_uk, self.w_uv if out is not None else None, self.pool_c, self.pool_kr,
                                   self.seq_len, self.table, q.shape[0], out, out_latent, lse, self.workspace, self.stream)

    def step(self, c_new, kr_new, q, q_rope, *, out=None, out_latent=None, lse=None, reserve=True):
        batch = q.shape[0]
        if reserve:
            self._reserve([1] * batch)
        self.ctx.decode_step_paged(self.pool_c, self.pool_kr, self.tail_c, self.seq_len, self.table, c_new, kr_new,
                                   self.hyp_A, self.hyp_a, self.hyp_G, q, q_rope, self.w_uk,
                                   self.w_uv if out is not None else None, batch, out, out_latent, lse, self.workspace,
                                   self.stream)
        self.h_len[:batch] += 1

    def prefill_chunk(self, q, q_rope, c, kr, *, out, max_past_slots: int, n_new=None, w_out=None):
        batch, T = c.shape[0], c.shape[1]
        n_host = [T] * batch if n_new is None else [int(x) for x in n_new]
        self._reserve(n_host)
        n_dev = None if n_new is None else torch.tensor(n_host, dtype=torch.int32, device=self.device)
        scratch = torch.empty(self.ctx.prefill_step_scratch_bytes(batch, T, max_past_slots), dtype=torch.uint8,
                              device=self.device)
        self.ctx.prefill_step_paged(self.pool_c, self.pool_kr, self.tail_c, self.seq_len, self.table, q, q_rope, c, kr,
                                    n_dev, self.hyp_A, self.hyp_a, self.hyp_G, self.w_uk, self.w_uv, batch, T,
                                    max_past_slots, out, w_out, scratch, self.workspace, self.stream)
        self.h_len[:batch] += np.asarray(n_host)
        return scratch

    def fork(self, src_index):
        """Beam reordering: sequence b continues what was sequence src_index[b] (host integers).  Complete pages are
        shared; every continuation gets a page of its own for the page being written to -- the source's own, taken
        over, when it is the source's only continuation.  Sequences nobody continues give their pages back."""
        src_index = [int(x) for x in src_index]
        batch = len(src_index)
        if self._alt is None:
            self._alt = [torch.zeros_like(self.table), torch.empty_like(self.tail_c), torch.zeros_like(self.seq_len)]
        uses = {s: src_index.count(s) for s in set(src_index)}
        new_table = np.full_like(self.h_table, -1)
        new_len = np.zeros_like(self.h_len)
        fresh = np.zeros(batch, np.int32)
        for b, s in enumerate(src_index):
            nxt = min(int(self.h_len[s]) // self.stride, self.max_slots - 1)
            pw = nxt // self.page_slots
            new_table[b, :pw] = self.h_table[s, :pw]
            for p in new_table[b, :pw]:
                self.refs[p] += 1
            own = int(self.h_table[s, pw])
            if uses[s] == 1 and own >= 0:     # take the source's page over
                self.refs[own] += 1
                fresh[b] = own
            else:
                fresh[b] = self._alloc()
            new_table[b, pw] = fresh[b]
            new_len[b] = self.h_len[s]
        self.ctx.cache_fork_paged(self.pool_c, self.pool_kr, self.table, self.tail_c, self.seq_len,
                                  torch.tensor(src_index, dtype=torch.int32, device=self.device),
                                  torch.from_numpy(fresh).to(self.device), batch, self._alt[0], self._alt[1], self._alt[2],
                                  self.workspace, self.stream)
        for b in range(self.max_batch):       # the old sequences let go of their pages
            for p in self.h_table[b]:
                if p >= 0:
                    self._release(int(p))
        self.h_table, self.h_len = new_table, new_len
        cur = [self.table, self.tail_c, self.seq_len]
        self.table, self.tail_c, self.seq_len = self._alt
        self._alt = cur
        # the kernel wrote rows 0 .. batch-1 of the new table up to the page being written to; what lies above is
        # whatever the buffer held, and is replaced (the whole table is uploaded) before an append reaches it

    def device_status(self) -> int:
        return self.ctx.device_status(self.workspace, self.stream)
