"""Seeded synthetic inputs shaped like the paper's decoder models.

The paper's decoder (Experimental Setup; appendix "Hyper-parameter Details")
has 512 attention dims, 8 heads of 64, latent r=256, decoupled-RoPE dim 32 and
a hyper-network mapping r -> 64; its datasets and trained weights are not
available, so Gaussian tensors of those shapes (and scaled-up variants) stand
in for them.

Everything here is *input preparation*: projections of the token stream
x -> q, q_rope, c = LayerNorm(x W_r), k_rope, the rotary rotation, the
sinusoidal table behind the hyper-network's positional branch, and rounding
to the storage dtype.  None of it is part of the attention path proper, which
starts from these tensors.  All values handed out are exactly representable
in the storage dtype (fp32 or bf16) and are returned as float32 arrays, so the
CPU oracle and the GPU path consume bit-identical numbers.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, Optional, Tuple, Union

import numpy as np

BLOCK = 1024  # token positions generated per RNG block (makes sub-ranges reproducible)


# --------------------------------------------------------------------------
# storage rounding
# --------------------------------------------------------------------------
def bf16_bits(x: np.ndarray) -> np.ndarray:
    """float -> bf16 bit patterns (uint16), round-to-nearest-even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bits_to_f32(b: np.ndarray) -> np.ndarray:
    """bf16 bit patterns (uint16) -> the float32 values they denote."""
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_round(x: np.ndarray) -> np.ndarray:
    """Round to the nearest bf16 value, returned as float32."""
    return bits_to_f32(bf16_bits(x))


def storage_round(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round once to the storage dtype ('f32' or 'bf16'); result is float32."""
    if dtype == "bf16":
        return bf16_round(x)
    if dtype == "f32":
        return np.ascontiguousarray(x, dtype=np.float32)
    raise ValueError(f"unknown storage dtype {dtype!r}")


# --------------------------------------------------------------------------
# pieces of the model that sit in front of the attention path
# --------------------------------------------------------------------------
def layer_norm(x: np.ndarray, eps: float = 1e-5) -> np.ndarray:
    """Non-affine LayerNorm over the last axis (gamma=1, beta=0)."""
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    return (x - mu) / np.sqrt(var + eps)


def rope_rotate(v: np.ndarray, pos: np.ndarray, base: float = 10000.0) -> np.ndarray:
    """Rotary embedding on the last axis: pair (2k, 2k+1) is rotated by
    pos * base**(-2k/d).  `pos` broadcasts against v[..., 0]."""
    d = v.shape[-1]
    assert d % 2 == 0
    k = np.arange(d // 2, dtype=np.float64)
    theta = np.asarray(pos, dtype=np.float64)[..., None] * base ** (-2.0 * k / d)
    cs, sn = np.cos(theta), np.sin(theta)
    out = np.empty(v.shape, dtype=np.float64)
    a, b = v[..., 0::2], v[..., 1::2]
    out[..., 0::2] = a * cs - b * sn
    out[..., 1::2] = a * sn + b * cs
    return out


def sinusoidal_pe(pos: np.ndarray, dim: int, base: float = 10000.0) -> np.ndarray:
    """Sinusoidal positional embedding: [.., 2k] = sin(pos/base^(2k/dim)),
    [.., 2k+1] = cos(same)."""
    assert dim % 2 == 0
    k = np.arange(dim // 2, dtype=np.float64)
    ang = np.asarray(pos, dtype=np.float64)[..., None] / base ** (2.0 * k / dim)
    out = np.empty(ang.shape[:-1] + (dim,), dtype=np.float64)
    out[..., 0::2] = np.sin(ang)
    out[..., 1::2] = np.cos(ang)
    return out


# --------------------------------------------------------------------------
# workload descriptions
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class Workload:
    name: str
    dtype: str                                  # storage: 'f32' | 'bf16'
    batch: int
    d_model: int
    n_heads: int
    d_head: int
    r: int
    d_rope: int
    stride: int
    prefix: Union[int, Tuple[int, int]]         # fixed, or uniform on [lo, hi] inclusive
    steps: int                                  # decode steps after the prefix
    seed: int
    d_hyper: int = 64

    @property
    def max_prefix(self) -> int:
        return self.prefix if isinstance(self.prefix, int) else self.prefix[1]

    @property
    def max_tokens(self) -> int:
        return self.max_prefix + self.steps

    @property
    def max_slots(self) -> int:
        return -(-self.max_tokens // self.stride)

    def scaled(self, **kw) -> "Workload":
        """A copy with some fields replaced (reduced sizes for quick tests)."""
        d = dict(self.__dict__)
        d.update(kw)
        return Workload(**d)


_SEED = 20250513
WORKLOADS: Dict[str, Workload] = {
    # batch 1, 256-token prefix + 64 decode steps, fp32 end to end
    "tiny_f32": Workload("tiny_f32", "f32", 1, 256, 4, 64, 64, 32, 2, 256, 64, _SEED + 0),
    # the paper's decoder shape: the headline configuration
    "speech_bf16": Workload("speech_bf16", "bf16", 16, 512, 8, 64, 256, 32, 2, 1024, 256, _SEED + 1),
    "long_bf16": Workload("long_bf16", "bf16", 8, 4096, 32, 128, 512, 64, 4, 32768, 128, _SEED + 2),
    "ragged_bf16": Workload("ragged_bf16", "bf16", 256, 2048, 16, 128, 512, 64, 2, (512, 4096), 64, _SEED + 3),
    # parallel prefill form, sequence length 4096, no decode steps
    "prefill_s2": Workload("prefill_s2", "bf16", 8, 2048, 16, 128, 512, 64, 2, 4096, 0, _SEED + 4),
    "prefill_s4": Workload("prefill_s4", "bf16", 8, 2048, 16, 128, 512, 64, 4, 4096, 0, _SEED + 4),
    # supplement, not one of the benchmark configurations: the headline's per-sequence shape with the
    # batch scaled until the cache (302 MB) no longer fits the last-level cache, to show what the
    # decode kernel streams at that head / latent shape
    "speech_b1024_bf16": Workload("speech_b1024_bf16", "bf16", 1024, 512, 8, 64, 256, 32, 2, 1024, 16, _SEED + 5),
}


def prefix_lengths(wl: Workload) -> np.ndarray:
    """Per-sequence prefix length, int32[batch]."""
    if isinstance(wl.prefix, int):
        return np.full(wl.batch, wl.prefix, dtype=np.int32)
    lo, hi = wl.prefix
    rng = np.random.default_rng([wl.seed, 0xA11CE])
    return rng.integers(lo, hi + 1, size=wl.batch).astype(np.int32)


# --------------------------------------------------------------------------
# weights
# --------------------------------------------------------------------------
@dataclass
class Weights:
    # generation-side projections (never seen by the library)
    W_Q: np.ndarray      # [d_model, n_heads*d_head]
    W_QR: np.ndarray     # [d_model, n_heads*d_rope]
    W_r: np.ndarray      # [d_model, r]
    W_KR: np.ndarray     # [d_model, d_rope]
    # attention-path weights, storage-rounded, float32
    W_K: np.ndarray      # [r, n_heads*d_head]   keys  = C_hat W_K
    W_V: np.ndarray      # [r, n_heads*d_head]   values = C_hat W_V
    w_uk: np.ndarray     # [n_heads, d_head, r]  w_uk[h,k,n] = W_K[n, h*d_head+k]
    w_uv: np.ndarray     # [n_heads, r, d_head]  w_uv[h,n,k] = W_V[n, h*d_head+k]
    w_uk_lib: np.ndarray  # [n_heads, r, d_head] the library's layout of w_uk (contraction innermost)
    w_uv_lib: np.ndarray  # [n_heads, d_head, r] the library's layout of w_uv
    hyp_A: np.ndarray    # [d_hyper, r]          Linear on the latent c_i
    hyp_B: np.ndarray    # [d_hyper, r]          Linear on the positional embedding
    hyp_G: np.ndarray    # [max_slots, d_hyper]  row j-1 = hyp_B @ pe_j (slot j, 1-based)


def make_weights(wl: Workload, max_slots: Optional[int] = None) -> Weights:
    rng = np.random.default_rng([wl.seed, 0xBEEF])
    d, nh, dh, r, dr, dy = wl.d_model, wl.n_heads, wl.d_head, wl.r, wl.d_rope, wl.d_hyper

    def gauss(fan_in, *shape):
        return rng.standard_normal(shape) / np.sqrt(fan_in)

    W_Q = gauss(d, d, nh * dh)
    W_QR = gauss(d, d, nh * dr)
    W_r = gauss(d, d, r)
    W_KR = gauss(d, d, dr)
    W_K = storage_round(gauss(r, r, nh * dh), wl.dtype)
    W_V = storage_round(gauss(r, r, nh * dh), wl.dtype)
    hyp_A = storage_round(gauss(r, dy, r), wl.dtype)
    hyp_B = gauss(r, dy, r)
    ms = wl.max_slots if max_slots is None else max_slots
    pe = sinusoidal_pe(np.arange(1, ms + 1), r)            # slot index j is 1-based
    hyp_G = storage_round(pe @ hyp_B.T, wl.dtype)
    w_uk = np.ascontiguousarray(W_K.reshape(r, nh, dh).transpose(1, 2, 0))
    w_uv = np.ascontiguousarray(W_V.reshape(r, nh, dh).transpose(1, 0, 2))
    w_uk_lib = np.ascontiguousarray(w_uk.transpose(0, 2, 1))
    w_uv_lib = np.ascontiguousarray(w_uv.transpose(0, 2, 1))
    return Weights(W_Q, W_QR, W_r, W_KR, W_K, W_V, w_uk, w_uv, w_uk_lib, w_uv_lib, hyp_A, hyp_B, hyp_G)


# --------------------------------------------------------------------------
# token streams
# --------------------------------------------------------------------------
@dataclass
class Tokens:
    """Per-token inputs of one sequence for positions [p0, p1) (0-based)."""
    p0: int
    p1: int
    c: np.ndarray                   # [n, r]              LayerNorm(x W_r)
    kr: np.ndarray                  # [n, d_rope]         rotated shared key
    q: Optional[np.ndarray]         # [n, n_heads, d_head]
    q_rope: Optional[np.ndarray]    # [n, n_heads, d_rope] rotated


def _x_block(wl: Workload, b: int, blk: int) -> np.ndarray:
    rng = np.random.default_rng([wl.seed, 0x70CE, b, blk])
    return rng.standard_normal((BLOCK, wl.d_model), dtype=np.float32)


def make_tokens(wl: Workload, wts: Weights, b: int, p0: int, p1: int,
                want_q: bool = True) -> Tokens:
    """Inputs of sequence `b` for token positions p0 <= p < p1.

    x ~ N(0,1) i.i.d.; q = x W_Q; q_rope = RoPE_p(x W_QR); c = LN(x W_r);
    kr = RoPE_p(x W_KR); each rounded once to the storage dtype.  Position p is
    0-based (token i = p+1 in the paper's numbering).
    """
    assert 0 <= p0 <= p1
    n = p1 - p0
    nh, dh, r, dr = wl.n_heads, wl.d_head, wl.r, wl.d_rope
    gen = np.float64 if wl.d_model <= 512 else np.float32
    c = np.empty((n, r), np.float32)
    kr = np.empty((n, dr), np.float32)
    q = np.empty((n, nh, dh), np.float32) if want_q else None
    qr = np.empty((n, nh, dr), np.float32) if want_q else None
    W_r, W_KR = wts.W_r.astype(gen), wts.W_KR.astype(gen)
    if want_q:
        W_Q, W_QR = wts.W_Q.astype(gen), wts.W_QR.astype(gen)
    for blk in range(p0 // BLOCK, -(-p1 // BLOCK) if n else 0):
        lo, hi = max(p0, blk * BLOCK), min(p1, (blk + 1) * BLOCK)
        x = _x_block(wl, b, blk)[lo - blk * BLOCK: hi - blk * BLOCK].astype(gen)
        pos = np.arange(lo, hi)
        o = slice(lo - p0, hi - p0)
        c[o] = storage_round(layer_norm((x @ W_r).astype(np.float64)), wl.dtype)
        kr[o] = storage_round(rope_rotate((x @ W_KR).astype(np.float64), pos), wl.dtype)
        if want_q:
            q[o] = storage_round(x @ W_Q, wl.dtype).reshape(-1, nh, dh)
            qr[o] = storage_round(
                rope_rotate((x @ W_QR).astype(np.float64).reshape(-1, nh, dr), pos[:, None]),
                wl.dtype)
    return Tokens(p0, p1, c, kr, q, qr)


# --------------------------------------------------------------------------
# inputs of the whole-layer call: the token stream itself and the projection weights
# --------------------------------------------------------------------------
@dataclass
class LayerWeights:
    """Projection weights around the attention path, output-major ([out_features, d_model]),
    storage-rounded, float32."""
    w_q: np.ndarray      # [n_heads*d_head, d_model]
    w_qr: np.ndarray     # [n_heads*d_rope, d_model]
    w_r: np.ndarray      # [r, d_model]
    w_kr: np.ndarray     # [d_rope, d_model]
    w_o: np.ndarray      # [d_model, n_heads*d_head]


def make_layer_weights(wl: Workload, wts: Weights) -> LayerWeights:
    """The generation-side projections of `wts`, transposed and rounded to the storage dtype, plus
    an output projection W_O ~ N(0,1)/sqrt(n_heads*d_head)."""
    rnd = lambda a: np.ascontiguousarray(storage_round(np.ascontiguousarray(a.T), wl.dtype))
    rng = np.random.default_rng([wl.seed, 0x0B0E])
    k = wl.n_heads * wl.d_head
    w_o = storage_round(rng.standard_normal((wl.d_model, k)) / np.sqrt(k), wl.dtype)
    return LayerWeights(rnd(wts.W_Q), rnd(wts.W_QR), rnd(wts.W_r), rnd(wts.W_KR), w_o)


def make_x(wl: Workload, b: int, p0: int, p1: int) -> np.ndarray:
    """Token inputs x [p1 - p0, d_model] of sequence `b`, rounded to the storage dtype (the same
    stream make_tokens projects)."""
    out = np.empty((p1 - p0, wl.d_model), np.float32)
    for blk in range(p0 // BLOCK, -(-p1 // BLOCK) if p1 > p0 else 0):
        lo, hi = max(p0, blk * BLOCK), min(p1, (blk + 1) * BLOCK)
        out[lo - p0: hi - p0] = storage_round(_x_block(wl, b, blk)[lo - blk * BLOCK: hi - blk * BLOCK], wl.dtype)
    return out

