"""Float64 CPU oracle for Multi-head Temporal Latent Attention (MTLA).

TEST INFRASTRUCTURE ONLY.  This module is the reference the HIP library is
checked against.  It may be imported by the tests, by the smoke check and by
the benchmark's CPU-baseline leg, never by the product path, and it shares no
code with the HIP kernels.  It is written for legibility, not speed: every
function follows one passage of the paper (arxiv 2505.13544) in the paper's
own order, in float64, with numpy matmuls as the only library steps.

Index conventions.  The paper counts tokens i = 1, 2, ... and slots
j = ceil(i/s).  Arrays here are 0-based: token position p = i-1 lives in slot
index p // s, and a new slot opens when p % s == 0 (the paper's condition that
i leaves the remainder 1 when divided by s, which for s = 1 is read as: every
token opens a slot).

Readings of the paper taken here (all are pinned by tests):
  * Eq. (infer-linear): the merge weight is a scalar, so the product of the
    two 64-vectors is a dot product, as the matrix product of Eq.
    (train-linear) implies.
  * Eq. (train-linear): W[m, n] = sigmoid(<Linear(pe_{ceil(m/s)}), Linear(c_n)>).
  * "Chunk masking": W[m, n] is kept iff n is in the same chunk of s as m and
    n <= m, so that row m of C_hat' is the temporary slot state that step m of
    incremental inference sees.
  * Eq. (with-rope): the logits are divided by sqrt(d_h) only.
  * Per head h: q_tilde = W_K^(h) q^(h), out^(h) = o_latent^(h) W_V^(h); the
    output projection W_O belongs to the layer functions at the end of the file.
  * The layer around the path (Eqs. (query), (low-rank), (softmax); Section
    "Decoupled Rotary Position Embedding in MTLA"): the RoPE queries come from
    a projection of their own, W_QR [n_h d_R, d] (the rotated vectors are d_R
    wide, Eq. (query)'s are d_h wide); the shared RoPE key is k^R = RoPE(x W_KR)
    of the un-merged token stream; rotation pairs are (2k, 2k+1), angle
    pos * base^(-2k/d_R), base 10000, pos = i - 1; LayerNorm acts on c = x W_r
    before the hyper-network and the cache see it (eps 1e-5, optional affine).

Parity status: every function below is pinned (tests/test_oracle_pins.py).
"""
from __future__ import annotations

import math
from typing import List, Optional, Sequence, Tuple

import numpy as np

F = np.float64


def sigmoid(z):
    return 1.0 / (1.0 + np.exp(-np.asarray(z, dtype=F)))


# ---------------------------------------------------------------------------
# Section "Inference using MTLA": hyper-network, cache update, attention
# ---------------------------------------------------------------------------
def merge_weight(c, hyp_A, hyp_a, g_row) -> float:
    """Eq. (infer-linear): w_i = sigmoid(<Linear(c_i), Linear(pe_j)>).

    c      [r]         post-LayerNorm latent of token i
    hyp_A  [d_y, r]    weight of Linear(c); hyp_a [d_y] its bias or None
    g_row  [d_y]       Linear(pe_j) for the token's slot j = ceil(i/s)
    """
    y = np.asarray(hyp_A, F) @ np.asarray(c, F)
    if hyp_a is not None:
        y = y + np.asarray(hyp_a, F)
    return float(sigmoid(y @ np.asarray(g_row, F)))


class LatentCache:
    """Compressed temporal-latent cache of ONE sequence (C_hat, K_hat^R, i)."""

    def __init__(self, r: int, d_rope: int, stride: int):
        assert stride >= 1
        self.r, self.d_rope, self.s = r, d_rope, stride
        self.C: List[np.ndarray] = []     # slots of C_hat, each [r]
        self.KR: List[np.ndarray] = []    # slots of K_hat^R, each [d_rope]
        self.i = 0                        # tokens seen

    def append(self, c, kr, w: float) -> Tuple[int, bool]:
        """Cache update rule of Section "Inference using MTLA" and its RoPE-key
        counterpart in Section "Decoupled Rotary Position Embedding".
        Returns (0-based slot index the token went to, whether it opened it)."""
        c, kr = np.asarray(c, F), np.asarray(kr, F)
        self.i += 1
        j = -(-self.i // self.s)                    # ceil(i/s), 1-based slot
        is_new = (self.i - 1) % self.s == 0
        if is_new:
            self.C.append(w * c)                    # C_hat = Concat(C_hat, w_i c_i)
            self.KR.append(kr.copy())               # K_hat^R = Concat(K_hat^R, k^R_i)
        else:
            self.C[j - 1] = self.C[j - 1] + w * c   # c_hat_j += w_i c_i
            self.KR[j - 1] = kr.copy()              # k_hat^R_j = k^R_i
        assert len(self.C) == j == len(self.KR)
        return j - 1, is_new

    @property
    def n_slots(self) -> int:
        return len(self.C)

    def arrays(self) -> Tuple[np.ndarray, np.ndarray]:
        return (np.stack(self.C) if self.C else np.zeros((0, self.r)),
                np.stack(self.KR) if self.KR else np.zeros((0, self.d_rope)))


def append_token(cache: LatentCache, c, kr, hyp_A, hyp_a, hyp_G,
                 w_override: Optional[float] = None):
    """One token through the hyper-network and the update rule.
    hyp_G [max_slots, d_y]: row j-1 holds Linear(pe_j).
    Returns (w, slot, is_new)."""
    j0 = cache.i // cache.s                         # 0-based slot of token i = cache.i + 1
    w = merge_weight(c, hyp_A, hyp_a, hyp_G[j0]) if w_override is None else float(w_override)
    slot, is_new = cache.append(c, kr, w)
    assert slot == j0
    return w, slot, is_new


def softmax_scale(d_head: int) -> float:
    """Eq. (with-rope): logits are divided by sqrt(d_h)."""
    return 1.0 / math.sqrt(d_head)


def decode_attn(cache: LatentCache, q, q_rope, w_uk, w_uv, scale: float):
    """Eq. (with-rope) for one new query against the live cache, per head.

    q [n_h, d_h]; q_rope [n_h, d_rope] (rotated); w_uk [n_h, d_h, r] holds the
    per-head W_K^(h) transposed; w_uv [n_h, r, d_h] holds the per-head W_V^(h).
    Returns out [n_h, d_h], out_latent [n_h, r], lse [n_h], probs [n_h, slots].
    """
    C_hat, KR_hat = cache.arrays()
    q, q_rope = np.asarray(q, F), np.asarray(q_rope, F)
    n_h = q.shape[0]
    out = np.zeros((n_h, np.asarray(w_uv).shape[2]), F)
    out_lat = np.zeros((n_h, cache.r), F)
    lse = np.zeros(n_h, F)
    probs = np.zeros((n_h, cache.n_slots), F)
    for h in range(n_h):
        q_tilde = q[h] @ np.asarray(w_uk[h], F)             # W_K absorbed into the query: [r]
        e = (C_hat @ q_tilde + KR_hat @ q_rope[h]) * scale  # logits over the slots
        m = e.max()
        p = np.exp(e - m)
        z = p.sum()
        p = p / z
        probs[h] = p
        lse[h] = m + math.log(z)
        out_lat[h] = p @ C_hat                              # softmax(.) C_hat
        out[h] = out_lat[h] @ np.asarray(w_uv[h], F)        # ... W_V (W_O is outside)
    return out, out_lat, lse, probs


def decode_sequence(c, kr, q, q_rope, hyp_A, hyp_a, hyp_G, w_uk, w_uv, stride: int,
                    scale: float, w_override: Optional[Sequence[float]] = None,
                    cache: Optional[LatentCache] = None):
    """Token-by-token inference over a whole sequence: update, then attend.
    Returns dict with per-token out, out_latent, lse, w, slot, is_new, n_slots
    and the final cache."""
    T = len(c)
    cache = cache or LatentCache(np.asarray(c).shape[1], np.asarray(kr).shape[1], stride)
    res = dict(out=[], out_latent=[], lse=[], w=[], slot=[], is_new=[], n_slots=[])
    for t in range(T):
        w, slot, is_new = append_token(cache, c[t], kr[t], hyp_A, hyp_a, hyp_G,
                                       None if w_override is None else w_override[t])
        o, ol, l, _ = decode_attn(cache, q[t], q_rope[t], w_uk, w_uv, scale)
        for k, v in zip(("out", "out_latent", "lse", "w", "slot", "is_new", "n_slots"),
                        (o, ol, l, w, slot, is_new, cache.n_slots)):
            res[k].append(v)
    res = {k: np.asarray(v) for k, v in res.items()}
    res["cache"] = cache
    return res


# ---------------------------------------------------------------------------
# Section "MTLA Training with Stride-aware Causal Mask": the parallel form
# ---------------------------------------------------------------------------
def hyper_weight_matrix(C, hyp_A, hyp_a, hyp_G, stride: int) -> np.ndarray:
    """Eq. (train-linear): W = sigmoid(Linear(PE) x Linear(C)^T), [T, T].
    PE repeats pe_j s times, so row m (0-based) uses hyp_G[m // s]."""
    C = np.asarray(C, F)
    T = C.shape[0]
    lin_c = C @ np.asarray(hyp_A, F).T                      # [T, d_y]
    if hyp_a is not None:
        lin_c = lin_c + np.asarray(hyp_a, F)
    lin_pe = np.asarray(hyp_G, F)[np.arange(T) // stride]   # [T, d_y], replicated
    return sigmoid(lin_pe @ lin_c.T)


def chunk_mask(T: int, stride: int) -> np.ndarray:
    """Keep W[m, n] iff n lies in m's chunk of `stride` tokens and n <= m."""
    m = np.arange(T)[:, None]
    n = np.arange(T)[None, :]
    return (m // stride == n // stride) & (n <= m)


def stride_aware_mask(T: int, stride: int) -> np.ndarray:
    """Allowed[m, n] of the stride-aware causal mask.  In the paper's 1-based
    indices: n == m, or n < m and n mod s == 0.  0-based: column n is 1-based
    n+1."""
    m = np.arange(T)[:, None]
    n = np.arange(T)[None, :]
    return (n == m) | ((n < m) & ((n + 1) % stride == 0))


def partial_states(C, W_masked) -> np.ndarray:
    """C_hat' = W C: the length-T sequence of temporary/final slot states."""
    return np.asarray(W_masked, F) @ np.asarray(C, F)


def prefill_attn(q, q_rope, C, KR, w_uk, w_uv, stride: int, scale: float,
                 hyp_A=None, hyp_a=None, hyp_G=None,
                 w: Optional[np.ndarray] = None, rows: Optional[Sequence[int]] = None):
    """Parallel (training/prefill) form for one sequence.

    q [T, n_h, d_h], q_rope [T, n_h, d_rope], C [T, r], KR [T, d_rope].
    Merge weights come from the hyper-network (hyp_*), or, if `w` [T] is
    given, W[m, n] = w[n] (the in-chunk columns of W do not depend on m).
    `rows` restricts the queries evaluated (C_hat' is always built in full).
    Returns out [R, n_h, d_h], out_latent [R, n_h, r], lse [R, n_h],
    C_hat' [T, r].
    """
    q, q_rope, C, KR = (np.asarray(a, F) for a in (q, q_rope, C, KR))
    T = C.shape[0]
    if w is None:
        W = hyper_weight_matrix(C, hyp_A, hyp_a, hyp_G, stride)
    else:
        W = np.broadcast_to(np.asarray(w, F)[None, :], (T, T))
    C_prime = partial_states(C, np.where(chunk_mask(T, stride), W, 0.0))
    allowed = stride_aware_mask(T, stride)
    rows = np.arange(T) if rows is None else np.asarray(rows)
    n_h = q.shape[1]
    out = np.zeros((len(rows), n_h, np.asarray(w_uv).shape[2]), F)
    out_lat = np.zeros((len(rows), n_h, C.shape[1]), F)
    lse = np.zeros((len(rows), n_h), F)
    for h in range(n_h):
        q_tilde = q[rows, h] @ np.asarray(w_uk[h], F)                 # [R, r]
        e = (q_tilde @ C_prime.T + q_rope[rows, h] @ KR.T) * scale    # [R, T]
        e = np.where(allowed[rows], e, -np.inf)
        m = e.max(axis=1, keepdims=True)
        p = np.exp(e - m)
        z = p.sum(axis=1, keepdims=True)
        p = p / z
        lse[:, h] = (m + np.log(z))[:, 0]
        out_lat[:, h] = p @ C_prime
        out[:, h] = out_lat[:, h] @ np.asarray(w_uv[h], F)
    return out, out_lat, lse, C_prime


# ---------------------------------------------------------------------------
# Closed forms stated by the paper
# ---------------------------------------------------------------------------
def cache_slots(T: int, stride: int) -> int:
    """t = ceil(T / s)."""
    return -(-T // stride)


def cache_elements_per_token(r: int, d_rope: int, stride: int, layers: int = 1) -> float:
    """Average KV-cache elements per token: (r + d_h^R) l / s."""
    return (r + d_rope) * layers / stride


# ---------------------------------------------------------------------------
# The layer around the path: Eqs. (query), (low-rank), (softmax)'s W_O, and the
# decoupled RoPE of Section "Decoupled Rotary Position Embedding in MTLA".
# Weights are given output-major, [out_features, in_features].
# ---------------------------------------------------------------------------
def layer_norm(v, eps: float = 1e-5, gamma=None, beta=None) -> np.ndarray:
    """Layer normalisation of one vector (the one applied to C = X W_r)."""
    v = np.asarray(v, F)
    mean = v.sum() / v.size
    var = ((v - mean) ** 2).sum() / v.size
    y = (v - mean) / math.sqrt(var + eps)
    if gamma is not None:
        y = y * np.asarray(gamma, F)
    if beta is not None:
        y = y + np.asarray(beta, F)
    return y


def rope(v, pos: int, base: float = 10000.0) -> np.ndarray:
    """Rotary position embedding of one vector at position pos: the pair
    (v[2k], v[2k+1]) is turned by the angle pos * base^(-2k/d)."""
    v = np.asarray(v, F)
    d = v.shape[-1]
    out = np.empty_like(v)
    for k in range(d // 2):
        ang = pos * base ** (-2.0 * k / d)
        cs, sn = math.cos(ang), math.sin(ang)
        out[..., 2 * k] = v[..., 2 * k] * cs - v[..., 2 * k + 1] * sn
        out[..., 2 * k + 1] = v[..., 2 * k] * sn + v[..., 2 * k + 1] * cs
    return out


def layer_front(x, pos: int, w_q, w_qr, w_r, w_kr, n_heads: int, ln_eps: float = 1e-5,
                rope_base: float = 10000.0, ln_gamma=None, ln_beta=None):
    """x [d] at 0-based position pos -> q [n_h, d_h] (Eq. (query)), q_rope
    [n_h, d_R] (rotated), c [r] = LayerNorm(x W_r) (Eq. (low-rank)), kr [d_R]
    (rotated, one head shared by all query heads)."""
    x = np.asarray(x, F)
    q = (np.asarray(w_q, F) @ x).reshape(n_heads, -1)
    q_rope = rope((np.asarray(w_qr, F) @ x).reshape(n_heads, -1), pos, rope_base)
    c = layer_norm(np.asarray(w_r, F) @ x, ln_eps, ln_gamma, ln_beta)
    kr = rope(np.asarray(w_kr, F) @ x, pos, rope_base)
    return q, q_rope, c, kr


def layer_decode_step(cache: LatentCache, x, w_q, w_qr, w_r, w_kr, w_o, hyp_A, hyp_a, hyp_G, w_uk, w_uv,
                      scale: float, ln_eps: float = 1e-5, rope_base: float = 10000.0, ln_gamma=None, ln_beta=None):
    """One token through one MTLA attention layer: projections, cache update,
    attention over the cache (Eq. (with-rope)), output projection W_O
    [d, n_h d_h] (Eq. (softmax)).  Returns (y [d], out [n_h, d_h], w, slot)."""
    n_heads = np.asarray(w_uk).shape[0]
    pos = cache.i                                    # the new token is number i = cache.i + 1
    q, q_rope, c, kr = layer_front(x, pos, w_q, w_qr, w_r, w_kr, n_heads, ln_eps, rope_base, ln_gamma, ln_beta)
    w, slot, _ = append_token(cache, c, kr, hyp_A, hyp_a, hyp_G)
    out, _, _, _ = decode_attn(cache, q, q_rope, w_uk, w_uv, scale)
    y = np.asarray(w_o, F) @ out.reshape(-1)
    return y, out, w, slot



def layer_prefill(x, w_q, w_qr, w_r, w_kr, w_o, hyp_A, hyp_a, hyp_G, w_uk, w_uv, stride: int, scale: float,
                  ln_eps: float = 1e-5, rope_base: float = 10000.0, ln_gamma=None, ln_beta=None,
                  rows: Optional[Sequence[int]] = None):
    """A whole sequence x [T, d] through one MTLA attention layer in the parallel
    form: Q = X W_Q (Eq. (query)), C = LayerNorm(X W_r) (Eq. (low-rank)), the
    rotated Q^R and K^R with row m at position m (Section "Decoupled Rotary
    Position Embedding in MTLA"), attention under the stride-aware causal mask
    on C_hat' and the uncompressed K^R (last paragraph of that section), and
    Y = concat_h(O_h) W_O (Eq. (softmax)).  `rows` restricts the rows of Y that
    are evaluated.  Returns (y [R, d], out [R, n_h, d_h])."""
    x = np.asarray(x, F)
    T = x.shape[0]
    n_heads = np.asarray(w_uk).shape[0]
    Q = (x @ np.asarray(w_q, F).T).reshape(T, n_heads, -1)
    QR_raw = (x @ np.asarray(w_qr, F).T).reshape(T, n_heads, -1)
    KR_raw = x @ np.asarray(w_kr, F).T
    C_raw = x @ np.asarray(w_r, F).T
    QR = np.stack([rope(QR_raw[m], m, rope_base) for m in range(T)])
    KR = np.stack([rope(KR_raw[m], m, rope_base) for m in range(T)])
    C = np.stack([layer_norm(C_raw[m], ln_eps, ln_gamma, ln_beta) for m in range(T)])
    out, _, _, _ = prefill_attn(Q, QR, C, KR, w_uk, w_uv, stride, scale, hyp_A=hyp_A, hyp_a=hyp_a, hyp_G=hyp_G,
                                rows=rows)
    y = out.reshape(out.shape[0], -1) @ np.asarray(w_o, F).T
    return y, out
