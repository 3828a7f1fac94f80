"""Pins for the float64 oracle: every check here compares the oracle with
something other than itself -- values worked out by hand from the paper's
formulas (tests/golden), closed forms, textbook routines written locally, or a
second independent route through the paper's equations (incremental inference
vs. the masked parallel form).  CPU only."""
import math
import os

import numpy as np
import pytest

from oracle import mtla_oracle as O

GOLD = os.path.join(os.path.dirname(__file__), "golden")


# ------------------------------------------------------------------ helpers
def rand_problem(seed, T, n_h=2, d_h=4, r=8, d_rope=4, d_y=6, s=2, bias=True):
    g = np.random.default_rng(seed)
    n_slots = -(-T // s)
    return dict(
        c=g.standard_normal((T, r)), kr=g.standard_normal((T, d_rope)),
        q=g.standard_normal((T, n_h, d_h)), q_rope=g.standard_normal((T, n_h, d_rope)),
        hyp_A=g.standard_normal((d_y, r)) / math.sqrt(r),
        hyp_a=g.standard_normal(d_y) * 0.3 if bias else None,
        hyp_G=g.standard_normal((n_slots, d_y)),
        w_uk=g.standard_normal((n_h, d_h, r)) / math.sqrt(r),
        w_uv=g.standard_normal((n_h, r, d_h)) / math.sqrt(r),
        stride=s, scale=1.0 / math.sqrt(d_h))


def run_incremental(P, w_override=None):
    return O.decode_sequence(P["c"], P["kr"], P["q"], P["q_rope"], P["hyp_A"], P["hyp_a"],
                             P["hyp_G"], P["w_uk"], P["w_uv"], P["stride"], P["scale"],
                             w_override=w_override)


def textbook_attention(q, K, V, scale):
    """softmax(q K^T * scale) V for one query (Preliminaries, first equation)."""
    e = [sum(qi * ki for qi, ki in zip(q, k)) * scale for k in K]
    m = max(e)
    p = [math.exp(x - m) for x in e]
    z = sum(p)
    return [sum(p[k] / z * V[k][d] for k in range(len(K))) for d in range(len(V[0]))]


# ------------------------------------------------- cache length, slot index
@pytest.mark.parametrize("s", [1, 2, 3, 4, 5])
def test_cache_length_is_ceil_T_over_s(s):
    g = np.random.default_rng(s)
    cache = O.LatentCache(3, 2, s)
    for T in range(1, 4 * s + 1):
        slot, is_new = cache.append(g.standard_normal(3), g.standard_normal(2), 0.5)
        assert cache.n_slots == math.ceil(T / s) == O.cache_slots(T, s)
        assert slot == math.ceil(T / s) - 1
        # a slot opens exactly when the 1-based token index leaves remainder 1 (every token for s=1)
        assert is_new == (T % s == 1 or s == 1)


def test_cache_elements_per_token_closed_form():
    # r = 4 d_h, d_h^R = d_h / 2  =>  9 d_h l / (2 s); 2.25 d_h l at s = 2
    for d_h in (32, 64, 128):
        for s in (1, 2, 3, 4):
            for l in (1, 9):
                assert O.cache_elements_per_token(4 * d_h, d_h // 2, s, l) == pytest.approx(9 * d_h * l / (2 * s))
    assert O.cache_elements_per_token(256, 32, 2, 1) == 2.25 * 64
    # the paper's decoder: MHA keeps 2 d_h n_h = 1024 elements per token and layer, MTLA 144 at s=2
    assert 2 * 64 * 8 / O.cache_elements_per_token(256, 32, 2) == pytest.approx(1024 / 144)


# ------------------------------------------------- golden: worked example
def _read_worked_example():
    toks, states = [], {}
    for line in open(os.path.join(GOLD, "worked_example_s2.txt")):
        f = line.split()
        if not f or f[0].startswith("#"):
            continue
        if f[0] == "tok":
            toks.append((float(f[2]), [float(f[3]), float(f[4])]))
        elif f[0] == "state":
            states[int(f[1])] = np.array([float(x) for x in f[2:]]).reshape(-1, 2)
    return toks, states


def test_worked_example_s2_values():
    toks, states = _read_worked_example()
    cache = O.LatentCache(2, 2, 2)
    for i, (w, c) in enumerate(toks, start=1):
        cache.append(np.array(c), np.array([float(i), -float(i)]), w)
        C_hat, KR_hat = cache.arrays()
        assert np.array_equal(C_hat, states[i]), (i, C_hat)
        # RoPE-key slot holds the newest key folded into it
        assert np.array_equal(KR_hat[-1], [float(i), -float(i)])
    assert np.array_equal(cache.arrays()[1], [[2.0, -2.0], [4.0, -4.0]])


# ------------------------------------------------- golden: mask
def _read_masks():
    out, cur = {}, None
    for line in open(os.path.join(GOLD, "stride_aware_mask.txt")):
        f = line.split()
        if not f or f[0].startswith("#"):
            continue
        if f[0] == "mask":
            cur = (int(f[1].split("=")[1]), int(f[2].split("=")[1]))
            out[cur] = []
        else:
            out[cur].append([int(x) for x in f])
    return {k: np.array(v, dtype=bool) for k, v in out.items()}


def test_stride_aware_mask_matches_hand_written_matrices():
    for (s, T), M in _read_masks().items():
        assert M.shape == (T, T)
        assert np.array_equal(O.stride_aware_mask(T, s), M), (s, T)


@pytest.mark.parametrize("s", [1, 2, 3, 4, 5])
def test_mask_row_counts_equal_cache_length(s):
    T = 23
    A = O.stride_aware_mask(T, s)
    for m in range(1, T + 1):                     # 1-based row
        assert A[m - 1].sum() == math.ceil(m / s)
        for n in range(1, T + 1):                 # literal sentence of the paper, 1-based
            assert A[m - 1, n - 1] == ((n == m) or (n < m and n % s == 0))
    if s == 1:
        assert np.array_equal(A, np.tril(np.ones((T, T), bool)))


def test_chunk_mask_is_block_diagonal_lower_triangular():
    T, s = 11, 3
    K = O.chunk_mask(T, s)
    for m in range(1, T + 1):
        for n in range(1, T + 1):
            assert K[m - 1, n - 1] == (math.ceil(n / s) == math.ceil(m / s) and n <= m)


# ------------------------------------------------- hyper-network
def test_merge_weight_special_cases():
    r = 5
    c = np.array([0.3, -1.2, 2.0, 0.0, 0.7])
    eye = np.eye(r)
    for k in range(r):                            # A = I, Linear(pe) = e_k  ->  sigmoid(c_k)
        assert O.merge_weight(c, eye, None, eye[k]) == pytest.approx(1 / (1 + math.exp(-c[k])), abs=1e-15)
    # zero positional branch -> sigmoid(0) = 1/2 whatever c is
    assert O.merge_weight(c, eye, None, np.zeros(r)) == 0.5
    # bias enters Linear(c): A = 0, a = e_0 * 2, g = e_0 * 3 -> sigmoid(6)
    a = np.zeros(r); a[0] = 2.0
    g = np.zeros(r); g[0] = 3.0
    assert O.merge_weight(c, np.zeros((r, r)), a, g) == pytest.approx(1 / (1 + math.exp(-6.0)), abs=1e-15)
    # scalar from two vectors: a dot product, i.e. symmetric under a joint permutation of d_y
    A = np.random.default_rng(0).standard_normal((4, r)); gg = np.array([1.0, -2.0, 0.5, 3.0])
    perm = [2, 0, 3, 1]
    assert O.merge_weight(c, A, None, gg) == pytest.approx(O.merge_weight(c, A[perm], None, gg[perm]), abs=1e-15)
    hand = 1 / (1 + math.exp(-sum(gg[k] * sum(A[k, n] * c[n] for n in range(r)) for k in range(4))))
    assert O.merge_weight(c, A, None, gg) == pytest.approx(hand, abs=1e-14)


def test_weights_in_unit_interval_and_training_matrix_matches_inference():
    P = rand_problem(3, T=13, s=3)
    inc = run_incremental(P)
    assert np.all((inc["w"] > 0) & (inc["w"] < 1))
    W = O.hyper_weight_matrix(P["c"], P["hyp_A"], P["hyp_a"], P["hyp_G"], 3)
    K = O.chunk_mask(13, 3)
    for n in range(13):
        col = W[K[:, n], n]                       # entries of column n kept by the chunk mask
        assert np.allclose(col, inc["w"][n], rtol=0, atol=1e-15)   # constant, and equal to inference w_n


# ------------------------------------------------- attention: closed forms
def test_first_s_tokens_return_the_single_slot():
    for s in (1, 2, 3, 4):
        P = rand_problem(10 + s, T=s, s=s)
        inc = run_incremental(P)
        cache = O.LatentCache(8, 4, s)
        for t in range(s):
            O.append_token(cache, P["c"][t], P["kr"][t], P["hyp_A"], P["hyp_a"], P["hyp_G"])
            if s > 1 or t == 0:
                assert cache.n_slots == 1
                for h in range(2):
                    assert np.allclose(inc["out_latent"][t, h], cache.C[0], atol=1e-15)


@pytest.mark.parametrize("s", [1, 2, 3, 4])
def test_a_complete_slot_depends_on_its_own_tokens_only(s):
    # Two sequences that start with the same P tokens and go on differently: the floor(P/s) slots that the
    # common tokens complete are the same rows in both caches, to the last bit, whatever follows (the update rule after Eq. (infer-linear): a
    # slot sums only its own s tokens, each weighted from its own latent and its slot's row of G).  This is what
    # lets beams read the rows of a common prompt from one stored copy.  The slot the prompt leaves open, and the
    # outputs, do differ.
    P_len, T = 7, 13
    A = rand_problem(40 + s, T=T, s=s)
    g = np.random.default_rng(90 + s)
    B = dict(A)
    B["c"] = np.concatenate([A["c"][:P_len], g.standard_normal((T - P_len, 8))])
    B["kr"] = np.concatenate([A["kr"][:P_len], g.standard_normal((T - P_len, 4))])
    caches = []
    for prob in (A, B):
        cache = O.LatentCache(8, 4, s)
        for t in range(T):
            O.append_token(cache, prob["c"][t], prob["kr"][t], prob["hyp_A"], prob["hyp_a"], prob["hyp_G"])
        caches.append(cache)
    done = P_len // s
    for j in range(done):
        assert np.array_equal(caches[0].C[j], caches[1].C[j]) and np.array_equal(caches[0].KR[j], caches[1].KR[j])
    assert not np.allclose(caches[0].C[done], caches[1].C[done])
    # and a slot is the plain weighted sum of its tokens, written out here without the cache
    for j in range(done):
        acc = np.zeros(8)
        for t in range(j * s, j * s + s):
            z = float((A["hyp_A"] @ A["c"][t] + A["hyp_a"]) @ A["hyp_G"][j])
            acc = acc + 1.0 / (1.0 + math.exp(-z)) * A["c"][t]
        assert np.allclose(caches[0].C[j], acc, rtol=0, atol=1e-14)
        assert np.array_equal(caches[0].KR[j], A["kr"][j * s + s - 1])


def test_softmax_rows_sum_to_one_and_output_in_hull():
    P = rand_problem(5, T=12, s=3)
    cache = O.LatentCache(8, 4, 3)
    for t in range(12):
        O.append_token(cache, P["c"][t], P["kr"][t], P["hyp_A"], P["hyp_a"], P["hyp_G"])
        out, lat, lse, probs = O.decode_attn(cache, P["q"][t], P["q_rope"][t], P["w_uk"], P["w_uv"], P["scale"])
        assert probs.shape == (2, math.ceil((t + 1) / 3))
        assert np.allclose(probs.sum(axis=1), 1.0, atol=1e-14)
        C_hat, _ = cache.arrays()
        assert np.all(lat <= C_hat.max(axis=0) + 1e-12) and np.all(lat >= C_hat.min(axis=0) - 1e-12)


def test_rope_key_slot_holds_latest_token():
    for s in (1, 2, 3, 4):
        for T in range(1, 3 * s + 2):
            cache = O.LatentCache(2, 3, s)
            for i in range(1, T + 1):
                cache.append(np.zeros(2), np.full(3, float(i)), 1.0)
            _, KR_hat = cache.arrays()
            for j in range(1, cache.n_slots + 1):
                assert np.all(KR_hat[j - 1] == min(j * s, T))


# ------------------------------------------------- MLA reduction + explicit form
def explicit_attention_per_head(P, C_hat, KR_hat, q, q_rope):
    """Keys and values written out: K = C_hat W_K, V = C_hat W_V per head, the
    shared RoPE key appended to every head's key, one textbook softmax each."""
    n_h, d_h, r = P["w_uk"].shape
    outs = []
    for h in range(n_h):
        W_K_h = P["w_uk"][h].T                    # [r, d_h]
        W_V_h = P["w_uv"][h]                      # [r, d_h]
        K = [list(C_hat[k] @ W_K_h) + list(KR_hat[k]) for k in range(len(C_hat))]
        V = [list(C_hat[k] @ W_V_h) for k in range(len(C_hat))]
        outs.append(textbook_attention(list(q[h]) + list(q_rope[h]), K, V, P["scale"]))
    return np.array(outs)


def test_s1_unit_weights_reduce_to_mla_causal_attention():
    T = 9
    P = rand_problem(7, T=T, s=1)
    inc = run_incremental(P, w_override=np.ones(T))
    for t in range(T):                            # MLA: cache is C itself, ordinary causal attention
        ref = explicit_attention_per_head(P, P["c"][:t + 1], P["kr"][:t + 1], P["q"][t], P["q_rope"][t])
        assert np.allclose(inc["out"][t], ref, atol=1e-12)
    assert inc["cache"].n_slots == T
    assert np.allclose(inc["cache"].arrays()[0], P["c"], atol=0)


@pytest.mark.parametrize("s", [2, 3, 4])
def test_absorbed_equals_explicit_keys_and_values(s):
    T = 11
    P = rand_problem(20 + s, T=T, s=s)
    cache = O.LatentCache(8, 4, s)
    for t in range(T):
        O.append_token(cache, P["c"][t], P["kr"][t], P["hyp_A"], P["hyp_a"], P["hyp_G"])
        out, _, _, _ = O.decode_attn(cache, P["q"][t], P["q_rope"][t], P["w_uk"], P["w_uv"], P["scale"])
        C_hat, KR_hat = cache.arrays()
        ref = explicit_attention_per_head(P, C_hat, KR_hat, P["q"][t], P["q_rope"][t])
        assert np.allclose(out, ref, atol=1e-12)


def test_lse_is_log_of_the_normaliser():
    P = rand_problem(31, T=7, s=2)
    cache = O.LatentCache(8, 4, 2)
    for t in range(7):
        O.append_token(cache, P["c"][t], P["kr"][t], P["hyp_A"], P["hyp_a"], P["hyp_G"])
    _, _, lse, _ = O.decode_attn(cache, P["q"][6], P["q_rope"][6], P["w_uk"], P["w_uv"], P["scale"])
    C_hat, KR_hat = cache.arrays()
    for h in range(2):
        qt = P["w_uk"][h].T @ P["q"][6, h]
        z = sum(math.exp((C_hat[k] @ qt + KR_hat[k] @ P["q_rope"][6, h]) * P["scale"]) for k in range(4))
        assert lse[h] == pytest.approx(math.log(z), abs=1e-12)


# ------------------------------------------------- incremental == parallel (brute force)
def brute_force_parallel(P, T, s):
    """Training form with everything materialised, in plain loops and the
    paper's 1-based indices: PE replicated s times, W = sigmoid(Lin(PE) Lin(C)^T),
    chunk mask, C_hat' = W C, T x T logits with the uncompressed K^R, mask,
    softmax, explicit values."""
    n_h, d_h, r = P["w_uk"].shape
    lin_c = [P["hyp_A"] @ P["c"][n] + (P["hyp_a"] if P["hyp_a"] is not None else 0) for n in range(T)]
    Cp = np.zeros((T, r))
    for m in range(1, T + 1):
        jm = math.ceil(m / s)
        for n in range(1, T + 1):
            if math.ceil(n / s) == jm and n <= m:
                W_mn = 1 / (1 + math.exp(-float(P["hyp_G"][jm - 1] @ lin_c[n - 1])))
                Cp[m - 1] += W_mn * P["c"][n - 1]
    out = np.zeros((T, n_h, d_h))
    for h in range(n_h):
        K = Cp @ P["w_uk"][h].T
        V = Cp @ P["w_uv"][h]
        for m in range(1, T + 1):
            cols = [n for n in range(1, T + 1) if n == m or (n < m and n % s == 0)]
            Kc = [list(K[n - 1]) + list(P["kr"][n - 1]) for n in cols]
            Vc = [list(V[n - 1]) for n in cols]
            out[m - 1, h] = textbook_attention(list(P["q"][m - 1, h]) + list(P["q_rope"][m - 1, h]), Kc, Vc, P["scale"])
    return out, Cp


@pytest.mark.parametrize("s", [1, 2, 3, 4])
@pytest.mark.parametrize("T", [1, 5, 12, 13])
def test_incremental_equals_masked_parallel_equals_brute_force(s, T):
    P = rand_problem(100 * s + T, T=T, s=s)
    inc = run_incremental(P)
    out, lat, lse, Cp = O.prefill_attn(P["q"], P["q_rope"], P["c"], P["kr"], P["w_uk"], P["w_uv"], s, P["scale"],
                                       hyp_A=P["hyp_A"], hyp_a=P["hyp_a"], hyp_G=P["hyp_G"])
    bf_out, bf_Cp = brute_force_parallel(P, T, s)
    assert np.allclose(inc["out"], out, atol=1e-12)
    assert np.allclose(inc["out_latent"], lat, atol=1e-12)
    assert np.allclose(inc["lse"], lse, atol=1e-12)
    assert np.allclose(out, bf_out, atol=1e-12)
    assert np.allclose(Cp, bf_Cp, atol=1e-13)
    # final slot states of the cache are rows s, 2s, ... (and the last row) of C_hat'
    C_hat, KR_hat = inc["cache"].arrays()
    last_rows = [min(j * s, T) - 1 for j in range(1, math.ceil(T / s) + 1)]
    assert np.allclose(C_hat, Cp[last_rows], atol=1e-13)
    assert np.array_equal(KR_hat, P["kr"][last_rows])


def test_parallel_form_with_given_weights_and_row_subset():
    T, s = 13, 3
    P = rand_problem(77, T=T, s=s)
    inc = run_incremental(P)
    rows = [0, 4, 5, 12]
    out, lat, lse, _ = O.prefill_attn(P["q"], P["q_rope"], P["c"], P["kr"], P["w_uk"], P["w_uv"], s, P["scale"],
                                      w=inc["w"], rows=rows)
    assert np.allclose(out, inc["out"][rows], atol=1e-12)
    assert np.allclose(lat, inc["out_latent"][rows], atol=1e-12)
    assert np.allclose(lse, inc["lse"][rows], atol=1e-12)


# ------------------------------------------------- the pins bite: planted mistakes are caught
def _parallel_vs_incremental_gap(P, T, s):
    inc = run_incremental(P)
    out, _, _, _ = O.prefill_attn(P["q"], P["q_rope"], P["c"], P["kr"], P["w_uk"], P["w_uv"], s, P["scale"],
                                  hyp_A=P["hyp_A"], hyp_a=P["hyp_a"], hyp_G=P["hyp_G"])
    return np.abs(inc["out"] - out).max()


def test_planted_mistakes_are_detected(monkeypatch):
    T, s = 12, 3
    P = rand_problem(5, T=T, s=s)
    assert _parallel_vs_incremental_gap(P, T, s) < 1e-12
    # ordinary causal mask instead of the stride-aware one
    with monkeypatch.context() as mp:
        mp.setattr(O, "stride_aware_mask", lambda T, s: np.tril(np.ones((T, T), bool)))
        assert _parallel_vs_incremental_gap(P, T, s) > 1e-3
    # off-by-one in the mask's "n mod s == 0" (0-based n instead of 1-based)
    with monkeypatch.context() as mp:
        mp.setattr(O, "stride_aware_mask",
                   lambda T, s: (np.arange(T)[None] == np.arange(T)[:, None])
                   | ((np.arange(T)[None] < np.arange(T)[:, None]) & (np.arange(T)[None] % s == 0)))
        assert _parallel_vs_incremental_gap(P, T, s) > 1e-3
    # streaming-encoder style chunk mask that also lets later in-chunk tokens through
    with monkeypatch.context() as mp:
        mp.setattr(O, "chunk_mask", lambda T, s: np.arange(T)[:, None] // s == np.arange(T)[None] // s)
        assert _parallel_vs_incremental_gap(P, T, s) > 1e-3
    # RoPE key averaged instead of overwritten
    with monkeypatch.context() as mp:
        orig = O.LatentCache.append

        def bad(self, c, kr, w):
            slot, is_new = orig(self, c, kr, w)
            if not is_new:
                self.KR[slot] = 0.5 * self.KR[slot]
            return slot, is_new
        mp.setattr(O.LatentCache, "append", bad)
        assert _parallel_vs_incremental_gap(P, T, s) > 1e-3
    # wrong softmax scale (sqrt(d_h + d_rope)) breaks the explicit-form pin
    P2 = rand_problem(6, T=6, s=2)
    cache = O.LatentCache(8, 4, 2)
    for t in range(6):
        O.append_token(cache, P2["c"][t], P2["kr"][t], P2["hyp_A"], P2["hyp_a"], P2["hyp_G"])
    C_hat, KR_hat = cache.arrays()
    good = explicit_attention_per_head(P2, C_hat, KR_hat, P2["q"][5], P2["q_rope"][5])
    bad_out, _, _, _ = O.decode_attn(cache, P2["q"][5], P2["q_rope"][5], P2["w_uk"], P2["w_uv"], 1 / math.sqrt(8))
    assert np.abs(bad_out - good).max() > 1e-3
    assert O.softmax_scale(4) == 0.5 and O.softmax_scale(64) == 0.125
