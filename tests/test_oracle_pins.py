"""Pins of the fp64 oracle to things other than itself (CPU only).

The paper prints no worked numeric example of attention, so the oracle is
pinned by: a dense brute force that materialises the literal mask matrix B of
Eq. 8, torch's CPU library routines (scaled_dot_product_attention, rms_norm,
silu), closed forms, locality/causality invariants, the GQA replication
invariant, the early-exit and prefix invariants of the stack (Fig. 3), and the
cache-size numbers the paper does print (tests/golden/kv_cache_tokens_per_gb.txt).
"""
import math
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle
import yoco_synth as ys

HERE = os.path.dirname(os.path.abspath(__file__))


def rand_qkv(seed, T, Hq, Hkv, d):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((T, Hq, d)), rng.standard_normal((T, Hkv, d)),
            rng.standard_normal((T, Hkv, d)))


def brute_force(Q, K, V, mask_fn, scale):
    """Dense T x N scores, the literal additive mask matrix with -inf, row
    softmax, product. Written independently of the oracle (element loops for
    the mask, no max subtraction: tiny inputs only)."""
    Tq, Hq, d = Q.shape
    N, Hkv, _ = K.shape
    G = Hq // Hkv
    O = np.zeros((Tq, Hq, d))
    for h in range(Hq):
        S = np.zeros((Tq, N))
        for i in range(Tq):
            for j in range(N):
                S[i, j] = scale * sum(Q[i, h, e] * K[j, h // G, e] for e in range(d))
                S[i, j] += 0.0 if mask_fn(i, j) else -np.inf
        E = np.exp(S)
        P = E / E.sum(axis=1, keepdims=True)
        for i in range(Tq):
            for e in range(d):
                O[i, h, e] = sum(P[i, j] * V[j, h // G, e] for j in range(N))
    return O


# ------------------------------------------------------------------ SWA (Eq. 8)
@pytest.mark.parametrize("T,C", [(16, 4), (13, 1), (12, 12), (9, 50), (16, 5)])
def test_swa_matches_brute_force_with_literal_mask(T, C):
    Q, K, V = rand_qkv(1, T, 2, 2, 8)
    ref = brute_force(Q, K, V, lambda i, j: i - C < j <= i, 0.37)
    assert np.abs(oracle.swa(Q, K, V, C, 0.37) - ref).max() < 1e-12


def test_swa_gqa_matches_brute_force():
    Q, K, V = rand_qkv(2, 10, 6, 2, 4)
    ref = brute_force(Q, K, V, lambda i, j: i - 3 < j <= i, 0.5)
    assert np.abs(oracle.swa(Q, K, V, 3, 0.5) - ref).max() < 1e-12


def sdpa(Q, K, V, mask, scale):
    """torch CPU library attention in float64; Q [Tq,Hq,d], K/V [N,Hkv,d]."""
    G = Q.shape[1] // K.shape[1]
    q = torch.from_numpy(Q).permute(1, 0, 2)[None]
    k = torch.from_numpy(K).permute(1, 0, 2).repeat_interleave(G, dim=0)[None]
    v = torch.from_numpy(V).permute(1, 0, 2).repeat_interleave(G, dim=0)[None]
    o = F.scaled_dot_product_attention(q, k, v, attn_mask=torch.from_numpy(mask), scale=scale)
    return o[0].permute(1, 0, 2).numpy()


def test_swa_matches_library_attention_with_band_mask():
    T, C, d = 96, 17, 16
    Q, K, V = rand_qkv(3, T, 4, 2, d)
    i, j = np.arange(T)[:, None], np.arange(T)[None, :]
    band = (j <= i) & (j > i - C)
    ref = sdpa(Q, K, V, band, 1 / np.sqrt(d))
    assert np.abs(oracle.swa(Q, K, V, C, 1 / np.sqrt(d)) - ref).max() < 1e-12


@pytest.mark.parametrize("C", [64, 65, 1000])
def test_swa_window_at_least_T_is_full_causal_attention(C):
    T, d = 64, 8
    Q, K, V = rand_qkv(4, T, 2, 2, d)
    q = torch.from_numpy(Q).permute(1, 0, 2)[None]
    k = torch.from_numpy(K).permute(1, 0, 2)[None]
    v = torch.from_numpy(V).permute(1, 0, 2)[None]
    ref = F.scaled_dot_product_attention(q, k, v, is_causal=True)[0].permute(1, 0, 2).numpy()
    assert np.abs(oracle.swa(Q, K, V, C, 1 / np.sqrt(d)) - ref).max() < 1e-12


def test_swa_window_one_returns_v():
    Q, K, V = rand_qkv(5, 20, 3, 3, 8)
    assert np.array_equal(oracle.swa(Q, K, V, 1, 0.3), V)


def test_swa_equal_keys_gives_running_mean_of_v():
    T, C = 40, 7
    Q, K, V = rand_qkv(6, T, 2, 1, 8)
    K[:] = K[0]
    O = oracle.swa(Q, K, V, C, 0.9)
    for i in range(T):
        mean = V[max(0, i - C + 1):i + 1, 0].mean(axis=0)
        assert np.abs(O[i] - mean).max() < 1e-13


def test_swa_constant_v_and_key_count():
    T, C = 30, 6
    Q, K, V = rand_qkv(7, T, 2, 2, 4)
    V[:] = 1.0        # output = sum of the row's probabilities = 1
    assert np.abs(oracle.swa(Q, K, V, C, 1.0) - 1.0).max() < 1e-14
    # one-hot V columns expose the weights: row i has exactly min(i+1, C) non-zeros
    Vh = np.zeros((T, 1, T))
    Vh[np.arange(T), 0, np.arange(T)] = 1.0
    W = oracle.swa(Q[:, :1], K[:, :1], Vh, C, 1.0)[:, 0]     # [T, T] = the probabilities
    for i in range(T):
        nz = np.nonzero(W[i])[0]
        assert len(nz) == min(i + 1, C) and nz.min() == max(0, i - C + 1) and nz.max() == i
    assert np.abs(W.sum(axis=1) - 1).max() < 1e-14


def test_swa_locality():
    T, C, j = 50, 8, 20
    Q, K, V = rand_qkv(8, T, 2, 2, 4)
    O0 = oracle.swa(Q, K, V, C, 0.5)
    K2, V2 = K.copy(), V.copy()
    K2[j] += 1.0
    V2[j] -= 2.0
    changed = np.nonzero(np.abs(oracle.swa(Q, K2, V2, C, 0.5) - O0).max(axis=(1, 2)) > 0)[0]
    assert changed.tolist() == list(range(j, j + C))


def test_swa_scale_matters_and_sign():
    # a transposed operand, dropped scale or flipped sign would fail here:
    # two keys, scores s*q.k; closed form of a 2-way softmax
    Q = np.array([[[0.0, 0.0]], [[1.0, 2.0]]])
    K = np.array([[[3.0, -1.0]], [[0.5, 0.25]]])
    V = np.array([[[1.0, 0.0]], [[0.0, 1.0]]])
    s0, s1 = 0.7 * (3.0 - 2.0), 0.7 * (0.5 + 0.5)
    p0 = np.exp(s0) / (np.exp(s0) + np.exp(s1))
    O = oracle.swa(Q, K, V, 2, 0.7)
    assert np.allclose(O[1, 0], [p0, 1 - p0], atol=1e-15)
    assert np.array_equal(O[0, 0], [1.0, 0.0])


# -------------------------------------------------------- cross-attention (Eq. 3)
@pytest.mark.parametrize("q_pos0,Tq,N", [(0, 12, 12), (5, 4, 12), (11, 1, 12)])
def test_cross_attn_matches_brute_force(q_pos0, Tq, N):
    rng = np.random.default_rng(9)
    Q = rng.standard_normal((Tq, 4, 8))
    K, V = rng.standard_normal((N, 2, 8)), rng.standard_normal((N, 2, 8))
    ref = brute_force(Q, K, V, lambda i, j: j <= q_pos0 + i, 0.41)
    assert np.abs(oracle.cross_attn(Q, K, V, q_pos0, 0.41) - ref).max() < 1e-12


def test_cross_attn_same_tokens_is_causal_self_attention_and_wide_swa():
    T, d = 48, 16
    Q, K, V = rand_qkv(10, T, 6, 2, d)
    i, j = np.arange(T)[:, None], np.arange(T)[None, :]
    ref = sdpa(Q, K, V, j <= i, 1 / np.sqrt(d))
    got = oracle.cross_attn(Q, K, V, 0, 1 / np.sqrt(d))
    assert np.abs(got - ref).max() < 1e-12
    assert np.abs(got - oracle.swa(Q, K, V, T, 1 / np.sqrt(d))).max() < 1e-13


def test_cross_attn_decode_is_last_row_and_causal():
    T, d = 33, 8
    Q, K, V = rand_qkv(11, T, 4, 1, d)
    full = oracle.cross_attn(Q, K, V, 0, 0.3)
    dec = oracle.cross_attn(Q[T - 1:], K, V, T - 1, 0.3)
    assert np.abs(dec[0] - full[T - 1]).max() < 1e-14
    K2 = K.copy()
    K2[20] += 3.0
    changed = np.nonzero(np.abs(oracle.cross_attn(Q, K2, V, 0, 0.3) - full).max(axis=(1, 2)) > 0)[0]
    assert changed.min() == 20 and len(changed) == T - 20


def test_gqa_replication_invariant():
    T, d, G = 24, 8, 3
    Q, K, V = rand_qkv(12, T, 6, 2, d)
    Kr, Vr = np.repeat(K, G, axis=1), np.repeat(V, G, axis=1)
    assert np.array_equal(oracle.swa(Q, K, V, 5, 0.4), oracle.swa(Q, Kr, Vr, 5, 0.4))
    assert np.array_equal(oracle.cross_attn(Q, K, V, 0, 0.4), oracle.cross_attn(Q, Kr, Vr, 0, 0.4))


# ---------------------------------------------------- RMSNorm, Eq. 2, SwiGLU
def test_rmsnorm_and_global_kv_against_library():
    rng = np.random.default_rng(13)
    X, g = rng.standard_normal((7, 32)), rng.standard_normal(32)
    ref = F.rms_norm(torch.from_numpy(X), (32,), torch.from_numpy(g), eps=1e-6).numpy()
    assert np.abs(oracle.rmsnorm(X, g, 1e-6) - ref).max() < 1e-14
    # closed form: a constant row c maps to gain * c / sqrt(c^2 + eps)
    c = np.full((1, 32), -3.0)
    assert np.allclose(oracle.rmsnorm(c, g, 1e-6), g * -3.0 / np.sqrt(9 + 1e-6), atol=1e-15)
    WK, WV = rng.standard_normal((32, 16)), rng.standard_normal((32, 16))
    Kh, Vh = oracle.global_kv(X, g, WK, WV, Hkv=2)
    assert Kh.shape == (7, 2, 8)
    assert np.abs(Kh.reshape(7, 16) - ref @ WK).max() < 1e-13
    assert np.abs(Vh.reshape(7, 16) - ref @ WV).max() < 1e-13
    # W_K = I picks the normalised rows themselves; head h holds columns [h*d, (h+1)*d)
    Ki, _ = oracle.global_kv(X, g, np.eye(32), np.eye(32), Hkv=4)
    assert np.abs(Ki[:, 1, :] - ref[:, 8:16]).max() < 1e-14


def test_global_kv_with_the_norm_behind_the_projections_is_the_same_cache():
    """Eq. 2 in the form the fused write call takes: (1 / rms(x)) * (x (diag(g) W)) equals RMSNorm(x) W to rounding
    (1e-12 of the largest entry), against the library's rms_norm as well as against oracle.global_kv; the factor is
    the library norm's own (a row of ones has factor 1 / sqrt(1 + eps)); a wrong eps, a dropped gain or a factor
    applied per column would each break the equality."""
    rng = np.random.default_rng(17)
    X, g = rng.standard_normal((9, 48)) * 3.0, rng.standard_normal(48)
    WK, WV = rng.standard_normal((48, 24)), rng.standard_normal((48, 24))
    Kh, Vh = oracle.global_kv(X, g, WK, WV, Hkv=3)
    Kr, Vr, rs = oracle.global_kv_scaled_form(X, g, WK, WV, Hkv=3)
    assert Kr.shape == (9, 3, 8) and rs.shape == (9,)
    big = max(np.abs(Kh).max(), np.abs(Vh).max())
    assert np.abs(Kr * rs[:, None, None] - Kh).max() <= 1e-12 * big
    assert np.abs(Vr * rs[:, None, None] - Vh).max() <= 1e-12 * big
    lib = F.rms_norm(torch.from_numpy(X), (48,), torch.from_numpy(g), eps=1e-6).numpy()
    assert np.abs((Kr * rs[:, None, None]).reshape(9, 24) - lib @ WK).max() <= 1e-12 * big
    ones = np.ones((1, 48))
    assert abs(oracle.global_kv_scaled_form(ones, g, WK, WV, Hkv=3)[2][0] - 1.0 / math.sqrt(1.0 + 1e-6)) < 1e-15
    # planted mistakes in copies of the scaled form
    assert np.abs(Kr * (1.0 / np.sqrt((X * X).mean(-1)))[:, None, None] - Kh).max() > 1e-9 * big          # eps dropped
    assert np.abs((X @ WK).reshape(9, 3, 8) * rs[:, None, None] - Kh).max() > 1e-3 * big                   # gain dropped
    assert np.abs(Kr * (1.0 / np.sqrt((X * X).sum(-1) + 1e-6))[:, None, None] - Kh).max() > 1e-3 * big     # sum for mean


def test_swish_against_library():
    x = np.linspace(-30, 30, 241)
    assert np.abs(oracle.swish(x) - F.silu(torch.from_numpy(x)).numpy()).max() < 1e-13
    assert oracle.swish(0.0) == 0.0 and abs(oracle.swish(40.0) - 40.0) < 1e-12


def test_swiglu_against_library():
    rng = np.random.default_rng(14)
    X = rng.standard_normal((5, 16))
    WG, W1, W2 = rng.standard_normal((16, 24)), rng.standard_normal((16, 24)), rng.standard_normal((24, 16))
    t = torch.from_numpy
    ref = ((F.silu(t(X) @ t(WG)) * (t(X) @ t(W1))) @ t(W2)).numpy()
    assert np.abs(oracle.swiglu(X, WG, W1, W2) - ref).max() < 1e-13


# --------------------------------------------------------- the stack (Fig. 2, 3)
SMALL = dict(d_model=32, Hq=4, Hkv_self=2, Hkv=1, d=8, n_self=2, n_cross=2, window=6, ffn=48, vocab=50, eps=1e-6)


def test_early_exit_equals_full_forward_last_row():
    w = ys.stack_weights(0, SMALL, "f32")
    for k in ("self", "cross"):          # larger weights so attention is not near-uniform
        for L in w[k]:
            for n in ("W_Q", "W_K", "W_V"):
                if n in L:
                    L[n] = L[n] * 30
    tok = ys.tokens(0, 40, 50)
    full = oracle.yoco_stack(tok, w, "full")
    ee = oracle.yoco_stack(tok, w, "early_exit")
    assert full.shape == (40, 50) and ee.shape == (1, 50)
    assert np.abs(ee[0] - full[-1]).max() < 1e-12


def test_prefix_invariance_decoder_only_behaviour():
    w = ys.stack_weights(1, SMALL, "f32")
    tok = ys.tokens(1, 30, 50)
    full = oracle.yoco_stack(tok, w, "full")
    for t in (0, 5, 6, 17):
        short = oracle.yoco_stack(tok[:t + 1], w, "early_exit")
        assert np.abs(short[0] - full[t]).max() < 1e-12


# ------------------------------------- rolling-window cache (section 3.2, 2.3 footnote)
@pytest.mark.parametrize("T,C", [(23, 5), (9, 1), (12, 12), (7, 30), (33, 8)])
def test_rolling_cache_matches_brute_force_over_full_history(T, C):
    """Feeding the rows one by one through a ring of C slots gives, at every
    position (before the first wrap, at it, and several wraps later), the row of
    the literal-mask definition computed over the whole history."""
    Q, K, V = rand_qkv(11, T, 4, 2, 8)
    ref = brute_force(Q, K, V, lambda i, j: i - C < j <= i, 0.41)
    ring = oracle.RollingWindowCache(C, 2, 8)
    assert ring.K.shape == (C, 2, 8) and ring.V.shape == (C, 2, 8)      # O(C) rows whatever T is
    for p_ in range(T):
        ring.write(p_, K[p_], V[p_])
        assert np.abs(ring.attend(Q[p_], p_, 0.41) - ref[p_]).max() < 1e-12, p_


def test_rolling_cache_forgets_exactly_position_p_minus_C():
    """After position p is written, changing the history at p - C (overwritten)
    cannot matter, while changing p - C + 1 (the oldest kept row) must."""
    C, T = 6, 20
    Q, K, V = rand_qkv(12, T, 2, 2, 8)

    def last_row(Kx, Vx):
        ring = oracle.RollingWindowCache(C, 2, 8)
        for p_ in range(T):
            ring.write(p_, Kx[p_], Vx[p_])
        return ring.attend(Q[T - 1], T - 1, 0.5)

    base = last_row(K, V)
    K2, V2 = K.copy(), V.copy()
    K2[T - 1 - C] += 3.0
    V2[T - 1 - C] -= 2.0
    assert np.array_equal(last_row(K2, V2), base)
    V3 = V.copy()
    V3[T - C] += 1.0
    assert np.abs(last_row(K, V3) - base).max() > 1e-3


def test_token_by_token_stack_equals_all_at_once_stack():
    """An autoregressive model gives the same logits whether the prompt is
    processed at once or one token at a time (sections 2 and 2.3); the sequence
    is several windows long so the rings wrap."""
    w = ys.stack_weights(2, SMALL, "f32")
    for k in ("self", "cross"):
        for L in w[k]:
            for n in ("W_Q", "W_K", "W_V"):
                if n in L:
                    L[n] = L[n] * 30
    tok = ys.tokens(2, 29, 50)
    full = oracle.yoco_stack(tok, w, "full")
    step = oracle.yoco_stack_generate(tok, w)
    assert step.shape == full.shape
    assert np.abs(step - full).max() < 1e-11


def test_stack_matches_library_composition():
    """The same stack assembled from torch library ops (rms_norm, sdpa with
    masks, silu) in float64."""
    w = ys.stack_weights(2, SMALL, "f32")
    tok = ys.tokens(2, 25, 50)
    T, Hq, d, eps = 25, SMALL["Hq"], SMALL["d"], 1e-6
    t = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64))
    rn = lambda x, g: F.rms_norm(x, (x.shape[-1],), t(g), eps=eps)
    ffn = lambda x, L: (F.silu(x @ t(L["W_G"])) * (x @ t(L["W_1"]))) @ t(L["W_2"])
    i, j = np.arange(T)[:, None], np.arange(T)[None, :]
    band, causal = (j <= i) & (j > i - SMALL["window"]), j <= i
    X = t(w["embed"])[torch.from_numpy(tok)]
    for L in w["self"]:
        xn = rn(X, L["ln1"])
        A = sdpa((xn @ t(L["W_Q"])).reshape(T, Hq, d).numpy(), (xn @ t(L["W_K"])).reshape(T, 2, d).numpy(),
                 (xn @ t(L["W_V"])).reshape(T, 2, d).numpy(), band, 1 / np.sqrt(d))
        Y = t(A).reshape(T, Hq * d) @ t(L["W_O"]) + X
        X = ffn(rn(Y, L["ln2"]), L) + Y
    xn = rn(X, w["kv"]["ln"])
    Kh, Vh = (xn @ t(w["kv"]["W_K"])).reshape(T, 1, d).numpy(), (xn @ t(w["kv"]["W_V"])).reshape(T, 1, d).numpy()
    for L in w["cross"]:
        A = sdpa((rn(X, L["ln1"]) @ t(L["W_Q"])).reshape(T, Hq, d).numpy(), Kh, Vh, causal, 1 / np.sqrt(d))
        Y = t(A).reshape(T, Hq * d) @ t(L["W_O"]) + X
        X = ffn(rn(Y, L["ln2"]), L) + Y
    ref = (rn(X, w["final_ln"]) @ t(w["W_out"])).numpy()
    assert np.abs(oracle.yoco_stack(tok, w, "full") - ref).max() < 1e-12


# ------------------------------------------------ the paper's printed cache numbers
def test_cache_arithmetic_matches_paper_numbers():
    vals = {}
    with open(os.path.join(HERE, "golden", "kv_cache_tokens_per_gb.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                k, v = line.split()
                vals[k] = float(v)
    per_tok = oracle.kv_cache_bytes_per_token(int(vals["kv_heads"]), int(vals["head_dim"]), int(vals["elem_bytes"]))
    per_tok_tf = oracle.kv_cache_bytes_per_token(int(vals["kv_heads"]), int(vals["head_dim"]),
                                                 int(vals["elem_bytes"]), cached_layers=int(vals["layers"]))
    assert 2 ** 30 // per_tok == vals["yoco_tokens_per_gib"]
    assert round(2 ** 30 / per_tok_tf / 1000, 1) == vals["transformer_tokens_per_gib_rounded_to_0.1k"]
    assert per_tok_tf / per_tok == vals["reduction_factor"]


def test_8_bit_cache_arithmetic_matches_the_papers_65b_example():
    vals = {}
    with open(os.path.join(HERE, "golden", "kv_cache_65b_512k_8bit.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                k, v = line.split()
                vals[k] = int(v)
    per_tok = oracle.kv_cache_bytes_per_token(vals["kv_heads"], vals["head_dim"], vals["elem_bytes"], cached_layers=vals["layers"])
    assert round(per_tok * vals["tokens"] / 1e9) == vals["gigabytes_rounded"]
    # the same model with YOCO's single global pair needs 1/80 of that
    assert per_tok // oracle.kv_cache_bytes_per_token(vals["kv_heads"], vals["head_dim"], vals["elem_bytes"]) == vals["layers"]


# ---------------------------------------------------------------- input module
def test_bf16_rounding_is_rne_and_idempotent():
    x = np.array([1.0, 1.00390625, 1.01171875, -2.5, 3.1415927, 1e-30, 65504.0], dtype=np.float32)
    r = ys.round_to(x, "bf16")
    ref = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(r, ref)
    assert np.array_equal(ys.round_to(r, "bf16"), r)
    big = np.random.default_rng(0).standard_normal(100000).astype(np.float32)
    assert np.array_equal(ys.round_to(big, "bf16"), torch.from_numpy(big).to(torch.bfloat16).float().numpy())


# ------------------------------------------------ gated retention (Eq. 4-7)
def rand_gret(seed, T, H, dk, dv, lo=0.6):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((T, H, dk)), rng.standard_normal((T, H, dk)), rng.standard_normal((T, H, dv)),
            lo + (1.0 - lo) * rng.random((T, H)))


def gret_brute_force(Q, K, V, gamma, scale):
    """o_n = sum_{m<=n} (prod_{i=m+1..n} gamma_i) (q_n . k_m) v_m with scalar loops."""
    T, H, dk = Q.shape
    O = np.zeros((T, H, V.shape[2]))
    for h in range(H):
        for n in range(T):
            for m in range(n + 1):
                decay = 1.0
                for i in range(m + 1, n + 1):
                    decay *= gamma[i, h]
                dot = sum(Q[n, h, e] * K[m, h, e] for e in range(dk))
                O[n, h] += scale * decay * dot * V[m, h]
    return O


def test_gret_parallel_matches_brute_force():
    Q, K, V, gamma = rand_gret(21, 11, 2, 4, 3)
    assert np.abs(oracle.gret_parallel(Q, K, V, gamma, 0.7) - gret_brute_force(Q, K, V, gamma, 0.7)).max() < 1e-12


@pytest.mark.parametrize("chunk", [1, 4, 7, 16, 64])
def test_gret_three_forms_agree(chunk):
    """Section 3.1: the parallel, recurrent and chunkwise forms are equivalent
    (appendix B); the last chunk is ragged for chunk = 7 and 16."""
    Q, K, V, gamma = rand_gret(22, 37, 3, 8, 6)
    par = oracle.gret_parallel(Q, K, V, gamma, 0.3)
    rec, S = oracle.gret_recurrent(Q, K, V, gamma, 0.3)
    chk, R = oracle.gret_chunkwise(Q, K, V, gamma, 0.3, chunk)
    assert np.abs(rec - par).max() < 1e-11
    assert np.abs(chk - par).max() < 1e-11
    assert np.abs(R - S).max() < 1e-11


def test_gret_state_carries_across_a_split():
    """Processing rows [0, 20) and then [20, 37) with the carried state equals one pass."""
    Q, K, V, gamma = rand_gret(23, 37, 2, 8, 8)
    full = oracle.gret_parallel(Q, K, V, gamma, 1.0)
    o1, S1 = oracle.gret_chunkwise(Q[:20], K[:20], V[:20], gamma[:20], 1.0, 8)
    o2, S2 = oracle.gret_chunkwise(Q[20:], K[20:], V[20:], gamma[20:], 1.0, 8, S0=S1)
    o3, S3 = oracle.gret_recurrent(Q[20:], K[20:], V[20:], gamma[20:], 1.0, S0=S1)
    assert np.abs(np.concatenate([o1, o2]) - full).max() < 1e-11
    assert np.abs(o3 - o2).max() < 1e-11 and np.abs(S3 - S2).max() < 1e-11


def test_gret_closed_forms():
    Q, K, V, _ = rand_gret(24, 15, 2, 4, 4)
    T = Q.shape[0]
    # gamma = 1: plain causal linear attention, o_n = q_n . sum_{m<=n} k_m^T v_m
    ones = np.ones((T, 2))
    ref = np.zeros_like(V)
    for h in range(2):
        S = np.zeros((4, 4))
        for n in range(T):
            S += np.outer(K[n, h], V[n, h])
            ref[n, h] = Q[n, h] @ S
    assert np.abs(oracle.gret_parallel(Q, K, V, ones, 1.0) - ref).max() < 1e-12
    # gamma = 0: only the diagonal term survives (the empty product is 1)
    diag = np.einsum("the,the->th", Q, K)[..., None] * V
    for fn in (lambda: oracle.gret_parallel(Q, K, V, 0 * ones, 1.0), lambda: oracle.gret_recurrent(Q, K, V, 0 * ones, 1.0)[0]):
        assert np.abs(fn() - diag).max() < 1e-12
    # a constant decay g: D_nm = g^(n-m) (retention with a fixed decay)
    g = 0.9
    D = np.tril(g ** (np.arange(T)[:, None] - np.arange(T)[None, :]).clip(0))
    ref = np.stack([(Q[:, h] @ K[:, h].T * D) @ V[:, h] for h in range(2)], axis=1)
    assert np.abs(oracle.gret_parallel(Q, K, V, g * ones, 1.0) - ref).max() < 1e-12


def test_gret_is_causal_and_scale_is_linear():
    Q, K, V, gamma = rand_gret(25, 12, 1, 4, 4)
    base = oracle.gret_parallel(Q, K, V, gamma, 1.0)
    K2, V2, g2 = K.copy(), V.copy(), gamma.copy()
    K2[8:] += 1.0
    V2[8:] -= 1.0
    g2[8:] *= 0.5
    assert np.array_equal(oracle.gret_parallel(Q, K2, V2, g2, 1.0)[:8], base[:8])
    assert np.abs(oracle.gret_parallel(Q, K, V, gamma, 0.25) - 0.25 * base).max() < 1e-13


def test_gret_decay_and_group_norm_against_library():
    rng = np.random.default_rng(26)
    X, W = rng.standard_normal((9, 16)), rng.standard_normal((16, 3))
    ref = torch.exp(F.logsigmoid(torch.from_numpy(X @ W)) / 16.0).numpy()       # sigmoid(z)^(1/tau)
    got = oracle.gret_decay(X, W, 16.0)
    assert np.abs(got - ref).max() < 1e-14 and (got > 0).all() and (got < 1).all()
    O = rng.standard_normal((9, 3, 8)) * 3 + 1
    ref = F.group_norm(torch.from_numpy(O.reshape(9, 24)), 3, eps=1e-6).numpy().reshape(9, 3, 8)
    assert np.abs(oracle.group_norm_heads(O, 1e-6) - ref).max() < 1e-12


def test_mhgr_matches_library_composition():
    """Eq. 7 assembled from torch ops (cumulative log-decays, masked product,
    group_norm, silu) against the oracle."""
    rng = np.random.default_rng(27)
    T, dm, H, dh, tau = 14, 16, 2, 8, 16.0
    X = rng.standard_normal((T, dm))
    Ws = {n: rng.standard_normal((dm, dm)) * 0.3 for n in ("W_Q", "W_K", "W_V", "W_G", "W_O")}
    Wg = rng.standard_normal((dm, H))
    got = oracle.mhgr(X, Ws["W_Q"], Ws["W_K"], Ws["W_V"], Wg, Ws["W_G"], Ws["W_O"], H, tau, 0.5)
    x = torch.from_numpy(X)
    q, k, v = ((x @ torch.from_numpy(Ws[n])).view(T, H, dh).transpose(0, 1) for n in ("W_Q", "W_K", "W_V"))
    G = (F.logsigmoid(x @ torch.from_numpy(Wg)) / tau).cumsum(0).transpose(0, 1)          # [H,T]
    mask = (G[:, :, None] - G[:, None, :] + torch.full((T, T), float("-inf"), dtype=torch.float64).triu(1)).exp()
    heads = ((0.5 * q @ k.transpose(1, 2)) * mask) @ v                                     # [H,T,dh]
    y = F.group_norm(heads.transpose(0, 1).reshape(T, H * dh), H, eps=1e-6)
    ref = ((F.silu(x @ torch.from_numpy(Ws["W_G"])) * y) @ torch.from_numpy(Ws["W_O"])).numpy()
    assert np.abs(got - ref).max() < 1e-10


GRET_SMALL = dict(SMALL, Hkv_self=4, self_kind="gret", tau=4.0)


def test_gret_stack_early_exit_prefix_and_generation_invariants():
    """The stack with a gated-retention self-decoder: early exit = last row of the full forward (Fig. 3), a
    prefix's logits do not depend on later tokens, and token-by-token generation with the recurrent state
    (Eq. 5) reproduces the all-at-once forward, which uses the parallel form (Eq. 4)."""
    w = ys.stack_weights(3, GRET_SMALL, "f32")
    for k in ("self", "cross"):
        for L in w[k]:
            for n in ("W_Q", "W_K", "W_V"):
                if n in L:
                    L[n] = L[n] * 30
    tok = ys.tokens(3, 23, 50)
    full = oracle.yoco_stack(tok, w, "full")
    assert np.abs(oracle.yoco_stack(tok, w, "early_exit")[0] - full[-1]).max() < 1e-11
    assert np.abs(oracle.yoco_stack(tok[:9], w, "early_exit")[0] - full[8]).max() < 1e-11
    assert np.abs(oracle.yoco_stack_generate(tok, w) - full).max() < 1e-10
    # and it is a different model from the sliding-window variant with the same shared matrices
    w_swa = ys.stack_weights(3, dict(SMALL, Hkv_self=4), "f32")
    assert np.abs(oracle.yoco_stack(tok, w_swa, "full") - oracle.yoco_stack(tok, ys.stack_weights(3, GRET_SMALL, "f32"), "full")).max() > 1e-4


# ---------------------------------------------------------------- 8-bit cache codes (section 1 names 8-bit KV quantisation)
def _rows(seed, shape, spread=True):
    rng = np.random.default_rng(seed)
    X = rng.standard_normal(shape).astype(np.float32)
    if spread:      # rows of very different magnitude: a scale taken over the wrong axis cannot pass
        X *= np.exp2(rng.integers(-12, 12, size=shape[:-1])).astype(np.float32)[..., None]
    return X


def test_int8_codes_half_step_property_and_extremes():
    X = _rows(0, (50, 3, 128))
    X[7, 1] = 0.0
    codes, scale = oracle.kv_quantise_int8(X)
    assert codes.dtype == np.int8 and scale.dtype == np.float32 and scale.shape == X.shape[:-1]
    assert codes.min() >= -127 and codes.max() <= 127
    a = np.abs(X).max(axis=-1)
    # the scale is max|row| / 127 and the largest element sits on the last code
    np.testing.assert_allclose(scale.astype(np.float64), a.astype(np.float64) / 127.0, rtol=1e-6)
    top = np.take_along_axis(codes, np.abs(X).argmax(axis=-1)[..., None], axis=-1)[..., 0]
    nz = a > 0
    assert np.all(np.abs(top[nz]) == 127)
    assert np.all(codes[7, 1] == 0) and scale[7, 1] == 0
    # nearest code: no element is further than half a step (plus float32 rounding) from its value
    err = np.abs(oracle.kv_dequantise_int8(codes, scale) - X.astype(np.float64))
    assert np.all(err <= 0.5 * scale.astype(np.float64)[..., None] * (1 + 1e-5))
    # and half a step is reached: the rounding is to nearest, not towards zero (whose error reaches a full step)
    assert (err / np.maximum(scale.astype(np.float64)[..., None], 1e-300)).max() > 0.49


def test_int8_codes_symmetries():
    X = _rows(1, (40, 2, 64))
    codes, scale = oracle.kv_quantise_int8(X)
    cn, sn = oracle.kv_quantise_int8(-X)
    assert np.array_equal(cn, -codes) and np.array_equal(sn, scale)            # odd in x: round-half-even, no offset
    c8, s8 = oracle.kv_quantise_int8(X * np.float32(8.0))
    assert np.array_equal(c8, codes) and np.array_equal(s8, scale * np.float32(8.0))   # powers of two are exact in float32
    # a row does not depend on the other rows or heads
    Y = X.copy()
    Y[3, 0] *= 100.0
    cy, sy = oracle.kv_quantise_int8(Y)
    keep = np.ones(X.shape[:-1], bool)
    keep[3, 0] = False
    assert np.array_equal(cy[keep], codes[keep]) and np.array_equal(sy[keep], scale[keep])


def test_int8_codes_exact_on_representable_rows_and_ties():
    # a row that is already integer codes times a power of two comes back unchanged
    rng = np.random.default_rng(2)
    c = rng.integers(-127, 128, size=(16, 32)).astype(np.int8)
    c[:, 0] = 127
    X = c.astype(np.float32) * np.float32(2.0 ** -5) * np.float32(127.0) / np.float32(127.0)
    codes, scale = oracle.kv_quantise_int8(X)
    assert np.array_equal(codes, c)
    # halves round to the even neighbour: with max 127 the multiplier is exactly 1
    X = np.array([[127.0, 0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 126.5]], dtype=np.float32)
    codes, scale = oracle.kv_quantise_int8(X)
    assert codes.tolist() == [[127, 0, 2, 2, 0, -2, -2, 126]] and scale[0] == 1.0


def test_int8_codes_against_library_quantiser():
    X = _rows(3, (64, 128))
    codes, scale = oracle.kv_quantise_int8(X)
    q = torch.quantize_per_channel(torch.from_numpy(X), torch.from_numpy(scale.astype(np.float64)),
                                   torch.zeros(64, dtype=torch.int64), 0, torch.qint8)
    lib = q.int_repr().numpy()
    # the library multiplies by 1/scale, the oracle by 127/max: the two may differ by one code on a rare near-tie
    diff = np.abs(lib.astype(np.int32) - codes.astype(np.int32))
    assert diff.max() <= 1 and (diff != 0).sum() <= 3
    np.testing.assert_allclose(q.dequantize().numpy()[diff == 0], oracle.kv_dequantise_int8(codes, scale)[diff == 0], rtol=1e-6)


def test_cross_attn_int8_is_attention_over_the_coded_rows_and_within_its_bound():
    T, Hq, Hkv, d = 96, 4, 2, 32
    scale = 1.0 / math.sqrt(d)
    q, k, v = ys.qkv(4, T, Hq, Hkv, d, 1.0, "f32")
    exact = oracle.cross_attn(q[-3:], k, v, T - 3, scale)
    coded = oracle.cross_attn_int8(q[-3:], k, v, T - 3, scale)
    err = np.abs(coded - exact).max()
    bound = oracle.cross_attn_int8_error_bound(q[-3:], k, v, scale)
    assert 0 < err <= bound, (err, bound)
    # the codes, not the originals, are what is attended to: replacing K^, V^ by their coded values changes nothing
    kq = oracle.kv_dequantise_int8(*oracle.kv_quantise_int8(k)).astype(np.float32)
    vq = oracle.kv_dequantise_int8(*oracle.kv_quantise_int8(v)).astype(np.float32)
    again = oracle.cross_attn_int8(q[-3:], kq, vq, T - 3, scale)
    np.testing.assert_allclose(again, coded, rtol=0, atol=1e-6)
    # a coarser grid (every second code) must violate the bound's leading term scaling: error grows about 2x
    k2, s2 = oracle.kv_quantise_int8(k)
    coarse = oracle.cross_attn(q[-3:], (2 * np.rint(k2 / 2.0)) * s2.astype(np.float64)[..., None], vq, T - 3, scale)
    assert np.abs(coarse - exact).max() > err


def int8_bound_worst_case(D_target=0.05, d=32, t=2.0 ** -7):
    """Rows built so that both terms of the 8-bit error bound are (almost) attained. Two cache rows, one KV head.
    K: element 0 = 127 s fixes the row maximum (scale exactly s); the other elements sit 0.499 s above code 10 in
    row 0 and 0.499 s below it in row 1, so the coded rows are equal and the exact scores differ by
    scale * ||q||_1 * 0.998 s, q being constant and positive there. V: element 0 = 127 t, the others 0.499 t above code
    +126 (row 0) and above code -126 (row 1): every coded value is 0.499 t too low and the two rows are almost
    +-max|V| in the first half of the dims (the second half holds small values). Returns q [1,1,d], K, V [2,1,d] (float32, all values exact) and the scale."""
    s = np.float32(2.0 ** -5)
    off = np.float32(0.4990234375)                       # 511/1024: exact in float32 next to small integers
    K = np.zeros((2, 1, d), dtype=np.float32)
    K[:, 0, 0] = 127 * s
    K[0, 0, 1:] = (10 + off) * s
    K[1, 0, 1:] = (10 - off) * s
    V = np.zeros((2, 1, d), dtype=np.float32)
    V[:, 0, 0] = 127 * np.float32(t)
    V[0, 0, 1:] = (126 + off) * np.float32(t)
    V[1, 0, 1:] = (-126 + off) * np.float32(t)
    V[:, 0, d // 2:] = off * np.float32(t)              # half of the dims small: the largest |V|, not a typical one, sets the bound
    scale = 1.0 / math.sqrt(d)
    # D = scale * ||q||_1 * 1.001 * 127 s / 254  ->  the constant q value that gives D_target
    qv = D_target / (scale * (d - 1) * 1.001 * float(s) / 2)
    q = np.zeros((1, 1, d), dtype=np.float32)
    q[0, 0, 1:] = np.float32(qv)
    return q, K, V, scale


@pytest.mark.parametrize("D_target", [0.01, 0.05, 0.3])
def test_int8_error_bound_is_attained_from_below_and_never_exceeded(D_target):
    """The bound is held from both sides: on rows that sit half a code step off, aligned with the query, the true
    error reaches 90 % of it (a bound twice too large fails here), and it stays below it (a bound too small fails)."""
    q, K, V, scale = int8_bound_worst_case(D_target)
    codes, sc = oracle.kv_quantise_int8(K)
    assert np.array_equal(codes[0], codes[1]) and sc[0, 0] == np.float32(2.0 ** -5)      # the construction holds
    exact = oracle.cross_attn(q, K, V, 1, scale)
    coded = oracle.cross_attn_int8(q, K, V, 1, scale)
    err = np.abs(coded - exact).max()
    bound = oracle.cross_attn_int8_error_bound(q, K, V, scale)
    assert 0.90 * bound <= err <= bound, (err, bound, err / bound)
    # closed form of this case: the coded rows tie (weights 1/2, 1/2), the exact weights are (1 +- tanh(delta/2))/2
    delta = scale * float(q.astype(np.float64).sum()) * 0.998046875 * 2.0 ** -5
    t = 2.0 ** -7
    want = 0.4990234375 * t + math.tanh(0.5 * delta) * 126 * t
    assert abs(err - want) <= 1e-9 * want, (err, want)


def test_int8_error_bound_terms_scale_as_the_derivation_says():
    """V-only case (q = 0: every weight is exact) leaves the half-step term alone; doubling every magnitude doubles
    the bound's V term and leaves D-dependence to the K term."""
    q, K, V, scale = int8_bound_worst_case(0.05)
    q0 = np.zeros_like(q)
    b0 = oracle.cross_attn_int8_error_bound(q0, K, V, scale)
    assert abs(b0 - 1.001 * 127 * 2.0 ** -7 / 254) <= 1e-15
    err0 = np.abs(oracle.cross_attn_int8(q0, K, V, 1, scale) - oracle.cross_attn(q0, K, V, 1, scale)).max()
    assert 0.99 * b0 <= err0 <= b0
    assert abs(oracle.cross_attn_int8_error_bound(q0, K, 2 * V, scale) - 2 * b0) <= 1e-15
    # random rows stay inside it with room to spare (it is a worst case, not a typical one)
    qr, kr, vr = ys.qkv(11, 64, 2, 1, 32, 1.0, "f32")
    e = np.abs(oracle.cross_attn_int8(qr[-1:], kr, vr, 63, scale) - oracle.cross_attn(qr[-1:], kr, vr, 63, scale)).max()
    assert 0 < e < 0.5 * oracle.cross_attn_int8_error_bound(qr[-1:], kr, vr, scale)


def test_stack_with_8_bit_cache_keeps_the_generation_and_early_exit_invariants():
    """cache_bits = 8 changes K^, V^ to their coded values and nothing else: early exit still equals the last row of
    the full forward, token-by-token generation still equals the all-at-once forward (rows are coded one by one, each
    with its own scale), and the logits move by little but not by nothing."""
    c = ys.CONFIGS["tiny_fp32"]
    s = dict(c["stack"], n_self=1, n_cross=2)
    w = ys.stack_weights(3, s, "f32")
    tok = ys.tokens(5, 40, s["vocab"])
    plain = oracle.yoco_stack(tok, w, "full")
    w8 = dict(w, cache_bits=8)
    full = oracle.yoco_stack(tok, w8, "full")
    np.testing.assert_allclose(oracle.yoco_stack(tok, w8, "early_exit")[0], full[-1], rtol=0, atol=1e-12)
    np.testing.assert_allclose(oracle.yoco_stack_generate(tok, w8), full, rtol=0, atol=1e-10)
    diff = np.abs(full - plain).max()
    assert 0 < diff < 0.02 * np.abs(plain).max()
    np.testing.assert_allclose(full[0], oracle.yoco_stack(tok[:1], w8, "full")[0], rtol=0, atol=1e-12)   # still a decoder-only model
