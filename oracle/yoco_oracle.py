"""Plain fp64 definitions of what the YOCO attention hot path computes.

TEST INFRASTRUCTURE ONLY (see the package docstring). Every function is the
definition from the paper written out with numpy in float64: no tiling, no
online softmax, no split-KV, no fusion. A matrix product may serve as a step.
Positions are 0-based here; the paper counts from 1.

Pins (tests/test_oracle_pins.py): brute-force dense masked softmax on tiny
inputs, torch's CPU scaled_dot_product_attention / rms_norm / silu as library
routines, closed forms (equal keys -> running mean, window 1 -> V, constant V),
locality and causality under perturbation, GQA replication, the early-exit and
prefix invariants of the stack, and the paper's cache-size arithmetic
(section 4.4, the KV-cache-per-token figure: 128K tokens per GB at 65B).
The rolling-window cache and the token-by-token stack are pinned to the
windowed definition (a literal-mask brute force over the full history) and to
the all-at-once stack, whose outputs an autoregressive model must reproduce.
Gated retention (Eq. 4-7): the parallel form is the definition written out
(products of the decays); it is pinned by a brute-force triple loop, by the
paper's own statement that the parallel, recurrent and chunkwise forms give the
same result (also across a split of the sequence with a carried state), by
the closed forms gamma = 1 (causal prefix sums) and gamma -> 0 (only the
diagonal term), and GroupNorm by torch's group_norm.
The 8-bit cache codes are pinned by the half-step error property, the
extremes (the largest element gets +-127, a zero row gets zeros), sign and
power-of-two scaling symmetries, torch's per-channel quantiser as a library
routine, and the attention over them by its derived error bound.
No function here is "parity unpinned".

Readings of points the paper leaves open:
  * `scale` is an explicit argument; Eq. 8 prints no 1/sqrt(d), Eq. 3 defers
    to "standard multi-head attention". The configurations use 1/sqrt(d).
  * Eq. 8's mask  i - C < j <= i  means a row sees itself and the C-1 keys
    before it: min(i+1, C) keys.
  * GQA: query head h reads KV head h // (Hq // Hkv).
  * LN is RMSNorm with its own gain vector and eps = 1e-6, no bias.
"""
import numpy as np

F64 = np.float64


def _softmax_weighted_sum(q, Kj, Vj, scale):
    """softmax_j(scale * q.k_j) applied to the rows v_j (one query, one head).

    q [d], Kj [n,d], Vj [n,d] -> [d]. The max is subtracted before exp, which
    leaves the softmax unchanged and avoids overflow.
    """
    s = scale * (Kj @ q)
    p = np.exp(s - s.max())
    p = p / p.sum()
    return p @ Vj


def swa_row(Q, K, V, i, h, window, scale):
    """Row i, head h of sliding-window attention (section 3.2, Eq. 8).

    B_ij = 0 iff i - C < j <= i, so the visible keys are j in
    [max(0, i-C+1), i]. Q [T,Hq,d]; K, V [T,Hkv,d]; returns [d] float64.
    """
    Hq, Hkv = Q.shape[1], K.shape[1]
    g = h // (Hq // Hkv)
    j0 = max(0, i - window + 1)
    q = np.asarray(Q[i, h], dtype=F64)
    Kj = np.asarray(K[j0:i + 1, g], dtype=F64)
    Vj = np.asarray(V[j0:i + 1, g], dtype=F64)
    return _softmax_weighted_sum(q, Kj, Vj, scale)


def swa(Q, K, V, window, scale):
    """head_h = softmax(Q_h K_h^T + B) V_h for every row and head (Eq. 8),
    before the output projection W_O. Returns [T,Hq,d] float64."""
    T, Hq, _ = Q.shape
    O = np.empty((T, Hq, V.shape[2]), dtype=F64)
    for h in range(Hq):
        for i in range(T):
            O[i, h] = swa_row(Q, K, V, i, h, window, scale)
    return O


def rmsnorm(X, gain, eps=1e-6):
    """RMSNorm, the paper's LN (section 2.1): x / sqrt(mean(x^2) + eps) * gain."""
    X = np.asarray(X, dtype=F64)
    ms = (X * X).mean(axis=-1, keepdims=True)
    return X / np.sqrt(ms + eps) * np.asarray(gain, dtype=F64)


def global_kv(X, gain, W_K, W_V, Hkv, eps=1e-6):
    """Global KV cache of the cross-decoder (section 2.2, Eq. 2):
    K^ = LN(X^{L/2}) W_K,  V^ = LN(X^{L/2}) W_V, reshaped to [T,Hkv,d]."""
    Xn = rmsnorm(X, gain, eps)
    Kh = Xn @ np.asarray(W_K, dtype=F64)
    Vh = Xn @ np.asarray(W_V, dtype=F64)
    T = X.shape[0]
    return Kh.reshape(T, Hkv, -1), Vh.reshape(T, Hkv, -1)


def global_kv_scaled_form(X, gain, W_K, W_V, Hkv, eps=1e-6):
    """Eq. 2 with the RMSNorm moved behind the projections (section 2.2, Eq. 2; section 2.1: LN = RMSNorm).
    RMSNorm(x) W = (x / rms(x) * g) W = (1 / rms(x)) * (x (diag(g) W)), so the un-normalised rows times the
    gain-scaled weights, and one factor per row, carry the same cache. Returns (K_raw, V_raw [T,Hkv,d],
    row_scale [T]) with K^ = K_raw * row_scale[:, None, None]."""
    X = np.asarray(X, dtype=F64)
    g = np.asarray(gain, dtype=F64)
    row_scale = 1.0 / np.sqrt((X * X).mean(axis=-1) + eps)
    Kraw = X @ (g[:, None] * np.asarray(W_K, dtype=F64))
    Vraw = X @ (g[:, None] * np.asarray(W_V, dtype=F64))
    T = X.shape[0]
    return Kraw.reshape(T, Hkv, -1), Vraw.reshape(T, Hkv, -1), row_scale


def cross_attn_row(Q, Khat, Vhat, i, h, q_pos0, scale):
    """Row i, head h of the cross-decoder's attention (section 2.2, Eq. 3):
    standard causal attention of the query at absolute position q_pos0 + i
    over cache rows j <= q_pos0 + i, with grouped-query heads."""
    Hq, Hkv = Q.shape[1], Khat.shape[1]
    g = h // (Hq // Hkv)
    p = q_pos0 + i
    q = np.asarray(Q[i, h], dtype=F64)
    Kj = np.asarray(Khat[:p + 1, g], dtype=F64)
    Vj = np.asarray(Vhat[:p + 1, g], dtype=F64)
    return _softmax_weighted_sum(q, Kj, Vj, scale)


def cross_attn(Q, Khat, Vhat, q_pos0, scale):
    """Attention(Q^, K^, V^) of Eq. 3 for Tq query rows; decode is Tq = 1 with
    q_pos0 = len - 1 (the new token's own row is already in the cache: Eq. 2
    comes before Eq. 3 and the mask is j <= i). Returns [Tq,Hq,d] float64."""
    Tq, Hq, _ = Q.shape
    O = np.empty((Tq, Hq, Vhat.shape[2]), dtype=F64)
    for h in range(Hq):
        for i in range(Tq):
            O[i, h] = cross_attn_row(Q, Khat, Vhat, i, h, q_pos0, scale)
    return O


def swish(x):
    """swish(x) = x * sigmoid(x) (sections 2.1 and 3.1)."""
    x = np.asarray(x, dtype=F64)
    return x / (1.0 + np.exp(-x))


def swiglu(X, W_G, W_1, W_2):
    """SwiGLU(X) = (swish(X W_G) * X W_1) W_2 with swish(x) = x * sigmoid(x)
    (section 2.1)."""
    X = np.asarray(X, dtype=F64)
    a = X @ np.asarray(W_G, dtype=F64)
    b = X @ np.asarray(W_1, dtype=F64)
    return ((a / (1.0 + np.exp(-a))) * b) @ np.asarray(W_2, dtype=F64)


def yoco_stack(tokens, w, mode="full"):
    """Decoder-decoder stack (section 2, Eq. 1-3, Fig. 2) -> logits.

    w: dict with 'embed' [vocab,dm]; 'self' = list of layers with keys
    ln1, W_Q, W_K, W_V, W_O, ln2, W_G, W_1, W_2 (and, when w['self_kind'] ==
    'gret', W_gamma [dm,Hq] and W_gate [dm,Hq*d] with the temperature w['tau']:
    the self-decoder then uses gated retention, Eq. 7); 'kv' = {ln, W_K, W_V};
    'cross' = list of layers with keys ln1, W_Q, W_O, ln2, W_G, W_1, W_2;
    'final_ln', 'W_out'; ints 'Hq', 'Hkv_self', 'Hkv', 'd', 'window'; 'eps';
    optional 'cache_bits' = 8: the global cache holds 8-bit codes (kv_quantise_int8).
    mode 'full': every row goes through the cross-decoder -> logits [T,vocab].
    mode 'early_exit' (Fig. 3, section 2.3): the self-decoder and Eq. 2 run on
    all rows, only the last row enters the cross-decoder -> logits [1,vocab].
    """
    Hq, d, eps = w["Hq"], w["d"], w["eps"]
    scale = 1.0 / np.sqrt(d)
    X = np.asarray(w["embed"], dtype=F64)[np.asarray(tokens)]
    T = X.shape[0]
    for L in w["self"]:                                   # Eq. 1
        Xn = rmsnorm(X, L["ln1"], eps)
        if w.get("self_kind", "swa") == "gret":           # section 3.1: multi-head gated retention (Eq. 7)
            Y = mhgr(Xn, L["W_Q"], L["W_K"], L["W_V"], L["W_gamma"], L["W_gate"], L["W_O"], Hq, w["tau"], scale, eps) + X
        else:                                             # section 3.2: sliding-window attention (Eq. 8)
            Q = (Xn @ np.asarray(L["W_Q"], F64)).reshape(T, Hq, d)
            K = (Xn @ np.asarray(L["W_K"], F64)).reshape(T, w["Hkv_self"], d)
            V = (Xn @ np.asarray(L["W_V"], F64)).reshape(T, w["Hkv_self"], d)
            A = swa(Q, K, V, w["window"], scale).reshape(T, Hq * d)
            Y = A @ np.asarray(L["W_O"], F64) + X
        X = swiglu(rmsnorm(Y, L["ln2"], eps), L["W_G"], L["W_1"], L["W_2"]) + Y
    Khat, Vhat = global_kv(X, w["kv"]["ln"], w["kv"]["W_K"], w["kv"]["W_V"], w["Hkv"], eps)  # Eq. 2
    if w.get("cache_bits") == 8:                          # the cache stores 8-bit codes: attention sees what they stand for
        Khat = kv_dequantise_int8(*kv_quantise_int8(Khat))
        Vhat = kv_dequantise_int8(*kv_quantise_int8(Vhat))
    if mode == "early_exit":
        X, q_pos0 = X[T - 1:T], T - 1
    elif mode == "full":
        q_pos0 = 0
    else:
        raise ValueError(mode)
    Tq = X.shape[0]
    for L in w["cross"]:                                  # Eq. 3
        Qh = (rmsnorm(X, L["ln1"], eps) @ np.asarray(L["W_Q"], F64)).reshape(Tq, Hq, d)
        A = cross_attn(Qh, Khat, Vhat, q_pos0, scale).reshape(Tq, Hq * d)
        Y = A @ np.asarray(L["W_O"], F64) + X
        X = swiglu(rmsnorm(Y, L["ln2"], eps), L["W_G"], L["W_1"], L["W_2"]) + Y
    return rmsnorm(X, w["final_ln"], eps) @ np.asarray(w["W_out"], F64)


class RollingWindowCache:
    """Self-decoder cache for token-by-token generation with sliding-window
    attention (section 3.2: the window bounds what a row can see; the footnote
    of section 2.3 and Table 1: the self-decoder keeps O(C) rows, not O(N)).

    A ring of C rows for one layer and one sequence: the row of position p is
    kept in slot p mod C, where it replaces position p - C, which the mask
    i - C < j <= i hides from every later row.
    """

    def __init__(self, C, Hkv, d):
        self.C = C
        self.K = np.zeros((C, Hkv, d), dtype=F64)
        self.V = np.zeros((C, Hkv, d), dtype=F64)

    def write(self, p, k, v):
        """k, v [Hkv,d]: the projected row of position p."""
        self.K[p % self.C] = k
        self.V[p % self.C] = v

    def attend(self, q, p, scale):
        """Eq. 8 for the row at position p (already written): q [Hq,d] -> [Hq,d].
        The visible positions max(0, p-C+1) .. p are gathered from their slots."""
        Hq, Hkv = q.shape[0], self.K.shape[1]
        slots = [j % self.C for j in range(max(0, p - self.C + 1), p + 1)]
        out = np.empty((Hq, self.V.shape[2]), dtype=F64)
        for h in range(Hq):
            g = h // (Hq // Hkv)
            out[h] = _softmax_weighted_sum(np.asarray(q[h], dtype=F64), self.K[slots, g], self.V[slots, g], scale)
        return out


def yoco_stack_generate(tokens, w):
    """The decoder-decoder stack run one token at a time (Fig. 3 "Generation",
    section 2.3): each self-decoder layer keeps a RollingWindowCache, Eq. 2
    appends one row to the global cache, and the cross-decoder attends to the
    rows written so far. Same weights dict as yoco_stack; returns the logits of
    every position, [T,vocab], which an autoregressive model must produce
    identically whether the prompt is processed at once or token by token."""
    Hq, d, eps = w["Hq"], w["d"], w["eps"]
    scale = 1.0 / np.sqrt(d)
    gret = w.get("self_kind", "swa") == "gret"
    rings = [RollingWindowCache(w["window"], w["Hkv_self"], d) for _ in w["self"]]
    states = [None for _ in w["self"]]                    # gated retention keeps S_n (Eq. 5) instead of a ring
    Khat, Vhat = [], []
    out = []
    for p, tok in enumerate(np.asarray(tokens)):
        x = np.asarray(w["embed"], dtype=F64)[tok][None]              # [1,dm]
        for li, (L, ring) in enumerate(zip(w["self"], rings)):
            xn = rmsnorm(x, L["ln1"], eps)
            q = (xn @ np.asarray(L["W_Q"], F64)).reshape(Hq, d)
            kr = (xn @ np.asarray(L["W_K"], F64)).reshape(w["Hkv_self"], d)
            vr = (xn @ np.asarray(L["W_V"], F64)).reshape(w["Hkv_self"], d)
            if gret:
                o, states[li] = gret_recurrent(q[None], kr[None], vr[None], gret_decay(xn, L["W_gamma"], w["tau"]), scale,
                                               S0=states[li])
                g = xn @ np.asarray(L["W_gate"], F64)
                a = (g / (1.0 + np.exp(-g))) * group_norm_heads(o, eps).reshape(1, Hq * d)
            else:
                ring.write(p, kr, vr)
                a = ring.attend(q, p, scale).reshape(1, Hq * d)
            y = a @ np.asarray(L["W_O"], F64) + x
            x = swiglu(rmsnorm(y, L["ln2"], eps), L["W_G"], L["W_1"], L["W_2"]) + y
        kh, vh = global_kv(x, w["kv"]["ln"], w["kv"]["W_K"], w["kv"]["W_V"], w["Hkv"], eps)
        if w.get("cache_bits") == 8:
            kh = kv_dequantise_int8(*kv_quantise_int8(kh))
            vh = kv_dequantise_int8(*kv_quantise_int8(vh))
        Khat.append(kh[0])
        Vhat.append(vh[0])
        Kc, Vc = np.stack(Khat), np.stack(Vhat)
        for L in w["cross"]:
            qh = (rmsnorm(x, L["ln1"], eps) @ np.asarray(L["W_Q"], F64)).reshape(1, Hq, d)
            a = cross_attn(qh, Kc, Vc, p, scale).reshape(1, Hq * d)
            y = a @ np.asarray(L["W_O"], F64) + x
            x = swiglu(rmsnorm(y, L["ln2"], eps), L["W_G"], L["W_1"], L["W_2"]) + y
        out.append((rmsnorm(x, w["final_ln"], eps) @ np.asarray(w["W_out"], F64))[0])
    return np.stack(out)


# ---------------------------------------------------------------- gated retention
def gret_decay(X, W_gamma, tau):
    """gamma = sigmoid(X W_gamma)^(1/tau) (section 3.1, Eq. 4): one decay in (0, 1)
    per token and head. X [T,dm], W_gamma [dm,H] -> gamma [T,H]."""
    z = np.asarray(X, dtype=F64) @ np.asarray(W_gamma, dtype=F64)
    return (1.0 / (1.0 + np.exp(-z))) ** (1.0 / tau)


def gret_parallel(Q, K, V, gamma, scale):
    """Parallel form of gated retention (Eq. 4): (Q K^T * D) V per head with
    D_nm = prod_{i=m+1..n} gamma_i for n >= m (1 on the diagonal) and 0 above.
    Q, K [T,H,dk]; V [T,H,dv]; gamma [T,H] -> [T,H,dv]. `scale` multiplies
    Q K^T (the equation prints none; it cancels in the GroupNorm of Eq. 7)."""
    T, H, _ = Q.shape
    Q, K, V, gamma = (np.asarray(a, dtype=F64) for a in (Q, K, V, gamma))
    O = np.zeros((T, H, V.shape[2]), dtype=F64)
    for h in range(H):
        D = np.zeros((T, T), dtype=F64)
        for n in range(T):
            for m in range(n + 1):
                D[n, m] = np.prod(gamma[m + 1:n + 1, h])
        O[:, h] = (scale * (Q[:, h] @ K[:, h].T) * D) @ V[:, h]
    return O


def gret_recurrent(Q, K, V, gamma, scale, S0=None):
    """Recurrent form (Eq. 5): S_n = gamma_n S_{n-1} + K_n^T V_n, o_n = Q_n S_n.
    S0 [H,dk,dv] is the state before the first row (zeros if None).
    Returns (O [T,H,dv], S_T [H,dk,dv])."""
    T, H, dk = Q.shape
    dv = V.shape[2]
    Q, K, V, gamma = (np.asarray(a, dtype=F64) for a in (Q, K, V, gamma))
    S = np.zeros((H, dk, dv), dtype=F64) if S0 is None else np.array(S0, dtype=F64)
    O = np.zeros((T, H, dv), dtype=F64)
    for n in range(T):
        for h in range(H):
            S[h] = gamma[n, h] * S[h] + np.outer(K[n, h], V[n, h])
            O[n, h] = scale * (Q[n, h] @ S[h])
    return O, S


def gret_chunkwise(Q, K, V, gamma, scale, chunk, S0=None):
    """Chunkwise recurrent form (Eq. 6, appendix B). Within chunk [i], with
    beta_j the product of the chunk's decays up to and including row j:
      inner  = (Q K^T * D) V,  D(j,k) = beta_j / beta_k for k <= j, else 0
      cross  = (Q R_{i-1}) * beta_j                      (row-wise)
      R_i    = K^T (V * beta_last / beta_j) + beta_last R_{i-1}
    (Eq. 6 prints D(j,k) with j and k exchanged; the proof in appendix B and
    Eq. 4 fix the reading used here.) The last chunk may be shorter.
    Returns (O [T,H,dv], R_last [H,dk,dv])."""
    T, H, dk = Q.shape
    dv = V.shape[2]
    Q, K, V, gamma = (np.asarray(a, dtype=F64) for a in (Q, K, V, gamma))
    R = np.zeros((H, dk, dv), dtype=F64) if S0 is None else np.array(S0, dtype=F64)
    O = np.zeros((T, H, dv), dtype=F64)
    for c0 in range(0, T, chunk):
        c1 = min(T, c0 + chunk)
        for h in range(H):
            beta = np.cumprod(gamma[c0:c1, h])
            q, k, v = Q[c0:c1, h], K[c0:c1, h], V[c0:c1, h]
            D = np.tril(beta[:, None] / beta[None, :])
            inner = (scale * (q @ k.T) * D) @ v
            cross = scale * (q @ R[h]) * beta[:, None]
            O[c0:c1, h] = inner + cross
            R[h] = k.T @ (v * (beta[-1] / beta)[:, None]) + beta[-1] * R[h]
    return O, R


def group_norm_heads(O, eps=1e-6):
    """GroupNorm_h of Eq. 7 with one group per head and no learned affine:
    every head's dv-vector is shifted to zero mean and scaled to unit variance
    (biased variance, eps inside the root). O [..., H, dv]."""
    O = np.asarray(O, dtype=F64)
    mu = O.mean(axis=-1, keepdims=True)
    var = ((O - mu) ** 2).mean(axis=-1, keepdims=True)
    return (O - mu) / np.sqrt(var + eps)


def mhgr(X, W_Q, W_K, W_V, W_gamma, W_G, W_O, H, tau, scale, eps=1e-6):
    """Multi-head gated retention (Eq. 7): (swish(X W_G) * GroupNorm_h(heads)) W_O
    with head_i = gRet(X) in its parallel form; no rotation Theta (the
    configurations use no positional encoding). X [T,dm] -> [T,dm]."""
    X = np.asarray(X, dtype=F64)
    T = X.shape[0]
    Q = (X @ np.asarray(W_Q, F64)).reshape(T, H, -1)
    K = (X @ np.asarray(W_K, F64)).reshape(T, H, -1)
    V = (X @ np.asarray(W_V, F64)).reshape(T, H, -1)
    Y = group_norm_heads(gret_parallel(Q, K, V, gret_decay(X, W_gamma, tau), scale), eps).reshape(T, -1)
    a = X @ np.asarray(W_G, F64)
    return ((a / (1.0 + np.exp(-a))) * Y) @ np.asarray(W_O, F64)


# ---------------------------------------------------------------- 8-bit global cache
def kv_quantise_int8(X):
    """Symmetric 8-bit codes of cache rows, one scale per (row, KV head).

    The paper only names 8-bit KV quantisation as the common remedy for cache
    size (section 1, the 65B example) and gives no scheme; this is the plain
    absmax one. For a row x of d numbers, all arithmetic in float32 because a
    rounding decides the integer:  a = max|x|,  scale = a / 127,
    code_e = round-half-even(x_e * (127 / a)) in [-127, 127]; a zero row has
    scale 0 and codes 0. X [..., d] -> (codes int8 [..., d], scale float32 [...]).
    """
    X = np.asarray(X, dtype=np.float32)
    a = np.abs(X).max(axis=-1)
    pos = a > 0
    safe = np.where(pos, a, np.float32(1))
    inv = np.where(pos, np.float32(127) / safe, np.float32(0)).astype(np.float32)
    scale = np.where(pos, a / np.float32(127), np.float32(0)).astype(np.float32)
    y = (X * inv[..., None]).astype(np.float32)
    codes = np.clip(np.rint(y), -127, 127).astype(np.int8)
    return codes, scale


def kv_dequantise_int8(codes, scale):
    """The values an 8-bit cache stands for: code * scale, exact in float64."""
    return np.asarray(codes, dtype=F64) * np.asarray(scale, dtype=F64)[..., None]


def cross_attn_int8(Q, Khat, Vhat, q_pos0, scale):
    """Eq. 3 over a cache that stores K^ and V^ as 8-bit codes: the rows are
    quantised when written and attention runs on the values the codes stand for."""
    Kq = kv_dequantise_int8(*kv_quantise_int8(Khat))
    Vq = kv_dequantise_int8(*kv_quantise_int8(Vhat))
    return cross_attn(Q, Kq, Vq, q_pos0, scale)


def cross_attn_int8_error_bound(Q, Khat, Vhat, scale):
    """A tight upper bound on |cross_attn_int8 - cross_attn| for every output element.

    Every element of a row moves by at most half a code step, h = max|row|/254
    (plus float32 rounding of the scale, covered by the 1.001), and a coded
    value never exceeds its row's maximum. With O = sum_j p_j v_j over the
    exact rows and O' = sum_j p'_j v'_j over the coded ones,
        O' - O = sum_j p'_j (v'_j - v_j) + sum_j (p'_j - p_j) v_j.
    The first sum is a convex combination of V moves: at most hv = max_j h(v_j).
    For the second, a score moves by at most D = scale * max_i ||q_i||_1 *
    max_j h(k_j), so p'_j is proportional to p_j * exp(delta_j) with |delta_j| <= D;
    the total variation between two such distributions is largest when a set of
    weight 1/(1 + e^D) moves up by D and the rest down by D, where it equals
    tanh(D/2), so sum_j |p'_j - p_j| <= 2 tanh(D/2). Total:
        hv + 2 tanh(D/2) max|V^|.
    Both terms are attained (rows sitting half a step off their codes), which is
    what the pins use to hold the bound from above and from below.
    """
    Q = np.asarray(Q, dtype=F64)
    vmax = np.abs(np.asarray(Vhat, dtype=F64)).max()
    hk = 1.001 * np.abs(np.asarray(Khat, dtype=F64)).max() / 254.0
    hv = 1.001 * vmax / 254.0
    D = scale * np.abs(Q).sum(axis=-1).max() * hk
    return hv + 2.0 * np.tanh(0.5 * D) * vmax


def kv_cache_bytes_per_token(Hkv, d, elem_bytes, cached_layers=1):
    """Bytes of K plus V kept per token. YOCO keeps one global pair whatever the
    depth (cached_layers = 1, Table 1); a Transformer keeps one per layer."""
    return 2 * Hkv * d * elem_bytes * cached_layers
