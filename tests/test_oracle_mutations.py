"""The pins must be able to fail: each plausible mistake planted in a copy of
the oracle's attention (a wrong window bound, a dropped scale, a wrong GQA map,
a transposed operand, a missing max shift, softmax over the wrong axis ...) is
caught by the same kind of checks tests/test_oracle_pins.py applies to the real
oracle (dense brute force with the literal mask, torch's library attention,
closed forms). CPU only; nothing here touches the HIP path."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle


def make_attention(window_lo=lambda i, C: max(0, i - C + 1), window_hi=lambda i: i, use_scale=True, gqa=lambda h, G: h // G,
                   normalise=True, value_from_keys=False):
    """A copy of the oracle's row definition with switches for planted mistakes."""
    def attn(Q, K, V, C, scale):
        T, Hq, _ = Q.shape
        G = Hq // K.shape[1]
        O = np.zeros((T, Hq, V.shape[2]))
        for h in range(Hq):
            g = min(gqa(h, G), K.shape[1] - 1)
            for i in range(T):
                j0, j1 = window_lo(i, C), min(window_hi(i), T - 1)
                s = (scale if use_scale else 1.0) * (K[j0:j1 + 1, g] @ Q[i, h])
                p = np.exp(s - s.max())
                if normalise:
                    p = p / p.sum()
                O[i, h] = p @ (K if value_from_keys else V)[j0:j1 + 1, g]
        return O
    return attn


def library_reference(Q, K, V, C, scale):
    T = Q.shape[0]
    G = Q.shape[1] // K.shape[1]
    i, j = np.arange(T)[:, None], np.arange(T)[None, :]
    band = torch.from_numpy((j <= i) & (j > i - C))
    q = torch.from_numpy(Q).permute(1, 0, 2)[None]
    k = torch.from_numpy(K).permute(1, 0, 2).repeat_interleave(G, dim=0)[None]
    v = torch.from_numpy(V).permute(1, 0, 2).repeat_interleave(G, dim=0)[None]
    return F.scaled_dot_product_attention(q, k, v, attn_mask=band, scale=scale)[0].permute(1, 0, 2).numpy()


def battery(attn):
    """True if `attn` passes the pins (library attention on a GQA band case, window-1, equal keys)."""
    rng = np.random.default_rng(0)
    Q, K, V = rng.standard_normal((40, 4, 8)), rng.standard_normal((40, 2, 8)), rng.standard_normal((40, 2, 8))
    if np.abs(attn(Q, K, V, 7, 0.6) - library_reference(Q, K, V, 7, 0.6)).max() > 1e-12:
        return False
    if not np.array_equal(attn(Q, K, V, 1, 0.6), np.repeat(V, 2, axis=1)):
        return False
    Ke = np.broadcast_to(K[:1], K.shape).copy()
    O = attn(Q, Ke, V, 5, 0.6)
    for i in (0, 3, 20):
        if np.abs(O[i, 0] - V[max(0, i - 4):i + 1, 0].mean(axis=0)).max() > 1e-13:
            return False
    return True


def test_the_unmutated_copy_and_the_oracle_pass():
    assert battery(make_attention())
    assert battery(lambda Q, K, V, C, s: oracle.swa(Q, K, V, C, s))


MUTANTS = {
    "window one key too long": dict(window_lo=lambda i, C: max(0, i - C)),
    "window one key too short": dict(window_lo=lambda i, C: max(0, min(i, i - C + 2))),
    "not causal (sees the next key)": dict(window_hi=lambda i: i + 1),
    "scale dropped": dict(use_scale=False),
    "GQA map interleaved instead of grouped": dict(gqa=lambda h, G: h % 2),
    "GQA map always head 0": dict(gqa=lambda h, G: 0),
    "softmax not normalised": dict(normalise=False),
    "values taken from K": dict(value_from_keys=True),
}


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_pins_catch_planted_mistake(name):
    assert not battery(make_attention(**MUTANTS[name])), name


# ---- the rolling-window cache: planted mistakes in a copy of the ring
def make_ring_attention(slot=lambda p, C: p % C, first=lambda p, C: max(0, p - C + 1), slots_in_ring=lambda C: C):
    """Attention through a ring of slots, as a function with the signature of
    the battery's `attn`, with switches for planted mistakes."""
    def attn(Q, K, V, C, scale):
        T, Hq, _ = Q.shape
        G = Hq // K.shape[1]
        n = slots_in_ring(C)
        Kr, Vr = np.zeros((n,) + K.shape[1:]), np.zeros((n,) + V.shape[1:])
        O = np.zeros((T, Hq, V.shape[2]))
        for p in range(T):
            Kr[slot(p, C) % n], Vr[slot(p, C) % n] = K[p], V[p]
            idx = [slot(j, C) % n for j in range(first(p, C), p + 1)]
            for h in range(Hq):
                s = scale * (Kr[idx, h // G] @ Q[p, h])
                w = np.exp(s - s.max())
                O[p, h] = (w / w.sum()) @ Vr[idx, h // G]
        return O
    return attn


def oracle_ring(Q, K, V, C, scale):
    ring = oracle.RollingWindowCache(C, K.shape[1], K.shape[2])
    out = []
    for p in range(Q.shape[0]):
        ring.write(p, K[p], V[p])
        out.append(ring.attend(Q[p], p, scale))
    return np.stack(out)


def test_the_unmutated_ring_and_the_oracle_ring_pass():
    assert battery(make_ring_attention())
    assert battery(oracle_ring)


RING_MUTANTS = {
    "slot = p mod (C+1) with C slots": dict(slot=lambda p, C: p % (C + 1)),
    "ring one slot short": dict(slots_in_ring=lambda C: max(1, C - 1)),
    "gathers C+1 positions": dict(first=lambda p, C: max(0, p - C)),
    "gathers C-1 positions": dict(first=lambda p, C: max(0, min(p, p - C + 2))),
    "slot order reversed": dict(slot=lambda p, C: C - 1 - p % C, first=lambda p, C: max(0, p - C)),
}


@pytest.mark.parametrize("name", sorted(RING_MUTANTS))
def test_pins_catch_planted_ring_mistake(name):
    assert not battery(make_ring_attention(**RING_MUTANTS[name])), name


# ---- gated retention: planted mistakes in copies of the recurrent and chunkwise forms
def make_gret(first=lambda m: m + 1, decay_after_add=False, d_transposed=False, cross_decay=True, value_decay=True,
              carry_decay=True, chunk=5):
    """Returns (parallel, recurrent, chunkwise) copies with switches for planted mistakes."""
    def parallel(Q, K, V, gamma, scale):
        T, H, _ = Q.shape
        O = np.zeros((T, H, V.shape[2]))
        for h in range(H):
            D = np.zeros((T, T))
            for n in range(T):
                for m in range(n + 1):
                    D[n, m] = np.prod(gamma[first(m):n + 1, h])
            O[:, h] = (scale * (Q[:, h] @ K[:, h].T) * D) @ V[:, h]
        return O

    def recurrent(Q, K, V, gamma, scale):
        T, H, dk = Q.shape
        S = np.zeros((H, dk, V.shape[2]))
        O = np.zeros((T, H, V.shape[2]))
        for n in range(T):
            for h in range(H):
                kv = np.outer(K[n, h], V[n, h])
                S[h] = gamma[n, h] * (S[h] + kv) if decay_after_add else gamma[n, h] * S[h] + kv
                O[n, h] = scale * (Q[n, h] @ S[h])
        return O

    def chunkwise(Q, K, V, gamma, scale):
        T, H, dk = Q.shape
        R = np.zeros((H, dk, V.shape[2]))
        O = np.zeros((T, H, V.shape[2]))
        for c0 in range(0, T, chunk):
            c1 = min(T, c0 + chunk)
            for h in range(H):
                beta = np.cumprod(gamma[c0:c1, h])
                q, k, v = Q[c0:c1, h], K[c0:c1, h], V[c0:c1, h]
                D = np.tril(beta[None, :] / beta[:, None]) if d_transposed else np.tril(beta[:, None] / beta[None, :])
                O[c0:c1, h] = (scale * (q @ k.T) * D) @ v + scale * (q @ R[h]) * (beta[:, None] if cross_decay else 1.0)
                vd = v * (beta[-1] / beta)[:, None] if value_decay else v
                R[h] = k.T @ vd + (beta[-1] if carry_decay else 1.0) * R[h]
        return O
    return parallel, recurrent, chunkwise


def gret_battery(fn):
    """True if `fn(Q, K, V, gamma, scale)` passes the pins: scalar-loop brute force, gamma = 1 prefix sums."""
    rng = np.random.default_rng(3)
    T, H = 13, 2
    Q, K, V = rng.standard_normal((T, H, 4)), rng.standard_normal((T, H, 4)), rng.standard_normal((T, H, 3))
    gamma = 0.5 + 0.5 * rng.random((T, H))
    ref = np.zeros((T, H, 3))
    for h in range(H):
        for n in range(T):
            for m in range(n + 1):
                decay = 1.0
                for i in range(m + 1, n + 1):
                    decay *= gamma[i, h]
                ref[n, h] += 0.7 * decay * (Q[n, h] @ K[m, h]) * V[m, h]
    if np.abs(fn(Q, K, V, gamma, 0.7) - ref).max() > 1e-11:
        return False
    ones = np.ones((T, H))
    pre = np.stack([np.stack([Q[n, h] @ (K[:n + 1, h].T @ V[:n + 1, h]) for h in range(H)]) for n in range(T)])
    return np.abs(fn(Q, K, V, ones, 1.0) - pre).max() < 1e-11


def test_the_unmutated_gret_copies_and_the_oracle_pass():
    for fn in make_gret():
        assert gret_battery(fn)
    assert gret_battery(oracle.gret_parallel)
    assert gret_battery(lambda *a: oracle.gret_recurrent(*a)[0])
    assert gret_battery(lambda Q, K, V, g, s: oracle.gret_chunkwise(Q, K, V, g, s, 5)[0])
    assert gret_battery(lambda Q, K, V, g, s: oracle.gret_chunkwise(Q, K, V, g, s, 64)[0])


GRET_MUTANTS = {
    "decay product starts one row early": (0, dict(first=lambda m: m)),
    "decay product starts one row late": (0, dict(first=lambda m: m + 2)),
    "state decayed after the new term is added": (1, dict(decay_after_add=True)),
    "inner-chunk decay matrix with rows and columns exchanged (as Eq. 6 prints it)": (2, dict(d_transposed=True)),
    "cross-chunk term without its row decay": (2, dict(cross_decay=False)),
    "chunk state without the value decay": (2, dict(value_decay=False)),
    "chunk state carried without the chunk's total decay": (2, dict(carry_decay=False)),
}


@pytest.mark.parametrize("name", sorted(GRET_MUTANTS))
def test_pins_catch_planted_gret_mistake(name):
    which, kw = GRET_MUTANTS[name]
    assert not gret_battery(make_gret(**kw)[which]), name


# ---------------------------------------------------------------- 8-bit cache codes
def make_quantiser(levels=127.0, rounding=np.rint, axis=-1, clip=127, scale_levels=127.0):
    """A copy of the oracle's absmax quantiser with switches for planted mistakes."""
    def quant(X):
        X = np.asarray(X, dtype=np.float32)
        a = np.abs(X).max(axis=axis, keepdims=True)
        safe = np.where(a > 0, a, np.float32(1))
        inv = np.where(a > 0, np.float32(levels) / safe, np.float32(0)).astype(np.float32)
        scale = np.where(a > 0, a / np.float32(scale_levels), np.float32(0)).astype(np.float32)
        codes = np.clip(rounding((X * inv).astype(np.float32)), -clip, clip).astype(np.int8)
        if axis != -1:                                   # one scale per column of a row block, handed to every row
            scale = np.broadcast_to(scale.max(axis=-1, keepdims=True), X.shape[:-1] + (1,))
        return codes, np.ascontiguousarray(scale[..., 0])
    return quant


def quantiser_battery(quant):
    """True if `quant` passes the pins of the real quantiser (half-step property, extremes, oddness, ties)."""
    rng = np.random.default_rng(0)
    X = rng.standard_normal((30, 2, 64)).astype(np.float32)
    X *= np.exp2(rng.integers(-10, 10, size=(30, 2))).astype(np.float32)[..., None]
    codes, scale = quant(X)
    if scale.shape != (30, 2) or np.abs(codes.astype(np.int32)).max() > 127:
        return False
    a = np.abs(X).max(axis=-1).astype(np.float64)
    if np.abs(scale.astype(np.float64) / (a / 127.0) - 1).max() > 1e-6:
        return False
    err = np.abs(codes.astype(np.float64) * scale.astype(np.float64)[..., None] - X)
    if np.any(err > 0.5 * scale.astype(np.float64)[..., None] * (1 + 1e-5)):
        return False
    cn, _ = quant(-X)
    if not np.array_equal(cn, -codes):
        return False
    ties = np.array([[127.0, 0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 126.5]], dtype=np.float32)
    return quant(ties)[0].tolist() == [[127, 0, 2, 2, 0, -2, -2, 126]]


QUANT_MUTANTS = {
    "128 levels": dict(levels=128.0, clip=128, scale_levels=128.0),
    "codes use 128, scale uses 127": dict(levels=128.0),
    "truncation": dict(rounding=np.trunc),
    "floor": dict(rounding=np.floor),
    "round half away from zero": dict(rounding=lambda y: np.sign(y) * np.floor(np.abs(y) + 0.5)),
    "scale over the heads axis": dict(axis=-2),
    "clip at 126": dict(clip=126),
}


def test_the_unmutated_quantiser_and_the_oracle_pass():
    assert quantiser_battery(make_quantiser())
    assert quantiser_battery(oracle.kv_quantise_int8)
    rng = np.random.default_rng(5)
    X = rng.standard_normal((9, 3, 32)).astype(np.float32)
    c0, s0 = make_quantiser()(X)
    c1, s1 = oracle.kv_quantise_int8(X)
    assert np.array_equal(c0, c1) and np.array_equal(s0, s1)


@pytest.mark.parametrize("name", sorted(QUANT_MUTANTS))
def test_pins_catch_planted_quantiser_mistake(name):
    assert not quantiser_battery(make_quantiser(**QUANT_MUTANTS[name])), name


# ---------------------------------------------------------------- 8-bit cache: the error bound
def make_int8_bound(step_div=254.0, weight_term=lambda D: 2.0 * np.tanh(0.5 * D), q_norm=lambda Q: np.abs(Q).sum(axis=-1).max(),
                    v_step=True, v_mag=lambda V: np.abs(V).max(), use_scale=True):
    """A copy of the oracle's bound on |attention over codes - attention over the rows| with switches for planted mistakes."""
    def bound(Q, K, V, scale):
        Q, K, V = (np.asarray(x, dtype=np.float64) for x in (Q, K, V))
        hk = 1.001 * np.abs(K).max() / step_div
        hv = 1.001 * np.abs(V).max() / step_div
        D = (scale if use_scale else 1.0) * q_norm(Q) * hk
        return (hv if v_step else 0.0) + weight_term(D) * v_mag(V)
    return bound


def int8_bound_battery(bound):
    """True if `bound` holds from both sides on the constructed worst cases of tests/test_oracle_pins.py."""
    from test_oracle_pins import int8_bound_worst_case
    for D_target in (0.01, 0.05, 0.3):
        q, K, V, scale = int8_bound_worst_case(D_target)
        err = np.abs(oracle.cross_attn_int8(q, K, V, 1, scale) - oracle.cross_attn(q, K, V, 1, scale)).max()
        b = bound(q, K, V, scale)
        if not (0.90 * b <= err <= b):
            return False
    q, K, V, scale = int8_bound_worst_case(0.05)
    q0 = np.zeros_like(q)
    err0 = np.abs(oracle.cross_attn_int8(q0, K, V, 1, scale) - oracle.cross_attn(q0, K, V, 1, scale)).max()
    b0 = bound(q0, K, V, scale)
    return bool(0.99 * b0 <= err0 <= b0)


INT8_BOUND_MUTANTS = {
    "a whole code step instead of half": dict(step_div=127.0),
    "a quarter step": dict(step_div=508.0),
    "weights within exp(+-2D), summed (twice too loose)": dict(weight_term=lambda D: np.expm1(2.0 * D)),
    "tanh(D/2) without the factor 2": dict(weight_term=lambda D: np.tanh(0.5 * D)),
    "tanh(D/4)": dict(weight_term=lambda D: 2.0 * np.tanh(0.25 * D)),
    "largest |q| instead of the 1-norm": dict(q_norm=lambda Q: np.abs(Q).max()),
    "2-norm of q instead of the 1-norm": dict(q_norm=lambda Q: np.sqrt((Q ** 2).sum(axis=-1)).max()),
    "V step dropped": dict(v_step=False),
    "mean |V| instead of the largest": dict(v_mag=lambda V: np.abs(V).mean()),
    "softmax scale dropped": dict(use_scale=False),
}


def test_the_unmutated_int8_bound_and_the_oracle_pass():
    assert int8_bound_battery(make_int8_bound())
    assert int8_bound_battery(oracle.cross_attn_int8_error_bound)


@pytest.mark.parametrize("name", sorted(INT8_BOUND_MUTANTS))
def test_pins_catch_planted_int8_bound_mistake(name):
    assert not int8_bound_battery(make_int8_bound(**INT8_BOUND_MUTANTS[name])), name
