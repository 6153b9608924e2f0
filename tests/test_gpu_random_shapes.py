"""Randomly drawn small shapes (fixed seeds) for every call, against the fp64
oracle: lengths around the tile and chunk sizes, windows from 1 to beyond T,
GQA ratios with and without a fast path, head dims with and without one,
ragged batches. Same tolerances as the other parity tests."""
import math

import numpy as np
import pytest
import torch

import oracle
import yoco_synth as ys

pytestmark = pytest.mark.gpu

TD = {"f32": torch.float32, "bf16": torch.bfloat16}


@pytest.fixture(scope="module")
def yoco():
    import paper_2405_05254_amd as y
    y.lib()
    assert torch.cuda.is_available()
    return y


def dev(a, dtype):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda").to(TD[dtype])


def host(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def check(got, ref, dtype, what, relative=False):
    unit = max(1.0, float(np.abs(ref).max())) if relative else 1.0
    st = ys.error_stats(got / unit, ref / unit)
    tol = ys.TOL[dtype]
    assert np.isfinite(got).all(), what
    assert st["max_abs"] <= tol["max_abs"] and st["mean_rel"] <= tol["mean_rel"], (what, st)


def draw_heads(rng):
    Hkv = int(rng.integers(1, 4))
    return Hkv * int(rng.choice([1, 1, 2, 3, 4, 5, 7, 8, 12, 16])), Hkv


def draw_len(rng, hi=420):
    """Lengths that favour the neighbourhoods of 64 / 128 / 256."""
    base = int(rng.choice([1, 32, 63, 64, 65, 127, 128, 129, 192, 255, 256, 257, 320, 383, 384]))
    return max(1, min(hi, base + int(rng.integers(-1, 2))))


@pytest.mark.parametrize("seed", range(24))
def test_swa_prefill_random_shape(yoco, seed):
    rng = np.random.default_rng(1000 + seed)
    dtype = "bf16" if seed % 3 else "f32"
    d = 128 if (dtype == "bf16" and seed % 4) else int(rng.choice([32, 64, 72, 128]))
    Hq, Hkv = draw_heads(rng)
    B, T = int(rng.integers(1, 3)), draw_len(rng)
    window = int(rng.choice([1, 2, 31, 64, 65, 100, 128, 200, T, T + 50]))
    scale = 1.0 / math.sqrt(d)
    what = "swa %s" % ((dtype, B, T, Hq, Hkv, d, window),)
    print(what, flush=True)
    q = ys.normal(rng, (B, T, Hq, d), 1.0, dtype)
    k = ys.normal(rng, (B, T, Hkv, d), 1.0, dtype)
    v = ys.normal(rng, (B, T, Hkv, d), 1.0, dtype)
    o = host(yoco.swa_prefill(dev(q, dtype), dev(k, dtype), dev(v, dtype), window, scale))
    for b in range(B):
        check(o[b], oracle.swa(q[b], k[b], v[b], window, scale), dtype, what)


@pytest.mark.parametrize("seed", range(16))
def test_cache_write_prefill_and_decode_random_shape(yoco, seed):
    """Rows written in two pieces, then causal prefill rows and a decode step over the same cache."""
    rng = np.random.default_rng(2000 + seed)
    dtype = "bf16" if seed % 3 else "f32"
    d = 128 if (dtype == "bf16" and seed % 4) else int(rng.choice([32, 64, 128]))
    Hq, Hkv = draw_heads(rng)
    B = int(rng.integers(1, 4))
    N_cap = draw_len(rng, 700) + int(rng.integers(0, 300))
    lens = [int(rng.integers(1, N_cap + 1)) for _ in range(B)]
    scale = 1.0 / math.sqrt(d)
    what = "cache %s" % ((dtype, B, Hq, Hkv, d, N_cap, lens),)
    print(what, flush=True)
    cache = yoco.KVCache(B, Hkv, d, N_cap, TD[dtype])
    for p in cache.planes():
        p.fill_(float("nan"))
    K = [ys.normal(rng, (n, Hkv, d), 1.0, dtype) for n in lens]
    V = [ys.normal(rng, (n, Hkv, d), 1.0, dtype) for n in lens]
    for b, n in enumerate(lens):
        cut = int(rng.integers(0, n + 1))
        yoco.global_kv_write(cache, dev(K[b][:cut], dtype), dev(V[b][:cut], dtype), b, 0)
        yoco.global_kv_write(cache, dev(K[b][cut:], dtype), dev(V[b][cut:], dtype), b, cut)
    qd = ys.normal(rng, (B, Hq, d), 1.0, dtype)
    nbytes, _ = yoco.cross_attn_decode_workspace(cache, Hq)
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    od = host(yoco.cross_attn_decode(cache, dev(qd, dtype), torch.tensor(lens, dtype=torch.int64, device="cuda"), scale, ws))
    for b, n in enumerate(lens):
        check(od[b], oracle.cross_attn(qd[b:b + 1], K[b], V[b], n - 1, scale)[0], dtype, what + " decode b=%d" % b)
        Tq = int(rng.integers(1, min(n, 150) + 1))
        q_pos0 = n - Tq
        qp = ys.normal(rng, (Tq, Hq, d), 1.0, dtype)
        op = host(yoco.cross_attn_prefill(cache, dev(qp, dtype), b, q_pos0, scale, workspace=ws if seed % 2 else None))
        check(op, oracle.cross_attn(qp, K[b], V[b], q_pos0, scale), dtype, what + " prefill b=%d Tq=%d" % (b, Tq))


@pytest.mark.parametrize("seed", range(12))
def test_coded_cache_random_shape(yoco, seed):
    """8-bit global cache: rows written in pieces of mixed source dtypes plus one appended row per sequence, then a
    decode step and a few exit rows, against the oracle's attention over its own codes of the same rows."""
    rng = np.random.default_rng(5000 + seed)
    d = 128
    Hkv = int(rng.integers(1, 4))
    Hq = Hkv * int(rng.choice([1, 2, 3, 4, 5, 8, 16]))
    B = int(rng.integers(1, 4))
    N_cap = draw_len(rng, 700) + int(rng.integers(0, 300))
    lens = [int(rng.integers(1, N_cap + 1)) for _ in range(B)]
    std = float(rng.choice([0.05, 1.0, 6.0]))
    scale = 1.0 / math.sqrt(d)
    what = "coded cache %s" % ((B, Hq, Hkv, N_cap, lens, std),)
    print(what, flush=True)
    cache = yoco.KVCache(B, Hkv, d, N_cap, torch.int8)
    cache.mem.fill_(0xFF)
    K = [ys.normal(rng, (n, Hkv, d), std, "bf16") for n in lens]
    V = [ys.normal(rng, (n, Hkv, d), std, "bf16") for n in lens]
    for b, n in enumerate(lens):                       # all rows but the last: two pieces, one given as f32 and one as bf16
        cut = int(rng.integers(0, n))
        yoco.global_kv_write(cache, dev(K[b][:cut], "f32"), dev(V[b][:cut], "f32"), b, 0)
        yoco.global_kv_write(cache, dev(K[b][cut:n - 1], "bf16"), dev(V[b][cut:n - 1], "bf16"), b, cut)
    pos = torch.tensor([n - 1 for n in lens], dtype=torch.int64, device="cuda")
    yoco.kv_cache_append(cache, dev(np.stack([K[b][-1] for b in range(B)]), "bf16"), dev(np.stack([V[b][-1] for b in range(B)]), "bf16"),
                         pos, False)
    qd = ys.normal(rng, (B, Hq, d), 1.0, "bf16")
    nbytes, _ = yoco.cross_attn_decode_workspace(cache, Hq)
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    od = host(yoco.cross_attn_decode(cache, dev(qd, "bf16"), pos + 1, scale, ws))
    for b, n in enumerate(lens):
        check(od[b], oracle.cross_attn_int8(qd[b:b + 1], K[b], V[b], n - 1, scale)[0], "bf16", what + " decode b=%d" % b, relative=True)
        Tq = int(rng.integers(1, min(n, 8) + 1))
        qp = ys.normal(rng, (Tq, Hq, d), 1.0, "bf16")
        op = host(yoco.cross_attn_prefill(cache, dev(qp, "bf16"), b, n - Tq, scale, workspace=ws))
        check(op, oracle.cross_attn_int8(qp, K[b], V[b], n - Tq, scale), "bf16", what + " exit rows b=%d Tq=%d" % (b, Tq), relative=True)


@pytest.mark.parametrize("seed", range(12))
def test_rolling_cache_decode_random_shape(yoco, seed):
    rng = np.random.default_rng(3000 + seed)
    dtype = "bf16" if seed % 2 else "f32"
    d = 128 if dtype == "bf16" else int(rng.choice([32, 64]))
    Hq, Hkv = draw_heads(rng)
    C = int(rng.choice([1, 7, 64, 100, 128, 300]))
    B = int(rng.integers(1, 4))
    lens = [int(rng.integers(1, 3 * C + 20)) for _ in range(B)]
    scale = 1.0 / math.sqrt(d)
    what = "ring %s" % ((dtype, B, Hq, Hkv, d, C, lens),)
    print(what, flush=True)
    ring = yoco.KVCache(B, Hkv, d, C, TD[dtype])
    for p in ring.planes():
        p.fill_(float("nan"))
    K = [ys.normal(rng, (n, Hkv, d), 1.0, dtype) for n in lens]
    V = [ys.normal(rng, (n, Hkv, d), 1.0, dtype) for n in lens]
    for b, n in enumerate(lens):
        cut = int(rng.integers(0, n))
        yoco.swa_cache_write(ring, dev(K[b][:cut], dtype), dev(V[b][:cut], dtype), b, 0)
        yoco.swa_cache_write(ring, dev(K[b][cut:n - 1], dtype), dev(V[b][cut:n - 1], dtype), b, cut)
    ln = torch.tensor(lens, dtype=torch.int64, device="cuda")
    yoco.kv_cache_append(ring, dev(np.stack([K[b][-1] for b in range(B)]), dtype), dev(np.stack([V[b][-1] for b in range(B)]), dtype),
                         ln - 1, True)
    q = ys.normal(rng, (B, Hq, d), 1.0, dtype)
    nbytes, _ = yoco.cross_attn_decode_workspace(ring, Hq)
    o = host(yoco.swa_decode(ring, dev(q, dtype), ln, scale, torch.empty(nbytes, dtype=torch.uint8, device="cuda")))
    for b, n in enumerate(lens):
        Qb = np.zeros((n, Hq, d), dtype=np.float32)
        Qb[n - 1] = q[b]
        ref = np.stack([oracle.swa_row(Qb, K[b], V[b], n - 1, h, C, scale) for h in range(Hq)])
        check(o[b], ref, dtype, what + " b=%d" % b)


@pytest.mark.parametrize("seed", range(16))
def test_gated_retention_random_shape(yoco, seed):
    rng = np.random.default_rng(4000 + seed)
    dtype = "bf16" if seed % 4 else "f32"
    chunked = dtype == "bf16" and seed % 2 == 1
    dk, dv = (128, 128) if chunked else (int(rng.choice([32, 64, 128])), int(rng.choice([32, 64, 72, 128])))
    B, H = int(rng.integers(1, 3)), int(rng.integers(1, 4))
    T = draw_len(rng, 700) + int(rng.integers(0, 300))
    chunk = int(rng.choice([128, 256, 384, 512]))
    gn, carry = bool(rng.integers(0, 2)), bool(rng.integers(0, 2))
    scale = 1.0 / math.sqrt(dk)
    what = "gret %s" % ((dtype, chunked, B, T, H, dk, dv, chunk, gn, carry),)
    print(what, flush=True)
    q, k, v, lg = ys.gret_inputs(4000 + seed, B, T, H, dk, dv, 1.0, dtype, mean_log_decay=float(rng.choice([0.004, 0.04, 0.3])))
    S0 = rng.standard_normal((B, H, dv, dk)).astype(np.float32) if carry else None
    s_out = torch.empty(B, H, dv, dk, dtype=torch.float32, device="cuda")
    ws = None
    if chunked:
        nbytes = yoco.gret_prefill_workspace(B, T, H, dk, dv, chunk, yoco.BF16)
        assert nbytes > 0
        ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    o = yoco.gret_prefill(dev(q, dtype), dev(k, dtype), dev(v, dtype), torch.from_numpy(lg).cuda(), scale, chunk=chunk, group_norm=gn,
                          state_in=None if S0 is None else torch.from_numpy(S0).cuda(), state_out=s_out, workspace=ws)
    torch.cuda.synchronize()
    refs_o, refs_s = [], []
    for b in range(B):
        s0 = None if S0 is None else np.transpose(S0[b], (0, 2, 1))
        ro, rs = oracle.gret_recurrent(q[b], k[b], v[b], np.exp(lg[b].astype(np.float64)), scale, S0=s0)
        refs_o.append(oracle.group_norm_heads(ro, 1e-6) if gn else ro)
        refs_s.append(np.transpose(rs, (0, 2, 1)))
    check(host(o), np.stack(refs_o), dtype, what, relative=not gn)
    unit = max(1.0, float(np.abs(np.stack(refs_s)).max()))
    err = np.abs(host(s_out) - np.stack(refs_s)).max() / unit
    assert err <= (2e-3 if chunked else 1e-4), (what, err)
