"""Parity of the HIP path (through the C ABI) with the fp64 oracle, element by
element on the same seeded inputs. Tolerances: fp32 paths max-abs and
sum|err|/sum|ref| <= 1e-4; bf16 paths max-abs <= 2e-2 and sum-ratio <= 2e-3.
Sizes span several tiles and ragged tails; full-size cases sample outputs the
oracle computes one by one."""
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
    y.lib()                       # fails loudly if libyoco.so is not built
    assert torch.cuda.is_available()
    return y


def dev(a, dtype):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda").to(TD[dtype])


def host(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def check(got, ref, dtype, what):
    st = ys.error_stats(got, ref)
    tol = ys.TOL[dtype]
    print("%s: max_abs %.3e mean_rel %.3e" % (what, st["max_abs"], st["mean_rel"]), flush=True)
    assert np.isfinite(got).all(), what
    assert st["max_abs"] <= tol["max_abs"] and st["mean_rel"] <= tol["mean_rel"], (what, st)


# ------------------------------------------------------------------- SWA prefill
SWA_CASES = [
    # dtype, B, T, Hq, Hkv, d, window, std
    ("f32", 1, 512, 4, 4, 64, 128, 1.0),       # the tiny fp32 configuration
    ("f32", 2, 333, 6, 2, 32, 50, 1.0),        # ragged, GQA, batch
    ("f32", 1, 1, 2, 2, 64, 4, 1.0),           # a single token
    ("f32", 1, 70, 2, 1, 64, 1, 1.0),          # window 1: o = v
    ("f32", 1, 70, 2, 1, 72, 1000, 1.0),       # window >= T: full causal; d not a multiple of 64
    ("bf16", 1, 2500, 4, 2, 128, 1024, 0.5),   # several tiles + ragged tail, GQA
    ("bf16", 2, 1300, 3, 3, 128, 300, 0.5),    # window not a multiple of the tile
    ("bf16", 1, 777, 2, 2, 128, 5000, 1.0),    # window >= T
    ("bf16", 1, 640, 2, 2, 128, 64, 2.0),      # window smaller than a tile, peaky softmax
    ("bf16", 1, 129, 2, 1, 128, 128, 0.5),
    ("bf16", 1, 300, 2, 2, 64, 100, 0.5),      # bf16 shape without a fast path
    ("bf16", 1, 200, 2, 2, 128, 1, 0.5),       # window 1 on the MFMA path: o = v
    ("bf16", 3, 130, 2, 1, 128, 40, 0.5),      # batch of ragged two-tile sequences
    ("bf16", 1, 1500, 2, 2, 128, 700, 4.0),    # large scores: the running max keeps growing (rescale path)
    ("bf16", 1, 5, 1, 1, 128, 3, 1.0),         # fewer rows than a wavefront
]


@pytest.mark.parametrize("dtype,B,T,Hq,Hkv,d,window,std", SWA_CASES)
def test_swa_prefill_matches_oracle(yoco, dtype, B, T, Hq, Hkv, d, window, std):
    print("swa case", dtype, B, T, Hq, Hkv, d, window, flush=True)
    scale = 1.0 / math.sqrt(d)
    qs, ks, vs = zip(*[ys.qkv(100 + b, T, Hq, Hkv, d, std, dtype) for b in range(B)])
    if std > 2.0:                 # large scores, unit-scale values: the absolute bound is for outputs of order 1
        vs = tuple(v / np.float32(std) for v in vs)       # a power of two: still exact in bf16
    q, k, v = (dev(np.stack(x), dtype) for x in (qs, ks, vs))
    o = yoco.swa_prefill(q, k, v, window, scale)
    torch.cuda.synchronize()
    for b in range(B):
        ref = oracle.swa(qs[b], ks[b], vs[b], window, scale)
        check(host(o[b]), ref, dtype, "swa b=%d" % b)


def test_swa_scale_zero_and_negative_use_the_generic_path(yoco):
    """scale <= 0 is outside the MFMA kernel's domain (it tracks max(s) before scaling); the call still answers."""
    T, H, d, C = 150, 2, 128, 37
    qn, kn, vn = ys.qkv(7, T, H, H, d, 0.5, "bf16")
    for scale in (0.0, -0.05):
        o = yoco.swa_prefill(dev(qn[None], "bf16"), dev(kn[None], "bf16"), dev(vn[None], "bf16"), C, scale)
        torch.cuda.synchronize()
        check(host(o[0]), oracle.swa(qn, kn, vn, C, scale), "bf16", "swa scale %g" % scale)


def check_scaled(got, ref, what):
    """bf16 bounds with the absolute one scaled by the output's magnitude (the output's own rounding grows with it)."""
    st = ys.error_stats(got, ref)
    tol = ys.TOL["bf16"]
    big = max(1.0, float(np.abs(ref).max()))
    print("%s: max_abs %.3e (outputs up to %.3e) mean_rel %.3e" % (what, st["max_abs"], big, st["mean_rel"]), flush=True)
    assert np.isfinite(got).all(), what
    assert st["max_abs"] <= tol["max_abs"] * big and st["mean_rel"] <= tol["mean_rel"], (what, st)


def edge_values(seed, shape, kind):
    """V tensors at the two ends of the matrix-core path's documented domain, inside it: 'large' has |v| up to 6e4
    (fp16's largest finite value is 65504), 'small' has |v| around 1e-4, most of it above fp16's smallest normal 2^-14
    and part of it below (those elements lose low bits, at most 2^-25 each)."""
    rng = np.random.default_rng(seed)
    x = rng.standard_normal(shape).astype(np.float32)
    if kind == "large":
        v = ys.round_to(np.clip(x * np.float32(2.0e4), -6.0e4, 6.0e4), "bf16")
        assert np.abs(v).max() < 65504 and np.abs(v).max() > 5.9e4
    else:
        v = ys.round_to(x * np.float32(1.0e-4), "bf16")
        assert 0 < (np.abs(v) < 2.0 ** -14).mean() < 0.6
    return v


@pytest.mark.parametrize("kind", ["large", "small"])
def test_swa_prefill_at_the_edges_of_the_fp16_value_domain(yoco, kind):
    T, Hq, Hkv, d, C = 700, 4, 2, 128, 200
    scale = 1.0 / math.sqrt(d)
    qn, kn, _ = ys.qkv(300, T, Hq, Hkv, d, 1.0, "bf16")
    vn = edge_values(301, (T, Hkv, d), kind)
    o = yoco.swa_prefill(dev(qn[None], "bf16"), dev(kn[None], "bf16"), dev(vn[None], "bf16"), C, scale)
    torch.cuda.synchronize()
    ref = oracle.swa(qn, kn, vn, C, scale)
    if kind == "large":
        check_scaled(host(o[0]), ref, "swa |v| up to 6e4")
    else:                                                # compare in units of 1e-4 so that the bf16 bounds apply as they stand
        check(host(o[0]) * 1e4, ref * 1e4, "bf16", "swa |v| ~ 1e-4")


@pytest.mark.parametrize("kind", ["large", "small"])
def test_cross_attn_prefill_at_the_edges_of_the_fp16_value_domain(yoco, kind):
    Hq, Hkv, d, N, Tq = 6, 2, 128, 900, 400
    scale = 1.0 / math.sqrt(d)
    cache = yoco.KVCache(1, Hkv, d, N, torch.bfloat16)
    cache.mem.zero_()
    kn = ys.normal(np.random.default_rng(310), (N, Hkv, d), 1.0, "bf16")
    vn = edge_values(311, (N, Hkv, d), kind)
    yoco.global_kv_write(cache, dev(kn, "bf16"), dev(vn, "bf16"), 0, 0)
    qn = ys.normal(np.random.default_rng(312), (Tq, Hq, d), 1.0, "bf16")
    o = yoco.cross_attn_prefill(cache, dev(qn, "bf16"), 0, N - Tq, scale)
    torch.cuda.synchronize()
    ref = oracle.cross_attn(qn, kn, vn, N - Tq, scale)
    if kind == "large":
        check_scaled(host(o), ref, "cross prefill |v| up to 6e4")
    else:
        check(host(o) * 1e4, ref * 1e4, "bf16", "cross prefill |v| ~ 1e-4")


def test_swa_prefill_headline_shape_sampled(yoco):
    """T=32768, 24 heads, d=128, window 1024 (the benchmark's launch), checked on
    sampled (row, head) outputs including the window and tile edges."""
    c = ys.CONFIGS["swa_prefill_32k"]
    T, H, d, C = c["T"], c["Hq"], c["d"], c["window"]
    scale = 1.0 / math.sqrt(d)
    qn, kn, vn = ys.qkv(c["seed"], T, H, H, d, c["std"], "bf16")
    q, k, v = (dev(x[None], "bf16") for x in (qn, kn, vn))
    o = yoco.swa_prefill(q, k, v, C, scale)
    torch.cuda.synchronize()
    on = host(o[0])
    assert np.isfinite(on).all()
    rng = np.random.default_rng(5)
    rows = [0, 1, 63, 64, 127, 128, C - 1, C, C + 1, 2 * C, T - 129, T - 128, T - 1] + rng.integers(0, T, 180).tolist()
    got, ref = [], []
    for n, i in enumerate(rows):
        h = int(rng.integers(0, H)) if n >= 13 else n % H
        got.append(on[i, h])
        ref.append(oracle.swa_row(qn, kn, vn, i, h, C, scale))
    check(np.array(got), np.array(ref), "bf16", "swa 32k sampled")


# ------------------------------------------------- global KV write + cross prefill
def make_cache(yoco, B, Hkv, d, N_cap, dtype, seeds, n_rows, std=1.0):
    cache = yoco.KVCache(B, Hkv, d, N_cap, TD[dtype])
    cache.mem.zero_()
    ks, vs = [], []
    for b in range(B):
        rng = np.random.default_rng(seeds + b)
        kb, vb = ys.normal(rng, (n_rows[b], Hkv, d), std, dtype), ys.normal(rng, (n_rows[b], Hkv, d), std, dtype)
        ks.append(kb)
        vs.append(vb)
        # written in two pieces to exercise pos0
        cut = n_rows[b] // 3
        yoco.global_kv_write(cache, dev(kb[:cut], dtype), dev(vb[:cut], dtype), b, 0)
        yoco.global_kv_write(cache, dev(kb[cut:], dtype), dev(vb[cut:], dtype), b, cut)
    return cache, ks, vs


@pytest.mark.parametrize("dtype,src", [("f32", "f32"), ("bf16", "bf16"), ("bf16", "f32")])
def test_global_kv_write_layout_is_exact(yoco, dtype, src):
    B, Hkv, d, N = 2, 3, 64, 37
    cache = yoco.KVCache(B, Hkv, d, N, TD[dtype])
    cache.mem.zero_()
    rng = np.random.default_rng(3)
    k, v = ys.normal(rng, (20, Hkv, d), 1.0, src), ys.normal(rng, (20, Hkv, d), 1.0, src)
    yoco.global_kv_write(cache, dev(k, src), dev(v, src), 1, 9)
    torch.cuda.synchronize()
    Kp, Vp = (host(p) for p in cache.planes())
    expect_k, expect_v = np.zeros((B, Hkv, N, d)), np.zeros((B, Hkv, N, d))
    expect_k[1, :, 9:29] = ys.round_to(k, dtype).transpose(1, 0, 2)
    expect_v[1, :, 9:29] = ys.round_to(v, dtype).transpose(1, 0, 2)
    assert np.array_equal(Kp, expect_k) and np.array_equal(Vp, expect_v)   # bit-exact, nothing else touched


@pytest.mark.parametrize("dtype,src", [("f32", "f32"), ("bf16", "bf16"), ("bf16", "f32")])
def test_global_kv_write_scaled_folds_the_norm_of_eq2(yoco, dtype, src):
    """yoco_global_kv_write_scaled takes x (diag(g) W_K), x (diag(g) W_V) and 1 / rms(x) (oracle.global_kv_scaled_form)
    and must cache RMSNorm(x) W (oracle.global_kv): bit for bit the float32 product rounded once to the cache dtype
    (the rounding that decides the stored bits is taken in float32 on both sides), and within the dtype's bound of the
    fp64 Eq. 2; rows outside the write stay untouched and a null factor is the plain write."""
    B, Hkv, d, N, n, pos0, dm = 2, 3, 64, 50, 23, 11, 96
    rng = np.random.default_rng(71)
    X = rng.standard_normal((n, dm)) * 2.0
    g = 1.0 + 0.1 * rng.standard_normal(dm)
    WK, WV = (rng.standard_normal((dm, Hkv * d)) * 0.1 for _ in range(2))
    Kr, Vr, rs = oracle.global_kv_scaled_form(X, g, WK, WV, Hkv)
    kr, vr = ys.round_to(Kr, src), ys.round_to(Vr, src)              # what the caller's GEMM hands over, in its dtype
    rs32 = rs.astype(np.float32)
    cache = yoco.KVCache(B, Hkv, d, N, TD[dtype])
    cache.mem.zero_()
    yoco.global_kv_write_scaled(cache, dev(kr, src), dev(vr, src), torch.from_numpy(rs32).cuda(), 1, pos0)
    torch.cuda.synchronize()
    Kp, Vp = (host(p) for p in cache.planes())
    want_k = ys.round_to((kr.astype(np.float32) * rs32[:, None, None]).astype(np.float32), dtype).astype(np.float64)
    want_v = ys.round_to((vr.astype(np.float32) * rs32[:, None, None]).astype(np.float32), dtype).astype(np.float64)
    expect_k, expect_v = np.zeros((B, Hkv, N, d)), np.zeros((B, Hkv, N, d))
    expect_k[1, :, pos0:pos0 + n] = want_k.transpose(1, 0, 2)
    expect_v[1, :, pos0:pos0 + n] = want_v.transpose(1, 0, 2)
    assert np.array_equal(Kp, expect_k) and np.array_equal(Vp, expect_v)
    Kh, Vh = oracle.global_kv(X, g, WK, WV, Hkv)
    check(Kp[1, :, pos0:pos0 + n].transpose(1, 0, 2), Kh, "bf16" if "bf16" in (dtype, src) else "f32", "K^ of Eq. 2 via the scaled write")
    check(Vp[1, :, pos0:pos0 + n].transpose(1, 0, 2), Vh, "bf16" if "bf16" in (dtype, src) else "f32", "V^ of Eq. 2 via the scaled write")


CROSS_CASES = [
    # dtype, Hq, Hkv, d, N, q_pos0, Tq
    ("f32", 4, 1, 64, 512, 0, 512),        # the tiny fp32 configuration
    ("f32", 6, 3, 32, 200, 150, 50),
    ("bf16", 6, 2, 128, 1500, 0, 1500),
    ("bf16", 3, 1, 128, 1500, 800, 700),   # continuation chunk
    ("bf16", 4, 4, 128, 900, 899, 1),      # one query row
    ("bf16", 4, 2, 64, 300, 0, 300),
]


@pytest.mark.parametrize("dtype,Hq,Hkv,d,N,q_pos0,Tq", CROSS_CASES)
def test_cross_attn_prefill_matches_oracle(yoco, dtype, Hq, Hkv, d, N, q_pos0, Tq):
    print("cross case", dtype, Hq, Hkv, d, N, q_pos0, Tq, flush=True)
    scale = 1.0 / math.sqrt(d)
    cache, ks, vs = make_cache(yoco, 2, Hkv, d, N + 5, dtype, 40, [N, N])
    qn = ys.normal(np.random.default_rng(41), (Tq, Hq, d), 1.0, dtype)
    o = yoco.cross_attn_prefill(cache, dev(qn, dtype), 1, q_pos0, scale)
    torch.cuda.synchronize()
    check(host(o), oracle.cross_attn(qn, ks[1], vs[1], q_pos0, scale), dtype, "cross prefill")


@pytest.mark.parametrize("dtype,Hq,Hkv,d,N,q_pos0,Tq", [
    ("bf16", 6, 2, 128, 3000, 2999, 1),      # the exit row of an early-exit prefill
    ("bf16", 6, 2, 128, 3000, 1500, 5),
    ("bf16", 4, 4, 128, 700, 0, 8),          # rows 0..7: the first sees one key
    ("f32", 4, 1, 64, 512, 511, 1),
    ("bf16", 10, 2, 128, 900, 890, 3),       # G = 5: the 16-rows-per-step streaming kernel
    ("bf16", 22, 2, 128, 1900, 1890, 4),     # G = 11: two launches, 6 + 5 heads
])
def test_cross_attn_prefill_few_rows_with_workspace(yoco, dtype, Hq, Hkv, d, N, q_pos0, Tq):
    """With a workspace, calls of up to 8 rows are split over the cache like decode;
    the result is the same operation and is bit-identical to the decode call."""
    scale = 1.0 / math.sqrt(d)
    cache, ks, vs = make_cache(yoco, 2, Hkv, d, N, dtype, 60, [N, N])
    qn = ys.normal(np.random.default_rng(61), (Tq, Hq, d), 1.0, dtype)
    nbytes, _ = yoco.cross_attn_decode_workspace(cache, Hq)
    ws = torch.full((nbytes // 4,), float("nan"), dtype=torch.float32, device="cuda")
    o = yoco.cross_attn_prefill(cache, dev(qn, dtype), 1, q_pos0, scale, workspace=ws)
    o_plain = yoco.cross_attn_prefill(cache, dev(qn, dtype), 1, q_pos0, scale)
    torch.cuda.synchronize()
    ref = oracle.cross_attn(qn, ks[1], vs[1], q_pos0, scale)
    check(host(o), ref, dtype, "cross prefill, few rows, split")
    check(host(o_plain), ref, dtype, "cross prefill, few rows, one workgroup per head")


# ------------------------------------------------------------------------ decode
DECODE_CASES = [
    # dtype, Hq, Hkv, d, N_cap, lens
    ("f32", 4, 1, 64, 512, [512]),                       # the tiny fp32 configuration
    ("f32", 4, 2, 32, 300, [1, 300, 77]),
    ("bf16", 6, 2, 128, 5000, [5000, 1, 1237]),           # GQA 3:1
    ("bf16", 4, 4, 128, 70000, [69999]),                  # many splits, G = 1
    ("bf16", 8, 2, 128, 3000, [2049, 255]),               # G = 4
    ("bf16", 6, 2, 128, 600, [0, 600]),                   # an empty sequence gives zeros
    ("bf16", 10, 2, 128, 900, [900]),                     # G = 5: 16 rows per wavefront step
    ("bf16", 16, 2, 128, 4100, [4100, 33]),               # G = 8, several splits, a ragged tail
    ("bf16", 7, 1, 128, 2500, [2500, 1, 0]),              # G = 7
    ("bf16", 9, 1, 128, 1500, [1500, 129]),               # G = 9: two launches, 5 + 4 heads
    ("bf16", 32, 2, 128, 6000, [5999, 600]),              # G = 16: two launches of 8 heads
    ("bf16", 34, 2, 128, 600, [600]),                     # G = 17: beyond the streaming kernels (generic split kernels)
    ("bf16", 4, 2, 64, 400, [400, 13]),
    ("bf16", 4, 2, 128, 400, [0, 400, 17]),               # one split: pass 1 stores the output itself; an empty sequence
]


@pytest.mark.parametrize("dtype,Hq,Hkv,d,N_cap,lens", DECODE_CASES)
def test_cross_attn_decode_matches_oracle(yoco, dtype, Hq, Hkv, d, N_cap, lens):
    print("decode case", dtype, Hq, Hkv, d, N_cap, lens, flush=True)
    B = len(lens)
    scale = 1.0 / math.sqrt(d)
    cache, ks, vs = make_cache(yoco, B, Hkv, d, N_cap, dtype, 50, [N_cap] * B)   # rows past lens must be ignored
    qn = ys.normal(np.random.default_rng(51), (B, Hq, d), 1.0, dtype)
    nbytes, splits = yoco.cross_attn_decode_workspace(cache, Hq)
    ws = torch.full((nbytes // 4,), float("nan"), dtype=torch.float32, device="cuda")
    o = yoco.cross_attn_decode(cache, dev(qn, dtype), torch.tensor(lens, dtype=torch.int64, device="cuda"), scale, ws)
    torch.cuda.synchronize()
    on = host(o)
    for b, n in enumerate(lens):
        if n == 0:
            assert np.array_equal(on[b], np.zeros((Hq, d)))
            continue
        ref = oracle.cross_attn(qn[b:b + 1], ks[b], vs[b], n - 1, scale)[0]
        check(on[b], ref, dtype, "decode b=%d len=%d splits=%d" % (b, n, splits))
    # the merge is deterministic: a second call gives the same bits
    o2 = yoco.cross_attn_decode(cache, dev(qn, dtype), torch.tensor(lens, dtype=torch.int64, device="cuda"), scale, ws)
    assert torch.equal(o, o2)


@pytest.mark.parametrize("Hq,Hkv,std,N,lens", [
    (6, 2, 4.0, 3000, [3000, 2049, 31]),      # scores of +-100: a few rows carry all the weight, the running maximum keeps moving
    (16, 2, 4.0, 2100, [2100, 1]),            # the same with 8 heads per KV head
    (6, 2, 0.05, 1500, [1500, 700]),          # nearly uniform weights over the whole cache
    (32, 2, 1.0, 777, [777, 776]),            # 16 heads per KV head, lengths one apart around a step boundary
])
def test_cross_attn_decode_peaky_and_flat_weights(yoco, Hq, Hkv, std, N, lens):
    """The decode step at the two ends of the softmax: large scores (the output rescale runs often and P's bf16
    high part + remainder must carry weights that differ by many orders of magnitude) and nearly equal ones."""
    d, B = 128, len(lens)
    scale = 1.0 / math.sqrt(d)
    cache, ks, vs = make_cache(yoco, B, Hkv, d, N, "bf16", 150, [N] * B, std=std)
    qn = ys.normal(np.random.default_rng(151), (B, Hq, d), std, "bf16")
    nbytes, splits = yoco.cross_attn_decode_workspace(cache, Hq)
    ws = torch.full((nbytes // 4,), float("nan"), dtype=torch.float32, device="cuda")
    o = yoco.cross_attn_decode(cache, dev(qn, "bf16"), torch.tensor(lens, dtype=torch.int64, device="cuda"), scale, ws)
    torch.cuda.synchronize()
    on = host(o)
    for b, n in enumerate(lens):
        ref = oracle.cross_attn(qn[b:b + 1], ks[b], vs[b], n - 1, scale)[0]
        check_scaled(on[b], ref, "decode std=%g G=%d b=%d len=%d splits=%d" % (std, Hq // Hkv, b, n, splits))


def test_cross_attn_decode_full_size_eight_heads_per_kv_head(yoco):
    """A 65B-like head layout (64 query heads over 8 KV heads, section 4.4's GQA setting) on 4 x 32768 rows:
    four (sequence, KV head) pairs, all 8 heads of each, against the oracle on the same bits."""
    B, N, Hq, Hkv, d = 4, 32768, 64, 8, 128
    scale = 1.0 / math.sqrt(d)
    cache = yoco.KVCache(B, Hkv, d, N, torch.bfloat16)
    Kp, Vp = cache.planes()
    Kp.copy_(ys.device_normal(Kp.shape, 700, 1.0, torch.bfloat16, "cuda"))
    Vp.copy_(ys.device_normal(Vp.shape, 701, 1.0, torch.bfloat16, "cuda"))
    q = ys.device_normal((B, Hq, d), 702, 1.0, torch.bfloat16, "cuda")
    lens = torch.tensor([N, N - 1, 20000, N], dtype=torch.int64, device="cuda")
    nbytes, splits = yoco.cross_attn_decode_workspace(cache, Hq)
    o = yoco.cross_attn_decode(cache, q, lens, scale, torch.empty(nbytes, dtype=torch.uint8, device="cuda"))
    torch.cuda.synchronize()
    on, qn, G = host(o), host(q), Hq // Hkv
    got, ref = [], []
    for b, g in ((0, 0), (1, 3), (2, 5), (3, 7)):
        n = int(lens[b])
        Kh, Vh = host(Kp[b, g])[:, None, :], host(Vp[b, g])[:, None, :]
        for h in range(g * G, (g + 1) * G):
            got.append(on[b, h])
            ref.append(oracle.cross_attn_row(qn[b:b + 1, h:h + 1], Kh, Vh, 0, 0, n - 1, scale))
    check(np.array(got), np.array(ref), "bf16", "decode 4 x 32K, 64:8 heads, splits=%d" % splits)


@pytest.mark.parametrize("name", ["decode_b16_32k", "decode_b1_512k"])
def test_cross_attn_decode_full_size(yoco, name):
    """The benchmark's decode launches (16 x 32K and 1 x 512K caches, 24:8 heads),
    every output row checked against the oracle on the same bits."""
    c = ys.CONFIGS[name]
    B, N, Hq, Hkv, d = c["B"], c["N"], c["Hq"], c["Hkv"], c["d"]
    scale = 1.0 / math.sqrt(d)
    cache = yoco.KVCache(B, Hkv, d, N, torch.bfloat16)
    Kp, Vp = cache.planes()
    Kp.copy_(ys.device_normal(Kp.shape, c["seed"], c["std"], torch.bfloat16, "cuda"))
    Vp.copy_(ys.device_normal(Vp.shape, c["seed"] + 1, c["std"], torch.bfloat16, "cuda"))
    q = ys.device_normal((B, Hq, d), c["seed"] + 2, c["std"], torch.bfloat16, "cuda")
    lens = torch.full((B,), N, dtype=torch.int64, device="cuda")
    nbytes, splits = yoco.cross_attn_decode_workspace(cache, Hq)
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    o = yoco.cross_attn_decode(cache, q, lens, scale, ws)
    torch.cuda.synchronize()
    on, qn = host(o), host(q)
    got, ref = [], []
    G = Hq // Hkv
    for b in range(B):
        for g in range(Hkv):
            if B > 1 and (b * Hkv + g) % 5:      # 16 x 8 heads: every fifth (b, g) pair
                continue
            Kh, Vh = host(Kp[b, g])[:, None, :], host(Vp[b, g])[:, None, :]
            for h in range(g * G, (g + 1) * G):
                got.append(on[b, h])
                ref.append(oracle.cross_attn_row(qn[b:b + 1, h:h + 1], Kh, Vh, 0, 0, N - 1, scale))
    check(np.array(got), np.array(ref), "bf16", "%s splits=%d" % (name, splits))


# --------------------------------------------------------------- early-exit flow
def test_tiny_stack_early_exit_matches_full_and_oracle(yoco):
    from paper_2405_05254_amd.stack import YocoStack
    c = ys.CONFIGS["tiny_fp32"]
    w = ys.stack_weights(c["seed"], c["stack"], "f32")
    tok = ys.tokens(c["seed"], c["T"], c["stack"]["vocab"])
    st = YocoStack(w, torch.float32)
    t = torch.from_numpy(tok).cuda()
    full = host(st.forward_full(t))
    ee_dec = host(st.forward_early_exit(t, decode_kernel=True)[0])
    ee_pre = host(st.forward_early_exit(t, decode_kernel=False)[0])
    ref = oracle.yoco_stack(tok, w, "full")
    print("early-exit vs full (gpu): %.3e / %.3e; full vs oracle: %.3e" % (
        np.abs(ee_dec[0] - full[-1]).max(), np.abs(ee_pre[0] - full[-1]).max(), np.abs(full - ref).max()), flush=True)
    assert np.abs(ee_dec[0] - full[-1]).max() <= 1e-3     # the paper's early-exit invariant (Fig. 3)
    assert np.abs(ee_pre[0] - full[-1]).max() <= 1e-3
    assert np.abs(full - ref).max() <= 1e-3               # logits against the fp64 oracle stack
    assert np.abs(ee_dec[0] - oracle.yoco_stack(tok, w, "early_exit")[0]).max() <= 1e-3


def test_tiny_stack_with_the_norm_folded_into_the_cache_write(yoco):
    """The same stack with Eq. 2's RMSNorm folded into the cache write (raw rows times gain-scaled weights, 1 / rms on
    the write call): logits against the fp64 oracle stack and against the unfused GPU stack."""
    from paper_2405_05254_amd.stack import YocoStack
    c = ys.CONFIGS["tiny_fp32"]
    w = ys.stack_weights(c["seed"], c["stack"], "f32")
    w["kv"]["ln"] = (1.0 + 0.2 * np.random.default_rng(5).standard_normal(w["kv"]["ln"].shape)).astype(np.float32)   # a gain that matters
    tok = ys.tokens(c["seed"], c["T"], c["stack"]["vocab"])
    t = torch.from_numpy(tok).cuda()
    fused = host(YocoStack(w, torch.float32, fused_kv_norm=True).forward_full(t))
    plain = host(YocoStack(w, torch.float32).forward_full(t))
    ref = oracle.yoco_stack(tok, w, "full")
    print("fused-norm stack vs oracle %.3e, vs unfused stack %.3e" % (np.abs(fused - ref).max(), np.abs(fused - plain).max()), flush=True)
    assert np.abs(fused - ref).max() <= 1e-3
    assert np.abs(fused - plain).max() <= 1e-4


def test_bf16_stack_early_exit_matches_full(yoco):
    """The end-to-end architecture (d_model 2048, 16 x 128 heads, 12 + 12 layers,
    window 1024) at a reduced length above the window: early-exit logits against
    the GPU full forward."""
    from paper_2405_05254_amd.stack import YocoStack
    c = ys.CONFIGS["e2e_early_exit_128k"]
    s = dict(c["stack"], n_self=3, n_cross=3, vocab=4096)
    T = 3000
    w = ys.stack_weights(c["seed"], s, "bf16")
    tok = torch.from_numpy(ys.tokens(c["seed"], T, s["vocab"])).cuda()
    st = YocoStack(w, torch.bfloat16)
    full_last = host(st.forward_full(tok, rows=slice(T - 1, T)))
    ee = host(st.forward_early_exit(tok)[0])
    err = np.abs(ee - full_last).max()
    print("bf16 stack early-exit vs full: %.3e (logit scale %.3f)" % (err, np.abs(full_last).max()), flush=True)
    assert err <= 1e-3


def test_e2e_early_exit_128k(yoco):
    """End-to-end configuration at full size: random-init stack (d_model 2048,
    16 x 128 heads, 12 SWA + 12 cross layers, window 1024, FFN 5632, vocab
    32000), T = 131072, bf16 attention. The global cache is written once; the
    early-exit prefill sends only the last position through the cross-decoder
    and its logits are compared with the GPU full forward (a full-length fp64
    stack is out of reach: ~160 TFLOP). The kernels are checked against the
    oracle on the stack's real layer inputs: sampled SWA rows of the first and
    last self-decoder layers, sampled cross-attention rows of the last
    cross-decoder layer, and the decode call of the last position."""
    from paper_2405_05254_amd.stack import YocoStack
    c = ys.CONFIGS["e2e_early_exit_128k"]
    s, T = c["stack"], c["T"]
    H, d, C = s["Hq"], s["d"], s["window"]
    scale = 1.0 / math.sqrt(d)
    with torch.no_grad():
        w = ys.stack_weights_device(c["seed"], s, torch.bfloat16, "cuda")
        tok = torch.from_numpy(ys.tokens(c["seed"], T, s["vocab"])).cuda()
        st = YocoStack(w, torch.bfloat16)
        del w
        last_self = "self%d" % (s["n_self"] - 1)
        last_cross = "cross%d" % (s["n_cross"] - 1)
        st.capture = {"self0": None, last_self: None}
        print("e2e: self-decoder", flush=True)
        X = st.self_decoder(tok)
        cache = st.write_cache(X)
        swa_caps = dict(st.capture)
        st.capture = None
        x_last = X[T - 1:T].contiguous()
        print("e2e: early exit", flush=True)
        ee_dec = host(st.logits(st.cross_decoder_decode(x_last, cache, T)))
        ee_pre = host(st.logits(st.cross_decoder_rows(x_last, cache, T - 1)))
        print("e2e: full forward", flush=True)
        st.capture = {last_cross: None}
        XF = st.cross_decoder_rows(X, cache, 0)
        full_last = host(st.logits(XF[T - 1:T]))
        qc, oc = st.capture[last_cross]
        torch.cuda.synchronize()
    e_dec, e_pre = np.abs(ee_dec - full_last).max(), np.abs(ee_pre - full_last).max()
    print("e2e early-exit vs full forward, last-token logits: decode kernel %.3e, prefill kernel %.3e "
          "(max |logit| %.3f)" % (e_dec, e_pre, np.abs(full_last).max()), flush=True)
    assert np.isfinite(full_last).all()
    assert e_pre <= 1e-3 and e_dec <= 1e-3            # the early-exit invariant (Fig. 3)

    # ---- teacher-forced oracle checks on the real layer inputs
    rng = np.random.default_rng(9)
    for name, (q, k, v, o) in swa_caps.items():
        rows = [0, 1, C - 1, C, C + 1, 127, 128, T - 1] + rng.integers(0, T, 248).tolist()
        got, ref = [], []
        for i in rows:
            h = int(rng.integers(0, H))
            j0 = max(0, i - C + 1)
            # the window of row i, re-based to local row i - j0 (Eq. 8 on the slice)
            ref.append(oracle.swa_row(host(q[i:i + 1, h:h + 1]).repeat(i - j0 + 1, axis=0), host(k[j0:i + 1, h:h + 1]),
                                      host(v[j0:i + 1, h:h + 1]), i - j0, 0, C, scale))
            got.append(host(o[i, h]))
        check(np.array(got), np.array(ref), "bf16", "e2e %s sampled rows" % name)
    Kp, Vp = cache.planes()
    got, ref = [], []
    for i in [0, 63, 64, 4095, T // 2, T - 2, T - 1]:
        h = int(rng.integers(0, H))
        Kh, Vh = host(Kp[0, h, :i + 1])[:, None, :], host(Vp[0, h, :i + 1])[:, None, :]
        ref.append(oracle.cross_attn_row(host(qc[i:i + 1, h:h + 1]), Kh, Vh, 0, 0, i, scale))
        got.append(host(oc[i, h]))
    check(np.array(got), np.array(ref), "bf16", "e2e %s sampled rows" % last_cross)
