"""The 8-bit global K^/V^ cache: codes and scales written by the library
bit-exactly against the oracle's float32 absmax rule (read back through the
documented block layout), and attention over the codes against the oracle's
fp64 attention over the same coded rows (bf16 bounds), and against the
uncoded rows within the oracle's derived error bound."""
import math

import numpy as np
import pytest
import torch

import oracle
import yoco_synth as ys

pytestmark = pytest.mark.gpu

TD = {"f32": torch.float32, "bf16": torch.bfloat16}
D = 128


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


def read_cache(cache):
    """(codes int16 [B,Hkv,NB*64,128], scales float32 [B,Hkv,NB*64]) of both planes, decoded from the documented block
    layout: 8192 code bytes in matrix-operand order (K signed, V as code + 128 and transposed), then 64 scales in row order."""
    r, e = np.meshgrid(np.arange(64), np.arange(D), indexing="ij")
    k_off = ((((r // 4) % 4) * 2 + e // 64) * 64 + ((e % 64) // 16) * 16 + 4 * (r // 16) + r % 4) * 16 + e % 16
    v_off = ((e // 16) * 64 + (r // 16) * 16 + e % 16) * 16 + r % 16
    assert len(np.unique(k_off)) == 8192 and len(np.unique(v_off)) == 8192       # both are permutations of the block
    out = []
    for plane, off, signed in zip(cache.blocks(), (k_off, v_off), (True, False)):
        raw = plane.cpu().numpy()
        B, Hkv, NB, _ = raw.shape
        by = raw[..., :8192][..., off]                                            # [B,Hkv,NB,64,128]
        codes = by.view(np.int8).astype(np.int16) if signed else by.astype(np.int16) - 128
        scales = np.ascontiguousarray(raw[..., 8192:]).view(np.float32).reshape(B, Hkv, NB * 64)
        out.append((codes.reshape(B, Hkv, NB * 64, D), scales))
    return out


def spread_rows(rng, shape, dtype):
    """Rows whose magnitudes span many binades, one all-zero, one with a single non-zero."""
    x = rng.standard_normal(shape) * np.exp2(rng.integers(-14, 14, size=shape[:-1]))[..., None]
    x[0, 0] = 0.0
    if shape[0] > 1:
        x[1, 0] = 0.0
        x[1, 0, 5] = -3.0
    return ys.round_to(x.astype(np.float32), dtype)


# ------------------------------------------------------------ coding rows (exact)
@pytest.mark.parametrize("src", ["f32", "bf16"])
@pytest.mark.parametrize("N_cap,pos0,n", [(64, 0, 64), (100, 0, 1), (100, 37, 63), (300, 60, 200), (1000, 999, 1), (130, 0, 0),
                                              (1000, 0, 1000), (640, 128, 512), (700, 1, 698)])
def test_global_kv_write_codes_are_exact(yoco, src, N_cap, pos0, n):
    B, Hkv = 2, 3
    rng = np.random.default_rng(N_cap * 7 + pos0 + n)
    cache = yoco.KVCache(B, Hkv, D, N_cap, torch.int8)
    cache.mem.fill_(0xAB)                                  # untouched bytes must stay as they are
    k = spread_rows(rng, (max(n, 2), Hkv, D), src)[:n]
    v = spread_rows(rng, (max(n, 2), Hkv, D), src)[:n]
    empty = torch.empty(0, Hkv, D, device="cuda", dtype=TD[src])
    yoco.global_kv_write(cache, dev(k, src) if n else empty, dev(v, src) if n else empty, 1, pos0)
    torch.cuda.synchronize()
    (kc, ks), (vc, vs) = read_cache(cache)
    for name, x, codes, scales in (("k", k, kc, ks), ("v", v, vc, vs)):
        if n:
            rc, rs = oracle.kv_quantise_int8(x.astype(np.float32))          # [n,Hkv,128], [n,Hkv]
            assert np.array_equal(codes[1, :, pos0:pos0 + n], rc.transpose(1, 0, 2).astype(np.int16)), name
            assert np.array_equal(scales[1, :, pos0:pos0 + n].view(np.uint32), rs.T.copy().view(np.uint32)), name
        # nothing else was written: sequence 0 and the rows around keep the fill pattern (0xAB as a K byte or as a V byte)
        fillc = 0xAB - 256 if name == "k" else 0xAB - 128
        assert np.all(codes[0] == fillc) and np.all(codes[1, :, :pos0] == fillc) and np.all(codes[1, :, pos0 + n:] == fillc)
        fill = np.frombuffer(bytes([0xAB] * 4), dtype=np.float32)[0]
        keep = np.ones(scales.shape, bool)
        keep[1, :, pos0:pos0 + n] = False
        assert np.all(scales[keep].view(np.uint32) == fill.view(np.uint32))


@pytest.mark.parametrize("src", ["f32", "bf16"])
@pytest.mark.parametrize("N_cap,pos0,n", [(300, 60, 200), (100, 37, 63), (640, 128, 512)])
def test_global_kv_write_scaled_codes_the_scaled_rows(yoco, src, N_cap, pos0, n):
    """The write that folds the norm of Eq. 2 over an 8-bit cache: every row is multiplied by its factor in float32 and
    then coded by the same rule, so codes and scales equal the oracle's quantiser on float32(x * factor), bit for bit
    (block-aligned runs and ragged head / tail rows take different kernels)."""
    B, Hkv = 2, 3
    rng = np.random.default_rng(N_cap + pos0 + n)
    cache = yoco.KVCache(B, Hkv, D, N_cap, torch.int8)
    cache.mem.fill_(0xAB)
    k = spread_rows(rng, (n, Hkv, D), src)
    v = spread_rows(rng, (n, Hkv, D), src)
    rs = np.exp2(rng.uniform(-3, 3, size=n)).astype(np.float32)
    yoco.global_kv_write_scaled(cache, dev(k, src), dev(v, src), torch.from_numpy(rs).cuda(), 1, pos0)
    torch.cuda.synchronize()
    (kc, ks), (vc, vs) = read_cache(cache)
    for name, x, codes, scales in (("k", k, kc, ks), ("v", v, vc, vs)):
        scaled = (x.astype(np.float32) * rs[:, None, None]).astype(np.float32)
        rc, rsc = oracle.kv_quantise_int8(scaled)
        assert np.array_equal(codes[1, :, pos0:pos0 + n], rc.transpose(1, 0, 2).astype(np.int16)), name
        assert np.array_equal(scales[1, :, pos0:pos0 + n].view(np.uint32), rsc.T.copy().view(np.uint32)), name
        fillc = 0xAB - 256 if name == "k" else 0xAB - 128
        assert np.all(codes[0] == fillc) and np.all(codes[1, :, :pos0] == fillc) and np.all(codes[1, :, pos0 + n:] == fillc)


def test_append_codes_rows_at_device_positions(yoco):
    B, Hkv, N_cap = 5, 2, 200
    rng = np.random.default_rng(11)
    cache = yoco.KVCache(B, Hkv, D, N_cap, torch.int8)
    cache.mem.fill_(0x11)
    k = spread_rows(rng, (B, Hkv, D), "bf16")
    v = spread_rows(rng, (B, Hkv, D), "bf16")
    pos = np.array([0, 63, 64, -1, 200], dtype=np.int64)      # the last two are skipped: negative, beyond the capacity
    yoco.kv_cache_append(cache, dev(k, "bf16"), dev(v, "bf16"), torch.from_numpy(pos).cuda(), False)
    torch.cuda.synchronize()
    (kc, ks), (vc, vs) = read_cache(cache)
    for x, codes, scales, fillc in ((k, kc, ks, 0x11), (v, vc, vs, 0x11 - 128)):
        rc, rs = oracle.kv_quantise_int8(x.astype(np.float32))
        for b in range(3):
            assert np.array_equal(codes[b, :, pos[b]], rc[b].astype(np.int16))
            assert np.array_equal(scales[b, :, pos[b]].view(np.uint32), rs[b].view(np.uint32))
            other = np.ones(codes.shape[2], bool)
            other[pos[b]] = False
            assert np.all(codes[b][:, other] == fillc)
        assert np.all(codes[3:] == fillc)
    with pytest.raises(yoco.YocoError):
        yoco.kv_cache_append(cache, dev(k, "bf16"), dev(v, "bf16"), torch.from_numpy(pos).cuda(), True)


# ------------------------------------------------------------ attention over the codes
def decode_case(yoco, seed, B, Hq, Hkv, N_cap, lens, std=1.0, want_splits=None):
    scale = 1.0 / math.sqrt(D)
    rng = np.random.default_rng(seed)
    cache = yoco.KVCache(B, Hkv, D, N_cap, torch.int8)
    cache.mem.fill_(0xFF)                                   # unwritten scales read as NaN: masked rows must not leak
    K = ys.normal(rng, (B, N_cap, Hkv, D), std, "bf16")
    V = ys.normal(rng, (B, N_cap, Hkv, D), std, "bf16")
    q = ys.normal(rng, (B, Hq, D), std, "bf16")
    for b in range(B):
        n = max(int(lens[b]), 0)
        if n:
            yoco.global_kv_write(cache, dev(K[b, :n], "bf16"), dev(V[b, :n], "bf16"), b, 0)
    nbytes, splits = yoco.cross_attn_decode_workspace(cache, Hq)
    if want_splits is not None:
        assert splits == want_splits, (splits, want_splits)
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    o = host(yoco.cross_attn_decode(cache, dev(q, "bf16"), torch.tensor(lens, dtype=torch.int64, device="cuda"), scale, ws))
    assert np.isfinite(o).all()
    tol = ys.TOL["bf16"]
    for b in range(B):
        n = min(max(int(lens[b]), 0), N_cap)
        if n == 0:
            assert np.all(o[b] == 0)
            continue
        ref = oracle.cross_attn_int8(q[b:b + 1], K[b, :n], V[b, :n], n - 1, scale)[0]
        st = ys.error_stats(o[b], ref)
        print("int8 decode seed %d b %d len %d splits %d: max_abs %.3e mean_rel %.3e" % (seed, b, n, splits, st["max_abs"], st["mean_rel"]),
              flush=True)
        big = max(1.0, float(np.abs(ref).max()))             # the bf16 output's own rounding grows with its magnitude
        assert st["max_abs"] <= tol["max_abs"] * big and st["mean_rel"] <= tol["mean_rel"], st
        exact = oracle.cross_attn(q[b:b + 1], K[b, :n], V[b, :n], n - 1, scale)[0]
        bound = oracle.cross_attn_int8_error_bound(q[b:b + 1], K[b, :n], V[b, :n], scale)
        assert np.abs(o[b] - exact).max() <= bound + tol["max_abs"] * big
    return o


@pytest.mark.parametrize("Hq,Hkv", [(2, 2), (4, 2), (6, 2), (8, 2), (10, 2), (16, 2), (32, 2), (13, 1)])
def test_decode_over_codes_every_group_size(yoco, Hq, Hkv):
    decode_case(yoco, 100 + Hq, 3, Hq, Hkv, 700, [700, 333, 64])


def test_decode_over_codes_ragged_lengths_and_block_edges(yoco):
    decode_case(yoco, 7, 10, 6, 2, 520, [0, 1, 63, 64, 65, 255, 256, 257, 520, 9999])


@pytest.mark.parametrize("B,Hkv,N_cap,lens,splits", [
    (2, 2, 500, [500, 123], 1),              # a cache of under 512 rows is never split
    (2, 2, 5000, [5000, 1234], 10),          # ceil(5000 / 512) rows-limited splits
    (1, 1, 40000, [40000], 79),
    (1, 1, 140000, [139999], 256),           # one workgroup per CU: the most a launch uses
])
def test_decode_over_codes_any_split_count(yoco, B, Hkv, N_cap, lens, splits):
    """The split count follows from the shape (one workgroup per CU, at least 512 rows per split): shapes that give
    1, 10, 79 and 256 splits, ragged last splits included."""
    decode_case(yoco, 20 + splits, B, 3 * Hkv, Hkv, N_cap, lens, want_splits=splits)


def test_decode_over_codes_large_and_small_magnitudes(yoco):
    decode_case(yoco, 31, 2, 6, 2, 600, [600, 77], std=8.0)
    decode_case(yoco, 32, 2, 6, 2, 600, [600, 77], std=0.01)


def test_decode_is_reproducible_and_does_not_touch_the_cache(yoco):
    scale = 1.0 / math.sqrt(D)
    rng = np.random.default_rng(5)
    cache = yoco.KVCache(2, 2, D, 3000, torch.int8)
    cache.mem.zero_()
    K = ys.normal(rng, (3000, 2, D), 1.0, "bf16")
    for b in range(2):
        yoco.global_kv_write(cache, dev(K, "bf16"), dev(K[::-1].copy(), "bf16"), b, 0)
    before = cache.mem.clone()
    q = dev(ys.normal(rng, (2, 6, D), 1.0, "bf16"), "bf16")
    lens = torch.tensor([3000, 2999], dtype=torch.int64, device="cuda")
    nbytes, _ = yoco.cross_attn_decode_workspace(cache, 6)
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    a = yoco.cross_attn_decode(cache, q, lens, scale, ws).clone()
    ws.fill_(0x7F)
    b = yoco.cross_attn_decode(cache, q, lens, scale, ws)
    assert torch.equal(a, b) and torch.equal(cache.mem, before)


def test_exit_rows_over_codes(yoco):
    """The few-row form of cross_attn_prefill (the exit row of an early-exit prefill) over an 8-bit cache."""
    scale = 1.0 / math.sqrt(D)
    T, Hq, Hkv = 900, 6, 2
    q, k, v = ys.qkv(9, T, Hq, Hkv, D, 1.0, "bf16")
    cache = yoco.KVCache(2, Hkv, D, T, torch.int8)
    cache.mem.fill_(0xFF)
    yoco.global_kv_write(cache, dev(k, "bf16"), dev(v, "bf16"), 1, 0)
    nbytes, _ = yoco.cross_attn_decode_workspace(cache, Hq)
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    o = host(yoco.cross_attn_prefill(cache, dev(q[T - 3:], "bf16"), 1, T - 3, scale, workspace=ws))
    ref = oracle.cross_attn_int8(q[T - 3:], k, v, T - 3, scale)
    st = ys.error_stats(o, ref)
    print("int8 exit rows: max_abs %.3e mean_rel %.3e" % (st["max_abs"], st["mean_rel"]), flush=True)
    assert st["max_abs"] <= ys.TOL["bf16"]["max_abs"] and st["mean_rel"] <= ys.TOL["bf16"]["mean_rel"]
    with pytest.raises(yoco.YocoError):                      # many rows: no kernel reads codes for a whole prefill
        yoco.cross_attn_prefill(cache, dev(q[:64], "bf16"), 1, 0, scale, workspace=ws)


def test_full_size_decode_over_codes_sampled(yoco):
    """16 sequences x 32768 rows, 24:8 heads, the launch the benchmark times: three (sequence, KV head) pairs
    against the oracle. Rows are drawn on the device and coded by the library; the oracle codes the same rows."""
    B, N, Hq, Hkv = 16, 32768, 24, 8
    scale = 1.0 / math.sqrt(D)
    cache = yoco.KVCache(B, Hkv, D, N, torch.int8)
    rows = {}
    for b in range(B):
        k = ys.device_normal((N, Hkv, D), 1000 + b, 1.0, torch.bfloat16, "cuda")
        v = ys.device_normal((N, Hkv, D), 2000 + b, 1.0, torch.bfloat16, "cuda")
        yoco.global_kv_write(cache, k, v, b, 0)
        if b in (0, 7, 15):
            rows[b] = (host(k), host(v))
    q = ys.device_normal((B, Hq, D), 3, 1.0, torch.bfloat16, "cuda")
    lens_h = [N - 37 * b for b in range(B)]
    lens = torch.tensor(lens_h, dtype=torch.int64, device="cuda")
    nbytes, splits = yoco.cross_attn_decode_workspace(cache, Hq)
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    o = host(yoco.cross_attn_decode(cache, q, lens, scale, ws))
    qh = host(q)
    G = Hq // Hkv
    for b, g in ((0, 0), (7, 3), (15, 7)):
        n = lens_h[b]
        K, V = rows[b]
        ref = oracle.cross_attn_int8(qh[b:b + 1, g * G:(g + 1) * G], K[:n, g:g + 1], V[:n, g:g + 1], n - 1, scale)[0]
        st = ys.error_stats(o[b, g * G:(g + 1) * G], ref)
        print("int8 full-size decode (b %d, g %d), %d splits: max_abs %.3e mean_rel %.3e" % (b, g, splits, st["max_abs"], st["mean_rel"]),
              flush=True)
        assert st["max_abs"] <= ys.TOL["bf16"]["max_abs"] and st["mean_rel"] <= ys.TOL["bf16"]["mean_rel"], st


# ------------------------------------------------------------ the stack over an 8-bit global cache
def test_stack_with_coded_cache_prefill_and_generation(yoco):
    """A small bf16 stack (head_dim 128, window 64) whose global cache holds 8-bit codes: early-exit prefill of 150
    tokens, then 30 decode steps, against the fp64 oracle stack that codes its K^, V^ rows the same way; and the
    distance to the stack with an uncoded cache, which the codes may move only a little."""
    from paper_2405_05254_amd.stack import YocoStack
    s = dict(d_model=256, Hq=4, Hkv_self=2, Hkv=2, d=128, n_self=2, n_cross=2, window=64, ffn=512, vocab=500, eps=1e-6)
    w = ys.stack_weights(21, s, "bf16")
    T0, steps = 150, 30
    tok = ys.tokens(22, T0 + steps, s["vocab"])
    ref8 = oracle.yoco_stack(tok, dict(w, cache_bits=8), "full")
    ref = oracle.yoco_stack(tok, w, "full")
    t = torch.from_numpy(tok).cuda()
    out = {}
    for name, cdt in (("int8", torch.int8), ("bf16", None)):
        st = YocoStack(w, torch.bfloat16, cache_dtype=cdt)
        state = st.new_generation_state(T0 + steps)
        logits = [host(st.prefill(t[:T0], state))[0]]
        for i in range(steps):
            logits.append(host(st.decode_step(t[T0 + i], state))[0])
        out[name] = np.stack(logits)
    big = np.abs(ref).max()
    e8 = np.abs(out["int8"] - ref8[T0 - 1:]).max()
    e16 = np.abs(out["bf16"] - ref[T0 - 1:]).max()
    moved = np.abs(ref8 - ref).max()
    print("stack, coded cache vs its oracle %.3e; uncoded cache vs its oracle %.3e; codes move the oracle's logits by %.3e (scale %.3f)"
          % (e8, e16, moved, big), flush=True)
    # bf16 kernels and bf16 K^, V^ rows (coded after that rounding, which can flip a code here and there)
    assert e8 <= 0.02 * big and e16 <= 0.02 * big
    assert moved <= 0.02 * big
