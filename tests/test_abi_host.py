"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every symbol include/yoco.h declares, sizes the cache as the paper's Table 1
says (one K/V pair per token whatever the depth), and rejects bad arguments
before anything is launched."""
import ctypes as C
import os
import re

import pytest

import paper_2405_05254_amd as yoco
from paper_2405_05254_amd import binding as yb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "yoco.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(yoco_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = yoco.lib()
    names = declared_symbols()
    assert {"yoco_swa_prefill", "yoco_global_kv_write", "yoco_cross_attn_prefill", "yoco_cross_attn_decode"} <= set(names)
    for n in names:
        assert hasattr(L, n), n
    assert yoco.version() >= 100


def test_cache_bytes_follow_table_1():
    # bytes per token = 2 * Hkv * d * sizeof, independent of the number of layers
    assert yoco.kv_cache_bytes(1, 8, 128, 1, yoco.BF16) == 4096
    assert yoco.kv_cache_bytes(1, 8, 128, 524288, yoco.BF16) == 2147483648     # 512K-token cache
    assert yoco.kv_cache_bytes(16, 8, 128, 32768, yoco.BF16) == 2147483648     # 16 x 32K
    assert yoco.kv_cache_bytes(1, 16, 128, 131072, yoco.BF16) == 1073741824
    assert yoco.kv_cache_bytes(1, 1, 64, 512, yoco.F32) == 2 * 512 * 64 * 4
    # the paper's 65B example (section 4.4): 128K tokens per GiB
    assert 2 ** 30 // yoco.kv_cache_bytes(1, 16, 128, 1, yoco.BF16) == 131072


def test_cache_init_fills_descriptor_and_checks_memory():
    L = yoco.lib()
    d = yb._Cache()
    need = yoco.kv_cache_bytes(2, 4, 64, 100, yoco.BF16)
    base = 0x7f0000000000          # never dereferenced by the host-only call
    assert L.yoco_kv_cache_init(base, need, 2, 4, 64, 100, yoco.BF16, C.byref(d)) == 0
    assert d.k == base and d.v == base + need // 2 and (d.B, d.Hkv, d.d, d.N_cap) == (2, 4, 64, 100)
    assert L.yoco_kv_cache_init(base, need - 1, 2, 4, 64, 100, yoco.BF16, C.byref(d)) == -4
    assert b"cache memory" in L.yoco_last_error_string()
    assert L.yoco_kv_cache_init(base + 16, need, 2, 4, 64, 100, yoco.BF16, C.byref(d)) == -3
    assert L.yoco_kv_cache_init(None, need, 2, 4, 64, 100, yoco.BF16, C.byref(d)) == -1


@pytest.mark.parametrize("args,code", [
    ((0, 8, 128, 10, 1), -1), ((1, 8, 128, 0, 1), -1), ((1, 8, 12, 10, 1), -3),
    ((1, 8, 512, 10, 1), -2), ((1, 8, 128, 10, 7), -2),
])
def test_cache_bytes_rejects_bad_sizes(args, code):
    n = C.c_size_t()
    assert yoco.lib().yoco_kv_cache_bytes(*args, C.byref(n)) == code
    assert yoco.lib().yoco_last_error_string() != b""


def test_calls_validate_before_launching():
    """Every failure below is found on the host: nothing reaches the GPU (there is none here)."""
    L = yoco.lib()
    p = 0x7f0000000000
    # swa_prefill
    assert L.yoco_swa_prefill(None, p, p, p, 1, 8, 4, 4, 64, 4, 1.0, 0, None) == -1
    assert L.yoco_swa_prefill(p, p, p, p, 1, 8, 6, 4, 64, 4, 1.0, 0, None) == -1      # Hq % Hkv
    assert L.yoco_swa_prefill(p, p, p, p, 1, 8, 4, 4, 64, 0, 1.0, 0, None) == -1      # window 0
    assert L.yoco_swa_prefill(p, p, p, p, 1, 0, 4, 4, 64, 4, 1.0, 0, None) == -1      # T 0
    assert L.yoco_swa_prefill(p, p + 4, p, p, 1, 8, 4, 4, 64, 4, 1.0, 0, None) == -3  # alignment
    assert L.yoco_swa_prefill(p, p, p, p, 1, 8, 4, 4, 60, 4, 1.0, 0, None) == -3      # d % 8
    assert L.yoco_swa_prefill(p, p, p, p, 1, 8, 4, 4, 64, 4, 1.0, 5, None) == -2      # dtype
    d = yb._Cache()
    need = yoco.kv_cache_bytes(2, 2, 64, 100, yoco.BF16)
    assert L.yoco_kv_cache_init(p, need, 2, 2, 64, 100, yoco.BF16, C.byref(d)) == 0
    # global_kv_write
    assert L.yoco_global_kv_write(C.byref(d), p, p, 2, 0, 1, 1, None) == -1            # b out of range
    assert L.yoco_global_kv_write(C.byref(d), p, p, 0, 99, 2, 1, None) == -1           # beyond capacity
    assert L.yoco_global_kv_write(C.byref(d), p, p, 0, -1, 1, 1, None) == -1
    assert L.yoco_global_kv_write(C.byref(d), None, None, 0, 5, 0, 1, None) == 0       # empty write is a no-op
    assert L.yoco_global_kv_write(None, p, p, 0, 0, 1, 1, None) == -1
    # cross_attn_prefill
    assert L.yoco_cross_attn_prefill(C.byref(d), p, p, 0, 98, 4, 4, 1.0, None, 0, None) == -1   # beyond capacity
    assert L.yoco_cross_attn_prefill(C.byref(d), p, p, 0, 0, 0, 4, 1.0, None, 0, None) == -1
    assert L.yoco_cross_attn_prefill(C.byref(d), p, p, 0, 0, 4, 3, 1.0, None, 0, None) == -1    # Hq % Hkv
    assert L.yoco_cross_attn_prefill(C.byref(d), p, p, 0, 0, 4, 4, 1.0, p + 4, 1 << 20, None) == -3   # workspace alignment
    # decode: workspace sizing and checks
    n, s = C.c_size_t(), C.c_int()
    assert L.yoco_cross_attn_decode_workspace(C.byref(d), 4, C.byref(n), C.byref(s)) == 0
    assert s.value >= 1 and n.value == 2 * 4 * s.value * (64 + 4) * 4
    assert L.yoco_cross_attn_decode(C.byref(d), p, p, p, 4, 1.0, p, n.value - 1, None) == -4
    assert L.yoco_cross_attn_decode(C.byref(d), p, p, None, 4, 1.0, p, n.value, None) == -1
    assert b"null" in L.yoco_last_error_string()
    # the variant with the static scratch: arguments and size are refused on the host, before any device call
    assert L.yoco_cross_attn_decode_noalloc(C.byref(d), p, p, None, 4, 1.0, None) == -1
    assert L.yoco_cross_attn_decode_noalloc(None, p, p, p, 4, 1.0, None) == -1
    big = yb._Cache()
    big.k, big.v, big.B, big.Hkv, big.d, big.dtype, big.N_cap = p, p, 64, 8, 256, yoco.BF16, 100
    assert L.yoco_cross_attn_decode_workspace(C.byref(big), 64, C.byref(n), C.byref(s)) == 0
    assert n.value > yoco.NOALLOC_SCRATCH_BYTES
    assert L.yoco_cross_attn_decode_noalloc(C.byref(big), p, p, p, 64, 1.0, None) == -4
    assert b"static scratch" in L.yoco_last_error_string()


def test_decode_splits_fill_the_chip():
    L = yoco.lib()
    p = 0x7f0000000000
    for B, N in ((1, 524288), (16, 32768)):
        d = yb._Cache()
        assert L.yoco_kv_cache_init(p, yoco.kv_cache_bytes(B, 8, 128, N, yoco.BF16), B, 8, 128, N, yoco.BF16, C.byref(d)) == 0
        n, s = C.c_size_t(), C.c_int()
        assert L.yoco_cross_attn_decode_workspace(C.byref(d), 24, C.byref(n), C.byref(s)) == 0
        assert B * 8 * s.value >= 256           # at least one workgroup per CU (256 CUs)
        assert n.value < 0.01 * 2 * B * 8 * N * 128 * 2   # partials cost < 1 % of the cache bytes


def test_generation_calls_validate_before_launching():
    """The rolling-cache entry points: host-side failures only (no GPU here)."""
    L = yoco.lib()
    p = 0x7f0000000000
    d = yb._Cache()
    need = yoco.kv_cache_bytes(2, 2, 64, 16, yoco.BF16)
    assert L.yoco_kv_cache_init(p, need, 2, 2, 64, 16, yoco.BF16, C.byref(d)) == 0
    # swa_cache_write: positions may exceed the capacity (it is a ring), but not be negative
    assert L.yoco_swa_cache_write(C.byref(d), p, p, 0, -1, 1, 1, None) == -1
    assert L.yoco_swa_cache_write(C.byref(d), p, p, 2, 0, 1, 1, None) == -1             # b out of range
    assert L.yoco_swa_cache_write(C.byref(d), p, p, 0, 0, -3, 1, None) == -1
    assert L.yoco_swa_cache_write(C.byref(d), p, p + 8, 0, 0, 4, 1, None) == -3
    assert L.yoco_swa_cache_write(C.byref(d), p, p, 0, 0, 4, 7, None) == -2             # dtype
    assert L.yoco_swa_cache_write(C.byref(d), None, None, 0, 1000, 0, 1, None) == 0      # empty write is a no-op
    assert L.yoco_swa_cache_write(None, p, p, 0, 0, 1, 1, None) == -1
    # kv_cache_append
    assert L.yoco_kv_cache_append(C.byref(d), p, p, None, 1, 1, None) == -1
    assert L.yoco_kv_cache_append(C.byref(d), p, p, p + 4, 1, 1, None) == -3            # pos alignment
    assert L.yoco_kv_cache_append(C.byref(d), p + 2, p, p, 0, 1, None) == -3
    assert L.yoco_kv_cache_append(C.byref(d), p, p, p, 0, 9, None) == -2
    # swa_decode
    n, s = C.c_size_t(), C.c_int()
    assert L.yoco_cross_attn_decode_workspace(C.byref(d), 4, C.byref(n), C.byref(s)) == 0
    assert L.yoco_swa_decode(C.byref(d), p, None, None, p, p, 4, 1.0, p, n.value - 1, None) == -4
    assert L.yoco_swa_decode(C.byref(d), p, None, None, p, p, 3, 1.0, p, n.value, None) == -1       # Hq % Hkv
    assert L.yoco_swa_decode(C.byref(d), p, None, None, p, None, 4, 1.0, p, n.value, None) == -1
    assert L.yoco_swa_decode(C.byref(d), p, None, None, p, p, 4, 1.0, p + 1, n.value, None) == -3
    assert L.yoco_swa_decode(C.byref(d), p, p, None, p, p, 4, 1.0, p, n.value, None) == -1          # k_new without v_new
    assert L.yoco_swa_decode(C.byref(d), p, p, p + 8, p, p, 4, 1.0, p, n.value, None) == -3


def test_gated_retention_calls_validate_before_launching():
    L = yoco.lib()
    p = 0x7f0000000000
    n = C.c_size_t()
    # workspace sizing: only bf16, dk = dv = 128, chunk a multiple of 128 has a chunkwise path
    assert L.yoco_gret_prefill_workspace(1, 1000, 4, 128, 128, 256, yoco.BF16, C.byref(n)) == 0
    # cumulative decays, one fp32 state per chunk, two per segment (here every chunk is its own segment), and two
    # small decay tables, each rounded up to 256 bytes
    bh, nc, nseg, state = 4, 4, 4, 128 * 128 * 4
    up = lambda x: (x + 255) // 256 * 256
    assert n.value == up(bh * nc * 256 * 4) + up(bh * nc * state) + 2 * up(bh * nseg * state) + up(bh * nc * 4) + up(bh * nseg * 4)
    assert L.yoco_gret_prefill_workspace(1, 32768, 24, 128, 128, 256, yoco.BF16, C.byref(n)) == 0
    bh, nc, nseg = 24, 128, 32                      # long inputs: segments of 4 chunks
    assert n.value == up(bh * nc * 256 * 4) + up(bh * nc * state) + 2 * up(bh * nseg * state) + up(bh * nc * 4) + up(bh * nseg * 4)
    for args in ((1, 1000, 4, 64, 128, 256, yoco.BF16), (1, 1000, 4, 128, 128, 256, yoco.F32), (1, 1000, 4, 128, 128, 200, yoco.BF16)):
        assert L.yoco_gret_prefill_workspace(*args, C.byref(n)) == 0 and n.value == 0
    assert L.yoco_gret_prefill_workspace(1, 1000, 4, 128, 128, 0, yoco.BF16, C.byref(n)) == -1
    assert L.yoco_gret_prefill_workspace(1, 1000, 4, 100, 128, 256, yoco.BF16, C.byref(n)) == -3
    assert L.yoco_gret_prefill_workspace(1, 1000, 4, 128, 128, 256, yoco.BF16, None) == -1

    def prefill(q=p, k=p, v=p, g=p, o=p, s_in=None, s_out=None, B=1, T=10, H=2, dk=128, dv=128, chunk=256, eps=1e-6, dt=yoco.BF16,
                ws=None, wsb=0, gate=None):
        return L.yoco_gret_prefill(q, k, v, g, gate, o, s_in, s_out, B, T, H, dk, dv, chunk, 1.0, 1, eps, dt, ws, wsb, None)
    assert prefill(q=None) == -1
    assert prefill(g=None) == -1
    assert prefill(v=p + 8) == -3
    assert prefill(g=p + 2) == -3
    assert prefill(gate=p + 8) == -3
    assert prefill(s_in=p + 4) == -3
    assert prefill(ws=p + 16, wsb=1 << 30) == -3
    assert prefill(T=-1) == -1
    assert prefill(H=0) == -1
    assert prefill(chunk=0) == -1
    assert prefill(eps=-1.0) == -1
    assert prefill(dt=3) == -2
    assert prefill(dk=12) == -3
    assert prefill(dk=264) == -2
    assert prefill(dk=256, dv=256, dt=yoco.F32) == -2                  # valid dims, but no kernel above 128
    assert b"no kernel" in L.yoco_last_error_string()
    assert prefill(T=0, q=None, k=None, v=None, g=None, o=None) == 0   # empty prompt, no state to copy

    def decode(q=p, k=p, v=p, g=p, o=p, st=p, B=2, H=2, dk=128, dv=128, eps=1e-6, dt=yoco.BF16, gate=None):
        return L.yoco_gret_decode(q, k, v, g, gate, o, st, B, H, dk, dv, 1.0, 1, eps, dt, None)
    assert decode(st=None) == -1
    assert decode(o=p + 2) == -3
    assert decode(gate=p + 4) == -3
    assert decode(B=0) == -1
    assert decode(dv=4) == -3
    assert decode(dt=-1) == -2
    assert decode(dk=136, dt=yoco.F32) == -2


def test_eight_bit_cache_sizes_and_validation():
    """The 8-bit global cache: 64-row blocks of 8448 bytes, head_dim 128 only, no rolling use; host-side checks."""
    L = yoco.lib()
    p = 0x7f0000000000
    assert yoco.kv_cache_bytes(1, 1, 128, 64, yoco.INT8) == 2 * 8448
    assert yoco.kv_cache_bytes(1, 1, 128, 65, yoco.INT8) == 2 * 2 * 8448          # a started block is a whole block
    assert yoco.kv_cache_bytes(16, 8, 128, 32768, yoco.INT8) == 2 * 16 * 8 * 512 * 8448
    # 132 bytes per token, head and plane: 0.516 of the bf16 cache
    assert yoco.kv_cache_bytes(1, 8, 128, 524288, yoco.INT8) / yoco.kv_cache_bytes(1, 8, 128, 524288, yoco.BF16) == 132 / 256
    n = C.c_size_t()
    assert L.yoco_kv_cache_bytes(1, 8, 64, 100, yoco.INT8, C.byref(n)) == -2             # head_dim 128 only
    d = yb._Cache()
    need = yoco.kv_cache_bytes(2, 2, 128, 100, yoco.INT8)
    assert L.yoco_kv_cache_init(p, need, 2, 2, 128, 100, yoco.INT8, C.byref(d)) == 0
    assert d.k == p and d.v == p + need // 2 and d.dtype == yoco.INT8
    assert L.yoco_kv_cache_init(p, need - 1, 2, 2, 128, 100, yoco.INT8, C.byref(d)) == -4
    # writes and appends take f32 or bf16 rows; the usual range checks apply
    assert L.yoco_global_kv_write(C.byref(d), p, p, 0, 99, 2, 1, None) == -1
    assert L.yoco_global_kv_write(C.byref(d), p, p, 0, 0, 1, yoco.INT8, None) == -2       # rows are never given as codes
    assert L.yoco_global_kv_write(C.byref(d), None, None, 0, 5, 0, 1, None) == 0
    assert L.yoco_kv_cache_append(C.byref(d), p, p, p, 1, 1, None) == -2                  # no 8-bit ring
    assert b"rolling" in L.yoco_last_error_string()
    assert L.yoco_swa_cache_write(C.byref(d), p, p, 0, 0, 1, 1, None) == -2
    ws, s = C.c_size_t(), C.c_int()
    assert L.yoco_cross_attn_decode_workspace(C.byref(d), 4, C.byref(ws), C.byref(s)) == 0
    assert L.yoco_swa_decode(C.byref(d), p, None, None, p, p, 4, 1.0, p, ws.value, None) == -2
    # many-row prefill over the codes has no kernel; without a workspace the few-row form cannot run either
    assert L.yoco_cross_attn_prefill(C.byref(d), p, p, 0, 0, 50, 4, 1.0, None, 0, None) == -2
    assert L.yoco_cross_attn_prefill(C.byref(d), p, p, 0, 0, 2, 4, 1.0, None, 0, None) == -2
    assert b"8-bit" in L.yoco_last_error_string()
    # more than 16 query heads per KV head: refused before any launch
    assert L.yoco_cross_attn_decode_workspace(C.byref(d), 34, C.byref(ws), C.byref(s)) == 0
    assert L.yoco_cross_attn_decode(C.byref(d), p, p, p, 34, 1.0, p, ws.value, None) == -2
    assert L.yoco_cross_attn_decode(C.byref(d), p, p, p, 4, 1.0, p, 16, None) == -4
