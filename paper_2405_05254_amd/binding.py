"""ctypes binding of include/yoco.h: same names, argument marshalling only."""
import ctypes as C
import os

import torch

F32, BF16, INT8 = 0, 1, 2
_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB = None


class YocoError(RuntimeError):
    pass


class _Cache(C.Structure):
    _fields_ = [("k", C.c_void_p), ("v", C.c_void_p), ("B", C.c_int32), ("Hkv", C.c_int32),
                ("d", C.c_int32), ("dtype", C.c_int32), ("N_cap", C.c_int64)]


def lib_path():
    """The in-tree libyoco.so (the only build this binding loads)."""
    return os.path.join(_PKG, "libyoco.so")


def lib():
    """Load libyoco.so (built by paper_2405_05254_amd/build.py); fail loudly if absent."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = lib_path()
    if not os.path.exists(path):
        raise YocoError("libyoco.so is not built: run `python -m paper_2405_05254_amd.build` "
                        "(or __graft_entry__.build()); there is no fallback path")
    L = C.CDLL(path)
    vp, i32, i64, f32, sz = C.c_void_p, C.c_int, C.c_int64, C.c_float, C.c_size_t
    L.yoco_version.restype = i32
    L.yoco_last_error_string.restype = C.c_char_p
    L.yoco_kv_cache_bytes.argtypes = [i32, i32, i32, i64, i32, C.POINTER(sz)]
    L.yoco_kv_cache_init.argtypes = [vp, sz, i32, i32, i32, i64, i32, C.POINTER(_Cache)]
    L.yoco_swa_prefill.argtypes = [vp, vp, vp, vp, i32, i64, i32, i32, i32, i64, f32, i32, vp]
    L.yoco_global_kv_write.argtypes = [C.POINTER(_Cache), vp, vp, i32, i64, i64, i32, vp]
    L.yoco_global_kv_write_scaled.argtypes = [C.POINTER(_Cache), vp, vp, vp, i32, i64, i64, i32, vp]
    L.yoco_cross_attn_prefill.argtypes = [C.POINTER(_Cache), vp, vp, i32, i64, i64, i32, f32, vp, sz, vp]
    L.yoco_cross_attn_decode_workspace.argtypes = [C.POINTER(_Cache), i32, C.POINTER(sz), C.POINTER(i32)]
    L.yoco_cross_attn_decode.argtypes = [C.POINTER(_Cache), vp, vp, vp, i32, f32, vp, sz, vp]
    L.yoco_cross_attn_decode_noalloc.argtypes = [C.POINTER(_Cache), vp, vp, vp, i32, f32, vp]
    L.yoco_swa_cache_write.argtypes = [C.POINTER(_Cache), vp, vp, i32, i64, i64, i32, vp]
    L.yoco_kv_cache_append.argtypes = [C.POINTER(_Cache), vp, vp, vp, i32, i32, vp]
    L.yoco_swa_decode.argtypes = [C.POINTER(_Cache), vp, vp, vp, vp, vp, i32, f32, vp, sz, vp]
    L.yoco_gret_prefill_workspace.argtypes = [i32, i64, i32, i32, i32, i32, i32, C.POINTER(sz)]
    L.yoco_gret_prefill.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, i32, i64, i32, i32, i32, i32, f32, i32, f32, i32, vp, sz, vp]
    L.yoco_gret_decode.argtypes = [vp, vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, f32, i32, f32, i32, vp]
    L.yoco_ceiling_mfma.argtypes = [vp, vp, i32, i32, vp]
    L.yoco_ceiling_attn_loop.argtypes = [vp, vp, i32, i32, i32, vp]
    L.yoco_ceiling_stream_read.argtypes = [vp, sz, vp, i32, vp]
    for name in ("yoco_ceiling_mfma", "yoco_ceiling_attn_loop", "yoco_ceiling_stream_read", "yoco_kv_cache_bytes", "yoco_kv_cache_init", "yoco_swa_prefill", "yoco_global_kv_write", "yoco_global_kv_write_scaled",
                 "yoco_cross_attn_prefill", "yoco_cross_attn_decode_workspace", "yoco_cross_attn_decode", "yoco_cross_attn_decode_noalloc",
                 "yoco_swa_cache_write", "yoco_kv_cache_append", "yoco_swa_decode",
                 "yoco_gret_prefill_workspace", "yoco_gret_prefill", "yoco_gret_decode"):
        getattr(L, name).restype = i32
    _LIB = L
    return L


def _check(rc):
    if rc != 0:
        raise YocoError("libyoco error %d: %s" % (rc, lib().yoco_last_error_string().decode()))


def _dtype(t):
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise YocoError("unsupported tensor dtype %s" % t.dtype)


def _dev(t, name):
    if not t.is_cuda:
        raise YocoError("%s must be a device tensor" % name)
    if not t.is_contiguous():
        raise YocoError("%s must be contiguous" % name)
    return t.data_ptr()


def _out(out, like, name="out"):
    """The output tensor: a fresh one shaped like `like`, or the caller's, which must be exactly that tensor's
    shape, dtype and device (the C ABI sees only a pointer and would write past a shorter or narrower buffer)."""
    if out is None:
        return torch.empty_like(like, memory_format=torch.contiguous_format)
    if out.shape != like.shape or out.dtype != like.dtype or out.device != like.device:
        raise YocoError("%s must be %s %s on %s, got %s %s on %s" % (name, tuple(like.shape), like.dtype, like.device,
                                                                    tuple(out.shape), out.dtype, out.device))
    return out


def _ws(workspace):
    """(pointer, bytes) of an optional workspace tensor on the current device."""
    if workspace is None:
        return None, 0
    ptr = _dev(workspace, "workspace")
    if workspace.device.index != torch.cuda.current_device():
        raise YocoError("workspace must live on the current device")
    return ptr, workspace.numel() * workspace.element_size()


def _stream():
    return torch.cuda.current_stream().cuda_stream


def version():
    return lib().yoco_version()


def kv_cache_bytes(B, Hkv, d, N_cap, dtype):
    n = C.c_size_t()
    _check(lib().yoco_kv_cache_bytes(B, Hkv, d, N_cap, dtype, C.byref(n)))
    return n.value


class KVCache:
    """The once-only global K^/V^ cache, or (N_cap = window) the rolling cache of one self-decoder layer:
    torch owns the memory, the descriptor is yoco_kv_cache."""

    def __init__(self, B, Hkv, d, N_cap, dtype=torch.bfloat16, device="cuda"):
        if dtype not in (torch.float32, torch.bfloat16, torch.int8):
            raise YocoError("unsupported cache dtype %s" % dtype)
        code = {torch.float32: F32, torch.bfloat16: BF16, torch.int8: INT8}[dtype]
        self.bytes = kv_cache_bytes(B, Hkv, d, N_cap, code)
        self.mem = torch.empty(self.bytes, dtype=torch.uint8, device=device)
        self.desc = _Cache()
        _check(lib().yoco_kv_cache_init(self.mem.data_ptr(), self.bytes, B, Hkv, d, N_cap, code, C.byref(self.desc)))
        self.B, self.Hkv, self.d, self.N_cap, self.dtype = B, Hkv, d, N_cap, dtype
        self.io_dtype = torch.bfloat16 if dtype == torch.int8 else dtype     # of the queries and outputs on this cache

    def planes(self):
        """Views [B,Hkv,N_cap,d] of the K and V planes (for tests and for filling synthetic caches)."""
        if self.dtype == torch.int8:
            raise YocoError("an 8-bit cache is a run of blocks, not a [B,Hkv,N_cap,d] array: use blocks()")
        half = self.bytes // 2
        shape = (self.B, self.Hkv, self.N_cap, self.d)
        return (self.mem[:half].view(self.dtype).view(shape), self.mem[half:].view(self.dtype).view(shape))

    def blocks(self):
        """Byte views [B,Hkv,ceil(N_cap/64),8448] of the K and V planes of an 8-bit cache: per block 8192 code bytes
        in the order yoco.h documents, then the 64 float32 scales of the block's rows."""
        if self.dtype != torch.int8:
            raise YocoError("blocks() is the layout of an 8-bit cache")
        half = self.bytes // 2
        shape = (self.B, self.Hkv, (self.N_cap + 63) // 64, 8448)
        return self.mem[:half].view(shape), self.mem[half:].view(shape)


def swa_prefill(q, k, v, window, scale, out=None):
    """q [B,T,Hq,d]; k, v [B,T,Hkv,d] -> o [B,T,Hq,d] (yoco_swa_prefill)."""
    B, T, Hq, d = q.shape
    Hkv = k.shape[2]
    if k.shape != (B, T, Hkv, d) or v.shape != k.shape or k.dtype != q.dtype or v.dtype != q.dtype:
        raise YocoError("q/k/v shapes or dtypes disagree")
    o = _out(out, q)
    _check(lib().yoco_swa_prefill(_dev(q, "q"), _dev(k, "k"), _dev(v, "v"), _dev(o, "o"), B, T, Hq, Hkv, d,
                                  window, scale, _dtype(q), _stream()))
    return o


def global_kv_write(cache, k, v, b, pos0):
    """k, v [n,Hkv,d] rows -> cache rows [pos0, pos0+n) of sequence b (yoco_global_kv_write)."""
    n = k.shape[0]
    if n and (k.shape != (n, cache.Hkv, cache.d) or v.shape != k.shape or v.dtype != k.dtype):
        raise YocoError("k/v rows do not match the cache")
    _check(lib().yoco_global_kv_write(C.byref(cache.desc), _dev(k, "k") if n else None, _dev(v, "v") if n else None,
                                      b, pos0, n, _dtype(k), _stream()))


def global_kv_write_scaled(cache, k, v, row_scale, b, pos0):
    """k, v [n,Hkv,d] un-normalised projections x (diag(g) W), row_scale float32 [n] = 1/rms(x): rows are scaled in
    float32 and stored like global_kv_write (yoco_global_kv_write_scaled)."""
    n = k.shape[0]
    if n and (k.shape != (n, cache.Hkv, cache.d) or v.shape != k.shape or v.dtype != k.dtype):
        raise YocoError("k/v rows do not match the cache")
    if row_scale.dtype != torch.float32 or row_scale.shape != (n,):
        raise YocoError("row_scale must be float32 [n]")
    _check(lib().yoco_global_kv_write_scaled(C.byref(cache.desc), _dev(k, "k") if n else None, _dev(v, "v") if n else None,
                                             _dev(row_scale, "row_scale") if n else None, b, pos0, n, _dtype(k), _stream()))


def cross_attn_prefill(cache, q, b, q_pos0, scale, out=None, workspace=None):
    """q [Tq,Hq,d] -> o [Tq,Hq,d], causal over the cache of sequence b (yoco_cross_attn_prefill).
    workspace: optional device scratch tensor (see cross_attn_decode_workspace) for few-row calls."""
    Tq, Hq, d = q.shape
    if d != cache.d or q.dtype != cache.io_dtype:
        raise YocoError("q does not match the cache")
    o = _out(out, q)
    ws_ptr, ws_bytes = _ws(workspace)
    _check(lib().yoco_cross_attn_prefill(C.byref(cache.desc), _dev(q, "q"), _dev(o, "o"), b, q_pos0, Tq, Hq, scale,
                                         ws_ptr, ws_bytes, _stream()))
    return o


def cross_attn_decode_workspace(cache, Hq):
    n, s = C.c_size_t(), C.c_int()
    _check(lib().yoco_cross_attn_decode_workspace(C.byref(cache.desc), Hq, C.byref(n), C.byref(s)))
    return n.value, s.value


def cross_attn_decode(cache, q, lens, scale, workspace, out=None):
    """q [B,Hq,d], lens int64 [B] (device) -> o [B,Hq,d] (yoco_cross_attn_decode)."""
    B, Hq, d = q.shape
    if B != cache.B or d != cache.d or q.dtype != cache.io_dtype:
        raise YocoError("q does not match the cache")
    if lens.dtype != torch.int64 or lens.shape != (B,):
        raise YocoError("lens must be int64 [B]")
    o = _out(out, q)
    _check(lib().yoco_cross_attn_decode(C.byref(cache.desc), _dev(q, "q"), _dev(o, "o"), _dev(lens, "lens"), Hq,
                                        scale, *_ws(workspace), _stream()))
    return o


NOALLOC_SCRATCH_BYTES = 4 << 20


def cross_attn_decode_noalloc(cache, q, lens, scale, out):
    """yoco_cross_attn_decode_noalloc: the decode step with the library's static scratch instead of a workspace.
    `out` is required (this wrapper allocates nothing either)."""
    B, Hq, d = q.shape
    if B != cache.B or d != cache.d or q.dtype != cache.io_dtype:
        raise YocoError("q does not match the cache")
    if lens.dtype != torch.int64 or lens.shape != (B,):
        raise YocoError("lens must be int64 [B]")
    if out is None:
        raise YocoError("out is required")
    o = _out(out, q)
    _check(lib().yoco_cross_attn_decode_noalloc(C.byref(cache.desc), _dev(q, "q"), _dev(o, "o"), _dev(lens, "lens"), Hq,
                                                scale, _stream()))
    return o


def swa_cache_write(ring, k, v, b, pos0):
    """k, v [n,Hkv,d] rows of positions pos0.. -> ring slots (pos0 + r) mod N_cap of sequence b (yoco_swa_cache_write)."""
    n = k.shape[0]
    if n and (k.shape != (n, ring.Hkv, ring.d) or v.shape != k.shape or v.dtype != k.dtype):
        raise YocoError("k/v rows do not match the cache")
    _check(lib().yoco_swa_cache_write(C.byref(ring.desc), _dev(k, "k") if n else None, _dev(v, "v") if n else None,
                                      b, pos0, n, _dtype(k), _stream()))


def kv_cache_append(cache, k, v, pos, ring):
    """k, v [B,Hkv,d], pos int64 [B] (device): one row per sequence at slot pos[b] (mod N_cap if ring)
    (yoco_kv_cache_append)."""
    if k.shape != (cache.B, cache.Hkv, cache.d) or v.shape != k.shape or v.dtype != k.dtype:
        raise YocoError("k/v rows do not match the cache")
    if pos.dtype != torch.int64 or pos.shape != (cache.B,):
        raise YocoError("pos must be int64 [B]")
    _check(lib().yoco_kv_cache_append(C.byref(cache.desc), _dev(k, "k"), _dev(v, "v"), _dev(pos, "pos"), int(bool(ring)),
                                      _dtype(k), _stream()))


def swa_decode(ring, q, lens, scale, workspace, out=None, k_new=None, v_new=None):
    """q [B,Hq,d], lens int64 [B] (device, tokens so far including the new one) -> o [B,Hq,d] (yoco_swa_decode).
    k_new, v_new [B,Hkv,d]: the new token's rows, stored by the same call; None when they were appended before."""
    B, Hq, d = q.shape
    if B != ring.B or d != ring.d or q.dtype != ring.dtype:
        raise YocoError("q does not match the cache")
    if lens.dtype != torch.int64 or lens.shape != (B,):
        raise YocoError("lens must be int64 [B]")
    if (k_new is None) != (v_new is None):
        raise YocoError("k_new and v_new go together")
    if k_new is not None and (k_new.shape != (B, ring.Hkv, d) or v_new.shape != k_new.shape or k_new.dtype != ring.dtype
                              or v_new.dtype != ring.dtype):
        raise YocoError("k_new/v_new do not match the cache")
    o = _out(out, q)
    _check(lib().yoco_swa_decode(C.byref(ring.desc), _dev(q, "q"), _dev(k_new, "k_new") if k_new is not None else None,
                                 _dev(v_new, "v_new") if v_new is not None else None, _dev(o, "o"), _dev(lens, "lens"), Hq, scale,
                                 *_ws(workspace), _stream()))
    return o


def gret_prefill_workspace(B, T, H, dk, dv, chunk, dtype):
    n = C.c_size_t()
    _check(lib().yoco_gret_prefill_workspace(B, T, H, dk, dv, chunk, dtype, C.byref(n)))
    return n.value


def _state(t, name, B, H, dk, dv):
    if t is None:
        return None
    if t.dtype != torch.float32 or t.shape != (B, H, dv, dk):
        raise YocoError("%s must be float32 [B,H,dv,dk]" % name)
    return _dev(t, name)


def gret_prefill(q, k, v, log_gamma, scale, chunk=256, group_norm=True, eps=1e-6, state_in=None, state_out=None,
                 workspace=None, out=None, gate=None):
    """q, k [B,T,H,dk]; v [B,T,H,dv]; log_gamma float32 [B,T,H] -> o [B,T,H,dv] (yoco_gret_prefill).
    States are float32 [B,H,dv,dk]; workspace: device tensor from gret_prefill_workspace bytes (None: recurrent path);
    gate: optional tensor like v, the output is multiplied by swish(gate)."""
    B, T, H, dk = q.shape
    dv = v.shape[3]
    if k.shape != q.shape or v.shape[:3] != q.shape[:3] or k.dtype != q.dtype or v.dtype != q.dtype:
        raise YocoError("q/k/v shapes or dtypes disagree")
    if log_gamma.dtype != torch.float32 or log_gamma.shape != (B, T, H):
        raise YocoError("log_gamma must be float32 [B,T,H]")
    if gate is not None and (gate.shape != v.shape or gate.dtype != v.dtype):
        raise YocoError("gate must match v")
    o = _out(out, v)
    ws_ptr, ws_bytes = _ws(workspace)
    _check(lib().yoco_gret_prefill(_dev(q, "q") if T else None, _dev(k, "k") if T else None, _dev(v, "v") if T else None,
                                   _dev(log_gamma, "log_gamma") if T else None,
                                   _dev(gate, "gate") if (T and gate is not None) else None, _dev(o, "o") if T else None,
                                   _state(state_in, "state_in", B, H, dk, dv), _state(state_out, "state_out", B, H, dk, dv),
                                   B, T, H, dk, dv, chunk, scale, int(bool(group_norm)), eps, _dtype(q), ws_ptr, ws_bytes,
                                   _stream()))
    return o


def gret_decode(q, k, v, log_gamma, state, scale, group_norm=True, eps=1e-6, out=None, gate=None):
    """q, k [B,H,dk]; v [B,H,dv]; log_gamma float32 [B,H]; state float32 [B,H,dv,dk], updated in place
    -> o [B,H,dv] (yoco_gret_decode)."""
    B, H, dk = q.shape
    dv = v.shape[2]
    if k.shape != q.shape or v.shape[:2] != q.shape[:2] or k.dtype != q.dtype or v.dtype != q.dtype:
        raise YocoError("q/k/v shapes or dtypes disagree")
    if log_gamma.dtype != torch.float32 or log_gamma.shape != (B, H):
        raise YocoError("log_gamma must be float32 [B,H]")
    if gate is not None and (gate.shape != v.shape or gate.dtype != v.dtype):
        raise YocoError("gate must match v")
    o = _out(out, v)
    _check(lib().yoco_gret_decode(_dev(q, "q"), _dev(k, "k"), _dev(v, "v"), _dev(log_gamma, "log_gamma"),
                                  _dev(gate, "gate") if gate is not None else None, _dev(o, "o"),
                                  _state(state, "state", B, H, dk, dv), B, H, dk, dv, scale, int(bool(group_norm)), eps,
                                  _dtype(q), _stream()))
    return o


def ceiling_mfma(seed, sink, iters, workgroups):
    """Launch the MFMA-only loop (yoco_ceiling_mfma); returns the flops of the launch."""
    _check(lib().yoco_ceiling_mfma(_dev(seed, "seed"), _dev(sink, "sink"), iters, workgroups, _stream()))
    return workgroups * 8 * 8 * iters * 32768.0


def ceiling_attn_loop(seed, sink, iters, workgroups, mode):
    """Launch the attention inner loop on its own (yoco_ceiling_attn_loop; mode 1: LDS-fed products, 2: with the
    softmax work); returns the flops of the launch."""
    _check(lib().yoco_ceiling_attn_loop(_dev(seed, "seed"), _dev(sink, "sink"), iters, workgroups, mode, _stream()))
    return workgroups * 8 * 32 * iters * 32768.0


def ceiling_stream_read(buf, sink, workgroups):
    """Launch the streaming read of `buf` (yoco_ceiling_stream_read); returns the bytes read."""
    nbytes = buf.numel() * buf.element_size()
    _check(lib().yoco_ceiling_stream_read(_dev(buf, "buf"), nbytes, _dev(sink, "sink"), workgroups, _stream()))
    return float(nbytes)
