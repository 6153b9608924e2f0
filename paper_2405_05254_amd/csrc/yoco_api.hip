// C ABI of libyoco: argument validation and dispatch. No kernels here; the one device object is the static scratch
// array of yoco_cross_attn_decode_noalloc.
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>

#include <mutex>

#include "yoco_common.h"

namespace {

thread_local char g_err[256] = "";

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

int hip_result(hipError_t e, const char* what) {
  if (e == hipSuccess) return YOCO_OK;
  return fail(YOCO_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

bool aligned16(const void* p) { return (((uintptr_t)p) & 15u) == 0; }
size_t elem_bytes(int dtype) { return dtype == YOCO_F32 ? 4 : 2; }
bool dtype_ok(int dtype) { return dtype == YOCO_F32 || dtype == YOCO_BF16; }                 // tensors
bool cache_dtype_ok(int dtype) { return dtype_ok(dtype) || dtype == YOCO_INT8; }             // cache planes
int io_dtype(const yoco_kv_cache& c) { return c.dtype == YOCO_INT8 ? YOCO_BF16 : c.dtype; }  // of q and o on this cache
// Bytes of one sequence's share of a plane (all its KV heads).
size_t plane_bytes_per_seq(const yoco_kv_cache& c) {
  if (c.dtype == YOCO_INT8) return (size_t)c.Hkv * yoco::i8_plane_bytes(c.N_cap);
  return (size_t)c.Hkv * c.N_cap * c.d * elem_bytes(c.dtype);
}

int check_cache(const yoco_kv_cache* c) {
  if (!c) return fail(YOCO_ERR_INVALID_ARG, "cache descriptor is null");
  if (!c->k || !c->v) return fail(YOCO_ERR_INVALID_ARG, "cache planes are null");
  if (c->B <= 0 || c->Hkv <= 0 || c->N_cap <= 0) return fail(YOCO_ERR_INVALID_ARG, "cache has a non-positive size");
  if (!cache_dtype_ok(c->dtype)) return fail(YOCO_ERR_UNSUPPORTED, "cache dtype %d", c->dtype);
  if (c->d <= 0 || c->d > 256) return fail(YOCO_ERR_UNSUPPORTED, "head_dim %d not in [8, 256]", c->d);
  if (c->dtype == YOCO_INT8 && !yoco::cache_i8_supported(c->d))
    return fail(YOCO_ERR_UNSUPPORTED, "an 8-bit cache needs head_dim 128, not %d", c->d);
  if (c->d % 8) return fail(YOCO_ERR_ALIGNMENT, "head_dim %d is not a multiple of 8", c->d);
  if (!aligned16(c->k) || !aligned16(c->v)) return fail(YOCO_ERR_ALIGNMENT, "cache planes are not 16-byte aligned");
  return YOCO_OK;
}

int check_heads(int Hq, int Hkv) {
  if (Hq <= 0 || Hkv <= 0) return fail(YOCO_ERR_INVALID_ARG, "non-positive head count");
  if (Hq % Hkv) return fail(YOCO_ERR_INVALID_ARG, "Hq %d is not a multiple of Hkv %d", Hq, Hkv);
  if (Hq > 65535) return fail(YOCO_ERR_UNSUPPORTED, "Hq %d exceeds the grid limit", Hq);
  return YOCO_OK;
}

// Splits of the decode pass. Streaming reads on MI355X are fastest with few,
// long, contiguous streams: one workgroup per CU, each of its wavefronts
// walking its own contiguous range (measured: 6.9 TB/s at 256 workgroups,
// 6.0 TB/s at 2048). At least 512 rows per split. A pure function of the
// cache shape and the device: the workspace query and the decode call agree.
int decode_splits(const yoco_kv_cache* c) {
  static const int cus = [] {                     // initialised once, thread-safe
    int dev = 0, n = 0;
    const bool ok = hipGetDevice(&dev) == hipSuccess &&
                    hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0;
    (void)hipGetLastError();
    return ok ? n : 256;                          // no device visible (host-only sizing): MI355X has 256 CUs
  }();
  const int64_t target = cus;
  const int64_t units = (int64_t)c->B * c->Hkv;
  int64_t s = (target + units - 1) / units;
  const int64_t by_rows = (c->N_cap + 511) / 512;
  if (s > by_rows) s = by_rows;
  if (s < 1) s = 1;
  if (s > 1024) s = 1024;
  // More (sequence, KV head) units than CUs, and not a multiple of them: the workgroups of a ragged last round run
  // with part of the chip idle (384 units on 256 CUs measured 5.7 TB/s at 4096 rows). Two to four splits per unit
  // make the count a multiple again, as long as a split keeps at least 1024 rows (below that the merge launch costs
  // more than the balance gains: 41 us against 39 us at 1024 rows).
  if (s == 1 && units > cus && units % cus != 0) {
    for (int64_t t = 2; t <= 4; ++t)
      if ((units * t) % cus == 0 && c->N_cap / t >= 1024) { s = t; break; }
  }
  return (int)s;
}

// Split-KV attention of one query token per sequence of `c`: pass 1 + merge.
// `lens` (device) or, when it is null, `fixed_len` (host) gives the visible rows.
// k_new / v_new (both null or both rows [B,Hkv,d] of the cache dtype): the new token's row is stored at slot
// lens[b] - 1 (ring: modulo the capacity) by the same call and attended to.
int run_decode(const yoco_kv_cache& c, const void* q, void* o, const int64_t* lens, int64_t fixed_len, int Hq, float scale,
               float* ws, int splits, hipStream_t s, const char* what, const void* k_new = nullptr, const void* v_new = nullptr,
               int ring = 0) {
  hipError_t e;
  if (c.dtype == YOCO_INT8) {
    if (!yoco::decode_i8_supported(c, Hq))
      return fail(YOCO_ERR_UNSUPPORTED, "%s: an 8-bit cache serves up to 16 query heads per KV head, not %d", what, Hq / c.Hkv);
    if (k_new) return fail(YOCO_ERR_UNSUPPORTED, "%s: no fused append into an 8-bit cache", what);
    e = yoco::launch_decode_i8(c, q, lens, fixed_len, Hq, scale, ws, splits, o, s);
    if (splits == 1) return hip_result(e, what);
  } else if (yoco::decode_bf16_supported(c, Hq)) {
    e = yoco::launch_decode_bf16(c, q, lens, fixed_len, Hq, scale, ws, splits, o, k_new, v_new, ring, s);
    if (splits == 1) return hip_result(e, what);      // one split: pass 1 wrote the output
  } else {
    if (k_new) {                                      // no fused path for this shape: append, then attend
      e = yoco::launch_kv_append(c, k_new, v_new, lens, -1, ring, c.dtype, s);
      if (e != hipSuccess) return hip_result(e, what);
    }
    e = yoco::launch_decode_generic(c, q, lens, fixed_len, Hq, scale, ws, splits, s);
  }
  if (e != hipSuccess) return hip_result(e, what);
  return hip_result(yoco::launch_decode_merge(ws, o, c.B, Hq, c.d, splits, io_dtype(c), s), what);
}

int check_gret_shape(int B, int64_t T, int H, int dk, int dv, int dtype) {
  if (B <= 0 || H <= 0 || T < 0) return fail(YOCO_ERR_INVALID_ARG, "non-positive B or H, or negative T");
  if (B > 65535 || H > 65535) return fail(YOCO_ERR_UNSUPPORTED, "B %d or H %d exceeds the grid limit", B, H);
  if (!dtype_ok(dtype)) return fail(YOCO_ERR_UNSUPPORTED, "dtype %d", dtype);
  if (dk <= 0 || dv <= 0 || dk > 256 || dv > 256) return fail(YOCO_ERR_UNSUPPORTED, "head dims %d, %d not in [8, 256]", dk, dv);
  if (dk % 8 || dv % 8) return fail(YOCO_ERR_ALIGNMENT, "head dims %d, %d are not multiples of 8", dk, dv);
  return YOCO_OK;
}

// ---- static scratch for callers that cannot allocate (yoco_cross_attn_decode_noalloc). Every GPU the library
// runs on holds its own copy of the array, at its own address, until the process ends. In host code the array's name is
// only a handle for hipGetSymbolAddress; kernels and copies get the per-device address looked up below.
constexpr size_t kScratchBytes = YOCO_NOALLOC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mutex;

// Device address of `scratch` on the current device, looked up once per device with that device current.
int scratch_of_current_device(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_result(e, "hipGetDevice");
  if (dev < 0 || dev >= kMaxDevices) return fail(YOCO_ERR_UNSUPPORTED, "device index %d outside [0, %d)", dev, kMaxDevices);
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return hip_result(e, "hipGetSymbolAddress(scratch)");
    if (!p) return fail(YOCO_ERR_HIP, "hipGetSymbolAddress(scratch) returned a null address");
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return YOCO_OK;
}

constexpr int64_t kFewRows = 8;   // query rows up to which the prefill call splits over the cache like decode

}  // namespace

#pragma GCC visibility push(default)
extern "C" {

int yoco_version(void) { return 100; }

const char* yoco_last_error_string(void) { return g_err; }

int yoco_kv_cache_bytes(int B, int Hkv, int d, int64_t N_cap, int dtype, size_t* bytes) {
  if (!bytes) return fail(YOCO_ERR_INVALID_ARG, "bytes is null");
  if (B <= 0 || Hkv <= 0 || d <= 0 || N_cap <= 0) return fail(YOCO_ERR_INVALID_ARG, "non-positive size");
  if (!cache_dtype_ok(dtype)) return fail(YOCO_ERR_UNSUPPORTED, "dtype %d", dtype);
  if (d % 8) return fail(YOCO_ERR_ALIGNMENT, "head_dim %d is not a multiple of 8", d);
  if (d > 256) return fail(YOCO_ERR_UNSUPPORTED, "head_dim %d exceeds 256", d);
  if (dtype == YOCO_INT8) {
    if (!yoco::cache_i8_supported(d)) return fail(YOCO_ERR_UNSUPPORTED, "an 8-bit cache needs head_dim 128, not %d", d);
    *bytes = (size_t)2 * B * Hkv * (size_t)yoco::i8_plane_bytes(N_cap);
    return YOCO_OK;
  }
  *bytes = (size_t)2 * B * Hkv * (size_t)N_cap * d * elem_bytes(dtype);
  return YOCO_OK;
}

int yoco_kv_cache_init(void* mem, size_t bytes, int B, int Hkv, int d, int64_t N_cap, int dtype, yoco_kv_cache* out) {
  if (!out) return fail(YOCO_ERR_INVALID_ARG, "out is null");
  if (!mem) return fail(YOCO_ERR_INVALID_ARG, "mem is null");
  size_t need = 0;
  int rc = yoco_kv_cache_bytes(B, Hkv, d, N_cap, dtype, &need);
  if (rc) return rc;
  if (bytes < need) return fail(YOCO_ERR_WORKSPACE, "cache memory %zu < %zu bytes", bytes, need);
  if (((uintptr_t)mem) & 255u) return fail(YOCO_ERR_ALIGNMENT, "cache memory is not 256-byte aligned");
  out->k = mem;
  out->v = (char*)mem + need / 2;
  out->B = B;
  out->Hkv = Hkv;
  out->d = d;
  out->dtype = dtype;
  out->N_cap = N_cap;
  return YOCO_OK;
}

int yoco_swa_prefill(const void* q, const void* k, const void* v, void* o, int B, int64_t T, int Hq, int Hkv, int d,
                     int64_t window, float scale, int dtype, void* stream) {
  if (!q || !k || !v || !o) return fail(YOCO_ERR_INVALID_ARG, "null tensor pointer");
  if (B <= 0 || T <= 0 || window <= 0) return fail(YOCO_ERR_INVALID_ARG, "non-positive B, T or window");
  if (B > 65535) return fail(YOCO_ERR_UNSUPPORTED, "B %d exceeds the grid limit", B);
  int rc = check_heads(Hq, Hkv);
  if (rc) return rc;
  if (!dtype_ok(dtype)) return fail(YOCO_ERR_UNSUPPORTED, "dtype %d", dtype);
  if (d <= 0 || d > 256) return fail(YOCO_ERR_UNSUPPORTED, "head_dim %d not in [8, 256]", d);
  if (d % 8) return fail(YOCO_ERR_ALIGNMENT, "head_dim %d is not a multiple of 8", d);
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o))
    return fail(YOCO_ERR_ALIGNMENT, "tensor pointer not 16-byte aligned");
  yoco::AttnView a;
  a.q = q; a.k = k; a.v = v; a.o = o;
  a.q_stride_t = (int64_t)Hq * d;
  a.q_stride_b = T * a.q_stride_t;
  a.kv_stride_n = (int64_t)Hkv * d;
  a.kv_stride_h = d;
  a.kv_stride_b = T * a.kv_stride_n;
  a.Tq = T; a.q_pos0 = 0;
  a.window = window > T ? T : window;
  a.Hq = Hq; a.Hkv = Hkv; a.d = d; a.B = B; a.scale = scale;
  if (yoco::swa_mfma_supported(a, dtype)) return hip_result(yoco::launch_swa_mfma(a, (hipStream_t)stream), "swa_prefill");
  return hip_result(yoco::launch_attn_generic(a, dtype, (hipStream_t)stream), "swa_prefill");
}

int yoco_global_kv_write_scaled(const yoco_kv_cache* c, const void* k, const void* v, const float* row_scale, int b, int64_t pos0,
                                int64_t n, int src_dtype, void* stream) {
  int rc = check_cache(c);
  if (rc) return rc;
  if (n < 0) return fail(YOCO_ERR_INVALID_ARG, "negative row count");
  if (b < 0 || b >= c->B) return fail(YOCO_ERR_INVALID_ARG, "sequence %d outside [0, %d)", b, c->B);
  if (pos0 < 0 || pos0 + n > c->N_cap)
    return fail(YOCO_ERR_INVALID_ARG, "rows [%lld, %lld) outside the cache capacity %lld", (long long)pos0,
                (long long)(pos0 + n), (long long)c->N_cap);
  if (!dtype_ok(src_dtype)) return fail(YOCO_ERR_UNSUPPORTED, "source dtype %d", src_dtype);
  if (n == 0) return YOCO_OK;
  if (!k || !v) return fail(YOCO_ERR_INVALID_ARG, "null row pointer");
  if (!aligned16(k) || !aligned16(v)) return fail(YOCO_ERR_ALIGNMENT, "row pointer not 16-byte aligned");
  if (row_scale && (((uintptr_t)row_scale) & 3u)) return fail(YOCO_ERR_ALIGNMENT, "row_scale is not 4-byte aligned");
  if (c->dtype == YOCO_INT8) {
    if (n * c->Hkv > (int64_t)1 << 32) return fail(YOCO_ERR_UNSUPPORTED, "too many rows for one call");
    if (c->Hkv > 65535) return fail(YOCO_ERR_UNSUPPORTED, "Hkv %d exceeds the grid limit", c->Hkv);
    return hip_result(yoco::launch_kv_code_i8(*c, k, v, row_scale, b, pos0, n, nullptr, src_dtype, (hipStream_t)stream), "global_kv_write");
  }
  return hip_result(yoco::launch_kv_write(*c, k, v, row_scale, b, pos0, 0, n, src_dtype, (hipStream_t)stream), "global_kv_write");
}

int yoco_global_kv_write(const yoco_kv_cache* c, const void* k, const void* v, int b, int64_t pos0, int64_t n,
                         int src_dtype, void* stream) {
  return yoco_global_kv_write_scaled(c, k, v, nullptr, b, pos0, n, src_dtype, stream);
}

int yoco_swa_cache_write(const yoco_kv_cache* ring, const void* k, const void* v, int b, int64_t pos0, int64_t n,
                         int src_dtype, void* stream) {
  int rc = check_cache(ring);
  if (rc) return rc;
  if (ring->dtype == YOCO_INT8) return fail(YOCO_ERR_UNSUPPORTED, "a rolling window cache cannot be 8-bit");
  if (n < 0) return fail(YOCO_ERR_INVALID_ARG, "negative row count");
  if (b < 0 || b >= ring->B) return fail(YOCO_ERR_INVALID_ARG, "sequence %d outside [0, %d)", b, ring->B);
  if (pos0 < 0) return fail(YOCO_ERR_INVALID_ARG, "negative position %lld", (long long)pos0);
  if (pos0 > INT64_MAX - n) return fail(YOCO_ERR_INVALID_ARG, "positions overflow");
  if (!dtype_ok(src_dtype)) return fail(YOCO_ERR_UNSUPPORTED, "source dtype %d", src_dtype);
  if (n == 0) return YOCO_OK;
  if (!k || !v) return fail(YOCO_ERR_INVALID_ARG, "null row pointer");
  if (!aligned16(k) || !aligned16(v)) return fail(YOCO_ERR_ALIGNMENT, "row pointer not 16-byte aligned");
  const int64_t r0 = n > ring->N_cap ? n - ring->N_cap : 0;     // earlier rows would be overwritten by later ones
  return hip_result(yoco::launch_kv_write(*ring, k, v, nullptr, b, pos0, r0, n, src_dtype, (hipStream_t)stream), "swa_cache_write");
}

int yoco_kv_cache_append(const yoco_kv_cache* c, const void* k, const void* v, const int64_t* pos, int ring,
                         int src_dtype, void* stream) {
  int rc = check_cache(c);
  if (rc) return rc;
  if (!dtype_ok(src_dtype)) return fail(YOCO_ERR_UNSUPPORTED, "source dtype %d", src_dtype);
  if (!k || !v || !pos) return fail(YOCO_ERR_INVALID_ARG, "null pointer");
  if (!aligned16(k) || !aligned16(v)) return fail(YOCO_ERR_ALIGNMENT, "row pointer not 16-byte aligned");
  if (((uintptr_t)pos) & 7u) return fail(YOCO_ERR_ALIGNMENT, "pos is not 8-byte aligned");
  if (c->dtype == YOCO_INT8) {
    if (ring) return fail(YOCO_ERR_UNSUPPORTED, "a rolling window cache cannot be 8-bit");
    return hip_result(yoco::launch_kv_code_i8(*c, k, v, nullptr, 0, 0, c->B, pos, src_dtype, (hipStream_t)stream), "kv_cache_append");
  }
  return hip_result(yoco::launch_kv_append(*c, k, v, pos, 0, ring, src_dtype, (hipStream_t)stream), "kv_cache_append");
}

int yoco_cross_attn_prefill(const yoco_kv_cache* c, const void* q, void* o, int b, int64_t q_pos0, int64_t Tq, int Hq,
                            float scale, void* workspace, size_t workspace_bytes, void* stream) {
  int rc = check_cache(c);
  if (rc) return rc;
  rc = check_heads(Hq, c->Hkv);
  if (rc) return rc;
  if (!q || !o) return fail(YOCO_ERR_INVALID_ARG, "null tensor pointer");
  if (!aligned16(q) || !aligned16(o)) return fail(YOCO_ERR_ALIGNMENT, "tensor pointer not 16-byte aligned");
  if (b < 0 || b >= c->B) return fail(YOCO_ERR_INVALID_ARG, "sequence %d outside [0, %d)", b, c->B);
  if (Tq <= 0 || q_pos0 < 0) return fail(YOCO_ERR_INVALID_ARG, "non-positive Tq or negative q_pos0");
  if (q_pos0 + Tq > c->N_cap)
    return fail(YOCO_ERR_INVALID_ARG, "query positions up to %lld exceed the cache capacity %lld",
                (long long)(q_pos0 + Tq), (long long)c->N_cap);
  const size_t eb = elem_bytes(io_dtype(*c));
  const size_t seq_bytes = plane_bytes_per_seq(*c);
  if (workspace && !aligned16(workspace)) return fail(YOCO_ERR_ALIGNMENT, "workspace not 16-byte aligned");
  if (workspace && Tq <= kFewRows) {
    // A few rows cannot fill the chip one workgroup per query tile: treat each
    // row as a decode step of a one-sequence cache, split over the rows it sees.
    yoco_kv_cache one = *c;
    one.B = 1;
    one.k = (char*)c->k + (size_t)b * seq_bytes;
    one.v = (char*)c->v + (size_t)b * seq_bytes;
    const int splits = decode_splits(&one);
    const size_t need = (size_t)Hq * splits * yoco::partial_stride(c->d) * sizeof(float);
    if (workspace_bytes >= need) {
      for (int64_t i = 0; i < Tq; ++i) {
        rc = run_decode(one, (const char*)q + (size_t)i * Hq * c->d * eb, (char*)o + (size_t)i * Hq * c->d * eb, nullptr,
                        q_pos0 + i + 1, Hq, scale, (float*)workspace, splits, (hipStream_t)stream, "cross_attn_prefill (split)");
        if (rc) return rc;
      }
      return YOCO_OK;
    }
  }
  if (c->dtype == YOCO_INT8)
    return fail(YOCO_ERR_UNSUPPORTED, "cross_attn_prefill over an 8-bit cache serves up to %d rows and needs the decode workspace",
                (int)kFewRows);
  yoco::AttnView a;
  a.q = q; a.o = o;
  a.k = (const char*)c->k + (size_t)b * seq_bytes;
  a.v = (const char*)c->v + (size_t)b * seq_bytes;
  a.q_stride_t = (int64_t)Hq * c->d;
  a.q_stride_b = 0;
  a.kv_stride_n = c->d;
  a.kv_stride_h = c->N_cap * c->d;
  a.kv_stride_b = 0;
  a.Tq = Tq; a.q_pos0 = q_pos0;
  a.window = q_pos0 + Tq;          // every earlier row is visible
  a.Hq = Hq; a.Hkv = c->Hkv; a.d = c->d; a.B = 1; a.scale = scale;
  if (yoco::swa_mfma_supported(a, c->dtype))
    return hip_result(yoco::launch_swa_mfma(a, (hipStream_t)stream), "cross_attn_prefill");
  return hip_result(yoco::launch_attn_generic(a, c->dtype, (hipStream_t)stream), "cross_attn_prefill");
}

int yoco_cross_attn_decode_workspace(const yoco_kv_cache* c, int Hq, size_t* bytes, int* splits) {
  if (!c || !bytes || !splits) return fail(YOCO_ERR_INVALID_ARG, "null argument");
  if (c->B <= 0 || c->Hkv <= 0 || c->N_cap <= 0 || c->d <= 0) return fail(YOCO_ERR_INVALID_ARG, "cache has a non-positive size");
  int rc = check_heads(Hq, c->Hkv);
  if (rc) return rc;
  const int s = decode_splits(c);
  *splits = s;
  *bytes = (size_t)c->B * Hq * s * yoco::partial_stride(c->d) * sizeof(float);
  return YOCO_OK;
}

int yoco_cross_attn_decode(const yoco_kv_cache* c, const void* q, void* o, const int64_t* lens, int Hq, float scale,
                           void* workspace, size_t workspace_bytes, void* stream) {
  int rc = check_cache(c);
  if (rc) return rc;
  rc = check_heads(Hq, c->Hkv);
  if (rc) return rc;
  if (!q || !o || !lens || !workspace) return fail(YOCO_ERR_INVALID_ARG, "null pointer");
  if (!aligned16(q) || !aligned16(o) || !aligned16(workspace))
    return fail(YOCO_ERR_ALIGNMENT, "pointer not 16-byte aligned");
  if (c->B > 65535) return fail(YOCO_ERR_UNSUPPORTED, "B %d exceeds the grid limit", c->B);
  size_t need = 0;
  int splits = 0;
  rc = yoco_cross_attn_decode_workspace(c, Hq, &need, &splits);
  if (rc) return rc;
  if (workspace_bytes < need) return fail(YOCO_ERR_WORKSPACE, "workspace %zu < %zu bytes", workspace_bytes, need);
  return run_decode(*c, q, o, lens, 0, Hq, scale, (float*)workspace, splits, (hipStream_t)stream, "cross_attn_decode");
}

int yoco_cross_attn_decode_noalloc(const yoco_kv_cache* c, const void* q, void* o, const int64_t* lens, int Hq, float scale,
                                   void* stream) {
  // Validate the shape and the size first: a call that is too large must fail before anything touches the device.
  int rc = check_cache(c);
  if (rc) return rc;
  if (!q || !o || !lens) return fail(YOCO_ERR_INVALID_ARG, "null pointer");
  size_t need = 0;
  int splits = 0;
  rc = yoco_cross_attn_decode_workspace(c, Hq, &need, &splits);
  if (rc) return rc;
  if (need > kScratchBytes)
    return fail(YOCO_ERR_WORKSPACE, "cross_attn_decode_noalloc: the partial results need %zu bytes, the static scratch holds %zu",
                need, kScratchBytes);
  void* ptr = nullptr;
  rc = scratch_of_current_device(&ptr);
  if (rc) return rc;
  // Every partial the merge reads is written by pass 1 of the same call (empty splits included), so nothing in the
  // array has to be cleared between calls.
  return yoco_cross_attn_decode(c, q, o, lens, Hq, scale, ptr, kScratchBytes, stream);
}

int yoco_swa_decode(const yoco_kv_cache* ring, const void* q, const void* k_new, const void* v_new, void* o,
                    const int64_t* lens, int Hq, float scale, void* workspace, size_t workspace_bytes, void* stream) {
  // The ring holds exactly the rows the window admits and a softmax-weighted
  // sum does not depend on the order of its terms, so a decode step over the
  // ring, with lens clamped to its capacity (the kernels do), is Eq. 8.
  int rc = check_cache(ring);
  if (rc) return rc;
  if (ring->dtype == YOCO_INT8) return fail(YOCO_ERR_UNSUPPORTED, "a rolling window cache cannot be 8-bit");
  rc = check_heads(Hq, ring->Hkv);
  if (rc) return rc;
  if (!q || !o || !lens || !workspace) return fail(YOCO_ERR_INVALID_ARG, "null pointer");
  if (!aligned16(q) || !aligned16(o) || !aligned16(workspace))
    return fail(YOCO_ERR_ALIGNMENT, "pointer not 16-byte aligned");
  if (ring->B > 65535) return fail(YOCO_ERR_UNSUPPORTED, "B %d exceeds the grid limit", ring->B);
  if ((k_new == nullptr) != (v_new == nullptr)) return fail(YOCO_ERR_INVALID_ARG, "k_new and v_new must both be given or both be null");
  if (k_new && (!aligned16(k_new) || !aligned16(v_new))) return fail(YOCO_ERR_ALIGNMENT, "new row pointer not 16-byte aligned");
  size_t need = 0;
  int splits = 0;
  rc = yoco_cross_attn_decode_workspace(ring, Hq, &need, &splits);
  if (rc) return rc;
  if (workspace_bytes < need) return fail(YOCO_ERR_WORKSPACE, "workspace %zu < %zu bytes", workspace_bytes, need);
  return run_decode(*ring, q, o, lens, 0, Hq, scale, (float*)workspace, splits, (hipStream_t)stream, "swa_decode", k_new, v_new, 1);
}

int yoco_gret_prefill_workspace(int B, int64_t T, int H, int dk, int dv, int chunk, int dtype, size_t* bytes) {
  if (!bytes) return fail(YOCO_ERR_INVALID_ARG, "bytes is null");
  int rc = check_gret_shape(B, T, H, dk, dv, dtype);
  if (rc) return rc;
  if (chunk <= 0) return fail(YOCO_ERR_INVALID_ARG, "non-positive chunk");
  *bytes = yoco::gret_chunk_supported(B, T, H, dk, dv, chunk, dtype) ? yoco::gret_chunk_workspace(B, T, H, chunk) : 0;
  return YOCO_OK;
}

int yoco_gret_prefill(const void* q, const void* k, const void* v, const float* log_gamma, const void* gate, void* o,
                      const float* state_in, float* state_out, int B, int64_t T, int H, int dk, int dv, int chunk,
                      float scale, int group_norm, float eps, int dtype, void* workspace, size_t workspace_bytes,
                      void* stream) {
  int rc = check_gret_shape(B, T, H, dk, dv, dtype);
  if (rc) return rc;
  if (chunk <= 0) return fail(YOCO_ERR_INVALID_ARG, "non-positive chunk");
  if (!(eps >= 0.f)) return fail(YOCO_ERR_INVALID_ARG, "negative eps");
  if (state_in && !aligned16(state_in)) return fail(YOCO_ERR_ALIGNMENT, "state_in not 16-byte aligned");
  if (state_out && !aligned16(state_out)) return fail(YOCO_ERR_ALIGNMENT, "state_out not 16-byte aligned");
  if (workspace && (((uintptr_t)workspace) & 255u)) return fail(YOCO_ERR_ALIGNMENT, "workspace not 256-byte aligned");
  if (T == 0) {
    if (!state_out || state_out == state_in) return YOCO_OK;
    const size_t nb = (size_t)B * H * dk * dv * sizeof(float);
    if (state_in) return hip_result(hipMemcpyAsync(state_out, state_in, nb, hipMemcpyDeviceToDevice, (hipStream_t)stream), "gret_prefill");
    return hip_result(yoco::launch_fill_zero(state_out, nb / sizeof(float), (hipStream_t)stream), "gret_prefill");
  }
  if (!q || !k || !v || !log_gamma || !o) return fail(YOCO_ERR_INVALID_ARG, "null tensor pointer");
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o) || (gate && !aligned16(gate)) || (((uintptr_t)log_gamma) & 3u))
    return fail(YOCO_ERR_ALIGNMENT, "tensor pointer not aligned");
  yoco::GretView a;
  a.q = q; a.k = k; a.v = v; a.o = o; a.log_gamma = log_gamma; a.gate = gate;
  a.state_in = state_in; a.state_out = state_out;
  a.T = T; a.B = B; a.H = H; a.dk = dk; a.dv = dv;
  a.scale = scale; a.eps = eps; a.group_norm = group_norm != 0;
  if (workspace && yoco::gret_chunk_supported(B, T, H, dk, dv, chunk, dtype) &&
      workspace_bytes >= yoco::gret_chunk_workspace(B, T, H, chunk))
    return hip_result(yoco::launch_gret_chunk(a, chunk, workspace, (hipStream_t)stream), "gret_prefill (chunkwise)");
  if (!yoco::gret_recurrent_supported(a))
    return fail(YOCO_ERR_UNSUPPORTED, "gated retention: dk %d, dv %d have no kernel (at most 128)", dk, dv);
  return hip_result(yoco::launch_gret_recurrent(a, dtype, (hipStream_t)stream), "gret_prefill");
}

int yoco_gret_decode(const void* q, const void* k, const void* v, const float* log_gamma, const void* gate, void* o, float* state,
                     int B, int H, int dk, int dv, float scale, int group_norm, float eps, int dtype, void* stream) {
  int rc = check_gret_shape(B, 1, H, dk, dv, dtype);
  if (rc) return rc;
  if (!(eps >= 0.f)) return fail(YOCO_ERR_INVALID_ARG, "negative eps");
  if (!q || !k || !v || !log_gamma || !o || !state) return fail(YOCO_ERR_INVALID_ARG, "null pointer");
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o) || !aligned16(state) || (gate && !aligned16(gate)) ||
      (((uintptr_t)log_gamma) & 3u))
    return fail(YOCO_ERR_ALIGNMENT, "pointer not aligned");
  yoco::GretView a;
  a.q = q; a.k = k; a.v = v; a.o = o; a.log_gamma = log_gamma; a.gate = gate;
  a.state_in = state; a.state_out = state;
  a.T = 1; a.B = B; a.H = H; a.dk = dk; a.dv = dv;
  a.scale = scale; a.eps = eps; a.group_norm = group_norm != 0;
  if (!yoco::gret_recurrent_supported(a))
    return fail(YOCO_ERR_UNSUPPORTED, "gated retention: dk %d, dv %d have no kernel (at most 128)", dk, dv);
  return hip_result(yoco::launch_gret_recurrent(a, dtype, (hipStream_t)stream), "gret_decode");
}

int yoco_ceiling_mfma(const void* seed, void* sink, int iters, int workgroups, void* stream) {
  if (!seed || !sink) return fail(YOCO_ERR_INVALID_ARG, "null pointer");
  if (!aligned16(seed)) return fail(YOCO_ERR_ALIGNMENT, "seed not 16-byte aligned");
  if (iters <= 0 || workgroups <= 0) return fail(YOCO_ERR_INVALID_ARG, "non-positive iters or workgroups");
  return hip_result(yoco::launch_mfma_ceiling(seed, sink, iters, workgroups, (hipStream_t)stream), "ceiling_mfma");
}

int yoco_ceiling_attn_loop(const void* seed, void* sink, int iters, int workgroups, int mode, void* stream) {
  if (!seed || !sink) return fail(YOCO_ERR_INVALID_ARG, "null pointer");
  if (!aligned16(seed)) return fail(YOCO_ERR_ALIGNMENT, "seed not 16-byte aligned");
  if (iters <= 0 || workgroups <= 0) return fail(YOCO_ERR_INVALID_ARG, "non-positive iters or workgroups");
  if (mode != 1 && mode != 2) return fail(YOCO_ERR_INVALID_ARG, "mode %d is neither 1 (LDS-fed products) nor 2 (with the softmax work)", mode);
  return hip_result(yoco::launch_attn_loop_ceiling(seed, sink, iters, workgroups, mode, (hipStream_t)stream), "ceiling_attn_loop");
}

int yoco_ceiling_stream_read(const void* buf, size_t bytes, void* sink, int workgroups, void* stream) {
  if (!buf || !sink) return fail(YOCO_ERR_INVALID_ARG, "null pointer");
  if (!aligned16(buf) || bytes % 16) return fail(YOCO_ERR_ALIGNMENT, "buffer not 16-byte aligned or size not a multiple of 16");
  if (bytes == 0 || workgroups <= 0) return fail(YOCO_ERR_INVALID_ARG, "empty buffer or non-positive workgroups");
  return hip_result(yoco::launch_stream_read(buf, bytes, sink, workgroups, (hipStream_t)stream), "ceiling_stream_read");
}

}  // extern "C"
#pragma GCC visibility pop
