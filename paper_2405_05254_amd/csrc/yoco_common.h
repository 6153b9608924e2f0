// Shared declarations of libyoco's translation units (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "yoco.h"

namespace yoco {

typedef unsigned short bf16_t;  // raw bfloat16 bits

__device__ __forceinline__ float bf16_to_f32(bf16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// Round to nearest even; NaN stays NaN (quiet).
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}

template <typename T> struct Elem;
template <> struct Elem<float> {
  static __device__ __forceinline__ float load(const float* p) { return *p; }
  static __device__ __forceinline__ void store(float* p, float x) { *p = x; }
};
template <> struct Elem<bf16_t> {
  static __device__ __forceinline__ float load(const bf16_t* p) { return bf16_to_f32(*p); }
  static __device__ __forceinline__ void store(bf16_t* p, float x) { *p = f32_to_bf16(x); }
};

// Addressing of one attention problem family. Strides are in elements.
struct AttnView {
  const void* q;   // [.., Tq, Hq, d]
  const void* k;
  const void* v;
  void* o;         // [.., Tq, Hq, d]
  int64_t q_stride_b, q_stride_t;          // o uses the same strides
  int64_t kv_stride_b, kv_stride_h, kv_stride_n;
  int64_t Tq;       // query rows per sequence
  int64_t q_pos0;   // absolute position of query row 0
  int64_t window;   // keys visible per row (>= 1); INT64_MAX/2 = unbounded
  int Hq, Hkv, d, B;
  float scale;
};

// One gated-retention problem (section 3.1). q, k: [B,T,H,dk]; v, o: [B,T,H,dv];
// log_gamma: [B,T,H] fp32, the natural log of the decays; states: [B,H,dv,dk]
// fp32 (the transpose of S = K^T V), either may be null; gate: like v, may be null.
struct GretView {
  const void* q;
  const void* k;
  const void* v;
  void* o;
  const float* log_gamma;
  const void* gate;          // [B,T,H,dv] or null: the output is multiplied by swish(gate) (Eq. 7)
  const float* state_in;
  float* state_out;
  int64_t T;
  int B, H, dk, dv;
  float scale, eps;
  int group_norm;
};

// Launchers (each returns the hipError_t of its launch).
hipError_t launch_attn_generic(const AttnView& a, int dtype, hipStream_t s);
hipError_t launch_decode_generic(const yoco_kv_cache& c, const void* q, const int64_t* lens, int64_t fixed_len, int Hq,
                                 float scale, float* ws, int splits, hipStream_t s);
hipError_t launch_decode_merge(const float* ws, void* o, int B, int Hq, int d, int splits, int dtype,
                               hipStream_t s);
hipError_t launch_kv_write(const yoco_kv_cache& c, const void* k, const void* v, const float* row_scale, int b, int64_t pos0, int64_t r0,
                           int64_t n, int src_dtype, hipStream_t s);
hipError_t launch_kv_append(const yoco_kv_cache& c, const void* k, const void* v, const int64_t* pos, int64_t bias, int ring,
                            int src_dtype, hipStream_t s);   // slot = pos[b] + bias

bool gret_recurrent_supported(const GretView& a);
hipError_t launch_gret_recurrent(const GretView& a, int dtype, hipStream_t s);
hipError_t launch_fill_zero(float* p, size_t n, hipStream_t s);
// Chunkwise form on the matrix cores (bf16, dk = dv = 128).
bool gret_chunk_supported(int B, int64_t T, int H, int dk, int dv, int chunk, int dtype);
size_t gret_chunk_workspace(int B, int64_t T, int H, int chunk);
hipError_t launch_gret_chunk(const GretView& a, int chunk, void* workspace, hipStream_t s);

// bf16, d = 128 fast paths. `supported` functions are host-side predicates.
bool swa_mfma_supported(const AttnView& a, int dtype);
hipError_t launch_swa_mfma(const AttnView& a, hipStream_t s);
bool decode_bf16_supported(const yoco_kv_cache& c, int Hq);
// With one split and a non-null o_direct the kernel normalises and stores the output itself (no merge pass).
// k_new / v_new ([B,Hkv,128] bf16, or null): also store and attend to the new token's row at slot lens[b] - 1.
hipError_t launch_decode_bf16(const yoco_kv_cache& c, const void* q, const int64_t* lens, int64_t fixed_len, int Hq, float scale,
                              float* ws, int splits, void* o_direct, const void* k_new, const void* v_new, int ring,
                              hipStream_t s);

// 8-bit global cache (cache_i8.hip), head_dim 128: a plane per (sequence, KV head) is a run of 64-row blocks, each
// 8192 code bytes followed by the rows' 64 fp32 scales in row order. Byte offsets of (block row rho, dim e) inside a block:
constexpr int kI8BlockRows = 64;
constexpr int kI8ScaleOffset = 64 * 128;                 // bytes from the start of a block to its scales
constexpr int kI8BlockBytes = kI8ScaleOffset + 64 * 4;   // 8448 = 33 * 256
__host__ __device__ inline int64_t i8_plane_bytes(int64_t N_cap) { return ((N_cap + 63) / 64) * kI8BlockBytes; }
__host__ __device__ inline int i8_k_offset(int rho, int e) {      // K plane: signed code bytes
  return (((((rho >> 2) & 3) * 2 + (e >> 6)) * 64) + ((e >> 4) & 3) * 16 + 4 * (rho >> 4) + (rho & 3)) * 16 + (e & 15);
}
__host__ __device__ inline int i8_v_offset(int rho, int e) {      // V plane: bytes code + 128, transposed
  return (((e >> 4) * 64) + (rho >> 4) * 16 + (e & 15)) * 16 + (rho & 15);
}
bool cache_i8_supported(int d);
bool decode_i8_supported(const yoco_kv_cache& c, int Hq);
// pos == null: rows [n,Hkv,128] of sequence b to slots pos0 ..; pos != null: one row per sequence to slot pos[b].
// row_scale (or null): float32 [n], every source row is multiplied by its entry (in float32) before it is coded.
hipError_t launch_kv_code_i8(const yoco_kv_cache& c, const void* k, const void* v, const float* row_scale, int b, int64_t pos0, int64_t n,
                             const int64_t* pos, int src_dtype, hipStream_t s);
hipError_t launch_decode_i8(const yoco_kv_cache& c, const void* q, const int64_t* lens, int64_t fixed_len, int Hq, float scale,
                            float* ws, int splits, void* o_direct, hipStream_t s);   // q, o bf16

// Measured-ceiling microbenchmarks (ceilings.hip).
hipError_t launch_mfma_ceiling(const void* seed, void* sink, int iters, int workgroups, hipStream_t s);
hipError_t launch_attn_loop_ceiling(const void* seed, void* sink, int iters, int workgroups, int mode, hipStream_t s);
hipError_t launch_stream_read(const void* buf, size_t bytes, void* sink, int workgroups, hipStream_t s);

// Partial result of one split, per (b, h, split): o[0..d), then the running max
// m (natural-log units) and sum l, padded so every row starts 16-byte aligned.
__host__ __device__ inline size_t partial_stride(int d) { return (size_t)d + 4; }

}  // namespace yoco
