// Generic attention kernels (any head_dim <= 256, fp32 or bf16 storage, fp32
// arithmetic on the vector ALU). They serve the fp32 configuration and every
// shape the MFMA / streaming fast paths do not cover. One wavefront owns one
// (sequence, query row, query head) and walks its visible keys 64 at a time:
// lane j scores key j (Eq. 8 / Eq. 3: scale * q.k), the wave reduces max and
// sum, then every lane accumulates its own slice of the head dimension over
// the 64 weighted value rows.
#include "yoco_common.h"

namespace yoco {

constexpr int kWaves = 4;        // wavefronts (query rows) per workgroup
constexpr int kMaxD = 256;

// LDS traffic of one wave is ordered by the hardware; this keeps the compiler
// from moving a lane's read above another lane's write.
__device__ __forceinline__ void lds_wave_sync() {
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  __builtin_amdgcn_wave_barrier();
}

__device__ __forceinline__ float wave_max(float x) {
  for (int o = 32; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o));
  return x;
}
__device__ __forceinline__ float wave_sum(float x) {
  for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o);
  return x;
}

// Online softmax state of one wave over keys [j_lo, j_hi] of one KV head.
// q_s: this wave's query in LDS (fp32, d entries). p_s: 64 floats of LDS.
// On return (m, l) are the running max / sum and acc[t] holds dimension
// lane + 64 t of the unnormalised output.
template <typename T>
__device__ __forceinline__ void attend_range(const T* __restrict__ kbase, const T* __restrict__ vbase,
                                             int64_t stride_n, int64_t j_lo, int64_t j_hi, int d, float scale,
                                             const float* q_s, float* p_s, float& m, float& l, float acc[4]) {
  const int lane = threadIdx.x & 63;
  for (int64_t c0 = j_lo; c0 <= j_hi; c0 += 64) {
    const int64_t j = c0 + lane;
    const bool valid = j <= j_hi;
    float s = -INFINITY;
    if (valid) {
      const T* kr = kbase + j * stride_n;
      float dot = 0.f;
      for (int e = 0; e < d; ++e) dot = fmaf(q_s[e], Elem<T>::load(kr + e), dot);
      s = dot * scale;
    }
    const float m_new = fmaxf(m, wave_max(s));       // finite: key c0 is valid
    const float alpha = __expf(m - m_new);            // m = -inf on the first chunk -> 0
    const float p = valid ? __expf(s - m_new) : 0.f;
    l = l * alpha + wave_sum(p);
    m = m_new;
    p_s[lane] = p;
    lds_wave_sync();
    const int n = (int)((j_hi - c0 + 1 < 64) ? (j_hi - c0 + 1) : 64);
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const int e = lane + 64 * t;
      if (e < d) {
        float a = acc[t] * alpha;
        const T* vr = vbase + c0 * stride_n + e;
        for (int jj = 0; jj < n; ++jj) a = fmaf(p_s[jj], Elem<T>::load(vr + jj * stride_n), a);
        acc[t] = a;
      }
    }
    lds_wave_sync();
  }
}

template <typename T>
__global__ void __launch_bounds__(64 * kWaves) attn_generic_kernel(AttnView a) {
  __shared__ float q_s[kWaves][kMaxD];
  __shared__ float p_s[kWaves][64];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int64_t i = (int64_t)blockIdx.x * kWaves + wave;
  const int h = blockIdx.y, b = blockIdx.z;
  if (i >= a.Tq) return;                      // whole wave leaves; no block-wide barrier below
  const int g = h / (a.Hq / a.Hkv);
  const T* q = (const T*)a.q + b * a.q_stride_b + i * a.q_stride_t + (int64_t)h * a.d;
  for (int e = lane; e < a.d; e += 64) q_s[wave][e] = Elem<T>::load(q + e);
  lds_wave_sync();
  const int64_t pos = a.q_pos0 + i;
  const int64_t j_lo = (pos - a.window + 1 > 0) ? pos - a.window + 1 : 0;
  const T* kb = (const T*)a.k + b * a.kv_stride_b + g * a.kv_stride_h;
  const T* vb = (const T*)a.v + b * a.kv_stride_b + g * a.kv_stride_h;
  float m = -INFINITY, l = 0.f, acc[4] = {0.f, 0.f, 0.f, 0.f};
  attend_range<T>(kb, vb, a.kv_stride_n, j_lo, pos, a.d, a.scale, q_s[wave], p_s[wave], m, l, acc);
  T* o = (T*)a.o + b * a.q_stride_b + i * a.q_stride_t + (int64_t)h * a.d;
  const float inv = 1.f / l;
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    const int e = lane + 64 * t;
    if (e < a.d) Elem<T>::store(o + e, acc[t] * inv);
  }
}

hipError_t launch_attn_generic(const AttnView& a, int dtype, hipStream_t s) {
  dim3 grid((unsigned)((a.Tq + kWaves - 1) / kWaves), a.Hq, a.B);
  if (dtype == YOCO_F32)
    hipLaunchKernelGGL(attn_generic_kernel<float>, grid, dim3(64 * kWaves), 0, s, a);
  else
    hipLaunchKernelGGL(attn_generic_kernel<bf16_t>, grid, dim3(64 * kWaves), 0, s, a);
  return hipGetLastError();
}

// ---- decode, pass 1 (generic): one wave per (sequence, query head, split).
template <typename T>
__global__ void __launch_bounds__(64) decode_generic_kernel(yoco_kv_cache c, const T* __restrict__ q,
                                                            const int64_t* __restrict__ lens, int64_t fixed_len, int Hq,
                                                            float scale, float* __restrict__ ws, int splits) {
  __shared__ float q_s[kMaxD];
  __shared__ float p_s[64];
  const int lane = threadIdx.x;
  const int sp = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  const int d = c.d, g = h / (Hq / c.Hkv);
  int64_t len = lens ? lens[b] : fixed_len;         // a host-known length serves the few-row prefill case
  len = len < 0 ? 0 : (len > c.N_cap ? c.N_cap : len);
  const int64_t chunk = (len + splits - 1) / splits;
  const int64_t j_lo = sp * chunk;
  const int64_t j_hi = ((j_lo + chunk < len) ? j_lo + chunk : len) - 1;
  for (int e = lane; e < d; e += 64) q_s[e] = Elem<T>::load(q + ((int64_t)b * Hq + h) * d + e);
  lds_wave_sync();
  const int64_t head_off = ((int64_t)b * c.Hkv + g) * c.N_cap * d;
  float m = -INFINITY, l = 0.f, acc[4] = {0.f, 0.f, 0.f, 0.f};
  if (j_lo <= j_hi)
    attend_range<T>((const T*)c.k + head_off, (const T*)c.v + head_off, d, j_lo, j_hi, d, scale, q_s, p_s, m, l, acc);
  float* w = ws + (((size_t)b * Hq + h) * splits + sp) * partial_stride(d);
  if (lane == 0) { w[d] = m; w[d + 1] = l; }
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    const int e = lane + 64 * t;
    if (e < d) w[e] = acc[t];
  }
}

hipError_t launch_decode_generic(const yoco_kv_cache& c, const void* q, const int64_t* lens, int64_t fixed_len, int Hq,
                                 float scale, float* ws, int splits, hipStream_t s) {
  dim3 grid(splits, Hq, c.B);
  if (c.dtype == YOCO_F32)
    hipLaunchKernelGGL(decode_generic_kernel<float>, grid, dim3(64), 0, s, c, (const float*)q, lens, fixed_len, Hq, scale, ws, splits);
  else
    hipLaunchKernelGGL(decode_generic_kernel<bf16_t>, grid, dim3(64), 0, s, c, (const bf16_t*)q, lens, fixed_len, Hq, scale, ws, splits);
  return hipGetLastError();
}

// ---- decode, pass 2: merge the splits of one (sequence, query head) by
// log-sum-exp: o = sum_s e^{m_s-M} o_s / sum_s e^{m_s-M} l_s.
// Phase 1 finds M, phase 2 puts the factors e^{m_s-M} in LDS, phase 3 has
// thread (sl, dl) add splits sl, sl+nsl, ... for dimensions 4dl..4dl+3 with
// independent 128-bit loads; the nsl partial sums are then added in order.
// Assignment and order are fixed (no atomics): results are bit-reproducible.
constexpr int kMaxSplits = 1024;

template <typename T>
__global__ void __launch_bounds__(256) decode_merge_kernel(const float* __restrict__ ws, T* __restrict__ o, int d,
                                                           int splits) {
  __shared__ float sF[kMaxSplits];
  __shared__ float sRed[8];
  __shared__ __attribute__((aligned(16))) float sO[1024];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const size_t bh = blockIdx.x;
  const size_t ps = partial_stride(d);
  const float* w = ws + bh * splits * ps;
  float M = -INFINITY;
  for (int s = tid; s < splits; s += 256) M = fmaxf(M, w[s * ps + d]);
  M = wave_max(M);
  if (lane == 0) sRed[wave] = M;
  __syncthreads();
  M = fmaxf(fmaxf(sRed[0], sRed[1]), fmaxf(sRed[2], sRed[3]));
  float L = 0.f;
  for (int s = tid; s < splits; s += 256) {
    const float ms = w[s * ps + d];
    const float f = (ms == -INFINITY) ? 0.f : __expf(ms - M);        // empty split (or no row at all)
    sF[s] = f;
    L = fmaf(f, w[s * ps + d + 1], L);
  }
  L = wave_sum(L);
  if (lane == 0) sRed[4 + wave] = L;
  __syncthreads();
  L = ((sRed[4] + sRed[5]) + sRed[6]) + sRed[7];
  const int nd = d >> 2;               // 128-bit groups per row
  const int nsl = 256 / nd;            // split lanes
  const int sl = tid / nd, dl = tid - sl * nd;
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  if (sl < nsl) {
#pragma unroll 4
    for (int s = sl; s < splits; s += nsl) {
      const float f = sF[s];
      const float4 x = *(const float4*)(w + s * ps + 4 * dl);
      acc.x = fmaf(f, x.x, acc.x);
      acc.y = fmaf(f, x.y, acc.y);
      acc.z = fmaf(f, x.z, acc.z);
      acc.w = fmaf(f, x.w, acc.w);
    }
    *(float4*)(sO + sl * d + 4 * dl) = acc;
  }
  __syncthreads();
  const float inv = (L > 0.f) ? 1.f / L : 0.f;                        // no visible row -> zeros
  for (int e = tid; e < d; e += 256) {
    float x = 0.f;
    for (int k = 0; k < nsl; ++k) x += sO[k * d + e];
    Elem<T>::store(o + bh * d + e, x * inv);
  }
}

hipError_t launch_decode_merge(const float* ws, void* o, int B, int Hq, int d, int splits, int dtype,
                               hipStream_t s) {
  if (splits > kMaxSplits) return hipErrorInvalidValue;
  dim3 grid((unsigned)(B * Hq));
  if (dtype == YOCO_F32)
    hipLaunchKernelGGL(decode_merge_kernel<float>, grid, dim3(256), 0, s, ws, (float*)o, d, splits);
  else
    hipLaunchKernelGGL(decode_merge_kernel<bf16_t>, grid, dim3(256), 0, s, ws, (bf16_t*)o, d, splits);
  return hipGetLastError();
}

// ---- global KV write: rows [n,Hkv,d] -> planes [B][Hkv][N_cap][d] of the cache
// dtype. Pure data movement (plus the cast): each thread moves 8 consecutive
// elements of K and of V with 128-bit accesses; 16 threads cover a 256-byte
// bf16 row on both sides.
typedef unsigned int kvw_u32x4 __attribute__((ext_vector_type(4)));
typedef float kvw_f32x4 __attribute__((ext_vector_type(4)));

template <typename S> struct Row8;
template <> struct Row8<float> {
  kvw_f32x4 lo, hi;
  __device__ __forceinline__ void load(const float* p) { lo = *(const kvw_f32x4*)p; hi = *(const kvw_f32x4*)(p + 4); }
  __device__ __forceinline__ float get(int i) const { return i < 4 ? lo[i] : hi[i - 4]; }
};
template <> struct Row8<bf16_t> {
  kvw_u32x4 w;
  __device__ __forceinline__ void load(const bf16_t* p) { w = *(const kvw_u32x4*)p; }
  __device__ __forceinline__ float get(int i) const {
    const unsigned x = w[i >> 1];
    return __uint_as_float((i & 1) ? (x & 0xffff0000u) : (x << 16));
  }
};
template <typename S>
__device__ __forceinline__ void store8(float* p, const Row8<S>& r) {
  kvw_f32x4 a = {r.get(0), r.get(1), r.get(2), r.get(3)}, b = {r.get(4), r.get(5), r.get(6), r.get(7)};
  *(kvw_f32x4*)p = a;
  *(kvw_f32x4*)(p + 4) = b;
}
__device__ __forceinline__ void store8(bf16_t* p, const Row8<bf16_t>& r) { *(kvw_u32x4*)p = r.w; }   // same dtype: bit copy
__device__ __forceinline__ void store8(bf16_t* p, const Row8<float>& r) {
  kvw_u32x4 w;
#pragma unroll
  for (int i = 0; i < 4; ++i) w[i] = (unsigned)f32_to_bf16(r.get(2 * i)) | ((unsigned)f32_to_bf16(r.get(2 * i + 1)) << 16);
  *(kvw_u32x4*)p = w;
}

// Rows r0 .. n-1 of k, v [n,Hkv,d] -> cache rows of sequence b. Row r goes to
// slot pos0 + r, taken modulo N_cap: the identity for the global cache (the
// host has checked pos0 + n <= N_cap), the ring slot for a rolling cache
// (whose caller passes r0 = max(0, n - N_cap), so no two rows share a slot).
template <typename S, typename D>
__global__ void __launch_bounds__(256) kv_write_kernel(yoco_kv_cache c, const S* __restrict__ k,
                                                       const S* __restrict__ v, const float* __restrict__ row_scale, int b,
                                                       int64_t pos0, int64_t r0, int64_t n) {
  const int d8 = c.d / 8;
  const int64_t total = (n - r0) * c.Hkv * d8;           // groups of 8 elements
  for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total;
       idx += (int64_t)gridDim.x * blockDim.x) {
    const int e8 = (int)(idx % d8);
    const int g = (int)((idx / d8) % c.Hkv);
    const int64_t r = r0 + idx / ((int64_t)d8 * c.Hkv);
    int64_t slot = pos0 + r;
    if (slot >= c.N_cap) slot %= c.N_cap;
    const int64_t src = (r * c.Hkv + g) * c.d + e8 * 8;
    const int64_t dst = (((int64_t)b * c.Hkv + g) * c.N_cap + slot) * c.d + e8 * 8;
    Row8<S> kr, vr;
    kr.load(k + src);
    vr.load(v + src);
    if (row_scale) {                                       // Eq. 2 with the norm's 1/rms applied after the projections
      const float rs = row_scale[r];
      Row8<float> ks, vs;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        ks.lo[i] = kr.get(i) * rs;
        ks.hi[i] = kr.get(4 + i) * rs;
        vs.lo[i] = vr.get(i) * rs;
        vs.hi[i] = vr.get(4 + i) * rs;
      }
      store8((D*)c.k + dst, ks);
      store8((D*)c.v + dst, vs);
    } else {
      store8((D*)c.k + dst, kr);
      store8((D*)c.v + dst, vr);
    }
  }
}

// One row per sequence at a device-side position: k, v [B,Hkv,d]; sequence b's
// row goes to slot pos[b] + bias (ring: modulo N_cap). Out-of-range positions write
// nothing.
template <typename S, typename D>
__global__ void __launch_bounds__(256) kv_append_kernel(yoco_kv_cache c, const S* __restrict__ k,
                                                        const S* __restrict__ v, const int64_t* __restrict__ pos,
                                                        int64_t bias, int ring) {
  const int d8 = c.d / 8;
  const int64_t total = (int64_t)c.B * c.Hkv * d8;
  for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total;
       idx += (int64_t)gridDim.x * blockDim.x) {
    const int e8 = (int)(idx % d8);
    const int g = (int)((idx / d8) % c.Hkv);
    const int b = (int)(idx / ((int64_t)d8 * c.Hkv));
    int64_t slot = pos[b] + bias;
    if (slot < 0) continue;
    if (slot >= c.N_cap) {
      if (!ring) continue;
      slot %= c.N_cap;
    }
    const int64_t src = ((int64_t)b * c.Hkv + g) * c.d + e8 * 8;
    const int64_t dst = (((int64_t)b * c.Hkv + g) * c.N_cap + slot) * c.d + e8 * 8;
    Row8<S> kr, vr;
    kr.load(k + src);
    vr.load(v + src);
    store8((D*)c.k + dst, kr);
    store8((D*)c.v + dst, vr);
  }
}

hipError_t launch_kv_write(const yoco_kv_cache& c, const void* k, const void* v, const float* row_scale, int b, int64_t pos0, int64_t r0,
                           int64_t n, int src_dtype, hipStream_t s) {
  const int64_t total = (n - r0) * c.Hkv * (c.d / 8);
  int64_t blocks = (total + 255) / 256;
  if (blocks > 16384) blocks = 16384;
  dim3 grid((unsigned)blocks), block(256);
  if (src_dtype == YOCO_F32 && c.dtype == YOCO_F32)
    hipLaunchKernelGGL((kv_write_kernel<float, float>), grid, block, 0, s, c, (const float*)k, (const float*)v, row_scale, b, pos0, r0, n);
  else if (src_dtype == YOCO_F32 && c.dtype == YOCO_BF16)
    hipLaunchKernelGGL((kv_write_kernel<float, bf16_t>), grid, block, 0, s, c, (const float*)k, (const float*)v, row_scale, b, pos0, r0, n);
  else if (src_dtype == YOCO_BF16 && c.dtype == YOCO_F32)
    hipLaunchKernelGGL((kv_write_kernel<bf16_t, float>), grid, block, 0, s, c, (const bf16_t*)k, (const bf16_t*)v, row_scale, b, pos0, r0, n);
  else
    hipLaunchKernelGGL((kv_write_kernel<bf16_t, bf16_t>), grid, block, 0, s, c, (const bf16_t*)k, (const bf16_t*)v, row_scale, b, pos0, r0, n);
  return hipGetLastError();
}

hipError_t launch_kv_append(const yoco_kv_cache& c, const void* k, const void* v, const int64_t* pos, int64_t bias, int ring,
                            int src_dtype, hipStream_t s) {
  const int64_t total = (int64_t)c.B * c.Hkv * (c.d / 8);
  int64_t blocks = (total + 255) / 256;
  if (blocks > 16384) blocks = 16384;
  dim3 grid((unsigned)blocks), block(256);
  if (src_dtype == YOCO_F32 && c.dtype == YOCO_F32)
    hipLaunchKernelGGL((kv_append_kernel<float, float>), grid, block, 0, s, c, (const float*)k, (const float*)v, pos, bias, ring);
  else if (src_dtype == YOCO_F32 && c.dtype == YOCO_BF16)
    hipLaunchKernelGGL((kv_append_kernel<float, bf16_t>), grid, block, 0, s, c, (const float*)k, (const float*)v, pos, bias, ring);
  else if (src_dtype == YOCO_BF16 && c.dtype == YOCO_F32)
    hipLaunchKernelGGL((kv_append_kernel<bf16_t, float>), grid, block, 0, s, c, (const bf16_t*)k, (const bf16_t*)v, pos, bias, ring);
  else
    hipLaunchKernelGGL((kv_append_kernel<bf16_t, bf16_t>), grid, block, 0, s, c, (const bf16_t*)k, (const bf16_t*)v, pos, bias, ring);
  return hipGetLastError();
}

}  // namespace yoco
