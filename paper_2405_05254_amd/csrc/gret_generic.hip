// Gated retention in its recurrent form (section 3.1, Eq. 5):
//   S_n = gamma_n S_{n-1} + K_n^T V_n,   o_n = scale * Q_n S_n,
// optionally followed by the per-head GroupNorm of Eq. 7 (no learned affine)
// and the multiplication by swish(gate) of the same equation.
// fp32 arithmetic on the vector ALU for any storage dtype and head dims up to
// 128. It is the decode step of the self-decoder (one row per sequence, the
// state read and written once: HBM-bound) and the prefill path of every shape
// the chunkwise MFMA kernels do not cover; the chunk size plays no part here
// because the recurrent and chunkwise forms are the same function.
//
// One workgroup owns one (sequence, head) and keeps the whole state in
// registers, transposed: thread (rr = tid / 32, kk = tid % 32) holds
// S^T[ev][4 kk .. 4 kk + 3] for the rows ev = rr + 8 r. A row of S^T is
// contiguous along the key dimension, so the 32 lanes of a half wavefront
// read and write 512 contiguous bytes, and o[ev] = q . S^T[ev] is a butterfly
// over those 32 lanes: no LDS and no barrier on the path without GroupNorm.
#include "yoco_common.h"

namespace yoco {

namespace {

constexpr int kMaxDim = 128;
constexpr int kRowsPerThread = kMaxDim / 8;

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

template <typename T> __device__ __forceinline__ f32x4 load4(const T* p);
template <> __device__ __forceinline__ f32x4 load4<float>(const float* p) { return *(const f32x4*)p; }
template <> __device__ __forceinline__ f32x4 load4<bf16_t>(const bf16_t* p) {
  const u32x2 w = *(const u32x2*)p;
  f32x4 r = {__uint_as_float(w[0] << 16), __uint_as_float(w[0] & 0xffff0000u), __uint_as_float(w[1] << 16),
             __uint_as_float(w[1] & 0xffff0000u)};
  return r;
}

__device__ __forceinline__ float half_wave_sum(float x) {      // over the 32 lanes that share tid / 32
  for (int o = 16; o > 0; o >>= 1) x += __shfl_xor(x, o);
  return x;
}

// Sum of one value per thread over the workgroup; every thread gets the result.
__device__ __forceinline__ float block_sum(float x, float* red) {
  for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o);
  __syncthreads();                                  // the previous use of red[] is over
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = x;
  __syncthreads();
  return red[0] + red[1] + red[2] + red[3];
}

template <typename T>
__global__ void __launch_bounds__(256) gret_recurrent_kernel(GretView a) {
  __shared__ float red[4];
  const int h = blockIdx.x, b = blockIdx.y;
  const int kk = threadIdx.x & 31, rr = threadIdx.x >> 5;
  const int ek = kk * 4;
  const bool k_on = ek < a.dk;
  const int n_rows = (a.dv - rr + 7) / 8;                 // rows rr, rr + 8, ... below dv

  f32x4 S[kRowsPerThread];
  const size_t st_off = ((size_t)b * a.H + h) * a.dv * a.dk;
#pragma unroll
  for (int r = 0; r < kRowsPerThread; ++r) {
    S[r] = f32x4{0.f, 0.f, 0.f, 0.f};
    if (a.state_in && k_on && r < n_rows) S[r] = *(const f32x4*)(a.state_in + st_off + (size_t)(rr + 8 * r) * a.dk + ek);
  }

  const T* q = (const T*)a.q + ((size_t)b * a.T * a.H + h) * a.dk;
  const T* k = (const T*)a.k + ((size_t)b * a.T * a.H + h) * a.dk;
  const T* v = (const T*)a.v + ((size_t)b * a.T * a.H + h) * a.dv;
  T* o = (T*)a.o + ((size_t)b * a.T * a.H + h) * a.dv;
  const float* g = a.log_gamma + (size_t)b * a.T * a.H + h;
  const float inv_dv = 1.f / (float)a.dv;

  for (int64_t n = 0; n < a.T; ++n) {
    const float gamma = __expf(g[n * a.H]);
    f32x4 kf = {0.f, 0.f, 0.f, 0.f}, qf = kf;
    if (k_on) {
      kf = load4<T>(k + n * a.H * a.dk + ek);
      qf = load4<T>(q + n * a.H * a.dk + ek);
    }
    float out[kRowsPerThread];
    float sum = 0.f;
    const bool store_state = a.state_out && k_on && n == a.T - 1;
#pragma unroll
    for (int r = 0; r < kRowsPerThread; ++r) {
      out[r] = 0.f;
      if (r < n_rows) {
        const float vv = Elem<T>::load(v + n * a.H * a.dv + rr + 8 * r);
        S[r] = gamma * S[r] + kf * vv;
        // the final state leaves row by row, while later rows of a decode step are still arriving
        if (store_state) *(f32x4*)(a.state_out + st_off + (size_t)(rr + 8 * r) * a.dk + ek) = S[r];
        const float part = qf[0] * S[r][0] + qf[1] * S[r][1] + qf[2] * S[r][2] + qf[3] * S[r][3];
        out[r] = a.scale * half_wave_sum(part);
        sum += out[r];
      }
    }
    if (a.group_norm) {
      // every lane of a half wavefront holds the same out[]: count each row once
      const float mean = block_sum(kk == 0 ? sum : 0.f, red) * inv_dv;
      float sq = 0.f;
#pragma unroll
      for (int r = 0; r < kRowsPerThread; ++r)
        if (r < n_rows) sq += (out[r] - mean) * (out[r] - mean);
      const float var = block_sum(kk == 0 ? sq : 0.f, red) * inv_dv;
      const float rstd = rsqrtf(var + a.eps);
#pragma unroll
      for (int r = 0; r < kRowsPerThread; ++r) out[r] = (out[r] - mean) * rstd;
    }
    if (kk == 0) {
      const T* gate = a.gate ? (const T*)a.gate + ((size_t)b * a.T * a.H + h) * a.dv + n * a.H * a.dv : nullptr;
#pragma unroll
      for (int r = 0; r < kRowsPerThread; ++r)
        if (r < n_rows) {
          float y = out[r];
          if (gate) {                                   // swish gate of Eq. 7: y * g * sigmoid(g)
            const float gv = Elem<T>::load(gate + rr + 8 * r);
            y *= gv / (1.f + __expf(-gv));
          }
          Elem<T>::store(o + n * a.H * a.dv + rr + 8 * r, y);
        }
    }
  }

}

// ---- the decode step (T = 1) at dk = dv = 128, state updated in place: same thread -> state mapping as above, but
// written for the memory system. The small operands are requested before the state, so that the first rows can be
// worked on as soon as they land (loads come back in issue order); the state moves in four quarters of four rows per
// thread with two quarters in flight, and a quarter is stored as soon as it is updated, so the launch reads and writes
// at the same time instead of in two phases; the 16 row sums of a thread are reduced together (at every exchange a
// lane keeps half of its rows: 16 exchanges instead of 80), after which lane pair kk / 2 of a half wavefront holds
// row rr + 8 (kk / 2).
template <typename T>
__global__ void __launch_bounds__(256) gret_decode_kernel(GretView a) {
  constexpr int kDim = 128;
  __shared__ float red[4];
  const int h = blockIdx.x, b = blockIdx.y;
  const int kk = threadIdx.x & 31, rr = threadIdx.x >> 5;
  const int ek = kk * 4;
  const size_t bh = (size_t)b * a.H + h;
  const T* q = (const T*)a.q + bh * kDim;
  const T* k = (const T*)a.k + bh * kDim;
  const T* v = (const T*)a.v + bh * kDim;
  float* st = a.state_out + bh * kDim * kDim + (size_t)rr * kDim + ek;    // row rr + 8 r is 8 r rows further

  const float gamma = __expf(a.log_gamma[bh]);
  const f32x4 kf = load4<T>(k + ek), qf = load4<T>(q + ek);
  float vv[16];
#pragma unroll
  for (int r = 0; r < 16; ++r) vv[r] = Elem<T>::load(v + rr + 8 * r);

  f32x4 S[16];
  auto load_quarter = [&](int qt) {
#pragma unroll
    for (int r = 4 * qt; r < 4 * qt + 4; ++r) S[r] = __builtin_nontemporal_load((const f32x4*)(st + (size_t)r * 8 * kDim));
  };
  float part[16];
  load_quarter(0);
  load_quarter(1);
#pragma unroll
  for (int qt = 0; qt < 4; ++qt) {
    if (qt + 2 < 4) load_quarter(qt + 2);
#pragma unroll
    for (int r = 4 * qt; r < 4 * qt + 4; ++r) {
      S[r] = gamma * S[r] + kf * vv[r];
      __builtin_nontemporal_store(S[r], (f32x4*)(st + (size_t)r * 8 * kDim));
      part[r] = qf[0] * S[r][0] + qf[1] * S[r][1] + qf[2] * S[r][2] + qf[3] * S[r][3];
    }
  }
  // reduce-scatter over the 32 lanes of the half wavefront
#pragma unroll
  for (int w = 8, o = 16; w >= 1; w >>= 1, o >>= 1) {       // w rows stay per lane after the exchange with lane ^ o
    const bool upper = (kk & o) != 0;
#pragma unroll
    for (int i = 0; i < w; ++i) {
      const float send = upper ? part[i] : part[i + w];
      const float keep = upper ? part[i + w] : part[i];
      part[i] = keep + __shfl_xor(send, o);
    }
  }
  float out = a.scale * (part[0] + __shfl_xor(part[0], 1));
  const int ev = rr + 8 * (kk >> 1);                         // the row this lane pair holds: bit o of kk chose its half at exchange o
  if (a.group_norm) {
    const float inv_dv = 1.f / (float)kDim;
    const float mean = block_sum((kk & 1) ? 0.f : out, red) * inv_dv;
    const float dlt = out - mean;
    const float var = block_sum((kk & 1) ? 0.f : dlt * dlt, red) * inv_dv;
    out = dlt * rsqrtf(var + a.eps);
  }
  if (!(kk & 1)) {
    if (a.gate) {                                            // swish gate of Eq. 7: y * g * sigmoid(g)
      const float gv = Elem<T>::load((const T*)a.gate + bh * kDim + ev);
      out *= gv / (1.f + __expf(-gv));
    }
    Elem<T>::store((T*)a.o + bh * kDim + ev, out);
  }
}

__global__ void __launch_bounds__(256) fill_zero_kernel(float* p, size_t n) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = 0.f;
}

}  // namespace

// A fill kernel, not a memset: a caller may be capturing the stream into a graph.
hipError_t launch_fill_zero(float* p, size_t n, hipStream_t s) {
  size_t blocks = (n + 255) / 256;
  if (blocks > 4096) blocks = 4096;
  if (blocks == 0) return hipSuccess;
  hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)blocks), dim3(256), 0, s, p, n);
  return hipGetLastError();
}

bool gret_recurrent_supported(const GretView& a) {
  return a.dk <= kMaxDim && a.dv <= kMaxDim && a.dk % 4 == 0 && a.B <= 65535;
}

hipError_t launch_gret_recurrent(const GretView& a, int dtype, hipStream_t s) {
  dim3 grid(a.H, a.B), block(256);
  if (a.T == 1 && a.dk == 128 && a.dv == 128 && a.state_in && a.state_in == a.state_out) {   // the decode step
    if (dtype == YOCO_F32)
      hipLaunchKernelGGL(gret_decode_kernel<float>, grid, block, 0, s, a);
    else
      hipLaunchKernelGGL(gret_decode_kernel<bf16_t>, grid, block, 0, s, a);
    return hipGetLastError();
  }
  if (dtype == YOCO_F32)
    hipLaunchKernelGGL(gret_recurrent_kernel<float>, grid, block, 0, s, a);
  else
    hipLaunchKernelGGL(gret_recurrent_kernel<bf16_t>, grid, block, 0, s, a);
  return hipGetLastError();
}

}  // namespace yoco
