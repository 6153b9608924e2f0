// Two microbenchmarks that tell what this GPU can do, so that the fractions of
// the published peaks can be read against measured ceilings (clocks under load
// are below their nominal value, and the MFMA rate depends on the operand
// data). They are measurement aids, not part of the attention path.
#include "mfma_util.h"
#include "yoco_common.h"

namespace yoco {

namespace {

// Back-to-back v_mfma_f32_32x32x16_bf16 on register operands: four independent
// accumulator chains per wavefront, two wavefronts per SIMD (the occupancy of
// the prefill kernel). Operands are read once from `seed` (the caller decides
// whether they are zeros or random values).
__global__ void __launch_bounds__(512) mfma_ceiling_kernel(const u32x4* __restrict__ seed, float* __restrict__ sink,
                                                           int iters) {
  const int t = threadIdx.x;
  const bf16x8 a = __builtin_bit_cast(bf16x8, seed[t]);
  const bf16x8 b = __builtin_bit_cast(bf16x8, seed[512 + t]);
  f32x16 acc[4];
#pragma unroll
  for (int c = 0; c < 4; ++c)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[c][r] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int u = 0; u < 8; ++u) acc[u & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[u & 3], 0, 0, 0);
  }
  float r = 0.f;
#pragma unroll
  for (int c = 0; c < 4; ++c)
#pragma unroll
    for (int i = 0; i < 16; ++i) r += acc[c][i];
  if (r == 1.2345678f) sink[0] = r;            // keeps the chains alive; practically never taken
}

// The inner loop of flash attention without the rest of the kernel (no staging, masks, barriers or tile walk): what the
// matrix pipe sustains when it is fed the way the prefill kernel feeds it. Two wavefronts per SIMD, 32 MFMAs per trip.
//   mode 1: the A operand of every MFMA is a fresh 128-bit LDS fragment (conflict-free pattern, read four ahead);
//   mode 2: mode 1 plus, after every second MFMA, the softmax work of two scores (2 fma, 2 exp2, one fp16 pack, one
//           dot2 for the row sum): 32 scores per lane and 32 MFMAs, the ratio of the attention loop at head_dim 128.
// LDS is filled from `seed` (16 KiB, repeated).
template <int MODE>
__global__ void __launch_bounds__(512) attn_loop_ceiling_kernel(const u32x4* __restrict__ seed, float* __restrict__ sink, int iters) {
  __shared__ __attribute__((aligned(1024))) char lds[65536];
  for (int i = threadIdx.x; i < 4096; i += 512) ((u32x4*)lds)[i] = seed[i & 1023];
  __syncthreads();
  const int t = threadIdx.x, lane = t & 63, lq = lane & 31, hf = lane >> 5;
  const int off0 = lq * 256 + ((hf ^ (lq & 15)) << 4);     // row lq, 16-byte chunk hf ^ (row & 15): one fragment, no bank conflicts
  const lds_char* lb = (const lds_char*)lds;
  auto frag = [&](int f, int it) __attribute__((always_inline)) {
    return __builtin_bit_cast(bf16x8, *(const __attribute__((address_space(3))) u32x4*)(lb + ((off0 ^ ((f & 7) << 5)) + ((f >> 3) & 3) * 8192 + (it & 1) * 32768)));
  };
  const bf16x8 b = __builtin_bit_cast(bf16x8, seed[512 + (t & 511)]);
  f32x16 acc[4];
#pragma unroll
  for (int c = 0; c < 4; ++c)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[c][r] = 0.f;
  float sc[16], l = 0.f, cs = 0.37f, cm = 0.01f;
#pragma unroll
  for (int j = 0; j < 16; ++j) sc[j] = __uint_as_float((seed[(t + j) & 1023][0] & 0x007fffffu) | 0x3f000000u) - 0.75f;   // scores in [-0.25, 0.25)
  asm volatile("" : "+v"(cs), "+v"(cm));
  for (int it = 0; it < iters; ++it) {
    constexpr int kAhead = 4;
    bf16x8 fr[32 + kAhead];
#pragma unroll
    for (int f = 0; f < kAhead; ++f) fr[f] = frag(f, it);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < 32; ++i) {
      if (i + kAhead < 32) fr[i + kAhead] = frag(i + kAhead, it);
      acc[i & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[i], b, acc[i & 3], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      if (MODE == 2 && (i & 1)) {
        float& s0 = sc[i & 15];
        float& s1 = sc[(i + 1) & 15];
        asm volatile("" : "+v"(s0), "+v"(s1));               // the scores change from MFMA to MFMA in the real loop: no hoisting
        const unsigned w = pack_f16(__builtin_amdgcn_exp2f(fmaf(s0, cs, -cm)), __builtin_amdgcn_exp2f(fmaf(s1, cs, -cm)));
        l = __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2, w), __builtin_bit_cast(f16x2, 0x3c003c00u), l, false);
        asm volatile("" : "+v"(l));
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  float r = l;
#pragma unroll
  for (int c = 0; c < 4; ++c)
#pragma unroll
    for (int i = 0; i < 16; ++i) r += acc[c][i];
  if (r == 1.2345678f) sink[0] = r;
}

// Streaming read: every workgroup walks its own contiguous share with 128-bit
// nontemporal loads, sixteen in flight per lane (the access pattern of decode).
__global__ void __launch_bounds__(256) stream_read_kernel(const u32x4* __restrict__ buf, size_t n16, unsigned* __restrict__ sink) {
  const size_t per = (n16 + gridDim.x - 1) / gridDim.x;
  const size_t lo = (size_t)blockIdx.x * per, hi = lo + per < n16 ? lo + per : n16;
  unsigned x = 0;
  size_t i = lo + threadIdx.x;
  constexpr int kDepth = 16;                       // 128-bit loads in flight per lane
  for (; i + (kDepth - 1) * 256 < hi; i += kDepth * 256) {
    u32x4 v[kDepth];
#pragma unroll
    for (int u = 0; u < kDepth; ++u) v[u] = __builtin_nontemporal_load(buf + i + u * 256);
#pragma unroll
    for (int u = 0; u < kDepth; ++u) x ^= v[u][0] ^ v[u][1] ^ v[u][2] ^ v[u][3];
  }
  for (; i < hi; i += 256) {
    const u32x4 v = __builtin_nontemporal_load(buf + i);
    x ^= v[0] ^ v[1] ^ v[2] ^ v[3];
  }
  if (x == 0x9e3779b9u) sink[0] = x;
}

}  // namespace

hipError_t launch_mfma_ceiling(const void* seed, void* sink, int iters, int workgroups, hipStream_t s) {
  hipLaunchKernelGGL(mfma_ceiling_kernel, dim3(workgroups), dim3(512), 0, s, (const u32x4*)seed, (float*)sink, iters);
  return hipGetLastError();
}

hipError_t launch_attn_loop_ceiling(const void* seed, void* sink, int iters, int workgroups, int mode, hipStream_t s) {
  if (mode == 1)
    hipLaunchKernelGGL(attn_loop_ceiling_kernel<1>, dim3(workgroups), dim3(512), 0, s, (const u32x4*)seed, (float*)sink, iters);
  else
    hipLaunchKernelGGL(attn_loop_ceiling_kernel<2>, dim3(workgroups), dim3(512), 0, s, (const u32x4*)seed, (float*)sink, iters);
  return hipGetLastError();
}

hipError_t launch_stream_read(const void* buf, size_t bytes, void* sink, int workgroups, hipStream_t s) {
  hipLaunchKernelGGL(stream_read_kernel, dim3(workgroups), dim3(256), 0, s, (const u32x4*)buf, bytes / 16, (unsigned*)sink);
  return hipGetLastError();
}

}  // namespace yoco
