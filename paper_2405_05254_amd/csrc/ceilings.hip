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

hipError_t launch_stream_read(const void* buf, size_t bytes, void* sink, int workgroups, hipStream_t s) {
  hipLaunchKernelGGL(stream_read_kernel, dim3(workgroups), dim3(256), 0, s, (const u32x4*)buf, bytes / 16, (unsigned*)sink);
  return hipGetLastError();
}

}  // namespace yoco
