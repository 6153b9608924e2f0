// The global K^/V^ cache in 8 bits (section 1 names 8-bit KV quantisation as the
// usual way to shrink the cache; the scheme here is plain absmax coding, one
// fp32 scale per row and KV head): the kernels that code rows into it and the
// split-KV decode pass that reads it. head_dim 128.
//
// Memory layout of a plane (one per sequence and KV head): blocks of 64 rows,
// 8448 bytes = 33 x 256 each: 8192 code bytes, then the 64 fp32 scales of the
// rows in row order. The code bytes are ordered so that each of the eight 1 KiB
// loads a wavefront issues per block (lane l reads bytes 16 l .. 16 l + 15) is
// a ready matrix-core operand:
//   K plane, code as a signed byte; row r, dim e sits at
//     ((((r / 4) % 4) * 2 + e / 64) * 64 + ((e % 64) / 16) * 16 + 4 * (r / 16) + r % 4) * 16 + e % 16
//     (load tau * 2 + half holds, for lane (n, qg), 16 dims of row 16 (n / 4) + 4 tau + n % 4);
//   V plane, byte = code + 128, transposed; row r, dim e sits at
//     ((e / 16) * 64 + (r / 16) * 16 + e % 16) * 16 + r % 16
//     (load t holds, for lane (n, qg), the 16 rows 16 qg .. of dim 16 t + n).
//
// Coding rule (float32 throughout, because a rounding decides the integer):
// a = max|x| over the row, scale = a / 127, code = rint(x * (127 / a)) clamped
// to +-127; a zero row has scale 0 and codes 0.
#include "yoco_common.h"

namespace yoco {

namespace {

constexpr int kD = 128;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kNegBig = -1.0e30f;

typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));

// ---------------------------------------------------------------- coding rows into the cache
// One wavefront per (row, KV head, K or V): lane l holds elements 2l and 2l + 1.
// pos == null: rows [n,Hkv,128] of sequence b_fixed go to slots pos0 + row;
// pos != null: one row per sequence ([B,Hkv,128]) goes to slot pos[b], skipped when outside [0, N_cap).
template <typename S>
__global__ void __launch_bounds__(256) kv_code_i8_kernel(yoco_kv_cache c, const S* __restrict__ k, const S* __restrict__ v,
                                                         const float* __restrict__ row_scale, int b_fixed, int64_t pos0, int64_t n,
                                                         const int64_t* __restrict__ pos) {
  const int lane = threadIdx.x & 63;
  const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (wave >= n * c.Hkv * 2) return;                       // uniform over the wavefront
  const int which = (int)(wave & 1);
  const int g = (int)((wave >> 1) % c.Hkv);
  const int64_t row = (wave >> 1) / c.Hkv;
  int b = b_fixed;
  int64_t slot = pos0 + row;
  if (pos) {
    b = (int)row;
    slot = pos[b];
    if (slot < 0 || slot >= c.N_cap) return;
  }
  const S* src = (which ? v : k) + (row * c.Hkv + g) * kD + lane * 2;
  const float rs = row_scale ? row_scale[row] : 1.f;       // the row as it is cached: float32(x * rs), then the coding rule
  const float x0 = Elem<S>::load(src) * rs, x1 = Elem<S>::load(src + 1) * rs;
  float a = fmaxf(fabsf(x0), fabsf(x1));
#pragma unroll
  for (int off = 32; off; off >>= 1) a = fmaxf(a, __shfl_xor(a, off));
  const float inv = a > 0.f ? 127.f / a : 0.f;
  const float scale = a > 0.f ? a / 127.f : 0.f;
  const float y0 = fminf(fmaxf(rintf(x0 * inv), -127.f), 127.f);
  const float y1 = fminf(fmaxf(rintf(x1 * inv), -127.f), 127.f);
  char* blk = (char*)(which ? c.v : c.k) + ((int64_t)b * c.Hkv + g) * i8_plane_bytes(c.N_cap) + (slot >> 6) * kI8BlockBytes;
  const int rho = (int)(slot & 63);
  if (which) {            // transposed plane: the row's bytes lie 16 apart
    blk[i8_v_offset(rho, lane * 2)] = (char)((int)y0 + 128);
    blk[i8_v_offset(rho, lane * 2 + 1)] = (char)((int)y1 + 128);
  } else {                // two neighbouring dims share a 16-byte piece
    *(unsigned short*)(blk + i8_k_offset(rho, lane * 2)) = (unsigned short)(((unsigned)(int)y0 & 0xffu) | (((unsigned)(int)y1 & 0xffu) << 8));
  }
  if (lane == 0) *(float*)(blk + kI8ScaleOffset + 4 * rho) = scale;
}

// Whole 64-row blocks: one workgroup per (block, KV head, plane), thread (rho = t / 4, part = t % 4) codes dims
// 32 part .. 32 part + 31 of block row rho. K codes leave as two 16-byte pieces per thread; V codes are transposed
// through LDS so that they leave as 16-byte pieces too. k, v point at the source row of the first block.
template <typename S> struct Row32;
template <> struct Row32<float> {
  static __device__ __forceinline__ void load(const float* p, float (&x)[32]) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const f32x4 a = *(const f32x4*)(p + 4 * i);
#pragma unroll
      for (int j = 0; j < 4; ++j) x[4 * i + j] = a[j];
    }
  }
};
template <> struct Row32<bf16_t> {
  static __device__ __forceinline__ void load(const bf16_t* p, float (&x)[32]) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const u32x4 a = *(const u32x4*)(p + 8 * i);
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        x[8 * i + 2 * j] = __uint_as_float(a[j] << 16);
        x[8 * i + 2 * j + 1] = __uint_as_float(a[j] & 0xffff0000u);
      }
    }
  }
};

template <typename S>
__global__ void __launch_bounds__(256) kv_code_i8_block_kernel(yoco_kv_cache c, const S* __restrict__ k, const S* __restrict__ v,
                                                               const float* __restrict__ row_scale, int b, int64_t blk0) {
  __shared__ __attribute__((aligned(16))) unsigned char tile[kI8ScaleOffset];
  const int t = threadIdx.x, rho = t >> 2, part = t & 3;
  const int g = blockIdx.y, which = blockIdx.z;
  const S* src = (which ? v : k) + (((int64_t)blockIdx.x * 64 + rho) * c.Hkv + g) * kD + part * 32;
  float x[32];
  Row32<S>::load(src, x);
  if (row_scale) {
    const float rs = row_scale[(int64_t)blockIdx.x * 64 + rho];
#pragma unroll
    for (int i = 0; i < 32; ++i) x[i] *= rs;
  }
  float a = 0.f;
#pragma unroll
  for (int i = 0; i < 32; ++i) a = fmaxf(a, fabsf(x[i]));
  a = fmaxf(a, __shfl_xor(a, 1));
  a = fmaxf(a, __shfl_xor(a, 2));
  const float inv = a > 0.f ? 127.f / a : 0.f;
  const float scale = a > 0.f ? a / 127.f : 0.f;
  int code[32];
#pragma unroll
  for (int i = 0; i < 32; ++i) code[i] = (int)fminf(fmaxf(rintf(x[i] * inv), -127.f), 127.f);
  char* blk = (char*)(which ? c.v : c.k) + ((int64_t)b * c.Hkv + g) * i8_plane_bytes(c.N_cap) + (blk0 + blockIdx.x) * kI8BlockBytes;
  if (which) {
#pragma unroll
    for (int i = 0; i < 32; ++i) tile[i8_v_offset(rho, part * 32 + i)] = (unsigned char)(code[i] + 128);
    __syncthreads();
    *(u32x4*)(blk + t * 32) = *(const u32x4*)(tile + t * 32);
    *(u32x4*)(blk + t * 32 + 16) = *(const u32x4*)(tile + t * 32 + 16);
  } else {
#pragma unroll
    for (int piece = 0; piece < 2; ++piece) {
      u32x4 w;
#pragma unroll
      for (int d4 = 0; d4 < 4; ++d4) {
        unsigned u = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) u |= ((unsigned)code[piece * 16 + d4 * 4 + j] & 0xffu) << (8 * j);
        w[d4] = u;
      }
      *(u32x4*)(blk + i8_k_offset(rho, part * 32 + piece * 16)) = w;
    }
  }
  if (part == 0) *(float*)(blk + kI8ScaleOffset + 4 * rho) = scale;
}

// ---------------------------------------------------------------- decode pass 1 over the coded cache
// Both contractions run on the matrix cores, whose operands are exactly what the block layout delivers:
//   scores  S^T[row][head] = K[row][dim] . q[head][dim]      v_mfma_i32_16x16x64_i8, K codes as loaded (no conversion);
//           q is split into two int8 parts per head, q = s1 * hi + (s1 / 254) * lo, which keeps 16 bits below max|q|
//   output  O^T[dim][head] += V^T[dim][row] . w[row][head]   v_mfma_f32_16x16x32_f16, V codes turned into exact fp16
//           integers (2 VALU ops per 4 codes), w = softmax weight * row scale in fp16, kept <= 1 by running its own maximum
// Lane (n = lane % 16, qg = lane / 16) owns head n (lanes n >= G idle along) and rows 16 qg .. 16 qg + 15 of a block,
// so up to 16 query heads per KV head cost the same as one.
__device__ __forceinline__ f16x2 as_f16x2(unsigned x) { return __builtin_bit_cast(f16x2, x); }

// Two code bytes (code + 128) -> two exact fp16 integers: a byte under exponent bits 0x64 is 1024 + byte, then - (1024 + 128).
template <unsigned SEL>
__device__ __forceinline__ unsigned codes_f16(unsigned w) {
  const unsigned p = __builtin_amdgcn_perm(0x64646464u, w, SEL);
  return __builtin_bit_cast(unsigned, as_f16x2(p) - (f16x2){(_Float16)1152.f, (_Float16)1152.f});
}
// 8 code bytes (two dwords) -> the 8 fp16 of one MFMA operand
__device__ __forceinline__ f16x8 codes8_f16(unsigned w0, unsigned w1) {
  const u32x4 r = {codes_f16<0x04010400u>(w0), codes_f16<0x04030402u>(w0), codes_f16<0x04010400u>(w1), codes_f16<0x04030402u>(w1)};
  return __builtin_bit_cast(f16x8, r);
}
__device__ __forceinline__ unsigned pack_f16(float a, float b) {      // round to nearest even
  return __builtin_bit_cast(unsigned, (f16x2){(_Float16)a, (_Float16)b});
}

struct Block {             // what a lane holds of one 64-row block
  u32x4 k[8];              // [tau * 2 + half]: K codes of row 16 (n / 4) + 4 tau + n % 4, dims 64 half + 16 qg ..
  u32x4 v[8];              // [t]: V codes of dim 16 t + n, rows 16 qg .. 16 qg + 15
  float ks, vs;            // scales of row `lane`: one coalesced 256-byte load per plane
};

struct State {
  float m, l, mo;          // running max of the scores, partial sum of weights, running max of score + log2(row scale of V)
  f32x4 o[8];              // O^T[16 t + 4 qg + i][n], relative to 2^mo
};

template <bool TAIL>
__device__ __forceinline__ void step(State& st, const i32x4 (&qhi)[2], const i32x4 (&qlo)[2], float qs, const Block& x, int qg,
                                     int nvalid, float (*sc)[64]) {
  // Lane (n, qg) needs the scales of rows 16 qg .. 16 qg + 15: pass them through the wavefront's own LDS lines
  // (a wavefront's LDS operations complete in order, so no barrier is involved).
  const int lane = threadIdx.x & 63;
  sc[0][lane] = x.ks;
  sc[1][lane] = x.vs;
  f32x4 ks[4], vs[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    ks[i] = *(const f32x4*)&sc[0][qg * 16 + i * 4];
    vs[i] = *(const f32x4*)&sc[1][qg * 16 + i * 4];
    if (TAIL) {   // rows past the end hold whatever the memory held (NaN bits included): zero their scales before any arithmetic
#pragma unroll
      for (int j = 0; j < 4; ++j)
        if (qg * 16 + i * 4 + j >= nvalid) { ks[i][j] = 0.f; vs[i][j] = 0.f; }
    }
  }
  float s[16], t[16];
  float smax = -INFINITY, tmax = -INFINITY;
#pragma unroll
  for (int tau = 0; tau < 4; ++tau) {
    i32x4 hi = {0, 0, 0, 0}, lo = {0, 0, 0, 0};
    hi = __builtin_amdgcn_mfma_i32_16x16x64_i8(__builtin_bit_cast(i32x4, x.k[tau * 2]), qhi[0], hi, 0, 0, 0);
    hi = __builtin_amdgcn_mfma_i32_16x16x64_i8(__builtin_bit_cast(i32x4, x.k[tau * 2 + 1]), qhi[1], hi, 0, 0, 0);
    lo = __builtin_amdgcn_mfma_i32_16x16x64_i8(__builtin_bit_cast(i32x4, x.k[tau * 2]), qlo[0], lo, 0, 0, 0);
    lo = __builtin_amdgcn_mfma_i32_16x16x64_i8(__builtin_bit_cast(i32x4, x.k[tau * 2 + 1]), qlo[1], lo, 0, 0, 0);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int r = tau * 4 + i;
      float a = (float)(__mul24(hi[i], 254) + lo[i]) * (ks[tau][i] * qs);   // |hi| < 2^21
      float b = a + __builtin_amdgcn_logf(vs[tau][i]);               // log2; a zero row of V gets -inf, weight 0
      if (TAIL && (qg * 16 + r >= nvalid)) { a = -INFINITY; b = -INFINITY; }   // rows past the end get weight 0
      s[r] = a;
      t[r] = b;
      smax = fmaxf(smax, a);
      tmax = fmaxf(tmax, b);
    }
  }
  // the four lanes of a head share the maxima: their rows meet in the same accumulators
  smax = fmaxf(smax, __shfl_xor(smax, 16));
  smax = fmaxf(smax, __shfl_xor(smax, 32));
  tmax = fmaxf(tmax, __shfl_xor(tmax, 16));
  tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
  const float m_new = fmaxf(st.m, smax), mo_new = fmaxf(st.mo, tmax);
  float psum = 0.f, w[16];
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    psum += __builtin_amdgcn_exp2f(s[r] - m_new);
    w[r] = __builtin_amdgcn_exp2f(t[r] - mo_new);
  }
  st.l = st.l * __builtin_amdgcn_exp2f(st.m - m_new) + psum;
  st.m = m_new;
  if (__builtin_amdgcn_ballot_w64(mo_new != st.mo)) {                  // rare once the stream has met its large scores
    const float alpha = __builtin_amdgcn_exp2f(st.mo - mo_new);
#pragma unroll
    for (int tt = 0; tt < 8; ++tt) st.o[tt] *= alpha;
    st.mo = mo_new;
  }
  const u32x4 pa = {pack_f16(w[0], w[1]), pack_f16(w[2], w[3]), pack_f16(w[4], w[5]), pack_f16(w[6], w[7])};
  const u32x4 pb = {pack_f16(w[8], w[9]), pack_f16(w[10], w[11]), pack_f16(w[12], w[13]), pack_f16(w[14], w[15])};
#pragma unroll
  for (int tt = 0; tt < 8; ++tt) {
    st.o[tt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(codes8_f16(x.v[tt][0], x.v[tt][1]), __builtin_bit_cast(f16x8, pa), st.o[tt], 0, 0, 0);
    st.o[tt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(codes8_f16(x.v[tt][2], x.v[tt][3]), __builtin_bit_cast(f16x8, pb), st.o[tt], 0, 0, 0);
  }
}

// Workgroup = 4 wavefronts on one (sequence, KV head, split); each wavefront walks a contiguous run of blocks,
// the next block's loads in flight while the current one is reduced. q, o are bf16.
// GMAX sizes the merge buffers (4 or 16 heads per KV head); G = Hq / Hkv <= GMAX is the real group size.
template <int GMAX>
__global__ void __launch_bounds__(256, 2) decode_i8_kernel(yoco_kv_cache c, const bf16_t* __restrict__ q,
                                                        const int64_t* __restrict__ lens, int64_t fixed_len, int Hq, float scale_log2,
                                                        float* __restrict__ ws, int splits, bf16_t* __restrict__ o_direct) {
  __shared__ float red_o[4][GMAX][kD];
  __shared__ float red_ml[4][GMAX][2];
  const int G = Hq / c.Hkv;
  __shared__ __attribute__((aligned(16))) float scales[4][2][64];
  const int sp = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int n = lane & 15, qg = lane >> 4;

  const int64_t len_raw = lens ? lens[b] : fixed_len;
  const int64_t len = len_raw < 0 ? 0 : (len_raw > c.N_cap ? c.N_cap : len_raw);
  const int64_t chunk = (((len + splits - 1) / splits) + 255) & ~(int64_t)255;   // rows per split, 256 | chunk
  const int64_t j_lo = sp * chunk;
  const int64_t j_hi = (j_lo + chunk < len) ? j_lo + chunk : len;
  const int64_t sub = chunk >> 2;                                                // rows per wave, 64 | sub
  const int64_t w_lo = j_lo + wave * sub;
  const int64_t w_hi = (w_lo + sub < j_hi) ? w_lo + sub : j_hi;

  // The query of head n as two int8 operands: dims 64 half + 16 qg + j in byte j of half `half`.
  i32x4 qhi[2] = {{0, 0, 0, 0}, {0, 0, 0, 0}}, qlo[2] = {{0, 0, 0, 0}, {0, 0, 0, 0}};
  float qs = 0.f;
  {
    float x[32];
#pragma unroll
    for (int i = 0; i < 32; ++i) x[i] = 0.f;
    if (n < G) {
      const bf16_t* qp = q + ((int64_t)b * Hq + g * G + n) * kD + qg * 16;
#pragma unroll
      for (int half = 0; half < 2; ++half) {
        const u32x4 a = *(const u32x4*)(qp + half * 64), bq = *(const u32x4*)(qp + half * 64 + 8);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const unsigned w = i < 4 ? a[i] : bq[i - 4];
          x[half * 16 + 2 * i] = __uint_as_float(w << 16);
          x[half * 16 + 2 * i + 1] = __uint_as_float(w & 0xffff0000u);
        }
      }
    }
    float amax = 0.f;
#pragma unroll
    for (int i = 0; i < 32; ++i) amax = fmaxf(amax, fabsf(x[i]));
    amax = fmaxf(amax, __shfl_xor(amax, 16));
    amax = fmaxf(amax, __shfl_xor(amax, 32));
    const float s1 = amax / 127.f, s2 = amax / 32258.f;                          // 32258 = 127 * 254
    const float inv1 = amax > 0.f ? 127.f / amax : 0.f, inv2 = amax > 0.f ? 32258.f / amax : 0.f;
#pragma unroll
    for (int half = 0; half < 2; ++half) {
#pragma unroll
      for (int wd = 0; wd < 4; ++wd) {
        unsigned ph = 0, pl = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const float v = x[half * 16 + wd * 4 + j];
          const float h = fminf(fmaxf(rintf(v * inv1), -127.f), 127.f);
          const float lo = fminf(fmaxf(rintf(fmaf(-h, s1, v) * inv2), -127.f), 127.f);
          ph |= ((unsigned)(int)h & 0xffu) << (8 * j);
          pl |= ((unsigned)(int)lo & 0xffu) << (8 * j);
        }
        qhi[half][wd] = (int)ph;
        qlo[half][wd] = (int)pl;
      }
    }
    qs = s2 * scale_log2;
  }

  State st;
  st.m = kNegBig;
  st.mo = kNegBig;
  st.l = 0.f;
#pragma unroll
  for (int tt = 0; tt < 8; ++tt) st.o[tt] = (f32x4){0.f, 0.f, 0.f, 0.f};

  const int64_t plane = ((int64_t)b * c.Hkv + g) * (i8_plane_bytes(c.N_cap) / 16);   // in 16-byte units
  const u32x4* kp = (const u32x4*)c.k + plane;
  const u32x4* vp = (const u32x4*)c.v + plane;

  if (w_lo < w_hi) {
    Block nx;
    auto load = [&](int64_t row0) {                       // row0 is a multiple of 64
      const int64_t base = (row0 >> 6) * (kI8BlockBytes / 16);
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        nx.k[u] = __builtin_nontemporal_load(kp + base + u * 64 + lane);
        nx.v[u] = __builtin_nontemporal_load(vp + base + u * 64 + lane);
      }
      nx.ks = __builtin_nontemporal_load((const float*)(kp + base + kI8ScaleOffset / 16) + lane);
      nx.vs = __builtin_nontemporal_load((const float*)(vp + base + kI8ScaleOffset / 16) + lane);
    };
    load(w_lo);
    int64_t row0 = w_lo;
    for (; row0 + 64 < w_hi; row0 += 64) {
      const Block cur = nx;
      load(row0 + 64);
      step<false>(st, qhi, qlo, qs, cur, qg, 64, scales[wave]);
    }
    step<true>(st, qhi, qlo, qs, nx, qg, (int)(w_hi - row0), scales[wave]);   // last block of the run, 1..64 rows
  }

  // One state per head and wavefront: gather the partial sums of the four row groups, rebase the output on 2^m.
  float l = st.l;
  l += __shfl_xor(l, 16);
  l += __shfl_xor(l, 32);
  const float f = __builtin_amdgcn_exp2f(st.mo - st.m);   // the output's own maximum differs by the V scales: finite
  if (n < G) {
#pragma unroll
    for (int tt = 0; tt < 8; ++tt)
#pragma unroll
      for (int i = 0; i < 4; ++i) red_o[wave][n][tt * 16 + qg * 4 + i] = st.o[tt][i] * f;
    if (qg == 0) { red_ml[wave][n][0] = st.m; red_ml[wave][n][1] = l; }
  }
  __syncthreads();
  for (int t = threadIdx.x; t < G * kD; t += 256) {
    const int h = t / kD, e = t % kD;
    const float M = fmaxf(fmaxf(red_ml[0][h][0], red_ml[1][h][0]), fmaxf(red_ml[2][h][0], red_ml[3][h][0]));
    float ls = 0.f, o = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const float fw = __builtin_amdgcn_exp2f(red_ml[w][h][0] - M);
      ls = fmaf(fw, red_ml[w][h][1], ls);
      o = fmaf(fw, red_o[w][h][e], o);
    }
    if (o_direct) {
      o_direct[((size_t)b * Hq + g * G + h) * kD + e] = f32_to_bf16(ls > 0.f ? o / ls : 0.f);
      continue;
    }
    float* out = ws + (((size_t)b * Hq + g * G + h) * splits + sp) * partial_stride(kD);
    out[e] = o;
    if (e == 0) {
      out[kD] = (ls > 0.f) ? M * kLn2 : -INFINITY;
      out[kD + 1] = ls;
    }
  }
}

}  // namespace

bool cache_i8_supported(int d) { return d == kD; }

bool decode_i8_supported(const yoco_kv_cache& c, int Hq) {
  if (c.dtype != YOCO_INT8 || c.d != kD) return false;
  const int G = Hq / c.Hkv;
  return G >= 1 && G <= 16 && c.Hkv <= 65535;
}

hipError_t launch_kv_code_i8(const yoco_kv_cache& c, const void* k, const void* v, const float* row_scale, int b, int64_t pos0,
                             int64_t n, const int64_t* pos, int src_dtype, hipStream_t s) {
  // rows [r0, r1) of the source, one wavefront per (row, head, plane)
  auto by_rows = [&](int64_t r0, int64_t r1, int64_t slot0) {
    if (r1 <= r0) return;
    const int64_t waves = (r1 - r0) * c.Hkv * 2;
    const size_t skip = (size_t)r0 * c.Hkv * kD;
    dim3 grid((unsigned)((waves + 3) / 4)), block(256);
    const float* rs = row_scale ? row_scale + r0 : nullptr;
    if (src_dtype == YOCO_F32)
      hipLaunchKernelGGL(kv_code_i8_kernel<float>, grid, block, 0, s, c, (const float*)k + skip, (const float*)v + skip, rs, b, slot0, r1 - r0, pos);
    else
      hipLaunchKernelGGL(kv_code_i8_kernel<bf16_t>, grid, block, 0, s, c, (const bf16_t*)k + skip, (const bf16_t*)v + skip, rs, b, slot0, r1 - r0, pos);
  };
  if (pos) {                                  // one row per sequence at device-side positions
    by_rows(0, c.B, 0);
    return hipGetLastError();
  }
  // rows that fill whole 64-row blocks go block by block, the ragged head and tail row by row
  const int64_t end = pos0 + n;
  const int64_t first_full = ((pos0 + 63) / 64) * 64, last_full = (end / 64) * 64;
  if (last_full <= first_full) {
    by_rows(0, n, pos0);
    return hipGetLastError();
  }
  by_rows(0, first_full - pos0, pos0);
  {
    const size_t skip = (size_t)(first_full - pos0) * c.Hkv * kD;
    dim3 grid((unsigned)((last_full - first_full) / 64), c.Hkv, 2), block(256);
    const float* rs = row_scale ? row_scale + (first_full - pos0) : nullptr;
    if (src_dtype == YOCO_F32)
      hipLaunchKernelGGL(kv_code_i8_block_kernel<float>, grid, block, 0, s, c, (const float*)k + skip, (const float*)v + skip, rs, b, first_full / 64);
    else
      hipLaunchKernelGGL(kv_code_i8_block_kernel<bf16_t>, grid, block, 0, s, c, (const bf16_t*)k + skip, (const bf16_t*)v + skip, rs, b, first_full / 64);
  }
  by_rows(last_full - pos0, n, last_full);
  return hipGetLastError();
}

hipError_t launch_decode_i8(const yoco_kv_cache& c, const void* q, const int64_t* lens, int64_t fixed_len, int Hq, float scale,
                            float* ws, int splits, void* o_direct, hipStream_t s) {
  bf16_t* od = splits == 1 ? (bf16_t*)o_direct : nullptr;
  dim3 grid(splits, c.Hkv, c.B), block(256);
  const float sl2 = scale * kLog2e;
  const bf16_t* qp = (const bf16_t*)q;
  const int G = Hq / c.Hkv;
  if (G < 1 || G > 16) return hipErrorInvalidValue;
  if (G <= 4)
    hipLaunchKernelGGL(decode_i8_kernel<4>, grid, block, 0, s, c, qp, lens, fixed_len, Hq, sl2, ws, splits, od);
  else
    hipLaunchKernelGGL(decode_i8_kernel<16>, grid, block, 0, s, c, qp, lens, fixed_len, Hq, sl2, ws, splits, od);
  return hipGetLastError();
}

}  // namespace yoco
