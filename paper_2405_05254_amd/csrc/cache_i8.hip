// The global K^/V^ cache in 8 bits (section 1 names 8-bit KV quantisation as the
// usual way to shrink the cache; the scheme here is plain absmax coding, one
// fp32 scale per row and KV head): the kernels that code rows into it and the
// split-KV decode pass that reads it. head_dim 128.
//
// Memory layout of a plane (one per sequence and KV head): blocks of 64 rows;
// a block is 64 x 128 code bytes (byte = code + 128, code in [-127, 127])
// followed by the 64 fp32 scales of its rows, 8448 bytes = 33 x 256 in all, so a
// wavefront streams a block with eight 1 KiB loads plus one 256-byte line and
// never leaves contiguous memory. The scale of block row rho sits at index
// (rho % 8) * 8 + rho / 8: the 8 lanes that share rows rho = r, r + 8, ... of a
// step find their 8 scales in one 32-byte piece.
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

// ---------------------------------------------------------------- coding rows into the cache
// One wavefront per (row, KV head, K or V): lane l holds elements 2l and 2l + 1.
// pos == null: rows [n,Hkv,128] of sequence b_fixed go to slots pos0 + row;
// pos != null: one row per sequence ([B,Hkv,128]) goes to slot pos[b], skipped when outside [0, N_cap).
template <typename S>
__global__ void __launch_bounds__(256) kv_code_i8_kernel(yoco_kv_cache c, const S* __restrict__ k, const S* __restrict__ v,
                                                         int b_fixed, int64_t pos0, int64_t n, const int64_t* __restrict__ pos) {
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
  const float x0 = Elem<S>::load(src), x1 = Elem<S>::load(src + 1);
  float a = fmaxf(fabsf(x0), fabsf(x1));
#pragma unroll
  for (int off = 32; off; off >>= 1) a = fmaxf(a, __shfl_xor(a, off));
  const float inv = a > 0.f ? 127.f / a : 0.f;
  const float scale = a > 0.f ? a / 127.f : 0.f;
  const float y0 = fminf(fmaxf(rintf(x0 * inv), -127.f), 127.f);
  const float y1 = fminf(fmaxf(rintf(x1 * inv), -127.f), 127.f);
  const unsigned w = (unsigned)((int)y0 + 128) | ((unsigned)((int)y1 + 128) << 8);
  char* blk = (char*)(which ? c.v : c.k) + ((int64_t)b * c.Hkv + g) * i8_plane_bytes(c.N_cap) + (slot >> 6) * kI8BlockBytes;
  const int rho = (int)(slot & 63);
  *(unsigned short*)(blk + rho * kD + lane * 2) = (unsigned short)w;
  if (lane == 0) *(float*)(blk + kI8ScaleOffset + 4 * i8_scale_index(rho)) = scale;
}

// ---------------------------------------------------------------- decode pass 1 over the coded cache
__device__ __forceinline__ f16x2 as_f16x2(unsigned x) { return __builtin_bit_cast(f16x2, x); }

// Two code bytes -> two exact fp16 integers: the byte under exponent bits 0x64 is 1024 + byte, then - (1024 + 128).
template <unsigned SEL>
__device__ __forceinline__ f16x2 codes_f16(unsigned w) {
  const unsigned p = __builtin_amdgcn_perm(0x64646464u, w, SEL);
  return as_f16x2(p) - (f16x2){(_Float16)1152.f, (_Float16)1152.f};
}
__device__ __forceinline__ void row_codes_f16(const u32x4& w, f16x2 (&out)[8]) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    out[2 * i] = codes_f16<0x04010400u>(w[i]);       // bytes 0, 1
    out[2 * i + 1] = codes_f16<0x04030402u>(w[i]);   // bytes 2, 3
  }
}

template <int CTRL>
__device__ __forceinline__ float dpp_add(float x) {
  int y = __builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xf, 0xf, true);
  return x + __int_as_float(y);
}
__device__ __forceinline__ float row8_sum(float x) {   // sum over 8 consecutive lanes, every lane gets the total
  x = dpp_add<0xB1>(x);    // quad_perm [1,0,3,2]
  x = dpp_add<0x4E>(x);    // quad_perm [2,3,0,1]
  x = dpp_add<0x141>(x);   // row_half_mirror: quads 0<->1, 2<->3
  return x;
}

constexpr int R = 8;       // rows per lane and step; 8 lanes share a row, so a step is one 64-row block

template <int G>
struct State {
  float m[G], l[G], o[G][16];
};

struct Block {             // what a lane holds of one block: 16 code bytes of 8 rows of K and V, and those rows' scales
  u32x4 k[R], v[R];
  f32x4 ks[2], vs[2];
};

template <int G, bool TAIL>
__device__ __forceinline__ void step(State<G>& st, const f16x2 (&qh)[G][8], const Block& x, float scale_log2, int r, int nvalid) {
  float s[R][G];
#pragma unroll
  for (int u = 0; u < R; ++u) {
    f16x2 kk[8];
    row_codes_f16(x.k[u], kk);
    const float f = x.ks[u >> 2][u & 3] * scale_log2;
#pragma unroll
    for (int h = 0; h < G; ++h) {
      float a = 0.f;
#pragma unroll
      for (int i = 0; i < 8; ++i) a = __builtin_amdgcn_fdot2(qh[h][i], kk[i], a, false);
      a = row8_sum(a) * f;
      if (TAIL && (u * 8 + r >= nvalid)) a = -INFINITY;     // also discards whatever an unwritten scale holds
      s[u][h] = a;
    }
  }
  float pv[R][G];
#pragma unroll
  for (int h = 0; h < G; ++h) {
    float mx = s[0][h];
#pragma unroll
    for (int u = 1; u < R; ++u) mx = fmaxf(mx, s[u][h]);
    const float m_new = fmaxf(st.m[h], mx);
    const float alpha = __builtin_amdgcn_exp2f(st.m[h] - m_new);
    float psum = 0.f;
#pragma unroll
    for (int u = 0; u < R; ++u) {
      const float p = __builtin_amdgcn_exp2f(s[u][h] - m_new);
      psum += p;
      const float w = p * x.vs[u >> 2][u & 3];
      pv[u][h] = (TAIL && (u * 8 + r >= nvalid)) ? 0.f : w;
    }
    st.l[h] = st.l[h] * alpha + psum;
    st.m[h] = m_new;
#pragma unroll
    for (int i = 0; i < 16; ++i) st.o[h][i] *= alpha;
  }
#pragma unroll
  for (int u = 0; u < R; ++u) {
    f16x2 vv[8];
    row_codes_f16(x.v[u], vv);
#pragma unroll
    for (int h = 0; h < G; ++h) {
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        st.o[h][2 * i] = fmaf(pv[u][h], (float)vv[i][0], st.o[h][2 * i]);
        st.o[h][2 * i + 1] = fmaf(pv[u][h], (float)vv[i][1], st.o[h][2 * i + 1]);
      }
    }
  }
}

// Workgroup = 4 wavefronts on one (sequence, KV head, split); each wavefront walks a contiguous run of blocks,
// the next block's loads in flight while the current one is reduced. Every group of 8 lanes keeps its own online
// softmax state for the G query heads; states meet once at the end, as in the bf16 kernel. q, o are bf16.
template <int G>
__global__ void __launch_bounds__(256) decode_i8_kernel(yoco_kv_cache c, const bf16_t* __restrict__ q,
                                                        const int64_t* __restrict__ lens, int64_t fixed_len, int Hq, float scale_log2,
                                                        float* __restrict__ ws, int splits, bf16_t* __restrict__ o_direct) {
  __shared__ float red_o[4][G][kD];
  __shared__ float red_ml[4][G][2];
  const int sp = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int r = lane >> 3, seg = lane & 7;

  const int64_t len_raw = lens ? lens[b] : fixed_len;
  const int64_t len = len_raw < 0 ? 0 : (len_raw > c.N_cap ? c.N_cap : len_raw);
  const int64_t chunk = (((len + splits - 1) / splits) + 255) & ~(int64_t)255;   // rows per split, 256 | chunk
  const int64_t j_lo = sp * chunk;
  const int64_t j_hi = (j_lo + chunk < len) ? j_lo + chunk : len;
  const int64_t sub = chunk >> 2;                                                // rows per wave, 64 | sub
  const int64_t w_lo = j_lo + wave * sub;
  const int64_t w_hi = (w_lo + sub < j_hi) ? w_lo + sub : j_hi;

  f16x2 qh[G][8];
#pragma unroll
  for (int h = 0; h < G; ++h) {
    const bf16_t* qp = q + ((int64_t)b * Hq + g * G + h) * kD + seg * 16;
    const u32x4 lo = *(const u32x4*)qp, hi = *(const u32x4*)(qp + 8);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const unsigned w = i < 4 ? lo[i] : hi[i - 4];
      qh[h][i] = (f16x2){(_Float16)__uint_as_float(w << 16), (_Float16)__uint_as_float(w & 0xffff0000u)};
    }
  }

  State<G> st;
#pragma unroll
  for (int h = 0; h < G; ++h) {
    st.m[h] = kNegBig;
    st.l[h] = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) st.o[h][i] = 0.f;
  }

  const int64_t plane = ((int64_t)b * c.Hkv + g) * (i8_plane_bytes(c.N_cap) / 16);   // in 16-byte units
  const u32x4* kp = (const u32x4*)c.k + plane;
  const u32x4* vp = (const u32x4*)c.v + plane;

  if (w_lo < w_hi) {
    Block nx;
    auto load = [&](int64_t row0) {                       // row0 is a multiple of 64
      const int64_t base = (row0 >> 6) * (kI8BlockBytes / 16);
#pragma unroll
      for (int u = 0; u < R; ++u) {
        nx.k[u] = __builtin_nontemporal_load(kp + base + u * 64 + lane);
        nx.v[u] = __builtin_nontemporal_load(vp + base + u * 64 + lane);
      }
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        nx.ks[i] = __builtin_nontemporal_load((const f32x4*)(kp + base + kI8ScaleOffset / 16 + r * 2 + i));
        nx.vs[i] = __builtin_nontemporal_load((const f32x4*)(vp + base + kI8ScaleOffset / 16 + r * 2 + i));
      }
    };
    load(w_lo);
    int64_t row0 = w_lo;
    for (; row0 + 64 < w_hi; row0 += 64) {
      const Block cur = nx;
      load(row0 + 64);
      step<G, false>(st, qh, cur, scale_log2, r, 64);
    }
    step<G, true>(st, qh, nx, scale_log2, r, (int)(w_hi - row0));   // last block of the run, 1..64 rows
  }

  // merge the 8 lane groups of the wave
#pragma unroll
  for (int h = 0; h < G; ++h) {
    float M = st.m[h];
    M = fmaxf(M, __shfl_xor(M, 8));
    M = fmaxf(M, __shfl_xor(M, 16));
    M = fmaxf(M, __shfl_xor(M, 32));
    const float f = __builtin_amdgcn_exp2f(st.m[h] - M);
    float l = st.l[h] * f;
    l += __shfl_xor(l, 8);
    l += __shfl_xor(l, 16);
    l += __shfl_xor(l, 32);
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      float x = st.o[h][i] * f;
      x += __shfl_xor(x, 8);
      x += __shfl_xor(x, 16);
      x += __shfl_xor(x, 32);
      st.o[h][i] = x;
    }
    if (lane < 8) {
#pragma unroll
      for (int i = 0; i < 16; ++i) red_o[wave][h][seg * 16 + i] = st.o[h][i];
      if (lane == 0) { red_ml[wave][h][0] = M; red_ml[wave][h][1] = l; }
    }
  }
  __syncthreads();
  for (int t = threadIdx.x; t < G * kD; t += 256) {
    const int h = t / kD, e = t % kD;
    const float M = fmaxf(fmaxf(red_ml[0][h][0], red_ml[1][h][0]), fmaxf(red_ml[2][h][0], red_ml[3][h][0]));
    float l = 0.f, o = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const float f = __builtin_amdgcn_exp2f(red_ml[w][h][0] - M);
      l = fmaf(f, red_ml[w][h][1], l);
      o = fmaf(f, red_o[w][h][e], o);
    }
    if (o_direct) {
      o_direct[((size_t)b * Hq + g * G + h) * kD + e] = f32_to_bf16(l > 0.f ? o / l : 0.f);
      continue;
    }
    float* out = ws + (((size_t)b * Hq + g * G + h) * splits + sp) * partial_stride(kD);
    out[e] = o;
    if (e == 0) {
      out[kD] = (l > 0.f) ? M * kLn2 : -INFINITY;
      out[kD + 1] = l;
    }
  }
}

}  // namespace

bool cache_i8_supported(int d) { return d == kD; }

bool decode_i8_supported(const yoco_kv_cache& c, int Hq) {
  if (c.dtype != YOCO_INT8 || c.d != kD) return false;
  const int G = Hq / c.Hkv;
  return G >= 1 && G <= 4 && c.Hkv <= 65535;
}

hipError_t launch_kv_code_i8(const yoco_kv_cache& c, const void* k, const void* v, int b, int64_t pos0, int64_t n,
                             const int64_t* pos, int src_dtype, hipStream_t s) {
  const int64_t rows = pos ? c.B : n;
  const int64_t waves = rows * c.Hkv * 2;
  dim3 grid((unsigned)((waves + 3) / 4)), block(256);
  if (src_dtype == YOCO_F32)
    hipLaunchKernelGGL(kv_code_i8_kernel<float>, grid, block, 0, s, c, (const float*)k, (const float*)v, b, pos0, rows, pos);
  else
    hipLaunchKernelGGL(kv_code_i8_kernel<bf16_t>, grid, block, 0, s, c, (const bf16_t*)k, (const bf16_t*)v, b, pos0, rows, pos);
  return hipGetLastError();
}

hipError_t launch_decode_i8(const yoco_kv_cache& c, const void* q, const int64_t* lens, int64_t fixed_len, int Hq, float scale,
                            float* ws, int splits, void* o_direct, hipStream_t s) {
  bf16_t* od = splits == 1 ? (bf16_t*)o_direct : nullptr;
  dim3 grid(splits, c.Hkv, c.B), block(256);
  const float sl2 = scale * kLog2e;
  const bf16_t* qp = (const bf16_t*)q;
  switch (Hq / c.Hkv) {
    case 1: hipLaunchKernelGGL(decode_i8_kernel<1>, grid, block, 0, s, c, qp, lens, fixed_len, Hq, sl2, ws, splits, od); break;
    case 2: hipLaunchKernelGGL(decode_i8_kernel<2>, grid, block, 0, s, c, qp, lens, fixed_len, Hq, sl2, ws, splits, od); break;
    case 3: hipLaunchKernelGGL(decode_i8_kernel<3>, grid, block, 0, s, c, qp, lens, fixed_len, Hq, sl2, ws, splits, od); break;
    case 4: hipLaunchKernelGGL(decode_i8_kernel<4>, grid, block, 0, s, c, qp, lens, fixed_len, Hq, sl2, ws, splits, od); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace yoco
