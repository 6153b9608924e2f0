// Split-KV decode of the cross-decoder's attention (Eq. 3 with one query row
// per sequence), bf16 cache, head_dim 128. HBM-bound: every byte of the shared
// K^/V^ planes is read exactly once per call, with 128-bit loads that cover
// whole 256-byte rows (16 lanes per row, 4 rows = 1 KiB contiguous per wave
// load), and all G query heads of a KV head are served from that one read.
//
// Workgroup = 4 wavefronts on one (sequence, KV head, split). Each wavefront
// streams a contiguous quarter of the split, 32 rows (16 KiB of K and V) per step,
// with the next step's loads in flight while the current one is reduced; each group of
// 16 lanes keeps its own online-softmax state (m, l, o[8 dims]) per query head,
// so the streaming loop has no cross-group traffic. States are merged once at
// the end (lane groups by shuffles, wavefronts through LDS) and written as one
// partial (m, l, o[128]) per (sequence, query head, split).
#include "yoco_common.h"

namespace yoco {

namespace {

constexpr int kD = 128;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kNegBig = -1.0e30f;   // "no row seen yet": finite, so m - m never makes NaN

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float dot2_bf16(unsigned a, unsigned b, float c) {
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a), __builtin_bit_cast(bf16x2_t, b), c, false);
}
__device__ __forceinline__ float bf_lo(unsigned x) { return __uint_as_float(x << 16); }
__device__ __forceinline__ float bf_hi(unsigned x) { return __uint_as_float(x & 0xffff0000u); }

// Sum over the 16 lanes of a DPP row; every lane ends with the total.
template <int CTRL>
__device__ __forceinline__ float dpp_add(float x) {
  int y = __builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xf, 0xf, true);
  return x + __int_as_float(y);
}
__device__ __forceinline__ float row16_sum(float x) {
  x = dpp_add<0xB1>(x);    // quad_perm [1,0,3,2]
  x = dpp_add<0x4E>(x);    // quad_perm [2,3,0,1]
  x = dpp_add<0x141>(x);   // row_half_mirror: quads 0<->1, 2<->3
  x = dpp_add<0x140>(x);   // row_mirror: halves 0<->1
  return x;
}

template <int G>
struct State {
  float m[G], l[G], o[G][8];
};

// One step: R rows per lane group (rows u*4 + r of the 4R-row step).
// nvalid = rows of this step that exist (4R in the steady state).
template <int G, int R, bool TAIL>
__device__ __forceinline__ void step(State<G>& st, const u32x4 (&kq)[G], const u32x4 (&kr)[R], const u32x4 (&vr)[R],
                                     float scale_log2, int r, int nvalid) {
  float s[R][G];
#pragma unroll
  for (int u = 0; u < R; ++u) {
#pragma unroll
    for (int h = 0; h < G; ++h) {
      float a = dot2_bf16(kq[h][0], kr[u][0], 0.f);
      a = dot2_bf16(kq[h][1], kr[u][1], a);
      a = dot2_bf16(kq[h][2], kr[u][2], a);
      a = dot2_bf16(kq[h][3], kr[u][3], a);
      a = row16_sum(a) * scale_log2;
      if (TAIL && (u * 4 + r >= nvalid)) a = -INFINITY;
      s[u][h] = a;
    }
  }
#pragma unroll
  for (int h = 0; h < G; ++h) {
    float mx = s[0][h];
#pragma unroll
    for (int u = 1; u < R; ++u) mx = fmaxf(mx, s[u][h]);
    const float m_new = fmaxf(st.m[h], mx);
    const float alpha = __builtin_amdgcn_exp2f(st.m[h] - m_new);
    float p[R], psum = 0.f;
#pragma unroll
    for (int u = 0; u < R; ++u) {
      p[u] = __builtin_amdgcn_exp2f(s[u][h] - m_new);
      psum += p[u];
    }
    st.l[h] = st.l[h] * alpha + psum;
    st.m[h] = m_new;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      float a0 = st.o[h][2 * i] * alpha, a1 = st.o[h][2 * i + 1] * alpha;
#pragma unroll
      for (int u = 0; u < R; ++u) {
        a0 = fmaf(p[u], bf_lo(vr[u][i]), a0);
        a1 = fmaf(p[u], bf_hi(vr[u][i]), a1);
      }
      st.o[h][2 * i] = a0;
      st.o[h][2 * i + 1] = a1;
    }
  }
}

// APPEND: the call also stores the new token's K/V row (k_new, v_new: [B,Hkv,128]) at slot lens[b] - 1 (modulo
// the capacity for a rolling cache) and attends to it. The row is taken from registers wherever the stream
// meets its slot, so nothing is read back that this launch writes.
template <int G, int R, bool APPEND>
__global__ void __launch_bounds__(256) decode_bf16_kernel(yoco_kv_cache c, const bf16_t* __restrict__ q,
                                                          const int64_t* __restrict__ lens, int64_t fixed_len, int Hq, float scale_log2,
                                                          float* __restrict__ ws, int splits, bf16_t* __restrict__ o_direct,
                                                          const bf16_t* __restrict__ k_new, const bf16_t* __restrict__ v_new,
                                                          int ring) {
  constexpr int kRowsPerStep = 4 * R;
  __shared__ float red_o[4][G][kD];
  __shared__ float red_ml[4][G][2];
  const int sp = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int r = lane >> 4, seg = lane & 15;

  const int64_t len_raw = lens ? lens[b] : fixed_len;   // a host-known length serves the few-row prefill case
  const int64_t len = len_raw < 0 ? 0 : (len_raw > c.N_cap ? c.N_cap : len_raw);
  const int64_t chunk = (((len + splits - 1) / splits) + 127) & ~(int64_t)127;  // rows per split, 128 | chunk
  const int64_t j_lo = sp * chunk;
  const int64_t j_hi = (j_lo + chunk < len) ? j_lo + chunk : len;
  const int64_t sub = chunk >> 2;                                               // rows per wave, 32 | sub
  const int64_t w_lo = j_lo + wave * sub;
  const int64_t w_hi = (w_lo + sub < j_hi) ? w_lo + sub : j_hi;

  u32x4 kq[G];
#pragma unroll
  for (int h = 0; h < G; ++h)
    kq[h] = *(const u32x4*)(q + ((int64_t)b * Hq + g * G + h) * kD + seg * 8);

  State<G> st;
#pragma unroll
  for (int h = 0; h < G; ++h) {
    st.m[h] = kNegBig;
    st.l[h] = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) st.o[h][i] = 0.f;
  }

  const int64_t plane = ((int64_t)b * c.Hkv + g) * c.N_cap * (kD / 8);          // in 16-byte units
  const u32x4* kp = (const u32x4*)c.k + plane + seg;
  const u32x4* vp = (const u32x4*)c.v + plane + seg;

  int64_t slot = -1;                                   // where the new row goes (APPEND), -1 = nowhere
  u32x4 knew = {0, 0, 0, 0}, vnew = knew;
  if (APPEND) {
    const int64_t pos = len_raw - 1;
    if (pos >= 0 && (ring || pos < c.N_cap)) slot = pos >= c.N_cap ? pos % c.N_cap : pos;
    knew = *(const u32x4*)(k_new + ((int64_t)b * c.Hkv + g) * kD + seg * 8);
    vnew = *(const u32x4*)(v_new + ((int64_t)b * c.Hkv + g) * kD + seg * 8);
    if (slot >= j_lo && slot < j_hi && wave == 0 && lane < 32) {      // the split that owns the slot stores the row
      u32x4* dst = (u32x4*)(lane < 16 ? c.k : c.v) + plane + slot * (kD / 8) + seg;
      *dst = lane < 16 ? knew : vnew;
    }
  }

  if (w_lo < w_hi) {
    const int64_t last = w_hi - 1;
    u32x4 kn[R], vn[R];
    auto load = [&](int64_t row0) {
#pragma unroll
      for (int u = 0; u < R; ++u) {
        int64_t row = row0 + u * 4 + r;
        row = row < last ? row : last;                 // clamped rows are masked in the tail step
        kn[u] = __builtin_nontemporal_load(kp + row * (kD / 8));
        vn[u] = __builtin_nontemporal_load(vp + row * (kD / 8));
        if (APPEND && row == slot) {                   // the new row comes from the registers, not from memory
          kn[u] = knew;
          vn[u] = vnew;
        }
      }
    };
    load(w_lo);
    int64_t row0 = w_lo;
    for (; row0 + kRowsPerStep < w_hi; row0 += kRowsPerStep) {   // steps followed by another step
      u32x4 kc[R], vc[R];
#pragma unroll
      for (int u = 0; u < R; ++u) { kc[u] = kn[u]; vc[u] = vn[u]; }
      load(row0 + kRowsPerStep);
      step<G, R, false>(st, kq, kc, vc, scale_log2, r, kRowsPerStep);
    }
    step<G, R, true>(st, kq, kn, vn, scale_log2, r, (int)(w_hi - row0));   // last step, 1..4R rows
  }

  // merge the 4 lane groups of the wave
#pragma unroll
  for (int h = 0; h < G; ++h) {
    float M = st.m[h];
    M = fmaxf(M, __shfl_xor(M, 16));
    M = fmaxf(M, __shfl_xor(M, 32));
    const float f = __builtin_amdgcn_exp2f(st.m[h] - M);
    float l = st.l[h] * f;
    l += __shfl_xor(l, 16);
    l += __shfl_xor(l, 32);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      float x = st.o[h][i] * f;
      x += __shfl_xor(x, 16);
      x += __shfl_xor(x, 32);
      st.o[h][i] = x;
    }
    if (lane < 16) {
#pragma unroll
      for (int i = 0; i < 8; ++i) red_o[wave][h][seg * 8 + i] = st.o[h][i];
      if (lane == 0) { red_ml[wave][h][0] = M; red_ml[wave][h][1] = l; }
    }
  }
  __syncthreads();
  // merge the 4 waves; thread t owns (head t / 128, dimension t % 128)
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
    if (o_direct) {          // a single split is the whole answer: normalise and store, no merge pass
      o_direct[((size_t)b * Hq + g * G + h) * kD + e] = f32_to_bf16(l > 0.f ? o / l : 0.f);
      continue;
    }
    float* out = ws + (((size_t)b * Hq + g * G + h) * splits + sp) * partial_stride(kD);
    out[e] = o;
    if (e == 0) {
      out[kD] = (l > 0.f) ? M * kLn2 : -INFINITY;    // the merge pass works with natural exponents
      out[kD + 1] = l;
    }
  }
}

}  // namespace

bool decode_bf16_supported(const yoco_kv_cache& c, int Hq) {
  if (c.dtype != YOCO_BF16 || c.d != kD) return false;
  const int G = Hq / c.Hkv;
  return G >= 1 && G <= 4 && c.Hkv <= 65535;
}

hipError_t launch_decode_bf16(const yoco_kv_cache& c, const void* q, const int64_t* lens, int64_t fixed_len, int Hq, float scale,
                              float* ws, int splits, void* o_direct, const void* k_new, const void* v_new, int ring,
                              hipStream_t s) {
  bf16_t* od = splits == 1 ? (bf16_t*)o_direct : nullptr;
  dim3 grid(splits, c.Hkv, c.B), block(256);
  const float sl2 = scale * kLog2e;
  const bf16_t* qp = (const bf16_t*)q;
  constexpr int R = 8;
  const bf16_t* kn = (const bf16_t*)k_new;
  const bf16_t* vn = (const bf16_t*)v_new;
#define YOCO_DECODE_LAUNCH(G)                                                                                                   \
  if (kn)                                                                                                                       \
    hipLaunchKernelGGL((decode_bf16_kernel<G, R, true>), grid, block, 0, s, c, qp, lens, fixed_len, Hq, sl2, ws, splits, od, kn, vn, ring); \
  else                                                                                                                          \
    hipLaunchKernelGGL((decode_bf16_kernel<G, R, false>), grid, block, 0, s, c, qp, lens, fixed_len, Hq, sl2, ws, splits, od, kn, vn, ring);
  switch (Hq / c.Hkv) {
    case 1: YOCO_DECODE_LAUNCH(1) break;
    case 2: YOCO_DECODE_LAUNCH(2) break;
    case 3: YOCO_DECODE_LAUNCH(3) break;
    case 4: YOCO_DECODE_LAUNCH(4) break;
    default: return hipErrorInvalidValue;
  }
#undef YOCO_DECODE_LAUNCH
  return hipGetLastError();
}

}  // namespace yoco
