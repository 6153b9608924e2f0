// Split-KV decode of the cross-decoder's attention (Eq. 3 with one query row
// per sequence), bf16 cache, head_dim 128. HBM-bound: every byte of the shared
// K^/V^ planes is read exactly once per call and all G query heads of a KV head
// are served from that one read.
//
// Workgroup = 4 wavefronts on one (sequence, KV head, split). Each wavefront
// streams a contiguous quarter of the split, 32 rows (16 KiB of K and V) per step,
// with the next step's loads in flight while the current one is reduced. States are
// merged once at the end (lanes by shuffles, wavefronts through LDS) and written as
// one partial (m, l, o[128]) per (sequence, query head, split).
//
// Two kernels share that frame. decode_bf16_mfma_kernel (further down) puts both
// products on the matrix cores and serves 1..16 heads per KV head at the rate of a
// plain streaming read. decode_bf16_kernel works on the vector ALU: 128-bit loads
// that cover whole 256-byte rows (16 lanes per row), each group of 16 lanes keeping
// its own online-softmax state (m, l, o[8 dims]) per query head; it serves the
// one-token sliding-window step, which also stores the new row.
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

// The call also stores the new token's K/V row (k_new, v_new: [B,Hkv,128]) at slot lens[b] - 1 (modulo
// the capacity for a rolling cache) and attends to it. The row is taken from registers wherever the stream
// meets its slot, so nothing is read back that this launch writes.
template <int G, int R>
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

  int64_t slot = -1;                                   // where the new row goes, -1 = nowhere
  u32x4 knew = {0, 0, 0, 0}, vnew = knew;
  {
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
        if (row == slot) {                             // the new row comes from the registers, not from memory
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


// ---- 1..16 query heads per KV head: both products on the matrix cores, so the stream stays HBM-bound whatever
// the group size (the heads are the 16 columns of the MFMA; unused columns carry zeros).
// Wavefront step = 32 rows. Scores: S[key, head] = K[key, :] . Q[head, :] as two 16-key tiles of four
// 16x16x32 products, K fragments loaded from the row-major plane as they are (lane = (key, 8-dim group)).
// Output: O^T[dim, head] += V^T[dim, key] P^T[key, head]; the V fragment (8 keys of one dim per lane) comes
// from the wavefront's own LDS staging rows through the transposing 64-bit read, which hands lane n of a
// 16-lane block the column n of the 4 x 16 tile whose row pieces the block's lanes address. Lane (head, qg)
// then owns dims 16 tt + 4 qg + i of its head in o[tt][i], next to that head's scores, so the online-softmax
// rescale is one factor per lane. P is fed as bf16 high part + bf16 remainder (two products), which keeps
// the weights at fp32-like precision; the row sum l is taken in fp32.
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

constexpr int kMRows = 32;        // rows per wavefront step
constexpr int kVStride = 288;     // bytes per staged V row: 256 + 32, the 4 rows of a transposing read fall in distinct banks
constexpr int kGMax = 16;

struct MState {
  float m, l;
  f32x4 o[8];
};

__device__ __forceinline__ bf16x8_t v_fragment(const unsigned char* lds_row_a, const unsigned char* lds_row_b) {
  const s16x4 a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)lds_row_a);
  const s16x4 b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)lds_row_b);
  const s16x8 ab = {a[0], a[1], a[2], a[3], b[0], b[1], b[2], b[3]};
  return __builtin_bit_cast(bf16x8_t, ab);
}

template <bool TAIL>
__device__ __forceinline__ void mfma_scores(float (&s)[8], const bf16x8_t (&qf)[4], const u32x4 (&kr)[8], float scale_log2,
                                            int qg, int nvalid) {
#pragma unroll
  for (int tau = 0; tau < 2; ++tau) {
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int t = 0; t < 4; ++t)
      acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, kr[tau * 4 + t]), qf[t], acc, 0, 0, 0);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      float a = acc[i] * scale_log2;
      if (TAIL && (tau * 16 + qg * 4 + i >= nvalid)) a = -INFINITY;
      s[tau * 4 + i] = a;
    }
  }
}

__device__ __forceinline__ void mfma_softmax_pv(MState& st, const float (&s)[8], const unsigned char* vst, int lane) {
  float smax = s[0];
#pragma unroll
  for (int i = 1; i < 8; ++i) smax = fmaxf(smax, s[i]);
  smax = fmaxf(smax, __shfl_xor(smax, 16));     // the four lanes of a head hold 8 rows each
  smax = fmaxf(smax, __shfl_xor(smax, 32));
  const float m_new = fmaxf(st.m, smax);
  float p[8], psum = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    p[i] = __builtin_amdgcn_exp2f(s[i] - m_new);
    psum += p[i];
  }
  const float alpha = __builtin_amdgcn_exp2f(st.m - m_new);
  st.l = st.l * alpha + psum;
  if (__builtin_amdgcn_ballot_w64(m_new != st.m)) {     // rare once the stream has met its large scores
#pragma unroll
    for (int tt = 0; tt < 8; ++tt) st.o[tt] *= alpha;
  }
  st.m = m_new;
  // weights as two bf16 operands: the upper 16 bits, and the upper 16 bits of what those leave
  u32x4 ph, pl;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const unsigned a = __float_as_uint(p[2 * i]), b = __float_as_uint(p[2 * i + 1]);
    const float ra = p[2 * i] - __uint_as_float(a & 0xffff0000u), rb = p[2 * i + 1] - __uint_as_float(b & 0xffff0000u);
    ph[i] = (a >> 16) | (b & 0xffff0000u);
    pl[i] = (__float_as_uint(ra) >> 16) | (__float_as_uint(rb) & 0xffff0000u);
  }
  const bf16x8_t bh = __builtin_bit_cast(bf16x8_t, ph), bl = __builtin_bit_cast(bf16x8_t, pl);
  // the block of 16 lanes with index kg reads rows 4 kg .. 4 kg + 3 of either 16-row tile: lane s of the block
  // addresses row 4 kg + s / 4, dims 16 tt + 4 (s % 4) .. + 3
  const int sl = lane & 15, kg = lane >> 4;
  const unsigned char* ra = vst + (4 * kg + (sl >> 2)) * kVStride + (sl & 3) * 8;
  const unsigned char* rb = ra + 16 * kVStride;
#pragma unroll
  for (int tt = 0; tt < 8; ++tt) {
    const bf16x8_t vf = v_fragment(ra + tt * 32, rb + tt * 32);
    st.o[tt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, bh, st.o[tt], 0, 0, 0);
    st.o[tt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, bl, st.o[tt], 0, 0, 0);
  }
}

template <bool APPEND>
__global__ void __launch_bounds__(256) decode_bf16_mfma_kernel(yoco_kv_cache c, const bf16_t* __restrict__ q,
                                                               const int64_t* __restrict__ lens, int64_t fixed_len, int Hq,
                                                               float scale_log2, float* __restrict__ ws, int splits,
                                                               bf16_t* __restrict__ o_direct, const bf16_t* __restrict__ k_new,
                                                               const bf16_t* __restrict__ v_new, int ring) {
  // V staging of the four wavefronts (4 x 32 rows x 288 B) during the stream, the merge buffers after it
  constexpr int kStageBytes = kMRows * kVStride;
  constexpr int kRedBytes = 4 * kGMax * kD * 4;
  __shared__ __attribute__((aligned(16))) unsigned char smem[(4 * kStageBytes > kRedBytes) ? 4 * kStageBytes : kRedBytes];
  __shared__ float red_ml[4][kGMax][2];
  float (*red_o)[kGMax][kD] = (float (*)[kGMax][kD])smem;
  const int G = Hq / c.Hkv;
  const int sp = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int n = lane & 15, qg = lane >> 4;
  unsigned char* vst = smem + wave * kStageBytes;

  const int64_t len_raw = lens ? lens[b] : fixed_len;
  const int64_t len = len_raw < 0 ? 0 : (len_raw > c.N_cap ? c.N_cap : len_raw);
  const int64_t chunk = (((len + splits - 1) / splits) + 127) & ~(int64_t)127;  // rows per split, 128 | chunk
  const int64_t j_lo = sp * chunk;
  const int64_t j_hi = (j_lo + chunk < len) ? j_lo + chunk : len;
  const int64_t sub = chunk >> 2;                                               // rows per wave, 32 | sub
  const int64_t w_lo = j_lo + wave * sub;
  const int64_t w_hi = (w_lo + sub < j_hi) ? w_lo + sub : j_hi;

  // lane (head n, dim group qg) holds dims 32 t + 8 qg .. + 7 of its head's query for t = 0..3
  bf16x8_t qf[4];
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    u32x4 x = {0, 0, 0, 0};
    if (n < G) x = *(const u32x4*)(q + ((int64_t)b * Hq + g * G + n) * kD + t * 32 + qg * 8);
    qf[t] = __builtin_bit_cast(bf16x8_t, x);
  }

  MState st;
  st.m = kNegBig;
  st.l = 0.f;
#pragma unroll
  for (int tt = 0; tt < 8; ++tt) st.o[tt] = (f32x4){0.f, 0.f, 0.f, 0.f};

  const int64_t plane = ((int64_t)b * c.Hkv + g) * c.N_cap * (kD / 8);          // in 16-byte units
  const u32x4* kp = (const u32x4*)c.k + plane + qg;                             // K: lane = (row n of a tile, dims 8 qg ..)
  const u32x4* vp = (const u32x4*)c.v + plane + n;                              // V: lane = (row qg of four, 16-byte piece n)

  // APPEND: the new token's row goes to slot lens[b] - 1 (modulo the capacity for a rolling cache) and is attended
  // to from registers wherever the stream meets its slot, so nothing is read back that this launch writes.
  int64_t slot = -1;
  u32x4 knew[4] = {}, vnew = {0, 0, 0, 0};
  if (APPEND) {
    const int64_t pos = len_raw - 1;
    if (pos >= 0 && (ring || pos < c.N_cap)) slot = pos >= c.N_cap ? pos % c.N_cap : pos;
    const bf16_t* kn = k_new + ((int64_t)b * c.Hkv + g) * kD;
#pragma unroll
    for (int t = 0; t < 4; ++t) knew[t] = *(const u32x4*)(kn + t * 32 + qg * 8);
    vnew = *(const u32x4*)(v_new + ((int64_t)b * c.Hkv + g) * kD + n * 8);
    if (slot >= j_lo && slot < j_hi && wave == 0 && lane < 32) {      // the split that owns the slot stores the row
      const u32x4 x = *(const u32x4*)((lane < 16 ? kn : v_new + ((int64_t)b * c.Hkv + g) * kD) + n * 8);
      *((u32x4*)(lane < 16 ? c.k : c.v) + plane + slot * (kD / 8) + n) = x;
    }
  }

  if (w_lo < w_hi) {
    const int64_t last = w_hi - 1;
    u32x4 kr[8], vr[8];
    auto load_k = [&](int64_t row0) {
#pragma unroll
      for (int tau = 0; tau < 2; ++tau) {
        int64_t row = row0 + tau * 16 + n;
        row = row < last ? row : last;                 // clamped rows are masked in the tail step
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          kr[tau * 4 + t] = __builtin_nontemporal_load(kp + row * (kD / 8) + t * 4);
          if (APPEND && row == slot) kr[tau * 4 + t] = knew[t];
        }
      }
    };
    auto load_v = [&](int64_t row0) {
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        int64_t row = row0 + u * 4 + qg;
        row = row < last ? row : last;                 // a written row: finite values under weight 0
        vr[u] = __builtin_nontemporal_load(vp + row * (kD / 8));
        if (APPEND && row == slot) vr[u] = vnew;
      }
    };
    auto stage_v = [&]() {
#pragma unroll
      for (int u = 0; u < 8; ++u) *(u32x4*)(vst + (u * 4 + qg) * kVStride + n * 16) = vr[u];
    };
    load_k(w_lo);
    load_v(w_lo);
    int64_t row0 = w_lo;
    float s[8];
    for (; row0 + kMRows < w_hi; row0 += kMRows) {      // steps followed by another step
      stage_v();
      load_v(row0 + kMRows);
      mfma_scores<false>(s, qf, kr, scale_log2, qg, kMRows);
      load_k(row0 + kMRows);
      mfma_softmax_pv(st, s, vst, lane);
    }
    stage_v();
    mfma_scores<true>(s, qf, kr, scale_log2, qg, (int)(w_hi - row0));   // last step, 1..32 rows
    mfma_softmax_pv(st, s, vst, lane);
  }

  // One state per head and wavefront: the four lanes of a head sum their row sums; then the merge over wavefronts.
  float l = st.l;
  l += __shfl_xor(l, 16);
  l += __shfl_xor(l, 32);
  __syncthreads();                                       // every wavefront is done with its staging rows
  if (n < G) {
#pragma unroll
    for (int tt = 0; tt < 8; ++tt)
#pragma unroll
      for (int i = 0; i < 4; ++i) red_o[wave][n][tt * 16 + qg * 4 + i] = st.o[tt][i];
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
      out[kD] = (ls > 0.f) ? M * kLn2 : -INFINITY;      // the merge pass works with natural exponents
      out[kD + 1] = ls;
    }
  }
}

}  // namespace

bool decode_bf16_supported(const yoco_kv_cache& c, int Hq) {
  if (c.dtype != YOCO_BF16 || c.d != kD) return false;
  const int G = Hq / c.Hkv;
  return G >= 1 && G <= 16 && c.Hkv <= 65535;
}

// Every call without an append, and append calls with 5..16 heads per KV head, take the matrix-core kernel (HBM-bound
// at every group size). The one-token sliding-window step (append, window of about a thousand rows, up to 4 heads
// per KV head) keeps the vector-ALU kernel, whose shorter prologue and merge win on streams of a few steps per wavefront.
hipError_t launch_decode_bf16(const yoco_kv_cache& c, const void* q, const int64_t* lens, int64_t fixed_len, int Hq, float scale,
                              float* ws, int splits, void* o_direct, const void* k_new, const void* v_new, int ring,
                              hipStream_t s) {
  bf16_t* od = splits == 1 ? (bf16_t*)o_direct : nullptr;
  dim3 grid(splits, c.Hkv, c.B), block(256);
  const float sl2 = scale * kLog2e;
  const bf16_t* qp = (const bf16_t*)q;
  const bf16_t* kn = (const bf16_t*)k_new;
  const bf16_t* vn = (const bf16_t*)v_new;
  const int G = Hq / c.Hkv;
  if (G < 1 || G > kGMax) return hipErrorInvalidValue;
  if (!kn) {
    hipLaunchKernelGGL(decode_bf16_mfma_kernel<false>, grid, block, 0, s, c, qp, lens, fixed_len, Hq, sl2, ws, splits, od, kn, vn, ring);
    return hipGetLastError();
  }
  switch (G) {
    case 1: hipLaunchKernelGGL((decode_bf16_kernel<1, 8>), grid, block, 0, s, c, qp, lens, fixed_len, Hq, sl2, ws, splits, od, kn, vn, ring); break;
    case 2: hipLaunchKernelGGL((decode_bf16_kernel<2, 8>), grid, block, 0, s, c, qp, lens, fixed_len, Hq, sl2, ws, splits, od, kn, vn, ring); break;
    case 3: hipLaunchKernelGGL((decode_bf16_kernel<3, 8>), grid, block, 0, s, c, qp, lens, fixed_len, Hq, sl2, ws, splits, od, kn, vn, ring); break;
    case 4: hipLaunchKernelGGL((decode_bf16_kernel<4, 8>), grid, block, 0, s, c, qp, lens, fixed_len, Hq, sl2, ws, splits, od, kn, vn, ring); break;
    default:
      hipLaunchKernelGGL(decode_bf16_mfma_kernel<true>, grid, block, 0, s, c, qp, lens, fixed_len, Hq, sl2, ws, splits, od, kn, vn, ring);
  }
  return hipGetLastError();
}

}  // namespace yoco
