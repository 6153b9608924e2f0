// Flash-style attention prefill on bf16 MFMA for gfx950, head_dim 128.
// Serves yoco_swa_prefill (Eq. 8: causal window of C keys) and
// yoco_cross_attn_prefill (Eq. 3: causal over the global cache, GQA) through
// one kernel: a query at absolute position p sees keys j with p - C < j <= p.
//
// Workgroup = 4 wavefronts, 128 query rows of one head; wavefront w owns rows
// 32w .. 32w+31. Keys are walked in tiles of 64, only tiles that intersect
// some row's window are visited, and a wavefront skips the 32-key half tiles
// that none of its own rows can see.
//
// Orientation: S^T = K Q^T and O^T = V^T P^T with v_mfma_f32_32x32x16_bf16, so
// a query is a lane column (lane % 32) and keys / head dims run along the
// accumulator registers: the softmax max and sum are in-lane plus one swap
// with lane ^ 32, and the P^T accumulator registers are, as they stand, the B
// operand of the second product (the V^T operand is read from LDS with the
// transposing ds_read_b64_tr_b16 in the matching key order).
//
// Precision: S^T uses bf16 products (exact in fp32). P is rounded to fp16, not
// bf16, and V is converted bf16 -> fp16 (exact for |v| in [2^-14, 65504]) when
// it is staged, so the second product runs on the fp16 MFMA at the same rate:
// with bf16 P the rounding of P alone costs as much error as the rounding of
// the bf16 output, and the two together exceed a 2e-3 mean relative error.
// |v| >= 65520 is outside this kernel's domain (it overflows fp16).
//
// K and V tiles are staged global -> registers -> LDS (double buffered, the
// next tile's loads are in flight while the current one is computed). LDS
// rows are 256 B; K is XOR-swizzled in 16-byte chunks and V in 32-byte chunks
// so both operand read patterns are bank-conflict free.
#include "yoco_common.h"

namespace yoco {

namespace {

constexpr int kD = 128;          // head dimension
constexpr int kBN = 64;          // keys per tile
constexpr int kNQ = 32;          // query rows per wavefront
constexpr int kWaves = 4;
constexpr int kBM = kNQ * kWaves;
constexpr int kTileBytes = kBN * kD * 2;     // 16 KiB
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kNegBig = -1.0e30f;
constexpr float kLazyLog2 = 8.0f;            // rescale only when the max grows by more than 2^8

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef __attribute__((address_space(3))) char lds_char;

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));

// Two fp32 -> packed fp16, round to nearest even.
__device__ __forceinline__ unsigned pack_f16(float a, float b) {
  f32x2 v = {a, b};
  return __builtin_bit_cast(unsigned, __builtin_convertvector(v, f16x2));
}
// Two packed bf16 -> two packed fp16. Exact for magnitudes in [2^-14, 65504]
// (bf16 carries 8 significant bits, fp16 11); smaller ones lose low bits or
// flush (absolute error below 2^-25), larger ones overflow.
__device__ __forceinline__ unsigned bf16x2_to_f16x2(unsigned x) {
  return pack_f16(__uint_as_float(x << 16), __uint_as_float(x & 0xffff0000u));
}

__device__ __forceinline__ unsigned pack_bf16(float a, float b) {
  f32x2 v = {a, b};
  return __builtin_bit_cast(unsigned, __builtin_convertvector(v, bf16x2));
}

__device__ __forceinline__ float other_half(float x) {        // value held by lane ^ 32
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float((threadIdx.x & 32) ? r[0] : r[1]);
}

struct Args {
  AttnView a;
  int n_qtiles;       // query tiles per (sequence, head)
  int total;          // workgroups
  int64_t n_keys;     // keys that exist (rows beyond are never read)
};

__global__ void __launch_bounds__(256, 2) swa_mfma_kernel(Args g) {
  __shared__ __attribute__((aligned(1024))) char smem[2][2][kTileBytes];   // [buffer][K, V]
  const AttnView& a = g.a;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int hf = lane >> 5, lq = lane & 31;

  // ---- workgroup -> (sequence, head, query tile). Workgroups are dealt to
  // the 8 XCDs round robin; give each XCD a contiguous run of tiles so that
  // neighbouring query tiles (which share K/V tiles) meet in one L2. Within a
  // KV head the G query heads of a tile are adjacent; later (heavier under a
  // causal mask) query tiles go first.
  const int bid = blockIdx.x;
  const int per = g.total >> 3, rem = g.total & 7, xcd = bid & 7;
  const int logical = xcd * per + (xcd < rem ? xcd : rem) + (bid >> 3);
  const int G = a.Hq / a.Hkv;
  const int hh = logical % G;
  const int qt = g.n_qtiles - 1 - (logical / G) % g.n_qtiles;
  const int kvh = (logical / (G * g.n_qtiles)) % a.Hkv;
  const int b = logical / (G * g.n_qtiles * a.Hkv);
  const int h = kvh * G + hh;

  const int64_t i0 = (int64_t)qt * kBM;                 // first query row of the workgroup
  const int64_t p0 = a.q_pos0 + i0;                     // its absolute position
  const int64_t win = a.window;
  // key tiles that intersect the window of some row of the workgroup
  int64_t rows_here = a.Tq - i0 < kBM ? a.Tq - i0 : kBM;
  const int64_t lo_key = p0 - win + 1 > 0 ? p0 - win + 1 : 0;
  const int64_t hi_key = p0 + rows_here - 1;
  const int jt_lo = (int)(lo_key / kBN), jt_hi = (int)(hi_key / kBN);

  const bf16_t* kg = (const bf16_t*)a.k + b * a.kv_stride_b + kvh * a.kv_stride_h;
  const bf16_t* vg = (const bf16_t*)a.v + b * a.kv_stride_b + kvh * a.kv_stride_h;

  // ---- staging assignment: thread -> 16-byte chunk c16 of rows srow + 16 i
  const int c16 = tid & 15, srow = tid >> 4;
  u32x4 kst[4], vst[4];
  auto load_tile = [&](int jt) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      int64_t row = (int64_t)jt * kBN + srow + 16 * i;
      row = row < g.n_keys ? row : g.n_keys - 1;        // clamped rows are masked below
      kst[i] = *(const u32x4*)(kg + row * a.kv_stride_n + c16 * 8);
      vst[i] = *(const u32x4*)(vg + row * a.kv_stride_n + c16 * 8);
    }
  };
  auto store_tile = [&](int buf) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int row = srow + 16 * i;
      *(u32x4*)(&smem[buf][0][row * 256 + ((c16 ^ (row & 15)) << 4)]) = kst[i];
      u32x4 vh = {bf16x2_to_f16x2(vst[i][0]), bf16x2_to_f16x2(vst[i][1]), bf16x2_to_f16x2(vst[i][2]),
                  bf16x2_to_f16x2(vst[i][3])};
      *(u32x4*)(&smem[buf][1][row * 256 + (((((c16 >> 1) ^ (row & 7)) << 1) | (c16 & 1)) << 4)]) = vh;
    }
  };

  // ---- Q^T fragments (B operand): lane holds query lq, dims ks*16 + hf*8 .. +8
  const int64_t iw = i0 + wave * kNQ;                   // first row of the wavefront
  int64_t iq = iw + lq;
  const bool q_valid = iq < a.Tq;
  if (!q_valid) iq = a.Tq - 1;
  const bf16_t* qg = (const bf16_t*)a.q + b * a.q_stride_b + iq * a.q_stride_t + (int64_t)h * kD;
  bf16x8 qf[8];
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) qf[ks] = __builtin_bit_cast(bf16x8, *(const u32x4*)(qg + ks * 16 + hf * 8));

  // ---- per-lane LDS byte offsets of the operand fragments (within a tile)
  // K (A operand of S^T): row mb*32 + lq, chunk (ks*2 + hf) ^ (row & 15)
  int koff[8];
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) koff[ks] = lq * 256 + ((((ks << 1) | hf) ^ (lq & 15)) << 4);
  // V^T (A operand of O^T) via transposing reads: lane s = lane % 16 of a block
  // of 16 supplies row z = hf*4 + s/4 (+ t*16 + half*8), dims (mb*2 + db)*16 + 4*(s%4)
  const int s16 = lane & 15, db = (lane >> 4) & 1, z = hf * 4 + (s16 >> 2);
  int voff[4];
#pragma unroll
  for (int mb = 0; mb < 4; ++mb) voff[mb] = z * 256 + ((((mb << 1) | db) ^ z) << 5) + ((s16 & 3) << 3);

  const float c = a.scale * kLog2e;                     // scores are kept raw; exponents use s * c
  const float lazy_raw = kLazyLog2 / c;
  float m_used = kNegBig, l_lane = 0.f;
  f32x16 acc_o[4];
#pragma unroll
  for (int mb = 0; mb < 4; ++mb)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc_o[mb][r] = 0.f;

  const int pw_lo = (int)(p0 + wave * kNQ - (int64_t)jt_lo * kBN);      // wave's first position, relative to tile jt_lo
  const int pq_rel0 = pw_lo + lq;                                        // this lane's query, same origin
  const int win32 = win > (1 << 30) ? (1 << 30) : (int)win;

  load_tile(jt_lo);
  store_tile(0);
  __syncthreads();

  for (int jt = jt_lo; jt <= jt_hi; ++jt) {
    const int buf = (jt - jt_lo) & 1;
    if (jt < jt_hi) load_tile(jt + 1);
    const int j0r = (jt - jt_lo) * kBN;                 // tile's first key, relative origin
    // half tiles (32 keys) this wavefront needs: some row sees some key
    bool need[2];
#pragma unroll
    for (int mb = 0; mb < 2; ++mb) {
      const int k_lo = j0r + mb * 32, k_hi = k_lo + 31;
      need[mb] = (k_lo <= pw_lo + kNQ - 1) && (k_hi > pw_lo - win32);
    }
    if (need[0] || need[1]) {
      lds_char* kb = (lds_char*)&smem[buf][0][0];
      lds_char* vb = (lds_char*)&smem[buf][1][0];
      // ---- S^T = K Q^T
      f32x16 acc_s[2];
#pragma unroll
      for (int mb = 0; mb < 2; ++mb) {
#pragma unroll
        for (int r = 0; r < 16; ++r) acc_s[mb][r] = 0.f;
        if (need[mb]) {
#pragma unroll
          for (int ks = 0; ks < 8; ++ks) {
            const bf16x8 kf = __builtin_bit_cast(bf16x8, *(const __attribute__((address_space(3))) u32x4*)(kb + koff[ks] + mb * 32 * 256));
            acc_s[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], acc_s[mb], 0, 0, 0);
          }
        }
      }
      // ---- mask: full visibility iff every key <= every row and inside every window
      const bool full = (j0r + kBN - 1 <= pw_lo) && (j0r > pw_lo + kNQ - 1 - win32) && need[0] && need[1];
      if (!full) {
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int key = j0r + mb * 32 + (r >> 2) * 8 + hf * 4 + (r & 3);
            const bool ok = need[mb] && ((unsigned)(pq_rel0 - key) < (unsigned)win32);
            acc_s[mb][r] = ok ? acc_s[mb][r] : -INFINITY;
          }
      }
      // ---- online softmax (per query = per lane pair l, l^32)
      float mx = acc_s[0][0];
#pragma unroll
      for (int r = 1; r < 16; ++r) mx = fmaxf(mx, acc_s[0][r]);
#pragma unroll
      for (int r = 0; r < 16; ++r) mx = fmaxf(mx, acc_s[1][r]);
      mx = fmaxf(mx, other_half(mx));
      const bool grow = mx > m_used + lazy_raw;
      if (__builtin_amdgcn_ballot_w64(grow) != 0) {
        const float m_new = grow ? mx : m_used;
        const float alpha = __builtin_amdgcn_exp2f((m_used - m_new) * c);
        m_used = m_new;
        l_lane *= alpha;
#pragma unroll
        for (int mb = 0; mb < 4; ++mb)
#pragma unroll
          for (int r = 0; r < 16; ++r) acc_o[mb][r] *= alpha;
      }
      const float mc = m_used * c;
      unsigned pk[2][8];
      float psum = 0.f;
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int r = 0; r < 16; r += 2) {
          const float p0f = __builtin_amdgcn_exp2f(fmaf(acc_s[mb][r], c, -mc));
          const float p1f = __builtin_amdgcn_exp2f(fmaf(acc_s[mb][r + 1], c, -mc));
          psum += p0f + p1f;
          pk[mb][r >> 1] = pack_f16(p0f, p1f);
        }
      l_lane += psum;
      // ---- O^T += V^T P^T ; k-step t covers keys t*16 .. t*16+15 of the tile
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        if (need[t >> 1]) {
          const int pb = (t & 1) * 4;
          u32x4 pu = {pk[t >> 1][pb], pk[t >> 1][pb + 1], pk[t >> 1][pb + 2], pk[t >> 1][pb + 3]};
          const f16x8 pf = __builtin_bit_cast(f16x8, pu);
#pragma unroll
          for (int mb = 0; mb < 4; ++mb) {
            const s16x4 v0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(vb + voff[mb] + (t * 16) * 256));
            const s16x4 v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(vb + voff[mb] + (t * 16 + 8) * 256));
            u32x2 a0 = __builtin_bit_cast(u32x2, v0), a1 = __builtin_bit_cast(u32x2, v1);
            u32x4 vu = {a0[0], a0[1], a1[0], a1[1]};
            acc_o[mb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, vu), pf, acc_o[mb], 0, 0, 0);
          }
        }
      }
    }
    if (jt < jt_hi) store_tile(buf ^ 1);
    __syncthreads();
  }

  // ---- normalise and store O (bf16, rounded once)
  const float l_tot = l_lane + other_half(l_lane);
  const float inv = 1.f / l_tot;
  if (q_valid) {
    bf16_t* og = (bf16_t*)a.o + b * a.q_stride_b + iq * a.q_stride_t + (int64_t)h * kD;
#pragma unroll
    for (int mb = 0; mb < 4; ++mb)
#pragma unroll
      for (int rq = 0; rq < 4; ++rq) {
        u32x2 w = {pack_bf16(acc_o[mb][rq * 4] * inv, acc_o[mb][rq * 4 + 1] * inv),
                   pack_bf16(acc_o[mb][rq * 4 + 2] * inv, acc_o[mb][rq * 4 + 3] * inv)};
        *(u32x2*)(og + mb * 32 + rq * 8 + hf * 4) = w;
      }
  }
}

}  // namespace

bool swa_mfma_supported(const AttnView& a, int dtype) {
  if (dtype != YOCO_BF16 || a.d != kD) return false;
  if (!(a.scale > 0.f) || !(a.scale < 1e30f)) return false;      // the kernel tracks max(s) and multiplies by scale later
  if (a.q_pos0 + a.Tq >= (1LL << 30)) return false;                 // 32-bit relative positions inside the kernel
  const int64_t n_qtiles = (a.Tq + kBM - 1) / kBM;
  const int64_t total = n_qtiles * a.Hq * a.B;
  return total < (1LL << 31);
}

hipError_t launch_swa_mfma(const AttnView& a, hipStream_t s) {
  Args g;
  g.a = a;
  g.n_qtiles = (int)((a.Tq + kBM - 1) / kBM);
  g.total = g.n_qtiles * a.Hq * a.B;
  g.n_keys = a.q_pos0 + a.Tq;
  hipLaunchKernelGGL(swa_mfma_kernel, dim3(g.total), dim3(256), 0, s, g);
  return hipGetLastError();
}

}  // namespace yoco
