// Flash-style attention prefill on bf16 MFMA for gfx950, head_dim 128.
// Serves yoco_swa_prefill (Eq. 8: causal window of C keys) and
// yoco_cross_attn_prefill (Eq. 3: causal over the global cache, GQA) through
// one kernel: a query at absolute position p sees keys j with p - C < j <= p.
//
// Workgroup = 4 wavefronts, 128 query rows of one head; wavefront w owns rows
// 32w .. 32w+31. Keys are walked in tiles of 64, only tiles that intersect
// some row's window are visited, and a wavefront skips the tiles that none of
// its own rows can see; the mask is applied only on the tiles that need it.
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
// Tiles are double buffered in LDS and the next tile is in flight (global ->
// registers) while the current one is computed. LDS rows are 256 B; K is XOR-swizzled
// in 16-byte chunks and V in 32-byte chunks so both operand read patterns are
// bank-conflict free.
#include <type_traits>

#include "mfma_util.h"
#include "yoco_common.h"

namespace yoco {

namespace {

constexpr int kD = 128;          // head dimension
constexpr int kBN = 64;          // keys per tile
constexpr int kNQ = 32;          // query rows per wavefront
constexpr int kWaves = 4;
constexpr int kThreads = kWaves * 64;
constexpr int kStageRows = 1024 / kThreads;   // 16-byte chunks of a K (or V) tile per thread
constexpr int kStageStep = kThreads / 16;     // rows between a thread's chunks
constexpr int kBM = kNQ * kWaves;
constexpr int kTileBytes = kBN * kD * 2;     // 16 KiB
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kNegBig = -1.0e30f;
constexpr float kLazyLog2 = 8.0f;            // rescale only when the max grows by more than 2^8

struct Args {
  AttnView a;
  int n_qtiles;       // query tiles per (sequence, head)
  int total;          // workgroups
  int64_t n_keys;     // keys that exist (rows beyond are never read)
};

__global__ void __launch_bounds__(kThreads, 2) swa_mfma_kernel(Args g) {
  // Two tile buffers as distinct arrays, so that the compiler can tell the
  // stores of the next tile from the operand reads of the current one.
  __shared__ __attribute__((aligned(1024))) char k_a[kTileBytes], k_b[kTileBytes];
  __shared__ __attribute__((aligned(1024))) char v_a[kTileBytes], v_b[kTileBytes];
  const AttnView& a = g.a;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);      // wavefront-uniform: scalar branches below
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

  // ---- tile walk. The n_t tiles of this workgroup are visited in the cyclic
  // order "tile index mod n_t" (any order is valid for an online softmax):
  // neighbouring query tiles, which share all but two of their key tiles and
  // run at the same time on the same XCD, then touch the same key tile at the
  // same step, so a tile comes from HBM once and from L2 for its other readers.
  const int n_t = jt_hi - jt_lo + 1;
  const int rot = n_t - jt_lo % n_t;                      // step s visits tile jt_lo + (s + rot) % n_t
  auto tile_of = [&](int s) { return jt_lo + (s + rot) % n_t; };

  // ---- tile staging: global -> registers -> LDS for both K and V. (LDS-direct
  // loads were measured slower here: a wavefront's later LDS reads queue behind
  // its pending global_load_lds, which exposes one memory latency per tile.)
  // V is converted to fp16 on the way. The rows of step s+1 are published
  // during the first product of step s, and the loads of step s+2 follow them.
  const int c16 = tid & 15, srow = tid >> 4;             // thread -> 16-byte chunk c16 of rows srow + 16 i
  const uint32_t row_bytes = (uint32_t)a.kv_stride_n * 2u;
  // LDS byte offsets of row srow (row srow + 16 i is 4096 i further: the
  // swizzles depend on row & 15 / row & 7 only, which 16 i does not change)
  const int kst_off = srow * 256 + ((c16 ^ (srow & 15)) << 4);
  const int vst_off = srow * 256 + (((((c16 >> 1) ^ (srow & 7)) << 1) | (c16 & 1)) << 4);
  u32x4 kst[kStageRows], vst[kStageRows];
  auto load_row = [&](int jt, int i) {
    const int64_t tile_row0 = (int64_t)jt * kBN;
    const int lim = (int)(g.n_keys - 1 - tile_row0 < kBN - 1 ? g.n_keys - 1 - tile_row0 : kBN - 1);   // last row that exists
    const int lrow = srow + kStageStep * i;
    const int grow = lrow < lim ? lrow : lim;             // rows past the end repeat the last one (masked later)
    const uint32_t off = (uint32_t)grow * row_bytes + (uint32_t)(c16 << 4);
    kst[i] = *(const u32x4*)((const char*)(kg + tile_row0 * a.kv_stride_n) + off);
    vst[i] = *(const u32x4*)((const char*)(vg + tile_row0 * a.kv_stride_n) + off);
  };
  auto load_tile = [&](int jt) {
#pragma unroll
    for (int i = 0; i < kStageRows; ++i) load_row(jt, i);
  };
  auto store_row = [&](char* k_dst, char* v_dst, int i) {
    u32x4 vh = {bf16x2_to_f16x2(vst[i][0]), bf16x2_to_f16x2(vst[i][1]), bf16x2_to_f16x2(vst[i][2]),
                bf16x2_to_f16x2(vst[i][3])};
    *(u32x4*)(k_dst + kst_off + i * (kStageStep * 256)) = kst[i];
    *(u32x4*)(v_dst + vst_off + i * (kStageStep * 256)) = vh;
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
  // K (A operand of S^T): row mb*32 + lq, chunk (ks*2 + hf) ^ (row & 15). The
  // chunk field is bits 4..7 of the offset, so k-step ks is koff0 ^ (ks << 5).
  const int koff0 = lq * 256 + ((hf ^ (lq & 15)) << 4);
  // V^T (A operand of O^T) via transposing reads: lane s = lane % 16 of a block
  // of 16 supplies row z = hf*4 + s/4 (+ t*16 + half*8), dims (mb*2 + db)*16 + 4*(s%4),
  // 32-byte chunk (mb*2 + db) ^ z: dim block mb is voff0 ^ (mb << 6).
  const int s16 = lane & 15, db = (lane >> 4) & 1, z = hf * 4 + (s16 >> 2);
  const int voff0 = z * 256 + ((db ^ z) << 5) + ((s16 & 3) << 3);

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

  // ---- prologue: tile of step 0 into buffer a, tile of step 1 in flight
  load_tile(tile_of(0));
#pragma unroll
  for (int i = 0; i < kStageRows; ++i) store_row(k_a, v_a, i);
  if (n_t > 1) load_tile(tile_of(1));
  __syncthreads();
  // Q is complete here; saying so keeps the loop free of waits on it (the
  // tile prefetch loads issued inside the loop must stay in flight).
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) asm volatile("" : "+v"(qf[ks]));

  // ---- one step = one key tile (64 keys) for this wavefront:
  //   [S^T = K Q^T  with  publishing the staged rows of the next step's tile
  //    and issuing the loads of the tile after it]
  //   mask (edge tiles only), running max, lazy rescale
  //   [weights and O^T += V^T P^T]
  // The first and third part each mix MFMA with vector work in one basic block,
  // so the two wavefronts that share a SIMD (one per resident workgroup) can
  // overlap their pipes in most phase combinations.
  auto step = [&](int st, char* k_cur, char* v_cur, char* k_nxt, char* v_nxt) {
    const int jt = tile_of(st);
    const int j0r = (jt - jt_lo) * kBN;                 // tile's first key, relative origin
    // does some row of this wavefront see some key of the tile? / every row every key?
    const bool need = (j0r <= pw_lo + kNQ - 1) && (j0r + kBN - 1 > pw_lo - win32);
    const bool full = (j0r + kBN - 1 <= pw_lo) && (j0r > pw_lo + kNQ - 1 - win32);
    // the same for the two 32-key halves: on edge tiles a wavefront multiplies only the halves it needs
    const bool need0 = need && (j0r + 31 > pw_lo - win32);
    const bool need1 = need && (j0r + 32 <= pw_lo + kNQ - 1);
    const bool both = need0 && need1;
    const bool stage = st + 1 < n_t, prefetch = st + 2 < n_t;
    lds_char* kb = (lds_char*)k_cur;
    lds_char* vb = (lds_char*)v_cur;
    int kbase = koff0, vbase = voff0;
    asm volatile("" : "+v"(kbase), "+v"(vbase));        // keep the 12 derived offsets out of long-lived registers
    auto kfrag = [&](int ks, int mb) {
      return __builtin_bit_cast(bf16x8, *(const __attribute__((address_space(3))) u32x4*)(kb + (kbase ^ (ks << 5)) + mb * 32 * 256));
    };
    const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    f32x16 s0 = zero, s1 = zero;                         // keys 0..31 and 32..63 of the tile
    if (both && prefetch) {
      // the common case, one basic block: 16 MFMAs, the 4 staged rows, 8 loads
      const int jt2 = tile_of(st + 2);
      // raised issue priority while this wavefront feeds the matrix pipe: the
      // other wavefront of the SIMD fills in with its vector work (measured -4 %)
      __builtin_amdgcn_s_setprio(2);
      // operand fragments are read two k-steps (4 MFMAs) ahead of their use
      bf16x8 f0[8], f1[8];
      f0[0] = kfrag(0, 0); f1[0] = kfrag(0, 1);
      f0[1] = kfrag(1, 0); f1[1] = kfrag(1, 1);
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        if (ks + 2 < 8) { f0[ks + 2] = kfrag(ks + 2, 0); f1[ks + 2] = kfrag(ks + 2, 1); }
        s0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f0[ks], qf[ks], ks == 0 ? zero : s0, 0, 0, 0);
        s1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f1[ks], qf[ks], ks == 0 ? zero : s1, 0, 0, 0);
        // a staged row is published and its registers reloaded at once: the
        // loads go out a pair at a time between the products, not as a burst
        if ((ks & 1) && (ks >> 1) % (4 / kStageRows) == 0) {
          store_row(k_nxt, v_nxt, (ks >> 1) / (4 / kStageRows));
          load_row(jt2, (ks >> 1) / (4 / kStageRows));
        }
        __builtin_amdgcn_sched_barrier(0);
      }
      __builtin_amdgcn_s_setprio(0);
    } else {
      if (need0) {
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) s0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kfrag(ks, 0), qf[ks], ks == 0 ? zero : s0, 0, 0, 0);
      }
      if (need1) {
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) s1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kfrag(ks, 1), qf[ks], ks == 0 ? zero : s1, 0, 0, 0);
      }
      if (stage) {
#pragma unroll
        for (int i = 0; i < kStageRows; ++i) store_row(k_nxt, v_nxt, i);
      }
      if (prefetch) load_tile(tile_of(st + 2));
    }
    if (need) {
      if (!full) {                                       // keys outside (p - C, p] of this lane's query
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = j0r + (r >> 2) * 8 + hf * 4 + (r & 3);
          s0[r] = (need0 && (unsigned)(pq_rel0 - key) < (unsigned)win32) ? s0[r] : -INFINITY;
          s1[r] = (need1 && (unsigned)(pq_rel0 - key - 32) < (unsigned)win32) ? s1[r] : -INFINITY;
        }
      }
      // ---- online softmax (a query is the lane pair l, l ^ 32); the
      // accumulators are rescaled only when the max grows by more than 2^kLazyLog2
      float mx = fmaxf(s0[0], s1[0]);
#pragma unroll
      for (int r = 1; r < 16; ++r) mx = fmaxf(mx, fmaxf(s0[r], s1[r]));
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
      unsigned pk0[8], pk1[8];
      const unsigned ones = 0x3c003c00u;                // (1.0, 1.0) in fp16
#pragma unroll
      for (int r = 0; r < 16; r += 2) {
        pk0[r >> 1] = pack_f16(__builtin_amdgcn_exp2f(fmaf(s0[r], c, -mc)), __builtin_amdgcn_exp2f(fmaf(s0[r + 1], c, -mc)));
        pk1[r >> 1] = pack_f16(__builtin_amdgcn_exp2f(fmaf(s1[r], c, -mc)), __builtin_amdgcn_exp2f(fmaf(s1[r + 1], c, -mc)));
        // the row sum uses the rounded weights, the ones the second product sees
        l_lane = __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2, pk0[r >> 1]), __builtin_bit_cast(f16x2, ones), l_lane, false);
        l_lane = __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2, pk1[r >> 1]), __builtin_bit_cast(f16x2, ones), l_lane, false);
      }
      // ---- O^T += V^T P^T ; k-step t covers keys t*16 .. t*16+15 of the tile
      __builtin_amdgcn_s_setprio(1);
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        if (!both && !((t >> 1) ? need1 : need0)) continue;   // a skipped half has zero weights
        const unsigned* pk = (t >> 1) ? pk1 : pk0;
        const int pb = (t & 1) * 4;
        u32x4 pu = {pk[pb], pk[pb + 1], pk[pb + 2], pk[pb + 3]};
        const f16x8 pf = __builtin_bit_cast(f16x8, pu);
#pragma unroll
        for (int mb = 0; mb < 4; ++mb) {
          const s16x4 v0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(vb + (vbase ^ (mb << 6)) + (t * 16) * 256));
          const s16x4 v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(vb + (vbase ^ (mb << 6)) + (t * 16 + 8) * 256));
          u32x2 a0 = __builtin_bit_cast(u32x2, v0), a1 = __builtin_bit_cast(u32x2, v1);
          u32x4 vu = {a0[0], a0[1], a1[0], a1[1]};
          acc_o[mb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, vu), pf, acc_o[mb], 0, 0, 0);
        }
      }
      __builtin_amdgcn_s_setprio(0);
    }
    __syncthreads();
  };
  for (int st = 0; st < n_t; st += 2) {
    step(st, k_a, v_a, k_b, v_b);
    if (st + 1 >= n_t) break;
    step(st + 1, k_b, v_b, k_a, v_a);
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
  hipLaunchKernelGGL(swa_mfma_kernel, dim3(g.total), dim3(kThreads), 0, s, g);
  return hipGetLastError();
}

}  // namespace yoco
