// Chunkwise gated retention on the matrix cores (section 3.1, Eq. 6; the
// equivalence with Eq. 4 and Eq. 5 is appendix B). bf16, dk = dv = 128.
//
// With G_j the sum of log2(gamma) from the first row of j's chunk up to and
// including j, chunk [i] of one head computes
//   U_i      = K^T (V * 2^(G_last - G_j))                local state of the chunk
//   R_i      = U_i + 2^G_last R_{i-1}                    state after the chunk
//   O_[i]    = scale * ((Q K^T * D) V + (Q R_{i-1}) * 2^(G_j)),  D(j,k) = 2^(G_j - G_k), k <= j
// in four launches:
//   0  cumulative decays G (one wavefront per chunk)
//   1  the states, scanned inside a segment: a workgroup walks a run of consecutive chunks of one head with the
//      running state L in its accumulators (L <- 2^G_last L + U_i after each chunk; fp16 MFMA, V scaled while
//      staged) and leaves, for every chunk but the first of the run, the state before the chunk *within the
//      segment* in fp32. U_i itself never reaches memory. The run's total goes out in fp32 as well.
//   2  the scan across segments (a few states per head, element-wise), leaving the state before each segment
//   3  outputs, one workgroup per 128 query rows: R_{i-1} = (state before the chunk within its segment) +
//      2^(decay since the segment's start) * (state before the segment), formed in fp32 while it is staged and
//      split into two bf16 planes hi + lo (16 significant bits, fp32's exponent range: no scaling to track, and
//      both feed the bf16 MFMA against the bf16 Q as it stands); the cross-chunk product R_{i-1}^T Q^T (bf16 MFMA on both planes) scaled per
//      row, then the key tiles of the chunk up to the diagonal as in the sliding-window kernel, with the decay
//      2^(G_j - G_k) in place of the softmax; optional GroupNorm and swish gate (Eq. 7) before the store.
// States are stored transposed ([dv][dk]); this is also the layout of
// the caller's state_in / state_out.
//
// Orientation, tiling, LDS swizzles, the fp16 second product (P rounded to fp16,
// V converted while staged) are those of swa_mfma.hip, for the same reasons.
// Launch 1 converts K as well (both operands of its product are fp16), and the
// weights scale * s * decay are not bounded by 1 as softmax weights are: |k|,
// |v| and |scale * q.k| of 65520 or more are outside these kernels' domain.
#include "mfma_util.h"
#include "yoco_common.h"

namespace yoco {

namespace {

constexpr int kD = 128;
constexpr int kBN = 64;                       // keys per tile
constexpr int kBM = 128;                      // query rows per workgroup of launch 3
constexpr int kTileBytes = kBN * kD * 2;      // 16 KiB
constexpr int kState = kD * kD;               // elements of one state
constexpr int kMaxChunk = 1024;
constexpr float kLog2e = 1.4426950408889634f;

struct ChunkArgs {
  GretView a;
  int chunk, nc;       // rows per chunk, chunks per sequence
  int seg, nseg;       // chunks per segment, segments per sequence
  float* gc;           // [B][H][nc * chunk]   cumulative log2 decay within the chunk, inclusive
  float* rw;           // [B][H][nc][dv][dk]   state before the chunk within its segment
  float* seg_total;    // [B][H][nseg][dv][dk] state a segment adds, started from zero
  float* seg_init;     // [B][H][nseg][dv][dk] state before the segment
  float* gpre;         // [B][H][nc]           log2 decay from the start of the chunk's segment to the start of the chunk
  float* gseg;         // [B][H][nseg]         log2 decay over the whole segment
};

__device__ __forceinline__ int64_t last_row_of_chunk(const ChunkArgs& g, int c) {
  const int64_t e = (int64_t)(c + 1) * g.chunk;
  return (e < g.a.T ? e : g.a.T) - 1;
}

// ---- launch 0: G. One wavefront per (chunk, head, sequence); lane l owns chunk / 64 consecutive rows.
__global__ void __launch_bounds__(64) gret_cumdecay_kernel(ChunkArgs g) {
  const int c = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  const int lane = threadIdx.x, rpl = g.chunk / 64;
  const int64_t row0 = (int64_t)c * g.chunk + lane * rpl;
  float x[kMaxChunk / 64];
  float acc = 0.f;
#pragma unroll
  for (int i = 0; i < kMaxChunk / 64; ++i) {
    if (i < rpl) {
      const int64_t row = row0 + i;
      acc += row < g.a.T ? g.a.log_gamma[((int64_t)b * g.a.T + row) * g.a.H + h] * kLog2e : 0.f;
      x[i] = acc;
    }
  }
  float incl = acc;
  for (int o = 1; o < 64; o <<= 1) {
    const float t = __shfl_up(incl, o);
    if (lane >= o) incl += t;
  }
  const float before = incl - acc;
  float* out = g.gc + (((int64_t)b * g.a.H + h) * g.nc + c) * g.chunk + lane * rpl;
#pragma unroll
  for (int i = 0; i < kMaxChunk / 64; ++i)
    if (i < rpl) out[i] = x[i] + before;
}

// Byte offset of 16-byte chunk c16 of row `row` in a 64-row tile, "transposing read" layout
// (32-byte chunk XOR row & 7), and the per-lane base of the transposing fragment reads.
__device__ __forceinline__ int tr_store_off(int row, int c16) {
  return row * 256 + (((((c16 >> 1) ^ (row & 7)) << 1) | (c16 & 1)) << 4);
}

// A (or B) operand fragment of 32 dims x 16 keys from a [64 keys][128 dims] fp16 tile: lane l gets dim
// blk * 32 + l % 32 and, with hf = l / 32, the keys t*16 + hf*4 + 0..3 then t*16 + 8 + hf*4 + 0..3.
__device__ __forceinline__ f16x8 tr_frag(lds_char* tile, int base, int blk, int t) {
  const s16x4 v0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(tile + (base ^ (blk << 6)) + (t * 16) * 256));
  const s16x4 v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(tile + (base ^ (blk << 6)) + (t * 16 + 8) * 256));
  const u32x2 a0 = __builtin_bit_cast(u32x2, v0), a1 = __builtin_bit_cast(u32x2, v1);
  const u32x4 vu = {a0[0], a0[1], a1[0], a1[1]};
  return __builtin_bit_cast(f16x8, vu);
}

// ---- launch 1: the states of a segment. Workgroup = 4 wavefronts, each a 64 x 64 block of L^T = sum (V * w)^T K;
// at every chunk boundary inside the segment the block is stored and decayed by the next chunk's 2^G_last.
__global__ void __launch_bounds__(256, 3) gret_chunk_state_kernel(ChunkArgs g) {
  __shared__ __attribute__((aligned(1024))) char k_t[kTileBytes], v_t[kTileBytes];
  const GretView& a = g.a;
  // heads vary fastest over the grid: workgroups that run together read neighbouring 256-byte segments of the same rows
  const int h = blockIdx.x, sg = blockIdx.y, b = blockIdx.z;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int hf = lane >> 5, lq = lane & 31;
  const int64_t bh = (int64_t)b * a.H + h;
  const int first = sg * g.seg;                                       // first chunk of the segment
  const int c_end = first + g.seg < g.nc ? first + g.seg : g.nc;
  const int64_t r0 = (int64_t)first * g.chunk;
  const int64_t last = last_row_of_chunk(g, c_end - 1);               // last row of the segment
  const float* gc = g.gc + bh * g.nc * g.chunk;                       // indexed by the row within the sequence
  const bf16_t* kg = (const bf16_t*)a.k + ((int64_t)b * a.T * a.H + h) * kD;
  const bf16_t* vg = (const bf16_t*)a.v + ((int64_t)b * a.T * a.H + h) * kD;
  const int64_t row_stride = (int64_t)a.H * kD;

  const int c16 = tid & 15, srow = tid >> 4;
  const int s16 = lane & 15, db = (lane >> 4) & 1, z = hf * 4 + (s16 >> 2);
  const int fbase = z * 256 + ((db ^ z) << 5) + ((s16 & 3) << 3);
  const int mb0 = (wave >> 1) * 2, nb0 = (wave & 1) * 2;

  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int tiles_per_chunk = g.chunk / kBN;
  const int n_tiles = (int)((last - r0) / kBN) + 1;
  u32x4 kr[4], vr[4];
  float w[4];
  auto load_tile = [&](int t0) {
    const float g_last = gc[last_row_of_chunk(g, first + t0 / tiles_per_chunk)];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int64_t row = r0 + (int64_t)t0 * kBN + srow + 16 * i;
      const int64_t grow = row <= last ? row : last;                // rows past the end weigh nothing
      w[i] = row <= last ? __builtin_amdgcn_exp2f(g_last - gc[grow]) : 0.f;
      kr[i] = *(const u32x4*)(kg + grow * row_stride + c16 * 8);
      vr[i] = *(const u32x4*)(vg + grow * row_stride + c16 * 8);
    }
  };
  load_tile(0);
  float gsum = 0.f;                                                  // log2 decay from the segment's start (thread 0 keeps it)
  if (tid == 0) g.gpre[bh * g.nc + first] = 0.f;
  for (int t0 = 0; t0 < n_tiles; ++t0) {
    if (t0 > 0 && t0 % tiles_per_chunk == 0) {                       // a chunk of the segment ends here
      const int c = first + t0 / tiles_per_chunk;                    // the chunk that starts
      const float decay = __builtin_amdgcn_exp2f(gc[last_row_of_chunk(g, c)]);
      int lane_off = (mb0 * 32 + hf * 4) * kD + nb0 * 32 + lq;       // kept local: 64 hoisted store addresses cost an occupancy step
      asm volatile("" : "+v"(lane_off));
      float* rw = g.rw + (bh * g.nc + c) * kState + lane_off;
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            rw[(i * 32 + (r >> 2) * 8 + (r & 3)) * kD + j * 32] = acc[i][j][r];
            acc[i][j][r] *= decay;
          }
      if (tid == 0) g.gpre[bh * g.nc + c] = (gsum += gc[last_row_of_chunk(g, c - 1)]);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int lrow = srow + 16 * i;
      u32x4 kh, vh;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        kh[e] = bf16x2_to_f16x2(kr[i][e]);
        vh[e] = pack_f16(__uint_as_float(vr[i][e] << 16) * w[i], __uint_as_float(vr[i][e] & 0xffff0000u) * w[i]);
      }
      *(u32x4*)(k_t + tr_store_off(lrow, c16)) = kh;
      *(u32x4*)(v_t + tr_store_off(lrow, c16)) = vh;
    }
    if (t0 + 1 < n_tiles) load_tile(t0 + 1);                        // in flight during the products
    __syncthreads();
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const f16x8 a0 = tr_frag((lds_char*)v_t, fbase, mb0, t), a1 = tr_frag((lds_char*)v_t, fbase, mb0 + 1, t);
      const f16x8 b0 = tr_frag((lds_char*)k_t, fbase, nb0, t), b1 = tr_frag((lds_char*)k_t, fbase, nb0 + 1, t);
      acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a0, b0, acc[0][0], 0, 0, 0);
      acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a0, b1, acc[0][1], 0, 0, 0);
      acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a1, b0, acc[1][0], 0, 0, 0);
      acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a1, b1, acc[1][1], 0, 0, 0);
    }
    __syncthreads();
  }
  if (tid == 0) g.gseg[bh * g.nseg + sg] = gsum + gc[last];
  float* u = g.seg_total + (bh * g.nseg + sg) * kState;
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = (mb0 + i) * 32 + (r >> 2) * 8 + hf * 4 + (r & 3);
        u[row * kD + (nb0 + j) * 32 + lq] = acc[i][j][r];
      }
}

// ---- launch 2: scan over the segments; thread owns 4 consecutive elements of the state. The totals of a group of
// segments are loaded together (independent addresses) before the dependent updates run.
__global__ void __launch_bounds__(256) gret_state_scan_kernel(ChunkArgs g) {
  constexpr int kAhead = 8;
  const GretView& a = g.a;
  const int h = blockIdx.y, b = blockIdx.z;
  const int e = (blockIdx.x * 256 + threadIdx.x) * 4;
  const int64_t bh = (int64_t)b * a.H + h;
  typedef float f32x4 __attribute__((ext_vector_type(4)));
  f32x4 R = {0.f, 0.f, 0.f, 0.f};
  if (a.state_in) R = *(const f32x4*)(a.state_in + bh * kState + e);
  for (int s0 = 0; s0 < g.nseg; s0 += kAhead) {
    f32x4 U[kAhead];
    float alpha[kAhead];
#pragma unroll
    for (int i = 0; i < kAhead; ++i) {
      const int sg = s0 + i < g.nseg ? s0 + i : g.nseg - 1;
      U[i] = __builtin_nontemporal_load((const f32x4*)(g.seg_total + (bh * g.nseg + sg) * kState + e));
      alpha[i] = __builtin_amdgcn_exp2f(g.gseg[bh * g.nseg + sg]);
    }
#pragma unroll
    for (int i = 0; i < kAhead; ++i) {
      if (s0 + i < g.nseg) {
        *(f32x4*)(g.seg_init + (bh * g.nseg + s0 + i) * kState + e) = R;
        R = U[i] + alpha[i] * R;
      }
    }
  }
  if (a.state_out) *(f32x4*)(a.state_out + bh * kState + e) = R;
}

// ---- launch 3: outputs. Workgroup = 4 wavefronts = 128 query rows of one head, all in one chunk.
__global__ void __launch_bounds__(256, 2) gret_chunk_output_kernel(ChunkArgs g) {
  __shared__ __attribute__((aligned(1024))) char k_a[kTileBytes], k_b[kTileBytes];
  __shared__ __attribute__((aligned(1024))) char v_a[kTileBytes], v_b[kTileBytes];
  __shared__ __attribute__((aligned(16))) float g_a[kBN], g_b[kBN];
  const GretView& a = g.a;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int hf = lane >> 5, lq = lane & 31;
  const int h = blockIdx.x, b = blockIdx.z;              // heads vary fastest over the grid, as in launch 1
  const int64_t bh = (int64_t)b * a.H + h;

  const int64_t i0 = (int64_t)blockIdx.y * kBM;           // first query row of the workgroup
  const int c = (int)(i0 / g.chunk);
  const int64_t c0 = (int64_t)c * g.chunk;
  const int64_t rows_here = a.T - i0 < kBM ? a.T - i0 : kBM;
  const int jt_lo = (int)(c0 / kBN), jt_hi = (int)((i0 + rows_here - 1) / kBN);
  const int n_t = jt_hi - jt_lo + 1;

  const bf16_t* kg = (const bf16_t*)a.k + ((int64_t)b * a.T * a.H + h) * kD;
  const bf16_t* vg = (const bf16_t*)a.v + ((int64_t)b * a.T * a.H + h) * kD;
  const uint32_t row_bytes = (uint32_t)a.H * kD * 2u;
  const float* gc = g.gc + bh * g.nc * g.chunk;            // indexed by the row within the sequence

  // ---- staging: global -> registers -> LDS; K rows keep 16-byte chunks XOR row & 15, V rows 32-byte chunks XOR row & 7
  const int c16 = tid & 15, srow = tid >> 4;
  const int kst_off = srow * 256 + ((c16 ^ (srow & 15)) << 4);
  const int vst_off = tr_store_off(srow, c16);
  u32x4 kst[4], vst[4];
  float gst = 0.f;
  auto load_tile = [&](int jt) {
    const int64_t tile_row0 = (int64_t)jt * kBN;
    const int lim = (int)(a.T - 1 - tile_row0 < kBN - 1 ? a.T - 1 - tile_row0 : kBN - 1);   // last row that exists
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int lrow = srow + 16 * i;
      const int grow = lrow < lim ? lrow : lim;            // rows past the end repeat the last one (masked later)
      const uint32_t off = (uint32_t)grow * row_bytes + (uint32_t)(c16 << 4);
      kst[i] = *(const u32x4*)((const char*)(kg + tile_row0 * a.H * kD) + off);
      vst[i] = *(const u32x4*)((const char*)(vg + tile_row0 * a.H * kD) + off);
    }
    if (tid < kBN) gst = gc[tile_row0 + tid];                // padded up to whole chunks: always in bounds
  };
  auto store_tile = [&](char* k_dst, char* v_dst, float* g_dst) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const u32x4 vh = {bf16x2_to_f16x2(vst[i][0]), bf16x2_to_f16x2(vst[i][1]), bf16x2_to_f16x2(vst[i][2]),
                        bf16x2_to_f16x2(vst[i][3])};
      *(u32x4*)(k_dst + kst_off + i * 4096) = kst[i];
      *(u32x4*)(v_dst + vst_off + i * 4096) = vh;
    }
    if (tid < kBN) g_dst[tid] = gst;
  };

  // ---- Q^T fragments (B operand): lane holds query lq, dims ks*16 + hf*8 .. +8
  int64_t iq = i0 + wave * 32 + lq;
  const bool q_valid = iq < a.T;
  if (!q_valid) iq = a.T - 1;
  const bf16_t* qg = (const bf16_t*)a.q + (((int64_t)b * a.T + iq) * a.H + h) * kD;
  bf16x8 qf[8];
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) qf[ks] = __builtin_bit_cast(bf16x8, *(const u32x4*)(qg + ks * 16 + hf * 8));
  const float gq = gc[iq];

  const int koff0 = lq * 256 + ((hf ^ (lq & 15)) << 4);
  const int s16 = lane & 15, db = (lane >> 4) & 1, z = hf * 4 + (s16 >> 2);
  const int voff0 = z * 256 + ((db ^ z) << 5) + ((s16 & 3) << 3);

  f32x16 acc_o[4];
#pragma unroll
  for (int mb = 0; mb < 4; ++mb)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc_o[mb][r] = 0.f;

  // ---- cross-chunk part: O^T = R_{i-1}^T Q^T, then every query column times scale * 2^(G_q). R_{i-1} is put
  // together in fp32 from the state before the chunk within its segment and the decayed state before
  // the segment, and its two bf16 planes (128 x 128 each) pass through the four tile buffers, laid out like K tiles.
  const int sg = c / g.seg, first = sg * g.seg;
  const bool has_local = c > first;
  const bool has_init = sg > 0 || a.state_in != nullptr;
  const bool has_past = has_local || has_init;
  if (has_past) {
    typedef float f32x4 __attribute__((ext_vector_type(4)));
    const float* rw = g.rw + (bh * g.nc + c) * kState;
    const float* si = g.seg_init + (bh * g.nseg + sg) * kState;
    const float fpre = has_init ? __builtin_amdgcn_exp2f(g.gpre[bh * g.nc + c]) : 0.f;
    // every load of this part, and the first key tile after them, is issued before anything waits
    f32x4 wl[8][2], wi[8][2];
#pragma unroll
    for (int i = 0; i < 8; ++i) {                                   // rows srow + 16 i of both planes
      const int off = (srow + 16 * i) * kD + c16 * 8;
#pragma unroll
      for (int p = 0; p < 2; ++p) {
        wl[i][p] = has_local ? *(const f32x4*)(rw + off + 4 * p) : (f32x4){0.f, 0.f, 0.f, 0.f};
        wi[i][p] = has_init ? *(const f32x4*)(si + off + 4 * p) : (f32x4){0.f, 0.f, 0.f, 0.f};
      }
    }
    load_tile(jt_lo);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      u32x4 hi, lo;
#pragma unroll
      for (int p = 0; p < 2; ++p)
#pragma unroll
        for (int e = 0; e < 2; ++e) {
          const float x0 = fmaf(fpre, wi[i][p][2 * e], wl[i][p][2 * e]);
          const float x1 = fmaf(fpre, wi[i][p][2 * e + 1], wl[i][p][2 * e + 1]);
          const unsigned hw = pack_bf16(x0, x1);
          hi[2 * p + e] = hw;
          lo[2 * p + e] = pack_bf16(x0 - __uint_as_float(hw << 16), x1 - __uint_as_float(hw & 0xffff0000u));
        }
      *(u32x4*)((i >= 4 ? k_b : k_a) + kst_off + (i & 3) * 4096) = hi;
      *(u32x4*)((i >= 4 ? v_b : v_a) + kst_off + (i & 3) * 4096) = lo;
    }
    __syncthreads();
#pragma unroll
    for (int mb = 0; mb < 4; ++mb) {
      lds_char* ph = (lds_char*)((mb >> 1) ? k_b : k_a) + (mb & 1) * 32 * 256;
      lds_char* pl = (lds_char*)((mb >> 1) ? v_b : v_a) + (mb & 1) * 32 * 256;
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        const bf16x8 ah = __builtin_bit_cast(bf16x8, *(const __attribute__((address_space(3))) u32x4*)(ph + (koff0 ^ (ks << 5))));
        const bf16x8 al = __builtin_bit_cast(bf16x8, *(const __attribute__((address_space(3))) u32x4*)(pl + (koff0 ^ (ks << 5))));
        acc_o[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, qf[ks], acc_o[mb], 0, 0, 0);
        acc_o[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al, qf[ks], acc_o[mb], 0, 0, 0);
      }
    }
    const float f = a.scale * __builtin_amdgcn_exp2f(gq);
#pragma unroll
    for (int mb = 0; mb < 4; ++mb)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc_o[mb][r] *= f;
    __syncthreads();                                              // the buffers are free for the key tiles
  } else {
    load_tile(jt_lo);
  }
  store_tile(k_a, v_a, g_a);
  if (n_t > 1) load_tile(jt_lo + 1);
  __syncthreads();

  // ---- inner-chunk part: key tiles from the chunk's first row up to the diagonal
  const int64_t pw_lo = i0 + wave * 32;                 // first row of the wavefront
  const int64_t pq = pw_lo + lq;                        // this lane's query row
  auto step = [&](int st, char* k_cur, char* v_cur, float* g_cur, char* k_nxt, char* v_nxt, float* g_nxt) {
    const int64_t j0 = (int64_t)(jt_lo + st) * kBN;     // first key of the tile
    const bool need0 = j0 <= pw_lo + 31;                // some row of the wavefront sees keys 0..31 of the tile
    const bool need1 = j0 + 32 <= pw_lo + 31;           //                              ... keys 32..63
    const bool full = j0 + kBN - 1 <= pw_lo;            // every row sees every key
    lds_char* kb = (lds_char*)k_cur;
    lds_char* vb = (lds_char*)v_cur;
    auto kfrag = [&](int ks, int mb) {
      return __builtin_bit_cast(bf16x8, *(const __attribute__((address_space(3))) u32x4*)(kb + (koff0 ^ (ks << 5)) + mb * 32 * 256));
    };
    const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    f32x16 s0 = zero, s1 = zero;
    if (need0) {
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) s0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kfrag(ks, 0), qf[ks], ks == 0 ? zero : s0, 0, 0, 0);
    }
    if (need1) {
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) s1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kfrag(ks, 1), qf[ks], ks == 0 ? zero : s1, 0, 0, 0);
    }
    if (need0) {
      // weights: scale * s * 2^(G_q - G_k); keys after the query (diagonal tiles only) weigh nothing
      typedef float f32x4 __attribute__((ext_vector_type(4)));
      unsigned pk0[8], pk1[8];
#pragma unroll
      for (int rq = 0; rq < 4; ++rq) {
        const f32x4 gk0 = *(const f32x4*)(g_cur + rq * 8 + hf * 4);
        const f32x4 gk1 = *(const f32x4*)(g_cur + 32 + rq * 8 + hf * 4);
        float p0[4], p1[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int64_t key = j0 + rq * 8 + hf * 4 + e;
          p0[e] = s0[rq * 4 + e] * a.scale * __builtin_amdgcn_exp2f(gq - gk0[e]);
          p1[e] = s1[rq * 4 + e] * a.scale * __builtin_amdgcn_exp2f(gq - gk1[e]);
          if (!full) {
            p0[e] = key <= pq ? p0[e] : 0.f;
            p1[e] = (need1 && key + 32 <= pq) ? p1[e] : 0.f;
          }
        }
        pk0[rq * 2] = pack_f16(p0[0], p0[1]);
        pk0[rq * 2 + 1] = pack_f16(p0[2], p0[3]);
        pk1[rq * 2] = pack_f16(p1[0], p1[1]);
        pk1[rq * 2 + 1] = pack_f16(p1[2], p1[3]);
      }
      // O^T += V^T P^T ; k-step t covers keys t*16 .. t*16+15 of the tile
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        if ((t >> 1) && !need1) continue;               // a skipped half has zero weights
        const unsigned* pk = (t >> 1) ? pk1 : pk0;
        const int pb = (t & 1) * 4;
        const u32x4 pu = {pk[pb], pk[pb + 1], pk[pb + 2], pk[pb + 3]};
        const f16x8 pf = __builtin_bit_cast(f16x8, pu);
#pragma unroll
        for (int mb = 0; mb < 4; ++mb)
          acc_o[mb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(tr_frag(vb, voff0, mb, t), pf, acc_o[mb], 0, 0, 0);
      }
    }
    if (st + 1 < n_t) store_tile(k_nxt, v_nxt, g_nxt);
    if (st + 2 < n_t) load_tile(jt_lo + st + 2);
    __syncthreads();
  };
  for (int st = 0; st < n_t; st += 2) {
    step(st, k_a, v_a, g_a, k_b, v_b, g_b);
    if (st + 1 >= n_t) break;
    step(st + 1, k_b, v_b, g_b, k_a, v_a, g_a);
  }

  // ---- GroupNorm over the head's 128 values of each query (held by the lane pair l, l ^ 32), then store
  float mean = 0.f, rstd = 1.f;
  if (a.group_norm) {
    float sum = 0.f;
#pragma unroll
    for (int mb = 0; mb < 4; ++mb)
#pragma unroll
      for (int r = 0; r < 16; ++r) sum += acc_o[mb][r];
    sum += other_half(sum);
    mean = sum * (1.f / kD);
    float sq = 0.f;
#pragma unroll
    for (int mb = 0; mb < 4; ++mb)
#pragma unroll
      for (int r = 0; r < 16; ++r) sq += (acc_o[mb][r] - mean) * (acc_o[mb][r] - mean);
    sq += other_half(sq);
    rstd = rsqrtf(sq * (1.f / kD) + a.eps);
  }
  if (q_valid) {
    const int64_t row_off = (((int64_t)b * a.T + iq) * a.H + h) * kD;
    bf16_t* og = (bf16_t*)a.o + row_off;
    const bf16_t* gg = a.gate ? (const bf16_t*)a.gate + row_off : nullptr;
#pragma unroll
    for (int mb = 0; mb < 4; ++mb)
#pragma unroll
      for (int rq = 0; rq < 4; ++rq) {
        float y[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) y[e] = (acc_o[mb][rq * 4 + e] - mean) * rstd;
        if (gg) {                                         // swish gate of Eq. 7: y * g * sigmoid(g)
          const u32x2 gw = *(const u32x2*)(gg + mb * 32 + rq * 8 + hf * 4);
          const float gv[4] = {__uint_as_float(gw[0] << 16), __uint_as_float(gw[0] & 0xffff0000u),
                               __uint_as_float(gw[1] << 16), __uint_as_float(gw[1] & 0xffff0000u)};
#pragma unroll
          for (int e = 0; e < 4; ++e) y[e] *= gv[e] / (1.f + __expf(-gv[e]));
        }
        const u32x2 w = {pack_bf16(y[0], y[1]), pack_bf16(y[2], y[3])};
        *(u32x2*)(og + mb * 32 + rq * 8 + hf * 4) = w;
      }
  }
}

size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

}  // namespace

bool gret_chunk_supported(int B, int64_t T, int H, int dk, int dv, int chunk, int dtype) {
  if (dtype != YOCO_BF16 || dk != kD || dv != kD) return false;
  if (chunk % kBM || chunk > kMaxChunk) return false;
  if (T <= 0 || (T + kBM - 1) / kBM > 65535) return false;          // query blocks are the grid's y dimension
  return B <= 65535;
}

// Chunks per segment: long enough that the states written per chunk are the only state traffic, short enough that
// the state launch still fills the chip at its occupancy (3 workgroups on each of 256 CUs) when the shape allows it.
int gret_segment_chunks(int B, int H, int nc) {
  int64_t s = (int64_t)nc * B * H / 768;
  if (s < 1) s = 1;
  if (s > 16) s = 16;
  return (int)s;
}

size_t gret_chunk_workspace(int B, int64_t T, int H, int chunk) {
  const size_t nc = (size_t)((T + chunk - 1) / chunk), bh = (size_t)B * H;
  const size_t seg = (size_t)gret_segment_chunks(B, H, (int)nc), nseg = (nc + seg - 1) / seg;
  return align256(bh * nc * chunk * sizeof(float)) + align256(bh * nc * kState * sizeof(float)) +
         2 * align256(bh * nseg * kState * sizeof(float)) + align256(bh * nc * sizeof(float)) + align256(bh * nseg * sizeof(float));
}

hipError_t launch_gret_chunk(const GretView& a, int chunk, void* workspace, hipStream_t s) {
  ChunkArgs g;
  g.a = a;
  g.chunk = chunk;
  g.nc = (int)((a.T + chunk - 1) / chunk);
  g.seg = gret_segment_chunks(a.B, a.H, g.nc);
  g.nseg = (g.nc + g.seg - 1) / g.seg;
  const size_t bh = (size_t)a.B * a.H;
  char* p = (char*)workspace;
  g.gc = (float*)p;
  p += align256(bh * g.nc * chunk * sizeof(float));
  g.rw = (float*)p;
  p += align256(bh * g.nc * kState * sizeof(float));
  g.seg_total = (float*)p;
  p += align256(bh * g.nseg * kState * sizeof(float));
  g.seg_init = (float*)p;
  p += align256(bh * g.nseg * kState * sizeof(float));
  g.gpre = (float*)p;
  p += align256(bh * g.nc * sizeof(float));
  g.gseg = (float*)p;
  hipLaunchKernelGGL(gret_cumdecay_kernel, dim3(g.nc, a.H, a.B), dim3(64), 0, s, g);
  hipLaunchKernelGGL(gret_chunk_state_kernel, dim3(a.H, g.nseg, a.B), dim3(256), 0, s, g);
  hipLaunchKernelGGL(gret_state_scan_kernel, dim3(kState / 1024, a.H, a.B), dim3(256), 0, s, g);
  hipLaunchKernelGGL(gret_chunk_output_kernel, dim3(a.H, (unsigned)((a.T + kBM - 1) / kBM), a.B), dim3(256), 0, s, g);
  return hipGetLastError();
}

}  // namespace yoco
