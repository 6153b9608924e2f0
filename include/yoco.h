/*
 * libyoco -- the attention hot path of YOCO ("You Only Cache Once",
 * arXiv 2405.05254) for AMD MI355X (gfx950).
 *
 * Operations, each a hand-written HIP kernel behind a plain C ABI:
 *   yoco_swa_prefill          sliding-window attention of the self-decoder
 *                             (section 3.2, Eq. 8)
 *   yoco_global_kv_write      store rows of the once-only global K^/V^ cache
 *                             (section 2.2, Eq. 2; the projection is the caller's)
 *   yoco_cross_attn_prefill   causal GQA attention of Tq query rows over the
 *                             global cache (section 2.2, Eq. 3)
 *   yoco_cross_attn_decode    the same for one new token per sequence, split
 *                             over the cache and merged by log-sum-exp
 *   yoco_swa_cache_write, yoco_kv_cache_append, yoco_swa_decode
 *                             token-by-token generation: the self-decoder's
 *                             rolling window cache (section 3.2) and batched
 *                             one-row appends
 *   yoco_gret_prefill, yoco_gret_decode
 *                             gated retention (section 3.1, Eq. 4-7), chunkwise
 *                             for prompts and recurrent for generation
 *
 * Conventions
 *   - Every pointer named q/k/v/o/lens/workspace/mem is DEVICE memory owned by
 *     the caller. The library allocates nothing, frees nothing and keeps no
 *     pointer after a call returns (the cache descriptor is a plain struct the
 *     caller holds). Pointers must be 16-byte aligned.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls only enqueue work; they never synchronise.
 *   - Tensors are dense and row-major; the last index is contiguous.
 *     [T,H,d] means element (t,h,e) at offset ((t*H)+h)*d + e.
 *   - Positions are 0-based. `scale` multiplies q.k before the softmax (the
 *     paper's Eq. 8 prints none; Eq. 3 defers to standard attention, whose
 *     value is 1/sqrt(d)).
 *   - GQA: query head h reads KV head h / (Hq / Hkv); Hq must be a multiple of
 *     Hkv.
 *   - Every call validates its arguments before launching anything and
 *     returns YOCO_OK (0) or a negative yoco_status; a failing call has no
 *     side effect. yoco_last_error_string() describes the last failure on the
 *     calling thread.
 *   - Arithmetic: products of the stored dtype, fp32 accumulation and fp32
 *     softmax; outputs are rounded once (to nearest even) to the dtype.
 *   - Calls on different streams may run concurrently as long as they do not
 *     share a workspace, a state, or cache rows one of them writes; the
 *     library keeps no state of its own between calls.
 */
#ifndef YOCO_H
#define YOCO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum yoco_status {
  YOCO_OK = 0,
  YOCO_ERR_INVALID_ARG = -1, /* null pointer, non-positive size, out-of-range position */
  YOCO_ERR_UNSUPPORTED = -2, /* dtype / head_dim / group size with no kernel */
  YOCO_ERR_ALIGNMENT = -3,   /* pointer not 16-byte aligned or d not a multiple of 8 */
  YOCO_ERR_WORKSPACE = -4,   /* workspace or cache memory too small */
  YOCO_ERR_HIP = -5          /* the HIP runtime refused a launch */
} yoco_status;

typedef enum yoco_dtype {
  YOCO_F32 = 0,
  YOCO_BF16 = 1,
  YOCO_INT8 = 2 /* only as the dtype of a global cache, see below */
} yoco_dtype;

/*
 * Descriptor of the global KV cache (section 2.2: one K^/V^ pair per sequence,
 * shared by all cross-decoder layers; Table 1: O((N+L)D) memory).
 * Layout in the caller's memory block: a K plane followed by a V plane, each
 * [B][Hkv][N_cap][d] -- head-major, so the rows one KV head streams during
 * decode are contiguous (d * sizeof(dtype) bytes each, 256 B at d=128 bf16).
 * Bytes per cached token = 2 * Hkv * d * sizeof(dtype), whatever the depth.
 */
typedef struct yoco_kv_cache {
  void* k;          /* device: K plane */
  void* v;          /* device: V plane */
  int32_t B;        /* sequences */
  int32_t Hkv;      /* KV heads */
  int32_t d;        /* head dimension */
  int32_t dtype;    /* yoco_dtype */
  int64_t N_cap;    /* rows per sequence the planes can hold */
} yoco_kv_cache;

/*
 * The 8-bit global cache (dtype YOCO_INT8; section 1 names 8-bit KV quantisation
 * as the usual way to shrink the cache, the paper prescribes no scheme). Rows
 * are coded when they are written, by yoco_global_kv_write and
 * yoco_kv_cache_append, one fp32 scale per row and KV head, all in float32:
 *   a = max|x| over the row's d numbers,  scale = a / 127,
 *   code_e = round-half-even(x_e * (127 / a)), in [-127, 127]
 * (a zero row: scale 0, codes 0), and the row stands for code_e * scale.
 * Every element is off by at most scale / 2 = max|x| / 254. Attention reads the
 * codes: yoco_cross_attn_decode, and yoco_cross_attn_prefill for up to 8 rows
 * with the decode workspace (the exit row of an early-exit prefill); q and o
 * are bf16. head_dim must be 128 and Hq / Hkv at most 16. A rolling window
 * cache cannot be 8-bit.
 * Layout of a plane per (sequence, KV head): ceil(N_cap / 64) blocks of 64 rows,
 * 8448 bytes each: 8192 code bytes, then the rows' 64 fp32 scales in row order;
 * 132 bytes per cached token, KV head and plane instead of 256 in bf16. The
 * code bytes are ordered as the matrix cores take them. Row r (0..63) of a
 * block, dim e (0..127):
 *   K plane, code as a signed byte, at offset
 *     ((((r/4)%4)*2 + e/64)*64 + ((e%64)/16)*16 + 4*(r/16) + r%4)*16 + e%16
 *   V plane, byte = code + 128, stored transposed, at offset
 *     ((e/16)*64 + (r/16)*16 + e%16)*16 + r%16
 * Decode keeps 16 bits of each query below the largest |q| of its head (two
 * int8 parts) and rounds each softmax weight times row scale to fp16.
 */

/* Bytes the cache needs: 2 * B * Hkv * N_cap * d * sizeof(dtype); for
 * YOCO_INT8 2 * B * Hkv * ceil(N_cap / 64) * 8448. Host only. */
int yoco_kv_cache_bytes(int B, int Hkv, int d, int64_t N_cap, int dtype, size_t* bytes);

/* Fill `out` for a caller-allocated block `mem` of `bytes` bytes (device
 * memory, 256-byte aligned). Host only; the memory is not touched. */
int yoco_kv_cache_init(void* mem, size_t bytes, int B, int Hkv, int d, int64_t N_cap, int dtype,
                       yoco_kv_cache* out);

/*
 * Sliding-window attention, Eq. 8 without the W_O product:
 *   o[b,i,h,:] = sum_j softmax_j(scale * q[b,i,h,:] . k[b,j,g,:]) v[b,j,g,:],
 *   j in [max(0, i-window+1), i],  g = h / (Hq/Hkv)
 * (the mask  i - C < j <= i : a row sees itself and the window-1 keys before).
 * q, o: [B,T,Hq,d]; k, v: [B,T,Hkv,d]; all of `dtype`. window >= 1; a window
 * >= T is plain causal attention.
 * Domain of the bf16, d = 128 matrix-core path: the softmax weights and V enter
 * the second product as fp16 (fp32 accumulation), so |v| must stay below 65504
 * (a larger bf16 value becomes infinite there); |v| under 2^-14 loses low bits
 * or flushes to zero, an absolute error below 2^-25 per element. q and k have
 * no such limit (bf16 products, exact in fp32). fp32 inputs, other head
 * dimensions and scale <= 0 run on fp32 vector kernels without this limit.
 */
int yoco_swa_prefill(const void* q, const void* k, const void* v, void* o, int B, int64_t T, int Hq,
                     int Hkv, int d, int64_t window, float scale, int dtype, void* stream);

/*
 * Store n projected rows K^[pos0..pos0+n), V^[pos0..pos0+n) of sequence b into
 * the cache (Eq. 2 is computed by the caller: RMSNorm and the two GEMMs).
 * k, v: [n,Hkv,d] of `src_dtype`; rows are converted to the cache dtype
 * (round to nearest even; coded as above for an 8-bit cache). Requires
 * 0 <= pos0, pos0 + n <= N_cap, 0 <= b < B.
 * n == 0 is a no-op.
 */
int yoco_global_kv_write(const yoco_kv_cache* c, const void* k, const void* v, int b, int64_t pos0,
                         int64_t n, int src_dtype, void* stream);

/*
 * The same write with the RMSNorm of Eq. 2 folded in (section 2.2, Eq. 2 with
 * LN = RMSNorm, section 2.1): since RMSNorm(x) W = (1 / rms(x)) * (x (diag(g) W)),
 * the caller can skip the normalisation pass over X^{L/2}, multiply the raw
 * rows by the gain-scaled weights diag(g) W_K, diag(g) W_V, and hand over those
 * products together with one float32 factor per row, row_scale[r] =
 * 1 / sqrt(mean(x_r^2) + eps) (device memory, [n]). Every element is multiplied
 * by its row's factor in float32 and then cast (or coded, for an 8-bit cache)
 * exactly as yoco_global_kv_write does. row_scale == NULL is
 * yoco_global_kv_write.
 */
int yoco_global_kv_write_scaled(const yoco_kv_cache* c, const void* k, const void* v, const float* row_scale,
                                int b, int64_t pos0, int64_t n, int src_dtype, void* stream);

/*
 * Cross-decoder attention of Eq. 3 for Tq query rows of sequence b; row i has
 * absolute position q_pos0 + i and attends to cache rows j <= q_pos0 + i
 * (causal). q, o: [Tq,Hq,d] of the cache dtype (bf16 for an 8-bit cache).
 * Requires q_pos0 + Tq <= N_cap;
 * the rows read must have been written.
 * workspace: optional device scratch (NULL = none), 16-byte aligned. With at
 * least yoco_cross_attn_decode_workspace(c, Hq) bytes, a call with Tq <= 8 rows
 * (the exit row of an early-exit prefill, Fig. 3) is split over the cache like
 * a decode step instead of walking it with one workgroup per head. The result
 * is the same operation either way.
 * A bf16 cache with d = 128 and more than 8 rows runs on the same matrix-core
 * path as yoco_swa_prefill, with the same domain: cached |v| below 65504, and
 * |v| under 2^-14 read with an absolute error below 2^-25.
 */
int yoco_cross_attn_prefill(const yoco_kv_cache* c, const void* q, void* o, int b, int64_t q_pos0,
                            int64_t Tq, int Hq, float scale, void* workspace, size_t workspace_bytes,
                            void* stream);

/* Workspace for yoco_cross_attn_decode on this cache with Hq query heads:
 * `splits` partial results (running max, sum, d-vector in fp32) per
 * (sequence, query head). Host only. */
int yoco_cross_attn_decode_workspace(const yoco_kv_cache* c, int Hq, size_t* bytes, int* splits);

/*
 * One decode step of a cross-decoder layer (Fig. 3 "Generation"): for every
 * sequence b one query token; q, o: [B,Hq,d] of the cache dtype (bf16 for an
 * 8-bit cache). lens: device
 * int64 [B]; sequence b attends to cache rows [0, lens[b]) -- its own row has
 * been written before the call (Eq. 2 precedes Eq. 3, the mask is j <= i).
 * lens[b] is clamped to [0, N_cap]; a sequence with lens[b] == 0 gets zeros.
 * Pass 1 reduces each split of the cache to (max, sum, vector) for all query
 * heads of a KV head in one read; pass 2 merges the splits by log-sum-exp in
 * a fixed order (no atomics: results are bit-reproducible).
 */
int yoco_cross_attn_decode(const yoco_kv_cache* c, const void* q, void* o, const int64_t* lens, int Hq,
                           float scale, void* workspace, size_t workspace_bytes, void* stream);

/*
 * yoco_cross_attn_decode for callers that cannot allocate device memory or
 * carry a workspace: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc. Same operation, same kernels and bit-identical
 * results; the split partials live in a static device array inside the library
 * (YOCO_NOALLOC_SCRATCH_BYTES per GPU the library runs on, held until the
 * process ends) instead of a caller workspace. The call allocates and frees
 * nothing. A shape whose partials (yoco_cross_attn_decode_workspace) exceed the
 * array is refused with YOCO_ERR_WORKSPACE before anything is launched.
 * All calls on one GPU share that GPU's array: two calls that overlap in time
 * on one GPU (different streams or threads) race; calls on one stream are
 * ordered. Nothing in the array needs clearing between calls (pass 1 writes
 * every partial the merge reads).
 */
#define YOCO_NOALLOC_SCRATCH_BYTES ((size_t)4 << 20)
int yoco_cross_attn_decode_noalloc(const yoco_kv_cache* c, const void* q, void* o, const int64_t* lens, int Hq,
                                   float scale, void* stream);

/*
 * ---- Token-by-token generation through the self-decoder ----
 * Sliding-window attention needs only the last C rows of a layer's K and V
 * (section 3.2, Eq. 8; the footnote of section 2.3 and Table 1 count this
 * cache as O(C) per self-decoder layer, constant in the sequence length).
 * The rolling cache is a yoco_kv_cache whose N_cap is the window C, used as a
 * ring: the row of position p lives in slot p mod C, where it replaces
 * position p - C, which no later row can see. One such cache per
 * self-decoder layer; yoco_kv_cache_bytes / _init size and describe it.
 */

/*
 * Store n rows K[pos0..pos0+n), V[pos0..pos0+n) of sequence b into a rolling
 * cache (after a prefill: the rows a later decode step can still see).
 * k, v: [n,Hkv,d] of `src_dtype`. Row pos0 + r goes to slot (pos0 + r) mod
 * N_cap; when n > N_cap only the last N_cap rows are stored. pos0 >= 0,
 * 0 <= b < B; n == 0 is a no-op.
 */
int yoco_swa_cache_write(const yoco_kv_cache* ring, const void* k, const void* v, int b, int64_t pos0,
                         int64_t n, int src_dtype, void* stream);

/*
 * Append one row per sequence, at positions known only on the device (a decode
 * step of a batch whose sequences have different lengths). k, v: [B,Hkv,d] of
 * `src_dtype`; pos: device int64 [B]. Sequence b's row goes to slot pos[b]
 * (ring == 0: the global cache of Eq. 2) or pos[b] mod N_cap (ring != 0: a
 * rolling cache). A sequence with pos[b] < 0, or with pos[b] >= N_cap when
 * ring == 0, is skipped (nothing is written for it).
 */
int yoco_kv_cache_append(const yoco_kv_cache* c, const void* k, const void* v, const int64_t* pos, int ring,
                         int src_dtype, void* stream);

/*
 * One decode step of a self-decoder layer: Eq. 8 for one new token per
 * sequence. q, o: [B,Hq,d] of the cache dtype. lens: device int64 [B], the
 * number of tokens of sequence b so far including the new one (the mask
 * includes j = i). k_new, v_new: the new token's rows, [B,Hkv,d] of the cache
 * dtype, which the call stores at slot (lens[b] - 1) mod N_cap before
 * attending (sequences with lens[b] <= 0 store nothing); or both NULL when
 * the rows have been appended already (yoco_kv_cache_append). The row attends to
 * the min(lens[b], N_cap) rows the ring holds, which are exactly positions
 * lens[b]-N_cap .. lens[b]-1; the order of the slots is irrelevant to a
 * softmax-weighted sum. Same two passes, workspace
 * (yoco_cross_attn_decode_workspace on this ring) and reproducibility as
 * yoco_cross_attn_decode.
 */
int yoco_swa_decode(const yoco_kv_cache* ring, const void* q, const void* k_new, const void* v_new, void* o,
                    const int64_t* lens, int Hq, float scale, void* workspace, size_t workspace_bytes, void* stream);

/*
 * ---- Gated retention, the paper's other self-decoder module (section 3.1) ----
 * Per head, with decays gamma_n in (0, 1] given as log_gamma[b,n,h] = ln gamma_n
 * (fp32; Eq. 4: gamma = sigmoid(X W_gamma)^(1/tau), computed by the caller):
 *   o_n = scale * sum_{m <= n} (prod_{i=m+1..n} gamma_i) (q_n . k_m) v_m      (Eq. 4)
 * which equals the recurrence S_n = gamma_n S_{n-1} + k_n^T v_n, o_n = scale * q_n S_n
 * (Eq. 5) and the chunkwise form of Eq. 6. q, k: [B,T,H,dk]; v, o: [B,T,H,dv],
 * all of `dtype`. Eq. 4 prints no scale; any value cancels in the GroupNorm.
 * The rotation Theta of Eq. 4 is the caller's (q and k arrive rotated, or not).
 * group_norm != 0 applies Eq. 7's GroupNorm_h to every head's dv-vector before
 * it is stored: (o - mean) / sqrt(var + eps), no learned affine. gate (NULL =
 * none; else like v, the caller's X W_G) multiplies the result by swish(gate) =
 * gate * sigmoid(gate), the gate of Eq. 7; W_O is the caller's.
 * States are fp32 [B,H,dv,dk]: element (e_v, e_k) is S[e_k][e_v] of Eq. 5, i.e.
 * S is stored transposed so that its rows run along the key dimension.
 * state_in: the state before row 0 (NULL = zeros); state_out: receives the
 * state after the last row (NULL = not stored); they may be the same memory.
 * Domain of the chunkwise bf16 path: its products run on fp16 operands, so
 * |k|, |v| and |scale * q.k| must stay below 65504 (magnitudes under 2^-14
 * lose low bits or flush, an absolute error below 2^-25); the recurrent
 * kernel computes in fp32 and has no such limit.
 */

/* Scratch bytes yoco_gret_prefill needs for its chunkwise path on this shape
 * (0 when the shape has no such path and the recurrent kernel serves it). Host only. */
int yoco_gret_prefill_workspace(int B, int64_t T, int H, int dk, int dv, int chunk, int dtype, size_t* bytes);

/*
 * Gated retention over T rows per sequence (prefill; Eq. 6 with chunk size
 * `chunk`, the paper uses 256). bf16 with dk = dv = 128 and chunk a multiple
 * of 128 runs chunkwise on the matrix cores when `workspace` holds at least
 * yoco_gret_prefill_workspace() bytes (device memory, 256-byte aligned); every
 * other case runs the recurrence, which computes the same function (dk, dv <=
 * 128). T == 0 copies state_in to state_out.
 */
int yoco_gret_prefill(const void* q, const void* k, const void* v, const float* log_gamma, const void* gate, void* o,
                      const float* state_in, float* state_out, int B, int64_t T, int H, int dk, int dv, int chunk,
                      float scale, int group_norm, float eps, int dtype, void* workspace, size_t workspace_bytes,
                      void* stream);

/*
 * One generation step (Eq. 5) for one new row per sequence: q, k: [B,H,dk];
 * v, gate, o: [B,H,dv]; log_gamma: [B,H]; state: [B,H,dv,dk] fp32, updated in place.
 */
int yoco_gret_decode(const void* q, const void* k, const void* v, const float* log_gamma, const void* gate, void* o, float* state,
                     int B, int H, int dk, int dv, float scale, int group_norm, float eps, int dtype, void* stream);

/*
 * ---- Measured ceilings (measurement aids for the benchmark, not part of the path) ----
 * yoco_ceiling_mfma: `workgroups` workgroups of 8 wavefronts each issue
 * 8 * iters back-to-back v_mfma_f32_32x32x16_bf16 (32768 flops each) on
 * operands read once from `seed` (device, 16384 bytes: zeros and random values
 * give different rates, the clock follows the data); flops per launch =
 * workgroups * 8 * 8 * iters * 32768. `sink`: 4 device bytes, practically never
 * written. yoco_ceiling_stream_read: reads `bytes` (a multiple of 16) of `buf`
 * once with 128-bit nontemporal loads, `workgroups` contiguous shares.
 * yoco_ceiling_attn_loop: the inner loop of flash attention on its own (no
 * staging, masks, barriers or tile walk), same operands, `workgroups`
 * workgroups of 8 wavefronts, 32 * iters MFMAs per wavefront. mode 1: every
 * MFMA takes its A operand as a fresh 128-bit LDS fragment; mode 2: the same
 * plus the softmax work of two scores (2 fma, 2 exp2, fp16 pack, row-sum dot2)
 * after every second MFMA, the ratio of the prefill kernel at head_dim 128.
 * flops per launch = workgroups * 8 * 32 * iters * 32768.
 */
int yoco_ceiling_mfma(const void* seed, void* sink, int iters, int workgroups, void* stream);
int yoco_ceiling_attn_loop(const void* seed, void* sink, int iters, int workgroups, int mode, void* stream);
int yoco_ceiling_stream_read(const void* buf, size_t bytes, void* sink, int workgroups, void* stream);

/* Description of the last failure on the calling thread ("" if none). */
const char* yoco_last_error_string(void);

/* Library version, e.g. 100 = 0.1.0. */
int yoco_version(void);

#ifdef __cplusplus
}
#endif
#endif /* YOCO_H */
