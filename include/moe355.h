/*
 * moe355 -- forward pass of one Mixture-of-Experts layer on AMD MI355X (gfx950),
 * with FP8 (e4m3) block-scaled expert GEMMs and a Router Replay mode.
 *
 * The operations follow the paper's statement of the problem:
 *   - Router Replay (section 2.4.4): the expert choices made by the router at
 *     rollout time are recorded and reused verbatim when the layer is evaluated
 *     again, instead of being recomputed.
 *   - FP8 rollout (section 3.1.2): weights arrive block-wise quantised to FP8
 *     and activations are quantised to FP8 on the fly, in the dense linear layers as well as the MoE layers.
 * The paper gives no formulas for the layer; each entry point below states the
 * definition it implements.
 *
 * Conventions
 *   - Every data pointer is a DEVICE pointer owned by the caller.  The library
 *     neither frees nor keeps it after the call returns.
 *   - All work is enqueued on the HIP stream given to moe_create(); calls return
 *     without synchronising.  A context must not be used from two threads at once.
 *   - Notation: T tokens, d hidden size, E experts, k experts per token, F expert
 *     FFN width, N = T*k assignments.  d and F must be multiples of 128.
 *   - bf16 values are passed as uint16_t bit patterns, e4m3 codes as uint8_t
 *     (OCP "FN" variant: bias 7, max 448, no infinities, 0x7F/0xFF = NaN).
 *   - Return value: 0 on success, a negative MOE_E* code otherwise.  On an error
 *     detected by argument validation nothing has been enqueued.
 *   - An empty batch is legal: with T == 0 (or rows == 0 for the calls that take a row
 *     count) the arrays that would have no elements may be null; the routing calls then
 *     only write offsets[0..E] = 0 and the other calls enqueue nothing.
 */
#ifndef MOE355_H
#define MOE355_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MOE_OK        0
#define MOE_EINVAL   -1   /* null pointer, bad shape, d or F not a multiple of 128, k > E, block != 128 */
#define MOE_EHIP     -2   /* a HIP runtime call or kernel launch failed */
#define MOE_EBADIDS  -3   /* moe_check_ids found an expert id outside [0,E), or one repeated inside a token */
#define MOE_ENOMEM   -4   /* workspace allocation failed */

typedef struct moe_ctx moe_ctx;

typedef struct {
    int32_t T;  /* tokens per call (upper bound is not needed: exact); T*k <= 2^30, T*d < 2^31 */
    int32_t d;  /* hidden size, multiple of 128 */
    int32_t E;  /* experts, 1..256 */
    int32_t k;  /* experts per token, 1..min(E,16) */
    int32_t F;  /* expert FFN width, multiple of 128; F*d < 2^32 */
} moe_dims;

/* Create a context for one layer shape.  Allocates the internal device workspace
 * (chunk histograms, the tile work list, and the quantised hidden activations
 * hq [N,F] u8 + hs [F/128][N] f32).  hip_stream is a hipStream_t (NULL = default
 * stream).  The device current at creation must be current at every later call. */
int moe_create(moe_ctx** out, const moe_dims* dims, void* hip_stream);
int moe_destroy(moe_ctx* ctx);
const char* moe_strerror(int code);

/* Routed mode.  logit[t,e] = sum_c x[t,c]*W_router[e,c] (fp32 accumulation);
 * score = logit + sel_bias[e] (sel_bias may be NULL = 0; it affects selection
 * only).  topk_idx[t,0..k-1] = the k experts of largest score in descending
 * score order, equal scores resolved towards the lower expert index.
 * topk_w[t,j] = softmax over the k selected unbiased logits.  Then the stable
 * permutation of moe_route_replay is built from topk_idx.
 *   x_bf16 [T,d] row-major; W_router [E,d] fp32 row-major; sel_bias [E] or NULL.
 *   Outputs: topk_idx [T,k] i32, topk_w [T,k] f32, offsets [E+1] i32,
 *   perm [N] i32, inv_perm [N] i32.
 * k must equal the context's k. */
int moe_route(moe_ctx* ctx, const uint16_t* x_bf16, const float* W_router, const float* sel_bias,
              int32_t k, int32_t* topk_idx, float* topk_w,
              int32_t* offsets, int32_t* perm, int32_t* inv_perm);

/* Router Replay mode (section 2.4.4).  logged_idx/logged_w are copied verbatim to
 * topk_idx/topk_w: no router GEMM, no softmax, no renormalisation.  x_bf16 is
 * accepted for symmetry with moe_route and is not read (may be NULL).
 * The permutation is the stable counting sort of flat assignments i = t*k+j by
 * expert id: offsets[e] = number of assignments with id < e, offsets[E] = N;
 * inv_perm[i] = offsets[id_i] + #{i' < i : id_i' = id_i}; perm[inv_perm[i]] = i.
 * Ids outside [0,E) never fault; their assignments are skipped and a device flag
 * is raised that moe_check_ids reports.  An id that repeats an earlier slot of the same
 * token raises a second flag (also reported by moe_check_ids); the permutation is still the
 * stable sort of the ids as given. */
int moe_route_replay(moe_ctx* ctx, const uint16_t* x_bf16, const int32_t* logged_idx,
                     const float* logged_w, int32_t* topk_idx, float* topk_w,
                     int32_t* offsets, int32_t* perm, int32_t* inv_perm);

/* moe_route_replay for callers that cannot allocate device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  It needs no context: the permutation's workspace (per-chunk
 * histograms) lives in a static 512 KiB device array inside the library, which bounds the batch at
 * T*k <= 1048576 assignments (MOE_EINVAL beyond that; also for E > 256, k > min(E,16), null pointers).  The
 * call enqueues kernels only (no hipMalloc, no hipFree, no hipMemset) on hip_stream (NULL = default stream),
 * on the current device.  Same outputs, bit for bit, as moe_route_replay.
 *   id_flags: two ints of device memory owned by the caller, or NULL.  The call first clears them, then
 *   id_flags[0] is set if an id lies outside [0,E) and id_flags[1] if an id repeats inside a token (with NULL
 *   the flags go to the library's array and are not reported).
 * Every call on one GPU uses the same array: calls that overlap on a GPU (different streams or threads) race;
 * calls in stream order do not.  T == 0: only offsets[0..E] = 0 is written. */
int moe_route_replay_noalloc(void* hip_stream, int32_t T, int32_t E, int32_t k,
                             const int32_t* logged_idx, const float* logged_w,
                             int32_t* topk_idx, float* topk_w, int32_t* offsets,
                             int32_t* perm, int32_t* inv_perm, int32_t* id_flags);

/* Ids-only Router Replay (section 2.4.4 read literally: the router's DECISIONS are reused).  The logged
 * expert ids are copied to topk_idx; the gate weights are recomputed from this engine's own logits,
 * topk_w[t,j] = softmax over logit[t, logged_idx[t,0..k-1]] (same logits, same arithmetic as moe_route, so
 * logging moe_route's own ids reproduces its weights bit for bit).  No selection bias takes part.  Then the
 * permutation is built as in moe_route_replay.  Ids outside [0,E) never fault: their weight is computed
 * from logit 0, their assignments are skipped and moe_check_ids reports them.
 *   x_bf16 [T,d]; W_router [E,d] fp32; logged_idx [T,k] i32; outputs as moe_route. */
int moe_route_replay_ids(moe_ctx* ctx, const uint16_t* x_bf16, const float* W_router,
                         const int32_t* logged_idx, int32_t* topk_idx, float* topk_w,
                         int32_t* offsets, int32_t* perm, int32_t* inv_perm);

/* Synchronises the stream and returns MOE_EBADIDS if any routing call on this
 * context since the last check met an expert id outside [0,E), or (replay calls) a
 * logged id that occurs twice inside one token; else MOE_OK.  Clears both flags. */
int moe_check_ids(moe_ctx* ctx);

/* Per-row FP8 quantisation with optional fan-out to expert order.
 * For each input row r and each group g of `block` (=128) consecutive columns:
 *   amax = max|x[r,g]|; s = amax/448 in fp32 (1.0 if amax = 0);
 *   code = e4m3(x/s), fp32 division, round to nearest even, saturating.
 * dst_rows == NULL: output row r receives input row r (fanout must be 1).
 * Otherwise output rows dst_rows[r*fanout + j], j < fanout, all receive the
 * quantised input row r (pass inv_perm and fanout = k to build the expert-ordered
 * activation matrix in one pass over x).
 *   x_bf16 [rows_in, cols]; q [rows_out, cols] u8 with rows_out = rows_in*fanout;
 *   scales [cols/128][rows_out] f32, group-major: the scale of output row p and
 *   column group g is scales[g*rows_out + p] (one contiguous plane per 128-column
 *   block, the order in which the grouped GEMM walks them).  cols must be a
 *   multiple of 128.
 * Does not use the context's T/d: any rows_in >= 0 and cols are accepted. */
int moe_quantize_fp8(moe_ctx* ctx, const uint16_t* x_bf16, int64_t rows_in, int32_t cols,
                     int32_t block, const int32_t* dst_rows, int32_t fanout,
                     uint8_t* q, float* scales);

/* Block-wise FP8 quantisation of a weight matrix (section 3.1.2: the weight-update path quantises
 * the trainer's weights block-wise before handing them to the FP8 rollout engine).  One fp32 scale per
 * 128x128 block: s = amax/448 (1.0 for an all-zero block), code = e4m3(w/s) with fp32 division, round
 * to nearest even, saturating: the weight format moe_expert_ffn_fp8 and moe_linear_fp8 consume.
 *   w_bf16 [rows, cols] row-major, rows and cols multiples of 128 (an [E,F,d] tensor is passed as
 *   rows = E*F, cols = d); q [rows, cols] u8; scales [rows/128, cols/128] f32. */
int moe_quantize_weights_fp8(moe_ctx* ctx, const uint16_t* w_bf16, int64_t rows, int32_t cols,
                             uint8_t* q, float* scales);

/* Dense block-scaled FP8 linear layer (section 3.1.2 applies FP8 to the dense linear layers as well as to the MoE layers):
 *   y[p,n] = sum_kb xs[kb,p]*ws[n/128,kb] * sum_{c in block kb} xq[p,c]*Wq[n,c],  fp32 out.
 * The grouped down-projection kernel with one group that owns every row.
 *   xq [rows,K] u8 and xs [K/128][rows] f32 as written by moe_quantize_fp8 (dst_rows = NULL);
 *   Wq [NOUT,K] u8; ws [NOUT/128, K/128] f32; y [rows,NOUT] f32.  K and NOUT multiples of 128.
 * Uses the context's work-list storage: ceil(rows/256)*ceil(NOUT/256) must not exceed
 * (T*k/256 + E) * (F/128 + ceil(d/256)) of the context's dims, else MOE_EINVAL; NOUT*K must be
 * below 2^32 (MOE_EINVAL otherwise). */
int moe_linear_fp8(moe_ctx* ctx, const uint8_t* xq, const float* xs, int32_t rows, int32_t K,
                   const uint8_t* Wq, const float* ws, int32_t NOUT, float* y);

/* Grouped SwiGLU expert FFN on expert-sorted rows.  For expert e and rows
 * p in [offsets[e], offsets[e+1]):
 *   g[p,f] = sum_kb xs[kb,p]*s1[e,f/128,kb] * sum_{c in block kb} xq[p,c]*W1[e,f,c]
 *   u[p,f] = the same with W3, s3
 *   h = g/(1+exp(-g)) * u (fp32), quantised per row per 128 columns exactly like
 *       moe_quantize_fp8 -> hq, hs (kept in the context workspace)
 *   y_perm[p,c] = sum_fb hs[fb,p]*s2[e,c/128,fb] * sum_{f in block fb} hq[p,f]*W2[e,c,f]
 * FP8 products are accumulated in fp32 on the matrix cores, one 128-wide block at
 * a time, and each block's partial sum is scaled in fp32.
 *   xq_perm [N,d] u8; xs_perm [d/128][N] f32 (group-major, as moe_quantize_fp8 writes
 *   it); offsets [E+1] i32 (device);
 *   W1,W3 [E,F,d] u8; W2 [E,d,F] u8; s1,s3 [E,F/128,d/128] f32; s2 [E,d/128,F/128] f32;
 *   y_perm [N,d] f32. */
int moe_expert_ffn_fp8(moe_ctx* ctx, const uint8_t* xq_perm, const float* xs_perm,
                       const int32_t* offsets, const uint8_t* W1, const uint8_t* W3,
                       const uint8_t* W2, const float* s1, const float* s3, const float* s2,
                       float* y_perm);

/* The same FFN with the token gather fused into the gate/up GEMM: xq_tok [T,d] u8 and xs_tok [d/128][T] f32
 * are the activations quantised ONCE per token, in token order (moe_quantize_fp8 with dst_rows = NULL);
 * expert-sorted row p reads token perm[p]/k.  perm [N] i32 and offsets [E+1] i32 are the ones a routing call
 * wrote for this batch; the call keeps no routing state of its own.  A perm entry that names a token
 * beyond T-1 reads token T-1 instead of faulting.  No expert-ordered copy of the activations exists: the
 * layer saves its k-fold write and re-read.  Results are bit-identical to moe_expert_ffn_fp8 on the
 * gathered rows. */
int moe_expert_ffn_fp8_gather(moe_ctx* ctx, const uint8_t* xq_tok, const float* xs_tok, const int32_t* perm,
                              const int32_t* offsets, const uint8_t* W1, const uint8_t* W3,
                              const uint8_t* W2, const float* s1, const float* s3, const float* s2,
                              float* y_perm);

/* Weighted combine back to token order:
 *   y[t,c] = bf16( sum_{j<k} topk_w[t,j] * y_perm[inv_perm[t*k+j], c] ),
 * fp32 fused multiply-adds in slot order, one rounding to bf16 at the end.
 *   y_perm [N,d] f32; inv_perm [N] i32; topk_w [T,k] f32; y_bf16 [T,d].
 *   y_f32 [T,d] f32 or NULL: if given, also receives the fp32 sums before the rounding (a parity aid: the
 *   rounded outputs of two implementations differ by whole bf16 steps wherever their sums straddle a rounding
 *   boundary, the sums themselves show the actual difference). */
int moe_combine(moe_ctx* ctx, const float* y_perm, const int32_t* inv_perm, const float* topk_w,
                uint16_t* y_bf16, float* y_f32);

/* Length-based load balancing before rollout (paper section 3.1.1): distributes n samples over
 * n_groups worker groups so that the groups' total predicted generation lengths are about equal.
 * The paper states the goal only; the rule taken is longest-first list scheduling: samples are
 * visited by decreasing pred_len (equal lengths by increasing index) and each goes to the group
 * with the smallest running total that still has room (lowest group index on equal totals).
 * equal_count != 0: group g takes at most n / n_groups + (g < n % n_groups) samples, i.e. the
 * batches of synchronous data-parallel workers stay equal-sized; 0: no limit.
 * Host-side scheduling step: ALL pointers are HOST pointers, no context, no stream, no GPU work.
 *   pred_len [n] in, >= 0;  group_of [n] out;  order [n] out: sample indices group after group,
 *   inside a group in the order handed out;  bounds [n_groups+1] out: group g owns
 *   order[bounds[g] .. bounds[g+1]);  totals [n_groups] out: summed pred_len per group.
 * MOE_EINVAL on a null pointer (pred_len/group_of/order may be null when n == 0), n < 0,
 * n_groups < 1 or a negative length; MOE_ENOMEM if temporary host memory cannot be had. */
int moe_balance_lengths(const int64_t* pred_len, int64_t n, int32_t n_groups, int32_t equal_count,
                        int32_t* group_of, int64_t* order, int64_t* bounds, int64_t* totals);

/* Copies the hidden activations written by the last expert-FFN call on this context into
 * caller-owned device buffers: hq_out [N,F] u8, hs_out [F/128][N] f32 (group-major).  Enqueued on the
 * context's stream.  For stage-isolated checks. */
int moe_debug_copy_hidden(moe_ctx* ctx, uint8_t* hq_out, float* hs_out);

/* Measured ceilings for benchmarks (neither is part of the layer; both enqueue on the context's stream).
 * moe_probe_copy: a plain streaming device copy of `bytes` bytes (multiple of 16) from src to dst, both
 *   device pointers owned by the caller: 2*bytes / its duration is what HBM delivers to a kernel that
 *   does nothing else.
 * moe_probe_fp8_mfma: `blocks` workgroups of 8 waves run `steps` times the matrix work one wave of the grouped
 *   GEMM does per 128-wide K block (8 sub-tile products of two 32x32x64 FP8 matrix instructions, random operand
 *   bits held in registers: no LDS, no memory), scaled != 0: each product folded into its accumulator with 16
 *   fp32 multiply-adds as per-block scaling requires.  FLOP = blocks * 8 waves * steps * 16 * 2*32*32*64.
 *   sink: one float of device memory (practically never written). */
int moe_probe_copy(moe_ctx* ctx, const void* src, void* dst, int64_t bytes);
int moe_probe_fp8_mfma(moe_ctx* ctx, int32_t blocks, int32_t steps, int32_t scaled, float* sink);

/* Kernel timing for benchmarks.  While enabled, moe_expert_ffn_fp8 brackets its two
 * GEMM kernels with HIP events on the context's stream (at most 512 calls are kept
 * between reads).  moe_profile_read synchronises the stream, writes the MEAN
 * duration in milliseconds of {gate/up GEMM, down GEMM} over the recorded calls to
 * ms[0..1] and the number of calls to *calls, and clears the record. */
int moe_profile_enable(moe_ctx* ctx, int32_t on);
int moe_profile_read(moe_ctx* ctx, float* ms, int32_t* calls);

/* Library version string. */
const char* moe_version(void);

#ifdef __cplusplus
}
#endif
#endif /* MOE355_H */
