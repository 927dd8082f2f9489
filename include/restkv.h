/*
 * restkv.h -- C ABI of the ReST-KV eviction path for AMD MI355X (gfx950).
 *
 * One call sequence compresses the KV cache of ONE transformer layer at prefill
 * time (the paper evicts once, after prefill; App. B):
 *
 *     restkv_prepare_wo   (once per layer's weights, not per request)
 *     restkv_score   ->  restkv_smooth  ->  restkv_select  ->  restkv_compact
 *
 * Notation (0-indexed): Hq query heads, Hkv KV heads, G = Hq/Hkv, d head_dim,
 * L cached tokens, W observation-window queries (the last W positions),
 * P = L - W evictable prefix tokens, B per-KV-head budget (the W window tokens
 * are always kept and count towards B).
 *
 * Pointers: every pointer argument except the parameter block is a DEVICE
 * pointer owned by the caller; the parameter block is a HOST pointer that is
 * read before the call returns.  The library allocates nothing, frees nothing
 * and never synchronises: each call validates its arguments on the host,
 * enqueues kernels on `stream` (a hipStream_t; NULL = the default stream) and
 * returns.  Scratch memory comes from the caller as `workspace` of at least
 * restkv_workspace_bytes() bytes, 256-byte aligned; its contents are undefined
 * between calls and calls that share a workspace must be ordered on one stream.
 *
 * Errors: every entry point returns RESTKV_OK (0) or a negative code; nothing is
 * enqueued when an error is returned, except RESTKV_EHIP, which reports a launch
 * failure of the HIP runtime and may leave earlier kernels of that call queued.
 * No entry point throws, aborts or prints.
 *
 * Design readings that the paper leaves open and no independent check can pin
 * ("parity unpinned"): the mean over the G query heads of a KV head (score), and
 * the way the fixed kernel size k widens under the adaptive window (smooth).
 */
#ifndef RESTKV_H_
#define RESTKV_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define RESTKV_OK            0
#define RESTKV_EINVAL       (-1)  /* null pointer, inconsistent shape, budget outside (W, L], ... */
#define RESTKV_EUNSUPPORTED (-2)  /* head_dim not in {64,128}, unknown dtype, G*W too large ...   */
#define RESTKV_EWORKSPACE   (-3)  /* workspace missing, misaligned or too small                   */
#define RESTKV_EHIP         (-4)  /* the HIP runtime refused a launch                             */

#define RESTKV_F32  0   /* q, k, v and the compacted cache are IEEE binary32 */
#define RESTKV_BF16 1   /* ... are bfloat16                                   */

/*
 * Ablation variants (Sec. 4, ablation table; App. on the ablation study), selected through
 * restkv_params.variant.  0 is the method itself.
 *   indicator (restkv_score):  RESTKV_IND_ATTENTION   A[n], the attention weight alone
 *                              RESTKV_IND_VALUE_NORM  A[n] * ||v_n||_2  (gram is ignored by both)
 *   group reduction:           RESTKV_GROUP_MAX       largest indicator among the G query heads
 *                                                     of a KV head instead of their mean
 *   temporal (restkv_smooth):  RESTKV_TEMPORAL_MEAN   plain mean over the W window queries
 *                              RESTKV_TEMPORAL_INV_EMA the EMA recursion run from the newest
 *                                                     query to the oldest (oldest weighs alpha)
 *   spatial pooling:           RESTKV_POOL_MAX        maximum over the window instead of the mean
 * "No temporal smoothing" is ema_alpha = 1, "no spatial smoothing" base_window = 1 with
 * adaptive = 0, fixed average pooling adaptive = 0.  restkv_score_smooth runs the two separate
 * calls for any variant other than 0.
 */
#define RESTKV_IND_RECONSTRUCTION 0
#define RESTKV_IND_ATTENTION      1
#define RESTKV_IND_VALUE_NORM     2
#define RESTKV_GROUP_MAX          (1 << 2)
#define RESTKV_TEMPORAL_MEAN      (1 << 4)
#define RESTKV_TEMPORAL_INV_EMA   (2 << 4)
#define RESTKV_POOL_MAX           (1 << 6)

typedef void* restkv_stream_t;    /* a hipStream_t */

/*
 * Problem statement of one layer (Sec. 3.2, Definition 3.1: the layer's cache
 * <K_T, V_T>, the recent queries, the head's output projection and the budget B).
 */
typedef struct restkv_params {
  int32_t n_q_heads;     /* Hq                                                         */
  int32_t n_kv_heads;    /* Hkv, divides Hq                                            */
  int32_t head_dim;      /* d: 64 or 128                                               */
  int32_t seq_len;       /* L                                                          */
  int32_t window;        /* W = S_w, 1 <= W < L                                        */
  int32_t budget;        /* B, W < B <= L                                              */
  int32_t dtype;         /* RESTKV_F32 or RESTKV_BF16                                  */
  int32_t causal;        /* 1: window query i sees keys 0 .. L-W+i ; 0: all L keys     */
  float   scale;         /* logit scale; 0 selects 1/sqrt(d) (Eq. softmax)             */
  float   ema_alpha;     /* alpha of the EMA recursion: weight of the newest query     */
  int32_t base_window;   /* k: odd >= 1, the fixed kernel size of App. B               */
  int32_t adaptive;      /* 1: W_s and gamma_shift from D_front/D_rear ; 0: W_s=k, 0   */
  float   beta;          /* scaling factor of the adaptive window (> L / 2^30 when adaptive) */
  int32_t variant;       /* 0: the method; else a sum of RESTKV_IND_*, RESTKV_GROUP_MAX,
                            RESTKV_TEMPORAL_*, RESTKV_POOL_MAX (ablation variants, see below) */
  int64_t q_stride_h;    /* elements between query heads  (0: W*d)                     */
  int64_t q_stride_t;    /* elements between window queries (0: d)                     */
  int64_t kv_stride_h;   /* elements between KV heads     (0: L*d)                     */
  int64_t kv_stride_t;   /* elements between tokens       (0: d); rows are d-contiguous*/
  int64_t ld_score;      /* row stride (floats) of score / ema / final (0: P; >= P)    */
} restkv_params;

/* Bytes of scratch the four calls below need for these parameters (0 if invalid). */
size_t restkv_workspace_bytes(const restkv_params* p);

/*
 * Gram matrices of the per-head output projection (Eq. mha: MHA = z W_O, with W_O
 * the head's rows of the layer's projection).  The indicator only needs
 * ||x W_O^h||_2, which depends on M_h = W_O^h W_O^hT alone.
 *   w_o   [Hq*d, d_model] float32, row-major, "z @ W_O" orientation: rows
 *         h*d .. (h+1)*d-1 belong to query head h (a framework weight stored
 *         [out,in] must be passed transposed).
 *   gram  [Hq, d, d] float32 out; symmetric by construction (restkv_score relies
 *         on M_h[i][j] == M_h[j][i] and reads the upper triangle only).
 * Weight-only: run once per layer, not per request.  Accumulates in float64.
 */
int restkv_prepare_wo(const restkv_params* p, const float* w_o, int64_t d_model,
                      float* gram, restkv_stream_t stream);

/*
 * Layer-wise reconstruction indicator (Sec. 3.2, Eq. rec_ei; derivation App. A):
 * for every query head h, window query i and prefix token n
 *     I[h,i,n] = A[n] / (1 - A[n]) * || (z_{h,i} - v_n) W_O^h ||_2 ,
 * A = softmax(scale * q_{h,i} K^T) over the visible keys (Eq. softmax), z = A V.
 * The token holding the largest weight of a query is evaluated by the equivalent
 * leave-one-out form (Eq. ori with Eq. relation), which stays finite as A -> 1.
 * Output is the mean over the G query heads of each KV head:
 *     score[g,i,n] = (1/G) sum_{h in g} I[h,i,n]          [Hkv, W, ld_score] float32
 *   q     [Hq, W, d]  (strides q_stride_*),  k, v  [Hkv, L, d] (strides kv_stride_*)
 *   gram  [Hq, d, d] from restkv_prepare_wo (any symmetric matrices), or NULL for
 *         W_O W_O^T = identity.
 * Columns n >= P of `score` are not written.
 * The squared distance is evaluated as z M z^T - 2 (z M) v_n^T + v_n M v_n^T in FP32; when the
 * three terms cancel (v_n W_O within a few 1e-3 of z W_O, relative to their norms) the rounding
 * residue of that sum enters by its magnitude (matrix-core kernels) or clamped at zero (FP32
 * kernels): the result then is a small non-negative number where the exact one is near zero.
 */
int restkv_score(const restkv_params* p, const void* q, const void* k, const void* v,
                 const float* gram, float* score, void* workspace, size_t workspace_bytes,
                 restkv_stream_t stream);

/*
 * restkv_score with the attention statistics of the window queries taken from the caller's
 * own attention kernel instead of a pass over the cache (App. B: at prefill the statistics the
 * method needs are already there; Sec. 5: only the attention output of a small query window
 * is needed).  The usual pair a fused attention kernel returns:
 *   attn_out [Hq, W, d] float32, contiguous: softmax(scale q K^T) V of the W window queries over
 *            exactly the keys restkv_score would let them see (query i: keys 0 .. L-W+i when
 *            causal), same scale;
 *   lse      [Hq, W] float32: natural logarithm of each row's softmax denominator.
 * Everything else as restkv_score; the attention pass and its merge are replaced by a pass
 * over [Hq, W, d].  Without the unnormalised sums of a pass of its own the library cannot
 * evaluate a dominant key by the leave-one-out form: a key that holds more than about 0.9 of a
 * query's attention is scored through Eq. rec_ei in FP32 and loses accuracy as 1 - A
 * vanishes (relative error about 4e-6 / (1 - A)^2); every other key meets the same bound as
 * restkv_score.
 */
int restkv_score_from_attention(const restkv_params* p, const void* q, const void* k, const void* v,
                                const float* gram, const float* attn_out, const float* lse, float* score,
                                void* workspace, size_t workspace_bytes, restkv_stream_t stream);

/*
 * Spatial-temporal smoothing (Sec. 3.3).
 *   ema[g,n]   = EMA over the W window queries of score[g,:,n] (newest weighs alpha)
 *   D_front/D_rear = mean index of the per-query top-min(B,P) tokens of the raw
 *                score, over the first floor(W/2) / the remaining queries
 *   W_s   = k + 2 floor(|D_rear - D_front| / beta)
 *   gamma = floor((D_front - D_rear)/beta) (+1 unless D_front - D_rear > 0)
 *   final[g,n] = (1/W_s) sum_{j=-floor(W_s/2)+gamma}^{floor(W_s/2)+gamma} ema[g,n+j]
 *                (Eq. final_ei; terms outside [0,P) are zero)
 * adaptive = 0 or W = 1 gives W_s = k, gamma = 0.
 *   score [Hkv, W, ld] in;  ema [Hkv, ld] out (may be NULL: kept in workspace);
 *   final [Hkv, ld] out;  aws_info [Hkv, 2] int32 out = {W_s, gamma} (may be NULL);
 *   aws_d [Hkv, 2] float64 out = {D_front, D_rear} (may be NULL).
 */
int restkv_smooth(const restkv_params* p, const float* score, float* ema, float* final_score,
                  int32_t* aws_info, double* aws_d, void* workspace, size_t workspace_bytes,
                  restkv_stream_t stream);

/*
 * restkv_score followed by restkv_smooth as ONE call, with the same outputs (score
 * included).  Where the shape allows it (bf16 inputs on the matrix-core path, G padded
 * to a power of two in {4, 8}, G * W <= 256, adaptive window on, P >= 32768) the score
 * pass itself accumulates the EMA (as the weighted sum that the recursion of Sec. 3.3
 * unrolls to) and the per-query top-B statistics of the adaptive window, from brackets
 * that a short pass over 8192 sampled keys provides, so that the raw score is written
 * once and not read again; otherwise the two calls run one after the other.  A query
 * whose bracket fails is redone exactly from `score`.  Workspace as reported by
 * restkv_workspace_bytes (it covers this call).
 */
int restkv_score_smooth(const restkv_params* p, const void* q, const void* k, const void* v,
                        const float* gram, float* score, float* ema, float* final_score,
                        int32_t* aws_info, double* aws_d, void* workspace, size_t workspace_bytes,
                        restkv_stream_t stream);

/*
 * Per-head selection (Sec. 3.3, Eq. topk): the B - W prefix tokens with the
 * largest final[g, 0..P) (equal values: lower index wins), written in ascending
 * position order and followed by the window tokens P .. L-1.
 *   final [Hkv, ld] in;  idx [Hkv, B] int32 out.
 * Uses the workspace (samples, per-chunk counters, candidates); like every call
 * here it allocates nothing and returns RESTKV_EWORKSPACE if the workspace is
 * NULL, misaligned or smaller than restkv_workspace_bytes().
 */
int restkv_select(const restkv_params* p, const float* final_score, int32_t* idx,
                  void* workspace, size_t workspace_bytes, restkv_stream_t stream);

/*
 * Non-uniform budgets (App. C of the paper pairs the indicator with layer-wise and head-wise
 * allocation).  A layer-wise budget is just `budget` of that layer's parameter block; the
 * two calls below take a budget per KV head instead:
 *   head_budget [Hkv] int32 on the device; entry g is used as min(max(b, W + 1), budget), so
 *   `budget` of the parameter block is the largest budget and stays the row stride of idx,
 *   k_out and v_out.
 * restkv_smooth_b uses min(head_budget[g], P) in place of min(B, P) for the per-query top-B
 * statistics of head g; restkv_select_b keeps head_budget[g] - W prefix tokens of head g,
 * appends the W window tokens, and fills idx[g, head_budget[g] .. B) with -1, which
 * restkv_compact turns into zero rows.  Everything else as restkv_smooth / restkv_select.
 */
int restkv_smooth_b(const restkv_params* p, const float* score, const int32_t* head_budget, float* ema,
                    float* final_score, int32_t* aws_info, double* aws_d, void* workspace,
                    size_t workspace_bytes, restkv_stream_t stream);
int restkv_select_b(const restkv_params* p, const float* final_score, const int32_t* head_budget,
                    int32_t* idx, void* workspace, size_t workspace_bytes, restkv_stream_t stream);

/*
 * restkv_select for callers that cannot allocate device memory or hand over a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same result as
 * restkv_select (same kernels); the scratch is an array inside the library's device image, one
 * copy per GPU that lives until the process ends (restkv_select_static_capacity() bytes, 4 MiB).
 * Returns RESTKV_EWORKSPACE, with nothing enqueued, when the shape needs more than that: about
 * 0.5 KiB per 4096 prefix positions and KV head (240 KV heads fit at 128k tokens).  The call
 * allocates nothing and frees nothing (the first call on a GPU looks up the array's address
 * once).  Every call on a GPU uses that GPU's one array: calls that overlap in time on one GPU
 * (different streams or host threads) race; calls ordered on one stream are safe, and each call
 * clears what it needs cleared itself.
 */
int restkv_select_static(const restkv_params* p, const float* final_score, int32_t* idx,
                         restkv_stream_t stream);
size_t restkv_select_static_capacity(void);

/*
 * Gather of the kept rows (Eq. topk): k_out[g,j,:] = k[g, idx[g,j], :], same for v.
 *   idx [Hkv, B] int32 in, entries in [0, L) (an entry outside is written as zeros);
 *   k_out, v_out [Hkv, B, d] out, contiguous, dtype of the inputs.
 */
int restkv_compact(const restkv_params* p, const void* k, const void* v, const int32_t* idx,
                   void* k_out, void* v_out, restkv_stream_t stream);

/*
 * Profiling aid (not part of the method): every kernel launch of a selected stage
 * is bracketed by two HIP events on the caller's stream.  stage_mask: bit s selects
 * stage s (see restkv_stage_name), -1 selects all, 0 turns timing off.  A bracket
 * costs a few microseconds of idle GPU, so timing all stages slows a layer by
 * about a tenth; timing one stage is nearly free.
 * restkv_timing_read() blocks until those events have completed, adds the elapsed
 * milliseconds and the number of launches per stage into ms[] / launches[] (host
 * arrays of n_stages >= RESTKV_N_STAGES entries) and forgets them.  Disabled by
 * default; enabling or disabling also forgets pending records.  Not thread-safe
 * against concurrent launches on other host threads beyond a mutex on the records.
 */
#define RESTKV_N_STAGES 10
int restkv_timing_enable(int stage_mask);
int restkv_timing_read(double* ms, int64_t* launches, int n_stages);
const char* restkv_stage_name(int stage);   /* "gram", "attn_partial", ... */

/*
 * Measurement aid, no part of the eviction path: one plain streaming kernel (16-byte loads
 * and stores, reads and writes interleaved step by step, no arithmetic beyond an XOR) that reads
 * read_bytes from src and writes write_bytes to dst, so that a kernel's HBM rate can be set
 * against what the part delivers for the same byte mix.
 * src, dst: DEVICE pointers (16-byte aligned), caller-owned, must not overlap; read_bytes and
 * write_bytes multiples of 16; either may be 0.  Result: 32-bit word i of dst = i XOR (all
 * words the writing thread read in earlier steps), i.e. dst[i] = i for an all-zero source.
 * Asynchronous on `stream`; RESTKV_EINVAL for null, misaligned or odd-sized arguments.
 */
int restkv_stream_reference(const void* src, size_t read_bytes, void* dst, size_t write_bytes,
                            void* stream);

/*
 * Debug aid: with on != 0 restkv_score runs bf16 inputs through the FP32 vector kernels
 * instead of the MFMA kernels (same stages, every product in FP32).  Process-wide.
 */
int restkv_debug_force_fp32(int on);

/* Static description of an error code. */
const char* restkv_strerror(int code);

/* Library version (major*10000 + minor*100 + patch). */
int restkv_version(void);

#ifdef __cplusplus
}
#endif
#endif /* RESTKV_H_ */
