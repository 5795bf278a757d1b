/*
 * srft_kv.h -- C ABI of the fused SRFT int4 KV-cache quantizer for AMD MI355X (gfx950).
 *
 * Write path (paper Sec. 3.2 steps 1-4, Sec. 5.1 item 1, Sec. 7.1), per head-dim vector x in fp16:
 *     u = s * x                      s in {-1,+1}^d, fixed per plan                       (Eq. 1)
 *     z = pack(F u)                  F the unitary DFT, real packing of Eq. 2             (Eq. 1-2)
 *     w = lambda * z                 per-channel rescale                                  (Sec. 5.1)
 *     scale_j = max_{k in group j} |w_k| / 7,  groups = runs of g packed indices          (Sec. 7.1)
 *     q_k = rint(w_k / scale_j) in [-7, 7]   (round half to even)                         (Sec. 3.2 step 4)
 *     byte_i = (q_{2i+1} << 4) | (q_{2i} & 0xF)                                           (Sec. 3.2 (ii))
 * Read path (the inverse kernel of Sec. 7.1): unpack nibbles (4-bit two's complement), times
 * scale_j, divide by max(lambda_k, 1e-6), unpack Eq. 2, unitary inverse DFT, times s, round to fp16.
 *
 * Stored record per vector: d/2 code bytes and d/g fp32 scales, in two separate arrays.
 *
 * Conventions
 *   - "dev" pointers are device (HBM) addresses on the GPU that was current when the plan was
 *     created; "host" pointers are ordinary host memory.  The caller owns every buffer it passes;
 *     the library allocates only the plan's own constant tables and frees them in srft_plan_destroy.
 *   - Calls that take a stream enqueue on it and return without synchronising.  hip_stream is a
 *     hipStream_t passed as void* (NULL = the default stream).
 *   - Every function returns SRFT_OK (0) or a negative srft_status; nothing aborts or throws.
 *     All argument checks happen before the first HIP call.
 *   - Supported shapes: d a multiple of 32 with 32 <= d <= 256 (so 96 = 2^5 * 3 is covered; the
 *     transform is applied as a dense d x d contraction, which needs no power-of-two length);
 *     group_size g = 32 (the deployed format, the fast path), 16, or any multiple of 32 that divides d
 *     (g = d is the per-token quantizer of Sec. 3.2 step 3).
 */
#ifndef SRFT_KV_H
#define SRFT_KV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct srft_plan srft_plan_t;   /* opaque; owned by the library */

typedef enum srft_status {
    SRFT_OK             =  0,
    SRFT_ERR_NULL       = -1,   /* a required pointer is NULL */
    SRFT_ERR_BAD_D      = -2,   /* d not a multiple of 32 in [32, 256] */
    SRFT_ERR_BAD_GROUP  = -3,   /* group_size not 16 and not a multiple of 32 dividing d */
    SRFT_ERR_BAD_LAMBDA = -4,   /* a lambda is not finite, not > 0, or max/min exceeds 2^16 */
    SRFT_ERR_ALIGN      = -5,   /* a device pointer is not aligned as documented */
    SRFT_ERR_HIP        = -6,   /* a HIP call failed; see srft_last_hip_error() */
    SRFT_ERR_BAD_N      = -7,   /* n_vec < 0, count < 0 or byte count negative */
    SRFT_ERR_MISMATCH   = -8,   /* plans of one call differ in d, group_size, code width or device */
    SRFT_ERR_BAD_BITS   = -9,   /* code width not 4 or 8 */
    SRFT_ERR_BAD_TRANSFORM = -10 /* transform not one of srft_transform */
} srft_status;

/*
 * Build a plan: the constants of one (layer, K|V) pair.                 (Eq. 1; Sec. 5.1; Sec. 7.1-7.2)
 *   out          receives the plan (host pointer to a host pointer).
 *   d            head dimension.
 *   group_size   g, the number of consecutive packed indices sharing one scale.
 *   sign_seed    the sign diagonal is the splitmix64 stream started at this seed: s_n = -1 iff the
 *                top bit of the n-th output is set (the signs are fixed when the plan is made, Sec. 3.1).
 *   lambda_host  d floats > 0 on the host, or NULL for all ones.  Copied; not kept.
 * Allocates device tables on the current GPU (about 4*d*d bytes) and copies them once.
 */
int srft_plan_create(srft_plan_t** out, int d, int group_size, uint64_t sign_seed,
                     const float* lambda_host);

/*
 * The same with a chosen code width.                                   (Sec. 3.2 steps 3-4: b in {4, 8})
 *   bits = 4   the format above (srft_plan_create is this case).
 *   bits = 8   scale_j = max |w_k| / 127, q_k = rint(w_k / scale_j) in [-127, 127], one two's-complement byte per
 *              value: codes are [n_vec, d] bytes, byte k = q_k; the record is d + 4 d/g bytes.  Every entry point
 *              that takes codes then takes this layout (srft_plan_code_bytes tells the row size).
 */
int srft_plan_create_bits(srft_plan_t** out, int d, int group_size, int bits, uint64_t sign_seed,
                          const float* lambda_host);

/*
 * The same with a chosen mixing matrix: the comparator of Sec. 1 / Sec. 3.1.
 *   SRFT_TRANSFORM_DFT       the real-packed unitary DFT of Eq. 1-2 (every other create call is this case).
 *   SRFT_TRANSFORM_HADAMARD  the orthonormal Walsh-Hadamard matrix in natural order, H[k][n] = (-1)^popcount(k & n)
 *                            / sqrt(d): sign diagonal, lambda, quantizer and record are unchanged, which makes the
 *                            pipeline the SRHT the paper compares against.  d must be a power of two (else
 *                            SRFT_ERR_BAD_D).  Runs on the plain kernels (the folded forms use DFT symmetries).
 */
typedef enum srft_transform { SRFT_TRANSFORM_DFT = 0, SRFT_TRANSFORM_HADAMARD = 1 } srft_transform;
int srft_plan_create_ex(srft_plan_t** out, int d, int group_size, int bits, int transform, uint64_t sign_seed,
                        const float* lambda_host);

/* Free the plan and its device tables.  NULL is accepted.  Work already enqueued must have finished. */
int srft_plan_destroy(srft_plan_t* plan);

/*
 * Write path over n_vec vectors.                                        (Sec. 3.2 steps 1-4, Sec. 7.1)
 *   x_f16_dev   [n_vec, d] row-major IEEE fp16, 16-byte aligned.        read only
 *   codes_dev   [n_vec, d/2] bytes ([n_vec, d] for an 8-bit plan), 16-byte aligned.   written
 *   scales_dev  [n_vec, d/g] fp32, 4-byte aligned.                      written
 * n_vec == 0 is a successful no-op; n_vec > 2^33 is SRFT_ERR_BAD_N (tile indices are 32-bit).  Inputs must be finite.  A group whose abs-max / 7 is below
 * 2^-100 is stored as scale 0 with all-zero codes.
 */
int srft_kv_quantize(const srft_plan_t* plan, const void* x_f16_dev, int64_t n_vec,
                     uint8_t* codes_dev, float* scales_dev, void* hip_stream);

/*
 * Read path over n_vec vectors: the inverse of srft_kv_quantize.        (Sec. 7.1; sentence after Eq. 2)
 *   codes_dev   [n_vec, d/2] bytes ([n_vec, d] for an 8-bit plan), 16-byte aligned.   read only
 *   scales_dev  [n_vec, d/g] fp32, 4-byte aligned.                      read only
 *   out_f16_dev [n_vec, d] fp16 (round to nearest even), 16-byte aligned.  written
 * Nibble 0x8 decodes as -8 (byte 0x80 as -128 at 8 bits).
 */
int srft_kv_dequantize(const srft_plan_t* plan, const uint8_t* codes_dev, const float* scales_dev,
                       int64_t n_vec, void* out_f16_dev, void* hip_stream);

/*
 * Write path / read path over several plans in one launch.     (Sec. 7.2: one stored transform per layer and
 * K|V; a decode step appends a few vectors to every one of them, so a launch per plan is all latency.)
 *   plans, *_dev arrays, n_vec   HOST arrays of `count` entries; entry i describes one call of
 *                                srft_kv_quantize / srft_kv_dequantize (same shapes, alignment and ownership;
 *                                the *_dev entries are device addresses).  The arrays are read before the call
 *                                returns and not kept.
 *   count                        number of entries; 0 is a successful no-op.  Entries with n_vec[i] == 0 are
 *                                skipped (their pointers are not looked at).
 * All plans must share d, group_size, code width, transform and device (else SRFT_ERR_MISMATCH); signs and lambda
 * may differ.
 * Every entry is validated before anything is enqueued.  Up to 64 entries go into one kernel launch; longer
 * lists take several launches on the same stream.  Results are bit-identical to the per-plan calls.
 * Buffers of different entries must not overlap.
 */
int srft_kv_quantize_batched(const srft_plan_t* const* plans, const void* const* x_f16_dev,
                             const int64_t* n_vec, uint8_t* const* codes_dev, float* const* scales_dev,
                             int count, void* hip_stream);
int srft_kv_dequantize_batched(const srft_plan_t* const* plans, const uint8_t* const* codes_dev,
                               const float* const* scales_dev, const int64_t* n_vec,
                               void* const* out_f16_dev, int count, void* hip_stream);

/*
 * The write path with the transform done as FFT butterflies on the vector ALU, in fp32: a complex FFT of half the
 * length and a Hermitian unpack (Sec. 3.2; the form of the kernel of Sec. 7.1) in place of the matrix-core contraction
 * that srft_kv_quantize uses.  Same arguments and the same record, except that scales_dev must be 16-byte aligned; for
 * plans with d = 128 or 256, g = 32, 4-bit codes and the DFT (else SRFT_ERR_BAD_D / _BAD_GROUP / _BAD_BITS /
 * _BAD_TRANSFORM).  At d = 128 a lane holds a whole vector; at d = 256 two lanes share one and exchange
 * registers.
 * It exists so that the two forms can be timed side by side (bench.py --butterfly); it is the slower one on this
 * machine, and codes may differ from srft_kv_quantize's where a value sits at a rounding boundary.
 */
int srft_kv_quantize_butterfly(const srft_plan_t* plan, const void* x_f16_dev, int64_t n_vec,
                               uint8_t* codes_dev, float* scales_dev, void* hip_stream);

/*
 * The transform alone, quantization disabled: w = lambda * pack(F (s * x)) in fp32.  (Eq. 1-2, Sec. 5.1)
 *   x_f16_dev [n_vec, d] fp16, 16-byte aligned; w_f32_dev [n_vec, d] fp32, 16-byte aligned, written.
 * Same kernel as the write path up to the abs-max; exists so that the transform can be checked
 * on its own (orthonormality, closed forms).
 */
int srft_kv_forward_f32(const srft_plan_t* plan, const void* x_f16_dev, int64_t n_vec,
                        float* w_f32_dev, void* hip_stream);

/*
 * Scores of queries against stored keys, without reconstructing the keys.    (Sec. 1: the decode step streams the
 * stored prefix before attention reads it; Eq. 1 and the sentence after Eq. 2: the transform is orthogonal.)
 *     scores[i][t] = < q_i , k_t >,   k_t the read path's reconstruction of key t (before its fp16 rounding)
 * computed as < Q (s * q_i) / max(lambda, 1e-6) , code_t * scale_t >: only the record of the keys is read.
 *   q_f16_dev      [n_q, d] fp16, 16-byte aligned, 1 <= n_q <= 32 (e.g. the query heads sharing one KV head).
 *   codes_dev      [n_keys, d/2] bytes, 16-byte aligned;  scales_dev [n_keys, d/g] fp32: the plan's record.
 *   scores_dev     [n_q, n_keys] fp32, row-major, written.
 *   workspace_dev  srft_scores_workspace_bytes(plan) bytes of device memory (about 1 MiB), 16-byte aligned,
 *                  overwritten; two calls that may run at the same time need a workspace each.
 * For plans with d a multiple of 64, 4-bit codes and g >= 32 (else SRFT_ERR_BAD_D / _BAD_BITS / _BAD_GROUP).
 * Enqueues two kernels on the stream: transform of the queries into the scan's operand layout, then the scan.
 */
int64_t srft_scores_workspace_bytes(const srft_plan_t* plan);
int srft_kv_scores(const srft_plan_t* plan, const void* q_f16_dev, int n_q, const uint8_t* codes_dev,
                   const float* scales_dev, int64_t n_keys, float* scores_dev, void* workspace_dev,
                   void* hip_stream);

/*
 * Weighted sums of stored values, without reconstructing the values: the other half of attention over the stored
 * cache.    (Sec. 1 and Sec. 7.2: attention reads the prefix the cache holds; Eq. 1-2: the transform is linear.)
 *     out[i] = sum_t weights[i][t] * v_t,   v_t the read path's reconstruction of value t (before its fp16 rounding)
 * computed as one inverse transform per query of  sum_t weights[i][t] * code_t * scale_t : only the record is read.
 *   weights_f32_dev [n_q, n_keys] fp32 row-major, 4-byte aligned, 1 <= n_q <= 32 (e.g. softmax of srft_kv_scores).
 *   codes_dev       [n_keys, d/2] bytes, 16-byte aligned;  scales_dev [n_keys, d/g] fp32: the plan's record.
 *   out_f32_dev     [n_q, d] fp32, written.
 *   workspace_dev   srft_attend_workspace_bytes(plan) bytes of device memory (about 34 MiB at d = 128), 16-byte aligned,
 *                   overwritten; calls that may run at the same time need a workspace each.
 * n_keys >= 1.  For plans with d a multiple of 64, 4-bit codes and g >= 32 (else SRFT_ERR_BAD_D / _BAD_BITS /
 * _BAD_GROUP).  Enqueues three kernels: partial sums per workgroup (fp32, on the matrix cores), their sum in a fixed
 * order (two levels), and the inverse transform.  The result does not depend on timing.
 */
int64_t srft_attend_workspace_bytes(const srft_plan_t* plan);
int srft_kv_attend(const srft_plan_t* plan, const float* weights_f32_dev, int n_q, const uint8_t* codes_dev,
                   const float* scales_dev, int64_t n_keys, float* out_f32_dev, void* workspace_dev,
                   void* hip_stream);

/*
 * One decode step of attention over a stored cache: out = softmax(softmax_scale * q K^T) V with K and V read from
 * their records (plan_k, plan_v: same d, own signs and lambda each).    (Sec. 1; Sec. 7.2)
 * On one stream: srft_kv_scores, whose scan also keeps the maximum of softmax_scale * score per row; then the weighted
 * sums of srft_kv_attend, whose kernel forms the weights exp(softmax_scale * score - maximum) from the raw scores as it
 * loads them, carries their sums along and divides by them at the end (the scores are written once and read once; the
 * row softmax has no pass of its own).  q_f16_dev [n_q, d] fp16 (16-byte aligned),
 * out_f32_dev [n_q, d] fp32; workspace_dev: srft_decode_attention_workspace_bytes(plan_k, plan_v, n_q, n_keys) bytes,
 * 256-byte aligned (it holds the n_q x n_keys scores).  Shapes and limits as for the two calls it is made of.
 */
int64_t srft_decode_attention_workspace_bytes(const srft_plan_t* plan_k, const srft_plan_t* plan_v, int n_q,
                                              int64_t n_keys);
int srft_kv_decode_attention(const srft_plan_t* plan_k, const srft_plan_t* plan_v, const void* q_f16_dev, int n_q,
                             const uint8_t* k_codes_dev, const float* k_scales_dev, const uint8_t* v_codes_dev,
                             const float* v_scales_dev, int64_t n_keys, float softmax_scale, float* out_f32_dev,
                             void* workspace_dev, void* hip_stream);

/*
 * srft_kv_scores for callers that cannot allocate device memory or pass a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, checks and results as
 * srft_kv_scores without workspace_dev: the workspace is a static device array inside the library (1 MiB + 32 KiB
 * per GPU, held until the process ends; its address is looked up when the plan is created).  Calls no hipMalloc,
 * hipFree or other allocating routine.  A plan whose srft_scores_workspace_bytes exceeds that array is refused with
 * SRFT_ERR_BAD_N (no plan this library creates does).  Every call on one GPU uses the same array: calls that may
 * overlap on one GPU (different streams, or threads) race -- order them, or use srft_kv_scores with a workspace each.
 */
int srft_kv_scores_static(const srft_plan_t* plan, const void* q_f16_dev, int n_q, const uint8_t* codes_dev,
                          const float* scales_dev, int64_t n_keys, float* scores_dev, void* hip_stream);

/*
 * Cache manager: int4 store + fp16 residual window + dequantized-prefix cache.   (Sec. 7.2: the cache class,
 * items (i)-(iv), and its paragraph on the residual window: 16 tokens.)
 *
 * One cache holds n_plans (layer, K|V) plans of one shape, each with n_seq sequences (batch x kv_heads) that grow
 * in lock-step.  All device buffers belong to the caller, one per plan, in a paged layout whose page is the
 * residual window of R tokens:
 *     codes_dev[p]     [capacity/R][n_seq][R][d/2]  bytes      the int4 store ([..][d] at 8 bits)  (16-byte aligned)
 *     scales_dev[p]    [capacity/R][n_seq][R][d/g]  fp32                                  (4-byte aligned)
 *     view_f16_dev[p]  [capacity/R][n_seq][R][d]    fp16       what attention reads       (16-byte aligned)
 * Token j of sequence q is at page j / R, slot j % R.  In the view, tokens below srft_cache_quantized_tokens() hold
 * what the store decodes to (the dequantized prefix, written once when their page is flushed, never again: an
 * update costs O(1) in the prefix length); tokens from there up to srft_cache_tokens() are the residual window,
 * exact fp16 copies of what was appended.  The store holds the quantized tokens only.
 *
 * srft_cache_create   records the geometry and the pointers (host arrays of n_plans entries, copied); no HIP
 *                     calls.  capacity_tokens must be a positive multiple of residual_tokens (>= 1).
 * srft_cache_append   new_f16_dev: host array of n_plans device pointers, each [n_seq, t, d] fp16 (16-byte
 *                     aligned): t new tokens per sequence.  Enqueues: a copy of the tokens into the view; then, if
 *                     one or more pages became full, ONE batched quantize of those pages over all plans and one
 *                     batched dequantize of them back into the view.  Exceeding the capacity is SRFT_ERR_BAD_N
 *                     (nothing is enqueued).  The result does not depend on how the tokens are split into calls.
 * srft_cache_rebuild_view  dequantizes the whole store into the view again (for a caller that dropped or
 *                     overwrote the view); O(prefix).  The window part of the view is not touched.
 * Calls on one cache must be made from one thread at a time and enqueued on one stream (or ordered by the caller).
 */
typedef struct srft_cache srft_cache_t;
int srft_cache_create(srft_cache_t** out, const srft_plan_t* const* plans, int n_plans, int n_seq,
                      int64_t capacity_tokens, int residual_tokens, uint8_t* const* codes_dev,
                      float* const* scales_dev, void* const* view_f16_dev);
int srft_cache_destroy(srft_cache_t* cache);     /* NULL is accepted; the buffers stay the caller's */
int srft_cache_append(srft_cache_t* cache, const void* const* new_f16_dev, int t, void* hip_stream);
int srft_cache_rebuild_view(srft_cache_t* cache, void* hip_stream);
int64_t srft_cache_tokens(const srft_cache_t* cache);              /* tokens per sequence, or a negative status */
int64_t srft_cache_quantized_tokens(const srft_cache_t* cache);    /* of which in the int4 store */

/*
 * Calibration statistic for lambda: per-channel abs-max of the transform output over a batch.  (Sec. 7.1: lambda is
 * the reciprocal of that maximum; Sec. 7.2: one static calibration over whole windows.)
 *   x_f16_dev  [n_vec, d] fp16, 16-byte aligned.                                         read only
 *   amax_dev   d fp32 on the device, 4-byte aligned, all >= 0: a RUNNING maximum.  On return amax_dev[k] =
 *              max(old amax_dev[k], max over the n_vec vectors of |w_k|), w = lambda * pack(F (s * x)) with the
 *              plan's lambda.  Zero it before the first batch; call once per batch of the calibration window.
 *              With a plan created with lambda_host = NULL, w is the plain SRFT output.
 * Updated with atomic maxima: calls on the same amax_dev may overlap.
 */
int srft_kv_channel_absmax(const srft_plan_t* plan, const void* x_f16_dev, int64_t n_vec, float* amax_dev,
                           void* hip_stream);

/*
 * lambda from that statistic, on the host: lambda_k = 1 / amax_k (Sec. 7.1).  Two cases the paper does not cover:
 * a channel whose amax is below 2^-16 of the largest is treated as if it were at that floor (srft_plan_create
 * accepts max/min lambda up to 2^16), and an all-zero statistic gives lambda = 1.  amax_host: d finite floats >= 0
 * (else SRFT_ERR_BAD_LAMBDA); lambda_host: d floats, written.  No HIP calls.
 */
int srft_lambda_from_absmax(const float* amax_host, int d, float* lambda_host);

/* Plan introspection (host side, no HIP calls). */
int srft_plan_d(const srft_plan_t* plan);             /* d, or a negative status */
int srft_plan_group_size(const srft_plan_t* plan);    /* g */
int srft_plan_groups(const srft_plan_t* plan);        /* d / g: scales per vector */
int srft_plan_code_bytes(const srft_plan_t* plan);    /* code bytes per vector: d / 2 at 4 bits, d at 8 */
int srft_plan_bits(const srft_plan_t* plan);          /* 4 or 8 */
/* Which form of the transform the plan's launches run: path 0 = write, 1 = read; returns 0 = the whole matrix
 * (plain form), 1 = folded once, 2 = folded twice (the factorisations that the symmetries of Eq. 1-2 allow; the
 * record is the same in every form), or SRFT_ERR_NULL / SRFT_ERR_BAD_N. */
int srft_plan_form(const srft_plan_t* plan, int path);
int srft_plan_get_signs(const srft_plan_t* plan, int8_t* out_host /* d entries, each -1 or +1 */);

/*
 * Launch shape: both kernels are persistent (a fixed grid loops over tiles of 32 vectors).
 * max_workgroups > 0 caps the grid of this plan's launches (to leave compute units to other streams, or to
 * check that results do not depend on the grid); 0 restores the default (compute units x resident workgroups
 * per unit).  Results are bit-identical for every grid size.  The library reads no environment variables.
 */
int srft_plan_set_max_workgroups(srft_plan_t* plan, int max_workgroups);

const char* srft_status_string(int status);
int srft_last_hip_error(void);    /* the hipError_t of the most recent SRFT_ERR_HIP on this thread */

#ifdef __cplusplus
}
#endif
#endif /* SRFT_KV_H */
