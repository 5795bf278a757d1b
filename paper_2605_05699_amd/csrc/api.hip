// api.hip -- the C entry points of the write path, the read path and what sits around them: argument checks
// (all before the first HIP call), grid sizing, launches.
#include <algorithm>
#include <atomic>
#include <cmath>

#include "common.h"

namespace {

int launch_quantize(const srft_plan* p, const void* x, long long n, uint8_t* codes, float* scales, float* wout,
                    int out, hipStream_t st) {
    const long long n_tiles = (n + kTileVecs - 1) / kTileVecs;
    long long grid = p->max_wgs > 0 ? p->max_wgs : p->grid_q;
    if (grid > n_tiles) grid = n_tiles;
    int threads = 0;
    const quantize_kernel_t kernel = srft_plan_quantize_kernel(p, out, &threads);
    if (!kernel) return SRFT_ERR_BAD_D;
    const bool fold4 = p->fold4_q && out == kOutCodes, fold = p->fold_q && (out == kOutCodes || out == kOutAmax);
    // the twice-folded form carries the matrix scaling inside its per-channel factors
    const float unscale = fold4 ? 1.0f : p->unscale_w;
    hipLaunchKernelGGL(kernel, dim3((unsigned)grid), dim3(threads), 0, st,
                       fold4 ? p->wfold4 : fold ? p->wfold : p->wfrag, (const uint4*)x, n, (uint2*)codes, scales,
                       (float4*)wout, unscale, unscale / (p->bits == 8 ? 127.0f : 7.0f), p->gw);
    SRFT_HIP(hipGetLastError());
    return SRFT_OK;
}

int launch_dequantize(const srft_plan* p, const uint8_t* codes, const float* scales, long long n, void* out,
                      hipStream_t st) {
    const long long n_tiles = (n + kTileVecs - 1) / kTileVecs;
    long long grid = p->max_wgs > 0 ? p->max_wgs : p->grid_dq;
    if (grid > n_tiles) grid = n_tiles;
    int threads = 0;
    const dequantize_kernel_t kernel = srft_plan_dequantize_kernel(p, &threads);
    if (!kernel) return SRFT_ERR_BAD_D;
    hipLaunchKernelGGL(kernel, dim3((unsigned)grid), dim3(threads), 0, st, srft_plan_read_table(p),
                       (const uint2*)codes, scales, n, (uint4*)out, srft_plan_read_unscale(p), p->gw);
    SRFT_HIP(hipGetLastError());
    return SRFT_OK;
}

// One batched launch: the segment table is complete except for first_block, which is laid out here.
// Every segment gets at least one workgroup and at most one per tile; when the tiles of all segments
// exceed the persistent grid, workgroups are shared out in proportion to the tiles.
int launch_batched(const srft_plan* p, srft_batch_args& a, bool write_path, hipStream_t st) {
    long long budget = p->max_wgs > 0 ? p->max_wgs : (write_path ? p->grid_q : p->grid_dq);
    long long total_tiles = 0;
    for (int i = 0; i < a.count; ++i) total_tiles += (a.n_vec[i] + kTileVecs - 1) / kTileVecs;
    int next = 0;
    for (int i = 0; i < a.count; ++i) {
        const long long tiles = (a.n_vec[i] + kTileVecs - 1) / kTileVecs;
        long long blocks = total_tiles <= budget ? tiles : tiles * budget / total_tiles;
        if (blocks < 1) blocks = 1;
        if (blocks > tiles) blocks = tiles;
        a.first_block[i] = next;
        next += (int)blocks;
    }
    a.first_block[a.count] = next;
    batched_kernel_t kernel = nullptr;
    int threads = 0;
    if (write_path) {
        if (p->fold4_q) {
            kernel = srft_pick_quantize_fold4_batched(p->bits);
            threads = 256;
        } else if (p->fold_q) {
            kernel = srft_pick_quantize_fold_batched(p->d, p->bits, p->gm == kGroupWide);
            threads = p->d;
        } else {
            kernel = p->bits == 8 ? srft_pick_quantize_plain_batched_b8(p->d, p->slabs_q, p->gm)
                                  : srft_pick_quantize_plain_batched_b4(p->d, p->slabs_q, p->gm);
            threads = 2 * p->d / p->slabs_q;
        }
    } else if (p->fold4_dq) {
        kernel = srft_pick_dequantize_fold4_batched(p->d, p->bits);
        threads = p->d;
    } else {
        kernel = p->bits == 8 ? srft_pick_dequantize_batched_b8(p->d, p->slabs_dq, p->gm, p->fold_dq)
                              : srft_pick_dequantize_batched_b4(p->d, p->slabs_dq, p->gm, p->fold_dq);
        threads = 2 * p->d / p->slabs_dq;
    }
    if (!kernel) return SRFT_ERR_BAD_D;
    hipLaunchKernelGGL(kernel, dim3((unsigned)next), dim3(threads), 0, st, a, p->gw);
    SRFT_HIP(hipGetLastError());
    return SRFT_OK;
}

}  // namespace

// Shared body of the two batched entry points.  in1 / out1 are NULL arrays where the path has no such buffer.
int srft_run_batched(const srft_plan_t* const* plans, const void* const* in0, const void* const* in1,
                     void* const* out0, void* const* out1, const int64_t* n_vec, int count, bool write_path,
                     hipStream_t st) {
    if (count < 0) return SRFT_ERR_BAD_N;
    if (count == 0) return SRFT_OK;
    if (!plans || !in0 || !out0 || !n_vec || (write_path ? !out1 : !in1)) return SRFT_ERR_NULL;
    // validate everything before the first launch: a bad segment must not leave half a batch enqueued
    for (int i = 0; i < count; ++i) {
        if (!plans[i]) return SRFT_ERR_NULL;
        if (!srft_plans_compatible(plans[i], plans[0])) return SRFT_ERR_MISMATCH;
        if (n_vec[i] < 0 || n_vec[i] > kMaxVectors) return SRFT_ERR_BAD_N;
        if (n_vec[i] == 0) continue;
        const void* small = write_path ? (const void*)out1[i] : in1[i];       // the scales
        if (!in0[i] || !out0[i] || !small) return SRFT_ERR_NULL;
        if (!srft_aligned(in0[i], 16) || !srft_aligned(out0[i], 16) || !srft_aligned(small, 4)) return SRFT_ERR_ALIGN;
    }
    srft_batch_args a;
    a.count = 0;
    for (int i = 0; i <= count; ++i) {
        if (i < count && n_vec[i] > 0) {
            const int k = a.count++;
            a.frag[k] = write_path ? (plans[i]->fold4_q ? plans[i]->wfold4 : plans[i]->fold_q ? plans[i]->wfold : plans[i]->wfrag)
                                   : srft_plan_read_table(plans[i]);
            a.in0[k] = in0[i];
            a.in1[k] = write_path ? nullptr : in1[i];
            a.out0[k] = out0[i];
            a.out1[k] = write_path ? out1[i] : nullptr;
            a.n_vec[k] = n_vec[i];
            a.unscale[k] = write_path ? plans[i]->unscale_w : srft_plan_read_unscale(plans[i]);
        }
        if (a.count == kMaxBatch || (i == count && a.count > 0)) {
            const int rc = launch_batched(plans[0], a, write_path, st);
            if (rc != SRFT_OK) return rc;
            a.count = 0;
        }
    }
    return SRFT_OK;
}

// ---------------------------------------------------------------------------------------------------------
// Workspace of srft_kv_scores_static: a file-scope device array, so that the entry point allocates nothing.
// Every GPU the library runs on holds its own copy of the array at its own address until the process ends.
// In host code the array's name is only a stand-in for the symbol: the device address comes from
// hipGetSymbolAddress, once per device with that device current, and only that address is ever handed to a
// kernel.
// ---------------------------------------------------------------------------------------------------------
constexpr size_t kScoresQfragBytesMax = (size_t)(kMaxD / 16) * 2 * 64 * 16;                    // 32 KiB at d = 256
constexpr size_t kScoresScratchBytes = kScoresQfragBytesMax + (size_t)kMaxScoreWorkgroups * 64 * 4;   // + 1 MiB
static __device__ __align__(256) unsigned char scratch[kScoresScratchBytes];

constexpr int kMaxDevices = 64;
static std::atomic<void*> g_scratch_ptr[kMaxDevices];

// The address of `scratch` on `device`, which must be the current device; resolved on the first call per device.
int srft_scores_scratch_prepare(int device) {
    if (device < 0 || device >= kMaxDevices) return SRFT_ERR_HIP;
    if (g_scratch_ptr[device].load(std::memory_order_acquire)) return SRFT_OK;
    void* ptr = nullptr;
    SRFT_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
    if (!ptr) return srft_hip_fail(hipErrorInvalidSymbol);
    g_scratch_ptr[device].store(ptr, std::memory_order_release);
    return SRFT_OK;
}

extern "C" {

int srft_kv_quantize(const srft_plan_t* plan, const void* x_f16_dev, int64_t n_vec, uint8_t* codes_dev,
                     float* scales_dev, void* hip_stream) {
    if (!plan) return SRFT_ERR_NULL;
    if (n_vec < 0 || n_vec > kMaxVectors) return SRFT_ERR_BAD_N;
    if (n_vec == 0) return SRFT_OK;
    if (!x_f16_dev || !codes_dev || !scales_dev) return SRFT_ERR_NULL;
    if (!srft_aligned(x_f16_dev, 16) || !srft_aligned(codes_dev, 16) || !srft_aligned(scales_dev, 4)) return SRFT_ERR_ALIGN;
    return launch_quantize(plan, x_f16_dev, n_vec, codes_dev, scales_dev, nullptr, kOutCodes, (hipStream_t)hip_stream);
}

int srft_kv_quantize_butterfly(const srft_plan_t* plan, const void* x_f16_dev, int64_t n_vec, uint8_t* codes_dev,
                               float* scales_dev, void* hip_stream) {
    if (!plan) return SRFT_ERR_NULL;
    if (plan->d != 128 && plan->d != 256) return SRFT_ERR_BAD_D;
    if (plan->gm != kGroup32) return SRFT_ERR_BAD_GROUP;
    if (plan->bits != 4) return SRFT_ERR_BAD_BITS;
    if (plan->transform != SRFT_TRANSFORM_DFT) return SRFT_ERR_BAD_TRANSFORM;
    if (n_vec < 0 || n_vec > kMaxVectors) return SRFT_ERR_BAD_N;
    if (n_vec == 0) return SRFT_OK;
    if (!x_f16_dev || !codes_dev || !scales_dev || !plan->bfly) return SRFT_ERR_NULL;
    if (!srft_aligned(x_f16_dev, 16) || !srft_aligned(codes_dev, 16) || !srft_aligned(scales_dev, 16)) return SRFT_ERR_ALIGN;
    return srft_launch_quantize_butterfly(plan->d, plan->bfly, x_f16_dev, n_vec, codes_dev, scales_dev, plan->max_wgs,
                                          (hipStream_t)hip_stream);
}

int srft_kv_forward_f32(const srft_plan_t* plan, const void* x_f16_dev, int64_t n_vec, float* w_f32_dev,
                        void* hip_stream) {
    if (!plan) return SRFT_ERR_NULL;
    if (n_vec < 0 || n_vec > kMaxVectors) return SRFT_ERR_BAD_N;
    if (n_vec == 0) return SRFT_OK;
    if (!x_f16_dev || !w_f32_dev) return SRFT_ERR_NULL;
    if (!srft_aligned(x_f16_dev, 16) || !srft_aligned(w_f32_dev, 16)) return SRFT_ERR_ALIGN;
    return launch_quantize(plan, x_f16_dev, n_vec, nullptr, nullptr, w_f32_dev, kOutRaw, (hipStream_t)hip_stream);
}

int srft_kv_channel_absmax(const srft_plan_t* plan, const void* x_f16_dev, int64_t n_vec, float* amax_dev,
                           void* hip_stream) {
    if (!plan) return SRFT_ERR_NULL;
    if (n_vec < 0 || n_vec > kMaxVectors) return SRFT_ERR_BAD_N;
    if (n_vec == 0) return SRFT_OK;
    if (!x_f16_dev || !amax_dev) return SRFT_ERR_NULL;
    if (!srft_aligned(x_f16_dev, 16) || !srft_aligned(amax_dev, 4)) return SRFT_ERR_ALIGN;
    return launch_quantize(plan, x_f16_dev, n_vec, nullptr, nullptr, amax_dev, kOutAmax, (hipStream_t)hip_stream);
}

int64_t srft_scores_workspace_bytes(const srft_plan_t* plan) {
    if (!plan) return SRFT_ERR_NULL;
    // the A fragments of up to 32 queries: d/16 k-steps x (hi, lo) x 64 lanes x 16 bytes, then 64 floats per
    // workgroup that absorb the stores of lanes without a valid (query, key)
    return (int64_t)(plan->d / 16) * 2 * 64 * 16 + (int64_t)kMaxScoreWorkgroups * 64 * 4;
}

static int scores_with_row_max(const srft_plan_t* plan, const void* q_f16_dev, int n_q, const uint8_t* codes_dev,
                               const float* scales_dev, int64_t n_keys, float* scores_dev, void* workspace_dev,
                               unsigned int* row_max, float sign, void* hip_stream) {
    if (!plan) return SRFT_ERR_NULL;
    if (plan->d % 64 != 0) return SRFT_ERR_BAD_D;
    if (plan->bits != 4) return SRFT_ERR_BAD_BITS;
    if (plan->gm == kGroup16) return SRFT_ERR_BAD_GROUP;
    if (n_q < 1 || n_q > 32 || n_keys < 0 || n_keys > kMaxVectors) return SRFT_ERR_BAD_N;
    if (n_keys == 0) return SRFT_OK;
    if (!q_f16_dev || !codes_dev || !scales_dev || !scores_dev || !workspace_dev) return SRFT_ERR_NULL;
    if (!srft_aligned(q_f16_dev, 16) || !srft_aligned(codes_dev, 16) || !srft_aligned(scales_dev, 4) || !srft_aligned(scores_dev, 4) ||
        !srft_aligned(workspace_dev, 16))
        return SRFT_ERR_ALIGN;
    hipStream_t st = (hipStream_t)hip_stream;
    uint4* qfrag = (uint4*)workspace_dev;
    float* dump = (float*)((char*)qfrag + (size_t)(plan->d / 16) * 2 * 64 * 16);
    // the write path's plain kernel transforms the queries and stores them as the scan's MFMA operands
    // (and clears the row maxima, if the caller wants them)
    const int rc = launch_quantize(plan, q_f16_dev, n_q, (uint8_t*)row_max, plan->inv_lam2, (float*)qfrag,
                                     n_q <= 16 ? kOutQFrag16 : kOutQFrag32, st);
    if (rc != SRFT_OK) return rc;
    return srft_launch_scores(plan, qfrag, dump, n_q, codes_dev, scales_dev, n_keys, scores_dev, row_max, sign, st);
}

int srft_kv_scores(const srft_plan_t* plan, const void* q_f16_dev, int n_q, const uint8_t* codes_dev,
                   const float* scales_dev, int64_t n_keys, float* scores_dev, void* workspace_dev, void* hip_stream) {
    return scores_with_row_max(plan, q_f16_dev, n_q, codes_dev, scales_dev, n_keys, scores_dev, workspace_dev, nullptr,
                               1.0f, hip_stream);
}

int srft_kv_scores_static(const srft_plan_t* plan, const void* q_f16_dev, int n_q, const uint8_t* codes_dev,
                          const float* scales_dev, int64_t n_keys, float* scores_dev, void* hip_stream) {
    if (!plan) return SRFT_ERR_NULL;
    // the static workspace holds the operands of up to 32 queries at d <= 256 and the dump slots of the largest
    // grid: anything a plan can ask for; a larger request is refused, never served from elsewhere
    if (srft_scores_workspace_bytes(plan) > (int64_t)kScoresScratchBytes) return SRFT_ERR_BAD_N;
    if (plan->device < 0 || plan->device >= kMaxDevices) return SRFT_ERR_HIP;
    void* ws = g_scratch_ptr[plan->device].load(std::memory_order_acquire);   // resolved when the plan was created
    if (!ws) return SRFT_ERR_NULL;
    return srft_kv_scores(plan, q_f16_dev, n_q, codes_dev, scales_dev, n_keys, scores_dev, ws, hip_stream);
}

static int attend_supported(const srft_plan_t* plan) {
    if (plan->d % 64 != 0) return SRFT_ERR_BAD_D;
    if (plan->bits != 4) return SRFT_ERR_BAD_BITS;
    if (plan->gm == kGroup16) return SRFT_ERR_BAD_GROUP;
    return SRFT_OK;
}

int64_t srft_attend_workspace_bytes(const srft_plan_t* plan) {
    if (!plan) return SRFT_ERR_NULL;
    return (int64_t)srft_attend_workspace_floats(plan->d) * 4;
}

int srft_kv_attend(const srft_plan_t* plan, const float* weights_f32_dev, int n_q, const uint8_t* codes_dev,
                   const float* scales_dev, int64_t n_keys, float* out_f32_dev, void* workspace_dev, void* hip_stream) {
    if (!plan) return SRFT_ERR_NULL;
    const int rc = attend_supported(plan);
    if (rc != SRFT_OK) return rc;
    if (n_q < 1 || n_q > 32 || n_keys < 1 || n_keys > kMaxVectors) return SRFT_ERR_BAD_N;
    if (!weights_f32_dev || !codes_dev || !scales_dev || !out_f32_dev || !workspace_dev) return SRFT_ERR_NULL;
    if (!srft_aligned(weights_f32_dev, 4) || !srft_aligned(codes_dev, 16) || !srft_aligned(scales_dev, 4) ||
        !srft_aligned(out_f32_dev, 4) || !srft_aligned(workspace_dev, 16))
        return SRFT_ERR_ALIGN;
    return srft_launch_attend(plan, weights_f32_dev, n_q, codes_dev, scales_dev, n_keys, out_f32_dev,
                              (float*)workspace_dev, nullptr, 1.0f, (hipStream_t)hip_stream);
}

int64_t srft_decode_attention_workspace_bytes(const srft_plan_t* plan_k, const srft_plan_t* plan_v, int n_q,
                                              int64_t n_keys) {
    if (!plan_k || !plan_v) return SRFT_ERR_NULL;
    if (n_q < 1 || n_q > 32 || n_keys < 1 || n_keys > kMaxVectors) return SRFT_ERR_BAD_N;
    const int64_t scores = ((int64_t)n_q * n_keys * 4 + 255) / 256 * 256;
    return scores + kRowMaxCopies * 32 * 4 + std::max(srft_scores_workspace_bytes(plan_k), srft_attend_workspace_bytes(plan_v));
}

int srft_kv_decode_attention(const srft_plan_t* plan_k, const srft_plan_t* plan_v, const void* q_f16_dev, int n_q,
                             const uint8_t* k_codes_dev, const float* k_scales_dev, const uint8_t* v_codes_dev,
                             const float* v_scales_dev, int64_t n_keys, float softmax_scale, float* out_f32_dev,
                             void* workspace_dev, void* hip_stream) {
    if (!plan_k || !plan_v) return SRFT_ERR_NULL;
    int rc = attend_supported(plan_v);
    if (rc != SRFT_OK) return rc;
    if (plan_k->d != plan_v->d || plan_k->device != plan_v->device) return SRFT_ERR_MISMATCH;
    if (n_q < 1 || n_q > 32 || n_keys < 1 || n_keys > kMaxVectors || !std::isfinite(softmax_scale)) return SRFT_ERR_BAD_N;
    if (!out_f32_dev || !workspace_dev || !v_codes_dev || !v_scales_dev) return SRFT_ERR_NULL;
    if (!srft_aligned(workspace_dev, 256) || !srft_aligned(out_f32_dev, 4) || !srft_aligned(v_codes_dev, 16) ||
        !srft_aligned(v_scales_dev, 4))
        return SRFT_ERR_ALIGN;
    float* scores = (float*)workspace_dev;
    unsigned int* row_max = (unsigned int*)((char*)workspace_dev + ((int64_t)n_q * n_keys * 4 + 255) / 256 * 256);
    void* rest = (char*)row_max + kRowMaxCopies * 32 * 4;
    hipStream_t st = (hipStream_t)hip_stream;
    // Scores of the queries against the stored keys, the scan keeping the maximum of softmax_scale * score per row;
    // then the stored values weighted with exp(softmax_scale * score - maximum), formed from the raw scores as the
    // value-side kernel loads them, the sums of those weights carried along and divided out at the end: the row
    // softmax has no pass of its own.  The same workspace serves both steps, which run one after the other.
    rc = scores_with_row_max(plan_k, q_f16_dev, n_q, k_codes_dev, k_scales_dev, n_keys, scores, rest, row_max,
                             softmax_scale < 0.0f ? -1.0f : 1.0f, hip_stream);
    if (rc != SRFT_OK) return rc;
    return srft_launch_attend(plan_v, scores, n_q, v_codes_dev, v_scales_dev, n_keys, out_f32_dev, (float*)rest,
                              row_max, softmax_scale, st);
}

int srft_lambda_from_absmax(const float* amax_host, int d, float* lambda_host) {
    if (!amax_host || !lambda_host) return SRFT_ERR_NULL;
    if (d < 1) return SRFT_ERR_BAD_D;
    float top = 0.0f;
    for (int k = 0; k < d; ++k) {
        if (!std::isfinite(amax_host[k]) || amax_host[k] < 0.0f) return SRFT_ERR_BAD_LAMBDA;
        top = std::fmax(top, amax_host[k]);
    }
    // lambda_k = 1 / amax_k; channels below 2^-16 of the largest are held there, which keeps max/min of lambda
    // within what srft_plan_create accepts; an all-zero batch gives all ones
    const float floor_ = std::ldexp(top, -16);
    for (int k = 0; k < d; ++k) lambda_host[k] = top > 0.0f ? 1.0f / std::fmax(amax_host[k], floor_) : 1.0f;
    return SRFT_OK;
}

int srft_kv_dequantize(const srft_plan_t* plan, const uint8_t* codes_dev, const float* scales_dev, int64_t n_vec,
                       void* out_f16_dev, void* hip_stream) {
    if (!plan) return SRFT_ERR_NULL;
    if (n_vec < 0 || n_vec > kMaxVectors) return SRFT_ERR_BAD_N;
    if (n_vec == 0) return SRFT_OK;
    if (!codes_dev || !scales_dev || !out_f16_dev) return SRFT_ERR_NULL;
    if (!srft_aligned(codes_dev, 16) || !srft_aligned(scales_dev, 4) || !srft_aligned(out_f16_dev, 16)) return SRFT_ERR_ALIGN;
    return launch_dequantize(plan, codes_dev, scales_dev, n_vec, out_f16_dev, (hipStream_t)hip_stream);
}

int srft_kv_quantize_batched(const srft_plan_t* const* plans, const void* const* x_f16_dev, const int64_t* n_vec,
                             uint8_t* const* codes_dev, float* const* scales_dev, int count, void* hip_stream) {
    return srft_run_batched(plans, x_f16_dev, nullptr, (void* const*)codes_dev, (void* const*)scales_dev, n_vec, count,
                       true, (hipStream_t)hip_stream);
}

int srft_kv_dequantize_batched(const srft_plan_t* const* plans, const uint8_t* const* codes_dev,
                               const float* const* scales_dev, const int64_t* n_vec, void* const* out_f16_dev,
                               int count, void* hip_stream) {
    return srft_run_batched(plans, (const void* const*)codes_dev, (const void* const*)scales_dev, out_f16_dev, nullptr,
                       n_vec, count, false, (hipStream_t)hip_stream);
}

const char* srft_status_string(int status) {
    switch (status) {
        case SRFT_OK: return "ok";
        case SRFT_ERR_NULL: return "required pointer is NULL";
        case SRFT_ERR_BAD_D: return "unsupported head dimension (need a multiple of 32 in [32, 256])";
        case SRFT_ERR_BAD_GROUP: return "unsupported group size (need 16, or a multiple of 32 that divides d)";
        case SRFT_ERR_BAD_LAMBDA: return "lambda must be finite, > 0 and span at most 2^16";
        case SRFT_ERR_ALIGN: return "device pointer is misaligned";
        case SRFT_ERR_HIP: return "HIP call failed (see srft_last_hip_error)";
        case SRFT_ERR_BAD_N: return "negative or malformed size";
        case SRFT_ERR_MISMATCH: return "plans of one call must share d, group size, code width and device";
        case SRFT_ERR_BAD_BITS: return "unsupported code width (need 4 or 8 bits)";
        case SRFT_ERR_BAD_TRANSFORM: return "unknown transform";
        default: return "unknown status";
    }
}

}  // extern "C"
