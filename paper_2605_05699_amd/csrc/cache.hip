// cache.hip -- cache manager: host bookkeeping around the batched kernels (int4 store, fp16 residual window,
// dequantized view), and the small scatter kernel that places new tokens in the paged view.
#include <algorithm>
#include <new>

#include "common.h"

namespace {

// Cache append: the new tokens of every plan, [n_seq][t][units] 16-byte units each, go to their place in the paged
// fp16 view [block][n_seq][R][units]: token pos0 + j of sequence q lands in block (pos0 + j) / R, slot (pos0 + j) % R.
// a.in0[p] / a.out0[p] are plan p's new tokens and view.  A few kilobytes per step: one thread per unit.
__global__ void __launch_bounds__(256)
srft_cache_scatter_kernel(const srft_batch_args a, int n_seq, int t, int units, int R, long long pos0) {
    const long long per_plan = (long long)n_seq * t * units, total = per_plan * a.count;
    for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < total; i += (long long)gridDim.x * 256) {
        const int p = (int)(i / per_plan);
        const long long r = i % per_plan;
        const int u = (int)(r % units);
        const long long st = r / units;
        const int tok = (int)(st % t), seq = (int)(st / t);
        const long long token = pos0 + tok, block = token / R;
        const int slot = (int)(token % R);
        reinterpret_cast<uint4*>(a.out0[p])[((block * n_seq + seq) * R + slot) * units + u] =
            reinterpret_cast<const uint4*>(a.in0[p])[r];
    }
}

}  // namespace

extern "C" {

int srft_cache_create(srft_cache_t** out, const srft_plan_t* const* plans, int n_plans, int n_seq,
                      int64_t capacity_tokens, int residual_tokens, uint8_t* const* codes_dev,
                      float* const* scales_dev, void* const* view_f16_dev) {
    if (!out) return SRFT_ERR_NULL;
    *out = nullptr;
    if (!plans || !codes_dev || !scales_dev || !view_f16_dev) return SRFT_ERR_NULL;
    if (n_plans < 1 || n_seq < 1 || residual_tokens < 1 || capacity_tokens < residual_tokens ||
        capacity_tokens % residual_tokens != 0 || capacity_tokens * n_seq > kMaxVectors)
        return SRFT_ERR_BAD_N;
    for (int i = 0; i < n_plans; ++i) {
        if (!plans[i] || !codes_dev[i] || !scales_dev[i] || !view_f16_dev[i]) return SRFT_ERR_NULL;
        if (!srft_plans_compatible(plans[i], plans[0])) return SRFT_ERR_MISMATCH;
        if (!srft_aligned(codes_dev[i], 16) || !srft_aligned(scales_dev[i], 4) || !srft_aligned(view_f16_dev[i], 16))
            return SRFT_ERR_ALIGN;
    }
    srft_cache* c = new (std::nothrow) srft_cache();
    if (!c) return SRFT_ERR_HIP;
    c->plans.assign(plans, plans + n_plans);
    c->codes.assign(codes_dev, codes_dev + n_plans);
    c->scales.assign(scales_dev, scales_dev + n_plans);
    c->view.assign(view_f16_dev, view_f16_dev + n_plans);
    c->n_seq = n_seq;
    c->R = residual_tokens;
    c->capacity = capacity_tokens;
    *out = c;
    return SRFT_OK;
}

int srft_cache_destroy(srft_cache_t* cache) {
    delete cache;
    return SRFT_OK;
}

int64_t srft_cache_tokens(const srft_cache_t* cache) { return cache ? cache->tokens : SRFT_ERR_NULL; }
int64_t srft_cache_quantized_tokens(const srft_cache_t* cache) { return cache ? cache->quantized : SRFT_ERR_NULL; }

// quantize (and read back into the view) or only read back the tokens [first, first + count) of every plan;
// both are multiples of R, so the range is contiguous in the paged layout
static int cache_convert(const srft_cache* c, int64_t first, int64_t count, bool quantize, hipStream_t st) {
    const size_t np = c->plans.size();
    const int d = c->plans[0]->d, G = d / c->plans[0]->g;
    const int64_t v0 = first * c->n_seq, nv = count * c->n_seq;          // vectors
    std::vector<const void*> x(np), cd(np), sc(np);
    std::vector<void*> xo(np), cdo(np), sco(np);
    std::vector<int64_t> n(np, nv);
    for (size_t i = 0; i < np; ++i) {
        xo[i] = (char*)c->view[i] + v0 * d * 2;
        cdo[i] = c->codes[i] + v0 * (d * c->plans[0]->bits / 8);
        sco[i] = c->scales[i] + v0 * G;
        x[i] = xo[i];
        cd[i] = cdo[i];
        sc[i] = sco[i];
    }
    if (quantize) {
        const int rc = srft_run_batched(c->plans.data(), x.data(), nullptr, cdo.data(), sco.data(), n.data(), (int)np,
                                   true, st);
        if (rc != SRFT_OK) return rc;
    }
    return srft_run_batched(c->plans.data(), cd.data(), sc.data(), xo.data(), nullptr, n.data(), (int)np, false, st);
}

int srft_cache_append(srft_cache_t* cache, const void* const* new_f16_dev, int t, void* hip_stream) {
    if (!cache) return SRFT_ERR_NULL;
    if (t < 0 || cache->tokens + t > cache->capacity) return SRFT_ERR_BAD_N;
    if (t == 0) return SRFT_OK;
    if (!new_f16_dev) return SRFT_ERR_NULL;
    const size_t np = cache->plans.size();
    for (size_t i = 0; i < np; ++i) {
        if (!new_f16_dev[i]) return SRFT_ERR_NULL;
        if (!srft_aligned(new_f16_dev[i], 16)) return SRFT_ERR_ALIGN;
    }
    hipStream_t st = (hipStream_t)hip_stream;
    const int units = cache->plans[0]->d / 8;
    // 1. the new tokens join the window: an exact fp16 copy into the view
    for (size_t p0 = 0; p0 < np; p0 += kMaxBatch) {
        srft_batch_args a;
        a.count = (int)std::min<size_t>(kMaxBatch, np - p0);
        for (int k = 0; k < a.count; ++k) {
            a.in0[k] = new_f16_dev[p0 + k];
            a.out0[k] = cache->view[p0 + k];
        }
        const long long total = (long long)a.count * cache->n_seq * t * units;
        const unsigned grid = (unsigned)std::min<long long>((total + 255) / 256, 4096);
        hipLaunchKernelGGL(srft_cache_scatter_kernel, dim3(grid), dim3(256), 0, st, a, cache->n_seq, t, units, cache->R,
                           (long long)cache->tokens);
        SRFT_HIP(hipGetLastError());
    }
    cache->tokens += t;
    // 2. every window that is now full is quantized into the store and replaced, in the view, by what the store
    //    decodes to (the window is "re-quantized when full"; the dequantized prefix is refreshed only here)
    const int64_t full = cache->tokens / cache->R * cache->R;
    if (full > cache->quantized) {
        const int rc = cache_convert(cache, cache->quantized, full - cache->quantized, true, st);
        if (rc != SRFT_OK) return rc;
        cache->quantized = full;
    }
    return SRFT_OK;
}

int srft_cache_rebuild_view(srft_cache_t* cache, void* hip_stream) {
    if (!cache) return SRFT_ERR_NULL;
    if (cache->quantized == 0) return SRFT_OK;
    return cache_convert(cache, 0, cache->quantized, false, (hipStream_t)hip_stream);
}

}  // extern "C"
