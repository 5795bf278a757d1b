// Row statistics of the softmax between the two halves of attention over the stored cache: for every row of
// scale * x its maximum m and 1 / sum exp(scale x - m).  The value-side kernel turns the raw scores into weights
// with them as it loads the scores, so the scores are read twice (here and there) and never rewritten.
// Rows are long (the number of keys) and few (the queries sharing a KV head), so every row is split into chunks:
// a first kernel leaves each chunk's maximum and its sum of exponentials relative to that maximum (one pass: a
// thread keeps a running maximum and rescales its running sum when the maximum moves), a second one combines the
// chunk results of a row in a fixed order.
#include "../device_util.h"

namespace {

constexpr int kSoftmaxThreads = 256;
constexpr int kSoftmaxMaxChunks = 1024;
constexpr int kSoftmaxBatch = 16;                // loads a thread has in flight

// (m, s) <- combination of (m, s) and (m2, s2): maxima and sums of exponentials relative to them
__device__ __forceinline__ void combine(float& m, float& s, float m2, float s2) {
    const float mn = fmaxf(m, m2);
    // an empty part has m = -inf and s = 0: exp(-inf - mn) = 0 unless both are empty (then s stays 0)
    const float a = (m == mn) ? 1.0f : __expf(m - mn), b = (m2 == mn) ? 1.0f : __expf(m2 - mn);
    s = s * a + s2 * b;
    m = mn;
}

// the (m, s) of all threads of the workgroup, combined lane by lane and wavefront by wavefront in a fixed order
__device__ __forceinline__ void block_combine(float& m, float& s, float2* red) {
    for (int off = 32; off > 0; off >>= 1) {
        const float m2 = __shfl_xor(m, off, 64), s2 = __shfl_xor(s, off, 64);
        combine(m, s, m2, s2);
    }
    const int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) red[wave] = make_float2(m, s);
    __syncthreads();
    m = red[0].x;
    s = red[0].y;
    for (int i = 1; i < kSoftmaxThreads / 64; ++i) combine(m, s, red[i].x, red[i].y);
}

// stats[row][chunk] = (max of scale x over the chunk, sum of exp(scale x - that max))
__global__ void __launch_bounds__(kSoftmaxThreads)
srft_softmax_chunk_stats_kernel(const float* __restrict__ x, long long n, long long chunk, float scale,
                                float2* __restrict__ stats) {
    __shared__ float2 red[kSoftmaxThreads / 64];
    const float* row = x + (long long)blockIdx.y * n;
    const long long lo = (long long)blockIdx.x * chunk, hi = min(n, lo + chunk);
    float m = -INFINITY, s = 0.0f;
    for (long long t0 = lo + threadIdx.x; t0 < hi; t0 += (long long)kSoftmaxBatch * kSoftmaxThreads) {
        float v[kSoftmaxBatch];
#pragma unroll
        for (int i = 0; i < kSoftmaxBatch; ++i) {            // coalesced: a wavefront's load covers 256 contiguous bytes
            const long long t = t0 + (long long)i * kSoftmaxThreads;
            v[i] = t < hi ? scale * row[t] : -INFINITY;
        }
        float bm = v[0];
#pragma unroll
        for (int i = 1; i < kSoftmaxBatch; ++i) bm = fmaxf(bm, v[i]);
        float bs = 0.0f;
#pragma unroll
        for (int i = 0; i < kSoftmaxBatch; ++i) bs += __expf(v[i] - bm);       // exp(-inf) = 0 for the slots past the end
        combine(m, s, bm, bs);
    }
    block_combine(m, s, red);
    if (threadIdx.x == 0) stats[(long long)blockIdx.y * gridDim.x + blockIdx.x] = make_float2(m, s);
}

// row_stats[row] = (max of scale x over the row, 1 / sum of exp(scale x - that max))
__global__ void __launch_bounds__(kSoftmaxThreads)
srft_softmax_row_stats_kernel(const float2* __restrict__ stats, int chunks, float2* __restrict__ row_stats) {
    __shared__ float2 red[kSoftmaxThreads / 64];
    const float2* rs = stats + (long long)blockIdx.x * chunks;
    float m = -INFINITY, s = 0.0f;
    for (int c = threadIdx.x; c < chunks; c += kSoftmaxThreads) combine(m, s, rs[c].x, rs[c].y);
    block_combine(m, s, red);
    if (threadIdx.x == 0) row_stats[blockIdx.x] = make_float2(m, 1.0f / s);
}

}  // namespace

// chunk_stats: room for rows x kSoftmaxMaxChunks float pairs (srft_softmax_stats_bytes); row_stats: rows float pairs
int64_t srft_softmax_stats_bytes(int rows) { return (int64_t)rows * (kSoftmaxMaxChunks + 1) * 8; }

int srft_launch_softmax_row_stats(const float* x, int rows, long long n, float scale, void* chunk_stats,
                                  float2* row_stats, hipStream_t st) {
    // 4 Ki scores per workgroup (one batch of loads per thread), at most kSoftmaxMaxChunks chunks per row
    long long chunks = (n + kSoftmaxBatch * kSoftmaxThreads - 1) / (kSoftmaxBatch * kSoftmaxThreads);
    if (chunks > kSoftmaxMaxChunks) chunks = kSoftmaxMaxChunks;
    const long long chunk = (n + chunks - 1) / chunks;
    chunks = (n + chunk - 1) / chunk;
    hipLaunchKernelGGL(srft_softmax_chunk_stats_kernel, dim3((unsigned)chunks, (unsigned)rows), dim3(kSoftmaxThreads), 0,
                       st, x, n, chunk, scale, (float2*)chunk_stats);
    SRFT_HIP(hipGetLastError());
    hipLaunchKernelGGL(srft_softmax_row_stats_kernel, dim3((unsigned)rows), dim3(kSoftmaxThreads), 0, st,
                       (const float2*)chunk_stats, (int)chunks, row_stats);
    SRFT_HIP(hipGetLastError());
    return SRFT_OK;
}
