// Row softmax between the two halves of attention over the stored cache: x <- exp(scale x - max) / sum, in place.
// Rows are long (the number of keys) and few (the queries sharing a KV head), so every row is split into chunks:
// a first kernel leaves each chunk's maximum and its sum of exponentials relative to that maximum, a second one
// combines the chunk results of its row (every workgroup redoes that small reduction, in the same order) and
// normalises its own chunk.  Two reads and one write of the scores.
#include "../device_util.h"

namespace {

constexpr int kSoftmaxThreads = 256;
constexpr int kSoftmaxMaxChunks = 1024;

__device__ __forceinline__ float block_reduce(float v, float* red, bool take_max) {
    for (int off = 32; off > 0; off >>= 1) {
        const float o = __shfl_xor(v, off, 64);
        v = take_max ? fmaxf(v, o) : v + o;
    }
    const int wave = threadIdx.x >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[wave] = v;
    __syncthreads();
    float r = red[0];
    for (int i = 1; i < kSoftmaxThreads / 64; ++i) r = take_max ? fmaxf(r, red[i]) : r + red[i];
    return r;
}

// stats[row][chunk] = (max of scale x over the chunk, sum of exp(scale x - that max))
__global__ void __launch_bounds__(kSoftmaxThreads)
srft_softmax_stats_kernel(const float* __restrict__ x, long long n, long long chunk, float scale, float2* __restrict__ stats) {
    __shared__ float red[kSoftmaxThreads / 64];
    const float* row = x + (long long)blockIdx.y * n;
    const long long lo = (long long)blockIdx.x * chunk, hi = min(n, lo + chunk);
    float m = -INFINITY;
    for (long long t = lo + threadIdx.x; t < hi; t += kSoftmaxThreads) m = fmaxf(m, scale * row[t]);
    m = block_reduce(m, red, true);
    float sum = 0.0f;
    for (long long t = lo + threadIdx.x; t < hi; t += kSoftmaxThreads) sum += __expf(scale * row[t] - m);
    sum = block_reduce(sum, red, false);
    if (threadIdx.x == 0) stats[(long long)blockIdx.y * gridDim.x + blockIdx.x] = make_float2(m, sum);
}

__global__ void __launch_bounds__(kSoftmaxThreads)
srft_softmax_apply_kernel(float* __restrict__ x, long long n, long long chunk, float scale, const float2* __restrict__ stats) {
    const float2* rs = stats + (long long)blockIdx.y * gridDim.x;
    float m = -INFINITY;
    for (int c = 0; c < (int)gridDim.x; ++c) m = fmaxf(m, rs[c].x);
    float sum = 0.0f;
    for (int c = 0; c < (int)gridDim.x; ++c) sum += rs[c].y * __expf(rs[c].x - m);
    const float inv = 1.0f / sum;
    float* row = x + (long long)blockIdx.y * n;
    const long long lo = (long long)blockIdx.x * chunk, hi = min(n, lo + chunk);
    for (long long t = lo + threadIdx.x; t < hi; t += kSoftmaxThreads) row[t] = __expf(scale * row[t] - m) * inv;
}

}  // namespace

// stats: room for rows x kSoftmaxMaxChunks float pairs (srft_softmax_stats_bytes)
int64_t srft_softmax_stats_bytes(int rows) { return (int64_t)rows * kSoftmaxMaxChunks * 8; }

int srft_launch_softmax_rows(float* x, int rows, long long n, float scale, void* stats, hipStream_t st) {
    long long chunks = (n + 16383) / 16384;                  // 16 Ki scores per workgroup, at most kSoftmaxMaxChunks chunks
    if (chunks > kSoftmaxMaxChunks) chunks = kSoftmaxMaxChunks;
    const long long chunk = (n + chunks - 1) / chunks;
    chunks = (n + chunk - 1) / chunk;
    hipLaunchKernelGGL(srft_softmax_stats_kernel, dim3((unsigned)chunks, (unsigned)rows), dim3(kSoftmaxThreads), 0, st,
                       (const float*)x, n, chunk, scale, (float2*)stats);
    SRFT_HIP(hipGetLastError());
    hipLaunchKernelGGL(srft_softmax_apply_kernel, dim3((unsigned)chunks, (unsigned)rows), dim3(kSoftmaxThreads), 0, st, x,
                       n, chunk, scale, (const float2*)stats);
    SRFT_HIP(hipGetLastError());
    return SRFT_OK;
}
