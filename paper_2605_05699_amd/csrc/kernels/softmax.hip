// Row softmax between the two halves of attention over the stored cache: x <- exp(scale x - max) / sum, in place.
// One workgroup per row, three passes over the row (maximum, sum of exponentials, normalisation); rows are a few
// megabytes at most and there are at most 32 of them, so this is a utility, not a hot kernel.
#include "../device_util.h"

namespace {

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
    for (int i = 1; i < (int)(blockDim.x >> 6); ++i) r = take_max ? fmaxf(r, red[i]) : r + red[i];
    return r;
}

__global__ void __launch_bounds__(1024)
srft_softmax_rows_kernel(float* __restrict__ x, long long n, float scale) {
    __shared__ float red[16];
    float* row = x + (long long)blockIdx.x * n;
    float m = -INFINITY;
    for (long long t = threadIdx.x; t < n; t += blockDim.x) m = fmaxf(m, scale * row[t]);
    m = block_reduce(m, red, true);
    float sum = 0.0f;
    for (long long t = threadIdx.x; t < n; t += blockDim.x) {
        const float e = __expf(scale * row[t] - m);
        row[t] = e;
        sum += e;
    }
    sum = block_reduce(sum, red, false);
    const float inv = 1.0f / sum;
    for (long long t = threadIdx.x; t < n; t += blockDim.x) row[t] *= inv;
}

}  // namespace

int srft_launch_softmax_rows(float* x, int rows, long long n, float scale, hipStream_t st) {
    hipLaunchKernelGGL(srft_softmax_rows_kernel, dim3((unsigned)rows), dim3(1024), 0, st, x, n, scale);
    SRFT_HIP(hipGetLastError());
    return SRFT_OK;
}
