// stream.hip -- measurement aids, not part of the method: plain streaming kernels whose rate is what the memory
// system offers a kernel with a given traffic shape.  Built into a library of its own (libsrft_measure.so).
#include <hip/hip_runtime.h>

#include <cstdint>

#include "srft_measure.h"

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void stream_store(uint4* p, uint4 v) {
    __builtin_nontemporal_store(__builtin_bit_cast(u32x4, v), reinterpret_cast<u32x4*>(p));
}
__device__ __forceinline__ uint4 stream_load(const uint4* p) {
    return __builtin_bit_cast(uint4, __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p)));
}

__global__ void __launch_bounds__(256)
srft_copy_kernel(uint4* __restrict__ dst, const uint4* __restrict__ src, long long n_units) {
    const long long stride = (long long)gridDim.x * blockDim.x;
    for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < n_units; i += stride)
        dst[i] = src[i];
}

// Streaming kernel with a given read : write byte mix per tile and no arithmetic to speak of: every
// workgroup walks tiles, reads r_units 16-byte units and writes w_units units per tile, all coalesced.
// Its rate is the ceiling the memory system offers a kernel with the same traffic shape.
// STREAM: non-temporal loads and stores (what the read path uses)
// CHUNK: 16-byte units a thread reads next to each other (1: a wavefront's load covers 1 KiB contiguously; 4: every
// lane reads 64 contiguous bytes with four loads, so that each load touches a quarter of every cache line it visits)
template <int RU, bool STREAM, int CHUNK = 1>   // RU = ceil(r_units / 256): loads per thread and tile, all issued before any is used
__global__ void __launch_bounds__(256)
srft_mix_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, long long n_tiles, int r_units, int w_units,
                int die_map) {
    // die_map: workgroup b runs on accelerator die b mod 8 (the hardware deals workgroups round-robin); each die then
    // gets one contiguous eighth of the tiles, walked by its workgroups with stride gridDim / 8.  Otherwise tile =
    // blockIdx + k gridDim, so that neighbouring tiles go to different dies.
    long long t0 = blockIdx.x, stride = gridDim.x, t_end = n_tiles;
    if (die_map && (gridDim.x & 7) == 0 && n_tiles >= (long long)gridDim.x) {
        const long long per_die = (n_tiles + 7) >> 3, die = blockIdx.x & 7;
        stride = gridDim.x >> 3;
        t0 = die * per_die + (blockIdx.x >> 3);
        t_end = n_tiles < (die + 1) * per_die ? n_tiles : (die + 1) * per_die;
    }
    for (long long t = t0; t < t_end; t += stride) {
        const uint4* s = src + t * r_units;
        uint4 v[RU] = {};
        if (r_units > 0) {                       // uniform; r_units = 0 is the write-only stream
#pragma unroll
            for (int i = 0; i < RU; ++i) {
                const int u = CHUNK == 1 ? threadIdx.x + 256 * i
                                         : (int)threadIdx.x * CHUNK + i % CHUNK + 256 * CHUNK * (i / CHUNK);
                v[i] = STREAM ? stream_load(&s[u < r_units ? u : r_units - 1]) : s[u < r_units ? u : r_units - 1];
            }
        }
        // every thread consumes what it loaded, here: only w_units of the 256 threads store, and without this the
        // compiler sinks the loads into the storing threads' branch, so that the others read nothing
#pragma unroll
        for (int i = 0; i < RU; ++i) asm volatile("" ::"v"(v[i].x), "v"(v[i].y), "v"(v[i].z), "v"(v[i].w));
        uint4 acc = v[0];
#pragma unroll
        for (int i = 1; i < RU; ++i) { acc.x ^= v[i].x; acc.y ^= v[i].y; acc.z ^= v[i].z; acc.w ^= v[i].w; }
        uint4* d = dst + t * w_units;
        for (int u = threadIdx.x; u < w_units; u += 256) {
            if (STREAM) stream_store(&d[u], acc);
            else d[u] = acc;
        }
    }
}

bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }
thread_local int g_last_hip_error = 0;
#define MEASURE_HIP(call)                                \
    do {                                                 \
        hipError_t e_ = (call);                          \
        if (e_ != hipSuccess) {                          \
            g_last_hip_error = (int)e_;                  \
            return SRFT_ERR_HIP;                         \
        }                                                \
    } while (0)

}  // namespace

extern "C" {

int srft_stream_copy(void* dst_dev, const void* src_dev, int64_t n_bytes, void* hip_stream) {
    if (n_bytes < 0 || n_bytes % 16 != 0) return SRFT_ERR_BAD_N;
    if (n_bytes == 0) return SRFT_OK;
    if (!dst_dev || !src_dev) return SRFT_ERR_NULL;
    if (!aligned16(dst_dev) || !aligned16(src_dev)) return SRFT_ERR_ALIGN;
    int dev = 0, cus = 0;
    MEASURE_HIP(hipGetDevice(&dev));
    MEASURE_HIP(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
    const long long units = n_bytes / 16;
    long long grid = (long long)cus * 8;
    if (grid > (units + 255) / 256) grid = (units + 255) / 256;
    hipLaunchKernelGGL(srft_copy_kernel, dim3((unsigned)grid), dim3(256), 0, (hipStream_t)hip_stream, (uint4*)dst_dev,
                       (const uint4*)src_dev, units);
    MEASURE_HIP(hipGetLastError());
    return SRFT_OK;
}

int srft_stream_mix(const void* src_dev, void* dst_dev, int64_t n_tiles, int read_bytes_per_tile,
                    int write_bytes_per_tile, int workgroups, int access, void* hip_stream) {
    const int nontemporal = access;
    if (n_tiles < 0 || read_bytes_per_tile < 0 || write_bytes_per_tile < 0 || read_bytes_per_tile % 16 ||
        write_bytes_per_tile % 16 || read_bytes_per_tile + write_bytes_per_tile == 0 || workgroups < 0)
        return SRFT_ERR_BAD_N;
    if (n_tiles == 0) return SRFT_OK;
    if (!src_dev || !dst_dev) return SRFT_ERR_NULL;
    if (!aligned16(src_dev) || !aligned16(dst_dev)) return SRFT_ERR_ALIGN;
    int dev = 0, cus = 0;
    MEASURE_HIP(hipGetDevice(&dev));
    MEASURE_HIP(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
    long long grid = workgroups > 0 ? workgroups : (long long)cus * 3;
    if (grid > n_tiles) grid = n_tiles;
    const int r_units = read_bytes_per_tile / 16, w_units = write_bytes_per_tile / 16;
    const int ru = r_units > 0 ? (r_units + 255) / 256 : 1;
    const bool stream = (nontemporal & 1) != 0, chunk4 = (nontemporal & 2) != 0;
    if (chunk4 && r_units % 1024 != 0) return SRFT_ERR_BAD_N;
    void (*kernel)(const uint4*, uint4*, long long, int, int, int) = nullptr;
#define SRFT_MIX_CASE(N)                                                                                          \
    case N:                                                                                                       \
        kernel = chunk4 ? (stream ? srft_mix_kernel<N, true, 4> : srft_mix_kernel<N, false, 4>)                  \
                        : (stream ? srft_mix_kernel<N, true> : srft_mix_kernel<N, false>);                       \
        break;
    switch (ru) {
        SRFT_MIX_CASE(1) SRFT_MIX_CASE(2) SRFT_MIX_CASE(3) SRFT_MIX_CASE(4)
        SRFT_MIX_CASE(5) SRFT_MIX_CASE(6) SRFT_MIX_CASE(7) SRFT_MIX_CASE(8)
        default: return SRFT_ERR_BAD_N;         // at most 32 KiB read per tile
    }
#undef SRFT_MIX_CASE
    hipLaunchKernelGGL(kernel, dim3((unsigned)grid), dim3(256), 0, (hipStream_t)hip_stream, (const uint4*)src_dev,
                       (uint4*)dst_dev, (long long)n_tiles, r_units, w_units, (nontemporal & 4) ? 1 : 0);
    MEASURE_HIP(hipGetLastError());
    return SRFT_OK;
}

int srft_measure_last_hip_error(void) { return g_last_hip_error; }

}  // extern "C"
