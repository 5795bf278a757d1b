// Write path at d = 128 with the transform as FFT butterflies on the vector ALU instead of a matrix-core
// contraction: the form the paper's kernel has (Sec. 3.2: the real transform through a complex FFT of half the
// length and a Hermitian unpack; Sec. 7.1), kept so that the two forms can be timed side by side on this machine.
// Same record as srft_kv_quantize (Sec. 3.2 steps 1-4, Sec. 5.1, Sec. 7.1); fp32 arithmetic throughout, as in the
// paper's kernel.
//
// One vector per lane, entirely in registers: no cross-lane exchange at all (a mapping of a vector onto several
// lanes adds DPP / swizzle moves on top of the same arithmetic).  A wavefront takes 64 vectors per step:
//   1. the 64 rows (16 KiB) are loaded with coalesced 16-byte loads and pass through LDS, from which every lane
//      reads its own row (padded rows: conflict-free);
//   2. u = s * x (sign bit of the packed fp16 pairs), conversion to fp32, z_m = u_2m + i u_2m+1;
//   3. complex FFT of length 64, radix 2, decimation in time, fully unrolled with compile-time twiddles (trivial
//      and eighth-turn factors cost no general multiply);
//   4. Hermitian unpack to the bins 0 .. 64, the packing of Eq. 2, times lambda sqrt(2/d) (one constant per packed index);
//   5. per group of 32 packed indices: abs-max, scale, round to nearest even, nibble pack -- all inside the lane;
//   6. every lane stores its 64 code bytes and 4 scales.
#include "../device_util.h"

namespace {

constexpr double kPi = 3.14159265358979323846264338327950288;

// cos / sin of 2 pi k / n at compile time (Taylor series after reduction to the first octant)
constexpr double series_sin(double x) {
    double term = x, sum = x;
    for (int i = 1; i < 12; ++i) {
        term *= -x * x / ((2 * i) * (2 * i + 1));
        sum += term;
    }
    return sum;
}
constexpr double series_cos(double x) {
    double term = 1.0, sum = 1.0;
    for (int i = 1; i < 12; ++i) {
        term *= -x * x / ((2 * i - 1) * (2 * i));
        sum += term;
    }
    return sum;
}
constexpr double cos_turn(int k, int n) {        // cos(2 pi k / n)
    k = ((k % n) + n) % n;
    if (2 * k > n) k = n - k;                    // cos is even about half a turn
    if (4 * k > n) return -cos_turn(n - 2 * k, 2 * n);          // cos(pi - x) = -cos x, x = 2 pi (n - 2k) / (2n)
    if (8 * k > n) return series_sin(2.0 * kPi * (n - 4 * k) / (4.0 * n));      // cos(pi/2 - y) = sin y
    return series_cos(2.0 * kPi * k / n);
}
constexpr double sin_turn(int k, int n) { return cos_turn(4 * k - n, 4 * n); }   // sin x = cos(x - pi/2)

constexpr int bit_reverse6(int i) {
    int r = 0;
    for (int b = 0; b < 6; ++b) r |= ((i >> b) & 1) << (5 - b);
    return r;
}

// one stage of the radix-2 decimation-in-time FFT over 64 complex points held in registers; M = butterfly span
template <int M, int J = 0>
__device__ __forceinline__ void fft64_stage(float (&re)[64], float (&im)[64]) {
    if constexpr (J < 32) {
        constexpr int t = J % (M / 2), base = (J / (M / 2)) * M + t, other = base + M / 2;
        // W = exp(-2 pi i t / M) = c - i s
        constexpr float c = (float)cos_turn(t, M), s = (float)sin_turn(t, M);
        float br, bi;
        if constexpr (t == 0) {
            br = re[other];
            bi = im[other];
        } else if constexpr (4 * t == M) {       // W = -i
            br = im[other];
            bi = -re[other];
        } else {                                 // (c - i s)(x + i y) = (c x + s y) + i (c y - s x)
            br = fmaf(c, re[other], s * im[other]);
            bi = fmaf(c, im[other], -s * re[other]);
        }
        const float ar = re[base], ai = im[base];
        re[base] = ar + br;
        im[base] = ai + bi;
        re[other] = ar - br;
        im[other] = ai - bi;
        fft64_stage<M, J + 1>(re, im);
    }
}

// bins k and 64 - k of the length-128 real transform from the length-64 complex one (k = 1 .. 31):
//   E = (Z_k + conj Z_{64-k}) / 2 (the transform of the even inputs), O = (Z_k - conj Z_{64-k}) / (2i) (of the odd ones),
//   Y_k = E + W^k O,  Y_{64-k} = conj(E - W^k O),  W = exp(-2 pi i / 128).  The halves are left to the constants cl.
// In place: the packed value z_p lands in re[p] for p < 64 and in im[p - 64] for p >= 64, so that the 128 packed
// values take the registers of the 64 complex ones (a second array would halve the wavefronts per SIMD).
template <int K>
__device__ __forceinline__ void unpack_pairs(float (&re)[64], float (&im)[64], const float* __restrict__ cl) {
    if constexpr (K < 32) {
        constexpr float c = (float)cos_turn(K, 128), s = (float)sin_turn(K, 128);
        const float er = re[K] + re[64 - K], ei = im[K] - im[64 - K];       // 2 E
        const float orr = im[K] + im[64 - K], oi = re[64 - K] - re[K];      // 2 O = (Z_k - conj Z_{64-k}) / i
        const float tr = fmaf(c, orr, s * oi), ti = fmaf(c, oi, -s * orr);  // 2 W^k O
        re[K] = (er + tr) * cl[K];                // z[K]
        im[K] = (ei + ti) * cl[64 + K];           // z[64 + K]
        re[64 - K] = (er - tr) * cl[64 - K];      // z[64 - K]
        im[64 - K] = (ti - ei) * cl[128 - K];     // z[128 - K]
        unpack_pairs<K + 1>(re, im, cl);
    }
}

// x   : [n_vec][16] 16-byte units of fp16
// cl  : 128 floats: lambda_p times the packing constant of index p (1/sqrt d for DC and Nyquist, sqrt(2/d) / 2 elsewhere:
//       the 1/2 of the unpack is inside), then 4 dwords per row unit: sign-bit masks of the 128 inputs as packed fp16 pairs
// (one wavefront per SIMD with the whole register file: measured 103 us per 1,048,576 vectors against 128 us for two
// wavefronts per SIMD within 211 registers each)
__global__ void __launch_bounds__(64, 1)
srft_quantize_butterfly_kernel(const float* __restrict__ cl, const uint4* __restrict__ x, long long n_vec,
                               uint4* __restrict__ codes, float4* __restrict__ scales) {
    constexpr int U = 16, ROW = U + 1;
    __shared__ uint4 tile[64 * ROW];
    const int lane = threadIdx.x;
    const long long n_blocks = (n_vec + 63) / 64;
    const uint4* masks = reinterpret_cast<const uint4*>(cl + 128);
    for (long long blk = blockIdx.x; blk < n_blocks; blk += gridDim.x) {
        const long long row0 = blk * 64;
        const int lim = (int)min((long long)63, n_vec - 1 - row0);       // rows past the end alias to the last row
        // 1. coalesced load, through LDS, to one row per lane
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int u = lane + 64 * i, r = u / U, c = u % U;
            tile[r * ROW + c] = x[(row0 + min(r, lim)) * U + c];
        }
        __syncthreads();
        float re[64], im[64];
#pragma unroll
        for (int c = 0; c < U; ++c) {
            uint4 v = tile[lane * ROW + c];
            const uint4 m = masks[c];
            v.x ^= m.x; v.y ^= m.y; v.z ^= m.z; v.w ^= m.w;               // u = s * x
            const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {                                 // pair m = 4 c + j: (u_2m, u_2m+1), bit-reversed place
                const half2v h = __builtin_bit_cast(half2v, w[j]);
                re[bit_reverse6(4 * c + j)] = (float)h[0];
                im[bit_reverse6(4 * c + j)] = (float)h[1];
            }
        }
        __syncthreads();                         // the tile is free for the next step's loads
        // 3. complex FFT of length 64
        fft64_stage<2>(re, im);
        fft64_stage<4>(re, im);
        fft64_stage<8>(re, im);
        fft64_stage<16>(re, im);
        fft64_stage<32>(re, im);
        fft64_stage<64>(re, im);
        // 4. Hermitian unpack and the packing of Eq. 2, times lambda, in place: z_p = re[p] (p < 64), im[p - 64] (p >= 64)
        {
            const float dc = (re[0] + im[0]) * cl[0];        // DC: sum of all inputs
            const float ny = (re[0] - im[0]) * cl[64];       // Nyquist: even minus odd inputs
            re[0] = dc;
            im[0] = ny;
            re[32] = re[32] * cl[32];            // bin 32: W^32 = -i, Y = E - i O with E = Re Z_32, O = Im Z_32
            im[32] = -im[32] * cl[96];
        }
        unpack_pairs<1>(re, im, cl);
        // 5. quantizer, one group of 32 packed indices after the other
        uint32_t packed[16];
        float sc[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float* zg = j < 2 ? &re[32 * j] : &im[32 * (j - 2)];
            float mx = fmaxf(fabsf(zg[0]), fabsf(zg[1]));
#pragma unroll
            for (int v = 2; v < 32; ++v) mx = fmaxf(mx, fabsf(zg[v]));
            float scale = mx * (1.0f / 7.0f);
            float inv = __builtin_amdgcn_rcpf(scale);
            if (!(scale >= kMinScale)) { scale = 0.0f; inv = 0.0f; }
            sc[j] = scale;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                constexpr float kMagic = 12582912.0f + 8.0f;
                constexpr uint32_t kMagicBits = 0x4B400000u;
                const float* f = &zg[8 * q];
                uint32_t p = __float_as_uint(fmaf(f[7], inv, kMagic));
#pragma unroll
                for (int i = 6; i >= 0; --i) p = shl4_add(p, __float_as_uint(fmaf(f[i], inv, kMagic)));
                uint32_t k = 0;
#pragma unroll
                for (int i = 0; i < 8; ++i) k += kMagicBits << (4 * i);
                packed[4 * j + q] = (p - k) ^ 0x88888888u;
            }
        }
        // 6. stores: 64 code bytes and 4 scales per lane (lanes past the end rewrite the last row with the same bytes)
        const long long row = row0 + min(lane, lim);
#pragma unroll
        for (int i = 0; i < 4; ++i)
            codes[row * 4 + i] = make_uint4(packed[4 * i], packed[4 * i + 1], packed[4 * i + 2], packed[4 * i + 3]);
        scales[row] = make_float4(sc[0], sc[1], sc[2], sc[3]);
    }
}

}  // namespace

int srft_launch_quantize_butterfly(const float* table_dev, const void* x, long long n_vec, uint8_t* codes, float* scales,
                                   int max_workgroups, hipStream_t st) {
    int blocks = 0, dev = 0, cus = 0;
    SRFT_HIP(hipOccupancyMaxActiveBlocksPerMultiprocessor(&blocks, srft_quantize_butterfly_kernel, 64, 0));
    SRFT_HIP(hipGetDevice(&dev));
    SRFT_HIP(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
    long long grid = max_workgroups > 0 ? max_workgroups : (long long)cus * (blocks > 0 ? blocks : 1);
    const long long n_blocks = (n_vec + 63) / 64;
    if (grid > n_blocks) grid = n_blocks;
    hipLaunchKernelGGL(srft_quantize_butterfly_kernel, dim3((unsigned)grid), dim3(64), 0, st, table_dev,
                       (const uint4*)x, n_vec, (uint4*)codes, (float4*)scales);
    SRFT_HIP(hipGetLastError());
    return SRFT_OK;
}
