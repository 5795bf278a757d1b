// Write path at d = 128 (and, further down, d = 256) with the transform as FFT butterflies on the vector ALU instead of a matrix-core
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


// ---- d = 256: one vector on two lanes ------------------------------------------------------------------------
// 256 fp32 values and the temporaries of the transform do not fit one lane, so lanes l and l + 32 share vector l
// (32 vectors per wavefront and step).  The complex FFT of length 128 over z_m = u_2m + i u_2m+1 is split by one
// decimation-in-time step: lane part 0 transforms the even m (A), part 1 the odd m (B), each a length-64 FFT in
// registers (the same code as above).  One v_permlane32_swap of a register with itself leaves the lower lanes' value
// and the upper lanes' value in both lanes, so every pair index j = 0 .. 32 is worked by both lanes from the same four
// values A_j, B_j, A_{64-j}, B_{64-j} with the same compile-time twiddles, without LDS:
//   Z_j = A_j + W^j B_j,  Z_{64+j} = A_j - W^j B_j,  Z_{64-j} = A_{64-j} + W^{64-j} B_{64-j},  Z_{128-j} = A_{64-j} - ...
// Part 0 takes the pair of bins (j, 128 - j), part 1 the pair (64 - j, 64 + j), whose unpack twiddle exp(-2 pi i k/256)
// at k = 64 - j is the one at k = j with cosine and sine exchanged.  Each pair consumes four registers and gives four
// packed values; they land in four groups per lane -- part 0: packed 0..31, 128..159, 96..127, 224..255; part 1:
// 64..95, 192..223, 32..63, 160..191 -- so the quantizer stays inside the lane.  j = 0 gives DC and Nyquist (part 0)
// and the two values of bin 64 (part 1).
//
// cl: 256 floats as for d = 128 (bins 0 and 64 are the ones without the factor 1/2), then 32 x 4 dwords of sign masks.

// the lower lanes' (part 0) and the upper lanes' (part 1) value of v, in every lane
__device__ __forceinline__ void both_parts(float v, float& lower, float& upper) {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    lower = __uint_as_float(r[0]);
    upper = __uint_as_float(r[1]);
}

// pair j of the two-lane unpack; X / Xi collect positions j, Y / Yi positions 32 - j of this lane's four groups
template <int J>
__device__ __forceinline__ void unpack256(float (&X)[32], float (&Xi)[32], float (&Y)[32], float (&Yi)[32],
                                          const float (&re)[64], const float (&im)[64],
                                          const float4* __restrict__ clp, bool part) {
    if constexpr (J <= 32) {
        constexpr float c1 = (float)cos_turn(J, 128), s1 = (float)sin_turn(J, 128);            // W_128^J
        constexpr float c2 = (float)cos_turn(64 - J, 128), s2 = (float)sin_turn(64 - J, 128);  // W_128^(64-J)
        constexpr float cu = (float)cos_turn(J, 256), su = (float)sin_turn(J, 256);            // W_256^J
        float ar, ai, br, bi, ar2, ai2, br2, bi2;
        both_parts(re[J], ar, br);
        both_parts(im[J], ai, bi);
        both_parts(re[64 - J], ar2, br2);
        both_parts(im[64 - J], ai2, bi2);
        const float tr1 = fmaf(c1, br, s1 * bi), ti1 = fmaf(c1, bi, -s1 * br);
        const float tr2 = fmaf(c2, br2, s2 * bi2), ti2 = fmaf(c2, bi2, -s2 * br2);
        // part 0: (Z_J, Z_{128-J});  part 1: (Z_{64-J}, Z_{64+J})
        const float zkr = part ? ar2 + tr2 : ar + tr1, zki = part ? ai2 + ti2 : ai + ti1;
        const float zmr = part ? ar - tr1 : ar2 - tr2, zmi = part ? ai - ti1 : ai2 - ti2;
        const float c = part ? su : cu, s = part ? cu : su;                                     // W_256^k, k = J or 64 - J
        const float er = zkr + zmr, ei = zki - zmi;
        const float orr = zki + zmi, oi = zmr - zkr;
        const float tr = fmaf(c, orr, s * oi), ti = fmaf(c, oi, -s * orr);
        const float4 k4 = clp[J];                   // lambda and packing constants of bins k (re, im) and 128 - k (re, im)
        const float skr = (er + tr) * k4.x, ski = (ei + ti) * k4.y, smr = (er - tr) * k4.z, smi = (ti - ei) * k4.w;
        if constexpr (J < 32) {
            X[J] = part ? smr : skr;
            Xi[J] = part ? smi : ski;
        }
        Y[32 - J] = part ? skr : smr;
        Yi[32 - J] = part ? ski : smi;
        unpack256<J + 1>(X, Xi, Y, Yi, re, im, clp, part);
    }
}

// abs-max, scale and nibble pack of one group of 32 values held by a lane
__device__ __forceinline__ void quantize_group32(const float (&z)[32], uint4& packed, float& scale_out) {
    float mx = fmaxf(fabsf(z[0]), fabsf(z[1]));
#pragma unroll
    for (int v = 2; v < 32; ++v) mx = fmaxf(mx, fabsf(z[v]));
    float scale = mx * (1.0f / 7.0f);
    float inv = __builtin_amdgcn_rcpf(scale);
    if (!(scale >= kMinScale)) { scale = 0.0f; inv = 0.0f; }
    scale_out = scale;
    uint32_t w[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        constexpr float kMagic = 12582912.0f + 8.0f;
        constexpr uint32_t kMagicBits = 0x4B400000u;
        uint32_t p = __float_as_uint(fmaf(z[8 * q + 7], inv, kMagic));
#pragma unroll
        for (int i = 6; i >= 0; --i) p = shl4_add(p, __float_as_uint(fmaf(z[8 * q + i], inv, kMagic)));
        uint32_t k = 0;
#pragma unroll
        for (int i = 0; i < 8; ++i) k += kMagicBits << (4 * i);
        w[q] = (p - k) ^ 0x88888888u;
    }
    packed = make_uint4(w[0], w[1], w[2], w[3]);
}

// (one wavefront per SIMD: within 256 registers the compiler spills 444 bytes and the kernel is a quarter slower)
__global__ void __launch_bounds__(64, 1)
srft_quantize_butterfly256_kernel(const float* __restrict__ cl, const uint4* __restrict__ x, long long n_vec,
                                  uint4* __restrict__ codes, float* __restrict__ scales) {
    constexpr int U = 32, ROW = U + 1;           // 16-byte units per input row, padded
    __shared__ uint4 tile[32 * ROW];
    __shared__ float4 clp_s[2][33];
    const int lane = threadIdx.x, vec = lane & 31;
    const bool part = lane >= 32;
    // constants of the pairs, per part: bins k and 128 - k with k = j (part 0) or 64 - j (part 1); j = 0: bins 0, 128, 64, 192
    for (int t = lane; t < 66; t += 64) {
        const int pt = t / 33, j = t % 33, k = pt ? 64 - j : j;
        clp_s[pt][j] = j == 0 ? make_float4(cl[0], cl[128], cl[64], cl[192])
                              : make_float4(cl[k], cl[128 + k], cl[128 - k], cl[256 - k]);
    }
    const uint4* masks = reinterpret_cast<const uint4*>(cl + 256);
    const long long n_blocks = (n_vec + 31) / 32;
    for (long long blk = blockIdx.x; blk < n_blocks; blk += gridDim.x) {
        const long long row0 = blk * 32;
        const int lim = (int)min((long long)31, n_vec - 1 - row0);       // rows past the end alias to the last row
        __syncthreads();                         // the tile of the previous step has been read
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int u = lane + 64 * i, r = u / U, c = u % U;
            tile[r * ROW + c] = x[(row0 + min(r, lim)) * U + c];
        }
        __syncthreads();
        float re[64], im[64];
#pragma unroll
        for (int c = 0; c < U; ++c) {            // unit c holds the complex samples m = 4c .. 4c+3; this lane takes m = 2j + part
            uint4 v = tile[vec * ROW + c];
            const uint4 m = masks[c];
            v.x ^= m.x; v.y ^= m.y; v.z ^= m.z; v.w ^= m.w;               // u = s * x
            const half2v h0 = __builtin_bit_cast(half2v, part ? v.y : v.x);   // j = 2c
            const half2v h1 = __builtin_bit_cast(half2v, part ? v.w : v.z);   // j = 2c + 1
            re[bit_reverse6(2 * c)] = (float)h0[0];
            im[bit_reverse6(2 * c)] = (float)h0[1];
            re[bit_reverse6(2 * c + 1)] = (float)h1[0];
            im[bit_reverse6(2 * c + 1)] = (float)h1[1];
        }
        fft64_stage<2>(re, im);
        fft64_stage<4>(re, im);
        fft64_stage<8>(re, im);
        fft64_stage<16>(re, im);
        fft64_stage<32>(re, im);
        fft64_stage<64>(re, im);
        const float4* clp = clp_s[part ? 1 : 0];
        float X[32], Xi[32], Y[32], Yi[32];
        {
            float a0r, b0r, a0i, b0i;
            both_parts(re[0], a0r, b0r);
            both_parts(im[0], a0i, b0i);
            const float pr = a0r + b0r, pi = a0i + b0i;                   // Z_0
            const float qr = a0r - b0r, qi = a0i - b0i;                   // Z_64
            const float4 k4 = clp[0];
            X[0] = part ? qr * k4.z : (pr + pi) * k4.x;                   // bin 64 (real part) | DC
            Xi[0] = part ? -qi * k4.w : (pr - pi) * k4.y;                 // bin 64 (imaginary part) | Nyquist
        }
        unpack256<1>(X, Xi, Y, Yi, re, im, clp, part);
        uint4 pk[4];
        float sc[4];
        quantize_group32(X, pk[0], sc[0]);
        quantize_group32(Xi, pk[1], sc[1]);
        quantize_group32(Y, pk[2], sc[2]);
        quantize_group32(Yi, pk[3], sc[3]);
        // groups of this lane: X, Xi, Y, Yi = 0, 4, 3, 7 (part 0) or 2, 6, 1, 5 (part 1)
        const int g0 = part ? 2 : 0, g1 = part ? 6 : 4, g2 = part ? 1 : 3, g3 = part ? 5 : 7;
        const long long row = row0 + min(vec, lim);       // lanes past the end rewrite the last row with the same bytes
        codes[row * 8 + g0] = pk[0];
        codes[row * 8 + g1] = pk[1];
        codes[row * 8 + g2] = pk[2];
        codes[row * 8 + g3] = pk[3];
        scales[row * 8 + g0] = sc[0];
        scales[row * 8 + g1] = sc[1];
        scales[row * 8 + g2] = sc[2];
        scales[row * 8 + g3] = sc[3];
    }
}

}  // namespace

int srft_launch_quantize_butterfly(int d, const float* table_dev, const void* x, long long n_vec, uint8_t* codes,
                                   float* scales, int max_workgroups, hipStream_t st) {
    int blocks = 0, dev = 0, cus = 0;
    const int per_block = d == 256 ? 32 : 64;    // vectors per wavefront and step
    if (d == 256) SRFT_HIP(hipOccupancyMaxActiveBlocksPerMultiprocessor(&blocks, srft_quantize_butterfly256_kernel, 64, 0));
    else SRFT_HIP(hipOccupancyMaxActiveBlocksPerMultiprocessor(&blocks, srft_quantize_butterfly_kernel, 64, 0));
    SRFT_HIP(hipGetDevice(&dev));
    SRFT_HIP(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
    long long grid = max_workgroups > 0 ? max_workgroups : (long long)cus * (blocks > 0 ? blocks : 1);
    const long long n_blocks = (n_vec + per_block - 1) / per_block;
    if (grid > n_blocks) grid = n_blocks;
    if (d == 256)
        hipLaunchKernelGGL(srft_quantize_butterfly256_kernel, dim3((unsigned)grid), dim3(64), 0, st, table_dev,
                           (const uint4*)x, n_vec, (uint4*)codes, scales);
    else
        hipLaunchKernelGGL(srft_quantize_butterfly_kernel, dim3((unsigned)grid), dim3(64), 0, st, table_dev,
                           (const uint4*)x, n_vec, (uint4*)codes, (float4*)scales);
    SRFT_HIP(hipGetLastError());
    return SRFT_OK;
}
