// quantize_tiles.h -- write path, plain form: the kernel template and its per-plan and batched kernels.
#ifndef SRFT_QUANTIZE_TILES_H
#define SRFT_QUANTIZE_TILES_H
#include "device_util.h"

// ------------------------------------------------------------------------------------------
// write path
// ------------------------------------------------------------------------------------------
// wfrag : [D/32 slabs][D/16 k-steps][hi, lo][64 lanes] 16-byte A-operand fragments of W
// x     : [n_vec][D/8] 16-byte units of fp16 input
// S     : slabs (= quantization groups) per wavefront; the workgroup has D / (32 S) wavefronts.  With S = 2
//         every B fragment read from LDS feeds four MFMAs instead of two and half as many wavefronts read the
//         tile; the price is a 2 x larger register-resident slab (at d = 256 it only fits with one wavefront
//         per SIMD, the slab in the accumulation half of the register file).
// OUT   : kOutCodes: the quantizer.  kOutRaw: store the fp32 coefficients w instead (srft_kv_forward_f32).
//         kOutAmax: no per-vector output; every lane keeps the running maximum of |w| of its 16 channels over the
//         tiles it sees, lanes are reduced once at the end and one atomic max per channel and workgroup goes
//         to wout, read as float[d] (srft_kv_channel_absmax: the statistic lambda is calibrated from, Sec. 7.1).
//         kOutQFrag32 / kOutQFrag16: the vectors are queries of srft_kv_scores (one tile at most): w times
//         scales[p] (there: 1 / (lambda max(lambda, 1e-6))), split into fp16 hi + lo and stored to wout as the
//         A fragments of the scores kernel with 32 or 16 rows of queries (layouts described there).
// GM    : group mode.  kGroup32: one scale per slab (g = 32, the deployed format).  kGroup16: one scale per
//         lane (g = 16; a lane's 16 outputs are one group, no cross-lane step).  kGroupWide: g = 32 * gw with
//         gw >= 2 slabs per group, up to the per-token case g = d; the slab maxima meet in LDS, which costs
//         two more barriers per tile.
// The work of one workgroup: tiles t0, t0 + stride, ... of one plan's n_vec vectors (t0 < number of tiles).
// BITS  : 4 (two nibbles per byte) or 8 (one byte per value, scale = abs-max / 127; Sec. 3.2 steps 3-4)
template <int D, int S, int OUT, int GM, int BITS>
__device__ __forceinline__ void
srft_quantize_tiles(const uint4* __restrict__ wfrag, const uint4* __restrict__ x, long long n_vec,
                    uint2* __restrict__ codes, float* __restrict__ scales, float4* __restrict__ wout,
                    float unscale, float scale_mul, int gw, const int t0, const int stride) {
    constexpr int G = D / 32;            // quantization groups per vector = slabs of the matrix
    constexpr int T = D / 16;            // MFMA k-steps
    constexpr int U = D / 8;             // 16-byte units per input row
    constexpr int ROW = U + 1;           // padded LDS row (odd number of units: conflict-free b128 reads)
    constexpr int NT = 64 * G / S;       // threads per workgroup
    constexpr int PER = 2 * S;           // 16-byte units each thread moves per tile (32 * U = PER * NT)
    constexpr int TB = (T < 8) ? T : 8;  // B fragments read from LDS ahead of their MFMAs
    static_assert(G % S == 0, "slabs per wavefront must divide the number of groups");
    __shared__ uint4 lds[2][kTileVecs * ROW];
    __shared__ float gmax[GM == kGroupWide ? kTileVecs * G : 1];     // per (vector, slab) abs-max

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane & 31, half = lane >> 5;
    // tile indices are 32-bit (the host bounds n_vec), so that the uniform index arithmetic stays scalar
    const int n_tiles = (int)((n_vec + kTileVecs - 1) / kTileVecs);
    const int last_lim = (int)(n_vec - 1 - (long long)(n_tiles - 1) * kTileVecs);   // last valid row of the last tile

    half8 ahi[S][T], alo[S][T];
#pragma unroll
    for (int s = 0; s < S; ++s)
#pragma unroll
        for (int t = 0; t < T; ++t) {
            ahi[s][t] = __builtin_bit_cast(half8, wfrag[(((wave * S + s) * T + t) * 2 + 0) * 64 + lane]);
            alo[s][t] = __builtin_bit_cast(half8, wfrag[(((wave * S + s) * T + t) * 2 + 1) * 64 + lane]);
        }

    // The PER prefetched units of one tile live in separately named registers (PER = 2 uses a and b only).
    // Addresses are a uniform tile base (scalar registers) plus a 32-bit per-lane offset; rows past the end
    // alias to the last row through `lim`, the index of the last valid row of the tile (uniform).
    auto fetch1 = [&](uint4& v, int i, const uint4* tile_base, int lim) __attribute__((always_inline)) {
        const int u = tid + i * NT, r = u / U, c = u % U;
        v = tile_base[(unsigned)(min(r, lim) * U + c)];
    };
    auto fetch = [&](uint4& a, uint4& b, uint4& c, uint4& d, int tile) __attribute__((always_inline)) {
        if (tile > n_tiles - 1) tile = n_tiles - 1;          // prefetch past the end re-reads the last tile
        const long long row0 = (long long)tile * kTileVecs;
        const int lim = (tile == n_tiles - 1) ? last_lim : kTileVecs - 1;
        const uint4* tile_base = x + row0 * U;
        fetch1(a, 0, tile_base, lim);
        fetch1(b, 1, tile_base, lim);
        if constexpr (PER > 2) { fetch1(c, 2, tile_base, lim); fetch1(d, 3, tile_base, lim); }
    };
    auto put1 = [&](int buf, const uint4& v, int i) __attribute__((always_inline)) {
        const int u = tid + i * NT, r = u / U, c = u % U;
        lds[buf][r * ROW + c] = v;
    };
    auto to_lds = [&](int buf, const uint4& a, const uint4& b, const uint4& c, const uint4& d) __attribute__((always_inline)) {
        put1(buf, a, 0);
        put1(buf, b, 1);
        if constexpr (PER > 2) { put1(buf, c, 2); put1(buf, d, 3); }
    };
    float cmax[OUT == kOutAmax ? S : 1][16] = {};            // running per-channel maxima (kOutAmax)
    if constexpr (OUT == kOutQFrag32 || OUT == kOutQFrag16) {
        // the scores set-up launch (one workgroup) also clears the row maxima that the scan will update with atomic
        // maxima, when the caller wants them: `codes` then points to kRowMaxCopies x 32 words
        if (codes) {                             // uniform
            unsigned int* words = reinterpret_cast<unsigned int*>(codes);
            for (int i = tid; i < kRowMaxCopies * 32; i += NT) words[i] = 0u;
        }
    }
    using Acc = Accs<S>;
    auto contract = [&](int b, Acc& accs) __attribute__((always_inline)) {
        const uint4* rowp = &lds[b][col * ROW + half];
        each_acc(accs, [&](floatx16& acc, int) __attribute__((always_inline)) { acc = floatx16{0}; });
#pragma unroll
        for (int t0 = 0; t0 < T; t0 += TB) {
            half8 bf[TB];
#pragma unroll
            for (int t = 0; t < TB; ++t)
                if (t0 + t < T) bf[t] = __builtin_bit_cast(half8, rowp[2 * (t0 + t)]);
#pragma unroll
            for (int t = 0; t < TB; ++t)
                if (t0 + t < T) {
                    each_acc(accs, [&](floatx16& acc, int s) __attribute__((always_inline)) {
                        acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(ahi[s][t0 + t], bf[t], acc, 0, 0, 0);
                        acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(alo[s][t0 + t], bf[t], acc, 0, 0, 0);
                    });
                }
        }
    };
    // vector-ALU tail of one tile: per-group abs-max, scale, int4 codes, stores
    auto finish = [&](Acc& accs, int tile) __attribute__((always_inline)) {
        const long long row0 = (long long)tile * kTileVecs;
        const int lim = (tile == n_tiles - 1) ? last_lim : kTileVecs - 1;     // uniform
        const int c = min(col, lim);                                      // alias rows past the end
        if constexpr (OUT == kOutAmax) {
            // rows past the end repeat the last row, which changes no maximum
            each_acc(accs, [&](floatx16& acc, int s) __attribute__((always_inline)) {
#pragma unroll
                for (int v = 0; v < 16; ++v) cmax[s][v] = fmaxf(cmax[s][v], fabsf(acc[v]));
            });
        } else if constexpr (OUT == kOutQFrag32 || OUT == kOutQFrag16) {
            // lane (query col, half) holds the packed indices p0 .. p0 + 15 of its query: code units p0 / 8 and
            // p0 / 8 + 1, whole.  Fragment element e of a unit is packed index 8 unit + e / 2 + 4 (e % 2) (the
            // 4-bit decode order of the read path).  Rows of queries that do not exist are zero.
            uint4* frag = reinterpret_cast<uint4*>(wout);
            const int q = col;
            each_acc(accs, [&](floatx16& acc, int s) __attribute__((always_inline)) {
                const int p0 = 32 * (wave * S + s) + 16 * half;
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    half8 hi, lo;
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const int pp = 8 * i + (e / 2) + 4 * (e % 2);
                        const float v = q <= lim ? (acc[pp] * unscale) * scales[p0 + pp] : 0.0f;
                        hi[e] = (_Float16)v;
                        lo[e] = (_Float16)(v - (float)hi[e]);
                    }
                    const int u = p0 / 8 + i;
                    if constexpr (OUT == kOutQFrag16) {
                        // MFMA row 4 a + i' carries query 2 i' + a (a < 2) or 8 + 2 i' + (a - 2); lane = 16 (u % 4) + row
                        const int row = q < 8 ? 4 * (q % 2) + q / 2 : 4 * (2 + q % 2) + (q - 8) / 2;
                        if (q < 16) {
                            frag[((u / 4) * 2 + 0) * 64 + 16 * (u % 4) + row] = __builtin_bit_cast(uint4, hi);
                            frag[((u / 4) * 2 + 1) * 64 + 16 * (u % 4) + row] = __builtin_bit_cast(uint4, lo);
                        }
                    } else {
                        // MFMA row 8 (v / 4) + 4 h + v % 4 carries query 2 v + h; lane = 32 (u % 2) + row
                        const int row = 8 * ((q / 2) / 4) + 4 * (q % 2) + (q / 2) % 4;
                        frag[((u / 2) * 2 + 0) * 64 + 32 * (u % 2) + row] = __builtin_bit_cast(uint4, hi);
                        frag[((u / 2) * 2 + 1) * 64 + 32 * (u % 2) + row] = __builtin_bit_cast(uint4, lo);
                    }
                }
            });
        } else if constexpr (OUT == kOutRaw) {
            each_acc(accs, [&](floatx16& acc, int s) __attribute__((always_inline)) {
                const int slab = wave * S + s;
                float4* o = wout + (row0 * D) / 4 + (unsigned)((c * D + 32 * slab + 16 * half) / 4);
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    o[i] = make_float4(acc[4 * i] * unscale, acc[4 * i + 1] * unscale,
                                       acc[4 * i + 2] * unscale, acc[4 * i + 3] * unscale);
            });
        } else {
            float mm[S];
            each_acc(accs, [&](floatx16& acc, int s) __attribute__((always_inline)) {
                float m = fmaxf(fabsf(acc[0]), fabsf(acc[1]));
#pragma unroll
                for (int v = 2; v < 16; ++v) m = fmaxf(m, fabsf(acc[v]));
                if constexpr (GM != kGroup16) m = other_half_max(m);
                mm[s] = m;
            });
            if constexpr (GM == kGroupWide) {
                __syncthreads();                             // the previous tile's maxima have been read
#pragma unroll
                for (int s = 0; s < S; ++s) gmax[col * G + wave * S + s] = mm[s];
                __syncthreads();
#pragma unroll
                for (int s = 0; s < S; ++s) {
                    const int first = (wave * S + s) / gw * gw;
                    float m = gmax[col * G + first];
                    for (int i = 1; i < gw; ++i) m = fmaxf(m, gmax[col * G + first + i]);
                    mm[s] = m;
                }
            }
            each_acc(accs, [&](floatx16& acc, int s) __attribute__((always_inline)) {
                const int slab = wave * S + s;
                float scale = mm[s] * scale_mul;             // scale_mul = fl(2^-e / 7): abs-max / 7
                float inv = unscale * __builtin_amdgcn_rcpf(scale);
                if (!(scale >= kMinScale)) { scale = 0.0f; inv = 0.0f; }
                if constexpr (BITS == 8) {       // 16 bytes per lane; a row is D / 16 such units
                    const uint4 packed = make_uint4(pack4_bytes(acc, 0, inv), pack4_bytes(acc, 4, inv),
                                                    pack4_bytes(acc, 8, inv), pack4_bytes(acc, 12, inv));
                    (reinterpret_cast<uint4*>(codes) + row0 * (D / 16))[(unsigned)(c * (D / 16) + 2 * slab + half)] = packed;
                } else {
                    uint2 packed;
                    packed.x = pack8(acc, 0, inv);
                    packed.y = pack8(acc, 8, inv);
                    (codes + row0 * (D / 16))[(unsigned)(c * (D / 16) + 2 * slab + half)] = packed;
                }
                // lanes that hold the same group store the same value to the same place
                if constexpr (GM == kGroup16) (scales + row0 * (2 * G))[(unsigned)(c * (2 * G) + 2 * slab + half)] = scale;
                else if constexpr (GM == kGroup32) (scales + row0 * G)[(unsigned)(c * G + slab)] = scale;
                else (scales + row0 * (G / gw))[(unsigned)(c * (G / gw) + slab / gw)] = scale;
            });
        }
    };

    const int m = (n_tiles - 1 - t0) / stride + 1;           // tiles of this workgroup
    uint4 pa0, pa1, pa2, pa3, pb0, pb1, pb2, pb3;
    Acc acc_a, acc_b;
    fetch(pa0, pa1, pa2, pa3, t0);
    fetch(pb0, pb1, pb2, pb3, t0 + stride);
    hold_in_registers(ahi, alo);                 // the matrix slab has arrived before the pipeline starts
    to_lds(0, pa0, pa1, pa2, pa3);
    fetch(pa0, pa1, pa2, pa3, t0 + 2 * stride);
    // stage 0
    __syncthreads();
    contract(0, acc_a);
    to_lds(1, pb0, pb1, pb2, pb3);
    fetch(pb0, pb1, pb2, pb3, t0 + 3 * stride);
    int k = 1;
    for (; k + 1 < m; k += 2) {
        const int tk = t0 + k * stride;
        __syncthreads();                         // stage k (odd)
        rotate_priority(k);
        contract(1, acc_b);
        finish(acc_a, tk - stride);
        to_lds(0, pa0, pa1, pa2, pa3);
        fetch(pa0, pa1, pa2, pa3, tk + 3 * stride);
        __syncthreads();                         // stage k + 1 (even)
        rotate_priority(k + 1);
        contract(0, acc_a);
        finish(acc_b, tk);
        to_lds(1, pb0, pb1, pb2, pb3);
        fetch(pb0, pb1, pb2, pb3, tk + 4 * stride);
    }
    if (k < m) {                                 // one more odd stage
        const int tk = t0 + k * stride;
        __syncthreads();
        contract(1, acc_b);
        finish(acc_a, tk - stride);
        finish(acc_b, tk);
    } else {
        finish(acc_a, t0 + (k - 1) * stride);
    }
    if constexpr (OUT == kOutAmax) {
        // lanes of one half hold the same 16 channels for 32 different vectors: butterfly over the 32, then one
        // atomic per channel (non-negative floats order like their bit patterns)
        unsigned int* amax = reinterpret_cast<unsigned int*>(wout);
#pragma unroll
        for (int s = 0; s < S; ++s)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                float mx = cmax[s][v];
#pragma unroll
                for (int step = 1; step < 32; step *= 2) mx = fmaxf(mx, __shfl_xor(mx, step, 64));
                if (col == 0) atomic_max_nonneg(&amax[32 * (wave * S + s) + 16 * half + v], mx * unscale);
            }
    }
}

template <int D, int S, int OUT, int GM, int BITS>
__global__ void __launch_bounds__(2 * D / S)
srft_quantize_kernel(const uint4* __restrict__ wfrag, const uint4* __restrict__ x, long long n_vec,
                     uint2* __restrict__ codes, float* __restrict__ scales, float4* __restrict__ wout,
                     float unscale, float scale_mul, int gw) {
    srft_quantize_tiles<D, S, OUT, GM, BITS>(wfrag, x, n_vec, codes, scales, wout, unscale, scale_mul, gw, blockIdx.x,
                                       gridDim.x);       // the grid never exceeds the number of tiles
}

// Several plans in one launch: segment i of the table is served by workgroups first_block[i] .. first_block[i+1]-1.
template <int D, int S, int GM, int BITS>
__global__ void __launch_bounds__(2 * D / S)
srft_quantize_batched_kernel(const srft_batch_args a, int gw) {
    const int i = srft_segment_of_block(a, blockIdx.x);
    srft_quantize_tiles<D, S, kOutCodes, GM, BITS>(a.frag[i], (const uint4*)a.in0[i], a.n_vec[i], (uint2*)a.out0[i],
                                         (float*)a.out1[i], nullptr, a.unscale[i],
                                         a.unscale[i] / (BITS == 8 ? 127.0f : 7.0f), gw,
                                         blockIdx.x - a.first_block[i], a.first_block[i + 1] - a.first_block[i]);
}

#endif  // SRFT_QUANTIZE_TILES_H
