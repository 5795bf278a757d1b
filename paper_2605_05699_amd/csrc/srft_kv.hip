// srft_kv.hip -- fused SRFT int4 KV-cache quantizer / dequantizer for MI355X (gfx950).
//
// How the path is mapped to CDNA4
// -------------------------------
// Per vector the method is: sign flip, unitary real DFT with the real packing of Eq. 2, per-channel
// lambda, per-group abs-max, round to int4, nibble pack (Sec. 3.2, Sec. 5.1, Sec. 7.1).  Sign, DFT,
// packing and lambda are all linear, so together they are ONE real d x d matrix
//     W = diag(lambda) * Q * diag(s),        Q = pack o F   (orthogonal),
// and the read path is the matrix  R = diag(s) * Q^T * diag(1 / max(lambda, 1e-6)).
// At 5.6 TB/s a d = 128 vector has about 37 compute-unit clocks; a butterfly FFT plus the fp16
// conversions needs about 3000 vector-ALU lane operations per vector, more than the 64 lanes x 37
// clocks available, whereas the matrix cores do the dense product with time to spare.  So the
// transform runs on MFMA (v_mfma_f32_32x32x16_f16) and the vector ALU only does the quantizer.
//
// Exactness: x is fp16, hence an exact MFMA operand.  W is split on the host into two fp16
// matrices W = Whi + Wlo (after a power-of-two scaling that keeps Wlo out of the fp16 denormal
// range); both products accumulate into the same fp32 accumulator, which gives about 22 bits of W.
// On the read path the codes (integers in [-8, 7]) are exact fp16 operands; the per-(vector, group)
// scale cannot enter the matrix, so each group's 32 codes are contracted separately (K = 32) and
// the partial results are combined as  x = sum_j scale_j * P_j  on the vector ALU in fp32.
//
// Work decomposition (plain forms): a workgroup has d/32 wavefronts and walks over tiles of 32 vectors
// (persistent grid).  Wavefront w owns the 32 output rows 32w..32w+31 -- on the write path that is
// exactly quantization group w, so the abs-max needs a single cross-lane step -- and keeps its
// 32 x d slab of the matrix (hi and lo) in registers for the whole launch.  The 32 x d operand tile
// (inputs, or decoded codes) is loaded once per workgroup with coalesced 16-byte accesses, staged in
// LDS (double buffered, one barrier per tile, reached by every thread) and read by every wavefront.
// The MFMA row order inside a slab is permuted on the host so that a lane ends up holding 16
// CONSECUTIVE outputs: 16 nibbles = one 8-byte store on the write path, 16 fp16 = two 16-byte
// stores on the read path, with no cross-lane shuffles.
//
// Folded forms (d = 128 and 256 on the write path, 128 / 192 / 256 on the read path): two symmetries of Q
// let every output pair share two half-length partial sums, which halves the matrix work; they are
// described at srft_quantize_fold_tiles and at the FOLD parameter of srft_dequantize_tiles.
//
// Around the two paths: the same kernels serving several plans in one launch (a segment table passed as a
// kernel argument), the per-channel abs-max statistic lambda is calibrated from, an 8-bit code width, the
// Walsh-Hadamard matrix in place of the DFT (the comparator of Sec. 3.1), scores of queries against the stored
// record without reconstructing the keys, and a host-side cache manager (int4 store, fp16 residual window,
// dequantized view) built on the batched launches.
//
// The kernels run at the socket's power limit with a throttled clock, so what shortens them is work per vector
// (matrix instructions, vector instructions, LDS traffic), not more parallelism: see the folded forms.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <cstdint>
#include <cstring>
#include <new>
#include <type_traits>
#include <vector>

#include "srft_kv.h"

namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

// Streaming (non-temporal) accesses for data touched once.  Measured: they help the read path (codes in, fp16
// rows out: +3 %) and hurt the write path (its 16-byte code pieces and 4-byte scales combine worse), so only the
// read path uses them.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ void stream_store(uint4* p, uint4 v) {
    __builtin_nontemporal_store(__builtin_bit_cast(u32x4, v), reinterpret_cast<u32x4*>(p));
}
__device__ __forceinline__ uint4 stream_load(const uint4* p) {
    return __builtin_bit_cast(uint4, __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p)));
}
__device__ __forceinline__ uint2 stream_load(const uint2* p) {
    return __builtin_bit_cast(uint2, __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(p)));
}

constexpr int kTileVecs = 32;          // vectors per tile = N of the 32x32x16 MFMA
constexpr int kMaxScoreWorkgroups = 4096;   // scores kernel: largest grid (each workgroup owns 256 bytes of workspace)
constexpr int kMaxD = 256;
#ifndef SRFT_LEAN_ALT_MAX
#define SRFT_LEAN_ALT_MAX 8              // read path: slabs x groups up to which two accumulator sets alternate
#endif
constexpr float kMinScale = 7.888609052210118e-31f;   // 2^-100: below this a group is stored as zero

// ------------------------------------------------------------------------------------------
// device helpers
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ float other_half_max(float m) {
    // lanes l and l^32 hold the two halves of one vector's group: one v_permlane32_swap.
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(m), __float_as_uint(m), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

// Make the loop-invariant matrix fragments "used" here, so that the wait for their loads is placed
// before the main loop and not inside it (where it would also wait for the loop's own prefetches).
template <int N>
__device__ __forceinline__ void hold_in_registers(half8 (&a)[N], half8 (&b)[N]) {
#pragma unroll
    for (int i = 0; i < N; ++i) asm volatile("" : "+v"(a[i]), "+v"(b[i]));
}
template <int N, int M>
__device__ __forceinline__ void hold_in_registers(half8 (&a)[N][M], half8 (&b)[N][M]) {
#pragma unroll
    for (int i = 0; i < N; ++i)
#pragma unroll
        for (int j = 0; j < M; ++j) asm volatile("" : "+v"(a[i][j]), "+v"(b[i][j]));
}

// The instruction arbiter of a compute unit favours its oldest wavefronts: of the workgroups that share a unit the
// one dispatched first ran 25 % ahead of the others and left the unit early, while the kernel waited for the
// last one.  Every workgroup therefore walks through the four wavefront priorities, one per stage, offset by its
// place in the dispatch order: over four stages each has held each priority once, and they finish together
// (end times of the workgroups 440..620 us -> 565..600 us at d = 128, 8 M vectors; launches 1.5-3.5 % shorter, the
// scores kernel 5-12 %).  Not used where two workgroups per unit take turns on one accumulator set (the folded
// write path at d = 256), which measured 1 % slower with it.
__device__ __forceinline__ void rotate_priority(int stage) {
    switch (((int)(blockIdx.x * 4 / gridDim.x) + stage) & 3) {
        case 0: __builtin_amdgcn_s_setprio(0); break;
        case 1: __builtin_amdgcn_s_setprio(1); break;
        case 2: __builtin_amdgcn_s_setprio(2); break;
        default: __builtin_amdgcn_s_setprio(3); break;
    }
}

template <int N> struct Accs;          // one 32x32 accumulator tile per slab, as named registers
template <> struct Accs<1> { floatx16 a; };
template <> struct Accs<2> { floatx16 a, b; };
template <class F> __device__ __forceinline__ void each_acc(Accs<1>& p, F f) { f(p.a, 0); }
template <class F> __device__ __forceinline__ void each_acc(Accs<2>& p, F f) { f(p.a, 0); f(p.b, 1); }

// Eight values already multiplied by 1/scale -> eight two's-complement nibbles in one dword.
// Adding 1.5*2^23 + 8 rounds to nearest-even and leaves q + 8 (1..15) in the low four bits above a
// constant bit pattern; a shift-add chain concatenates the nibbles (no borrows because q + 8 > 0),
// the constant is subtracted once and flipping bit 3 of each nibble turns q + 8 into q mod 16.
__device__ __forceinline__ uint32_t shl4_add(uint32_t p, uint32_t x) {
    uint32_t r;                                  // (p << 4) + x as ONE instruction (the compiler prefers shift + 3-way add)
    asm("v_lshl_add_u32 %0, %1, 4, %2" : "=v"(r) : "v"(p), "v"(x));
    return r;
}
__device__ __forceinline__ uint32_t pack8(const floatx16& acc, int base, float inv) {
    constexpr float kMagic = 12582912.0f + 8.0f;
    constexpr uint32_t kMagicBits = 0x4B400000u;
    uint32_t p = __float_as_uint(fmaf(acc[base + 7], inv, kMagic));
#pragma unroll
    for (int i = 6; i >= 0; --i) p = shl4_add(p, __float_as_uint(fmaf(acc[base + i], inv, kMagic)));
    uint32_t k = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) k += kMagicBits << (4 * i);
    return (p - k) ^ 0x88888888u;
}

// Four values already multiplied by 1/scale -> four two's-complement bytes in one dword (8-bit output).
// Adding 1.5 * 2^23 rounds to nearest-even and leaves q mod 256 in the low byte of the bit pattern.
__device__ __forceinline__ uint32_t pack4_bytes(const floatx16& acc, int base, float inv) {
    constexpr float kMagic = 12582912.0f;
    const uint32_t a = __float_as_uint(fmaf(acc[base], inv, kMagic)), b = __float_as_uint(fmaf(acc[base + 1], inv, kMagic));
    const uint32_t c = __float_as_uint(fmaf(acc[base + 2], inv, kMagic)), d = __float_as_uint(fmaf(acc[base + 3], inv, kMagic));
    const uint32_t lo = __builtin_amdgcn_perm(b, a, 0x0c0c0400u);       // byte 0 of a, byte 0 of b, 0, 0
    const uint32_t hi = __builtin_amdgcn_perm(d, c, 0x0c0c0400u);
    return (hi << 16) | lo;
}

// ------------------------------------------------------------------------------------------
// Both kernels are software pipelines over the tiles T_0, T_1, ... of a workgroup (T_k = blockIdx +
// k * gridDim).  Stage k starts with the only barrier of the stage and then, in ONE straight-line
// block, (1) contracts T_k from LDS buffer k % 2 on the matrix cores, (2) runs the vector-ALU tail of
// T_{k-1} (quantizer and stores, or scaling / conversion / stores) on the accumulators the previous
// stage left behind, and (3) moves T_{k+1} from its prefetch registers into LDS buffer (k+1) % 2 and
// refills those registers with T_{k+3}.  (1) and (2) are independent, so one wavefront keeps the MFMA
// pipe and the vector ALU busy together.  The barrier of stage k makes T_k visible and also proves
// that every wavefront has finished reading buffer (k+1) % 2, which (3) overwrites.
//
// Rows past the end of the input alias to the last row, in the loads AND in the stores: surplus lanes
// compute the last vector again and store the same bytes to the same place.  Prefetches past the last
// tile re-read the last tile.  So no memory operation in the loop is conditional, the hardware wait
// counters are exact, and stores and younger prefetches stay in flight while older data is consumed.
// Every branch in the kernels is uniform over the workgroup.
// ------------------------------------------------------------------------------------------

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
enum { kGroup16 = 0, kGroup32 = 1, kGroupWide = 2 };
enum { kOutCodes = 0, kOutRaw = 1, kOutAmax = 2, kOutQFrag32 = 3, kOutQFrag16 = 4 };
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
                if (col == 0) atomicMax(&amax[32 * (wave * S + s) + 16 * half + v], __float_as_uint(mx * unscale));
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

// ------------------------------------------------------------------------------------------
// write path, folded form: half the matrix work, for d a multiple of 128 and g = 32
// ------------------------------------------------------------------------------------------
// Rows k and d/2 - k of the cosine block of Q differ only by the factor (-1)^n, and so do (up to a sign)
// rows k and d/2 - k of the sine block.  With  E_k = sum over even n,  O_k = sum over odd n  of Q[k][n] u_n:
//     z_k       = E_k + O_k        z_{d/2-k}     =   E_k - O_k          (cosine block, packed index p = k)
//     z_{d/2+k} = E'_k + O'_k      z_{d-k}       = -(E'_k - O'_k)       (sine block)
// so only the rows k < d/4 are contracted, each over half of the inputs.  A workgroup has d/64 wavefronts: the
// first half owns the cosine block, the second half the sine block, 32 values of k each; a wavefront keeps an
// E slab (contracted with the even-n inputs) and an O slab (odd-n inputs), each 32 rows x d/2.  The inputs
// are split into even and odd positions when the tile is staged in LDS.  A lane holds k = 16 h + v (v < 16)
// and produces a "direct" run of 16 packed indices (ascending with v) and a "mirror" run (descending).
// lambda of the direct index is folded into the rows; the mirror value is rho_k (E - O) with
// rho = +-lambda_mirror / lambda_direct.
//
// The mirror run of a lane is p_top - 16h - v: one index above a 16-aligned block.  Each lane therefore takes
// the bottom element of its block from its neighbour: the h = 0 lane from the h = 1 lane of the same vector (one
// v_permlane32_swap), the h = 1 lane from another wavefront, through LDS (`xch`, one slot per group: the value of
// packed index 32 * slot).  The four indices without a partner go the same way: k = 0 gives DC (direct) and
// Nyquist (mirror top of the first cosine wavefront, slot d/64); the first sine wavefront has no k = 0 of its own
// and uses that row pair for the quarter bins, E = row d/4 and O = row 3d/4 (slots d/128 and 3d/128), and takes
// Nyquist as its direct element 0.  Values are exchanged already multiplied by their lambda.
// A tile's exchange values are written at the end of the stage that contracts it and read after the next
// barrier, in the stage that quantizes it.
//
// BITS: 4 or 8, as on the plain path.  WIDE: g = 32 gw with gw >= 2, up to the per-token case g = d: the maxima
// of the 32-runs meet in LDS (gmax), which costs one more barrier per tile, in the middle of the stage.
//
// wfold : [d/64 waves][E, O][d/32 k-steps][hi, lo][64 lanes] fragments, then [d/64 waves][64 lanes][4] x 4 floats rho
template <int D, int BITS, bool WIDE>
__device__ __forceinline__ void
srft_quantize_fold_tiles(const uint4* __restrict__ wfold, const uint4* __restrict__ x, long long n_vec,
                         uint2* __restrict__ codes, float* __restrict__ scales, float unscale, float scale_mul,
                         int gw, const int t0, const int stride) {
    constexpr int M = D / 64;            // wavefronts per workgroup
    constexpr int G = D / 32;            // groups per vector
    constexpr int T = D / 32;            // k-steps per slab (K = D / 2)
    constexpr int U = D / 8;             // 16-byte units per input row
    constexpr int ROW = U + 1;
    constexpr int NT = 64 * M;
    constexpr int DUMMY = 2 * M + 1;     // exchange slot for values nobody reads
    constexpr bool LEAN = (D >= 256);    // registers for one accumulator set only
    static_assert(M % 2 == 0, "the cosine and the sine block each need whole wavefronts");
    __shared__ uint4 lds[2][kTileVecs * ROW];
    __shared__ float xch[2][(DUMMY + 1) * kTileVecs];
    __shared__ float gmax[WIDE ? 2 : 1][WIDE ? kTileVecs * G : 1];     // maxima of the 32-runs of a tile (WIDE)

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane & 31, half = lane >> 5;
    const int n_tiles = (int)((n_vec + kTileVecs - 1) / kTileVecs);
    const int last_lim = (int)(n_vec - 1 - (long long)(n_tiles - 1) * kTileVecs);
    const bool sine = wave >= M / 2;
    const int wk = sine ? wave - M / 2 : wave;               // which 32 values of k
    const bool quarter = (wave == M / 2);                    // the wavefront that carries the quarter bins
    const int base_d = (sine ? D / 2 : 0) + 32 * wk;         // first packed index of the direct group
    const int p_top = (sine ? D : D / 2) - 32 * wk;          // packed index of mirror element v = 0, h = 0
    const int slot_out = (half || quarter) ? DUMMY : p_top / 32;
    const int slot_e = (quarter && !half) ? M / 2 : DUMMY;   // where this lane's E[0] and O[0] go as they are:
    const int slot_o = (quarter && !half) ? 3 * M / 2 : DUMMY;       // the quarter bins, or nowhere
    const int slot_in = p_top / 32 - 1;                      // bottom of the mirror group

    half8 ehi[T], elo[T], ohi[T], olo[T];
#pragma unroll
    for (int t = 0; t < T; ++t) {
        ehi[t] = __builtin_bit_cast(half8, wfold[(((wave * 2 + 0) * T + t) * 2 + 0) * 64 + lane]);
        elo[t] = __builtin_bit_cast(half8, wfold[(((wave * 2 + 0) * T + t) * 2 + 1) * 64 + lane]);
        ohi[t] = __builtin_bit_cast(half8, wfold[(((wave * 2 + 1) * T + t) * 2 + 0) * 64 + lane]);
        olo[t] = __builtin_bit_cast(half8, wfold[(((wave * 2 + 1) * T + t) * 2 + 1) * 64 + lane]);
    }
    // rho: in registers, or (large d, where registers are short) in LDS, re-read for every tile
    constexpr bool RHO_LDS = (D >= 256);
    __shared__ uint4 rho_s[RHO_LDS ? 4 * NT : 1];
    float rho[16];
    {
        const uint4* rp = wfold + M * 2 * T * 2 * 64 + (wave * 64 + lane) * 4;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint4 r = rp[i];
            if constexpr (RHO_LDS) rho_s[i * NT + tid] = r;
            rho[4 * i] = __uint_as_float(r.x); rho[4 * i + 1] = __uint_as_float(r.y);
            rho[4 * i + 2] = __uint_as_float(r.z); rho[4 * i + 3] = __uint_as_float(r.w);
        }
    }
    auto load_rho = [&]() __attribute__((always_inline)) {
        if constexpr (RHO_LDS) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const uint4 r = rho_s[i * NT + tid];
                rho[4 * i] = __uint_as_float(r.x); rho[4 * i + 1] = __uint_as_float(r.y);
                rho[4 * i + 2] = __uint_as_float(r.z); rho[4 * i + 3] = __uint_as_float(r.w);
            }
        }
    };

    // each thread moves two pairs of adjacent units (32 contiguous bytes each) per tile: pair q = tid + i NT
    auto fetch2 = [&](uint4& a, uint4& b, int i, const uint4* tile_base, int lim) __attribute__((always_inline)) {
        const int q = tid + i * NT, r = q / (U / 2), c = q % (U / 2);
        const uint4* src = tile_base + (unsigned)(min(r, lim) * U + 2 * c);
        a = src[0];
        b = src[1];
    };
    auto fetch = [&](uint4& a, uint4& b, uint4& c, uint4& d, int tile) __attribute__((always_inline)) {
        if (tile > n_tiles - 1) tile = n_tiles - 1;
        const int lim = (tile == n_tiles - 1) ? last_lim : kTileVecs - 1;
        const uint4* tile_base = x + (long long)tile * kTileVecs * U;
        fetch2(a, b, 0, tile_base, lim);
        fetch2(c, d, 1, tile_base, lim);
    };
    // 16 consecutive inputs -> the 8 at even and the 8 at odd positions
    auto put2 = [&](int buf, const uint4& a, const uint4& b, int i) __attribute__((always_inline)) {
        const int q = tid + i * NT, r = q / (U / 2), c = q % (U / 2);
        constexpr uint32_t kLo = 0x05040100u, kHi = 0x07060302u;
        lds[buf][r * ROW + 2 * c] = make_uint4(__builtin_amdgcn_perm(a.y, a.x, kLo), __builtin_amdgcn_perm(a.w, a.z, kLo),
                                               __builtin_amdgcn_perm(b.y, b.x, kLo), __builtin_amdgcn_perm(b.w, b.z, kLo));
        lds[buf][r * ROW + 2 * c + 1] = make_uint4(__builtin_amdgcn_perm(a.y, a.x, kHi), __builtin_amdgcn_perm(a.w, a.z, kHi),
                                                   __builtin_amdgcn_perm(b.y, b.x, kHi), __builtin_amdgcn_perm(b.w, b.z, kHi));
    };
    auto to_lds = [&](int buf, const uint4& a, const uint4& b, const uint4& c, const uint4& d) __attribute__((always_inline)) {
        // The first use of the prefetched registers stays here, behind the tail's stores.  The scheduler otherwise
        // moves the (cheap) byte permutes to the top of the stage or above its barrier, and the wait for the
        // loads with them, where it also drains the younger loads and the stores.
        __builtin_amdgcn_sched_barrier(0);
        put2(buf, a, b, 0);
        put2(buf, c, d, 1);
    };
    auto contract = [&](int b, floatx16& e, floatx16& o) __attribute__((always_inline)) {
        const uint4* rowp = &lds[b][col * ROW + 2 * half];      // unit pair 2t + half: [even][odd]
        e = floatx16{0};
        o = floatx16{0};
#pragma unroll
        for (int t = 0; t < T; ++t) {
            const half8 be = __builtin_bit_cast(half8, rowp[4 * t]);
            const half8 bo = __builtin_bit_cast(half8, rowp[4 * t + 1]);
            e = __builtin_amdgcn_mfma_f32_32x32x16_f16(ehi[t], be, e, 0, 0, 0);
            o = __builtin_amdgcn_mfma_f32_32x32x16_f16(ohi[t], bo, o, 0, 0, 0);
            e = __builtin_amdgcn_mfma_f32_32x32x16_f16(elo[t], be, e, 0, 0, 0);
            o = __builtin_amdgcn_mfma_f32_32x32x16_f16(olo[t], bo, o, 0, 0, 0);
        }
    };
    // what other wavefronts need of the tile just contracted
    auto publish = [&](int b, const floatx16& e, const floatx16& o) __attribute__((always_inline)) {
        float* slots = &xch[b][col];
        float rho0 = rho[0];
        if constexpr (RHO_LDS) rho0 = __uint_as_float(rho_s[tid].x);
        slots[slot_out * kTileVecs] = rho0 * (e[0] - o[0]);
        slots[slot_e * kTileVecs] = e[0];                    // straight-line code: no branch splits the stage
        slots[slot_o * kTileVecs] = o[0];
    };
    auto pack8v = [&](float f0, float f1, float f2, float f3, float f4, float f5, float f6, float f7, float inv)
                      __attribute__((always_inline)) {
        constexpr float kMagic = 12582912.0f + 8.0f;
        constexpr uint32_t kMagicBits = 0x4B400000u;
        uint32_t p = __float_as_uint(fmaf(f7, inv, kMagic));
        p = shl4_add(p, __float_as_uint(fmaf(f6, inv, kMagic)));
        p = shl4_add(p, __float_as_uint(fmaf(f5, inv, kMagic)));
        p = shl4_add(p, __float_as_uint(fmaf(f4, inv, kMagic)));
        p = shl4_add(p, __float_as_uint(fmaf(f3, inv, kMagic)));
        p = shl4_add(p, __float_as_uint(fmaf(f2, inv, kMagic)));
        p = shl4_add(p, __float_as_uint(fmaf(f1, inv, kMagic)));
        p = shl4_add(p, __float_as_uint(fmaf(f0, inv, kMagic)));
        uint32_t k = 0;
#pragma unroll
        for (int i = 0; i < 8; ++i) k += kMagicBits << (4 * i);
        return (p - k) ^ 0x88888888u;
    };
    auto pack4v = [&](float f0, float f1, float f2, float f3, float inv) __attribute__((always_inline)) {
        constexpr float kMagic = 12582912.0f;    // q mod 256 in the low byte of the bit pattern
        const uint32_t a = __float_as_uint(fmaf(f0, inv, kMagic)), b2 = __float_as_uint(fmaf(f1, inv, kMagic));
        const uint32_t c2 = __float_as_uint(fmaf(f2, inv, kMagic)), d2 = __float_as_uint(fmaf(f3, inv, kMagic));
        return (__builtin_amdgcn_perm(d2, c2, 0x0c0c0400u) << 16) | __builtin_amdgcn_perm(b2, a, 0x0c0c0400u);
    };
    auto scale_of = [&](float m, float& scale, float& inv) __attribute__((always_inline)) {
        scale = m * scale_mul;
        inv = unscale * __builtin_amdgcn_rcpf(scale);
        if (!(scale >= kMinScale)) { scale = 0.0f; inv = 0.0f; }
    };
    // vector-ALU tail of one tile, whose exchange values are in xch[b]
    auto finish = [&](int b, floatx16& e, floatx16& o, int tile) __attribute__((always_inline)) {
        const long long row0 = (long long)tile * kTileVecs;
        const int lim = (tile == n_tiles - 1) ? last_lim : kTileVecs - 1;
        const int c = min(col, lim);
        float below = xch[b][slot_in * kTileVecs + col];                 // packed index 32 * slot_in
        float nyquist = xch[b][M * kTileVecs + col];
        asm volatile("" : "+v"(below), "+v"(nyquist));       // read by every lane: no branch around the loads
        float dv[16], mv[16];
        load_rho();
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            dv[v] = e[v] + o[v];
            mv[v] = rho[v] * (e[v] - o[v]);
        }
        dv[0] = (quarter && !half) ? nyquist : dv[0];
        // bottom element of this lane's aligned mirror block
        const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(mv[0]), __float_as_uint(mv[0]), false, false);
        const float bottom = half ? below : __uint_as_float(sw[1]);      // [1]: the upper lanes' value, in all lanes
        float md = fmaxf(fabsf(dv[0]), fabsf(dv[1])), mm = fmaxf(fabsf(bottom), fabsf(mv[1]));
#pragma unroll
        for (int v = 2; v < 16; ++v) {
            md = fmaxf(md, fabsf(dv[v]));
            mm = fmaxf(mm, fabsf(mv[v]));
        }
        md = other_half_max(md);
        mm = other_half_max(mm);
        if constexpr (WIDE) {                    // the runs of one group meet in LDS (buffer b: free since stage k - 2)
            gmax[b][col * G + base_d / 32] = md;
            gmax[b][col * G + slot_in] = mm;
            __syncthreads();
            const int jd = base_d / 32 / gw * gw, jm = slot_in / gw * gw;
            md = gmax[b][col * G + jd];
            mm = gmax[b][col * G + jm];
            for (int i = 1; i < gw; ++i) {
                md = fmaxf(md, gmax[b][col * G + jd + i]);
                mm = fmaxf(mm, gmax[b][col * G + jm + i]);
            }
        }
        float sd, id, sm, im;
        scale_of(md, sd, id);
        scale_of(mm, sm, im);
        if constexpr (BITS == 8) {               // 16 values = 16 bytes: the same unit indices, in 16-byte units
            const uint4 pd = make_uint4(pack4v(dv[0], dv[1], dv[2], dv[3], id), pack4v(dv[4], dv[5], dv[6], dv[7], id),
                                        pack4v(dv[8], dv[9], dv[10], dv[11], id), pack4v(dv[12], dv[13], dv[14], dv[15], id));
            const uint4 pm = make_uint4(pack4v(bottom, mv[15], mv[14], mv[13], im), pack4v(mv[12], mv[11], mv[10], mv[9], im),
                                        pack4v(mv[8], mv[7], mv[6], mv[5], im), pack4v(mv[4], mv[3], mv[2], mv[1], im));
            uint4* crow = reinterpret_cast<uint4*>(codes) + row0 * (D / 16);
            crow[(unsigned)(c * (D / 16) + base_d / 16 + half)] = pd;
            crow[(unsigned)(c * (D / 16) + p_top / 16 - 1 - half)] = pm;
        } else {
            uint2 pd, pm;
            pd.x = pack8v(dv[0], dv[1], dv[2], dv[3], dv[4], dv[5], dv[6], dv[7], id);
            pd.y = pack8v(dv[8], dv[9], dv[10], dv[11], dv[12], dv[13], dv[14], dv[15], id);
            pm.x = pack8v(bottom, mv[15], mv[14], mv[13], mv[12], mv[11], mv[10], mv[9], im);
            pm.y = pack8v(mv[8], mv[7], mv[6], mv[5], mv[4], mv[3], mv[2], mv[1], im);
            uint2* crow = codes + row0 * (D / 16);
            crow[(unsigned)(c * (D / 16) + base_d / 16 + half)] = pd;
            crow[(unsigned)(c * (D / 16) + p_top / 16 - 1 - half)] = pm;
        }
        // both halves store the same values
        if constexpr (WIDE) {
            float* srow = scales + row0 * (G / gw);
            srow[(unsigned)(c * (G / gw) + base_d / 32 / gw)] = sd;
            srow[(unsigned)(c * (G / gw) + slot_in / gw)] = sm;
        } else {
            float* srow = scales + row0 * G;
            srow[(unsigned)(c * G + base_d / 32)] = sd;
            srow[(unsigned)(c * G + slot_in)] = sm;
        }
    };

    const int m = (n_tiles - 1 - t0) / stride + 1;
    uint4 pa0, pa1, pa2, pa3, pb0, pb1, pb2, pb3;
    floatx16 ea, oa, eb, ob;
    fetch(pa0, pa1, pa2, pa3, t0);
    fetch(pb0, pb1, pb2, pb3, t0 + stride);
    hold_in_registers(ehi, elo);
    hold_in_registers(ohi, olo);
    to_lds(0, pa0, pa1, pa2, pa3);
    fetch(pa0, pa1, pa2, pa3, t0 + 2 * stride);
    if constexpr (LEAN) {
        // One accumulator set.  Stage k: barrier; quantize T_{k-1} out of the accumulators (its exchange values,
        // in xch[(k-1) & 1], became visible with the barrier); contract T_k into them; fill LDS for T_{k+1};
        // publish T_k's exchange values into xch[k & 1].  Within a wavefront the two halves do not overlap; two
        // workgroups per compute unit overlap each other.
        __syncthreads();                         // stage 0: nothing to quantize yet
        contract(0, ea, oa);
        to_lds(1, pb0, pb1, pb2, pb3);
        fetch(pb0, pb1, pb2, pb3, t0 + 3 * stride);
        publish(0, ea, oa);
        // two stages per trip, so that the two prefetch register sets keep their names: selecting them by a
        // branch makes the compiler copy the loaded registers at the end of the stage, behind a wait for
        // every load and store in flight
        int k = 1;
        for (; k + 1 < m; k += 2) {
            const int tk = t0 + k * stride;
            __syncthreads();                     // stage k (odd)
            finish(0, ea, oa, tk - stride);
            __builtin_amdgcn_sched_barrier(0);   // no second accumulator set: the tail ends before the MFMAs begin
            contract(1, ea, oa);
            to_lds(0, pa0, pa1, pa2, pa3);
            fetch(pa0, pa1, pa2, pa3, tk + 3 * stride);
            publish(1, ea, oa);
            __syncthreads();                     // stage k + 1 (even)
            finish(1, ea, oa, tk);
            __builtin_amdgcn_sched_barrier(0);
            contract(0, ea, oa);
            to_lds(1, pb0, pb1, pb2, pb3);
            fetch(pb0, pb1, pb2, pb3, tk + 4 * stride);
            publish(0, ea, oa);
        }
        if (k < m) {                             // one more odd stage
            const int tk = t0 + k * stride;
            __syncthreads();
            finish(0, ea, oa, tk - stride);
            __builtin_amdgcn_sched_barrier(0);
            contract(1, ea, oa);
            publish(1, ea, oa);
            __syncthreads();
            finish(1, ea, oa, tk);
        } else {
            __syncthreads();
            finish(0, ea, oa, t0 + (k - 1) * stride);
        }
        return;
    }
    // stage 0
    __syncthreads();
    contract(0, ea, oa);
    to_lds(1, pb0, pb1, pb2, pb3);
    fetch(pb0, pb1, pb2, pb3, t0 + 3 * stride);
    publish(0, ea, oa);
    int k = 1;
    for (; k + 1 < m; k += 2) {
        const int tk = t0 + k * stride;
        __syncthreads();                         // stage k (odd)
        rotate_priority(k);
        contract(1, eb, ob);
        finish(0, ea, oa, tk - stride);
        to_lds(0, pa0, pa1, pa2, pa3);
        fetch(pa0, pa1, pa2, pa3, tk + 3 * stride);
        publish(1, eb, ob);
        __syncthreads();                         // stage k + 1 (even)
        rotate_priority(k + 1);
        contract(0, ea, oa);
        finish(1, eb, ob, tk);
        to_lds(1, pb0, pb1, pb2, pb3);
        fetch(pb0, pb1, pb2, pb3, tk + 4 * stride);
        publish(0, ea, oa);
    }
    if (k < m) {                                 // one more odd stage
        const int tk = t0 + k * stride;
        __syncthreads();
        contract(1, eb, ob);
        finish(0, ea, oa, tk - stride);
        publish(1, eb, ob);
        __syncthreads();
        finish(1, eb, ob, tk);
    } else {
        __syncthreads();
        finish(0, ea, oa, t0 + (k - 1) * stride);
    }
}

// two wavefronts per SIMD (8 per compute unit): the register allocator is told to stay within 256 VGPRs
template <int D, int BITS, bool WIDE>
__global__ void __launch_bounds__(D, 2)
srft_quantize_fold_kernel(const uint4* __restrict__ wfold, const uint4* __restrict__ x, long long n_vec,
                          uint2* __restrict__ codes, float* __restrict__ scales, float4* __restrict__,
                          float unscale, float scale_mul, int gw) {
    srft_quantize_fold_tiles<D, BITS, WIDE>(wfold, x, n_vec, codes, scales, unscale, scale_mul, gw, blockIdx.x,
                                            gridDim.x);
}

// Several plans in one launch (a decode step appends a few hundred vectors to each of many (layer, K|V)
// caches: one launch per plan would be all launch latency).  Segment i = plan i's constants and buffers; it
// is served by workgroups first_block[i] .. first_block[i+1]-1, each walking that segment's tiles with
// that many as stride.  The table travels as a kernel argument.
constexpr int kMaxBatch = 64;       // the table is about 3.5 KiB of the 4 KiB a kernel may take as arguments
struct srft_batch_args {
    int count;
    int first_block[kMaxBatch + 1];
    const uint4* frag[kMaxBatch];
    const void* in0[kMaxBatch];      // write path: x      read path: codes
    const void* in1[kMaxBatch];      //                    read path: scales
    void* out0[kMaxBatch];           // write path: codes  read path: out
    void* out1[kMaxBatch];           // write path: scales
    long long n_vec[kMaxBatch];
    float unscale[kMaxBatch];
};
static_assert(sizeof(srft_batch_args) + sizeof(int) <= 4096, "kernel arguments are limited to 4 KiB");
__device__ __forceinline__ int srft_segment_of_block(const srft_batch_args& a, int block) {
    int i = 0;
    while (i + 1 < a.count && a.first_block[i + 1] <= block) ++i;     // uniform; count is small
    return i;
}

template <int D, int S, int GM, int BITS>
__global__ void __launch_bounds__(2 * D / S)
srft_quantize_batched_kernel(const srft_batch_args a, int gw) {
    const int i = srft_segment_of_block(a, blockIdx.x);
    srft_quantize_tiles<D, S, kOutCodes, GM, BITS>(a.frag[i], (const uint4*)a.in0[i], a.n_vec[i], (uint2*)a.out0[i],
                                         (float*)a.out1[i], nullptr, a.unscale[i],
                                         a.unscale[i] / (BITS == 8 ? 127.0f : 7.0f), gw,
                                         blockIdx.x - a.first_block[i], a.first_block[i + 1] - a.first_block[i]);
}

template <int D, int BITS, bool WIDE>
__global__ void __launch_bounds__(D, 2)
srft_quantize_fold_batched_kernel(const srft_batch_args a, int gw) {
    const int i = srft_segment_of_block(a, blockIdx.x);
    srft_quantize_fold_tiles<D, BITS, WIDE>(a.frag[i], (const uint4*)a.in0[i], a.n_vec[i], (uint2*)a.out0[i],
                                            (float*)a.out1[i], a.unscale[i], a.unscale[i] / (BITS == 8 ? 127.0f : 7.0f),
                                            gw, blockIdx.x - a.first_block[i], a.first_block[i + 1] - a.first_block[i]);
}

// ------------------------------------------------------------------------------------------
// read path
// ------------------------------------------------------------------------------------------
// One dword of eight nibbles -> eight exact fp16 codes, as four packed pairs (n_m, n_{m+4}).
// 0x6400 | u is the fp16 number 1024 + u; with u = q + 8 a packed fp16 subtract of 1032 leaves q.
// A nibble one position higher (bits 4..7 of the 16-bit half) gives 1024 + 16 u instead; times 1/16 minus 72
// is q again (exact), which saves the shift: ten vector-ALU operations per dword.
__device__ __forceinline__ uint32_t and_or(uint32_t v, uint32_t mask, uint32_t bits) {
    uint32_t r;                                  // one instruction; `bits` is kept in a vector register
    asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(r) : "v"(v), "s"(mask), "v"(bits));
    return r;
}
__device__ __forceinline__ uint4 decode8(uint32_t v) {
    v ^= 0x88888888u;
    const half2v bias = {(_Float16)1032.0f, (_Float16)1032.0f};
    const half2v sixteenth = {(_Float16)0.0625f, (_Float16)0.0625f}, bias16 = {(_Float16)72.0f, (_Float16)72.0f};
    const uint32_t one_k = 0x64006400u, w = v >> 8;
    uint4 o;
    o.x = __builtin_bit_cast(uint32_t, __builtin_bit_cast(half2v, and_or(v, 0x000F000Fu, one_k)) - bias);
    o.y = __builtin_bit_cast(uint32_t, __builtin_bit_cast(half2v, and_or(v, 0x00F000F0u, one_k)) * sixteenth - bias16);
    o.z = __builtin_bit_cast(uint32_t, __builtin_bit_cast(half2v, and_or(w, 0x000F000Fu, one_k)) - bias);
    o.w = __builtin_bit_cast(uint32_t, __builtin_bit_cast(half2v, and_or(w, 0x00F000F0u, one_k)) * sixteenth - bias16);
    return o;
}

// One dword of four two's-complement bytes -> four exact fp16 codes as the packed pairs (b0, b2) and (b1, b3):
// flipping bit 7 gives u = q + 128 in 0..255, 0x6400 | u is 1024 + u, minus 1152 is q.
__device__ __forceinline__ uint2 decode4_bytes(uint32_t v) {
    v ^= 0x80808080u;
    const half2v bias = {(_Float16)1152.0f, (_Float16)1152.0f};
    const uint32_t one_k = 0x64006400u;
    uint2 o;
    o.x = __builtin_bit_cast(uint32_t, __builtin_bit_cast(half2v, and_or(v, 0x00FF00FFu, one_k)) - bias);
    o.y = __builtin_bit_cast(uint32_t, __builtin_bit_cast(half2v, and_or(v >> 8, 0x00FF00FFu, one_k)) - bias);
    return o;
}

// Two fp32 values -> packed fp16, round to nearest even.  The empty asm keeps the compiler from fusing
// the preceding multiply-add into a mixed-precision fma in some copies of this code and not in others:
// every path rounds fp32 -> fp16 the same way, so a vector's output does not depend on where in the
// batch it sits or on the launch shape.
__device__ __forceinline__ uint32_t pack_half2(float a, float b) {
    asm volatile("" : "+v"(a), "+v"(b));
    const half2v h = {(_Float16)a, (_Float16)b};
    return __builtin_bit_cast(uint32_t, h);
}

// rfrag : [D/32 waves][D/32 groups][2 k-steps][hi, lo][64 lanes] 16-byte A-operand fragments of R
// codes : [n_vec][D/16] 8-byte units; scales : [n_vec][D/32]; out : [n_vec][D/8] 16-byte units of fp16
//
// Within a tile the groups are contracted one after the other (K = 32 each), into accumulators that
// alternate, so that  o += scale_j * P_j  of one group runs on the vector ALU while the next group is
// on the matrix cores; the last group of a tile has an accumulator of its own and is folded in under
// the first group of the next tile.
//
// A lane ends up with 16 consecutive fp16 of one vector (32 bytes); stored directly that would be 16-byte
// pieces 256 bytes apart.  The finished tile is therefore staged in LDS (stage k stages T_{k-1}) and
// written out one stage later by all threads as fully coalesced 16-byte-per-lane stores of the
// contiguous 32 x 2D-byte block (stage k flushes T_{k-2}).  The per-vector scales reach the lanes through
// LDS as well: they are loaded once per workgroup, coalesced, together with the codes.
// S : output slabs per wavefront (the workgroup has D / (32 S) wavefronts), as on the write path.
// KS: MFMA k-steps (of 16 codes) contracted under one scale: 2 for g >= 32 (g = 32 * gw, gw slabs of codes
//     share a scale), 1 for g = 16.  "Group" below means one such run of 16 * KS codes.
// FOLD: half the matrix work, for d a multiple of 64 and g >= 32.  Every row of Q satisfies
//     Q[p][n + d/2] = (-1)^p Q[p][n]   (DC and Nyquist rows: +1; cos and sin rows of bin k: (-1)^k, and the
//     packed index p has the parity of k), so with  A_n = sum over even p,  B_n = sum over odd p  of
//     Q[p][n] z_p  the outputs are  x_n = s_n (A_n + B_n)  and  x_{n+d/2} = s_{n+d/2} (A_n - B_n),  n < d/2.
//     A byte holds an even p in its low and an odd p in its high nibble, so the two operands are the low and
//     the high nibbles.  Wavefront w owns n = 32w .. 32w+31: slab 0 is A, slab 1 is B (S = 2, KS = 1: per
//     group of 32 codes one k-step of 16 even and one of 16 odd codes), rows scaled by s_n on the host;
//     the relative sign s_n s_{n+d/2} is applied to the packed fp16 bits.  rfrag is then
//     [D/64 waves][A, B][D/32 groups][hi, lo][64 lanes], followed by [D/64 waves][64 lanes][2] sign masks.
// BITS: 4, or 8 (one two's-complement byte per code).  A "code unit" is 16 codes: 8 bytes at 4 bits, 16 at 8.
//     At 8 bits a dword gives the pairs (b0, b2) and (b1, b3): again even and odd p apart, so FOLD applies as is.
template <int D, int S, int KS, bool FOLD, int BITS>
__device__ __forceinline__ void
srft_dequantize_tiles(const uint4* __restrict__ rfrag, const uint2* __restrict__ codes_raw,
                      const float* __restrict__ scales, long long n_vec, uint4* __restrict__ out,
                      float unscale, int gw, const int t0, const int stride) {
    constexpr int G = FOLD ? D / 32 : D / 32 * (2 / KS);  // groups per vector as contracted
    constexpr int NSMAX = D / 16;         // most scales a vector can have (g = 16)
    constexpr bool kPerStep = (KS == 1 && !FOLD);         // g = 16: a scale per k-step of the full matrix
    const int ns = kPerStep ? D / 16 : D / 32 / gw;       // scales per vector
    static_assert(!FOLD || (S == 2 && KS == 1 && D % 64 == 0), "the folded form pairs an A and a B slab");
    constexpr int U = D / 8;             // 16-byte units per decoded row (D fp16)
    constexpr int ROW = U + 1;
    constexpr int C = D / 16;            // code units (16 codes) per row
    using CodeUnit = std::conditional_t<BITS == 8, uint4, uint2>;
    const CodeUnit* __restrict__ codes = reinterpret_cast<const CodeUnit*>(codes_raw);
    constexpr int NT = 2 * D / S;
    constexpr int SROW = NSMAX + 1;      // padded row of the scale tile (floats)
    constexpr int PS = (32 * NSMAX + NT - 1) / NT;      // scale floats a thread may have to carry (1 or 2)
    static_assert((D / 32) % S == 0 && (S == 1 || S == 2), "one or two slabs per wavefront");
    // Two slabs of a large matrix leave no room for alternating accumulators: one accumulator set, each group
    // folded in as soon as it is done, the tile staged in the stage that computes it.
    constexpr bool LEAN = (S == 2 && (D / 32 > 4 || FOLD));
    __shared__ uint4 dec[2][kTileVecs * ROW];    // decoded codes of T_k in dec[k % 2]
    __shared__ uint4 stg[2][kTileVecs * ROW];    // finished fp16 rows of T_k in stg[k % 2]
    __shared__ float scl[2][kTileVecs * SROW];   // scales (times 2^-e) of T_k in scl[k % 2]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane & 31, half = lane >> 5;
    // tile indices are 32-bit (the host bounds n_vec), so that the uniform index arithmetic stays scalar
    const int n_tiles = (int)((n_vec + kTileVecs - 1) / kTileVecs);
    const int last_lim = (int)(n_vec - 1 - (long long)(n_tiles - 1) * kTileVecs);   // last valid row of the last tile

    half8 rhi[S * G][KS], rlo[S * G][KS];        // [s * G + group][k-step within the group]
#pragma unroll
    for (int s = 0; s < S; ++s)
#pragma unroll
        for (int j = 0; j < G; ++j)
#pragma unroll
            for (int t = 0; t < KS; ++t) {
                const int slab = wave * S + s, kstep = j * KS + t;
                const int f = FOLD ? slab * G + j : slab * (D / 16) + kstep;
                rhi[s * G + j][t] = __builtin_bit_cast(half8, rfrag[(f * 2 + 0) * 64 + lane]);
                rlo[s * G + j][t] = __builtin_bit_cast(half8, rfrag[(f * 2 + 1) * 64 + lane]);
            }
    uint4 flip0 = {}, flip1 = {};                // sign-bit masks of this lane's 16 outputs n + d/2 (FOLD)
    if constexpr (FOLD) {
        const uint4* masks = rfrag + (D / 32) * G * 2 * 64;
        flip0 = masks[(wave * 64 + lane) * 2];
        flip1 = masks[(wave * 64 + lane) * 2 + 1];
        asm volatile("" : "+v"(flip0.x), "+v"(flip0.y), "+v"(flip0.z), "+v"(flip0.w));
        asm volatile("" : "+v"(flip1.x), "+v"(flip1.y), "+v"(flip1.z), "+v"(flip1.w));
    }

    // each thread decodes S 8-byte units of the 32 x D/2 code tile (32 * C = S * NT units) and carries up to
    // PS floats of the 32 x ns scale tile (float e = tid + i * NT; past the end it re-reads the last one)
    // Addresses are a uniform tile base (scalar registers) plus a 32-bit per-lane offset; rows past the end
    // alias to the last row through `lim`, the index of the last valid row of the tile (uniform).
    auto fetch1 = [&](CodeUnit& v, int i, const CodeUnit* tile_base, int lim) __attribute__((always_inline)) {
        const int u = tid + i * NT, r = u / C, c = u % C;
        v = stream_load(&tile_base[(unsigned)(min(r, lim) * C + c)]);
    };
    auto fetch_scale = [&](float& sc, int i, const float* tile_base, int lim) __attribute__((always_inline)) {
        int e = tid + i * NT;
        if (e > 32 * ns - 1) e = 32 * ns - 1;
        const int r = e / ns, j = e % ns;
        sc = tile_base[(unsigned)(min(r, lim) * ns + j)];
    };
    auto fetch = [&](CodeUnit& c0, CodeUnit& c1, float& s0, float& s1, int tile) __attribute__((always_inline)) {
        if (tile > n_tiles - 1) tile = n_tiles - 1;
        const long long row0 = (long long)tile * kTileVecs;
        const int lim = (tile == n_tiles - 1) ? last_lim : kTileVecs - 1;
        const CodeUnit* code_base = codes + row0 * C;
        const float* scale_base = scales + row0 * ns;
        fetch1(c0, 0, code_base, lim);
        if constexpr (S > 1) fetch1(c1, 1, code_base, lim);
        fetch_scale(s0, 0, scale_base, lim);
        if constexpr (PS > 1) fetch_scale(s1, 1, scale_base, lim);
    };
    auto put1 = [&](int b, const CodeUnit& v, int i) __attribute__((always_inline)) {
        const int u = tid + i * NT, r = u / C, c = u % C;
        if constexpr (BITS == 8) {               // .x: bytes 0 and 2 (even p), .y: bytes 1 and 3 (odd p) of a dword
            const uint2 a = decode4_bytes(v.x), b2 = decode4_bytes(v.y), c2 = decode4_bytes(v.z), d2 = decode4_bytes(v.w);
            if constexpr (FOLD) {
                dec[b][r * ROW + 2 * c] = make_uint4(a.x, b2.x, c2.x, d2.x);
                dec[b][r * ROW + 2 * c + 1] = make_uint4(a.y, b2.y, c2.y, d2.y);
            } else {
                dec[b][r * ROW + 2 * c] = make_uint4(a.x, a.y, b2.x, b2.y);
                dec[b][r * ROW + 2 * c + 1] = make_uint4(c2.x, c2.y, d2.x, d2.y);
            }
        } else {
            const uint4 lo = decode8(v.x), hi = decode8(v.y);
            if constexpr (FOLD) {                // .x .z hold the even, .y .w the odd nibbles of a dword
                dec[b][r * ROW + 2 * c] = make_uint4(lo.x, lo.z, hi.x, hi.z);
                dec[b][r * ROW + 2 * c + 1] = make_uint4(lo.y, lo.w, hi.y, hi.w);
            } else {
                dec[b][r * ROW + 2 * c] = lo;
                dec[b][r * ROW + 2 * c + 1] = hi;
            }
        }
    };
    auto put_scale = [&](int b, float sc, int i) __attribute__((always_inline)) {
        const int e = tid + i * NT;
        if (e < 32 * ns) scl[b][(e / ns) * SROW + e % ns] = sc * unscale;
    };
    auto to_lds = [&](int b, const CodeUnit& c0, const CodeUnit& c1, float s0, float s1) __attribute__((always_inline)) {
        put1(b, c0, 0);
        if constexpr (S > 1) put1(b, c1, 1);
        put_scale(b, s0, 0);
        if constexpr (PS > 1) put_scale(b, s1, 1);
    };
    // scale of contracted group j: its own at g = 16 and g = 32, shared by gw groups at g = 32 * gw
    auto scale_of = [&](int b, int j) __attribute__((always_inline)) { return scl[b][col * SROW + (kPerStep ? j : j / gw)]; };
    // The last group of a tile is folded in one stage later, under group 0 of the next tile (which uses
    // acc0); with an even number of groups it can live in acc1, otherwise it needs a register set of its own.
    floatx16 o[S], acc0[S], acc1[S], acc_odd[S];
    auto& acc_last = (G % 2 == 0) ? acc1 : acc_odd;
    auto group = [&](int b, int j, floatx16 (&acc)[S]) {
        const uint4* rowp = &dec[b][col * ROW + half];
#pragma unroll
        for (int s = 0; s < S; ++s) acc[s] = floatx16{0};
        if constexpr (FOLD) {                    // unit 2j + half of the row: [even codes][odd codes]
#pragma unroll
            for (int s = 0; s < S; ++s) {
                const half8 bf = __builtin_bit_cast(half8, rowp[4 * j + half + s]);
                acc[s] = __builtin_amdgcn_mfma_f32_32x32x16_f16(rhi[s * G + j][0], bf, acc[s], 0, 0, 0);
                acc[s] = __builtin_amdgcn_mfma_f32_32x32x16_f16(rlo[s * G + j][0], bf, acc[s], 0, 0, 0);
            }
            return;
        }
#pragma unroll
        for (int t = 0; t < KS; ++t) {
            const half8 bf = __builtin_bit_cast(half8, rowp[2 * (j * KS + t)]);
#pragma unroll
            for (int s = 0; s < S; ++s) {
                acc[s] = __builtin_amdgcn_mfma_f32_32x32x16_f16(rhi[s * G + j][t], bf, acc[s], 0, 0, 0);
                acc[s] = __builtin_amdgcn_mfma_f32_32x32x16_f16(rlo[s * G + j][t], bf, acc[s], 0, 0, 0);
            }
        }
    };
    // o (+)= sc * acc
    auto fold = [&](const floatx16 (&acc)[S], float sc, bool first) {
#pragma unroll
        for (int s = 0; s < S; ++s)
#pragma unroll
            for (int v = 0; v < 16; ++v) o[s][v] = first ? acc[s][v] * sc : fmaf(acc[s][v], sc, o[s][v]);
    };
    // the finished outputs of this lane, rounded to fp16, into the staging tile b
    auto stage_out = [&](int b) __attribute__((always_inline)) {
        if constexpr (FOLD) {
            uint4* dst = &stg[b][col * ROW + 4 * wave + 2 * half];
            uint32_t lo[8], hi[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                lo[i] = pack_half2(o[0][2 * i] + o[1][2 * i], o[0][2 * i + 1] + o[1][2 * i + 1]);
                hi[i] = pack_half2(o[0][2 * i] - o[1][2 * i], o[0][2 * i + 1] - o[1][2 * i + 1]);
            }
            dst[0] = make_uint4(lo[0], lo[1], lo[2], lo[3]);
            dst[1] = make_uint4(lo[4], lo[5], lo[6], lo[7]);
            dst[U / 2] = make_uint4(hi[0] ^ flip0.x, hi[1] ^ flip0.y, hi[2] ^ flip0.z, hi[3] ^ flip0.w);
            dst[U / 2 + 1] = make_uint4(hi[4] ^ flip1.x, hi[5] ^ flip1.y, hi[6] ^ flip1.z, hi[7] ^ flip1.w);
            return;
        }
#pragma unroll
        for (int s = 0; s < S; ++s) {
            uint4* dst = &stg[b][col * ROW + 4 * (wave * S + s) + 2 * half];
            dst[0] = make_uint4(pack_half2(o[s][0], o[s][1]), pack_half2(o[s][2], o[s][3]),
                                pack_half2(o[s][4], o[s][5]), pack_half2(o[s][6], o[s][7]));
            dst[1] = make_uint4(pack_half2(o[s][8], o[s][9]), pack_half2(o[s][10], o[s][11]),
                                pack_half2(o[s][12], o[s][13]), pack_half2(o[s][14], o[s][15]));
        }
    };
    // staging tile b -> global rows of `tile`: fully coalesced 16-byte stores, 2 S per thread
    auto flush = [&](int b, int tile) __attribute__((always_inline)) {
        const long long row0 = (long long)tile * kTileVecs;
        const int lim = (tile == n_tiles - 1) ? last_lim : kTileVecs - 1;
        uint4* tile_base = out + row0 * U;
#pragma unroll
        for (int i = 0; i < 2 * S; ++i) {
            const int u = tid + i * NT, r = u / U, c = u % U;
            stream_store(&tile_base[(unsigned)(min(r, lim) * U + c)], stg[b][r * ROW + c]);   // rows past the end alias to the last row
        }
    };
    // all groups of the tile in dec[b] (scales in scl[b]); `prev`: first fold in the last group of the
    // previous tile, whose scale is s_prev_last, and stage that tile in stg[b_prev]
    auto tile_body = [&](int b, bool prev, float s_prev_last, int b_prev) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < G; ++j) {
            auto& acc = (j == G - 1) ? acc_last : ((j & 1) ? acc1 : acc0);
            if (j == 0 && prev) {
                // acc_last still holds the last group of the previous tile
                if constexpr (G > 1) {
                    group(b, 0, acc);
                    fold(acc_last, s_prev_last, false);
                    stage_out(b_prev);
                } else {
                    fold(acc_last, s_prev_last, true);
                    stage_out(b_prev);
                    group(b, 0, acc);
                }
            } else {
                group(b, j, acc);
            }
            if (j >= 1) fold((j - 1) & 1 ? acc1 : acc0, scale_of(b, j - 1), j == 1);
            // with many groups, keep the scheduler from reading every group's fragments up front
            if constexpr (G > 4) __builtin_amdgcn_sched_barrier(0);
        }
    };

    // With few groups two accumulator sets fit: group j + 1 is on the matrix cores while group j is folded in.
    constexpr bool LEAN_ALT = LEAN && (S * G <= SRFT_LEAN_ALT_MAX);
    auto lean_body = [&](int b) __attribute__((always_inline)) {
        if constexpr (LEAN_ALT) {
            group(b, 0, acc0);
#pragma unroll
            for (int j = 1; j < G; ++j) {
                group(b, j, (j & 1) ? acc1 : acc0);
                fold((j & 1) ? acc0 : acc1, scale_of(b, j - 1), j == 1);
            }
            fold(((G - 1) & 1) ? acc1 : acc0, scale_of(b, G - 1), G == 1);
        } else {
#pragma unroll
            for (int j = 0; j < G; ++j) {
                group(b, j, acc0);
                fold(acc0, scale_of(b, j), j == 0);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        stage_out(b);
    };

    const int m = (n_tiles - 1 - t0) / stride + 1;
    CodeUnit pa0, pa1, pb0, pb1;                 // prefetched code units of the next two tiles
    float pas, pat, pbs, pbt;                    // and up to two floats each of their scale tiles
    float s_last;                                // scale of the last group of the tile contracted last
    fetch(pa0, pa1, pas, pat, t0);
    fetch(pb0, pb1, pbs, pbt, t0 + stride);
    hold_in_registers(rhi, rlo);
    to_lds(0, pa0, pa1, pas, pat);
    fetch(pa0, pa1, pas, pat, t0 + 2 * stride);
    if constexpr (LEAN) {
        // stage k: barrier; flush T_{k-1}; contract, fold and stage T_k; decode T_{k+1}.  Two stages per trip,
        // so that the two prefetch register sets keep their names (selecting them by a branch makes the compiler
        // copy the loaded registers at the end of the stage, behind a wait for every load and store in flight).
        __syncthreads();                         // stage 0: nothing to flush yet
        lean_body(0);
        to_lds(1, pb0, pb1, pbs, pbt);
        fetch(pb0, pb1, pbs, pbt, t0 + 3 * stride);
        int k = 1;
        for (; k + 1 < m; k += 2) {
            const int tk = t0 + k * stride;
            __syncthreads();                     // stage k (odd)
            rotate_priority(k);
            flush(0, tk - stride);
            lean_body(1);
            to_lds(0, pa0, pa1, pas, pat);
            fetch(pa0, pa1, pas, pat, tk + 3 * stride);
            __syncthreads();                     // stage k + 1 (even)
            rotate_priority(k + 1);
            flush(1, tk);
            lean_body(0);
            to_lds(1, pb0, pb1, pbs, pbt);
            fetch(pb0, pb1, pbs, pbt, tk + 4 * stride);
        }
        if (k < m) {                             // one more odd stage
            const int tk = t0 + k * stride;
            __syncthreads();
            flush(0, tk - stride);
            lean_body(1);
            __syncthreads();
            flush(1, tk);
        } else {
            __syncthreads();
            flush(0, t0 + (k - 1) * stride);
        }
        return;
    }
    // stage 0
    __syncthreads();
    tile_body(0, false, 0.0f, 0);
    s_last = scale_of(0, G - 1);
    to_lds(1, pb0, pb1, pbs, pbt);
    fetch(pb0, pb1, pbs, pbt, t0 + 3 * stride);
    // stage k: barrier; flush T_{k-2}; contract T_k (staging T_{k-1} under its first group); decode T_{k+1}
    int stage_no = 1;
    auto odd_stage = [&](int tk, auto flush_first) __attribute__((always_inline)) {      // T_k in dec[1]
        __syncthreads();
        rotate_priority(stage_no++);
        if constexpr (decltype(flush_first)::value) flush(1, tk - 2 * stride);
        tile_body(1, true, s_last, 0);
        s_last = scale_of(1, G - 1);
        to_lds(0, pa0, pa1, pas, pat);
        fetch(pa0, pa1, pas, pat, tk + 3 * stride);
    };
    auto even_stage = [&](int tk) __attribute__((always_inline)) {                       // T_k in dec[0]
        __syncthreads();
        rotate_priority(stage_no++);
        flush(0, tk - 2 * stride);
        tile_body(0, true, s_last, 1);
        s_last = scale_of(0, G - 1);
        to_lds(1, pb0, pb1, pbs, pbt);
        fetch(pb0, pb1, pbs, pbt, tk + 3 * stride);
    };
    int k = 1;
    if (k + 1 < m) {                             // stages 1 and 2: nothing to flush in stage 1 yet
        odd_stage(t0 + stride, std::false_type{});
        even_stage(t0 + 2 * stride);
        k = 3;
    }
    for (; k + 1 < m; k += 2) {
        odd_stage(t0 + k * stride, std::true_type{});
        even_stage(t0 + (k + 1) * stride);
    }
    // the last group of the last tile is still in acc_last; up to two staged tiles are unflushed
    if (k < m) {                                 // one more odd stage: T_k in dec[1]
        const int tk = t0 + k * stride;
        __syncthreads();
        if (k >= 2) flush(1, tk - 2 * stride);
        tile_body(1, true, s_last, 0);
        s_last = scale_of(1, G - 1);
        __syncthreads();                         // every thread is done reading stg[1]
        fold(acc_last, s_last, G == 1);
        stage_out(1);
        flush(0, tk - stride);
        __syncthreads();
        flush(1, tk);
    } else {                                     // the last stage was even (or stage 0): T_{k-1} in dec[0]
        const int tl = t0 + (k - 1) * stride;
        __syncthreads();                         // every thread is done reading stg[0]
        fold(acc_last, s_last, G == 1);
        stage_out(0);
        if (k >= 2) flush(1, tl - stride);
        __syncthreads();
        flush(0, tl);
    }
}

template <int D, int S, int KS, bool FOLD, int BITS>
__global__ void __launch_bounds__(2 * D / S)
srft_dequantize_kernel(const uint4* __restrict__ rfrag, const uint2* __restrict__ codes,
                       const float* __restrict__ scales, long long n_vec, uint4* __restrict__ out,
                       float unscale, int gw) {
    srft_dequantize_tiles<D, S, KS, FOLD, BITS>(rfrag, codes, scales, n_vec, out, unscale, gw, blockIdx.x, gridDim.x);
}

template <int D, int S, int KS, bool FOLD, int BITS>
__global__ void __launch_bounds__(2 * D / S)
srft_dequantize_batched_kernel(const srft_batch_args a, int gw) {
    const int i = srft_segment_of_block(a, blockIdx.x);
    srft_dequantize_tiles<D, S, KS, FOLD, BITS>(a.frag[i], (const uint2*)a.in0[i], (const float*)a.in1[i], a.n_vec[i],
                                    (uint4*)a.out0[i], a.unscale[i], gw, blockIdx.x - a.first_block[i],
                                    a.first_block[i + 1] - a.first_block[i]);
}

// ------------------------------------------------------------------------------------------
// scores against the stored keys, in the rotated domain
// ------------------------------------------------------------------------------------------
// <q, k_t> with k_t = s * Q^T (code * scale / lambda) equals <q', code * scale> with q' = Q (s * q) / lambda:
// the transform is orthogonal, so the keys never have to be reconstructed; the kernel reads the 4-bit record
// only (d/2 + 4 d/g bytes per key instead of the 2d of a dequantized prefix) and writes n_q floats per key.
//
// Up to 32 queries are the 32 rows of the MFMA A operand (hi + lo fp16 of q', in registers for the whole
// launch), the keys are the columns: the read path with the queries in place of the matrix.  One wavefront
// per workgroup, each walking its own tiles of 32 keys: codes are loaded coalesced, decoded into LDS (which
// transposes them into B fragments), contracted group by group and folded with the group scales.
//
// Step 1: q' = w / (lambda * max(lambda, 1e-6)) with w = lambda * Q (s * q), split into fp16 hi + lo and laid out as
// A fragments.  The write path's plain kernel does it, in its kOutQFrag32 / kOutQFrag16 modes (one launch).
// Two layouts, both chosen so that the first ceil(n_q / 2) result registers of the lanes hold all the queries
// (a small group of queries costs few stores):
//   32 rows (n_q > 16; v_mfma_f32_32x32x16_f16): [d/32 groups][2 k-steps][hi, lo][64 lanes]; MFMA row i (lane half
//     h = (i / 4) % 2, register v = 4 (i / 8) + i % 4 of the result) carries query 2 v + h.
//   16 rows (R16, n_q <= 16; v_mfma_f32_16x16x32_f16, half the matrix-core time): [d/32 groups][hi, lo][64 lanes];
//     lane l holds row l % 16 and the 8 codes of unit 4 j + l / 16 of group j.  MFMA row r = 4 a + i (result register i
//     of the lanes 16 a .. 16 a + 15) carries query 2 i + a for a < 2 and 8 + 2 i + (a - 2) for a >= 2.
//
// Step 2.  codes [n_keys][D/16] 8-byte units, scales [n_keys][ns], out [n_q][n_keys] fp32.
// NV: result registers a lane stores per tile (NV >= ceil(n_q / 2), a power of two; 16 with 32 rows, <= 8 with 16).
// Every lane stores NV times per tile whatever n_q and the tile are: a lane without a valid (query, key) writes
// to its own slot of `dump` (64 floats per workgroup, never read).  So the number of memory operations per stage
// is fixed, the wait counters are exact, and the codes are prefetched two tiles ahead in two named register
// sets (two stages per trip), as on the read path.
template <int D, int NV, bool R16>
__global__ void __launch_bounds__(64, (D <= 128 || R16) ? 2 : 1)
srft_scores_kernel(const uint4* __restrict__ qfrag, const uint2* __restrict__ codes, const float* __restrict__ scales,
                   long long n_keys, float* __restrict__ out, int n_q, int gw, float* __restrict__ dump) {
    constexpr int G = D / 32, U = D / 8, ROW = U + 1, C = D / 16;
    constexpr int PER = C / 2;           // 8-byte code units per lane and tile (32 C units, 64 lanes)
    constexpr int SROW = G + 1;
    constexpr int PS = (32 * G + 63) / 64;
    constexpr int NF = R16 ? G : 2 * G;  // A fragments (hi, lo each)
    static_assert(D % 64 == 0, "whole code units per lane");
    static_assert(R16 ? NV <= 8 : NV == 16, "16 rows hold up to 16 queries");
    __shared__ uint4 dec[2][kTileVecs * ROW];
    __shared__ float scl[2][kTileVecs * SROW];
    const int lane = threadIdx.x, col = lane & 31, half = lane >> 5;
    const int ns = G / gw;
    const int n_tiles = (int)((n_keys + kTileVecs - 1) / kTileVecs);
    const int last_lim = (int)(n_keys - 1 - (long long)(n_tiles - 1) * kTileVecs);
    const int t0 = blockIdx.x, stride = gridDim.x;
    float* const my_dump = dump + (size_t)blockIdx.x * 64 + lane;

    half8 qhi[NF], qlo[NF];
#pragma unroll
    for (int f = 0; f < NF; ++f) {
        qhi[f] = __builtin_bit_cast(half8, qfrag[(f * 2 + 0) * 64 + lane]);
        qlo[f] = __builtin_bit_cast(half8, qfrag[(f * 2 + 1) * 64 + lane]);
    }
    struct Set { uint2 pc[PER]; float ps[PS]; };
    auto fetch = [&](Set& r, int tile) __attribute__((always_inline)) {
        if (tile > n_tiles - 1) tile = n_tiles - 1;
        const int lim = (tile == n_tiles - 1) ? last_lim : kTileVecs - 1;
        const uint2* cb = codes + (long long)tile * kTileVecs * C;
        const float* sb = scales + (long long)tile * kTileVecs * ns;
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int u = lane + 64 * i, rr = u / C, c = u % C;
            r.pc[i] = stream_load(&cb[(unsigned)(min(rr, lim) * C + c)]);
        }
#pragma unroll
        for (int i = 0; i < PS; ++i) {
            int e = lane + 64 * i;
            if (e > 32 * ns - 1) e = 32 * ns - 1;
            r.ps[i] = sb[(unsigned)(min(e / ns, lim) * ns + e % ns)];
        }
    };
    auto to_lds = [&](int b, const Set& r) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int u = lane + 64 * i, rr = u / C, c = u % C;
            dec[b][rr * ROW + 2 * c] = decode8(r.pc[i].x);
            dec[b][rr * ROW + 2 * c + 1] = decode8(r.pc[i].y);
        }
#pragma unroll
        for (int i = 0; i < PS; ++i) {
            int e = lane + 64 * i;
            if (e > 32 * ns - 1) e = 32 * ns - 1;        // surplus lanes rewrite the last scale: no branch
            scl[b][(e / ns) * SROW + e % ns] = r.ps[i];
        }
    };
    // lane (key, a) stores val[v] to row 2 v + a of out for v < its number of valid rows, elsewhere to its dump slot
    auto store_rows = [&](const float (&val)[NV], long long key, int a) __attribute__((always_inline)) {
        const int nv_lane = key < n_keys ? (n_q - a + 1) >> 1 : 0;
        long long at = (long long)a * n_keys + key;          // index of (row a, key); only used where it is valid
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            float* dst = v < nv_lane ? out + at : my_dump;
            *dst = val[v];
            at += 2 * n_keys;
        }
        // With many queries the kernel mostly writes; letting a tile's stores complete before the next stage
        // measured 3-5 % faster than keeping them in flight (s_waitcnt vmcnt(0); the other counters at their maximum).
        if constexpr (NV >= 8) __builtin_amdgcn_s_waitcnt(0x0F70);
    };
    // scores of the tile in dec[b] / scl[b]
    auto tile_scores = [&](int b, int tile) __attribute__((always_inline)) {
        if constexpr (R16) {
            // two MFMAs of 16 keys each per group (K = 32 codes = the whole group); lane l: key l % 16 (+ 16 c),
            // code unit 4 j + l / 16; result register i of lane l: MFMA row 4 (l / 16) + i
            const int key16 = lane & 15, a4 = lane >> 4;
            floatx4 o[2], acc0[2], acc1[2];
            auto group = [&](int j, floatx4 (&acc)[2]) __attribute__((always_inline)) {
#pragma unroll
                for (int c = 0; c < 2; ++c) {
                    const half8 bf = __builtin_bit_cast(half8, dec[b][(16 * c + key16) * ROW + 4 * j + a4]);
                    acc[c] = __builtin_amdgcn_mfma_f32_16x16x32_f16(qhi[j], bf, floatx4{0, 0, 0, 0}, 0, 0, 0);
                    acc[c] = __builtin_amdgcn_mfma_f32_16x16x32_f16(qlo[j], bf, acc[c], 0, 0, 0);
                }
            };
            auto fold = [&](int j, const floatx4 (&acc)[2]) __attribute__((always_inline)) {
#pragma unroll
                for (int c = 0; c < 2; ++c) {
                    const float sc = scl[b][(16 * c + key16) * SROW + j / gw];
#pragma unroll
                    for (int i = 0; i < 4; ++i) o[c][i] = j == 0 ? acc[c][i] * sc : fmaf(acc[c][i], sc, o[c][i]);
                }
            };
            group(0, acc0);
#pragma unroll
            for (int j = 1; j < G; ++j) {
                group(j, (j & 1) ? acc1 : acc0);
                fold(j - 1, (j & 1) ? acc0 : acc1);
                __builtin_amdgcn_sched_barrier(0);
            }
            fold(G - 1, ((G - 1) & 1) ? acc1 : acc0);
            // One swap per register puts the 32 keys of a row into one register: afterwards lane l holds key
            // 16 (l / 32) + l % 16; x[i] is MFMA row 4 a + i with a = (l % 32) / 16 (queries 2 i + a), y[i] is row
            // 4 (a + 2) + i (queries 8 + 2 i + a): val[v] = query 2 v + a.
            float x[4], y[4], val[NV];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(o[0][i]), __float_as_uint(o[1][i]),
                                                                 false, false);
                x[i] = __uint_as_float(sw[0]);
                y[i] = __uint_as_float(sw[1]);
            }
#pragma unroll
            for (int v = 0; v < NV; ++v) val[v] = v < 4 ? x[v] : y[v < 4 ? 0 : v - 4];
            store_rows(val, (long long)tile * kTileVecs + 16 * half + key16, (lane & 31) >> 4);
        } else {
            floatx16 o, acc0, acc1;
            const uint4* rowp = &dec[b][col * ROW + half];
            auto group = [&](int j, floatx16& acc) __attribute__((always_inline)) {
                acc = floatx16{0};
#pragma unroll
                for (int t = 0; t < 2; ++t) {
                    const half8 bf = __builtin_bit_cast(half8, rowp[2 * (2 * j + t)]);
                    acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(qhi[2 * j + t], bf, acc, 0, 0, 0);
                    acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(qlo[2 * j + t], bf, acc, 0, 0, 0);
                }
            };
            auto fold = [&](int j, const floatx16& acc) __attribute__((always_inline)) {
                const float sc = scl[b][col * SROW + j / gw];
#pragma unroll
                for (int v = 0; v < 16; ++v) o[v] = j == 0 ? acc[v] * sc : fmaf(acc[v], sc, o[v]);
            };
            // group j + 1 is on the matrix cores while group j is folded in; the scheduling barrier keeps the
            // compiler from reading every group's fragments up front (registers)
            group(0, acc0);
#pragma unroll
            for (int j = 1; j < G; ++j) {
                group(j, (j & 1) ? acc1 : acc0);
                fold(j - 1, (j & 1) ? acc0 : acc1);
                __builtin_amdgcn_sched_barrier(0);
            }
            fold(G - 1, ((G - 1) & 1) ? acc1 : acc0);
            float val[NV];
#pragma unroll
            for (int v = 0; v < NV; ++v) val[v] = o[v];
            store_rows(val, (long long)tile * kTileVecs + col, half);
        }
    };

    const int m = (n_tiles - 1 - t0) / stride + 1;       // the grid never exceeds the tiles
    Set ra, rb;
    fetch(ra, t0);
    fetch(rb, t0 + stride);
    hold_in_registers(qhi, qlo);
    to_lds(0, ra);
    // stage k: barrier (one wavefront: it orders the LDS writes before the reads); prefetch T_{k+2} into the set
    // that the previous stage decoded (the loads go out ahead of this stage's burst of stores); scores of T_k;
    // decode T_{k+1}
    __syncthreads();
    fetch(ra, t0 + 2 * stride);
    tile_scores(0, t0);
    to_lds(1, rb);
    int k = 1;
    for (; k + 1 < m; k += 2) {
        const int tk = t0 + k * stride;
        __syncthreads();                         // stage k (odd)
        rotate_priority(k);
        fetch(rb, tk + 2 * stride);
        tile_scores(1, tk);
        to_lds(0, ra);
        __syncthreads();                         // stage k + 1 (even)
        rotate_priority(k + 1);
        fetch(ra, tk + 3 * stride);
        tile_scores(0, tk + stride);
        to_lds(1, rb);
    }
    if (k < m) {
        __syncthreads();
        tile_scores(1, t0 + k * stride);
    }
}

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
template <int RU, bool STREAM>   // RU = ceil(r_units / 256): loads per thread and tile, all issued before any is used
__global__ void __launch_bounds__(256)
srft_mix_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, long long n_tiles, int r_units, int w_units) {
    for (long long t = blockIdx.x; t < n_tiles; t += gridDim.x) {
        const uint4* s = src + t * r_units;
        uint4 v[RU] = {};
        if (r_units > 0) {                       // uniform; r_units = 0 is the write-only stream
#pragma unroll
            for (int i = 0; i < RU; ++i) {
                const int u = threadIdx.x + 256 * i;
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

// ------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------
thread_local int g_last_hip_error = 0;

int hip_fail(hipError_t e) {
    g_last_hip_error = (int)e;
    return SRFT_ERR_HIP;
}
#define SRFT_HIP(call)                                   \
    do {                                                 \
        hipError_t e_ = (call);                          \
        if (e_ != hipSuccess) return hip_fail(e_);       \
    } while (0)

// double -> IEEE fp16 bits, round to nearest even, subnormals kept, overflow to infinity.
uint16_t f16_bits(double v) {
    const uint16_t sign = std::signbit(v) ? 0x8000u : 0u;
    double a = std::fabs(v);
    if (std::isnan(v)) return 0x7E00u;
    if (a >= 65520.0) return sign | 0x7C00u;
    if (a == 0.0) return sign;
    int e;
    std::frexp(a, &e);                    // a = m * 2^e, m in [0.5, 1)
    int E = e - 1;                        // a in [2^E, 2^(E+1))
    if (E < -14) E = -14;                 // subnormal range shares the quantum 2^-24
    const double r = std::nearbyint(std::ldexp(a, 10 - E));   // exact scaling, ties to even
    int mant = (int)r;                    // in [0, 2048]
    if (mant >= 2048) { mant = 1024; ++E; }
    if (mant < 1024) return sign | (uint16_t)mant;            // subnormal (E == -14)
    return sign | (uint16_t)(((E + 15) << 10) | (mant - 1024));
}

double f16_value(uint16_t b) {
    const int e = (b >> 10) & 0x1F, m = b & 0x3FF;
    double v = (e == 0) ? std::ldexp((double)m, -24) : std::ldexp((double)(m + 1024), e - 25);
    return (b & 0x8000u) ? -v : v;
}

uint64_t splitmix64_next(uint64_t& state) {
    state += 0x9E3779B97F4A7C15ull;
    uint64_t z = state;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

// Q[k][n] of the packed unitary real DFT (Eq. 1-2), rfft sign convention.
// Entry of the orthonormal Walsh-Hadamard matrix in natural order: (-1)^popcount(k & n) / sqrt(d).
double hadamard_entry(int d, int k, int n) {
    return (__builtin_popcount((unsigned)(k & n)) & 1 ? -1.0 : 1.0) / std::sqrt((double)d);
}

double q_entry(int d, int k, int n) {
    const int h = d / 2;
    const double pi = 3.14159265358979323846;
    if (k == 0) return 1.0 / std::sqrt((double)d);
    if (k == h) return ((n & 1) ? -1.0 : 1.0) / std::sqrt((double)d);
    const int kk = (k < h) ? k : k - h;
    const double ang = 2.0 * pi * (double)((long long)kk * n % d) / (double)d;
    return (k < h) ? std::sqrt(2.0 / d) * std::cos(ang) : -std::sqrt(2.0 / d) * std::sin(ang);
}

// slab row i of the 32x32 MFMA result (row = 8r + 4h + c) <-> output 16h + 4r + c of the slab,
// so that the 16 accumulators of a lane (r = v / 4, c = v % 4) are outputs 16h .. 16h + 15.
int slab_output_of_row(int i) {
    const int r = i / 8, h = (i / 4) % 2, c = i % 4;
    return 16 * h + 4 * r + c;
}

}  // namespace

struct srft_plan {
    int d = 0, g = 0, bits = 4, transform = 0, device = 0;
    uint64_t seed = 0;
    std::vector<int8_t> signs;
    uint4* wfrag = nullptr;     // write-path matrix fragments (device)
    uint4* rfrag = nullptr;     // read-path matrix fragments (device)
    uint4* rfold = nullptr;     // read-path fragments of the folded form (device), when fold_dq
    uint4* wfold = nullptr;     // write-path fragments of the folded form (device), when fold_q
    float* inv_lam2 = nullptr;  // 1 / (lambda * max(lambda, 1e-6)) per channel (device): scores in the rotated domain
    int grid_scores = 0;        // persistent grid of the scores kernel (32 rows of queries)
    int grid_scores16 = 0;      // the same with 16 rows
    bool fold_dq = false;       // read path contracts even and odd codes separately (half the matrix work)
    bool fold_q = false;        // write path contracts even and odd inputs separately (half the matrix work)
    float unscale_w = 1.0f;     // 2^-e of the write matrix
    float unscale_r = 1.0f;
    int grid_q = 0, grid_dq = 0;    // default persistent grid sizes
    int slabs_q = 1, slabs_dq = 1;  // slabs of the matrix per wavefront in the write / read kernel
    int gm = 1, gw = 1;             // group mode (kGroup16 / kGroup32 / kGroupWide) and slabs per group
    int max_wgs = 0;
};

struct srft_cache {
    std::vector<const srft_plan*> plans;
    std::vector<uint8_t*> codes;
    std::vector<float*> scales;
    std::vector<void*> view;
    int n_seq = 0, R = 0;
    int64_t capacity = 0, tokens = 0, quantized = 0;
};

namespace {

typedef void (*quantize_kernel_t)(const uint4*, const uint4*, long long, uint2*, float*, float4*, float, float, int);
typedef void (*dequantize_kernel_t)(const uint4*, const uint2*, const float*, long long, uint4*, float, int);

// The kernel instance for a plan: d, slabs per wavefront, group mode.
template <int D, int S, int BITS>
quantize_kernel_t quantize_codes_instance(int gm) {
    switch (gm) {
        case kGroup16: return srft_quantize_kernel<D, S, kOutCodes, kGroup16, BITS>;
        case kGroupWide: return srft_quantize_kernel<D, S, kOutCodes, kGroupWide, BITS>;
        default: return srft_quantize_kernel<D, S, kOutCodes, kGroup32, BITS>;
    }
}
template <int D, int S>
quantize_kernel_t quantize_instance(int out, int gm, int bits) {
    if (out == kOutRaw) return srft_quantize_kernel<D, S, kOutRaw, kGroup32, 4>;
    if (out == kOutAmax) return srft_quantize_kernel<D, S, kOutAmax, kGroup32, 4>;
    if constexpr (S == 1 && D % 64 == 0) {       // the scores set-up always runs one slab per wavefront
        if (out == kOutQFrag32) return srft_quantize_kernel<D, 1, kOutQFrag32, kGroup32, 4>;
        if (out == kOutQFrag16) return srft_quantize_kernel<D, 1, kOutQFrag16, kGroup32, 4>;
    }
    return bits == 8 ? quantize_codes_instance<D, S, 8>(gm) : quantize_codes_instance<D, S, 4>(gm);
}
template <int D>
quantize_kernel_t quantize_instance(int slabs, int out, int gm, bool fold, int bits) {
    if constexpr (D % 128 == 0) {
        if (fold && out == kOutCodes && gm != kGroup16) {
            if (gm == kGroupWide)
                return bits == 8 ? srft_quantize_fold_kernel<D, 8, true> : srft_quantize_fold_kernel<D, 4, true>;
            return bits == 8 ? srft_quantize_fold_kernel<D, 8, false> : srft_quantize_fold_kernel<D, 4, false>;
        }
    }
    if constexpr ((D / 32) % 2 == 0) {
        if (slabs == 2) return quantize_instance<D, 2>(out, gm, bits);
    }
    return quantize_instance<D, 1>(out, gm, bits);
}
template <int D, int BITS>
dequantize_kernel_t dequantize_instance_bits(int slabs, int gm, bool fold) {
    if constexpr ((D / 32) % 2 == 0) {
        if (fold && gm != kGroup16) return srft_dequantize_kernel<D, 2, 1, true, BITS>;
        if (slabs == 2)
            return gm == kGroup16 ? srft_dequantize_kernel<D, 2, 1, false, BITS>
                                  : srft_dequantize_kernel<D, 2, 2, false, BITS>;
    }
    return gm == kGroup16 ? srft_dequantize_kernel<D, 1, 1, false, BITS> : srft_dequantize_kernel<D, 1, 2, false, BITS>;
}
template <int D>
dequantize_kernel_t dequantize_instance(int slabs, int gm, bool fold, int bits) {
    return bits == 8 ? dequantize_instance_bits<D, 8>(slabs, gm, fold) : dequantize_instance_bits<D, 4>(slabs, gm, fold);
}

template <int D>
int occupancy_grids(srft_plan* p, int cus) {
    int bq = 0, bd = 0;
    SRFT_HIP(hipOccupancyMaxActiveBlocksPerMultiprocessor(&bq, quantize_instance<D>(p->slabs_q, kOutCodes, p->gm, p->fold_q, p->bits),
                                                          p->fold_q ? D : 2 * D / p->slabs_q, 0));
    SRFT_HIP(hipOccupancyMaxActiveBlocksPerMultiprocessor(&bd, dequantize_instance<D>(p->slabs_dq, p->gm, p->fold_dq, p->bits),
                                                          2 * D / p->slabs_dq, 0));
    p->grid_q = cus * (bq > 0 ? bq : 1);
    p->grid_dq = cus * (bd > 0 ? bd : 1);
    if constexpr (D % 64 == 0) {
        int bs = 0;
        SRFT_HIP(hipOccupancyMaxActiveBlocksPerMultiprocessor(&bs, srft_scores_kernel<D, 16, false>, 64, 0));
        p->grid_scores = cus * (bs > 0 ? bs : 1);
        SRFT_HIP(hipOccupancyMaxActiveBlocksPerMultiprocessor(&bs, srft_scores_kernel<D, 8, true>, 64, 0));
        p->grid_scores16 = cus * (bs > 0 ? bs : 1);
    }
    return SRFT_OK;
}

template <int D>
int launch_quantize(const srft_plan* p, const void* x, long long n, uint8_t* codes, float* scales,
                    float* wout, int out, hipStream_t st) {
    const long long n_tiles = (n + kTileVecs - 1) / kTileVecs;
    long long grid = p->max_wgs > 0 ? p->max_wgs : p->grid_q;
    if (grid > n_tiles) grid = n_tiles;
    const bool fold = p->fold_q && out == kOutCodes;
    const int slabs = (out == kOutQFrag32 || out == kOutQFrag16) ? 1 : p->slabs_q;
    const quantize_kernel_t kernel = quantize_instance<D>(slabs, out, p->gm, fold, p->bits);
    hipLaunchKernelGGL(kernel, dim3((unsigned)grid), dim3(fold ? D : 2 * D / slabs), 0, st,
                       fold ? p->wfold : p->wfrag, (const uint4*)x, n,
                       (uint2*)codes, scales, (float4*)wout, p->unscale_w, p->unscale_w / (p->bits == 8 ? 127.0f : 7.0f),
                       p->gw);
    SRFT_HIP(hipGetLastError());
    return SRFT_OK;
}

template <int D>
int launch_dequantize(const srft_plan* p, const uint8_t* codes, const float* scales, long long n, void* out,
                      hipStream_t st) {
    const long long n_tiles = (n + kTileVecs - 1) / kTileVecs;
    long long grid = p->max_wgs > 0 ? p->max_wgs : p->grid_dq;
    if (grid > n_tiles) grid = n_tiles;
    const dequantize_kernel_t kernel = dequantize_instance<D>(p->slabs_dq, p->gm, p->fold_dq, p->bits);
    hipLaunchKernelGGL(kernel, dim3((unsigned)grid), dim3(2 * D / p->slabs_dq), 0, st,
                       p->fold_dq ? p->rfold : p->rfrag, (const uint2*)codes,
                       scales, n, (uint4*)out, p->unscale_r, p->gw);
    SRFT_HIP(hipGetLastError());
    return SRFT_OK;
}

typedef void (*quantize_batched_kernel_t)(const srft_batch_args, int);
typedef void (*dequantize_batched_kernel_t)(const srft_batch_args, int);

template <int D, int S, int BITS>
quantize_batched_kernel_t quantize_batched_instance_gm(int gm) {
    return gm == kGroup16 ? srft_quantize_batched_kernel<D, S, kGroup16, BITS>
         : gm == kGroupWide ? srft_quantize_batched_kernel<D, S, kGroupWide, BITS>
                            : srft_quantize_batched_kernel<D, S, kGroup32, BITS>;
}
template <int D>
quantize_batched_kernel_t quantize_batched_instance(int slabs, int gm, bool fold, int bits) {
    if constexpr (D % 128 == 0) {
        if (fold && gm != kGroup16) {
            if (gm == kGroupWide)
                return bits == 8 ? srft_quantize_fold_batched_kernel<D, 8, true>
                                 : srft_quantize_fold_batched_kernel<D, 4, true>;
            return bits == 8 ? srft_quantize_fold_batched_kernel<D, 8, false>
                             : srft_quantize_fold_batched_kernel<D, 4, false>;
        }
    }
    if constexpr ((D / 32) % 2 == 0) {
        if (slabs == 2)
            return bits == 8 ? quantize_batched_instance_gm<D, 2, 8>(gm) : quantize_batched_instance_gm<D, 2, 4>(gm);
    }
    return bits == 8 ? quantize_batched_instance_gm<D, 1, 8>(gm) : quantize_batched_instance_gm<D, 1, 4>(gm);
}
template <int D, int BITS>
dequantize_batched_kernel_t dequantize_batched_instance_bits(int slabs, int gm, bool fold) {
    if constexpr ((D / 32) % 2 == 0) {
        if (fold && gm != kGroup16) return srft_dequantize_batched_kernel<D, 2, 1, true, BITS>;
        if (slabs == 2)
            return gm == kGroup16 ? srft_dequantize_batched_kernel<D, 2, 1, false, BITS>
                                  : srft_dequantize_batched_kernel<D, 2, 2, false, BITS>;
    }
    return gm == kGroup16 ? srft_dequantize_batched_kernel<D, 1, 1, false, BITS>
                          : srft_dequantize_batched_kernel<D, 1, 2, false, BITS>;
}
template <int D>
dequantize_batched_kernel_t dequantize_batched_instance(int slabs, int gm, bool fold, int bits) {
    return bits == 8 ? dequantize_batched_instance_bits<D, 8>(slabs, gm, fold)
                     : dequantize_batched_instance_bits<D, 4>(slabs, gm, fold);
}

// One batched launch: the segment table is complete except for first_block, which is laid out here.
// Every segment gets at least one workgroup and at most one per tile; when the tiles of all segments
// exceed the persistent grid, workgroups are shared out in proportion to the tiles.
template <int D>
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
    const int slabs = write_path ? p->slabs_q : p->slabs_dq;
    if (write_path)
        hipLaunchKernelGGL(quantize_batched_instance<D>(slabs, p->gm, p->fold_q, p->bits), dim3((unsigned)next),
                           dim3(p->fold_q ? D : 2 * D / slabs), 0, st, a, p->gw);
    else
        hipLaunchKernelGGL(dequantize_batched_instance<D>(slabs, p->gm, p->fold_dq, p->bits), dim3((unsigned)next),
                           dim3(2 * D / slabs), 0, st, a, p->gw);
    SRFT_HIP(hipGetLastError());
    return SRFT_OK;
}

#define SRFT_DISPATCH_D(d, fn, ...)                       \
    switch (d) {                                          \
        case 32:  return fn<32>(__VA_ARGS__);             \
        case 64:  return fn<64>(__VA_ARGS__);             \
        case 96:  return fn<96>(__VA_ARGS__);             \
        case 128: return fn<128>(__VA_ARGS__);            \
        case 160: return fn<160>(__VA_ARGS__);            \
        case 192: return fn<192>(__VA_ARGS__);            \
        case 224: return fn<224>(__VA_ARGS__);            \
        case 256: return fn<256>(__VA_ARGS__);            \
        default:  return SRFT_ERR_BAD_D;                  \
    }

template <int D>
int launch_scores(const srft_plan* p, uint4* qfrag, float* dump, int n_q, const uint8_t* codes,
                  const float* scales, long long n_keys, float* out, hipStream_t st) {
    if constexpr (D % 64 == 0) {
        const bool r16 = n_q <= 16;             // 16 MFMA rows are enough: half the matrix-core time
        const long long n_tiles = (n_keys + kTileVecs - 1) / kTileVecs;
        long long grid = p->max_wgs > 0 ? p->max_wgs : (r16 ? p->grid_scores16 : p->grid_scores);
        if (grid > n_tiles) grid = n_tiles;
        if (grid > kMaxScoreWorkgroups) grid = kMaxScoreWorkgroups;      // each has its 64 floats of `dump`
        const int nv = (n_q + 1) / 2;            // result registers a lane has to store
        auto kernel = nv <= 1 ? srft_scores_kernel<D, 1, true> : nv <= 2 ? srft_scores_kernel<D, 2, true>
                    : nv <= 4 ? srft_scores_kernel<D, 4, true> : nv <= 8 ? srft_scores_kernel<D, 8, true>
                                                                         : srft_scores_kernel<D, 16, false>;
        hipLaunchKernelGGL(kernel, dim3((unsigned)grid), dim3(64), 0, st, (const uint4*)qfrag,
                           (const uint2*)codes, scales, n_keys, out, n_q, p->gw, dump);
        SRFT_HIP(hipGetLastError());
        return SRFT_OK;
    } else {
        return SRFT_ERR_BAD_D;
    }
}

int dispatch_occupancy(srft_plan* p, int cus) { SRFT_DISPATCH_D(p->d, occupancy_grids, p, cus) }
int dispatch_scores(const srft_plan* p, uint4* qfrag, float* dump, int n_q, const uint8_t* c,
                    const float* s, long long n, float* o, hipStream_t st) {
    SRFT_DISPATCH_D(p->d, launch_scores, p, qfrag, dump, n_q, c, s, n, o, st)
}
int dispatch_quantize(const srft_plan* p, const void* x, long long n, uint8_t* c, float* s, float* w, int out,
                      hipStream_t st) { SRFT_DISPATCH_D(p->d, launch_quantize, p, x, n, c, s, w, out, st) }
int dispatch_dequantize(const srft_plan* p, const uint8_t* c, const float* s, long long n, void* o,
                        hipStream_t st) { SRFT_DISPATCH_D(p->d, launch_dequantize, p, c, s, n, o, st) }

int dispatch_batched(const srft_plan* p, srft_batch_args& a, bool write_path, hipStream_t st) {
    SRFT_DISPATCH_D(p->d, launch_batched, p, a, write_path, st)
}

// Slabs per wavefront: 1, or 2 where the number of groups is even and the table (or the tuning override in
// the environment) says so.
int default_slabs(int d, const char* env_name, int table_value) {
    int s = table_value;
    if (const char* e = std::getenv(env_name)) s = std::atoi(e);
    if (s != 2 || (d / 32) % 2 != 0) s = 1;
    return s;
}

bool aligned(const void* p, size_t a) { return ((uintptr_t)p & (a - 1)) == 0; }

// The kernels index tiles of 32 vectors with 32-bit integers and look a few grid strides ahead.
constexpr int64_t kMaxVectors = (int64_t)1 << 33;

// Scale a matrix by the power of two that puts its largest magnitude in [2^13, 2^14) and split every
// entry into fp16 hi + fp16 lo.  Returns the exponent e (entries were multiplied by 2^e).
int split_hi_lo(const std::vector<double>& m, std::vector<uint16_t>& hi, std::vector<uint16_t>& lo) {
    double mx = 0.0;
    for (double v : m) mx = std::fmax(mx, std::fabs(v));
    int e2;
    std::frexp(mx, &e2);                 // mx in [2^(e2-1), 2^e2)
    const int e = 14 - e2;
    hi.resize(m.size());
    lo.resize(m.size());
    for (size_t i = 0; i < m.size(); ++i) {
        const double v = std::ldexp(m[i], e);
        hi[i] = f16_bits(v);
        lo[i] = f16_bits(v - f16_value(hi[i]));
    }
    return e;
}

}  // namespace

extern "C" {

int srft_plan_create(srft_plan_t** out, int d, int group_size, uint64_t sign_seed, const float* lambda_host) {
    return srft_plan_create_bits(out, d, group_size, 4, sign_seed, lambda_host);
}

int srft_plan_create_bits(srft_plan_t** out, int d, int group_size, int bits, uint64_t sign_seed,
                          const float* lambda_host) {
    return srft_plan_create_ex(out, d, group_size, bits, SRFT_TRANSFORM_DFT, sign_seed, lambda_host);
}

int srft_plan_create_ex(srft_plan_t** out, int d, int group_size, int bits, int transform, uint64_t sign_seed,
                        const float* lambda_host) {
    if (!out) return SRFT_ERR_NULL;
    *out = nullptr;
    if (bits != 4 && bits != 8) return SRFT_ERR_BAD_BITS;
    if (transform != SRFT_TRANSFORM_DFT && transform != SRFT_TRANSFORM_HADAMARD) return SRFT_ERR_BAD_TRANSFORM;
    if (d < 32 || d > kMaxD || d % 32 != 0) return SRFT_ERR_BAD_D;
    if (transform == SRFT_TRANSFORM_HADAMARD && (d & (d - 1)) != 0) return SRFT_ERR_BAD_D;
    if (!(group_size == 16 || (group_size >= 32 && group_size % 32 == 0 && d % group_size == 0))) return SRFT_ERR_BAD_GROUP;
    std::vector<double> lam(d, 1.0);
    if (lambda_host) {
        double lo = INFINITY, hi = 0.0;
        for (int k = 0; k < d; ++k) {
            const float v = lambda_host[k];
            if (!std::isfinite(v) || !(v > 0.0f)) return SRFT_ERR_BAD_LAMBDA;
            lam[k] = (double)v;
            lo = std::fmin(lo, lam[k]);
            hi = std::fmax(hi, lam[k]);
        }
        if (hi / lo > 65536.0) return SRFT_ERR_BAD_LAMBDA;
    }

    srft_plan* p = new (std::nothrow) srft_plan();
    if (!p) return SRFT_ERR_HIP;
    p->d = d;
    p->g = group_size;
    p->bits = bits;
    p->transform = transform;
    p->gm = group_size == 16 ? kGroup16 : (group_size == 32 ? kGroup32 : kGroupWide);
    p->gw = group_size <= 32 ? 1 : group_size / 32;
    p->seed = sign_seed;
    p->signs.resize(d);
    uint64_t state = sign_seed;
    for (int n = 0; n < d; ++n) p->signs[n] = (splitmix64_next(state) >> 63) ? -1 : 1;

    // W[k][n] = lambda_k Q[k][n] s_n ; R[n][k] = s_n Q[k][n] / max(lambda_k, 1e-6)
    std::vector<double> W((size_t)d * d), R((size_t)d * d);
    for (int k = 0; k < d; ++k)
        for (int n = 0; n < d; ++n) {
            const double q = (transform == SRFT_TRANSFORM_HADAMARD ? hadamard_entry(d, k, n) : q_entry(d, k, n)) *
                             (double)p->signs[n];
            W[(size_t)k * d + n] = lam[k] * q;
            R[(size_t)n * d + k] = q / std::fmax(lam[k], 1e-6);
        }
    std::vector<uint16_t> whi, wlo, rhi, rlo;
    p->unscale_w = (float)std::ldexp(1.0, -split_hi_lo(W, whi, wlo));
    p->unscale_r = (float)std::ldexp(1.0, -split_hi_lo(R, rhi, rlo));

    // A-operand fragments: lane l holds row l % 32 of the slab and contraction indices 8 (l / 32) + e.
    const int G = d / 32, T = d / 16;
    std::vector<uint16_t> wf((size_t)G * T * 2 * 64 * 8), rf((size_t)G * G * 2 * 2 * 64 * 8);
    for (int w = 0; w < G; ++w)
        for (int l = 0; l < 64; ++l) {
            const int row = 32 * w + slab_output_of_row(l % 32), kh = l / 32;
            for (int t = 0; t < T; ++t)           // write path: contraction index = input position n
                for (int e = 0; e < 8; ++e) {
                    const size_t src = (size_t)row * d + (16 * t + 8 * kh + e);
                    wf[((((size_t)w * T + t) * 2 + 0) * 64 + l) * 8 + e] = whi[src];
                    wf[((((size_t)w * T + t) * 2 + 1) * 64 + l) * 8 + e] = wlo[src];
                }
            // read path: group j, run of 8 codes 4j + 2t + kh; element e <-> code e/2 + 4 (e % 2) of the run at
            // 4 bits (nibble pairs (n0, n4), (n1, n5), ...), code {0, 2, 1, 3, 4, 6, 5, 7}[e] at 8 bits (byte pairs
            // (b0, b2), (b1, b3) of each dword): the orders in which the kernel's decode lays the codes out
            static const int byte_order[8] = {0, 2, 1, 3, 4, 6, 5, 7};
            for (int j = 0; j < G; ++j)
                for (int t = 0; t < 2; ++t)
                    for (int e = 0; e < 8; ++e) {
                        const int k = 8 * (4 * j + 2 * t + kh) + (bits == 8 ? byte_order[e] : (e / 2) + 4 * (e % 2));
                        const size_t src = (size_t)row * d + k;
                        rf[(((((size_t)w * G + j) * 2 + t) * 2 + 0) * 64 + l) * 8 + e] = rhi[src];
                        rf[(((((size_t)w * G + j) * 2 + t) * 2 + 1) * 64 + l) * 8 + e] = rlo[src];
                    }
        }

    p->slabs_q = default_slabs(d, "SRFT_SLABS_Q", d == 64 ? 2 : 1);
    p->slabs_dq = default_slabs(d, "SRFT_SLABS_DQ", (d == 256 || d == 64) ? 2 : 1);
    // Folded read path where it applies and pays (d = 128, 192, 256; g >= 32); SRFT_FOLD_DQ=0 turns it off (tuning).
    p->fold_dq = (d % 64 == 0) && d >= 128 && p->gm != kGroup16 &&    // at d = 64 it gains nothing
                 transform == SRFT_TRANSFORM_DFT;                      // (the symmetries are the DFT's)
    if (const char* e = std::getenv("SRFT_FOLD_DQ")) p->fold_dq = p->fold_dq && std::atoi(e) != 0;
    std::vector<uint16_t> rfold;
    if (p->fold_dq) {
        p->slabs_dq = 2;
        // A (even p) and B (odd p) fragments of wavefront w: row n = 32w + (output of MFMA row l % 32); group j,
        // lane half kh, element e <-> packed index 32j + 16 kh + off[e] (+ 1 for B), off[] being the order in
        // which the kernel lays out the decoded low nibbles of an 8-byte unit: (n0, n4, n2, n6) of each dword.
        // (at 8 bits: bytes 0 and 2 of each of the four dwords)
        static const int off4[8] = {0, 4, 2, 6, 8, 12, 10, 14}, off8[8] = {0, 2, 4, 6, 8, 10, 12, 14};
        const int* off = bits == 8 ? off8 : off4;
        const int waves = d / 64;
        const size_t frag_halves = (size_t)waves * 2 * G * 2 * 64 * 8;
        rfold.assign(frag_halves + (size_t)waves * 64 * 16, 0);
        for (int w = 0; w < waves; ++w)
            for (int l = 0; l < 64; ++l) {
                const int n = 32 * w + slab_output_of_row(l % 32), kh = l / 32;
                for (int ab = 0; ab < 2; ++ab)
                    for (int j = 0; j < G; ++j)
                        for (int e = 0; e < 8; ++e) {
                            const size_t src = (size_t)n * d + (32 * j + 16 * kh + off[e] + ab);
                            const size_t dst = (((size_t)(w * 2 + ab) * G + j) * 2) * 64;
                            rfold[((dst + 0) + l) * 8 + e] = rhi[src];
                            rfold[((dst + 64) + l) * 8 + e] = rlo[src];
                        }
                // sign-bit masks for this lane's outputs n + d/2, n = 32w + 16 kh + v: s_n s_{n+d/2} < 0
                for (int v = 0; v < 16; ++v) {
                    const int nn = 32 * w + 16 * kh + v;
                    rfold[frag_halves + ((size_t)w * 64 + l) * 16 + v] =
                        (p->signs[nn] * p->signs[nn + d / 2] < 0) ? 0x8000u : 0u;
                }
            }
    }
    // Folded write path where it applies (d a multiple of 128, g >= 32); SRFT_FOLD_Q=0 turns it off (tuning).
    p->fold_q = (d % 128 == 0) && p->gm != kGroup16 && transform == SRFT_TRANSFORM_DFT;
    if (const char* e = std::getenv("SRFT_FOLD_Q")) p->fold_q = p->fold_q && std::atoi(e) != 0;
    std::vector<uint16_t> wfold;
    if (p->fold_q) {
        // Wavefront w < M/2 owns cosine rows k = 32w + i, the others sine rows; row i of its E (O) slab is row
        // p = k (cosine) or d/2 + k (sine) of W restricted to even (odd) n.  The first sine wavefront has no k = 0:
        // there E is row d/4 and O is row 3d/4.  k-step t, lane half kh, element e <-> n = 32t + 16kh + 2e (+ 1).
        const int M = d / 64, TF = d / 32;
        const size_t frag_halves = (size_t)M * 2 * TF * 2 * 64 * 8;
        wfold.assign(frag_halves + (size_t)M * 64 * 16 * 2, 0);          // rho: 16 floats = 32 halves per lane
        for (int w = 0; w < M; ++w) {
            const bool sine = w >= M / 2;
            const int wk = sine ? w - M / 2 : w;
            for (int l = 0; l < 64; ++l) {
                const int kh = l / 32, k = 32 * wk + slab_output_of_row(l % 32);
                for (int eo = 0; eo < 2; ++eo) {
                    int prow = sine ? d / 2 + k : k;
                    if (sine && k == 0) prow = eo == 0 ? d / 4 : 3 * d / 4;
                    for (int t = 0; t < TF; ++t)
                        for (int e = 0; e < 8; ++e) {
                            const size_t src = (size_t)prow * d + (32 * t + 16 * kh + 2 * e + eo);
                            const size_t dst = (((size_t)(w * 2 + eo) * TF + t) * 2) * 64;
                            wfold[((dst + 0) + l) * 8 + e] = whi[src];
                            wfold[((dst + 64) + l) * 8 + e] = wlo[src];
                        }
                }
                // rho of this lane's 16 values k = 32 wk + 16 kh + v: lambda_mirror / lambda_direct, negated in the
                // sine block; 0 where there is no mirror value (k = 0 of the sine block)
                for (int v = 0; v < 16; ++v) {
                    const int kk = 32 * wk + 16 * kh + v;
                    const int pd = sine ? d / 2 + kk : kk, pm = sine ? d - kk : d / 2 - kk;
                    float r = 0.0f;
                    if (!(sine && kk == 0)) r = (float)((sine ? -1.0 : 1.0) * lam[pm] / lam[pd]);
                    uint32_t bits;
                    std::memcpy(&bits, &r, 4);
                    const size_t at = frag_halves + (((size_t)w * 64 + l) * 16 + v) * 2;
                    wfold[at] = (uint16_t)(bits & 0xFFFFu);
                    wfold[at + 1] = (uint16_t)(bits >> 16);
                }
            }
        }
    }
    hipError_t e = hipGetDevice(&p->device);
    int cus = 0;
    if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, p->device);
    if (e == hipSuccess) e = hipMalloc((void**)&p->wfrag, wf.size() * 2);
    if (e == hipSuccess) e = hipMalloc((void**)&p->rfrag, rf.size() * 2);
    if (e == hipSuccess) e = hipMemcpy(p->wfrag, wf.data(), wf.size() * 2, hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy(p->rfrag, rf.data(), rf.size() * 2, hipMemcpyHostToDevice);
    std::vector<float> il2(d);
    for (int k = 0; k < d; ++k) il2[k] = (float)(1.0 / (lam[k] * std::fmax(lam[k], 1e-6)));
    if (e == hipSuccess) e = hipMalloc((void**)&p->inv_lam2, d * sizeof(float));
    if (e == hipSuccess) e = hipMemcpy(p->inv_lam2, il2.data(), d * sizeof(float), hipMemcpyHostToDevice);
    if (e == hipSuccess && p->fold_q) e = hipMalloc((void**)&p->wfold, wfold.size() * 2);
    if (e == hipSuccess && p->fold_q) e = hipMemcpy(p->wfold, wfold.data(), wfold.size() * 2, hipMemcpyHostToDevice);
    if (e == hipSuccess && p->fold_dq) e = hipMalloc((void**)&p->rfold, rfold.size() * 2);
    if (e == hipSuccess && p->fold_dq) e = hipMemcpy(p->rfold, rfold.data(), rfold.size() * 2, hipMemcpyHostToDevice);
    int rc = (e == hipSuccess) ? dispatch_occupancy(p, cus) : hip_fail(e);
    if (rc != SRFT_OK) {
        srft_plan_destroy(p);
        return rc;
    }
    *out = p;
    return SRFT_OK;
}

int srft_plan_destroy(srft_plan_t* plan) {
    if (!plan) return SRFT_OK;
    hipError_t e1 = plan->wfrag ? hipFree(plan->wfrag) : hipSuccess;
    hipError_t e2 = plan->rfrag ? hipFree(plan->rfrag) : hipSuccess;
    hipError_t e3 = plan->rfold ? hipFree(plan->rfold) : hipSuccess;
    if (plan->wfold) {
        const hipError_t e4 = hipFree(plan->wfold);
        if (e3 == hipSuccess) e3 = e4;
    }
    if (plan->inv_lam2) {
        const hipError_t e5 = hipFree(plan->inv_lam2);
        if (e3 == hipSuccess) e3 = e5;
    }
    delete plan;
    if (e1 != hipSuccess) return hip_fail(e1);
    if (e2 != hipSuccess) return hip_fail(e2);
    if (e3 != hipSuccess) return hip_fail(e3);
    return SRFT_OK;
}

int srft_kv_quantize(const srft_plan_t* plan, const void* x_f16_dev, int64_t n_vec, uint8_t* codes_dev,
                     float* scales_dev, void* hip_stream) {
    if (!plan) return SRFT_ERR_NULL;
    if (n_vec < 0 || n_vec > kMaxVectors) return SRFT_ERR_BAD_N;
    if (n_vec == 0) return SRFT_OK;
    if (!x_f16_dev || !codes_dev || !scales_dev) return SRFT_ERR_NULL;
    if (!aligned(x_f16_dev, 16) || !aligned(codes_dev, 16) || !aligned(scales_dev, 4)) return SRFT_ERR_ALIGN;
    return dispatch_quantize(plan, x_f16_dev, n_vec, codes_dev, scales_dev, nullptr, kOutCodes, (hipStream_t)hip_stream);
}

int srft_kv_forward_f32(const srft_plan_t* plan, const void* x_f16_dev, int64_t n_vec, float* w_f32_dev,
                        void* hip_stream) {
    if (!plan) return SRFT_ERR_NULL;
    if (n_vec < 0 || n_vec > kMaxVectors) return SRFT_ERR_BAD_N;
    if (n_vec == 0) return SRFT_OK;
    if (!x_f16_dev || !w_f32_dev) return SRFT_ERR_NULL;
    if (!aligned(x_f16_dev, 16) || !aligned(w_f32_dev, 16)) return SRFT_ERR_ALIGN;
    return dispatch_quantize(plan, x_f16_dev, n_vec, nullptr, nullptr, w_f32_dev, kOutRaw, (hipStream_t)hip_stream);
}

int srft_kv_channel_absmax(const srft_plan_t* plan, const void* x_f16_dev, int64_t n_vec, float* amax_dev,
                           void* hip_stream) {
    if (!plan) return SRFT_ERR_NULL;
    if (n_vec < 0 || n_vec > kMaxVectors) return SRFT_ERR_BAD_N;
    if (n_vec == 0) return SRFT_OK;
    if (!x_f16_dev || !amax_dev) return SRFT_ERR_NULL;
    if (!aligned(x_f16_dev, 16) || !aligned(amax_dev, 4)) return SRFT_ERR_ALIGN;
    return dispatch_quantize(plan, x_f16_dev, n_vec, nullptr, nullptr, amax_dev, kOutAmax, (hipStream_t)hip_stream);
}

int64_t srft_scores_workspace_bytes(const srft_plan_t* plan) {
    if (!plan) return SRFT_ERR_NULL;
    // the A fragments of up to 32 queries: d/16 k-steps x (hi, lo) x 64 lanes x 16 bytes, then 64 floats per
    // workgroup that absorb the stores of lanes without a valid (query, key)
    return (int64_t)(plan->d / 16) * 2 * 64 * 16 + (int64_t)kMaxScoreWorkgroups * 64 * 4;
}

int srft_kv_scores(const srft_plan_t* plan, const void* q_f16_dev, int n_q, const uint8_t* codes_dev,
                   const float* scales_dev, int64_t n_keys, float* scores_dev, void* workspace_dev, void* hip_stream) {
    if (!plan) return SRFT_ERR_NULL;
    if (plan->d % 64 != 0) return SRFT_ERR_BAD_D;
    if (plan->bits != 4) return SRFT_ERR_BAD_BITS;
    if (plan->gm == kGroup16) return SRFT_ERR_BAD_GROUP;
    if (n_q < 1 || n_q > 32 || n_keys < 0 || n_keys > kMaxVectors) return SRFT_ERR_BAD_N;
    if (n_keys == 0) return SRFT_OK;
    if (!q_f16_dev || !codes_dev || !scales_dev || !scores_dev || !workspace_dev) return SRFT_ERR_NULL;
    if (!aligned(q_f16_dev, 16) || !aligned(codes_dev, 16) || !aligned(scales_dev, 4) || !aligned(scores_dev, 4) ||
        !aligned(workspace_dev, 16))
        return SRFT_ERR_ALIGN;
    hipStream_t st = (hipStream_t)hip_stream;
    uint4* qfrag = (uint4*)workspace_dev;
    float* dump = (float*)((char*)qfrag + (size_t)(plan->d / 16) * 2 * 64 * 16);
    // the write path's plain kernel transforms the queries and stores them as the scan's MFMA operands
    const int rc = dispatch_quantize(plan, q_f16_dev, n_q, nullptr, plan->inv_lam2, (float*)qfrag,
                                     n_q <= 16 ? kOutQFrag16 : kOutQFrag32, st);
    if (rc != SRFT_OK) return rc;
    return dispatch_scores(plan, qfrag, dump, n_q, codes_dev, scales_dev, n_keys, scores_dev, st);
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
    if (!aligned(codes_dev, 16) || !aligned(scales_dev, 4) || !aligned(out_f16_dev, 16)) return SRFT_ERR_ALIGN;
    return dispatch_dequantize(plan, codes_dev, scales_dev, n_vec, out_f16_dev, (hipStream_t)hip_stream);
}

// Shared body of the two batched entry points.  in1 / out1 are NULL arrays where the path has no such buffer.
static int run_batched(const srft_plan_t* const* plans, const void* const* in0, const void* const* in1,
                       void* const* out0, void* const* out1, const int64_t* n_vec, int count, bool write_path,
                       hipStream_t st) {
    if (count < 0) return SRFT_ERR_BAD_N;
    if (count == 0) return SRFT_OK;
    if (!plans || !in0 || !out0 || !n_vec || (write_path ? !out1 : !in1)) return SRFT_ERR_NULL;
    // validate everything before the first launch: a bad segment must not leave half a batch enqueued
    for (int i = 0; i < count; ++i) {
        if (!plans[i]) return SRFT_ERR_NULL;
        if (plans[i]->d != plans[0]->d || plans[i]->g != plans[0]->g || plans[i]->bits != plans[0]->bits ||
            plans[i]->transform != plans[0]->transform || plans[i]->device != plans[0]->device)
            return SRFT_ERR_MISMATCH;
        if (n_vec[i] < 0 || n_vec[i] > kMaxVectors) return SRFT_ERR_BAD_N;
        if (n_vec[i] == 0) continue;
        const void* small = write_path ? (const void*)out1[i] : in1[i];       // the scales
        if (!in0[i] || !out0[i] || !small) return SRFT_ERR_NULL;
        if (!aligned(in0[i], 16) || !aligned(out0[i], 16) || !aligned(small, 4)) return SRFT_ERR_ALIGN;
    }
    srft_batch_args a;
    a.count = 0;
    for (int i = 0; i <= count; ++i) {
        if (i < count && n_vec[i] > 0) {
            const int k = a.count++;
            a.frag[k] = write_path ? (plans[i]->fold_q ? plans[i]->wfold : plans[i]->wfrag)
                                   : (plans[i]->fold_dq ? plans[i]->rfold : plans[i]->rfrag);
            a.in0[k] = in0[i];
            a.in1[k] = write_path ? nullptr : in1[i];
            a.out0[k] = out0[i];
            a.out1[k] = write_path ? out1[i] : nullptr;
            a.n_vec[k] = n_vec[i];
            a.unscale[k] = write_path ? plans[i]->unscale_w : plans[i]->unscale_r;
        }
        if (a.count == kMaxBatch || (i == count && a.count > 0)) {
            const int rc = dispatch_batched(plans[0], a, write_path, st);
            if (rc != SRFT_OK) return rc;
            a.count = 0;
        }
    }
    return SRFT_OK;
}

int srft_kv_quantize_batched(const srft_plan_t* const* plans, const void* const* x_f16_dev, const int64_t* n_vec,
                             uint8_t* const* codes_dev, float* const* scales_dev, int count, void* hip_stream) {
    return run_batched(plans, x_f16_dev, nullptr, (void* const*)codes_dev, (void* const*)scales_dev, n_vec, count,
                       true, (hipStream_t)hip_stream);
}

int srft_kv_dequantize_batched(const srft_plan_t* const* plans, const uint8_t* const* codes_dev,
                               const float* const* scales_dev, const int64_t* n_vec, void* const* out_f16_dev,
                               int count, void* hip_stream) {
    return run_batched(plans, (const void* const*)codes_dev, (const void* const*)scales_dev, out_f16_dev, nullptr,
                       n_vec, count, false, (hipStream_t)hip_stream);
}

// ---------------------------------------------------------------------------------------------------------
// cache manager (host bookkeeping around the batched kernels)
// ---------------------------------------------------------------------------------------------------------
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
        if (plans[i]->d != plans[0]->d || plans[i]->g != plans[0]->g || plans[i]->bits != plans[0]->bits ||
            plans[i]->transform != plans[0]->transform || plans[i]->device != plans[0]->device)
            return SRFT_ERR_MISMATCH;
        if (!aligned(codes_dev[i], 16) || !aligned(scales_dev[i], 4) || !aligned(view_f16_dev[i], 16))
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
        const int rc = run_batched(c->plans.data(), x.data(), nullptr, cdo.data(), sco.data(), n.data(), (int)np,
                                   true, st);
        if (rc != SRFT_OK) return rc;
    }
    return run_batched(c->plans.data(), cd.data(), sc.data(), xo.data(), nullptr, n.data(), (int)np, false, st);
}

int srft_cache_append(srft_cache_t* cache, const void* const* new_f16_dev, int t, void* hip_stream) {
    if (!cache) return SRFT_ERR_NULL;
    if (t < 0 || cache->tokens + t > cache->capacity) return SRFT_ERR_BAD_N;
    if (t == 0) return SRFT_OK;
    if (!new_f16_dev) return SRFT_ERR_NULL;
    const size_t np = cache->plans.size();
    for (size_t i = 0; i < np; ++i) {
        if (!new_f16_dev[i]) return SRFT_ERR_NULL;
        if (!aligned(new_f16_dev[i], 16)) return SRFT_ERR_ALIGN;
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

int srft_plan_d(const srft_plan_t* plan) { return plan ? plan->d : SRFT_ERR_NULL; }
int srft_plan_group_size(const srft_plan_t* plan) { return plan ? plan->g : SRFT_ERR_NULL; }
int srft_plan_groups(const srft_plan_t* plan) { return plan ? plan->d / plan->g : SRFT_ERR_NULL; }
int srft_plan_code_bytes(const srft_plan_t* plan) { return plan ? plan->d * plan->bits / 8 : SRFT_ERR_NULL; }
int srft_plan_bits(const srft_plan_t* plan) { return plan ? plan->bits : SRFT_ERR_NULL; }

int srft_plan_get_signs(const srft_plan_t* plan, int8_t* out_host) {
    if (!plan || !out_host) return SRFT_ERR_NULL;
    std::memcpy(out_host, plan->signs.data(), plan->signs.size());
    return SRFT_OK;
}

int srft_plan_set_max_workgroups(srft_plan_t* plan, int max_workgroups) {
    if (!plan) return SRFT_ERR_NULL;
    if (max_workgroups < 0) return SRFT_ERR_BAD_N;
    plan->max_wgs = max_workgroups;
    return SRFT_OK;
}

int srft_stream_copy(void* dst_dev, const void* src_dev, int64_t n_bytes, void* hip_stream) {
    if (n_bytes < 0 || n_bytes % 16 != 0) return SRFT_ERR_BAD_N;
    if (n_bytes == 0) return SRFT_OK;
    if (!dst_dev || !src_dev) return SRFT_ERR_NULL;
    if (!aligned(dst_dev, 16) || !aligned(src_dev, 16)) return SRFT_ERR_ALIGN;
    int dev = 0, cus = 0;
    SRFT_HIP(hipGetDevice(&dev));
    SRFT_HIP(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
    const long long units = n_bytes / 16;
    long long grid = (long long)cus * 8;
    if (grid > (units + 255) / 256) grid = (units + 255) / 256;
    hipLaunchKernelGGL(srft_copy_kernel, dim3((unsigned)grid), dim3(256), 0, (hipStream_t)hip_stream, (uint4*)dst_dev,
                       (const uint4*)src_dev, units);
    SRFT_HIP(hipGetLastError());
    return SRFT_OK;
}

int srft_stream_mix(const void* src_dev, void* dst_dev, int64_t n_tiles, int read_bytes_per_tile,
                    int write_bytes_per_tile, int workgroups, void* hip_stream) {
    if (n_tiles < 0 || read_bytes_per_tile < 0 || write_bytes_per_tile < 0 || read_bytes_per_tile % 16 ||
        write_bytes_per_tile % 16 || read_bytes_per_tile + write_bytes_per_tile == 0 || workgroups < 0)
        return SRFT_ERR_BAD_N;
    if (n_tiles == 0) return SRFT_OK;
    if (!src_dev || !dst_dev) return SRFT_ERR_NULL;
    if (!aligned(src_dev, 16) || !aligned(dst_dev, 16)) return SRFT_ERR_ALIGN;
    int dev = 0, cus = 0;
    SRFT_HIP(hipGetDevice(&dev));
    SRFT_HIP(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
    long long grid = workgroups > 0 ? workgroups : (long long)cus * 3;
    if (grid > n_tiles) grid = n_tiles;
    const int r_units = read_bytes_per_tile / 16, w_units = write_bytes_per_tile / 16;
    const int ru = r_units > 0 ? (r_units + 255) / 256 : 1;
    const char* env = std::getenv("SRFT_MIX_STREAM");          // 1: non-temporal accesses (read on every call)
    const bool stream = env && std::atoi(env) != 0;
    void (*kernel)(const uint4*, uint4*, long long, int, int) = nullptr;
#define SRFT_MIX_CASE(N)                                                                                          \
    case N:                                                                                                       \
        kernel = stream ? srft_mix_kernel<N, true> : srft_mix_kernel<N, false>;                                  \
        break;
    switch (ru) {
        SRFT_MIX_CASE(1) SRFT_MIX_CASE(2) SRFT_MIX_CASE(3) SRFT_MIX_CASE(4)
        SRFT_MIX_CASE(5) SRFT_MIX_CASE(6) SRFT_MIX_CASE(7) SRFT_MIX_CASE(8)
        default: return SRFT_ERR_BAD_N;         // at most 32 KiB read per tile
    }
#undef SRFT_MIX_CASE
    hipLaunchKernelGGL(kernel, dim3((unsigned)grid), dim3(256), 0, (hipStream_t)hip_stream, (const uint4*)src_dev,
                       (uint4*)dst_dev, (long long)n_tiles, r_units, w_units);
    SRFT_HIP(hipGetLastError());
    return SRFT_OK;
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

int srft_last_hip_error(void) { return g_last_hip_error; }

}  // extern "C"
