// Scores of queries against the stored keys, in the rotated domain: the scan kernel and its launch.
#include "../device_util.h"

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
                   long long n_keys, float* __restrict__ out, int n_q, int gw, float* __restrict__ dump,
                   unsigned int* __restrict__ row_max, float sign) {
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
    // running maximum of sign * score over this lane's valid (query, key) pairs, per result register: what a softmax
    // over the rows needs first (row_max: nullptr, or kRowMaxCopies x 32 order-preserving codes of such maxima, see
    // srft_ordered_code, one copy updated with atomic maxima when the workgroup is done)
    float vmax[NV];
#pragma unroll
    for (int v = 0; v < NV; ++v) vmax[v] = -INFINITY;

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
            vmax[v] = fmaxf(vmax[v], v < nv_lane ? sign * val[v] : -INFINITY);
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
    if (row_max) {                               // uniform
        // lanes with the same a hold the same queries (2 v + a) for different keys: R16 a = bit 4 of the lane (after the
        // swap of tile_scores), else a = bit 5; the maximum runs over the other five lane bits
        constexpr int kABit = R16 ? 16 : 32;
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            float mx = vmax[v];
#pragma unroll
            for (int step = 1; step < 64; step *= 2)
                if (step != kABit) mx = fmaxf(mx, __shfl_xor(mx, step, 64));
            const int a = (lane & kABit) ? 1 : 0, q = 2 * v + a;
            if ((lane & (63 ^ kABit)) == 0 && q < n_q) {
                const unsigned int code = srft_ordered_code(mx);
                // kRowMaxCopies copies, a cache line each: atomics to one line are served one after the other
                unsigned int* slot = &row_max[(blockIdx.x % kRowMaxCopies) * 32 + q];
                atomicMax(slot, code);
            }
        }
    }
}

namespace {
template <int D>
int launch(const srft_plan* p, uint4* qfrag, float* dump, int n_q, const uint8_t* codes, const float* scales,
           long long n_keys, float* out, unsigned int* row_max, float sign, hipStream_t st) {
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
                           (const uint2*)codes, scales, n_keys, out, n_q, p->gw, dump, row_max, sign);
        SRFT_HIP(hipGetLastError());
        return SRFT_OK;
    } else {
        return SRFT_ERR_BAD_D;
    }
}
template <int D>
int occupancy(bool r16, int* blocks) {
    if constexpr (D % 64 == 0) {
        if (r16) SRFT_HIP(hipOccupancyMaxActiveBlocksPerMultiprocessor(blocks, srft_scores_kernel<D, 8, true>, 64, 0));
        else SRFT_HIP(hipOccupancyMaxActiveBlocksPerMultiprocessor(blocks, srft_scores_kernel<D, 16, false>, 64, 0));
        return SRFT_OK;
    } else {
        *blocks = 0;
        return SRFT_OK;
    }
}
}  // namespace

int srft_launch_scores(const srft_plan* p, uint4* qfrag, float* dump, int n_q, const uint8_t* codes,
                       const float* scales, long long n_keys, float* out, unsigned int* row_max, float sign,
                       hipStream_t st) {
    switch (p->d) {
        case 64: return launch<64>(p, qfrag, dump, n_q, codes, scales, n_keys, out, row_max, sign, st);
        case 128: return launch<128>(p, qfrag, dump, n_q, codes, scales, n_keys, out, row_max, sign, st);
        case 192: return launch<192>(p, qfrag, dump, n_q, codes, scales, n_keys, out, row_max, sign, st);
        case 256: return launch<256>(p, qfrag, dump, n_q, codes, scales, n_keys, out, row_max, sign, st);
        default: return SRFT_ERR_BAD_D;
    }
}
int srft_scores_occupancy(int d, bool r16, int* blocks) {
    switch (d) {
        case 64: return occupancy<64>(r16, blocks);
        case 128: return occupancy<128>(r16, blocks);
        case 192: return occupancy<192>(r16, blocks);
        case 256: return occupancy<256>(r16, blocks);
        default: *blocks = 0; return SRFT_OK;
    }
}
