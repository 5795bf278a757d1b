// dequantize_tiles.h -- read path (plain and folded forms): kernel template and kernels.
#ifndef SRFT_DEQUANTIZE_TILES_H
#define SRFT_DEQUANTIZE_TILES_H
#include "device_util.h"

#ifndef SRFT_DQ_HALF_PIPE
#define SRFT_DQ_HALF_PIPE 1            // folded read path with one accumulator per slab: pinned half-group pipeline
#endif

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
// FOLD: half the matrix work, for d a multiple of 64 and g >= 32 (run at d = 128 and 192; d = 256 has a kernel of its
//     own, dequantize_fold4_tiles.h, that folds twice).  Every row of Q satisfies
//     Q[p][n + d/2] = (-1)^p Q[p][n]   (DC and Nyquist rows: +1; cos and sin rows of bin k: (-1)^k, and the
//     packed index p has the parity of k), so with  A_n = sum over even p,  B_n = sum over odd p  of
//     Q[p][n] z_p  the outputs are  x_n = s_n (A_n + B_n)  and  x_{n+d/2} = s_{n+d/2} (A_n - B_n),  n < d/2.
//     A byte holds an even p in its low and an odd p in its high nibble, so the two operands are the low and
//     the high nibbles.  Wavefront w owns n = 32w .. 32w+31: slab 0 is A, slab 1 is B (S = 2, KS = 1: per
//     group of 32 codes one k-step of 16 even and one of 16 odd codes), rows scaled by s_n on the host;
//     the relative sign s_n s_{n+d/2} is applied to the packed fp16 bits.  There is room for one accumulator per slab;
//     the loop is pipelined at half-group granularity (see lean_body).  rfrag is then
//     [D/64 waves][A, B][D/32 groups][hi, lo][64 lanes], followed by [D/64 waves][64 lanes][2] sign masks.
// BITS: 4, or 8 (one two's-complement byte per code).  A "code unit" is 16 codes: 8 bytes at 4 bits, 16 at 8.
//     At 8 bits a dword gives the pairs (b0, b2) and (b1, b3): again even and odd p apart, so FOLD applies as is.
template <int D, int S, int KS, bool FOLD, int BITS>
__device__ __forceinline__ void
srft_dequantize_tiles(const uint4* __restrict__ rfrag, const uint2* __restrict__ codes_raw,
                      const float* __restrict__ scales, long long n_vec, uint4* __restrict__ out,
                      float unscale, int gw, const int t0, const int stride, const int t_end) {
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

    auto lean_body = [&](int b) __attribute__((always_inline)) {
        if constexpr (FOLD && SRFT_DQ_HALF_PIPE) {
            // One accumulator per slab, software-pipelined at half-group granularity.  The MFMA pairs go A_0, B_0, A_1,
            // B_1, ...; each result is folded in (16 multiply-adds) one half-step after its pair, under the other
            // slab's pair.  A wavefront issues in order, and a second MFMA cannot issue while the first occupies the
            // matrix pipe (32 clocks): the order is therefore pinned as  MFMA, 8 multiply-adds, MFMA, 8 multiply-adds,
            // so that the vector ALU has work exactly while the pipe is taken.  Left alone, the compiler puts the two
            // MFMAs back to back and the wavefront idles behind the second.
            // B fragments are read two half-steps ahead, the group scale one step ahead.
            const uint4* rowp = &dec[b][col * ROW + 2 * half];      // units 4j + 2 half (+ 1): even / odd codes of group j
            float sc = scale_of(b, 0), sc_next = sc;
            half8 fa = __builtin_bit_cast(half8, rowp[0]), fb = __builtin_bit_cast(half8, rowp[1]);
            half8 fa_next = fa, fb_next = fb;
            acc0[0] = __builtin_amdgcn_mfma_f32_32x32x16_f16(rhi[0][0], fa, floatx16{0}, 0, 0, 0);
            acc0[0] = __builtin_amdgcn_mfma_f32_32x32x16_f16(rlo[0][0], fa, acc0[0], 0, 0, 0);
            auto pin_half_step = [&]() __attribute__((always_inline)) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);      // one MFMA
                __builtin_amdgcn_sched_group_barrier(0x002, 8, 0);      // eight vector-ALU instructions
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x002, 8, 0);
            };
#pragma unroll
            for (int j = 0; j < G; ++j) {
                // B_j on the matrix pipe, A_j folded in
                __builtin_amdgcn_sched_barrier(0);
                if (j + 1 < G) fa_next = __builtin_bit_cast(half8, rowp[4 * (j + 1)]);
                acc0[1] = __builtin_amdgcn_mfma_f32_32x32x16_f16(rhi[G + j][0], fb, floatx16{0}, 0, 0, 0);
#pragma unroll
                for (int v = 0; v < 8; ++v) o[0][v] = j == 0 ? acc0[0][v] * sc : fmaf(acc0[0][v], sc, o[0][v]);
                acc0[1] = __builtin_amdgcn_mfma_f32_32x32x16_f16(rlo[G + j][0], fb, acc0[1], 0, 0, 0);
#pragma unroll
                for (int v = 8; v < 16; ++v) o[0][v] = j == 0 ? acc0[0][v] * sc : fmaf(acc0[0][v], sc, o[0][v]);
                pin_half_step();
                // A_{j+1} on the matrix pipe, B_j folded in
                __builtin_amdgcn_sched_barrier(0);
                if (j + 1 < G) {
                    fb_next = __builtin_bit_cast(half8, rowp[4 * (j + 1) + 1]);
                    sc_next = scale_of(b, j + 1);
                    acc0[0] = __builtin_amdgcn_mfma_f32_32x32x16_f16(rhi[j + 1][0], fa_next, floatx16{0}, 0, 0, 0);
                }
#pragma unroll
                for (int v = 0; v < 8; ++v) o[1][v] = j == 0 ? acc0[1][v] * sc : fmaf(acc0[1][v], sc, o[1][v]);
                if (j + 1 < G) acc0[0] = __builtin_amdgcn_mfma_f32_32x32x16_f16(rlo[j + 1][0], fa_next, acc0[0], 0, 0, 0);
#pragma unroll
                for (int v = 8; v < 16; ++v) o[1][v] = j == 0 ? acc0[1][v] * sc : fmaf(acc0[1][v], sc, o[1][v]);
                if (j + 1 < G) pin_half_step();
                sc = sc_next;
                fb = fb_next;
            }
            __builtin_amdgcn_sched_barrier(0);
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

    const int m = (t_end - 1 - t0) / stride + 1;            // tiles of this workgroup: t0, t0 + stride, ... < t_end
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
__global__ void __launch_bounds__(2 * D / S, 1)
srft_dequantize_kernel(const uint4* __restrict__ rfrag, const uint2* __restrict__ codes,
                       const float* __restrict__ scales, long long n_vec, uint4* __restrict__ out,
                       float unscale, int gw) {
    int t0, stride, t_end;
    if (!srft_tile_range(n_vec, t0, stride, t_end)) return;
    srft_dequantize_tiles<D, S, KS, FOLD, BITS>(rfrag, codes, scales, n_vec, out, unscale, gw, t0, stride, t_end);
}

template <int D, int S, int KS, bool FOLD, int BITS>
__global__ void __launch_bounds__(2 * D / S, 1)
srft_dequantize_batched_kernel(const srft_batch_args a, int gw) {
    const int i = srft_segment_of_block(a, blockIdx.x);
    srft_dequantize_tiles<D, S, KS, FOLD, BITS>(a.frag[i], (const uint2*)a.in0[i], (const float*)a.in1[i], a.n_vec[i],
                                    (uint4*)a.out0[i], a.unscale[i], gw, blockIdx.x - a.first_block[i],
                                    a.first_block[i + 1] - a.first_block[i],
                                    (int)((a.n_vec[i] + kTileVecs - 1) / kTileVecs));
}

#endif  // SRFT_DEQUANTIZE_TILES_H
