// dequantize_fold4_tiles.h -- read path at d = 128 and 256, folded twice: a quarter of the dense matrix work, half the
// scale fold of the once-folded form.
//
// With h = d/2 the inverse of Eq. 1-2 is  u_n = C_n + S_n,  C_n the sum over the packed indices p <= h (DC, the cosine
// rows, Nyquist) and S_n the sum over p > h (the sine rows) of Q[p][n] z_p.  C is even and S is odd under n -> d - n,
// and the two kinds of rows are whole groups of the record (p < h: the first d/64 groups, p >= h: the others), so each
// half is contracted from half of the groups only.  Under n -> h - n a row of bin k keeps its sign when k is even and
// flips it when k is odd (cosine), or the other way round (sine); p has the parity of k, and a code byte holds an even
// p in its low and an odd p in its high nibble.  With Ce, Co (Se, So) the partial sums over even and odd p:
//     C_m = Ce_m + Co_m,  C_{h-m} = Ce_m - Co_m,  S_m = So_m + Se_m,  S_{h-m} = So_m - Se_m,     m = 0 .. d/4,
//     u_m = C_m + S_m,  u_{d-m} = C_m - S_m,  u_{h-m} = C_{h-m} + S_{h-m},  u_{h+m} = C_{h-m} - S_{h-m}.
// Only m < d/4 is contracted, per class from K = 16 codes per group: d/4 MFMAs per tile of 32 vectors (d/2 once
// folded, d dense: 64 / 128 / 256 at d = 256), and every output sums d/64 group partial results instead of d/32.
//
// With NB = d/128 blocks of 32 values of m, wavefront w < NB holds the cosine classes (E = Ce, O = Co) of m = 32w ..
// 32w + 31, wavefront NB + w the sine classes (E = Se, O = -So, negated on the host) of the same m: every wavefront
// forms  own = E + O  and  send = E - O,  which is (C_m, C_{h-m}) on the cosine and (-S_{h-m}, S_m) on the sine side.
// `send` crosses to the partner wavefront through LDS (fp32), and every wavefront finishes two runs of 16 outputs
// per lane:
//     ascending   own + recv  ->  n = m          (cosine)   n = h + m   (sine)
//     descending  own - recv  ->  n = d - m      (cosine)   n = h - m   (sine, negated: undone by the sign masks)
// The sign diagonal is applied to the packed fp16 bits (one mask per output).  A descending run covers
// n0 - 15 .. n0 with n0 a multiple of 16: its top element belongs to the 16-byte block above, so every lane takes the
// bottom element of its block from the lane that owns the next 16 values of m: the other half of the wavefront
// (v_permlane32_swap), the next wavefront (through LDS; d = 256 only), or, above the last block, the row m = d/4 that
// no slab holds (Co and Se vanish there):
//     Ce at m = d/4  as a dot product on the vector ALU, one group of 16 even codes per wavefront,
//     So at m = d/4  in row m = 0 of the first sine wavefront's O slab, which is otherwise zero.
// The Nyquist code (packed index h, first code of the first sine group) is even under both reflections: it enters the
// cosine wavefronts as the addend (-1)^m code scale c of the first multiply-add of the E class.
//
// Stage k of a workgroup: barrier; flush T_{k-1} from the staging tile; contract T_k, write `send`; decode T_{k+1};
// barrier; read `recv`, finish, stage T_k.  The second barrier lets the staging tile and the exchange be single
// buffers.  (Decoding T_{k+1} after the second barrier instead would let the decoded tile be a single buffer too, and
// at d = 128 a fifth workgroup fit a compute unit: measured 2 - 3.5 % slower at both sizes.)
//
// Table (16-byte units), NW = d/64 wavefronts: [NW][E, O][d/64 groups][hi, lo][64 lanes] A-operand fragments;
// [NW][2 lane halves][6]: sign masks (8 dwords ascending run, 8 dwords descending run) and the 8 fp32 coefficients of
// row m = d/4 for the even codes of group w a lane of that half reads (the 32 lanes of a half share them: the kernel
// keeps them in LDS and reads them as broadcasts); [NW] per-wavefront constants (.x = Nyquist factor).
#ifndef SRFT_DEQUANTIZE_FOLD4_TILES_H
#define SRFT_DEQUANTIZE_FOLD4_TILES_H
#include "device_util.h"

// sizes of the table's parts (16-byte units) at head dimension d: NW = d/64 wavefronts, d/64 groups per half
constexpr int srft_rfold4_frag_units(int d) { return (d / 64) * 2 * (d / 64) * 2 * 64; }
constexpr int srft_rfold4_half_units(int d) { return (d / 64) * 2 * 6; }
constexpr int srft_rfold4_units(int d) { return srft_rfold4_frag_units(d) + srft_rfold4_half_units(d) + d / 64; }

template <int D, int BITS>
__device__ __forceinline__ void
srft_dequantize_fold4_tiles(const uint4* __restrict__ tab, const uint2* __restrict__ codes_raw,
                            const float* __restrict__ scales, long long n_vec, uint4* __restrict__ out,
                            float unscale, int gw, const int t0, const int stride, const int t_end) {
    static_assert(D == 128 || D == 256, "one or two blocks of 32 values of m per class");
    constexpr int NB = D / 128, NW = 2 * NB, GH = D / 64;      // m blocks per class, wavefronts, groups per half of the record
    constexpr int LG = D == 256 ? 3 : 2;                        // log2 of the groups per vector at g = 32
    constexpr int U = D / 8, ROW = U + 1, C = D / 16, NT = 64 * NW, SROW = D / 32 + 1;
    constexpr int kFragUnits = srft_rfold4_frag_units(D), kHalfUnits = srft_rfold4_half_units(D);
    using CodeUnit = std::conditional_t<BITS == 8, uint4, uint2>;
    const CodeUnit* __restrict__ codes = reinterpret_cast<const CodeUnit*>(codes_raw);
    const int sh = __builtin_ctz((unsigned)gw);  // g = 32 gw, gw a power of two: group j uses scale j >> sh
    const int ns = (D / 32) >> sh;               // scales per vector
    __shared__ uint4 dec[2][kTileVecs * ROW];    // decoded codes of T_k in dec[k % 2]: per code unit [even p][odd p]
    __shared__ uint4 stg[kTileVecs * ROW];       // finished fp16 rows of the tile staged last
    __shared__ uint4 xch[2 * NB * 4 * 64];       // [sent by: cosine, sine][m block][quarter][lane]: `send`, fp32
    __shared__ float scl[2][kTileVecs * SROW];   // scales (times 2^-e) of T_k in scl[k % 2]
    __shared__ float s_own32[2][32];             // own[m = 32] of the second cosine / sine wavefront (d = 256)
    __shared__ float s_neg64[32];                // -So at m = d/4, the row above the last block
    __shared__ float s_c64[NW][32];              // Ce at m = d/4: one partial sum per wavefront (group)
    // Stores that only some lanes make go to this array from the other lanes, a word per thread: the code between the
    // barriers stays one straight-line block (a branch after the pinned MFMA / multiply-add pipeline lets the
    // compiler sink the multiply-adds out of it).
    __shared__ float s_dump[NT];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);          // uniform: kept in a scalar register
    const int col = lane & 31, half = lane >> 5;
    const int sine = wave / NB, blk = wave % NB;
    const int n_tiles = (int)((n_vec + kTileVecs - 1) / kTileVecs);
    const int last_lim = (int)(n_vec - 1 - (long long)(n_tiles - 1) * kTileVecs);

    half8 rhi[2][GH], rlo[2][GH];                // [class][group]
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
        for (int j = 0; j < GH; ++j) {
            const int f = ((wave * 2 + c) * GH + j) * 2;
            rhi[c][j] = __builtin_bit_cast(half8, tab[(f + 0) * 64 + lane]);
            rlo[c][j] = __builtin_bit_cast(half8, tab[(f + 1) * 64 + lane]);
        }
    __shared__ uint4 s_half[kHalfUnits];   // per (wavefront, lane half): 4 units of sign masks, 2 of coefficients
    if (tid < kHalfUnits) s_half[tid] = tab[kFragUnits + tid];     // visible after the first barrier
    const float c_nyq = __uint_as_float(tab[kFragUnits + kHalfUnits + wave].x);   // uniform; 0 on the sine side
    const uint4* mine = &s_half[(wave * 2 + half) * 6];

    // ---- loads and decode: as in the once-folded kernel (two code units and one scale per thread) ----
    auto fetch1 = [&](CodeUnit& v, int i, const CodeUnit* tile_base, int lim) __attribute__((always_inline)) {
        const int u = tid + i * NT, r = u / C, c = u % C;
        v = stream_load(&tile_base[(unsigned)(min(r, lim) * C + c)]);
    };
    auto fetch = [&](CodeUnit& c0, CodeUnit& c1, float& s0, int tile) __attribute__((always_inline)) {
        if (tile > n_tiles - 1) tile = n_tiles - 1;
        const long long row0 = (long long)tile * kTileVecs;
        const int lim = (tile == n_tiles - 1) ? last_lim : kTileVecs - 1;
        fetch1(c0, 0, codes + row0 * C, lim);
        fetch1(c1, 1, codes + row0 * C, lim);
        int e = tid;
        if (e > 32 * ns - 1) e = 32 * ns - 1;
        s0 = (scales + row0 * ns)[(unsigned)(min(e >> (LG - sh), lim) * ns + (e & (ns - 1)))];
    };
    auto put1 = [&](int b, const CodeUnit& v, int i) __attribute__((always_inline)) {
        const int u = tid + i * NT, r = u / C, c = u % C;
        if constexpr (BITS == 8) {               // .x: bytes 0 and 2 (even p), .y: bytes 1 and 3 (odd p) of a dword
            const uint2 a = decode4_bytes(v.x), b2 = decode4_bytes(v.y), c2 = decode4_bytes(v.z), d2 = decode4_bytes(v.w);
            dec[b][r * ROW + 2 * c] = make_uint4(a.x, b2.x, c2.x, d2.x);
            dec[b][r * ROW + 2 * c + 1] = make_uint4(a.y, b2.y, c2.y, d2.y);
        } else {                                 // .x .z hold the even, .y .w the odd nibbles of a dword
            const uint4 lo = decode8(v.x), hi = decode8(v.y);
            dec[b][r * ROW + 2 * c] = make_uint4(lo.x, lo.z, hi.x, hi.z);
            dec[b][r * ROW + 2 * c + 1] = make_uint4(lo.y, lo.w, hi.y, hi.w);
        }
    };
    auto to_lds = [&](int b, const CodeUnit& c0, const CodeUnit& c1, float s0) __attribute__((always_inline)) {
        put1(b, c0, 0);
        put1(b, c1, 1);
        float* dst = tid < 32 * ns ? &scl[b][(tid >> (LG - sh)) * SROW + (tid & (ns - 1))] : &s_dump[tid];
        *dst = s0 * unscale;
    };

    floatx16 oE, oO, accE, accO, own;
    const int jb = GH * sine;                    // first group of this wavefront's half of the record
    // ---- contraction of the tile in dec[b], and what leaves this wavefront through LDS ----
    auto contract = [&](int b) __attribute__((always_inline)) {
        const uint4* rowp = &dec[b][col * ROW + 2 * half + 4 * jb];     // + 4 jj (+ 1): even / odd codes of group jb + jj
        const float* srow = &scl[b][col * SROW];
        const float code_n = (float)reinterpret_cast<const _Float16*>(&dec[b][col * ROW + D / 16])[0];
        const float t_n = code_n * srow[GH >> sh] * c_nyq;
        float sc = srow[jb >> sh], sc_next = sc;
        half8 fa_next = __builtin_bit_cast(half8, rowp[0]), fb = __builtin_bit_cast(half8, rowp[1]), fb_next = fb;
        accE = __builtin_amdgcn_mfma_f32_32x32x16_f16(rhi[0][0], fa_next, floatx16{0}, 0, 0, 0);
        accE = __builtin_amdgcn_mfma_f32_32x32x16_f16(rlo[0][0], fa_next, accE, 0, 0, 0);
        // One accumulator per class, pipelined at half-group granularity with the order pinned: MFMA, eight
        // multiply-adds, MFMA, eight multiply-adds (a wavefront issues in order; the vector ALU has work exactly
        // while the matrix pipe is taken).
        auto pin_half_step = [&]() __attribute__((always_inline)) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x002, 8, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x002, 8, 0);
        };
#pragma unroll
        for (int jj = 0; jj < GH; ++jj) {
            // O_jj on the matrix pipe, E_jj folded in
            __builtin_amdgcn_sched_barrier(0);
            if (jj + 1 < GH) fa_next = __builtin_bit_cast(half8, rowp[4 * (jj + 1)]);
            accO = __builtin_amdgcn_mfma_f32_32x32x16_f16(rhi[1][jj], fb, floatx16{0}, 0, 0, 0);
#pragma unroll
            for (int v = 0; v < 8; ++v) oE[v] = fmaf(accE[v], sc, jj == 0 ? ((v & 1) ? -t_n : t_n) : oE[v]);
            accO = __builtin_amdgcn_mfma_f32_32x32x16_f16(rlo[1][jj], fb, accO, 0, 0, 0);
#pragma unroll
            for (int v = 8; v < 16; ++v) oE[v] = fmaf(accE[v], sc, jj == 0 ? ((v & 1) ? -t_n : t_n) : oE[v]);
            pin_half_step();
            // E_{jj+1} on the matrix pipe, O_jj folded in
            __builtin_amdgcn_sched_barrier(0);
            if (jj + 1 < GH) {
                fb_next = __builtin_bit_cast(half8, rowp[4 * (jj + 1) + 1]);
                sc_next = srow[(jb + jj + 1) >> sh];
                accE = __builtin_amdgcn_mfma_f32_32x32x16_f16(rhi[0][jj + 1], fa_next, floatx16{0}, 0, 0, 0);
            }
#pragma unroll
            for (int v = 0; v < 8; ++v) oO[v] = jj == 0 ? accO[v] * sc : fmaf(accO[v], sc, oO[v]);
            if (jj + 1 < GH) accE = __builtin_amdgcn_mfma_f32_32x32x16_f16(rlo[0][jj + 1], fa_next, accE, 0, 0, 0);
#pragma unroll
            for (int v = 8; v < 16; ++v) oO[v] = jj == 0 ? accO[v] * sc : fmaf(accO[v], sc, oO[v]);
            if (jj + 1 < GH) pin_half_step();
            sc = sc_next;
            fb = fb_next;
        }
        __builtin_amdgcn_sched_barrier(0);
        // Ce at m = d/4: this wavefront's share is cosine group `wave`; a lane holds 8 of its 16 even codes
        {
            const half8 fx = __builtin_bit_cast(half8, dec[b][col * ROW + 2 * half + 4 * wave]);
            const uint4 cf0 = mine[4], cf1 = mine[5];
            const float cf[8] = {__uint_as_float(cf0.x), __uint_as_float(cf0.y), __uint_as_float(cf0.z), __uint_as_float(cf0.w),
                                 __uint_as_float(cf1.x), __uint_as_float(cf1.y), __uint_as_float(cf1.z), __uint_as_float(cf1.w)};
            float dot0 = 0.0f, dot1 = 0.0f;
#pragma unroll
            for (int e = 0; e < 8; e += 2) {
                dot0 = fmaf((float)fx[e], cf[e], dot0);
                dot1 = fmaf((float)fx[e + 1], cf[e + 1], dot1);
            }
            float part = (dot0 + dot1) * srow[wave >> sh];
            part += (wave == 0 && half == 0) ? t_n : 0.0f;
            const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(part), __float_as_uint(part), false, false);
            *(half == 0 ? &s_c64[wave][col] : &s_dump[tid]) = __uint_as_float(r[0]) + __uint_as_float(r[1]);
        }
        // row m = 0 of the first sine wavefront's O slab carried -So at m = d/4
        const bool hijack = (wave == NB) && (half == 0);
        *(hijack ? &s_neg64[col] : &s_dump[tid]) = oO[0];
        oO[0] = hijack ? 0.0f : oO[0];
        floatx16 snd;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            own[v] = oE[v] + oO[v];
            snd[v] = oE[v] - oO[v];
        }
        if constexpr (NB == 2) *((blk == 1 && half == 0) ? &s_own32[sine][col] : &s_dump[tid]) = own[0];
        uint4* xw = &xch[((sine * NB + blk) * 4) * 64 + lane];
#pragma unroll
        for (int q = 0; q < 4; ++q)
            xw[q * 64] = make_uint4(__float_as_uint(snd[4 * q]), __float_as_uint(snd[4 * q + 1]),
                                    __float_as_uint(snd[4 * q + 2]), __float_as_uint(snd[4 * q + 3]));
    };
    // ---- after the exchange: the two runs of this lane, rounded to fp16, signed, into the staging tile ----
    const int uA = (U / 2) * sine + 4 * blk + 2 * half;                    // 16-byte unit of the ascending run
    const int uD = (sine ? U / 2 : U) - 2 - 4 * blk - 2 * half;              // ... of the descending run's block
    auto finish = [&]() __attribute__((always_inline)) {
        const uint4* xr = &xch[(((1 - sine) * NB + blk) * 4) * 64 + lane];
        float rc[16];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const uint4 t = xr[q * 64];
            rc[4 * q] = __uint_as_float(t.x);
            rc[4 * q + 1] = __uint_as_float(t.y);
            rc[4 * q + 2] = __uint_as_float(t.z);
            rc[4 * q + 3] = __uint_as_float(t.w);
        }
        // bottom element of the descending block: (own - recv) at m0 + 16
        float c64 = s_c64[0][col] + s_c64[1][col];
        if constexpr (NW == 4) c64 += s_c64[2][col] + s_c64[3][col];
        float above = fmaf(c64, sine ? -1.0f : 1.0f, s_neg64[col]);      // the row above the last block
        if constexpr (NB == 2) {
            const float above32 = s_own32[sine][col] - __uint_as_float(xch[(((1 - sine) * NB + 1) * 4) * 64 + col].x);
            above = blk == 0 ? above32 : above;
        }
        float des[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) des[v] = own[v] - rc[v];
        const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(des[0]), __float_as_uint(des[0]), false, false);
        const float bottom = half ? above : __uint_as_float(sw[1]);
        uint32_t a[8], dd[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) a[i] = pack_half2(own[2 * i] + rc[2 * i], own[2 * i + 1] + rc[2 * i + 1]);
        dd[0] = pack_half2(bottom, des[15]);
#pragma unroll
        for (int i = 1; i < 8; ++i) dd[i] = pack_half2(des[16 - 2 * i], des[15 - 2 * i]);
        uint4* row = &stg[col * ROW];
        const uint4 mA0 = mine[0], mA1 = mine[1], mD0 = mine[2], mD1 = mine[3];
        row[uA] = make_uint4(a[0] ^ mA0.x, a[1] ^ mA0.y, a[2] ^ mA0.z, a[3] ^ mA0.w);
        row[uA + 1] = make_uint4(a[4] ^ mA1.x, a[5] ^ mA1.y, a[6] ^ mA1.z, a[7] ^ mA1.w);
        row[uD] = make_uint4(dd[0] ^ mD0.x, dd[1] ^ mD0.y, dd[2] ^ mD0.z, dd[3] ^ mD0.w);
        row[uD + 1] = make_uint4(dd[4] ^ mD1.x, dd[5] ^ mD1.y, dd[6] ^ mD1.z, dd[7] ^ mD1.w);
    };
    // staging tile -> global rows of `tile`: fully coalesced 16-byte stores, four per thread
    auto flush = [&](int tile) __attribute__((always_inline)) {
        const long long row0 = (long long)tile * kTileVecs;
        const int lim = (tile == n_tiles - 1) ? last_lim : kTileVecs - 1;
        uint4* tile_base = out + row0 * U;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int u = tid + i * NT, r = u / U, c = u % U;
            stream_store(&tile_base[(unsigned)(min(r, lim) * U + c)], stg[r * ROW + c]);   // rows past the end alias to the last row
        }
    };

    const int m = (t_end - 1 - t0) / stride + 1;            // tiles of this workgroup: t0, t0 + stride, ... < t_end
    CodeUnit pa0, pa1, pb0, pb1;
    float pas, pbs;
    fetch(pa0, pa1, pas, t0);
    fetch(pb0, pb1, pbs, t0 + stride);
    hold_in_registers(rhi, rlo);
    to_lds(0, pa0, pa1, pas);
    fetch(pa0, pa1, pas, t0 + 2 * stride);
    // Two stages per trip, so that the two prefetch register sets keep their names.
    __syncthreads();                             // stage 0: nothing to flush yet
    contract(0);
    to_lds(1, pb0, pb1, pbs);
    fetch(pb0, pb1, pbs, t0 + 3 * stride);
    __syncthreads();
    finish();
    int k = 1;
    for (; k + 1 < m; k += 2) {
        const int tk = t0 + k * stride;
        __syncthreads();                         // stage k (odd)
        rotate_priority(k);
        flush(tk - stride);
        contract(1);
        to_lds(0, pa0, pa1, pas);
        fetch(pa0, pa1, pas, tk + 3 * stride);
        __syncthreads();
        finish();
        __syncthreads();                         // stage k + 1 (even)
        rotate_priority(k + 1);
        flush(tk);
        contract(0);
        to_lds(1, pb0, pb1, pbs);
        fetch(pb0, pb1, pbs, tk + 4 * stride);
        __syncthreads();
        finish();
    }
    if (k < m) {                                 // one more odd stage
        const int tk = t0 + k * stride;
        __syncthreads();
        flush(tk - stride);
        contract(1);
        __syncthreads();
        finish();
        __syncthreads();
        flush(tk);
    } else {
        __syncthreads();
        flush(t0 + (k - 1) * stride);
    }
}

template <int D, int BITS>
__global__ void __launch_bounds__(D / 64 * 64, 2)
srft_dequantize_fold4_kernel(const uint4* __restrict__ tab, const uint2* __restrict__ codes,
                             const float* __restrict__ scales, long long n_vec, uint4* __restrict__ out,
                             float unscale, int gw) {
    int t0, stride, t_end;
    if (!srft_tile_range(n_vec, t0, stride, t_end)) return;
    srft_dequantize_fold4_tiles<D, BITS>(tab, codes, scales, n_vec, out, unscale, gw, t0, stride, t_end);
}

template <int D, int BITS>
__global__ void __launch_bounds__(D / 64 * 64, 2)
srft_dequantize_fold4_batched_kernel(const srft_batch_args a, int gw) {
    const int i = srft_segment_of_block(a, blockIdx.x);
    srft_dequantize_fold4_tiles<D, BITS>(a.frag[i], (const uint2*)a.in0[i], (const float*)a.in1[i], a.n_vec[i],
                                      (uint4*)a.out0[i], a.unscale[i], gw, blockIdx.x - a.first_block[i],
                                      a.first_block[i + 1] - a.first_block[i],
                                      (int)((a.n_vec[i] + kTileVecs - 1) / kTileVecs));
}

#endif  // SRFT_DEQUANTIZE_FOLD4_TILES_H
