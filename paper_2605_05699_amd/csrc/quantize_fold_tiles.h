// quantize_fold_tiles.h -- write path, folded form (half the matrix work): kernel template and kernels.
#ifndef SRFT_QUANTIZE_FOLD_TILES_H
#define SRFT_QUANTIZE_FOLD_TILES_H
#include "device_util.h"

// tuning constants (compile time)
#ifndef SRFT_QF_LEAN_MIN_D
#define SRFT_QF_LEAN_MIN_D 256
#endif
#ifndef SRFT_QF_RHO_LDS_MIN_D
#define SRFT_QF_RHO_LDS_MIN_D 256
#endif
#ifndef SRFT_QF_STAGE_OUT
#define SRFT_QF_STAGE_OUT 1          // the record goes through LDS and is stored as whole rows one stage later
#endif
#ifndef SRFT_QF_NT_STORE
#define SRFT_QF_NT_STORE 1           // non-temporal stores of the staged rows (+2.5 % at d = 128; nothing at d = 256)
#endif
#ifndef SRFT_QF_WG_PER_CU_256
#define SRFT_QF_WG_PER_CU_256 2
#endif

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
// AMAX: no record; every lane keeps the running maximum of |w| of its 32 packed indices (direct run, mirror run and
//       the bottom element of its mirror block: together the lanes of a vector cover every index once) over all the
//       tiles it sees; at the end the 32 vectors' lanes are reduced and one atomic maximum per channel goes to `amax`,
//       read as unsigned[d] (srft_kv_channel_absmax: the statistic lambda is calibrated from, Sec. 7.1).
template <int D, int BITS, bool WIDE, bool AMAX = false>
__device__ __forceinline__ void
srft_quantize_fold_tiles(const uint4* __restrict__ wfold, const uint4* __restrict__ x, long long n_vec,
                         uint2* __restrict__ codes, float* __restrict__ scales, float unscale, float scale_mul,
                         int gw, const int t0, const int stride, const int t_end, unsigned int* __restrict__ amax = nullptr) {
    constexpr int M = D / 64;            // wavefronts per workgroup
    constexpr int G = D / 32;            // groups per vector
    constexpr int T = D / 32;            // k-steps per slab (K = D / 2)
    constexpr int U = D / 8;             // 16-byte units per input row
    constexpr int ROW = U + 1;
    constexpr int NT = 64 * M;
    constexpr int DUMMY = 2 * M + 1;     // exchange slot for values nobody reads
    constexpr bool LEAN = (D >= SRFT_QF_LEAN_MIN_D);    // registers for one accumulator set only
    static_assert(M % 2 == 0, "the cosine and the sine block each need whole wavefronts");
    __shared__ uint4 lds[2][kTileVecs * ROW];
    __shared__ float xch[2][(DUMMY + 1) * kTileVecs];
    __shared__ float gmax[WIDE ? 2 : 1][WIDE ? kTileVecs * G : 1];     // maxima of the 32-runs of a tile (WIDE)
    // The record of a finished tile is staged here and stored one stage later, 16 bytes per thread over whole rows:
    // stored directly, a tile's record is 8-byte pieces and single floats, a write request each.
    constexpr bool STAGE = SRFT_QF_STAGE_OUT != 0 && !AMAX;
    static_assert(!AMAX || (BITS == 4 && !WIDE), "the statistic has one instance per d");
    constexpr int CU8 = (BITS == 8 ? D : D / 2) / 8;     // 8-byte units per code row
    constexpr int CROW = CU8 + 1;                        // padded: the lanes of a wavefront hit different banks
    __shared__ uint2 cstage[STAGE ? 2 : 1][STAGE ? kTileVecs * CROW : 1];
    __shared__ float sstage[STAGE ? 2 : 1][STAGE ? kTileVecs * G : 1];

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
    constexpr bool RHO_LDS = (D >= SRFT_QF_RHO_LDS_MIN_D);
    __shared__ uint4 rho_s[RHO_LDS ? 4 * NT : 1];
    float rho[16];
    float amd[AMAX ? 16 : 1] = {}, amm[AMAX ? 16 : 1] = {};     // running maxima of the direct and the mirror run (AMAX)
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
        if constexpr (AMAX) {                    // rows past the end alias to the last row: a maximum does not mind
            amm[0] = fmaxf(amm[0], fabsf(bottom));
            amd[0] = fmaxf(amd[0], fabsf(dv[0]));
#pragma unroll
            for (int v = 1; v < 16; ++v) {
                amd[v] = fmaxf(amd[v], fabsf(dv[v]));
                amm[v] = fmaxf(amm[v], fabsf(mv[v]));
            }
            return;
        }
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
        if constexpr (STAGE) {
            const int ns = WIDE ? G / gw : G;
            uint2* crow = &cstage[b][col * CROW];
            if constexpr (BITS == 8) {           // 16 values = 16 bytes = two 8-byte units
                crow[base_d / 8 + 2 * half] = make_uint2(pack4v(dv[0], dv[1], dv[2], dv[3], id), pack4v(dv[4], dv[5], dv[6], dv[7], id));
                crow[base_d / 8 + 2 * half + 1] = make_uint2(pack4v(dv[8], dv[9], dv[10], dv[11], id), pack4v(dv[12], dv[13], dv[14], dv[15], id));
                crow[p_top / 8 - 2 - 2 * half] = make_uint2(pack4v(bottom, mv[15], mv[14], mv[13], im), pack4v(mv[12], mv[11], mv[10], mv[9], im));
                crow[p_top / 8 - 1 - 2 * half] = make_uint2(pack4v(mv[8], mv[7], mv[6], mv[5], im), pack4v(mv[4], mv[3], mv[2], mv[1], im));
            } else {
                uint2 pd, pm;
                pd.x = pack8v(dv[0], dv[1], dv[2], dv[3], dv[4], dv[5], dv[6], dv[7], id);
                pd.y = pack8v(dv[8], dv[9], dv[10], dv[11], dv[12], dv[13], dv[14], dv[15], id);
                pm.x = pack8v(bottom, mv[15], mv[14], mv[13], mv[12], mv[11], mv[10], mv[9], im);
                pm.y = pack8v(mv[8], mv[7], mv[6], mv[5], mv[4], mv[3], mv[2], mv[1], im);
                crow[base_d / 16 + half] = pd;
                crow[p_top / 16 - 1 - half] = pm;
            }
            // both halves hold both scales: the lower lanes stage the direct group's, the upper lanes the mirror group's
            const int jd = WIDE ? base_d / 32 / gw : base_d / 32, jm = WIDE ? slot_in / gw : slot_in;
            sstage[b][col * ns + (half ? jm : jd)] = half ? sm : sd;
            return;
        }
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

    // staged record of `tile` -> global memory (rows past the end alias to the last row)
    auto flush = [&](int b, int tile) __attribute__((always_inline)) {
        if constexpr (STAGE) {
            const long long row0 = (long long)tile * kTileVecs;
            const int lim = (tile == n_tiles - 1) ? last_lim : kTileVecs - 1;
            constexpr int PIECES = CU8 / 2;              // 16-byte pieces per code row
            uint4* cbase = reinterpret_cast<uint4*>(codes) + row0 * PIECES;
#pragma unroll
            for (int i = 0; i < kTileVecs * PIECES / NT; ++i) {
                const int u = tid + i * NT, r = u / PIECES, pc = u % PIECES;
                const uint2 lo = cstage[b][r * CROW + 2 * pc], hi = cstage[b][r * CROW + 2 * pc + 1];
                
#if SRFT_QF_NT_STORE
            stream_store(&cbase[(unsigned)(min(r, lim) * PIECES + pc)], make_uint4(lo.x, lo.y, hi.x, hi.y));
#else
            cbase[(unsigned)(min(r, lim) * PIECES + pc)] = make_uint4(lo.x, lo.y, hi.x, hi.y);
#endif

            }
            const int ns = WIDE ? G / gw : G;            // 32 ns floats, next to each other in memory
            if (tid < kTileVecs * ns)
                (scales + row0 * ns)[(unsigned)(min(tid / ns, lim) * ns + tid % ns)] = sstage[b][tid];
        }
    };

    // AMAX: lanes of one half hold the same 32 indices for 32 different vectors: butterfly over the 32, then one atomic
    // per channel (non-negative floats order like their bit patterns)
    auto emit_amax = [&]() __attribute__((always_inline)) {
        if constexpr (AMAX) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                float md = amd[v], mm = amm[v];
#pragma unroll
                for (int step = 1; step < 32; step *= 2) {
                    md = fmaxf(md, __shfl_xor(md, step, 64));
                    mm = fmaxf(mm, __shfl_xor(mm, step, 64));
                }
                if (col == 0) {
                    atomic_max_nonneg(&amax[base_d + 16 * half + v], md * unscale);
                    atomic_max_nonneg(&amax[p_top - 16 * half - (v == 0 ? 16 : v)], mm * unscale);
                }
            }
        }
    };
    const int m = (t_end - 1 - t0) / stride + 1;            // tiles of this workgroup: t0, t0 + stride, ... < t_end
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
            if (k >= 2) flush(1, tk - 2 * stride);
            finish(0, ea, oa, tk - stride);
            __builtin_amdgcn_sched_barrier(0);   // no second accumulator set: the tail ends before the MFMAs begin
            contract(1, ea, oa);
            to_lds(0, pa0, pa1, pa2, pa3);
            fetch(pa0, pa1, pa2, pa3, tk + 3 * stride);
            publish(1, ea, oa);
            __syncthreads();                     // stage k + 1 (even)
            flush(0, tk - stride);
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
            if (k >= 2) flush(1, tk - 2 * stride);
            finish(0, ea, oa, tk - stride);
            __builtin_amdgcn_sched_barrier(0);
            contract(1, ea, oa);
            publish(1, ea, oa);
            __syncthreads();
            flush(0, tk - stride);
            finish(1, ea, oa, tk);
            if constexpr (STAGE) __syncthreads();
            flush(1, tk);
        } else {
            const int tl = t0 + (k - 1) * stride;
            __syncthreads();
            if (k >= 2) flush(1, tl - stride);
            finish(0, ea, oa, tl);
            if constexpr (STAGE) __syncthreads();
            flush(0, tl);
        }
        emit_amax();
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
        if (k >= 2) flush(1, tk - 2 * stride);
        contract(1, eb, ob);
        finish(0, ea, oa, tk - stride);
        to_lds(0, pa0, pa1, pa2, pa3);
        fetch(pa0, pa1, pa2, pa3, tk + 3 * stride);
        publish(1, eb, ob);
        __syncthreads();                         // stage k + 1 (even)
        rotate_priority(k + 1);
        flush(0, tk - stride);
        contract(0, ea, oa);
        finish(1, eb, ob, tk);
        to_lds(1, pb0, pb1, pb2, pb3);
        fetch(pb0, pb1, pb2, pb3, tk + 4 * stride);
        publish(0, ea, oa);
    }
    if (k < m) {                                 // one more odd stage
        const int tk = t0 + k * stride;
        __syncthreads();
        if (k >= 2) flush(1, tk - 2 * stride);
        contract(1, eb, ob);
        finish(0, ea, oa, tk - stride);
        publish(1, eb, ob);
        __syncthreads();
        flush(0, tk - stride);
        finish(1, eb, ob, tk);
        if constexpr (STAGE) __syncthreads();
        flush(1, tk);
    } else {
        const int tl = t0 + (k - 1) * stride;
        __syncthreads();
        if (k >= 2) flush(1, tl - stride);
        finish(0, ea, oa, tl);
        if constexpr (STAGE) __syncthreads();
        flush(0, tl);
    }
    emit_amax();
}

// two wavefronts per SIMD (8 per compute unit): the register allocator is told to stay within 256 VGPRs
template <int D, int BITS, bool WIDE>
__global__ void __launch_bounds__(D, (D >= 256 ? SRFT_QF_WG_PER_CU_256 : 2))
srft_quantize_fold_kernel(const uint4* __restrict__ wfold, const uint4* __restrict__ x, long long n_vec,
                          uint2* __restrict__ codes, float* __restrict__ scales, float4* __restrict__,
                          float unscale, float scale_mul, int gw) {
    int t0, stride, t_end;
    if (!srft_tile_range(n_vec, t0, stride, t_end)) return;
    srft_quantize_fold_tiles<D, BITS, WIDE>(wfold, x, n_vec, codes, scales, unscale, scale_mul, gw, t0, stride, t_end);
}

// the abs-max statistic through the folded contraction: amax is float[d] read as unsigned, updated with atomic maxima
// (at d = 256 the 32 running maxima do not fit beside the matrix in 256 registers, and with them in scratch the kernel
// takes twice as long: one workgroup per compute unit)
template <int D>
__global__ void __launch_bounds__(D, (D >= 256 ? 1 : 2))
srft_quantize_fold_amax_kernel(const uint4* __restrict__ wfold, const uint4* __restrict__ x, long long n_vec,
                               uint2* __restrict__, float* __restrict__, float4* __restrict__ amax, float unscale,
                               float scale_mul, int gw) {
    int t0, stride, t_end;
    if (!srft_tile_range(n_vec, t0, stride, t_end)) return;
    srft_quantize_fold_tiles<D, 4, false, true>(wfold, x, n_vec, nullptr, nullptr, unscale, scale_mul, gw, t0, stride, t_end,
                                                reinterpret_cast<unsigned int*>(amax));
}

template <int D, int BITS, bool WIDE>
__global__ void __launch_bounds__(D, (D >= 256 ? SRFT_QF_WG_PER_CU_256 : 2))
srft_quantize_fold_batched_kernel(const srft_batch_args a, int gw) {
    const int i = srft_segment_of_block(a, blockIdx.x);
    srft_quantize_fold_tiles<D, BITS, WIDE>(a.frag[i], (const uint4*)a.in0[i], a.n_vec[i], (uint2*)a.out0[i],
                                            (float*)a.out1[i], a.unscale[i], a.unscale[i] / (BITS == 8 ? 127.0f : 7.0f),
                                            gw, blockIdx.x - a.first_block[i], a.first_block[i + 1] - a.first_block[i],
                                            (int)((a.n_vec[i] + kTileVecs - 1) / kTileVecs));
}

#endif  // SRFT_QUANTIZE_FOLD_TILES_H
