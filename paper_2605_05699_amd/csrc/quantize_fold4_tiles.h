// quantize_fold4_tiles.h -- write path at d = 256, folded twice: a quarter of the dense matrix work.
//
// Split the input positions by n mod 4 into four classes and write the bin as k = k1 + 64 k2 (Eq. 1 with the
// sum over n regrouped; the transform stays exactly the one of Eq. 1-2).  With
//     C_c[k1] = sum over n = c (mod 4) of Q[k1][n] u_n          (cosine rows, k1 < 32)
//     S_c[k1] = sum over n = c (mod 4) of Q[128 + k1][n] u_n    (sine rows)
// the twiddle factors are inside the rows already, and what is left between the classes is a 4-point DFT whose
// factors are +-1 and +-i.  In packed indices (Eq. 2), with P = C0 + C2, M = C0 - C2, P' = C1 + C3, M' = C1 - C3,
// U = S0 + S2, V = S0 - S2, U' = S1 + S3, V' = S1 - S3:
//     z[k1]       = P + P'        z[128 - k1] = P - P'         (groups 0 and 3)
//     z[64 + k1]  = M + V'        z[64 - k1]  = M - V'         (groups 2 and 1)
//     z[128 + k1] = U + U'        z[256 - k1] = -(U - U')      (groups 4 and 7)
//     z[192 + k1] = V - M'        z[192 - k1] = -(V + M')      (groups 6 and 5)
// Only 32 cosine and 32 sine rows are contracted, each over a quarter of the inputs (K = 64): 64 MFMAs per tile of
// 32 vectors against 128 of the once-folded form and 256 of the dense one.
//
// A workgroup has four wavefronts, (cosine | sine) x (classes {0,2} | classes {1,3}).  Each contracts its two
// classes into accumulators a and c (row signs are chosen on the host so that every wavefront does the same):
//     keep = a + c,  send = a - c;   send goes to the wavefront that needs it through LDS (16 floats per lane),
//     after the next barrier:  recv = the send of wavefront (w + 1) mod 4,
//     direct run  = rho_d (keep + tau recv),   mirror run = rho_m (keep - tau recv)
// with rho = +-lambda of the packed index (lambda is NOT folded into the matrix here: the rows of all four
// wavefronts meet in sums, so they share one scaling) and tau = -1 for the cosine-odd wavefront, +1 elsewhere:
//     wave 0 (cos, 0|2): keep P,  send M   -> groups 0 (direct) and 3 (mirror), recv P'
//     wave 1 (cos, 1|3): keep M', send P'  -> groups 6 and 5, recv V
//     wave 2 (sin, 0|2): keep U,  send V   -> groups 4 and 7, recv U'
//     wave 3 (sin, 1|3): keep V', send U'  -> groups 2 and 1, recv M
// A lane holds k1 = 16 h + v (v < 16): a direct run of 16 packed indices (ascending) and a mirror run (descending),
// exactly as in the once-folded form, whose quantizer tail is reused: the mirror run sits one index above a
// 16-aligned block, lanes h = 0 take the bottom element of their block from lane h = 1 of the same vector, lanes
// h = 1 take it from LDS -- here the four bins k = 32, 96 (packed 32, 96, 160, 224).  Those come from the row
// k1 = 32, which is (-1)^(n/4) times a constant per class: the alternating sums A_c ride in the otherwise empty
// sine rows k1 = 0 (A1, A3 pre-multiplied by 1/sqrt 2):  z32 = A0 + Am, z96 = A0 - Am, z160 = -(A2 + Ap),
// z224 = A2 - Ap with Am = A1 - A3, Ap = A1 + A3.  The lanes k1 = 0 also carry DC (direct element 0 of wave 0),
// Nyquist = P0 - P0' (direct element 0 of wave 2, which computes it from the two published halves), and
// z64 = sqrt 2 M0, z192 = -sqrt 2 M0' (the rows k1 = 0 have the DC scaling 1/sqrt d; sqrt 2 is folded into rho).
//
// wf4: [4 waves][a, c][4 k-steps][hi, lo][64 lanes] 16-byte fragments, then [4 waves][rho_d[32], rho_m[32]] floats,
//      then [4 waves] (beta1, beta2, nyquist scale, tau).  All scalings by 2^-e of the matrix are inside rho / beta.
#ifndef SRFT_QUANTIZE_FOLD4_TILES_H
#define SRFT_QUANTIZE_FOLD4_TILES_H
#include "device_util.h"

constexpr int kFold4FragUnits = 4 * 2 * 4 * 2 * 64;          // 16-byte units of fragments in wf4
constexpr int kFold4RhoFloats = 4 * 64;
constexpr int kFold4Units = kFold4FragUnits + kFold4RhoFloats / 4 + 4;

template <int BITS>
__device__ __forceinline__ void
srft_quantize_fold4_tiles(const uint4* __restrict__ wf4, const uint4* __restrict__ x, long long n_vec,
                          uint2* __restrict__ codes, float* __restrict__ scales, float scale_mul, const int t0,
                          const int stride, const int t_end) {
    constexpr int D = 256;
    constexpr int G = D / 32;            // groups per vector
    constexpr int T = 4;                 // k-steps per class (K = 64)
    constexpr int U = D / 8;             // 16-byte units per input row
    constexpr int ROW = U + 1;
    constexpr int NT = 256;
    constexpr int NSLOT = 7;             // exchange slots per vector: A0, A2, Am, Ap, P0, P0', unused
    __shared__ uint4 lds[2][kTileVecs * ROW];            // the tile, split by class: row = [class][8 units]
    __shared__ uint4 exch[2][4][4][64];                  // send of every wavefront: [wave][4 x 4 floats][lane]
    __shared__ float xch[2][NSLOT * kTileVecs];
    __shared__ __align__(16) float rho_s[4][64];
    // the record of a finished tile, staged for coalesced stores one stage later: code rows of CROW 8-byte units
    // (one more than a row has, so that the lanes of a wavefront hit different banks), 8 scales per vector
    constexpr int CU8 = (BITS == 8 ? D : D / 2) / 8;     // 8-byte units per code row
    constexpr int CROW = CU8 + 1;
    __shared__ uint2 cstage[2][kTileVecs * CROW];
    __shared__ __align__(16) float sstage[2][kTileVecs * G];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane & 31, half = lane >> 5;
    const int n_tiles = (int)((n_vec + kTileVecs - 1) / kTileVecs);
    const int last_lim = (int)(n_vec - 1 - (long long)(n_tiles - 1) * kTileVecs);
    const bool sine = wave >= 2, odd = wave & 1;
    // packed index of the direct run's first element and of the mirror run's element (h = 0, v = 0)
    const int base_d = wave == 0 ? 0 : wave == 1 ? 192 : wave == 2 ? 128 : 64;
    const int p_top = wave == 0 ? 128 : wave == 1 ? 192 : wave == 2 ? 256 : 64;
    const int slot_in = p_top / 32 - 1;                  // group of the mirror run
    const int cls_a = odd ? 1 : 0, cls_c = odd ? 3 : 2;
    const bool k0 = (half == 0);                         // this lane's element 0 is k1 = 0
    const bool kill_keep = k0 && wave == 3, kill_recv = k0 && wave == 1;
    const bool take_nyquist = k0 && wave == 2;
    // what the k1 = 0 lanes publish: a[0], c[0] (wave 2: A0, A2), send[0], keep[0] (wave 3: Am, Ap; wave 0: keep = P0;
    // wave 1: send = P0'); everything else goes to the unused slot
    const int slot_a = (k0 && wave == 2) ? 0 : 6, slot_c = (k0 && wave == 2) ? 1 : 6;
    const int slot_s = !k0 ? 6 : wave == 3 ? 2 : wave == 1 ? 5 : 6;
    const int slot_k = !k0 ? 6 : wave == 3 ? 3 : wave == 0 ? 4 : 6;
    const int slot_x1 = (wave == 0 || wave == 3) ? 0 : 1, slot_x2 = (wave == 0 || wave == 3) ? 2 : 3;

    half8 ahi[T], alo[T], chi[T], clo[T];
#pragma unroll
    for (int t = 0; t < T; ++t) {
        ahi[t] = __builtin_bit_cast(half8, wf4[(((wave * 2 + 0) * T + t) * 2 + 0) * 64 + lane]);
        alo[t] = __builtin_bit_cast(half8, wf4[(((wave * 2 + 0) * T + t) * 2 + 1) * 64 + lane]);
        chi[t] = __builtin_bit_cast(half8, wf4[(((wave * 2 + 1) * T + t) * 2 + 0) * 64 + lane]);
        clo[t] = __builtin_bit_cast(half8, wf4[(((wave * 2 + 1) * T + t) * 2 + 1) * 64 + lane]);
    }
    {
        const float* rho_g = reinterpret_cast<const float*>(wf4 + kFold4FragUnits);
        rho_s[wave][lane] = rho_g[wave * 64 + lane];
    }
    const uint4 misc = wf4[kFold4FragUnits + kFold4RhoFloats / 4 + wave];
    const float beta1 = __uint_as_float(misc.x), beta2 = __uint_as_float(misc.y);
    const float nyq_scale = __uint_as_float(misc.z), tau = __uint_as_float(misc.w);

    // each thread moves one 64-byte chunk (32 consecutive inputs) per tile: chunk tid % 8 of row tid / 8
    const int frow = tid >> 3, fchunk = tid & 7;
    auto fetch = [&](uint4& a, uint4& b, uint4& c, uint4& d, int tile) __attribute__((always_inline)) {
        if (tile > n_tiles - 1) tile = n_tiles - 1;
        const int lim = (tile == n_tiles - 1) ? last_lim : kTileVecs - 1;
        const uint4* src = x + (long long)tile * kTileVecs * U + (unsigned)(min(frow, lim) * U + 4 * fchunk);
        a = src[0];          // plain loads: four loads touch every line, and non-temporal ones then fetch it again
        b = src[1];
        c = src[2];
        d = src[3];
    };
    // 32 consecutive inputs -> for each class the 8 that belong to it (positions c, c + 4, ... of the chunk)
    auto to_lds = [&](int buf, const uint4& a, const uint4& b, const uint4& c, const uint4& d) __attribute__((always_inline)) {
        constexpr uint32_t kLo = 0x05040100u, kHi = 0x07060302u;
        uint4* row = &lds[buf][frow * ROW + fchunk];
        row[0] = make_uint4(__builtin_amdgcn_perm(a.z, a.x, kLo), __builtin_amdgcn_perm(b.z, b.x, kLo),
                            __builtin_amdgcn_perm(c.z, c.x, kLo), __builtin_amdgcn_perm(d.z, d.x, kLo));
        row[8] = make_uint4(__builtin_amdgcn_perm(a.z, a.x, kHi), __builtin_amdgcn_perm(b.z, b.x, kHi),
                            __builtin_amdgcn_perm(c.z, c.x, kHi), __builtin_amdgcn_perm(d.z, d.x, kHi));
        row[16] = make_uint4(__builtin_amdgcn_perm(a.w, a.y, kLo), __builtin_amdgcn_perm(b.w, b.y, kLo),
                             __builtin_amdgcn_perm(c.w, c.y, kLo), __builtin_amdgcn_perm(d.w, d.y, kLo));
        row[24] = make_uint4(__builtin_amdgcn_perm(a.w, a.y, kHi), __builtin_amdgcn_perm(b.w, b.y, kHi),
                             __builtin_amdgcn_perm(c.w, c.y, kHi), __builtin_amdgcn_perm(d.w, d.y, kHi));
    };
    auto contract = [&](int b, floatx16& a, floatx16& c) __attribute__((always_inline)) {
        const uint4* rowa = &lds[b][col * ROW + 8 * cls_a + half];
        const uint4* rowc = &lds[b][col * ROW + 8 * cls_c + half];
        a = floatx16{0};
        c = floatx16{0};
#pragma unroll
        for (int t = 0; t < T; ++t) {
            const half8 ba = __builtin_bit_cast(half8, rowa[2 * t]);
            const half8 bc = __builtin_bit_cast(half8, rowc[2 * t]);
            a = __builtin_amdgcn_mfma_f32_32x32x16_f16(ahi[t], ba, a, 0, 0, 0);
            c = __builtin_amdgcn_mfma_f32_32x32x16_f16(chi[t], bc, c, 0, 0, 0);
            a = __builtin_amdgcn_mfma_f32_32x32x16_f16(alo[t], ba, a, 0, 0, 0);
            c = __builtin_amdgcn_mfma_f32_32x32x16_f16(clo[t], bc, c, 0, 0, 0);
        }
    };
    // end of the stage that contracts a tile: a <- keep = a + c; send = a - c goes to LDS together with what the
    // k1 = 0 lanes owe the other wavefronts (straight-line code: lanes with nothing to say write the unused slot)
    auto hand_over = [&](int b, floatx16& a, const floatx16& c) __attribute__((always_inline)) {
        float* slots = &xch[b][col];
        slots[slot_a * kTileVecs] = a[0];
        slots[slot_c * kTileVecs] = c[0];
        float send[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            send[v] = a[v] - c[v];
            a[v] = a[v] + c[v];
        }
        slots[slot_s * kTileVecs] = send[0];
        slots[slot_k * kTileVecs] = a[0];
#pragma unroll
        for (int i = 0; i < 4; ++i)
            exch[b][wave][i][lane] = make_uint4(__float_as_uint(send[4 * i]), __float_as_uint(send[4 * i + 1]),
                                                __float_as_uint(send[4 * i + 2]), __float_as_uint(send[4 * i + 3]));
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
        inv = __builtin_amdgcn_rcpf(scale);
        if (!(scale >= kMinScale)) { scale = 0.0f; inv = 0.0f; }
    };
    // vector-ALU tail of the tile whose keep is in `keep` and whose exchange values are in exch[b] / xch[b]
    auto finish = [&](int b, const floatx16& keep, int tile) __attribute__((always_inline)) {
        const long long row0 = (long long)tile * kTileVecs;
        const int lim = (tile == n_tiles - 1) ? last_lim : kTileVecs - 1;
        const int c = min(col, lim);
        float x1 = xch[b][slot_x1 * kTileVecs + col], x2 = xch[b][slot_x2 * kTileVecs + col];
        float n1 = xch[b][4 * kTileVecs + col], n2 = xch[b][5 * kTileVecs + col];
        asm volatile("" : "+v"(x1), "+v"(x2), "+v"(n1), "+v"(n2));      // read by every lane: no branch around the loads
        const float below = fmaf(beta2, x2, beta1 * x1);                // packed index 32 * slot_in
        const float nyquist = nyq_scale * (n1 - n2);
        float recv[16], rd[16], rm[16];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint4 r = exch[b][(wave + 1) & 3][i][lane];
            recv[4 * i] = __uint_as_float(r.x); recv[4 * i + 1] = __uint_as_float(r.y);
            recv[4 * i + 2] = __uint_as_float(r.z); recv[4 * i + 3] = __uint_as_float(r.w);
            const float4 d4 = *reinterpret_cast<const float4*>(&rho_s[wave][16 * half + 4 * i]);
            const float4 m4 = *reinterpret_cast<const float4*>(&rho_s[wave][32 + 16 * half + 4 * i]);
            rd[4 * i] = d4.x; rd[4 * i + 1] = d4.y; rd[4 * i + 2] = d4.z; rd[4 * i + 3] = d4.w;
            rm[4 * i] = m4.x; rm[4 * i + 1] = m4.y; rm[4 * i + 2] = m4.z; rm[4 * i + 3] = m4.w;
        }
        float dv[16], mv[16];
        {
            const float k0v = kill_keep ? 0.0f : keep[0], r0v = kill_recv ? 0.0f : recv[0];
            dv[0] = rd[0] * fmaf(r0v, tau, k0v);
            mv[0] = rm[0] * fmaf(r0v, -tau, k0v);
        }
#pragma unroll
        for (int v = 1; v < 16; ++v) {
            dv[v] = rd[v] * fmaf(recv[v], tau, keep[v]);
            mv[v] = rm[v] * fmaf(recv[v], -tau, keep[v]);
        }
        dv[0] = take_nyquist ? nyquist : dv[0];
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
        float sd, id, sm, im;
        scale_of(md, sd, id);
        scale_of(mm, sm, im);
        uint2* crow = &cstage[b][col * CROW];
        if constexpr (BITS == 8) {               // 16 values = 16 bytes = two 8-byte units
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
        sstage[b][col * G + (half ? slot_in : base_d / 32)] = half ? sm : sd;
    };

    // staged record of `tile` -> global memory: 16 bytes per thread, whole rows next to each other (rows past the end
    // alias to the last row); the first wavefront also moves the scales
    auto flush = [&](int b, int tile) __attribute__((always_inline)) {
        const long long row0 = (long long)tile * kTileVecs;
        const int lim = (tile == n_tiles - 1) ? last_lim : kTileVecs - 1;
        constexpr int PIECES = CU8 / 2;                  // 16-byte pieces per code row
        uint4* cbase = reinterpret_cast<uint4*>(codes) + row0 * PIECES;
#pragma unroll
        for (int i = 0; i < kTileVecs * PIECES / NT; ++i) {
            const int u = tid + i * NT, r = u / PIECES, pc = u % PIECES;
            const uint2 lo = cstage[b][r * CROW + 2 * pc], hi = cstage[b][r * CROW + 2 * pc + 1];
            cbase[(unsigned)(min(r, lim) * PIECES + pc)] = make_uint4(lo.x, lo.y, hi.x, hi.y);
        }
        if (wave == 0) {                                 // uniform per wavefront
            const int r = lane >> 1, hf = lane & 1;
            const float4 v = *reinterpret_cast<const float4*>(&sstage[b][r * G + 4 * hf]);
            reinterpret_cast<float4*>(scales + row0 * G)[(unsigned)(min(r, lim) * 2 + hf)] = v;
        }
    };

    const int m = (t_end - 1 - t0) / stride + 1;            // tiles of this workgroup: t0, t0 + stride, ... < t_end
    uint4 pa0, pa1, pa2, pa3, pb0, pb1, pb2, pb3;
    floatx16 aa, ca, ab, cb;                     // two accumulator sets; after hand_over the a of a set holds keep
    fetch(pa0, pa1, pa2, pa3, t0);
    fetch(pb0, pb1, pb2, pb3, t0 + stride);
    hold_in_registers(ahi, alo);
    hold_in_registers(chi, clo);
    to_lds(0, pa0, pa1, pa2, pa3);
    fetch(pa0, pa1, pa2, pa3, t0 + 2 * stride);
    // stage 0
    __syncthreads();
    contract(0, aa, ca);
    to_lds(1, pb0, pb1, pb2, pb3);
    fetch(pb0, pb1, pb2, pb3, t0 + 3 * stride);
    hand_over(0, aa, ca);
    int k = 1;
    for (; k + 1 < m; k += 2) {
        const int tk = t0 + k * stride;
        __syncthreads();                         // stage k (odd)
        rotate_priority(k);
        if (k >= 2) flush(1, tk - 2 * stride);
        contract(1, ab, cb);
        finish(0, aa, tk - stride);
        to_lds(0, pa0, pa1, pa2, pa3);
        fetch(pa0, pa1, pa2, pa3, tk + 3 * stride);
        hand_over(1, ab, cb);
        __syncthreads();                         // stage k + 1 (even)
        rotate_priority(k + 1);
        flush(0, tk - stride);
        contract(0, aa, ca);
        finish(1, ab, tk);
        to_lds(1, pb0, pb1, pb2, pb3);
        fetch(pb0, pb1, pb2, pb3, tk + 4 * stride);
        hand_over(0, aa, ca);
    }
    // finish(b, ...) stages into buffer b, flush(b, ...) stores it one barrier later
    if (k < m) {                                 // one more odd stage
        const int tk = t0 + k * stride;
        __syncthreads();
        if (k >= 2) flush(1, tk - 2 * stride);
        contract(1, ab, cb);
        finish(0, aa, tk - stride);
        hand_over(1, ab, cb);
        __syncthreads();
        flush(0, tk - stride);
        finish(1, ab, tk);
        __syncthreads();
        flush(1, tk);
    } else {
        const int tl = t0 + (k - 1) * stride;    // the last stage was even (or stage 0): its tile's keep is in aa
        __syncthreads();
        if (k >= 2) flush(1, tl - stride);
        finish(0, aa, tl);
        __syncthreads();
        flush(0, tl);
    }
}

template <int BITS>
__global__ void __launch_bounds__(256, 2)
srft_quantize_fold4_kernel(const uint4* __restrict__ wf4, const uint4* __restrict__ x, long long n_vec,
                           uint2* __restrict__ codes, float* __restrict__ scales, float4* __restrict__,
                           float, float scale_mul, int) {
    int t0, stride, t_end;
    if (!srft_tile_range(n_vec, t0, stride, t_end)) return;
    srft_quantize_fold4_tiles<BITS>(wf4, x, n_vec, codes, scales, scale_mul, t0, stride, t_end);
}

template <int BITS>
__global__ void __launch_bounds__(256, 2)
srft_quantize_fold4_batched_kernel(const srft_batch_args a, int) {
    const int i = srft_segment_of_block(a, blockIdx.x);
    srft_quantize_fold4_tiles<BITS>(a.frag[i], (const uint4*)a.in0[i], a.n_vec[i], (uint2*)a.out0[i],
                                    (float*)a.out1[i], 1.0f / (BITS == 8 ? 127.0f : 7.0f),
                                    blockIdx.x - a.first_block[i], a.first_block[i + 1] - a.first_block[i],
                                    (int)((a.n_vec[i] + kTileVecs - 1) / kTileVecs));
}

#endif  // SRFT_QUANTIZE_FOLD4_TILES_H
