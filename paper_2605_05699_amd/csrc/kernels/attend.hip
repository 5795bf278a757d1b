// Weighted sums of the stored values, in the rotated domain: the value side of attention over the int4 cache.
//
//     out_i = sum_t w[i][t] v_t,   v_t = s * Q^T (code_t * scale_t / max(lambda, 1e-6))    (the read path's value)
// The transform is linear, so the sum over the keys is taken on the codes,
//     acc_i[k] = sum_t w[i][t] * scale_t[group of k] * code_t[k],
// and ONE inverse transform per query follows:  out_i = s * Q^T (acc_i / max(lambda, 1e-6)).  The record is read once
// (d/2 + 4 d/g bytes per value instead of the 2 d of a dequantized prefix); no value is ever reconstructed.
//
// Step 1 (srft_attend_accumulate_kernel): a contraction over the keys on the matrix cores.  Per group j of 32
// channels, A = w[i][t] * scale_t[j] (up to 32 queries x 16 keys per MFMA, fp32 products split into fp16 hi + lo),
// B = the codes of the group (16 keys x 32 channels, exact fp16).  Both MFMA operands want the contraction index --
// here the key -- to run inside a lane, while the record is key-major: every thread takes the code units of 8
// consecutive keys (one 16-channel unit each), decodes them and transposes the 8 x 16 block in registers with byte
// permutes, so that one 16-byte LDS write is one channel's 8 keys = one lane's B fragment.
// One wavefront per workgroup; a wavefront owns a slab of up to 128 channels and a stripe of 64-key tiles, keeps
// its sums in the MFMA accumulators for the whole launch, and writes them once, to its slot of the workspace.
// Step 2 (srft_attend_finish_kernel): the partial sums of all workgroups are added in a fixed order (the result does
// not depend on timing) and multiplied by R = diag(s) Q^T diag(1 / max(lambda, 1e-6)) in fp32.
#include "../device_util.h"

namespace {

constexpr int kAttendTileKeys = 64;

// D: head dimension; GS: groups of 32 channels per wavefront (slab = 32 GS channels); SLABS = D / (32 GS)
// NQB: query rows the kernel carries (n_q <= NQB).  8 and 16 run on v_mfma_f32_16x16x32_f16 (16 query rows, 32 keys
// per instruction: half the matrix-core time and half the operand-forming work of the 32-row form), 32 on
// v_mfma_f32_32x32x16_f16.
// row_max: nullptr, or per query the ordered code of the maximum of sign(softmax_scale) * w over the keys: w then
// holds raw scores, the weight exp(softmax_scale * w - maximum) is formed as the scores are loaded, and the workgroup
// leaves the sum of its weights per query in den_part[stripe][32] (slab 0 only) for the final division.
template <int D, int GS, int NQB>
// (second bound: wavefronts per SIMD the register allocator aims for; LDS allows 8 / 7 / 5 workgroups per compute unit)
__global__ void __launch_bounds__(64, NQB <= 16 ? 3 : 2)
srft_attend_accumulate_kernel(const float* __restrict__ w, int n_q, const uint2* __restrict__ codes,
                              const float* __restrict__ scales, long long n_keys, int gw, float* __restrict__ part,
                              int stripes, const unsigned int* __restrict__ row_max, float softmax_scale,
                              float* __restrict__ den_part) {
    constexpr bool R16 = NQB <= 16;
    constexpr int ROWS = R16 ? 16 : 32;                      // rows of the MFMA A operand
    constexpr int G = D / 32, SLABS = G / GS, C = D / 16;    // C: 8-byte code units per row
    constexpr int UN = 2 * GS;                               // code units (16 channels) per key in the slab
    constexpr int SLOTS = 32 * GS + UN - 1;                  // B tile: one 16-byte slot per channel, one spare between units
    static_assert(G % GS == 0 && UN * 8 <= 64, "eight key blocks of UN threads each");
    // one buffer each: a workgroup is one wavefront, whose LDS accesses complete in program order
    __shared__ uint4 bt[8 * SLOTS];                          // [key block of 8][channel slot]: 8 keys of one channel
    __shared__ __align__(16) float st[GS * kAttendTileKeys]; // scales, [group][key]
    constexpr int WROW = kAttendTileKeys + 4;                // padded row: the query rows are read bank-conflict free
    __shared__ __align__(16) float wt[NQB * WROW];           // weights, [query][key] (rows past n_q hold zeros)
    const int lane = threadIdx.x;
    const int slab = blockIdx.x % SLABS, stripe = blockIdx.x / SLABS;
    const int ns = G / gw;                                   // scales per key
    const long long n_tiles = (n_keys + kAttendTileKeys - 1) / kAttendTileKeys;
    // transposing threads: key block kb (8 keys), unit u (16 channels of the slab)
    const int kb = lane / UN, u = lane % UN;
    const bool mover = lane < 8 * UN;

    using Acc = std::conditional_t<R16, floatx4, floatx16>;
    constexpr int NACC = R16 ? 2 * GS : GS;                  // 16 x 16 blocks (16 channels each) or 32 x 32 blocks
    Acc acc[NACC];
#pragma unroll
    for (int j = 0; j < NACC; ++j) acc[j] = Acc{0};

    // row maxima of softmax_scale * score (uniform: scalar registers); rows past n_q alias to the last row
    float rmax[NQB], wsum[NQB];
#pragma unroll
    for (int i = 0; i < NQB; ++i) {
        rmax[i] = 0.0f;
        wsum[i] = 0.0f;
    }
    if (row_max) {                               // uniform: lane l reads copy l, the wavefront takes the maximum
        static_assert(kRowMaxCopies == 64, "one copy per lane");
#pragma unroll
        for (int i = 0; i < NQB; ++i) {
            unsigned int code = row_max[lane * 32 + min(i, n_q - 1)];
#pragma unroll
            for (int step = 32; step > 0; step >>= 1) code = max(code, (unsigned int)__shfl_xor((int)code, step, 64));
            rmax[i] = fabsf(softmax_scale) * srft_ordered_value(code);
        }
    }
    struct Prefetch { uint2 c[8]; float s[GS]; };
    float wreg[NQB];                                         // weights of the next tile (one key per lane)
    // Addresses are a uniform tile base (scalar registers) plus a 32-bit lane offset; keys past the end alias to the
    // last key of the tile (`lim`, uniform) -- their weights are taken as zero below.
    const int kbm = mover ? kb : 0, um = mover ? u : 0;
    // codes of this thread's 8 keys x 1 unit; the tile's scales (one key per lane)
    auto fetch = [&](Prefetch& p, long long tile) __attribute__((always_inline)) {
        const long long t0 = tile * kAttendTileKeys;
        const int lim = (int)min((long long)(kAttendTileKeys - 1), n_keys - 1 - t0);
        const uint2* cbase = codes + t0 * C + slab * UN;
#pragma unroll
        for (int i = 0; i < 8; ++i) p.c[i] = cbase[(unsigned)(min(8 * kbm + i, lim) * C + um)];
        const float* sbase = scales + t0 * ns;
        const int rl = min(lane, lim);
#pragma unroll
        for (int j = 0; j < GS; ++j) p.s[j] = sbase[(unsigned)(rl * ns + (slab * GS + j) / gw)];
    };
    // the weights of key t0 + lane, one query after the other (each load covers 256 contiguous bytes of a row).
    // Every load is issued whatever n_q is (rows past n_q re-read the last row), so that all of them are in flight
    // at once; rows past n_q and keys past the end carry weight zero.
    auto fetch_w = [&](long long tile) __attribute__((always_inline)) {
        const long long t0 = tile * kAttendTileKeys;
        const int lim = (int)min((long long)(kAttendTileKeys - 1), n_keys - 1 - t0);
        const bool live = lane <= lim;
        const int rl = min(lane, lim);
        float v[NQB];
#pragma unroll
        for (int i = 0; i < NQB; ++i) v[i] = (w + (long long)min(i, n_q - 1) * n_keys + t0)[(unsigned)rl];
        if (row_max) {                           // uniform
#pragma unroll
            for (int i = 0; i < NQB; ++i) v[i] = __expf(fmaf(softmax_scale, v[i], -rmax[i]));
        }
#pragma unroll
        for (int i = 0; i < NQB; ++i) {
            wreg[i] = (live && i < n_q) ? v[i] : 0.0f;
            wsum[i] += wreg[i];
        }
    };
    // Codes -> B fragments.  The 8 keys x 16 channels block of this thread is transposed as bytes (a byte holds the
    // nibbles of channels 2 c and 2 c + 1): four 4 x 4 byte transposes give, per channel pair and half of the keys,
    // one dword with the bytes of keys 4 h .. 4 h + 3.  decode8 of such a dword yields the packed fp16 pairs
    // (key 0, key 2) and (key 1, key 3) of the even channel (.x, .z) and of the odd channel (.y, .w): a fragment holds
    // its 8 keys in the order 0 2 1 3 4 6 5 7, and the A operand is built in the same order (kKeyOrder).
    auto to_lds = [&](const Prefetch& p) __attribute__((always_inline)) {
        constexpr uint32_t kLo = 0x05040100u, kHi = 0x07060302u, kZipLo = 0x05010400u, kZipHi = 0x07030602u;
        // rows r0 .. r3 (dwords of four keys) -> t[c] = byte c of each row
        auto transpose4 = [&](uint32_t r0, uint32_t r1, uint32_t r2, uint32_t r3, uint32_t (&t)[4]) __attribute__((always_inline)) {
            const uint32_t a_lo = __builtin_amdgcn_perm(r1, r0, kZipLo), a_hi = __builtin_amdgcn_perm(r1, r0, kZipHi);
            const uint32_t b_lo = __builtin_amdgcn_perm(r3, r2, kZipLo), b_hi = __builtin_amdgcn_perm(r3, r2, kZipHi);
            t[0] = __builtin_amdgcn_perm(b_lo, a_lo, kLo);
            t[1] = __builtin_amdgcn_perm(b_lo, a_lo, kHi);
            t[2] = __builtin_amdgcn_perm(b_hi, a_hi, kLo);
            t[3] = __builtin_amdgcn_perm(b_hi, a_hi, kHi);
        };
        if (mover) {
            uint4* dst = &bt[kb * SLOTS + 17 * u];
#pragma unroll
            for (int side = 0; side < 2; ++side) {           // channels 0 .. 7 (.x of the units) and 8 .. 15 (.y)
                uint32_t t0[4], t1[4];
                if (side == 0) {
                    transpose4(p.c[0].x, p.c[1].x, p.c[2].x, p.c[3].x, t0);
                    transpose4(p.c[4].x, p.c[5].x, p.c[6].x, p.c[7].x, t1);
                } else {
                    transpose4(p.c[0].y, p.c[1].y, p.c[2].y, p.c[3].y, t0);
                    transpose4(p.c[4].y, p.c[5].y, p.c[6].y, p.c[7].y, t1);
                }
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const uint4 lo = decode8(t0[c]), hi = decode8(t1[c]);
                    dst[8 * side + 2 * c] = make_uint4(lo.x, lo.z, hi.x, hi.z);
                    dst[8 * side + 2 * c + 1] = make_uint4(lo.y, lo.w, hi.y, hi.w);
                }
            }
        }
#pragma unroll
        for (int j = 0; j < GS; ++j) st[j * kAttendTileKeys + lane] = p.s[j];
#pragma unroll
        for (int i = 0; i < NQB; ++i) wt[i * WROW + lane] = wreg[i];
    };
    // a = w * scale for this lane's 8 keys (in the fragments' key order) as fp16 hi + fp16 lo: hi is a truncated to
    // fp16 (two values per conversion), a - hi is exact in fp32, lo is that remainder truncated to fp16: about 21 bits
    auto split = [&](const float4& w0, const float4& w1, const float4& s0, const float4& s1, half8& ahi, half8& alo)
                     __attribute__((always_inline)) {
        const float wv[8] = {w0.x, w0.z, w0.y, w0.w, w1.x, w1.z, w1.y, w1.w};     // key order 0 2 1 3 4 6 5 7
        const float sc[8] = {s0.x, s0.z, s0.y, s0.w, s1.x, s1.z, s1.y, s1.w};
        uint32_t hh[4], ll[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float a0 = wv[2 * e] * sc[2 * e], a1 = wv[2 * e + 1] * sc[2 * e + 1];
            const auto h2 = __builtin_amdgcn_cvt_pkrtz(a0, a1);
            const auto l2 = __builtin_amdgcn_cvt_pkrtz(a0 - (float)h2[0], a1 - (float)h2[1]);
            hh[e] = __builtin_bit_cast(uint32_t, h2);
            ll[e] = __builtin_bit_cast(uint32_t, l2);
        }
        ahi = __builtin_bit_cast(half8, make_uint4(hh[0], hh[1], hh[2], hh[3]));
        alo = __builtin_bit_cast(half8, make_uint4(ll[0], ll[1], ll[2], ll[3]));
    };
    // The tile in bt / st / wt: acc += (w * scale_j) . codes_j over its 64 keys.  Steps (k-step, group) are software
    // pipelined: the LDS reads of step i + 1 (scales and B fragments) are issued before the arithmetic of step i, and
    // a scheduling barrier keeps them there; with one or two wavefronts per SIMD nothing else hides the LDS latency.
    // R16: k-steps of 32 keys.  A: lane = (query row m, key block k8): keys 32 ks + 8 k8 + e.  B: lane = (channel n of a
    //      block of 16, key block k8).  Result register r of a lane: query 4 (lane / 16) + r, channel n.
    // else: k-steps of 16 keys; lane (col, half): query row / channel col, keys 16 ks + 8 half + e.
    constexpr int KSTEPS = R16 ? 2 : 4, KKEYS = kAttendTileKeys / KSTEPS, NB = R16 ? 2 : 1;
    const int arow = R16 ? (lane & 15) : (lane & 31), k8 = R16 ? (lane >> 4) : (lane >> 5);
    struct Step { float4 s0, s1; uint4 b[NB]; };
    auto load_step = [&](Step& f, int ks, int j) __attribute__((always_inline)) {
        const float* sp = &st[j * kAttendTileKeys + KKEYS * ks + 8 * k8];
        f.s0 = *reinterpret_cast<const float4*>(sp);
        f.s1 = *reinterpret_cast<const float4*>(sp + 4);
#pragma unroll
        for (int c = 0; c < NB; ++c) {
            const int ch = 32 * j + (R16 ? 16 * c : 0) + arow;
            f.b[c] = bt[((KKEYS / 8) * ks + k8) * SLOTS + ch + ch / 16];
        }
    };
    auto contract = [&]() __attribute__((always_inline)) {
        float4 w0[KSTEPS], w1[KSTEPS];
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) {
            // MFMA rows past the NQB rows that wt holds (8 queries on the 16-row form) carry weight zero
            const float* wp = &wt[(arow < NQB ? arow : 0) * WROW + KKEYS * ks + 8 * k8];
            const float4 zero = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
            w0[ks] = arow < NQB ? *reinterpret_cast<const float4*>(wp) : zero;
            w1[ks] = arow < NQB ? *reinterpret_cast<const float4*>(wp + 4) : zero;
        }
        Step cur, nxt;
        load_step(cur, 0, 0);
#pragma unroll
        for (int it = 0; it < KSTEPS * GS; ++it) {
            const int ks = it / GS, j = it % GS;
            if (it + 1 < KSTEPS * GS) load_step(nxt, (it + 1) / GS, (it + 1) % GS);
            half8 ahi, alo;
            split(w0[ks], w1[ks], cur.s0, cur.s1, ahi, alo);
#pragma unroll
            for (int c = 0; c < NB; ++c) {
                const half8 bf = __builtin_bit_cast(half8, cur.b[c]);
                if constexpr (R16) {
                    acc[2 * j + c] = __builtin_amdgcn_mfma_f32_16x16x32_f16(ahi, bf, acc[2 * j + c], 0, 0, 0);
                    acc[2 * j + c] = __builtin_amdgcn_mfma_f32_16x16x32_f16(alo, bf, acc[2 * j + c], 0, 0, 0);
                } else {
                    acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ahi, bf, acc[j], 0, 0, 0);
                    acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(alo, bf, acc[j], 0, 0, 0);
                }
            }
            cur = nxt;
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // tiles of this stripe: stripe, stripe + stripes, ...; codes and scales are prefetched two tiles ahead in two named
    // register sets (two tiles per trip), the weights one tile ahead
    const long long m_tiles = stripe < n_tiles ? (n_tiles - 1 - stripe) / stripes + 1 : 0;
    Prefetch pa, pb;
    auto tile_of = [&](long long k) { return min(stripe + k * stripes, n_tiles - 1); };   // past the end: re-read the last
    if (m_tiles > 0) {
        fetch(pa, tile_of(0));
        fetch_w(tile_of(0));
        fetch(pb, tile_of(1));
        long long k = 0;
        for (; k + 1 < m_tiles; k += 2) {
            to_lds(pa);
            fetch_w(tile_of(k + 1));
            fetch(pa, tile_of(k + 2));
            __syncthreads();                     // one wavefront: orders the LDS writes before the reads
            contract();
            to_lds(pb);
            fetch_w(tile_of(k + 2));
            fetch(pb, tile_of(k + 3));
            __syncthreads();
            contract();
        }
        if (k < m_tiles) {
            to_lds(pa);
            __syncthreads();
            contract();
        }
    }
    // the sums of this workgroup's weights, lane by lane in a fixed order
    if (den_part && slab == 0) {                 // uniform
#pragma unroll
        for (int i = 0; i < NQB; ++i) {
            float t = wsum[i];
#pragma unroll
            for (int step = 32; step > 0; step >>= 1) t += __shfl_xor(t, step, 64);
            if (lane == 0) den_part[stripe * 32 + i] = t;
        }
    }
    // the sums of this workgroup: part[stripe][query][channel]
    float* dst = part + (long long)stripe * 32 * D;
    if constexpr (R16) {
        const int n = lane & 15, a4 = lane >> 4;
#pragma unroll
        for (int b = 0; b < NACC; ++b)
#pragma unroll
            for (int r = 0; r < 4; ++r) dst[(4 * a4 + r) * D + 32 * slab * GS + 16 * b + n] = acc[b][r];
    } else {
        // the accumulator of lane (col, half) holds rows (queries) 8 r + 4 half + i in register 4 r + i, column =
        // channel 32 j + col of the slab
        const int col = lane & 31, half = lane >> 5;
#pragma unroll
        for (int j = 0; j < GS; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int q = 8 * (v / 4) + 4 * half + (v % 4);
                dst[q * D + 32 * (slab * GS + j) + col] = acc[j][v];
            }
    }
}

// first level of the fixed-order sum: part2[c][i][n] = sum over the stripes c, c + kAttendFan, ... of part[stripe][i][n]
// (eight loads in flight per thread; the eight running sums are added in a fixed order).  With den_part, the blocks
// c = kAttendFan add the stripes' sums of weights of query i instead: den[i], thread by thread in a fixed order.
template <int D>
__global__ void __launch_bounds__(D)
srft_attend_reduce_kernel(const float* __restrict__ part, int stripes, float* __restrict__ part2,
                          const float* __restrict__ den_part, float* __restrict__ den) {
    __shared__ float red[D / 64];
    const int i = blockIdx.x, c = blockIdx.y, n = threadIdx.x;
    if (c == kAttendFan) {                       // uniform per block
        float t = 0.0f;
        for (int sidx = n; sidx < stripes; sidx += D) t += den_part[sidx * 32 + i];
#pragma unroll
        for (int step = 32; step > 0; step >>= 1) t += __shfl_xor(t, step, 64);
        if ((n & 63) == 0) red[n >> 6] = t;
        __syncthreads();
        if (n == 0) {
            float total = red[0];
            for (int k = 1; k < D / 64; ++k) total += red[k];
            den[i] = total;
        }
        return;
    }
    float sum[8] = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};
    for (int s0 = c; s0 < stripes; s0 += 8 * kAttendFan) {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int sidx = s0 + e * kAttendFan;
            sum[e] += sidx < stripes ? part[((long long)sidx * 32 + i) * D + n] : 0.0f;
        }
    }
    part2[((long long)c * 32 + i) * D + n] = ((sum[0] + sum[1]) + (sum[2] + sum[3])) + ((sum[4] + sum[5]) + (sum[6] + sum[7]));
}

// out[i][n] = sum_k rmat[k][n] * (sum over c of part2[c][i][k]) / den[i];  rmat[k][n] = s_n Q[k][n] / max(lambda_k, 1e-6);
// without den the divisor is 1.
// A workgroup of 4 D threads per query: quarter q of the threads adds the first-level sums c = q (mod 4) of channel n,
// then takes the quarter q of the k range of output n; both sets of four partial results meet in LDS, in a fixed order.
template <int D>
__global__ void __launch_bounds__(4 * D)
srft_attend_finish_kernel(const float* __restrict__ part2, const float* __restrict__ rmat, float* __restrict__ out,
                          const float* __restrict__ den) {
    __shared__ float quarter[4][D];
    __shared__ float accs[D];
    const int i = blockIdx.x, n = threadIdx.x % D, q = threadIdx.x / D;
    const float inv_den = den ? 1.0f / den[i] : 1.0f;
    float sum = 0.0f;
#pragma unroll
    for (int c = q; c < kAttendFan; c += 4) sum += part2[((long long)c * 32 + i) * D + n];
    quarter[q][n] = sum;
    __syncthreads();
    if (q == 0) accs[n] = (quarter[0][n] + quarter[1][n]) + (quarter[2][n] + quarter[3][n]);
    __syncthreads();
    float o = 0.0f;
#pragma unroll
    for (int k = 0; k < D / 4; ++k) o = fmaf(rmat[(q * (D / 4) + k) * D + n], accs[q * (D / 4) + k], o);   // all loads in flight
    quarter[q][n] = o;
    __syncthreads();
    if (q == 0) out[(long long)i * D + n] = ((quarter[0][n] + quarter[1][n]) + (quarter[2][n] + quarter[3][n])) * inv_den;
}

template <int D, int GS, int NQB>
int launch_rows(const srft_plan* p, const float* w, int n_q, const uint8_t* codes, const float* scales, long long n_keys,
                float* out, float* part, int stripes, const unsigned int* row_max, float softmax_scale, hipStream_t st) {
    constexpr int SLABS = D / 32 / GS;
    // workspace: part [kMaxAttendStripes][32][D], part2 [kAttendFan][32][D], den_part [kMaxAttendStripes][32], den [32]
    float* part2 = part + (size_t)kMaxAttendStripes * 32 * D;
    float* den_part = row_max ? part2 + (size_t)kAttendFan * 32 * D : nullptr;
    float* den = row_max ? den_part + (size_t)kMaxAttendStripes * 32 : nullptr;
    hipLaunchKernelGGL((srft_attend_accumulate_kernel<D, GS, NQB>), dim3((unsigned)(stripes * SLABS)), dim3(64), 0, st, w,
                       n_q, (const uint2*)codes, scales, n_keys, p->gw, part, stripes, row_max, softmax_scale, den_part);
    SRFT_HIP(hipGetLastError());
    hipLaunchKernelGGL(srft_attend_reduce_kernel<D>, dim3((unsigned)n_q, kAttendFan + (row_max ? 1 : 0)), dim3(D), 0, st,
                       (const float*)part, stripes, part2, (const float*)den_part, den);
    SRFT_HIP(hipGetLastError());
    hipLaunchKernelGGL(srft_attend_finish_kernel<D>, dim3((unsigned)n_q), dim3(4 * D), 0, st, (const float*)part2,
                       (const float*)p->rmat_f32, out, (const float*)den);
    SRFT_HIP(hipGetLastError());
    return SRFT_OK;
}

template <int D, int GS>
int launch(const srft_plan* p, const float* w, int n_q, const uint8_t* codes, const float* scales, long long n_keys,
           float* out, float* part, const unsigned int* row_max, float softmax_scale, hipStream_t st) {
    const int stripes = srft_attend_stripes(p, n_q, n_keys);
    if (n_q <= 8)
        return launch_rows<D, GS, 8>(p, w, n_q, codes, scales, n_keys, out, part, stripes, row_max, softmax_scale, st);
    if (n_q <= 16)
        return launch_rows<D, GS, 16>(p, w, n_q, codes, scales, n_keys, out, part, stripes, row_max, softmax_scale, st);
    return launch_rows<D, GS, 32>(p, w, n_q, codes, scales, n_keys, out, part, stripes, row_max, softmax_scale, st);
}

}  // namespace

int srft_attend_stripes(const srft_plan* p, int n_q, long long n_keys) {
    // workgroups per channel slab: what a compute unit holds at once (eight one-wavefront workgroups with 8 query
    // rows, seven with 16, five with 32), at most one per tile, at most kMaxAttendStripes
    const long long n_tiles = (n_keys + kAttendTileKeys - 1) / kAttendTileKeys;
    long long s = p->max_wgs > 0 ? p->max_wgs : (n_q <= 8 ? 8LL : n_q <= 16 ? 7LL : 5LL) * p->compute_units;
    if (s > kMaxAttendStripes) s = kMaxAttendStripes;
    if (s > n_tiles) s = n_tiles;
    return (int)(s < 1 ? 1 : s);
}

size_t srft_attend_workspace_floats(int d) {
    return (size_t)(kMaxAttendStripes + kAttendFan) * 32 * d + (size_t)(kMaxAttendStripes + kAttendFan) * 32;
}

int srft_launch_attend(const srft_plan* p, const float* w, int n_q, const uint8_t* codes, const float* scales,
                       long long n_keys, float* out, float* part, const unsigned int* row_max, float softmax_scale,
                       hipStream_t st) {
    switch (p->d) {
        case 64: return launch<64, 2>(p, w, n_q, codes, scales, n_keys, out, part, row_max, softmax_scale, st);
        case 128: return launch<128, 4>(p, w, n_q, codes, scales, n_keys, out, part, row_max, softmax_scale, st);
        case 192: return launch<192, 3>(p, w, n_q, codes, scales, n_keys, out, part, row_max, softmax_scale, st);
        case 256: return launch<256, 4>(p, w, n_q, codes, scales, n_keys, out, part, row_max, softmax_scale, st);
        default: return SRFT_ERR_BAD_D;
    }
}
