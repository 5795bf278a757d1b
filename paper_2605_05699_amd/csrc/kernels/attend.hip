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
template <int D, int GS>
__global__ void __launch_bounds__(64, 5)         // five one-wavefront workgroups per compute unit (LDS): within 256 VGPRs
srft_attend_accumulate_kernel(const float* __restrict__ w, int n_q, const uint2* __restrict__ codes,
                              const float* __restrict__ scales, long long n_keys, int gw, float* __restrict__ part,
                              int stripes) {
    constexpr int G = D / 32, SLABS = G / GS, C = D / 16;    // C: 8-byte code units per row
    constexpr int UN = 2 * GS;                               // code units (16 channels) per key in the slab
    constexpr int SLOTS = 32 * GS + UN;                      // B tile: one 16-byte slot per channel, one spare per unit
    static_assert(G % GS == 0 && UN * 8 <= 64, "eight key blocks of UN threads each");
    // one buffer each: a workgroup is one wavefront, whose LDS accesses complete in program order
    __shared__ uint4 bt[1][8 * SLOTS];                       // [key block of 8][channel slot]: 8 keys of one channel
    __shared__ __align__(16) float st[1][GS * kAttendTileKeys];   // scales, [group][key]
    constexpr int WROW = kAttendTileKeys + 4;                // padded row: the 32 query rows are read bank-conflict free
    __shared__ __align__(16) float wt[1][32 * WROW];         // weights, [query][key] (rows past n_q stay zero)
    const int lane = threadIdx.x, col = lane & 31, half = lane >> 5;
    const int slab = blockIdx.x % SLABS, stripe = blockIdx.x / SLABS;
    const int ns = G / gw;                                   // scales per key
    const long long n_tiles = (n_keys + kAttendTileKeys - 1) / kAttendTileKeys;
    // transposing threads: key block kb (8 keys), unit u (16 channels of the slab)
    const int kb = lane / UN, u = lane % UN;
    const bool mover = lane < 8 * UN;

    floatx16 acc[GS];
#pragma unroll
    for (int j = 0; j < GS; ++j) acc[j] = floatx16{0};

    // rows of wt that no query fills are read by the A operand: zero them once
    for (int i = n_q; i < 32; ++i) {
        wt[0][i * WROW + lane] = 0.0f;
    }
    struct Prefetch { uint2 c[8]; float s[GS]; };
    float wreg[32];                                          // weights of the next tile (one key per lane)
    // codes of this thread's 8 keys x 1 unit; the tile's scales (one key per lane); keys past the end alias to
    // the last key -- their weights are taken as zero below
    auto fetch = [&](Prefetch& p, long long tile) __attribute__((always_inline)) {
        const long long t0 = tile * kAttendTileKeys;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const long long t = min(t0 + 8 * (mover ? kb : 0) + i, n_keys - 1);
            p.c[i] = codes[t * C + slab * UN + (mover ? u : 0)];
        }
        const long long t = min(t0 + lane, n_keys - 1);
#pragma unroll
        for (int j = 0; j < GS; ++j) p.s[j] = scales[t * ns + (slab * GS + j) / gw];
    };
    // the weights of key t0 + lane, one query after the other (each load covers 256 contiguous bytes of a row);
    // keys past the end carry weight zero
    auto fetch_w = [&](long long tile) __attribute__((always_inline)) {
        const long long t = tile * kAttendTileKeys + lane;
        const bool live = t < n_keys;
        const long long tc = min(t, n_keys - 1);
#pragma unroll
        for (int i = 0; i < 32; ++i)
            if (i < n_q) {                       // uniform
                const float v = w[(long long)i * n_keys + tc];
                wreg[i] = live ? v : 0.0f;
            }
    };
    auto to_lds = [&](int b, const Prefetch& p) __attribute__((always_inline)) {
        // decode8 gives, per dword of 8 nibbles, the packed pairs (n0, n4), (n1, n5), (n2, n6), (n3, n7)
        uint4 lo[8], hi[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            lo[i] = decode8(p.c[i].x);
            hi[i] = decode8(p.c[i].y);
        }
        constexpr uint32_t kLo = 0x05040100u, kHi = 0x07060302u;
        auto put = [&](int c0, uint32_t d0, uint32_t d1, uint32_t d2, uint32_t d3, uint32_t d4, uint32_t d5,
                       uint32_t d6, uint32_t d7) __attribute__((always_inline)) {
            // d_i = (code of key i at channel c0, at channel c0 + 4): two channels' runs of 8 keys
            uint4* dst = &bt[b][kb * SLOTS + 17 * u];
            dst[c0] = make_uint4(__builtin_amdgcn_perm(d1, d0, kLo), __builtin_amdgcn_perm(d3, d2, kLo),
                                 __builtin_amdgcn_perm(d5, d4, kLo), __builtin_amdgcn_perm(d7, d6, kLo));
            dst[c0 + 4] = make_uint4(__builtin_amdgcn_perm(d1, d0, kHi), __builtin_amdgcn_perm(d3, d2, kHi),
                                     __builtin_amdgcn_perm(d5, d4, kHi), __builtin_amdgcn_perm(d7, d6, kHi));
        };
        if (mover) {
            put(0, lo[0].x, lo[1].x, lo[2].x, lo[3].x, lo[4].x, lo[5].x, lo[6].x, lo[7].x);
            put(1, lo[0].y, lo[1].y, lo[2].y, lo[3].y, lo[4].y, lo[5].y, lo[6].y, lo[7].y);
            put(2, lo[0].z, lo[1].z, lo[2].z, lo[3].z, lo[4].z, lo[5].z, lo[6].z, lo[7].z);
            put(3, lo[0].w, lo[1].w, lo[2].w, lo[3].w, lo[4].w, lo[5].w, lo[6].w, lo[7].w);
            put(8, hi[0].x, hi[1].x, hi[2].x, hi[3].x, hi[4].x, hi[5].x, hi[6].x, hi[7].x);
            put(9, hi[0].y, hi[1].y, hi[2].y, hi[3].y, hi[4].y, hi[5].y, hi[6].y, hi[7].y);
            put(10, hi[0].z, hi[1].z, hi[2].z, hi[3].z, hi[4].z, hi[5].z, hi[6].z, hi[7].z);
            put(11, hi[0].w, hi[1].w, hi[2].w, hi[3].w, hi[4].w, hi[5].w, hi[6].w, hi[7].w);
        }
#pragma unroll
        for (int j = 0; j < GS; ++j) st[b][j * kAttendTileKeys + lane] = p.s[j];
#pragma unroll
        for (int i = 0; i < 32; ++i)
            if (i < n_q) wt[b][i * WROW + lane] = wreg[i];
    };
    // the tile in bt[b] / st[b]: acc_j += (w * scale_j) . codes_j over its 64 keys
    auto contract = [&](int b) __attribute__((always_inline)) {
#pragma unroll
        for (int kap = 0; kap < 4; ++kap) {                  // k-steps of 16 keys; this lane: keys 16 kap + 8 half + e
            const float4 w0 = *reinterpret_cast<const float4*>(&wt[b][col * WROW + 16 * kap + 8 * half]);
            const float4 w1 = *reinterpret_cast<const float4*>(&wt[b][col * WROW + 16 * kap + 8 * half + 4]);
            const float wv[8] = {w0.x, w0.y, w0.z, w0.w, w1.x, w1.y, w1.z, w1.w};
#pragma unroll
            for (int j = 0; j < GS; ++j) {
                const float4 s0 = *reinterpret_cast<const float4*>(&st[b][j * kAttendTileKeys + 16 * kap + 8 * half]);
                const float4 s1 = *reinterpret_cast<const float4*>(&st[b][j * kAttendTileKeys + 16 * kap + 8 * half + 4]);
                const float sc[8] = {s0.x, s0.y, s0.z, s0.w, s1.x, s1.y, s1.z, s1.w};
                // a = w * scale as fp16 hi + fp16 lo: hi is a truncated to fp16 (two values per conversion), a - hi is exact
                // in fp32, lo is that remainder truncated to fp16: about 21 bits of a
                half8 ahi, alo;
#pragma unroll
                for (int e = 0; e < 8; e += 2) {
                    const float a0 = wv[e] * sc[e], a1 = wv[e + 1] * sc[e + 1];
                    const auto h2 = __builtin_amdgcn_cvt_pkrtz(a0, a1);
                    const auto l2 = __builtin_amdgcn_cvt_pkrtz(a0 - (float)h2[0], a1 - (float)h2[1]);
                    ahi[e] = h2[0]; ahi[e + 1] = h2[1];
                    alo[e] = l2[0]; alo[e + 1] = l2[1];
                }
                const int ch = 32 * j + col;
                const half8 bf = __builtin_bit_cast(half8, bt[b][(2 * kap + half) * SLOTS + ch + ch / 16]);
                acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ahi, bf, acc[j], 0, 0, 0);
                acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(alo, bf, acc[j], 0, 0, 0);
            }
        }
    };

    // tiles of this stripe: stripe, stripe + stripes, ...; codes, scales and weights are prefetched two tiles ahead
    // in two named register sets (two tiles per trip)
    const long long m = stripe < n_tiles ? (n_tiles - 1 - stripe) / stripes + 1 : 0;
    Prefetch pa, pb;
    auto tile_of = [&](long long k) { return min(stripe + k * stripes, n_tiles - 1); };   // past the end: re-read the last
    if (m > 0) {
        fetch(pa, tile_of(0));
        fetch_w(tile_of(0));
        fetch(pb, tile_of(1));
        long long k = 0;
        for (; k + 1 < m; k += 2) {
            to_lds(0, pa);
            fetch_w(tile_of(k + 1));
            fetch(pa, tile_of(k + 2));
            __syncthreads();                     // one wavefront: orders the LDS writes before the reads
            contract(0);
            to_lds(0, pb);
            fetch_w(tile_of(k + 2));
            fetch(pb, tile_of(k + 3));
            __syncthreads();
            contract(0);
        }
        if (k < m) {
            to_lds(0, pa);
            __syncthreads();
            contract(0);
        }
    }
    // the sums of this workgroup: part[stripe][query][channel]; the accumulator of lane (col, half) holds rows
    // (queries) 8 r + 4 half + i in register 4 r + i, column = channel 32 j + col of the slab
    float* dst = part + (long long)stripe * 32 * D;
#pragma unroll
    for (int j = 0; j < GS; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int q = 8 * (v / 4) + 4 * half + (v % 4);
            dst[q * D + 32 * (slab * GS + j) + col] = acc[j][v];
        }
}

// first level of the fixed-order sum: part2[c][i][n] = sum over the stripes c, c + kAttendFan, ... of part[stripe][i][n]
constexpr int kAttendFan = 16;
template <int D>
__global__ void __launch_bounds__(D)
srft_attend_reduce_kernel(const float* __restrict__ part, int stripes, float* __restrict__ part2) {
    const int i = blockIdx.x, c = blockIdx.y, n = threadIdx.x;
    float sum = 0.0f;
    for (int sidx = c; sidx < stripes; sidx += kAttendFan) sum += part[((long long)sidx * 32 + i) * D + n];
    part2[((long long)c * 32 + i) * D + n] = sum;
}

// out[i][n] = sum_k rmat[k][n] * (sum over c of part2[c][i][k]);  rmat[k][n] = s_n Q[k][n] / max(lambda_k, 1e-6)
template <int D>
__global__ void __launch_bounds__(D)
srft_attend_finish_kernel(const float* __restrict__ part2, const float* __restrict__ rmat, float* __restrict__ out) {
    __shared__ float accs[D];
    const int i = blockIdx.x, n = threadIdx.x;
    float sum = 0.0f;
#pragma unroll
    for (int c = 0; c < kAttendFan; ++c) sum += part2[((long long)c * 32 + i) * D + n];
    accs[n] = sum;
    __syncthreads();
    float o = 0.0f;
#pragma unroll 8
    for (int k = 0; k < D; ++k) o = fmaf(rmat[k * D + n], accs[k], o);
    out[(long long)i * D + n] = o;
}

template <int D, int GS>
int launch(const srft_plan* p, const float* w, int n_q, const uint8_t* codes, const float* scales, long long n_keys,
           float* out, float* part, int stripes, hipStream_t st) {
    constexpr int SLABS = D / 32 / GS;
    hipLaunchKernelGGL((srft_attend_accumulate_kernel<D, GS>), dim3((unsigned)(stripes * SLABS)), dim3(64), 0, st, w, n_q,
                       (const uint2*)codes, scales, n_keys, p->gw, part, stripes);
    SRFT_HIP(hipGetLastError());
    float* part2 = part + (size_t)kMaxAttendStripes * 32 * D;
    hipLaunchKernelGGL(srft_attend_reduce_kernel<D>, dim3((unsigned)n_q, kAttendFan), dim3(D), 0, st, (const float*)part,
                       stripes, part2);
    SRFT_HIP(hipGetLastError());
    hipLaunchKernelGGL(srft_attend_finish_kernel<D>, dim3((unsigned)n_q), dim3(D), 0, st, (const float*)part2,
                       (const float*)p->rmat_f32, out);
    SRFT_HIP(hipGetLastError());
    return SRFT_OK;
}

}  // namespace

int srft_attend_stripes(const srft_plan* p, long long n_keys) {
    // workgroups per launch: four per compute unit and slab, at most one per tile, at most kMaxAttendStripes
    const long long n_tiles = (n_keys + kAttendTileKeys - 1) / kAttendTileKeys;
    long long s = p->max_wgs > 0 ? p->max_wgs : 4LL * p->compute_units;
    if (s > kMaxAttendStripes) s = kMaxAttendStripes;
    if (s > n_tiles) s = n_tiles;
    return (int)(s < 1 ? 1 : s);
}

int srft_launch_attend(const srft_plan* p, const float* w, int n_q, const uint8_t* codes, const float* scales,
                       long long n_keys, float* out, float* part, hipStream_t st) {
    const int stripes = srft_attend_stripes(p, n_keys);
    switch (p->d) {
        case 64: return launch<64, 2>(p, w, n_q, codes, scales, n_keys, out, part, stripes, st);
        case 128: return launch<128, 4>(p, w, n_q, codes, scales, n_keys, out, part, stripes, st);
        case 192: return launch<192, 3>(p, w, n_q, codes, scales, n_keys, out, part, stripes, st);
        case 256: return launch<256, 4>(p, w, n_q, codes, scales, n_keys, out, part, stripes, st);
        default: return SRFT_ERR_BAD_D;
    }
}
