// plan.hip -- host side of a plan: the sign diagonal, the matrices W and R of the write and the read path, their
// fp16 hi + lo split in MFMA operand order (plain and folded forms), the choice of kernel instances, and the
// persistent grid sizes.
#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <new>

#include "common.h"

namespace {

thread_local int g_last_hip_error = 0;

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

// Table of the twice-folded write path (d = 256, g = 32): see quantize_fold4_tiles.h for what the kernel does with it.
// Wavefront w = 0 .. 3 is (cosine, classes 0|2), (cosine, 1|3), (sine, 0|2), (sine, 1|3).  Its two 32 x 64 slabs a
// and c hold, for k1 = 0 .. 31 and the inputs n = 4 n1 + class, the entries Q[k1][n] s_n (cosine) or Q[128 + k1][n] s_n
// (sine), the c slab of the odd-class wavefronts negated.  Row k1 = 0 of the sine slabs carries the row k = 32 of the
// transform instead, (-1)^n1 sqrt(2/d) s_n per class, times 1/sqrt 2 in the odd classes (not negated).
// lambda is applied after the contraction: rho_d / rho_m are +-lambda of the packed index a lane's value lands on,
// times the 2^-e of the fp16 scaling, times sqrt 2 for the two values of the rows k1 = 0 that are bins 64.
void build_fold4_table(const std::vector<int8_t>& signs, const std::vector<double>& lam, std::vector<uint32_t>& out) {
    const int d = 256, T = 4;
    std::vector<double> rows((size_t)4 * 2 * 32 * 64);
    for (int w = 0; w < 4; ++w)
        for (int ac = 0; ac < 2; ++ac) {
            const bool sine = w >= 2, oddw = w & 1;
            const int cls = (oddw ? 1 : 0) + 2 * ac;
            for (int k1 = 0; k1 < 32; ++k1)
                for (int n1 = 0; n1 < 64; ++n1) {
                    const int n = 4 * n1 + cls;
                    double v;
                    if (sine && k1 == 0) {
                        v = ((n1 & 1) ? -1.0 : 1.0) * std::sqrt(2.0 / d) * (oddw ? std::sqrt(0.5) : 1.0);
                    } else {
                        v = q_entry(d, sine ? d / 2 + k1 : k1, n);
                        if (oddw && ac == 1) v = -v;
                    }
                    rows[(((size_t)w * 2 + ac) * 32 + k1) * 64 + n1] = v * (double)signs[n];
                }
        }
    std::vector<uint16_t> hi, lo;
    const double u = std::ldexp(1.0, -split_hi_lo(rows, hi, lo));
    out.assign((size_t)srft_fold4_table_units() * 4, 0);
    uint16_t* frag = reinterpret_cast<uint16_t*>(out.data());
    for (int w = 0; w < 4; ++w)
        for (int ac = 0; ac < 2; ++ac)
            for (int t = 0; t < T; ++t)
                for (int l = 0; l < 64; ++l) {
                    const int k1 = slab_output_of_row(l % 32), kh = l / 32;
                    for (int e = 0; e < 8; ++e) {
                        const size_t src = (((size_t)w * 2 + ac) * 32 + k1) * 64 + (16 * t + 8 * kh + e);
                        const size_t dst = ((((size_t)(w * 2 + ac) * T + t) * 2) * 64);
                        frag[((dst + 0) + l) * 8 + e] = hi[src];
                        frag[((dst + 64) + l) * 8 + e] = lo[src];
                    }
                }
    float* rho = reinterpret_cast<float*>(out.data()) + (size_t)4 * 2 * T * 2 * 64 * 4;
    const double r2 = std::sqrt(2.0);
    for (int k1 = 0; k1 < 32; ++k1) {
        // direct runs: wave 0 -> k1, wave 1 -> 192 + k1, wave 2 -> 128 + k1, wave 3 -> 64 + k1
        rho[0 * 64 + k1] = (float)(u * lam[k1]);
        rho[1 * 64 + k1] = (float)(-u * lam[192 + k1] * (k1 == 0 ? r2 : 1.0));
        rho[2 * 64 + k1] = (float)(u * lam[128 + k1]);            // k1 = 0 is replaced by Nyquist in the kernel
        rho[3 * 64 + k1] = (float)(u * lam[64 + k1] * (k1 == 0 ? r2 : 1.0));
        // mirror runs: wave 0 -> 128 - k1, wave 1 -> 192 - k1, wave 2 -> 256 - k1, wave 3 -> 64 - k1 (none at k1 = 0)
        rho[0 * 64 + 32 + k1] = k1 ? (float)(u * lam[128 - k1]) : 0.0f;
        rho[1 * 64 + 32 + k1] = k1 ? (float)(-u * lam[192 - k1]) : 0.0f;
        rho[2 * 64 + 32 + k1] = k1 ? (float)(-u * lam[256 - k1]) : 0.0f;
        rho[3 * 64 + 32 + k1] = k1 ? (float)(-u * lam[64 - k1]) : 0.0f;
    }
    float* misc = rho + 4 * 64;          // per wave: beta1, beta2 (bottom of the mirror group), Nyquist scale, tau
    const float m0[4] = {(float)(u * lam[96]), (float)(-u * lam[96]), 0.0f, 1.0f};          // z96 = A0 - Am
    const float m1[4] = {(float)(-u * lam[160]), (float)(-u * lam[160]), 0.0f, -1.0f};      // z160 = -(A2 + Ap)
    const float m2[4] = {(float)(u * lam[224]), (float)(-u * lam[224]), (float)(u * lam[128]), 1.0f};   // z224 = A2 - Ap
    const float m3[4] = {(float)(u * lam[32]), (float)(u * lam[32]), 0.0f, 1.0f};           // z32 = A0 + Am
    std::memcpy(misc + 0, m0, 16);
    std::memcpy(misc + 4, m1, 16);
    std::memcpy(misc + 8, m2, 16);
    std::memcpy(misc + 12, m3, 16);
}

// Table of the twice-folded read path (d = 128 or 256, g >= 32): see dequantize_fold4_tiles.h for what the kernel
// does with it.  With NB = d/128 blocks of 32 values of m per class, wavefront w < NB holds cosine rows (packed
// indices p < h), w >= NB sine rows (p > h; p = h, Nyquist, has a zero column here and enters the cosine side as an
// addend), each for m = 32 (w mod NB) .. + 31; class 0 are the even, class 1 the odd p of a group; the odd class of
// the sine wavefronts is negated, and its row m = 0 in the first sine wavefront carries row m = d/4 instead.  Entries
// are Q[p][m] / max(lambda_p, 1e-6), without the sign diagonal, which the kernel applies through the masks.
// Returns the exponent e of the fp16 scaling.
int build_rfold4_table(int d, const std::vector<int8_t>& signs, const std::vector<double>& lam, int bits,
                       std::vector<uint32_t>& out) {
    const int h = d / 2, NB = d / 128, NW = 2 * NB, GH = d / 64;
    static const int off4[8] = {0, 4, 2, 6, 8, 12, 10, 14}, off8[8] = {0, 2, 4, 6, 8, 10, 12, 14};
    const int* off = bits == 8 ? off8 : off4;
    auto entry = [&](int p, int m) { return q_entry(d, p, m) / std::fmax(lam[p], 1e-6); };
    // [w][class][m row 0..31][group 0..GH-1][16 codes], then the h/2 coefficients of row m = d/4 (even p < h)
    const size_t coef0 = (size_t)NW * 2 * 32 * GH * 16;
    std::vector<double> rows(coef0 + h / 2);
    for (int w = 0; w < NW; ++w) {
        const int sine = w / NB, blk = w % NB;
        for (int c = 0; c < 2; ++c)
            for (int r = 0; r < 32; ++r)
                for (int jj = 0; jj < GH; ++jj)
                    for (int i = 0; i < 16; ++i) {
                        const int p = 32 * (GH * sine + jj) + 2 * i + c, m = 32 * blk + r;
                        double v = (sine && p == h) ? 0.0 : entry(p, (w == NB && c == 1 && m == 0) ? d / 4 : m);
                        if (sine && c == 1) v = -v;
                        rows[((((size_t)w * 2 + c) * 32 + r) * GH + jj) * 16 + i] = v;
                    }
    }
    for (int i = 0; i < h / 2; ++i) rows[coef0 + i] = entry(2 * i, d / 4);
    std::vector<uint16_t> hi, lo;
    const int e = split_hi_lo(rows, hi, lo);
    out.assign((size_t)srft_rfold4_table_units(d) * 4, 0);
    uint16_t* frag = reinterpret_cast<uint16_t*>(out.data());
    for (int w = 0; w < NW; ++w)
        for (int c = 0; c < 2; ++c)
            for (int jj = 0; jj < GH; ++jj)
                for (int l = 0; l < 64; ++l) {
                    const int r = slab_output_of_row(l % 32), kh = l / 32;
                    for (int el = 0; el < 8; ++el) {
                        const int i = (16 * kh + off[el]) / 2;          // even (or odd) code 2 i (+ 1) of the group
                        const size_t src = ((((size_t)w * 2 + c) * 32 + r) * GH + jj) * 16 + i;
                        const size_t dst = ((((size_t)(w * 2 + c) * GH + jj) * 2) * 64);
                        frag[((dst + 0) + l) * 8 + el] = hi[src];
                        frag[((dst + 64) + l) * 8 + el] = lo[src];
                    }
                }
    const size_t frag_units = (size_t)NW * 2 * GH * 2 * 64, half_units = (size_t)NW * 2 * 6;
    float* consts = reinterpret_cast<float*>(out.data() + (frag_units + half_units) * 4);
    for (int w = 0; w < NW; ++w) {
        const int sine = w / NB, blk = w % NB;
        for (int kh = 0; kh < 2; ++kh) {         // what the 32 lanes of a half share: 16 mask dwords, 8 coefficients
            const int m0 = 32 * blk + 16 * kh;
            const int n_asc = (sine ? h : 0) + m0, n_des = (sine ? h : d) - m0 - 16;
            uint32_t* mk = out.data() + (frag_units + (size_t)(w * 2 + kh) * 6) * 4;
            for (int i = 0; i < 8; ++i) {
                mk[i] = (signs[n_asc + 2 * i] < 0 ? 0x8000u : 0u) | (signs[n_asc + 2 * i + 1] < 0 ? 0x80000000u : 0u);
                // the sine side leaves the descending run negated: its masks carry the opposite sign
                const bool lo_neg = (signs[n_des + 2 * i] < 0) != (sine != 0), hi_neg = (signs[n_des + 2 * i + 1] < 0) != (sine != 0);
                mk[8 + i] = (lo_neg ? 0x8000u : 0u) | (hi_neg ? 0x80000000u : 0u);
            }
            // row m = d/4 over the even codes of cosine group w that a lane of this half reads as a B fragment
            float* coef = reinterpret_cast<float*>(mk + 16);
            for (int el = 0; el < 8; ++el) coef[el] = (float)std::ldexp(entry(32 * w + 16 * kh + off[el], d / 4), e);
        }
        consts[w * 4] = sine ? 0.0f : (float)std::ldexp(1.0 / (std::sqrt((double)d) * std::fmax(lam[h], 1e-6)), e);
    }
    return e;
}

// resident workgroups per compute unit of a kernel with `threads` threads per workgroup
int resident_blocks(const void* kernel, int threads, int* blocks) {
    *blocks = 0;
    SRFT_HIP(hipOccupancyMaxActiveBlocksPerMultiprocessor(blocks, kernel, threads, 0));
    if (*blocks < 1) *blocks = 1;
    return SRFT_OK;
}

int occupancy_grids(srft_plan* p, int cus) {
    int threads = 0, blocks = 0;
    const quantize_kernel_t qk = srft_plan_quantize_kernel(p, kOutCodes, &threads);
    int rc = resident_blocks((const void*)qk, threads, &blocks);
    if (rc != SRFT_OK) return rc;
    p->grid_q = cus * blocks;
    const dequantize_kernel_t dk = srft_plan_dequantize_kernel(p, &threads);
    rc = resident_blocks((const void*)dk, threads, &blocks);
    if (rc != SRFT_OK) return rc;
    p->grid_dq = cus * blocks;
    rc = srft_scores_occupancy(p->d, false, &blocks);
    if (rc != SRFT_OK) return rc;
    p->grid_scores = cus * (blocks > 0 ? blocks : 1);
    rc = srft_scores_occupancy(p->d, true, &blocks);
    if (rc != SRFT_OK) return rc;
    p->grid_scores16 = cus * (blocks > 0 ? blocks : 1);
    return SRFT_OK;
}

}  // namespace

int srft_hip_fail(hipError_t e) {
    g_last_hip_error = (int)e;
    return SRFT_ERR_HIP;
}

quantize_kernel_t srft_plan_quantize_kernel(const srft_plan* p, int out, int* threads) {
    if (out == kOutQFrag32 || out == kOutQFrag16) {      // the scores set-up always runs one slab per wavefront
        *threads = 2 * p->d;
        return srft_pick_quantize_aux(p->d, 1, out);
    }
    if (out == kOutAmax && p->fold_q) {                  // the statistic does not depend on the groups: folded wherever the table exists
        *threads = p->d;
        return srft_pick_quantize_fold_amax(p->d);
    }
    if (out != kOutCodes) {
        *threads = 2 * p->d / p->slabs_q;
        return srft_pick_quantize_aux(p->d, p->slabs_q, out);
    }
    if (p->fold4_q) {
        *threads = 256;
        return srft_pick_quantize_fold4(p->bits);
    }
    if (p->fold_q) {
        *threads = p->d;
        return srft_pick_quantize_fold(p->d, p->bits, p->gm == kGroupWide);
    }
    *threads = 2 * p->d / p->slabs_q;
    return p->bits == 8 ? srft_pick_quantize_plain_b8(p->d, p->slabs_q, p->gm)
                        : srft_pick_quantize_plain_b4(p->d, p->slabs_q, p->gm);
}

dequantize_kernel_t srft_plan_dequantize_kernel(const srft_plan* p, int* threads) {
    if (p->fold4_dq) {
        *threads = p->d;
        return srft_pick_dequantize_fold4(p->d, p->bits);
    }
    *threads = 2 * p->d / p->slabs_dq;
    return p->bits == 8 ? srft_pick_dequantize_b8(p->d, p->slabs_dq, p->gm, p->fold_dq)
                        : srft_pick_dequantize_b4(p->d, p->slabs_dq, p->gm, p->fold_dq);
}

bool srft_plans_compatible(const srft_plan* a, const srft_plan* b) {
    return a->d == b->d && a->g == b->g && a->bits == b->bits && a->transform == b->transform &&
           a->device == b->device && a->fold_q == b->fold_q && a->fold4_q == b->fold4_q && a->fold_dq == b->fold_dq &&
           a->fold4_dq == b->fold4_dq &&
           a->slabs_q == b->slabs_q && a->slabs_dq == b->slabs_dq;
}

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

    // Slabs of the matrix per wavefront: two where the table says so (and the number of groups is even).
    p->slabs_q = (d == 64) ? 2 : 1;
    p->slabs_dq = (d == 256 || d == 64) ? 2 : 1;
    // Folded read path where it applies and pays (d = 192; g >= 32); d = 128 and 256 have the twice-folded form below.
    p->fold_dq = (d % 64 == 0) && d >= 128 && d != 128 && d != 256 && p->gm != kGroup16 &&    // at d = 64 it gains nothing
                 transform == SRFT_TRANSFORM_DFT;                      // (the symmetries are the DFT's)
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
    // Folded write path where it applies (d a multiple of 128, g >= 32).
    p->fold_q = (d % 128 == 0) && p->gm != kGroup16 && transform == SRFT_TRANSFORM_DFT;
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
    // Twice-folded write path at d = 256 with the deployed group size; it replaces the once-folded form there.
    p->fold4_q = (d == 256) && p->gm == kGroup32 && transform == SRFT_TRANSFORM_DFT;
    std::vector<uint32_t> wfold4;
    if (p->fold4_q) build_fold4_table(p->signs, lam, wfold4);
    // Twice-folded read path at d = 128 and 256 (any g >= 32); it replaces the once-folded form there.
    p->fold4_dq = (d == 128 || d == 256) && p->gm != kGroup16 && transform == SRFT_TRANSFORM_DFT;
    std::vector<uint32_t> rfold4;
    if (p->fold4_dq) p->unscale_r4 = (float)std::ldexp(1.0, -build_rfold4_table(d, p->signs, lam, bits, rfold4));
    // Butterfly form of the write path (comparison kernel): per packed index lambda times the packing constant of
    // Eq. 2 -- 1/sqrt d for DC and Nyquist, sqrt(2/d) elsewhere, halved where the unpack leaves a factor 2 (every
    // bin except 0, d/4 and d/2) -- then the sign diagonal as sign-bit masks of the packed fp16 pairs.
    std::vector<float> bfly;
    if ((d == 128 || d == 256) && p->gm == kGroup32 && bits == 4 && transform == SRFT_TRANSFORM_DFT) {
        const int h = d / 2;
        bfly.resize(d + h);
        for (int k = 0; k < d; ++k) {
            const int bin = k < h ? k : k - h;
            double c = (k == 0 || k == h) ? 1.0 / std::sqrt((double)d) : std::sqrt(2.0 / d);
            if (bin != 0 && bin != d / 4) c *= 0.5;
            bfly[k] = (float)(lam[k] * c);
        }
        for (int j = 0; j < h; ++j) {
            const uint32_t m = (p->signs[2 * j] < 0 ? 0x8000u : 0u) | (p->signs[2 * j + 1] < 0 ? 0x80000000u : 0u);
            std::memcpy(&bfly[d + j], &m, 4);
        }
    }
    hipError_t e = hipGetDevice(&p->device);
    int cus = 0;
    if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, p->device);
    if (e == hipSuccess) e = hipMalloc((void**)&p->wfrag, wf.size() * 2);
    if (e == hipSuccess) e = hipMalloc((void**)&p->rfrag, rf.size() * 2);
    if (e == hipSuccess) e = hipMemcpy(p->wfrag, wf.data(), wf.size() * 2, hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy(p->rfrag, rf.data(), rf.size() * 2, hipMemcpyHostToDevice);
    std::vector<float> rmat((size_t)d * d);
    for (int n = 0; n < d; ++n)
        for (int k = 0; k < d; ++k) rmat[(size_t)k * d + n] = (float)R[(size_t)n * d + k];
    if (e == hipSuccess) e = hipMalloc((void**)&p->rmat_f32, rmat.size() * sizeof(float));
    if (e == hipSuccess) e = hipMemcpy(p->rmat_f32, rmat.data(), rmat.size() * sizeof(float), hipMemcpyHostToDevice);
    p->compute_units = cus;
    std::vector<float> il2(d);
    for (int k = 0; k < d; ++k) il2[k] = (float)(1.0 / (lam[k] * std::fmax(lam[k], 1e-6)));
    if (e == hipSuccess) e = hipMalloc((void**)&p->inv_lam2, d * sizeof(float));
    if (e == hipSuccess) e = hipMemcpy(p->inv_lam2, il2.data(), d * sizeof(float), hipMemcpyHostToDevice);
    if (e == hipSuccess && p->fold_q) e = hipMalloc((void**)&p->wfold, wfold.size() * 2);
    if (e == hipSuccess && p->fold_q) e = hipMemcpy(p->wfold, wfold.data(), wfold.size() * 2, hipMemcpyHostToDevice);
    if (e == hipSuccess && !bfly.empty()) e = hipMalloc((void**)&p->bfly, bfly.size() * 4);
    if (e == hipSuccess && !bfly.empty()) e = hipMemcpy(p->bfly, bfly.data(), bfly.size() * 4, hipMemcpyHostToDevice);
    if (e == hipSuccess && p->fold4_q) e = hipMalloc((void**)&p->wfold4, wfold4.size() * 4);
    if (e == hipSuccess && p->fold4_q) e = hipMemcpy(p->wfold4, wfold4.data(), wfold4.size() * 4, hipMemcpyHostToDevice);
    if (e == hipSuccess && p->fold4_dq) e = hipMalloc((void**)&p->rfold4, rfold4.size() * 4);
    if (e == hipSuccess && p->fold4_dq) e = hipMemcpy(p->rfold4, rfold4.data(), rfold4.size() * 4, hipMemcpyHostToDevice);
    if (e == hipSuccess && p->fold_dq) e = hipMalloc((void**)&p->rfold, rfold.size() * 2);
    if (e == hipSuccess && p->fold_dq) e = hipMemcpy(p->rfold, rfold.data(), rfold.size() * 2, hipMemcpyHostToDevice);
    int rc = (e == hipSuccess) ? occupancy_grids(p, cus) : srft_hip_fail(e);
    if (rc == SRFT_OK) rc = srft_scores_scratch_prepare(p->device);
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
    if (plan->rmat_f32) {
        const hipError_t e8 = hipFree(plan->rmat_f32);
        if (e3 == hipSuccess) e3 = e8;
    }
    if (plan->bfly) {
        const hipError_t e7 = hipFree(plan->bfly);
        if (e3 == hipSuccess) e3 = e7;
    }
    if (plan->wfold4) {
        const hipError_t e6 = hipFree(plan->wfold4);
        if (e3 == hipSuccess) e3 = e6;
    }
    if (plan->rfold4) {
        const hipError_t e9 = hipFree(plan->rfold4);
        if (e3 == hipSuccess) e3 = e9;
    }
    if (plan->inv_lam2) {
        const hipError_t e5 = hipFree(plan->inv_lam2);
        if (e3 == hipSuccess) e3 = e5;
    }
    delete plan;
    if (e1 != hipSuccess) return srft_hip_fail(e1);
    if (e2 != hipSuccess) return srft_hip_fail(e2);
    if (e3 != hipSuccess) return srft_hip_fail(e3);
    return SRFT_OK;
}

int srft_plan_d(const srft_plan_t* plan) { return plan ? plan->d : SRFT_ERR_NULL; }
int srft_plan_group_size(const srft_plan_t* plan) { return plan ? plan->g : SRFT_ERR_NULL; }
int srft_plan_groups(const srft_plan_t* plan) { return plan ? plan->d / plan->g : SRFT_ERR_NULL; }
int srft_plan_code_bytes(const srft_plan_t* plan) { return plan ? plan->d * plan->bits / 8 : SRFT_ERR_NULL; }
int srft_plan_bits(const srft_plan_t* plan) { return plan ? plan->bits : SRFT_ERR_NULL; }
int srft_plan_form(const srft_plan_t* plan, int path) {
    if (!plan) return SRFT_ERR_NULL;
    if (path == 0) return plan->fold4_q ? 2 : plan->fold_q ? 1 : 0;
    if (path == 1) return plan->fold4_dq ? 2 : plan->fold_dq ? 1 : 0;
    return SRFT_ERR_BAD_N;
}

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

int srft_last_hip_error(void) { return g_last_hip_error; }

}  // extern "C"
