// common.h -- shared declarations of the fused SRFT int4 KV-cache quantizer / dequantizer for MI355X (gfx950).
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
// Folded forms (d = 128 and 256 on the write path, 128 / 192 / 256 on the read path): symmetries of Q let
// outputs share half-length (folded once) or quarter-length (folded twice) partial sums, which halves or
// quarters the matrix work; they are described at srft_quantize_fold_tiles, in quantize_fold4_tiles.h, at
// the FOLD parameter of srft_dequantize_tiles and in dequantize_fold4_tiles.h.
//
// Around the two paths: the same kernels serving several plans in one launch (a segment table passed as a
// kernel argument), the per-channel abs-max statistic lambda is calibrated from, an 8-bit code width, the
// Walsh-Hadamard matrix in place of the DFT (the comparator of Sec. 3.1), scores of queries against the stored
// record without reconstructing the keys, and a host-side cache manager (int4 store, fp16 residual window,
// dequantized view) built on the batched launches.
//
// The kernels run at the socket's power limit with a throttled clock, so what shortens them is work per vector
// (matrix instructions, vector instructions, LDS traffic), not more parallelism: see the folded forms.
//
// Source layout: the kernel templates live in quantize_tiles.h (write path, plain form), quantize_fold_tiles.h and
// quantize_fold4_tiles.h (write path, folded forms), dequantize_tiles.h and dequantize_fold4_tiles.h (read path),
// kernels/scores.hip and kernels/attend.hip; every file under kernels/
// instantiates one family of them and exports a function that picks the instance for a plan; plan.hip builds
// the constant tables, api.hip holds the C entry points, cache.hip the cache manager.
#ifndef SRFT_COMMON_H
#define SRFT_COMMON_H

#include <hip/hip_runtime.h>

#include <cstdint>
#include <vector>

#include "srft_kv.h"

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kTileVecs = 32;          // vectors per tile = N of the 32x32x16 MFMA
constexpr int kMaxScoreWorkgroups = 4096;   // scores kernel: largest grid (each workgroup owns 256 bytes of workspace)
constexpr int kMaxD = 256;
constexpr int kMaxAttendStripes = 2048;      // value-side kernel: most workgroups per channel slab (each owns 32 x d floats of workspace)
constexpr int kAttendFan = 64;                // value-side kernel: first-level sums the partial results are added into
constexpr int kRowMaxCopies = 64;            // copies of the per-query score maxima (a cache line each), so that the scan's atomics spread
constexpr float kMinScale = 7.888609052210118e-31f;   // 2^-100: below this a group is stored as zero
// The kernels index tiles of 32 vectors with 32-bit integers and look a few grid strides ahead.
constexpr int64_t kMaxVectors = (int64_t)1 << 33;

// group mode of a plan.  kGroup32: one scale per slab (g = 32, the deployed format).  kGroup16: one scale per
// lane (g = 16).  kGroupWide: g = 32 * gw with gw >= 2 slabs per group, up to the per-token case g = d.
enum { kGroup16 = 0, kGroup32 = 1, kGroupWide = 2 };
// what the write-path kernel produces (see quantize_tiles.h)
enum { kOutCodes = 0, kOutRaw = 1, kOutAmax = 2, kOutQFrag32 = 3, kOutQFrag16 = 4 };

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

typedef void (*quantize_kernel_t)(const uint4*, const uint4*, long long, uint2*, float*, float4*, float, float, int);
typedef void (*dequantize_kernel_t)(const uint4*, const uint2*, const float*, long long, uint4*, float, int);
typedef void (*batched_kernel_t)(const srft_batch_args, int);

struct srft_plan {
    int d = 0, g = 0, bits = 4, transform = 0, device = 0;
    uint64_t seed = 0;
    std::vector<int8_t> signs;
    uint4* wfrag = nullptr;     // write-path matrix fragments (device)
    uint4* rfrag = nullptr;     // read-path matrix fragments (device)
    uint4* rfold = nullptr;     // read-path fragments of the folded form (device), when fold_dq
    uint4* wfold = nullptr;     // write-path fragments of the folded form (device), when fold_q
    uint4* wfold4 = nullptr;    // write-path table of the twice-folded form (device), when fold4_q
    uint4* rfold4 = nullptr;    // read-path table of the twice-folded form (device), when fold4_dq
    float* rmat_f32 = nullptr;  // R^T in fp32, [k][n] = s_n Q[k][n] / max(lambda_k, 1e-6) (device): the one inverse transform per
                                // query of srft_kv_attend
    int compute_units = 0;
    float* bfly = nullptr;      // table of the butterfly form of the write path (device), d = 128 or 256 / g = 32 / 4-bit only
    float* inv_lam2 = nullptr;  // 1 / (lambda * max(lambda, 1e-6)) per channel (device): scores in the rotated domain
    int grid_scores = 0;        // persistent grid of the scores kernel (32 rows of queries)
    int grid_scores16 = 0;      // the same with 16 rows
    bool fold_dq = false;       // read path contracts even and odd codes separately (half the matrix work)
    bool fold_q = false;        // write path contracts even and odd inputs separately (half the matrix work)
    bool fold4_q = false;       // write path contracts the inputs in four classes n mod 4 (a quarter of the work)
    bool fold4_dq = false;      // read path contracts (cosine | sine) x (even | odd) codes apart (a quarter of the work)
    float unscale_w = 1.0f;     // 2^-e of the write matrix
    float unscale_r = 1.0f;
    float unscale_r4 = 1.0f;    // 2^-e of the twice-folded read table
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

// ---- kernel instances, one function per translation unit under kernels/ (nullptr: no such instance) ----
// write path, plain form, codes out: d, slabs per wavefront (1 or 2), group mode; 4- and 8-bit codes
quantize_kernel_t srft_pick_quantize_plain_b4(int d, int slabs, int gm);
quantize_kernel_t srft_pick_quantize_plain_b8(int d, int slabs, int gm);
batched_kernel_t srft_pick_quantize_plain_batched_b4(int d, int slabs, int gm);
batched_kernel_t srft_pick_quantize_plain_batched_b8(int d, int slabs, int gm);
// write path, plain form, other outputs (kOutRaw, kOutAmax with `slabs`; kOutQFrag32 / kOutQFrag16 with one slab)
quantize_kernel_t srft_pick_quantize_aux(int d, int slabs, int out);
// write path, folded form (d = 128, 256)
quantize_kernel_t srft_pick_quantize_fold(int d, int bits, bool wide);
quantize_kernel_t srft_pick_quantize_fold_amax(int d);      // the abs-max statistic through the once-folded contraction
batched_kernel_t srft_pick_quantize_fold_batched(int d, int bits, bool wide);
// write path, folded twice (d = 256, g = 32); the size of its table in 16-byte units
quantize_kernel_t srft_pick_quantize_fold4(int bits);
batched_kernel_t srft_pick_quantize_fold4_batched(int bits);
int srft_fold4_table_units(void);
// read path
dequantize_kernel_t srft_pick_dequantize_b4(int d, int slabs, int gm, bool fold);
dequantize_kernel_t srft_pick_dequantize_b8(int d, int slabs, int gm, bool fold);
batched_kernel_t srft_pick_dequantize_batched_b4(int d, int slabs, int gm, bool fold);
batched_kernel_t srft_pick_dequantize_batched_b8(int d, int slabs, int gm, bool fold);
// read path, folded twice (d = 128 and 256, g >= 32); the size of its table in 16-byte units
dequantize_kernel_t srft_pick_dequantize_fold4(int d, int bits);
batched_kernel_t srft_pick_dequantize_fold4_batched(int d, int bits);
int srft_rfold4_table_units(int d);
// write path with the transform as FFT butterflies on the vector ALU (d = 128 or 256, g = 32, 4-bit; the comparison form)
int srft_launch_quantize_butterfly(int d, const float* table_dev, const void* x, long long n_vec, uint8_t* codes,
                                   float* scales, int max_workgroups, hipStream_t st);
// scores in the rotated domain: launch of the scan (kernels/scores.hip) and its resident workgroups per unit
// row_max: nullptr, or kRowMaxCopies x 32 cleared words: copy (workgroup mod kRowMaxCopies) receives, per query, the
// ordered code (srft_ordered_code) of the maximum of sign * score over that workgroup's keys
int srft_launch_scores(const srft_plan* p, uint4* qfrag, float* dump, int n_q, const uint8_t* codes,
                       const float* scales, long long n_keys, float* out, unsigned int* row_max, float sign,
                       hipStream_t st);
int srft_scores_occupancy(int d, bool r16, int* blocks_per_cu);

// weighted sums of the stored values in the rotated domain (kernels/attend.hip): workgroups per channel slab for
// n_q queries over n_keys values, and the three launches (partial sums per workgroup into `part`, their fixed-order
// reduction, the inverse transform).  row_max: nullptr (w holds the weights), or the kRowMaxCopies x 32 ordered codes of
// the maxima of sign(softmax_scale) * w over the keys, as srft_launch_scores leaves them: w then holds raw scores, the
// weights exp(softmax_scale * w - maximum) are formed as the scores are loaded, their sums are carried along and the
// result is divided by them (a row softmax without a pass of its own).
int srft_attend_stripes(const srft_plan* p, int n_q, long long n_keys);
size_t srft_attend_workspace_floats(int d);
int srft_launch_attend(const srft_plan* p, const float* w, int n_q, const uint8_t* codes, const float* scales,
                       long long n_keys, float* out, float* part, const unsigned int* row_max, float softmax_scale,
                       hipStream_t st);

// ---- host side (plan.hip, api.hip) ----
int srft_hip_fail(hipError_t e);         // records the error for srft_last_hip_error, returns SRFT_ERR_HIP
#define SRFT_HIP(call)                                   \
    do {                                                 \
        hipError_t e_ = (call);                          \
        if (e_ != hipSuccess) return srft_hip_fail(e_);  \
    } while (0)

// the kernels a plan launches, and their block sizes
quantize_kernel_t srft_plan_quantize_kernel(const srft_plan* p, int out, int* threads);
dequantize_kernel_t srft_plan_dequantize_kernel(const srft_plan* p, int* threads);
// the table and the matrix scaling the read-path kernel of a plan takes
inline const uint4* srft_plan_read_table(const srft_plan* p) { return p->fold4_dq ? p->rfold4 : p->fold_dq ? p->rfold : p->rfrag; }
inline float srft_plan_read_unscale(const srft_plan* p) { return p->fold4_dq ? p->unscale_r4 : p->unscale_r; }
// batched launches over plans that share shape and kernel choice (api.hip)
int srft_run_batched(const srft_plan_t* const* plans, const void* const* in0, const void* const* in1,
                     void* const* out0, void* const* out1, const int64_t* n_vec, int count, bool write_path,
                     hipStream_t st);
// true when two plans can share one batched launch or one cache (shape, code width, transform, device, kernel forms)
bool srft_plans_compatible(const srft_plan* a, const srft_plan* b);

// resolves, once per device, the device address of the static workspace of srft_kv_scores_static (api.hip);
// called with `device` current when a plan is created
int srft_scores_scratch_prepare(int device);

inline bool srft_aligned(const void* p, size_t a) { return ((uintptr_t)p & (a - 1)) == 0; }

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
        default:  return nullptr;                         \
    }

#endif  // SRFT_COMMON_H
