// device_util.h -- device-side helpers shared by the kernel templates.
#ifndef SRFT_DEVICE_UTIL_H
#define SRFT_DEVICE_UTIL_H

#include <type_traits>

#include "common.h"

// Streaming (non-temporal) accesses for data touched once.  Measured: non-temporal stores of full rows help both
// paths (+2.5 to +3 %); non-temporal loads help where one load instruction covers whole cache lines (the read
// path's code units) and cost up to 20 % where several loads of a lane share a line (the folded write paths, whose
// lanes read 32 or 64 contiguous bytes), so those loads stay plain.
__device__ __forceinline__ void stream_store(uint4* p, uint4 v) {
    __builtin_nontemporal_store(__builtin_bit_cast(u32x4, v), reinterpret_cast<u32x4*>(p));
}
__device__ __forceinline__ uint4 stream_load(const uint4* p) {
    return __builtin_bit_cast(uint4, __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p)));
}
__device__ __forceinline__ uint2 stream_load(const uint2* p) {
    return __builtin_bit_cast(uint2, __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(p)));
}

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

__device__ __forceinline__ int srft_segment_of_block(const srft_batch_args& a, int block) {
    int i = 0;
    while (i + 1 < a.count && a.first_block[i + 1] <= block) ++i;     // uniform; count is small
    return i;
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

// Running maximum of non-negative floats kept as their bit patterns (they order alike).  All workgroups of a launch
// update the same few cache lines at about the same time, and atomics to one line are served one after the other:
// the current value is read first (from L2, past the caches of this compute unit), and the atomic is only sent when
// it would raise it -- of N similar contributions about ln N do.
__device__ __forceinline__ void atomic_max_nonneg(unsigned int* p, float v) {
    const unsigned int bits = __float_as_uint(v);
    if (bits > __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) atomicMax(p, bits);
}

// An unsigned code of a float that orders like the float (negative floats: all bits flipped; others: sign bit set),
// so that an unsigned atomic maximum is a float maximum.  The code 0 lies below every float's: cleared memory is "no
// value yet".
__device__ __forceinline__ unsigned int srft_ordered_code(float f) {
    const unsigned int b = __float_as_uint(f);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}
__device__ __forceinline__ float srft_ordered_value(unsigned int c) {
    return __uint_as_float((c & 0x80000000u) ? (c & 0x7FFFFFFFu) : ~c);
}

// Which tiles a workgroup of a per-plan launch walks: first tile, stride, and the end (exclusive) of its range.
// SRFT_XCD_MAP = 0: tile = blockIdx + k gridDim over all tiles.  SRFT_XCD_MAP = 1: workgroups are dealt to the 8
// accelerator dies round-robin (die = blockIdx mod 8), and each die gets one contiguous eighth of the tiles, which
// its workgroups walk with stride gridDim / 8 (grids that are not a multiple of 8 fall back to the plain map).
#ifndef SRFT_XCD_MAP
#define SRFT_XCD_MAP 0
#endif
__device__ __forceinline__ bool srft_tile_range(long long n_vec, int& t0, int& stride, int& t_end) {
    const int n_tiles = (int)((n_vec + kTileVecs - 1) / kTileVecs);
    t0 = blockIdx.x;
    stride = gridDim.x;
    t_end = n_tiles;
#if SRFT_XCD_MAP
    if ((gridDim.x & 7) == 0 && n_tiles >= (int)gridDim.x) {
        const int per_die = (n_tiles + 7) >> 3, die = blockIdx.x & 7;
        stride = gridDim.x >> 3;
        t0 = die * per_die + (blockIdx.x >> 3);
        t_end = min(n_tiles, (die + 1) * per_die);
    }
#endif
    return t0 < t_end;
}

#endif  // SRFT_DEVICE_UTIL_H
