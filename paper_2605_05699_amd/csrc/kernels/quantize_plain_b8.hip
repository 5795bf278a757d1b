// Write path, plain form, 8-bit codes: every (d, slabs per wavefront, group mode) instance.
#include "../quantize_tiles.h"

namespace {
template <int D, int S>
quantize_kernel_t by_group_mode(int gm) {
    switch (gm) {
        case kGroup16: return srft_quantize_kernel<D, S, kOutCodes, kGroup16, 8>;
        case kGroupWide: return srft_quantize_kernel<D, S, kOutCodes, kGroupWide, 8>;
        default: return srft_quantize_kernel<D, S, kOutCodes, kGroup32, 8>;
    }
}
template <int D>
quantize_kernel_t pick(int slabs, int gm) {
    if constexpr ((D / 32) % 2 == 0) {
        if (slabs == 2) return by_group_mode<D, 2>(gm);
    }
    return by_group_mode<D, 1>(gm);
}
template <int D, int S>
batched_kernel_t batched_by_group_mode(int gm) {
    return gm == kGroup16 ? srft_quantize_batched_kernel<D, S, kGroup16, 8>
         : gm == kGroupWide ? srft_quantize_batched_kernel<D, S, kGroupWide, 8>
                            : srft_quantize_batched_kernel<D, S, kGroup32, 8>;
}
template <int D>
batched_kernel_t pick_batched(int slabs, int gm) {
    if constexpr ((D / 32) % 2 == 0) {
        if (slabs == 2) return batched_by_group_mode<D, 2>(gm);
    }
    return batched_by_group_mode<D, 1>(gm);
}
}  // namespace

quantize_kernel_t srft_pick_quantize_plain_b8(int d, int slabs, int gm) { SRFT_DISPATCH_D(d, pick, slabs, gm) }
batched_kernel_t srft_pick_quantize_plain_batched_b8(int d, int slabs, int gm) {
    SRFT_DISPATCH_D(d, pick_batched, slabs, gm)
}
