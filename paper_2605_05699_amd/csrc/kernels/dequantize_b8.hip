// Read path, 8-bit codes: every (d, slabs per wavefront, group mode, folded or plain) instance.
#include "../dequantize_tiles.h"

namespace {
template <int D>
dequantize_kernel_t pick(int slabs, int gm, bool fold) {
    if constexpr ((D / 32) % 2 == 0) {
        if constexpr (D != 128 && D != 256)      // d = 128 and 256 run the twice-folded kernel instead
            if (fold && gm != kGroup16) return srft_dequantize_kernel<D, 2, 1, true, 8>;
        if (slabs == 2)
            return gm == kGroup16 ? srft_dequantize_kernel<D, 2, 1, false, 8>
                                  : srft_dequantize_kernel<D, 2, 2, false, 8>;
    }
    return gm == kGroup16 ? srft_dequantize_kernel<D, 1, 1, false, 8> : srft_dequantize_kernel<D, 1, 2, false, 8>;
}
template <int D>
batched_kernel_t pick_batched(int slabs, int gm, bool fold) {
    if constexpr ((D / 32) % 2 == 0) {
        if constexpr (D != 128 && D != 256)      // d = 128 and 256 run the twice-folded kernel instead
            if (fold && gm != kGroup16) return srft_dequantize_batched_kernel<D, 2, 1, true, 8>;
        if (slabs == 2)
            return gm == kGroup16 ? srft_dequantize_batched_kernel<D, 2, 1, false, 8>
                                  : srft_dequantize_batched_kernel<D, 2, 2, false, 8>;
    }
    return gm == kGroup16 ? srft_dequantize_batched_kernel<D, 1, 1, false, 8>
                          : srft_dequantize_batched_kernel<D, 1, 2, false, 8>;
}
}  // namespace

dequantize_kernel_t srft_pick_dequantize_b8(int d, int slabs, int gm, bool fold) {
    SRFT_DISPATCH_D(d, pick, slabs, gm, fold)
}
batched_kernel_t srft_pick_dequantize_batched_b8(int d, int slabs, int gm, bool fold) {
    SRFT_DISPATCH_D(d, pick_batched, slabs, gm, fold)
}
