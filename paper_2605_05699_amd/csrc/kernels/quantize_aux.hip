// Write path, plain form, outputs other than codes: the raw coefficients (srft_kv_forward_f32), the per-channel
// abs-max statistic (srft_kv_channel_absmax) and the query operands of the scores kernel.
#include "../quantize_tiles.h"

namespace {
template <int D, int S>
quantize_kernel_t by_output(int out) {
    if (out == kOutRaw) return srft_quantize_kernel<D, S, kOutRaw, kGroup32, 4>;
    if (out == kOutAmax) return srft_quantize_kernel<D, S, kOutAmax, kGroup32, 4>;
    if constexpr (S == 1 && D % 64 == 0) {       // the scores set-up always runs one slab per wavefront
        if (out == kOutQFrag32) return srft_quantize_kernel<D, 1, kOutQFrag32, kGroup32, 4>;
        if (out == kOutQFrag16) return srft_quantize_kernel<D, 1, kOutQFrag16, kGroup32, 4>;
    }
    return nullptr;
}
template <int D>
quantize_kernel_t pick(int slabs, int out) {
    if constexpr ((D / 32) % 2 == 0) {
        if (slabs == 2) return by_output<D, 2>(out);
    }
    return by_output<D, 1>(out);
}
}  // namespace

quantize_kernel_t srft_pick_quantize_aux(int d, int slabs, int out) { SRFT_DISPATCH_D(d, pick, slabs, out) }
