// Write path, folded form (d = 128 and 256): 4- and 8-bit codes, g = 32 or wider groups.
#include "../quantize_fold_tiles.h"

namespace {
template <int D>
quantize_kernel_t pick(int bits, bool wide) {
    if (wide) return bits == 8 ? srft_quantize_fold_kernel<D, 8, true> : srft_quantize_fold_kernel<D, 4, true>;
    return bits == 8 ? srft_quantize_fold_kernel<D, 8, false> : srft_quantize_fold_kernel<D, 4, false>;
}
template <int D>
batched_kernel_t pick_batched(int bits, bool wide) {
    if (wide)
        return bits == 8 ? srft_quantize_fold_batched_kernel<D, 8, true> : srft_quantize_fold_batched_kernel<D, 4, true>;
    return bits == 8 ? srft_quantize_fold_batched_kernel<D, 8, false> : srft_quantize_fold_batched_kernel<D, 4, false>;
}
}  // namespace

quantize_kernel_t srft_pick_quantize_fold(int d, int bits, bool wide) {
    return d == 128 ? pick<128>(bits, wide) : d == 256 ? pick<256>(bits, wide) : nullptr;
}
quantize_kernel_t srft_pick_quantize_fold_amax(int d) {
    return d == 128 ? srft_quantize_fold_amax_kernel<128> : d == 256 ? srft_quantize_fold_amax_kernel<256> : nullptr;
}
batched_kernel_t srft_pick_quantize_fold_batched(int d, int bits, bool wide) {
    return d == 128 ? pick_batched<128>(bits, wide) : d == 256 ? pick_batched<256>(bits, wide) : nullptr;
}
