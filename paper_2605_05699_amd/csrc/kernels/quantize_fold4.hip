// Write path at d = 256, g = 32, folded twice (a quarter of the dense matrix work): 4- and 8-bit codes.
#include "../quantize_fold4_tiles.h"

quantize_kernel_t srft_pick_quantize_fold4(int bits) {
    return bits == 8 ? srft_quantize_fold4_kernel<8> : srft_quantize_fold4_kernel<4>;
}
batched_kernel_t srft_pick_quantize_fold4_batched(int bits) {
    return bits == 8 ? srft_quantize_fold4_batched_kernel<8> : srft_quantize_fold4_batched_kernel<4>;
}
int srft_fold4_table_units(void) { return kFold4Units; }

