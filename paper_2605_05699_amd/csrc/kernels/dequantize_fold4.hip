// Read path at d = 256, twice-folded form (g >= 32), 4- and 8-bit codes.
#include "../dequantize_fold4_tiles.h"

dequantize_kernel_t srft_pick_dequantize_fold4(int bits) {
    return bits == 8 ? srft_dequantize_fold4_kernel<8> : srft_dequantize_fold4_kernel<4>;
}
batched_kernel_t srft_pick_dequantize_fold4_batched(int bits) {
    return bits == 8 ? srft_dequantize_fold4_batched_kernel<8> : srft_dequantize_fold4_batched_kernel<4>;
}
int srft_rfold4_table_units(void) { return kRFold4Units; }
