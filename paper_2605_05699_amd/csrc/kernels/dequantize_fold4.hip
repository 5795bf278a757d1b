// Read path, twice-folded form (d = 128 and 256, g >= 32), 4- and 8-bit codes.
#include "../dequantize_fold4_tiles.h"

dequantize_kernel_t srft_pick_dequantize_fold4(int d, int bits) {
    if (d == 128) return bits == 8 ? srft_dequantize_fold4_kernel<128, 8> : srft_dequantize_fold4_kernel<128, 4>;
    if (d == 256) return bits == 8 ? srft_dequantize_fold4_kernel<256, 8> : srft_dequantize_fold4_kernel<256, 4>;
    return nullptr;
}
batched_kernel_t srft_pick_dequantize_fold4_batched(int d, int bits) {
    if (d == 128) return bits == 8 ? srft_dequantize_fold4_batched_kernel<128, 8> : srft_dequantize_fold4_batched_kernel<128, 4>;
    if (d == 256) return bits == 8 ? srft_dequantize_fold4_batched_kernel<256, 8> : srft_dequantize_fold4_batched_kernel<256, 4>;
    return nullptr;
}
int srft_rfold4_table_units(int d) { return srft_rfold4_units(d); }
