// Write path at d = 256, g = 32, folded twice (a quarter of the dense matrix work): 4- and 8-bit codes.
#include "../quantize_fold4_tiles.h"

quantize_kernel_t srft_pick_quantize_fold4(int bits) {
    return bits == 8 ? srft_quantize_fold4_kernel<8> : srft_quantize_fold4_kernel<4>;
}
batched_kernel_t srft_pick_quantize_fold4_batched(int bits) {
    return bits == 8 ? srft_quantize_fold4_batched_kernel<8> : srft_quantize_fold4_batched_kernel<4>;
}
int srft_fold4_table_units(void) { return kFold4Units; }

#ifdef SRFT_F4_TRACE
// work builds only: a buffer for per-stage cycle stamps
extern "C" void* srft_debug_buffer(size_t bytes) {
    void* p = nullptr;
    if (hipMalloc(&p, bytes) != hipSuccess || hipMemset(p, 0, bytes) != hipSuccess) return nullptr;
    if (hipMemcpyToSymbol(HIP_SYMBOL(srft_trace_buf), &p, sizeof(p)) != hipSuccess) return nullptr;
    return p;
}
#endif
