// fp8 (e4m3) kernels of the Stream-K GEMM (see streamk_kernels.h): the same byte footprint per stage
// as the 16-bit tiles with twice the k.
#include "streamk_kernels.h"
namespace streamk_detail {
void register_fp8(KernelEntry** t, int* n) {
    t[(*n)++] = make_entry<Cfg<SK_FP8_E4M3, 256, 256, 128, 2, 4, 32, 3, 2>>();
    t[(*n)++] = make_entry<Cfg<SK_FP8_E4M3, 256, 256, 128, 2, 2, 32, 3, 2, 1>>(1, 48);   // four waves: plans without split tiles and K >= 6144 (+2 - 3 %)
    t[(*n)++] = make_entry<Cfg<SK_FP8_E4M3, 128, 256, 128, 2, 4, 32, 3, 3>>();
    t[(*n)++] = make_entry<Cfg<SK_FP8_E4M3, 256, 256, 128, 2, 4, 32, 3, 2>>(3);             // variant 0's kernel under a number of its own
}
void register_fp8_atomic(KernelEntry** t, int* n) {
    t[(*n)++] = make_entry<Cfg<SK_FP8_E4M3, 256, 256, 128, 2, 4, 32, 3, 2>, true>();
    t[(*n)++] = make_entry<Cfg<SK_FP8_E4M3, 128, 256, 128, 2, 4, 32, 3, 3>, true>();
}
}  // namespace streamk_detail
