// bf16 kernels of the Stream-K GEMM with the atomic-add fix-up (see streamk_kernels.h).
#include "streamk_kernels.h"
namespace streamk_detail {
void register_bf16_atomic(KernelEntry** t, int* n) { add_16bit_tiles<SK_BF16, true>(t, n); }
}  // namespace streamk_detail
