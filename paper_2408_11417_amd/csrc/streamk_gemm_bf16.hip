// bf16 kernels of the Stream-K GEMM (see streamk_kernels.h).
#include "streamk_kernels.h"
namespace streamk_detail {
void register_bf16(KernelEntry** t, int* n) { add_16bit_tiles<SK_BF16>(t, n); }
}  // namespace streamk_detail
