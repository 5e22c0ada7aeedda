// gemm / batched_gemm with an operand contiguous along M or N (transposed on the way into LDS), bf16 inputs.
#include "ucl_launch.h"
namespace ucl {
static const VariantDesc kTable[] = {
    describe<KernelCfg<128, 128, 64, 2, 0, 0, kKContig, kMNContig>>(),
    describe<KernelCfg<128, 128, 64, 2, 0, 0, kMNContig, kKContig>>(),
    describe<KernelCfg<128, 128, 64, 2, 0, 0, kMNContig, kMNContig>>(),
    describe<KernelCfg<64, 64, 64, 2, 0, 0, kKContig, kMNContig>>(),
    describe<KernelCfg<64, 64, 64, 2, 0, 0, kMNContig, kKContig>>(),
    describe<KernelCfg<64, 64, 64, 2, 0, 0, kMNContig, kMNContig>>(),
};
VariantList variants_gemm_mn_bf16() { return {kTable, (int)(sizeof(kTable) / sizeof(kTable[0]))}; }
}  // namespace ucl
