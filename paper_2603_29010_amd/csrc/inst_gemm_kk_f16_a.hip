// gemm / batched_gemm, both operands contiguous along K, fp16 inputs, large tiles.
#include "ucl_launch.h"
namespace ucl {
static const VariantDesc kTable[] = {
    describe<KernelCfg<256, 256, 32, 4, 1, 0, kKContig, kKContig>>(),
    describe<KernelCfg<256, 256, 64, 2, 1, 0, kKContig, kKContig>>(),
    describe<KernelCfg<256, 128, 32, 4, 1, 0, kKContig, kKContig>>(),
    describe<KernelCfg<256, 128, 32, 3, 1, 0, kKContig, kKContig>>(),
};
VariantList variants_gemm_kk_f16_a() { return {kTable, (int)(sizeof(kTable) / sizeof(kTable[0]))}; }
}  // namespace ucl
