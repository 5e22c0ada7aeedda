// gemm / batched_gemm, both operands contiguous along K, bf16 inputs, 256x128 tiles.
#include "ucl_launch.h"
namespace ucl {
static const VariantDesc kTable[] = {
    describe<KernelCfg<256, 128, 32, 4, 0, 0, kKContig, kKContig>>(),
    describe<KernelCfg<256, 128, 32, 3, 0, 0, kKContig, kKContig>>(),
    describe<KernelCfg<256, 128, 64, 2, 0, 0, kKContig, kKContig>>(),
};
VariantList variants_gemm_kk_bf16_b() { return {kTable, (int)(sizeof(kTable) / sizeof(kTable[0]))}; }
}  // namespace ucl
