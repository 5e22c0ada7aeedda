// gemm / batched_gemm, both operands contiguous along K, fp16 inputs, 128x128 and 64x64 tiles.
#include "ucl_launch.h"
namespace ucl {
static const VariantDesc kTable[] = {
    describe<KernelCfg<128, 128, 64, 3, 1, 0, kKContig, kKContig>>(),
    describe<KernelCfg<128, 128, 32, 4, 1, 0, kKContig, kKContig>>(),
    describe<KernelCfg<128, 128, 32, 3, 1, 0, kKContig, kKContig>>(),
    describe<KernelCfg<128, 128, 64, 2, 1, 0, kKContig, kKContig>>(),
    describe<KernelCfg<64, 64, 32, 3, 1, 0, kKContig, kKContig>>(),
};
VariantList variants_gemm_kk_f16_b() { return {kTable, (int)(sizeof(kTable) / sizeof(kTable[0]))}; }
}  // namespace ucl
