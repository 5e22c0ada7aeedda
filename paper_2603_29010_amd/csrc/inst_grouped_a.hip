// grouped_gemm (per-group pointer tables, ragged M), operands contiguous along K, bf16, large tiles.
#include "ucl_launch.h"
namespace ucl {
static const VariantDesc kTable[] = {
    describe<KernelCfg<256, 256, 32, 4, 0, 1, kKContig, kKContig>>(),
    describe<KernelCfg<256, 256, 32, 5, 0, 1, kKContig, kKContig>>(),
    describe<KernelCfg<256, 256, 64, 2, 0, 1, kKContig, kKContig>>(),
    describe<KernelCfg<256, 128, 32, 4, 0, 1, kKContig, kKContig>>(),
    describe<KernelCfg<256, 128, 32, 3, 0, 1, kKContig, kKContig>>(),
};
VariantList variants_grouped_a() { return {kTable, (int)(sizeof(kTable) / sizeof(kTable[0]))}; }
}  // namespace ucl
