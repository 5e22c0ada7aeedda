// grouped_gemm (per-group pointer tables, ragged M), operands contiguous along K, small tiles and fp16.
#include "ucl_launch.h"
namespace ucl {
static const VariantDesc kTable[] = {
    describe<KernelCfg<128, 128, 64, 3, 0, 1, kKContig, kKContig>>(),
    describe<KernelCfg<128, 128, 64, 2, 0, 1, kKContig, kKContig>>(),
    describe<KernelCfg<64, 64, 32, 3, 0, 1, kKContig, kKContig>>(),
    describe<KernelCfg<256, 256, 32, 4, 1, 1, kKContig, kKContig>>(),
    describe<KernelCfg<256, 256, 64, 2, 1, 1, kKContig, kKContig>>(),
    describe<KernelCfg<128, 128, 64, 3, 1, 1, kKContig, kKContig>>(),
    describe<KernelCfg<64, 64, 32, 3, 1, 1, kKContig, kKContig>>(),
};
VariantList variants_grouped_b() { return {kTable, (int)(sizeof(kTable) / sizeof(kTable[0]))}; }
}  // namespace ucl
