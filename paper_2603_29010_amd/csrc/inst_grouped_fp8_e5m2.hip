// grouped_gemm with fp8 (e5m2) inputs: per-group pointer tables, ragged M, both operands contiguous along K.
#include "ucl_launch.h"
namespace ucl {
static const VariantDesc kTable[] = {
    describe<KernelCfg<256, 256, 64, 2, 3, 1, kKContig, kKContig>>(),
    describe<KernelCfg<128, 128, 64, 2, 3, 1, kKContig, kKContig>>(),
    describe<KernelCfg<64, 64, 64, 4, 3, 1, kKContig, kKContig>>(),
};
VariantList variants_grouped_fp8_e5m2() { return {kTable, (int)(sizeof(kTable) / sizeof(kTable[0]))}; }
}  // namespace ucl
