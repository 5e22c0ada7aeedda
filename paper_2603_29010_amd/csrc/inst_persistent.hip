// persistent tile scheduler (grid = CU slots, every workgroup walks the tile order with a stride of the grid size): built for the
// tiles whose kernels leave registers free for the loop: gemm / batched up to 128x128, grouped 64x64 (the grouped 128x128 kernel
// lands just above 256 registers per lane, which halves its occupancy); operands contiguous along K.
#include "ucl_launch.h"
namespace ucl {
static const VariantDesc kTable[] = {
    describe<KernelCfg<128, 128, 64, 2, 0, 0, kKContig, kKContig, 1>>(),
    describe<KernelCfg<128, 128, 32, 4, 0, 0, kKContig, kKContig, 1>>(),
    describe<KernelCfg<64, 64, 64, 4, 0, 0, kKContig, kKContig, 1>>(),
    describe<KernelCfg<128, 128, 32, 4, 1, 0, kKContig, kKContig, 1>>(),
    describe<KernelCfg<64, 64, 64, 4, 1, 0, kKContig, kKContig, 1>>(),
    describe<KernelCfg<64, 64, 64, 4, 0, 1, kKContig, kKContig, 1>>(),
};
VariantList variants_persistent() { return {kTable, (int)(sizeof(kTable) / sizeof(kTable[0]))}; }
}  // namespace ucl
