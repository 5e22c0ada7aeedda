// stream-K tile scheduler (grid = CU slots, every workgroup takes an equal run of (tile, 64-wide k range) iterations, parts of tiles are
// added up through the workspace): gemm / batched, operands contiguous along K, the tiles whose kernels leave registers free for the loop.
#include "ucl_launch.h"
namespace ucl {
static const VariantDesc kTable[] = {
    describe<KernelCfg<128, 128, 32, 4, 0, 0, kKContig, kKContig, 2>>(),
    describe<KernelCfg<128, 128, 64, 2, 0, 0, kKContig, kKContig, 2>>(),
    describe<KernelCfg<64, 64, 64, 4, 0, 0, kKContig, kKContig, 2>>(),
    describe<KernelCfg<128, 128, 32, 4, 1, 0, kKContig, kKContig, 2>>(),
};
VariantList variants_streamk() { return {kTable, (int)(sizeof(kTable) / sizeof(kTable[0]))}; }
}  // namespace ucl
