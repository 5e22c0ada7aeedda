// grouped_gemm with each group's B contiguous along N (row-major expert weights): B copied directly and read through the LDS transpose read.
#include "ucl_launch.h"
namespace ucl {
static const VariantDesc kTable[] = {
    describe<KernelCfg<256, 256, 64, 2, 0, 1, kKContig, kNDirect>>(),
    describe<KernelCfg<128, 128, 32, 4, 0, 1, kKContig, kNDirect>>(),
    describe<KernelCfg<64, 64, 32, 3, 0, 1, kKContig, kNDirect>>(),
    describe<KernelCfg<256, 256, 64, 2, 1, 1, kKContig, kNDirect>>(),
    describe<KernelCfg<64, 64, 32, 3, 1, 1, kKContig, kNDirect>>(),
};
VariantList variants_grouped_kn() { return {kTable, (int)(sizeof(kTable) / sizeof(kTable[0]))}; }
}  // namespace ucl
