// gemm / batched_gemm with fp8 inputs (e4m3 and e5m2), both operands contiguous along K: the loops of the 16-bit kernels on pairs of elements, two 8-bit MFMAs per fragment.
#include "ucl_launch.h"
namespace ucl {
static const VariantDesc kTable[] = {
    describe<KernelCfg<256, 256, 64, 2, 2, 0, kKContig, kKContig>>(),
    describe<KernelCfg<256, 128, 32, 3, 2, 0, kKContig, kKContig>>(),
    describe<KernelCfg<128, 128, 64, 2, 2, 0, kKContig, kKContig>>(),
    describe<KernelCfg<64, 64, 64, 4, 2, 0, kKContig, kKContig>>(),
    describe<KernelCfg<256, 256, 64, 2, 3, 0, kKContig, kKContig>>(),
    describe<KernelCfg<128, 128, 64, 2, 3, 0, kKContig, kKContig>>(),
    describe<KernelCfg<64, 64, 64, 4, 3, 0, kKContig, kKContig>>(),
};
VariantList variants_gemm_kk_fp8() { return {kTable, (int)(sizeof(kTable) / sizeof(kTable[0]))}; }
}  // namespace ucl
