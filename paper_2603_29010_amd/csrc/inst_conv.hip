// conv2d_fprop as implicit GEMM: A operand gathered from NHWC activations, filter KRSC contiguous along K.
#include "ucl_launch.h"
namespace ucl {
static const VariantDesc kTable[] = {
    describe<KernelCfg<256, 128, 64, 2, false, 2, kIm2col, kKContig>>(),
    describe<KernelCfg<256, 128, 32, 4, false, 2, kIm2col, kKContig>>(),
    describe<KernelCfg<128, 128, 64, 3, false, 2, kIm2col, kKContig>>(),
    describe<KernelCfg<128, 128, 32, 4, false, 2, kIm2col, kKContig>>(),
    describe<KernelCfg<64, 64, 64, 2, false, 2, kIm2col, kKContig>>(),
    describe<KernelCfg<256, 128, 32, 4, true, 2, kIm2col, kKContig>>(),
    describe<KernelCfg<128, 128, 64, 3, true, 2, kIm2col, kKContig>>(),
    describe<KernelCfg<64, 64, 64, 2, true, 2, kIm2col, kKContig>>(),
};
VariantList variants_conv() { return {kTable, (int)(sizeof(kTable) / sizeof(kTable[0]))}; }
}  // namespace ucl
