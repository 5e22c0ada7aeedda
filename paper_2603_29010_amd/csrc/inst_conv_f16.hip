// conv2d_fprop as implicit GEMM (A gathered from NHWC activations, filter KRSC contiguous along K), fp16.
#include "ucl_launch.h"
namespace ucl {
static const VariantDesc kTable[] = {
    describe<KernelCfg<256, 128, 32, 4, 1, 2, kIm2col, kKContig>>(),
    describe<KernelCfg<128, 128, 64, 3, 1, 2, kIm2col, kKContig>>(),
    describe<KernelCfg<64, 64, 32, 3, 1, 2, kIm2col, kKContig>>(),
};
VariantList variants_conv_f16() { return {kTable, (int)(sizeof(kTable) / sizeof(kTable[0]))}; }
}  // namespace ucl
