// conv2d_fprop as implicit GEMM (A gathered from NHWC activations, filter KRSC contiguous along K), bf16, 256x128 tiles.
#include "ucl_launch.h"
namespace ucl {
static const VariantDesc kTable[] = {
    describe<KernelCfg<256, 128, 32, 4, 0, 2, kIm2col, kKContig>>(),
    describe<KernelCfg<256, 128, 32, 3, 0, 2, kIm2col, kKContig>>(),
    describe<KernelCfg<256, 128, 64, 2, 0, 2, kIm2col, kKContig>>(),
};
VariantList variants_conv_a() { return {kTable, (int)(sizeof(kTable) / sizeof(kTable[0]))}; }
}  // namespace ucl
