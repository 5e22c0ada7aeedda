// conv2d_dgrad: rows are input pixels, A gathers the output gradient per tap, B reads filter rows w[k, r, s, :] (contiguous along C) directly.
#include "ucl_launch.h"
namespace ucl {
static const VariantDesc kTable[] = {
    describe<KernelCfg<256, 128, 32, 3, 0, 3, kIm2col, kNDirect>>(),
    describe<KernelCfg<256, 64, 32, 4, 0, 3, kIm2col, kNDirect>>(),
    describe<KernelCfg<128, 64, 32, 4, 0, 3, kIm2col, kNDirect>>(),
    describe<KernelCfg<128, 128, 32, 4, 0, 3, kIm2col, kNDirect>>(),
    describe<KernelCfg<64, 64, 32, 3, 0, 3, kIm2col, kNDirect>>(),
    describe<KernelCfg<128, 128, 32, 4, 1, 3, kIm2col, kNDirect>>(),
    describe<KernelCfg<64, 64, 32, 3, 1, 3, kIm2col, kNDirect>>(),
};
VariantList variants_conv_dgrad() { return {kTable, (int)(sizeof(kTable) / sizeof(kTable[0]))}; }
}  // namespace ucl
