// conv2d_dgrad, 3x3 / stride 1 / pad 1 / 128 or 64 output channels: the output gradient held in LDS as one resident patch per tile, taps mirrored.
#include "ucl_launch.h"
namespace ucl {
static const VariantDesc kTable[] = {
    describe<KernelCfg<256, 64, 32, 4, 0, 3, kHalo, kNDirect>>(),
    describe<KernelCfg<128, 64, 32, 4, 0, 3, kHalo, kNDirect>>(),
    describe<KernelCfg<256, 64, 32, 4, 1, 3, kHalo, kNDirect>>(),
    // 64 output channels
    describe<KernelCfg<256, 64, 32, 4, 0, 3, kHalo, kNDirect, 0, 64>>(),
    describe<KernelCfg<256, 128, 32, 4, 0, 3, kHalo, kNDirect, 0, 64>>(),
    describe<KernelCfg<256, 64, 32, 4, 1, 3, kHalo, kNDirect, 0, 64>>(),
};
VariantList variants_conv_dgrad_halo() { return {kTable, (int)(sizeof(kTable) / sizeof(kTable[0]))}; }
}  // namespace ucl
