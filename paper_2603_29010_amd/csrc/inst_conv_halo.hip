// conv2d_fprop, 3x3 / stride 1 / pad 1 / 64 or 128 channels: activations held in LDS as one resident patch per tile, 256x128 tiles.
#include "ucl_launch.h"
namespace ucl {
static const VariantDesc kTable[] = {
    describe<KernelCfg<256, 128, 32, 4, 0, 2, kHalo, kKContig>>(),
    describe<KernelCfg<256, 128, 32, 4, 1, 2, kHalo, kKContig>>(),
    // pixels of 128 channels (the 128-row tile with 64 columns leaves room for two workgroups per CU)
    describe<KernelCfg<256, 128, 32, 4, 0, 2, kHalo, kKContig, 0, 128>>(),
    describe<KernelCfg<128, 64, 32, 4, 0, 2, kHalo, kKContig, 0, 128>>(),
    describe<KernelCfg<256, 128, 32, 4, 1, 2, kHalo, kKContig, 0, 128>>(),
};
VariantList variants_conv_halo() { return {kTable, (int)(sizeof(kTable) / sizeof(kTable[0]))}; }
}  // namespace ucl
