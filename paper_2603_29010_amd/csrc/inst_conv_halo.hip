// conv2d_fprop, 3x3 / stride 1 / pad 1 / 64 channels: activations held in LDS as one resident patch per tile, 256x128 tiles.
#include "ucl_launch.h"
namespace ucl {
static const VariantDesc kTable[] = {
    describe<KernelCfg<256, 128, 32, 4, 0, 2, kHalo, kKContig>>(),
    describe<KernelCfg<256, 128, 32, 4, 1, 2, kHalo, kKContig>>(),
};
VariantList variants_conv_halo() { return {kTable, (int)(sizeof(kTable) / sizeof(kTable[0]))}; }
}  // namespace ucl
