// conv2d_wgrad: rows are output channels (A = the output gradient, contiguous along Kout, copied directly), columns (r, s, c) gathered from the activations, K = output pixels; split-K capable.
#include "ucl_launch.h"
namespace ucl {
static const VariantDesc kTable[] = {
    describe<KernelCfg<128, 128, 32, 4, 0, 4, kMDirect, kNDirect>>(),
    describe<KernelCfg<128, 128, 64, 2, 0, 4, kMDirect, kNDirect>>(),
    describe<KernelCfg<64, 64, 32, 3, 0, 4, kMDirect, kNDirect>>(),
    describe<KernelCfg<64, 64, 64, 4, 0, 4, kMDirect, kNDirect>>(),
    describe<KernelCfg<128, 128, 32, 4, 1, 4, kMDirect, kNDirect>>(),
    describe<KernelCfg<64, 64, 32, 3, 1, 4, kMDirect, kNDirect>>(),
};
VariantList variants_conv_wgrad() { return {kTable, (int)(sizeof(kTable) / sizeof(kTable[0]))}; }
}  // namespace ucl
