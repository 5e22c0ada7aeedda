// gemm / batched_gemm with A contiguous along M (column-major A), bf16: A goes straight into LDS and is read through the LDS transpose read; B contiguous along K or along N.
#include "ucl_launch.h"
namespace ucl {
static const VariantDesc kTable[] = {
    describe<KernelCfg<256, 256, 64, 2, 0, 0, kMDirect, kKContig>>(),
    describe<KernelCfg<128, 128, 32, 4, 0, 0, kMDirect, kKContig>>(),
    describe<KernelCfg<128, 128, 64, 2, 0, 0, kMDirect, kKContig>>(),
    describe<KernelCfg<64, 64, 32, 3, 0, 0, kMDirect, kKContig>>(),
    describe<KernelCfg<64, 64, 64, 4, 0, 0, kMDirect, kKContig>>(),
    describe<KernelCfg<256, 256, 64, 2, 0, 0, kMDirect, kNDirect>>(),
    describe<KernelCfg<128, 128, 32, 4, 0, 0, kMDirect, kNDirect>>(),
    describe<KernelCfg<128, 128, 64, 2, 0, 0, kMDirect, kNDirect>>(),
    describe<KernelCfg<64, 64, 32, 3, 0, 0, kMDirect, kNDirect>>(),
    describe<KernelCfg<64, 64, 64, 4, 0, 0, kMDirect, kNDirect>>(),
};
VariantList variants_gemm_mx_bf16() { return {kTable, (int)(sizeof(kTable) / sizeof(kTable[0]))}; }
}  // namespace ucl
