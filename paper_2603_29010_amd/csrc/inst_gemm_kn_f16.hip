// gemm / batched_gemm, A contiguous along K, B contiguous along N (both row-major), f16: B goes straight into LDS and is read through the LDS transpose read.
#include "ucl_launch.h"
namespace ucl {
static const VariantDesc kTable[] = {
    describe<KernelCfg<256, 256, 64, 2, 1, 0, kKContig, kNDirect>>(),
        describe<KernelCfg<128, 128, 32, 4, 1, 0, kKContig, kNDirect>>(),
    describe<KernelCfg<128, 128, 64, 2, 1, 0, kKContig, kNDirect>>(),
    describe<KernelCfg<64, 64, 32, 3, 1, 0, kKContig, kNDirect>>(),
};
VariantList variants_gemm_kn_f16() { return {kTable, (int)(sizeof(kTable) / sizeof(kTable[0]))}; }
}  // namespace ucl
