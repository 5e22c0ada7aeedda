// Registry of the built kernel variants: every instantiation unit contributes a table of these.
#pragma once
#include "ucl_device.h"

namespace ucl {

struct VariantDesc {
    int tile_m, tile_n, tile_k, stages;
    int dt;             // inputs: 0 bf16, 1 fp16, 2 fp8 e4m3, 3 fp8 e5m2 (8-bit inputs are handled as pairs: K, strides in 16-bit units)
    int mode;           // 0 gemm / batched, 1 grouped, 2 conv2d fprop, 3 conv2d dgrad, 4 conv2d wgrad
    int la, lb;         // 0: operand contiguous along K, 1: contiguous along M / N (register transpose); A only: 2 im2col gather,
                        // 3 resident patch; 4 (B) / 5 (A): contiguous along N / M, copied directly and read through the LDS transpose read
    int lds_bytes;
    int persistent;     // tile scheduler the kernel is built for: 0 one workgroup per tile, 1 persistent (grid = CU slots, workgroups
                        // walk the tile order), 2 stream-K (grid = CU slots, workgroups take equal runs of (tile, k range) iterations)
    int wgs_per_cu;     // workgroups of the kernel a CU is meant to hold (register budget it was built with)
    int patch_c;        // resident-patch kernels: channels per pixel of the tensor the patch holds (64 or 128), else 0
    hipError_t (*launch)(const KParams &p, const GroupTable *gt, int grid, hipStream_t stream);
    int (*resident)();          // workgroups one CU holds at a time (queried from the runtime)
};

struct VariantList {
    const VariantDesc *v;
    int n;
};

// one per instantiation unit
VariantList variants_gemm_kk_bf16_a();
VariantList variants_gemm_kk_bf16_b();
VariantList variants_gemm_kk_bf16_c();
VariantList variants_gemm_kk_bf16_d();
VariantList variants_gemm_kk_f16_a();
VariantList variants_gemm_kk_f16_b();
VariantList variants_gemm_mn_bf16();
VariantList variants_gemm_mn_f16();
VariantList variants_grouped_a();
VariantList variants_grouped_b();
VariantList variants_conv_a();
VariantList variants_conv_b();
VariantList variants_conv_f16();
VariantList variants_conv_halo();
VariantList variants_gemm_kn_bf16();
VariantList variants_gemm_kn_f16();
VariantList variants_gemm_mx_bf16();
VariantList variants_gemm_mx_f16();
VariantList variants_grouped_kn();
VariantList variants_persistent();
VariantList variants_streamk();
VariantList variants_grouped_fp8_e4m3();
VariantList variants_grouped_fp8_e5m2();
VariantList variants_gemm_kk_fp8();
VariantList variants_conv_dgrad();
VariantList variants_conv_dgrad_halo();
VariantList variants_conv_wgrad();

}  // namespace ucl
