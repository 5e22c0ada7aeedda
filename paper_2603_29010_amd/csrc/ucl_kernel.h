// The one mainloop of the library: an MFMA tile kernel for gfx950 (CDNA4, wave64), shared by
// gemm / batched_gemm / grouped_gemm / conv2d_fprop / conv2d_dgrad / conv2d_wgrad.  Included only by
// the instantiation units.
//
// Structure of a workgroup (256 threads = 4 waves, one per SIMD):
//   tile schedule  : workgroup id -> (batch or group, tile row, tile column), XCD-aware; with split-K also a K slice;
//                    under the persistent scheduler a walk over several tiles, under stream-K over tiles and
//                    parts of tiles (partial sums meet in a workspace and are added in a fixed order)
//   staging        : global -> LDS, `STAGES` buffers deep, 128-bit `buffer_load ... lds` (no VGPR round
//                    trip) for every operand form: rows contiguous along K, the gathered views of the
//                    three convolutions, and rows contiguous along M / N (copied as they are and read
//                    back through the LDS transpose read).  A fallback that loads M / N-contiguous
//                    operands into VGPRs and transposes them on the way into LDS serves matrices beyond
//                    the reach of 32-bit offsets.
//   LDS layout     : [rows][TK elements] (TK = 64 or 32: 128- or 64-byte rows of 16-byte chunks), chunk
//                    index XORed with a function of the row so that the 16-byte-per-lane MFMA
//                    fragment reads of 16 consecutive rows spread over all banks.
//   mainloop       : v_mfma_f32_16x16x32_{bf16,f16} (8-bit inputs: the 32-deep or the 128-deep fp8 MFMA on
//                    pairs of elements), fp32 accumulators held in registers, wave tile (TM/2) x (TN/2).
//   epilogue       : accumulators pass through a wave-private LDS patch to a row-contiguous layout;
//                    the `>>` chain runs on them in fp32 registers, one rounding to the output type,
//                    128-bit stores of whole row segments.
#pragma once
#include <cstddef>
#include <type_traits>
#include <utility>

#include "ucl_device.h"

namespace ucl {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2_t;
typedef __attribute__((ext_vector_type(8))) uint32_t u32x8_t;

#define UCL_LDS_PTR(p) ((__attribute__((address_space(3))) void *)(p))

// kIm2col gathers every filter tap of the activations from global memory again; kHalo (3x3 filter,
// unit stride and dilation, pad 1, 64 or 128 channels) copies the pixels a tile needs -- its rows plus one
// image row and one pixel on either side -- into LDS once and reads every tap from there (fprop: pixels
// of the activations; dgrad: pixels of the output gradient, taps mirrored).
// kNDirect (B only): B contiguous along N is copied row by row (k) straight into LDS like a
// K-contiguous operand and the MFMA fragments -- 8 consecutive k per lane -- come out of the LDS
// transpose read (ds_read_b64_tr_b16), so no register transpose and no 16-bit LDS writes are needed.
// kMDirect (A only) is the same for A contiguous along M.
enum OperandLayout { kKContig = 0, kMNContig = 1, kIm2col = 2, kHalo = 3, kNDirect = 4, kMDirect = 5 };

// Compile-time loop: register arrays (accumulators, fragments) must only ever be indexed by
// constants, or the compiler moves them to scratch memory.
template <class F, int... I>
__device__ __forceinline__ void static_for_impl(F &&f, std::integer_sequence<int, I...>) {
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void static_for(F &&f) {
    static_for_impl(f, std::make_integer_sequence<int, N>{});
}

// s_waitcnt immediate (gfx9 encoding) that waits only on the vector-memory counter.
__device__ constexpr int vmcnt_imm(int n) { return (n & 0xF) | ((n >> 4) << 14) | (0x7 << 4) | (0xF << 8); }

// Workgroup barrier of the pipelined mainloop: waits until at most `VM` of this wave's global -> LDS
// loads are outstanding and all of its LDS reads have returned, then s_barrier.  __syncthreads() is
// not used there: its release fence makes the compiler wait for EVERY outstanding global -> LDS load
// (it must treat them as LDS stores), which would drain the pipeline at each stage boundary.  The
// empty asm statements only stop the compiler from moving memory operations across the barrier.
template <int VM>
__device__ __forceinline__ void pipeline_barrier() {
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt((VM & 0xF) | ((VM >> 4) << 14) | (0x7 << 4) | (0x0 << 8));   // vmcnt(VM) lgkmcnt(0)
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

// XOR pattern of the LDS layout, for rows of CPR 16-byte chunks.  It depends on row mod 16 only, so
// any multiple-of-16 row offset (wave tile, MFMA block) leaves it unchanged.  An MFMA fragment read
// has 16 consecutive lanes on 16 consecutive rows at one logical chunk: with rows of 64 bytes the
// 16-byte slots hit are (row mod 4) * 4 + (chunk ^ swz), with rows of 128 bytes (row mod 2) * 8 +
// (chunk ^ swz), modulo the 16 slots of the banks -- both patterns make these 16 values distinct
// (measured: SQ_LDS_BANK_CONFLICT = 0).
template <int CPR>
__device__ __forceinline__ int lds_swz(int row) {
    if constexpr (CPR == 8) return (row & 7) ^ ((row >> 3) & 1);
    else return (row >> 2) & 3;
}

__device__ __forceinline__ float bits_to_f32(uint32_t raw16, int dtype) {
    if (dtype == UCL_BF16) return __uint_as_float(raw16 << 16);
    union { uint16_t u; _Float16 h; } c;
    c.u = (uint16_t)raw16;
    return (float)c.h;
}

// ---- epilogue operand access: 8 consecutive elements along n per lane ---------------------------

// Raw result of an 8-element load, decoded later so that several loads can be in flight at once.
struct Raw8 {
    u32x4_t lo, hi;     // packed: eight 16-bit patterns in lo.  Otherwise eight fp32 values in lo, hi.
    bool packed;
};

// Elements [idx, idx+8) of a tensor of type dtype; lanes with nvalid < 8 read only what exists
// (the rest decode to 0).  `vec`: base + idx is 16-byte aligned for every lane (host-checked).
__device__ __forceinline__ Raw8 load8(const void *base, int dtype, int64_t idx, bool vec, int nvalid) {
    Raw8 r;
    r.lo = u32x4_t{0, 0, 0, 0};
    r.hi = u32x4_t{0, 0, 0, 0};
    r.packed = false;
    if (nvalid <= 0) return r;
    if (vec && nvalid >= 8) {
        if (dtype == UCL_F32) {
            const u32x4_t *p = (const u32x4_t *)((const float *)base + idx);
            r.lo = p[0];
            r.hi = p[1];
        } else {
            r.lo = *(const u32x4_t *)((const uint16_t *)base + idx);
            r.packed = true;
        }
        return r;
    }
    float t[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        t[e] = 0.f;
        if (e < nvalid)
            t[e] = dtype == UCL_F32 ? ((const float *)base)[idx + e]
                                    : bits_to_f32(((const uint16_t *)base)[idx + e], dtype);
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        r.lo[e] = __float_as_uint(t[e]);
        r.hi[e] = __float_as_uint(t[4 + e]);
    }
    return r;
}

__device__ __forceinline__ void decode8(const Raw8 &r, int dtype, float (&out)[8]) {
    if (r.packed) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            out[2 * e] = bits_to_f32(r.lo[e] & 0xffffu, dtype);
            out[2 * e + 1] = bits_to_f32(r.lo[e] >> 16, dtype);
        }
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            out[e] = __uint_as_float(r.lo[e]);
            out[4 + e] = __uint_as_float(r.hi[e]);
        }
    }
}

__device__ __forceinline__ uint32_t f32_to_bits16(float v, int dtype) {
    if (dtype == UCL_BF16) {
        union { __bf16 b; uint16_t u; } c;
        c.b = (__bf16)v;                  // round to nearest even
        return c.u;
    }
    union { _Float16 h; uint16_t u; } c;
    c.h = (_Float16)v;                    // round to nearest even
    return c.u;
}

// One rounding to the stored type, then 128-bit stores where alignment allows.
__device__ __forceinline__ void store8(void *base, int dtype, int64_t idx, const float (&v)[8], bool vec, int nvalid) {
    if (nvalid <= 0) return;
    if (dtype == UCL_F32) {
        float *p = (float *)base + idx;
        if (vec && nvalid >= 8) {
            ((f32x4_t *)p)[0] = f32x4_t{v[0], v[1], v[2], v[3]};
            ((f32x4_t *)p)[1] = f32x4_t{v[4], v[5], v[6], v[7]};
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e)
                if (e < nvalid) p[e] = v[e];
        }
    } else {
        uint16_t *p = (uint16_t *)base + idx;
        uint32_t b[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) b[e] = f32_to_bits16(v[e], dtype);
        if (vec && nvalid >= 8) {
            *(u32x4_t *)p = u32x4_t{b[0] | (b[1] << 16), b[2] | (b[3] << 16), b[4] | (b[5] << 16), b[6] | (b[7] << 16)};
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e)
                if (e < nvalid) p[e] = (uint16_t)b[e];
        }
    }
}

// 1 / (1 + 2^-t): one exp2 and one reciprocal (both hardware approximations good to ~1 ulp), so an
// activation built on it costs two quarter-rate instructions per element instead of a full division.
__device__ __forceinline__ float sigmoid_exp2(float t) {
    return __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-t));
}
__device__ __forceinline__ float sigmoid_f32(float u) { return sigmoid_exp2(u * 1.4426950408889634f); }

// The element-wise activations of the vocabulary, fp32.
template <int OP>
__device__ __forceinline__ float act_f32(float x, float p0, float p1) {
    if constexpr (OP == UCL_EPI_RELU) return fmaxf(x, 0.f);
    else if constexpr (OP == UCL_EPI_LEAKY_RELU) return x > 0.f ? x : p0 * x;
    else if constexpr (OP == UCL_EPI_CLAMP) return fminf(fmaxf(x, p0), p1);
    else if constexpr (OP == UCL_EPI_HARDSWISH) return x * fminf(fmaxf(x + 3.f, 0.f), 6.f) * (1.f / 6.f);
    else if constexpr (OP == UCL_EPI_GELU_TANH) {
        // 0.5 (1 + tanh u) = sigmoid(2u),  u = sqrt(2/pi) (x + 0.044715 x^3); constants folded with log2(e)
        const float x2 = x * x;
        return x * sigmoid_exp2(x * (2.3022082011f + 0.1029432397f * x2));
    } else if constexpr (OP == UCL_EPI_SILU) return x * sigmoid_f32(x);
    else if constexpr (OP == UCL_EPI_SIGMOID) return sigmoid_f32(x);
    else if constexpr (OP == UCL_EPI_TANH) return tanhf(x);
    else if constexpr (OP == UCL_EPI_GELU_ERF) return 0.5f * x * (1.f + erff(x * 0.7071067811865476f));
    else if constexpr (OP == UCL_EPI_MISH) {
        // tanh(log(1 + e^x)) = w (w + 2) / (w (w + 2) + 2) with w = e^x; for large x the factor is 1
        const float w = __builtin_amdgcn_exp2f(fminf(x, 20.f) * 1.4426950408889634f);
        const float q = w * (w + 2.f);
        return x > 20.f ? x : x * (q * __builtin_amdgcn_rcpf(q + 2.f));
    } else if constexpr (OP == UCL_EPI_ELU) return x > 0.f ? x : p0 * expm1f(x);
    else return x;
}

// Where a lane stands in the output while it runs the chain: 8 consecutive columns of one row.
struct EpiCtx {
    int64_t m;          // row within the (sub)problem
    int n;              // first of the lane's 8 columns
    int nvalid;         // how many of them exist (<= 0: none; row out of range counts as none)
    int batch;          // batch index (bs multiplier)
    int group;          // grouped: index into per-group pointer tables, else -1
};

__device__ __forceinline__ const void *step_ptr(const EpiStepDev &s, int group) {
    if (group >= 0) return ((const void *const *)s.ptr)[group];
    return s.ptr;
}

__device__ __forceinline__ bool op_is_nvec(int op) {
    return op == UCL_EPI_BIAS || op == UCL_EPI_ROW_BROADCAST || op == UCL_EPI_PER_COL_SCALE;
}

// One step of the chain on the lane's 8 values.  If has_pre, `pre` is the step's tensor operand
// already fetched for exactly this position: an n-indexed vector or an AUX_LOAD row segment.
__device__ __forceinline__ void apply_step(float (&v)[8], const EpiStepDev &s, const EpiCtx &c, const Raw8 &pre,
                                           bool has_pre) {
    const int dt = s.dtype & 0xff;
    const bool vec = (s.dtype & 0x100) != 0;
    switch (s.op) {
    case UCL_EPI_SCALE:
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] *= s.p0;
        break;
    case UCL_EPI_BIAS:
    case UCL_EPI_ROW_BROADCAST:
    case UCL_EPI_PER_COL_SCALE: {
        float t[8];
        if (has_pre) decode8(pre, dt, t);
        else decode8(load8(step_ptr(s, c.group), dt, c.n, vec, c.nvalid), dt, t);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            if (s.op == UCL_EPI_PER_COL_SCALE) v[j] *= t[j];
            else v[j] += t[j];
        }
        break;
    }
    case UCL_EPI_PER_ROW_SCALE:
    case UCL_EPI_COL_BROADCAST: {
        float t = 0.f;
        if (c.nvalid > 0) {
            const void *base = step_ptr(s, c.group);
            t = dt == UCL_F32 ? ((const float *)base)[c.m] : bits_to_f32(((const uint16_t *)base)[c.m], dt);
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            if (s.op == UCL_EPI_PER_ROW_SCALE) v[j] *= t;
            else v[j] += t;
        }
        break;
    }
    case UCL_EPI_AUX_LOAD: {
        float t[8];
        if (has_pre) decode8(pre, dt, t);
        else decode8(load8(step_ptr(s, c.group), dt, (int64_t)c.batch * s.bs + c.m * s.ld + c.n, vec, c.nvalid), dt, t);
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] += s.p0 * t[j];
        break;
    }
    case UCL_EPI_AUX_STORE:
        store8((void *)step_ptr(s, c.group), dt, (int64_t)c.batch * s.bs + c.m * s.ld + c.n, v, vec, c.nvalid);
        break;
    case UCL_EPI_RELU:
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = act_f32<UCL_EPI_RELU>(v[j], s.p0, s.p1);
        break;
    case UCL_EPI_LEAKY_RELU:
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = act_f32<UCL_EPI_LEAKY_RELU>(v[j], s.p0, s.p1);
        break;
    case UCL_EPI_CLAMP:
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = act_f32<UCL_EPI_CLAMP>(v[j], s.p0, s.p1);
        break;
    case UCL_EPI_HARDSWISH:
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = act_f32<UCL_EPI_HARDSWISH>(v[j], s.p0, s.p1);
        break;
    case UCL_EPI_GELU_TANH:
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = act_f32<UCL_EPI_GELU_TANH>(v[j], s.p0, s.p1);
        break;
    case UCL_EPI_SILU:
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = act_f32<UCL_EPI_SILU>(v[j], s.p0, s.p1);
        break;
    case UCL_EPI_SIGMOID:
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = act_f32<UCL_EPI_SIGMOID>(v[j], s.p0, s.p1);
        break;
    case UCL_EPI_TANH:
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = act_f32<UCL_EPI_TANH>(v[j], s.p0, s.p1);
        break;
    case UCL_EPI_GELU_ERF:
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = act_f32<UCL_EPI_GELU_ERF>(v[j], s.p0, s.p1);
        break;
    case UCL_EPI_MISH:
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = act_f32<UCL_EPI_MISH>(v[j], s.p0, s.p1);
        break;
    case UCL_EPI_ELU:
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = act_f32<UCL_EPI_ELU>(v[j], s.p0, s.p1);
        break;
    default:
        break;
    }
}

// ------------------------------------------------------------------------------------------------

template <int TM_, int TN_, int TK_, int STAGES_, int DT_ /*inputs: 0 bf16, 1 fp16, 2 fp8 e4m3, 3 fp8 e5m2*/, int MODE_ /*0 gemm+batched, 1 grouped, 2 conv fprop, 3 conv dgrad, 4 conv wgrad*/,
          int LA_ /*OperandLayout of A*/, int LB_ /*OperandLayout of B*/, int SCHED_ = 0 /*tile scheduler: 0 default, 1 persistent, 2 stream-K*/,
          int PATCH_C_ = 0 /*kHalo: channels per pixel of the tensor the patch holds, 64 or 128 (0: 64 for fprop, 128 for dgrad)*/>
struct KernelCfg {
    static constexpr int TM = TM_, TN = TN_, TK = TK_, STAGES = STAGES_, MODE = MODE_, LA = LA_, LB = LB_;
    static constexpr int SCHED = SCHED_;
    static constexpr bool PERSIST = SCHED_ != 0;          // the workgroup walks several tiles (or pieces of tiles)
    static constexpr bool STREAMK = SCHED_ == 2;          // ... an equal run of (tile, 64-wide k range) iterations
    static_assert(SCHED_ >= 0 && SCHED_ <= 2, "tile scheduler code");
    static_assert(SCHED_ != 2 || (MODE_ == 0 && DT_ < 2), "stream-K: gemm / batched_gemm with 16-bit inputs");
    static constexpr int CPR = TK / 8;                            // 16-byte chunks per LDS row
    static constexpr int ROW_BYTES = TK * 2;
    static_assert(TK == 32 || TK == 64, "k-tile of 32 or 64 elements");
    static constexpr int DT = DT_;
    static_assert(DT_ >= 0 && DT_ <= 3, "input type code");
    static_assert(DT_ < 2 || (LA_ == kKContig && LB_ == kKContig), "8-bit inputs: both operands contiguous along K");
    static constexpr int WAVES_M = 2, WAVES_N = 2;
    static constexpr int WTM = TM / WAVES_M, WTN = TN / WAVES_N;  // wave tile
    static constexpr int MI = WTM / 16, NI = WTN / 16;            // 16x16 MFMA blocks per wave
    static constexpr int KSTEPS = TK / 32;                        // MFMA k-steps (32 elements) per k-tile
    static constexpr bool HALO = LA_ == kHalo;
    // kHalo: the stage buffers hold B only; A is a resident patch of PATCH_ROWS pixels (rows of 64 or
    // 128 channels = 128 or 256 bytes; fprop: activations, data gradient: the output gradient) behind
    // them, whose last row stays zero for padded taps to read.
    static constexpr int A_BYTES = HALO ? 0 : TM * TK * 2, B_BYTES = TN * TK * 2;
    static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
    static constexpr int PIPE_BYTES = STAGES * STAGE_BYTES;
    static constexpr int HALO_MAX = 59;                           // pixels kept before and behind the tile's own
    static constexpr int PATCH_ROWS = TM + 2 * HALO_MAX + 2;      // a whole number of 8-row wave copies
    static constexpr int PATCH_C = PATCH_C_ ? PATCH_C_ : MODE_ == 3 ? 128 : 64;
    static_assert(PATCH_C == 64 || PATCH_C == 128, "patch pixels of 64 or 128 channels");
    static constexpr int PATCH_ROW_BYTES = PATCH_C * 2;
    static constexpr int PATCH_BYTES = HALO ? PATCH_ROWS * PATCH_ROW_BYTES : 0;
    static_assert(PATCH_ROWS % 8 == 0, "one copy instruction of a wave fills a whole number of patch rows");
    static_assert(!HALO || (TK == 32 && STAGES >= 3 && ((MODE_ == 2 && LB_ == kKContig) || (MODE_ == 3 && LB_ == kNDirect))),
                  "patch kernels: pipelined loop, k-tiles of 32 channels of a tap");
    // epilogue staging: per wave 32 rows x (WTN + 4) fp32 (16 bytes of padding per row)
    static constexpr int EPI_LD = TN / 2 + 4;
    static constexpr int EPI_BYTES = 4 * 32 * EPI_LD * 4;
    static constexpr int LDS_BYTES = PIPE_BYTES + PATCH_BYTES > EPI_BYTES ? PIPE_BYTES + PATCH_BYTES : EPI_BYTES;
    static constexpr int A_ITERS = HALO ? 0 : TM * CPR / kThreads;   // 16-byte chunks per thread per stage
    static constexpr int B_ITERS = TN * CPR / kThreads;
    static constexpr int ROWS_PER_ITER = kThreads / CPR;          // rows covered by one 256-thread copy
    static_assert(TM % 64 == 0 && TN % 64 == 0, "wave tile is a multiple of 32x32 (two 16-row MFMA blocks per staged epilogue block)");
    static_assert(LDS_BYTES <= kLdsBytesPerCU, "stages x tile exceed LDS");
    // Register budget: smaller tiles are built to let several workgroups share a CU (512 registers per
    // lane and SIMD, accumulators included), so that one workgroup's loads and stores overlap another's
    // MFMAs -- that is what the short-K, bandwidth-bound problems need.
    static constexpr int MIN_WAVES = TM * TN >= 256 * 256 ? 1 : TM * TN >= 256 * 128 ? 2 : TM * TN >= 128 * 128 ? 3 : 4;
    using Groups = typename std::conditional<MODE == 1, GroupTable, NoGroupTable>::type;
};

// Buffer resource (4 SGPRs) over `bytes` bytes at `base`: raw buffer, no stride, range-checked.
// Loads through it whose offset is >= bytes return zero, which is how rows beyond the problem edge,
// the K tail and the conv halo become zeros in LDS without a branch or a second address.
typedef __amdgpu_buffer_rsrc_t rsrc_t;
typedef __attribute__((ext_vector_type(2))) float f32x2_t;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
typedef __attribute__((ext_vector_type(2))) _Float16 f16x2_t;
// Cache policy of accesses to data that is touched exactly once (residual loads, 16-bit output stores
// whose wave instruction covers whole 128-byte lines): the non-temporal bit.  Measured on the grouped
// GEMM and conv workloads: 9 % and 7 % shorter launches, because less dirty output waits in L2 for the
// write-back at the end of the kernel.  fp32 outputs keep the default policy: a lane's 32 bytes go out
// as two instructions that each cover half of every line, and streaming those half lines was 29 % slower.
constexpr int kAuxStream = 2;
constexpr uint32_t kOobOffset = 0x80000000u;   // never inside a resource (sizes are kept below 2^31)
__device__ __forceinline__ rsrc_t buffer_rsrc(const void *base, uint32_t bytes) {
    // word 3: 32-bit data format, raw (unstructured) addressing
    return __builtin_amdgcn_make_buffer_rsrc((void *)base, (short)0, (int)bytes, 0x00020000);
}

// D(16x16, fp32) += A(16x32) * B(32x16): lane L supplies row/column L % 16 and the 8 consecutive k
// starting at 8 * (L / 16) of both operands; it receives column L % 16, rows 4 * (L / 16) .. + 3 of D.
// (Of the two shapes of the 16-bit MFMA this one sustains the higher rate on random data under the
// power limit: measured 2.03 vs 1.81 PFLOP/s for loops of nothing but MFMAs.)
// Written as an asm statement with the accumulator tied to an accumulation register: the compiler's
// register allocator otherwise shuffles the 64 four-register accumulators of a wave tile between the
// two register files inside the loop.  The statements are volatile, so MFMAs, LDS reads and copy
// instructions issue in source order, which is how the loop below spaces them.
template <int DT>
__device__ __forceinline__ void mfma16(f32x4_t &c, const u32x4_t &a, const u32x4_t &b) {
    if constexpr (DT == 1) asm volatile("v_mfma_f32_16x16x32_f16 %0, %1, %2, %0" : "+a"(c) : "v"(a), "v"(b));
    else if constexpr (DT == 0) asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(c) : "v"(a), "v"(b));
    else {
        // 8-bit inputs.  The kernel handles them as pairs: one 16-bit unit of every address computation
        // is two fp8 values, so a 16-byte fragment is 16 consecutive k of a lane's row / column, and a
        // "k-step" is 64 of them.  The 8-bit MFMA takes 8 k per lane: the low and the high half of the
        // fragment go through one MFMA each.  Which k a lane's bytes stand for is the same for both
        // operands, and every k of the k-step is held by exactly one lane and half: the two MFMAs add
        // up the 64 products of the k-step.
        const u32x2_t a0{a[0], a[1]}, a1{a[2], a[3]}, b0{b[0], b[1]}, b1{b[2], b[3]};
        if constexpr (DT == 2) {
            asm volatile("v_mfma_f32_16x16x32_fp8_fp8 %0, %1, %2, %0" : "+a"(c) : "v"(a0), "v"(b0));
            asm volatile("v_mfma_f32_16x16x32_fp8_fp8 %0, %1, %2, %0" : "+a"(c) : "v"(a1), "v"(b1));
        } else {
            asm volatile("v_mfma_f32_16x16x32_bf8_bf8 %0, %1, %2, %0" : "+a"(c) : "v"(a0), "v"(b0));
            asm volatile("v_mfma_f32_16x16x32_bf8_bf8 %0, %1, %2, %0" : "+a"(c) : "v"(a1), "v"(b1));
        }
    }
}

// D(16x16, fp32) += A(16x128) * B(128x16), 8-bit operands: 32 bytes per lane and operand.
template <int DT>
__device__ __forceinline__ void mfma128(f32x4_t &c, const u32x8_t &a, const u32x8_t &b) {
    if constexpr (DT == 2) asm volatile("v_mfma_f32_16x16x128_f8f6f4 %0, %1, %2, %0" : "+a"(c) : "v"(a), "v"(b));
    else asm volatile("v_mfma_f32_16x16x128_f8f6f4 %0, %1, %2, %0 cbsz:1 blgp:1" : "+a"(c) : "v"(a), "v"(b));
}

// A pointer that is the same in every lane, moved into scalar registers.
__device__ __forceinline__ const char *uniform_ptr(const char *q) {
    const uint64_t v = (uint64_t)(uintptr_t)q;
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return (const char *)(uintptr_t)(((uint64_t)hi << 32) | lo);
}

// Forces the accumulator to hold its value in an accumulation register at this point of the program.
__device__ __forceinline__ void pin_acc(f32x4_t &c) { asm volatile("" : "+a"(c)); }

// Keeps a fragment register allocated up to this point of the program (see drain_asm_reads).
__device__ __forceinline__ void keep_alive(const u32x4_t &x) { asm volatile("" ::"v"(x)); }

// First of the n items dealt to row block mi when they are spread over the first half of the
// mblocks row blocks.
constexpr int bshare(int mi, int mblocks, int n) {
    const int h = mblocks >= 2 ? mblocks / 2 : 1;
    return (mi < h ? mi : h) * n / h;
}

template <class Cfg>
__global__ __launch_bounds__(kThreads, Cfg::MIN_WAVES) void ucl_tile_kernel(const KParams p_arg, const typename Cfg::Groups gt) {
    constexpr int TM = Cfg::TM, TN = Cfg::TN, TK = Cfg::TK, STAGES = Cfg::STAGES;
    constexpr int MI = Cfg::MI, NI = Cfg::NI, MODE = Cfg::MODE, LA = Cfg::LA, LB = Cfg::LB;
    constexpr int A_ITERS = Cfg::A_ITERS, B_ITERS = Cfg::B_ITERS;
    constexpr bool kAnyReg = (LA == kMNContig) || (LB == kMNContig);
    constexpr int DMA_PER_TILE = (LA != kMNContig ? A_ITERS : 0) + (LB != kMNContig ? B_ITERS : 0);
    constexpr int KSTEPS = Cfg::KSTEPS;
    constexpr int CPR = Cfg::CPR, ROW_BYTES = Cfg::ROW_BYTES, RPI = Cfg::ROWS_PER_ITER;

    __shared__ __attribute__((aligned(1024))) char smem[Cfg::LDS_BYTES];

    // ---- tile schedule ---------------------------------------------------------------------
    // Default scheduler: the grid has one workgroup per tile (per tile and K slice with split-K) and
    // the loop below runs once.  Persistent scheduler: the grid has one workgroup per CU slot (a
    // multiple of 8, so a workgroup stays on the tile run of its XCD) and walks the tile order with
    // a stride of the grid size.
    // Stream-K scheduler: as many whole rounds of tiles as the grid divides are walked like the persistent
    // scheduler walks them (sk_rounds tiles per workgroup: workgroups that run side by side work on neighbouring
    // tiles and share their operands in L2).  The (tile, 64-wide k range) pairs of the remaining tiles are numbered
    // tile by tile and the workgroup with run g (streamk_run) takes the sk_q of them from g * sk_q on.  The loop variable
    // counts the k steps the workgroup has behind it (sk_ipt per whole tile); one pass of the loop body is one piece:
    // a whole tile ends in the epilogue as usual; a part of a tile goes to the workspace, and the workgroup that
    // delivers the last part of a tile adds the parts up in k order and runs the epilogue.
    typedef const __attribute__((address_space(4))) KParams ConstKParams;
    int wg_first = blockIdx.x, sk_end = 0;
    if constexpr (Cfg::STREAMK) {
        ConstKParams *p0 = (ConstKParams *)__builtin_amdgcn_kernarg_segment_ptr();
        const int rest = (p0->total_tiles - p0->sk_rounds * (int)gridDim.x) * p0->sk_ipt;     // k steps of the remaining tiles
        const int mine0 = streamk_run(blockIdx.x, gridDim.x, p0->sk_deal, p0->sk_ipt, p0->sk_q) * p0->sk_q;
        const int mine_n = rest - mine0 < p0->sk_q ? rest - mine0 : p0->sk_q;
        wg_first = 0;
        sk_end = p0->sk_rounds * p0->sk_ipt + (mine_n > 0 ? mine_n : 0);
        if (sk_end == 0) return;
    }
    for (int wg_id = wg_first;;) {
    // The kernel arguments are read through a pointer into the argument segment (p_arg is the first
    // argument).  Persistent kernels make that pointer opaque once per tile: the compiler would
    // otherwise load every argument ahead of the loop and keep all of them in registers across it.
    ConstKParams *pp = (ConstKParams *)__builtin_amdgcn_kernarg_segment_ptr();
    if constexpr (Cfg::PERSIST) asm volatile("" : "+s"(pp));
    ConstKParams &p = *pp;
    (void)p_arg;
    int tid_ = threadIdx.x;
    // (persistent kernels: everything derived from the thread index is worked out again for every tile,
    // or the compiler keeps all of it in registers across the whole loop and runs out of them)
    if constexpr (Cfg::PERSIST) asm volatile("" : "+v"(tid_));
    const int tid = tid_;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / Cfg::WAVES_N, wn = wave % Cfg::WAVES_N;
    // split-K (gemm / batched / wgrad): the (slice, tile) pairs are numbered slice by slice and that numbering is
    // dealt to the XCDs in runs, like tiles are: the tiles of one K slice, which read the same rows of A and B,
    // run side by side on one XCD and share them in its L2
    int slice = 0;
    int t = 0;
    int sk_k0 = 0, sk_k1 = 0;           // stream-K: the piece's range of 64-wide k steps within its tile
    if constexpr ((MODE == 0 || MODE == 4) && !Cfg::PERSIST) {
        if (p.split_k > 1 && p.split_phase != 2) {
            t = xcd_remap(wg_id, p.total_tiles * p.split_k);
            slice = t / p.total_tiles;
            t -= slice * p.total_tiles;
        } else {
            t = xcd_remap(wg_id, p.total_tiles);
        }
    } else if constexpr (Cfg::STREAMK) {
        // (nothing of a piece is kept across the mainloop: streamk_piece works it out from the loop variable)
        const StreamKPiece pc = streamk_piece(wg_id, sk_end, p.sk_rounds, p.sk_ipt, p.sk_q, p.sk_deal);
        t = xcd_remap(pc.tile, p.total_tiles);
        sk_k0 = pc.k0;
        sk_k1 = pc.k1;
    } else {
        t = xcd_remap(wg_id, p.total_tiles);
    }
    int batch = 0, group = -1, tm, tn;
    int Mloc = p.M;
    const char *Ab = (const char *)p.A;
    const char *Bb = (const char *)p.B;
    char *Db = (char *)p.D;
    if constexpr (MODE == 1) {
        group = find_group(gt.tile_start, p.groups, t);
        t -= gt.tile_start[group];
        Mloc = gt.m[group];
        band_raster(t, (Mloc + TM - 1) / TM, p.tiles_n, p.raster, tm, tn);
        // The per-group pointers come out of device memory.  Where the compiler may not use a scalar load for them
        // (persistent kernels: the table is read again after the previous tile's stores) they arrive in vector
        // registers, and a buffer resource built on such a pointer makes every global -> LDS copy a readfirstlane
        // loop.  They are the same in every lane: say so.
        Ab = uniform_ptr((const char *)p.A_g[group]);
        Bb = uniform_ptr((const char *)p.B_g[group]);
        Db = (char *)uniform_ptr((const char *)p.D_g[group]);
    } else {
        batch = t / p.tiles_per_batch;
        t -= batch * p.tiles_per_batch;
        band_raster(t, p.tiles_m, p.tiles_n, p.raster, tm, tn);
        Ab += (int64_t)batch * p.a_bs * 2;
        Bb += (int64_t)batch * p.b_bs * 2;
    }
    const int m0 = tm * TM, n0 = tn * TN;
    int k_len = p.K;
    if constexpr ((MODE == 0 || MODE == 4) && !Cfg::PERSIST) {
        if (p.split_k > 1 || p.split_phase == 2) {
            // this slice's K range (a multiple of 64 long, so operand rows stay 16-byte aligned)
            const int kb = slice * p.k_per_slice;
            k_len = p.K - kb < p.k_per_slice ? p.K - kb : p.k_per_slice;
            // the second launch of a parallel split-K only adds up the partial tiles: with K = 0 the
            // loops below run no k-tile (their prologue copies land in LDS and are never read)
            if (p.split_phase == 2) k_len = 0;
            Ab += (int64_t)kb * (LA == kKContig ? 1 : p.lda) * 2;
            Bb += (int64_t)kb * (LB == kKContig ? 1 : p.ldb) * 2;
        }
    }
    if constexpr (Cfg::STREAMK) {
        const int kb = sk_k0 * 64;
        k_len = (sk_k1 * 64 < p.K ? sk_k1 * 64 : p.K) - kb;
        Ab += (int64_t)kb * (LA == kKContig ? 1 : p.lda) * 2;
        Bb += (int64_t)kb * (LB == kKContig ? 1 : p.ldb) * 2;
    }
    const int K = k_len;
    const int Kr = K > 0 ? K : 1;                      // rows of k a directly copied operand's resource covers (K = 0: see above)
    const int KT = (K + TK - 1) / TK;
    const bool k_tail = (K % TK) != 0;

    // ---- loader set-up -----------------------------------------------------------------------
    // Slot s = i*256 + tid of a stage holds row s/CPR = i*RPI + tid/CPR, chunk position tid%CPR; the
    // source chunk is that position XOR swz(row), the same for every i (RPI is a multiple of 16).
    const int l_row = tid / CPR;
    const int l_chunk = (tid % CPR) ^ lds_swz<CPR>(l_row);
    const int l_kc = l_chunk * 8;                        // first k of this thread's chunk within a k-tile
    // K-contiguous operands: one scalar buffer resource per operand over the tile's row panel, and per
    // thread one loop-invariant 32-bit byte offset per slot; the k position advances through the
    // scalar offset of the load, so a load costs no vector ALU instruction in the steady state.
    rsrc_t a_rsrc = buffer_rsrc(nullptr, 0), b_rsrc = buffer_rsrc(nullptr, 0);
    uint32_t a_off[LA == kMNContig || LA == kHalo ? 1 : A_ITERS], b_off[LB == kMNContig ? 1 : B_ITERS];
    int a_h0[LA == kIm2col ? A_ITERS : 1], a_w0[LA == kIm2col ? A_ITERS : 1];
    int a_ci = 0, a_r = 0, a_s = 0;                      // im2col: decomposition of k = l_kc + kt*TK
    u32x4_t a_stage[LA == kMNContig ? A_ITERS : 1], b_stage[LB == kMNContig ? B_ITERS : 1];

    if constexpr (LA == kKContig) {
        const int rows = Mloc - m0 < TM ? Mloc - m0 : TM;              // rows of the panel that exist
        a_rsrc = buffer_rsrc(Ab + (int64_t)m0 * p.lda * 2, (uint32_t)(((int64_t)(rows - 1) * p.lda + K) * 2));
#pragma unroll
        for (int i = 0; i < A_ITERS; ++i)
            a_off[i] = (uint32_t)(((int64_t)(i * RPI + l_row) * p.lda + l_kc) * 2);   // rows past the edge: out of range
    } else if constexpr (LA == kMDirect) {
        // the stage holds TK rows (k) of TM elements (m), laid out and swizzled like the kNDirect B stage
        constexpr int CPRA = TM / 8, RPIA = kThreads / CPRA;
        a_rsrc = buffer_rsrc(Ab + (int64_t)m0 * 2, (uint32_t)(((int64_t)(Kr - 1) * p.lda + (Mloc - m0)) * 2));
#pragma unroll
        for (int i = 0; i < A_ITERS; ++i) {
            const int row = i * RPIA + tid / CPRA;
            const int chunk = (tid % CPRA) ^ ((((row & 3) << 1) | (((row >> 3) & 3) << 3)) & (CPRA - 1));
            a_off[i] = (uint32_t)(((int64_t)row * p.lda + chunk * 8) * 2);
        }
    } else if constexpr (LA == kIm2col) {
        a_rsrc = buffer_rsrc(Ab, (uint32_t)p.a_bytes);
#pragma unroll
        for (int i = 0; i < A_ITERS; ++i) {
            int row = m0 + i * RPI + l_row;
            row = row < Mloc ? row : Mloc - 1;
            const int q = row % p.cQ;
            const int pq = row / p.cQ;
            const int pp = pq % p.cP;
            const int nb = pq / p.cP;
            if constexpr (MODE == 3) {
                // data gradient: the row is an INPUT pixel (h, w) = (pp, q); tap (r, s) pairs it with the
                // gradient pixel ((h + pad - r*dil) / stride, ...) where that division is exact.  The
                // gathered tensor is dy: "image" extents cH x cW = P x Q, cC = its channels.
                a_h0[i] = pp + p.pad_h;
                a_w0[i] = q + p.pad_w;
                a_off[i] = (uint32_t)(nb * p.cH * p.cW * p.cC * 2);
            } else {
                a_h0[i] = pp * p.str_h - p.pad_h;
                a_w0[i] = q * p.str_w - p.pad_w;
                // byte offset of x[nb, h0, w0, 0] (may be negative); only used at taps inside the image
                a_off[i] = (uint32_t)(((nb * p.cH + a_h0[i]) * p.cW + a_w0[i]) * p.cC * 2);
            }
        }
        a_ci = l_kc % p.cC;
        const int tap = l_kc / p.cC;
        a_r = tap / p.cS;
        a_s = tap % p.cS;
    }
    if constexpr (LB == kKContig) {
        const int rows = p.N - n0 < TN ? p.N - n0 : TN;
        b_rsrc = buffer_rsrc(Bb + (int64_t)n0 * p.ldb * 2, (uint32_t)(((int64_t)(rows - 1) * p.ldb + K) * 2));
#pragma unroll
        for (int i = 0; i < B_ITERS; ++i)
            b_off[i] = (uint32_t)(((int64_t)(i * RPI + l_row) * p.ldb + l_kc) * 2);
    }
    // kNDirect: the stage holds TK rows (k) of TN elements (n); slot s = i*256 + tid is row s / CPRB,
    // chunk position s % CPRB, filled from chunk position XOR nd_swz(row).  The resource starts at
    // column n0 of row 0 and ends with the matrix, so rows past K read zeros; columns past N read
    // elements of the following row, which only ever reach accumulators that are not stored.
    constexpr int CPRB = TN / 8, RPIB = kThreads / CPRB;          // chunks per row, rows per 256-thread copy
    auto nd_swz = [](int row) { return (((row & 3) << 1) | (((row >> 3) & 3) << 3)) & (CPRB - 1); };
    const int nd_row = tid / CPRB;
    // Per-slot state of the two gathered forms of such a B stage.
    // MODE 3 (data gradient): GEMM row k = (r*S + s)*Ko + ko of B is filter row w[ko, r, s, :]: the slot
    // keeps (ko, tap) of its row and steps ko by TK per k-tile.
    // MODE 4 (weight gradient): GEMM row k is output pixel (n, p, q), GEMM column (r, s, c): the slot's 8
    // columns are 8 channels of ONE tap (C is a multiple of 8), fixed for the whole loop; its pixel
    // steps by TK per k-tile.  Every slot reads x[n, p*stride - pad + r*dil, q*stride - pad + s*dil, c..c+7].
    constexpr bool kBGather = LB == kNDirect && (MODE == 3 || MODE == 4);
    int g_a[kBGather ? B_ITERS : 1], g_b[kBGather ? B_ITERS : 1];          // MODE 3: ko, tap   MODE 4: q, p
    int g_dh[MODE == 4 && kBGather ? B_ITERS : 1], g_dw[MODE == 4 && kBGather ? B_ITERS : 1];
    uint32_t g_img[MODE == 4 && kBGather ? B_ITERS : 1];                   // byte offset of the slot's image
    if constexpr (LB == kNDirect && MODE == 3) {
        b_rsrc = buffer_rsrc(Bb + (int64_t)n0 * 2, (uint32_t)(p.b_bytes - (int64_t)n0 * 2));
#pragma unroll
        for (int i = 0; i < B_ITERS; ++i) {
            const int row = i * RPIB + nd_row;
            const int chunk = (tid % CPRB) ^ nd_swz(row);
            b_off[i] = (uint32_t)(chunk * 16);
            g_b[i] = row / p.cC;
            g_a[i] = row - g_b[i] * p.cC;
        }
    } else if constexpr (LB == kNDirect && MODE == 4) {
        b_rsrc = buffer_rsrc(Bb, (uint32_t)p.b_bytes);
        const int kb = p.split_k > 1 && p.split_phase != 2 ? slice * p.k_per_slice : 0;
#pragma unroll
        for (int i = 0; i < B_ITERS; ++i) {
            const int row = i * RPIB + nd_row;
            const int chunk = (tid % CPRB) ^ nd_swz(row);
            const int n = n0 + chunk * 8;                       // first of the slot's 8 GEMM columns
            const int tap = n / p.cC, c = n - tap * p.cC;
            const int r = tap / p.cS, sx = tap - r * p.cS;
            // a column past N never reaches a stored accumulator: give it a tap far outside every image
            g_dh[i] = n < p.N ? r * p.dil_h - p.pad_h : -(1 << 28);
            g_dw[i] = sx * p.dil_w - p.pad_w;
            b_off[i] = (uint32_t)(c * 2);
            const int pix = kb + row;                            // (n, p, q) of the slot's row in k-tile 0
            const int pq = p.cP * p.cQ;
            const int img = pix / pq, rem = pix - img * pq;
            g_b[i] = rem / p.cQ;
            g_a[i] = rem - g_b[i] * p.cQ;
            g_img[i] = (uint32_t)img * (uint32_t)(p.cH * p.cW * p.cC * 2);
        }
    } else if constexpr (LB == kNDirect) {
        b_rsrc = buffer_rsrc(Bb + (int64_t)n0 * 2, (uint32_t)(((int64_t)(Kr - 1) * p.ldb + (p.N - n0)) * 2));
#pragma unroll
        for (int i = 0; i < B_ITERS; ++i) {
            const int row = i * RPIB + nd_row;
            const int chunk = (tid % CPRB) ^ nd_swz(row);
            b_off[i] = (uint32_t)(((int64_t)row * p.ldb + chunk * 8) * 2);
        }
    }
    // Offset of gathered slot i for the k-tile it stands at, then the slot steps on by one k-tile.
    auto b_gather_off = [&](auto i_, bool kok) __attribute__((always_inline)) -> uint32_t {
        constexpr int i = decltype(i_)::value;
        uint32_t off = kOobOffset;
        if constexpr (kBGather && MODE == 3) {
            if (kok) off = (uint32_t)((g_a[i] * (int)p.ldb + g_b[i] * p.N) * 2) + b_off[i];
            g_a[i] += TK;
            while (g_a[i] >= p.cC) { g_a[i] -= p.cC; ++g_b[i]; }
        } else if constexpr (kBGather && MODE == 4) {
            const int h = g_b[i] * p.str_h + g_dh[i], w = g_a[i] * p.str_w + g_dw[i];
            if (kok && (unsigned)h < (unsigned)p.cH && (unsigned)w < (unsigned)p.cW)
                off = g_img[i] + (uint32_t)((h * p.cW + w) * p.cC * 2) + b_off[i];
            g_a[i] += TK;
            while (g_a[i] >= p.cQ) {
                g_a[i] -= p.cQ;
                if (++g_b[i] == p.cP) { g_b[i] = 0; g_img[i] += (uint32_t)(p.cH * p.cW * p.cC * 2); }
            }
        }
        return off;
    };
    // Data gradient: offset of gather slot i of A at the tap (a_r, a_s) and channel offset a_ci the loader stands at.
    auto a_gather_off = [&](auto i_, bool kok) __attribute__((always_inline)) -> uint32_t {
        constexpr int i = decltype(i_)::value;
        if constexpr (LA == kIm2col && MODE == 3) {
            const int th = a_h0[i] - a_r * p.dil_h, tw = a_w0[i] - a_s * p.dil_w;
            int hh = th, ww = tw;
            bool ok = kok && th >= 0 && tw >= 0;
            if (p.str_h != 1) { hh = th / p.str_h; ok = ok && hh * p.str_h == th; }
            if (p.str_w != 1) { ww = tw / p.str_w; ok = ok && ww * p.str_w == tw; }
            ok = ok && hh < p.cH && ww < p.cW;
            return ok ? a_off[i] + (uint32_t)(((hh * p.cW + ww) * p.cC + a_ci) * 2) : kOobOffset;
        } else {
            return kOobOffset;
        }
    };

    // Resident activation patch (kHalo).  Output pixel m of a 3x3 / stride 1 / pad 1 convolution reads
    // input pixels m + dy*W + dx of the flattened [N*H*W] pixel sequence, except where the tap leaves
    // the image.  Patch row r holds pixel m0 - (W + 1) + r (one contiguous global range, rows outside
    // the tensor are zero-filled by the range check), its 16-byte chunks XOR-swizzled like a 128-byte
    // stage row.  Per 16-row MFMA block and lane, one byte says for each of the eight outer taps
    // whether it leaves the image at the lane's pixel (first / last column, first / last row, and the
    // four corner combinations); such a tap reads the zero row.
    // Pixels of 128 channels: rows of 256 bytes, sixteen chunks XORed with the row number (16 consecutive rows at
    // one logical chunk then hit 16 different 16-byte slots), four k-tiles per tap instead of two.
    // Data gradient (same filter geometry): input pixel m reads gradient pixels m - dy*W - dx, the taps mirrored,
    // from a patch of the output gradient.
    constexpr int PRB = Cfg::PATCH_ROW_BYTES, PCPR = PRB / 16, KPT = PRB / 64, kTapSign = MODE == 3 ? -1 : 1;
    auto patch_swz = [&](int r) __attribute__((always_inline)) -> int {
        if constexpr (PCPR == 8) return lds_swz<8>(r);
        else return r & 15;
    };
    constexpr int kPatchOff = Cfg::PIPE_BYTES, kZeroRow = Cfg::PIPE_BYTES + (Cfg::PATCH_ROWS - 1) * PRB;
    uint32_t h_flags[2] = {0u, 0u};                              // row blocks 0-3, 4-7
    int h_r0 = 0;
    if constexpr (LA == kHalo) {
        a_rsrc = buffer_rsrc(Ab, (uint32_t)p.a_bytes);
        const int halo = p.cW + 1;
        const int f_row_ = lane & 15;
        h_r0 = wm * Cfg::WTM + f_row_ + halo;
#pragma unroll
        for (int blk = 0; blk < MI; ++blk) {
            int pix = m0 + wm * Cfg::WTM + blk * 16 + f_row_;
            pix = pix < Mloc ? pix : Mloc - 1;
            const int w = pix % p.cW, h = (pix / p.cW) % p.cH;
            const bool w0 = w == 0, wl = w == p.cW - 1, h0 = h == 0, hl = h == p.cH - 1;
            const uint32_t f = (w0 ? 1u : 0u) | (wl ? 2u : 0u) | (h0 ? 4u : 0u) | (hl ? 8u : 0u) | (w0 || h0 ? 16u : 0u) |
                               (wl || h0 ? 32u : 0u) | (w0 || hl ? 64u : 0u) | (wl || hl ? 128u : 0u);
            h_flags[blk >> 2] |= f << (8 * (blk & 3));
        }
        constexpr int CHUNKS = Cfg::PATCH_ROWS * PCPR, SLOTS = (CHUNKS + kThreads - 1) / kThreads;
        static_assert(MI <= 8, "one flag byte per row block");
        // rows the tile does not need (the last one among them: TM + 2 halo < PATCH_ROWS) are copied
        // from an out-of-range offset, i.e. zero-filled
#pragma unroll
        for (int i = 0; i < SLOTS; ++i) {
            if (i * kThreads + wave * 64 < CHUNKS) {             // wave-uniform: the last slot may be partial
                const int q = i * kThreads + tid;                // 16-byte slot of the patch
                const int r = q / PCPR;
                const int chunk = (q % PCPR) ^ patch_swz(r);
                const int pix = m0 - halo + r;
                const bool ok = pix >= 0 && pix < Mloc && r < TM + 2 * halo;
                const uint32_t off = ok ? (uint32_t)(pix * PCPR + chunk) * 16u : kOobOffset;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(a_rsrc, UCL_LDS_PTR(smem + kPatchOff + (i * kThreads + wave * 64) * 16), 16, off, 0, 0, 0);
            }
        }
    }
    // Patch addressing of k-tile KT (32 of a tap's channels; dy, dx and the channel range are
    // compile-time): byte address of this lane's fragment chunk for row block 0.
    auto halo_base = [&](auto kt_) __attribute__((always_inline)) {
        constexpr int KT_ = decltype(kt_)::value, tap = KT_ / KPT, dy = kTapSign * (tap / 3 - 1), dx = kTapSign * (tap % 3 - 1);
        const int r = h_r0 + dy * p.cW + dx;
        const int chunk = ((KT_ % KPT) << 2) | (lane >> 4);
        return kPatchOff + r * PRB + ((chunk ^ patch_swz(r)) << 4);
    };
    // Fragment of row block BLK: one vector ALU instruction spreads the tap's flag bit over a register
    // (-1: the tap leaves the image at this lane's pixel), one merges the zero row's address in under
    // that mask, then the 128-bit LDS read.  Written as asm so that they stay where they are placed
    // between the MFMAs.
    auto halo_test = [&](auto kt_, auto blk_) __attribute__((always_inline)) -> int {
        constexpr int KT_ = decltype(kt_)::value, BLK = decltype(blk_)::value, tap = KT_ / KPT, dy = kTapSign * (tap / 3 - 1), dx = kTapSign * (tap % 3 - 1);
        constexpr int bit = dy == 0 ? (dx < 0 ? 0 : 1) : dx == 0 ? (dy < 0 ? 2 : 3) : 4 + (dx > 0 ? 1 : 0) + (dy > 0 ? 2 : 0);
        int dead = 0;
        if constexpr (dx != 0 || dy != 0)
            asm volatile("v_bfe_i32 %0, %1, %2, 1" : "=v"(dead) : "v"(h_flags[BLK >> 2]), "n"(8 * (BLK & 3) + bit));
        return dead;
    };
    auto halo_read = [&](auto kt_, auto blk_, int base, int dead) __attribute__((always_inline)) {
        constexpr int KT_ = decltype(kt_)::value, BLK = decltype(blk_)::value, tap = KT_ / KPT, dy = kTapSign * (tap / 3 - 1), dx = kTapSign * (tap % 3 - 1);
        int addr = base;
        if constexpr (dx != 0 || dy != 0)                        // the read adds BLK * 16 rows as its immediate offset
            asm volatile("v_bfi_b32 %0, %1, %2, %3" : "=v"(addr) : "v"(dead), "s"(kZeroRow - BLK * 16 * PRB), "v"(base));
        return *(const u32x4_t *)(smem + addr + BLK * 16 * PRB);
    };

    // Issue the copies of k-tile `kt` into stage buffer `buf`.  K-contiguous and im2col operands:
    // one 128-bit global -> LDS load per slot (lane L of a wave lands at dst + 16 L).  M/N-contiguous
    // operands: 128-bit loads into registers, written (transposed) by commit_regs.  CHECK_K adds the
    // K-tail test; full k-tiles skip it.
    // PART: 0 = both operands, 1 = A only, 2 = B only (the deep pipelines spread the two halves of a
    // stage's loads over different k-steps).
    auto issue_part = [&](auto check_k_, auto part_, int kt, int buf) __attribute__((always_inline)) {
        constexpr bool CHECK_K = decltype(check_k_)::value;
        constexpr int PART = decltype(part_)::value;
        char *sA = smem + buf * Cfg::STAGE_BYTES;
        char *sB = sA + Cfg::A_BYTES;
        const int k0 = kt * TK;
        const bool kok = !CHECK_K || (k0 + l_kc < K);
        if constexpr (PART == 2 || LA == kHalo) {
        } else if constexpr (LA == kKContig) {
#pragma unroll
            for (int i = 0; i < A_ITERS; ++i) {
                char *dst = sA + (i * kThreads + wave * 64) * 16;
                const uint32_t off = CHECK_K ? (kok ? a_off[i] : kOobOffset) : a_off[i];
                __builtin_amdgcn_raw_ptr_buffer_load_lds(a_rsrc, UCL_LDS_PTR(dst), 16, off, k0 * 2, 0, 0);
            }
        } else if constexpr (LA == kMDirect) {
            constexpr int RPIA = kThreads / (TM / 8);
            const uint32_t krow = (uint32_t)k0 * (uint32_t)p.lda * 2u;       // validated: K * lda * 2 < 2^31
#pragma unroll
            for (int i = 0; i < A_ITERS; ++i) {
                char *dst = sA + (i * kThreads + wave * 64) * 16;
                const uint32_t off = CHECK_K ? (k0 + i * RPIA + tid / (TM / 8) < K ? a_off[i] : kOobOffset) : a_off[i];
                __builtin_amdgcn_raw_ptr_buffer_load_lds(a_rsrc, UCL_LDS_PTR(dst), 16, off, krow, 0, 0);
            }
        } else if constexpr (LA == kIm2col) {
            if constexpr (MODE == 3) {
                static_for<A_ITERS>([&](auto i_) {
                    constexpr int i = decltype(i_)::value;
                    char *dst = sA + (i * kThreads + wave * 64) * 16;
                    const uint32_t off = a_gather_off(i_, kok);
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(a_rsrc, UCL_LDS_PTR(dst), 16, off, 0, 0, 0);
                });
            } else {
                const int dh = a_r * p.dil_h, dw = a_s * p.dil_w;
                const uint32_t tap_off = (uint32_t)(((dh * p.cW + dw) * p.cC + a_ci) * 2);
#pragma unroll
                for (int i = 0; i < A_ITERS; ++i) {
                    char *dst = sA + (i * kThreads + wave * 64) * 16;
                    const int h = a_h0[i] + dh, w = a_w0[i] + dw;
                    const bool ok = kok && (unsigned)h < (unsigned)p.cH && (unsigned)w < (unsigned)p.cW;
                    const uint32_t off = ok ? a_off[i] + tap_off : kOobOffset;
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(a_rsrc, UCL_LDS_PTR(dst), 16, off, 0, 0, 0);
                }
            }
            // advance k by one k-tile: (ci, s, r) += TK channels
            a_ci += TK;
            while (a_ci >= p.cC) {
                a_ci -= p.cC;
                if (++a_s == p.cS) { a_s = 0; ++a_r; }
            }
        } else {   // A contiguous along M: element (m, k) at k*lda + m
#pragma unroll
            for (int i = 0; i < A_ITERS; ++i) {
                const int s = i * kThreads + tid;
                const int krow = s / (TM / 8), mc = s % (TM / 8);
                int m = m0 + mc * 8;
                m = m + 8 <= Mloc ? m : Mloc - 8;                  // Mloc % 8 == 0 (validated)
                const int k = k0 + krow;
                a_stage[i] = k < K ? *(const u32x4_t *)(Ab + ((int64_t)k * p.lda + m) * 2) : u32x4_t{0, 0, 0, 0};
            }
        }
        if constexpr (PART == 1) {
        } else if constexpr (LB == kKContig) {
#pragma unroll
            for (int i = 0; i < B_ITERS; ++i) {
                char *dst = sB + (i * kThreads + wave * 64) * 16;
                const uint32_t off = CHECK_K ? (kok ? b_off[i] : kOobOffset) : b_off[i];
                __builtin_amdgcn_raw_ptr_buffer_load_lds(b_rsrc, UCL_LDS_PTR(dst), 16, off, k0 * 2, 0, 0);
            }
        } else if constexpr (kBGather) {
            static_for<B_ITERS>([&](auto i_) {
                constexpr int i = decltype(i_)::value;
                char *dst = sB + (i * kThreads + wave * 64) * 16;
                const uint32_t off = b_gather_off(i_, !CHECK_K || k0 + i * RPIB + nd_row < K);
                __builtin_amdgcn_raw_ptr_buffer_load_lds(b_rsrc, UCL_LDS_PTR(dst), 16, off, 0, 0, 0);
            });
        } else if constexpr (LB == kNDirect) {
            const uint32_t krow = (uint32_t)k0 * (uint32_t)p.ldb * 2u;       // validated: K * ldb * 2 < 2^31
#pragma unroll
            for (int i = 0; i < B_ITERS; ++i) {
                char *dst = sB + (i * kThreads + wave * 64) * 16;
                const uint32_t off = CHECK_K ? (k0 + i * RPIB + nd_row < K ? b_off[i] : kOobOffset) : b_off[i];
                __builtin_amdgcn_raw_ptr_buffer_load_lds(b_rsrc, UCL_LDS_PTR(dst), 16, off, krow, 0, 0);
            }
        } else {   // B contiguous along N: element (k, n) at k*ldb + n
#pragma unroll
            for (int i = 0; i < B_ITERS; ++i) {
                const int s = i * kThreads + tid;
                const int krow = s / (TN / 8), nc = s % (TN / 8);
                int n = n0 + nc * 8;
                n = n + 8 <= p.N ? n : p.N - 8;                    // N % 8 == 0 (validated)
                const int k = k0 + krow;
                b_stage[i] = k < K ? *(const u32x4_t *)(Bb + ((int64_t)k * p.ldb + n) * 2) : u32x4_t{0, 0, 0, 0};
            }
        }
    };
    // One copy instruction of k-tile `kt`: slot IDX counts the A slots first, then the B slots.  The
    // deep pipeline deals these out one at a time between the MFMAs (K-contiguous / im2col operands).
    auto issue_one = [&](auto check_k_, auto idx_, int kt, int buf) __attribute__((always_inline)) {
        constexpr bool CHECK_K = decltype(check_k_)::value;
        constexpr int IDX = decltype(idx_)::value;
        char *sA = smem + buf * Cfg::STAGE_BYTES;
        char *sB = sA + Cfg::A_BYTES;
        const int k0 = kt * TK;
        const bool kok = !CHECK_K || (k0 + l_kc < K);
        if constexpr (IDX < A_ITERS) {
            constexpr int i = IDX;
            char *dst = sA + (i * kThreads + wave * 64) * 16;
            if constexpr (LA == kKContig) {
                const uint32_t off = CHECK_K ? (kok ? a_off[i] : kOobOffset) : a_off[i];
                __builtin_amdgcn_raw_ptr_buffer_load_lds(a_rsrc, UCL_LDS_PTR(dst), 16, off, k0 * 2, 0, 0);
            } else if constexpr (LA == kMDirect) {
                constexpr int RPIA = kThreads / (TM / 8);
                const uint32_t off = CHECK_K ? (k0 + i * RPIA + tid / (TM / 8) < K ? a_off[i] : kOobOffset) : a_off[i];
                __builtin_amdgcn_raw_ptr_buffer_load_lds(a_rsrc, UCL_LDS_PTR(dst), 16, off, (uint32_t)k0 * (uint32_t)p.lda * 2u, 0, 0);
            } else {
                if constexpr (MODE == 3) {
                    const uint32_t off = a_gather_off(std::integral_constant<int, i>{}, kok);
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(a_rsrc, UCL_LDS_PTR(dst), 16, off, 0, 0, 0);
                } else {
                    const int dh = a_r * p.dil_h, dw = a_s * p.dil_w;
                    const uint32_t tap_off = (uint32_t)(((dh * p.cW + dw) * p.cC + a_ci) * 2);
                    const int h = a_h0[i] + dh, w = a_w0[i] + dw;
                    const bool ok = kok && (unsigned)h < (unsigned)p.cH && (unsigned)w < (unsigned)p.cW;
                    const uint32_t off = ok ? a_off[i] + tap_off : kOobOffset;
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(a_rsrc, UCL_LDS_PTR(dst), 16, off, 0, 0, 0);
                }
                if constexpr (i == A_ITERS - 1) {     // advance k by one k-tile: (ci, s, r) += TK channels
                    a_ci += TK;
                    while (a_ci >= p.cC) {
                        a_ci -= p.cC;
                        if (++a_s == p.cS) { a_s = 0; ++a_r; }
                    }
                }
            }
        } else {
            constexpr int i = IDX - A_ITERS;
            char *dst = sB + (i * kThreads + wave * 64) * 16;
            if constexpr (kBGather) {
                const uint32_t off = b_gather_off(std::integral_constant<int, i>{}, !CHECK_K || k0 + i * RPIB + nd_row < K);
                __builtin_amdgcn_raw_ptr_buffer_load_lds(b_rsrc, UCL_LDS_PTR(dst), 16, off, 0, 0, 0);
            } else if constexpr (LB == kNDirect) {
                const uint32_t off = CHECK_K ? (k0 + i * RPIB + nd_row < K ? b_off[i] : kOobOffset) : b_off[i];
                __builtin_amdgcn_raw_ptr_buffer_load_lds(b_rsrc, UCL_LDS_PTR(dst), 16, off, (uint32_t)k0 * (uint32_t)p.ldb * 2u, 0, 0);
            } else {
                const uint32_t off = CHECK_K ? (kok ? b_off[i] : kOobOffset) : b_off[i];
                __builtin_amdgcn_raw_ptr_buffer_load_lds(b_rsrc, UCL_LDS_PTR(dst), 16, off, k0 * 2, 0, 0);
            }
        }
    };
    auto issue_tile = [&](auto check_k_, int kt, int buf) __attribute__((always_inline)) {
        issue_part(check_k_, std::integral_constant<int, 0>{}, kt, buf);
    };
    // only the last k-tile can be partial
    auto issue = [&](int kt, int buf) {
        if (k_tail && kt == KT - 1) issue_tile(std::true_type{}, kt, buf);
        else issue_tile(std::false_type{}, kt, buf);
    };

    // Transposing write of the register-staged operands into stage buffer `buf`.
    auto commit_regs = [&](int buf) {
        char *sA = smem + buf * Cfg::STAGE_BYTES;
        char *sB = sA + Cfg::A_BYTES;
        if constexpr (LA == kMNContig) {
#pragma unroll
            for (int i = 0; i < A_ITERS; ++i) {
                const int s = i * kThreads + tid;
                const int krow = s / (TM / 8), mc = s % (TM / 8);
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const int row = mc * 8 + j;
                    const uint32_t w = a_stage[i][j >> 1];
                    const uint16_t e = (j & 1) ? (uint16_t)(w >> 16) : (uint16_t)(w & 0xffffu);
                    *(uint16_t *)(sA + row * ROW_BYTES + (((krow >> 3) ^ lds_swz<CPR>(row)) << 4) + (krow & 7) * 2) = e;
                }
            }
        }
        if constexpr (LB == kMNContig) {
#pragma unroll
            for (int i = 0; i < B_ITERS; ++i) {
                const int s = i * kThreads + tid;
                const int krow = s / (TN / 8), nc = s % (TN / 8);
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const int row = nc * 8 + j;
                    const uint32_t w = b_stage[i][j >> 1];
                    const uint16_t e = (j & 1) ? (uint16_t)(w >> 16) : (uint16_t)(w & 0xffffu);
                    *(uint16_t *)(sB + row * ROW_BYTES + (((krow >> 3) ^ lds_swz<CPR>(row)) << 4) + (krow & 7) * 2) = e;
                }
            }
        }
    };

    // Small tiles serve short, latency-bound problems: their bias vector (and, grouped, the pointer to
    // it) is requested here, ahead of the mainloop, instead of at the head of the epilogue where the
    // wave would sit out a memory round trip.  (The large tiles have no registers to spare for it.)
    constexpr bool kBiasAhead = Cfg::MIN_WAVES >= 4;
    Raw8 bias_ahead;
    bias_ahead.lo = bias_ahead.hi = u32x4_t{0u, 0u, 0u, 0u};
    bias_ahead.packed = false;
    if constexpr (kBiasAhead) {
        if (p.fused.enabled && p.fused.has_bias) {
            const int n_first = n0 + wn * Cfg::WTN + (lane % (Cfg::WTN / 8)) * 8;
            const void *bp = MODE == 1 ? ((const void *const *)p.fused.bias)[group] : p.fused.bias;
            bias_ahead = load8(bp, p.fused.bias_dt & 0xff, n_first, (p.fused.bias_dt & 0x100) != 0, p.N - n_first);
        }
    }

    // ---- accumulators and fragment addressing -----------------------------------------------
    f32x4_t acc[MI][NI];
    static_for<MI>([&](auto mi) {
        static_for<NI>([&](auto ni) { acc[mi][ni] = f32x4_t{0.f, 0.f, 0.f, 0.f}; });
    });

    const int f_row = lane & 15, f_kg = lane >> 4;
    // byte offset of this lane's fragment chunk inside its LDS row for k-step 0 (chunk f_kg XOR
    // swz(row)); k-step kk XORs it with kk*64 (chunk index 4kk + f_kg)
    const int f_x = (f_kg ^ lds_swz<CPR>(f_row)) << 4;
    const int a_frag_base = (wm * Cfg::WTM + f_row) * ROW_BYTES;
    const int b_frag_base = Cfg::A_BYTES + (wn * Cfg::WTN + f_row) * ROW_BYTES;
    auto frag = [&](const char *sbase, int base, int blk, int kk) __attribute__((always_inline)) {
        return *(const u32x4_t *)(sbase + base + blk * 16 * ROW_BYTES + (f_x ^ (kk << 6)));
    };
    // B fragment of column block `blk`, k-step `kk`.  kNDirect: lanes 16g .. 16g+15 need k = 8g .. 8g+7
    // of columns blk*16 + (lane % 16); one transpose read takes, per 16 lanes, 4 rows (k) x 16 columns
    // -- lane l addresses 4 consecutive n at row l/4, column group l%4 -- and returns to lane l the 4
    // consecutive k of column l, so two of them make the 8 k of a fragment.  Row & 3 = l / 4 and
    // (row >> 3) & 3 = g for every row a lane addresses, so its swizzle term is a constant.
    constexpr int NDB = LB == kNDirect ? NI : 1;
    int nd_addr[NDB];
    if constexpr (LB == kNDirect) {
        const int l = lane & 15, g = lane >> 4;
        const int xr = (((l >> 2) << 1) | (g << 3)) & (CPRB - 1);
        static_for<NI>([&](auto ni_) {
            constexpr int ni = decltype(ni_)::value;
            const int chunk = (wn * Cfg::WTN + ni * 16) / 8 + ((l & 3) >> 1);
            nd_addr[ni] = Cfg::A_BYTES + (8 * g + (l >> 2)) * (TN * 2) + ((chunk ^ xr) << 4) + (l & 1) * 8;
        });
    }
    auto fragB = [&](const char *sbase, auto blk_, int kk) __attribute__((always_inline)) {
        constexpr int blk = decltype(blk_)::value;
        if constexpr (LB == kNDirect) {
            // Written as asm: the compiler makes the builtin form of this read wait for every
            // outstanding global -> LDS copy (it cannot tell that they go to other buffers), which
            // drains the pipeline.  It therefore does not count these reads either: the code that
            // consumes them runs behind an explicit lgkmcnt(0) (the barrier of the pipelined loop,
            // the wait at the head of a k-tile in the two-buffer loop).
            const uint32_t q = (uint32_t)(uintptr_t)(sbase - smem) + (uint32_t)nd_addr[blk] + (uint32_t)(kk * 32 * (TN * 2));
            u32x2_t lo, hi;
            asm volatile("ds_read_b64_tr_b16 %0, %2\n\tds_read_b64_tr_b16 %1, %2 offset:%3"
                         : "=&v"(lo), "=&v"(hi)
                         : "v"(q), "n"(4 * (TN * 2)));
            return u32x4_t{lo[0], lo[1], hi[0], hi[1]};
        } else {
            return frag(sbase, b_frag_base, blk, kk);
        }
    };
    // A fragment of row block `blk`, k-step `kk`; kMDirect mirrors kNDirect.  Consecutive row blocks
    // are two chunks apart, i.e. bit 5 upward of the byte address, which the swizzle XORs but no
    // other term touches: the address of block blk is that of block 0 XOR (blk << 5).
    int md_addr = 0;
    if constexpr (LA == kMDirect) {
        const int l = lane & 15, g = lane >> 4;
        const int xr = (((l >> 2) << 1) | (g << 3)) & (TM / 8 - 1);
        const int chunk = (wm * Cfg::WTM) / 8 + ((l & 3) >> 1);
        md_addr = (8 * g + (l >> 2)) * (TM * 2) + ((chunk ^ xr) << 4) + (l & 1) * 8;
    }
    auto fragA = [&](const char *sbase, int blk, int kk) __attribute__((always_inline)) {
        if constexpr (LA == kMDirect) {
            const uint32_t q = ((uint32_t)(uintptr_t)(sbase - smem) + (uint32_t)md_addr + (uint32_t)(kk * 32 * (TM * 2))) ^ (uint32_t)(blk << 5);
            u32x2_t lo, hi;
            asm volatile("ds_read_b64_tr_b16 %0, %2\n\tds_read_b64_tr_b16 %1, %2 offset:%3"
                         : "=&v"(lo), "=&v"(hi)
                         : "v"(q), "n"(4 * (TM * 2)));
            return u32x4_t{lo[0], lo[1], hi[0], hi[1]};
        } else {
            return frag(sbase, a_frag_base, blk, kk);
        }
    };
    // The compiler does not count asm LDS reads, so with kMDirect a row block waits for its A fragment
    // itself: lgkmcnt(W).  The fragment was requested RA - 1 row blocks earlier and LDS reads return in
    // order, so it has arrived once at most W reads are outstanding, W being a number of reads known
    // to have been issued after it (2: the two transpose reads of the previous row block's request).
    auto a_ready = [&](auto w_) __attribute__((always_inline)) {
        constexpr int W = decltype(w_)::value;
        if constexpr (LA == kMDirect && W >= 0) __builtin_amdgcn_s_waitcnt((0xF) | (0x3 << 14) | (0x7 << 4) | (W << 8));
    };
    using I0 = std::integral_constant<int, 0>;
    using I1 = std::integral_constant<int, 1>;

    if constexpr (kAnyReg) {
        // ---- simple loop for operands that need the register transpose: prefetch distance 1 -----
        u32x4_t af[MI], bf[NI];
        issue(0, 0);
        commit_regs(0);
        for (int kt = 0; kt < KT; ++kt) {
            __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
            __syncthreads();
            if (kt + 1 < KT) issue(kt + 1, (kt + 1) % STAGES);
            const char *sbase = smem + (kt % STAGES) * Cfg::STAGE_BYTES;
            static_for<KSTEPS>([&](auto kk) {
                static_for<MI>([&](auto mi) { af[mi] = frag(sbase, a_frag_base, mi, kk); });
                static_for<NI>([&](auto ni) { bf[ni] = frag(sbase, b_frag_base, ni, kk); });
                // B fragment as the MFMA's first operand: the lane then holds 4 consecutive n per
                // accumulator, which is what the row-major store wants.
                static_for<MI>([&](auto mi) {
                    static_for<NI>([&](auto ni) { mfma16<Cfg::DT>(acc[mi][ni], bf[ni], af[mi]); });
                });
            });
            if (kt + 1 < KT) commit_regs((kt + 1) % STAGES);
        }
    } else if constexpr (STAGES == 2 && Cfg::DT >= 2) {
        // ---- 8-bit inputs, two stage buffers: one 128-deep MFMA per 16x16 block and k-tile -----------
        // A k-tile row is 128 bytes = 128 fp8 values.  The wide 8-bit MFMA (16x16x128) takes 32 bytes per
        // lane and operand: the lane's 16-byte fragments of both halves of the row side by side (which
        // k a byte stands for is the same for A and B, and every k of the row is held exactly once).
        // It does four times the work of the 32-deep form in twice the time, so the k-tile costs what a
        // 16-bit k-tile of the same bytes costs and carries twice the FLOPs.
        static_assert(KSTEPS == 2 && LA == kKContig && LB == kKContig, "128-byte rows of K-contiguous operands");
        u32x8_t b8[NI];
        issue_tile(std::true_type{}, 0, 0);
        issue_tile(std::true_type{}, 1, 1);
        auto pair = [&](const char *sbase, int base, auto blk_) __attribute__((always_inline)) {
            constexpr int blk = decltype(blk_)::value;
            const u32x4_t lo = frag(sbase, base, blk, 0), hi = frag(sbase, base, blk, 1);
            return u32x8_t{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
        };
        // The k-tile's MFMAs run in two halves with the barrier between them, as the k-steps of the 16-bit loop
        // below do.  First half: row blocks 0 .. MI/2-1 (their A fragments and all of B were read during the previous
        // k-tile); beside its MFMAs the A fragments of the other row blocks are read.  Barrier: this wave has every
        // fragment of the k-tile, k-tile kt+1 has landed (vmcnt 0), every wave is past its reads.  Second half, column
        // block by column block: beside its MFMAs the k-tile's own buffer is refilled with k-tile kt+2 and the
        // fragments of k-tile kt+1 are read -- B into the registers of the column block just finished, A of the
        // first row blocks into the registers the first half has released.  One set of B fragments and two half
        // sets of A (16 fragments of 32 bytes) are all the registers it takes, and LDS reads, copies and MFMAs are
        // spread evenly.  (Reading a k-tile's fragments in one burst at its head and refilling the buffer behind
        // its MFMAs took 1.7 us per k-tile for 0.85 us of MFMAs.)
        static_assert(MI % 2 == 0 && NI >= 2, "two halves of row blocks");
        constexpr int MH = MI / 2;
        u32x8_t a_lo[MH], a_hi[MH];
        pipeline_barrier<DMA_PER_TILE>();                          // k-tile 0 has landed
        static_for<MH>([&](auto mi) { a_lo[mi] = pair(smem, a_frag_base, mi); });
        static_for<NI>([&](auto ni) { b8[ni] = pair(smem, b_frag_base, ni); });
        for (int kt = 0; kt < KT; ++kt) {
            const int cur = kt & 1;
            const char *sc = smem + cur * Cfg::STAGE_BYTES, *sn = smem + (cur ^ 1) * Cfg::STAGE_BYTES;
            static_for<MH>([&](auto mi_) {
                constexpr int mi = decltype(mi_)::value;
                static_for<NI>([&](auto ni_) {
                    constexpr int ni = decltype(ni_)::value;
                    mfma128<Cfg::DT>(acc[mi][ni], b8[ni], a_lo[mi]);
                    if constexpr (ni == NI / 2) a_hi[mi] = pair(sc, a_frag_base, std::integral_constant<int, MH + mi>{});
                });
            });
            pipeline_barrier<0>();
            static_for<NI>([&](auto ni_) {
                constexpr int ni = decltype(ni_)::value;
                constexpr int d0 = ni * DMA_PER_TILE / NI, nd = (ni + 1) * DMA_PER_TILE / NI - d0;
                static_for<MH>([&](auto mi_) {
                    constexpr int mi = decltype(mi_)::value;
                    mfma128<Cfg::DT>(acc[MH + mi][ni], b8[ni], a_hi[mi]);
                    // copies of k-tile kt+2 into this k-tile's buffer, their even share per column block
                    static_for<(mi + 1) * nd / MH - mi * nd / MH>([&](auto j) {
                        issue_one(std::true_type{}, std::integral_constant<int, d0 + mi * nd / MH + decltype(j)::value>{}, kt + 2, cur);
                    });
                    // fragments of k-tile kt+1: B of the column block finished before this one, A of row block ni
                    if constexpr (mi == 1 % MH && ni >= 1) b8[ni - 1] = pair(sn, b_frag_base, std::integral_constant<int, ni - 1>{});
                    if constexpr (mi == MH - 1 && ni < MH) a_lo[ni] = pair(sn, a_frag_base, ni_);
                });
            });
            b8[NI - 1] = pair(sn, b_frag_base, std::integral_constant<int, NI - 1>{});
        }
    } else if constexpr (STAGES == 2) {
        // ---- two stage buffers, k-tiles of two k-steps --------------------------------------------
        // For tiles whose stage is too large for three buffers.  One k-tile is multiplied while the
        // next is in flight.  k-step 0 takes its A fragments through the ring (see below) and, beside
        // its MFMAs, reads ALL fragments of k-step 1; then the barrier: this wave has issued every
        // read of the tile, the next k-tile has landed (vmcnt 0), every wave is past its reads -- so
        // k-step 1, beside its MFMAs, refills the tile's own buffer with k-tile kt+2 and reads the
        // first fragments of k-tile kt+1.
        static_assert(KSTEPS == 2, "the two-buffer loop is written for k-tiles of two k-steps");
        constexpr int RA = MI % 4 == 0 ? 4 : 2;
        static_assert(MI % RA == 0, "ring slots must line up across k-tiles");
        u32x4_t ar[RA], af[MI], bq[2][NI];
        // the side instructions of a row block go out one (or their even share) behind each MFMA
        auto row_block = [&](auto mi_, const u32x4_t &a, auto pb_, auto ns_, auto w_, auto &&side) __attribute__((always_inline)) {
            constexpr int mi = decltype(mi_)::value, PB = decltype(pb_)::value, NS = decltype(ns_)::value;
            a_ready(w_);
            static_for<NI>([&](auto ni_) {
                constexpr int ni = decltype(ni_)::value;
                mfma16<Cfg::DT>(acc[mi][ni], bq[PB][ni], a);
                constexpr int s0 = ni * NS / NI, s1 = (ni + 1) * NS / NI;
                static_for<s1 - s0>([&](auto j) { side(std::integral_constant<int, s0 + decltype(j)::value>{}); });
            });
        };
        auto first_step = [&](const char *sc) __attribute__((always_inline)) {
            if constexpr (LB == kNDirect) __builtin_amdgcn_s_waitcnt((0xF) | (0x3 << 14) | (0x7 << 4) | (0x0 << 8));   // lgkmcnt(0)
            static_for<MI>([&](auto mi_) {
                constexpr int mi = decltype(mi_)::value;
                constexpr int ia = mi + RA - 1;
                // everything of k-step 1 is requested in the first half of the row blocks, so that the
                // barrier behind this k-step does not wait for LDS latency
                constexpr int b0 = bshare(mi, MI, NI), nb = bshare(mi + 1, MI, NI) - b0;
                constexpr int f0 = bshare(mi, MI, MI), nf = bshare(mi + 1, MI, MI) - f0;
                constexpr int na = ia < MI ? 1 : 0;
                auto side = [&](auto s_) __attribute__((always_inline)) {
                    constexpr int sx = decltype(s_)::value;
                    if constexpr (sx < na) ar[ia % RA] = fragA(sc, ia, 0);
                    else if constexpr (sx < na + nf) af[f0 + sx - na] = fragA(sc, f0 + sx - na, 1);
                    else bq[1][b0 + sx - na - nf] = fragB(sc, std::integral_constant<int, b0 + sx - na - nf>{}, 1);
                };
                // (the previous row block requested a ring fragment unless it was one of the last RA - 1 of this k-step)
                constexpr int W = (mi == 0 || mi + RA - 2 < MI) ? 2 : 0;
                row_block(mi_, ar[mi % RA], I0{}, std::integral_constant<int, na + nf + nb>{}, std::integral_constant<int, W>{}, side);
            });
        };
        auto last_step = [&](auto check_, const char *sn, int kt_load, int buf) __attribute__((always_inline)) {
            static_for<MI>([&](auto mi_) {
                constexpr int mi = decltype(mi_)::value;
                constexpr int ih = mi - (MI - (RA - 1));           // ring head of the next k-tile
                constexpr int na = ih >= 0 ? 1 : 0;
                constexpr int b0 = bshare(mi, MI, NI), nb = bshare(mi + 1, MI, NI) - b0;
                constexpr int d0 = mi * DMA_PER_TILE / MI, nd = (mi + 1) * DMA_PER_TILE / MI - d0;
                auto side = [&](auto s_) __attribute__((always_inline)) {
                    constexpr int sx = decltype(s_)::value;
                    if constexpr (sx < na) ar[ih] = fragA(sn, ih, 0);
                    else if constexpr (sx < na + nb) bq[0][b0 + sx - na] = fragB(sn, std::integral_constant<int, b0 + sx - na>{}, 0);
                    else issue_one(check_, std::integral_constant<int, d0 + sx - na - nb>{}, kt_load, buf);
                };
                // (af[] and bq[1] were complete at the barrier: no wait)
                row_block(mi_, af[mi], I1{}, std::integral_constant<int, na + nb + nd>{}, std::integral_constant<int, -1>{}, side);
            });
        };
        issue_tile(std::true_type{}, 0, 0);
        issue_tile(std::true_type{}, 1, 1);
        pipeline_barrier<DMA_PER_TILE>();
        static_for<RA - 1>([&](auto i) { ar[i] = fragA(smem, i, 0); });
        static_for<NI>([&](auto ni) { bq[0][ni] = fragB(smem, ni, 0); });
        const int KT_full = k_tail ? KT - 1 : KT;
        int kt = 0;
        auto ktile2 = [&](auto check_, auto cur_) __attribute__((always_inline)) {
            const int cur = cur_;
            first_step(smem + cur * Cfg::STAGE_BYTES);
            pipeline_barrier<0>();
            last_step(check_, smem + (cur ^ 1) * Cfg::STAGE_BYTES, kt + 2, cur);
            ++kt;
        };
        while (kt + 3 < KT_full) {                                 // steady state over the two buffers
            ktile2(std::false_type{}, I0{});
            ktile2(std::false_type{}, I1{});
        }
        while (kt < KT) ktile2(std::true_type{}, kt & 1);
        // The last k-tile has requested fragments of a k-tile that does not exist.  Reads issued as asm
        // are invisible to the compiler: it would hand their destination registers to the epilogue
        // while the data is still on its way.  Wait for them, and keep the registers allocated until then.
        if constexpr (LA == kMDirect || LB == kNDirect) {
            __builtin_amdgcn_s_waitcnt((0xF) | (0x3 << 14) | (0x7 << 4) | (0x0 << 8));   // lgkmcnt(0)
            static_for<RA>([&](auto i) { keep_alive(ar[i]); });
            static_for<MI>([&](auto i) { keep_alive(af[i]); });
            static_for<NI>([&](auto i) { keep_alive(bq[0][i]); keep_alive(bq[1][i]); });
        }
    } else if constexpr (LA == kHalo) {
        // ---- resident patch: 18 k-tiles (9 taps x 2 channel halves; data gradient: 36), fully unrolled
        // The same ring of A fragments and two B sets as the pipelined loop below, with every buffer
        // index, tap offset and border test a compile-time constant; only B is copied (k-tile
        // kt + STAGES - 1 into the buffer released by the barrier of k-tile kt).
        // (narrow wave tiles have two MFMAs per row block: a ring of four would request a fragment only 96 clocks
        // ahead of its use, less than an LDS read takes under load)
        constexpr int KT_ALL = 9 * KPT, RA = NI <= 2 && MI % 8 == 0 ? 8 : 4;
        static_assert(MI % RA == 0 && KSTEPS == 1, "ring slots line up across k-tiles");
        u32x4_t ar[RA], bq[2][NI];
        static_for<STAGES - 1>([&](auto s_) { issue_tile(std::false_type{}, decltype(s_)::value, decltype(s_)::value); });
        // The code below is straight-line, so the compiler would otherwise sink the zeroing of each
        // accumulator to just in front of its first MFMA -- closer than the matrix pipeline allows
        // after a register write, which it cannot know of an asm statement.  Pin the zeroing here.
        static_for<MI>([&](auto mi) {
            static_for<NI>([&](auto ni) { pin_acc(acc[mi][ni]); });
        });
        pipeline_barrier<(STAGES - 2) * DMA_PER_TILE>();
        int hb_c = halo_base(I0{}), hb_n = 0;
        static_for<RA - 1>([&](auto i) { ar[i] = halo_read(I0{}, i, hb_c, halo_test(I0{}, i)); });
        static_for<NI>([&](auto ni) { bq[0][ni] = fragB(smem, ni, 0); });
        static_for<KT_ALL>([&](auto kt_) {
            constexpr int kt = decltype(kt_)::value, PB = kt & 1;
            constexpr bool more = kt + 1 < KT_ALL, load = kt + STAGES - 1 < KT_ALL;
            constexpr int last_issued = kt + STAGES - 2 < KT_ALL - 1 ? kt + STAGES - 2 : KT_ALL - 1;
            constexpr int in_flight = last_issued - (kt + 1) > 0 ? last_issued - (kt + 1) : 0;   // k-tiles behind kt + 1
            using KN = std::integral_constant<int, more ? kt + 1 : kt>;
            const char *sn = smem + ((kt + 1) % STAGES) * Cfg::STAGE_BYTES;
            if constexpr (more) hb_n = halo_base(KN{});
            pipeline_barrier<in_flight * DMA_PER_TILE>();
            static_for<MI>([&](auto mi_) {
                constexpr int mi = decltype(mi_)::value;
                constexpr int ia = mi + RA - 1;
                constexpr bool a_cur = ia < MI, a_any = a_cur || more;
                using KA = std::integral_constant<int, a_cur ? kt : KN::value>;
                using BA = std::integral_constant<int, a_cur ? ia : ia - MI>;
                constexpr int b0 = more ? bshare(mi, MI, NI) : 0, nb = more ? bshare(mi + 1, MI, NI) - b0 : 0;
                constexpr int d0 = load ? mi * DMA_PER_TILE / MI : 0, nd = load ? (mi + 1) * DMA_PER_TILE / MI - d0 : 0;
                constexpr int NS = 2 + nb + nd;
                int dead = 0;
                auto side = [&](auto s_) __attribute__((always_inline)) {
                    constexpr int sx = decltype(s_)::value;
                    if constexpr (sx == 0) {
                        if constexpr (a_any) dead = halo_test(KA{}, BA{});
                    } else if constexpr (sx == 1) {
                        if constexpr (a_any) ar[ia % RA] = halo_read(KA{}, BA{}, a_cur ? hb_c : hb_n, dead);
                    } else if constexpr (sx < 2 + nb) {
                        bq[1 - PB][b0 + sx - 2] = fragB(sn, std::integral_constant<int, b0 + sx - 2>{}, 0);
                    } else {
                        issue_one(std::false_type{}, std::integral_constant<int, d0 + sx - 2 - nb>{}, kt + STAGES - 1,
                                  (kt + STAGES - 1) % STAGES);
                    }
                };
                static_for<NI>([&](auto ni_) {
                    constexpr int ni = decltype(ni_)::value;
                    mfma16<Cfg::DT>(acc[mi][ni], bq[PB][ni], ar[mi % RA]);
                    constexpr int s0 = ni * NS / NI, s1 = (ni + 1) * NS / NI;
                    static_for<s1 - s0>([&](auto j) { side(std::integral_constant<int, s0 + decltype(j)::value>{}); });
                });
            });
            hb_c = hb_n;
        });
    } else {
        // ---- software-pipelined loop ---------------------------------------------------------------
        // STAGES-1 k-tiles are in flight.  Registers hold the B fragments of the running k-step and
        // of the next one (two sets) and a ring of RA fragments of A: the MFMAs walk the wave tile
        // row block by row block (mi), and at the start of row block mi the A fragment of row block
        // mi + RA - 1 is requested -- past the last row block that is the first of the NEXT k-step,
        // so the ring runs across k-step and k-tile boundaries without a bubble.  The B fragments of
        // the next k-step and the copy instructions of the k-tile being fetched are dealt out over
        // the row blocks in the same way, one side instruction per MFMA (the MFMAs, reads and copies are
        // volatile asm statements or loads the compiler keeps in program order: the source order is
        // the issue order).
        // One barrier per k-tile, before its last k-step: then k-tile kt+1 has landed (explicit
        // vmcnt) and every wave is done with k-tile kt-1, whose buffer the last k-step refills with
        // k-tile kt+STAGES-1.  The k-steps before it read their own stage only and issue no copies.
        static_assert(STAGES >= 3, "the pipelined loop refills the buffer released one k-tile earlier");
        constexpr int RA = MI % 4 == 0 ? 4 : 2;                    // ring of A fragments
        static_assert(MI % RA == 0, "ring slots must line up across k-steps");
        // B sets alternate per k-step: with an odd number of k-steps per k-tile two k-tiles form one
        // unit of the loop (the K extent is rounded up to whole units; k-tiles past the end are
        // copied from out-of-range addresses, i.e. zeros).
        constexpr int TPU = KSTEPS % 2 ? 2 : 1;                    // k-tiles per unit
        u32x4_t ar[RA], bq[2][NI];

        // One k-step: fragment set PB of B, k-step KK of stage `sc`; the following k-step is KN of
        // stage `sn`.  DN > 0: also the copies of k-tile kt_load into buffer fill_buf.
        auto kstep = [&](auto pb_, auto kk_, auto kn_, const char *sc, const char *sn, auto check_, auto dn_, int kt_load,
                         int fill_buf) __attribute__((always_inline)) {
            constexpr int PB = decltype(pb_)::value, KK = decltype(kk_)::value, KN = decltype(kn_)::value;
            constexpr int DN = decltype(dn_)::value;
            // A k-step that issues no copies is not behind the k-tile's barrier: its directly copied B
            // fragments were requested with asm reads during the previous k-step, so it waits itself.
            if constexpr (LB == kNDirect && DN == 0) __builtin_amdgcn_s_waitcnt((0xF) | (0x3 << 14) | (0x7 << 4) | (0x0 << 8));   // lgkmcnt(0)
            static_for<MI>([&](auto mi_) {
                constexpr int mi = decltype(mi_)::value;
                constexpr int ia = mi + RA - 1;                    // A fragment requested in this row block
                // B fragments of the next k-step: all in the first half of the row blocks (its first MFMAs need them)
                constexpr int b0 = bshare(mi, MI, NI), nb = bshare(mi + 1, MI, NI) - b0;
                constexpr int d0 = mi * DN / MI, nd = (mi + 1) * DN / MI - d0;   // copies
                constexpr int NS = 1 + nb + nd;                    // side instructions of this row block
                auto side = [&](auto s_) __attribute__((always_inline)) {
                    constexpr int sx = decltype(s_)::value;
                    if constexpr (sx == 0) {
                        if constexpr (ia < MI) ar[ia % RA] = fragA(sc, ia, KK);
                        else ar[ia % RA] = fragA(sn, ia - MI, KN);
                    } else if constexpr (sx <= nb) {
                        bq[1 - PB][b0 + sx - 1] = fragB(sn, std::integral_constant<int, b0 + sx - 1>{}, KN);
                    } else {
                        issue_one(check_, std::integral_constant<int, d0 + sx - 1 - nb>{}, kt_load, fill_buf);
                    }
                };
                // B fragment as the MFMA's first operand: the lane then holds 4 consecutive n per
                // accumulator, which is what the row-major store wants.  The side instructions go
                // out one (or their even share) behind each MFMA, so that none of the gaps between
                // two MFMAs grows longer than the MFMA itself.
                a_ready(std::integral_constant<int, 2>{});
                static_for<NI>([&](auto ni_) {
                    constexpr int ni = decltype(ni_)::value;
                    mfma16<Cfg::DT>(acc[mi][ni], bq[PB][ni], ar[mi % RA]);
                    constexpr int s0 = ni * NS / NI, s1 = (ni + 1) * NS / NI;
                    static_for<s1 - s0>([&](auto j) { side(std::integral_constant<int, s0 + decltype(j)::value>{}); });
                });
            });
        };
        // One k-tile.  P0: B set of its first k-step.  cur / nxt / fill: buffers of k-tiles kt, kt+1 and
        // kt-1 (= kt+STAGES-1); constants in the unrolled steady loop, so that every LDS address
        // there is a loop-invariant register plus an immediate.
        auto ktile = [&](auto p0_, auto check_, auto cur_, auto nxt_, auto fill_, int kt) __attribute__((always_inline)) {
            constexpr int P0 = decltype(p0_)::value;
            const int cur = cur_, nxt = nxt_, fill = fill_;
            const char *sc = smem + cur * Cfg::STAGE_BYTES;
            static_for<KSTEPS - 1>([&](auto kk_) {
                constexpr int kk = decltype(kk_)::value;
                kstep(std::integral_constant<int, (P0 + kk) & 1>{}, kk_, std::integral_constant<int, kk + 1>{}, sc, sc,
                      check_, I0{}, 0, 0);
            });
            pipeline_barrier<(STAGES - 3) * DMA_PER_TILE>();
            kstep(std::integral_constant<int, (P0 + KSTEPS - 1) & 1>{}, std::integral_constant<int, KSTEPS - 1>{}, I0{}, sc,
                  smem + nxt * Cfg::STAGE_BYTES, check_, std::integral_constant<int, DMA_PER_TILE>{}, kt + STAGES - 1, fill);
        };

        // prologue: k-tiles 0 .. STAGES-2 on their way, k-tile 0 landed, first fragments in registers
        static_for<STAGES - 1>([&](auto s_) { issue_tile(std::true_type{}, decltype(s_)::value, decltype(s_)::value); });
        pipeline_barrier<(STAGES - 2) * DMA_PER_TILE>();
        static_for<RA - 1>([&](auto i) { ar[i] = fragA(smem, i, 0); });
        static_for<NI>([&](auto ni) { bq[0][ni] = fragB(smem, ni, 0); });

        const int KT_full = k_tail ? KT - 1 : KT;                  // complete k-tiles: loads skip the K-tail test
        const int KTP = (KT + TPU - 1) / TPU * TPU;
        int kt = 0;
        // steady state, unrolled over the ring of stage buffers (and over the B set parity)
        constexpr int UNR = STAGES * TPU;
        while (kt + UNR + STAGES - 2 < KT_full) {
            static_for<UNR>([&](auto u_) {
                constexpr int u = decltype(u_)::value;
                constexpr int c = u % STAGES;
                ktile(std::integral_constant<int, (u * KSTEPS) & 1>{}, std::false_type{}, std::integral_constant<int, c>{},
                      std::integral_constant<int, (c + 1) % STAGES>{}, std::integral_constant<int, (c + STAGES - 1) % STAGES>{}, kt);
                ++kt;
            });
        }
        // the rest, one unit at a time with the K-tail / past-the-end test on every copy
        int cur = 0;                                               // kt is a multiple of STAGES here
        while (kt < KTP) {
            static_for<TPU>([&](auto u_) {
                constexpr int u = decltype(u_)::value;
                const int nxt = cur + 1 == STAGES ? 0 : cur + 1;
                const int fill = cur == 0 ? STAGES - 1 : cur - 1;
                ktile(std::integral_constant<int, (u * KSTEPS) & 1>{}, std::true_type{}, cur, nxt, fill, kt);
                cur = nxt;
                ++kt;
            });
        }
        // (as at the end of the two-buffer loop: asm reads of a k-tile that does not exist are still in flight)
        if constexpr (LA == kMDirect || LB == kNDirect) {
            __builtin_amdgcn_s_waitcnt((0xF) | (0x3 << 14) | (0x7 << 4) | (0x0 << 8));   // lgkmcnt(0)
            static_for<RA>([&](auto i) { keep_alive(ar[i]); });
            static_for<NI>([&](auto i) { keep_alive(bq[0][i]); keep_alive(bq[1][i]); });
        }
    }

    // The MFMAs are asm statements, so the compiler does not know that the accumulators were written
    // by the matrix pipeline: keep the required distance to their first reader by hand.
    asm volatile("s_nop 15");
    asm volatile("s_nop 15");

    // ---- split-K: partial tiles through the workspace ---------------------------------------------
    // Slice s of tile t keeps its fp32 accumulators at partial[(s * tiles + t)][register][thread], one
    // 128-bit store per accumulator and thread.  Whoever adds the slices up reads them back in the same
    // layout, slice 0 first: the order of the additions is fixed, whichever workgroup does them.
    // Partial tiles are written and read with device-coherent accesses (they bypass the L2 of the XCD
    // the workgroup runs on: the eight L2s are not coherent with one another), so handing a tile from
    // one workgroup to another needs no write-back or invalidation of a whole cache, only the wait for
    // the stores' completion in front of the counter update.
    if constexpr ((MODE == 0 || MODE == 4) && !Cfg::PERSIST) {
        // (phase 2 with one slice: the slices were added up into slice 0 by the reduction kernel)
        if (p.split_k > 1 || p.split_phase == 2) {
            constexpr int64_t kTileElems = (int64_t)TM * TN;
            constexpr int kCoherent = 17;                  // cache policy bits sc0 | sc1: device scope
            // (slice and tile index are worked out again from the workgroup id rather than kept in
            // registers across the mainloop; split-K never runs under the persistent scheduler)
            int wg_again = blockIdx.x;
            asm volatile("" : "+s"(wg_again));
            const int pair = xcd_remap(wg_again, p.split_phase != 2 ? p.total_tiles * p.split_k : p.total_tiles);
            const int slice2 = p.split_phase != 2 ? pair / p.total_tiles : 0;
            const int t_lin = pair - slice2 * p.total_tiles;
            auto part_rsrc = [&](int sl) __attribute__((always_inline)) {
                return buffer_rsrc(p.ws_partials + ((int64_t)sl * p.total_tiles + t_lin) * kTileElems, (uint32_t)(kTileElems * 4));
            };
            if (p.split_phase != 2) {
                const rsrc_t mine = part_rsrc(slice2);
                static_for<MI>([&](auto mi) {
                    static_for<NI>([&](auto ni) {
                        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4_t, acc[mi][ni]), mine,
                                                               ((mi * NI + ni) * kThreads + tid) * 16, 0, kCoherent);
                    });
                });
                if (p.split_phase == 1) return;            // parallel mode, first launch: done
                // serial mode: the workgroup that arrives last at the tile's counter does the rest.  Its
                // partial tile has reached memory once the stores have completed (vmcnt 0); then count.
                __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
                __syncthreads();                           // (also: every wave is past its LDS reads and copies)
                if (tid == 0) *(volatile int *)smem = (int)atomicAdd(&p.ws_counters[t_lin], 1u);
                __syncthreads();
                const int arrived = *(volatile int *)smem;
                if (arrived != p.split_k - 1) return;
                if (tid == 0) atomicExch(&p.ws_counters[t_lin], 0u);      // leave the counter as it was found
            }
            constexpr int kRegs = MI * NI;
            if (p.split_k == 1) {
                // One slice: the sum the reduction kernel left in slice 0.  It is taken as it is (0 + x is x bit for
                // bit: a sum that started from +0 is never -0), sixteen accumulators' loads in flight at a time.
                const rsrc_t rs = part_rsrc(0);
                constexpr int kBatch = kRegs < 16 ? kRegs : 16;
                static_for<kRegs / kBatch>([&](auto b_) {
                    constexpr int r0 = decltype(b_)::value * kBatch;
                    u32x4_t v[kBatch];
                    static_for<kBatch>([&](auto j) { v[j] = __builtin_amdgcn_raw_buffer_load_b128(rs, ((r0 + j) * kThreads + tid) * 16, 0, kCoherent); });
                    static_for<kBatch>([&](auto j) {
                        constexpr int r = r0 + decltype(j)::value;
                        acc[r / NI][r % NI] = __builtin_bit_cast(f32x4_t, v[j]);
                        pin_acc(acc[r / NI][r % NI]);
                    });
                    asm volatile("" ::: "memory");
                });
            } else {
                static_for<MI>([&](auto mi) {
                    static_for<NI>([&](auto ni) {
                        acc[mi][ni] = f32x4_t{0.f, 0.f, 0.f, 0.f};
                        pin_acc(acc[mi][ni]);
                    });
                });
                // Several slices' loads are in flight at once (a thread's share of one slice of a small tile is a
                // few hundred bytes: one slice at a time would pay a memory round trip per slice); the additions
                // still happen in slice order.
                // (as many slices as fit into half of what the kernel's register budget leaves beside the
                // accumulators, at most 8; large tiles have a slice's worth of loads in flight anyway)
                constexpr int kFit = (512 / Cfg::MIN_WAVES - kRegs * 4) / 2 / (kRegs * 4);
                constexpr int U = kFit < 1 ? 1 : kFit > 8 ? 8 : kFit;
                int sl = 0;
                if constexpr (kFit >= 1) {
                    for (; sl + U <= p.split_k; sl += U) {
                        u32x4_t v[U][kRegs];
                        static_for<U>([&](auto u) {
                            const rsrc_t rs = part_rsrc(sl + u);
                            static_for<kRegs>([&](auto r) { v[u][r] = __builtin_amdgcn_raw_buffer_load_b128(rs, (r * kThreads + tid) * 16, 0, kCoherent); });
                        });
                        static_for<U>([&](auto u) {
                            static_for<MI>([&](auto mi) {
                                static_for<NI>([&](auto ni) {
                                    acc[mi][ni] += __builtin_bit_cast(f32x4_t, v[u][mi * NI + ni]);
                                    pin_acc(acc[mi][ni]);  // back into its accumulation register: the sums must not
                                                           // live in ordinary registers across the loop
                                });
                            });
                        });
                        asm volatile("" ::: "memory");
                    }
                }
                for (; sl < p.split_k; ++sl) {
                    const rsrc_t rs = part_rsrc(sl);
                    // (one row block at a time: the compiler would otherwise gather all of a slice's loads in
                    // front of the additions and need a second register file's worth of registers for them)
                    static_for<MI>([&](auto mi) {
                        static_for<NI>([&](auto ni) {
                            const u32x4_t v = __builtin_amdgcn_raw_buffer_load_b128(rs, ((mi * NI + ni) * kThreads + tid) * 16, 0, kCoherent);
                            acc[mi][ni] += __builtin_bit_cast(f32x4_t, v);
                            pin_acc(acc[mi][ni]);
                        });
                        asm volatile("" ::: "memory");
                    });
                }
            }
        }
    }

    // ---- stream-K: parts of a tile through the workspace -------------------------------------------
    // Workgroup g keeps at most two parts: the one that starts inside a tile (slot 2g) and the one that ends
    // inside a tile (slot 2g + 1).  Part s of a tile belongs to workgroup g_first + s, g_first owning the tile's
    // first iteration; part 0 is that workgroup's second kind, every later part its owner's first kind.  The
    // same device-coherent accesses, counter and fixed order of additions as split-K above.
    if constexpr (Cfg::STREAMK) {
        // (the piece is worked out again from the loop variable rather than kept in registers across the mainloop)
        int it_again = wg_id;
        asm volatile("" : "+s"(it_again));
        const StreamKPiece pc = streamk_piece(it_again, sk_end, p.sk_rounds, p.sk_ipt, p.sk_q, p.sk_deal);
        const int k0_again = pc.k0, k1_again = pc.k1;
        if (k0_again != 0 || k1_again != p.sk_ipt) {
            constexpr int64_t kTileElems = (int64_t)TM * TN;
            constexpr int kCoherent = 17;
            // the parts of remaining tile r: those of the workgroups whose runs meet its k steps [r, r + 1) * sk_ipt
            const int tile_again = pc.rest_tile;
            const int it0 = tile_again * p.sk_ipt;
            const int g_first = it0 / p.sk_q, n_parts = (it0 + p.sk_ipt - 1) / p.sk_q - g_first + 1;
            auto part_rsrc = [&](int slot) __attribute__((always_inline)) {
                return buffer_rsrc(p.ws_partials + (int64_t)slot * kTileElems, (uint32_t)(kTileElems * 4));
            };
            const rsrc_t mine = part_rsrc(2 * pc.g + (k0_again != 0 ? 0 : 1));
            static_for<MI>([&](auto mi) {
                static_for<NI>([&](auto ni) {
                    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4_t, acc[mi][ni]), mine,
                                                           ((mi * NI + ni) * kThreads + tid) * 16, 0, kCoherent);
                });
            });
            __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
            __syncthreads();                               // (also: every wave is past its LDS reads and copies)
            if (tid == 0) *(volatile int *)smem = (int)atomicAdd(&p.ws_counters[tile_again], 1u);
            __syncthreads();
            // (the same in every lane, and said so: a branch the compiler took for divergent would make the loop
            // variable, and with it every address and buffer resource of the next piece, a vector value)
            const int arrived = __builtin_amdgcn_readfirstlane(*(volatile int *)smem);
            if (arrived != n_parts - 1) {
                // not the last part: on to the workgroup's next piece
                wg_id = it_again + (k1_again - k0_again);
                if (wg_id >= sk_end) break;
                __syncthreads();
                continue;
            }
            if (tid == 0) atomicExch(&p.ws_counters[tile_again], 0u);
            static_for<MI>([&](auto mi) {
                static_for<NI>([&](auto ni) {
                    acc[mi][ni] = f32x4_t{0.f, 0.f, 0.f, 0.f};
                    pin_acc(acc[mi][ni]);
                });
            });
            // as in the split-K loop above: several parts' loads in flight where the registers allow, additions in part order
            constexpr int kRegs = MI * NI;
            constexpr int kFit = (512 / Cfg::MIN_WAVES - kRegs * 4) / 2 / (kRegs * 4);
            constexpr int U = kFit < 1 ? 1 : kFit > 8 ? 8 : kFit;
            int s_ = 0;
            if constexpr (kFit >= 1) {
                for (; s_ + U <= n_parts; s_ += U) {
                    u32x4_t v[U][kRegs];
                    static_for<U>([&](auto u) {
                        const rsrc_t rs = part_rsrc(2 * (g_first + s_ + u) + (s_ + u == 0 ? 1 : 0));
                        static_for<kRegs>([&](auto r) { v[u][r] = __builtin_amdgcn_raw_buffer_load_b128(rs, (r * kThreads + tid) * 16, 0, kCoherent); });
                    });
                    static_for<U>([&](auto u) {
                        static_for<MI>([&](auto mi) {
                            static_for<NI>([&](auto ni) {
                                acc[mi][ni] += __builtin_bit_cast(f32x4_t, v[u][mi * NI + ni]);
                                pin_acc(acc[mi][ni]);
                            });
                        });
                    });
                    asm volatile("" ::: "memory");
                }
            }
            for (; s_ < n_parts; ++s_) {
                const rsrc_t rs = part_rsrc(2 * (g_first + s_) + (s_ == 0 ? 1 : 0));
                static_for<MI>([&](auto mi) {
                    static_for<NI>([&](auto ni) {
                        const u32x4_t v = __builtin_amdgcn_raw_buffer_load_b128(rs, ((mi * NI + ni) * kThreads + tid) * 16, 0, kCoherent);
                        acc[mi][ni] += __builtin_bit_cast(f32x4_t, v);
                        pin_acc(acc[mi][ni]);
                    });
                    asm volatile("" ::: "memory");
                });
            }
        }
    }

    // ---- epilogue ---------------------------------------------------------------------------------
    // The accumulators leave the MFMA layout (a lane holds 4 consecutive n of ONE row per quad)
    // through a wave-private LDS patch, one 32-row block at a time, and come back as 8 consecutive
    // n per lane with the lanes of a row side by side.  The chain then runs on registers in that
    // layout, so bias / residual loads and the output stores are all full 128-bit accesses that
    // cover whole contiguous row segments.
    constexpr int WTN = Cfg::WTN, EPI_LD = Cfg::EPI_LD;
    constexpr int LPR = WTN / 8;              // lanes per staged row
    constexpr int RPP = 64 / LPR;             // rows per pass
    constexpr int PASSES = 32 / RPP;
    // tensor operands of an interpreted chain fetched ahead of use (others load in place); kernels that
    // share a CU with other workgroups have fewer registers and prefetch less
    constexpr bool kLean = Cfg::MIN_WAVES >= 2;
    constexpr int kMaxNVec = kLean ? 2 : 4, kMaxMat = kLean ? 1 : 2;
    __syncthreads();                          // every wave is done with the pipeline buffers
    // The chain is walked with a run-time step index.  Steps are read straight from the kernel
    // argument segment (constant address space, uniform index => scalar loads into SGPRs); `p` is
    // the kernel's first argument, so its step table sits at offsetof(KParams, steps).
    typedef const __attribute__((address_space(4))) EpiStepDev ConstStep;
    ConstStep *const ksteps = (ConstStep *)((const __attribute__((address_space(4))) char *)
                                                __builtin_amdgcn_kernarg_segment_ptr() + offsetof(KParams, steps));
    auto get_step = [&](int s) __attribute__((always_inline)) {
        EpiStepDev st;
        st.op = ksteps[s].op;
        st.dtype = ksteps[s].dtype;
        st.p0 = ksteps[s].p0;
        st.p1 = ksteps[s].p1;
        st.ptr = ksteps[s].ptr;
        st.ld = ksteps[s].ld;
        st.bs = ksteps[s].bs;
        return st;
    };
    float *stg = (float *)smem + wave * 32 * EPI_LD;
    const int e_row = lane / LPR, e_col = (lane % LPR) * 8;
    const int dtD = p.dtD;
    const bool dvec = p.d_vec != 0;
    const int n_steps = p.n_steps;

    EpiCtx c;
    c.batch = batch;
    c.group = group;
    c.n = n0 + wn * WTN + e_col;
    const int n_left = p.N - c.n;

    // passes whose residual segments are requested together, ahead of use
    constexpr int GRP = PASSES < 4 ? PASSES : 4;
    constexpr int GRP_I = Cfg::MIN_WAVES >= 3 ? 1 : (kLean && GRP > 2 ? 2 : GRP);     // pass group of the interpreted chain

    // accumulators of 32-row block `mi` -> this wave's staging patch (fp32).  acc needs constant
    // indices, and is only ever touched by code written directly in the kernel body (a closure that
    // holds a reference to it and is itself captured by another closure keeps it out of registers).
#define UCL_STAGE_BLOCK(mb)                                                                             \
    static_for<MI / 2>([&](auto mj) {                                                                   \
        if ((mb) == mj) {                                                                               \
            static_for<2>([&](auto h) {                                                                 \
                static_for<NI>([&](auto ni) {                                                           \
                    *(f32x4_t *)(stg + (h * 16 + f_row) * EPI_LD + ni * 16 + 4 * f_kg) = acc[2 * mj + h][ni]; \
                });                                                                                     \
            });                                                                                         \
        }                                                                                               \
    })
    auto staged_row = [&](int row, float (&v)[8]) __attribute__((always_inline)) {
        const f32x4_t lo = *(const f32x4_t *)(stg + row * EPI_LD + e_col);
        const f32x4_t hi = *(const f32x4_t *)(stg + row * EPI_LD + e_col + 4);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            v[e] = lo[e];
            v[4 + e] = hi[e];
        }
    };
    const int64_t d_batch_off = MODE == 1 ? 0 : (int64_t)batch * p.d_bs;

    // ---- fused form: act(alpha * acc + bias[n] + beta * R[m,n]) as straight-line code ---------------
    // All block / pass loops of the epilogue are REAL loops: their bodies are re-executed from the
    // instruction cache instead of existing once per pass.
    // (one 32-row block; the caller stages the block and loops over blocks, so that the accumulator
    // registers are read at exactly one place in the code)
    const __attribute__((address_space(4))) FusedEpi &f = p.fused;
    float bias8[8];
    const char *res_base = nullptr;       // residual, this lane's columns of row 0
    const char *res_u = nullptr;          // residual, element (0, 0) of this batch / group (wave-uniform)
    float alpha = 1.f;
    auto fused_block = [&](auto act_, int mi) __attribute__((always_inline)) {
        constexpr int ACT = decltype(act_)::value;
        const int m_blk = m0 + wm * Cfg::WTM + mi * 32;
#pragma clang loop unroll(disable)
        for (int pg = 0; pg < PASSES; pg += GRP) {
            // the residual segments of a whole group of passes are requested before any is used
            Raw8 res[GRP];
            if (f.has_res) {
                static_for<GRP>([&](auto u) {
                    const int m = m_blk + (pg + u) * RPP + e_row;
                    res[u] = load8(res_base, f.res_dt & 0xff, (int64_t)m * f.res_ld, (f.res_dt & 0x100) != 0,
                                   m < Mloc ? n_left : 0);
                });
            }
            static_for<GRP>([&](auto u) {
                const int row = (pg + u) * RPP + e_row;
                const int m = m_blk + row;
                float v[8];
                staged_row(row, v);
#pragma unroll
                for (int e = 0; e < 8; ++e) v[e] = v[e] * alpha + bias8[e];
                if (f.has_res) {
                    float t[8];
                    decode8(res[u], f.res_dt & 0xff, t);
#pragma unroll
                    for (int e = 0; e < 8; ++e) v[e] += f.beta * t[e];
                }
#pragma unroll
                for (int e = 0; e < 8; ++e) v[e] = act_f32<ACT>(v[e], f.act_p0, f.act_p1);
                store8(Db, dtD, d_batch_off + (int64_t)m * p.ldd + c.n, v, dvec, m < Mloc ? n_left : 0);
            });
        }
    };

    // Fast form of the same block for the common case (decided once per wave): every lane owns 8
    // existing columns and every tensor involved allows 128-bit access.  Rows are bounded by the
    // range check of buffer resources that cover exactly the wave's existing rows (stores past the
    // end are dropped, residual loads return zero), so the block is straight-line code: all residual
    // rows and all staged rows are requested up front and the arithmetic of one pass runs while the
    // data of the next is still on its way.
    const int w_rows = Mloc - (m0 + wm * Cfg::WTM) < Cfg::WTM ? Mloc - (m0 + wm * Cfg::WTM) : Cfg::WTM;
    const int d_esz = dtD == UCL_F32 ? 4 : 2;
    const int r_dt = f.res_dt & 0xff;
    const int r_esz = r_dt == UCL_F32 ? 4 : 2;
    rsrc_t d_rsrc = buffer_rsrc(nullptr, 0), r_rsrc = buffer_rsrc(nullptr, 0);
    uint32_t d_lane = 0, r_lane = 0, d_row_bytes = 0, r_row_bytes = 0;
    // fp32 output without a residual or with an fp32 one: a lane takes columns 4i..4i+3 and 4(i + LPR)..+3 of its row
    // instead of 8i..8i+7, so that each of its two 128-bit stores is, across the lanes of a row, one
    // contiguous run of whole lines (and can stream); with 8 consecutive columns per lane each store
    // instruction writes every other 16 bytes.
    const bool f_split = f.enabled && dtD == UCL_F32 && (!f.has_res || (f.res_dt & 0xff) == UCL_F32) && LPR * 16 >= 128;
    const int f_colA = f_split ? (lane % LPR) * 4 : e_col, f_colB = f_split ? f_colA + LPR * 4 : e_col + 4;
    auto fast_setup = [&]() __attribute__((always_inline)) {
        const int64_t col0 = n0 + wn * WTN;
        if (w_rows > 0) {
            d_rsrc = buffer_rsrc(Db + (d_batch_off + (int64_t)(m0 + wm * Cfg::WTM) * p.ldd + col0) * d_esz,
                                 (uint32_t)(((int64_t)(w_rows - 1) * p.ldd + WTN) * d_esz));
            if (f.has_res)
                r_rsrc = buffer_rsrc(res_u + ((int64_t)(m0 + wm * Cfg::WTM) * f.res_ld + col0) * r_esz,
                                     (uint32_t)(((int64_t)(w_rows - 1) * f.res_ld + WTN) * r_esz));
        }
        d_row_bytes = (uint32_t)(p.ldd * d_esz);
        r_row_bytes = (uint32_t)(f.res_ld * r_esz);
        d_lane = e_row * d_row_bytes + f_colA * d_esz;
        r_lane = e_row * r_row_bytes + f_colA * r_esz;        // (f_colA != e_col only with an fp32 residual)
    };
    // passes whose operands are requested together (all of a block where registers allow)
    constexpr int FG = Cfg::MIN_WAVES >= 2 && PASSES > 2 ? 2 : PASSES;
    // The block in three phases, each selected once per pass group by a wave-uniform branch instead of
    // per element: gather (staged fp32 * alpha + bias + beta * residual, by residual type), activation
    // (by opcode), conversion + store (by output type).  The values of the whole group stay in
    // registers between the phases.
    // The residual segments of a whole block (one 128-bit load per pass, two for fp32) are requested
    // one block ahead of their use: a load from HBM takes longer than a block's arithmetic, and a wave
    // that waited for it in every block would spend the epilogue waiting.
    static_assert(MI / 2 == 1 || (MI / 2) % 2 == 0, "blocks are taken in pairs");
    // (the registers suffice for the first 16 bytes per pass: the second half of an fp32 residual is
    // loaded where it is used; kernels with three or more workgroups per CU load everything in place)
    constexpr bool kResHi = false, kResAhead = Cfg::MIN_WAVES <= 2;
    struct ResRegs {
        u32x4_t lo[kResAhead ? PASSES : 1], hi[kResHi ? PASSES : 1];
    };
    auto res_issue = [&](int mi, ResRegs &r) __attribute__((always_inline)) {
        if constexpr (!kResAhead) return;
        const uint32_t r0 = r_lane + mi * 32 * r_row_bytes;
        static_for<kResAhead ? PASSES : 0>([&](auto u) { r.lo[u] = __builtin_amdgcn_raw_buffer_load_b128(r_rsrc, r0 + u * RPP * r_row_bytes, 0, kAuxStream); });
        if constexpr (kResHi) {
            if (r_dt == UCL_F32) {
                static_for<PASSES>([&](auto u) { r.hi[u] = __builtin_amdgcn_raw_buffer_load_b128(r_rsrc, r0 + u * RPP * r_row_bytes + 16, 0, kAuxStream); });
            }
        }
    };
    auto fast_block = [&](auto has_res_, int mi, const ResRegs &rr) __attribute__((always_inline)) {
        constexpr bool HAS_RES = decltype(has_res_)::value;
        constexpr int kAuxStore = LPR * 16 >= 128 ? kAuxStream : 0;   // streaming only where an instruction writes whole lines
        constexpr int FGX = HAS_RES && FG > 4 ? 4 : FG;       // with a residual in registers: smaller pass groups
        const float beta = f.beta, ap0 = f.act_p0, ap1 = f.act_p1;
        const uint32_t d0 = d_lane + mi * 32 * d_row_bytes;
        static_for<PASSES / FGX>([&](auto g_) {
            constexpr int P0 = decltype(g_)::value * FGX;
            float v[FGX][8];
            u32x4_t r_lo[FGX], r_hi[FGX];
            if constexpr (HAS_RES) {
                if constexpr (kResAhead) {
                    static_for<FGX>([&](auto u) { r_lo[u] = rr.lo[P0 + u]; });
                } else {
                    const uint32_t r0 = r_lane + mi * 32 * r_row_bytes;
                    static_for<FGX>([&](auto u) {
                        r_lo[u] = __builtin_amdgcn_raw_buffer_load_b128(r_rsrc, r0 + (P0 + u) * RPP * r_row_bytes, 0, kAuxStream);
                    });
                }
                if constexpr (kResHi) {
                    static_for<FGX>([&](auto u) { r_hi[u] = rr.hi[P0 + u]; });
                } else if (r_dt == UCL_F32) {
                    const uint32_t r0 = r_lane + mi * 32 * r_row_bytes;
                    const uint32_t hi_off = f_split ? LPR * 16 : 16;       // second column group of the lane
                    static_for<FGX>([&](auto u) {
                        r_hi[u] = __builtin_amdgcn_raw_buffer_load_b128(r_rsrc, r0 + (P0 + u) * RPP * r_row_bytes + hi_off, 0, kAuxStream);
                    });
                }
            }
            static_for<FGX>([&](auto u) {
                const f32x4_t lo = *(const f32x4_t *)(stg + ((P0 + u) * RPP + e_row) * EPI_LD + f_colA);
                const f32x4_t hi = *(const f32x4_t *)(stg + ((P0 + u) * RPP + e_row) * EPI_LD + f_colB);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    v[u][e] = lo[e] * alpha + bias8[e];
                    v[u][4 + e] = hi[e] * alpha + bias8[4 + e];
                }
            });
            if constexpr (HAS_RES) {
                if (r_dt == UCL_F32) {
                    static_for<FGX>([&](auto u) {
                        const f32x4_t fl = __builtin_bit_cast(f32x4_t, r_lo[u]), fh = __builtin_bit_cast(f32x4_t, r_hi[u]);
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            v[u][e] += beta * fl[e];
                            v[u][4 + e] += beta * fh[e];
                        }
                    });
                } else if (r_dt == UCL_BF16) {
                    static_for<FGX>([&](auto u) {
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const uint32_t w = r_lo[u][e];
                            v[u][2 * e] += beta * __builtin_bit_cast(float, w << 16);
                            v[u][2 * e + 1] += beta * __builtin_bit_cast(float, w & 0xffff0000u);
                        }
                    });
                } else {
                    static_for<FGX>([&](auto u) {
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const uint32_t w = r_lo[u][e];
                            const f16x2_t h = __builtin_bit_cast(f16x2_t, w);
                            v[u][2 * e] += beta * (float)h[0];
                            v[u][2 * e + 1] += beta * (float)h[1];
                        }
                    });
                }
            }
            switch (f.act) {
#define UCL_ACT_CASE(OP)                                                                   \
    case OP:                                                                               \
        static_for<FGX>([&](auto u) {                                                       \
            _Pragma("unroll") for (int e = 0; e < 8; ++e) v[u][e] = act_f32<OP>(v[u][e], ap0, ap1); \
        });                                                                                \
        break;
                UCL_ACT_CASE(UCL_EPI_RELU)
                UCL_ACT_CASE(UCL_EPI_GELU_TANH)
                UCL_ACT_CASE(UCL_EPI_GELU_ERF)
                UCL_ACT_CASE(UCL_EPI_SILU)
                UCL_ACT_CASE(UCL_EPI_SIGMOID)
                UCL_ACT_CASE(UCL_EPI_TANH)
                UCL_ACT_CASE(UCL_EPI_MISH)
                UCL_ACT_CASE(UCL_EPI_HARDSWISH)
                UCL_ACT_CASE(UCL_EPI_LEAKY_RELU)
                UCL_ACT_CASE(UCL_EPI_ELU)
                UCL_ACT_CASE(UCL_EPI_CLAMP)
#undef UCL_ACT_CASE
            default: break;
            }
            if (dtD == UCL_F32) {
                if (f_split) {
                    static_for<FGX>([&](auto u) {
                        const uint32_t off = d0 + (P0 + u) * RPP * d_row_bytes;
                        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4_t, f32x4_t{v[u][0], v[u][1], v[u][2], v[u][3]}), d_rsrc, off, 0, kAuxStore);
                        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4_t, f32x4_t{v[u][4], v[u][5], v[u][6], v[u][7]}), d_rsrc, off + LPR * 16, 0, kAuxStore);
                    });
                } else {
                    static_for<FGX>([&](auto u) {
                        const uint32_t off = d0 + (P0 + u) * RPP * d_row_bytes;
                        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4_t, f32x4_t{v[u][0], v[u][1], v[u][2], v[u][3]}), d_rsrc, off, 0, 0);
                        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4_t, f32x4_t{v[u][4], v[u][5], v[u][6], v[u][7]}), d_rsrc, off + 16, 0, 0);
                    });
                }
            } else if (dtD == UCL_BF16) {
                static_for<FGX>([&](auto u) {
                    u32x4_t o;
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        o[e] = __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2_t{v[u][2 * e], v[u][2 * e + 1]}, bf16x2_t));
                    __builtin_amdgcn_raw_buffer_store_b128(o, d_rsrc, d0 + (P0 + u) * RPP * d_row_bytes, 0, kAuxStore);
                });
            } else {
                static_for<FGX>([&](auto u) {
                    u32x4_t o;
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        o[e] = __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2_t{v[u][2 * e], v[u][2 * e + 1]}, f16x2_t));
                    __builtin_amdgcn_raw_buffer_store_b128(o, d_rsrc, d0 + (P0 + u) * RPP * d_row_bytes, 0, kAuxStore);
                });
            }
        });
    };

    if (f.enabled) {
        // uniform per wave: all 8-column groups of the wave exist and every access may be 128-bit
        const bool fast_ok = dvec && (n0 + wn * WTN + WTN <= p.N) && (!f.has_res || (f.res_dt & 0x100)) &&
                             (!f.has_bias || (f.bias_dt & 0x100));
#pragma unroll
        for (int e = 0; e < 8; ++e) bias8[e] = 0.f;
        if (f.has_bias) {
            const void *bp = group >= 0 ? ((const void *const *)f.bias)[group] : f.bias;
            if constexpr (kBiasAhead) decode8(bias_ahead, f.bias_dt & 0xff, bias8);
            else decode8(load8(bp, f.bias_dt & 0xff, c.n, (f.bias_dt & 0x100) != 0, n_left), f.bias_dt & 0xff, bias8);
            // (the split column mapping belongs to the fast form of the block)
            if (f_split && fast_ok) {
                const int64_t nb = n0 + wn * WTN;
                const int bdt = f.bias_dt & 0xff;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int64_t idx = nb + (e < 4 ? f_colA + e : f_colB + e - 4);
                    bias8[e] = bdt == UCL_F32 ? ((const float *)bp)[idx] : bits_to_f32(((const uint16_t *)bp)[idx], bdt);
                }
            }
        }
        if (f.has_res) {
            const void *rp = group >= 0 ? ((const void *const *)f.res)[group] : f.res;
            res_u = (const char *)rp + (int64_t)batch * f.res_bs * r_esz;
            res_base = res_u + (int64_t)c.n * r_esz;
        }
        if (f.has_scale) alpha = f.alpha;
        if (fast_ok) {
            fast_setup();
            // All block loops of the epilogue are REAL loops: their bodies are re-executed from the
            // instruction cache instead of existing once per block.
            // (two copies: without a residual the block issues no loads at all, so nothing ever makes
            // it wait for the stores in flight)
            if (f.has_res) {
                ResRegs ra, rb;
                res_issue(0, ra);
                if constexpr (!kResAhead) {
#pragma clang loop unroll(disable)
                    for (int mi = 0; mi < MI / 2; ++mi) {
                        UCL_STAGE_BLOCK(mi);
                        fast_block(std::true_type{}, mi, ra);
                    }
                } else if constexpr (MI / 2 >= 2) {
#pragma clang loop unroll(disable)
                    for (int mi = 0; mi < MI / 2; mi += 2) {          // two blocks per trip: the register sets alternate
                        res_issue(mi + 1, rb);
                        UCL_STAGE_BLOCK(mi);
                        fast_block(std::true_type{}, mi, ra);
                        if (mi + 2 < MI / 2) res_issue(mi + 2, ra);
                        UCL_STAGE_BLOCK(mi + 1);
                        fast_block(std::true_type{}, mi + 1, rb);
                    }
                } else {
                    UCL_STAGE_BLOCK(0);
                    fast_block(std::true_type{}, 0, ra);
                }
            } else {
                ResRegs none;
#pragma clang loop unroll(disable)
                for (int mi = 0; mi < MI / 2; ++mi) {
                    UCL_STAGE_BLOCK(mi);
                    fast_block(std::false_type{}, mi, none);
                }
            }
        } else {
#pragma clang loop unroll(disable)
            for (int mi = 0; mi < MI / 2; ++mi) {
                UCL_STAGE_BLOCK(mi);
                switch (f.act) {
#define UCL_FUSED_CASE(OP)                                                         \
    case OP:                                                                       \
        fused_block(std::integral_constant<int, OP>{}, mi);                        \
        break;
                    UCL_FUSED_CASE(UCL_EPI_RELU)
                    UCL_FUSED_CASE(UCL_EPI_GELU_TANH)
                    UCL_FUSED_CASE(UCL_EPI_GELU_ERF)
                    UCL_FUSED_CASE(UCL_EPI_SILU)
                    UCL_FUSED_CASE(UCL_EPI_SIGMOID)
                    UCL_FUSED_CASE(UCL_EPI_TANH)
                    UCL_FUSED_CASE(UCL_EPI_MISH)
                    UCL_FUSED_CASE(UCL_EPI_HARDSWISH)
                    UCL_FUSED_CASE(UCL_EPI_LEAKY_RELU)
                    UCL_FUSED_CASE(UCL_EPI_ELU)
                    UCL_FUSED_CASE(UCL_EPI_CLAMP)
#undef UCL_FUSED_CASE
                default:
                    fused_block(std::integral_constant<int, 0>{}, mi);
                    break;
                }
            }
        }
    } else {
    // ---- any other chain: interpreted step by step ----------------------------------------------------
        // n-indexed vectors (bias, column scale): the lane's 8 columns never change, fetch them once.
        // (All indexing of these small register arrays goes through static_for: constant indices only.)
        Raw8 nvec[kMaxNVec];
        int nvec_step[kMaxNVec], mat_step[kMaxMat];
        const char *mat_base[kMaxMat];            // AUX_LOAD operands: row-0 address of this lane's columns
        int64_t mat_ld[kMaxMat];
        int mat_dt[kMaxMat];
        int n_nvec = 0, n_mat = 0;
        static_for<kMaxNVec>([&](auto j) { nvec_step[j] = -1; });
        static_for<kMaxMat>([&](auto j) { mat_step[j] = -1; });
        for (int s = 0; s < n_steps; ++s) {
            const EpiStepDev st = get_step(s);
            const int op = st.op;
            if (op_is_nvec(op) && n_nvec < kMaxNVec) {
                static_for<kMaxNVec>([&](auto j) {
                    if (j == n_nvec) {
                        nvec_step[j] = s;
                        nvec[j] = load8(step_ptr(st, group), st.dtype & 0xff, c.n, (st.dtype & 0x100) != 0, n_left);
                    }
                });
                ++n_nvec;
            } else if (op == UCL_EPI_AUX_LOAD && n_mat < kMaxMat) {
                static_for<kMaxMat>([&](auto j) {
                    if (j == n_mat) {
                        const int esz = (st.dtype & 0xff) == UCL_F32 ? 4 : 2;
                        mat_step[j] = s;
                        mat_dt[j] = st.dtype;
                        mat_ld[j] = st.ld;
                        mat_base[j] = (const char *)step_ptr(st, group) + ((int64_t)batch * st.bs + c.n) * esz;
                    }
                });
                ++n_mat;
            }
        }

#pragma clang loop unroll(disable)
        for (int mi = 0; mi < MI / 2; ++mi) {
            UCL_STAGE_BLOCK(mi);
            const int m_blk = m0 + wm * Cfg::WTM + mi * 32;
            // passes run in groups: the matrix operands (residual) of a whole group are requested first,
            // so several row segments are in flight while the chain runs
#pragma clang loop unroll(disable)
            for (int pg = 0; pg < PASSES; pg += GRP_I) {
                Raw8 mat[GRP_I][kMaxMat];
                static_for<GRP_I>([&](auto u) {
                    const int m = m_blk + (pg + u) * RPP + e_row;
                    const int nv = m < Mloc ? n_left : 0;
                    static_for<kMaxMat>([&](auto j) {
                        if (j < n_mat)
                            mat[u][j] = load8(mat_base[j], mat_dt[j] & 0xff, (int64_t)m * mat_ld[j], (mat_dt[j] & 0x100) != 0, nv);
                    });
                });
                static_for<GRP_I>([&](auto u) {
                    const int row = (pg + u) * RPP + e_row;
                    const int m = m_blk + row;
                    c.m = m;
                    c.nvalid = m < Mloc ? n_left : 0;
                    float v[8];
                    staged_row(row, v);
                    for (int s = 0; s < n_steps; ++s) {
                        Raw8 pre;
                        pre.lo = u32x4_t{0, 0, 0, 0};
                        pre.hi = u32x4_t{0, 0, 0, 0};
                        pre.packed = false;
                        bool has_pre = false;
                        static_for<kMaxNVec>([&](auto j) {
                            if (nvec_step[j] == s) { pre = nvec[j]; has_pre = true; }
                        });
                        static_for<kMaxMat>([&](auto j) {
                            if (mat_step[j] == s) { pre = mat[u][j]; has_pre = true; }
                        });
                        apply_step(v, get_step(s), c, pre, has_pre);
                    }
                    store8(Db, dtD, d_batch_off + (int64_t)m * p.ldd + c.n, v, dvec, c.nvalid);
                });
            }
        }
    }
    if constexpr (!Cfg::PERSIST) {
        break;
    } else if constexpr (Cfg::STREAMK) {
        // the k steps of the piece are behind the workgroup
        const StreamKPiece pe = streamk_piece(wg_id, sk_end, p.sk_rounds, p.sk_ipt, p.sk_q, p.sk_deal);
        wg_id += pe.k1 - pe.k0;
        if (wg_id >= sk_end) break;
        __syncthreads();
    } else {
        wg_id += gridDim.x;
        if (wg_id >= p.total_tiles) break;
        __syncthreads();                                  // the next tile's copies overwrite the staging patch
    }
    }   // tile loop
#undef UCL_STAGE_BLOCK
}

}  // namespace ucl
