// Transform stage of the grammar's `pipeline(...)`: `transpose(tensor, NCL, NLC [, dtype_in, dtype_out])`
// (and NCHW <-> NHWC with H*W flattened): per batch a rows x cols matrix is written transposed, the
// element type converted on the way.  A pure HBM-bound kernel: 128-bit loads along the source's
// contiguous dimension, a 64x64 tile of fp32 words in LDS (row pitch 65 words, so both the row-wise
// writes and the column-wise reads touch 64 different banks per wave instruction), 128-bit stores
// along the destination's contiguous dimension.
#include <cstdio>

#include "ucl_device.h"

namespace ucl {
namespace {

typedef __attribute__((ext_vector_type(4))) uint32_t tu32x4_t;
typedef __attribute__((ext_vector_type(4))) float tf32x4_t;
typedef __attribute__((ext_vector_type(2))) float tf32x2_t;
typedef __attribute__((ext_vector_type(2))) __bf16 tbf16x2_t;
typedef __attribute__((ext_vector_type(2))) _Float16 tf16x2_t;
typedef __attribute__((ext_vector_type(8))) _Float16 tf16x8_t;

constexpr int kTile = 64, kPitch = 65;

template <int DT>
struct Elem {
    static constexpr int SIZE = DT == UCL_F32 ? 4 : 2;
    static constexpr int PER16 = 16 / SIZE;          // elements of a 128-bit access
};

// stored element -> fp32 (exact for all three types)
template <int DT>
__device__ __forceinline__ float decode(const char *p) {
    if constexpr (DT == UCL_F32) return *(const float *)p;
    else if constexpr (DT == UCL_F16) return (float)*(const _Float16 *)p;
    else return __builtin_bit_cast(float, (uint32_t)*(const uint16_t *)p << 16);
}
template <int DT>
__device__ __forceinline__ void decode16(const tu32x4_t &raw, float *v) {
    if constexpr (DT == UCL_F32) {
        const tf32x4_t f = __builtin_bit_cast(tf32x4_t, raw);
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = f[e];
    } else if constexpr (DT == UCL_F16) {
        // (the whole register group is reinterpreted at once: a bit cast of one indexed element of a
        // vector has been seen to pick element 0 for every index)
        const tf16x8_t h = __builtin_bit_cast(tf16x8_t, raw);
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = (float)h[e];
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            v[2 * e] = __builtin_bit_cast(float, raw[e] << 16);
            v[2 * e + 1] = __builtin_bit_cast(float, raw[e] & 0xffff0000u);
        }
    }
}
// fp32 -> stored element, round to nearest even
template <int DT>
__device__ __forceinline__ void encode(char *p, float x) {
    if constexpr (DT == UCL_F32) *(float *)p = x;
    else if constexpr (DT == UCL_F16) *(_Float16 *)p = (_Float16)x;
    else *(__bf16 *)p = (__bf16)x;
}
template <int DT>
__device__ __forceinline__ tu32x4_t encode16(const float *v) {
    tu32x4_t o;
    if constexpr (DT == UCL_F32) {
        o = __builtin_bit_cast(tu32x4_t, tf32x4_t{v[0], v[1], v[2], v[3]});
    } else if constexpr (DT == UCL_F16) {
#pragma unroll
        for (int e = 0; e < 4; ++e)
            o[e] = __builtin_bit_cast(uint32_t, __builtin_convertvector(tf32x2_t{v[2 * e], v[2 * e + 1]}, tf16x2_t));
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e)
            o[e] = __builtin_bit_cast(uint32_t, __builtin_convertvector(tf32x2_t{v[2 * e], v[2 * e + 1]}, tbf16x2_t));
    }
    return o;
}

// One 64x64 tile per workgroup.  vec_in / vec_out: the source rows / destination rows are 16-byte
// aligned and a whole number of 128-bit groups long, so a group never straddles the matrix edge.
template <int SRC, int DST>
__global__ __launch_bounds__(kThreads) void transpose_kernel(const char *src, char *dst, int rows, int cols, int tiles_r,
                                                             int tiles_c, int vec_in, int vec_out) {
    constexpr int ES = Elem<SRC>::SIZE, ED = Elem<DST>::SIZE, CI = Elem<SRC>::PER16, CO = Elem<DST>::PER16;
    __shared__ float tile[kTile * kPitch];
    const int tid = threadIdx.x;
    int t = blockIdx.x;
    const int tc = t % tiles_c;
    t /= tiles_c;
    const int tr = t % tiles_r;
    const int b = t / tiles_r;
    const int r0 = tr * kTile, c0 = tc * kTile;
    const int64_t plane = (int64_t)rows * cols;
    const char *s = src + (int64_t)b * plane * ES;
    char *d = dst + (int64_t)b * plane * ED;

    // source rows -> LDS: consecutive lanes take consecutive 128-bit groups of a row
    constexpr int GI = kTile / CI;                       // groups per tile row
#pragma unroll
    for (int i = 0; i < kTile * GI / kThreads; ++i) {
        const int q = i * kThreads + tid;
        const int r = q / GI, cc = (q % GI) * CI;
        const int gr = r0 + r, gc = c0 + cc;
        float v[CI];
#pragma unroll
        for (int e = 0; e < CI; ++e) v[e] = 0.f;
        if (gr < rows && gc < cols) {
            const char *p = s + ((int64_t)gr * cols + gc) * ES;
            if (vec_in) {
                // every byte is touched exactly once: non-temporal accesses keep the stream from
                // displacing itself in the caches (measured 5.3 -> 5.9 TB/s on a 308 MB problem)
                decode16<SRC>(__builtin_nontemporal_load((const tu32x4_t *)p), v);
            } else {
#pragma unroll
                for (int e = 0; e < CI; ++e)
                    if (gc + e < cols) v[e] = decode<SRC>(p + e * ES);
            }
        }
#pragma unroll
        for (int e = 0; e < CI; ++e) tile[r * kPitch + cc + e] = v[e];
    }
    __syncthreads();
    // LDS columns -> destination rows: consecutive lanes take consecutive 128-bit groups of a destination row
    constexpr int GO = kTile / CO;
#pragma unroll
    for (int i = 0; i < kTile * GO / kThreads; ++i) {
        const int q = i * kThreads + tid;
        const int c = q / GO, rr = (q % GO) * CO;
        const int gc = c0 + c, gr = r0 + rr;
        if (gc < cols && gr < rows) {
            float v[CO];
#pragma unroll
            for (int e = 0; e < CO; ++e) v[e] = tile[(rr + e) * kPitch + c];
            char *p = d + ((int64_t)gc * rows + gr) * ED;
            if (vec_out) {
                __builtin_nontemporal_store(encode16<DST>(v), (tu32x4_t *)p);
            } else {
#pragma unroll
                for (int e = 0; e < CO; ++e)
                    if (gr + e < rows) encode<DST>(p + e * ED, v[e]);
            }
        }
    }
}

thread_local char g_terr[256] = "";

template <int SRC, int DST>
hipError_t launch_t(const void *src, void *dst, int rows, int cols, int tiles_r, int tiles_c, int grid, int vi, int vo,
                    hipStream_t st) {
    hipLaunchKernelGGL((transpose_kernel<SRC, DST>), dim3(grid), dim3(kThreads), 0, st, (const char *)src, (char *)dst, rows, cols,
                       tiles_r, tiles_c, vi, vo);
    return hipGetLastError();
}

}  // namespace

const char *transpose_last_error() { return g_terr; }

ucl_status transpose_run(int64_t batch, int64_t rows, int64_t cols, const void *src, int32_t dt_src, void *dst, int32_t dt_dst,
                         void *stream) {
    g_terr[0] = 0;
    auto fail = [&](ucl_status st, const char *msg) {
        snprintf(g_terr, sizeof(g_terr), "%s", msg);
        return st;
    };
    auto valid = [](int dt) { return dt == UCL_F32 || dt == UCL_F16 || dt == UCL_BF16; };
    if (batch < 0 || rows < 0 || cols < 0) return fail(UCL_ERR_INVALID_ARG, "transpose extents must be non-negative");
    if (!valid(dt_src) || !valid(dt_dst)) return fail(UCL_ERR_INVALID_ARG, "transpose: element types must be fp32, fp16 or bf16");
    if (batch == 0 || rows == 0 || cols == 0) return UCL_OK;         // nothing to move
    if (!src || !dst) return fail(UCL_ERR_INVALID_ARG, "transpose: src and dst must be non-NULL device pointers");
    {
        // out of place only: a tile of the destination is written while other tiles of the source are still unread
        const uintptr_t s0 = reinterpret_cast<uintptr_t>(src), d0 = reinterpret_cast<uintptr_t>(dst);
        const uintptr_t sn = (uintptr_t)(batch * rows * cols) * (dt_src == UCL_F32 ? 4 : 2);
        const uintptr_t dn = (uintptr_t)(batch * rows * cols) * (dt_dst == UCL_F32 ? 4 : 2);
        if (s0 < d0 + dn && d0 < s0 + sn)
            return fail(UCL_ERR_INVALID_ARG, "transpose works out of place: the byte ranges of src and dst overlap");
    }
    if (rows >= (1ll << 31) - kTile || cols >= (1ll << 31) - kTile)
        return fail(UCL_ERR_UNSUPPORTED, "transpose: rows and cols must be below 2^31");
    const int64_t tiles_r = (rows + kTile - 1) / kTile, tiles_c = (cols + kTile - 1) / kTile;
    const int64_t grid = batch * tiles_r * tiles_c;
    if (grid >= (1ll << 31)) return fail(UCL_ERR_UNSUPPORTED, "transpose: more than 2^31 tiles of 64x64 elements");
    const int es = dt_src == UCL_F32 ? 4 : 2, ed = dt_dst == UCL_F32 ? 4 : 2;
    const int vi = (reinterpret_cast<uintptr_t>(src) % 16 == 0) && (cols % (16 / es) == 0);
    const int vo = (reinterpret_cast<uintptr_t>(dst) % 16 == 0) && (rows % (16 / ed) == 0);
    hipStream_t st = (hipStream_t)stream;
    hipError_t e = hipSuccess;
#define UCL_T_CASE(S, D) \
    if (dt_src == S && dt_dst == D) e = launch_t<S, D>(src, dst, (int)rows, (int)cols, (int)tiles_r, (int)tiles_c, (int)grid, vi, vo, st);
    UCL_T_CASE(UCL_F32, UCL_F32) UCL_T_CASE(UCL_F32, UCL_F16) UCL_T_CASE(UCL_F32, UCL_BF16)
    UCL_T_CASE(UCL_F16, UCL_F32) UCL_T_CASE(UCL_F16, UCL_F16) UCL_T_CASE(UCL_F16, UCL_BF16)
    UCL_T_CASE(UCL_BF16, UCL_F32) UCL_T_CASE(UCL_BF16, UCL_F16) UCL_T_CASE(UCL_BF16, UCL_BF16)
#undef UCL_T_CASE
    if (e != hipSuccess) {
        snprintf(g_terr, sizeof(g_terr), "transpose kernel launch failed: %s", hipGetErrorString(e));
        return UCL_ERR_LAUNCH;
    }
    return UCL_OK;
}

}  // namespace ucl
