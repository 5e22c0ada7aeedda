// Types shared by the host launch code and the gfx950 kernels of this library.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/ucl.h"

namespace ucl {

constexpr int kThreads = 256;         // 4 wavefronts of 64 lanes, one per SIMD of a CU
constexpr int kLdsBytesPerCU = 160 * 1024;

struct EpiStepDev {
    int32_t op;
    int32_t dtype;
    float p0, p1;
    const void *ptr;
    int64_t ld;
    int64_t bs;
};

// A chain of the common shape  act( alpha * acc + bias[n] + beta * R[m,n] )  -- any of the four parts
// optional, in that order -- is recognised on the host and runs through straight-line epilogue code;
// every other chain is interpreted step by step.
struct FusedEpi {
    int32_t enabled;
    int32_t has_scale, has_bias, has_res;
    int32_t act;                      // ucl_epi_op of the activation, 0 = none
    int32_t bias_dt, res_dt;          // ucl_dtype | 0x100 if 128-bit access is allowed
    int32_t pad_;
    float alpha, beta, act_p0, act_p1;
    const void *bias;                 // grouped: device table of per-group pointers
    const void *res;
    int64_t res_ld, res_bs;
};

// Kernel arguments, passed by value (kernarg segment).
struct KParams {
    const void *A;
    const void *B;
    void *D;
    const void *const *A_g;           // grouped: device tables of per-group pointers
    const void *const *B_g;
    void *const *D_g;
    int64_t lda, ldb, ldd;            // element stride of the non-contiguous dimension
    int64_t a_bs, b_bs, d_bs;         // batch strides (elements)
    int64_t a_bytes;                  // conv fprop / dgrad: size in bytes (< 2^31) of the tensor A is gathered from
    int64_t b_bytes;                  // conv dgrad: size of the filter in bytes; wgrad: of the activations B is gathered from
    int32_t M, N, K;                  // grouped: M unused (per-group table)
    int32_t tiles_m, tiles_n;         // per batch (non-grouped)
    int32_t tiles_per_batch, total_tiles;
    int32_t raster;                   // band width in tile rows
    int32_t dtD;                      // ucl_dtype of D
    int32_t d_vec;                    // 1: D (and aux tensors) may be accessed with 4-element vectors
    int32_t groups;
    // conv2d geometry (implicit-GEMM A operand): x [N,H,W,C]
    int32_t cH, cW, cC, cS, cP, cQ;
    int32_t pad_h, pad_w, str_h, str_w, dil_h, dil_w;
    int32_t n_steps;
    // split-K (gemm / batched): number of K slices (<= 1: none), K extent of a slice (multiple of 64),
    // phase 0 = one launch, the last workgroup to arrive at a tile adds up; 1 = write partial tiles only;
    // 2 = add up only
    int32_t split_k, k_per_slice, split_phase;
    int32_t sk_ipt, sk_q, sk_rounds;  // stream-K: 64-wide k steps per tile, k steps of the remaining tiles per workgroup, whole rounds
    int32_t sk_deal;                  // stream-K: remaining tiles if sk_q divides sk_ipt (runs are dealt k range by k range), else 0
    float *ws_partials;
    uint32_t *ws_counters;
    EpiStepDev steps[UCL_MAX_EPI_STEPS];   // must stay addressable as offsetof(KParams, steps)
    FusedEpi fused;
};

struct GroupTable {
    int32_t m[UCL_MAX_GROUPS];              // rows of each group
    int32_t tile_start[UCL_MAX_GROUPS + 1]; // prefix sum of tiles per group
};
struct NoGroupTable {};

// ---- tile schedule: the same code runs on the host (tests, introspection) and in the kernels ----

// Workgroups are dealt to the 8 XCDs round-robin by id, and each XCD has its own L2.  Give XCD x
// one contiguous run of the tile sequence so that the tiles resident on an XCD at the same time
// are neighbours and share A / B panels through that L2.  Bijective on [0, total).
__host__ __device__ inline int xcd_remap(int wg, int total) {
    const int q = total >> 3, r = total & 7;
    const int x = wg & 7, loc = wg >> 3;
    return x * q + (x < r ? x : r) + loc;
}

// Stream-K: the piece a workgroup stands at after `done` k steps of its run of `end` (see the kernel's tile loop).
// The first rounds * ipt k steps are whole tiles, tile number round * grid + workgroup; the rest is the workgroup's
// run [g * q, ...) of the k steps of the remaining tiles, numbered tile by tile.
struct StreamKPiece {
    int tile;        // in the numbering that xcd_remap deals to the XCDs
    int rest_tile;   // index among the remaining tiles (-1: a whole tile of the first rounds)
    int g;           // the workgroup's run (streamk_run)
    int k0, k1;      // 64-wide k steps [k0, k1) of the tile
};
// The run a workgroup takes: run g covers k steps [g * q, (g + 1) * q) of the remaining tiles.  Workgroups are
// taken in XCD-run order (u).  Where q divides ipt every tile falls into the same ipt / q k ranges, and the runs are
// dealt k range by k range: the workgroups of an XCD work on one k range of many tiles, which read the same
// columns of A and B rows and share them in its L2 (tile by tile they would share nothing).  Bijective on [0, grid).
__host__ __device__ inline int streamk_run(int wg, int grid, int deal_tiles, int ipt, int q) {
    const int u = xcd_remap(wg, grid);
    if (deal_tiles > 0) {
        const int parts = ipt / q;
        if (u < deal_tiles * parts) return (u % deal_tiles) * parts + u / deal_tiles;
    }
    return u;
}
#if defined(__HIPCC__)
__device__ inline StreamKPiece streamk_piece(int done, int end, int rounds, int ipt, int q, int deal_tiles) {
    StreamKPiece pc;
    const int grid = (int)gridDim.x;
    pc.g = streamk_run((int)blockIdx.x, grid, deal_tiles, ipt, q);
    if (done < rounds * ipt) {
        pc.tile = (done / ipt) * grid + (int)blockIdx.x;
        pc.rest_tile = -1;
        pc.k0 = 0;
        pc.k1 = ipt;
    } else {
        const int it = done - rounds * ipt + pc.g * q;
        pc.rest_tile = it / ipt;
        pc.tile = rounds * grid + pc.rest_tile;
        pc.k0 = it - pc.rest_tile * ipt;
        pc.k1 = pc.k0 + (end - done) < ipt ? pc.k0 + (end - done) : ipt;
    }
    return pc;
}
#endif

// Walk a tiles_m x tiles_n grid in bands of `gm` tile rows, column by column inside a band.
__host__ __device__ inline void band_raster(int t, int tiles_m, int tiles_n, int gm, int &tm, int &tn) {
    const int per_band = gm * tiles_n;
    const int band = t / per_band;
    const int first = band * gm;
    const int rows = (tiles_m - first) < gm ? (tiles_m - first) : gm;
    const int r = t - band * per_band;
    tm = first + r % rows;
    tn = r / rows;
}

// Largest g with tile_start[g] <= t  (tile_start[0] = 0, tile_start[groups] = total > t).
__host__ __device__ inline int find_group(const int32_t *tile_start, int groups, int t) {
    int lo = 0, hi = groups;          // invariant: tile_start[lo] <= t < tile_start[hi]
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (tile_start[mid] <= t) lo = mid; else hi = mid;
    }
    return lo;
}

}  // namespace ucl
