// Sanitizer driver for the host-only paths of the C ABI (test infrastructure): the SOL arithmetic for
// every operation kind, the tile schedule enumerated over ragged group tables, and the validation
// paths that return before any launch.  Linked against the library's host code with EMPTY kernel
// variant tables (no GPU is touched).  Exit code 0 and no ASan / UBSan report = pass.
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <set>
#include <tuple>
#include <vector>

#include "ucl.h"

static int fails = 0;
#define EXPECT(c) do { if (!(c)) { std::fprintf(stderr, "line %d: %s\n", __LINE__, #c); ++fails; } } while (0)

int main() {
    // ---- SOL for the six operation kinds, default and explicit hardware descriptors
    const int64_t Mg[5] = {128, 0, 2048, 640, 1};
    for (int op = UCL_OP_GEMM; op <= UCL_OP_CONV2D_WGRAD; ++op) {
        ucl_problem p;
        std::memset(&p, 0, sizeof p);
        p.op = op; p.dt_in = UCL_BF16; p.dt_out = UCL_F32;
        p.batch = 3; p.M = 300; p.N = 200; p.K = 64; p.groups = 5; p.M_g = Mg;
        p.cN = 2; p.cH = 9; p.cW = 7; p.cC = 16; p.cKout = 24; p.cR = 3; p.cS = 3;
        p.pad_h = p.pad_w = 1; p.stride_h = 2; p.stride_w = 1; p.dil_h = p.dil_w = 1;
        ucl_epilogue e;
        std::memset(&e, 0, sizeof e);
        e.n_steps = 3;
        e.steps[0].op = UCL_EPI_BIAS; e.steps[0].dtype = UCL_BF16;
        e.steps[1].op = UCL_EPI_AUX_LOAD; e.steps[1].dtype = UCL_F16;
        e.steps[2].op = UCL_EPI_PER_ROW_SCALE; e.steps[2].dtype = UCL_F32;
        p.epi = &e;
        ucl_sol_report r;
        EXPECT(ucl_sol_bound(&p, nullptr, &r) == UCL_OK);
        EXPECT(r.flops > 0 && r.bytes > 0 && r.t_sol >= r.t_compute && r.t_sol >= r.t_mem);
        ucl_hw hw = {1e15, 1e14, 3.35e12, 1500.0 / 1980.0, 1.0, 2e15};
        EXPECT(ucl_sol_bound(&p, &hw, &r) == UCL_OK);
        p.dt_in = UCL_FP8_E4M3;
        EXPECT(ucl_sol_bound(&p, &hw, &r) == UCL_OK && r.peak_flops == 2e15 * (1500.0 / 1980.0));
        hw.peak_bw = 0;
        EXPECT(ucl_sol_bound(&p, &hw, &r) == UCL_ERR_INVALID_ARG);
        p.dt_in = 99;
        EXPECT(ucl_sol_bound(&p, nullptr, &r) == UCL_ERR_INVALID_ARG);
        ucl_tuning t;
        p.dt_in = UCL_BF16;
        (void)ucl_select_tuning(&p, &t);                 // no variants are linked in: must fail cleanly
        int64_t bytes = -1;
        int32_t slices = -1;
        (void)ucl_workspace_size(&p, nullptr, &bytes, &slices);
    }
    EXPECT(ucl_sol_bound(nullptr, nullptr, nullptr) == UCL_ERR_INVALID_ARG);
    {
        ucl_problem p;
        std::memset(&p, 0, sizeof p);
        p.op = UCL_OP_GROUPED_GEMM; p.dt_in = p.dt_out = UCL_BF16; p.groups = 2; p.N = 8; p.K = 8;
        ucl_sol_report r;
        EXPECT(ucl_sol_bound(&p, nullptr, &r) == UCL_ERR_INVALID_ARG);      // M_g missing
        p.op = 77;
        EXPECT(ucl_sol_bound(&p, nullptr, &r) == UCL_ERR_INVALID_ARG);
    }
    // ---- tile schedule: a bijection for ragged group tables and every raster width
    for (int raster : {1, 2, 3, 4, 8, 16, 64}) {
        const std::vector<std::vector<int32_t>> tables = {{16}, {3, 0, 5, 1}, {1}, {0, 0, 7}, {9, 2}, {5, 5, 5, 5, 5, 5, 5, 5, 5}};
        for (const auto &tm : tables)
            for (int tn : {1, 3, 7, 16}) {
                int total = 0;
                for (int v : tm) total += v * tn;
                std::set<std::tuple<int, int, int>> seen;
                for (int wg = 0; wg < total; ++wg) {
                    int32_t g, a, b;
                    EXPECT(ucl_tile_map((int32_t)tm.size(), tm.data(), tn, raster, wg, &g, &a, &b) == UCL_OK);
                    EXPECT(g >= 0 && g < (int)tm.size() && a >= 0 && a < tm[g] && b >= 0 && b < tn);
                    seen.insert({g, a, b});
                }
                EXPECT((int)seen.size() == total);
                int32_t g, a, b;
                EXPECT(ucl_tile_map((int32_t)tm.size(), tm.data(), tn, raster, total, &g, &a, &b) == UCL_ERR_INVALID_ARG);
            }
    }
    // ---- validation that returns before any launch (16-byte aligned fake addresses, never dereferenced)
    void *P = reinterpret_cast<void *>(4096);
    EXPECT(ucl_gemm(0, 64, 64, P, UCL_BF16, 64, 1, P, UCL_BF16, 1, 64, P, UCL_BF16, 64, 1, nullptr, nullptr, nullptr) == UCL_ERR_INVALID_ARG);
    EXPECT(ucl_gemm(64, 64, 60, P, UCL_BF16, 60, 1, P, UCL_BF16, 1, 60, P, UCL_BF16, 64, 1, nullptr, nullptr, nullptr) == UCL_ERR_UNSUPPORTED);
    EXPECT(ucl_gemm(64, 64, 72, P, UCL_FP8_E4M3, 72, 1, P, UCL_FP8_E4M3, 1, 72, P, UCL_BF16, 64, 1, nullptr, nullptr, nullptr) == UCL_ERR_UNSUPPORTED);
    EXPECT(ucl_gemm(64, 64, 64, P, UCL_BF16, 64, 1, P, UCL_BF16, 1, 64, P, UCL_BF16, 64, 1, nullptr, nullptr, nullptr) == UCL_ERR_UNSUPPORTED);   // no kernels linked
    ucl_epilogue bad;
    std::memset(&bad, 0, sizeof bad);
    bad.n_steps = 9;
    EXPECT(ucl_gemm(64, 64, 64, P, UCL_BF16, 64, 1, P, UCL_BF16, 1, 64, P, UCL_BF16, 64, 1, &bad, nullptr, nullptr) == UCL_ERR_INVALID_ARG);
    const int64_t neg[2] = {64, -1};
    EXPECT(ucl_grouped_gemm(2, neg, 64, 64, (const void *const *)P, UCL_BF16, 64, 1, (const void *const *)P, UCL_BF16, 1, 64, (void *const *)P, UCL_BF16, 64, 1, nullptr, nullptr, nullptr) == UCL_ERR_INVALID_ARG);
    EXPECT(ucl_conv2d_fprop(1, 8, 8, 3, 8, 3, 3, 1, 1, 1, 1, 1, 1, P, UCL_BF16, P, UCL_BF16, P, UCL_BF16, nullptr, nullptr, nullptr) == UCL_ERR_UNSUPPORTED);
    EXPECT(ucl_conv2d_dgrad(1, 8, 8, 8, 12, 3, 3, 1, 1, 1, 1, 1, 1, P, UCL_BF16, P, UCL_BF16, P, UCL_BF16, nullptr, nullptr, nullptr) == UCL_ERR_UNSUPPORTED);
    EXPECT(ucl_conv2d_wgrad(1, 2, 2, 8, 8, 5, 5, 0, 0, 1, 1, 1, 1, P, UCL_BF16, P, UCL_BF16, P, UCL_BF16, nullptr, nullptr, nullptr) == UCL_ERR_INVALID_ARG);
    EXPECT(ucl_transpose(1, 64, 64, P, UCL_F32, P, UCL_F32, nullptr) == UCL_ERR_INVALID_ARG);
    EXPECT(ucl_transpose(0, 64, 64, nullptr, UCL_F32, nullptr, UCL_F32, nullptr) == UCL_OK);
    EXPECT(ucl_workspace_init(nullptr, 1 << 20, nullptr) == UCL_ERR_INVALID_ARG);
    EXPECT(ucl_workspace_init(P, 16, nullptr) == UCL_ERR_WORKSPACE);
    ucl_variant_info vi;
    EXPECT(ucl_num_variants() == 0 && ucl_variant(0, &vi) == UCL_ERR_INVALID_ARG);
    EXPECT(std::strlen(ucl_last_error()) > 0 && std::strlen(ucl_status_string(UCL_ERR_WORKSPACE)) > 0 && std::strlen(ucl_version()) > 0);
    if (fails) { std::fprintf(stderr, "%d checks failed\n", fails); return 1; }
    std::printf("host API sanitizer driver: ok\n");
    return 0;
}
