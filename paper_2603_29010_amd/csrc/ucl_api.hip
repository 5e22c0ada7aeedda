// Host side of the C ABI declared in include/ucl.h: argument validation with explanatory
// errors, the per-problem tile / stage selection table, the launch, and the SOL analysis.
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <vector>

#include <mutex>

#include "ucl_kernel.h"      // the epilogue's element-wise arithmetic (the split-K reduction kernel finishes simple chains itself)
#include "ucl_variants.h"

// Split-K workspace of ucl_gemm_static_workspace: counters followed by partial tiles, held by every
// GPU the library runs on until the process ends.  Host code never uses this name as an address: it
// asks the runtime for the array's device address once per device (static_workspace() below).
static __device__ __align__(256) unsigned char scratch[UCL_STATIC_WORKSPACE_BYTES];

namespace ucl {
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
// the transform stage lives in its own unit
ucl_status transpose_run(int64_t batch, int64_t rows, int64_t cols, const void *src, int32_t dt_src, void *dst, int32_t dt_dst,
                         void *stream);
const char *transpose_last_error();

namespace {

thread_local char g_err[512] = "";

ucl_status fail(ucl_status st, const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return st;
}

const std::vector<VariantDesc> &all_variants() {
    static const std::vector<VariantDesc> v = [] {
        std::vector<VariantDesc> out;
        for (VariantList l : {variants_gemm_kk_bf16_a(), variants_gemm_kk_bf16_b(), variants_gemm_kk_bf16_c(), variants_gemm_kk_bf16_d(), variants_gemm_kk_f16_a(), variants_gemm_kk_f16_b(), variants_gemm_mn_bf16(), variants_gemm_mn_f16(), variants_grouped_a(), variants_grouped_b(), variants_conv_a(), variants_conv_b(), variants_conv_f16(), variants_conv_halo(), variants_gemm_kn_bf16(), variants_gemm_kn_f16(), variants_gemm_mx_bf16(), variants_gemm_mx_f16(), variants_grouped_kn(), variants_conv_dgrad(), variants_conv_dgrad_halo(), variants_conv_wgrad(), variants_gemm_kk_fp8(), variants_persistent(), variants_grouped_fp8_e4m3(), variants_grouped_fp8_e5m2(), variants_streamk()})
            for (int i = 0; i < l.n; ++i) out.push_back(l.v[i]);
        return out;
    }();
    return v;
}

bool is8(int dt) { return dt == UCL_FP8_E4M3 || dt == UCL_FP8_E5M2; }
int elem_size(int dt) { return dt == UCL_F32 ? 4 : is8(dt) ? 1 : 2; }
bool is16(int dt) { return dt == UCL_F16 || dt == UCL_BF16; }
bool valid_dtype(int dt) { return dt == UCL_F32 || dt == UCL_F16 || dt == UCL_BF16; }     // outputs and epilogue tensors
const char *dtype_name(int dt) {
    return dt == UCL_F32 ? "fp32" : dt == UCL_F16 ? "fp16" : dt == UCL_BF16 ? "bf16" : dt == UCL_FP8_E4M3 ? "fp8_e4m3"
           : dt == UCL_FP8_E5M2 ? "fp8_e5m2" : "?";
}
// input type code of the kernel variants
int dt_code(int dt) { return dt == UCL_F16 ? 1 : dt == UCL_FP8_E4M3 ? 2 : dt == UCL_FP8_E5M2 ? 3 : 0; }
bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

bool op_has_tensor(int op) {
    switch (op) {
    case UCL_EPI_BIAS: case UCL_EPI_AUX_LOAD: case UCL_EPI_PER_ROW_SCALE: case UCL_EPI_PER_COL_SCALE:
    case UCL_EPI_ROW_BROADCAST: case UCL_EPI_COL_BROADCAST: case UCL_EPI_AUX_STORE:
        return true;
    default:
        return false;
    }
}
bool op_is_matrix(int op) { return op == UCL_EPI_AUX_LOAD || op == UCL_EPI_AUX_STORE; }

// ---- generic description of one launch, filled by the four entry points -------------------------
struct Launch {
    int mode = 0;                 // 0 gemm / batched, 1 grouped, 2 conv fprop, 3 conv dgrad, 4 conv wgrad
    int64_t batch = 1, M = 0, N = 0, K = 0;
    int la = 0, lb = 0;           // operand layouts
    int dt = 0;                   // input type code of the kernels: 0 bf16, 1 fp16, 2 fp8 e4m3, 3 fp8 e5m2
    int dtD = 0;
    int groups = 0;
    const int64_t *M_g = nullptr;
    int64_t max_Mg = 0, sum_Mg = 0;
    int patch_c = 0;              // conv: the problem fits the resident-patch kernels built for pixels of this many channels (0: none)
    bool ndirect_ok = false;      // B contiguous along N and small enough for 32-bit byte offsets: direct-copy kernels apply
    bool mdirect_ok = false;      // the same for A contiguous along M
};

// The resident-patch conv kernels hold pixels of 64 or 128 channels and address the taps of a 3x3 filter at unit
// stride / dilation with one pad pixel, the image row (plus one pixel) on either side of a tile in LDS.  fprop: the
// pixels are those of the activations (C channels); data gradient: those of the output gradient (Kout channels;
// P = H and Q = W follow from the geometry), taps mirrored.  Returns the channel count, 0 if the kernels do not apply.
int conv_patch_channels(int64_t W, int64_t channels, int64_t R, int64_t S, int64_t pad_h, int64_t pad_w, int64_t str_h,
                        int64_t str_w, int64_t dil_h, int64_t dil_w) {
    const bool ok = (channels == 64 || channels == 128) && R == 3 && S == 3 && pad_h == 1 && pad_w == 1 && str_h == 1 &&
                    str_w == 1 && dil_h == 1 && dil_w == 1 && W + 1 <= 59;
    return ok ? (int)channels : 0;
}

// Per-problem selection table: of the variants built for this (mode, input type, operand layouts)
// take the one with the smallest estimated time
//     ceil(tiles / 256) * ( tile FLOPs / (rate of a busy CU with this variant)
//                           + (fixed cost of a tile) / (workgroups of the variant that share a CU) ),
// i.e. the tiles dealt to the busiest CU one after the other, each paying its MFMA time at the rate
// measured for the variant (4096^3 bf16 problem, relative to the best variant) and its un-overlapped
// prologue + store time unless a co-resident workgroup hides it.  Large compute-bound problems thus get
// 256x256 tiles and the two-buffer loop, short-K / wide-output problems get the largest tile of which
// two workgroups fit on a CU, small problems the tile that fills the chip.
int64_t count_tiles(const Launch &L, int tm, int tn) {
    const int64_t tiles_n = (L.N + tn - 1) / tn;
    if (L.mode == 1) {
        int64_t t = 0;
        for (int g = 0; g < L.groups; ++g) t += (L.M_g[g] + tm - 1) / tm * tiles_n;
        return t;
    }
    return L.batch * ((L.M + tm - 1) / tm) * tiles_n;
}

// The wide epilogue path addresses a wave's row panel (up to 128 rows) with 32-bit byte offsets.
constexpr int64_t kMaxWideLd = 1ll << 21;

// Workgroups of a variant that fit on one CU: 512 registers per lane and SIMD (the kernels are built
// with a budget by tile area), 160 KB of LDS.
int workgroups_per_cu(const VariantDesc &v) {
    const int64_t area = (int64_t)v.tile_m * v.tile_n;
    const int by_regs = area >= 256 * 256 ? 1 : area >= 256 * 128 ? 2 : area >= 128 * 128 ? 3 : 4;
    const int by_lds = v.lds_bytes > 0 ? kLdsBytesPerCU / v.lds_bytes : 8;
    return by_regs < by_lds ? by_regs : by_lds;
}

// Rate of a CU that is busy with variant v, relative to the best variant (measured, see above).
double relative_rate(const VariantDesc &v) {
    const int64_t area = (int64_t)v.tile_m * v.tile_n;
    const bool two_buf = v.stages == 2 && v.tile_k == 64 && v.lb != 1 && v.la != 1;
    if (v.la == 1 || v.lb == 1) return area >= 128 * 128 ? 0.30 : 0.20;     // register-transposed operands
    const double nd = (v.lb == 4 ? 0.95 : 1.0) * (v.la == 5 ? 0.9 : 1.0);   // two LDS reads per fragment of a directly copied operand
    // conv from a resident patch: above the gather kernels.  (A 256-row tile with 128-channel pixels is alone on its
    // CU, with nothing to run while its 96 KB patch loads: measured 32 us against 27 us for the 128-row tile.)
    if (v.la == 3) return 2 * v.lds_bytes > kLdsBytesPerCU ? 0.65 : 0.85;
    if (area >= 256 * 256) return nd * (two_buf ? 1.00 : v.stages >= 5 ? 0.92 : 0.90);
    if (area >= 256 * 128) return nd * (two_buf ? 0.81 : v.stages == 3 ? 0.80 : 0.73);
    // (with a directly copied operand the two-buffer loop of this size measured below the 4-stage one)
    if (area >= 128 * 128) return nd * (two_buf ? (nd < 1.0 ? 0.62 : 0.86) : v.tile_k == 32 ? (v.stages >= 4 ? 0.67 : 0.65) : 0.58);
    return nd * (v.tile_k == 64 ? 0.49 : v.stages == 3 ? 0.41 : 0.37);
}

double estimate_seconds(const VariantDesc &v, const Launch &L) {
    const double kCuRate = 1.38e15 / 256;            // FLOP/s of one CU at the best variant's measured rate
    const double kCuStore = 4.6e12 / 256;            // B/s of output one CU gets when all CUs store
    const int wg = workgroups_per_cu(v);
    const int64_t tiles = count_tiles(L, v.tile_m, v.tile_n);
    const int64_t slots = 256 * (int64_t)wg;
    // tiles the busiest CU works through: they run wg at a time, a new set starting when slots free up
    const double per_cu = tiles <= slots ? (double)((tiles + 255) / 256) : (double)((tiles + slots - 1) / slots * wg);
    // the chip is power-limited: CUs run faster when fewer of them are busy (measured ~1.5x at 144 of 256)
    const double active = tiles / per_cu < 256.0 ? tiles / per_cu : 256.0;
    double boost = pow(256.0 / (active < 1.0 ? 1.0 : active), 0.7);
    if (boost > 1.5) boost = 1.5;
    // (8-bit inputs: K counts pairs, and the 8-bit MFMA used runs at the 16-bit rate per byte of operand)
    const double tile_flops = 2.0 * v.tile_m * v.tile_n * (double)L.K;
    const double out_bytes = (double)v.tile_m * v.tile_n * (L.dtD == UCL_F32 ? 4.0 : 2.0);
    const double fixed = 2.0e-6 + out_bytes / kCuStore;
    // co-resident workgroups hide about half of what perfect overlap of one's fixed cost with the
    // others' MFMA time would; a CU with a single tile has nothing to overlap with
    const double exposed = per_cu > 1.0 ? 0.5 * (1.0 + 1.0 / wg) : 1.0;
    // a variant built to share its CU runs below its rate when it has the CU to itself (one wave per SIMD
    // with the register budget of two: measured 0.7x for 256x128 tiles)
    const double alone = (wg >= 2 && per_cu < 2.0) ? 0.7 : 1.0;
    return per_cu * (tile_flops / (relative_rate(v) * alone * kCuRate * boost) + fixed * exposed);
}

constexpr int kNumCUs = 256;

// Slices a split-K launch of `total_tiles` tiles gets: as asked for, or (0) enough to give every CU a workgroup
// while each keeps at least 4 x 64 of K; slices are whole multiples of 64 along K.
// The weight gradient in parallel mode gets two workgroups per CU where the variant fits twice: its gathered operand
// leaves a lone workgroup waiting (measured 36.7 -> 32.6 us on 32x56x56x64 -> 128), and the streaming reduction
// kernel takes the extra partial tiles in its stride; the GEMMs measured best with one (256x256x16384: 15.0 us with
// 16 slices, 16.9 with 32).
int split_fill(const Launch &L, const VariantDesc &v, const ucl_tuning *tune) {
    return L.mode == 4 && tune->split_k_mode == UCL_SPLIT_K_PARALLEL && workgroups_per_cu(v) >= 2 ? 2 * kNumCUs : kNumCUs;
}
void split_slices(const Launch &L, int64_t want, int64_t total_tiles, int fill, int &slices, int &k_per_slice) {
    const int64_t kt = (L.K + 63) / 64;
    if (want == 0) {
        want = total_tiles >= fill ? 1 : (fill + total_tiles - 1) / total_tiles;
        if (want > kt / 4) want = kt / 4;
        if (want < 1) want = 1;
    }
    if (want > kt) want = kt;
    const int64_t per = (kt + want - 1) / want;
    k_per_slice = (int)(per * 64);
    slices = (int)((kt + per - 1) / per);
}

// Launch time of variant v under split-K, for the choice among the variants when the caller names no tile.
// What counts differs from the unsplit case.  Every CU has a workgroup, so the mainloop is bound by one of: the
// operand bytes all workgroups together copy into LDS (measured ~10 TB/s over the chip when they stream from
// HBM, ~16 TB/s when the operands stay in the L2s), the MFMA rate, or a workgroup's own chain of copies (stages-1
// k-tiles in flight, a round trip of ~1.5 us from HBM, ~0.8 us from L2).  The partial tiles then cross memory:
// in parallel mode through a streaming reduction kernel and two more launches (measured: 6 us plus 1 us per MB
// of partial tiles; chains the reduction kernel finishes itself need one launch less, which is the same for every
// tile and is left out of the comparison), in serial mode through the last workgroup of each tile, which reads all slices alone
// (measured 15-28 GB/s per workgroup).
double estimate_split_seconds(const VariantDesc &v, const Launch &L, const ucl_tuning *tune) {
    const int64_t tiles = count_tiles(L, v.tile_m, v.tile_n);
    int slices = 1, kps = 0;
    split_slices(L, tune->split_k_slices, tiles, split_fill(L, v, tune), slices, kps);
    if (slices <= 1) return estimate_seconds(v, L);
    const double wgs = (double)tiles * slices;
    const double rounds = ceil(wgs / (256.0 * workgroups_per_cu(v)));
    const double busy = wgs < 256.0 ? wgs / 256.0 : 1.0;
    const bool resident = (double)L.batch * (L.M + L.N) * (double)L.K * 2.0 <= 32.0e6;
    const double copy_bytes = wgs * kps * (double)(v.tile_m + v.tile_n) * 2.0;
    const double flops = 2.0 * wgs * kps * (double)v.tile_m * v.tile_n;
    double main = copy_bytes / ((resident ? 16.0e12 : 10.0e12) * busy);
    const double mfma = flops / (relative_rate(v) * 1.38e15 * busy);
    if (mfma > main) main = mfma;
    const double chain = rounds * (kps / (double)v.tile_k) * (resident ? 0.8e-6 : 1.5e-6) / (v.stages > 1 ? v.stages - 1 : 1);
    if (chain > main) main = chain;
    const double tile_bytes = (double)v.tile_m * v.tile_n * 4.0;
    if (tune->split_k_mode == UCL_SPLIT_K_PARALLEL) return main + 6.0e-6 + wgs * tile_bytes / 1.0e12;
    return main + 3.0e-6 + slices * tile_bytes / (v.tile_m * v.tile_n >= 128 * 128 ? 15.0e9 : 28.0e9);
}

const VariantDesc *select_variant(const Launch &L, const ucl_tuning *tune) {
    const auto &vs = all_variants();
    const bool explicit_tune = tune && (tune->tile_m || tune->tile_n || tune->tile_k || tune->stages);
    const VariantDesc *best = nullptr;
    double best_t = 0;
    const int want_persistent = !tune ? 0 : tune->scheduler == UCL_SCHED_PERSISTENT ? 1 : tune->scheduler == UCL_SCHED_STREAM_K ? 2 : 0;
    for (const auto &v : vs) {
        if (v.mode != L.mode || v.dt != L.dt || v.persistent != want_persistent) continue;
        if (v.lb == 4 ? !(L.lb == 1 && L.ndirect_ok) : v.lb != L.lb) continue;
        if (L.mode == 2 || L.mode == 3) {
            // conv: the iterator knob picks between the per-tap gather (la 2) and the resident patch (la 3)
            const int it = tune ? tune->iterator : 0;
            if (v.la == 3 ? (L.patch_c != v.patch_c || it == UCL_ITER_ANALYTIC) : (v.la != 2 || it == UCL_ITER_FIXED_STRIDE_DILATION)) continue;
        } else if (v.la == 5 ? !(L.la == 1 && L.mdirect_ok) : v.la != L.la) {
            continue;
        }
        if (explicit_tune) {
            if (v.tile_m != tune->tile_m || v.tile_n != tune->tile_n || v.stages != tune->stages || v.tile_k != tune->tile_k)
                continue;
            // of several kernels with the named shape: the resident-patch one, else a direct-copy one, else the first
            if (v.la == 3) return &v;
            const bool direct = v.la == 5 || v.lb == 4;
            if (!best || (direct && !(best->la == 5 || best->lb == 4))) best = &v;
            continue;
        }
        const bool split = tune && tune->split_k_mode != UCL_SPLIT_K_NONE && tune->split_k_slices >= 0 && (L.mode == 0 || L.mode == 4);
        const double t = split ? estimate_split_seconds(v, L, tune) : estimate_seconds(v, L);
        if (!best || t < best_t) { best_t = t; best = &v; }
    }
    return best;
}

int default_raster(const VariantDesc &v, const Launch &L) {
    (void)L;
    // bands of ~1024 rows: an XCD's run of 32 consecutive tiles then covers a near-square block
    int gm = 1024 / v.tile_m;
    return gm < 1 ? 1 : gm;
}

ucl_status check_epilogue(const ucl_epilogue *epi, const Launch &L, KParams &kp) {
    kp.n_steps = 0;
    memset(&kp.fused, 0, sizeof(kp.fused));
    kp.fused.enabled = 1;             // the empty chain is the trivial fused form
    if (!epi) return UCL_OK;
    if (epi->n_steps < 0 || epi->n_steps > UCL_MAX_EPI_STEPS)
        return fail(UCL_ERR_INVALID_ARG, "epilogue has %d steps; the chain holds 0..%d", epi->n_steps, UCL_MAX_EPI_STEPS);
    for (int i = 0; i < epi->n_steps; ++i) {
        const ucl_epi_step &s = epi->steps[i];
        if (s.op < UCL_EPI_SCALE || s.op > UCL_EPI_AUX_STORE)
            return fail(UCL_ERR_INVALID_ARG, "epilogue step %d: unknown op code %d", i, s.op);
        EpiStepDev &d = kp.steps[i];
        d.op = s.op; d.dtype = s.dtype; d.p0 = s.p0; d.p1 = s.p1; d.ptr = s.ptr; d.ld = s.ld; d.bs = s.bs;
        if (op_has_tensor(s.op)) {
            if (!s.ptr) return fail(UCL_ERR_INVALID_ARG, "epilogue step %d needs a tensor operand but ptr is NULL", i);
            if (!valid_dtype(s.dtype)) return fail(UCL_ERR_INVALID_ARG, "epilogue step %d: bad tensor dtype %d", i, s.dtype);
            // 128-bit accesses of 8 (16-bit) or 4 (fp32) elements need 16-byte aligned rows
            const int per16 = 16 / elem_size(s.dtype);
            bool vec = true;
            if (L.mode != 1) vec = aligned16(s.ptr);
            // (grouped: the per-group pointers live on the device and are required to be 16-byte aligned)
            if (op_is_matrix(s.op)) {
                if (s.ld < L.N) return fail(UCL_ERR_INVALID_ARG, "epilogue step %d: ld=%lld is smaller than N=%lld", i, (long long)s.ld, (long long)L.N);
                vec = vec && (s.ld % per16 == 0) && (s.bs % per16 == 0) && s.ld <= kMaxWideLd;
            }
            if (vec) d.dtype |= 0x100;
        }
        if (s.op == UCL_EPI_CLAMP && !(s.p0 <= s.p1))
            return fail(UCL_ERR_INVALID_ARG, "epilogue step %d: clamp(min=%g, max=%g) has min > max", i, s.p0, s.p1);
    }
    kp.n_steps = epi->n_steps;
    // Recognise  [scale] [bias | row_broadcast] [aux_load] [one activation]  in that order.
    FusedEpi f;
    memset(&f, 0, sizeof(f));
    int i = 0;
    const int n = epi->n_steps;
    if (i < n && kp.steps[i].op == UCL_EPI_SCALE) { f.has_scale = 1; f.alpha = kp.steps[i].p0; ++i; }
    if (i < n && (kp.steps[i].op == UCL_EPI_BIAS || kp.steps[i].op == UCL_EPI_ROW_BROADCAST)) {
        f.has_bias = 1; f.bias = kp.steps[i].ptr; f.bias_dt = kp.steps[i].dtype; ++i;
    }
    if (i < n && kp.steps[i].op == UCL_EPI_AUX_LOAD) {
        f.has_res = 1; f.res = kp.steps[i].ptr; f.res_dt = kp.steps[i].dtype; f.beta = kp.steps[i].p0;
        f.res_ld = kp.steps[i].ld; f.res_bs = kp.steps[i].bs; ++i;
    }
    if (i < n) {
        switch (kp.steps[i].op) {
        case UCL_EPI_RELU: case UCL_EPI_GELU_TANH: case UCL_EPI_GELU_ERF: case UCL_EPI_SILU: case UCL_EPI_SIGMOID:
        case UCL_EPI_TANH: case UCL_EPI_MISH: case UCL_EPI_HARDSWISH: case UCL_EPI_LEAKY_RELU: case UCL_EPI_ELU:
        case UCL_EPI_CLAMP:
            f.act = kp.steps[i].op; f.act_p0 = kp.steps[i].p0; f.act_p1 = kp.steps[i].p1; ++i;
            break;
        default:
            break;
        }
    }
    f.enabled = (i == n);
    kp.fused = f;
    return UCL_OK;
}

// Layout of a 16-bit operand from its two strides: *layout = 0 (contiguous along K) or 1
// (contiguous along its M / N extent), *ld = stride of the other dimension.
ucl_status classify(const char *name, const void *ptr, int64_t k_stride, int64_t mn_stride, int64_t mn_extent,
                    int64_t K, int *layout, int64_t *ld) {
    if (!aligned16(ptr))
        return fail(UCL_ERR_UNSUPPORTED, "%s base pointer %p is not 16-byte aligned; 128-bit loads need (alignment * element_size) %% 16 == 0", name, ptr);
    if (k_stride != 1 && mn_stride != 1)
        return fail(UCL_ERR_UNSUPPORTED, "%s has strides (%lld, %lld): one of them must be 1 (RowMajor or ColumnMajor)", name,
                    (long long)mn_stride, (long long)k_stride);
    if (k_stride == 1 && mn_stride == 1 && mn_extent > 1 && K > 1)
        return fail(UCL_ERR_INVALID_ARG, "%s has both strides 1 with both extents > 1: elements would overlap", name);
    if (k_stride == 1 && (mn_stride != 1 || K % 8 == 0)) {
        if (K % 8 != 0)
            return fail(UCL_ERR_UNSUPPORTED, "%s is contiguous along K but K=%lld is not a multiple of 8 (alignment 8 x 2 bytes = 16)", name, (long long)K);
        if (mn_extent > 1) {
            if (mn_stride % 8 != 0)
                return fail(UCL_ERR_UNSUPPORTED, "%s leading stride %lld is not a multiple of 8 elements", name, (long long)mn_stride);
            if (mn_stride < K)
                return fail(UCL_ERR_INVALID_ARG, "%s leading stride %lld is smaller than its contiguous extent K=%lld", name, (long long)mn_stride, (long long)K);
        }
        *layout = 0;
        *ld = mn_extent > 1 ? mn_stride : K;
        return UCL_OK;
    }
    if (mn_extent % 8 != 0)
        return fail(UCL_ERR_UNSUPPORTED, "%s is contiguous along its M/N extent %lld, which is not a multiple of 8", name, (long long)mn_extent);
    if (K > 1) {
        if (k_stride % 8 != 0)
            return fail(UCL_ERR_UNSUPPORTED, "%s leading stride %lld is not a multiple of 8 elements", name, (long long)k_stride);
        if (k_stride < mn_extent)
            return fail(UCL_ERR_INVALID_ARG, "%s leading stride %lld is smaller than its contiguous extent %lld", name, (long long)k_stride, (long long)mn_extent);
    }
    *layout = 1;
    *ld = K > 1 ? k_stride : mn_extent;
    return UCL_OK;
}

ucl_status check_common(int64_t M, int64_t N, int64_t K, int dtA, int dtB, int dtD, const void *A, const void *B,
                        const void *D, bool fp8_ok = false) {
    if (M <= 0 || N <= 0 || K <= 0)
        return fail(UCL_ERR_INVALID_ARG, "extents must be positive, got M=%lld N=%lld K=%lld", (long long)M, (long long)N, (long long)K);
    if (M >= (1ll << 31) || N >= (1ll << 31) || K >= (1ll << 31))
        return fail(UCL_ERR_UNSUPPORTED, "extents must be below 2^31");
    if (!A || !B || !D) return fail(UCL_ERR_INVALID_ARG, "A, B and D must be non-NULL device pointers");
    if (is8(dtA) && dtA == dtB && !fp8_ok)
        return fail(UCL_ERR_UNSUPPORTED, "fp8 inputs are built for gemm, batched_gemm and grouped_gemm");
    if (!(is16(dtA) || is8(dtA)) || dtA != dtB)
        return fail(UCL_ERR_UNSUPPORTED, "inputs must both be bf16, both fp16 or both the same fp8 type (got %s, %s); accumulation is fp32", dtype_name(dtA), dtype_name(dtB));
    if (!valid_dtype(dtD)) return fail(UCL_ERR_INVALID_ARG, "bad output dtype %d", dtD);
    return UCL_OK;
}


// Fill kernel for the counter area of a split-K workspace (a kernel, not a memset node: the call may
// be captured into a HIP graph).  One 128-bit store per thread.
__global__ void zero_words_kernel(uint32_t *w) {
    ((u32x4 *)w)[blockIdx.x * blockDim.x + threadIdx.x] = u32x4{0u, 0u, 0u, 0u};
}

// Parallel split-K, between the two launches of the tile kernel: adds the slices of every partial tile up into
// slice 0, slice 0 first (the same order, starting from +0, as the tile kernel's own loop: the results are
// bit-identical).  A tile kernel that did this itself would have one workgroup per tile read all slices of its
// tile; here every 16 bytes of a tile are a thread's work, so that the whole chip streams the partial tiles.
typedef float f32x4 __attribute__((ext_vector_type(4)));
// (sixteen, then eight slices' loads in flight per thread: what the kernel moves per microsecond is what it has in
// flight; the additions stay in slice order.  V = f32x4, or float where 16-byte words would make too few workgroups
// to occupy the chip: the same additions per element either way.)
template <int U, class V>
__device__ inline void sum_slices(const V *src, int64_t stride, int slices, int &s, V &acc) {
    for (; s + U <= slices; s += U) {
        V v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) v[u] = __builtin_nontemporal_load(src + (s + u) * stride);
#pragma unroll
        for (int u = 0; u < U; ++u) acc += v[u];
    }
}
template <class V>
__device__ inline V sum_slices(const V *src, int64_t stride, int slices) {
    V acc = V();                     // +0 in every element
    int s = 0;
    sum_slices<16>(src, stride, slices, s, acc);
    sum_slices<8>(src, stride, slices, s, acc);
    sum_slices<1>(src, stride, slices, s, acc);
    return acc;
}
// `slice_stride` = floats per slice, `n` = elements of type V per slice
template <class V>
__global__ __launch_bounds__(256) void splitk_reduce_kernel(float *partials, int64_t slice_stride, int slices, int64_t n) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    constexpr int kPer = sizeof(V) / 4;
    ((V *)partials)[i] = sum_slices((const V *)partials + i, slice_stride / kPer, slices);
}
// Words of 16 bytes per slice below which the reduction runs one float per thread (fewer than two workgroups per CU otherwise).
constexpr int64_t kReduceScalarBelow = 2 * 256 * 256;

// The same reduction for launches whose chain has the form act(alpha * acc + bias[n] + beta * R[m, n]) (any part may be
// missing, the empty chain included): the
// reduction kernel runs the chain on the sums, with the tile kernel's own element-wise functions and in its order of
// operations (so the bits are the same), and stores D; the finishing launch of the tile kernel is not needed.
// A 16-byte word of a partial tile is accumulator (mi, ni) of one lane: four consecutive columns of one row (the
// layout the tile kernel stores: word = (mi * NI + ni) * 256 + thread; thread = wave * 64 + lane, wave = (row half,
// column half) of the tile; row = mi * 16 + lane % 16, column = ni * 16 + 4 * (lane / 16) inside the wave's quarter).
struct ReduceStore {
    float *partials;
    void *D;
    const void *bias, *res;
    int64_t slice_stride, n4, ldd, d_bs, res_ld, res_bs;
    int32_t slices, tile_m, tile_n, M, N, tiles_m, tiles_n, tiles_per_batch, raster;
    int32_t dtD, has_bias, bias_dt, has_res, res_dt, act;
    float alpha, beta, act_p0, act_p1;
};
template <class V>
__global__ __launch_bounds__(256) void splitk_reduce_store_kernel(const ReduceStore a) {
    constexpr int kPer = sizeof(V) / 4;                // 4: a thread per 16-byte word, 1: a thread per element
    const int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (j >= a.n4 * (4 / kPer)) return;
    const V acc = sum_slices((const V *)a.partials + j, a.slice_stride / kPer, a.slices);
    const int64_t i = kPer == 4 ? j : j >> 2;          // the 16-byte word
    const int e0 = kPer == 4 ? 0 : (int)(j & 3);       // the thread's (first) element in it
    const int words_per_tile = a.tile_m * a.tile_n / 4, ni_count = a.tile_n / 32;
    int t = (int)(i / words_per_tile);
    const int w = (int)(i - (int64_t)t * words_per_tile);
    const int reg = w >> 8, thread = w & 255, wave = thread >> 6, lane = thread & 63;
    const int m_loc = (wave >> 1) * (a.tile_m / 2) + (reg / ni_count) * 16 + (lane & 15);
    const int n_loc = (wave & 1) * (a.tile_n / 2) + (reg % ni_count) * 16 + 4 * (lane >> 4);
    const int batch = t / a.tiles_per_batch;
    t -= batch * a.tiles_per_batch;
    int tm, tn;
    band_raster(t, a.tiles_m, a.tiles_n, a.raster, tm, tn);
    const int m = tm * a.tile_m + m_loc, n = tn * a.tile_n + n_loc + e0;
    if (m >= a.M || n >= a.N) return;
    const int nvalid = a.N - n < kPer ? a.N - n : kPer;
    float x[kPer];
#pragma unroll
    for (int e = 0; e < kPer; ++e) {
        float b = 0.f;
        if (a.has_bias && e < nvalid)
            b = a.bias_dt == UCL_F32 ? ((const float *)a.bias)[n + e] : bits_to_f32(((const uint16_t *)a.bias)[n + e], a.bias_dt);
        float s;
        if constexpr (kPer == 4) s = acc[e]; else s = acc;
        x[e] = s * a.alpha + b;
    }
    if (a.has_res) {
        const int64_t rat = (int64_t)batch * a.res_bs + (int64_t)m * a.res_ld + n;
#pragma unroll
        for (int e = 0; e < kPer; ++e) {
            float r = 0.f;
            if (e < nvalid)
                r = a.res_dt == UCL_F32 ? ((const float *)a.res)[rat + e] : bits_to_f32(((const uint16_t *)a.res)[rat + e], a.res_dt);
            x[e] += a.beta * r;
        }
    }
    switch (a.act) {
#define UCL_ACT_CASE(OP)                                                                                      \
    case OP:                                                                                                  \
        _Pragma("unroll") for (int e = 0; e < kPer; ++e) x[e] = act_f32<OP>(x[e], a.act_p0, a.act_p1);         \
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
    const int64_t at = (int64_t)batch * a.d_bs + (int64_t)m * a.ldd + n;
    if (a.dtD == UCL_F32) {
        float *dst = (float *)a.D + at;
        if constexpr (kPer == 4) {
            if (nvalid == 4) {
                *(f32x4 *)dst = f32x4{x[0], x[1], x[2], x[3]};
                return;
            }
        }
#pragma unroll
        for (int e = 0; e < kPer; ++e)
            if (e < nvalid) dst[e] = x[e];
    } else {
        uint16_t *dst = (uint16_t *)a.D + at;
        uint32_t bits[kPer];
#pragma unroll
        for (int e = 0; e < kPer; ++e) bits[e] = f32_to_bits16(x[e], a.dtD);
        if constexpr (kPer == 4) {
            if (nvalid == 4) {
                typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
                *(u32x2 *)dst = u32x2{bits[0] | (bits[1] << 16), bits[2] | (bits[3] << 16)};
                return;
            }
        }
#pragma unroll
        for (int e = 0; e < kPer; ++e)
            if (e < nvalid) dst[e] = (uint16_t)bits[e];
    }
}

// split-K plan of a launch: slices (1 = none), K extent per slice, workspace bytes.
struct SplitPlan {
    int slices = 1;
    int k_per_slice = 0;
    int64_t bytes = 0;
    // stream-K: 64-wide k steps per tile, iterations per workgroup, workgroups (0: not a stream-K launch)
    int sk_ipt = 0, sk_q = 0, sk_rounds = 0, sk_grid = 0, sk_deal = 0;
};

ucl_status plan_split(const Launch &L, const VariantDesc &v, const ucl_tuning *tune, int64_t total_tiles, SplitPlan &sp) {
    sp = SplitPlan();
    if (!tune) return UCL_OK;
    if (tune->scheduler < UCL_SCHED_DEFAULT || tune->scheduler > UCL_SCHED_STREAM_K)
        return fail(UCL_ERR_INVALID_ARG, "scheduler=%d is not a ucl_tile_scheduler", tune->scheduler);
    if (tune->scheduler == UCL_SCHED_STREAM_K) {
        // every workgroup of a resident grid takes an equal run of (tile, 64-wide k range) iterations; a workgroup
        // leaves at most two parts of tiles in the workspace (two slots per workgroup behind the counters)
        if (tune->split_k_mode != UCL_SPLIT_K_NONE)
            return fail(UCL_ERR_UNSUPPORTED, "split-K and the stream_k scheduler cannot be combined");
        if (total_tiles > UCL_SPLIT_K_MAX_TILES)
            return fail(UCL_ERR_UNSUPPORTED, "the stream_k scheduler serves at most %d output tiles (this problem has %lld)", UCL_SPLIT_K_MAX_TILES, (long long)total_tiles);
        const int64_t ipt = (L.K + 63) / 64, all = total_tiles * ipt;
        if (all >= (1ll << 31)) return fail(UCL_ERR_UNSUPPORTED, "tiles x k steps exceeds 2^31");
        if (all == 0) return UCL_OK;
        // whole rounds of tiles go one tile per workgroup and round; the k steps of the tiles that are left are
        // dealt out evenly.  Fewer tiles than CU slots: no whole round, and only as many workgroups as it takes.
        const int64_t slots = (int64_t)kNumCUs * v.resident();
        int64_t grid = slots, rounds = total_tiles / slots;
        int64_t rest = (total_tiles - rounds * grid) * ipt, q = (rest + grid - 1) / grid;
        if (rounds == 0) {
            // (one workgroup per CU at most, or per tile if there are more tiles than CUs)
            if (grid > kNumCUs) grid = total_tiles > kNumCUs ? total_tiles : kNumCUs;
            if (grid > rest) grid = rest;
            q = (rest + grid - 1) / grid;
            // The workgroup that ends a tile reads the tile's other parts back one after the other, which costs it
            // about r k steps' time per part (measured: 1 for 64x64 tiles, whose parts are loaded several at a time,
            // 9 for 128x128); a run of q steps and ipt / q parts to add make q = sqrt(r ipt) the shortest path
            // through a tile.
            const double r = (int64_t)v.tile_m * v.tile_n >= 128 * 128 ? 9.0 : 1.0;
            const int64_t q_path = (int64_t)(sqrt(r * (double)ipt) + 0.5);
            if (q < q_path) q = q_path;
            if (q < 4) q = 4;
            if (q > ipt) q = ipt;
            // (a slightly longer run that divides the k steps of a tile: the runs can then be dealt k range by k range)
            for (int64_t d = q; d <= q + q / 4; ++d)
                if (ipt % d == 0) { q = d; break; }
            grid = (rest + q - 1) / q;
        }
        if (q > 0 && ipt % q == 0 && (total_tiles - rounds * grid) * (ipt / q) <= grid) sp.sk_deal = (int)(total_tiles - rounds * grid);
        sp.sk_ipt = (int)ipt;
        sp.sk_q = (int)q;
        sp.sk_rounds = (int)rounds;
        sp.sk_grid = (int)grid;
        sp.slices = q ? (int)((ipt + q - 2) / q + 1) : 1;    // parts a tile can fall into, at most
        if (sp.slices > ipt) sp.slices = (int)ipt;
        sp.bytes = UCL_WORKSPACE_COUNTER_BYTES + (int64_t)sp.sk_grid * 2 * v.tile_m * v.tile_n * 4;
        return UCL_OK;
    }
    if (tune->split_k_mode < UCL_SPLIT_K_NONE || tune->split_k_mode > UCL_SPLIT_K_PARALLEL)
        return fail(UCL_ERR_INVALID_ARG, "split_k_mode=%d is not a ucl_split_k_mode", tune->split_k_mode);
    if (tune->split_k_slices < 0) return fail(UCL_ERR_INVALID_ARG, "split_k_slices=%d must be >= 0", tune->split_k_slices);
    if (tune->split_k_mode == UCL_SPLIT_K_NONE) {
        if (tune->split_k_slices > 1)
            return fail(UCL_ERR_INVALID_ARG, "split_k_slices=%d with split_k_mode none: name serial or parallel", tune->split_k_slices);
        return UCL_OK;
    }
    if (L.mode != 0 && L.mode != 4) return fail(UCL_ERR_UNSUPPORTED, "split-K is built for gemm, batched_gemm and conv2d_wgrad");
    if (tune->scheduler == UCL_SCHED_PERSISTENT)
        return fail(UCL_ERR_UNSUPPORTED, "split-K and the persistent scheduler cannot be combined");
    split_slices(L, tune->split_k_slices, total_tiles, split_fill(L, v, tune), sp.slices, sp.k_per_slice);
    if (sp.slices <= 1) { sp = SplitPlan(); return UCL_OK; }
    if (total_tiles > UCL_SPLIT_K_MAX_TILES)
        return fail(UCL_ERR_UNSUPPORTED, "split-K serves at most %d output tiles (this problem has %lld)", UCL_SPLIT_K_MAX_TILES, (long long)total_tiles);
    if (total_tiles * sp.slices >= (1ll << 31)) return fail(UCL_ERR_UNSUPPORTED, "tiles x slices exceeds the grid limit");
    sp.bytes = UCL_WORKSPACE_COUNTER_BYTES + (int64_t)sp.slices * total_tiles * v.tile_m * v.tile_n * 4;
    return UCL_OK;
}

// Parallel split-K with up to this many slices lets the last launch of the tile kernel add them up itself.
constexpr int kReduceInTileKernel = 2;

ucl_status run(const Launch &L, KParams &kp, const ucl_tuning *tune, void *stream, bool clear_counters = false) {
    if (tune && (tune->iterator < 0 || tune->iterator > UCL_ITER_FIXED_STRIDE_DILATION))
        return fail(UCL_ERR_INVALID_ARG, "iterator=%d is not a ucl_conv_iterator", tune->iterator);
    // (the GEMM entry points ignore the iterator)
    if (tune && (L.mode == 2 || L.mode == 3) && tune->iterator == UCL_ITER_FIXED_STRIDE_DILATION && !L.patch_c)
        return fail(UCL_ERR_UNSUPPORTED, "the fixed_stride_dilation iterator serves a 3x3 filter with unit stride and dilation, pad 1 and W <= 58: conv2d_fprop with 64 or 128 input channels, conv2d_dgrad with 64 or 128 output channels");
    const VariantDesc *v = select_variant(L, tune);
    if (!v) {
        if (tune && (tune->tile_m || tune->tile_n || tune->tile_k || tune->stages)) {
            if (tune->tile_k != 32 && tune->tile_k != 64)
                return fail(UCL_ERR_UNSUPPORTED, "tile_k=%d: the built kernels stage K in steps of 32 or 64", tune->tile_k);
            const int64_t lds = (int64_t)(tune->tile_m + tune->tile_n) * tune->tile_k * 2 * tune->stages;
            if (lds > kLdsBytesPerCU)
                return fail(UCL_ERR_WORKSPACE, "tile %dx%dx%d with %d stages needs %lld bytes of LDS; a CU has %d",
                            tune->tile_m, tune->tile_n, tune->tile_k, tune->stages, (long long)lds, kLdsBytesPerCU);
            return fail(UCL_ERR_UNSUPPORTED, "no kernel built for tile %dx%dx%d, %d stages with these types/layouts; see ucl_variant()",
                        tune->tile_m, tune->tile_n, tune->tile_k, tune->stages);
        }
        if (tune && tune->scheduler == UCL_SCHED_PERSISTENT)
            return fail(UCL_ERR_UNSUPPORTED, "no kernel with the persistent tile scheduler is built for this combination of operation, input type and layouts");
        if (tune && tune->scheduler == UCL_SCHED_STREAM_K)
            return fail(UCL_ERR_UNSUPPORTED, "no kernel with the stream_k tile scheduler is built for this combination of operation, input type and layouts (gemm / batched_gemm, 16-bit inputs contiguous along K)");
        return fail(UCL_ERR_UNSUPPORTED, "no kernel built for this combination of operation, input type and layouts");
    }
    if (kp.ldd > kMaxWideLd) kp.d_vec = 0;
    int raster = tune ? tune->raster : 0;
    if (raster < 0 || raster > 64) return fail(UCL_ERR_INVALID_ARG, "raster=%d must be in 0..64", raster);
    if (raster == 0) raster = default_raster(*v, L);
    kp.raster = raster;
    kp.tiles_n = (int32_t)((L.N + v->tile_n - 1) / v->tile_n);
    GroupTable gt;
    int64_t total;
    if (L.mode == 1) {
        int64_t acc = 0;
        for (int g = 0; g < L.groups; ++g) {
            gt.m[g] = (int32_t)L.M_g[g];
            gt.tile_start[g] = (int32_t)acc;
            acc += (L.M_g[g] + v->tile_m - 1) / v->tile_m * kp.tiles_n;
        }
        for (int g = L.groups; g <= UCL_MAX_GROUPS; ++g) gt.tile_start[g] = (int32_t)acc;
        for (int g = L.groups; g < UCL_MAX_GROUPS; ++g) gt.m[g] = 0;
        total = acc;
        kp.tiles_m = 0;
        kp.tiles_per_batch = 0;
    } else {
        kp.tiles_m = (int32_t)((L.M + v->tile_m - 1) / v->tile_m);
        kp.tiles_per_batch = kp.tiles_m * kp.tiles_n;
        total = (int64_t)kp.tiles_per_batch * L.batch;
    }
    if (total >= (1ll << 31)) return fail(UCL_ERR_UNSUPPORTED, "problem needs %lld tiles; the grid is limited to 2^31-1", (long long)total);
    SplitPlan sp;
    if (ucl_status st = plan_split(L, *v, tune, total, sp)) return st;
    if (sp.sk_grid > 0) {
        if (!tune->workspace)
            return fail(UCL_ERR_WORKSPACE, "the stream_k scheduler needs a workspace of %lld bytes (ucl_workspace_size); tune->workspace is NULL", (long long)sp.bytes);
        if (!aligned16(tune->workspace)) return fail(UCL_ERR_WORKSPACE, "the workspace must be 16-byte aligned");
        if (tune->workspace_bytes < sp.bytes)
            return fail(UCL_ERR_WORKSPACE, "the stream_k scheduler with %d workgroups and tiles of %dx%d needs %lld bytes of workspace, got %lld",
                        sp.sk_grid, v->tile_m, v->tile_n, (long long)sp.bytes, (long long)tune->workspace_bytes);
        kp.sk_ipt = sp.sk_ipt;
        kp.sk_q = sp.sk_q;
        kp.sk_deal = sp.sk_deal;
        kp.sk_rounds = sp.sk_rounds;
        kp.ws_counters = (uint32_t *)tune->workspace;
        kp.ws_partials = (float *)((char *)tune->workspace + UCL_WORKSPACE_COUNTER_BYTES);
    } else if (sp.slices > 1) {
        if (!tune->workspace)
            return fail(UCL_ERR_WORKSPACE, "split-K with %d slices needs a workspace of %lld bytes (ucl_workspace_size); tune->workspace is NULL", sp.slices, (long long)sp.bytes);
        if (!aligned16(tune->workspace)) return fail(UCL_ERR_WORKSPACE, "the split-K workspace must be 16-byte aligned");
        if (tune->workspace_bytes < sp.bytes)
            return fail(UCL_ERR_WORKSPACE, "split-K with %d slices over %lld tiles of %dx%d needs %lld bytes of workspace, got %lld",
                        sp.slices, (long long)total, v->tile_m, v->tile_n, (long long)sp.bytes, (long long)tune->workspace_bytes);
        kp.split_k = sp.slices;
        kp.k_per_slice = sp.k_per_slice;
        kp.ws_counters = (uint32_t *)tune->workspace;
        kp.ws_partials = (float *)((char *)tune->workspace + UCL_WORKSPACE_COUNTER_BYTES);
    }
    // operand panels are addressed with 32-bit byte offsets inside range-checked buffer resources
    if (v->la == 0 && ((int64_t)v->tile_m * kp.lda + L.K) * 2 >= (1ll << 31))
        return fail(UCL_ERR_UNSUPPORTED, "A leading stride %lld too large: a %d-row panel must span less than 2 GiB", (long long)kp.lda, v->tile_m);
    if (v->lb == 0 && ((int64_t)v->tile_n * kp.ldb + L.K) * 2 >= (1ll << 31))
        return fail(UCL_ERR_UNSUPPORTED, "B leading stride %lld too large: a %d-row panel must span less than 2 GiB", (long long)kp.ldb, v->tile_n);
    kp.total_tiles = (int32_t)total;
    if (total == 0) return UCL_OK;     // grouped with every M_g == 0: nothing to do
    const GroupTable *gtp = L.mode == 1 ? &gt : nullptr;
    hipError_t e;
    if (sp.sk_grid > 0) {
        if (clear_counters) {
            hipLaunchKernelGGL(zero_words_kernel, dim3(UCL_WORKSPACE_COUNTER_BYTES / 16 / 256), dim3(256), 0, (hipStream_t)stream,
                               (uint32_t *)tune->workspace);
            e = hipGetLastError();
            if (e != hipSuccess) return fail(UCL_ERR_LAUNCH, "kernel launch failed: %s", hipGetErrorString(e));
        }
        e = v->launch(kp, gtp, sp.sk_grid, (hipStream_t)stream);
    } else if (sp.slices > 1 && tune->split_k_mode == UCL_SPLIT_K_PARALLEL) {
        kp.split_phase = 1;
        e = v->launch(kp, gtp, (int)(total * sp.slices), (hipStream_t)stream);
        bool finished = false;
        if (e == hipSuccess && sp.slices > kReduceInTileKernel) {
            // many slices: a launch of its own adds them up with the whole chip, the last launch then finds one slice
            const int64_t slice_floats = total * v->tile_m * v->tile_n, n4 = slice_floats / 4;
            const bool simple = kp.fused.enabled && kp.d_vec && L.mode != 1;
            if (simple) {
                // ... or none: a chain of the form act(alpha * acc + bias[n] + beta * R[m, n]) is run by the reduction kernel on the sums
                ReduceStore rs;
                rs.partials = kp.ws_partials; rs.D = kp.D; rs.bias = kp.fused.bias;
                rs.dtD = kp.dtD; rs.has_bias = kp.fused.has_bias; rs.bias_dt = kp.fused.bias_dt & 0xff; rs.act = kp.fused.act;
                rs.alpha = kp.fused.has_scale ? kp.fused.alpha : 1.f; rs.act_p0 = kp.fused.act_p0; rs.act_p1 = kp.fused.act_p1;
                rs.has_res = kp.fused.has_res; rs.res = kp.fused.res; rs.res_dt = kp.fused.res_dt & 0xff; rs.beta = kp.fused.beta;
                rs.res_ld = kp.fused.res_ld; rs.res_bs = kp.fused.res_bs;
                rs.slice_stride = slice_floats; rs.n4 = n4; rs.ldd = kp.ldd; rs.d_bs = kp.d_bs;
                rs.slices = sp.slices; rs.tile_m = v->tile_m; rs.tile_n = v->tile_n; rs.M = kp.M; rs.N = kp.N;
                rs.tiles_m = kp.tiles_m; rs.tiles_n = kp.tiles_n; rs.tiles_per_batch = kp.tiles_per_batch; rs.raster = kp.raster;
                if (n4 < kReduceScalarBelow)
                    hipLaunchKernelGGL(splitk_reduce_store_kernel<float>, dim3((unsigned)((slice_floats + 255) / 256)), dim3(256), 0, (hipStream_t)stream, rs);
                else
                    hipLaunchKernelGGL(splitk_reduce_store_kernel<f32x4>, dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, (hipStream_t)stream, rs);
                finished = true;
            } else if (n4 < kReduceScalarBelow) {
                hipLaunchKernelGGL(splitk_reduce_kernel<float>, dim3((unsigned)((slice_floats + 255) / 256)), dim3(256), 0, (hipStream_t)stream,
                                   kp.ws_partials, slice_floats, sp.slices, slice_floats);
            } else {
                hipLaunchKernelGGL(splitk_reduce_kernel<f32x4>, dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, (hipStream_t)stream,
                                   kp.ws_partials, slice_floats, sp.slices, n4);
            }
            e = hipGetLastError();
            kp.split_k = 1;
        }
        if (e == hipSuccess && !finished) {
            kp.split_phase = 2;
            e = v->launch(kp, gtp, (int)total, (hipStream_t)stream);
        }
    } else {
        if (clear_counters && sp.slices > 1) {
            // the static workspace is shared by every call on this GPU: start from zeroed counters whatever
            // an earlier call left behind (a fill kernel, so that the call can be captured into a graph)
            hipLaunchKernelGGL(zero_words_kernel, dim3(UCL_WORKSPACE_COUNTER_BYTES / 16 / 256), dim3(256), 0, (hipStream_t)stream,
                               (uint32_t *)tune->workspace);
            e = hipGetLastError();
            if (e != hipSuccess) return fail(UCL_ERR_LAUNCH, "kernel launch failed: %s", hipGetErrorString(e));
        }
        int64_t grid = total * sp.slices;
        if (v->persistent) {
            // one workgroup per CU slot; a multiple of 8 keeps each workgroup on the tile run of its XCD
            // (as many as the compiled kernel's registers and LDS let a CU hold, so that the whole grid is resident)
            const int64_t slots = (int64_t)kNumCUs * v->resident();
            if (grid > slots) grid = slots;
        }
        e = v->launch(kp, gtp, (int)grid, (hipStream_t)stream);
    }
    if (e != hipSuccess) return fail(UCL_ERR_LAUNCH, "kernel launch failed: %s", hipGetErrorString(e));
    return UCL_OK;
}

ucl_status gemm_like(int64_t batch, int64_t M, int64_t N, int64_t K,
                     const void *A, int dtA, int64_t a_rs, int64_t a_cs, int64_t a_bs,
                     const void *B, int dtB, int64_t b_rs, int64_t b_cs, int64_t b_bs,
                     void *D, int dtD, int64_t d_rs, int64_t d_cs, int64_t d_bs,
                     const ucl_epilogue *epi, const ucl_tuning *tune, void *stream, bool clear_counters = false) {
    g_err[0] = 0;
    if (batch <= 0) return fail(UCL_ERR_INVALID_ARG, "batch=%lld must be positive", (long long)batch);
    if (ucl_status st = check_common(M, N, K, dtA, dtB, dtD, A, B, D, /*fp8_ok=*/true)) return st;
    if (is8(dtA)) {
        // 8-bit inputs are handled as pairs of elements: from here on K and the strides of A and B count
        // 16-bit units, which the checks below require to be 16-byte aligned like those of 16-bit inputs
        if (a_cs != 1 || b_rs != 1)
            return fail(UCL_ERR_UNSUPPORTED, "fp8 inputs must both be contiguous along K (A row-major, B column-major)");
        if (K % 16 || (M > 1 && a_rs % 16) || (N > 1 && b_cs % 16) || (batch > 1 && (a_bs % 16 || b_bs % 16)))
            return fail(UCL_ERR_UNSUPPORTED, "fp8 inputs: K=%lld, the leading strides (%lld, %lld) and the batch strides must be multiples of 16 (alignment 16 x 1 byte = 16)",
                        (long long)K, (long long)a_rs, (long long)b_cs);
        K /= 2; a_rs /= 2; b_cs /= 2; a_bs /= 2; b_bs /= 2;
    }
    if (d_cs != 1)
        return fail(UCL_ERR_UNSUPPORTED, "D must be row-major (d_cs == 1, got %lld); for a column-major D swap the operands' roles: (A.B)^T = B^T.A^T", (long long)d_cs);
    if (d_rs < N && M > 1) return fail(UCL_ERR_INVALID_ARG, "d_rs=%lld is smaller than N=%lld", (long long)d_rs, (long long)N);
    if (batch > 1 && ((a_bs % 8) || (b_bs % 8)))
        return fail(UCL_ERR_UNSUPPORTED, "batch strides of A and B must be multiples of 8 elements (16-byte alignment of every batch)");
    Launch L;
    L.mode = 0; L.batch = batch; L.M = M; L.N = N; L.K = K; L.dt = dt_code(dtA); L.dtD = dtD;
    KParams kp;
    memset(&kp, 0, sizeof(kp));
    if (ucl_status st = classify("A", A, a_cs, a_rs, M, K, &L.la, &kp.lda)) return st;
    if (ucl_status st = classify("B", B, b_rs, b_cs, N, K, &L.lb, &kp.ldb)) return st;
    // direct copies of an N-contiguous B address it with 32-bit byte offsets from the start of a batch
    L.ndirect_ok = L.lb == 1 && ((K - 1) * kp.ldb + N) * 2 < (1ll << 31);
    L.mdirect_ok = L.la == 1 && ((K - 1) * kp.lda + M) * 2 < (1ll << 31);
    if (ucl_status st = check_epilogue(epi, L, kp)) return st;
    kp.A = A; kp.B = B; kp.D = D;
    kp.ldd = d_rs; kp.a_bs = a_bs; kp.b_bs = b_bs; kp.d_bs = d_bs;
    kp.M = (int32_t)M; kp.N = (int32_t)N; kp.K = (int32_t)K;
    kp.dtD = dtD;
    kp.d_vec = aligned16(D) && (d_rs % (16 / elem_size(dtD)) == 0) && (d_bs % (16 / elem_size(dtD)) == 0);
    return run(L, kp, tune, stream, clear_counters);
}

// ---- SOL ---------------------------------------------------------------------------------------

int64_t conv_out(int64_t in, int64_t pad, int64_t dil, int64_t ker, int64_t stride) {
    return (in + 2 * pad - dil * (ker - 1) - 1) / stride + 1;
}

ucl_status characterise(const ucl_problem *p, double *flops, double *bytes, int64_t *M_out, int64_t *N_out) {
    if (!p) return fail(UCL_ERR_INVALID_ARG, "problem is NULL");
    if (!(valid_dtype(p->dt_in) || is8(p->dt_in)) || !valid_dtype(p->dt_out)) return fail(UCL_ERR_INVALID_ARG, "bad dtype in problem");
    const double si = elem_size(p->dt_in), so = elem_size(p->dt_out);
    double rows = 0, N = 0, batch = 1;
    switch (p->op) {
    case UCL_OP_GEMM:
    case UCL_OP_BATCHED_GEMM: {
        batch = p->op == UCL_OP_GEMM ? 1 : (double)p->batch;
        if (p->M <= 0 || p->N <= 0 || p->K <= 0 || batch <= 0) return fail(UCL_ERR_INVALID_ARG, "extents must be positive");
        rows = (double)p->M; N = (double)p->N;
        *flops = 2.0 * batch * p->M * p->N * p->K;
        *bytes = batch * ((double)p->M * p->K + (double)p->K * p->N) * si + batch * (double)p->M * p->N * so;
        break;
    }
    case UCL_OP_GROUPED_GEMM: {
        if (p->groups <= 0 || !p->M_g || p->N <= 0 || p->K <= 0) return fail(UCL_ERR_INVALID_ARG, "grouped problem needs groups > 0, M_g, N, K");
        double sumM = 0;
        for (int g = 0; g < p->groups; ++g) {
            if (p->M_g[g] < 0) return fail(UCL_ERR_INVALID_ARG, "M_g[%d] is negative", g);
            sumM += (double)p->M_g[g];
        }
        rows = sumM; N = (double)p->N;
        *flops = 2.0 * sumM * p->N * p->K;
        // every group's A, B and D once
        *bytes = (sumM * p->K + (double)p->groups * p->K * p->N) * si + sumM * p->N * so;
        break;
    }
    case UCL_OP_CONV2D_FPROP:
    case UCL_OP_CONV2D_DGRAD:
    case UCL_OP_CONV2D_WGRAD: {
        if (p->cN <= 0 || p->cH <= 0 || p->cW <= 0 || p->cC <= 0 || p->cKout <= 0 || p->cR <= 0 || p->cS <= 0 ||
            p->stride_h <= 0 || p->stride_w <= 0 || p->dil_h <= 0 || p->dil_w <= 0 || p->pad_h < 0 || p->pad_w < 0)
            return fail(UCL_ERR_INVALID_ARG, "conv geometry must be positive (pads non-negative)");
        const int64_t P = conv_out(p->cH, p->pad_h, p->dil_h, p->cR, p->stride_h);
        const int64_t Q = conv_out(p->cW, p->pad_w, p->dil_w, p->cS, p->stride_w);
        if (P <= 0 || Q <= 0) return fail(UCL_ERR_INVALID_ARG, "conv output is empty");
        const double n_y = (double)p->cN * P * Q * (double)p->cKout, n_x = (double)p->cN * p->cH * p->cW * p->cC;
        const double n_w = (double)p->cKout * p->cR * p->cS * p->cC;
        // padded taps are counted, as a dense implicit GEMM executes them (the same count in all three directions)
        *flops = 2.0 * n_y * (double)(p->cR * p->cS * p->cC);
        if (p->op == UCL_OP_CONV2D_FPROP) {
            rows = (double)p->cN * P * Q; N = (double)p->cKout;
            *bytes = (n_x + n_w) * si + n_y * so;
        } else if (p->op == UCL_OP_CONV2D_DGRAD) {
            rows = (double)p->cN * p->cH * p->cW; N = (double)p->cC;
            *bytes = (n_y + n_w) * si + n_x * so;
        } else {
            rows = (double)p->cKout; N = (double)(p->cR * p->cS * p->cC);
            *bytes = (n_y + n_x) * si + n_w * so;
        }
        break;
    }
    default:
        return fail(UCL_ERR_INVALID_ARG, "unknown op kind %d", p->op);
    }
    if (p->epi) {
        if (p->epi->n_steps < 0 || p->epi->n_steps > UCL_MAX_EPI_STEPS) return fail(UCL_ERR_INVALID_ARG, "bad epilogue length");
        for (int i = 0; i < p->epi->n_steps; ++i) {
            const ucl_epi_step &s = p->epi->steps[i];
            if (!op_has_tensor(s.op)) continue;
            const double se = elem_size(s.dtype);
            const double groups = p->op == UCL_OP_GROUPED_GEMM ? p->groups : 1;
            if (op_is_matrix(s.op)) *bytes += batch * rows * N * se;
            else if (s.op == UCL_EPI_PER_ROW_SCALE || s.op == UCL_EPI_COL_BROADCAST) *bytes += rows * se;
            else *bytes += groups * N * se;
        }
    }
    if (M_out) *M_out = (int64_t)rows;
    if (N_out) *N_out = (int64_t)N;
    return UCL_OK;
}


// Device address of this GPU's copy of the static workspace, looked up once per device with that
// device current (each GPU holds its own copy at its own address).
constexpr int kMaxDevices = 64;
std::mutex g_static_mu;
void *g_static_ptr[kMaxDevices] = {};

ucl_status static_workspace(void **out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(UCL_ERR_LAUNCH, "hipGetDevice failed: %s", hipGetErrorString(e));
    if (dev < 0 || dev >= kMaxDevices) return fail(UCL_ERR_UNSUPPORTED, "device index %d outside [0, %d)", dev, kMaxDevices);
    std::lock_guard<std::mutex> lock(g_static_mu);
    if (!g_static_ptr[dev]) {
        void *ptr = nullptr;
        e = hipGetSymbolAddress((void **)&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr)
            return fail(UCL_ERR_LAUNCH, "hipGetSymbolAddress of the static workspace failed: %s", hipGetErrorString(e));
        g_static_ptr[dev] = ptr;
    }
    *out = g_static_ptr[dev];
    return UCL_OK;
}

// Launch description of a problem given as ucl_problem (packed operands), for the host-only queries.
ucl_status launch_from_problem(const ucl_problem *p, Launch &L) {
    double f, b;
    int64_t M = 0, N = 0;
    if (ucl_status st = characterise(p, &f, &b, &M, &N)) return st;
    if (!is16(p->dt_in) && !is8(p->dt_in)) return fail(UCL_ERR_UNSUPPORTED, "kernels take bf16, fp16 or fp8 inputs");
    if (is8(p->dt_in) && (p->op > UCL_OP_GROUPED_GEMM || p->a_layout != UCL_LAYOUT_K_CONTIGUOUS || p->b_layout != UCL_LAYOUT_K_CONTIGUOUS || p->K % 16))
        return fail(UCL_ERR_UNSUPPORTED, "fp8 inputs are built for gemm, batched_gemm and grouped_gemm with both operands contiguous along K, K a multiple of 16");
    L.mode = p->op == UCL_OP_GROUPED_GEMM ? 1 : p->op == UCL_OP_CONV2D_FPROP ? 2 : p->op == UCL_OP_CONV2D_DGRAD ? 3
             : p->op == UCL_OP_CONV2D_WGRAD ? 4 : 0;
    L.batch = p->op == UCL_OP_BATCHED_GEMM ? p->batch : 1;
    L.M = M; L.N = N;
    L.K = is8(p->dt_in) ? p->K / 2 : p->K;          // 8-bit inputs: the kernels count pairs
    if (L.mode >= 2) {
        const int64_t P = conv_out(p->cH, p->pad_h, p->dil_h, p->cR, p->stride_h), Q = conv_out(p->cW, p->pad_w, p->dil_w, p->cS, p->stride_w);
        L.K = L.mode == 2 ? p->cR * p->cS * p->cC : L.mode == 3 ? p->cR * p->cS * p->cKout : p->cN * P * Q;
    }
    L.groups = p->groups; L.M_g = p->M_g;
    if (L.mode == 2) {
        L.la = 2; L.lb = 0;
    } else if (L.mode == 3) {
        L.la = 2; L.lb = 1; L.ndirect_ok = true;
    } else if (L.mode == 4) {
        L.la = 1; L.lb = 1; L.ndirect_ok = L.mdirect_ok = true;
    } else {
        if ((p->a_layout != UCL_LAYOUT_K_CONTIGUOUS && p->a_layout != UCL_LAYOUT_MN_CONTIGUOUS) ||
            (p->b_layout != UCL_LAYOUT_K_CONTIGUOUS && p->b_layout != UCL_LAYOUT_MN_CONTIGUOUS))
            return fail(UCL_ERR_INVALID_ARG, "a_layout / b_layout must be ucl_operand_layout values");
        if (L.mode == 1 && p->a_layout != UCL_LAYOUT_K_CONTIGUOUS)
            return fail(UCL_ERR_UNSUPPORTED, "grouped_gemm is built for a row-major A");
        L.la = p->a_layout; L.lb = p->b_layout;
        // packed operands: the same reach test for directly copied rows as the launch path applies
        const int64_t Mmax = L.mode == 1 ? 0 : M;
        L.ndirect_ok = L.lb == 1 && ((L.K - 1) * N + N) * 2 < (1ll << 31);
        L.mdirect_ok = L.la == 1 && ((L.K - 1) * Mmax + Mmax) * 2 < (1ll << 31);
    }
    L.dt = dt_code(p->dt_in);
    L.dtD = p->dt_out;
    if (L.mode == 2)
        L.patch_c = conv_patch_channels(p->cW, p->cC, p->cR, p->cS, p->pad_h, p->pad_w, p->stride_h, p->stride_w, p->dil_h, p->dil_w);
    if (L.mode == 3)
        L.patch_c = conv_patch_channels(p->cW, p->cKout, p->cR, p->cS, p->pad_h, p->pad_w, p->stride_h, p->stride_w, p->dil_h, p->dil_w);
    if (L.mode == 1)
        for (int g = 0; g < L.groups; ++g) L.sum_Mg += L.M_g[g];
    return UCL_OK;
}


}  // namespace
}  // namespace ucl

using namespace ucl;

extern "C" {

ucl_status ucl_gemm(int64_t M, int64_t N, int64_t K, const void *A, int32_t dtA, int64_t a_rs, int64_t a_cs,
                    const void *B, int32_t dtB, int64_t b_rs, int64_t b_cs, void *D, int32_t dtD, int64_t d_rs,
                    int64_t d_cs, const ucl_epilogue *epi, const ucl_tuning *tune, void *stream) {
    return gemm_like(1, M, N, K, A, dtA, a_rs, a_cs, 0, B, dtB, b_rs, b_cs, 0, D, dtD, d_rs, d_cs, 0, epi, tune, stream);
}

ucl_status ucl_gemm_static_workspace(int64_t M, int64_t N, int64_t K, const void *A, int32_t dtA, int64_t a_rs, int64_t a_cs,
                                     const void *B, int32_t dtB, int64_t b_rs, int64_t b_cs, void *D, int32_t dtD, int64_t d_rs,
                                     int64_t d_cs, const ucl_epilogue *epi, const ucl_tuning *tune, void *stream) {
    g_err[0] = 0;
    if (!tune || tune->split_k_mode == UCL_SPLIT_K_NONE)
        return fail(UCL_ERR_INVALID_ARG, "ucl_gemm_static_workspace is the split-K form of ucl_gemm: tune must name split_k_mode serial or parallel");
    void *ws = nullptr;
    if (ucl_status st = static_workspace(&ws)) return st;
    ucl_tuning t = *tune;
    t.workspace = ws;                       // (the device address, never the array's name)
    t.workspace_bytes = UCL_STATIC_WORKSPACE_BYTES;
    const ucl_status st = gemm_like(1, M, N, K, A, dtA, a_rs, a_cs, 0, B, dtB, b_rs, b_cs, 0, D, dtD, d_rs, d_cs, 0, epi, &t, stream,
                                    /*clear_counters=*/t.split_k_mode == UCL_SPLIT_K_SERIAL);
    if (st == UCL_ERR_WORKSPACE) {
        // say which limit was hit: the message of the general path speaks of the caller's workspace
        char detail[384];
        snprintf(detail, sizeof(detail), "%s", g_err);
        return fail(UCL_ERR_WORKSPACE, "the static workspace holds %lld bytes: %s (use fewer slices, or ucl_gemm with a workspace of your own)",
                    (long long)UCL_STATIC_WORKSPACE_BYTES, detail);
    }
    return st;
}

ucl_status ucl_batched_gemm(int64_t batch, int64_t M, int64_t N, int64_t K, const void *A, int32_t dtA, int64_t a_rs,
                            int64_t a_cs, int64_t a_bs, const void *B, int32_t dtB, int64_t b_rs, int64_t b_cs,
                            int64_t b_bs, void *D, int32_t dtD, int64_t d_rs, int64_t d_cs, int64_t d_bs,
                            const ucl_epilogue *epi, const ucl_tuning *tune, void *stream) {
    return gemm_like(batch, M, N, K, A, dtA, a_rs, a_cs, a_bs, B, dtB, b_rs, b_cs, b_bs, D, dtD, d_rs, d_cs, d_bs, epi,
                     tune, stream);
}

ucl_status ucl_grouped_gemm(int32_t groups, const int64_t *M_g, int64_t N, int64_t K, const void *const *A_g,
                            int32_t dtA, int64_t a_rs, int64_t a_cs, const void *const *B_g, int32_t dtB, int64_t b_rs,
                            int64_t b_cs, void *const *D_g, int32_t dtD, int64_t d_rs, int64_t d_cs,
                            const ucl_epilogue *epi, const ucl_tuning *tune, void *stream) {
    g_err[0] = 0;
    if (groups <= 0 || groups > UCL_MAX_GROUPS)
        return fail(UCL_ERR_INVALID_ARG, "groups=%d must be in 1..%d", groups, UCL_MAX_GROUPS);
    if (!M_g) return fail(UCL_ERR_INVALID_ARG, "M_g (host array of group sizes) is NULL");
    Launch L;
    L.mode = 1; L.groups = groups; L.M_g = M_g; L.N = N; L.K = K; L.dt = dt_code(dtA); L.dtD = dtD;
    for (int g = 0; g < groups; ++g) {
        if (M_g[g] < 0 || M_g[g] >= (1ll << 31)) return fail(UCL_ERR_INVALID_ARG, "M_g[%d]=%lld must be in [0, 2^31)", g, (long long)M_g[g]);
        L.sum_Mg += M_g[g];
        if (M_g[g] > L.max_Mg) L.max_Mg = M_g[g];
    }
    if (ucl_status st = check_common(1, N, K, dtA, dtB, dtD, A_g, B_g, D_g, /*fp8_ok=*/true)) return st;
    if (a_cs != 1 || (b_rs != 1 && b_cs != 1))
        return fail(UCL_ERR_UNSUPPORTED, "grouped_gemm is built for A row-major (a_cs == 1) and B column-major (b_rs == 1) or row-major (b_cs == 1)");
    const bool b_row = b_rs != 1;             // B[k*b_rs + n]: contiguous along N
    int64_t ldb = b_row ? b_rs : b_cs;
    if (is8(dtA)) {
        // 8-bit inputs are handled as pairs of elements (see gemm_like): K and the leading strides count 16-bit units below
        if (b_row) return fail(UCL_ERR_UNSUPPORTED, "fp8 inputs must both be contiguous along K (A row-major, B column-major)");
        if (K % 16 || a_rs % 16 || ldb % 16)
            return fail(UCL_ERR_UNSUPPORTED, "fp8 inputs: K=%lld and the leading strides (%lld, %lld) must be multiples of 16 (alignment 16 x 1 byte = 16)",
                        (long long)K, (long long)a_rs, (long long)ldb);
        K /= 2; a_rs /= 2; ldb /= 2;
        L.K = K;
    }
    if (K % 8 || a_rs % 8 || ldb % 8 || a_rs < K || ldb < (b_row ? N : K))
        return fail(UCL_ERR_UNSUPPORTED, "K=%lld and the leading strides (%lld, %lld) must be multiples of 8 and at least the contiguous extent", (long long)K, (long long)a_rs, (long long)ldb);
    if (b_row) {
        if (N % 8) return fail(UCL_ERR_UNSUPPORTED, "B is contiguous along N=%lld, which is not a multiple of 8", (long long)N);
        if (((K - 1) * ldb + N) * 2 >= (1ll << 31))
            return fail(UCL_ERR_UNSUPPORTED, "a row-major B of a group must be smaller than 2 GiB (32-bit offsets)");
        L.lb = 1;
        L.ndirect_ok = true;
    }
    if (d_cs != 1 || d_rs < N) return fail(UCL_ERR_UNSUPPORTED, "D must be row-major with d_rs >= N");
    KParams kp;
    memset(&kp, 0, sizeof(kp));
    if (ucl_status st = check_epilogue(epi, L, kp)) return st;
    kp.A_g = A_g; kp.B_g = B_g; kp.D_g = D_g;
    kp.lda = a_rs; kp.ldb = ldb; kp.ldd = d_rs;
    kp.N = (int32_t)N; kp.K = (int32_t)K; kp.groups = groups; kp.dtD = dtD;
    kp.d_vec = d_rs % (16 / elem_size(dtD)) == 0;      // group base pointers are required to be 16-byte aligned
    return run(L, kp, tune, stream);
}

ucl_status ucl_conv2d_fprop(int64_t N, int64_t H, int64_t W, int64_t C, int64_t Kout, int64_t R, int64_t S,
                            int64_t pad_h, int64_t pad_w, int64_t stride_h, int64_t stride_w, int64_t dil_h,
                            int64_t dil_w, const void *x, int32_t dtX, const void *w, int32_t dtW, void *y, int32_t dtY,
                            const ucl_epilogue *epi, const ucl_tuning *tune, void *stream) {
    g_err[0] = 0;
    if (N <= 0 || H <= 0 || W <= 0 || C <= 0 || Kout <= 0 || R <= 0 || S <= 0)
        return fail(UCL_ERR_INVALID_ARG, "conv extents must be positive");
    if (pad_h < 0 || pad_w < 0 || stride_h <= 0 || stride_w <= 0 || dil_h <= 0 || dil_w <= 0)
        return fail(UCL_ERR_INVALID_ARG, "pads must be >= 0, strides and dilations > 0");
    const int64_t P = conv_out(H, pad_h, dil_h, R, stride_h), Q = conv_out(W, pad_w, dil_w, S, stride_w);
    if (P <= 0 || Q <= 0) return fail(UCL_ERR_INVALID_ARG, "conv output is empty (P=%lld, Q=%lld)", (long long)P, (long long)Q);
    const int64_t M = N * P * Q, Kg = R * S * C;
    if (ucl_status st = check_common(M, Kout, Kg, dtX, dtW, dtY, x, w, y)) return st;
    if (C % 8) return fail(UCL_ERR_UNSUPPORTED, "C=%lld must be a multiple of 8 so that a 128-bit load never straddles a filter tap", (long long)C);
    if (!aligned16(x) || !aligned16(w)) return fail(UCL_ERR_UNSUPPORTED, "x and w must be 16-byte aligned");
    if (N * H * W * C * 2 >= (1ll << 31)) return fail(UCL_ERR_UNSUPPORTED, "activation tensor must be smaller than 2 GiB (32-bit offsets)");
    if (H >= (1 << 24) || W >= (1 << 24) || pad_h >= (1 << 24) || pad_w >= (1 << 24))
        return fail(UCL_ERR_UNSUPPORTED, "image extents / pads must be below 2^24");
    Launch L;
    L.mode = 2; L.M = M; L.N = Kout; L.K = Kg; L.la = 2; L.lb = 0; L.dt = dt_code(dtX); L.dtD = dtY;
    L.patch_c = conv_patch_channels(W, C, R, S, pad_h, pad_w, stride_h, stride_w, dil_h, dil_w);
    KParams kp;
    memset(&kp, 0, sizeof(kp));
    if (ucl_status st = check_epilogue(epi, L, kp)) return st;
    kp.A = x; kp.B = w; kp.D = y;
    kp.a_bytes = N * H * W * C * 2;
    kp.lda = 0; kp.ldb = Kg; kp.ldd = Kout;
    kp.M = (int32_t)M; kp.N = (int32_t)Kout; kp.K = (int32_t)Kg; kp.dtD = dtY;
    kp.cH = (int32_t)H; kp.cW = (int32_t)W; kp.cC = (int32_t)C; kp.cS = (int32_t)S; kp.cP = (int32_t)P; kp.cQ = (int32_t)Q;
    kp.pad_h = (int32_t)pad_h; kp.pad_w = (int32_t)pad_w; kp.str_h = (int32_t)stride_h; kp.str_w = (int32_t)stride_w;
    kp.dil_h = (int32_t)dil_h; kp.dil_w = (int32_t)dil_w;
    kp.d_vec = aligned16(y) && (Kout % (16 / elem_size(dtY)) == 0);
    return run(L, kp, tune, stream);
}

// Shared checks of the two gradient entry points; P, Q of the forward geometry.
static ucl_status conv_grad_common(int64_t N, int64_t H, int64_t W, int64_t C, int64_t Kout, int64_t R, int64_t S,
                                   int64_t pad_h, int64_t pad_w, int64_t stride_h, int64_t stride_w, int64_t dil_h,
                                   int64_t dil_w, int64_t *P, int64_t *Q) {
    if (N <= 0 || H <= 0 || W <= 0 || C <= 0 || Kout <= 0 || R <= 0 || S <= 0)
        return fail(UCL_ERR_INVALID_ARG, "conv extents must be positive");
    if (pad_h < 0 || pad_w < 0 || stride_h <= 0 || stride_w <= 0 || dil_h <= 0 || dil_w <= 0)
        return fail(UCL_ERR_INVALID_ARG, "pads must be >= 0, strides and dilations > 0");
    *P = conv_out(H, pad_h, dil_h, R, stride_h);
    *Q = conv_out(W, pad_w, dil_w, S, stride_w);
    if (*P <= 0 || *Q <= 0) return fail(UCL_ERR_INVALID_ARG, "conv output is empty (P=%lld, Q=%lld)", (long long)*P, (long long)*Q);
    if (C % 8 || Kout % 8)
        return fail(UCL_ERR_UNSUPPORTED, "C=%lld and Kout=%lld must be multiples of 8 so that a 128-bit load never straddles a filter tap or a pixel", (long long)C, (long long)Kout);
    if (N * H * W * C * 2 >= (1ll << 31) || N * *P * *Q * Kout * 2 >= (1ll << 31) || Kout * R * S * C * 2 >= (1ll << 31))
        return fail(UCL_ERR_UNSUPPORTED, "activations, output gradient and filter must each be smaller than 2 GiB (32-bit offsets)");
    if (H >= (1 << 24) || W >= (1 << 24) || pad_h >= (1 << 24) || pad_w >= (1 << 24) || dil_h * R >= (1 << 24) || dil_w * S >= (1 << 24))
        return fail(UCL_ERR_UNSUPPORTED, "image extents, pads and dilated filter extents must be below 2^24");
    return UCL_OK;
}

ucl_status ucl_conv2d_dgrad(int64_t N, int64_t H, int64_t W, int64_t C, int64_t Kout, int64_t R, int64_t S,
                            int64_t pad_h, int64_t pad_w, int64_t stride_h, int64_t stride_w, int64_t dil_h,
                            int64_t dil_w, const void *dy, int32_t dtDy, const void *w, int32_t dtW, void *dx, int32_t dtDx,
                            const ucl_epilogue *epi, const ucl_tuning *tune, void *stream) {
    g_err[0] = 0;
    int64_t P = 0, Q = 0;
    if (ucl_status st = conv_grad_common(N, H, W, C, Kout, R, S, pad_h, pad_w, stride_h, stride_w, dil_h, dil_w, &P, &Q)) return st;
    const int64_t M = N * H * W, Kg = R * S * Kout;
    if (ucl_status st = check_common(M, C, Kg, dtDy, dtW, dtDx, dy, w, dx)) return st;
    if (!aligned16(dy) || !aligned16(w)) return fail(UCL_ERR_UNSUPPORTED, "dy and w must be 16-byte aligned");
    Launch L;
    L.mode = 3; L.M = M; L.N = C; L.K = Kg; L.la = 2; L.lb = 1; L.ndirect_ok = true; L.dt = dt_code(dtDy); L.dtD = dtDx;
    L.patch_c = conv_patch_channels(W, Kout, R, S, pad_h, pad_w, stride_h, stride_w, dil_h, dil_w);
    KParams kp;
    memset(&kp, 0, sizeof(kp));
    if (ucl_status st = check_epilogue(epi, L, kp)) return st;
    kp.A = dy; kp.B = w; kp.D = dx;
    kp.a_bytes = N * P * Q * Kout * 2;
    kp.b_bytes = Kout * R * S * C * 2;
    kp.lda = 0; kp.ldb = R * S * C; kp.ldd = C;
    kp.M = (int32_t)M; kp.N = (int32_t)C; kp.K = (int32_t)Kg; kp.dtD = dtDx;
    // the gathered tensor is dy: its extents take the place of the image's, the rows are input pixels
    kp.cH = (int32_t)P; kp.cW = (int32_t)Q; kp.cC = (int32_t)Kout; kp.cS = (int32_t)S; kp.cP = (int32_t)H; kp.cQ = (int32_t)W;
    kp.pad_h = (int32_t)pad_h; kp.pad_w = (int32_t)pad_w; kp.str_h = (int32_t)stride_h; kp.str_w = (int32_t)stride_w;
    kp.dil_h = (int32_t)dil_h; kp.dil_w = (int32_t)dil_w;
    kp.d_vec = aligned16(dx) && (C % (16 / elem_size(dtDx)) == 0);
    return run(L, kp, tune, stream);
}

ucl_status ucl_conv2d_wgrad(int64_t N, int64_t H, int64_t W, int64_t C, int64_t Kout, int64_t R, int64_t S,
                            int64_t pad_h, int64_t pad_w, int64_t stride_h, int64_t stride_w, int64_t dil_h,
                            int64_t dil_w, const void *dy, int32_t dtDy, const void *x, int32_t dtX, void *dw, int32_t dtDw,
                            const ucl_epilogue *epi, const ucl_tuning *tune, void *stream) {
    g_err[0] = 0;
    int64_t P = 0, Q = 0;
    if (ucl_status st = conv_grad_common(N, H, W, C, Kout, R, S, pad_h, pad_w, stride_h, stride_w, dil_h, dil_w, &P, &Q)) return st;
    const int64_t Ng = R * S * C, Kg = N * P * Q;
    if (ucl_status st = check_common(Kout, Ng, Kg, dtDy, dtX, dtDw, dy, x, dw)) return st;
    if (!aligned16(dy) || !aligned16(x)) return fail(UCL_ERR_UNSUPPORTED, "dy and x must be 16-byte aligned");
    Launch L;
    L.mode = 4; L.M = Kout; L.N = Ng; L.K = Kg; L.la = 1; L.lb = 1; L.ndirect_ok = L.mdirect_ok = true;
    L.dt = dt_code(dtDy); L.dtD = dtDw;
    KParams kp;
    memset(&kp, 0, sizeof(kp));
    if (ucl_status st = check_epilogue(epi, L, kp)) return st;
    kp.A = dy; kp.B = x; kp.D = dw;
    kp.b_bytes = N * H * W * C * 2;
    kp.lda = Kout; kp.ldb = 0; kp.ldd = Ng;
    kp.M = (int32_t)Kout; kp.N = (int32_t)Ng; kp.K = (int32_t)Kg; kp.dtD = dtDw;
    kp.cH = (int32_t)H; kp.cW = (int32_t)W; kp.cC = (int32_t)C; kp.cS = (int32_t)S; kp.cP = (int32_t)P; kp.cQ = (int32_t)Q;
    kp.pad_h = (int32_t)pad_h; kp.pad_w = (int32_t)pad_w; kp.str_h = (int32_t)stride_h; kp.str_w = (int32_t)stride_w;
    kp.dil_h = (int32_t)dil_h; kp.dil_w = (int32_t)dil_w;
    kp.d_vec = aligned16(dw) && (Ng % (16 / elem_size(dtDw)) == 0);
    return run(L, kp, tune, stream);
}

ucl_status ucl_transpose(int64_t batch, int64_t rows, int64_t cols, const void *src, int32_t dt_src, void *dst,
                         int32_t dt_dst, void *stream) {
    g_err[0] = 0;
    const ucl_status st = transpose_run(batch, rows, cols, src, dt_src, dst, dt_dst, stream);
    if (st != UCL_OK) return fail(st, "%s", transpose_last_error());
    return UCL_OK;
}

ucl_status ucl_sol_bound(const ucl_problem *p, const ucl_hw *hw, ucl_sol_report *out) {
    g_err[0] = 0;
    if (!out) return fail(UCL_ERR_INVALID_ARG, "report pointer is NULL");
    double flops = 0, bytes = 0;
    if (ucl_status st = characterise(p, &flops, &bytes, nullptr, nullptr)) return st;
    // Hardware limits: published peaks, scaled linearly by the clock ratios.
    ucl_hw mi355x = {2516.6e12, 157.3e12, 8.0e12, 1.0, 1.0, 5033.2e12};
    const ucl_hw &h = hw ? *hw : mi355x;
    if (!(h.peak_bw > 0) || !(h.compute_clock_ratio > 0) || !(h.memory_clock_ratio > 0))
        return fail(UCL_ERR_INVALID_ARG, "hardware descriptor needs positive peaks and clock ratios");
    const double peak = (p->dt_in == UCL_F32 ? h.peak_flops_f32 : is8(p->dt_in) ? h.peak_flops_8bit : h.peak_flops_16bit) * h.compute_clock_ratio;
    if (!(peak > 0)) return fail(UCL_ERR_INVALID_ARG, "hardware descriptor has no compute peak for %s inputs", dtype_name(p->dt_in));
    const double bw = h.peak_bw * h.memory_clock_ratio;
    out->flops = flops;
    out->bytes = bytes;
    out->peak_flops = peak;
    out->peak_bw = bw;
    out->ai = flops / bytes;
    out->ridge = peak / bw;
    out->t_compute = flops / peak;
    out->t_mem = bytes / bw;
    out->t_sol = out->t_compute > out->t_mem ? out->t_compute : out->t_mem;
    out->compute_bound = out->ai >= out->ridge ? 1 : 0;
    out->reserved = 0;
    return UCL_OK;
}

ucl_status ucl_select_tuning(const ucl_problem *p, ucl_tuning *out) {
    g_err[0] = 0;
    if (!out) return fail(UCL_ERR_INVALID_ARG, "output pointer is NULL");
    Launch L;
    if (ucl_status st = launch_from_problem(p, L)) return st;
    const VariantDesc *v = select_variant(L, nullptr);
    if (!v) return fail(UCL_ERR_UNSUPPORTED, "no kernel built for this problem");
    memset(out, 0, sizeof(*out));
    out->tile_m = v->tile_m; out->tile_n = v->tile_n; out->tile_k = v->tile_k; out->stages = v->stages;
    out->raster = default_raster(*v, L);
    out->iterator = v->la == 3 ? UCL_ITER_FIXED_STRIDE_DILATION : v->la == 2 ? UCL_ITER_ANALYTIC : UCL_ITER_DEFAULT;
    return UCL_OK;
}

ucl_status ucl_workspace_size(const ucl_problem *p, const ucl_tuning *tune, int64_t *bytes, int32_t *slices_out) {
    g_err[0] = 0;
    if (!bytes) return fail(UCL_ERR_INVALID_ARG, "output pointer is NULL");
    *bytes = 0;
    if (slices_out) *slices_out = 1;
    Launch L;
    if (ucl_status st = launch_from_problem(p, L)) return st;
    if (tune && (tune->iterator < 0 || tune->iterator > UCL_ITER_FIXED_STRIDE_DILATION))
        return fail(UCL_ERR_INVALID_ARG, "iterator=%d is not a ucl_conv_iterator", tune->iterator);
    const VariantDesc *v = select_variant(L, tune);
    if (!v) return fail(UCL_ERR_UNSUPPORTED, "no kernel built for this problem and tuning; see ucl_variant()");
    SplitPlan sp;
    if (ucl_status st = plan_split(L, *v, tune, count_tiles(L, v->tile_m, v->tile_n), sp)) return st;
    *bytes = sp.bytes;
    if (slices_out) *slices_out = sp.slices;
    return UCL_OK;
}

ucl_status ucl_workspace_init(void *workspace, int64_t workspace_bytes, void *stream) {
    g_err[0] = 0;
    if (!workspace || !aligned16(workspace)) return fail(UCL_ERR_INVALID_ARG, "workspace must be a 16-byte aligned device pointer");
    if (workspace_bytes < UCL_WORKSPACE_COUNTER_BYTES)
        return fail(UCL_ERR_WORKSPACE, "a split-K workspace holds at least its %d bytes of counters, got %lld", UCL_WORKSPACE_COUNTER_BYTES, (long long)workspace_bytes);
    hipLaunchKernelGGL(zero_words_kernel, dim3(UCL_WORKSPACE_COUNTER_BYTES / 16 / 256), dim3(256), 0, (hipStream_t)stream, (uint32_t *)workspace);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(UCL_ERR_LAUNCH, "kernel launch failed: %s", hipGetErrorString(e));
    return UCL_OK;
}

ucl_status ucl_tile_map(int32_t groups, const int32_t *tiles_m, int32_t tiles_n, int32_t raster, int32_t wg,
                        int32_t *group, int32_t *tile_m, int32_t *tile_n) {
    g_err[0] = 0;
    if (groups <= 0 || !tiles_m || tiles_n <= 0 || raster <= 0 || !group || !tile_m || !tile_n)
        return fail(UCL_ERR_INVALID_ARG, "bad arguments to ucl_tile_map");
    std::vector<int32_t> start(groups + 1, 0);
    for (int g = 0; g < groups; ++g) {
        if (tiles_m[g] < 0) return fail(UCL_ERR_INVALID_ARG, "tiles_m[%d] is negative", g);
        start[g + 1] = start[g] + tiles_m[g] * tiles_n;
    }
    const int total = start[groups];
    if (wg < 0 || wg >= total) return fail(UCL_ERR_INVALID_ARG, "wg=%d outside [0, %d)", wg, total);
    int t = xcd_remap(wg, total);
    const int g = find_group(start.data(), groups, t);
    t -= start[g];
    int tm, tn;
    band_raster(t, tiles_m[g], tiles_n, raster, tm, tn);
    *group = g; *tile_m = tm; *tile_n = tn;
    return UCL_OK;
}

int32_t ucl_num_variants(void) { return (int32_t)all_variants().size(); }

ucl_status ucl_variant(int32_t i, ucl_variant_info *out) {
    const auto &vs = all_variants();
    if (i < 0 || i >= (int)vs.size() || !out) return fail(UCL_ERR_INVALID_ARG, "variant index %d outside [0, %d)", i, (int)vs.size());
    const VariantDesc &v = vs[i];
    memset(out, 0, sizeof(*out));
    out->tile_m = v.tile_m; out->tile_n = v.tile_n; out->tile_k = v.tile_k; out->stages = v.stages;
    out->iterator = v.la == 3 ? UCL_ITER_FIXED_STRIDE_DILATION : v.la == 2 ? UCL_ITER_ANALYTIC : UCL_ITER_DEFAULT;
    out->op_class = v.mode;
    out->dt_in = v.dt == 1 ? UCL_F16 : v.dt == 2 ? UCL_FP8_E4M3 : v.dt == 3 ? UCL_FP8_E5M2 : UCL_BF16;
    out->a_layout = (v.la == 1 || v.la == 5) ? UCL_LAYOUT_MN_CONTIGUOUS : UCL_LAYOUT_K_CONTIGUOUS;
    out->b_layout = (v.lb == 1 || v.lb == 4) ? UCL_LAYOUT_MN_CONTIGUOUS : UCL_LAYOUT_K_CONTIGUOUS;
    out->a_path = v.la; out->b_path = v.lb;
    out->lds_bytes = v.lds_bytes;
    out->patch_channels = v.patch_c;
    out->scheduler = v.persistent == 2 ? UCL_SCHED_STREAM_K : v.persistent ? UCL_SCHED_PERSISTENT : UCL_SCHED_DEFAULT;
    return UCL_OK;
}

const char *ucl_status_string(ucl_status s) {
    switch (s) {
    case UCL_OK: return "UCL_OK";
    case UCL_ERR_INVALID_ARG: return "UCL_ERR_INVALID_ARG";
    case UCL_ERR_UNSUPPORTED: return "UCL_ERR_UNSUPPORTED";
    case UCL_ERR_WORKSPACE: return "UCL_ERR_WORKSPACE";
    case UCL_ERR_LAUNCH: return "UCL_ERR_LAUNCH";
    }
    return "UCL_ERR_?";
}

const char *ucl_last_error(void) { return g_err; }
const char *ucl_version(void) { return "ucl 0.1 (gfx950)"; }

}  // extern "C"
