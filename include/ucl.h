/*
 * ucl.h -- C ABI of the MI355X (gfx950) fused-epilogue GEMM / conv library.
 *
 * The operations are the ones the paper's kernel DSL names (Sec. 3 and the
 * appendix grammar, rule `operation`): gemm(), batched_gemm(),
 * grouped_gemm(expert_count=E), conv2d_fprop(kernel_h, kernel_w); their
 * configuration knobs (rule `configuration`: dtype triple, layouts, tile,
 * stages, alignment, swizzle, alpha/beta scaling) become plain arguments; the
 * `>>` epilogue chain (rule `epilogue_op`, Table (c)) becomes an ordered array
 * of steps that the kernel applies to the fp32 accumulator in registers before
 * the one rounding to the output type.  ucl_sol_bound is the paper's
 * Speed-of-Light analysis (Sec. 4.1) as a function.
 *
 * General conventions
 *   - Every tensor pointer is caller-owned DEVICE memory unless marked HOST.
 *     The library allocates nothing, frees nothing, keeps no pointer after a
 *     call returns, and never synchronises: each call validates its arguments
 *     on the host, then enqueues its kernel on `stream` (a hipStream_t passed
 *     as void*; NULL = the null stream) and returns: one kernel per call (two
 *     for split-K in PARALLEL mode; ucl_gemm_static_workspace in SERIAL mode
 *     puts a small fill kernel in front).
 *   - Strides are in ELEMENTS.  Inputs are UCL_BF16 or UCL_F16 (both operands
 *     the same type), accumulation is fp32, outputs are UCL_BF16, UCL_F16 or
 *     UCL_F32.  ucl_gemm, ucl_batched_gemm and ucl_grouped_gemm also take
 *     UCL_FP8_E4M3 or UCL_FP8_E5M2 inputs (both operands the same type, both
 *     contiguous along K; K, the leading strides and the batch strides
 *     multiples of 16).
 *   - Alignment (the paper's rule (alignment * element_size) % 16 == 0,
 *     grammar notes, constraint 3): A and B base pointers are 16-byte aligned,
 *     one of their two strides is 1 and the other a multiple of 8, and K (for
 *     K-contiguous operands) or M / N (for operands contiguous along M / N) is
 *     a multiple of 8.  D and the epilogue's tensor operands may have any N and
 *     any strides; they are accessed with 128-bit loads / stores when base and
 *     row starts are 16-byte aligned (leading and batch strides multiples of 8
 *     for 16-bit types, of 4 for fp32), element by element otherwise.  In
 *     ucl_grouped_gemm the per-group pointers live on the device, where the
 *     host cannot inspect them: every one of them must be 16-byte aligned,
 *     except those of vectors indexed by m (PER_ROW_SCALE, COL_BROADCAST),
 *     which are read element by element.
 *   - Errors: a nonzero ucl_status is returned BEFORE anything is launched;
 *     ucl_last_error() gives a thread-local sentence saying what was wrong and
 *     why (the paper's compiler explains failed validation the same way,
 *     Sec. 3 "Compilation").  Nothing aborts or throws.
 *   - Explicit tuning is honoured exactly or rejected, never silently replaced
 *     (Sec. 3: all choices explicit, no hidden defaults).  tune == NULL or an
 *     all-zero struct selects from the built-in per-problem table.
 */
#ifndef UCL_H_
#define UCL_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum ucl_status {
    UCL_OK = 0,
    UCL_ERR_INVALID_ARG = 1,   /* null pointer, non-positive extent, bad enum            */
    UCL_ERR_UNSUPPORTED = 2,   /* legal request outside what the kernels implement       */
    UCL_ERR_WORKSPACE = 3,     /* tile x stages exceeds the 160 KiB of LDS per CU, or the
                                  split-K workspace is missing, misaligned or too small  */
    UCL_ERR_LAUNCH = 4         /* the HIP runtime refused the launch                     */
} ucl_status;

/* UCL_FP8_E4M3 / UCL_FP8_E5M2 (the open-standard 8-bit formats: e4m3 without infinities, largest value
 * 448; e5m2 with IEEE-style infinities) are input types only. */
typedef enum ucl_dtype { UCL_F32 = 0, UCL_F16 = 1, UCL_BF16 = 2, UCL_FP8_E4M3 = 3, UCL_FP8_E5M2 = 4 } ucl_dtype;

/* Epilogue vocabulary: grammar rule `epilogue_op`.  v is the running fp32
 * value of output element (m, n); m = output row (GEMM row / flattened n,p,q
 * of a conv), n = output column (GEMM column / conv output channel). */
typedef enum ucl_epi_op {
    UCL_EPI_SCALE = 1,        /* scale(alpha)          v * p0                              */
    UCL_EPI_BIAS = 2,         /* bias()                v + vec[n]                          */
    UCL_EPI_AUX_LOAD = 3,     /* aux_load(id)          v + p0 * T[m*ld + n]  (residual; p0 = beta) */
    UCL_EPI_RELU = 4,
    UCL_EPI_GELU_TANH = 5,    /* gelu(), tanh form                                          */
    UCL_EPI_GELU_ERF = 6,     /* gelu(), erf form                                           */
    UCL_EPI_SILU = 7,
    UCL_EPI_SIGMOID = 8,
    UCL_EPI_TANH = 9,
    UCL_EPI_MISH = 10,
    UCL_EPI_HARDSWISH = 11,
    UCL_EPI_LEAKY_RELU = 12,  /* leaky_relu(alpha)     v > 0 ? v : p0 * v                  */
    UCL_EPI_ELU = 13,         /* elu(alpha)            v > 0 ? v : p0 * (exp(v) - 1)       */
    UCL_EPI_CLAMP = 14,       /* clip / clamp(min,max) min(max(v, p0), p1)                 */
    UCL_EPI_PER_ROW_SCALE = 15, /* per_row_scale()     v * vec[m]                          */
    UCL_EPI_PER_COL_SCALE = 16, /* per_col_scale(), per_channel_scale()   v * vec[n]       */
    UCL_EPI_ROW_BROADCAST = 17, /* row_broadcast(id)   v + vec[n]                          */
    UCL_EPI_COL_BROADCAST = 18, /* column_broadcast(id) v + vec[m]                         */
    UCL_EPI_AUX_STORE = 19    /* aux_store(id)         T[m*ld + n] = round(v); v unchanged */
} ucl_epi_op;

#define UCL_MAX_EPI_STEPS 8
#define UCL_MAX_GROUPS 256

/* One step of the chain.  ptr (device) is the step's tensor operand, of type
 * `dtype` (ucl_dtype): a vector of length N (ops indexed by n) or M (ops
 * indexed by m), or a matrix addressed as ptr[b*bs + m*ld + n] for AUX_LOAD /
 * AUX_STORE (b = batch index, bs = 0 shares it across batches).  In
 * ucl_grouped_gemm, ptr is instead a device array of `groups` pointers, one
 * operand per group, each indexed with the group's own m.  Steps without a
 * tensor ignore ptr. */
typedef struct ucl_epi_step {
    int32_t op;        /* ucl_epi_op */
    int32_t dtype;     /* ucl_dtype of ptr */
    float p0, p1;
    const void *ptr;
    int64_t ld;
    int64_t bs;
} ucl_epi_step;

typedef struct ucl_epilogue {
    int32_t n_steps;   /* 0..UCL_MAX_EPI_STEPS; NULL epilogue == 0 steps */
    int32_t reserved;
    ucl_epi_step steps[UCL_MAX_EPI_STEPS];
} ucl_epilogue;

/* How conv2d_fprop reads the activations, and conv2d_dgrad the output gradient
 * (`.with_iterator`).  ANALYTIC gathers every filter tap from global memory and serves
 * every geometry.  FIXED_STRIDE_DILATION (3x3 filter, unit stride and dilation, pad 1,
 * W <= 58; fprop: C = 64 or 128, dgrad: Kout = 64 or 128) copies the pixels a tile needs into LDS
 * once and reads all nine taps from there.  DEFAULT: the table takes the second where it
 * applies.  conv2d_wgrad accepts any valid value and ignores it. */
typedef enum ucl_conv_iterator {
    UCL_ITER_DEFAULT = 0,
    UCL_ITER_ANALYTIC = 1,
    UCL_ITER_FIXED_STRIDE_DILATION = 2
} ucl_conv_iterator;

/* `.with_split_k(mode=..., slices=...)`: the K extent is cut into `slices` ranges (multiples of 64)
 * that run as separate workgroups; their fp32 partial tiles pass through the caller's workspace and
 * are added in slice order 0, 1, 2, ... (a fixed order: results do not depend on timing), after
 * which the epilogue chain runs once.  SERIAL: one launch; the workgroup that finishes a tile last
 * (a counter per tile in the workspace) adds the slices up and runs the epilogue.  PARALLEL: the
 * slices are written by one launch and added up and finished by another; with more than two slices
 * a small reduction kernel between them adds the slices up with the whole GPU (three launches in
 * all, on the caller's stream; two where the chain has the form act(alpha * acc + bias[n] +
 * beta * R[m,n]) -- any part may be missing, the empty chain included -- and the rows of D are
 * 16-byte aligned: the reduction kernel then runs the chain on the sums and stores D itself).
 * Both give bit-identical results.  With no tile named in the same
 * ucl_tuning, the tile is chosen for the split-K launch (not as for the unsplit problem). */
typedef enum ucl_split_k_mode { UCL_SPLIT_K_NONE = 0, UCL_SPLIT_K_SERIAL = 1, UCL_SPLIT_K_PARALLEL = 2 } ucl_split_k_mode;

/* `.with_scheduler(tile=...)`.  DEFAULT: one workgroup per output tile, dealt out by the hardware as
 * CUs free up.  PERSISTENT: one workgroup per CU slot (a multiple of 8, so a workgroup stays on the
 * tile run of its XCD), each walking the tile order with a stride of the grid size; built for gemm,
 * batched_gemm and grouped_gemm with operands contiguous along K and tiles up to 128x128 (grouped:
 * 64x64; the larger tiles' kernels have no registers to spare for the loop; see ucl_variant()).
 * STREAM_K: one workgroup per CU slot; as many whole rounds of tiles as the grid divides are walked
 * as under PERSISTENT, and the K extent of the remaining tiles is cut into 64-wide steps that are
 * dealt out evenly, so that a workgroup may compute parts of tiles (fewer tiles than CU slots: no
 * whole round, at most one workgroup per CU, and runs long enough that adding a tile's parts up
 * does not take longer than computing them).  Parts pass through the
 * caller's workspace (as for split-K: ucl_workspace_size, ucl_workspace_init; two tile-sized slots
 * per workgroup behind the counters) and are added in k order by the workgroup that delivers a
 * tile's last part: results do not depend on timing.  Built for gemm and batched_gemm with 16-bit
 * inputs contiguous along K, tiles 128x128 and 64x64; cannot be combined with split-K.  Requests
 * outside what is built are rejected with UCL_ERR_UNSUPPORTED. */
typedef enum ucl_tile_scheduler { UCL_SCHED_DEFAULT = 0, UCL_SCHED_PERSISTENT = 1, UCL_SCHED_STREAM_K = 2 } ucl_tile_scheduler;

/* The first UCL_WORKSPACE_COUNTER_BYTES of a split-K workspace hold the per-tile counters. */
#define UCL_WORKSPACE_COUNTER_BYTES 65536
#define UCL_SPLIT_K_MAX_TILES (UCL_WORKSPACE_COUNTER_BYTES / 4)

/* Explicit kernel choice (`.with_tile`, `.with_stages`, `.with_swizzle`, `.with_iterator`,
 * `.with_split_k`, `.with_scheduler`).
 * tile_k (K extent of one LDS stage) is 32 or 64; stages is the number of LDS stage
 * buffers: 3 or more for operands contiguous along K (stages - 1 k-tiles are in
 * flight while one is being multiplied), or 2 with tile_k = 64 (each half of a
 * buffer is refilled as soon as it has been read).  Operands contiguous along M / N
 * use the same loops (their rows of k are copied directly and read back through the
 * LDS transpose read); a slower form with 2 buffers that transposes them in registers
 * serves matrices beyond the 2 GiB reach of 32-bit offsets.
 * Only built combinations are accepted (ucl_variant()); all four of tile_m, tile_n, tile_k,
 * stages zero = the table's choice.  raster = width, in tile rows, of the
 * bands the tile order walks column by column (1, 2, 4, 8, 16; the swizzle
 * knob's Identity1..8), 0 = table default.  The order is also XCD-aware:
 * workgroup ids that land on the same XCD (id mod 8) get neighbouring tiles.
 * iterator is a ucl_conv_iterator; the GEMM entry points accept any valid value and ignore it.
 * split_k_mode / split_k_slices (ucl_gemm, ucl_batched_gemm and ucl_conv2d_wgrad only; slices = 0 lets the library
 * choose, slices = 1 is no split): the library allocates nothing, so the caller passes
 * `workspace`, DEVICE memory, 16-byte aligned, of at least ucl_workspace_size() bytes.  SERIAL needs
 * the first UCL_WORKSPACE_COUNTER_BYTES to be zero when the call starts: clear them once with
 * ucl_workspace_init(); every call leaves them zero again.  Calls that share a workspace must not
 * overlap in time.  Without a split, workspace is ignored.
 * scheduler is a ucl_tile_scheduler; STREAM_K uses the workspace in the same way (zeroed counters, left zero). */
typedef struct ucl_tuning {
    int32_t tile_m, tile_n, tile_k, stages, raster;
    int32_t iterator;
    int32_t split_k_mode, split_k_slices;
    int32_t scheduler;
    int32_t reserved;
    void *workspace;
    int64_t workspace_bytes;
} ucl_tuning;

/* D[m,n] = E( sum_k A[m*a_rs + k*a_cs] * B[k*b_rs + n*b_cs] ), written to
 * D[m*d_rs + n*d_cs] (grammar `gemm_op`; layouts RowMajor / ColumnMajor are
 * the two stride patterns).  d_cs must be 1 (row-major D); for a column-major
 * D call with the operands' roles swapped, (A.B)^T = B^T.A^T. */
ucl_status ucl_gemm(int64_t M, int64_t N, int64_t K,
                    const void *A, int32_t dtA, int64_t a_rs, int64_t a_cs,
                    const void *B, int32_t dtB, int64_t b_rs, int64_t b_cs,
                    void *D, int32_t dtD, int64_t d_rs, int64_t d_cs,
                    const ucl_epilogue *epi, const ucl_tuning *tune, void *stream);

/* ucl_gemm with split-K for callers that cannot allocate a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments and results as
 * ucl_gemm with the same tune (which must name split_k_mode SERIAL or PARALLEL; tune->workspace and
 * tune->workspace_bytes are ignored), but the partial tiles and counters live in a workspace of
 * UCL_STATIC_WORKSPACE_BYTES that is part of the library's device code: every GPU the library runs
 * on holds one copy until the process ends.  The call allocates and frees nothing (the first call
 * on a device looks the array's address up; make that call outside a graph capture).  A problem
 * whose slices x tiles x tile_m x tile_n x 4 bytes of partial tiles (ucl_workspace_size) exceed the
 * static workspace is rejected with UCL_ERR_WORKSPACE before anything is launched.  All calls on a
 * GPU share that GPU's array: calls that overlap in time on one GPU race; the SERIAL form clears
 * the counter area with a small fill kernel ahead of the GEMM kernel, on the same stream. */
#define UCL_STATIC_WORKSPACE_BYTES (UCL_WORKSPACE_COUNTER_BYTES + (8 << 20))
ucl_status ucl_gemm_static_workspace(int64_t M, int64_t N, int64_t K,
                                     const void *A, int32_t dtA, int64_t a_rs, int64_t a_cs,
                                     const void *B, int32_t dtB, int64_t b_rs, int64_t b_cs,
                                     void *D, int32_t dtD, int64_t d_rs, int64_t d_cs,
                                     const ucl_epilogue *epi, const ucl_tuning *tune, void *stream);

/* Strided batched GEMM (grammar `batched_gemm_op`): the above for b in
 * [0, batch) with operands advanced by b * {a,b,d}_bs elements.  A batch
 * stride of 0 shares that operand. */
ucl_status ucl_batched_gemm(int64_t batch, int64_t M, int64_t N, int64_t K,
                            const void *A, int32_t dtA, int64_t a_rs, int64_t a_cs, int64_t a_bs,
                            const void *B, int32_t dtB, int64_t b_rs, int64_t b_cs, int64_t b_bs,
                            void *D, int32_t dtD, int64_t d_rs, int64_t d_cs, int64_t d_bs,
                            const ucl_epilogue *epi, const ucl_tuning *tune, void *stream);

/* Grouped GEMM (grammar `grouped_gemm_op`, expert_count = groups): `groups`
 * independent problems (M_g[g], N, K) in one launch.  M_g is a HOST array
 * (so the grid can be sized without a device round trip); M_g[g] == 0 is legal
 * and skips the group.  A_g, B_g, D_g are DEVICE arrays of `groups` device
 * pointers (the per-group pointer table); strides are shared by all groups.
 * A is row-major (a_cs == 1); B is column-major (b_rs == 1, stored [N][K]) or
 * row-major (b_cs == 1, stored [K][N], N a multiple of 8, each group's B below
 * 2 GiB).  groups <= UCL_MAX_GROUPS, M_g[g] < 2^31. */
ucl_status ucl_grouped_gemm(int32_t groups, const int64_t *M_g, int64_t N, int64_t K,
                            const void *const *A_g, int32_t dtA, int64_t a_rs, int64_t a_cs,
                            const void *const *B_g, int32_t dtB, int64_t b_rs, int64_t b_cs,
                            void *const *D_g, int32_t dtD, int64_t d_rs, int64_t d_cs,
                            const ucl_epilogue *epi, const ucl_tuning *tune, void *stream);

/* Forward convolution as an implicit GEMM (grammar `conv2d_fprop`, layouts
 * TensorNHWC): x [N,H,W,C], w [Kout,R,S,C], y [N,P,Q,Kout], all packed,
 *   y[n,p,q,k] = E( sum_{r,s,c} x[n, p*stride_h - pad_h + r*dil_h,
 *                                    q*stride_w - pad_w + s*dil_w, c] * w[k,r,s,c] )
 * with out-of-image taps contributing zero (cross-correlation, no filter flip),
 * P = (H + 2 pad_h - dil_h (R-1) - 1) / stride_h + 1, Q likewise.  The chain
 * sees m = (n*P + p)*Q + q and n = k, so bias() is per output channel and an
 * AUX_LOAD tensor is shaped like y (ld = Kout).  C must be a multiple of 8. */
ucl_status ucl_conv2d_fprop(int64_t N, int64_t H, int64_t W, int64_t C, int64_t Kout,
                            int64_t R, int64_t S, int64_t pad_h, int64_t pad_w,
                            int64_t stride_h, int64_t stride_w, int64_t dil_h, int64_t dil_w,
                            const void *x, int32_t dtX, const void *w, int32_t dtW,
                            void *y, int32_t dtY,
                            const ucl_epilogue *epi, const ucl_tuning *tune, void *stream);

/* Data gradient of the convolution above (grammar `conv2d_dgrad`), as an implicit GEMM of
 * N*H*W rows, C columns and R*S*Kout deep: dy [N,P,Q,Kout], w [Kout,R,S,C] -> dx [N,H,W,C],
 *   dx[n,h,w,c] = E( sum over (p,r), (q,s), k with p*stride_h - pad_h + r*dil_h == h and
 *                    q*stride_w - pad_w + s*dil_w == w of dy[n,p,q,k] * w[k,r,s,c] ),
 * P and Q as ucl_conv2d_fprop derives them from the same arguments (N, H, W, C describe the
 * ACTIVATIONS, i.e. the output of this call).  The chain sees m = (n*H + h)*W + w and n = c.
 * C and Kout must be multiples of 8, all three tensors packed, 16-byte aligned, below 2 GiB. */
ucl_status ucl_conv2d_dgrad(int64_t N, int64_t H, int64_t W, int64_t C, int64_t Kout,
                            int64_t R, int64_t S, int64_t pad_h, int64_t pad_w,
                            int64_t stride_h, int64_t stride_w, int64_t dil_h, int64_t dil_w,
                            const void *dy, int32_t dtDy, const void *w, int32_t dtW,
                            void *dx, int32_t dtDx,
                            const ucl_epilogue *epi, const ucl_tuning *tune, void *stream);

/* Weight gradient (grammar `conv2d_wgrad`), as an implicit GEMM of Kout rows, R*S*C columns and
 * N*P*Q deep: dy [N,P,Q,Kout], x [N,H,W,C] -> dw [Kout,R,S,C],
 *   dw[k,r,s,c] = E( sum_{n,p,q} dy[n,p,q,k] * x[n, p*stride_h - pad_h + r*dil_h,
 *                                                   q*stride_w - pad_w + s*dil_w, c] ),
 * out-of-image x contributing zero.  The chain sees m = k and n = (r*S + s)*C + c.  The deep
 * reduction over few output tiles is what split-K is for: tune->split_k_mode / workspace apply as
 * for ucl_gemm (ucl_workspace_size with UCL_OP_CONV2D_WGRAD).  Same size and alignment rules. */
ucl_status ucl_conv2d_wgrad(int64_t N, int64_t H, int64_t W, int64_t C, int64_t Kout,
                            int64_t R, int64_t S, int64_t pad_h, int64_t pad_w,
                            int64_t stride_h, int64_t stride_w, int64_t dil_h, int64_t dil_w,
                            const void *dy, int32_t dtDy, const void *x, int32_t dtX,
                            void *dw, int32_t dtDw,
                            const ucl_epilogue *epi, const ucl_tuning *tune, void *stream);

/* Transform stage of a `pipeline(...)` program (grammar `transpose_op`:
 * transpose(tensor, NCL, NLC [, dtype_in, dtype_out]); NCHW <-> NHWC is the same
 * with H*W flattened into L): src is `batch` packed row-major rows x cols matrices,
 * dst `batch` packed cols x rows matrices, and
 *   dst[b][c][r] = convert(src[b][r][c]),
 * the conversion between fp32 / fp16 / bf16 exact where the target holds the value
 * and round-to-nearest-even otherwise.  NCL -> NLC: rows = C, cols = L; NHWC -> NCHW:
 * rows = H*W, cols = C.  src and dst are DEVICE pointers owned by the caller; their byte
 * ranges must not overlap (an overlap is rejected with UCL_ERR_INVALID_ARG: a transpose in
 * place is not supported); any extents are accepted (zero extents do nothing), 16-byte aligned
 * pointers with cols*size(dt_src) and rows*size(dt_dst) multiples of 16 take the
 * 128-bit path.  Errors as for the other entry points, nothing is launched then. */
ucl_status ucl_transpose(int64_t batch, int64_t rows, int64_t cols, const void *src, int32_t dt_src,
                         void *dst, int32_t dt_dst, void *stream);

/* ---- Speed-of-Light analysis (paper Sec. 4.1, four steps) ------------------ */

typedef enum ucl_op_kind { UCL_OP_GEMM = 0, UCL_OP_BATCHED_GEMM = 1, UCL_OP_GROUPED_GEMM = 2,
                           UCL_OP_CONV2D_FPROP = 3, UCL_OP_CONV2D_DGRAD = 4, UCL_OP_CONV2D_WGRAD = 5 } ucl_op_kind;

/* Which extent of a GEMM operand is contiguous in memory (`.with_layout`): A RowMajor and
 * B ColumnMajor are contiguous along K, A ColumnMajor and B RowMajor along M / N. */
typedef enum ucl_operand_layout { UCL_LAYOUT_K_CONTIGUOUS = 0, UCL_LAYOUT_MN_CONTIGUOUS = 1 } ucl_operand_layout;

/* Problem characterisation input.  GEMM family: batch (1 for gemm), M, N, K;
 * grouped: groups and M_g (HOST), N, K.  Conv (fprop, dgrad, wgrad alike): N,H,W,C,Kout,R,S
 * and pads, strides, dilations of the forward convolution.  dt_in / dt_out are ucl_dtype.  The epilogue matters
 * only through the bytes of its tensor operands (each read or written once).
 * a_layout / b_layout (ucl_operand_layout, GEMM family only) do not change the
 * SOL figures; ucl_select_tuning needs them because the kernels built for an
 * operand depend on its layout. */
typedef struct ucl_problem {
    int32_t op;                 /* ucl_op_kind */
    int32_t dt_in, dt_out;
    int32_t groups;
    int64_t batch, M, N, K;
    const int64_t *M_g;         /* HOST, grouped only */
    int64_t cN, cH, cW, cC, cKout, cR, cS;
    int64_t pad_h, pad_w, stride_h, stride_w, dil_h, dil_w;
    const ucl_epilogue *epi;    /* may be NULL; pointers inside are not dereferenced */
    int32_t a_layout, b_layout; /* ucl_operand_layout */
} ucl_problem;

/* Hardware limits: published peaks at maximum clocks, scaled linearly by the
 * ratio current / maximum clock, as the paper's report does.  NULL selects
 * MI355X: 2516.6 TFLOP/s dense bf16 / fp16 MFMA (256 CUs x 2.4 GHz x 4096
 * FLOP/clk), 8.0 TB/s HBM3E, ratios 1. */
typedef struct ucl_hw {
    double peak_flops_16bit;    /* FLOP/s, dense, bf16 / fp16 inputs */
    double peak_flops_f32;      /* FLOP/s, fp32 inputs (unused by the built kernels) */
    double peak_bw;             /* B/s */
    double compute_clock_ratio; /* (0,1] */
    double memory_clock_ratio;  /* (0,1] */
    double peak_flops_8bit;     /* FLOP/s, dense, fp8 inputs (MI355X: 5033.2 TFLOP/s) */
} ucl_hw;

typedef struct ucl_sol_report {
    double flops;               /* 2 per multiply-accumulate; epilogue not counted        */
    double bytes;               /* every unique input element read once, every output written once */
    double peak_flops, peak_bw; /* clock-scaled                                           */
    double ai, ridge;           /* FLOP/byte                                              */
    double t_compute, t_mem, t_sol; /* seconds; t_sol = max(t_compute, t_mem)             */
    int32_t compute_bound;      /* 1 if ai >= ridge, else memory-bound                    */
    int32_t reserved;
} ucl_sol_report;

/* HOST only; touches no device.  Returns UCL_ERR_INVALID_ARG on a malformed problem. */
ucl_status ucl_sol_bound(const ucl_problem *p, const ucl_hw *hw, ucl_sol_report *out);

/* ---- Introspection (HOST only; used by tests and the benchmark) ------------ */

/* The tuning the selection table would pick for a problem: the launch path with
 * tune == NULL applies the same function to the same description (packed
 * operands assumed: leading strides equal to the contiguous extents).  A launch
 * that asks for split-K without naming a tile chooses its tile for the split
 * launch instead; ucl_workspace_size() follows that choice. */
ucl_status ucl_select_tuning(const ucl_problem *p, ucl_tuning *out);

/* Bytes of workspace a call on problem p with tuning `tune` needs (0 without a split):
 * UCL_WORKSPACE_COUNTER_BYTES + slices x tiles x tile_m x tile_n x 4.  *slices_out (may be NULL)
 * receives the number of K slices the call will use.  With the STREAM_K scheduler:
 * UCL_WORKSPACE_COUNTER_BYTES + workgroups x 2 x tile_m x tile_n x 4, *slices_out = the largest
 * number of parts a tile can fall into; the number of workgroups follows from how many of them a
 * CU holds, which is asked of the HIP runtime (this one query needs a device to be present). */
ucl_status ucl_workspace_size(const ucl_problem *p, const ucl_tuning *tune, int64_t *bytes, int32_t *slices_out);

/* Zero the counter area at the start of a split-K workspace (one small kernel on `stream`; no
 * memset node, so the call may be captured into a HIP graph).  Needed once per workspace. */
ucl_status ucl_workspace_init(void *workspace, int64_t workspace_bytes, void *stream);

/* The tile schedule, evaluated on the host with the same code the kernels run:
 * for workgroup id `wg` of a launch covering `groups` sub-problems with
 * tiles_m[g] x tiles_n tiles each (batched: every entry equal), return the
 * sub-problem index and tile coordinates it processes.  total = sum of
 * tiles_m[g] * tiles_n must be > wg >= 0. */
ucl_status ucl_tile_map(int32_t groups, const int32_t *tiles_m, int32_t tiles_n, int32_t raster,
                        int32_t wg, int32_t *group, int32_t *tile_m, int32_t *tile_n);

/* The kernel variants built in.  An explicit ucl_tuning must name the (tile_m,
 * tile_n, tile_k, stages[, iterator]) of a variant built for the call's operation,
 * input type and operand layouts. */
typedef struct ucl_variant_info {
    int32_t tile_m, tile_n, tile_k, stages;
    int32_t iterator;           /* ucl_conv_iterator (conv variants), else 0 */
    int32_t op_class;           /* 0 gemm + batched_gemm, 1 grouped_gemm, 2 conv2d_fprop, 3 conv2d_dgrad, 4 conv2d_wgrad */
    int32_t dt_in;              /* ucl_dtype of both inputs */
    int32_t a_layout, b_layout; /* ucl_operand_layout the variant serves (conv: 0) */
    int32_t a_path, b_path;     /* how the operand reaches LDS: 0 direct 128-bit copies of K-contiguous rows,
                                   1 through registers with a transposing write (fallback for matrices beyond the
                                   reach of 32-bit offsets), 2 per-tap gather (conv), 3 resident patch (conv),
                                   4 / 5 direct copies of rows contiguous along N / M, read back transposed */
    int32_t lds_bytes;          /* LDS a workgroup of the variant occupies */
    int32_t scheduler;          /* ucl_tile_scheduler the variant is built for */
    int32_t patch_channels;     /* resident-patch variants: channels per pixel they are built for (fprop: C, dgrad: Kout), else 0 */
} ucl_variant_info;
int32_t ucl_num_variants(void);
ucl_status ucl_variant(int32_t i, ucl_variant_info *out);

const char *ucl_status_string(ucl_status s);
const char *ucl_last_error(void);   /* thread-local; valid until the next call on this thread */
const char *ucl_version(void);

#ifdef __cplusplus
}
#endif
#endif /* UCL_H_ */
