/*
 * ucl_oracle.c -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * Plain, slow, fp64 CPU definitions of the operations the paper's DSL names
 * (grammar `operation`: gemm, batched_gemm, grouped_gemm, conv2d_fprop; and the
 * `>>` epilogue chain, grammar `epilogue_op`), plus the roofline arithmetic of
 * the paper's SOL analysis (Sec. 4.1, steps 1-4).  Only tests, the smoke check
 * and the CPU-baseline leg of the benchmark may call this file.  It shares no
 * code, header or table with the GPU library.
 *
 * Every operation is the textbook definition written out:
 *   GEMM      D[m,n] = E_{m,n}( sum_{k ascending} A[m,k] * B[k,n] )
 *   conv2d    y[n,p,q,ko] = E( sum_{r,s,c} x[n, p*sh-ph+r*dh, q*sw-pw+s*dw, c] * w[ko,r,s,c] )
 *             (cross-correlation, NHWC activations, KRSC filter, NPQK output,
 *              taps that fall outside the image contribute zero)
 * with E the epilogue chain applied left to right to the fp64 accumulator.
 * Inputs are the stored bit patterns (fp8 e4m3 / e5m2, bf16 / fp16 / fp32 / fp64) converted
 * exactly to double.  No blocking, no reordering; OpenMP splits output rows only.
 *
 * Pins (tests/test_oracle_*.py): closed forms (identity, all-ones, K=1 outer
 * product, delta/one-hot filters, all-ones 3x3 conv = 9C/6C/4C), the transpose
 * identity (A.B)^T = B^T.A^T through swapped strides, conv 1x1 == GEMM,
 * conv H=1 == 1-D correlation (numpy.correlate), explicit im2col x GEMM == direct
 * conv, brute-force pure-Python loops on tiny shapes, numpy fp64 matmul,
 * activation values from tests/golden/activations.txt, RNE rounding against
 * exhaustive fp16 round trips and hand-derived ties, and the SOL arithmetic
 * against the worked example the paper prints (Appendix, "Example SOL Report");
 * transpose: numpy's own transposition of the decoded array, a pure-Python index
 * loop, the involution T(T(x)) = x and rows = 1 / cols = 1 being plain copies.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>

/* ---- storage formats (oracle's own codes) -------------------------------- */
enum { ORC_E4M3 = 8, ORC_E5M2 = 9, ORC_BF16 = 16, ORC_F16 = 17, ORC_F32 = 32, ORC_F64 = 64 };

static double load_bf16(uint16_t h) {
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}

/* IEEE binary16: 1 sign, 5 exponent (bias 15), 10 fraction bits. */
static double load_f16(uint16_t h) {
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1f;
    int f = h & 0x3ff;
    double v;
    if (e == 0)
        v = ldexp((double)f, -24);               /* subnormal: f * 2^-10 * 2^-14 */
    else if (e == 31)
        v = f ? NAN : INFINITY;
    else
        v = ldexp(1.0 + (double)f / 1024.0, e - 15);
    return sign ? -v : v;
}

/* The two 8-bit floating-point formats of the DSL's DTYPE rule (fp8_e4m3, fp8_e5m2), in their
 * open-standard encodings.  e4m3: 1 sign, 4 exponent (bias 7), 3 fraction bits, no infinities, the
 * single NaN pattern S.1111.111, largest finite value 448.  e5m2: 1 sign, 5 exponent (bias 15),
 * 2 fraction bits, IEEE-style infinities and NaNs (binary16 cut to its top byte). */
static double load_e4m3(uint8_t b) {
    int sign = (b >> 7) & 1, e = (b >> 3) & 0xf, f = b & 7;
    double v;
    if (e == 15 && f == 7)
        v = NAN;
    else if (e == 0)
        v = ldexp((double)f, -9);                /* subnormal: f * 2^-3 * 2^-6 */
    else
        v = ldexp(1.0 + (double)f / 8.0, e - 7);
    return sign ? -v : v;
}

static double load_e5m2(uint8_t b) {
    int sign = (b >> 7) & 1, e = (b >> 2) & 0x1f, f = b & 3;
    double v;
    if (e == 31)
        v = f ? NAN : INFINITY;
    else if (e == 0)
        v = ldexp((double)f, -16);               /* subnormal: f * 2^-2 * 2^-14 */
    else
        v = ldexp(1.0 + (double)f / 4.0, e - 15);
    return sign ? -v : v;
}

/* Bytes one stored element of a format occupies (batch strides are counted in elements). */
static int elem_bytes(int dtype) {
    return dtype == ORC_F64 ? 8 : dtype == ORC_F32 ? 4 : (dtype == ORC_E4M3 || dtype == ORC_E5M2) ? 1 : 2;
}

double orc_load(const void *p, int dtype, int64_t i) {
    switch (dtype) {
    case ORC_E4M3: return load_e4m3(((const uint8_t *)p)[i]);
    case ORC_E5M2: return load_e5m2(((const uint8_t *)p)[i]);
    case ORC_BF16: return load_bf16(((const uint16_t *)p)[i]);
    case ORC_F16:  return load_f16(((const uint16_t *)p)[i]);
    case ORC_F32:  return (double)((const float *)p)[i];
    case ORC_F64:  return ((const double *)p)[i];
    }
    return NAN;
}

/* Round a double to the nearest value of a binary format with `mant` explicit
 * fraction bits, minimum normal exponent emin and maximum exponent emax, ties
 * to even, gradual underflow, overflow to infinity (IEEE 754 roundTiesToEven).
 * The scaling x/q is by a power of two, hence exact, so nearbyint (default
 * rounding mode = ties-to-even) performs the one and only rounding. */
static double round_format(double x, int mant, int emin, int emax) {
    if (x == 0.0 || isnan(x) || isinf(x)) return x;
    int e;
    frexp(x, &e);          /* |x| = f * 2^e, f in [0.5,1)  => floor(log2|x|) = e-1 */
    e -= 1;
    if (e < emin) e = emin;
    double q = ldexp(1.0, e - mant);             /* spacing of the format near x */
    double r = nearbyint(x / q) * q;
    double maxfin = ldexp(2.0 - ldexp(1.0, -mant), emax);
    if (fabs(r) > maxfin) r = copysign(INFINITY, x);
    return r;
}

double orc_round(double x, int dtype) {
    switch (dtype) {
    case ORC_BF16: return round_format(x, 7, -126, 127);
    case ORC_F16:  return round_format(x, 10, -14, 15);
    case ORC_F32:  return round_format(x, 23, -126, 127);
    default:       return x;
    }
}

void orc_round_array(const double *x, double *y, int64_t n, int dtype) {
    for (int64_t i = 0; i < n; ++i) y[i] = orc_round(x[i], dtype);
}

/* Encode an already-rounded value as the 16-bit pattern of bf16 / fp16
 * (used by the bit-exact tests). */
uint16_t orc_encode16(double x, int dtype) {
    double r = orc_round(x, dtype);
    if (dtype == ORC_BF16) {
        float f = (float)r;                      /* exact: bf16 values are floats */
        uint32_t u;
        memcpy(&u, &f, 4);
        return (uint16_t)(u >> 16);
    }
    /* fp16 */
    uint16_t s = signbit(r) ? 0x8000 : 0;
    double a = fabs(r);
    if (isnan(r)) return 0x7e00;
    if (isinf(r)) return s | 0x7c00;
    if (a == 0.0) return s;
    int e;
    double f = frexp(a, &e);                     /* a = f*2^e, f in [0.5,1) */
    e -= 1;                                      /* a = (2f)*2^e, 2f in [1,2) */
    if (e < -14) {
        return s | (uint16_t)llround(ldexp(a, 24));
    }
    uint16_t frac = (uint16_t)llround((2.0 * f - 1.0) * 1024.0);
    return s | (uint16_t)((e + 15) << 10) | frac;
}

/* ---- epilogue chain (paper grammar `epilogue_op`, Table (c)) -------------- */
enum {
    ORC_E_SCALE = 1,       /* scale(alpha)            v * p0                        */
    ORC_E_BIAS,            /* bias()                  v + vec[n]                    */
    ORC_E_AUX_LOAD,        /* aux_load(id)            v + p0 * T[m,n]  (residual)   */
    ORC_E_RELU,            /* relu()                  max(v, 0)                     */
    ORC_E_GELU_TANH,       /* gelu(), tanh form       v/2 (1 + tanh(c (v + .044715 v^3))) */
    ORC_E_GELU_ERF,        /* gelu(), erf form        v/2 (1 + erf(v / sqrt 2))     */
    ORC_E_SILU,            /* silu()                  v / (1 + e^-v)                */
    ORC_E_SIGMOID,         /* sigmoid()               1 / (1 + e^-v)                */
    ORC_E_TANH,            /* tanh()                                                */
    ORC_E_MISH,            /* mish()                  v tanh(log(1 + e^v))          */
    ORC_E_HARDSWISH,       /* hardswish()             v min(max(v + 3, 0), 6) / 6   */
    ORC_E_LEAKY_RELU,      /* leaky_relu(alpha)       v > 0 ? v : p0 v              */
    ORC_E_ELU,             /* elu(alpha)              v > 0 ? v : p0 (e^v - 1)      */
    ORC_E_CLAMP,           /* clip / clamp(min,max)   min(max(v, p0), p1)           */
    ORC_E_PER_ROW_SCALE,   /* per_row_scale()         v * vec[m]                    */
    ORC_E_PER_COL_SCALE,   /* per_col_scale(), per_channel_scale()   v * vec[n]     */
    ORC_E_ROW_BROADCAST,   /* row_broadcast(id)       v + vec[n]  (a 1xN row)       */
    ORC_E_COL_BROADCAST,   /* column_broadcast(id)    v + vec[m]  (an Mx1 column)   */
    ORC_E_AUX_STORE        /* aux_store(id)           T[m,n] = v ; v unchanged      */
};

typedef struct {
    int32_t op;
    int32_t dtype;         /* storage format of ptr                                 */
    double p0, p1;
    void *ptr;             /* vector (length N or M) or matrix with row stride ld   */
    int64_t ld;
} orc_step;

typedef struct {
    int32_t n_steps;
    int32_t pad_;
    orc_step steps[16];
} orc_chain;

static double softplus(double v) {
    /* log(1 + e^v) without overflow */
    return v > 0 ? v + log1p(exp(-v)) : log1p(exp(v));
}

/* Apply the chain to one accumulator value at output coordinate (m, n).
 * aux_store writes the value rounded to the aux tensor's format, stored as
 * double in a double-typed aux buffer (dtype says which rounding). */
double orc_epilogue(double v, int64_t m, int64_t n, const orc_chain *c) {
    if (!c) return v;
    for (int i = 0; i < c->n_steps; ++i) {
        const orc_step *s = &c->steps[i];
        switch (s->op) {
        case ORC_E_SCALE:         v = v * s->p0; break;
        case ORC_E_BIAS:
        case ORC_E_ROW_BROADCAST: v = v + orc_load(s->ptr, s->dtype, n); break;
        case ORC_E_COL_BROADCAST: v = v + orc_load(s->ptr, s->dtype, m); break;
        case ORC_E_AUX_LOAD:      v = v + s->p0 * orc_load(s->ptr, s->dtype, m * s->ld + n); break;
        case ORC_E_RELU:          v = v > 0 ? v : 0.0; break;
        case ORC_E_GELU_TANH:
            v = 0.5 * v * (1.0 + tanh(sqrt(2.0 / M_PI) * (v + 0.044715 * v * v * v)));
            break;
        case ORC_E_GELU_ERF:      v = 0.5 * v * (1.0 + erf(v / sqrt(2.0))); break;
        case ORC_E_SILU:          v = v / (1.0 + exp(-v)); break;
        case ORC_E_SIGMOID:       v = 1.0 / (1.0 + exp(-v)); break;
        case ORC_E_TANH:          v = tanh(v); break;
        case ORC_E_MISH:          v = v * tanh(softplus(v)); break;
        case ORC_E_HARDSWISH:     v = v * fmin(fmax(v + 3.0, 0.0), 6.0) / 6.0; break;
        case ORC_E_LEAKY_RELU:    v = v > 0 ? v : s->p0 * v; break;
        case ORC_E_ELU:           v = v > 0 ? v : s->p0 * expm1(v); break;
        case ORC_E_CLAMP:         v = fmin(fmax(v, s->p0), s->p1); break;
        case ORC_E_PER_ROW_SCALE: v = v * orc_load(s->ptr, s->dtype, m); break;
        case ORC_E_PER_COL_SCALE: v = v * orc_load(s->ptr, s->dtype, n); break;
        case ORC_E_AUX_STORE:
            ((double *)s->ptr)[m * s->ld + n] = orc_round(v, s->dtype);
            break;
        }
    }
    return v;
}

/* ---- GEMM family ---------------------------------------------------------- */

/* D (double, row-major, leading dimension N) for the listed output rows only:
 * rows == NULL means all rows 0..M-1 and n_rows is ignored.  Output row j of
 * Dout corresponds to problem row rows[j].  A and B are addressed with element
 * strides (row stride, column stride), so either storage order, or a
 * transposed view, is just a pair of strides.  If absacc != NULL it receives
 * sum_k |A[m,k]| |B[k,n]| (the scale of the rounding-error bound). */
void orc_gemm(int64_t M, int64_t N, int64_t K,
              const void *A, int dtA, int64_t a_rs, int64_t a_cs,
              const void *B, int dtB, int64_t b_rs, int64_t b_cs,
              const orc_chain *chain,
              const int64_t *rows, int64_t n_rows,
              double *Dout, double *absacc) {
    int64_t R = rows ? n_rows : M;
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < R; ++j) {
        int64_t m = rows ? rows[j] : j;
        for (int64_t n = 0; n < N; ++n) {
            double acc = 0.0, aacc = 0.0;
            for (int64_t k = 0; k < K; ++k) {
                double a = orc_load(A, dtA, m * a_rs + k * a_cs);
                double b = orc_load(B, dtB, k * b_rs + n * b_cs);
                acc += a * b;
                aacc += fabs(a) * fabs(b);
            }
            Dout[j * N + n] = orc_epilogue(acc, m, n, chain);
            if (absacc) absacc[j * N + n] = aacc;
        }
    }
}

/* Strided batched GEMM (grammar `batched_gemm_op`): the GEMM definition applied
 * to each batch b with operands offset by b times the batch stride (elements).
 * Tensor operands of the chain that are matrices advance by aux_bs elements per
 * batch; vectors are shared.  Dout is [batch][M][N]. */
void orc_batched_gemm(int64_t batch, int64_t M, int64_t N, int64_t K,
                      const void *A, int dtA, int64_t a_rs, int64_t a_cs, int64_t a_bs,
                      const void *B, int dtB, int64_t b_rs, int64_t b_cs, int64_t b_bs,
                      const orc_chain *chain, int64_t aux_bs,
                      double *Dout, double *absacc) {
    for (int64_t b = 0; b < batch; ++b) {
        orc_chain c;
        if (chain) {
            c = *chain;
            for (int i = 0; i < c.n_steps; ++i) {
                orc_step *s = &c.steps[i];
                if (s->op == ORC_E_AUX_LOAD) {
                    int esz = elem_bytes(s->dtype);
                    s->ptr = (char *)s->ptr + b * aux_bs * esz;
                } else if (s->op == ORC_E_AUX_STORE) {
                    s->ptr = (double *)s->ptr + b * aux_bs;
                }
            }
        }
        int esA = elem_bytes(dtA);
        int esB = elem_bytes(dtB);
        orc_gemm(M, N, K,
                 (const char *)A + b * a_bs * esA, dtA, a_rs, a_cs,
                 (const char *)B + b * b_bs * esB, dtB, b_rs, b_cs,
                 chain ? &c : NULL, NULL, 0,
                 Dout + b * M * N, absacc ? absacc + b * M * N : NULL);
    }
}

/* Grouped GEMM (grammar `grouped_gemm_op`, expert_count = groups): independent
 * problems (M_g, N, K), each with its own A_g, B_g and chain operands; results
 * packed one group after another in Dout, i.e. [sum_g M_g][N].  chains may be
 * NULL (identity epilogue) or an array of one chain per group. */
void orc_grouped_gemm(int32_t groups, const int64_t *M_g, int64_t N, int64_t K,
                      const void *const *A_g, int dtA, int64_t a_rs, int64_t a_cs,
                      const void *const *B_g, int dtB, int64_t b_rs, int64_t b_cs,
                      const orc_chain *chains,
                      double *Dout, double *absacc) {
    int64_t row0 = 0;
    for (int32_t g = 0; g < groups; ++g) {
        if (M_g[g] > 0)
            orc_gemm(M_g[g], N, K, A_g[g], dtA, a_rs, a_cs, B_g[g], dtB, b_rs, b_cs,
                     chains ? &chains[g] : NULL, NULL, 0,
                     Dout + row0 * N, absacc ? absacc + row0 * N : NULL);
        row0 += M_g[g];
    }
}

/* ---- conv2d forward (grammar `conv2d_fprop`, layouts TensorNHWC) ----------- */

int64_t orc_conv_out_dim(int64_t in, int64_t pad, int64_t dil, int64_t ker, int64_t stride) {
    return (in + 2 * pad - dil * (ker - 1) - 1) / stride + 1;
}

/* Direct convolution.  x [Nb,H,W,C], w [Ko,R,S,C], y [Nb,P,Q,Ko] as doubles.
 * The epilogue sees the output as a matrix with row index (n*P+p)*Q+q and
 * column index ko (output channel), so bias() is per output channel and
 * aux_load is a tensor shaped like y.  rows != NULL restricts the computation
 * to the listed flattened (n,p,q) positions; Dout row j <-> rows[j]. */
void orc_conv2d_fprop(int64_t Nb, int64_t H, int64_t W, int64_t C, int64_t Ko,
                      int64_t R, int64_t S,
                      int64_t pad_h, int64_t pad_w, int64_t stride_h, int64_t stride_w,
                      int64_t dil_h, int64_t dil_w,
                      const void *x, int dtX, const void *w, int dtW,
                      const orc_chain *chain,
                      const int64_t *rows, int64_t n_rows,
                      double *Dout, double *absacc) {
    int64_t P = orc_conv_out_dim(H, pad_h, dil_h, R, stride_h);
    int64_t Q = orc_conv_out_dim(W, pad_w, dil_w, S, stride_w);
    int64_t total = rows ? n_rows : Nb * P * Q;
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < total; ++j) {
        int64_t row = rows ? rows[j] : j;
        int64_t q = row % Q;
        int64_t p = (row / Q) % P;
        int64_t n = row / (Q * P);
        for (int64_t ko = 0; ko < Ko; ++ko) {
            double acc = 0.0, aacc = 0.0;
            for (int64_t r = 0; r < R; ++r) {
                int64_t h = p * stride_h - pad_h + r * dil_h;
                if (h < 0 || h >= H) continue;
                for (int64_t s = 0; s < S; ++s) {
                    int64_t ww = q * stride_w - pad_w + s * dil_w;
                    if (ww < 0 || ww >= W) continue;
                    for (int64_t c = 0; c < C; ++c) {
                        double xv = orc_load(x, dtX, ((n * H + h) * W + ww) * C + c);
                        double wv = orc_load(w, dtW, ((ko * R + r) * S + s) * C + c);
                        acc += xv * wv;
                        aacc += fabs(xv) * fabs(wv);
                    }
                }
            }
            Dout[j * Ko + ko] = orc_epilogue(acc, row, ko, chain);
            if (absacc) absacc[j * Ko + ko] = aacc;
        }
    }
}


/* Data gradient of the convolution above (grammar `conv2d_dgrad`): the adjoint of fprop with
 * respect to x.  dy [Nb,P,Q,Ko], w [Ko,R,S,C] -> dx [Nb,H,W,C],
 *   dx[n,h,w,c] = E( sum over (p,r), (q,s), ko with p*stride_h - pad_h + r*dil_h == h and
 *                    q*stride_w - pad_w + s*dil_w == w of dy[n,p,q,ko] * w[ko,r,s,c] ),
 * i.e. every product of fprop in which x[n,h,w,c] takes part, with the other factor's partner dy.
 * For a tap r the matching output row is p = (h + pad_h - r*dil_h) / stride_h when that division
 * is exact and 0 <= p < P.  The epilogue sees row index (n*H+h)*W+w and column index c. */
void orc_conv2d_dgrad(int64_t Nb, int64_t H, int64_t W, int64_t C, int64_t Ko,
                      int64_t R, int64_t S,
                      int64_t pad_h, int64_t pad_w, int64_t stride_h, int64_t stride_w,
                      int64_t dil_h, int64_t dil_w,
                      const void *dy, int dtY, const void *w, int dtW,
                      const orc_chain *chain,
                      const int64_t *rows, int64_t n_rows,
                      double *Dout, double *absacc) {
    int64_t P = orc_conv_out_dim(H, pad_h, dil_h, R, stride_h);
    int64_t Q = orc_conv_out_dim(W, pad_w, dil_w, S, stride_w);
    int64_t total = rows ? n_rows : Nb * H * W;
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < total; ++j) {
        int64_t row = rows ? rows[j] : j;
        int64_t wi = row % W;
        int64_t h = (row / W) % H;
        int64_t n = row / (W * H);
        for (int64_t c = 0; c < C; ++c) {
            double acc = 0.0, aacc = 0.0;
            for (int64_t r = 0; r < R; ++r) {
                int64_t th = h + pad_h - r * dil_h;
                if (th < 0 || th % stride_h != 0 || th / stride_h >= P) continue;
                int64_t p = th / stride_h;
                for (int64_t s2 = 0; s2 < S; ++s2) {
                    int64_t tw = wi + pad_w - s2 * dil_w;
                    if (tw < 0 || tw % stride_w != 0 || tw / stride_w >= Q) continue;
                    int64_t q = tw / stride_w;
                    for (int64_t ko = 0; ko < Ko; ++ko) {
                        double gv = orc_load(dy, dtY, ((n * P + p) * Q + q) * Ko + ko);
                        double wv = orc_load(w, dtW, ((ko * R + r) * S + s2) * C + c);
                        acc += gv * wv;
                        aacc += fabs(gv) * fabs(wv);
                    }
                }
            }
            Dout[j * C + c] = orc_epilogue(acc, row, c, chain);
            if (absacc) absacc[j * C + c] = aacc;
        }
    }
}

/* Weight gradient (grammar `conv2d_wgrad`): the adjoint of fprop with respect to w.
 * dy [Nb,P,Q,Ko], x [Nb,H,W,C] -> dw [Ko,R,S,C],
 *   dw[ko,r,s,c] = E( sum_{n,p,q} dy[n,p,q,ko] * x[n, p*stride_h - pad_h + r*dil_h,
 *                                                    q*stride_w - pad_w + s*dil_w, c] ),
 * out-of-image x = 0.  The epilogue sees dw as a Ko x (R*S*C) matrix: row ko, column (r*S+s)*C+c.
 * rows != NULL restricts the computation to the listed ko. */
void orc_conv2d_wgrad(int64_t Nb, int64_t H, int64_t W, int64_t C, int64_t Ko,
                      int64_t R, int64_t S,
                      int64_t pad_h, int64_t pad_w, int64_t stride_h, int64_t stride_w,
                      int64_t dil_h, int64_t dil_w,
                      const void *dy, int dtY, const void *x, int dtX,
                      const orc_chain *chain,
                      const int64_t *rows, int64_t n_rows,
                      double *Dout, double *absacc) {
    int64_t P = orc_conv_out_dim(H, pad_h, dil_h, R, stride_h);
    int64_t Q = orc_conv_out_dim(W, pad_w, dil_w, S, stride_w);
    int64_t total = rows ? n_rows : Ko;
    int64_t cols = R * S * C;
#pragma omp parallel for schedule(static) collapse(2)
    for (int64_t j = 0; j < total; ++j) {
        for (int64_t col = 0; col < cols; ++col) {
            int64_t ko = rows ? rows[j] : j;
            int64_t c = col % C;
            int64_t s2 = (col / C) % S;
            int64_t r = col / (C * S);
            double acc = 0.0, aacc = 0.0;
            for (int64_t n = 0; n < Nb; ++n) {
                for (int64_t p = 0; p < P; ++p) {
                    int64_t h = p * stride_h - pad_h + r * dil_h;
                    if (h < 0 || h >= H) continue;
                    for (int64_t q = 0; q < Q; ++q) {
                        int64_t ww = q * stride_w - pad_w + s2 * dil_w;
                        if (ww < 0 || ww >= W) continue;
                        double gv = orc_load(dy, dtY, ((n * P + p) * Q + q) * Ko + ko);
                        double xv = orc_load(x, dtX, ((n * H + h) * W + ww) * C + c);
                        acc += gv * xv;
                        aacc += fabs(gv) * fabs(xv);
                    }
                }
            }
            Dout[j * cols + col] = orc_epilogue(acc, ko, col, chain);
            if (absacc) absacc[j * cols + col] = aacc;
        }
    }
}

/* ---- SOL analysis (paper Sec. 4.1; Appendix "Example SOL Report") ---------- */

typedef struct {
    double flops, bytes;            /* problem characterisation                   */
    double peak_flops, peak_bw;     /* clock-scaled hardware limits               */
    double ai, ridge;               /* FLOP/byte                                  */
    double t_compute, t_mem, t_sol; /* seconds                                    */
    int32_t compute_bound;          /* 1 if ai >= ridge                           */
    int32_t pad_;
} orc_sol;

/* Transform stage of a `pipeline(...)` program (grammar `transpose_op`): per batch a rows x cols
 * matrix written transposed, dst[b][c][r] = src[b][r][c], as unrounded doubles (the caller rounds
 * to the target type with orc_round).  Three plain loops. */
void orc_transpose(int64_t batch, int64_t rows, int64_t cols, const void *src, int dtype, double *dst) {
    for (int64_t b = 0; b < batch; ++b)
        for (int64_t r = 0; r < rows; ++r)
            for (int64_t c = 0; c < cols; ++c)
                dst[(b * cols + c) * rows + r] = orc_load(src, dtype, (b * rows + r) * cols + c);
}

/* The four steps of the analysis, given work (flops, bytes) and published peaks
 * (FLOP/s and B/s at max clocks) scaled linearly by clock ratios. */
void orc_sol_bound(double flops, double bytes,
                   double peak_flops_at_max, double compute_clock_ratio,
                   double peak_bw_at_max, double mem_clock_ratio, orc_sol *out) {
    out->flops = flops;
    out->bytes = bytes;
    out->peak_flops = peak_flops_at_max * compute_clock_ratio;
    out->peak_bw = peak_bw_at_max * mem_clock_ratio;
    out->ai = flops / bytes;
    out->ridge = out->peak_flops / out->peak_bw;
    out->t_compute = flops / out->peak_flops;
    out->t_mem = bytes / out->peak_bw;
    out->t_sol = out->t_compute > out->t_mem ? out->t_compute : out->t_mem;
    out->compute_bound = out->ai >= out->ridge;
}

/* Work of a dense GEMM-shaped problem: 2 FLOPs per multiply-accumulate; every
 * unique input element read once and every output written once. */
double orc_gemm_flops(double batch, double M, double N, double K) { return 2.0 * batch * M * N * K; }
