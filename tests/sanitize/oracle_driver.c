/* Sanitizer driver for the CPU oracle (test infrastructure): every entry point of ucl_oracle.c on
 * small ragged problems, with buffers of exactly the size each call may touch, so that an access
 * past an operand or an undefined integer operation is reported by ASan / UBSan.  Exit code 0 and
 * no sanitizer report = pass.  Built and run by tests/test_sanitizers.py. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

typedef struct { int32_t op, dtype; double p0, p1; const void *ptr; int64_t ld; } step_t;
typedef struct { int32_t n_steps, pad_; step_t steps[16]; } chain_t;

double orc_load(const void *p, int dtype, int64_t i);
double orc_round(double x, int dtype);
uint16_t orc_encode16(double x, int dtype);
void orc_gemm(int64_t, int64_t, int64_t, const void *, int, int64_t, int64_t, const void *, int, int64_t, int64_t,
              const chain_t *, const int64_t *, int64_t, double *, double *);
void orc_batched_gemm(int64_t, int64_t, int64_t, int64_t, const void *, int, int64_t, int64_t, int64_t, const void *, int,
                      int64_t, int64_t, int64_t, const chain_t *, int64_t, double *, double *);
void orc_grouped_gemm(int32_t, const int64_t *, int64_t, int64_t, const void *const *, int, int64_t, int64_t,
                      const void *const *, int, int64_t, int64_t, const chain_t *, double *, double *);
void orc_conv2d_fprop(int64_t, int64_t, int64_t, int64_t, int64_t, int64_t, int64_t, int64_t, int64_t, int64_t, int64_t,
                      int64_t, int64_t, const void *, int, const void *, int, const chain_t *, const int64_t *, int64_t,
                      double *, double *);
void orc_conv2d_dgrad(int64_t, int64_t, int64_t, int64_t, int64_t, int64_t, int64_t, int64_t, int64_t, int64_t, int64_t,
                      int64_t, int64_t, const void *, int, const void *, int, const chain_t *, const int64_t *, int64_t,
                      double *, double *);
void orc_conv2d_wgrad(int64_t, int64_t, int64_t, int64_t, int64_t, int64_t, int64_t, int64_t, int64_t, int64_t, int64_t,
                      int64_t, int64_t, const void *, int, const void *, int, const chain_t *, const int64_t *, int64_t,
                      double *, double *);
void orc_transpose(int64_t, int64_t, int64_t, const void *, int, double *);
int64_t orc_conv_out_dim(int64_t, int64_t, int64_t, int64_t, int64_t);

enum { E4M3 = 8, E5M2 = 9, BF16 = 16, F16 = 17, F32 = 32 };

static uint32_t rng_state = 12345u;
static uint32_t rnd(void) { rng_state = rng_state * 1664525u + 1013904223u; return rng_state >> 8; }

/* n elements of `dtype` with small finite values, in a buffer of exactly n elements */
static void *fill(int dtype, int64_t n) {
    int es = dtype == F32 ? 4 : (dtype == E4M3 || dtype == E5M2) ? 1 : 2;
    unsigned char *p = malloc((size_t)(n * es) ? (size_t)(n * es) : 1);
    for (int64_t i = 0; i < n; ++i) {
        double v = (double)((int)(rnd() % 9) - 4) * 0.25;
        if (dtype == F32) ((float *)p)[i] = (float)v;
        else if (es == 2) ((uint16_t *)p)[i] = orc_encode16(v, dtype);
        else p[i] = (unsigned char)(dtype == E4M3 ? (rnd() % 0x78) : (rnd() % 0x7B)) | (unsigned char)((rnd() & 1) << 7);
    }
    return p;
}

int main(void) {
    int fails = 0;
    /* storage formats: every code of the narrow ones, and rounding of awkward values */
    for (int c = 0; c < 65536; ++c) { uint16_t h = (uint16_t)c; (void)orc_load(&h, F16, 0); (void)orc_load(&h, BF16, 0); }
    for (int c = 0; c < 256; ++c) { uint8_t b = (uint8_t)c; (void)orc_load(&b, E4M3, 0); (void)orc_load(&b, E5M2, 0); }
    const double odd[] = {0.0, -0.0, 1e-320, 1e-46, 6.1e-5, 65519.9, 65520.0, 3.4e38, 3.5e38, 1e308, INFINITY, -INFINITY, NAN};
    for (unsigned i = 0; i < sizeof(odd) / sizeof(odd[0]); ++i)
        for (int dt = BF16; dt <= F16; ++dt) { (void)orc_round(odd[i], dt); (void)orc_round(odd[i], F32); (void)orc_encode16(odd[i], dt); }

    /* gemm in all four layouts with a chain that touches a vector by n, a vector by m and a matrix */
    const int64_t M = 7, N = 5, K = 9;
    const int dts[] = {BF16, F16, E4M3, E5M2};
    for (int d = 0; d < 4; ++d) {
        void *A = fill(dts[d], M * K), *B = fill(dts[d], K * N);
        void *bias = fill(BF16, N), *rowv = fill(F32, M), *res = fill(F16, M * N);
        double *aux = malloc(sizeof(double) * M * N), *D = malloc(sizeof(double) * M * N), *S = malloc(sizeof(double) * M * N);
        chain_t ch; memset(&ch, 0, sizeof ch);
        ch.n_steps = 7;
        ch.steps[0] = (step_t){1, 0, 0.5, 0, NULL, 0};                /* scale */
        ch.steps[1] = (step_t){2, BF16, 0, 0, bias, 0};               /* bias */
        ch.steps[2] = (step_t){15, F32, 0, 0, rowv, 0};               /* per_row_scale */
        ch.steps[3] = (step_t){3, F16, -1.0, 0, res, N};              /* aux_load */
        ch.steps[4] = (step_t){19, BF16, 0, 0, aux, N};               /* aux_store */
        ch.steps[5] = (step_t){5, 0, 0, 0, NULL, 0};                  /* gelu_tanh */
        ch.steps[6] = (step_t){14, 0, -1.0, 1.0, NULL, 0};            /* clamp */
        for (int la = 0; la < 2; ++la)
            for (int lb = 0; lb < 2; ++lb) {
                orc_gemm(M, N, K, A, dts[d], la ? 1 : K, la ? M : 1, B, dts[d], lb ? N : 1, lb ? 1 : K, &ch, NULL, 0, D, S);
                for (int64_t i = 0; i < M * N; ++i) if (!isfinite(D[i]) || S[i] < 0) ++fails;
            }
        const int64_t rows[3] = {6, 0, 3};
        orc_gemm(M, N, K, A, dts[d], K, 1, B, dts[d], 1, K, NULL, rows, 3, D, NULL);
        free(A); free(B); free(bias); free(rowv); free(res); free(aux); free(D); free(S);
    }
    /* batched with a per-batch residual; grouped with an empty group */
    {
        const int64_t b = 3;
        void *A = fill(E5M2, b * M * K), *B = fill(E5M2, b * N * K), *res = fill(F32, b * M * N);
        double *D = malloc(sizeof(double) * b * M * N);
        chain_t ch; memset(&ch, 0, sizeof ch);
        ch.n_steps = 1; ch.steps[0] = (step_t){3, F32, 1.0, 0, res, N};
        orc_batched_gemm(b, M, N, K, A, E5M2, K, 1, M * K, B, E5M2, 1, K, N * K, &ch, M * N, D, NULL);
        orc_batched_gemm(b, M, N, K, A, E5M2, K, 1, 0, B, E5M2, 1, K, N * K, NULL, 0, D, NULL);     /* shared A */
        free(A); free(B); free(res); free(D);
        const int64_t Mg[4] = {3, 0, 5, 1};
        const void *Ap[4], *Bp[4];
        void *keep[8];
        for (int g = 0; g < 4; ++g) { keep[g] = fill(BF16, Mg[g] * K); keep[4 + g] = fill(BF16, N * K); Ap[g] = keep[g]; Bp[g] = keep[4 + g]; }
        double *Dg = malloc(sizeof(double) * 9 * N), *Sg = malloc(sizeof(double) * 9 * N);
        orc_grouped_gemm(4, Mg, N, K, Ap, BF16, K, 1, Bp, BF16, 1, K, NULL, Dg, Sg);
        for (int g = 0; g < 8; ++g) free(keep[g]);
        free(Dg); free(Sg);
    }
    /* the three convolutions on geometries with padding, stride and dilation, and a row subset */
    const int64_t geo[3][13] = {{2, 5, 6, 3, 4, 3, 3, 1, 1, 1, 1, 1, 1}, {1, 7, 5, 2, 3, 3, 2, 2, 0, 2, 1, 1, 2}, {1, 1, 9, 2, 2, 1, 5, 0, 2, 1, 3, 1, 1}};
    for (int g = 0; g < 3; ++g) {
        const int64_t *q = geo[g];
        const int64_t Nb = q[0], H = q[1], W = q[2], C = q[3], Ko = q[4], R = q[5], Sx = q[6];
        const int64_t P = orc_conv_out_dim(H, q[7], q[11], R, q[9]), Q = orc_conv_out_dim(W, q[8], q[12], Sx, q[10]);
        void *x = fill(BF16, Nb * H * W * C), *w = fill(BF16, Ko * R * Sx * C), *dy = fill(BF16, Nb * P * Q * Ko);
        double *y = malloc(sizeof(double) * Nb * P * Q * Ko), *dx = malloc(sizeof(double) * Nb * H * W * C), *dw = malloc(sizeof(double) * Ko * R * Sx * C);
        double *s1 = malloc(sizeof(double) * Nb * H * W * C);
        orc_conv2d_fprop(Nb, H, W, C, Ko, R, Sx, q[7], q[8], q[9], q[10], q[11], q[12], x, BF16, w, BF16, NULL, NULL, 0, y, NULL);
        orc_conv2d_dgrad(Nb, H, W, C, Ko, R, Sx, q[7], q[8], q[9], q[10], q[11], q[12], dy, BF16, w, BF16, NULL, NULL, 0, dx, s1);
        orc_conv2d_wgrad(Nb, H, W, C, Ko, R, Sx, q[7], q[8], q[9], q[10], q[11], q[12], dy, BF16, x, BF16, NULL, NULL, 0, dw, NULL);
        const int64_t last = Nb * P * Q - 1, rows2[2] = {last, 0}, rows3[2] = {Nb * H * W - 1, 0}, rows4[1] = {Ko - 1};
        orc_conv2d_fprop(Nb, H, W, C, Ko, R, Sx, q[7], q[8], q[9], q[10], q[11], q[12], x, BF16, w, BF16, NULL, rows2, 2, y, NULL);
        orc_conv2d_dgrad(Nb, H, W, C, Ko, R, Sx, q[7], q[8], q[9], q[10], q[11], q[12], dy, BF16, w, BF16, NULL, rows3, 2, dx, NULL);
        orc_conv2d_wgrad(Nb, H, W, C, Ko, R, Sx, q[7], q[8], q[9], q[10], q[11], q[12], dy, BF16, x, BF16, NULL, rows4, 1, dw, NULL);
        /* adjoint identity as a functional check of the run itself */
        orc_conv2d_fprop(Nb, H, W, C, Ko, R, Sx, q[7], q[8], q[9], q[10], q[11], q[12], x, BF16, w, BF16, NULL, NULL, 0, y, NULL);
        orc_conv2d_dgrad(Nb, H, W, C, Ko, R, Sx, q[7], q[8], q[9], q[10], q[11], q[12], dy, BF16, w, BF16, NULL, NULL, 0, dx, NULL);
        double lhs = 0, rhs = 0;
        for (int64_t i = 0; i < Nb * P * Q * Ko; ++i) lhs += orc_load(dy, BF16, i) * y[i];
        for (int64_t i = 0; i < Nb * H * W * C; ++i) rhs += dx[i] * orc_load(x, BF16, i);
        if (fabs(lhs - rhs) > 1e-9) { fprintf(stderr, "adjoint identity fails on geometry %d: %g vs %g\n", g, lhs, rhs); ++fails; }
        free(x); free(w); free(dy); free(y); free(dx); free(dw); free(s1);
    }
    /* transpose of a ragged batch */
    {
        void *src = fill(F16, 2 * 3 * 5);
        double *dst = malloc(sizeof(double) * 2 * 3 * 5);
        orc_transpose(2, 3, 5, src, F16, dst);
        free(src); free(dst);
    }
    if (fails) { fprintf(stderr, "%d checks failed\n", fails); return 1; }
    printf("oracle sanitizer driver: ok\n");
    return 0;
}
