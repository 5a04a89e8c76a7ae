/*
 * ffn_oracle.c -- TEST INFRASTRUCTURE ONLY.  Slow, plain fp64 CPU definition of the
 * operator chain the fused kernel evaluates.  Only tests, the smoke check and the
 * cpu_baseline leg of the benchmark may load this file; the product path never does.
 * It shares no code, header, table or helper with the HIP library.
 *
 * What is computed (paper: Background, Fig. "three common GEMM chains" (b)/(c);
 * Sec. 4.1 tile-graph description of the standard and the gated FFN):
 *
 *   standard : Y[i][j] = sum_n act( sum_k X[i][k] * W1[k][n] ) * W2[n][j]
 *   gated    : Y[i][j] = sum_n act( sum_k X[i][k] * W1[k][n] )
 *                              * ( sum_k X[i][k] * W3[k][n] ) * W2[n][j]
 *
 * The activation is applied to COMPLETE sums over k only (paper Sec. 4.3, pruning
 * Rule 3: partial sums must never reach the activation).
 *
 * All tensors row-major and contiguous: X[M][K], W1/W3[K][N1], W2[N1][N2].
 * Inputs are the already-rounded operand bit patterns (bf16 / fp16 / fp32); each element
 * is widened EXACTLY to double and all arithmetic is double.  Nothing is rounded between
 * the two products; the output stays double.
 *
 * Loop order is the definition written out: for each requested row, k then n for the
 * first product, n then j for the second.  Rows are independent and are spread over
 * OpenMP threads; there is no tiling, no BLAS, no reassociation inside a row.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORC_BF16 = 0, ORC_F16 = 1, ORC_F32 = 2 };
enum { ORC_IDENTITY = 0, ORC_RELU = 1, ORC_GELU_TANH = 2, ORC_SILU = 3 };

/* ---- exact widening of the three operand formats to double ------------------------ */

static inline double widen_bf16(uint16_t b) {
    /* bf16 is the upper half of an IEEE binary32 */
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}

static inline double widen_f16(uint16_t h) {
    /* IEEE binary16: 1 sign, 5 exponent (bias 15), 10 fraction */
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1f;
    int m = h & 0x3ff;
    double v;
    if (e == 0)
        v = ldexp((double)m, -24); /* zero and subnormals: m * 2^-10 * 2^-14 */
    else if (e == 31)
        v = m ? NAN : INFINITY;
    else
        v = ldexp((double)(m | 0x400), e - 25); /* (1 + m/1024) * 2^(e-15) */
    return sign ? -v : v;
}

static inline double load_elem(const void* p, int dtype, int64_t idx) {
    switch (dtype) {
        case ORC_BF16: return widen_bf16(((const uint16_t*)p)[idx]);
        case ORC_F16: return widen_f16(((const uint16_t*)p)[idx]);
        default: return (double)((const float*)p)[idx];
    }
}

/* ---- activations (the paper names only SiLU for the gated branch; ReLU and the tanh
 *      form of GELU are the workloads' choice; IDENTITY exists for closed-form tests) -- */

double orc_act(int act, double x) {
    switch (act) {
        case ORC_RELU: return x > 0.0 ? x : 0.0;
        case ORC_GELU_TANH: {
            const double c = 0.79788456080286535588; /* sqrt(2/pi) */
            return 0.5 * x * (1.0 + tanh(c * (x + 0.044715 * x * x * x)));
        }
        case ORC_SILU: return x / (1.0 + exp(-x));
        default: return x;
    }
}

/* ---- widening entry point (so a test can pin the conversions on their own) -------- */

void orc_widen(const void* src, int dtype, int64_t n, double* dst) {
    for (int64_t i = 0; i < n; ++i) dst[i] = load_elem(src, dtype, i);
}

/* ---- the chain itself ------------------------------------------------------------- */

/*
 * Computes the rows listed in rows[0..nrows) (rows == NULL means rows 0..nrows-1).
 * Y is nrows x N2 doubles, row r of Y belonging to input row rows[r].
 * If H_out != NULL it receives the activated (and gated) intermediate, nrows x N1.
 * W3 == NULL selects the standard chain.  Returns 0, or -1 on a bad argument.
 */
int orc_ffn_rows(const void* X, const void* W1, const void* W3, const void* W2, int dtype, int act,
                 int64_t M, int64_t K, int64_t N1, int64_t N2, const int64_t* rows, int64_t nrows,
                 double* Y, double* H_out) {
    if (!X || !W1 || !W2 || !Y) return -1;
    if (M < 0 || K < 0 || N1 < 0 || N2 < 0 || nrows < 0) return -1;
    if (dtype < ORC_BF16 || dtype > ORC_F32 || act < ORC_IDENTITY || act > ORC_SILU) return -1;
    for (int64_t r = 0; r < nrows; ++r) {
        int64_t i = rows ? rows[r] : r;
        if (i < 0 || i >= M) return -1;
    }
    int failed = 0;
#pragma omp parallel
    {
        double* g = (double*)malloc(sizeof(double) * (size_t)(N1 > 0 ? N1 : 1));
        double* u = (double*)malloc(sizeof(double) * (size_t)(N1 > 0 ? N1 : 1));
        if (!g || !u) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp barrier
        if (!failed) {
#pragma omp for schedule(dynamic, 1)
            for (int64_t r = 0; r < nrows; ++r) {
                const int64_t i = rows ? rows[r] : r;
                /* first product(s): complete sums over k */
                for (int64_t n = 0; n < N1; ++n) g[n] = 0.0;
                if (W3)
                    for (int64_t n = 0; n < N1; ++n) u[n] = 0.0;
                for (int64_t k = 0; k < K; ++k) {
                    const double x = load_elem(X, dtype, i * K + k);
                    for (int64_t n = 0; n < N1; ++n) g[n] += x * load_elem(W1, dtype, k * N1 + n);
                    if (W3)
                        for (int64_t n = 0; n < N1; ++n)
                            u[n] += x * load_elem(W3, dtype, k * N1 + n);
                }
                /* activation on complete sums, then the gate */
                for (int64_t n = 0; n < N1; ++n) {
                    double a = orc_act(act, g[n]);
                    if (W3) a *= u[n];
                    g[n] = a;
                }
                if (H_out)
                    for (int64_t n = 0; n < N1; ++n) H_out[r * N1 + n] = g[n];
                /* second product */
                double* y = Y + r * N2;
                for (int64_t j = 0; j < N2; ++j) y[j] = 0.0;
                for (int64_t n = 0; n < N1; ++n) {
                    const double a = g[n];
                    for (int64_t j = 0; j < N2; ++j) y[j] += a * load_elem(W2, dtype, n * N2 + j);
                }
            }
        }
        free(g);
        free(u);
    }
    return failed ? -1 : 0;
}

/* ---- convolution chains -------------------------------------------------------------
 *
 * The paper's second workload class (Evaluation, table "The configuration of conv chain":
 * IC, H, W, OC1, OC2, k1, k2): two convolutions back to back with an activation between
 * them.  As a formula, for batch b, pixel (h, w):
 *
 *   A[b][h][w][o] = act( sum_{kh<k1} sum_{kw<k1} sum_{ic<IC}
 *                        X[b][h+kh-p1][w+kw-p1][ic] * W1[kh][kw][ic][o] ),      p1 = k1/2
 *   Y[b][h][w][q] =      sum_{kh<k2} sum_{kw<k2} sum_{o<OC1}
 *                        A[b][h+kh-p2][w+kw-p2][o] * W2[kh][kw][o][q],          p2 = k2/2
 *
 * with X and A read as zero outside the image.  Readings (the paper gives only the table):
 * stride 1 and zero padding k/2, so that H x W is preserved; "convolution" is the
 * cross-correlation of deep-learning frameworks (no kernel flip); no bias; activations
 * channels-last (N H W C), weights [kh][kw][in][out].  With k1 = k2 = 1 this is exactly the
 * standard chain on the M = B*H*W pixel rows.  The activation sees complete sums over
 * (kh, kw, ic) only, as in the GEMM chain.  k1 and k2 must be odd.
 *
 * A_out (optional) receives the activated intermediate, B*H*W*OC1 doubles.
 * Returns 0, or -1 on a bad argument.
 */
static int conv_pass(const void* in_raw, const double* in_f64, int dtype, const void* Wt, int apply_act, int act,
                     int64_t B, int64_t H, int64_t W, int64_t CI, int64_t CO, int64_t k, double* out) {
    const int64_t p = k / 2;
    int failed = 0;
#pragma omp parallel
    {
        double* acc = (double*)malloc(sizeof(double) * (size_t)(CO > 0 ? CO : 1));
        if (!acc) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp barrier
        if (!failed) {
#pragma omp for schedule(dynamic, 4)
            for (int64_t pix = 0; pix < B * H * W; ++pix) {
                const int64_t b = pix / (H * W), h = (pix / W) % H, w = pix % W;
                for (int64_t o = 0; o < CO; ++o) acc[o] = 0.0;
                for (int64_t kh = 0; kh < k; ++kh) {
                    const int64_t hh = h + kh - p;
                    if (hh < 0 || hh >= H) continue; /* zero padding */
                    for (int64_t kw = 0; kw < k; ++kw) {
                        const int64_t ww = w + kw - p;
                        if (ww < 0 || ww >= W) continue;
                        const int64_t src = ((b * H + hh) * W + ww) * CI;
                        for (int64_t ci = 0; ci < CI; ++ci) {
                            const double x = in_f64 ? in_f64[src + ci] : load_elem(in_raw, dtype, src + ci);
                            const int64_t wrow = ((kh * k + kw) * CI + ci) * CO;
                            for (int64_t o = 0; o < CO; ++o) acc[o] += x * load_elem(Wt, dtype, wrow + o);
                        }
                    }
                }
                for (int64_t o = 0; o < CO; ++o) out[pix * CO + o] = apply_act ? orc_act(act, acc[o]) : acc[o];
            }
        }
        free(acc);
    }
    return failed ? -1 : 0;
}

int orc_conv_chain(const void* X, const void* W1, const void* W2, int dtype, int act, int64_t B, int64_t H,
                   int64_t W, int64_t IC, int64_t OC1, int64_t OC2, int64_t k1, int64_t k2, double* Y,
                   double* A_out) {
    if (!X || !W1 || !W2 || !Y) return -1;
    if (B < 0 || H < 0 || W < 0 || IC < 0 || OC1 < 0 || OC2 < 0) return -1;
    if (k1 < 1 || k2 < 1 || !(k1 & 1) || !(k2 & 1)) return -1;
    if (dtype < ORC_BF16 || dtype > ORC_F32 || act < ORC_IDENTITY || act > ORC_SILU) return -1;
    const int64_t npix = B * H * W;
    double* A = A_out ? A_out : (double*)malloc(sizeof(double) * (size_t)(npix * OC1 > 0 ? npix * OC1 : 1));
    if (!A) return -1;
    int rc = conv_pass(X, NULL, dtype, W1, 1, act, B, H, W, IC, OC1, k1, A);
    if (rc == 0) rc = conv_pass(NULL, A, dtype, W2, 0, act, B, H, W, OC1, OC2, k2, Y);
    if (!A_out) free(A);
    return rc;
}

int orc_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
