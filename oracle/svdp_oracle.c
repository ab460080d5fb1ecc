/*
 * CPU oracle for the decode step of a ReGLU FFN gated by a low-rank sparsity
 * predictor.  THIS IS TEST INFRASTRUCTURE, NOT A PRODUCT PATH: it exists so
 * that the HIP library can be checked element by element against a plain,
 * slow, obviously correct implementation.  Only the tests, the smoke entry and
 * the benchmark's cpu_baseline leg may call it.  It shares no code with the
 * HIP library.
 *
 * Every function is the plain definition written out: scalar loops, double
 * accumulation in index order, no blocking, no fusion, no reordering.  Inputs
 * are float arrays (an exact container for both fp32 and bfloat16 storage; the
 * caller decodes bf16 bit patterns exactly), outputs are double.
 *
 * OpenMP is used only across independent output elements; each output element
 * is still one sequential sum in index order, so results do not depend on the
 * thread count.
 *
 * Pins (see tests/test_oracle_pins.py): numpy matmul / flatnonzero reductions,
 * hand-worked integer example, true-sign mask => sparse == dense (Sec. 3),
 * full rank and b = 0 => mask == gate sign, Prop. A.1 / Prop. A.2 / Lemma A.3 /
 * Cor. A.7 of the paper's App. A, union identities, degree-2 homogeneity.
 * oracle_stack_glue: closed forms for RMS normalisation (unit RMS, scale
 * invariance).
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>

/* ---- dense ReGLU FFN (paper Sec. 3, eq. 1) ---------------------------------
 * y = W_down ( ReLU(W_gate x) (.) (W_up x) ), with W_down given transposed:
 * WdT[i][:] is column i of W_down, so y = sum_i z_i * WdT[i][:]  (App. A.2's
 * rank-one decomposition of the FFN output).
 * drelu != 0 applies ReLU to the up branch as well (paper Sec. 5.1, eq. 6).
 * Wg, Wu, WdT: [D][d] row-major; x: [B][d]; y: [B][d].
 * z_out (nullable): [B][D] receives the intermediate z.                      */
void oracle_dense_ffn(int d, int D, int B, const float *Wg, const float *Wu,
                      const float *WdT, const float *x, int drelu, double *y,
                      double *z_out)
{
    double *z = (double *)malloc(sizeof(double) * (size_t)(D > 0 ? D : 1));
    for (int t = 0; t < B; ++t) {
        const float *xt = x + (size_t)t * d;
#pragma omp parallel for schedule(static)
        for (int i = 0; i < D; ++i) {
            double g = 0.0, u = 0.0;
            for (int j = 0; j < d; ++j) g += (double)Wg[(size_t)i * d + j] * (double)xt[j];
            for (int j = 0; j < d; ++j) u += (double)Wu[(size_t)i * d + j] * (double)xt[j];
            double gp = g > 0.0 ? g : 0.0;
            if (drelu) u = u > 0.0 ? u : 0.0;
            z[i] = gp * u;
        }
        if (z_out)
            for (int i = 0; i < D; ++i) z_out[(size_t)t * D + i] = z[i];
#pragma omp parallel for schedule(static)
        for (int j = 0; j < d; ++j) {
            double acc = 0.0;
            for (int i = 0; i < D; ++i) acc += z[i] * (double)WdT[(size_t)i * d + j];
            y[(size_t)t * d + j] = acc;
        }
    }
    free(z);
}

/* ---- predictor scores (paper Sec. 4.1, eq. 2, before the step function) -----
 * s = (x P) Q^T + b, with P [d][r] and Q [D][r] row-major (P = B^T, Q = A in
 * the paper's notation A B x + b).  The rank-r intermediate t = x P is kept in
 * double, not rounded.  x: [B][d]; s: [B][D].                                  */
void oracle_predict(int d, int D, int r, int B, const float *P, const float *Q,
                    const float *b, const float *x, double *s)
{
    double *tv = (double *)malloc(sizeof(double) * (size_t)(r > 0 ? r : 1));
    for (int t = 0; t < B; ++t) {
        const float *xt = x + (size_t)t * d;
        for (int k = 0; k < r; ++k) {
            double acc = 0.0;
            for (int j = 0; j < d; ++j) acc += (double)xt[j] * (double)P[(size_t)j * r + k];
            tv[k] = acc;
        }
#pragma omp parallel for schedule(static)
        for (int i = 0; i < D; ++i) {
            double acc = 0.0;
            for (int k = 0; k < r; ++k) acc += tv[k] * (double)Q[(size_t)i * r + k];
            s[(size_t)t * D + i] = acc + (double)b[i];
        }
    }
    free(tv);
}

/* ---- mask and index list (eq. 2's step function; Alg. 4's nonzero) ----------
 * m_i = 1 iff s_i > 0 strictly (so 0, -0 and NaN give 0).  For B > 1 the mask
 * is the union over the B tokens.  idx receives the ascending list of set
 * neurons; the return value is its length.  m: [D] bytes; idx: [D].          */
int oracle_compact(int D, int B, const double *s, uint8_t *m, int32_t *idx)
{
    int nnz = 0;
    for (int i = 0; i < D; ++i) {
        uint8_t on = 0;
        for (int t = 0; t < B; ++t)
            if (s[(size_t)t * D + i] > 0.0) on = 1;
        m[i] = on;
        if (on) idx[nnz++] = i;
    }
    return nnz;
}

/* ---- sparse ReGLU FFN over an index list (Sec. 3; Alg. 3 / Alg. 4) ----------
 * For every token of the batch, over the SAME list idx[0..nnz):
 *   y = sum_{i in idx} ReLU(Wg[i]·x) * (Wu[i]·x) * WdT[i][:]
 * Rows outside the list are never touched.  h_out (nullable): [B][nnz].       */
void oracle_sparse_ffn(int d, int D, int B, const float *Wg, const float *Wu,
                       const float *WdT, const float *x, const int32_t *idx,
                       int nnz, int drelu, double *y, double *h_out)
{
    (void)D;
    double *h = (double *)malloc(sizeof(double) * (size_t)(nnz > 0 ? nnz : 1));
    for (int t = 0; t < B; ++t) {
        const float *xt = x + (size_t)t * d;
#pragma omp parallel for schedule(static)
        for (int n = 0; n < nnz; ++n) {
            size_t i = (size_t)idx[n];
            double g = 0.0, u = 0.0;
            for (int j = 0; j < d; ++j) g += (double)Wg[i * d + j] * (double)xt[j];
            for (int j = 0; j < d; ++j) u += (double)Wu[i * d + j] * (double)xt[j];
            double gp = g > 0.0 ? g : 0.0;
            if (drelu) u = u > 0.0 ? u : 0.0;
            h[n] = gp * u;
        }
        if (h_out)
            for (int n = 0; n < nnz; ++n) h_out[(size_t)t * nnz + n] = h[n];
#pragma omp parallel for schedule(static)
        for (int j = 0; j < d; ++j) {
            double acc = 0.0;
            for (int n = 0; n < nnz; ++n) acc += h[n] * (double)WdT[(size_t)idx[n] * d + j];
            y[(size_t)t * d + j] = acc;
        }
    }
    free(h);
}

/* ---- glue between stacked layers (not from the paper: the benchmark's
 * 32-layer stack carries the residual as x + y with RMS normalisation and
 * re-centres it on the next layer's token direction) -------------------------
 * v = x + y;  out = v / sqrt(mean(v^2) + eps) + shift                          */
void oracle_stack_glue(int d, const double *x, const double *y, const double *shift,
                       double eps, double *out)
{
    double ss = 0.0;
    for (int j = 0; j < d; ++j) {
        double v = x[j] + y[j];
        ss += v * v;
    }
    double inv = 1.0 / sqrt(ss / (double)d + eps);
    for (int j = 0; j < d; ++j) out[j] = (x[j] + y[j]) * inv + shift[j];
}
