/* Direct-loop CPU oracle for the ternary convolution / inner product and its
 * straight-through backward.  TEST INFRASTRUCTURE ONLY: nothing in the GPU
 * library includes, links or calls this file.
 *
 * Forward (Eq. 2, Alg. 1 step 8):  Z = X * (alpha W~), cross-correlation
 *   Z[n,p,q,o] = alpha * sum_{r,s,c} X[n, p*sh-ph+r*dh, q*sw-pw+s*dw, c] * W~[o,c,r,s]
 * and the multiplication-free form (alpha X) (+) W~ of the same equation.
 * Backward (Alg. 1 steps 9-10): ordinary back-propagation with T = alpha W~ in
 * place of W; the weight gradient dL/dT is handed to the float32 master weights
 * unchanged.
 *
 * Activations are NHWC float32 (bf16-valued inputs are widened exactly by the
 * caller), codes are int8 in [O][C][R][S] order, all accumulation is double,
 * outputs are double.  No blocking, no reordering: one plain loop nest per
 * output element.
 */
#include <stdint.h>
#include <stddef.h>

typedef struct {
    int32_t N, H, W, C;      /* input  NHWC */
    int32_t O, R, S;         /* filters [O][C][R][S] */
    int32_t sh, sw, ph, pw, dh, dw;
    int32_t P, Q;            /* output spatial size (given by the caller) */
} oracle_conv;

static double fwd_one(const oracle_conv* g, const float* X, const int8_t* code,
                      int n, int p, int q, int o)
{
    double acc = 0.0;
    for (int r = 0; r < g->R; ++r) {
        int ih = p * g->sh - g->ph + r * g->dh;
        if (ih < 0 || ih >= g->H) continue;
        for (int s = 0; s < g->S; ++s) {
            int iw = q * g->sw - g->pw + s * g->dw;
            if (iw < 0 || iw >= g->W) continue;
            const float* x = X + (((size_t)n * g->H + ih) * g->W + iw) * g->C;
            for (int c = 0; c < g->C; ++c) {
                int t = code[(((size_t)o * g->C + c) * g->R + r) * g->S + s];
                acc += (double)x[c] * (double)t;
            }
        }
    }
    return acc;
}

/* Full forward.  Y[n,p,q,o] = alpha * acc (+ bias[o] when bias != NULL). */
void twn_oracle_conv2d_fwd(const oracle_conv* g, const float* X, const int8_t* code,
                           const double* alpha_per_o, const double* bias, double* Y)
{
    long long total = (long long)g->N * g->P * g->Q;
#pragma omp parallel for schedule(static)
    for (long long pix = 0; pix < total; ++pix) {
        int q = (int)(pix % g->Q);
        int p = (int)((pix / g->Q) % g->P);
        int n = (int)(pix / ((long long)g->Q * g->P));
        for (int o = 0; o < g->O; ++o) {
            double v = alpha_per_o[o] * fwd_one(g, X, code, n, p, q, o);
            if (bias) v += bias[o];
            Y[pix * g->O + o] = v;
        }
    }
}

/* Forward without multiplications inside the sum: the (+) of Eq. 2.
 * Inputs with code +1 are added, inputs with code -1 are subtracted, zeros are
 * skipped; alpha scales the result once. */
void twn_oracle_conv2d_fwd_addsub(const oracle_conv* g, const float* X, const int8_t* code,
                                  const double* alpha_per_o, double* Y)
{
    long long total = (long long)g->N * g->P * g->Q;
#pragma omp parallel for schedule(static)
    for (long long pix = 0; pix < total; ++pix) {
        int q = (int)(pix % g->Q);
        int p = (int)((pix / g->Q) % g->P);
        int n = (int)(pix / ((long long)g->Q * g->P));
        for (int o = 0; o < g->O; ++o) {
            double plus = 0.0, minus = 0.0;
            for (int r = 0; r < g->R; ++r) {
                int ih = p * g->sh - g->ph + r * g->dh;
                if (ih < 0 || ih >= g->H) continue;
                for (int s = 0; s < g->S; ++s) {
                    int iw = q * g->sw - g->pw + s * g->dw;
                    if (iw < 0 || iw >= g->W) continue;
                    const float* x = X + (((size_t)n * g->H + ih) * g->W + iw) * g->C;
                    for (int c = 0; c < g->C; ++c) {
                        int t = code[(((size_t)o * g->C + c) * g->R + r) * g->S + s];
                        if (t > 0) plus += (double)x[c];
                        else if (t < 0) minus += (double)x[c];
                    }
                }
            }
            Y[pix * g->O + o] = alpha_per_o[o] * (plus - minus);
        }
    }
}

/* Forward at selected flattened NHWC output indices. */
void twn_oracle_conv2d_fwd_at(const oracle_conv* g, const float* X, const int8_t* code,
                              const double* alpha_per_o, const double* bias,
                              const int64_t* idx, int64_t n_idx, double* out)
{
#pragma omp parallel for schedule(dynamic, 64)
    for (long long i = 0; i < (long long)n_idx; ++i) {
        int64_t f = idx[i];
        int o = (int)(f % g->O); f /= g->O;
        int q = (int)(f % g->Q); f /= g->Q;
        int p = (int)(f % g->P); f /= g->P;
        int n = (int)f;
        double v = alpha_per_o[o] * fwd_one(g, X, code, n, p, q, o);
        if (bias) v += bias[o];
        out[i] = v;
    }
}

/* dX[n,h,w,c] = sum over (o,r,s) and the output positions (p,q) that read
 * input (h,w) through tap (r,s):  alpha_o * dY[n,p,q,o] * W~[o,c,r,s]. */
static double bwd_data_one(const oracle_conv* g, const float* dY, const int8_t* code,
                           const double* alpha_per_o, int n, int h, int w, int c)
{
    double acc = 0.0;
    for (int r = 0; r < g->R; ++r) {
        int th = h + g->ph - r * g->dh;
        if (th < 0 || th % g->sh != 0) continue;
        int p = th / g->sh;
        if (p >= g->P) continue;
        for (int s = 0; s < g->S; ++s) {
            int tw = w + g->pw - s * g->dw;
            if (tw < 0 || tw % g->sw != 0) continue;
            int q = tw / g->sw;
            if (q >= g->Q) continue;
            const float* dy = dY + (((size_t)n * g->P + p) * g->Q + q) * g->O;
            for (int o = 0; o < g->O; ++o) {
                int t = code[(((size_t)o * g->C + c) * g->R + r) * g->S + s];
                acc += alpha_per_o[o] * ((double)dy[o] * (double)t);
            }
        }
    }
    return acc;
}

void twn_oracle_conv2d_bwd_data(const oracle_conv* g, const float* dY, const int8_t* code,
                                const double* alpha_per_o, double* dX)
{
    long long total = (long long)g->N * g->H * g->W;
#pragma omp parallel for schedule(static)
    for (long long pix = 0; pix < total; ++pix) {
        int w = (int)(pix % g->W);
        int h = (int)((pix / g->W) % g->H);
        int n = (int)(pix / ((long long)g->W * g->H));
        for (int c = 0; c < g->C; ++c)
            dX[pix * g->C + c] = bwd_data_one(g, dY, code, alpha_per_o, n, h, w, c);
    }
}

void twn_oracle_conv2d_bwd_data_at(const oracle_conv* g, const float* dY, const int8_t* code,
                                   const double* alpha_per_o,
                                   const int64_t* idx, int64_t n_idx, double* out)
{
#pragma omp parallel for schedule(dynamic, 64)
    for (long long i = 0; i < (long long)n_idx; ++i) {
        int64_t f = idx[i];
        int c = (int)(f % g->C); f /= g->C;
        int w = (int)(f % g->W); f /= g->W;
        int h = (int)(f % g->H); f /= g->H;
        int n = (int)f;
        out[i] = bwd_data_one(g, dY, code, alpha_per_o, n, h, w, c);
    }
}

/* dW[o,c,r,s] = sum_{n,p,q} X[n, p*sh-ph+r*dh, q*sw-pw+s*dw, c] * dY[n,p,q,o].
 * This is dL/dT; it contains neither alpha nor the codes. */
static double bwd_weight_one(const oracle_conv* g, const float* X, const float* dY,
                             int o, int c, int r, int s)
{
    double acc = 0.0;
    for (int n = 0; n < g->N; ++n)
        for (int p = 0; p < g->P; ++p) {
            int ih = p * g->sh - g->ph + r * g->dh;
            if (ih < 0 || ih >= g->H) continue;
            for (int q = 0; q < g->Q; ++q) {
                int iw = q * g->sw - g->pw + s * g->dw;
                if (iw < 0 || iw >= g->W) continue;
                acc += (double)X[(((size_t)n * g->H + ih) * g->W + iw) * g->C + c]
                     * (double)dY[(((size_t)n * g->P + p) * g->Q + q) * g->O + o];
            }
        }
    return acc;
}

void twn_oracle_conv2d_bwd_weight(const oracle_conv* g, const float* X, const float* dY,
                                  double* dW)
{
    long long total = (long long)g->O * g->C * g->R * g->S;
#pragma omp parallel for schedule(static)
    for (long long i = 0; i < total; ++i) {
        long long f = i;
        int s = (int)(f % g->S); f /= g->S;
        int r = (int)(f % g->R); f /= g->R;
        int c = (int)(f % g->C); f /= g->C;
        int o = (int)f;
        dW[i] = bwd_weight_one(g, X, dY, o, c, r, s);
    }
}

void twn_oracle_conv2d_bwd_weight_at(const oracle_conv* g, const float* X, const float* dY,
                                     const int64_t* idx, int64_t n_idx, double* out)
{
#pragma omp parallel for schedule(dynamic, 4)
    for (long long i = 0; i < (long long)n_idx; ++i) {
        int64_t f = idx[i];
        int s = (int)(f % g->S); f /= g->S;
        int r = (int)(f % g->R); f /= g->R;
        int c = (int)(f % g->C); f /= g->C;
        int o = (int)f;
        out[i] = bwd_weight_one(g, X, dY, o, c, r, s);
    }
}

/* Inner product (the other meaning of * in Eq. 2):
 * Y[m,j] = alpha_j * sum_k X[m,k] * W~[j,k]  (+ bias[j]). */
void twn_oracle_gemm_fwd(const float* X, const int8_t* code, const double* alpha_per_row,
                         const double* bias, int64_t M, int64_t Nn, int64_t K, double* Y)
{
#pragma omp parallel for schedule(static)
    for (long long m = 0; m < (long long)M; ++m)
        for (long long j = 0; j < (long long)Nn; ++j) {
            double acc = 0.0;
            for (long long k = 0; k < (long long)K; ++k)
                acc += (double)X[m * K + k] * (double)code[j * K + k];
            double v = alpha_per_row[j] * acc;
            if (bias) v += bias[j];
            Y[m * Nn + j] = v;
        }
}

void twn_oracle_gemm_fwd_at(const float* X, const int8_t* code, const double* alpha_per_row,
                            const double* bias, int64_t M, int64_t Nn, int64_t K,
                            const int64_t* idx, int64_t n_idx, double* out)
{
    (void)M;
#pragma omp parallel for schedule(dynamic, 64)
    for (long long i = 0; i < (long long)n_idx; ++i) {
        long long m = idx[i] / Nn, j = idx[i] % Nn;
        double acc = 0.0;
        for (long long k = 0; k < (long long)K; ++k)
            acc += (double)X[m * K + k] * (double)code[j * K + k];
        double v = alpha_per_row[j] * acc;
        if (bias) v += bias[j];
        out[i] = v;
    }
}

int twn_oracle_max_threads(void)
{
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    return omp_get_max_threads();
#else
    return 1;
#endif
}
