/* CPU oracle for the dense-layer arithmetic of the packed iteration.
 *
 * TEST INFRASTRUCTURE ONLY: plain, slow, written from the definitions; shares
 * no code with the HIP library and is never on the product path.
 *
 * The paper (Salus, arXiv 1902.04610) runs the framework's own kernels and
 * fixes no arithmetic; what an iteration of a co-resident job computes is set
 * by the workload: a stack of dense layers  H_{l+1} = act(H_l . W_l)  (forward
 * pass, Section 2.1), plus the backward pass and parameter update for training
 * jobs.  Every function below is the textbook definition with the sum taken
 * in double precision in ascending index order and rounded once to float.
 *
 * Matrices are row-major: X is M x K, W is K x N, Y is M x N.
 * bf16 values are passed as their 16-bit patterns.
 *
 * Pins: tests/test_oracle_dense.py (identity / zero / one-hot weights, float64
 * library matmul, hand-computed bf16 roundings, finite differences for the
 * training step).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ACT_NONE = 0, ACT_RELU = 1, ACT_GELU = 2 };

static double activate(double z, int act)
{
    if (act == ACT_RELU) return z > 0.0 ? z : 0.0;
    if (act == ACT_GELU) return 0.5 * z * (1.0 + erf(z / sqrt(2.0)));   /* exact erf form */
    return z;
}

/* bfloat16 = upper 16 bits of an IEEE float; conversion rounds to nearest, ties to even. */
uint16_t orc_bf16_from_f32(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u); /* NaN stays NaN */
    uint32_t lower = u & 0xffffu, keep = u >> 16;
    if (lower > 0x8000u || (lower == 0x8000u && (keep & 1u))) keep += 1u;
    return (uint16_t)keep;
}

float orc_f32_from_bf16(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

void orc_round_bf16(const float *in, uint16_t *out, int64_t n)
{
    for (int64_t i = 0; i < n; ++i) out[i] = orc_bf16_from_f32(in[i]);
}

/* Y = act(X . W), float inputs. */
void orc_dense_f32(const float *X, const float *W, float *Y,
                   int64_t M, int64_t K, int64_t N, int act)
{
    double *acc = (double *)malloc((size_t)N * sizeof(double));
    for (int64_t m = 0; m < M; ++m) {
        for (int64_t n = 0; n < N; ++n) acc[n] = 0.0;
        for (int64_t k = 0; k < K; ++k) {
            double x = (double)X[m * K + k];
            for (int64_t n = 0; n < N; ++n) acc[n] += x * (double)W[k * N + n];
        }
        for (int64_t n = 0; n < N; ++n) Y[m * N + n] = (float)activate(acc[n], act);
    }
    free(acc);
}

/* Y = act(X . W), bf16 inputs, float output. */
void orc_dense_bf16(const uint16_t *X, const uint16_t *W, float *Y,
                    int64_t M, int64_t K, int64_t N, int act)
{
    double *acc = (double *)malloc((size_t)N * sizeof(double));
    for (int64_t m = 0; m < M; ++m) {
        for (int64_t n = 0; n < N; ++n) acc[n] = 0.0;
        for (int64_t k = 0; k < K; ++k) {
            double x = (double)orc_f32_from_bf16(X[m * K + k]);
            for (int64_t n = 0; n < N; ++n)
                acc[n] += x * (double)orc_f32_from_bf16(W[k * N + n]);
        }
        for (int64_t n = 0; n < N; ++n) Y[m * N + n] = (float)activate(acc[n], act);
    }
    free(acc);
}

/* dX = dY . W^T : dY is M x N, W is K x N, dX is M x K (bf16 inputs). */
void orc_dense_bwd_input_bf16(const uint16_t *dY, const uint16_t *W, float *dX,
                              int64_t M, int64_t K, int64_t N)
{
    for (int64_t m = 0; m < M; ++m)
        for (int64_t k = 0; k < K; ++k) {
            double s = 0.0;
            for (int64_t n = 0; n < N; ++n)
                s += (double)orc_f32_from_bf16(dY[m * N + n]) *
                     (double)orc_f32_from_bf16(W[k * N + n]);
            dX[m * K + k] = (float)s;
        }
}

/* dW = H^T . dY : H is M x K, dY is M x N, dW is K x N (bf16 inputs). */
void orc_dense_bwd_weight_bf16(const uint16_t *H, const uint16_t *dY, float *dW,
                               int64_t M, int64_t K, int64_t N)
{
    for (int64_t k = 0; k < K; ++k)
        for (int64_t n = 0; n < N; ++n) {
            double s = 0.0;
            for (int64_t m = 0; m < M; ++m)
                s += (double)orc_f32_from_bf16(H[m * K + k]) *
                     (double)orc_f32_from_bf16(dY[m * N + n]);
            dW[k * N + n] = (float)s;
        }
}

/* Mean softmax cross-entropy over M rows of N logits and its gradient
 * dlogits[m][n] = (softmax(z_m)[n] - [n == label_m]) / M. Returns the loss. */
double orc_softmax_xent(const float *logits, const int32_t *labels, float *dlogits,
                        int64_t M, int64_t N)
{
    double loss = 0.0;
    for (int64_t m = 0; m < M; ++m) {
        const float *z = logits + m * N;
        double zmax = z[0];
        for (int64_t n = 1; n < N; ++n) if (z[n] > zmax) zmax = z[n];
        double denom = 0.0;
        for (int64_t n = 0; n < N; ++n) denom += exp((double)z[n] - zmax);
        loss += -((double)z[labels[m]] - zmax - log(denom));
        for (int64_t n = 0; n < N; ++n) {
            double p = exp((double)z[n] - zmax) / denom;
            dlogits[m * N + n] = (float)((p - (n == labels[m] ? 1.0 : 0.0)) / (double)M);
        }
    }
    return loss / (double)M;
}

/* Plain SGD on float master weights, then the bf16 working copy is re-derived:
 * Wm <- Wm - lr * dW  (one float multiply, one float subtract), Wb <- bf16(Wm). */
void orc_sgd_update(float *Wm, uint16_t *Wb, const float *dW, float lr, int64_t n)
{
    for (int64_t i = 0; i < n; ++i) {
        volatile float step = lr * dW[i];   /* keep the product rounded to float: no fused multiply-add */
        Wm[i] = Wm[i] - step;
        Wb[i] = orc_bf16_from_f32(Wm[i]);
    }
}
