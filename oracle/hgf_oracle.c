/*
 * CPU oracle for the HGF linear layer -- TEST INFRASTRUCTURE, not the product.
 *
 * A plain, slow, obviously-correct implementation of Algorithm 1 ("HGF 1.0
 * Forward Pass, Inference Mode") of the Hybrid Gated Flow paper, written so that
 * each function can be checked against the paper by eye.  It shares no code,
 * layout, table or helper with the HIP library and is only ever called from the
 * tests, the smoke check and the benchmark's CPU-baseline leg.
 *
 * Readings taken where the paper's equations leave a detail open (all follow the
 * paper's appendix implementation, which is the one unambiguous statement):
 *   - the weight scale is the MEAN of |W| over the whole matrix (the definition in
 *     Sec. 2.2 is titled "absmax" but its equation is the mean), clamped to >= 1e-5;
 *   - Round() is round-half-to-even;
 *   - both quantisers form one correctly-rounded fp32 reciprocal scale
 *     (1/gamma_W, 127/gamma_x) and multiply every element by it in fp32;
 *   - gamma_x is clamped to >= 1e-5 so an all-zero token quantises to zeros.
 *
 * Every function is pinned by tests/test_oracle_pins.py against closed forms,
 * brute-force dense products and the values the paper prints.
 *
 * Build: gcc -O2 -fopenmp -ffp-contract=off -fPIC -shared hgf_oracle.c -lm
 */
#include <math.h>
#include <stdint.h>
#include <stddef.h>

/* Sec. 2.2, Def. "Absmax Quantization" (equations for gamma_W and W~):
 *   gamma_W = (1/(N K)) sum |W_ij|,  T = Clip(Round(W / gamma_W), -1, 1).
 * The sum is taken in fp64 and rounded once to fp32. */
void hgf_oracle_ternarize(const float *W, long N, long K, int8_t *T, float *gamma_w)
{
    double sum = 0.0;
    for (long i = 0; i < N * K; ++i)
        sum += fabs((double)W[i]);
    float gamma = (N * K > 0) ? (float)(sum / (double)(N * K)) : 0.0f;
    if (gamma < 1e-5f)
        gamma = 1e-5f;
    const float inv = 1.0f / gamma;
    for (long i = 0; i < N * K; ++i) {
        float q = rintf(W[i] * inv);          /* round-half-to-even in the default mode */
        if (q > 1.0f) q = 1.0f;
        if (q < -1.0f) q = -1.0f;
        T[i] = (int8_t)q;
    }
    *gamma_w = gamma;
}

/* Sec. 2.2.1, Def. "Dynamic Activation Quantization"; Algorithm 1, steps 1-2:
 *   gamma_x[m] = max_k |X[m,k]|,
 *   X~[m,k]    = Clip(Round(X[m,k] / gamma_x[m] * 127), -127, 127).
 * x holds the fp16 activations converted exactly to fp32.  s_x[m] = gamma_x[m]/127
 * is the per-token factor of the dequantisation in step 4. */
void hgf_oracle_quantize_act(const float *x, long M, long K, int8_t *xq, float *s_x,
                             int32_t *rowsum)
{
    for (long m = 0; m < M; ++m) {
        float amax = 0.0f;
        for (long k = 0; k < K; ++k) {
            float a = fabsf(x[m * K + k]);
            if (a > amax) amax = a;
        }
        if (amax < 1e-5f)
            amax = 1e-5f;
        const float inv = 127.0f / amax;
        int32_t sum = 0;
        for (long k = 0; k < K; ++k) {
            float q = rintf(x[m * K + k] * inv);
            if (q > 127.0f) q = 127.0f;
            if (q < -127.0f) q = -127.0f;
            xq[m * K + k] = (int8_t)q;
            sum += (int32_t)q;
        }
        s_x[m] = amax / 127.0f;
        if (rowsum)
            rowsum[m] = sum;
    }
}

/* Algorithm 1, step 3: Y_int = GEMM_Int8(X~, W~^T), exact in int32.
 * Written the way the proof of the "Complexity Reduction" theorem (Sec. 2.2.2)
 * states a ternary product: w = +1 adds x, w = -1 subtracts x, w = 0 skips. */
void hgf_oracle_int_gemm(const int8_t *T, const int8_t *xq, long M, long N, long K,
                         int32_t *acc)
{
#pragma omp parallel for schedule(static)
    for (long n = 0; n < N; ++n) {
        for (long m = 0; m < M; ++m) {
            int32_t s = 0;
            for (long k = 0; k < K; ++k) {
                int8_t w = T[n * K + k];
                if (w == 1)
                    s += xq[m * K + k];
                else if (w == -1)
                    s -= xq[m * K + k];
            }
            acc[m * N + n] = s;
        }
    }
}

/* Algorithm 1, steps 4-8, in fp64:
 *   step 4  Y_tern = Y_int * (gamma_x (x) gamma_W / 127)      = acc * (s_x[m] * s_w)
 *   step 5  H = X A          (the UN-quantised fp16 X; A stored [r, K] row-major)
 *   step 6  H = SiLU(H)      SiLU(h) = h * sigmoid(h)          (Sec. 2.3, Def. "Low-Rank Correction")
 *   step 7  Y_corr = H B     (B stored [N, r] row-major)
 *   step 8  Y = Y_tern + tanh(alpha) * Y_corr                  (Sec. 2.3.1, Def. "Gated Fusion")
 * alpha is one gate parameter per output channel (a scalar gate is the
 * constant vector).  rank may be 0: then Y = Y_tern.
 * y_tern_out / y_corr_out (nullable) return the two paths separately. */
void hgf_oracle_epilogue(const float *x, const int32_t *acc, const float *s_x, float s_w,
                         const float *A, const float *B, const float *alpha,
                         long M, long N, long K, long r,
                         double *y, double *y_tern_out, double *y_corr_out)
{
#pragma omp parallel for schedule(static)
    for (long m = 0; m < M; ++m) {
        double h[1024];                       /* r <= 1024 checked by the caller */
        for (long j = 0; j < r; ++j) {
            double s = 0.0;
            for (long k = 0; k < K; ++k)
                s += (double)A[j * K + k] * (double)x[m * K + k];
            h[j] = s / (1.0 + exp(-s));       /* s * sigmoid(s) */
        }
        for (long n = 0; n < N; ++n) {
            double yt = (double)acc[m * N + n] * ((double)s_x[m] * (double)s_w);
            double c = 0.0;
            for (long j = 0; j < r; ++j)
                c += (double)B[n * r + j] * h[j];
            double g = (r > 0) ? tanh((double)alpha[n]) : 0.0;
            y[m * N + n] = yt + g * c;
            if (y_tern_out) y_tern_out[m * N + n] = yt;
            if (y_corr_out) y_corr_out[m * N + n] = c;
        }
    }
}

/* The gated product of the paper's MLP (appendix implementation, block forward:
 * x + w3(SiLU(w1(n2 x)) * w2(n2 x))): elementwise z = SiLU(y_gate) * y_up with
 * SiLU(v) = v * sigmoid(v) (Sec. 2.3, Def. "Low-Rank Correction", states the activation),
 * in fp64 on the two layers' un-rounded outputs. */
void hgf_oracle_swiglu(const double *y_gate, const double *y_up, long M, long N, double *z)
{
    for (long i = 0; i < M * N; ++i)
        z[i] = (y_gate[i] / (1.0 + exp(-y_gate[i]))) * y_up[i];
}

/* LayerNorm in front of the activation quantiser (appendix implementation, BitLinear forward:
 * the backbone quantises layernorm(x) in fp32 while the correction path reads x itself):
 *   mu = mean_k x,  var = mean_k (x - mu)^2  (biased),  out = (x - mu) / sqrt(var + eps) * gamma + beta.
 * The two reductions are taken in fp64 and rounded once to fp32 (mu, and 1/sqrt(var + eps));
 * the elementwise part is fp32, one rounding per operation, in the order written above:
 * subtract, multiply by the reciprocal deviation, multiply by gamma, add beta.  The quantiser
 * that follows decides integers from these values, so the order is part of the definition. */
void hgf_oracle_layernorm(const float *x, long M, long K, const float *gamma, const float *beta,
                          float eps, float *out)
{
    for (long m = 0; m < M; ++m) {
        double sum = 0.0;
        for (long k = 0; k < K; ++k)
            sum += (double)x[m * K + k];
        const double mu = sum / (double)K;
        double ss = 0.0;
        for (long k = 0; k < K; ++k) {
            const double d = (double)x[m * K + k] - mu;
            ss += d * d;
        }
        const double var = ss / (double)K;
        const float mu32 = (float)mu;
        const float rstd = (float)(1.0 / sqrt(var + (double)eps));
        for (long k = 0; k < K; ++k) {
            float v = x[m * K + k] - mu32;
            v = v * rstd;
            v = v * gamma[k];
            v = v + beta[k];
            out[m * K + k] = v;
        }
    }
}
