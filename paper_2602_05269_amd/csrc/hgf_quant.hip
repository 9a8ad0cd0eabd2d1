// Fused per-token absmax int8 activation quantiser.
//
// Sec. 2.2.1 of the HGF paper (dynamic activation quantisation) and Algorithm 1, steps
// 1-2: gamma_x[m] = max_k |x[m,k]| and x_q = Clip(Round(x / gamma_x * 127), -127, 127).
// One fp32 reciprocal scale 127/gamma_x per token (IEEE division), one fp32 multiply and
// a round-half-to-even per element; gamma_x is clamped to >= 1e-5 so a zero token gives
// zeros.  One workgroup per token: the row is read twice (the second pass hits cache),
// the int8 row, s_x = gamma_x/127 and sum_k x_q are written once.  This is the stand-alone
// entry point's kernel and the prefill path's fall-back for rows that are longer than 16384
// columns or not 16-byte aligned; otherwise that path quantises with one wavefront per token
// inside prepare_kernel (same arithmetic, row kept in registers).
#include "hgf_internal.h"

namespace hgf {

namespace {

template <bool VEC>
__global__ __launch_bounds__(256) void quantize_kernel(const _Float16 *__restrict__ x, int K, int Kp,
                                                       int8_t *__restrict__ xq, float *__restrict__ s_x,
                                                       int32_t *__restrict__ rowsum)
{
    __shared__ float sh_max[4];
    __shared__ int sh_sum[4];
    const int m = blockIdx.x, tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const _Float16 *row = x + (size_t)m * K;
    int8_t *out = xq + (size_t)m * Kp;

    float amax = 0.0f;
    if (VEC) {
        const v8h *row8 = reinterpret_cast<const v8h *>(row);
        for (int i = tid; i < K / 8; i += 256) {
            const v8h v = row8[i];
#pragma unroll
            for (int j = 0; j < 8; ++j) amax = fmaxf(amax, fabsf((float)v[j]));
        }
    } else {
        for (int i = tid; i < K; i += 256) amax = fmaxf(amax, fabsf((float)row[i]));
    }
    amax = wave_max(amax);
    if (lane == 0) sh_max[wave] = amax;
    __syncthreads();
    amax = fmaxf(fmaxf(sh_max[0], sh_max[1]), fmaxf(sh_max[2], sh_max[3]));
    amax = fmaxf(amax, 1e-5f);
    const float inv = 127.0f / amax;

    int sum = 0;
    if (VEC) {
        const v8h *row8 = reinterpret_cast<const v8h *>(row);
        uint2 *out8 = reinterpret_cast<uint2 *>(out);
        for (int i = tid; i < Kp / 8; i += 256) {
            uint2 packed = make_uint2(0u, 0u);
            if (i < K / 8) {
                const v8h v = row8[i];
                uint32_t w[2] = {0u, 0u};
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const int q = quant1((float)v[j], inv);
                    sum += q;
                    w[j >> 2] |= (uint32_t)(q & 0xff) << (8 * (j & 3));
                }
                packed = make_uint2(w[0], w[1]);
            }
            out8[i] = packed;
        }
    } else {
        for (int i = tid; i < Kp; i += 256) {
            int q = 0;
            if (i < K) q = quant1((float)row[i], inv);
            sum += q;
            out[i] = (int8_t)q;
        }
    }
    sum = wave_sum(sum);
    if (lane == 0) sh_sum[wave] = sum;
    __syncthreads();
    if (tid == 0) {
        s_x[m] = amax / 127.0f;
        if (rowsum) rowsum[m] = sh_sum[0] + sh_sum[1] + sh_sum[2] + sh_sum[3];
    }
}

// LayerNorm fused into the quantiser (the appendix implementation's BitLinear normalises the
// backbone's input in fp32 before the absmax quantisation of Sec. 2.2.1; the correction path
// reads x itself): one workgroup per token, the normalised row is never written --
//   mu = mean x, var = mean (x - mu)^2 (biased), v = ((x - mu) * rstd) * gamma + beta, then
//   amax = max |v|, x_q = clip(rne(v * (127 / amax))).
// The two reductions are taken in fp64 in a fixed tree order and rounded once to fp32 (mu and
// rstd = 1 / sqrt(var + eps)); the elementwise part is fp32 with one rounding per operation, in
// exactly this order, because the integers x_q are decided from it.  The row is read four times
// (sum, squared deviations, absmax, rounding); after the first pass it comes from the caches.
__device__ inline double block_sum(double v, double *sh)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    __syncthreads();                 // the previous use of sh is over
    if (lane == 0) sh[wave] = v;
    __syncthreads();
    return ((sh[0] + sh[1]) + sh[2]) + sh[3];
}

__global__ __launch_bounds__(256) void ln_quantize_kernel(const _Float16 *__restrict__ x, int K, int Kp,
                                                          const float *__restrict__ gamma,
                                                          const float *__restrict__ beta, float eps,
                                                          int8_t *__restrict__ xq, float *__restrict__ s_x,
                                                          int32_t *__restrict__ rowsum)
{
    __shared__ double sh_d[4];
    __shared__ float sh_max[4];
    __shared__ int sh_sum[4];
    const int m = blockIdx.x, tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const _Float16 *row = x + (size_t)m * K;
    int8_t *out = xq + (size_t)m * Kp;

    double s = 0.0;
    for (int i = tid; i < K; i += 256) s += (double)(float)row[i];
    const double mu = block_sum(s, sh_d) / (double)K;
    double ss = 0.0;
    for (int i = tid; i < K; i += 256) {
        const double d = (double)(float)row[i] - mu;
        ss += d * d;
    }
    const double var = block_sum(ss, sh_d) / (double)K;
    const float mu32 = (float)mu;
    const float rstd = (float)(1.0 / sqrt(var + (double)eps));
    auto norm = [&](int i) {
        float v = (float)row[i] - mu32;
        v = v * rstd;
        v = v * gamma[i];
        v = v + (beta ? beta[i] : 0.0f);
        return v;
    };

    float amax = 0.0f;
    for (int i = tid; i < K; i += 256) amax = fmaxf(amax, fabsf(norm(i)));
    amax = wave_max(amax);
    if (lane == 0) sh_max[wave] = amax;
    __syncthreads();
    amax = fmaxf(fmaxf(sh_max[0], sh_max[1]), fmaxf(sh_max[2], sh_max[3]));
    amax = fmaxf(amax, 1e-5f);
    const float inv = 127.0f / amax;

    int sum = 0;
    for (int i = tid; i < Kp; i += 256) {
        int q = 0;
        if (i < K) q = quant1(norm(i), inv);
        sum += q;
        out[i] = (int8_t)q;
    }
    sum = wave_sum(sum);
    if (lane == 0) sh_sum[wave] = sum;
    __syncthreads();
    if (tid == 0) {
        s_x[m] = amax / 127.0f;
        if (rowsum) rowsum[m] = sh_sum[0] + sh_sum[1] + sh_sum[2] + sh_sum[3];
    }
}

}  // namespace

hipError_t launch_ln_quantize(const _Float16 *x, int M, int K, const float *gamma, const float *beta, float eps,
                              int8_t *xq, float *s_x, int32_t *rowsum, hipStream_t st)
{
    const int Kp = round_up(K, kTileCols);
    hipLaunchKernelGGL(ln_quantize_kernel, dim3(M), dim3(256), 0, st, x, K, Kp, gamma, beta, eps, xq, s_x, rowsum);
    return hipGetLastError();
}

hipError_t launch_quantize(const _Float16 *x, int M, int K, int8_t *xq, float *s_x, int32_t *rowsum,
                           hipStream_t st)
{
    const int Kp = round_up(K, kTileCols);
    if (K % 8 == 0)
        hipLaunchKernelGGL(quantize_kernel<true>, dim3(M), dim3(256), 0, st, x, K, Kp, xq, s_x, rowsum);
    else
        hipLaunchKernelGGL(quantize_kernel<false>, dim3(M), dim3(256), 0, st, x, K, Kp, xq, s_x, rowsum);
    return hipGetLastError();
}

}  // namespace hgf
