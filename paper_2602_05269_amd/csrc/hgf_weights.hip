// Offline weight path: absmean ternarisation and the 2-bit packed layout.
//
// Sec. 2.2 of the HGF paper (weight-quantisation definition): gamma_W is the mean of |W|
// over the whole matrix and T = Clip(Round(W / gamma_W), -1, 1).  The sum is taken in
// fp64 in a fixed order (per-block partial sums, then one block), rounded once to fp32
// and clamped to >= 1e-5; every element is then multiplied by the fp32 reciprocal and
// rounded half-to-even.
#include "hgf_internal.h"

namespace hgf {

namespace {

__device__ inline double block_sum_f64(double v, double *sh)
{
    const int t = threadIdx.x;
    sh[t] = v;
    __syncthreads();
    for (int s = blockDim.x / 2; s > 0; s >>= 1) {
        if (t < s) sh[t] += sh[t + s];
        __syncthreads();
    }
    return sh[0];
}

__global__ __launch_bounds__(256) void wsum_partial_kernel(const float *__restrict__ W, size_t n,
                                                           double *__restrict__ partials)
{
    __shared__ double sh[256];
    const size_t chunk = (n + gridDim.x - 1) / gridDim.x;
    const size_t lo = chunk * blockIdx.x;
    const size_t hi = lo + chunk < n ? lo + chunk : n;
    double s = 0.0;
    for (size_t i = lo + threadIdx.x; i < hi; i += blockDim.x) s += fabs((double)W[i]);
    s = block_sum_f64(s, sh);
    if (threadIdx.x == 0) partials[blockIdx.x] = s;
}

__global__ __launch_bounds__(256) void wsum_final_kernel(const double *__restrict__ partials, int nparts,
                                                         size_t n, float *__restrict__ s_w)
{
    __shared__ double sh[256];
    double s = 0.0;
    for (int i = threadIdx.x; i < nparts; i += blockDim.x) s += partials[i];
    s = block_sum_f64(s, sh);
    if (threadIdx.x == 0) {
        float g = (float)(s / (double)n);
        *s_w = g < 1e-5f ? 1e-5f : g;
    }
}

__device__ inline uint32_t ternary_code(float w, float inv)
{
    float q = rintf(w * inv);
    q = fminf(fmaxf(q, -1.0f), 1.0f);
    return (uint32_t)((int)q + 1);
}

// Position of packed word `idx`: tile = idx/256; within the tile, lane l = (idx%256)/4 and
// word t = idx%4 hold row 32*rb + (l%32), columns 128*kt + 32*t + 16*(l/32) + 0..15.
__device__ inline void word_position(size_t idx, int KT, int &row, int &kbase)
{
    const size_t tile = idx >> 8;
    const int within = (int)(idx & 255);
    const int l = within >> 2, t = within & 3;
    const int rb = (int)(tile / KT), kt = (int)(tile % KT);
    row = rb * kTileRows + (l & 31);
    kbase = kt * kTileCols + t * 32 + (l >> 5) * 16;
}

// One thread per packed 32-bit word: 16 codes of one row, 16 consecutive columns.
__global__ __launch_bounds__(256) void pack_kernel(const float *__restrict__ W, int N, int K, int KT,
                                                   const float *__restrict__ s_w,
                                                   uint32_t *__restrict__ packed, size_t nwords)
{
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= nwords) return;
    const float inv = 1.0f / *s_w;
    int row, kbase;
    word_position(idx, KT, row, kbase);
    uint32_t word = 0;
#pragma unroll
    for (int s = 0; s < 4; ++s) {
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const int k = kbase + 4 * s + b;
            uint32_t c = 1;                                    // padding decodes to 0
            if (row < N && k < K) c = ternary_code(W[(size_t)row * K + k], inv);
            word |= c << (8 * b + 2 * s);
        }
    }
    packed[idx] = word;
}

// One thread per packed word, writing its 16 values back as int8 -1/0/+1.
__global__ __launch_bounds__(256) void unpack_kernel(const uint32_t *__restrict__ packed, int N, int K, int KT,
                                                     int8_t *__restrict__ T, size_t nwords)
{
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= nwords) return;
    int row, kbase;
    word_position(idx, KT, row, kbase);
    if (row >= N) return;
    const uint32_t word = packed[idx];
#pragma unroll
    for (int s = 0; s < 4; ++s) {
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const int k = kbase + 4 * s + b;
            if (k < K) T[(size_t)row * K + k] = (int8_t)((int)((word >> (8 * b + 2 * s)) & 3u) - 1);
        }
    }
}

__global__ __launch_bounds__(256) void fill_kernel(uint4 *__restrict__ p, size_t n16, uint32_t word)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n16; i += stride) p[i] = make_uint4(word, word, word, word);
}

__global__ __launch_bounds__(256) void zero_words_kernel(uint32_t *__restrict__ p, size_t n)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0u;
}

}  // namespace

// Zeroes n 4-byte words at any 4-byte aligned address (a kernel, so it may be captured in a graph).
hipError_t launch_zero_words(void *p, size_t n, hipStream_t st)
{
    if (n == 0) return hipSuccess;
    hipLaunchKernelGGL(zero_words_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st,
                       reinterpret_cast<uint32_t *>(p), n);
    return hipGetLastError();
}

hipError_t launch_wsum(const float *W, size_t n, double *partials, float *s_w_out, hipStream_t st)
{
    hipLaunchKernelGGL(wsum_partial_kernel, dim3(kWsumBlocks), dim3(256), 0, st, W, n, partials);
    hipLaunchKernelGGL(wsum_final_kernel, dim3(1), dim3(256), 0, st, partials, kWsumBlocks, n, s_w_out);
    return hipGetLastError();
}

hipError_t launch_pack(const float *W, int N, int K, const float *s_w, uint32_t *packed, hipStream_t st)
{
    const int KT = round_up(K, kTileCols) / kTileCols;
    const size_t nwords = (size_t)(round_up(N, kTileRows) / kTileRows) * KT * 256;
    hipLaunchKernelGGL(pack_kernel, dim3((unsigned)((nwords + 255) / 256)), dim3(256), 0, st, W, N, K, KT, s_w,
                       packed, nwords);
    return hipGetLastError();
}

hipError_t launch_unpack(const uint32_t *packed, int N, int K, int8_t *T, hipStream_t st)
{
    const int KT = round_up(K, kTileCols) / kTileCols;
    const size_t nwords = (size_t)(round_up(N, kTileRows) / kTileRows) * KT * 256;
    hipLaunchKernelGGL(unpack_kernel, dim3((unsigned)((nwords + 255) / 256)), dim3(256), 0, st, packed, N, K, KT,
                       T, nwords);
    return hipGetLastError();
}

hipError_t launch_fill(void *p, size_t bytes, uint32_t word, hipStream_t st)
{
    const size_t n16 = bytes / 16;                               // callers pass multiples of 16
    unsigned blocks = (unsigned)((n16 + 255) / 256);
    if (blocks > 4096) blocks = 4096;
    if (blocks == 0) return hipSuccess;
    hipLaunchKernelGGL(fill_kernel, dim3(blocks), dim3(256), 0, st, (uint4 *)p, n16, word);
    return hipGetLastError();
}

}  // namespace hgf
