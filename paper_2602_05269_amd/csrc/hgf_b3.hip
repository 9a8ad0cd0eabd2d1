// Base-3 packing of the ternary weights, five per byte (1.6 bits per weight), and a decode
// kernel for a handful of tokens that reads it.
//
// The HGF paper calls its backbone "1.58-bit" (Sec. 4.1, Def. "Effective Bit-Width": log2 3 bits
// per ternary weight).  The 2-bit layout of the main path spends 0.42 bits per weight on a code
// that never occurs; five ternary digits fit one byte (3^5 = 243 <= 256), which is 20 % fewer
// bytes to stream at decode, where the weights are nearly all the traffic.  The price is the
// decode: a byte no longer splits into fields with a shift and a mask.
//
// Layout.  Row n of the [d_out, d_in] matrix is ceil(d_in / 5) bytes, padded to a multiple of 16
// so that every row starts 16-byte aligned and a lane's load is 16 bytes = 80 weights of one row;
// consecutive lanes read consecutive pieces of the row (coalesced).  Byte g of a row holds
// columns 5g .. 5g+4 as  b = sum_i (T[n, 5g+i] + 1) * 3^i ; columns past d_in count as T = 0, so
// padding bytes are 121.
//
// Kernel (Algorithm 1, steps 3, 4, 7, 8 for M <= 4; steps 1, 2, 5, 6 come from the decode
// prologue).  A 256-entry table in LDS maps a byte to its five codes as int8 (four in one
// 32-bit word, the fifth in a second), and the quantised tokens sit in LDS in the matching
// image (eight bytes per group of five columns: four values, then the fifth and three zeros),
// so a byte of weights costs one table read, one token read per token and two 4-way int8 dot
// products per token.  A wavefront takes whole rows: its lanes split the row's bytes and a
// cross-lane reduction adds their sums, for the int32 accumulators and for the rank-r
// up-projection alike.  Codes are T + 1; the per-token sum of x_q is subtracted at the end.
#include "hgf_internal.h"

namespace hgf {

namespace {

constexpr int kB3Group = 5;
constexpr int kB3MaxM = 4;
constexpr unsigned kB3PadByte = 121u;     // five zero weights

__host__ __device__ inline int b3_groups(int K) { return (K + kB3Group - 1) / kB3Group; }
__host__ __device__ inline int b3_row_bytes(int K) { return (b3_groups(K) + 15) / 16 * 16; }

// One thread per output byte.
__global__ __launch_bounds__(256) void pack_b3_kernel(const float *__restrict__ W, int N, int K, int Rb,
                                                      const float *__restrict__ s_w, unsigned char *__restrict__ out)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= (size_t)N * Rb) return;
    const int n = (int)(i / Rb), g = (int)(i % Rb);
    const float inv = 1.0f / *s_w;
    unsigned b = 0, p3 = 1;
#pragma unroll
    for (int d = 0; d < kB3Group; ++d) {
        const int k = g * kB3Group + d;
        int t = 0;
        if (k < K) {
            float q = rintf(W[(size_t)n * K + k] * inv);
            q = fminf(fmaxf(q, -1.0f), 1.0f);
            t = (int)q;
        }
        b += (unsigned)(t + 1) * p3;
        p3 *= 3;
    }
    out[i] = (unsigned char)b;
}

__global__ __launch_bounds__(256) void unpack_b3_kernel(const unsigned char *__restrict__ packed, int N, int K, int Rb,
                                                        int8_t *__restrict__ T)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= (size_t)N * K) return;
    const int n = (int)(i / K), k = (int)(i % K);
    unsigned b = packed[(size_t)n * Rb + k / kB3Group];
    for (int d = 0; d < k % kB3Group; ++d) b /= 3;
    T[i] = (int8_t)((int)(b % 3) - 1);
}

struct B3Params {
    const unsigned char *packed;   // [N, Rb]
    const int8_t *xq;              // [M, Kp]
    const float *s_x;
    const int32_t *rowsum;
    const _Float16 *h16;           // [M, hstride] SiLU(A x)
    const float *s_w;
    const _Float16 *B, *alpha;
    _Float16 *y;
    int32_t *acc_debug;
    int M, K, Kp, N, Rb, rank, hstride;
    int rows_per_wave;
};

__device__ inline int wave_sum_i(int v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ inline float wave_sum_f(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ inline int dot4(unsigned a, unsigned b, int c)
{
    return __builtin_amdgcn_sdot4((int)a, (int)b, c, false);
}

template <int MT>
__global__ __launch_bounds__(256) void b3_decode_kernel(B3Params p)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    uint2 *lut = reinterpret_cast<uint2 *>(lds);                       // 256 entries
    uint2 *xs = reinterpret_cast<uint2 *>(lds + 2048);                 // [MT][Rb] token slots
    float *hs = reinterpret_cast<float *>(lds + 2048 + (size_t)MT * p.Rb * 8);   // [MT][hstride] fp32

    const int tid = threadIdx.x, l = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    {   // the table: byte -> codes 0..3 in one word, code 4 in the next (bytes >= 243 never occur)
        unsigned b = (unsigned)tid, lo = 0;
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            lo |= (b % 3) << (8 * d);
            b /= 3;
        }
        lut[tid] = make_uint2(lo, b % 3);
    }
    // the tokens' image: slot g holds x_q[5g .. 5g+3] and x_q[5g+4]; columns past d_in are zero
    for (int i = tid; i < MT * p.Rb; i += 256) {
        const int m = i / p.Rb, g = i - m * p.Rb;
        unsigned v[kB3Group];
#pragma unroll
        for (int d = 0; d < kB3Group; ++d) {
            const int k = g * kB3Group + d;
            v[d] = (m < p.M && k < p.K) ? (unsigned)(unsigned char)p.xq[(size_t)m * p.Kp + k] : 0u;
        }
        xs[i] = make_uint2(v[0] | (v[1] << 8) | (v[2] << 16) | (v[3] << 24), v[4]);
    }
    for (int i = tid; i < MT * p.hstride; i += 256) {
        const int m = i / p.hstride;
        hs[i] = (p.rank > 0 && m < p.M) ? (float)p.h16[i] : 0.0f;
    }
    __syncthreads();

    const float s_w = *p.s_w;
    float scale[MT];
    int rs[MT];
#pragma unroll
    for (int m = 0; m < MT; ++m) {
        scale[m] = m < p.M ? p.s_x[m] * s_w : 0.0f;
        rs[m] = m < p.M ? p.rowsum[m] : 0;
    }
    const int pieces = p.Rb / 16;                   // 16-byte pieces of a row
    const rsrc_t wr = make_rsrc(p.packed, (unsigned)((size_t)p.N * p.Rb));
    const int wave = blockIdx.x * 4 + w;
    const int n_first = wave * p.rows_per_wave;
    const int n_end = min(n_first + p.rows_per_wave, p.N);

    // a row's pieces for this lane: piece l, l + 64, ...; up to kPieces of them are held in registers,
    // requested one row ahead
    constexpr int kPieces = 4;                      // 64 lanes x 4 x 16 bytes x 5 = 20480 columns
    v4u cur[kPieces], nxt[kPieces];
    auto request = [&](v4u (&dst)[kPieces], int n) {
#pragma unroll
        for (int q = 0; q < kPieces; ++q) {
            const int pc = l + 64 * q;
            dst[q] = buf_load16_stream(wr, (n < n_end && pc < pieces) ? (unsigned)n * p.Rb + pc * 16 : kOob);
        }
    };
    request(cur, n_first);
    for (int n = n_first; n < n_end; ++n) {
        request(nxt, n + 1);
        // epilogue operands of the row: two ranks of B per lane, the gate parameter
        float bj0 = 0.f, bj1 = 0.f, gate = 0.f;
        if (p.rank > 0) {
            const int j = 2 * l;
            if (j < p.rank) bj0 = (float)p.B[(size_t)n * p.rank + j];
            if (j + 1 < p.rank) bj1 = (float)p.B[(size_t)n * p.rank + j + 1];
            gate = tanhf((float)p.alpha[n]);
        }
        int acc[MT];
#pragma unroll
        for (int m = 0; m < MT; ++m) acc[m] = 0;
#pragma unroll
        for (int q = 0; q < kPieces; ++q) {
            const int pc = l + 64 * q;
            if (pc >= pieces) continue;
#pragma unroll
            for (int dw = 0; dw < 4; ++dw) {
                const unsigned word = cur[q][dw];
#pragma unroll
                for (int by = 0; by < 4; ++by) {
                    const unsigned b = (word >> (8 * by)) & 0xffu;
                    const uint2 codes = lut[b];
                    const int g = pc * 16 + dw * 4 + by;
#pragma unroll
                    for (int m = 0; m < MT; ++m) {
                        const uint2 xv = xs[m * p.Rb + g];
                        acc[m] = dot4(codes.x, xv.x, acc[m]);
                        acc[m] = dot4(codes.y, xv.y, acc[m]);
                    }
                }
            }
        }
#pragma unroll
        for (int m = 0; m < MT; ++m) {
            const int a = wave_sum_i(acc[m]) - rs[m];
            float c = 0.f;
            if (p.rank > 0) {
                const float h0 = 2 * l < p.rank ? hs[m * p.hstride + 2 * l] : 0.f;
                const float h1 = 2 * l + 1 < p.rank ? hs[m * p.hstride + 2 * l + 1] : 0.f;
                c = wave_sum_f(bj0 * h0 + bj1 * h1);
            }
            if (l == 0 && m < p.M) {
                p.y[(size_t)m * p.N + n] = (_Float16)((float)a * scale[m] + gate * c);
                if (p.acc_debug) p.acc_debug[(size_t)m * p.N + n] = a;
            }
        }
#pragma unroll
        for (int q = 0; q < kPieces; ++q) cur[q] = nxt[q];
    }
}

}  // namespace

size_t b3_packed_bytes(int d_out, int d_in) { return (size_t)d_out * b3_row_bytes(d_in); }

hipError_t launch_pack_b3(const float *W, int N, int K, const float *s_w, unsigned char *packed, hipStream_t st)
{
    const int Rb = b3_row_bytes(K);
    const size_t n = (size_t)N * Rb;
    hipLaunchKernelGGL(pack_b3_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, W, N, K, Rb, s_w, packed);
    return hipGetLastError();
}

hipError_t launch_unpack_b3(const unsigned char *packed, int N, int K, int8_t *T, hipStream_t st)
{
    const size_t n = (size_t)N * K;
    hipLaunchKernelGGL(unpack_b3_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, packed, N, K,
                       b3_row_bytes(K), T);
    return hipGetLastError();
}

// False: the shape does not fit this kernel (tokens' image beyond LDS, or a row beyond the
// registers that hold it).
bool b3_fits(int M, int K, int rank)
{
    if (M < 1 || M > kB3MaxM) return false;
    const int Rb = b3_row_bytes(K);
    if (Rb / 16 > 64 * 4) return false;
    const int mt = M <= 1 ? 1 : (M <= 2 ? 2 : 4);
    const size_t lds = 2048 + (size_t)mt * Rb * 8 + (size_t)mt * h_stride(rank > 0 ? rank : 1) * 4;
    return lds <= 150 * 1024;
}

hipError_t launch_b3_decode(const void *packed, const Workspace &ws, const _Float16 *h16, int M, const hgf_layer &L,
                            void *y, int32_t *acc_debug, hipStream_t st)
{
    B3Params p;
    p.packed = reinterpret_cast<const unsigned char *>(packed);
    p.xq = ws.xq;
    p.s_x = ws.s_x;
    p.rowsum = ws.rowsum;
    p.h16 = h16;
    p.s_w = L.s_w;
    p.B = reinterpret_cast<const _Float16 *>(L.B_f16);
    p.alpha = reinterpret_cast<const _Float16 *>(L.alpha_f16);
    p.y = reinterpret_cast<_Float16 *>(y);
    p.acc_debug = acc_debug;
    p.M = M;
    p.K = L.d_in;
    p.Kp = round_up(L.d_in, kTileCols);
    p.N = L.d_out;
    p.Rb = b3_row_bytes(L.d_in);
    p.rank = L.rank;
    p.hstride = h_stride(L.rank > 0 ? L.rank : 1);
    // about two workgroups per compute unit (each rebuilds the tokens' image, so fewer and longer
    // lived ones are cheaper), at least two rows per wavefront (the second row's request overlaps
    // the first row's arithmetic)
    int rows = (L.d_out + 2047) / 2048;
    if (rows < 2) rows = 2;
    p.rows_per_wave = rows;
    const int waves = (L.d_out + rows - 1) / rows;
    const int mt = M <= 1 ? 1 : (M <= 2 ? 2 : 4);
    const size_t lds = 2048 + (size_t)mt * p.Rb * 8 + (size_t)mt * p.hstride * 4;
    static const hipError_t attr = [] {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&b3_decode_kernel<1>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 150 * 1024);
        if (e == hipSuccess)
            e = hipFuncSetAttribute(reinterpret_cast<const void *>(&b3_decode_kernel<2>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, 150 * 1024);
        if (e == hipSuccess)
            e = hipFuncSetAttribute(reinterpret_cast<const void *>(&b3_decode_kernel<4>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, 150 * 1024);
        return e;
    }();
    if (attr != hipSuccess) return attr;
    const dim3 grid((waves + 3) / 4), block(256);
    if (mt == 1) hipLaunchKernelGGL(b3_decode_kernel<1>, grid, block, lds, st, p);
    else if (mt == 2) hipLaunchKernelGGL(b3_decode_kernel<2>, grid, block, lds, st, p);
    else hipLaunchKernelGGL(b3_decode_kernel<4>, grid, block, lds, st, p);
    return hipGetLastError();
}

}  // namespace hgf
