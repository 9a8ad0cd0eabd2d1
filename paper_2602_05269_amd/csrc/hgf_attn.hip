// Differential attention, one decode step (the block that consumes the HGF q/k/v projections).
//
// Sec. 2.4, Def. "Differential Attention": with Q = [Q1; Q2] and K = [K1; K2] split into two
// groups of heads,  O = (softmax(Q1 K1^T / sqrt(d_h)) - lambda softmax(Q2 K2^T / sqrt(d_h))) V.
// The appendix implementation fixes what the definition leaves open: q and k carry 2 n_heads
// heads of d_h = d_model / (2 n_heads) columns (the first n_heads are branch 1, the rest branch
// 2), v carries n_heads heads of the same d_h (V: d -> d/2), head h of both branches reads head
// h of v, the scores are scaled by 1/sqrt(d_h), and the difference is multiplied by 0.5.
//
// Decode: the newest token attends to every cached position 0 .. len-1 (itself included), so
// a step streams the K and V caches once: 6 len d_h bytes per head, nothing else of size.
// That is bandwidth-bound work with no reuse, so there are no matrix instructions here:
// coalesced 16-byte loads, dot products in the vector ALU, cross-lane reductions.
//   pass 1 (grid: chunks of 256 positions x heads x sequences): a workgroup loads its chunk
//     of K1, K2 and V rows of one head in one burst, forms both branches' scores, their chunk
//     maximum and exponentials (LDS), and both exp-weighted sums of the V rows, which it reads
//     once for the two; it writes (max, sum, weighted V) per branch to the workspace;
//   pass 2 (grid: heads x sequences): merges the chunks (rescaling by exp(max_chunk - max)),
//     normalises, forms (a1 - lambda a2) * 0.5 and stores fp16.
#include "hgf_internal.h"

namespace hgf {

namespace {

constexpr int kAttnChunk = 256;        // positions per workgroup of pass 1 (one per thread)

struct AttnParams {
    const _Float16 *q;                 // [B, 2 n_heads, d_h]
    const _Float16 *k;                 // [B, L_max, 2 n_heads, d_h]
    const _Float16 *v;                 // [B, L_max, n_heads, d_h]
    const int32_t *lens;               // [B]
    float *part;                       // [B, n_heads, chunks, 2, d_h + 2]
    _Float16 *out;                     // [B, n_heads, d_h]
    int B, L_max, n_heads, d_h, chunks;
    float lambda, scale;
};

// V8: 16-byte pieces of a head row (d_h / 8).  Lane (ps = l / V8, pc = l % V8) takes piece pc of
// the positions ps, ps + P, ... of its wavefront's 64 positions (P = 64 / V8 per instruction).
template <int V8>
__global__ __launch_bounds__(256) void diff_attn_chunk_kernel(AttnParams p)
{
    constexpr int P = 64 / V8, IT = 64 / P;
    __shared__ float sc[2][kAttnChunk];
    __shared__ float red[2][4];
    __shared__ float accs[4][2][V8 * 8];
    const int tid = threadIdx.x, l = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int chunk = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int len = min(max(p.lens[b], 0), p.L_max);
    const int d_h = V8 * 8;
    float *out = p.part + ((((size_t)b * p.n_heads + h) * p.chunks + chunk) * 2) * (d_h + 2);
    const int pos0 = chunk * kAttnChunk;
    if (pos0 >= len) {                  // nothing cached here: an empty part (exp(-inf) weight)
        if (tid < 2) {
            out[tid * (d_h + 2)] = -INFINITY;
            out[tid * (d_h + 2) + 1] = 0.f;
        }
        for (int e = tid; e < 2 * d_h; e += 256) out[(e / d_h) * (d_h + 2) + 2 + e % d_h] = 0.f;
        return;
    }
    const int ps = l / V8, pc = l % V8;
    const size_t krow = (size_t)2 * p.n_heads * d_h, vrow = (size_t)p.n_heads * d_h;
    const rsrc_t kr = make_rsrc(p.k + (size_t)b * p.L_max * krow, (unsigned)((size_t)len * krow * 2));
    const rsrc_t vr = make_rsrc(p.v + (size_t)b * p.L_max * vrow, (unsigned)((size_t)len * vrow * 2));
    // the burst: every K1 and K2 piece of this lane (rows past len lie beyond the descriptors: zeros)
    v4u k1[IT], k2[IT], vv[IT];
#pragma unroll
    for (int it = 0; it < IT; ++it) {
        const unsigned pos = (unsigned)(pos0 + w * 64 + it * P + ps);
        k1[it] = buf_load16_stream(kr, (unsigned)((pos * krow + (size_t)h * d_h + pc * 8) * 2));
        k2[it] = buf_load16_stream(kr, (unsigned)((pos * krow + (size_t)(p.n_heads + h) * d_h + pc * 8) * 2));
    }
    const _Float16 *qb = p.q + (size_t)b * krow;
    const v8h q1 = *reinterpret_cast<const v8h *>(qb + (size_t)h * d_h + pc * 8);
    const v8h q2 = *reinterpret_cast<const v8h *>(qb + (size_t)(p.n_heads + h) * d_h + pc * 8);

    // ---- scores of both branches
#pragma unroll
    for (int it = 0; it < IT; ++it) {
        const v8h a = __builtin_bit_cast(v8h, k1[it]), c = __builtin_bit_cast(v8h, k2[it]);
        float s1 = 0.f, s2 = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            s1 += (float)q1[e] * (float)a[e];
            s2 += (float)q2[e] * (float)c[e];
        }
#pragma unroll
        for (int o = 1; o < V8; o <<= 1) {
            s1 += __shfl_xor(s1, o, 64);
            s2 += __shfl_xor(s2, o, 64);
        }
        const int idx = w * 64 + it * P + ps;
        if (pc == 0) {
            const bool valid = pos0 + idx < len;
            sc[0][idx] = valid ? s1 * p.scale : -INFINITY;
            sc[1][idx] = valid ? s2 * p.scale : -INFINITY;
        }
    }
    // the V rows are requested now (the K registers are free again) and arrive during the softmax
#pragma unroll
    for (int it = 0; it < IT; ++it) {
        const unsigned pos = (unsigned)(pos0 + w * 64 + it * P + ps);
        vv[it] = buf_load16_stream(vr, (unsigned)((pos * vrow + (size_t)h * d_h + pc * 8) * 2));
    }
    __syncthreads();
    // ---- chunk maximum, exponentials and their sum: one position per thread
    float m[2], lsum[2];
#pragma unroll
    for (int br = 0; br < 2; ++br) {
        const float s = sc[br][tid];
        float mx = wave_max(s);
        if (l == 0) red[br][w] = mx;
        __syncthreads();
        mx = fmaxf(fmaxf(red[br][0], red[br][1]), fmaxf(red[br][2], red[br][3]));   // finite: position pos0 is valid
        const float e = expf(s - mx);
        sc[br][tid] = e;
        float sum = e;
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o, 64);
        __syncthreads();
        if (l == 0) red[br][w] = sum;
        __syncthreads();
        m[br] = mx;
        lsum[br] = (red[br][0] + red[br][1]) + (red[br][2] + red[br][3]);
        __syncthreads();
    }
    // ---- both branches' weighted sums of the V rows (read once)
    float a1[8], a2[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) a1[e] = a2[e] = 0.f;
#pragma unroll
    for (int it = 0; it < IT; ++it) {
        const int idx = w * 64 + it * P + ps;
        const float p1 = sc[0][idx], p2 = sc[1][idx];
        const v8h x = __builtin_bit_cast(v8h, vv[it]);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            a1[e] += p1 * (float)x[e];
            a2[e] += p2 * (float)x[e];
        }
    }
#pragma unroll
    for (int o = V8; o < 64; o <<= 1) {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            a1[e] += __shfl_xor(a1[e], o, 64);
            a2[e] += __shfl_xor(a2[e], o, 64);
        }
    }
    if (ps == 0) {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            accs[w][0][pc * 8 + e] = a1[e];
            accs[w][1][pc * 8 + e] = a2[e];
        }
    }
    __syncthreads();
    for (int e = tid; e < 2 * d_h; e += 256) {
        const int br = e / d_h, d = e % d_h;
        out[br * (d_h + 2) + 2 + d] = (accs[0][br][d] + accs[1][br][d]) + (accs[2][br][d] + accs[3][br][d]);
    }
    if (tid < 2) {
        out[tid * (d_h + 2)] = m[tid];
        out[tid * (d_h + 2) + 1] = lsum[tid];
    }
}

__global__ __launch_bounds__(128) void diff_attn_merge_kernel(AttnParams p)
{
    const int h = blockIdx.x, b = blockIdx.y, d = threadIdx.x;
    const int d_h = p.d_h;
    if (d >= d_h) return;
    const float *part = p.part + (((size_t)b * p.n_heads + h) * p.chunks) * 2 * (d_h + 2);
    const int len = min(max(p.lens[b], 0), p.L_max);
    const int used = (len + kAttnChunk - 1) / kAttnChunk;
    float a[2];
#pragma unroll
    for (int br = 0; br < 2; ++br) {
        float mx = -INFINITY;
        for (int c = 0; c < used; ++c) mx = fmaxf(mx, part[(c * 2 + br) * (d_h + 2)]);
        float sum = 0.f, acc = 0.f;
        for (int c = 0; c < used; ++c) {
            const float *q = part + (c * 2 + br) * (d_h + 2);
            const float wgt = expf(q[0] - mx);
            sum += q[1] * wgt;
            acc += q[2 + d] * wgt;
        }
        a[br] = used > 0 ? acc / sum : 0.f;
    }
    p.out[((size_t)b * p.n_heads + h) * d_h + d] = (_Float16)((a[0] - p.lambda * a[1]) * 0.5f);
}

}  // namespace

size_t diff_attn_workspace_bytes(int B, int L_max, int n_heads, int d_h)
{
    const size_t chunks = (size_t)(L_max + kAttnChunk - 1) / kAttnChunk;
    return (size_t)B * n_heads * chunks * 2 * (d_h + 2) * sizeof(float);
}

hipError_t launch_diff_attn(const void *q, const void *k, const void *v, const int32_t *lens, int B, int L_max,
                            int n_heads, int d_h, float lambda, void *out, void *workspace, hipStream_t st)
{
    AttnParams p;
    p.q = reinterpret_cast<const _Float16 *>(q);
    p.k = reinterpret_cast<const _Float16 *>(k);
    p.v = reinterpret_cast<const _Float16 *>(v);
    p.lens = lens;
    p.part = reinterpret_cast<float *>(workspace);
    p.out = reinterpret_cast<_Float16 *>(out);
    p.B = B;
    p.L_max = L_max;
    p.n_heads = n_heads;
    p.d_h = d_h;
    p.chunks = (L_max + kAttnChunk - 1) / kAttnChunk;
    p.lambda = lambda;
    p.scale = 1.0f / sqrtf((float)d_h);
    const dim3 grid(p.chunks, n_heads, B), block(256);
    switch (d_h / 8) {
        case 1: hipLaunchKernelGGL(diff_attn_chunk_kernel<1>, grid, block, 0, st, p); break;
        case 2: hipLaunchKernelGGL(diff_attn_chunk_kernel<2>, grid, block, 0, st, p); break;
        case 4: hipLaunchKernelGGL(diff_attn_chunk_kernel<4>, grid, block, 0, st, p); break;
        case 8: hipLaunchKernelGGL(diff_attn_chunk_kernel<8>, grid, block, 0, st, p); break;
        case 16: hipLaunchKernelGGL(diff_attn_chunk_kernel<16>, grid, block, 0, st, p); break;
        default: return hipErrorInvalidValue;
    }
    hipLaunchKernelGGL(diff_attn_merge_kernel, dim3(n_heads, B), dim3(128), 0, st, p);
    return hipGetLastError();
}

}  // namespace hgf
