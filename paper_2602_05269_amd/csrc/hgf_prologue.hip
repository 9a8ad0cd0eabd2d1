// Decode prologue (up to 64 tokens): one launch that quantises the activations and starts the
// correction path of every layer reading them.
//
// Algorithm 1 of the HGF paper, steps 1-2 (per-token absmax int8 quantisation,
// Sec. 2.2.1) and step 5 (H <- X A on the UN-quantised fp16 activations).  Workgroups
// 0..M-1 each quantise one token; the remaining workgroups hold four wavefronts, each
// computing one 16-rank-row tile of A x over one slice of d_in on the 16x16x32 f16 MFMA
// (rows = rank indices, columns = tokens) and writing its fp32 partial sums.  The slices
// are short enough that a wavefront issues all of its loads at once: the launch costs one
// memory round trip.  The consumer adds the slices in order (deterministic) and applies
// SiLU (step 6) while its weights are in flight.
#include "hgf_internal.h"

namespace hgf {

namespace {

constexpr int kRegVecs = 6;   // a token row of up to 6*256*8 = 12288 columns stays in registers

// One workgroup quantises one token row.  VEC: d_in % 8 == 0 (16-byte loads).
template <bool VEC>
__device__ void quantize_row(const ProParams &p, int m)
{
    __shared__ float sh_max[4];
    __shared__ int sh_sum[4];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const _Float16 *row = p.x + (size_t)m * p.K;
    int8_t *out = p.xq + (size_t)m * p.Kp;
    const int nvec = p.K / 8;
    const bool in_regs = VEC && nvec <= kRegVecs * 256;

    v8h keep[kRegVecs];
    float amax = 0.0f;
    if (VEC) {
        const v8h *row8 = reinterpret_cast<const v8h *>(row);
        if (in_regs) {
            const rsrc_t rr = make_rsrc(row, (unsigned)p.K * 2u);
#pragma unroll
            for (int r = 0; r < kRegVecs; ++r)
                keep[r] = __builtin_bit_cast(v8h, buf_load16(rr, (unsigned)(tid + r * 256) * 16u));
#pragma unroll
            for (int r = 0; r < kRegVecs; ++r)
#pragma unroll
                for (int j = 0; j < 8; ++j) amax = fmaxf(amax, fabsf((float)keep[r][j]));
        } else {
            for (int i = tid; i < nvec; i += 256) {
                const v8h v = row8[i];
#pragma unroll
                for (int j = 0; j < 8; ++j) amax = fmaxf(amax, fabsf((float)v[j]));
            }
        }
    } else {
        for (int i = tid; i < p.K; i += 256) amax = fmaxf(amax, fabsf((float)row[i]));
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
        auto quant8 = [&](const v8h v) {
            uint32_t w[2] = {0u, 0u};
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int q = quant1((float)v[j], inv);
                sum += q;
                w[j >> 2] |= (uint32_t)(q & 0xff) << (8 * (j & 3));
            }
            return make_uint2(w[0], w[1]);
        };
        if (in_regs) {
#pragma unroll
            for (int r = 0; r < kRegVecs; ++r) {
                const int i = tid + r * 256;
                if (i < nvec) out8[i] = quant8(keep[r]);
                else if (i < p.Kp / 8) out8[i] = make_uint2(0u, 0u);
            }
            for (int i = tid + kRegVecs * 256; i < p.Kp / 8; i += 256) out8[i] = make_uint2(0u, 0u);
        } else {
            for (int i = tid; i < p.Kp / 8; i += 256) out8[i] = i < nvec ? quant8(row8[i]) : make_uint2(0u, 0u);
        }
    } else {
        for (int i = tid; i < p.Kp; i += 256) {
            int q = 0;
            if (i < p.K) q = quant1((float)row[i], inv);
            sum += q;
            out[i] = (int8_t)q;
        }
    }
    sum = wave_sum(sum);
    if (lane == 0) sh_sum[wave] = sum;
    __syncthreads();
    if (tid == 0) {
        p.s_x[m] = amax / 127.0f;
        p.rowsum[m] = sh_sum[0] + sh_sum[1] + sh_sum[2] + sh_sum[3];
        if (p.amax_zero) p.amax_zero[m] = 0.0f;
    }
}

// One wavefront: rank tile `rt` of layer `g`, slice `sp` of d_in, every token tile.
// Lane (i = l%16, kb = l/16) holds A[rt*16+i][k] and x[tt*16+i][k] for the same eight k per
// MFMA: k = 64*kp + 16*kb + 0..7 and + 8..15 (two MFMAs per 64 columns), so a row is read
// 128 contiguous bytes at a time.  All loads of the slice are issued before the first MFMA.
template <int TT, bool VEC>
__device__ void corr_partial(const ProParams &p, int job)
{
    int g = 0;
    while (g + 1 < p.G && job >= p.job_start[g + 1]) ++g;
    const ProLayer &L = p.L[g];
    const int local = job - p.job_start[g];
    const int rt = local / p.S, sp = local % p.S;
    const int l = threadIdx.x & 63, i = l & 15, kb = l >> 4;
    const int j = rt * 16 + i;
    const bool j_ok = j < L.rank;
    const rsrc_t ar = make_rsrc(L.A, (unsigned)L.rank * p.K * 2u);
    const rsrc_t xr = make_rsrc(p.x, (unsigned)p.M * p.K * 2u);

    v4f acc[TT];
#pragma unroll
    for (int tt = 0; tt < TT; ++tt) acc[tt] = (v4f){0.f, 0.f, 0.f, 0.f};

    const int kp0 = sp * p.pairs_per_slice;
    const int kp1 = min(kp0 + p.pairs_per_slice, p.pairs);
    constexpr int UN = 8;                      // 64-column steps issued together
    for (int kpb = kp0; kpb < kp1; kpb += UN) {
        v8h a[UN][2];
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            const int k0 = (kpb + u) * 64 + kb * 16;
            const bool ok = j_ok && (kpb + u) < kp1;
            a[u][0] = buf_load8h<VEC>(ar, (unsigned)j * p.K + k0, p.K - k0, ok);
            a[u][1] = buf_load8h<VEC>(ar, (unsigned)j * p.K + k0 + 8, p.K - k0 - 8, ok);
        }
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) {
            const int m = tt * 16 + i;
            const bool m_ok = m < p.M;
            v8h b[UN][2];
#pragma unroll
            for (int u = 0; u < UN; ++u) {
                const int k0 = (kpb + u) * 64 + kb * 16;
                const bool ok = m_ok && (kpb + u) < kp1;
                b[u][0] = buf_load8h<VEC>(xr, (unsigned)m * p.K + k0, p.K - k0, ok);
                b[u][1] = buf_load8h<VEC>(xr, (unsigned)m * p.K + k0 + 8, p.K - k0 - 8, ok);
            }
#pragma unroll
            for (int u = 0; u < UN; ++u) {
                acc[tt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[u][0], b[u][0], acc[tt], 0, 0, 0);
                acc[tt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[u][1], b[u][1], acc[tt], 0, 0, 0);
            }
        }
    }
    // acc[tt][v]: rank index rt*16 + 4*kb + v, token tt*16 + i  ->  hpart[sp][m][rp]
#pragma unroll
    for (int tt = 0; tt < TT; ++tt) {
        const int m = tt * 16 + i;
        if (m < p.M)
            *reinterpret_cast<v4f *>(L.hpart + ((size_t)sp * p.M + m) * L.rp + rt * 16 + 4 * kb) = acc[tt];
    }
}

template <int TT, bool VEC>
__global__ __launch_bounds__(256) void prologue_kernel(ProParams p)
{
    const int qb = p.quantize ? p.M : 0;            // workgroups that quantise a token each
    if ((int)blockIdx.x < qb) {
        quantize_row<VEC>(p, blockIdx.x);
        return;
    }
    const int job = ((int)blockIdx.x - qb) * 4 + (threadIdx.x >> 6);
    if (job < p.job_start[p.G]) corr_partial<TT, VEC>(p, job);
}

// Adds the slices in order (deterministic), applies SiLU (Alg. 1 step 6) and writes fp16 rows of
// hstride (zero padded): one thread per (layer, token, rank), all its slices requested at once.
struct ReduceParams {
    const float *hpart[kMaxGroup];
    _Float16 *h16[kMaxGroup];
    int rank[kMaxGroup], rp[kMaxGroup], start[kMaxGroup + 1];
    int M, S, G;
};
__global__ __launch_bounds__(256) void hreduce_kernel(ReduceParams p)
{
    const int e = blockIdx.x * 256 + threadIdx.x;
    int g = 0;
#pragma unroll
    for (int i = 1; i < kMaxGroup; ++i)
        if (i < p.G && e >= p.start[i]) g = i;
    const int idx = e - p.start[g], rp = p.rp[g];
    const bool inside = e < p.start[p.G];
    const int j = idx % rp;
    const rsrc_t hr = make_rsrc(p.hpart[g], (unsigned)p.S * p.M * rp * 4u);
    float part[kMaxHSplit];
#pragma unroll
    for (int sp = 0; sp < kMaxHSplit; ++sp)
        part[sp] = __builtin_bit_cast(float, buf_load4(hr, ((unsigned)idx + (unsigned)sp * p.M * rp) * 4u,
                                                       inside && j < p.rank[g] && sp < p.S));
    float h = part[0];
#pragma unroll
    for (int sp = 1; sp < kMaxHSplit; ++sp) h += part[sp];
    if (inside) p.h16[g][idx] = (_Float16)silu(h);
}

}  // namespace

int prologue_slices(int M, int K)
{
    const int pairs = (K + 63) / 64;
    int s = (pairs + 7) / 8;                   // 512 columns per slice: one batch of loads
    (void)M;
    if (s > kMaxHSplit) s = kMaxHSplit;
    if (s < 1) s = 1;
    const int per = (pairs + s - 1) / s;
    return (pairs + per - 1) / per;
}

hipError_t launch_prologue(ProParams &p, _Float16 *const *h16, hipStream_t st)
{
    p.pairs = (p.K + 63) / 64;
    p.S = prologue_slices(p.M, p.K);
    p.pairs_per_slice = (p.pairs + p.S - 1) / p.S;
    int jobs = 0;
    bool aligned = (reinterpret_cast<uintptr_t>(p.x) % 16) == 0;
    for (int g = 0; g < p.G; ++g) {
        p.job_start[g] = jobs;
        if (p.L[g].rank > 0) {
            jobs += ((p.L[g].rank + 15) / 16) * p.S;
            aligned = aligned && (reinterpret_cast<uintptr_t>(p.L[g].A) % 16) == 0;
        }
    }
    p.job_start[p.G] = jobs;
    const bool vec = (p.K % 8 == 0) && aligned;
    const dim3 grid((p.quantize ? p.M : 0) + (jobs + 3) / 4), block(256);
    if (grid.x == 0) return hipSuccess;             // nothing to quantise, no correction path
    const int tt = (p.M + 15) / 16;
#define HGF_PRO(TT_)                                                                        \
    if (vec) hipLaunchKernelGGL((prologue_kernel<TT_, true>), grid, block, 0, st, p);       \
    else hipLaunchKernelGGL((prologue_kernel<TT_, false>), grid, block, 0, st, p)
    switch (tt) {
        case 1: HGF_PRO(1); break;
        case 2: HGF_PRO(2); break;
        case 3: HGF_PRO(3); break;
        default: HGF_PRO(4); break;
    }
#undef HGF_PRO
    if (h16 == nullptr) return hipGetLastError();   // the consumer adds the slices itself
    ReduceParams rp;
    rp.M = p.M;
    rp.S = p.S;
    rp.G = p.G;
    int total = 0;
    for (int g = 0; g < kMaxGroup; ++g) {
        rp.start[g] = total;
        rp.hpart[g] = g < p.G ? p.L[g].hpart : nullptr;
        rp.h16[g] = g < p.G ? h16[g] : nullptr;
        rp.rank[g] = g < p.G ? p.L[g].rank : 0;
        rp.rp[g] = g < p.G ? p.L[g].rp : 32;
        if (g < p.G && p.L[g].rank > 0) total += p.M * p.L[g].rp;
    }
    rp.start[kMaxGroup] = total;
    for (int g = p.G; g <= kMaxGroup; ++g) rp.start[g] = total;
    if (total > 0) hipLaunchKernelGGL(hreduce_kernel, dim3((total + 255) / 256), dim3(256), 0, st, rp);
    return hipGetLastError();
}

}  // namespace hgf
