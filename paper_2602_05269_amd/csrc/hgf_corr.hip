// Down-projection of the correction path: h16[m, j] = fp16( SiLU( sum_k A[j,k] x[m,k] ) ).
//
// Algorithm 1, steps 5-6 of the HGF paper (H <- X A; H <- SiLU(H)) on the UN-quantised
// fp16 activations, with SiLU(h) = h * sigmoid(h) (Sec. 2.3, low-rank correction).
// fp16 operands, fp32 accumulation on the 16x16x32 f16 MFMA: matrix rows are rank
// indices, matrix columns are tokens.  One wavefront owns one tile of 16 tokens and one
// slice of d_in and computes every rank tile for it, so x is read once.  With more than
// one slice the partial sums go to scratch and the last wavefront to arrive for a token
// tile adds them in slice order (deterministic), applies SiLU and writes fp16.
#include "hgf_internal.h"

namespace hgf {

namespace {

struct CorrParams {
    const _Float16 *x;
    const _Float16 *A;
    _Float16 *h16;
    float *hpart;
    int32_t *counters;
    int M, K, rank, hstride;
    int splits, ksteps, ksteps_per_split;   // k-steps of 32 columns
};

__device__ inline float silu(float h) { return h / (1.0f + expf(-h)); }

template <bool VEC>
__device__ inline v8h load8(const _Float16 *row, int k0, int K, bool row_ok)
{
    v8h v = {0, 0, 0, 0, 0, 0, 0, 0};
    if (!row_ok) return v;
    if (VEC) {
        if (k0 < K) v = *reinterpret_cast<const v8h *>(row + k0);   // K % 8 == 0: whole vector in range
    } else {
#pragma unroll
        for (int e = 0; e < 8; ++e)
            if (k0 + e < K) v[e] = row[k0 + e];
    }
    return v;
}

template <int RTN, bool VEC>
__global__ __launch_bounds__(64) void corr_down_kernel(CorrParams p)
{
    const int tt = blockIdx.x / p.splits, sp = blockIdx.x % p.splits;
    const int l = threadIdx.x, i = l & 15, kb = l >> 4;
    const int m = tt * 16 + i;
    const bool m_ok = m < p.M;
    const _Float16 *xrow = p.x + (size_t)(m_ok ? m : 0) * p.K;

    v4f acc[RTN];
#pragma unroll
    for (int rt = 0; rt < RTN; ++rt) acc[rt] = (v4f){0.f, 0.f, 0.f, 0.f};

    const int ks0 = sp * p.ksteps_per_split;
    const int ks1 = min(ks0 + p.ksteps_per_split, p.ksteps);
    for (int ks = ks0; ks < ks1; ++ks) {
        const int k0 = ks * 32 + kb * 8;
        const v8h b = load8<VEC>(xrow, k0, p.K, m_ok);
#pragma unroll
        for (int rt = 0; rt < RTN; ++rt) {
            const int j = rt * 16 + i;
            const bool j_ok = j < p.rank;
            const v8h a = load8<VEC>(p.A + (size_t)(j_ok ? j : 0) * p.K, k0, p.K, j_ok);
            acc[rt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, acc[rt], 0, 0, 0);
        }
    }

    // acc[rt][v] holds rank index rt*16 + 4*(l/16) + v for token tt*16 + (l%16)
    if (p.splits > 1) {
        // Partial sums cross workgroups (and XCDs, whose L2 caches are not coherent with each
        // other) as device-scope atomic stores and loads, which go to the point of coherence:
        // no cache write-back or invalidate.  The arrival counter moves once they are acknowledged.
        const int ntt = gridDim.x / p.splits;
        float *mine = p.hpart + ((size_t)(sp * ntt + tt) * RTN) * 256;
#pragma unroll
        for (int rt = 0; rt < RTN; ++rt)
#pragma unroll
            for (int v = 0; v < 4; ++v)
                __hip_atomic_store(&mine[(rt * 4 + v) * 64 + l], acc[rt][v], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        __builtin_amdgcn_s_waitcnt(0);
        int old = 0;
        if (l == 0) old = __hip_atomic_fetch_add(&p.counters[tt], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        old = __shfl(old, 0, 64);
        if (old != p.splits - 1) return;
        if (l == 0) __hip_atomic_exchange(&p.counters[tt], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
        for (int rt = 0; rt < RTN; ++rt) acc[rt] = (v4f){0.f, 0.f, 0.f, 0.f};
        for (int s = 0; s < p.splits; ++s) {
            const float *part = p.hpart + ((size_t)(s * ntt + tt) * RTN) * 256;
#pragma unroll
            for (int rt = 0; rt < RTN; ++rt)
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    acc[rt][v] += __hip_atomic_load(&part[(rt * 4 + v) * 64 + l], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }

    if (!m_ok) return;
    _Float16 *hrow = p.h16 + (size_t)m * p.hstride;
#pragma unroll
    for (int rt = 0; rt < RTN; ++rt) {
        const int j0 = rt * 16 + 4 * kb;
        v4h o;
#pragma unroll
        for (int v = 0; v < 4; ++v) o[v] = (j0 + v < p.rank) ? (_Float16)silu(acc[rt][v]) : (_Float16)0.0f;
        *reinterpret_cast<v4h *>(hrow + j0) = o;
    }
    if (RTN * 16 < p.hstride) {   // rank <= 16: the upper half of the 32-wide row is padding
        v4h z = {0, 0, 0, 0};
        *reinterpret_cast<v4h *>(hrow + 16 + 4 * kb) = z;
    }
}

template <int RTN>
hipError_t launch_rtn(const CorrParams &p, int grid, bool vec, hipStream_t st)
{
    if (vec)
        hipLaunchKernelGGL((corr_down_kernel<RTN, true>), dim3(grid), dim3(64), 0, st, p);
    else
        hipLaunchKernelGGL((corr_down_kernel<RTN, false>), dim3(grid), dim3(64), 0, st, p);
    return hipGetLastError();
}

}  // namespace

// Number of d_in slices the launcher uses (also sizes the scratch for the partial sums).
int corr_splits(int M, int K)
{
    const int ntt = (M + 15) / 16;
    const int ksteps = (K + 31) / 32;
    if (ntt > kNumCounters / 2) return 1;
    int s = (768 + ntt - 1) / ntt;          // aim at ~768 wavefronts
    if (s > kMaxHSplit) s = kMaxHSplit;
    if (s > ksteps / 2) s = ksteps / 2;     // at least two k-steps per slice
    if (s < 1) s = 1;
    const int per = (ksteps + s - 1) / s;
    return (ksteps + per - 1) / per;
}

size_t corr_scratch_bytes(int M, int K, int rank)
{
    if (rank <= 0) return 0;
    const int s = corr_splits(M, K);
    if (s == 1) return 0;
    return (size_t)s * ((M + 15) / 16) * h_rank_tiles(rank) * 64 * sizeof(v4f);
}

hipError_t launch_corr_down(const _Float16 *x, int M, int K, const _Float16 *A, int rank, const Workspace &ws,
                            hipStream_t st)
{
    CorrParams p;
    p.x = x;
    p.A = A;
    p.h16 = ws.h16;
    p.hpart = ws.hpart;
    p.counters = ws.counters + kNumCounters / 2;
    p.M = M;
    p.K = K;
    p.rank = rank;
    p.hstride = h_stride(rank);
    p.ksteps = (K + 31) / 32;
    p.splits = corr_splits(M, K);
    p.ksteps_per_split = (p.ksteps + p.splits - 1) / p.splits;
    const int ntt = (M + 15) / 16;
    const int grid = ntt * p.splits;
    const bool vec = (K % 8 == 0) && ((reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(A)) % 16 == 0);
    switch (h_rank_tiles(rank)) {
        case 1: return launch_rtn<1>(p, grid, vec, st);
        case 2: return launch_rtn<2>(p, grid, vec, st);
        case 4: return launch_rtn<4>(p, grid, vec, st);
        default: return launch_rtn<8>(p, grid, vec, st);
    }
}

}  // namespace hgf
