// Decode kernel (M <= 64 per launch column): packed ternary weights x int8 activations,
// fused with dequantisation, the rank-r up-projection and the gate.
//
// Algorithm 1 of the HGF paper, steps 3, 4, 7 and 8:
//   acc[m,n] = sum_k T[n,k] x_q[m,k]                       (exact int32)
//   y[m,n]   = acc * (s_x[m] s_w) + tanh(alpha[n]) * sum_j B[n,j] h[m,j]
// The weights are streamed from HBM exactly once with 16-byte loads per lane (1 KiB per
// wavefront instruction, one 64x64 tile); the 2-bit codes are widened to int8 in
// registers (a shift and a mask per four codes) and contracted on the 16x16x64 int8 MFMA
// with the 16 weight rows as matrix rows and up to 16 tokens as matrix columns.  Codes are
// T+1, so the MFMA accumulates sum (T+1) x_q and the per-token sum of x_q is subtracted
// once at the end: integer-exact, no per-weight subtract.
//
// Work split: one workgroup of four wavefronts per (row-block of 64 rows, slice of d_in);
// the wavefronts take the slice's tiles round-robin and add their partial tiles through
// LDS.  With more than one slice per row-block the partial sums are added into a zeroed
// int32 scratch with device-scope atomics (integer addition: order does not matter) and
// the last workgroup to arrive for the row-block swaps them back out (leaving zeros) and
// runs the epilogue.
#include "hgf_internal.h"

namespace hgf {

namespace {

struct DecodeParams {
    const v4u *packed;
    const int8_t *xq;
    const float *s_x;
    const int32_t *rowsum;
    const float *s_w;
    const _Float16 *B;
    const _Float16 *alpha;
    const _Float16 *h16;
    _Float16 *y;
    int32_t *acc_debug;
    int32_t *acc_ws;
    int32_t *counters;
    int M, N, Np, Kp, KS;
    int rank, hstride;
    int splits, ks_per_split;
};

template <int TT> struct ChunkOf { static constexpr int value = TT == 1 ? 32 : (TT == 2 ? 16 : 8); };

__device__ inline v4i widen_codes(uint32_t w)
{
    v4i a;
    a[0] = (int)(w & 0x03030303u);
    a[1] = (int)((w >> 2) & 0x03030303u);
    a[2] = (int)((w >> 4) & 0x03030303u);
    a[3] = (int)((w >> 6) & 0x03030303u);
    return a;
}

template <int TT>
__global__ __launch_bounds__(256) void decode_kernel(DecodeParams p)
{
    constexpr int CH = ChunkOf<TT>::value;         // k-steps staged in LDS at a time
    constexpr int ROWS = 16 * TT;                  // token rows staged
    constexpr int STRIDE = CH * 64 + 16;           // bytes per staged row (+16: bank spread)
    constexpr int STAGE_BYTES = ROWS * STRIDE;
    constexpr int RED_BYTES = 4 * 3 * TT * 64 * 16;
    constexpr int LDS_BYTES = STAGE_BYTES > RED_BYTES ? STAGE_BYTES : RED_BYTES;
    __shared__ __attribute__((aligned(16))) unsigned char lds[LDS_BYTES];
    __shared__ int sh_last;

    const int tid = threadIdx.x, w = tid >> 6, l = tid & 63;
    const int rb = blockIdx.x / p.splits, sp = blockIdx.x % p.splits;
    const int m0 = blockIdx.y * kMaxDecodeM;       // first token of this launch column
    const int mcount = min(p.M - m0, ROWS);
    const int ks0 = sp * p.ks_per_split;
    const int ks1 = min(ks0 + p.ks_per_split, p.KS);

    v4i acc[4][TT];
#pragma unroll
    for (int rt = 0; rt < 4; ++rt)
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) acc[rt][tt] = (v4i){0, 0, 0, 0};

    const v4u *tiles = p.packed + (size_t)rb * p.KS * 64 + l;   // + ks*64 per tile

    for (int c0 = ks0; c0 < ks1; c0 += CH) {
        const int nks = min(CH, ks1 - c0);
        // this wavefront's tiles of the chunk: issue every load before touching LDS
        v4u wq[CH / 4];
#pragma unroll
        for (int t = 0; t < CH / 4; ++t) {
            const int ks = c0 + w + 4 * t;
            wq[t] = (v4u){0x55555555u, 0x55555555u, 0x55555555u, 0x55555555u};
            if (ks < c0 + nks) wq[t] = __builtin_nontemporal_load(&tiles[(size_t)ks * 64]);
        }
        __syncthreads();                            // the previous chunk's reads are done
        const int pieces_per_row = nks * 4;         // 16-byte pieces
        for (int pc = tid; pc < ROWS * pieces_per_row; pc += 256) {
            const int row = pc / pieces_per_row, col = pc % pieces_per_row;
            uint4 v = make_uint4(0, 0, 0, 0);
            if (row < mcount)
                v = *reinterpret_cast<const uint4 *>(p.xq + (size_t)(m0 + row) * p.Kp + (size_t)c0 * 64 + col * 16);
            *reinterpret_cast<uint4 *>(lds + row * STRIDE + col * 16) = v;
        }
        __syncthreads();
#pragma unroll
        for (int t = 0; t < CH / 4; ++t) {
            const int kl = w + 4 * t;               // k-step within the chunk
            if (kl < nks) {
                v4i b[TT];
#pragma unroll
                for (int tt = 0; tt < TT; ++tt)
                    b[tt] = *reinterpret_cast<const v4i *>(lds + (tt * 16 + (l & 15)) * STRIDE + kl * 64 + (l >> 4) * 16);
#pragma unroll
                for (int rt = 0; rt < 4; ++rt) {
                    const v4i a = widen_codes(wq[t][rt]);
#pragma unroll
                    for (int tt = 0; tt < TT; ++tt)
                        acc[rt][tt] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, b[tt], acc[rt][tt], 0, 0, 0);
                }
            }
        }
    }

    // ---- add the four wavefronts' partial tiles: wavefront w ends up owning row tile w
    __syncthreads();
    {
        v4i *red = reinterpret_cast<v4i *>(lds);
#pragma unroll
        for (int rt = 0; rt < 4; ++rt) {
            if (rt != w) {
                const int slot = rt < w ? rt : rt - 1;
#pragma unroll
                for (int tt = 0; tt < TT; ++tt) red[((w * 3 + slot) * TT + tt) * 64 + l] = acc[rt][tt];
            }
        }
        __syncthreads();
    }
    v4i mine[TT];
    {
        const v4i *red = reinterpret_cast<const v4i *>(lds);
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) {
            v4i s = (v4i){0, 0, 0, 0};
#pragma unroll
            for (int rt = 0; rt < 4; ++rt)          // select acc[w][tt] without dynamic indexing
                if (rt == w) s = acc[rt][tt];
#pragma unroll
            for (int ws = 0; ws < 4; ++ws) {
                if (ws != w) {
                    const int slot = w < ws ? w : w - 1;
                    s += red[((ws * 3 + slot) * TT + tt) * 64 + l];
                }
            }
            mine[tt] = s;
        }
    }

    const int n0 = rb * 64 + w * 16;                // this wavefront's 16 output rows
    const int nl = n0 + 4 * (l >> 4);               // this lane's 4 consecutive rows
    const int ml = l & 15;                          // this lane's token within a token tile

    if (p.splits > 1) {
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) {
            const int m = tt * 16 + ml;
            if (m < mcount) {
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    __hip_atomic_fetch_add(&p.acc_ws[(size_t)m * p.Np + nl + v], mine[tt][v], __ATOMIC_RELAXED,
                                           __HIP_MEMORY_SCOPE_AGENT);
            }
        }
        __threadfence();
        __syncthreads();
        if (tid == 0) {
            const int old = __hip_atomic_fetch_add(&p.counters[rb], 1, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
            const int last = old == p.splits - 1;
            if (last) __hip_atomic_exchange(&p.counters[rb], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            sh_last = last;
        }
        __syncthreads();
        if (!sh_last) return;
        __threadfence();
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) {
            const int m = tt * 16 + ml;
            if (m < mcount) {
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    mine[tt][v] = __hip_atomic_exchange(&p.acc_ws[(size_t)m * p.Np + nl + v], 0, __ATOMIC_RELAXED,
                                                        __HIP_MEMORY_SCOPE_AGENT);
            }
        }
    }

    if (n0 >= p.N) return;                          // padding rows only

    // ---- correction up-projection: corr[m,n] = sum_j B[n,j] h[m,j] on the f16 MFMA
    v4f corr[TT];
#pragma unroll
    for (int tt = 0; tt < TT; ++tt) corr[tt] = (v4f){0.f, 0.f, 0.f, 0.f};
    if (p.rank > 0) {
        const int brow = n0 + (l & 15);
        const bool brow_ok = brow < p.N;
        const _Float16 *bptr = p.B + (size_t)(brow_ok ? brow : 0) * p.rank;
        const bool bvec = (p.rank % 8) == 0;
        for (int js = 0; js < p.hstride / 32; ++js) {
            const int j0 = js * 32 + (l >> 4) * 8;
            v8h a = {0, 0, 0, 0, 0, 0, 0, 0};
            if (brow_ok) {
                if (bvec) {
                    if (j0 < p.rank) a = *reinterpret_cast<const v8h *>(bptr + j0);
                } else {
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        if (j0 + e < p.rank) a[e] = bptr[j0 + e];
                }
            }
#pragma unroll
            for (int tt = 0; tt < TT; ++tt) {
                const int m = tt * 16 + ml;
                v8h b = {0, 0, 0, 0, 0, 0, 0, 0};
                if (m < mcount) b = *reinterpret_cast<const v8h *>(p.h16 + (size_t)(m0 + m) * p.hstride + j0);
                corr[tt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, corr[tt], 0, 0, 0);
            }
        }
    }

    // ---- dequantise, gate, store
    const float s_w = *p.s_w;
    float g[4] = {0.f, 0.f, 0.f, 0.f};
    if (p.rank > 0) {
#pragma unroll
        for (int v = 0; v < 4; ++v)
            if (nl + v < p.N) g[v] = tanhf((float)p.alpha[nl + v]);
    }
    const bool nvec = (p.N % 4) == 0;
#pragma unroll
    for (int tt = 0; tt < TT; ++tt) {
        const int m = tt * 16 + ml;
        if (m >= mcount) continue;
        const size_t mg = (size_t)(m0 + m);
        const float scale = p.s_x[mg] * s_w;
        const int rs = p.rowsum[mg];
        int a[4];
        v4h o;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            a[v] = mine[tt][v] - rs;
            o[v] = (_Float16)((float)a[v] * scale + g[v] * corr[tt][v]);
        }
        if (nvec && nl + 3 < p.N) {
            *reinterpret_cast<v4h *>(p.y + mg * p.N + nl) = o;
            if (p.acc_debug) *reinterpret_cast<v4i *>(p.acc_debug + mg * p.N + nl) = (v4i){a[0], a[1], a[2], a[3]};
        } else {
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                if (nl + v < p.N) {
                    p.y[mg * p.N + nl + v] = o[v];
                    if (p.acc_debug) p.acc_debug[mg * p.N + nl + v] = a[v];
                }
            }
        }
    }
}

int g_target_wgs = 512;

}  // namespace

void set_decode_target_wgs(int v) { g_target_wgs = v > 0 ? v : 512; }

hipError_t launch_decode(const Workspace &ws, int M, const hgf_layer &L, _Float16 *y, int32_t *acc_debug,
                         hipStream_t st)
{
    DecodeParams p;
    p.packed = reinterpret_cast<const v4u *>(L.W_packed);
    p.xq = ws.xq;
    p.s_x = ws.s_x;
    p.rowsum = ws.rowsum;
    p.s_w = L.s_w;
    p.B = reinterpret_cast<const _Float16 *>(L.B_f16);
    p.alpha = reinterpret_cast<const _Float16 *>(L.alpha_f16);
    p.h16 = ws.h16;
    p.y = y;
    p.acc_debug = acc_debug;
    p.acc_ws = ws.acc;
    p.counters = ws.counters;
    p.M = M;
    p.N = L.d_out;
    p.Np = round_up(L.d_out, kTile);
    p.Kp = round_up(L.d_in, kTile);
    p.KS = p.Kp / kTile;
    p.rank = L.rank;
    p.hstride = h_stride(L.rank);

    const int RB = p.Np / kTile;
    const int cols = (M + kMaxDecodeM - 1) / kMaxDecodeM;
    int splits = 1;
    const bool can_split = cols == 1 && RB <= kNumCounters / 2 &&
                           (size_t)round_up(M, 16) * p.Np * sizeof(int32_t) <= kAccZeroBytes;
    if (can_split) {
        splits = (g_target_wgs + RB - 1) / RB;
        if (splits > p.KS / 4) splits = p.KS / 4;   // at least one tile per wavefront
        if (splits < 1) splits = 1;
    }
    p.ks_per_split = (p.KS + splits - 1) / splits;
    p.splits = (p.KS + p.ks_per_split - 1) / p.ks_per_split;

    const dim3 grid(RB * p.splits, cols), block(256);
    const int mt = cols > 1 ? 4 : (M + 15) / 16;
    switch (mt) {
        case 1: hipLaunchKernelGGL(decode_kernel<1>, grid, block, 0, st, p); break;
        case 2: hipLaunchKernelGGL(decode_kernel<2>, grid, block, 0, st, p); break;
        case 3: hipLaunchKernelGGL(decode_kernel<3>, grid, block, 0, st, p); break;
        default: hipLaunchKernelGGL(decode_kernel<4>, grid, block, 0, st, p); break;
    }
    return hipGetLastError();
}

// Until the dedicated MFMA prefill kernel lands, large M runs as columns of 64 tokens.
hipError_t launch_prefill(const Workspace &ws, int M, const hgf_layer &L, _Float16 *y, int32_t *acc_debug,
                          hipStream_t st)
{
    return launch_decode(ws, M, L, y, acc_debug, st);
}

}  // namespace hgf
