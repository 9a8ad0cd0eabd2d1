// Decode kernel (up to 64 tokens per launch column): packed ternary weights x int8
// activations, fused with dequantisation, the rank-r up-projection and the gate.
//
// Algorithm 1 of the HGF paper, steps 3, 4, 7 and 8:
//   acc[m,n] = sum_k T[n,k] x_q[m,k]                       (exact int32)
//   y[m,n]   = acc * (s_x[m] s_w) + tanh(alpha[n]) * sum_j B[n,j] h[m,j]
// The weights are streamed from HBM exactly once with 16-byte loads per lane: one
// wavefront instruction fetches one 1 KiB tile (16 rows x 256 columns).  The 2-bit codes
// are widened to int8 in registers (a shift and a mask per four codes) and contracted on
// the 16x16x64 int8 MFMA with the 16 weight rows as matrix rows and up to 16 tokens as
// matrix columns.  Codes are T+1, so the MFMA accumulates sum (T+1) x_q and the per-token
// sum of x_q is subtracted once at the end: integer-exact, no per-weight subtract.
//
// Work split: a workgroup of four wavefronts covers RW row-blocks of 16 rows, with KW =
// 4/RW wavefronts sharing each row-block's tiles round-robin along d_in and adding their
// partial tiles through LDS.  The quantised activations of the current stretch of d_in
// sit in LDS, shared by the four wavefronts; only lanes whose token exists read them.
// Every wavefront issues all weight loads of a batch before it consumes the first, so a
// compute unit keeps tens of KiB in flight.  Nothing crosses workgroups: no atomics.
#include "hgf_internal.h"

namespace hgf {

namespace {

__device__ inline v4i widen_codes(uint32_t w)
{
    v4i a;
    a[0] = (int)(w & 0x03030303u);
    a[1] = (int)((w >> 2) & 0x03030303u);
    a[2] = (int)((w >> 4) & 0x03030303u);
    a[3] = (int)((w >> 6) & 0x03030303u);
    return a;
}

__device__ inline float silu(float h) { return h / (1.0f + expf(-h)); }

template <int TT>
__global__ __launch_bounds__(256) void decode_kernel(DecodeParams p)
{
#ifndef HGF_PF1
#define HGF_PF1 8
#endif
    constexpr int PF = TT == 1 ? HGF_PF1 : (TT == 2 ? 8 : 4);   // weight tiles in flight per wavefront
    constexpr int XPRE = 4;                                 // activation pieces per thread fetched up front
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];

    const int tid = threadIdx.x, l = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    // this workgroup's layer: every candidate is read at a fixed kernel-argument offset (one
    // batch of scalar loads) and selected, instead of a dependent load at a computed offset
    DecLayer L = p.L[0];
    int wg0 = 0;
#pragma unroll
    for (int i = 1; i < kMaxGroup; ++i) {
        if (i < p.G && (int)blockIdx.x >= p.wg_start[i]) {
            L = p.L[i];
            wg0 = p.wg_start[i];
        }
    }
    const int rw = w / p.KW, kw = w % p.KW;
    const int rb = ((int)blockIdx.x - wg0) * p.RW + rw;   // this wavefront's row-block
    const bool rb_ok = rb < L.RBn;
    const int m0 = blockIdx.y * kMaxDecodeM;        // first token of this launch column
    const int mcount = min(p.M - m0, 16 * TT);
    const int ml = l & 15, kb = l >> 4;
    const int n0 = rb * kTileRows;                   // this wavefront's 16 output rows
    const int nl = n0 + 4 * kb;                      // this lane's 4 consecutive rows
    const bool owner = rb_ok && kw == 0;             // runs the epilogue of the row-block

    // Loads are issued smallest and most urgent first, the weight stream last, all without
    // branches, so that everything is in flight together and the small results can be
    // consumed while the weights are still arriving.

    // ---- (1) partial sums of A x for the first element this thread turns into SiLU(A x)
    const rsrc_t hr = p.hmode == 0 ? make_rsrc(L.hpart, (unsigned)p.S * p.M * L.hstride * 4u)
                                   : make_rsrc(L.h16, (unsigned)p.M * L.hstride * 2u);
    const int htotal = L.rank > 0 ? mcount * L.hstride : 0;
    float hpre[kMaxHSplit];
    {
        const int m = tid / L.hstride, j = tid - m * L.hstride;
        const bool ok = tid < htotal && j < L.rank;
        const unsigned row = (unsigned)(m0 + m) * L.hstride + j;
        if (p.hmode == 0) {
#pragma unroll
            for (int sp = 0; sp < kMaxHSplit; ++sp)
                hpre[sp] = __builtin_bit_cast(float, buf_load4(hr, (row + (unsigned)sp * p.M * L.hstride) * 4u,
                                                               ok && sp < p.S));
        } else {
            hpre[0] = (float)half_bits(buf_load2(hr, row * 2u, ok));
        }
    }

    // ---- (2) the first pieces of the quantised activations (16 bytes each)
    const int cend0 = min(p.CT, p.KT);
    const rsrc_t xr = make_rsrc(p.xq + (size_t)m0 * p.Kp, (unsigned)mcount * p.Kp);
    v4u xpre[XPRE];
    {
        const int pieces_per_row = cend0 * 16;
        const int total = mcount * pieces_per_row;
#pragma unroll
        for (int u = 0; u < XPRE; ++u) {
            const int pc = tid + u * 256;
            const int row = pc / pieces_per_row, col = pc - row * pieces_per_row;
            xpre[u] = buf_load16(xr, (unsigned)row * p.Kp + col * 16, pc < total);
        }
    }

    // ---- (3) epilogue operands of the wavefront that owns the row-block
    constexpr int JS = HGF_MAX_RANK / 32;
    v8h breg[JS];
    float alpha_f[4];
    {
        const rsrc_t br = make_rsrc(L.B, L.rank > 0 ? (unsigned)L.N * L.rank * 2u : 0u);
        const rsrc_t ar = make_rsrc(L.alpha, L.rank > 0 ? (unsigned)L.N * 2u : 0u);
        const int brow = n0 + ml;
        const bool brow_ok = owner && brow < L.N;
        const bool bvec = (L.rank % 8) == 0;
#pragma unroll
        for (int js = 0; js < JS; ++js) {
            const int j0 = js * 32 + kb * 8;
            breg[js] = bvec ? buf_load8h<true>(br, (unsigned)brow * L.rank + j0, L.rank - j0, brow_ok)
                            : buf_load8h<false>(br, (unsigned)brow * L.rank + j0, L.rank - j0, brow_ok);
        }
#pragma unroll
        for (int v = 0; v < 4; ++v) alpha_f[v] = (float)half_bits(buf_load2(ar, (unsigned)(nl + v) * 2u, owner && nl + v < L.N));
    }
    const float s_w = *L.s_w;
    float sx_pre[TT];
    int rs_pre[TT];
    {
        const rsrc_t sr = make_rsrc(p.s_x + m0, (unsigned)mcount * 4u);
        const rsrc_t rr = make_rsrc(p.rowsum + m0, (unsigned)mcount * 4u);
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) {
            sx_pre[tt] = __builtin_bit_cast(float, buf_load4(sr, (unsigned)(tt * 16 + ml) * 4u, owner));
            rs_pre[tt] = (int)buf_load4(rr, (unsigned)(tt * 16 + ml) * 4u, owner);
        }
    }

    // ---- (4) first batch of weight tiles: the bulk of the bytes
    const v4u *rb_tiles = L.packed + (size_t)(rb_ok ? rb : 0) * p.KT * 64;
    int kt0 = kw;
    int cend = cend0;
    v4u wq[PF];
    {
        const rsrc_t wr = make_rsrc(rb_tiles, rb_ok ? (unsigned)cend * kTileBytes : 0u);
#pragma unroll
        for (int t = 0; t < PF; ++t) wq[t] = buf_load16_stream(wr, (unsigned)(kt0 + t * p.KW) * kTileBytes + l * 16);
    }

    // ---- SiLU(A x) of this launch column's tokens into LDS (fp16 rows of hstride)
    _Float16 *hs = reinterpret_cast<_Float16 *>(lds + p.h_off);
    if (tid < htotal) {
        float h = hpre[0];
        if (p.hmode == 0) {
#pragma unroll
            for (int sp = 1; sp < kMaxHSplit; ++sp) h += hpre[sp];   // slice order: deterministic
            h = silu(h);
        }
        hs[tid] = (_Float16)h;
    }
    for (int idx = tid + 256; idx < htotal; idx += 256) {            // more than 256 elements: M*hstride > 256
        const int m = idx / L.hstride, j = idx - m * L.hstride;
        const unsigned row = (unsigned)(m0 + m) * L.hstride + j;
        float h = 0.f;
        if (p.hmode == 0) {
            float part[kMaxHSplit];
#pragma unroll
            for (int sp = 0; sp < kMaxHSplit; ++sp)
                part[sp] = __builtin_bit_cast(float, buf_load4(hr, (row + (unsigned)sp * p.M * L.hstride) * 4u,
                                                               j < L.rank && sp < p.S));
#pragma unroll
            for (int sp = 0; sp < kMaxHSplit; ++sp) h += part[sp];
            h = silu(h);
        } else {
            h = (float)half_bits(buf_load2(hr, row * 2u, j < L.rank));
        }
        hs[idx] = (_Float16)h;
    }

    v4i acc[TT];
#pragma unroll
    for (int tt = 0; tt < TT; ++tt) acc[tt] = (v4i){0, 0, 0, 0};

    for (int c0 = 0; c0 < p.KT; c0 += p.CT) {        // stretches of d_in staged in LDS
        cend = min(c0 + p.CT, p.KT);
        if (c0 > 0) {
            kt0 = c0 + kw;
            const rsrc_t wr = make_rsrc(rb_tiles, rb_ok ? (unsigned)cend * kTileBytes : 0u);
#pragma unroll
            for (int t = 0; t < PF; ++t) wq[t] = buf_load16_stream(wr, (unsigned)(kt0 + t * p.KW) * kTileBytes + l * 16);
            __syncthreads();                         // the previous stretch has been consumed
        }
        {   // stage x_q[:, c0*256 .. cend*256) into LDS, 16 bytes per thread and step
            const int pieces_per_row = (cend - c0) * 16;
            const int total = mcount * pieces_per_row;
            int first = 0;
            if (c0 == 0) {
#pragma unroll
                for (int u = 0; u < XPRE; ++u) {
                    const int pc = tid + u * 256;
                    const int row = pc / pieces_per_row, col = pc - row * pieces_per_row;
                    if (pc < total) *reinterpret_cast<v4u *>(lds + row * p.xstride + col * 16) = xpre[u];
                }
                first = XPRE * 256;
            }
            for (int pc = first + tid; pc < total; pc += 256) {
                const int row = pc / pieces_per_row, col = pc - row * pieces_per_row;
                const v4u v = buf_load16(xr, (unsigned)row * p.Kp + (unsigned)c0 * kTileCols + col * 16);
                *reinterpret_cast<v4u *>(lds + row * p.xstride + col * 16) = v;
            }
        }
        __syncthreads();
        while (true) {
#pragma unroll
            for (int t = 0; t < PF; ++t) {
                const int kt = kt0 + t * p.KW;
                if (kt < cend) {
                    const unsigned char *xrow = lds + (kt - c0) * kTileCols + kb * 16;
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const v4i a = widen_codes(wq[t][q]);
#pragma unroll
                        for (int tt = 0; tt < TT; ++tt) {
                            v4i b = (v4i){0, 0, 0, 0};
                            if (tt * 16 + ml < mcount)
                                b = *reinterpret_cast<const v4i *>(xrow + (tt * 16 + ml) * p.xstride + q * 64);
                            acc[tt] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, b, acc[tt], 0, 0, 0);
                        }
                    }
                }
            }
            kt0 += p.KW * PF;
            if (kt0 >= cend) break;
            const rsrc_t wr = make_rsrc(rb_tiles, rb_ok ? (unsigned)cend * kTileBytes : 0u);
#pragma unroll
            for (int t = 0; t < PF; ++t) wq[t] = buf_load16_stream(wr, (unsigned)(kt0 + t * p.KW) * kTileBytes + l * 16);
        }
    }

    // ---- add the KW partial tiles of a row-block: its first wavefront ends up owning it
    if (p.KW > 1) {
        __syncthreads();                             // the activations in LDS are no longer needed
        v4i *red = reinterpret_cast<v4i *>(lds);
        if (kw > 0) {
#pragma unroll
            for (int tt = 0; tt < TT; ++tt) red[((w * TT) + tt) * 64 + l] = acc[tt];
        }
        __syncthreads();
        if (kw > 0) return;
        for (int o = 1; o < p.KW; ++o) {
#pragma unroll
            for (int tt = 0; tt < TT; ++tt) acc[tt] += red[(((w + o) * TT) + tt) * 64 + l];
        }
    }
    if (!rb_ok || n0 >= L.N) return;

    // ---- correction up-projection: corr[m,n] = sum_j B[n,j] h[m,j] on the f16 MFMA
    v4f corr[TT];
#pragma unroll
    for (int tt = 0; tt < TT; ++tt) corr[tt] = (v4f){0.f, 0.f, 0.f, 0.f};
    if (L.rank > 0) {
#pragma unroll
        for (int js = 0; js < JS; ++js) {
            if (js * 32 < L.hstride) {
                const int j0 = js * 32 + kb * 8;
#pragma unroll
                for (int tt = 0; tt < TT; ++tt) {
                    const int m = tt * 16 + ml;
                    v8h b = {0, 0, 0, 0, 0, 0, 0, 0};
                    if (m < mcount) b = *reinterpret_cast<const v8h *>(hs + m * L.hstride + j0);
                    corr[tt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(breg[js], b, corr[tt], 0, 0, 0);
                }
            }
        }
    }

    // ---- dequantise, gate, store
    float gate[4];
#pragma unroll
    for (int v = 0; v < 4; ++v) gate[v] = L.rank > 0 ? tanhf(alpha_f[v]) : 0.f;
    const bool nvec = (L.N % 4) == 0;
#pragma unroll
    for (int tt = 0; tt < TT; ++tt) {
        const int m = tt * 16 + ml;
        if (m >= mcount) continue;
        const size_t mg = (size_t)(m0 + m);
        const float scale = sx_pre[tt] * s_w;
        const int rs = rs_pre[tt];
        int a[4];
        v4h o;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            a[v] = acc[tt][v] - rs;
            o[v] = (_Float16)((float)a[v] * scale + gate[v] * corr[tt][v]);
        }
        if (nvec && nl + 3 < L.N) {
            *reinterpret_cast<v4h *>(L.y + mg * L.N + nl) = o;
            if (L.acc_debug) *reinterpret_cast<v4i *>(L.acc_debug + mg * L.N + nl) = (v4i){a[0], a[1], a[2], a[3]};
        } else {
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                if (nl + v < L.N) {
                    L.y[mg * L.N + nl + v] = o[v];
                    if (L.acc_debug) L.acc_debug[mg * L.N + nl + v] = a[v];
                }
            }
        }
    }
}

int g_target_wgs = 512;
constexpr int kDecodeLdsBudget = 64 * 1024;

}  // namespace

void set_decode_target_wgs(int v) { g_target_wgs = v > 0 ? v : 512; }

// Fills in the launch shape of a group whose layers, activations and outputs are set.
hipError_t launch_decode(DecodeParams &p, int d_in, hipStream_t st)
{
    const int M = p.M;
    p.Kp = round_up(d_in, kTileCols);
    p.KT = p.Kp / kTileCols;
    int rb_total = 0, hstride_max = 32;
    for (int g = 0; g < p.G; ++g) {
        rb_total += p.L[g].RBn;
        if (p.L[g].hstride > hstride_max) hstride_max = p.L[g].hstride;
    }
    // the widest row coverage per workgroup that still gives the chip enough workgroups
    // and leaves each wavefront a short run of tiles
    p.RW = 4;
    while (p.RW > 1 && ((rb_total + p.RW - 1) / p.RW < g_target_wgs || p.KT > 16)) p.RW /= 2;
    while (p.RW < 4 && p.KT < 4 / p.RW) p.RW *= 2;   // no more wavefronts per row-block than tiles
    p.KW = 4 / p.RW;
    int wgs = 0;
    for (int g = 0; g < p.G; ++g) {
        p.wg_start[g] = wgs;
        wgs += (p.L[g].RBn + p.RW - 1) / p.RW;
    }
    p.wg_start[p.G] = wgs;

    const int cols = (M + kMaxDecodeM - 1) / kMaxDecodeM;
    const int mrows = cols > 1 ? kMaxDecodeM : M;
    const int mt = (mrows + 15) / 16;
    const size_t hbytes = (size_t)mrows * hstride_max * sizeof(_Float16);
    // stretch of d_in staged in LDS: as long as fits the budget (whole rows for small M)
    int ct = (int)(((kDecodeLdsBudget - hbytes) / mrows - 16) / kTileCols);
    if (ct > p.KT) ct = p.KT;
    if (ct < 1) ct = 1;
    p.CT = ct;
    p.xstride = ct * kTileCols + 16;
    size_t stage = (size_t)mrows * p.xstride;
    const size_t red = (size_t)4 * mt * 64 * 16;
    if (stage < red) stage = red;
    p.h_off = (int)stage;
    const size_t lds = stage + hbytes;

    const dim3 grid(wgs, cols), block(256);
    switch (mt) {
        case 1: hipLaunchKernelGGL(decode_kernel<1>, grid, block, lds, st, p); break;
        case 2: hipLaunchKernelGGL(decode_kernel<2>, grid, block, lds, st, p); break;
        case 3: hipLaunchKernelGGL(decode_kernel<3>, grid, block, lds, st, p); break;
        default: hipLaunchKernelGGL(decode_kernel<4>, grid, block, lds, st, p); break;
    }
    return hipGetLastError();
}

}  // namespace hgf
