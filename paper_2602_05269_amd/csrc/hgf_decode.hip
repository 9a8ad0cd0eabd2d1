// Decode kernel (up to 64 tokens): packed ternary weights x int8 activations, fused with
// dequantisation, the rank-r up-projection and the gate.
//
// Algorithm 1 of the HGF paper, steps 3, 4, 6, 7 and 8:
//   acc[m,n] = sum_k T[n,k] x_q[m,k]                       (exact int32)
//   h[m,j]   = SiLU(sum over the prologue's slices of (A x)[m,j])
//   y[m,n]   = acc * (s_x[m] s_w) + tanh(alpha[n]) * sum_j B[n,j] h[m,j]
// The weights are streamed from HBM exactly once with 16-byte loads per lane: one
// wavefront instruction fetches one 1 KiB tile (32 rows x 128 columns).  The 2-bit codes
// are widened to int8 in registers (a shift and a mask per four codes) and contracted on
// the 32x32x32 int8 MFMA with the 32 weight rows as matrix rows and up to 32 tokens as
// matrix columns.  Codes are T+1, so the MFMA accumulates sum (T+1) x_q and the per-token
// sum of x_q is subtracted once at the end: integer-exact, no per-weight subtract.
//
// Work split: a workgroup covers RW row-blocks of 32 rows, with KW wavefronts sharing each
// row-block's tiles round-robin along d_in and adding their partial tiles through LDS
// (RW*KW = 4 or 8 wavefronts).  The quantised activations of the current stretch of
// d_in sit in LDS, shared by all wavefronts; only lanes whose token exists read them.
// Every load of the kernel is issued in one burst at its start, smallest first and the
// weight stream last, without branches (guards are selects on buffer-descriptor offsets),
// so that all of it is in flight together.  Nothing crosses workgroups: no atomics.
#include "hgf_internal.h"

namespace hgf {

namespace {

typedef __attribute__((address_space(3))) void *lds_ptr_t;

// TG: token groups of 32 (1 or 2).  PAIR: the gated pair of two layers (a constant of the kernel:
// the single wavefront that finishes a row-block runs the epilogue, and what it does not need
// should not be in its way).
template <int TG, bool PAIR>
__global__ __launch_bounds__(512) void decode_kernel(DecodeParams p)
{
    constexpr int PF = TG == 1 ? 6 : 4;       // weight tiles in flight per wavefront (4 ... 10 measured within 3 %; 16: 10 % slower)
    constexpr int JS = HGF_MAX_RANK / 16;           // steps of the 32x32x16 f16 MFMA over the rank
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];

    const int tid = threadIdx.x, nthreads = blockDim.x, l = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    // this workgroup's layer: every candidate is read at a fixed kernel-argument offset (one
    // batch of scalar loads) and selected, instead of a dependent load at a computed offset
    const int rw = w / p.KW, kw = w % p.KW;
    constexpr bool pair = PAIR;
    DecLayer L = p.L[0];
    int wg0 = 0;
#pragma unroll
    for (int i = 1; i < kMaxGroup; ++i) {
        if (i < p.G && (pair ? rw == i : (int)blockIdx.x >= p.wg_start[i])) {
            L = p.L[i];
            wg0 = pair ? 0 : p.wg_start[i];
        }
    }
    // first row-block of the workgroup and this wavefront's (pair: the same one in both layers)
    const int rb_first = pair ? (int)blockIdx.x : ((int)blockIdx.x - wg0) * p.RW;
    const int rb = pair ? rb_first : rb_first + rw;
    const bool rb_ok = rb < L.RBn;
    const int mcount = p.M;                          // tokens (<= 32*TG)
    const int jl = l & 31, hf = l >> 5;              // matrix column / row index, and k-half
    const int n0 = rb * kTileRows;                   // this wavefront's 32 output rows
    const bool owner = rb_ok && kw == 0;             // runs the epilogue of the row-block

    // ---- (1) the prologue's partial sums of A x, [slice][token][hstride] fp32: a thread takes four
    //      consecutive ranks of one token and adds their slices in order (Alg. 1 step 5 is complete
    //      with that sum; SiLU, step 6, follows below).  The first eight slices of its first two
    //      quadruples are requested here, with everything else of the kernel's start.
    //      (pair: each half of the workgroup brings its own layer's rows)
    constexpr int HV = 2, HS = 8;
    const int hthreads = pair ? nthreads / 2 : nthreads;
    const int htid = pair ? tid - rw * hthreads : tid;
    const int hquads = L.rank > 0 ? mcount * L.hstride / 4 : 0;
    const int hwritten = (L.rank + 15) / 16 * 16;    // ranks the prologue's tiles cover (those past the rank: zeros)
    const unsigned hslice = (unsigned)mcount * L.hstride * 4u;
    const rsrc_t hr = make_rsrc(L.hpart, L.rank > 0 ? (unsigned)p.S * hslice : 0u);
    auto hquad_ok = [&](int it) { return it < hquads && (it * 4) % L.hstride < hwritten; };
    v4f hpre[HV][HS];
#pragma unroll
    for (int u = 0; u < HV; ++u)
#pragma unroll
        for (int sl = 0; sl < HS; ++sl)
            hpre[u][sl] = __builtin_bit_cast(v4f, buf_load16(hr, (unsigned)(htid + u * hthreads) * 16u + (unsigned)sl * hslice,
                                                             hquad_ok(htid + u * hthreads) && sl < p.S));

    // ---- (2) the quantised activations of the first stretch of d_in, straight into LDS: one
    //      request moves up to 1 KiB of one token's row (the rows keep their 16 bytes of padding,
    //      so a request never crosses a row), the wavefronts take the requests in turn, and all
    //      of them are in flight together with everything below -- through registers the rows
    //      took a trip to L2 per eight pieces, which cost 0.7 us per token
    const int cend0 = min(p.CT, p.KT);
    const rsrc_t xr = make_rsrc(p.xq, (unsigned)mcount * p.Kp);
    const int nwaves = nthreads >> 6;
    auto stage_tokens = [&](int c0, int c1) __attribute__((always_inline)) {
        const int row_bytes = (c1 - c0) * kTileCols;
        const int per_row = (row_bytes + 1023) / 1024;
        for (int i = w; i < mcount * per_row; i += nwaves) {
            const int row = i / per_row, pc = i - row * per_row;
            const int at = pc * 1024 + l * 16;
            if (at < row_bytes)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(xr, (lds_ptr_t)(lds + row * p.xstride + pc * 1024), 16,
                                                         (int)((unsigned)row * p.Kp + (unsigned)c0 * kTileCols + at), 0, 0, 0);
        }
    };
    stage_tokens(0, cend0);

    // ---- (3) epilogue operands: gate parameter of the workgroup's rows, B rows and the
    //      token scales of the wavefront that owns the row-block
    float alpha_pre;
    {
        // thread t < 32 RW takes row t of the workgroup's rows; in a pair threads 0..31 take the
        // rows of layer 0 and threads 32..63 the same rows of layer 1 (two guarded requests with
        // uniform descriptors and a select: a per-lane descriptor would be a loop)
        const DecLayer &L0 = pair ? p.L[0] : L;
        const rsrc_t ar0 = make_rsrc(L0.alpha, L0.rank > 0 ? (unsigned)L0.N * 2u : 0u);
        const rsrc_t ar1 = make_rsrc(p.L[1].alpha, pair && p.L[1].rank > 0 ? (unsigned)p.L[1].N * 2u : 0u);
        const int n = rb_first * kTileRows + (pair ? (tid & (kTileRows - 1)) : tid);
        const bool first = !pair || tid < kTileRows;
        const float a0 = (float)half_bits(buf_load2(ar0, (unsigned)n * 2u, first && tid < p.RW * kTileRows && n < L0.N));
        const float a1 = (float)half_bits(buf_load2(ar1, (unsigned)n * 2u, !first && tid < p.RW * kTileRows && n < p.L[1].N));
        alpha_pre = first ? a0 : a1;
    }
    v8h breg[JS];
    {
        const rsrc_t br = make_rsrc(L.B, L.rank > 0 ? (unsigned)L.N * L.rank * 2u : 0u);
        const int brow = n0 + jl;
        const bool brow_ok = owner && brow < L.N;
        const bool bvec = (L.rank % 8) == 0;
#pragma unroll
        for (int js = 0; js < JS; ++js) {
            const int j0 = js * 16 + hf * 8;
            breg[js] = bvec ? buf_load8h<true>(br, (unsigned)brow * L.rank + j0, L.rank - j0, brow_ok)
                            : buf_load8h<false>(br, (unsigned)brow * L.rank + j0, L.rank - j0, brow_ok);
        }
    }
    const float s_w = *L.s_w;
    float sx_pre[TG];
    int rs_pre[TG];
    {
        const rsrc_t sr = make_rsrc(p.s_x, (unsigned)mcount * 4u);
        const rsrc_t rr = make_rsrc(p.rowsum, (unsigned)mcount * 4u);
#pragma unroll
        for (int tg = 0; tg < TG; ++tg) {
            sx_pre[tg] = __builtin_bit_cast(float, buf_load4(sr, (unsigned)(tg * 32 + jl) * 4u, owner));
            rs_pre[tg] = (int)buf_load4(rr, (unsigned)(tg * 32 + jl) * 4u, owner);
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

    // ---- SiLU(A x) of the tokens and tanh(alpha) into LDS
    _Float16 *hs = reinterpret_cast<_Float16 *>(lds + p.h_off + (pair ? rw * p.h_each : 0));
    float *gs = reinterpret_cast<float *>(lds + p.g_off);
    {
        // the slices past the eighth (long d_in) and the quadruples past the second (many tokens)
        // cost further trips to L2
        auto finish = [&](int it, v4f h, int s0) __attribute__((always_inline)) {
            for (; s0 < p.S; s0 += HS) {
                v4f part[HS];
#pragma unroll
                for (int sl = 0; sl < HS; ++sl)
                    part[sl] = __builtin_bit_cast(v4f, buf_load16(hr, (unsigned)it * 16u + (unsigned)(s0 + sl) * hslice,
                                                                  hquad_ok(it) && s0 + sl < p.S));
#pragma unroll
                for (int sl = 0; sl < HS; ++sl) h += part[sl];
            }
            v4h o;
#pragma unroll
            for (int v = 0; v < 4; ++v) o[v] = (_Float16)silu(h[v]);
            if (it < hquads) *reinterpret_cast<v4h *>(hs + it * 4) = o;
        };
#pragma unroll
        for (int u = 0; u < HV; ++u) {
            v4f h = hpre[u][0];
#pragma unroll
            for (int sl = 1; sl < HS; ++sl) h += hpre[u][sl];
            finish(htid + u * hthreads, h, HS);
        }
        for (int it = htid + HV * hthreads; it < hquads; it += hthreads) finish(it, (v4f){0.f, 0.f, 0.f, 0.f}, 0);
    }
    if (tid < p.RW * kTileRows) {
        const int grank = pair ? (tid >= kTileRows ? p.L[1].rank : p.L[0].rank) : L.rank;
        gs[tid] = grank > 0 ? tanhf(alpha_pre) : 0.f;
    }

    v16i acc[TG];
#pragma unroll
    for (int tg = 0; tg < TG; ++tg) acc[tg] = (v16i){};

    for (int c0 = 0; c0 < p.KT; c0 += p.CT) {        // stretches of d_in staged in LDS
        cend = min(c0 + p.CT, p.KT);
        if (c0 > 0) {
            kt0 = c0 + kw;
            const rsrc_t wr = make_rsrc(rb_tiles, rb_ok ? (unsigned)cend * kTileBytes : 0u);
#pragma unroll
            for (int t = 0; t < PF; ++t) wq[t] = buf_load16_stream(wr, (unsigned)(kt0 + t * p.KW) * kTileBytes + l * 16);
            __syncthreads();                         // the previous stretch has been consumed
        }
        // x_q[:, c0*128 .. cend*128) is on its way into LDS (the first stretch since the kernel's
        // start): every wavefront waits for its own requests, then for the others'
        if (c0 > 0) stage_tokens(c0, cend);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        while (true) {
#pragma unroll
            for (int t = 0; t < PF; ++t) {
                const int kt = kt0 + t * p.KW;
                if (kt < cend) {
                    const unsigned char *xrow = lds + (kt - c0) * kTileCols + hf * 16;
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const v4i a = widen_codes(wq[t][q]);
#pragma unroll
                        for (int tg = 0; tg < TG; ++tg) {
                            v4i b = (v4i){0, 0, 0, 0};
                            if (tg * 32 + jl < mcount)
                                b = *reinterpret_cast<const v4i *>(xrow + (tg * 32 + jl) * p.xstride + q * 32);
                            acc[tg] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, acc[tg], 0, 0, 0);
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
        // (a partial tile as four pieces of 16 bytes per lane, piece by piece across the lanes:
        //  whole accumulators side by side, 64 bytes apart, put four lanes on every bank)
        v4i *red = reinterpret_cast<v4i *>(lds);
        const int slot0 = w - rw - 1;               // the non-owning wavefronts, densely numbered
        if (kw > 0) {
#pragma unroll
            for (int tg = 0; tg < TG; ++tg)
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    red[(((slot0 * TG) + tg) * 4 + c) * 64 + l] =
                        (v4i){acc[tg][4 * c], acc[tg][4 * c + 1], acc[tg][4 * c + 2], acc[tg][4 * c + 3]};
        }
        __syncthreads();
        if (kw > 0 && !pair) return;
        if (kw == 0) {
            for (int o = 1; o < p.KW; ++o) {
#pragma unroll
                for (int tg = 0; tg < TG; ++tg)
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        const v4i t = red[((((slot0 + o) * TG) + tg) * 4 + c) * 64 + l];
#pragma unroll
                        for (int i = 0; i < 4; ++i) acc[tg][4 * c + i] += t[i];
                    }
            }
        }
    }
    if (pair && p.KW == 1) __syncthreads();          // (pair: the staged activations give way to the exchange)
    // live: this wavefront finishes a row-block.  In a pair every wavefront stays for the
    // barrier over which the gate's outputs pass to the wavefront that holds the up rows.
    const bool live = kw == 0 && rb_ok && n0 < L.N;
    if (!live && !pair) return;

    // ---- correction up-projection: corr[m,n] = sum_j B[n,j] h[m,j] on the f16 MFMA
    v16f corr[TG];
#pragma unroll
    for (int tg = 0; tg < TG; ++tg) corr[tg] = (v16f){};
    if (live && L.rank > 0) {
#pragma unroll
        for (int js = 0; js < JS; ++js) {
            if (js * 16 < L.hstride) {
                const int j0 = js * 16 + hf * 8;
#pragma unroll
                for (int tg = 0; tg < TG; ++tg) {
                    const int m = tg * 32 + jl;
                    v8h b = {0, 0, 0, 0, 0, 0, 0, 0};
                    if (m < mcount) b = *reinterpret_cast<const v8h *>(hs + m * L.hstride + j0);
                    corr[tg] = __builtin_amdgcn_mfma_f32_32x32x16_f16(breg[js], b, corr[tg], 0, 0, 0);
                }
            }
        }
    }

    // ---- dequantise, gate, store.  Element 4*q + v of a lane's accumulator is row
    //      8*q + 4*hf + v of the row-block, for the token of the lane.
    //      Pair: the wavefront with the gate rows leaves its fp32 outputs in LDS; after a barrier
    //      the wavefront with the same rows of `up` (same lanes, same elements) multiplies its own
    //      by SiLU of them -- neither layer's output goes to memory -- and stores the product.
    const bool nvec = (L.N % 4) == 0;
    float *exch = reinterpret_cast<float *>(lds + p.exch_off);
    for (int pass = 0; pass < (pair ? 2 : 1); ++pass) {
        if (pair && pass == 1) __syncthreads();
        if (!live || (pair && rw != pass)) continue;
        const bool gate_side = pair && rw == 0;
#pragma unroll
        for (int tg = 0; tg < TG; ++tg) {
            const int m = tg * 32 + jl;
            const bool m_ok = m < mcount;
            const float scale = sx_pre[tg] * s_w;
            const int rs = rs_pre[tg];
            float zmax = 0.f;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int r0 = 8 * q + 4 * hf;           // first of 4 consecutive rows within the row-block
                const int nl = n0 + r0;
                int a[4];
                v4h o;
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    a[v] = acc[tg][4 * q + v] - rs;
                    float yv = (float)a[v] * scale + gs[rw * kTileRows + r0 + v] * corr[tg][4 * q + v];
                    if (gate_side) {
                        exch[(tg * 16 + 4 * q + v) * 64 + l] = yv;
                    } else if (pair) {
                        yv = silu(exch[(tg * 16 + 4 * q + v) * 64 + l]) * yv;
                    }
                    o[v] = (_Float16)yv;
                    if (nl + v < L.N) zmax = fmaxf(zmax, fabsf((float)o[v]));
                }
                if (!m_ok) continue;
                const size_t at = (size_t)m * L.N + nl;
                if (nvec && nl + 3 < L.N) {
                    if (!gate_side) *reinterpret_cast<v4h *>(L.y + at) = o;
                    if (L.acc_debug) *reinterpret_cast<v4i *>(L.acc_debug + at) = (v4i){a[0], a[1], a[2], a[3]};
                } else {
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        if (nl + v < L.N) {
                            if (!gate_side) L.y[at + v] = o[v];
                            if (L.acc_debug) L.acc_debug[at + v] = a[v];
                        }
                    }
                }
            }
            if (pair && !gate_side && p.amax_out) {
                // per token: the larger of the two lanes that hold its rows, then one atomic
                // (non-negative floats order like their bit patterns)
                zmax = fmaxf(zmax, __shfl_xor(zmax, 32, 64));
                if (hf == 0 && m_ok)
                    atomicMax(reinterpret_cast<unsigned *>(p.amax_out) + m, __builtin_bit_cast(unsigned, zmax));
            }
        }
    }
}

constexpr int kTargetWaves = 2048;            // wavefronts a launch aims at when it splits d_in
constexpr int kDecodeLdsBudget = 144 * 1024;   // one workgroup of 512 threads per compute unit anyway

}  // namespace

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
    const int tgroups = (M + 31) / 32;
    // wavefronts per row-block: enough to give the chip kTargetWaves wavefronts, at most
    // one per tile and eight per workgroup (two per SIMD, so each keeps 256 registers)
    int kw = 1;
    while (kw < 8 && kw * 2 <= p.KT && rb_total * kw < kTargetWaves) kw *= 2;
    if (p.pair) {
        // a workgroup per row-block index, two sets of up to four wavefronts (gate rows, up rows)
        if (p.G != 2 || p.L[0].N != p.L[1].N) return hipErrorInvalidValue;
        // (up to 16 tokens two per set: workgroups of 256 threads, several to a compute unit and
        //  the whole grid in one round -- 21.0 against 25.7 us for the 7B-shape pair at one token, 25.9
        //  against 30.4 at 16; from 24 tokens on the staged tokens make four per set the faster shape)
        const int per_set = M <= 16 ? 2 : 4;
        if (kw > per_set) kw = per_set;
    }
    p.KW = kw;
    p.RW = p.pair ? 2 : (kw >= 4 ? 1 : 4 / kw);
    // From a dozen tokens on the staged activations are what a workgroup mostly loads and what
    // limits how many of them a compute unit holds: then four row-blocks share one stage, two
    // wavefronts each (measured on the 7B-shape FFN: 47 against 53 us per block at 16 tokens, 58
    // against 66 at 32, 88 against 103 at 56; at 8 tokens 43 either way).
    if (!p.pair && kw == 4 && M > 12) {
        p.KW = 2;
        p.RW = 4;
    }
    const int nwaves = p.RW * p.KW;
    int wgs = 0;
    for (int g = 0; g < p.G; ++g) {
        p.wg_start[g] = wgs;
        wgs += (p.L[g].RBn + p.RW - 1) / p.RW;
    }
    p.wg_start[p.G] = wgs;
    if (p.pair) wgs = p.L[0].RBn;

    const size_t heach = ((size_t)M * hstride_max * sizeof(_Float16) + 15) & ~size_t(15);
    const size_t hbytes = heach * (p.pair ? 2 : 1);
    p.h_each = (int)heach;
    const size_t gbytes = (size_t)p.RW * kTileRows * sizeof(float);
    // stretch of d_in staged in LDS: as long as fits the budget (whole rows for small M)
    int ct = (int)(((kDecodeLdsBudget - hbytes - gbytes) / M - 16) / kTileCols);
    if (ct > p.KT) ct = p.KT;
    if (ct < 1) ct = 1;
    p.CT = ct;
    p.xstride = ct * kTileCols + 16;
    size_t stage = (size_t)M * p.xstride;
    size_t red = (size_t)(nwaves - p.RW) * tgroups * 64 * sizeof(v16i);
    p.exch_off = (int)red;                     // pair: the gate's fp32 outputs, behind the partial tiles
    if (p.pair) red += (size_t)tgroups * 16 * 64 * sizeof(float);
    if (stage < red) stage = red;
    stage = (stage + 15) & ~size_t(15);
    p.h_off = (int)stage;
    p.g_off = (int)(stage + ((hbytes + 15) & ~size_t(15)));
    const size_t lds = p.g_off + gbytes;

    if (lds > 160 * 1024) return hipErrorInvalidValue;
    static const hipError_t attr = [] {
        const void *const kernels[] = {reinterpret_cast<const void *>(&decode_kernel<1, false>),
                                       reinterpret_cast<const void *>(&decode_kernel<2, false>),
                                       reinterpret_cast<const void *>(&decode_kernel<1, true>),
                                       reinterpret_cast<const void *>(&decode_kernel<2, true>)};
        for (const void *k : kernels) {
            const hipError_t e = hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
            if (e != hipSuccess) return e;
        }
        return hipSuccess;
    }();
    if (attr != hipSuccess) return attr;
    const dim3 grid(wgs), block(64 * nwaves);
    if (p.pair) {
        if (tgroups == 1) hipLaunchKernelGGL((decode_kernel<1, true>), grid, block, lds, st, p);
        else hipLaunchKernelGGL((decode_kernel<2, true>), grid, block, lds, st, p);
    } else {
        if (tgroups == 1) hipLaunchKernelGGL((decode_kernel<1, false>), grid, block, lds, st, p);
        else hipLaunchKernelGGL((decode_kernel<2, false>), grid, block, lds, st, p);
    }
    return hipGetLastError();
}

}  // namespace hgf
