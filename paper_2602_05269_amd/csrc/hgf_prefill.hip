// Prefill kernel (more than 40 tokens; groups of few rows from 65): the ternary x int8 contraction as a dense int8 MFMA GEMM,
// fused with dequantisation, the rank-r up-projection and the gate.
//
// Algorithm 1 of the HGF paper, steps 3, 4, 7 and 8 (see hgf_decode.hip for the formulas).
// At hundreds of tokens the layer is a dense contraction (4*M int8 ops per weight byte), so
// it is tiled for the matrix cores: a workgroup of four wavefronts owns 256 output rows x
// 128 tokens; each wavefront owns 64 rows (two packed row-blocks) x 128 tokens = 8
// accumulator tiles of the 32x32x32 int8 MFMA (the full-rate int8 shape on gfx950: the
// 16x16x64 shape issues at half the rate), so each widened weight operand (7 VALU ops)
// feeds four MFMAs and each activation operand read from LDS feeds two.
// Weights never touch LDS: a wavefront loads its own packed tiles (16 bytes per lane per
// row-block per 128 columns), widens the 2-bit codes in registers and uses them as the
// MFMA's row operand.  The quantised activations of the 128 tokens are loaded straight
// into LDS (four buffers, requested four steps ahead, one barrier per 128 columns) and are
// shared by the four wavefronts.  Codes are T+1; the per-token sum of x_q is subtracted in
// the epilogue (integer-exact).
#include "hgf_internal.h"

namespace hgf {

namespace {

constexpr int kPN = 256;            // output rows per workgroup: four wavefronts x two row-blocks
constexpr int kPM = 128;            // tokens per workgroup at most (the LDS buffers hold that many)

struct PrefillLayer {
    const v4u *packed;
    const float *s_w;
    const _Float16 *B;
    const _Float16 *alpha;
    const _Float16 *h16;
    _Float16 *y;
    int N, RBn, rank;
    int nb_start;                  // first of this layer's row tiles among the launch's
};

// One launch covers every layer of a group (layers that read the same activations): the tail of
// one layer's tiles -- compute units left with a single workgroup, which does not keep the
// matrix cores busy on its own -- fills up with the next layer's.
struct PrefillParams {
    const int8_t *xq;
    const float *s_x;
    const int32_t *rowsum;
    int32_t *acc_debug;            // single-layer launches only
    int M, Kp, KT, hstride, G;
    int NB;                        // row tiles of all layers
    int MB;                        // token tiles
    // Workgroups go to the 8 XCDs round-robin by their index, and each XCD has its own L2: XCD
    // (xr, xt) of an rx x tx arrangement (rx * tx = 8) takes the row tiles = xr (mod rx) and the
    // token tiles = xt (mod tx), nbl x mbl of them at most, row tiles first -- so an L2 holds
    // 1/rx of the weights and sees 1/tx of the activations.
    int rx, tx, nbl, mbl;
    // SwiGLU pair (PAIR kernels): L[0] is the gate projection, L[1] the up projection, of one
    // shape.  A wavefront takes the SAME row-block of both (a workgroup: 128 rows x 2 layers)
    // and stores z = SiLU(y_gate) * y_up to L[1].y; neither y goes to memory.
    int32_t *acc_debug2;           // pair: the up projection's accumulators (nullable)
    float *amax_out;               // pair, nullable: per-token max |z| (zeroed before; atomic max)
    PrefillLayer L[kMaxGroup];
};

typedef __attribute__((address_space(3))) void *lds_ptr_t;

// LDS image of a kPM x 128 activation tile: row r at byte 128*r, its eight 16-byte pieces
// permuted by XOR with ((r div 2) mod 8): rows are 128 bytes, so rows r and r+1 differ in
// their bank half and the pair index picks the 16-byte group -- the sixteen lanes that read
// the same piece of consecutive rows in one LDS cycle hit sixteen different groups (the
// counters went from 48 % to 12 % conflict cycles against XOR with r mod 8) -- without padding (padding is impossible: an LDS-direct load
// writes 64 lanes x 16 bytes contiguously).
__device__ inline unsigned piece_slot(unsigned piece, unsigned row) { return piece ^ ((row >> 1) & 7u); }

// JS: steps of the 32x32x16 f16 MFMA over the (padded) rank = hstride / 16; 0 without correction.
// PM: tokens per workgroup, 128 or 64 (each widened weight operand then feeds two MFMAs instead
// of four, each activation operand still two); the launcher picks the width whose rounds of
// two workgroups per compute unit cost less.  The main loop keeps the matrix core about 85 %
// busy per clock with one workgroup in residence and 90 % with two; under either the chip's power
// management holds the clock near 1.6 GHz.
template <int JS, int PM, bool PAIR>
__global__ __launch_bounds__(256, 2) void prefill_kernel(PrefillParams p)
{
    constexpr int kPG = PM / 32;                         // token groups of 32 per wavefront
    constexpr int kXP = PM * kTileCols / (256 * 16);     // 16-byte activation pieces per thread and step
    // four separately declared activation buffers: the compiler can then prove that an
    // LDS-direct load into one does not alias the reads of another and leaves it in flight
    __shared__ __attribute__((aligned(1024))) unsigned char xs0[PM * kTileCols];
    __shared__ __attribute__((aligned(1024))) unsigned char xs1[PM * kTileCols];
    __shared__ __attribute__((aligned(1024))) unsigned char xs2[PM * kTileCols];
    __shared__ __attribute__((aligned(1024))) unsigned char xs3[PM * kTileCols];
    __shared__ float gs[kPN];                            // tanh(alpha) of the workgroup's rows

    const int tid = threadIdx.x, l = tid & 63, jl = l & 31, hf = l >> 5;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int xcd = blockIdx.x & 7, within = blockIdx.x >> 3;
    const int nbg = (within % p.nbl) * p.rx + xcd % p.rx, mb = (within / p.nbl) * p.tx + xcd / p.rx;
    if (nbg >= p.NB || mb >= p.MB) return;           // padding of the arrangement
    int g = 0;
    while (!PAIR && g + 1 < p.G && nbg >= p.L[g + 1].nb_start) ++g;
    const PrefillLayer &L = p.L[g];
    const int nb = nbg - L.nb_start;
    // this wavefront's first row-block; its second is the next one (PAIR: the same one of layer 1)
    const int rb0 = PAIR ? nb * (kPN / kTileRows / 2) + w : nb * (kPN / kTileRows) + w * 2;
    const int m0 = mb * PM;
    const int mrows = min(PM, p.M - m0);

    rsrc_t wr[2];
#pragma unroll
    for (int rb = 0; rb < 2; ++rb) {
        const int rbi = PAIR ? rb0 : rb0 + rb;
        const bool ok = rbi < L.RBn;
        const v4u *packed = PAIR ? p.L[rb].packed : L.packed;
        wr[rb] = make_rsrc(packed + (size_t)(ok ? rbi : 0) * p.KT * 64, ok ? (unsigned)p.KT * kTileBytes : 0u);
    }
    const rsrc_t xr = make_rsrc(p.xq + (size_t)m0 * p.Kp, (unsigned)mrows * p.Kp);

    if (!PAIR) {   // gate table
        const rsrc_t ar = make_rsrc(L.alpha, L.rank > 0 ? (unsigned)L.N * 2u : 0u);
        const int n = nb * kPN + tid;
        const float a = (float)half_bits(buf_load2(ar, (unsigned)n * 2u, n < L.N));
        gs[tid] = L.rank > 0 ? tanhf(a) : 0.f;
    } else {       // entry (2 w' + rb') * 32 + r: row (4 nb + w') * 32 + r of layer rb'
        const int lay = (tid >> 5) & 1;
        const int n = (nb * (kPN / kTileRows / 2) + (tid >> 6)) * kTileRows + (tid & 31);
        const rsrc_t ar0 = make_rsrc(p.L[0].alpha, p.L[0].rank > 0 ? (unsigned)p.L[0].N * 2u : 0u);
        const rsrc_t ar1 = make_rsrc(p.L[1].alpha, p.L[1].rank > 0 ? (unsigned)p.L[1].N * 2u : 0u);
        const float a0 = (float)half_bits(buf_load2(ar0, (unsigned)n * 2u, lay == 0 && n < p.L[0].N));
        const float a1 = (float)half_bits(buf_load2(ar1, (unsigned)n * 2u, lay == 1 && n < p.L[1].N));
        const int rank = lay == 0 ? p.L[0].rank : p.L[1].rank;
        gs[tid] = rank > 0 ? tanhf(lay == 0 ? a0 : a1) : 0.f;
    }

    // the weight scale(s) and the per-token scales of this lane's tokens, requested now, used in the epilogue
    const float s_w = *L.s_w;
    const float s_w2 = PAIR ? *p.L[1].s_w : s_w;
    float sx[kPG];
    int rs[kPG];
    {
        const rsrc_t sr = make_rsrc(p.s_x, (unsigned)p.M * 4u);
        const rsrc_t rr = make_rsrc(p.rowsum, (unsigned)p.M * 4u);
#pragma unroll
        for (int tg = 0; tg < kPG; ++tg) {
            sx[tg] = __builtin_bit_cast(float, buf_load4(sr, (unsigned)(m0 + tg * 32 + jl) * 4u));
            rs[tg] = (int)buf_load4(rr, (unsigned)(m0 + tg * 32 + jl) * 4u);
        }
    }

    // Activation staging: instruction i of wavefront w fills LDS bytes [(4i+w) KiB, +1 KiB):
    // lane L writes row 8(4i+w) + L/8, slot L%8, which holds piece slot ^ ((row/2)%8).  Rows
    // beyond the last token lie outside the descriptor and arrive as zeros.
    unsigned xsrc[kXP];
#pragma unroll
    for (int i = 0; i < kXP; ++i) {
        const unsigned row = (unsigned)(4 * i + w) * 8 + (l >> 3);
        xsrc[i] = row * p.Kp + piece_slot(l & 7, row) * 16;
    }
    // The step enters the addresses as a scalar offset (no vector arithmetic per request); a
    // request beyond the last step repeats the last step's (in bounds, never used).
    const int kt_last = p.KT - 1;
    auto stage = [&](unsigned char *buf, v4u (&wfill)[2], int kt) {   // request step kt
        const int ks = min(kt, kt_last);
#pragma unroll
        for (int rb = 0; rb < 2; ++rb)
            wfill[rb] = __builtin_bit_cast(v4u, __builtin_amdgcn_raw_buffer_load_b128(wr[rb], l * 16, ks * kTileBytes, 0));
#pragma unroll
        for (int i = 0; i < kXP; ++i)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(xr, (lds_ptr_t)(buf + (4 * i + w) * 1024), 16, (int)xsrc[i],
                                                     ks * kTileCols, 0, 0);
    };
    // Activation reads: lane (jl, hf) reads piece 2*t + hf of rows 32*tg + jl
    unsigned xoff[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) xoff[t] = (unsigned)jl * kTileCols + piece_slot(2 * t + hf, jl) * 16;

    v16i acc[2][kPG];
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
        for (int tg = 0; tg < kPG; ++tg) acc[rb][tg] = (v16i){};

    // One quarter of a step: the activation operands of 32 columns (piece pair t) for every
    // token group, and the 2 x kPG MFMAs that use them.
    auto reads = [&](const unsigned char *xbase, int t, v4i (&b)[kPG]) {
#pragma unroll
        for (int tg = 0; tg < kPG; ++tg)
            b[tg] = *reinterpret_cast<const v4i *>(xbase + xoff[t] + tg * 32 * kTileCols);
    };
    auto widen = [&](const v4u (&wuse)[2], int t, v4i (&a)[2]) {
#pragma unroll
        for (int rb = 0; rb < 2; ++rb) a[rb] = widen_codes(wuse[rb][t]);
    };
    auto mfmas = [&](const v4i (&a)[2], const v4i (&b)[kPG]) {
#pragma unroll
        for (int rb = 0; rb < 2; ++rb)
#pragma unroll
            for (int tg = 0; tg < kPG; ++tg)
                acc[rb][tg] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[rb], b[tg], acc[rb][tg], 0, 0, 0);
    };

    // Software pipeline.  Memory: four steps (4 x 128 columns) are in LDS or on their way; every
    // step issues 2 + kXP vector memory operations per wavefront (2 weight loads, kXP LDS-direct
    // loads).  Registers: the operands of a quarter are read from LDS and its weight codes widened
    // while the MFMAs of the quarter before run -- the instructions are dealt out between the
    // MFMAs (one MFMA, two vector instructions, every other time an LDS read), so that they issue
    // while the matrix core is busy with the MFMA before them -- also across the step boundary:
    // the barrier that opens step kt+1 stands before the last quarter of step kt:
    //   quarters 0..2 of step kt (each: request the next quarter's operands, then the MFMAs);
    //   wait until this wavefront's loads of step kt+1 have landed (those of steps kt+2 and
    //   kt+3 may stay in flight) and its LDS reads of step kt have returned; barrier: everyone's
    //   have; request quarter 0 of step kt+1 and, from memory, step kt+4 into the buffer and the
    //   weight registers step kt used, between the MFMAs of quarter 3.
    // The barrier is the bare instruction (the fence of __syncthreads would wait for all
    // loads in flight); the empty asm statements keep the compiler from moving memory
    // operations across it, the scheduling barriers from sinking the LDS reads below the
    // MFMAs that are to hide them.  Beyond the last step the descriptors return zeros, never used.
    constexpr int kLoads = 2 * (2 + kXP);            // two steps' worth may stay in flight
    constexpr int kWaitTwoStepsInFlight = (kLoads & 0xF) | (7 << 4) | (0 << 8) | ((kLoads >> 4) << 14);
    constexpr int kLoads3 = 3 * (2 + kXP);
    constexpr int kWaitThreeStepsInFlight = (kLoads3 & 0xF) | (7 << 4) | (15 << 8) | ((kLoads3 >> 4) << 14);
    v4i b0[kPG], b1[kPG], a0[2], a1[2];
    constexpr int kMfma = 0x008, kValu = 0x002, kLdsRead = 0x100, kVmemRead = 0x020;    // instruction classes of the scheduler hints
#define HGF_QUARTER(XREAD, WREAD, TREAD, BREAD, AREAD, AUSE, BUSE)        \
    do {                                                          \
        reads(XREAD, TREAD, BREAD);                               \
        widen(WREAD, TREAD, AREAD);                               \
        mfmas(AUSE, BUSE);                                        \
        _Pragma("unroll") for (int i_ = 0; i_ < 2 * kPG; ++i_) {  \
            __builtin_amdgcn_sched_group_barrier(kMfma, 1, 0);    \
            __builtin_amdgcn_sched_group_barrier(kValu, 2, 0);    \
            if (i_ % 2 == 0) __builtin_amdgcn_sched_group_barrier(kLdsRead, 1, 0); \
        }                                                         \
        __builtin_amdgcn_sched_barrier(0);                        \
    } while (0)
#define HGF_STEP(XCUR, WCUR, XNEXT, WNEXT, KT)                    \
    do {                                                          \
        HGF_QUARTER(XCUR, WCUR, 1, b1, a1, a0, b0);               \
        HGF_QUARTER(XCUR, WCUR, 2, b0, a0, a1, b1);               \
        HGF_QUARTER(XCUR, WCUR, 3, b1, a1, a0, b0);               \
        __builtin_amdgcn_s_waitcnt(kWaitTwoStepsInFlight);        \
        asm volatile("" ::: "memory");                            \
        __builtin_amdgcn_s_barrier();                             \
        asm volatile("" ::: "memory");                            \
        reads(XNEXT, 0, b0);                                      \
        widen(WNEXT, 0, a0);                                      \
        mfmas(a1, b1);                                            \
        stage(XCUR, WCUR, (KT) + 4);                              \
        _Pragma("unroll") for (int i_ = 0; i_ < 2 * kPG; ++i_) {  \
            __builtin_amdgcn_sched_group_barrier(kMfma, 1, 0);    \
            __builtin_amdgcn_sched_group_barrier(kValu, 2, 0);    \
            if (i_ % 2 == 0) __builtin_amdgcn_sched_group_barrier(kLdsRead, 1, 0); \
            else __builtin_amdgcn_sched_group_barrier(kVmemRead, 2, 0); \
        }                                                         \
        __builtin_amdgcn_sched_barrier(0);                        \
    } while (0)

    v4u w0[2], w1[2], w2[2], w3[2];
    stage(xs0, w0, 0);
    stage(xs1, w1, 1);
    stage(xs2, w2, 2);
    stage(xs3, w3, 3);
    __builtin_amdgcn_s_waitcnt(kWaitThreeStepsInFlight);
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    reads(xs0, 0, b0);
    widen(w0, 0, a0);
    __builtin_amdgcn_sched_barrier(0);
    int kt = 0;
    for (; kt + 3 < p.KT; kt += 4) {
        HGF_STEP(xs0, w0, xs1, w1, kt);
        HGF_STEP(xs1, w1, xs2, w2, kt + 1);
        HGF_STEP(xs2, w2, xs3, w3, kt + 2);
        HGF_STEP(xs3, w3, xs0, w0, kt + 3);
    }
    if (kt < p.KT) HGF_STEP(xs0, w0, xs1, w1, kt);
    if (kt + 1 < p.KT) HGF_STEP(xs1, w1, xs2, w2, kt + 1);
    if (kt + 2 < p.KT) HGF_STEP(xs2, w2, xs3, w3, kt + 2);
#undef HGF_STEP
#undef HGF_QUARTER
    __syncthreads();                 // gs is complete; every wavefront is done with the activation buffers

    // ---- epilogue: correction up-projection on the f16 MFMA, gate, dequantise, store.
    //      Element 4*q + v of an accumulator is row 8*q + 4*hf + v of the row-block, for the
    //      token of the lane.
    // SiLU(A x) of the tokens goes into the (now free) activation buffers: rows of JS*32
    // bytes with the same XOR permutation of the 16-byte pieces, the image of all PM tokens
    // cut into buffer-sized stretches (xs0 then xs1 for 128 tokens, xs0 then xs3 for 64);
    // the B rows of both row-blocks go to registers.  All of it is requested in one burst:
    // one memory round trip for the whole epilogue.
    constexpr int kRowBytes = JS * 32, kPieces = JS * 2, kMask = (kPieces < 8 ? kPieces : 8) - 1;
    constexpr unsigned kBufBytes = PM * kTileCols;
    if constexpr (PAIR) {
        // ---- SwiGLU pair: acc[0] holds this wavefront's row-block of the gate projection and
        //      acc[1] the same rows of the up projection, element for element in the same
        //      lanes, so z = SiLU(y_gate) * y_up forms in registers.  SiLU(A x) of the gate
        //      goes to (xs0, xs1), of the up projection to (xs2, xs3); direct stores.
        auto hplace2 = [&](int lay, unsigned byte) -> unsigned char * {
            unsigned char *a = lay ? xs2 : xs0, *b = lay ? xs3 : xs1;
            return byte < kBufBytes ? a + byte : b + (byte - kBufBytes);
        };
        v8h breg[2][JS > 0 ? JS : 1];
        if (JS > 0) {
#pragma unroll
            for (int lay = 0; lay < 2; ++lay) {
                // (a layer without correction has no rows: an empty descriptor reads zeros)
                const rsrc_t hr = make_rsrc(p.L[lay].h16 + (size_t)m0 * p.hstride,
                                            p.L[lay].rank > 0 ? (unsigned)mrows * p.hstride * 2u : 0u);
#pragma unroll
                for (int i = 0; i < PM * kRowBytes / 4096; ++i) {
                    const unsigned byte = (unsigned)(4 * i + w) * 1024 + l * 16;
                    const unsigned row = byte / kRowBytes, slot = (byte % kRowBytes) / 16;
                    const unsigned piece = slot ^ (row & kMask);
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(hr, (lds_ptr_t)hplace2(lay, (unsigned)(4 * i + w) * 1024), 16,
                                                             (int)(row * (unsigned)p.hstride * 2u + piece * 16), 0, 0, 0);
                }
            }
#pragma unroll
            for (int lay = 0; lay < 2; ++lay) {
                const int rank = p.L[lay].rank;
                const rsrc_t br = make_rsrc(p.L[lay].B, (unsigned)p.L[lay].N * rank * 2u);
                const bool bvec = (rank % 8) == 0;
                const int brow = rb0 * kTileRows + jl;
                const bool ok = rank > 0 && brow < p.L[lay].N;
#pragma unroll
                for (int js = 0; js < JS; ++js) {
                    const int j0 = js * 16 + hf * 8;
                    breg[lay][js] = bvec ? buf_load8h<true>(br, (unsigned)brow * rank + j0, rank - j0, ok)
                                         : buf_load8h<false>(br, (unsigned)brow * rank + j0, rank - j0, ok);
                }
            }
            __syncthreads();         // waits for the loads above and makes the staged rows visible
        }
        const int N = p.L[1].N;
        _Float16 *const z = p.L[1].y;
        const bool nvec = (N % 4) == 0;
        const int n0 = rb0 * kTileRows;
#pragma unroll
        for (int tg = 0; tg < kPG; ++tg) {
            const int m = m0 + tg * 32 + jl;
            const float scale_g = sx[tg] * s_w, scale_u = sx[tg] * s_w2;
            v16f corr[2] = {(v16f){}, (v16f){}};
            if (JS > 0) {
                const unsigned row = (unsigned)tg * 32 + jl;
#pragma unroll
                for (int js = 0; js < JS; ++js) {
                    const unsigned piece = (unsigned)(js * 2 + hf) ^ (row & kMask);
#pragma unroll
                    for (int lay = 0; lay < 2; ++lay) {
                        const unsigned char *hrow = hplace2(lay, (unsigned)tg * 32 * kRowBytes) + jl * kRowBytes;
                        const v8h b = *reinterpret_cast<const v8h *>(hrow + piece * 16);
                        corr[lay] = __builtin_amdgcn_mfma_f32_32x32x16_f16(breg[lay][js], b, corr[lay], 0, 0, 0);
                    }
                }
            }
            float zmax = 0.f;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int r0 = 8 * q + 4 * hf;
                const int nl = n0 + r0;
                int ag[4], au[4];
                v4h o;
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    ag[v] = acc[0][tg][4 * q + v] - rs[tg];
                    au[v] = acc[1][tg][4 * q + v] - rs[tg];
                    const float yg = (float)ag[v] * scale_g + gs[(w * 2 + 0) * kTileRows + r0 + v] * corr[0][4 * q + v];
                    const float yu = (float)au[v] * scale_u + gs[(w * 2 + 1) * kTileRows + r0 + v] * corr[1][4 * q + v];
                    o[v] = (_Float16)(silu(yg) * yu);
                    if (nl + v < N) zmax = fmaxf(zmax, fabsf((float)o[v]));
                }
                if (m < p.M) {
                    const size_t at = (size_t)m * N + nl;
                    if (nvec && nl + 3 < N) {
                        *reinterpret_cast<v4h *>(z + at) = o;
                        if (p.acc_debug) *reinterpret_cast<v4i *>(p.acc_debug + at) = (v4i){ag[0], ag[1], ag[2], ag[3]};
                        if (p.acc_debug2) *reinterpret_cast<v4i *>(p.acc_debug2 + at) = (v4i){au[0], au[1], au[2], au[3]};
                    } else {
#pragma unroll
                        for (int v = 0; v < 4; ++v) {
                            if (nl + v < N) {
                                z[at + v] = o[v];
                                if (p.acc_debug) p.acc_debug[at + v] = ag[v];
                                if (p.acc_debug2) p.acc_debug2[at + v] = au[v];
                            }
                        }
                    }
                }
            }
            if (p.amax_out) {        // per token: the larger of its two lanes, then one atomic
                zmax = fmaxf(zmax, __shfl_xor(zmax, 32, 64));
                if (hf == 0 && m < p.M && n0 < N)
                    atomicMax(reinterpret_cast<unsigned *>(p.amax_out) + m, __builtin_bit_cast(unsigned, zmax));
            }
        }
        return;
    }
    auto hplace = [&](unsigned byte) -> unsigned char * {
        return byte < kBufBytes ? xs0 + byte : (PM == 64 ? xs3 : xs1) + (byte - kBufBytes);
    };
    v8h breg[2][JS > 0 ? JS : 1];
    if (JS > 0) {
        const rsrc_t hr = make_rsrc(L.h16 + (size_t)m0 * p.hstride, (unsigned)mrows * p.hstride * 2u);
#pragma unroll
        for (int i = 0; i < PM * kRowBytes / 4096; ++i) {    // 4 KiB per instruction of the four wavefronts
            const unsigned byte = (unsigned)(4 * i + w) * 1024 + l * 16;
            const unsigned row = byte / kRowBytes, slot = (byte % kRowBytes) / 16;
            const unsigned piece = slot ^ (row & kMask);
            __builtin_amdgcn_raw_ptr_buffer_load_lds(hr, (lds_ptr_t)hplace((unsigned)(4 * i + w) * 1024), 16,
                                                     (int)(row * (unsigned)p.hstride * 2u + piece * 16), 0, 0, 0);
        }
        const int rank = L.rank;
        const rsrc_t br = make_rsrc(L.B, (unsigned)L.N * rank * 2u);
        const bool bvec = (rank % 8) == 0;
#pragma unroll
        for (int rb = 0; rb < 2; ++rb) {
            const int brow = (rb0 + rb) * kTileRows + jl;
#pragma unroll
            for (int js = 0; js < JS; ++js) {
                const int j0 = js * 16 + hf * 8;
                breg[rb][js] = bvec ? buf_load8h<true>(br, (unsigned)brow * rank + j0, rank - j0, brow < L.N)
                                    : buf_load8h<false>(br, (unsigned)brow * rank + j0, rank - j0, brow < L.N);
            }
        }
        __syncthreads();             // waits for the loads above and makes the staged rows visible
    }
    const int N = L.N;
    _Float16 *const y = L.y;
    const bool nvec = (N % 4) == 0;
    const int nw0 = rb0 * kTileRows;                 // first of this wavefront's 64 output rows
    // Coalesced store path: a token's 64 outputs of this wavefront are 128 contiguous bytes of
    // y.  The fp16 results of 32 tokens at a time are transposed through a wavefront-private
    // LDS patch (32 rows of 128 bytes, 16-byte pieces permuted like the activation tile's) and
    // leave as 16-byte stores, eight lanes per token (non-temporal: 13 to 67 MB of output per
    // launch would otherwise push the weights out of the L2s).  Needs the whole 64-row strip in
    // range and 16-byte aligned rows of y; otherwise (ragged d_out, or the int32 debug output)
    // direct stores.
    const bool wide = (N % 8) == 0 && nw0 + 64 <= N && p.acc_debug == nullptr;
    unsigned char *patch = (PM == 64 ? (w < 2 ? xs1 : xs2) : (w < 2 ? xs2 : xs3)) + (w & 1) * 4096;

#pragma unroll
    for (int tg = 0; tg < kPG; ++tg) {
        const int m = m0 + tg * 32 + jl;
        const float scale = sx[tg] * s_w;
        v16f corr[2] = {(v16f){}, (v16f){}};
        if (JS > 0) {
            const unsigned row = (unsigned)tg * 32 + jl;
            const unsigned char *hrow = hplace((unsigned)tg * 32 * kRowBytes) + jl * kRowBytes;
#pragma unroll
            for (int js = 0; js < JS; ++js) {
                const unsigned piece = (unsigned)(js * 2 + hf) ^ (row & kMask);
                const v8h b = *reinterpret_cast<const v8h *>(hrow + piece * 16);
#pragma unroll
                for (int rb = 0; rb < 2; ++rb)
                    corr[rb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(breg[rb][js], b, corr[rb], 0, 0, 0);
            }
        }
#pragma unroll
        for (int rb = 0; rb < 2; ++rb) {
            const int n0 = nw0 + rb * kTileRows;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int r0 = 8 * q + 4 * hf;
                const int nl = n0 + r0;
                int a[4];
                v4h o;
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    a[v] = acc[rb][tg][4 * q + v] - rs[tg];
                    o[v] = (_Float16)((float)a[v] * scale + gs[(w * 2 + rb) * kTileRows + r0 + v] * corr[rb][4 * q + v]);
                }
                if (wide) {
                    *reinterpret_cast<v4h *>(patch + jl * kTileCols + piece_slot(rb * 4 + q, jl) * 16 + hf * 8) = o;
                } else if (m < p.M) {
                    const size_t at = (size_t)m * N + nl;
                    if (nvec && nl + 3 < N) {
                        *reinterpret_cast<v4h *>(y + at) = o;
                        if (p.acc_debug) *reinterpret_cast<v4i *>(p.acc_debug + at) = (v4i){a[0], a[1], a[2], a[3]};
                    } else {
#pragma unroll
                        for (int v = 0; v < 4; ++v) {
                            if (nl + v < N) {
                                y[at + v] = o[v];
                                if (p.acc_debug) p.acc_debug[at + v] = a[v];
                            }
                        }
                    }
                }
            }
        }
        if (wide) {
            // the patch is private to the wavefront: its own LDS writes are complete once
            // the read below has been ordered after them (same wavefront, in-order LDS)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int tok = i * 8 + (l >> 3), piece = l & 7;
                const v4u v = *reinterpret_cast<const v4u *>(patch + tok * kTileCols + piece_slot(piece, tok) * 16);
                const int mm = m0 + tg * 32 + tok;
                if (mm < p.M) __builtin_nontemporal_store(v, reinterpret_cast<v4u *>(y + (size_t)mm * N + nw0 + piece * 8));
            }
        }
    }
}

}  // namespace

// Layers [0, G) read the same quantised activations (the workspace's); consecutive layers whose
// correction paths have the same padded rank share a launch.
// pair_out != nullptr: the SwiGLU pair (G == 2; layers[0] gate, layers[1] up): ys[1] receives
// z = SiLU(y_gate) * y_up, ys[0] is unused.
hipError_t launch_prefill(const Workspace &ws, _Float16 *const *h16, int M, const hgf_layer *layers, int G,
                          void *const *ys, int32_t *acc_debug, hipStream_t st, const PairOut *pair_out)
{
    static int num_cus = 0;
    if (num_cus == 0) {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) {
            (void)hipGetLastError();
            n = 256;
        }
        num_cus = n;
    }
    auto steps_of = [](const hgf_layer &L) { return L.rank > 0 ? h_stride(L.rank) / 16 : 0; };
    const bool pair = pair_out != nullptr;
    if (pair && (G != 2 || layers[0].d_out != layers[1].d_out)) return hipErrorInvalidValue;
    // pair: the two correction paths must pad to one width (a zero rank rides along with the other's)
    const int pair_steps = pair ? (steps_of(layers[0]) > steps_of(layers[1]) ? steps_of(layers[0]) : steps_of(layers[1])) : 0;
    for (int first = 0; first < G;) {
        int n = 1;
        while (!acc_debug && !pair && first + n < G && steps_of(layers[first + n]) == steps_of(layers[first])) ++n;
        if (pair) n = 2;
        PrefillParams p;
        p.xq = ws.xq;
        p.s_x = ws.s_x;
        p.rowsum = ws.rowsum;
        p.acc_debug = acc_debug;
        p.acc_debug2 = pair ? pair_out->acc_debug2 : nullptr;
        p.amax_out = pair ? pair_out->amax_out : nullptr;
        p.M = M;
        p.Kp = round_up(layers[first].d_in, kTileCols);
        p.KT = p.Kp / kTileCols;
        p.hstride = pair ? (pair_steps > 0 ? pair_steps * 16 : 32) : h_stride(layers[first].rank > 0 ? layers[first].rank : 1);
        p.G = n;
        p.NB = 0;
        for (int g = 0; g < n; ++g) {
            const hgf_layer &L = layers[first + g];
            PrefillLayer &P = p.L[g];
            P.packed = reinterpret_cast<const v4u *>(L.W_packed);
            P.s_w = L.s_w;
            P.B = reinterpret_cast<const _Float16 *>(L.B_f16);
            P.alpha = reinterpret_cast<const _Float16 *>(L.alpha_f16);
            P.h16 = h16[first + g];
            P.y = reinterpret_cast<_Float16 *>(ys[first + g]);
            P.N = L.d_out;
            P.RBn = round_up(L.d_out, kTileRows) / kTileRows;
            P.rank = L.rank;
            P.nb_start = p.NB;
            p.NB += (L.d_out + kPN - 1) / kPN;
        }
        if (pair) {
            p.L[1].nb_start = 0;
            p.NB = (layers[0].d_out + kPN / 2 - 1) / (kPN / 2);    // a workgroup: 128 rows of both layers
        }
        for (int g = n; g < kMaxGroup; ++g) p.L[g] = p.L[0];
        // Tile width.  Two workgroups fit a compute unit, so the tiles run in rounds of
        // 2 x num_cus; a round of 256 x 64 tiles costs a little over half a round of 256 x 128
        // tiles (each widened weight operand feeds two MFMAs instead of four).  Take the width
        // whose whole rounds cost less: the wide tile unless its last round would be mostly empty.
        const int slots = 2 * num_cus;
        const int rounds_wide = (p.NB * ((M + kPM - 1) / kPM) + slots - 1) / slots;
        const int rounds_narrow = (p.NB * ((M + 63) / 64) + slots - 1) / slots;
        const bool narrow = rounds_narrow * 21 < rounds_wide * 40;
        const int pm = narrow ? 64 : kPM;
        p.MB = (M + pm - 1) / pm;
        // the arrangement that moves the fewest bytes into the L2s: tx copies of the weights,
        // rx copies of the quantised activations
        double wbytes = 0.0;
        for (int g = 0; g < n; ++g) wbytes += (double)p.L[g].RBn * p.KT * kTileBytes;
        const double xbytes = (double)M * p.Kp;
        p.rx = 8;
        for (int rx = 4; rx >= 1; rx /= 2)
            if ((8 / rx) * wbytes + rx * xbytes < (8 / p.rx) * wbytes + p.rx * xbytes) p.rx = rx;
        p.tx = 8 / p.rx;
        p.nbl = (p.NB + p.rx - 1) / p.rx;
        p.mbl = (p.MB + p.tx - 1) / p.tx;
        const dim3 grid(8 * p.nbl * p.mbl), block(256);
#define HGF_PREFILL(JS)                                                                              \
    do {                                                                                             \
        if (pair) {                                                                                  \
            if (narrow) hipLaunchKernelGGL((prefill_kernel<JS, 64, true>), grid, block, 0, st, p);   \
            else hipLaunchKernelGGL((prefill_kernel<JS, 128, true>), grid, block, 0, st, p);         \
        } else {                                                                                     \
            if (narrow) hipLaunchKernelGGL((prefill_kernel<JS, 64, false>), grid, block, 0, st, p);  \
            else hipLaunchKernelGGL((prefill_kernel<JS, 128, false>), grid, block, 0, st, p);        \
        }                                                                                            \
    } while (0)
        switch (pair ? pair_steps : steps_of(layers[first])) {
            case 0: HGF_PREFILL(0); break;
            case 2: HGF_PREFILL(2); break;
            case 4: HGF_PREFILL(4); break;
            default: HGF_PREFILL(8); break;
        }
#undef HGF_PREFILL
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        first += n;
    }
    return hipSuccess;
}

}  // namespace hgf
