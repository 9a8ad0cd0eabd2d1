// Decode for a handful of tokens (M <= 4): every step of the layer in ONE persistent
// launch, for up to four layers that read the same activations.
//
// Algorithm 1 of the HGF paper, steps 1-8.  At batch 1 a layer is a single pass over the
// packed weights, a few microseconds of HBM time; launch gaps and dependent memory round
// trips cost as much, so the whole layer runs in one launch whose workgroups (one per
// compute unit) each take every nwg-th row-block of 32 output rows ("unit") and keep a
// ring of weight tiles in flight from the first instruction to the last.
//
// A workgroup has seven streaming wavefronts and one service wavefront.
//   streaming: request the token rows and the first ring of weight tiles; quantise the
//     tokens into LDS (steps 1-2; the int8 row never goes to memory); then per unit,
//     contract tiles w, w+7, ... of d_in on the int8 MFMA over 2-bit codes (step 3),
//     refilling each ring slot as it is consumed, and post the partial int32 tile to an
//     LDS mailbox.
//   service: computes one slice of A x (step 5) on the f16 MFMA and writes its fp32
//     partial sums to a device-wide exchange buffer; collects every slice of the group,
//     adds them in order and applies SiLU (step 6); then per unit adds the seven posted
//     tiles, dequantises (step 4), applies the up-projection on the f16 MFMA and the gate
//     (steps 7-8) and stores.  It issues no weight loads, so its waits never stall the stream.
//
// Exchange of the partial sums: the buffer holds a sentinel bit pattern (all ones: a NaN
// that arithmetic on fp16 inputs cannot produce) wherever no value has been written.
// Producers store with device scope; consumers re-read with device scope until no word is
// the sentinel.  No flag, no fence: every word is either the sentinel or final.  Two
// buffers alternate by a launch counter kept in the workspace: each launch fills the one
// the next launch will use with sentinels, and the last workgroup to finish advances the
// counter.  Every wait is bounded; on expiry a sticky word is set in the workspace and the
// affected outputs are NaN.
#include "hgf_internal.h"

namespace hgf {

namespace {

constexpr int kStream = 7;             // streaming wavefronts per workgroup (wavefront 7 is the service one)
constexpr int kXV = 4;                 // 16-byte pieces of a token row per streaming thread: 448*4*8 >= kMaxFusedK
constexpr int kPF = 6;                 // weight tiles in flight per streaming wavefront.  More than the
                                       // bandwidth-delay product needs only lengthens every queue, and with
                                       // it the round trips of the exchange below.
constexpr int kMaxUnits = 16;          // units per workgroup at most: each has a mailbox slot of its own
constexpr int kLdsPolls = 1 << 22;     // bound of a wait on LDS (about a second)
constexpr int kMemPolls = 1 << 18;     // bound of a wait on the exchange buffer (about a second)
constexpr unsigned kSentinel = 0xFFFFFFFFu;
constexpr int kHsStride = HGF_MAX_RANK;  // halves per (layer, token) row of SiLU(A x) in LDS
constexpr int kJS = HGF_MAX_RANK / 16;   // steps of the 32x32x16 f16 MFMA over the rank

struct Control {                       // LDS words shared by the two sides of a workgroup
    int arrived[kMaxUnits];            // streaming wavefronts that have posted the unit
};

typedef __attribute__((address_space(3))) void *lds_ptr_t;

__device__ __forceinline__ int lds_load(const int *p) { return __hip_atomic_load(p, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP); }

__device__ __forceinline__ v4u buf_load16_agent(rsrc_t r, unsigned off, bool ok = true)
{
    return __builtin_bit_cast(v4u, __builtin_amdgcn_raw_buffer_load_b128(r, (int)(ok ? off : kOob), 0, 16));
}

// Cheap transcendental forms for the service wavefront, whose latency is the tail of the
// launch (hardware exp2 and reciprocal, about 1 ulp each; the results are rounded to fp16
// or multiply an fp16-bound term).
__device__ __forceinline__ float exp_fast(float v) { return __builtin_amdgcn_exp2f(v * 1.44269504088896340736f); }
__device__ __forceinline__ float silu_fast(float h) { return h * __builtin_amdgcn_rcpf(1.0f + exp_fast(-h)); }
__device__ __forceinline__ float tanh_fast(float a) { return 1.0f - 2.0f * __builtin_amdgcn_rcpf(1.0f + exp_fast(2.0f * a)); }

// unit -> layer of the group (ustart is the running sum of row-blocks)
__device__ __forceinline__ int layer_of(const FusedParams &p, int u)
{
    int g = 0;
#pragma unroll
    for (int i = 1; i < kMaxGroup; ++i)
        if (i < p.G && u >= p.ustart[i]) g = i;
    return g;
}

// ------------------------------------------------------------------ streaming side
__device__ __forceinline__ void streaming_wave(const FusedParams &p, unsigned char *lds, Control *ctl, float *sh_max, int *sh_sum,
                               float *sh_sx, int *sh_rs, int c, int nunits)
{
    const int tid = threadIdx.x, l = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int jl = l & 31, hf = l >> 5;
    constexpr int nthreads = kStream * 64;

    // ---- (1) the first token row
    const rsrc_t xr = make_rsrc(p.x, (unsigned)p.M * p.K * 2u);
    v8h keep[kXV];
#pragma unroll
    for (int r = 0; r < kXV; ++r) {
        const int i = tid + r * nthreads;
        keep[r] = __builtin_bit_cast(v8h, buf_load16(xr, (unsigned)i * 16u, i * 8 < p.K));
    }

    // ---- (2) the ring of weight tiles.  The load cursor (li, lj) runs kPF tiles ahead of
    //      the MFMA cursor; tile j of a unit is column tile 7*j + w of its row-block.
    //      The layers' bases and extents sit in scalar registers: the cursor selects, it never loads.
    const void *pk0 = p.L[0].packed, *pk1 = p.L[1].packed, *pk2 = p.L[2].packed, *pk3 = p.L[3].packed;
    const unsigned by0 = (unsigned)p.L[0].RBn * p.KT * kTileBytes, by1 = (unsigned)p.L[1].RBn * p.KT * kTileBytes,
                   by2 = (unsigned)p.L[2].RBn * p.KT * kTileBytes, by3 = (unsigned)p.L[3].RBn * p.KT * kTileBytes;
    const int us1 = p.G > 1 ? p.ustart[1] : 0x7fffffff, us2 = p.G > 2 ? p.ustart[2] : 0x7fffffff,
              us3 = p.G > 3 ? p.ustart[3] : 0x7fffffff;
    int li = 0, lj = 0;
    const void *lbase = nullptr;
    unsigned lbytes = 0, lrow = 0;
    auto load_unit = [&]() {            // the load cursor has entered unit li
        const bool valid = li < nunits; // past the last unit: every load reads zeros
        const int u = valid ? c + li * p.nwg : c;
        int first = 0;
        lbase = pk0;
        lbytes = by0;
        if (u >= us1) { lbase = pk1; lbytes = by1; first = us1; }
        if (u >= us2) { lbase = pk2; lbytes = by2; first = us2; }
        if (u >= us3) { lbase = pk3; lbytes = by3; first = us3; }
        if (!valid) lbytes = 0;
        lrow = (unsigned)(u - first) * p.KT;
    };
    load_unit();
    v4u wq[kPF];
    auto issue = [&](v4u &dst) {
        const int kt = lj * kStream + w;
        const rsrc_t wr = make_rsrc(lbase, lbytes);
        dst = buf_load16_stream(wr, kt < p.KT ? (lrow + kt) * kTileBytes + l * 16 : kOob);
        if (++lj == p.TPW) {
            lj = 0;
            ++li;
            load_unit();
        }
    };
#pragma unroll
    for (int t = 0; t < kPF; ++t) issue(wq[t]);

    // ---- per-token absmax int8 quantisation into LDS (Sec. 2.2.1), one token after the other
    const int nvec_p = p.Kp / 8;
    auto quantise_row = [&](int m) {
        float amax = 0.0f;
#pragma unroll
        for (int r = 0; r < kXV; ++r)
            if (r * nthreads < nvec_p)  // (compute only: the loads themselves are unconditional)
#pragma unroll
                for (int e = 0; e < 8; ++e) amax = fmaxf(amax, fabsf((float)keep[r][e]));
        amax = wave_max(amax);
        if (l == 0) sh_max[w] = amax;
        __syncthreads();
        amax = sh_max[0];
#pragma unroll
        for (int i = 1; i < kStream; ++i) amax = fmaxf(amax, sh_max[i]);
        amax = fmaxf(amax, 1e-5f);
        const float inv = 127.0f / amax;
        int sum = 0;
#pragma unroll
        for (int r = 0; r < kXV; ++r) {
            if (r * nthreads >= nvec_p) continue;
            const int i = tid + r * nthreads;
            uint32_t q2[2] = {0u, 0u};
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int q = quant1((float)keep[r][e], inv);
                sum += q;
                q2[e >> 2] |= (uint32_t)(q & 0xff) << (8 * (e & 3));
            }
            if (i < nvec_p) *reinterpret_cast<uint2 *>(lds + m * p.xstride + i * 8) = make_uint2(q2[0], q2[1]);
        }
        sum = wave_sum(sum);
        if (l == 0) sh_sum[w] = sum;
        __syncthreads();
        if (tid == 0) {
            int s = sh_sum[0];
#pragma unroll
            for (int i = 1; i < kStream; ++i) s += sh_sum[i];
            sh_sx[m] = amax / 127.0f;
            sh_rs[m] = s;
        }
    };
    quantise_row(0);                    // outside the loop: its wait must not cover the loads behind it
    for (int m = 1; m < p.M; ++m) {
#pragma unroll
        for (int r = 0; r < kXV; ++r) {
            const int i = tid + r * nthreads;
            keep[r] = __builtin_bit_cast(v8h, buf_load16(xr, ((unsigned)m * p.K + (unsigned)i * 8u) * 2u, i * 8 < p.K));
        }
        quantise_row(m);
    }
    // the token scales written by thread 0 after the last barrier reach the service side
    // through the release/acquire pair on `arrived`

    // ---- contraction: one ring slot per step
    int *tiles = reinterpret_cast<int *>(lds + p.tile_off);
    int ci = 0, cj = 0;                 // MFMA cursor: unit, tile within the unit
    v16i acc = (v16i){};
    // (the refill of a slot is unconditional, straight-line code: a load under a branch makes
    //  the compiler's wait for the OTHER slots stricter at every join, until it waits for all)
    while (ci < nunits) {
#pragma unroll
        for (int t = 0; t < kPF; ++t) {
            const int kt = cj * kStream + w;
            if (kt < p.KT && ci < nunits) {
                // tokens are the matrix rows (lane jl < M holds 16 int8 of token jl), the 32 weight
                // rows the matrix columns: lane n < 32 ends up with acc[m] for tokens m = 0..3
                const unsigned char *xrow = lds + kt * kTileCols + hf * 16;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const v4i wcodes = widen_codes(wq[t][q]);
                    v4i xv = (v4i){0, 0, 0, 0};
                    if (jl < p.M) xv = *reinterpret_cast<const v4i *>(xrow + jl * p.xstride + q * 32);
                    acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(xv, wcodes, acc, 0, 0, 0);
                }
            }
            issue(wq[t]);
            if (++cj == p.TPW) {
                if (ci < nunits) {      // the unit is complete: add its partial tile to the unit's
                                        // [token][row] sums in LDS (integer adds: any order, same result;
                                        // no wait, no inner loop: either would cost the ring its precise waits)
                    if (l < 32) {
#pragma unroll
                        for (int m = 0; m < kMaxFusedM; ++m)
                            if (m < p.M)
                                __hip_atomic_fetch_add(tiles + (ci * kMaxFusedM + m) * kTileRows + l, acc[m], __ATOMIC_RELAXED,
                                                       __HIP_MEMORY_SCOPE_WORKGROUP);
                    }
                    if (l == 0)
                        __hip_atomic_fetch_add(&ctl->arrived[ci], 1, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
                    acc = (v16i){};
                }
                cj = 0;
                ++ci;
            }
        }
    }
}

// ------------------------------------------------------------------ service side
// One slice of A x: rank tile `rt` of layer `g`, slice `sp` of d_in, all tokens.  Lane
// (i = l%16, kb = l/16) holds A[rt*16+i][k] and x[i][k] for the same eight k per MFMA:
// k = 64*kp + 16*kb + 0..7 and + 8..15, so a row is read 128 contiguous bytes at a time.
constexpr int kUN = 8;                 // 64-column steps requested together
struct JobRegs {
    v8h a[kUN][2], b[kUN][2];
};
__device__ __forceinline__ void job_decode(const FusedParams &p, int job, int &g, int &rt, int &sp)
{
    g = 0;
#pragma unroll
    for (int i = 1; i < kMaxGroup; ++i)
        if (i < p.G && job >= p.job_start[i]) g = i;
    const int local = job - p.job_start[g];
    rt = local / p.S;
    sp = local % p.S;
}
__device__ __forceinline__ void job_load(const FusedParams &p, JobRegs &r, int g, int rt, int kpb, int kp1)
{
    const int l = threadIdx.x & 63, i = l & 15, kb = l >> 4;
    const int j = rt * 16 + i, rank = p.L[g].rank;
    const bool j_ok = j < rank, m_ok = i < p.M;
    const rsrc_t ar = make_rsrc(p.A[g], (unsigned)rank * p.K * 2u);
    const rsrc_t xr = make_rsrc(p.x, (unsigned)p.M * p.K * 2u);
#pragma unroll
    for (int u = 0; u < kUN; ++u) {
        const int k0 = (kpb + u) * 64 + kb * 16;
        const bool ok = (kpb + u) < kp1;
        r.a[u][0] = buf_load8h<true>(ar, (unsigned)j * p.K + k0, p.K - k0, ok && j_ok);
        r.a[u][1] = buf_load8h<true>(ar, (unsigned)j * p.K + k0 + 8, p.K - k0 - 8, ok && j_ok);
        r.b[u][0] = buf_load8h<true>(xr, (unsigned)i * p.K + k0, p.K - k0, ok && m_ok);
        r.b[u][1] = buf_load8h<true>(xr, (unsigned)i * p.K + k0 + 8, p.K - k0 - 8, ok && m_ok);
    }
}
__device__ __forceinline__ v4f job_mfma(const JobRegs &r, v4f acc)
{
#pragma unroll
    for (int u = 0; u < kUN; ++u) {
        acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(r.a[u][0], r.b[u][0], acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(r.a[u][1], r.b[u][1], acc, 0, 0, 0);
    }
    return acc;
}

// Requests the epilogue operands of unit `u` into LDS with LDS-direct loads (no registers
// held, nothing to wait for until the epilogue): the 32 rows of B as 16-byte pieces in
// column-major order (piece cp of row r at slot 32*cp + r, so the MFMA operand reads of 32
// rows are conflict-free), then the 32 gate parameters.  Rows beyond d_out and pieces beyond
// the rank arrive as zeros.
__device__ __forceinline__ void stage_unit(const FusedParams &p, unsigned char *dst, int u)
{
    const int l = threadIdx.x & 63, r = l & 31;
    const int g = layer_of(p, u);
    const DecLayer &L = p.L[g];
    if (L.rank == 0) return;
    const int n0 = (u - p.ustart[g]) * kTileRows;
    const rsrc_t br = make_rsrc(L.B, (unsigned)L.N * L.rank * 2u);
    const rsrc_t ar = make_rsrc(L.alpha, ((unsigned)L.N * 2u + 3u) & ~3u);
    const int ninstr = L.hstride / 16;
    for (int k = 0; k < ninstr; ++k) {
        const int cp = 2 * k + (l >> 5);
        const bool ok = cp * 8 < L.rank && n0 + r < L.N;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(br, (lds_ptr_t)(dst + k * 1024), 16,
                                                 (int)(ok ? (unsigned)((n0 + r) * L.rank + cp * 8) * 2u : kOob), 0, 0, 0);
    }
    __builtin_amdgcn_raw_ptr_buffer_load_lds(ar, (lds_ptr_t)(dst + p.unit_alpha), 4,
                                             (int)(l < 16 && n0 + 2 * l < L.N ? (unsigned)(n0 * 2 + l * 4) : kOob), 0, 0, 0);
}

// corr[m] of lane n = sum_j h[m][j] B[n][j] on the 32x32x16 f16 MFMA, tokens as matrix rows.
// Every LDS operand is requested before the first MFMA; two accumulators halve the chain.
template <int JS>
__device__ __forceinline__ v16f corr_unit(const _Float16 *hrow, const unsigned char *brow, bool token)
{
    v8h hv[JS], bv[JS];
#pragma unroll
    for (int js = 0; js < JS; ++js) {
        hv[js] = (v8h){0, 0, 0, 0, 0, 0, 0, 0};
        if (token) hv[js] = *reinterpret_cast<const v8h *>(hrow + js * 16);
        bv[js] = *reinterpret_cast<const v8h *>(brow + js * 1024);
    }
    v16f c0 = (v16f){}, c1 = (v16f){};
#pragma unroll
    for (int js = 0; js < JS; js += 2) {
        c0 = __builtin_amdgcn_mfma_f32_32x32x16_f16(hv[js], bv[js], c0, 0, 0, 0);
        c1 = __builtin_amdgcn_mfma_f32_32x32x16_f16(hv[js + 1], bv[js + 1], c1, 0, 0, 0);
    }
    return c0 + c1;
}

__device__ __forceinline__ void service_wave(const FusedParams &p, unsigned char *lds, Control *ctl, const float *sh_sx,
                             const int *sh_rs, int c, int nunits)
{
    const int l = threadIdx.x & 63, jl = l & 31, hf = l >> 5;
    const int njobs = p.job_start[p.G];
    bool failed = false;

    // ---- which exchange buffer this launch uses
    const unsigned epoch = (unsigned)__hip_atomic_load(p.flags, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    unsigned char *mine = p.mail + (size_t)(epoch & 1u) * kMailBytes;
    unsigned char *other = p.mail + (size_t)((epoch & 1u) ^ 1u) * kMailBytes;

    {   // the units' [token][row] sums start at zero (before any LDS-direct load: an LDS access
        // behind one makes the compiler wait for it)
        int *tiles = reinterpret_cast<int *>(lds + p.tile_off);
        for (int e = l; e < nunits * kMaxFusedM * kTileRows; e += 64) tiles[e] = 0;
    }
    // ---- requests, all up front: the epilogue operands of every unit (LDS-direct; issued first
    //      because the compiler drains the queue before a loop of such loads), the layers'
    //      weight scales (four guarded loads; absent layers read zero), then the operands of
    //      the first slice of A x
    unsigned char *ustage = lds + p.unit_off;
    for (int i = 0; i < nunits; ++i) stage_unit(p, ustage + i * p.unit_stride, c + i * p.nwg);
    const unsigned swb0 = buf_load4(make_rsrc(p.L[0].s_w, nunits > 0 ? 4u : 0u), 0u);
    const unsigned swb1 = buf_load4(make_rsrc(p.L[1].s_w, nunits > 0 && p.G > 1 ? 4u : 0u), 0u);
    const unsigned swb2 = buf_load4(make_rsrc(p.L[2].s_w, nunits > 0 && p.G > 2 ? 4u : 0u), 0u);
    const unsigned swb3 = buf_load4(make_rsrc(p.L[3].s_w, nunits > 0 && p.G > 3 ? 4u : 0u), 0u);
    int job = p.nwg - 1 - c;            // the highest workgroups, which own the fewest units, come first
    JobRegs jr;
    int g = 0, rt = 0, sp = 0, kp0 = 0, kp1 = 0;
    if (job < njobs) {
        job_decode(p, job, g, rt, sp);
        kp0 = sp * p.pairs_per_slice;
        kp1 = min(kp0 + p.pairs_per_slice, p.pairs);
        job_load(p, jr, g, rt, kp0, kp1);
    }
    // The quantiser's barriers.  Bare barriers: this wavefront shares no data with the others
    // at them (a fence would make it wait for everything it has just requested); only the
    // zeroed control words must have landed.  Its slice of A x goes between the first two, in
    // the time the others spend quantising.
    auto job_compute = [&]() {
        v4f acc = {0.f, 0.f, 0.f, 0.f};
        acc = job_mfma(jr, acc);
        for (int kpb = kp0 + kUN; kpb < kp1; kpb += kUN) {
            job_load(p, jr, g, rt, kpb, kp1);
            acc = job_mfma(jr, acc);
        }
        return acc;
    };
    auto job_store = [&](v4f acc) {
        // acc[v]: rank index rt*16 + 4*kb + v of token i  ->  [sp][i][hstride] of layer g
        const int i = l & 15, kb = l >> 4, hstride = p.L[g].hstride;
        const rsrc_t hr = make_rsrc(mine + (size_t)g * kMailLayerBytes, (unsigned)kMailLayerBytes);
        buf_store16_agent(hr, i < p.M ? (unsigned)(((sp * p.M + i) * hstride + rt * 16 + 4 * kb) * 4) : kOob, acc);
    };
    if (nunits > 0) {
        __builtin_amdgcn_s_waitcnt(0xC07F);          // lgkmcnt(0) only
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
    }
    {
        v4f acc = {0.f, 0.f, 0.f, 0.f};
        if (job < njobs) acc = job_compute();
        // A read of the staged operands, placed where it costs nothing: the compiler orders it
        // behind the LDS-direct loads, and these have landed once the job's operands (requested
        // after them) are here.  Without it the first LDS access further down would wait for
        // every outstanding memory operation -- the store below included, whose
        // acknowledgement takes microseconds while the weight stream saturates the memory.
        asm volatile("" ::"v"(*reinterpret_cast<volatile int *>(lds + p.unit_off)) : "memory");
        if (job < njobs) {
            job_store(acc);
            job += p.nwg;
        }
    }
    if (nunits > 0) {
        for (int b = 1; b < 2 * p.M; ++b) {
            asm volatile("" ::: "memory");
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
        }
    }
    while (job < njobs) {
        job_decode(p, job, g, rt, sp);
        kp0 = sp * p.pairs_per_slice;
        kp1 = min(kp0 + p.pairs_per_slice, p.pairs);
        job_load(p, jr, g, rt, kp0, kp1);
        job_store(job_compute());
        job += p.nwg;
    }
    // ---- my share of the sentinels the next launch expects to find in the other buffer.
    //      Placed where nothing waits for the stores: behind the first LDS access that follows
    //      the LDS-direct loads (the compiler makes that access wait for every outstanding
    //      memory operation, stores included), and well before the end of the launch.
    auto fill_other = [&]() {
        const rsrc_t orr = make_rsrc(other, (unsigned)kMailBytes);
        const v4f s4 = __builtin_bit_cast(v4f, (v4u){kSentinel, kSentinel, kSentinel, kSentinel});
        for (unsigned v = (unsigned)c * 64u + l; v < (unsigned)(kMailBytes / 16); v += (unsigned)p.nwg * 64u)
            buf_store16_agent(orr, v * 16u, s4);
    };
    if (nunits == 0) fill_other();

    if (nunits > 0) {
        // ---- collect every slice: h[g][m][j] = SiLU(sum_sp partial) (step 6).  A lane takes four
        //      consecutive ranks of one (layer, token); the layers of the group are laid end to
        //      end so that a single batch of loads -- one round trip -- usually covers them all.
        //      The loads are guarded by their offsets, never by branches.
        // (values first, selects after: a select between two loads from the kernel arguments
        //  would be turned into a load at a per-lane address, through a private copy)
        const int rk0 = p.L[0].rank, rk1 = p.L[1].rank, rk2 = p.L[2].rank, rk3 = p.L[3].rank;
        const int hs0 = p.L[0].hstride, hs1 = p.L[1].hstride, hs2 = p.L[2].hstride, hs3 = p.L[3].hstride;
        // running end of each layer's (token, four ranks) groups
        const int ge0 = rk0 > 0 ? p.M * hs0 / 4 : 0;
        const int ge1 = ge0 + (p.G > 1 && rk1 > 0 ? p.M * hs1 / 4 : 0);
        const int ge2 = ge1 + (p.G > 2 && rk2 > 0 ? p.M * hs2 / 4 : 0);
        const int ge3 = ge2 + (p.G > 3 && rk3 > 0 ? p.M * hs3 / 4 : 0);
        const rsrc_t mr = make_rsrc(mine, (unsigned)kMailBytes);
        _Float16 *hs = reinterpret_cast<_Float16 *>(lds + p.h_off);
        for (int f0 = 0; f0 < ge3; f0 += 64) {
            const int f = f0 + l;
            int gg = 0, first = 0, rank = rk0, hstride = hs0;                // per lane
            if (f >= ge0) { gg = 1; first = ge0; rank = rk1; hstride = hs1; }
            if (f >= ge1) { gg = 2; first = ge1; rank = rk2; hstride = hs2; }
            if (f >= ge2) { gg = 3; first = ge2; rank = rk3; hstride = hs3; }
            const bool inside = f < ge3;
            const int idx = f - first;                                       // (token, four ranks) within the layer
            const int j = (idx * 4) % hstride;
            const bool wanted = inside && j < (rank + 15) / 16 * 16;         // ranks covered by the producers' tiles
            const unsigned at = (unsigned)gg * (unsigned)kMailLayerBytes + (unsigned)idx * 16u;
            const unsigned step = (unsigned)p.M * hstride * 4u;
            v4f part[kFusedSplit];
            int polls = 0;
            while (true) {
                bool ready = true;
#pragma unroll
                for (int sl = 0; sl < kFusedSplit; ++sl) {
                    const v4u raw = buf_load16_agent(mr, at + (unsigned)sl * step, wanted && sl < p.S);
                    ready = ready && raw[0] != kSentinel && raw[1] != kSentinel && raw[2] != kSentinel &&
                            raw[3] != kSentinel;
                    part[sl] = __builtin_bit_cast(v4f, raw);
                }
                if (__builtin_amdgcn_ballot_w64(!ready) == 0) break;
                if (++polls >= kMemPolls) {
                    failed = true;
                    break;
                }
                __builtin_amdgcn_s_sleep(2);
            }
            v4f h = part[0];
#pragma unroll
            for (int sl = 1; sl < kFusedSplit; ++sl) h += part[sl];         // slice order: deterministic
            if (inside) {
                v4h o;
#pragma unroll
                for (int v = 0; v < 4; ++v) o[v] = (j + v < rank) ? (_Float16)silu_fast(h[v]) : (_Float16)0.0f;
                *reinterpret_cast<v4h *>(hs + (gg * p.M + idx * 4 / hstride) * kHsStride + j) = o;
            }
        }

        // ---- per unit: lane n < 32 owns output row n of the unit for every token
        const int *tiles = reinterpret_cast<const int *>(lds + p.tile_off);
        const _Float16 bad = __builtin_bit_cast(_Float16, (unsigned short)0x7e00);
        fill_other();
        // the layers' output descriptions in scalar registers: the loop selects, it never loads
        _Float16 *const y0 = p.L[0].y, *const y1 = p.L[1].y, *const y2 = p.L[2].y, *const y3 = p.L[3].y;
        int32_t *const d0 = p.L[0].acc_debug, *const d1 = p.L[1].acc_debug, *const d2 = p.L[2].acc_debug,
                       *const d3 = p.L[3].acc_debug;
        const int N0 = p.L[0].N, N1 = p.L[1].N, N2 = p.L[2].N, N3 = p.L[3].N;
        const int us1 = p.G > 1 ? p.ustart[1] : 0x7fffffff, us2 = p.G > 2 ? p.ustart[2] : 0x7fffffff,
                  us3 = p.G > 3 ? p.ustart[3] : 0x7fffffff;
        for (int i = 0; i < nunits; ++i) {
            const unsigned char *op = ustage + i * p.unit_stride;
            const int u = c + i * p.nwg;
            int gg = 0, ufirst = 0, LN = N0, Lrank = rk0, Lhstride = hs0;
            _Float16 *Ly = y0;
            int32_t *Ldbg = d0;
            unsigned swb = swb0;
            if (u >= us1) { gg = 1; ufirst = us1; LN = N1; Lrank = rk1; Lhstride = hs1; Ly = y1; Ldbg = d1; swb = swb1; }
            if (u >= us2) { gg = 2; ufirst = us2; LN = N2; Lrank = rk2; Lhstride = hs2; Ly = y2; Ldbg = d2; swb = swb2; }
            if (u >= us3) { gg = 3; ufirst = us3; LN = N3; Lrank = rk3; Lhstride = hs3; Ly = y3; Ldbg = d3; swb = swb3; }
            const int n0 = (u - ufirst) * kTileRows;
            int polls = 0;
            while (!failed && lds_load(&ctl->arrived[i]) < kStream) {
                if (++polls >= kLdsPolls) {
                    failed = true;
                    if (l == 0) __hip_atomic_store(p.flags + 2, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    break;
                }
                __builtin_amdgcn_s_sleep(1);
            }
            // corr[m] of lane n: sum_j h[m][j] B[n0+n][j]  (tokens as matrix rows, as in the streaming side)
            v16f corr = (v16f){};
            float gate = 0.f;
            if (Lrank > 0) {
                gate = tanh_fast((float)*reinterpret_cast<const _Float16 *>(op + p.unit_alpha + jl * 2));
                const _Float16 *hrow = hs + (gg * p.M + jl) * kHsStride + hf * 8;
                const unsigned char *brow = op + (hf * 32 + jl) * 16;
                switch (Lhstride / 16) {
                    case 2: corr = corr_unit<2>(hrow, brow, jl < p.M); break;
                    case 4: corr = corr_unit<4>(hrow, brow, jl < p.M); break;
                    default: corr = corr_unit<8>(hrow, brow, jl < p.M); break;
                }
            }
            const int n = n0 + l;
            if (l < 32 && n < LN) {
                const float s_w = __builtin_bit_cast(float, swb);
#pragma unroll
                for (int m = 0; m < kMaxFusedM; ++m) {
                    if (m < p.M) {
                        const int a = tiles[(i * kMaxFusedM + m) * kTileRows + l] - sh_rs[m];
                        _Float16 o = (_Float16)((float)a * (sh_sx[m] * s_w) + gate * corr[m]);
                        if (failed) o = bad;
                        Ly[(size_t)m * LN + n] = o;
                        if (Ldbg) Ldbg[(size_t)m * LN + n] = a;
                    }
                }
            }
        }
    }

    // ---- the last workgroup to get here advances the launch counter
    if (failed && l == 0) __hip_atomic_store(p.flags + 2, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (l == 0) {
        const int done = __hip_atomic_fetch_add(p.flags + 1, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (done == p.nwg - 1) {
            __hip_atomic_store(p.flags + 1, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(p.flags, (int)(epoch + 1u), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

__global__ __launch_bounds__(512) void fused_kernel(FusedParams p)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    __shared__ Control ctl;
    __shared__ float sh_max[8], sh_sx[kMaxFusedM];
    __shared__ int sh_sum[8], sh_rs[kMaxFusedM];

    const int c = blockIdx.x;
    const int total = p.ustart[p.G];
    const int nunits = c < total ? (total - c + p.nwg - 1) / p.nwg : 0;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    if (w == kStream) {
        if ((threadIdx.x & 63) == 0) {
#pragma unroll
            for (int i = 0; i < kMaxUnits; ++i) ctl.arrived[i] = 0;
        }
        service_wave(p, lds, &ctl, sh_sx, sh_rs, c, nunits);
    } else if (nunits > 0) {
        streaming_wave(p, lds, &ctl, sh_max, sh_sum, sh_sx, sh_rs, c, nunits);
    }
}

int g_num_cus = 0, g_device = -1;
constexpr size_t kFusedLdsMax = 144 * 1024;

}  // namespace

// Fills in the launch shape of a group whose layers, activations and outputs are set
// (M <= kMaxFusedM, d_in % 8 == 0, d_in <= kMaxFusedK, ranks multiples of 8, x and every A
// and B 16-byte aligned, alpha 4-byte aligned).
// False: the group does not fit this path (too many units per workgroup, or LDS).
bool plan_fused(FusedParams &p, size_t *lds_bytes)
{
    // The workgroups exchange partial sums within the launch, so all of them must be resident
    // at once: at most one per compute unit, and only if the occupancy query confirms that a
    // unit holds this kernel at its largest LDS request (asked once per device).
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) {
        (void)hipGetLastError();
        return false;
    }
    if (g_num_cus == 0 || dev != g_device) {
        int n = 0, per_cu = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
            hipFuncSetAttribute(reinterpret_cast<const void *>(fused_kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)kFusedLdsMax) != hipSuccess ||
            hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fused_kernel, 512, kFusedLdsMax) != hipSuccess ||
            per_cu < 1) {
            (void)hipGetLastError();
            return false;
        }
        g_num_cus = n > 0 ? n : 1;
        g_device = dev;
    }
    const int M = p.M;
    p.Kp = round_up(p.K, kTileCols);
    p.KT = p.Kp / kTileCols;
    p.TPW = (p.KT + kStream - 1) / kStream;
    int units = 0, hstride_max = 32;
    for (int g = 0; g < p.G; ++g) {
        p.ustart[g] = units;
        units += p.L[g].RBn;
        if (p.L[g].rank > 0 && p.L[g].hstride > hstride_max) hstride_max = p.L[g].hstride;
    }
    p.ustart[p.G] = units;

    // slices of A x: 512 columns each, at most kFusedSplit and 64 (slice, token) rows per layer
    p.pairs = (p.K + 63) / 64;
    int s = (p.pairs + 7) / 8;
    if (s > kFusedSplit) s = kFusedSplit;
    if (s > 64 / M) s = 64 / M;
    p.pairs_per_slice = (p.pairs + s - 1) / s;
    p.S = (p.pairs + p.pairs_per_slice - 1) / p.pairs_per_slice;
    int jobs = 0;
    for (int g = 0; g < p.G; ++g) {
        p.job_start[g] = jobs;
        if (p.L[g].rank > 0) jobs += ((p.L[g].rank + 15) / 16) * p.S;
    }
    p.job_start[p.G] = jobs;
    int nwg = units > jobs ? units : jobs;
    if (nwg > g_num_cus) nwg = g_num_cus;      // one resident workgroup per compute unit
    p.nwg = nwg;
    const int per_wg = (units + nwg - 1) / nwg;
    if (per_wg > kMaxUnits) return false;

    p.xstride = p.Kp + 16;
    size_t off = ((size_t)M * p.xstride + 15) & ~size_t(15);
    p.tile_off = (int)off;
    off += (size_t)per_wg * kMaxFusedM * kTileRows * sizeof(int);
    p.h_off = (int)off;
    off += (size_t)p.G * M * kHsStride * sizeof(_Float16);
    off = (off + 1023) & ~size_t(1023);
    p.unit_off = (int)off;                     // per unit: B rows (64 bytes per padded rank), then 256 bytes of alpha
    p.unit_alpha = 64 * hstride_max;
    p.unit_stride = p.unit_alpha + 256;
    off += (size_t)per_wg * p.unit_stride;
    *lds_bytes = off;
    return off <= kFusedLdsMax;
}

hipError_t launch_fused(const FusedParams &p, size_t lds_bytes, hipStream_t st)
{
    hipLaunchKernelGGL(fused_kernel, dim3(p.nwg), dim3(512), lds_bytes, st, p);
    return hipGetLastError();
}

}  // namespace hgf
