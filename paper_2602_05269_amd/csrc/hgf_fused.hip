// Fused decode launch for a handful of tokens (M <= 4): every step of the layer in ONE
// kernel, for up to four layers that read the same activations.
//
// Algorithm 1 of the HGF paper, steps 1-8.  At batch 1 the layer is a single pass over
// the packed weights; split over several launches, the launch-to-launch gaps and each
// launch's own memory round trips cost as much as the pass itself.  Here
//   * the first `ncorr` workgroups compute fp32 partial sums of A x (step 5) on the
//     16x16x32 f16 MFMA, one wavefront per (layer, 16-rank tile, 512-column slice), and
//     publish them with device-coherent stores followed by one counter increment;
//   * every other workgroup requests, in one burst, its token rows, its epilogue operands
//     and its first weight tiles; quantises the tokens itself into LDS while the weights
//     are in flight (steps 1-2: the quantised row never goes to memory); waits for the
//     counter; adds the slices in order, applies SiLU (step 6) and proceeds as the stand-
//     alone decode kernel: int8 MFMA over 2-bit codes (step 3), dequantisation (step 4),
//     up-projection on the f16 MFMA and gate (steps 7-8).
// Workgroups are dispatched in index order, so the correction workgroups hold their
// resources before any workgroup that waits for them; the wait is bounded all the same
// (on expiry the workgroup's outputs are NaN and a sticky flag is set in the workspace).
// The last decode workgroup to finish clears the counters for the next launch.
#include "hgf_internal.h"

namespace hgf {

namespace {

constexpr int kXV = 6;                 // 16-byte pieces of a token row per thread (256 threads: 12288 columns)
constexpr int kSpinLimit = 1 << 20;    // polls of the counter before giving up (about a second)

// One wavefront: rank tile `rt` of layer `g`, slice `sp` of d_in, all (<= 4) tokens.
// Lane (i = l%16, kb = l/16) holds A[rt*16+i][k] and x[i][k] for the same eight k per MFMA:
// k = 64*kp + 16*kb + 0..7 and + 8..15, so a row is read 128 contiguous bytes at a time.
__device__ void corr_job(const FusedParams &p, int job)
{
    int g = 0;
    while (g + 1 < p.G && job >= p.job_start[g + 1]) ++g;
    const DecLayer &L = p.L[g];
    const int local = job - p.job_start[g];
    const int rt = local / p.S, sp = local % p.S;
    const int l = threadIdx.x & 63, i = l & 15, kb = l >> 4;
    const int j = rt * 16 + i;
    const bool j_ok = j < L.rank, m_ok = i < p.M;
    const rsrc_t ar = make_rsrc(p.A[g], (unsigned)L.rank * p.K * 2u);
    const rsrc_t xr = make_rsrc(p.x, (unsigned)p.M * p.K * 2u);

    v4f acc = {0.f, 0.f, 0.f, 0.f};
    const int kp0 = sp * p.pairs_per_slice;
    const int kp1 = min(kp0 + p.pairs_per_slice, p.pairs);
    constexpr int UN = 8;                      // 64-column steps requested together
    for (int kpb = kp0; kpb < kp1; kpb += UN) {
        v8h a[UN][2], b[UN][2];
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            const int k0 = (kpb + u) * 64 + kb * 16;
            const bool ok = (kpb + u) < kp1;
            a[u][0] = buf_load8h<true>(ar, (unsigned)j * p.K + k0, p.K - k0, ok && j_ok);
            a[u][1] = buf_load8h<true>(ar, (unsigned)j * p.K + k0 + 8, p.K - k0 - 8, ok && j_ok);
            b[u][0] = buf_load8h<true>(xr, (unsigned)i * p.K + k0, p.K - k0, ok && m_ok);
            b[u][1] = buf_load8h<true>(xr, (unsigned)i * p.K + k0 + 8, p.K - k0 - 8, ok && m_ok);
        }
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[u][0], b[u][0], acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[u][1], b[u][1], acc, 0, 0, 0);
        }
    }
    // acc[v]: rank index rt*16 + 4*kb + v of token i  ->  hpart[sp][i][hstride]
    const rsrc_t hr = make_rsrc(L.hpart, (unsigned)p.S * p.M * L.hstride * 4u);
    buf_store16_agent(hr, m_ok ? (unsigned)(((sp * p.M + i) * L.hstride + rt * 16 + 4 * kb) * 4) : kOob, acc);
}

__global__ __launch_bounds__(512) void fused_kernel(FusedParams p)
{
    constexpr int PF = 8;                           // weight tiles in flight per wavefront
    constexpr int JS = HGF_MAX_RANK / 16;           // steps of the 32x32x16 f16 MFMA over the rank
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    __shared__ float sh_max[8], sh_sx[kMaxFusedM];
    __shared__ int sh_sum[8], sh_rs[kMaxFusedM], sh_expired;

    const int tid = threadIdx.x, nthreads = blockDim.x, l = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6), nw = nthreads >> 6;

    // ======================= correction workgroups =======================
    if ((int)blockIdx.x < p.ncorr) {
        const int job = (int)blockIdx.x * nw + w;
        if (job < p.job_start[p.G]) corr_job(p, job);
        __builtin_amdgcn_s_waitcnt(0);              // the stores have been acknowledged
        asm volatile("" ::: "memory");
        __syncthreads();
        if (tid == 0) __hip_atomic_fetch_add(p.flags, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return;
    }

    // ========================= decode workgroups =========================
    const int wg = (int)blockIdx.x - p.ncorr;
    DecLayer L = p.L[0];
    int wg0 = 0;
#pragma unroll
    for (int i = 1; i < kMaxGroup; ++i) {
        if (i < p.G && wg >= p.wg_start[i]) {
            L = p.L[i];
            wg0 = p.wg_start[i];
        }
    }
    const int rw = w / p.KW, kw = w % p.KW;
    const int rb_first = (wg - wg0) * p.RW;          // first row-block of the workgroup
    const int rb = rb_first + rw;                    // this wavefront's row-block
    const bool rb_ok = rb < L.RBn;
    const int jl = l & 31, hf = l >> 5;              // matrix column / row index, and k-half
    const int n0 = rb * kTileRows;                   // this wavefront's 32 output rows
    const bool owner = rb_ok && kw == 0;             // runs the epilogue of the row-block

    // ---- (1) the first token row, 16 bytes per thread and piece
    const rsrc_t xr = make_rsrc(p.x, (unsigned)p.M * p.K * 2u);
    v8h keep[kXV];
#pragma unroll
    for (int r = 0; r < kXV; ++r) {
        const int i = tid + r * nthreads;
        keep[r] = __builtin_bit_cast(v8h, buf_load16(xr, (unsigned)i * 16u, i * 8 < p.K));
    }

    // ---- (2) epilogue operands: gate parameter of the workgroup's rows, B rows of the owner
    float alpha_pre;
    {
        const rsrc_t ar = make_rsrc(L.alpha, L.rank > 0 ? (unsigned)L.N * 2u : 0u);
        const int n = rb_first * kTileRows + tid;
        alpha_pre = (float)half_bits(buf_load2(ar, (unsigned)n * 2u, tid < p.RW * kTileRows && n < L.N));
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

    // ---- (3) first batch of weight tiles: the bulk of the bytes
    const v4u *rb_tiles = L.packed + (size_t)(rb_ok ? rb : 0) * p.KT * 64;
    const rsrc_t wr = make_rsrc(rb_tiles, rb_ok ? (unsigned)p.KT * kTileBytes : 0u);
    int kt0 = kw;
    v4u wq[PF];
#pragma unroll
    for (int t = 0; t < PF; ++t) wq[t] = buf_load16_stream(wr, (unsigned)(kt0 + t * p.KW) * kTileBytes + l * 16);

    // ---- per-token absmax int8 quantisation into LDS (Sec. 2.2.1), one token after the other
    // (the first row is handled outside the loop: its wait must not cover the loads behind it)
    const int nvec_p = p.Kp / 8;
    auto quantise_row = [&](int m) {
        float amax = 0.0f;
#pragma unroll
        for (int r = 0; r < kXV; ++r)
#pragma unroll
            for (int e = 0; e < 8; ++e) amax = fmaxf(amax, fabsf((float)keep[r][e]));
        amax = wave_max(amax);
        if (l == 0) sh_max[w] = amax;
        __syncthreads();
        amax = sh_max[0];
        for (int i = 1; i < nw; ++i) amax = fmaxf(amax, sh_max[i]);
        amax = fmaxf(amax, 1e-5f);
        const float inv = 127.0f / amax;
        int sum = 0;
#pragma unroll
        for (int r = 0; r < kXV; ++r) {
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
            for (int i = 1; i < nw; ++i) s += sh_sum[i];
            sh_sx[m] = amax / 127.0f;
            sh_rs[m] = s;
        }
    };
    quantise_row(0);
    for (int m = 1; m < p.M; ++m) {
#pragma unroll
        for (int r = 0; r < kXV; ++r) {
            const int i = tid + r * nthreads;
            keep[r] = __builtin_bit_cast(v8h, buf_load16(xr, ((unsigned)m * p.K + (unsigned)i * 8u) * 2u, i * 8 < p.K));
        }
        quantise_row(m);
    }

    // ---- wait for the correction workgroups (bounded)
    if (tid == 0) {
        int expired = 0;
        if (p.ncorr > 0) {
            int polls = 0;
            while (__hip_atomic_load(p.flags, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < p.ncorr) {
                if (++polls >= kSpinLimit) {
                    expired = 1;
                    __hip_atomic_store(p.flags + 2, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    break;
                }
                __builtin_amdgcn_s_sleep(2);
            }
        }
        sh_expired = expired;
    }
    __syncthreads();
    const bool expired = sh_expired != 0;

    // ---- SiLU(A x) of the tokens (fp16 rows of hstride) and tanh(alpha) into LDS
    _Float16 *hs = reinterpret_cast<_Float16 *>(lds + p.h_off);
    float *gs = reinterpret_cast<float *>(lds + p.g_off);
    const rsrc_t hr = make_rsrc(L.hpart, L.rank > 0 ? (unsigned)p.S * p.M * L.hstride * 4u : 0u);
    const int htotal = L.rank > 0 ? p.M * L.hstride : 0;
    for (int idx = tid; idx < htotal; idx += nthreads) {
        const int j = idx % L.hstride;
        float part[kMaxHSplit];
#pragma unroll
        for (int sp = 0; sp < kMaxHSplit; ++sp)
            part[sp] = __builtin_bit_cast(float, buf_load4_agent(hr, ((unsigned)idx + (unsigned)sp * p.M * L.hstride) * 4u,
                                                                 j < L.rank && sp < p.S));
        float h = part[0];
#pragma unroll
        for (int sp = 1; sp < kMaxHSplit; ++sp) h += part[sp];        // slice order: deterministic
        hs[idx] = (_Float16)silu(h);
    }
    if (tid < p.RW * kTileRows) gs[tid] = L.rank > 0 ? tanhf(alpha_pre) : 0.f;
    __syncthreads();

    // ---- ternary x int8 contraction: this wavefront's tiles kw, kw + KW, ...
    v16i acc = (v16i){};
    while (true) {
#pragma unroll
        for (int t = 0; t < PF; ++t) {
            const int kt = kt0 + t * p.KW;
            if (kt < p.KT) {
                const unsigned char *xrow = lds + kt * kTileCols + hf * 16;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const v4i a = widen_codes(wq[t][q]);
                    v4i b = (v4i){0, 0, 0, 0};
                    if (jl < p.M) b = *reinterpret_cast<const v4i *>(xrow + jl * p.xstride + q * 32);
                    acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, acc, 0, 0, 0);
                }
            }
        }
        kt0 += p.KW * PF;
        if (kt0 >= p.KT) break;
#pragma unroll
        for (int t = 0; t < PF; ++t) wq[t] = buf_load16_stream(wr, (unsigned)(kt0 + t * p.KW) * kTileBytes + l * 16);
    }

    // ---- add the KW partial tiles of a row-block: its first wavefront ends up owning it
    if (p.KW > 1) {
        __syncthreads();                             // the activations in LDS are no longer needed
        v16i *red = reinterpret_cast<v16i *>(lds);
        const int slot0 = w - rw - 1;               // the non-owning wavefronts, densely numbered
        if (kw > 0) red[slot0 * 64 + l] = acc;
        __syncthreads();
        if (kw > 0) return;
        for (int o = 1; o < p.KW; ++o) acc += red[(slot0 + o) * 64 + l];
    }

    if (rb_ok && n0 < L.N) {
        // ---- correction up-projection: corr[m,n] = sum_j B[n,j] h[m,j] on the f16 MFMA
        v16f corr = (v16f){};
        if (L.rank > 0) {
#pragma unroll
            for (int js = 0; js < JS; ++js) {
                if (js * 16 < L.hstride) {
                    v8h b = {0, 0, 0, 0, 0, 0, 0, 0};
                    if (jl < p.M) b = *reinterpret_cast<const v8h *>(hs + jl * L.hstride + js * 16 + hf * 8);
                    corr = __builtin_amdgcn_mfma_f32_32x32x16_f16(breg[js], b, corr, 0, 0, 0);
                }
            }
        }
        // ---- dequantise, gate, store.  Element 4*q + v of a lane's accumulator is row
        //      8*q + 4*hf + v of the row-block, for the token of the lane.
        if (jl < p.M) {
            const int m = jl;
            const bool nvec = (L.N % 4) == 0;
            const float scale = sh_sx[m] * s_w;
            const int rs = sh_rs[m];
            const _Float16 bad = __builtin_bit_cast(_Float16, (unsigned short)0x7e00);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int r0 = 8 * q + 4 * hf;
                const int nl = n0 + r0;
                int a[4];
                v4h o;
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    a[v] = acc[4 * q + v] - rs;
                    o[v] = (_Float16)((float)a[v] * scale + gs[rw * kTileRows + r0 + v] * corr[4 * q + v]);
                    if (expired) o[v] = bad;
                }
                const size_t at = (size_t)m * L.N + nl;
                if (nvec && nl + 3 < L.N) {
                    *reinterpret_cast<v4h *>(L.y + at) = o;
                    if (L.acc_debug) *reinterpret_cast<v4i *>(L.acc_debug + at) = (v4i){a[0], a[1], a[2], a[3]};
                } else {
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        if (nl + v < L.N) {
                            L.y[at + v] = o[v];
                            if (L.acc_debug) L.acc_debug[at + v] = a[v];
                        }
                    }
                }
            }
        }
    }

    // ---- the last decode workgroup to get here leaves the counters zero for the next launch
    if (w == 0 && l == 0) {
        const int done = __hip_atomic_fetch_add(p.flags + 1, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (done == p.wg_start[p.G] - 1) {
            __hip_atomic_store(p.flags, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(p.flags + 1, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

}  // namespace

// Fills in the launch shape of a group whose layers, activations and outputs are set
// (M <= kMaxFusedM, d_in % 8 == 0, d_in <= kMaxFusedK, x and every A 16-byte aligned).
hipError_t launch_fused(FusedParams &p, hipStream_t st)
{
    const int M = p.M;
    p.Kp = round_up(p.K, kTileCols);
    p.KT = p.Kp / kTileCols;
    int rb_total = 0, hstride_max = 32;
    for (int g = 0; g < p.G; ++g) {
        rb_total += p.L[g].RBn;
        if (p.L[g].hstride > hstride_max) hstride_max = p.L[g].hstride;
    }
    // wavefronts per row-block: as for the stand-alone decode kernel
    int kw = 1;
    while (kw < 8 && kw * 2 <= p.KT && rb_total * kw < decode_target_waves()) kw *= 2;
    p.KW = kw;
    p.RW = kw >= 4 ? 1 : 4 / kw;
    const int nwaves = p.RW * p.KW;
    int wgs = 0;
    for (int g = 0; g < p.G; ++g) {
        p.wg_start[g] = wgs;
        wgs += (p.L[g].RBn + p.RW - 1) / p.RW;
    }
    p.wg_start[p.G] = wgs;

    // correction jobs: slices of 512 columns, at most kMaxHSplit of them
    p.pairs = (p.K + 63) / 64;
    int s = (p.pairs + 7) / 8;
    if (s > kMaxHSplit) s = kMaxHSplit;
    if (s > 64 / M) s = 64 / M;                 // the workspace holds 64 (slice, token) rows per layer
    p.pairs_per_slice = (p.pairs + s - 1) / s;
    p.S = (p.pairs + p.pairs_per_slice - 1) / p.pairs_per_slice;
    int jobs = 0;
    for (int g = 0; g < p.G; ++g) {
        p.job_start[g] = jobs;
        if (p.L[g].rank > 0) jobs += ((p.L[g].rank + 15) / 16) * p.S;
    }
    p.job_start[p.G] = jobs;
    p.ncorr = (jobs + nwaves - 1) / nwaves;

    const size_t hbytes = (size_t)M * hstride_max * sizeof(_Float16);
    const size_t gbytes = (size_t)p.RW * kTileRows * sizeof(float);
    p.xstride = p.Kp + 16;
    size_t stage = (size_t)M * p.xstride;
    const size_t red = (size_t)(nwaves - p.RW) * 64 * sizeof(v16i);
    if (stage < red) stage = red;
    stage = (stage + 15) & ~size_t(15);
    p.h_off = (int)stage;
    p.g_off = (int)(stage + ((hbytes + 15) & ~size_t(15)));
    const size_t lds = p.g_off + gbytes;

    hipLaunchKernelGGL(fused_kernel, dim3(p.ncorr + wgs), dim3(64 * nwaves), lds, st, p);
    return hipGetLastError();
}

}  // namespace hgf
