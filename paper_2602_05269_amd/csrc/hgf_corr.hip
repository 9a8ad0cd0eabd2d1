// Down-projection of the correction path for many tokens (the prefill path):
//   h16[m, j] = fp16( SiLU( sum_k A[j,k] x[m,k] ) ).
//
// Algorithm 1, steps 5-6 of the HGF paper (H <- X A; H <- SiLU(H)) on the UN-quantised
// fp16 activations, with SiLU(h) = h * sigmoid(h) (Sec. 2.3, low-rank correction).
// A skinny GEMM on the 32x32x16 f16 MFMA: matrix rows are rank indices (so a lane ends up
// with four consecutive ranks of one token: 8-byte stores), matrix columns are tokens.
// One workgroup of four wavefronts owns 32 tokens and one tile of 32 ranks of one layer
// (the rank tiles of every layer of the group are numbered through: all layers that read the
// same activations share one launch, which fills the chip where a single layer's 64 token
// tiles would not).  On the prefill path the tiles share their launch with the activation
// quantiser as well (prepare_kernel below).  x and A are streamed through LDS in
// stretches of KC columns with LDS-direct loads (whole row pieces, coalesced; double
// buffered, requested one stretch ahead); each wavefront multiplies a quarter of the stretch
// for every rank tile; the four partial tiles meet in LDS at the end and the first
// wavefront adds them in order (deterministic), applies SiLU and writes fp16.
#include "hgf_internal.h"

namespace hgf {

namespace {

struct CorrParams {
    const _Float16 *x;
    const _Float16 *A;                          // the layer of a ragged launch; of a grouped launch: A4[g]
    _Float16 *h16;
    int M, K, rank, hstride;
    int steps;                                  // stretches of KC columns
    // grouped launch: blockIdx.y walks the 32-rank tiles of up to four layers that read the same x
    int G;
    const _Float16 *A4[kMaxGroup];
    _Float16 *h4[kMaxGroup];
    int rank4[kMaxGroup], hstride4[kMaxGroup];
    int tile_start[kMaxGroup + 1];
};

typedef __attribute__((address_space(3))) void *lds_ptr_t;

// Staged rows are permuted in units of 16 bytes by XOR with (row mod 16): rows are a multiple
// of 256 bytes, so the sixteen lanes that read the same piece of consecutive rows in one LDS
// cycle land on sixteen different 16-byte bank groups.
__device__ inline unsigned slot_of(unsigned piece, unsigned row) { return piece ^ (row & 15u); }

// RT: rank tiles of 32 covering the padded row of h16 (1, 2 or 4).  KC: columns per stretch.
// (bx, by): token tile and rank tile of the workgroup.
template <int RT, int KC>
__device__ inline void corr_down_tile(const CorrParams &p, const int bx, const int by)
{
    constexpr int kRowB = KC * 2;               // bytes per staged row
    constexpr int kPieces = kRowB / 16;         // 16-byte pieces per row = lanes per row of an LDS-direct load
    constexpr int kRowsPerInst = 64 / kPieces;
    constexpr int kXInst = 32 / kRowsPerInst / 4;        // LDS-direct loads per wavefront for x ...
    constexpr int kAInst = RT * 32 / kRowsPerInst / 4;   // ... and for A, per stretch
    // separately declared buffers: the compiler can prove an LDS-direct load into one stage
    // does not alias the reads of the other and leaves it in flight
    __shared__ __attribute__((aligned(1024))) unsigned char xs0[32 * kRowB], xs1[32 * kRowB];
    __shared__ __attribute__((aligned(1024))) unsigned char as0[RT * 32 * kRowB], as1[RT * 32 * kRowB];

    const int tid = threadIdx.x, l = tid & 63, jl = l & 31, hf = l >> 5;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int m0 = bx * 32;
    const int mrows = min(32, p.M - m0);
    // this workgroup's layer and first rank (RT tiles of 32 from there)
    int g = 0;
#pragma unroll
    for (int i = 1; i < kMaxGroup; ++i)
        if (i < p.G && by >= p.tile_start[i]) g = i;
    const int j_first = (by - p.tile_start[g]) * 32 * RT;
    const int rank = p.rank4[g], hstride = p.hstride4[g];
    _Float16 *const h16 = p.h4[g];
    const int arows = min(RT * 32, rank - j_first);          // rows of A this workgroup reads (may be <= 0)
    const rsrc_t xr = make_rsrc(p.x + (size_t)m0 * p.K, (unsigned)mrows * p.K * 2u);
    const rsrc_t ar = make_rsrc(p.A4[g] + (size_t)j_first * p.K, arows > 0 ? (unsigned)arows * p.K * 2u : 0u);

    // Staging: one instruction moves 1 KiB = kRowsPerInst rows; lane L writes row
    // kRowsPerInst*ii + L/kPieces, slot L%kPieces.  Rows beyond the last token / rank lie
    // outside the descriptors and arrive as zeros; columns beyond d_in are guarded (they
    // would otherwise read the next row).
    auto stage = [&](unsigned char *xb, unsigned char *ab, int st) {
        const int k0 = st * KC;
#pragma unroll
        for (int i = 0; i < kXInst; ++i) {
            const unsigned ii = 4 * i + w, row = kRowsPerInst * ii + l / kPieces;
            const int col = k0 + (int)slot_of(l % kPieces, row) * 8;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(xr, (lds_ptr_t)(xb + ii * 1024), 16,
                                                     (int)(col < p.K ? (row * p.K + col) * 2u : kOob), 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < kAInst; ++i) {
            const unsigned ii = 4 * i + w, row = kRowsPerInst * ii + l / kPieces;
            const int col = k0 + (int)slot_of(l % kPieces, row) * 8;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(ar, (lds_ptr_t)(ab + ii * 1024), 16,
                                                     (int)(col < p.K ? (row * p.K + col) * 2u : kOob), 0, 0, 0);
        }
    };

    v16f acc[RT];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) acc[rt] = (v16f){};

    // Wavefront w multiplies columns (KC/4)*w .. of the stretch: KC/64 MFMA k-steps of 16;
    // lane (jl, hf) reads piece (KC/32)*w + 2*u + hf of row jl (tokens) / 32*rt + jl (ranks).
    auto compute = [&](const unsigned char *xb, const unsigned char *ab) {
#pragma unroll
        for (int u = 0; u < KC / 64; ++u) {
            const unsigned piece = (KC / 32) * w + 2 * u + hf;
            const v8h b = *reinterpret_cast<const v8h *>(xb + jl * kRowB + slot_of(piece, jl) * 16);
#pragma unroll
            for (int rt = 0; rt < RT; ++rt) {
                const unsigned row = rt * 32 + jl;
                const v8h a = *reinterpret_cast<const v8h *>(ab + row * kRowB + slot_of(piece, row) * 16);
                acc[rt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, acc[rt], 0, 0, 0);
            }
        }
    };

    // A step waits for its own stage only (the next one stays in flight), meets the others at
    // a bare barrier, computes, waits until its LDS reads have RETURNED (the compiler sinks
    // MFMAs and the waits for their operands below the barrier otherwise, so reads would still
    // be queued while the buffers are handed over), meets the others again (everyone is done
    // reading) and requests the stage after next into the same buffers.  The wait matters at
    // the end of the row: the requests beyond the last stretch are out of range, so their
    // zeros come back without a memory round trip and would overtake reads still in flight.
    constexpr int kLoads = kXInst + kAInst;     // vector memory operations per wavefront and stage
    constexpr int kWaitNextInFlight = (kLoads & 0xF) | (7 << 4) | (15 << 8) | ((kLoads >> 4) << 14);
#define HGF_CSTEP(XC, AC, ST)                                  \
    do {                                                       \
        __builtin_amdgcn_s_waitcnt(kWaitNextInFlight);         \
        asm volatile("" ::: "memory");                         \
        __builtin_amdgcn_s_barrier();                          \
        asm volatile("" ::: "memory");                         \
        compute(XC, AC);                                       \
        __builtin_amdgcn_s_waitcnt(0xC07F);     /* lgkmcnt(0) */ \
        asm volatile("" ::: "memory");                         \
        __builtin_amdgcn_s_barrier();                          \
        asm volatile("" ::: "memory");                         \
        stage(XC, AC, (ST) + 2);                               \
    } while (0)
    stage(xs0, as0, 0);
    stage(xs1, as1, 1);
    int st = 0;
    for (; st + 1 < p.steps; st += 2) {
        HGF_CSTEP(xs0, as0, st);
        HGF_CSTEP(xs1, as1, st + 1);
    }
    if (st < p.steps) HGF_CSTEP(xs0, as0, st);
#undef HGF_CSTEP
    __syncthreads();                             // drains the unused tail loads; buffers are free

    // ---- add the four partial tiles (through the A buffers), SiLU, store
    // 4 KiB * RT each: wavefront 1 -> as0, 2 -> as1, 3 -> second part of as0
    float *red = reinterpret_cast<float *>(w == 2 ? as1 : (w == 3 ? as0 + RT * 4096 : as0));
    if (w > 0) {
#pragma unroll
        for (int rt = 0; rt < RT; ++rt)
#pragma unroll
            for (int e = 0; e < 16; ++e) red[(rt * 16 + e) * 64 + l] = acc[rt][e];
    }
    __syncthreads();
    if (w > 0) return;
#pragma unroll
    for (int s = 1; s < 4; ++s) {
        const float *part = reinterpret_cast<const float *>(s == 2 ? as1 : (s == 3 ? as0 + RT * 4096 : as0));
#pragma unroll
        for (int rt = 0; rt < RT; ++rt)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[rt][e] += part[(rt * 16 + e) * 64 + l];
    }

    // acc[rt][4q+v]: rank rt*32 + 8q + 4hf + v of token m0 + jl
    const int m = m0 + jl;
    if (m >= p.M) return;
    _Float16 *hrow = h16 + (size_t)m * hstride;
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int j0 = j_first + rt * 32 + 8 * q + 4 * hf;
            v4h o;
#pragma unroll
            for (int v = 0; v < 4; ++v) o[v] = (j0 + v < rank) ? (_Float16)silu(acc[rt][4 * q + v]) : (_Float16)0.0f;
            *reinterpret_cast<v4h *>(hrow + j0) = o;
        }
    }
}

template <int RT, int KC>
__global__ __launch_bounds__(256) void corr_down_kernel(CorrParams p)
{
    corr_down_tile<RT, KC>(p, blockIdx.x, blockIdx.y);
}

// The activation quantiser (Sec. 2.2.1 of the HGF paper; Algorithm 1, steps 1-2; the arithmetic
// of quantize_kernel, bit for bit) with one wavefront per token: the row stays in registers
// between the absmax pass and the rounding pass (NV 16-byte pieces per lane: d_in <= 512 NV),
// so x is read once and nothing goes through LDS.
struct QuantParams {
    const _Float16 *x;
    int8_t *xq;
    float *s_x;
    int32_t *rowsum;
    int M, K, Kp;
};

template <int NV>
__device__ inline void quantize_row(const QuantParams &q, const int m, const int l)
{
    if (m >= q.M) return;
    const rsrc_t xr = make_rsrc(q.x + (size_t)m * q.K, (unsigned)q.K * 2u);
    v4u raw[NV];
#pragma unroll
    for (int i = 0; i < NV; ++i) raw[i] = buf_load16(xr, (unsigned)(i * 64 + l) * 16u);   // beyond the row: zeros
    float amax = 0.0f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const v8h v = __builtin_bit_cast(v8h, raw[i]);
#pragma unroll
        for (int j = 0; j < 8; ++j) amax = fmaxf(amax, fabsf((float)v[j]));
    }
    amax = fmaxf(wave_max(amax), 1e-5f);
    const float inv = 127.0f / amax;
    int sum = 0;
    uint2 *out8 = reinterpret_cast<uint2 *>(q.xq + (size_t)m * q.Kp);
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const v8h v = __builtin_bit_cast(v8h, raw[i]);
        uint32_t w[2] = {0u, 0u};
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int c = quant1((float)v[j], inv);
            sum += c;
            w[j >> 2] |= (uint32_t)(c & 0xff) << (8 * (j & 3));
        }
        if ((i * 64 + l) * 8 < q.Kp) out8[i * 64 + l] = make_uint2(w[0], w[1]);
    }
    sum = wave_sum(sum);
    if (l == 0) {
        q.s_x[m] = amax / 127.0f;
        if (q.rowsum) q.rowsum[m] = sum;
    }
}

// Both halves of the preparation of a group of prefill layers in one launch: the first
// `ncorr` workgroups are the down-projection tiles (few, long: a dozen dependent memory
// round trips each), the rest quantise four tokens each (many, short) and fill the compute
// units the tiles leave idle.  Both only read x.
template <int NV>
__global__ __launch_bounds__(256) void prepare_kernel(CorrParams p, QuantParams q, int ncorr, int token_tiles)
{
    const int b = blockIdx.x;
    if (b < ncorr) {
        corr_down_tile<1, 256>(p, b % token_tiles, b / token_tiles);
    } else {
        const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
        quantize_row<NV>(q, (b - ncorr) * 4 + w, threadIdx.x & 63);
    }
}

// d_in % 8 != 0 (rows not 16-byte aligned): one thread per (token, rank) pair with plain
// loads.  Slow and simple, for odd shapes only.
__global__ __launch_bounds__(256) void corr_down_ragged_kernel(CorrParams p)
{
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (size_t)p.M * p.hstride) return;
    const int m = (int)(idx / p.hstride), j = (int)(idx % p.hstride);
    float h = 0.f;
    if (j < p.rank) {
        const _Float16 *xrow = p.x + (size_t)m * p.K, *arow = p.A + (size_t)j * p.K;
        for (int k = 0; k < p.K; ++k) h += (float)arow[k] * (float)xrow[k];
        h = silu(h);
    }
    p.h16[idx] = (_Float16)h;
}

}  // namespace

// Layers 0..G-1 read the same x; layer g's result goes to h16[g] ([M, h_stride(rank[g])] fp16).
// With xq != nullptr the quantised activations, their scales and sums are produced as well --
// in the same launch where the shapes allow it, by launch_quantize before otherwise.
hipError_t launch_corr_down(const _Float16 *x, int M, int K, int G, const _Float16 *const *A, const int *rank,
                            _Float16 *const *h16, int8_t *xq, float *s_x, int32_t *rowsum, hipStream_t st)
{
    CorrParams p;
    p.x = x;
    p.M = M;
    p.K = K;
    bool vec = (K % 8 == 0) && (reinterpret_cast<uintptr_t>(x) % 16 == 0);
    for (int g = 0; g < G; ++g) vec = vec && (rank[g] == 0 || reinterpret_cast<uintptr_t>(A[g]) % 16 == 0);
    const bool together = vec && xq != nullptr && K <= 512 * 32;
    if (xq != nullptr && !together) {
        const hipError_t e = launch_quantize(x, M, K, xq, s_x, rowsum, st);
        if (e != hipSuccess) return e;
    }
    if (!vec) {
        for (int g = 0; g < G; ++g) {
            if (rank[g] == 0) continue;
            p.A = A[g];
            p.h16 = h16[g];
            p.rank = rank[g];
            p.hstride = h_stride(rank[g]);
            const size_t n = (size_t)M * p.hstride;
            hipLaunchKernelGGL(corr_down_ragged_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, p);
        }
        return hipGetLastError();
    }
    int tiles = 0;
    p.G = G;
    for (int g = 0; g < kMaxGroup; ++g) {
        p.tile_start[g] = tiles;
        p.A4[g] = g < G ? A[g] : nullptr;
        p.h4[g] = g < G ? h16[g] : nullptr;
        p.rank4[g] = g < G ? rank[g] : 0;
        p.hstride4[g] = g < G ? h_stride(rank[g]) : 32;
        if (g < G && rank[g] > 0) tiles += p.hstride4[g] / 32;     // tiles cover the padded row: every column is written
    }
    p.tile_start[kMaxGroup] = tiles;
    p.steps = (K + 255) / 256;
    const int token_tiles = (M + 31) / 32;
    if (together) {
        QuantParams q;
        q.x = x;
        q.xq = xq;
        q.s_x = s_x;
        q.rowsum = rowsum;
        q.M = M;
        q.K = K;
        q.Kp = round_up(K, kTileCols);
        const int ncorr = token_tiles * tiles;
        const dim3 grid(ncorr + (M + 3) / 4), block(256);
        const int pieces = (q.Kp + 511) / 512;
        if (pieces <= 8) hipLaunchKernelGGL(prepare_kernel<8>, grid, block, 0, st, p, q, ncorr, token_tiles);
        else if (pieces <= 16) hipLaunchKernelGGL(prepare_kernel<16>, grid, block, 0, st, p, q, ncorr, token_tiles);
        else hipLaunchKernelGGL(prepare_kernel<32>, grid, block, 0, st, p, q, ncorr, token_tiles);
        return hipGetLastError();
    }
    if (tiles == 0) return hipSuccess;
    hipLaunchKernelGGL((corr_down_kernel<1, 256>), dim3(token_tiles, tiles), dim3(256), 0, st, p);
    return hipGetLastError();
}

}  // namespace hgf
