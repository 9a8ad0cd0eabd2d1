// Internal declarations shared by the HIP sources of libhgf (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>
#include <stddef.h>

#include "../../include/hgf.h"

namespace hgf {

constexpr int kTileRows = 32;        // a packed tile covers 32 rows ...
constexpr int kTileCols = 128;       // ... by 128 columns of 2-bit codes
constexpr int kTileBytes = 1024;
// Tokens the two-launch decode path handles (4 token tiles of 16).  It is taken up to 40 tokens
// always and up to 64 for groups of few rows (takes_decode_path in hgf_api.hip): on the 7B-shape
// FFN block it costs 43 us at 8 tokens, 58 at 32, 82 at 48, where the prefill path costs the same
// 91-95 us for anything from 41 to 128.
constexpr int kMaxDecodeM = 64;
constexpr int kMaxGroup = 4;         // layers reading the same activations launched together

typedef int v4i __attribute__((ext_vector_type(4)));
typedef unsigned int v4u __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef _Float16 v4h __attribute__((ext_vector_type(4)));

// ---- branch-free guarded loads ---------------------------------------------------------
// A load inside a conditional makes the compiler wait for every outstanding load at the
// join, which serialises the memory pipeline.  These helpers go through a buffer
// descriptor instead: an offset at or beyond the descriptor's size reads as zero, so a
// guard becomes a select on the offset and the loads stay back to back.
typedef __amdgpu_buffer_rsrc_t rsrc_t;
constexpr unsigned kOob = 0xFFFFFF00u;         // beyond any descriptor in this library
__device__ inline rsrc_t make_rsrc(const void *base, unsigned bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, (int)bytes, 0x00020000);
}
__device__ inline v4u buf_load16(rsrc_t r, unsigned off, bool ok = true)
{
    return __builtin_bit_cast(v4u, __builtin_amdgcn_raw_buffer_load_b128(r, (int)(ok ? off : kOob), 0, 0));
}
__device__ inline v4u buf_load16_stream(rsrc_t r, unsigned off)   // read-once data: non-temporal
{
    return __builtin_bit_cast(v4u, __builtin_amdgcn_raw_buffer_load_b128(r, (int)off, 0, 2));
}
__device__ inline unsigned buf_load4(rsrc_t r, unsigned off, bool ok = true)
{
    return (unsigned)__builtin_amdgcn_raw_buffer_load_b32(r, (int)(ok ? off : kOob), 0, 0);
}
__device__ inline unsigned short buf_load2(rsrc_t r, unsigned off, bool ok = true)
{
    return (unsigned short)__builtin_amdgcn_raw_buffer_load_b16(r, (int)(ok ? off : kOob), 0, 0);
}
__device__ inline _Float16 half_bits(unsigned short u) { return __builtin_bit_cast(_Float16, u); }
// Eight consecutive fp16 of a row-major matrix behind `r`, starting at element `elem`;
// elements at column >= cols_left read as zero.  VEC: the eight are 16-byte aligned and
// all in range or all out.
template <bool VEC>
__device__ inline v8h buf_load8h(rsrc_t r, unsigned elem, int cols_left, bool ok)
{
    if (VEC) return __builtin_bit_cast(v8h, buf_load16(r, elem * 2u, ok && cols_left > 0));
    v8h v;
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = half_bits(buf_load2(r, (elem + e) * 2u, ok && e < cols_left));
    return v;
}

// Same, visible to every compute unit of the device: partial results that one workgroup
// writes and another reads within a single launch bypass the per-XCD L2 (sc1).
__device__ inline unsigned buf_load4_agent(rsrc_t r, unsigned off, bool ok = true)
{
    return (unsigned)__builtin_amdgcn_raw_buffer_load_b32(r, (int)(ok ? off : kOob), 0, 16);
}
__device__ inline void buf_store16_agent(rsrc_t r, unsigned off, v4f v)
{
    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(v4u, v), r, (int)off, 0, 16);
}

// ---- arithmetic shared by the kernels ---------------------------------------------------
// Four bytes of 2-bit codes (T+1) -> the four int8 operand registers of one MFMA.
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
// Wave-wide reductions with the result in every lane.  The lanes of a row of 16 exchange
// through the data-parallel-primitive modifiers of the vector ALU (xor 1, xor 2, mirror within
// 8, mirror within 16: four dependent instructions); the four rows are then combined from
// scalar reads of one lane each.  (A shuffle through LDS per butterfly step costs an LDS
// round trip each: six in a row were half a microsecond of the decode chain.)
template <int CTRL>
__device__ inline int dpp_move(int v)
{
    return __builtin_amdgcn_update_dpp(v, v, CTRL, 0xF, 0xF, false);
}
__device__ inline float wave_max(float v)
{
    v = fmaxf(v, __builtin_bit_cast(float, dpp_move<0xB1>(__builtin_bit_cast(int, v))));    // quad_perm [1,0,3,2]
    v = fmaxf(v, __builtin_bit_cast(float, dpp_move<0x4E>(__builtin_bit_cast(int, v))));    // quad_perm [2,3,0,1]
    v = fmaxf(v, __builtin_bit_cast(float, dpp_move<0x141>(__builtin_bit_cast(int, v))));   // row_half_mirror
    v = fmaxf(v, __builtin_bit_cast(float, dpp_move<0x140>(__builtin_bit_cast(int, v))));   // row_mirror
    const int b = __builtin_bit_cast(int, v);
    const float r0 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 0));
    const float r1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 16));
    const float r2 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 32));
    const float r3 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 48));
    return fmaxf(fmaxf(r0, r1), fmaxf(r2, r3));
}
__device__ inline int wave_sum(int v)
{
    v += dpp_move<0xB1>(v);
    v += dpp_move<0x4E>(v);
    v += dpp_move<0x141>(v);
    v += dpp_move<0x140>(v);
    return __builtin_amdgcn_readlane(v, 0) + __builtin_amdgcn_readlane(v, 16) + __builtin_amdgcn_readlane(v, 32) +
           __builtin_amdgcn_readlane(v, 48);
}
// Sec. 2.2.1 activation quantiser: round half to even, clip to [-127, 127].
__device__ inline int quant1(float x, float inv)
{
    float q = rintf(x * inv);
    q = fminf(fmaxf(q, -127.0f), 127.0f);
    return (int)q;
}

inline int round_up(int v, int m) { return (v + m - 1) / m * m; }
inline size_t align256(size_t v) { return (v + 255) & ~size_t(255); }

// ---- workspace layout -------------------------------------------------------------
// [ flags | exchange buffers of the single-launch path | x_q | s_x | rowsum | h16 | h partials |
//   weight-quantiser sums ]   (hgf_workspace_init zeroes the flags and fills the exchange
//   buffers with the sentinel pattern)
constexpr int kNumFlags = 64;                              // int32 words: launch counter, arrival count, sticky error
constexpr size_t kZeroBytes = size_t(kNumFlags) * 4;
constexpr int kWsumBlocks = 1024;                          // fp64 partial sums of |W|
constexpr int kMaxHSplit = 32;                             // k-splits of the rank-r down-projection

struct Workspace {
    int32_t *flags;      // zero region: [0] correction workgroups done, [1] decode workgroups done,
                         // [2] sticky: a bounded wait ran out
    unsigned char *mail; // two exchange buffers of kMailBytes, sentinel-filled between launches
    unsigned char *xchg; // two sets of kStackSetBytes for the whole-stack launch, likewise
    int8_t *xq;
    float *s_x;
    int32_t *rowsum;
    _Float16 *h16;       // large M: kMaxGroup x [M, h_stride] SiLU(A x), zero padded (one per layer of a group)
    size_t h16_each;     // bytes per layer
    float *hslices;      // decode: kMaxGroup x [S, M, h_stride] fp32 partial sums of A x
    size_t hslices_each; // bytes per layer of a group
    double *wsum;        // [kWsumBlocks]
    size_t bytes;        // total bytes needed
};

// Carves `base` for a call of the given sizes (base may be null: sizes only).  `groups`: layers
// that may share one launch (kMaxGroup for layer lists, 1 for a single layer); `with_stack`:
// include the exchange regions of the whole-stack launch (else `xchg` is null).
Workspace carve_workspace(void *base, int M, int d_in, int d_out, int rank, int groups = kMaxGroup,
                          bool with_stack = true);

__host__ __device__ inline int h_rank_tiles(int rank)   // rank tiles of 16, rounded to a power of two (1, 2, 4, 8)
{
    int t = (rank + 15) / 16, p = 1;
    while (p < t) p *= 2;
    return p;
}
__host__ __device__ inline int h_stride(int rank)       // row stride of h16 in elements (multiple of 32)
{
    int s = 16 * h_rank_tiles(rank);
    return s < 32 ? 32 : s;
}

// ---- grouped launches: up to kMaxGroup layers that read the same activations ----------

struct ProLayer {
    const _Float16 *A;   // [rank, K]
    float *hpart;        // [S, M, rp] fp32 partial sums of A x
    int rank, rp;
};
struct ProParams {
    const _Float16 *x;
    unsigned char *mail; // two exchange buffers of kMailBytes, sentinel-filled between launches
    unsigned char *xchg; // two sets of kStackSetBytes for the whole-stack launch, likewise
    int8_t *xq;
    float *s_x;
    int32_t *rowsum;
    float *amax_zero;    // nullable: [M] floats the quantising workgroups set to zero (a later kernel's atomic max)
    int quantize;        // 0: x_q, s_x and the row sums are already there (the LayerNorm quantiser wrote them)
    int M, K, Kp, G;
    ProLayer L[kMaxGroup];
    int job_start[kMaxGroup + 1];
    int S, pairs, pairs_per_slice;   // slices of d_in; 64-column steps in all and per slice
};

struct DecLayer {
    const v4u *packed;
    const float *s_w;
    const _Float16 *B;
    const _Float16 *alpha;
    const _Float16 *h16;     // [M, hstride] fp16 SiLU(A x), zero padded (the base-3 path; the prefill path has its own)
    const float *hpart;      // [S][M][hstride] fp32 slices of A x from the prologue (the decode kernel adds them itself)
    _Float16 *y;
    int32_t *acc_debug;
    int N, RBn, rank, hstride;
};
struct DecodeParams {
    const int8_t *xq;
    const float *s_x;
    const int32_t *rowsum;
    int M, Kp, KT, G;
    int S;                   // slices of A x the prologue wrote
    DecLayer L[kMaxGroup];
    int wg_start[kMaxGroup + 1];
    int RW, KW;              // row-blocks per workgroup, wavefronts per row-block (RW*KW = 4 or 8)
    int CT, xstride;         // tiles of d_in staged in LDS at a time; bytes per staged row
    int h_off, g_off;        // byte offsets in LDS of the SiLU(A x) rows and of the tanh(alpha) table
    // SwiGLU pair (G == 2, both layers of one shape): a workgroup takes the SAME row-block of
    // layer 0 (gate) and layer 1 (up), one half of its wavefronts each, and stores
    // z = SiLU(y_gate) * y_up to L[1].y; L[0].y is unused.
    int pair;
    int h_each, exch_off;    // pair: bytes per layer of the SiLU(A x) rows in LDS; offset of the y_gate exchange
    float *amax_out;         // pair, nullable: per-token max |z| (zeroed before the launch; combined with atomic max)
};

// Single persistent launch for a handful of tokens: every workgroup quantises the tokens
// itself, streams its share of the row-blocks ("units") and exchanges the partial sums of
// A x with the others through a sentinel-filled buffer in the workspace.
constexpr int kMaxFusedM = 4;
constexpr int kMaxFusedK = 12288;
constexpr int kFusedSplit = 24;                               // slices of d_in at most (512 columns each)
constexpr size_t kMailLayerBytes = size_t(64) * HGF_MAX_RANK * 4;   // 64 (slice, token) rows of fp32 per layer
constexpr size_t kMailBytes = kMailLayerBytes * kMaxGroup;    // one exchange buffer; the workspace holds two
struct FusedParams {
    const _Float16 *x;            // [M, K] fp16
    int M, K, Kp, KT, TPW, G;     // TPW: tiles of a unit per streaming wavefront
    DecLayer L[kMaxGroup];        // h16 unused
    const _Float16 *A[kMaxGroup];
    int ustart[kMaxGroup + 1];    // running sum of the layers' row-blocks
    int job_start[kMaxGroup + 1]; // running sum of the layers' (rank tile, slice) jobs
    int nwg;                      // workgroups of the launch
    int S, pairs, pairs_per_slice;
    int xstride, tile_off, h_off; // LDS: bytes per quantised token row; offsets of the units' int32 sums and of SiLU(A x)
    int unit_off, unit_stride, unit_alpha;   // LDS: staged epilogue operands (B rows, alpha) per unit
    unsigned char *mail;          // two exchange buffers of kMailBytes
    int32_t *flags;               // [0] launch counter, [1] workgroups done, [2] sticky: a wait ran out
};

// One persistent launch over a list of phases (groups of layers) for a handful of tokens.
// Sized so that the whole description fits the 4 KiB of kernel arguments.
constexpr int kStackMaxLayers = 48;
constexpr int kStackMaxPhases = 36;
constexpr size_t kStackActBytes = size_t(6) << 20;     // per set: exchange copies of the layers' outputs ...
constexpr size_t kStackSetBytes = size_t(8) << 20;     // ... followed by the partial sums of A x
struct StackLayer {                                    // 64 bytes
    const v4u *packed;
    const float *s_w;
    const _Float16 *A, *B, *alpha;
    _Float16 *y;
    int N, rank;
    unsigned act_off;             // byte offset of the output's exchange copy ([M][N] fp16, N % 8 == 0)
    int reserved;
};
struct StackPhase {                                    // 24 bytes
    const _Float16 *x_ext;        // the tokens, when they were written before the launch; else null
    int K;
    short first_layer, G;
    unsigned src_off;             // else: byte offset of their exchange copy
    unsigned mail_off;            // byte offset of the phase's partial sums of A x
};
// Time stamps of the whole-stack launch (a measurement aid, off unless a buffer is set): each
// role's first lane notes the device-wide 100 MHz clock at fixed points of kTracePhases
// consecutive phases; the words leave through LDS at the end of the launch.
constexpr int kTraceRoles = 11;       // contracting wavefronts 0..7, slice wavefront, unit wavefront, loader 0
constexpr int kTracePhases = 4;
constexpr int kTraceIds = 8;
struct StackParams {
    int M, nphases, nwg, trace_ph0;   // trace_ph0: first traced phase
    unsigned long long *trace;        // null, or [nwg][kTraceRoles][kTracePhases][kTraceIds] time stamps
    int32_t *flags;               // [2] sticky error, [4] launch counter, [5] workgroups done, [6], [7] extents used
    unsigned char *xchg;          // two sets of kStackSetBytes
    unsigned act_used, mail_used;
    int xstride, h_par, tile_off, tile_par, h_off, unit_off, unit_stride, unit_alpha, jx_off, ring_off, ring_slots;   // LDS layout
    int mem_polls, lds_polls;     // tries after which a wait for another workgroup / another wavefront gives up
    StackPhase ph[kStackMaxPhases];
    StackLayer L[kStackMaxLayers];
};
static_assert(sizeof(StackParams) <= 4096, "kernel arguments");

// ---- kernel launchers (each validates nothing: the ABI layer has done it) -----------
hipError_t launch_wsum(const float *W, size_t n, double *partials, float *s_w_out, hipStream_t st);
hipError_t launch_pack(const float *W, int N, int K, const float *s_w, uint32_t *packed, hipStream_t st);
hipError_t launch_unpack(const uint32_t *packed, int N, int K, int8_t *T, hipStream_t st);
hipError_t launch_fill(void *p, size_t bytes, uint32_t word, hipStream_t st);   // whole 16-byte units, 16-byte aligned
hipError_t launch_zero_words(void *p, size_t n, hipStream_t st);
hipError_t launch_quantize(const _Float16 *x, int M, int K, int8_t *xq, float *s_x, int32_t *rowsum,
                           hipStream_t st);
hipError_t launch_ln_quantize(const _Float16 *x, int M, int K, const float *gamma, const float *beta, float eps,
                              int8_t *xq, float *s_x, int32_t *rowsum, hipStream_t st);
hipError_t launch_corr_down(const _Float16 *x, int M, int K, int G, const _Float16 *const *A, const int *rank,
                            _Float16 *const *h16, int8_t *xq, float *s_x, int32_t *rowsum, hipStream_t st);
int prologue_slices(int M, int K);
hipError_t launch_prologue(ProParams &p, _Float16 *const *h16, hipStream_t st);
hipError_t launch_decode(DecodeParams &p, int d_in, hipStream_t st);
// What a plan or a launch of one of the persistent kernels came to.
enum class Launch { kRan, kNoFit, kRefused };
bool plan_fused(FusedParams &p, size_t *lds_bytes);
hipError_t launch_fused(const FusedParams &p, size_t lds_bytes, hipStream_t st);
bool plan_stack(StackParams &p, size_t *lds_bytes);
void set_stack_wait_limit(int tries);
void set_stack_trace(unsigned long long *buf, size_t bytes, int first_phase);
hipError_t launch_stack(const StackParams &p, size_t lds_bytes, hipStream_t st);
struct PairOut {                 // extra outputs of a SwiGLU pair launch (both nullable)
    int32_t *acc_debug2;         // the up projection's int32 accumulators
    float *amax_out;             // per-token max |z|
};
hipError_t launch_prefill(const Workspace &ws, _Float16 *const *h16, int M, const hgf_layer *layers, int G,
                          void *const *ys, int32_t *acc_debug, hipStream_t st, const PairOut *pair_out = nullptr);

// differential attention, one decode step
size_t diff_attn_workspace_bytes(int B, int L_max, int n_heads, int d_h);
hipError_t launch_diff_attn(const void *q, const void *k, const void *v, const int32_t *lens, int B, int L_max,
                            int n_heads, int d_h, float lambda, void *out, void *workspace, hipStream_t st);

// base-3 packing (five ternary weights per byte) and its few-token decode kernel
size_t b3_packed_bytes(int d_out, int d_in);
hipError_t launch_pack_b3(const float *W, int N, int K, const float *s_w, unsigned char *packed, hipStream_t st);
hipError_t launch_unpack_b3(const unsigned char *packed, int N, int K, int8_t *T, hipStream_t st);
bool b3_fits(int M, int K, int rank);
hipError_t launch_b3_decode(const void *packed, const Workspace &ws, const _Float16 *h16, int M, const hgf_layer &L,
                            void *y, int32_t *acc_debug, hipStream_t st);

}  // namespace hgf
