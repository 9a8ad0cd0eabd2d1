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
constexpr int kMaxDecodeM = 64;      // decode kernel handles up to 4 token tiles of 16
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

inline int round_up(int v, int m) { return (v + m - 1) / m * m; }
inline size_t align256(size_t v) { return (v + 255) & ~size_t(255); }

// ---- workspace layout -------------------------------------------------------------
// [ zero region: split-K int32 accumulators | arrival counters ]  (zero between calls)
// [ x_q | s_x | rowsum | h16 | h partials | weight-quantiser partial sums ]
constexpr size_t kAccZeroBytes = size_t(64) * 32768 * 4;   // 8 MiB of int32 accumulators
constexpr int kNumCounters = 16384;                        // int32 arrival counters
constexpr size_t kZeroBytes = kAccZeroBytes + size_t(kNumCounters) * 4;
constexpr int kWsumBlocks = 1024;                          // fp64 partial sums of |W|
constexpr int kMaxHSplit = 32;                             // k-splits of the rank-r down-projection

struct Workspace {
    int32_t *acc;        // zero region
    int32_t *counters;   // zero region: [0, 8192) decode row-blocks, [8192, 16384) h tiles
    int8_t *xq;
    float *s_x;
    int32_t *rowsum;
    _Float16 *h16;       // large M: [M, h_stride] SiLU(A x), zero padded
    float *hslices;      // decode: kMaxGroup x [S, M, h_stride] fp32 partial sums of A x
    size_t hslices_each; // bytes per layer of a group
    double *wsum;        // [kWsumBlocks]
    size_t bytes;        // total bytes needed
};

// Carves `base` for a call of the given sizes (base may be null: sizes only).
Workspace carve_workspace(void *base, int M, int d_in, int d_out, int rank);

inline int h_rank_tiles(int rank)   // rank tiles of 16, rounded to a power of two (1, 2, 4, 8)
{
    int t = (rank + 15) / 16, p = 1;
    while (p < t) p *= 2;
    return p;
}
inline int h_stride(int rank)       // row stride of h16 in elements (multiple of 32)
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
    int8_t *xq;
    float *s_x;
    int32_t *rowsum;
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
    const float *hpart;      // [S, M, hstride] fp32 partial sums of A x from the prologue
    _Float16 *y;
    int32_t *acc_debug;
    int N, RBn, rank, hstride;
};
struct DecodeParams {
    const int8_t *xq;
    const float *s_x;
    const int32_t *rowsum;
    int M, Kp, KT, G;
    DecLayer L[kMaxGroup];
    int wg_start[kMaxGroup + 1];
    int RW, KW;              // row-blocks per workgroup, wavefronts per row-block (RW*KW = 4 or 8)
    int CT, xstride;         // tiles of d_in staged in LDS at a time; bytes per staged row
    int S;                   // slices of the correction partial sums
    int h_off, g_off;        // byte offsets in LDS of the SiLU(A x) rows and of the tanh(alpha) table
};

// ---- kernel launchers (each validates nothing: the ABI layer has done it) -----------
hipError_t launch_wsum(const float *W, size_t n, double *partials, float *s_w_out, hipStream_t st);
hipError_t launch_pack(const float *W, int N, int K, const float *s_w, uint32_t *packed, hipStream_t st);
hipError_t launch_unpack(const uint32_t *packed, int N, int K, int8_t *T, hipStream_t st);
hipError_t launch_fill_zero(void *p, size_t bytes, hipStream_t st);
hipError_t launch_quantize(const _Float16 *x, int M, int K, int8_t *xq, float *s_x, int32_t *rowsum,
                           hipStream_t st);
hipError_t launch_corr_down(const _Float16 *x, int M, int K, const _Float16 *A, int rank,
                            const Workspace &ws, hipStream_t st);
int prologue_slices(int M, int K);
hipError_t launch_prologue(ProParams &p, hipStream_t st);
hipError_t launch_decode(DecodeParams &p, int d_in, hipStream_t st);
void set_decode_target_wgs(int v);
hipError_t launch_prefill(const Workspace &ws, int M, const hgf_layer &L, _Float16 *y, int32_t *acc_debug,
                          hipStream_t st);

}  // namespace hgf
