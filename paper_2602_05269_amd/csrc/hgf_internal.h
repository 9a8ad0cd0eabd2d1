// Internal declarations shared by the HIP sources of libhgf (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>
#include <stddef.h>

#include "../../include/hgf.h"

namespace hgf {

constexpr int kTile = 64;            // packing granule in both dimensions
constexpr int kTileBytes = 1024;     // one 64x64 tile of 2-bit codes
constexpr int kMaxDecodeM = 64;      // decode kernel handles up to 4 token tiles of 16

typedef int v4i __attribute__((ext_vector_type(4)));
typedef unsigned int v4u __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef _Float16 v4h __attribute__((ext_vector_type(4)));

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
    _Float16 *h16;       // [M, h_stride] SiLU(A x), zero padded
    float *hpart;        // [splits, M16, rp]
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

// ---- kernel launchers (each validates nothing: the ABI layer has done it) -----------
hipError_t launch_wsum(const float *W, size_t n, double *partials, float *s_w_out, hipStream_t st);
hipError_t launch_pack(const float *W, int N, int K, const float *s_w, uint32_t *packed, hipStream_t st);
hipError_t launch_unpack(const uint32_t *packed, int N, int K, int8_t *T, hipStream_t st);
hipError_t launch_fill_zero(void *p, size_t bytes, hipStream_t st);
hipError_t launch_quantize(const _Float16 *x, int M, int K, int8_t *xq, float *s_x, int32_t *rowsum,
                           hipStream_t st);
int corr_splits(int M, int K);
size_t corr_scratch_bytes(int M, int K, int rank);
hipError_t launch_corr_down(const _Float16 *x, int M, int K, const _Float16 *A, int rank,
                            const Workspace &ws, hipStream_t st);
hipError_t launch_decode(const Workspace &ws, int M, const hgf_layer &L, _Float16 *y, int32_t *acc_debug,
                         hipStream_t st);
void set_decode_target_wgs(int v);
hipError_t launch_prefill(const Workspace &ws, int M, const hgf_layer &L, _Float16 *y, int32_t *acc_debug,
                          hipStream_t st);

}  // namespace hgf
