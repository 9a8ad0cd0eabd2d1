// Measurement aid: the rate the matrix cores sustain on a loop of nothing but the prefill
// kernel's MFMA (v_mfma_i32_32x32x32_i8, eight independent accumulators per wavefront, operands
// in registers, no memory traffic), for three kinds of operand values.  The chip lowers its clock
// under the switching power of the matrix cores, so the sustained rate depends on the data; the
// figure for "codes 0..2 against random int8" is what a perfect prefill kernel could reach on
// this layer's operands, and is the yardstick the design notes quote beside the published peak.
#include "hgf_internal.h"

#include <vector>

namespace hgf {
namespace {

__global__ __launch_bounds__(256, 2) void mfma_probe_kernel(const v4i *ops, unsigned long long *out, int iters)
{
    v4i a[4], b[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        a[i] = ops[i * 256 + threadIdx.x];
        b[i] = ops[(4 + i) * 256 + threadIdx.x];
    }
    const unsigned long long w0 = wall_clock64(), c0 = clock64();
    v16i acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = (v16i){};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int j = 0; j < 8; ++j)
                acc[j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[(u + j) & 3], b[j & 3], acc[j], 0, 0, 0);
    }
    const unsigned long long w1 = wall_clock64(), c1 = clock64();
    int s = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) s += acc[j][0];
    if (threadIdx.x == 0) {
        out[blockIdx.x * 2] = w1 - w0;          // 100 MHz ticks
        out[blockIdx.x * 2 + 1] = c1 - c0;      // shader clock cycles
    }
    if (s == 0x7fffffff) out[0] = 0;            // keeps the accumulators alive
}

}  // namespace
}  // namespace hgf

using namespace hgf;

extern "C" hgf_status hgf_probe_mfma_rate(int operand_kind, int iters, double *tops_out, double *ghz_out, void *stream)
{
    if (!tops_out || !ghz_out) return HGF_ERR_NULL;
    if (operand_kind < 0 || operand_kind > 2 || iters < 1 || iters > (1 << 20)) return HGF_ERR_SHAPE;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
        return HGF_ERR_DEVICE;
    const int wgs = 2 * cus;                    // two workgroups of four wavefronts per compute unit
    // operands: a[] (the weight side) then b[] (the activation side), 4 x 256 lanes x 16 bytes each
    std::vector<uint32_t> host(8 * 256 * 4);
    uint64_t state = 0x9E3779B97F4A7C15ull;     // splitmix64
    auto next = [&]() {
        uint64_t z = (state += 0x9E3779B97F4A7C15ull);
        z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
        z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
        return (uint32_t)((z ^ (z >> 31)) >> 16);
    };
    for (size_t i = 0; i < host.size(); ++i) {
        const bool weight_side = i < host.size() / 2;
        uint32_t v = 0;
        for (int byte = 0; byte < 4; ++byte) {
            uint32_t c;
            if (operand_kind == 0) c = 1;                                   // constant
            else if (operand_kind == 1 && weight_side) c = next() % 3;      // codes 0..2
            else c = next() & 0xff;                                         // random int8
            v |= c << (8 * byte);
        }
        host[i] = v;
    }
    v4i *ops = nullptr;
    unsigned long long *out = nullptr;
    if (hipMalloc(&ops, host.size() * 4) != hipSuccess) return HGF_ERR_DEVICE;
    if (hipMalloc(&out, (size_t)wgs * 16) != hipSuccess) {
        (void)hipFree(ops);
        return HGF_ERR_DEVICE;
    }
    hipEvent_t e0 = nullptr, e1 = nullptr;
    hgf_status rc = HGF_ERR_DEVICE;
    const int reps = 10;
    float ms = 0.f;
    unsigned long long first[2] = {0, 0};
    if (hipMemcpyAsync(ops, host.data(), host.size() * 4, hipMemcpyHostToDevice, st) != hipSuccess) goto done;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) goto done;
    for (int r = 0; r < reps; ++r) hipLaunchKernelGGL(mfma_probe_kernel, dim3(wgs), dim3(256), 0, st, ops, out, iters);   // warm-up: lets the clock settle
    if (hipEventRecord(e0, st) != hipSuccess) goto done;
    for (int r = 0; r < reps; ++r) hipLaunchKernelGGL(mfma_probe_kernel, dim3(wgs), dim3(256), 0, st, ops, out, iters);
    if (hipEventRecord(e1, st) != hipSuccess || hipEventSynchronize(e1) != hipSuccess) goto done;
    if (hipGetLastError() != hipSuccess || hipEventElapsedTime(&ms, e0, e1) != hipSuccess) goto done;
    if (hipMemcpy(first, out, sizeof(first), hipMemcpyDeviceToHost) != hipSuccess) goto done;
    *tops_out = (double)wgs * 4 * iters * 32 * 65536.0 * reps / (ms * 1e-3) / 1e12;
    *ghz_out = first[0] ? (double)first[1] / ((double)first[0] * 10.0) : 0.0;     // cycles per nanosecond
    rc = HGF_OK;
done:
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    (void)hipFree(ops);
    (void)hipFree(out);
    return rc;
}
