// C ABI of libhgf: host-side argument validation, workspace carving and dispatch.
// Every check happens before the first HIP call, so the error paths run without a GPU.
#include "hgf_internal.h"

#include <utility>
#include <vector>

namespace hgf {

Workspace carve_workspace(void *base, int M, int d_in, int d_out, int rank, int groups, bool with_stack)
{
    Workspace ws;
    char *p = reinterpret_cast<char *>(base);
    size_t off = 0;
    auto take = [&](size_t bytes) {
        char *r = p ? p + off : nullptr;
        off += align256(bytes);
        return r;
    };
    ws.flags = reinterpret_cast<int32_t *>(take(kZeroBytes));
    ws.mail = reinterpret_cast<unsigned char *>(take(2 * kMailBytes));
    ws.xchg = with_stack ? reinterpret_cast<unsigned char *>(take(2 * kStackSetBytes)) : nullptr;
    const int Kp = round_up(d_in, kTileCols);
    ws.xq = reinterpret_cast<int8_t *>(take((size_t)M * Kp));
    ws.s_x = reinterpret_cast<float *>(take((size_t)M * 4));
    ws.rowsum = reinterpret_cast<int32_t *>(take((size_t)M * 4));
    ws.h16_each = align256((size_t)M * h_stride(rank > 0 ? rank : 1) * 2);
    ws.h16 = reinterpret_cast<_Float16 *>(take(ws.h16_each * groups));
    // two-launch decode path: per layer of a group kMaxHSplit slices of [M, h_stride] partial sums
    const int Md = M < kMaxDecodeM ? M : kMaxDecodeM;
    ws.hslices_each = rank > 0 ? align256((size_t)kMaxHSplit * Md * h_stride(rank) * sizeof(float)) : 0;
    ws.hslices = reinterpret_cast<float *>(take(ws.hslices_each * groups));
    ws.wsum = reinterpret_cast<double *>(take(size_t(kWsumBlocks) * 8));
    (void)d_out;
    ws.bytes = off;
    return ws;
}

namespace {

bool dims_ok(int d_in, int d_out) { return d_in >= 1 && d_out >= 1 && d_in <= HGF_MAX_DIM && d_out <= HGF_MAX_DIM; }
bool tokens_ok(int M, int d_in, int d_out)
{
    if (M < 1) return false;
    const long long big = (long long)M * (d_in > d_out ? d_in : d_out);
    return big < (1LL << 31);
}
bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

hgf_status check_layer(const hgf_layer *L, int M)
{
    if (!L) return HGF_ERR_NULL;
    if (!dims_ok(L->d_in, L->d_out) || L->rank < 0 || L->rank > HGF_MAX_RANK) return HGF_ERR_SHAPE;
    if (!tokens_ok(M, L->d_in, L->d_out)) return HGF_ERR_SHAPE;
    if (!L->W_packed || !L->s_w) return HGF_ERR_NULL;
    if (L->rank > 0 && (!L->A_f16 || !L->B_f16 || !L->alpha_f16)) return HGF_ERR_NULL;
    if (!aligned16(L->W_packed)) return HGF_ERR_ALIGN;
    if (L->ln_gamma && !(L->ln_eps >= 0.0f)) return HGF_ERR_SHAPE;
    return HGF_OK;
}

hgf_status from_hip(hipError_t e) { return e == hipSuccess ? HGF_OK : HGF_ERR_DEVICE; }

// Which of the two paths a group of layers takes.  Up to 40 tokens the two-launch decode path
// always; from 41 to 64 (what its kernel handles) only groups of few rows, whose prefill grids
// would be a handful of 256-row tiles (7B-shape FFN at 64 tokens: the down projection, 4096 rows,
// takes 52 us on the decode path and 60 on the prefill path; up + gate, 22016 rows, 41 and 33).
bool takes_decode_path(int M, const hgf_layer *layers, int G, bool pair)
{
    if (M <= 40) return true;
    if (M > kMaxDecodeM || pair) return false;
    long long rows = 0;
    for (int g = 0; g < G; ++g) rows += layers[g].d_out;
    return rows <= 8192;
}

// Profiling aid: event pairs recorded around main-kernel launches, by kind (0 decode, 1 prefill).
bool g_profile = false;
int g_launch_level = 2;      // 0: two launches per group, 1: one persistent launch per group, 2: per stack
std::vector<std::pair<hipEvent_t, hipEvent_t>> g_events[2];
std::vector<hipEvent_t> g_event_pool;

hipEvent_t take_event()
{
    hipEvent_t e = nullptr;
    if (!g_event_pool.empty()) {
        e = g_event_pool.back();
        g_event_pool.pop_back();
    } else if (hipEventCreate(&e) != hipSuccess) {
        e = nullptr;
    }
    return e;
}

// Records an event pair around a main-kernel launch when profiling is on.
struct ProfileScope {
    hipEvent_t e0 = nullptr, e1 = nullptr;
    hipStream_t st;
    int kind;
    ProfileScope(int kind_, hipStream_t st_) : st(st_), kind(kind_)
    {
        if (!g_profile) return;
        e0 = take_event();
        e1 = take_event();
        if (e0 && e1) (void)hipEventRecord(e0, st);
    }
    ~ProfileScope()
    {
        if (e0 && e1) {
            (void)hipEventRecord(e1, st);
            g_events[kind].emplace_back(e0, e1);
        }
    }
};

// Decode (M <= kMaxDecodeM): `G` layers that read the same activations `x` run as two launches:
// the fused prologue (quantiser + partial sums of every A x) and one grouped main kernel.
//
// `pair` (G == 2): the SwiGLU pair -- layers[0] is the gate projection, layers[1] the up
// projection; the one output ys[1] receives SiLU(y_gate) * y_up, amax_out (nullable) the
// per-token max of its magnitude, acc_debug2 (nullable) the up projection's accumulators.
hgf_status run_decode_group(const void *x, int M, const hgf_layer *layers, int G, void *const *ys,
                            int32_t *acc_debug, const Workspace &ws, hipStream_t st, bool pair = false,
                            float *amax_out = nullptr, int32_t *acc_debug2 = nullptr)
{
    const int K = layers[0].d_in;
    const bool ln = layers[0].ln_gamma != nullptr;   // (such a layer is always a group of its own)
    bool fused = !pair && !ln && g_launch_level >= 1 && M <= kMaxFusedM && K % 8 == 0 && K <= kMaxFusedK && aligned16(x);
    for (int g = 0; g < G; ++g)
        fused = fused && (layers[g].rank == 0 ||
                          (layers[g].rank % 8 == 0 && aligned16(layers[g].A_f16) && aligned16(layers[g].B_f16) &&
                           (reinterpret_cast<uintptr_t>(layers[g].alpha_f16) & 3u) == 0));
    if (fused) {
        FusedParams fp;
        fp.x = reinterpret_cast<const _Float16 *>(x);
        fp.M = M;
        fp.K = K;
        fp.G = G;
        fp.flags = ws.flags;
        fp.mail = ws.mail;
        for (int g = 0; g < G; ++g) {
            const hgf_layer &L = layers[g];
            DecLayer &D = fp.L[g];
            D.packed = reinterpret_cast<const v4u *>(L.W_packed);
            D.s_w = L.s_w;
            D.B = reinterpret_cast<const _Float16 *>(L.B_f16);
            D.alpha = reinterpret_cast<const _Float16 *>(L.alpha_f16);
            D.h16 = nullptr;
            D.hpart = nullptr;
            D.y = reinterpret_cast<_Float16 *>(ys[g]);
            D.acc_debug = acc_debug;
            D.N = L.d_out;
            D.RBn = round_up(L.d_out, kTileRows) / kTileRows;
            D.rank = L.rank;
            D.hstride = h_stride(L.rank > 0 ? L.rank : 1);
            fp.A[g] = reinterpret_cast<const _Float16 *>(L.A_f16);
        }
        size_t lds_bytes = 0;
        if (plan_fused(fp, &lds_bytes)) {
            ProfileScope prof(0, st);
            return from_hip(launch_fused(fp, lds_bytes, st));
        }
    }
    ProParams pp;
    pp.x = reinterpret_cast<const _Float16 *>(x);
    pp.xq = ws.xq;
    pp.s_x = ws.s_x;
    pp.rowsum = ws.rowsum;
    pp.amax_zero = pair ? amax_out : nullptr;
    pp.quantize = ln ? 0 : 1;
    pp.M = M;
    pp.K = K;
    pp.Kp = round_up(K, kTileCols);
    pp.G = G;
    DecodeParams dp;
    dp.xq = ws.xq;
    dp.s_x = ws.s_x;
    dp.rowsum = ws.rowsum;
    dp.M = M;
    dp.G = G;
    dp.pair = pair ? 1 : 0;
    dp.amax_out = pair ? amax_out : nullptr;
    for (int g = 0; g < G; ++g) {
        const hgf_layer &L = layers[g];
        float *slices = reinterpret_cast<float *>(reinterpret_cast<char *>(ws.hslices) + ws.hslices_each * g);
        pp.L[g].A = reinterpret_cast<const _Float16 *>(L.A_f16);
        pp.L[g].hpart = slices;
        pp.L[g].rank = L.rank;
        pp.L[g].rp = h_stride(L.rank > 0 ? L.rank : 1);
        DecLayer &D = dp.L[g];
        D.packed = reinterpret_cast<const v4u *>(L.W_packed);
        D.s_w = L.s_w;
        D.B = reinterpret_cast<const _Float16 *>(L.B_f16);
        D.alpha = reinterpret_cast<const _Float16 *>(L.alpha_f16);
        D.h16 = nullptr;
        D.hpart = slices;                           // (the main kernel adds the slices of A x itself: no reducing launch)
        D.y = reinterpret_cast<_Float16 *>(ys[g]);
        D.acc_debug = (pair && g == 1) ? acc_debug2 : acc_debug;
        D.N = L.d_out;
        D.RBn = round_up(L.d_out, kTileRows) / kTileRows;
        D.rank = L.rank;
        D.hstride = h_stride(L.rank > 0 ? L.rank : 1);
    }
    dp.S = prologue_slices(M, K);
    if (ln && launch_ln_quantize(pp.x, M, K, layers[0].ln_gamma, layers[0].ln_beta, layers[0].ln_eps, ws.xq, ws.s_x,
                                 ws.rowsum, st) != hipSuccess)
        return HGF_ERR_DEVICE;
    if (launch_prologue(pp, nullptr, st) != hipSuccess) return HGF_ERR_DEVICE;
    ProfileScope prof(0, st);
    return from_hip(launch_decode(dp, K, st));
}

// Large M: per group of layers that read the same activations, one launch for the quantiser
// and the down-projections with SiLU of all layers (both read x), then one launch of the int8
// MFMA prefill kernel over the tiles of all layers.
hgf_status run_large_group(const void *x, int M, const hgf_layer *layers, int G, void *const *ys,
                           int32_t *acc_debug, const Workspace &ws, hipStream_t st, const PairOut *pair_out = nullptr)
{
    const _Float16 *xh = reinterpret_cast<const _Float16 *>(x);
    const int K = layers[0].d_in;
    const _Float16 *A[kMaxGroup];
    _Float16 *h16[kMaxGroup];
    int rank[kMaxGroup];
    for (int g = 0; g < G; ++g) {
        A[g] = reinterpret_cast<const _Float16 *>(layers[g].A_f16);
        rank[g] = layers[g].rank;
        h16[g] = reinterpret_cast<_Float16 *>(reinterpret_cast<char *>(ws.h16) + ws.h16_each * g);
    }
    if (pair_out && pair_out->amax_out &&
        launch_zero_words(pair_out->amax_out, (size_t)M, st) != hipSuccess)
        return HGF_ERR_DEVICE;
    const bool ln = layers[0].ln_gamma != nullptr;   // (such a layer is always a group of its own)
    if (ln && launch_ln_quantize(xh, M, K, layers[0].ln_gamma, layers[0].ln_beta, layers[0].ln_eps, ws.xq, ws.s_x,
                                 ws.rowsum, st) != hipSuccess)
        return HGF_ERR_DEVICE;
    if (launch_corr_down(xh, M, K, G, A, rank, h16, ln ? nullptr : ws.xq, ws.s_x, ws.rowsum, st) != hipSuccess)
        return HGF_ERR_DEVICE;
    ProfileScope prof(1, st);
    return from_hip(launch_prefill(ws, h16, M, layers, G, ys, acc_debug, st, pair_out));
}

// ---- the scratch of hgf_linear_forward_static: what the workspace argument brings to
//      hgf_linear_forward (launch counter, exchange buffers, x_q, scales, SiLU(A x), partial
//      sums), for callers that can bring none.  Every GPU the library runs on holds its own
//      copy of this array at its own address until the process ends; host code reaches it only
//      through the address hipGetSymbolAddress returns with that GPU current.
constexpr size_t kStaticScratchBytes = size_t(8) << 20;
constexpr int kMaxDevices = 64;
}  // namespace
}  // namespace hgf

static __device__ __align__(256) unsigned char scratch[hgf::kStaticScratchBytes];

namespace hgf {
namespace {

unsigned char *g_scratch_ptr[kMaxDevices];      // per device: the array's address there (null: not asked yet)

Workspace carve_static(void *base, int M, const hgf_layer *L)
{
    return carve_workspace(base, M, L->d_in, L->d_out, L->rank, /*groups=*/1, /*with_stack=*/false);
}

// The device address of `scratch` on the current device, set up on first use: the address is
// looked up and the control words and exchange buffers are put into the state
// hgf_workspace_init leaves them in (fill kernels on `st`, ahead of the caller's work).
hgf_status static_scratch(hipStream_t st, unsigned char **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        (void)hipGetLastError();
        return HGF_ERR_DEVICE;
    }
    if (!g_scratch_ptr[dev]) {
        unsigned char *ptr = nullptr;
        if (hipGetSymbolAddress(reinterpret_cast<void **>(&ptr), HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
            (void)hipGetLastError();
            return HGF_ERR_DEVICE;
        }
        const Workspace ws = carve_workspace(ptr, 1, 1, 1, 0, 1, false);
        if (launch_fill(ws.flags, align256(kZeroBytes), 0u, st) != hipSuccess ||
            launch_fill(ws.mail, 2 * kMailBytes, 0xFFFFFFFFu, st) != hipSuccess)
            return HGF_ERR_DEVICE;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return HGF_OK;
}

}  // namespace
}  // namespace hgf

using namespace hgf;

extern "C" {

const char *hgf_status_string(int status)
{
    switch (status) {
        case HGF_OK: return "HGF_OK";
        case HGF_ERR_NULL: return "HGF_ERR_NULL: a required pointer is NULL";
        case HGF_ERR_SHAPE: return "HGF_ERR_SHAPE: a dimension is out of range";
        case HGF_ERR_ALIGN: return "HGF_ERR_ALIGN: a buffer is not 16-byte aligned";
        case HGF_ERR_UNSUPPORTED: return "HGF_ERR_UNSUPPORTED";
        case HGF_ERR_WORKSPACE: return "HGF_ERR_WORKSPACE: workspace missing or too small";
        case HGF_ERR_DEVICE: return "HGF_ERR_DEVICE: the HIP runtime refused a launch";
        default: return "HGF: unknown status";
    }
}

int hgf_version(void) { return 100; }

int hgf_padded_k(int d_in) { return (d_in >= 1 && d_in <= HGF_MAX_DIM) ? round_up(d_in, kTileCols) : 0; }

size_t hgf_packed_weight_bytes(int d_out, int d_in)
{
    if (!dims_ok(d_in, d_out)) return 0;
    return (size_t)(round_up(d_out, kTileRows) / kTileRows) * (round_up(d_in, kTileCols) / kTileCols) * kTileBytes;
}

size_t hgf_workspace_bytes(int M_max, int d_in_max, int d_out_max, int rank_max)
{
    if (!dims_ok(d_in_max, d_out_max) || rank_max < 0 || rank_max > HGF_MAX_RANK) return 0;
    if (!tokens_ok(M_max, d_in_max, d_out_max)) return 0;
    return carve_workspace(nullptr, M_max, d_in_max, d_out_max, rank_max).bytes;
}

hgf_status hgf_workspace_init(void *workspace, size_t workspace_bytes, void *stream)
{
    if (!workspace) return HGF_ERR_NULL;
    if (!aligned16(workspace)) return HGF_ERR_ALIGN;
    const Workspace ws = carve_workspace(workspace, 1, 1, 1, 0);
    if (workspace_bytes < ws.bytes) return HGF_ERR_WORKSPACE;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    if (launch_fill(ws.flags, align256(kZeroBytes), 0u, st) != hipSuccess) return HGF_ERR_DEVICE;
    if (launch_fill(ws.mail, 2 * kMailBytes, 0xFFFFFFFFu, st) != hipSuccess) return HGF_ERR_DEVICE;
    return from_hip(launch_fill(ws.xchg, 2 * kStackSetBytes, 0xFFFFFFFFu, st));
}

hgf_status hgf_quantize_pack_weights(const float *W, int d_out, int d_in, void *packed_out, float *s_w_out,
                                     void *workspace, size_t workspace_bytes, void *stream)
{
    if (!W || !packed_out || !s_w_out) return HGF_ERR_NULL;
    if (!dims_ok(d_in, d_out)) return HGF_ERR_SHAPE;
    if (!aligned16(packed_out)) return HGF_ERR_ALIGN;
    if (!workspace) return HGF_ERR_WORKSPACE;
    const Workspace ws = carve_workspace(workspace, 1, 1, 1, 0);
    if (workspace_bytes < ws.bytes) return HGF_ERR_WORKSPACE;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    if (launch_wsum(W, (size_t)d_out * d_in, ws.wsum, s_w_out, st) != hipSuccess) return HGF_ERR_DEVICE;
    return from_hip(launch_pack(W, d_out, d_in, s_w_out, reinterpret_cast<uint32_t *>(packed_out), st));
}

hgf_status hgf_unpack_weights(const void *packed, int d_out, int d_in, int8_t *T_out, void *stream)
{
    if (!packed || !T_out) return HGF_ERR_NULL;
    if (!dims_ok(d_in, d_out)) return HGF_ERR_SHAPE;
    if (!aligned16(packed)) return HGF_ERR_ALIGN;
    return from_hip(launch_unpack(reinterpret_cast<const uint32_t *>(packed), d_out, d_in, T_out,
                                  reinterpret_cast<hipStream_t>(stream)));
}

hgf_status hgf_quantize_activations(const void *x_f16, int M, int d_in, int8_t *xq_out, float *s_x_out,
                                    int32_t *rowsum_out, void *stream)
{
    if (!x_f16 || !xq_out || !s_x_out) return HGF_ERR_NULL;
    if (!dims_ok(d_in, 1) || !tokens_ok(M, d_in, 1)) return HGF_ERR_SHAPE;
    if (!aligned16(x_f16) || !aligned16(xq_out)) return HGF_ERR_ALIGN;
    return from_hip(launch_quantize(reinterpret_cast<const _Float16 *>(x_f16), M, d_in, xq_out, s_x_out, rowsum_out,
                                    reinterpret_cast<hipStream_t>(stream)));
}

hgf_status hgf_layernorm_quantize_activations(const void *x_f16, int M, int d_in, const float *ln_gamma,
                                              const float *ln_beta, float ln_eps, int8_t *xq_out, float *s_x_out,
                                              int32_t *rowsum_out, void *stream)
{
    if (!x_f16 || !xq_out || !s_x_out || !ln_gamma) return HGF_ERR_NULL;
    if (!dims_ok(d_in, 1) || !tokens_ok(M, d_in, 1) || !(ln_eps >= 0.0f)) return HGF_ERR_SHAPE;
    if (!aligned16(x_f16) || !aligned16(xq_out)) return HGF_ERR_ALIGN;
    return from_hip(launch_ln_quantize(reinterpret_cast<const _Float16 *>(x_f16), M, d_in, ln_gamma, ln_beta, ln_eps,
                                       xq_out, s_x_out, rowsum_out, reinterpret_cast<hipStream_t>(stream)));
}

hgf_status hgf_linear_forward(const void *x_f16, int M, const hgf_layer *L, void *y_f16, int32_t *acc_debug,
                              void *workspace, size_t workspace_bytes, void *stream)
{
    if (!x_f16 || !y_f16) return HGF_ERR_NULL;
    const hgf_status s = check_layer(L, M);
    if (s != HGF_OK) return s;
    if (!aligned16(x_f16) || !aligned16(y_f16) || (acc_debug && !aligned16(acc_debug))) return HGF_ERR_ALIGN;
    if (!workspace) return HGF_ERR_WORKSPACE;
    if (!aligned16(workspace)) return HGF_ERR_ALIGN;
    const Workspace ws = carve_workspace(workspace, M, L->d_in, L->d_out, L->rank);
    if (workspace_bytes < ws.bytes) return HGF_ERR_WORKSPACE;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    if (takes_decode_path(M, L, 1, false)) {
        void *ys[1] = {y_f16};
        return run_decode_group(x_f16, M, L, 1, ys, acc_debug, ws, st);
    }
    void *ys1[1] = {y_f16};
    return run_large_group(x_f16, M, L, 1, ys1, acc_debug, ws, st);
}

hgf_status hgf_swiglu_forward(const void *x_f16, int M, const hgf_layer *gate, const hgf_layer *up, void *z_f16,
                              float *amax_out, int32_t *acc_debug_gate, int32_t *acc_debug_up, void *workspace,
                              size_t workspace_bytes, void *stream)
{
    if (!x_f16 || !z_f16) return HGF_ERR_NULL;
    hgf_status s = check_layer(gate, M);
    if (s == HGF_OK) s = check_layer(up, M);
    if (s != HGF_OK) return s;
    if (gate->d_in != up->d_in || gate->d_out != up->d_out) return HGF_ERR_SHAPE;
    if (gate->ln_gamma || up->ln_gamma) return HGF_ERR_UNSUPPORTED;   // (each would need a quantisation of its own)
    if (!aligned16(x_f16) || !aligned16(z_f16) || (acc_debug_gate && !aligned16(acc_debug_gate)) ||
        (acc_debug_up && !aligned16(acc_debug_up)) || (reinterpret_cast<uintptr_t>(amax_out) & 3u))
        return HGF_ERR_ALIGN;
    if (!workspace) return HGF_ERR_WORKSPACE;
    if (!aligned16(workspace)) return HGF_ERR_ALIGN;
    const int rank_max = gate->rank > up->rank ? gate->rank : up->rank;
    const Workspace ws = carve_workspace(workspace, M, gate->d_in, gate->d_out, rank_max);
    if (workspace_bytes < ws.bytes) return HGF_ERR_WORKSPACE;
    // the prefill kernel stages both layers' SiLU(A x) at one row width
    if (M > 40 && gate->rank > 0 && up->rank > 0 && h_stride(gate->rank) != h_stride(up->rank))
        return HGF_ERR_UNSUPPORTED;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    const hgf_layer pairL[2] = {*gate, *up};
    void *ys[2] = {nullptr, z_f16};
    if (takes_decode_path(M, pairL, 2, true))
        return run_decode_group(x_f16, M, pairL, 2, ys, acc_debug_gate, ws, st, true, amax_out, acc_debug_up);
    const PairOut po = {acc_debug_up, amax_out};
    return run_large_group(x_f16, M, pairL, 2, ys, acc_debug_gate, ws, st, &po);
}

namespace {
bool attn_dims_ok(int B, int L_max, int n_heads, int d_h)
{
    if (B < 1 || L_max < 1 || n_heads < 1 || d_h < 8 || d_h > 128 || (d_h & (d_h - 1)) != 0) return false;
    // the caches are addressed with 32-bit byte offsets per sequence
    return (long long)L_max * 2 * n_heads * d_h * 2 < (1LL << 31) && (long long)B * n_heads < (1LL << 16);
}
}  // namespace

size_t hgf_diff_attention_workspace_bytes(int B, int L_max, int n_heads, int d_h)
{
    return attn_dims_ok(B, L_max, n_heads, d_h) ? diff_attn_workspace_bytes(B, L_max, n_heads, d_h) : 0;
}

hgf_status hgf_diff_attention_decode(const void *q_f16, const void *k_cache_f16, const void *v_cache_f16,
                                     const int32_t *lens, int B, int L_max, int n_heads, int d_h, float lambda,
                                     void *out_f16, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!q_f16 || !k_cache_f16 || !v_cache_f16 || !lens || !out_f16) return HGF_ERR_NULL;
    if (!attn_dims_ok(B, L_max, n_heads, d_h)) return HGF_ERR_SHAPE;
    if (!aligned16(q_f16) || !aligned16(k_cache_f16) || !aligned16(v_cache_f16) ||
        (reinterpret_cast<uintptr_t>(out_f16) & 1u) || (reinterpret_cast<uintptr_t>(lens) & 3u))
        return HGF_ERR_ALIGN;
    if (!workspace || workspace_bytes < diff_attn_workspace_bytes(B, L_max, n_heads, d_h)) return HGF_ERR_WORKSPACE;
    if (!aligned16(workspace)) return HGF_ERR_ALIGN;
    return from_hip(launch_diff_attn(q_f16, k_cache_f16, v_cache_f16, lens, B, L_max, n_heads, d_h, lambda, out_f16,
                                     workspace, reinterpret_cast<hipStream_t>(stream)));
}

size_t hgf_packed_weight_bytes_b3(int d_out, int d_in)
{
    if (!dims_ok(d_in, d_out)) return 0;
    return b3_packed_bytes(d_out, d_in);
}

hgf_status hgf_quantize_pack_weights_b3(const float *W, int d_out, int d_in, void *packed_out, float *s_w_out,
                                        void *workspace, size_t workspace_bytes, void *stream)
{
    if (!W || !packed_out || !s_w_out) return HGF_ERR_NULL;
    if (!dims_ok(d_in, d_out)) return HGF_ERR_SHAPE;
    if (!aligned16(packed_out)) return HGF_ERR_ALIGN;
    if (!workspace) return HGF_ERR_WORKSPACE;
    const Workspace ws = carve_workspace(workspace, 1, 1, 1, 0);
    if (workspace_bytes < ws.bytes) return HGF_ERR_WORKSPACE;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    if (launch_wsum(W, (size_t)d_out * d_in, ws.wsum, s_w_out, st) != hipSuccess) return HGF_ERR_DEVICE;
    return from_hip(launch_pack_b3(W, d_out, d_in, s_w_out, reinterpret_cast<unsigned char *>(packed_out), st));
}

hgf_status hgf_unpack_weights_b3(const void *packed, int d_out, int d_in, int8_t *T_out, void *stream)
{
    if (!packed || !T_out) return HGF_ERR_NULL;
    if (!dims_ok(d_in, d_out)) return HGF_ERR_SHAPE;
    if (!aligned16(packed)) return HGF_ERR_ALIGN;
    return from_hip(launch_unpack_b3(reinterpret_cast<const unsigned char *>(packed), d_out, d_in, T_out,
                                     reinterpret_cast<hipStream_t>(stream)));
}

hgf_status hgf_linear_forward_b3(const void *x_f16, int M, const hgf_layer *L, void *y_f16, int32_t *acc_debug,
                                 void *workspace, size_t workspace_bytes, void *stream)
{
    if (!x_f16 || !y_f16) return HGF_ERR_NULL;
    const hgf_status s = check_layer(L, M);
    if (s != HGF_OK) return s;
    if (!aligned16(x_f16) || !aligned16(y_f16)) return HGF_ERR_ALIGN;
    if (!workspace) return HGF_ERR_WORKSPACE;
    if (!aligned16(workspace)) return HGF_ERR_ALIGN;
    const Workspace ws = carve_workspace(workspace, M, L->d_in, L->d_out, L->rank);
    if (workspace_bytes < ws.bytes) return HGF_ERR_WORKSPACE;
    if (L->ln_gamma || !b3_fits(M, L->d_in, L->rank)) return HGF_ERR_UNSUPPORTED;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    // steps 1, 2, 5, 6 of Algorithm 1: the decode prologue (quantiser, partial sums of A x, their sum and SiLU)
    ProParams pp;
    pp.x = reinterpret_cast<const _Float16 *>(x_f16);
    pp.xq = ws.xq;
    pp.s_x = ws.s_x;
    pp.rowsum = ws.rowsum;
    pp.amax_zero = nullptr;
    pp.quantize = 1;
    pp.M = M;
    pp.K = L->d_in;
    pp.Kp = round_up(L->d_in, kTileCols);
    pp.G = 1;
    pp.L[0].A = reinterpret_cast<const _Float16 *>(L->A_f16);
    pp.L[0].hpart = ws.hslices;
    pp.L[0].rank = L->rank;
    pp.L[0].rp = h_stride(L->rank > 0 ? L->rank : 1);
    _Float16 *h16[kMaxGroup] = {ws.h16, nullptr, nullptr, nullptr};
    if (launch_prologue(pp, h16, st) != hipSuccess) return HGF_ERR_DEVICE;
    return from_hip(launch_b3_decode(L->W_packed, ws, ws.h16, M, *L, y_f16, acc_debug, st));
}

size_t hgf_static_scratch_bytes(void) { return kStaticScratchBytes; }

size_t hgf_static_scratch_needed(int M, int d_in, int d_out, int rank)
{
    if (!dims_ok(d_in, d_out) || rank < 0 || rank > HGF_MAX_RANK || !tokens_ok(M, d_in, d_out)) return 0;
    return carve_workspace(nullptr, M, d_in, d_out, rank, 1, false).bytes;
}

hgf_status hgf_linear_forward_static(const void *x_f16, int M, const hgf_layer *L, void *y_f16, int32_t *acc_debug,
                                     void *stream)
{
    if (!x_f16 || !y_f16) return HGF_ERR_NULL;
    const hgf_status s = check_layer(L, M);
    if (s != HGF_OK) return s;
    if (!aligned16(x_f16) || !aligned16(y_f16) || (acc_debug && !aligned16(acc_debug))) return HGF_ERR_ALIGN;
    if (carve_static(nullptr, M, L).bytes > kStaticScratchBytes) return HGF_ERR_WORKSPACE;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    unsigned char *base = nullptr;
    const hgf_status ss = static_scratch(st, &base);
    if (ss != HGF_OK) return ss;
    const Workspace ws = carve_static(base, M, L);
    void *ys[1] = {y_f16};
    const bool profiling = g_profile;           // (the profiling aid creates events: not from here)
    g_profile = false;
    const hgf_status r = takes_decode_path(M, L, 1, false) ? run_decode_group(x_f16, M, L, 1, ys, acc_debug, ws, st)
                                          : run_large_group(x_f16, M, L, 1, ys, acc_debug, ws, st);
    g_profile = profiling;
    return r;
}

hgf_status hgf_stack_forward(const hgf_layer *layers, int n_layers, void *const *slots, int n_slots, int M,
                             void *workspace, size_t workspace_bytes, void *stream)
{
    if (!layers || !slots) return HGF_ERR_NULL;
    if (n_layers < 1 || n_slots < 1) return HGF_ERR_SHAPE;
    int d_in_max = 1, d_out_max = 1, rank_max = 0;
    for (int i = 0; i < n_layers; ++i) {
        const hgf_layer &L = layers[i];
        const hgf_status s = check_layer(&L, M);
        if (s != HGF_OK) return s;
        if (L.src_slot < 0 || L.src_slot >= n_slots || L.dst_slot < 0 || L.dst_slot >= n_slots ||
            L.src_slot == L.dst_slot)
            return HGF_ERR_SHAPE;
        if (!slots[L.src_slot] || !slots[L.dst_slot]) return HGF_ERR_NULL;
        if (!aligned16(slots[L.src_slot]) || !aligned16(slots[L.dst_slot])) return HGF_ERR_ALIGN;
        if (L.d_in > d_in_max) d_in_max = L.d_in;
        if (L.d_out > d_out_max) d_out_max = L.d_out;
        if (L.rank > rank_max) rank_max = L.rank;
    }
    if (!workspace) return HGF_ERR_WORKSPACE;
    if (!aligned16(workspace)) return HGF_ERR_ALIGN;
    const Workspace ws = carve_workspace(workspace, M, d_in_max, d_out_max, rank_max);
    if (workspace_bytes < ws.bytes) return HGF_ERR_WORKSPACE;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);

    // groups: consecutive layers reading the same slot with the same d_in, none of which writes
    // that slot or a slot another member writes
    struct Group { int first, G; bool stackable; };
    std::vector<Group> groups;
    for (int i = 0; i < n_layers;) {
        int G = 1;
        while (i + G < n_layers && G < kMaxGroup) {
            const hgf_layer &C = layers[i + G];
            bool ok = C.src_slot == layers[i].src_slot && C.d_in == layers[i].d_in && !C.ln_gamma && !layers[i].ln_gamma;
            for (int j = i; ok && j < i + G; ++j) ok = layers[j].dst_slot != C.dst_slot;
            if (!ok) break;
            ++G;
        }
        const int K = layers[i].d_in;
        bool stackable = g_launch_level >= 2 && M <= kMaxFusedM && K % 8 == 0 && K <= kMaxFusedK && !layers[i].ln_gamma;
        for (int g = 0; g < G && stackable; ++g) {
            const hgf_layer &L = layers[i + g];
            stackable = L.d_out % 8 == 0 &&
                        (L.rank == 0 || (L.rank % 8 == 0 && aligned16(L.A_f16) && aligned16(L.B_f16) &&
                                         (reinterpret_cast<uintptr_t>(L.alpha_f16) & 3u) == 0));
        }
        groups.push_back({i, G, stackable});
        i += G;
    }

    auto run_group = [&](const Group &gr) -> hgf_status {
        const void *x = slots[layers[gr.first].src_slot];
        if (takes_decode_path(M, layers + gr.first, gr.G, false)) {
            void *ys[kMaxGroup];
            for (int g = 0; g < gr.G; ++g) ys[g] = slots[layers[gr.first + g].dst_slot];
            return run_decode_group(x, M, layers + gr.first, gr.G, ys, nullptr, ws, st);
        }
        void *ys[kMaxGroup];
        for (int g = 0; g < gr.G; ++g) ys[g] = slots[layers[gr.first + g].dst_slot];
        return run_large_group(x, M, layers + gr.first, gr.G, ys, nullptr, ws, st);
    };

    // Runs groups [a, b), all stackable, as one persistent launch.  kNoFit: they do not fit one
    // (nothing was enqueued; the groups then run one by one); kRefused: the runtime refused it.
    auto run_stack = [&](size_t a, size_t b) -> Launch {
        StackParams sp;
        sp.M = M;
        sp.nphases = (int)(b - a);
        sp.flags = ws.flags;
        sp.xchg = ws.xchg;
        int nl = 0;
        size_t act = 0;
        for (size_t gi = a; gi < b; ++gi) {
            const Group &gr = groups[gi];
            StackPhase &P = sp.ph[gi - a];
            P.K = layers[gr.first].d_in;
            P.first_layer = (short)nl;
            P.G = (short)gr.G;
            // the tokens: the latest earlier layer of this launch that writes the slot, else the slot itself
            const int src = layers[gr.first].src_slot;
            P.x_ext = reinterpret_cast<const _Float16 *>(slots[src]);
            P.src_off = 0;
            for (int j = 0; j < nl; ++j) {
                if (layers[groups[a].first + j].dst_slot == src) {
                    P.x_ext = nullptr;
                    P.src_off = sp.L[j].act_off;
                }
            }
            for (int g = 0; g < gr.G; ++g) {
                const hgf_layer &L = layers[gr.first + g];
                StackLayer &D = sp.L[nl++];
                D.packed = reinterpret_cast<const v4u *>(L.W_packed);
                D.s_w = L.s_w;
                D.A = reinterpret_cast<const _Float16 *>(L.A_f16);
                D.B = reinterpret_cast<const _Float16 *>(L.B_f16);
                D.alpha = reinterpret_cast<const _Float16 *>(L.alpha_f16);
                D.y = reinterpret_cast<_Float16 *>(slots[L.dst_slot]);
                D.N = L.d_out;
                D.rank = L.rank;
                D.act_off = (unsigned)act;
                D.reserved = 0;
                act += align256((size_t)M * L.d_out * 2);
            }
        }
        if (act > kStackActBytes) return Launch::kNoFit;
        sp.act_used = (unsigned)act;
        size_t lds_bytes = 0;
        if (!plan_stack(sp, &lds_bytes)) return Launch::kNoFit;
        ProfileScope prof(0, st);
        return launch_stack(sp, lds_bytes, st) == hipSuccess ? Launch::kRan : Launch::kRefused;
    };

    size_t gi = 0;
    while (gi < groups.size()) {
        // the longest run of stackable groups that fits one launch's description
        size_t ge = gi;
        int nl = 0;
        size_t act = 0;
        while (ge < groups.size() && groups[ge].stackable && (int)(ge - gi) < kStackMaxPhases &&
               nl + groups[ge].G <= kStackMaxLayers) {
            size_t add = 0;
            for (int g = 0; g < groups[ge].G; ++g) add += align256((size_t)M * layers[groups[ge].first + g].d_out * 2);
            if (act + add > kStackActBytes) break;
            act += add;
            nl += groups[ge].G;
            ++ge;
        }
        if (ge - gi >= 2) {
            const Launch r = run_stack(gi, ge);
            if (r == Launch::kRefused) return HGF_ERR_DEVICE;
            if (r == Launch::kRan) {
                gi = ge;
                continue;
            }
        }
        if (ge == gi) ge = gi + 1;
        for (; gi < ge; ++gi) {
            const hgf_status s = run_group(groups[gi]);
            if (s != HGF_OK) return s;
        }
    }
    return HGF_OK;
}

void hgf_profile_enable(int on) { g_profile = on != 0; }

hgf_status hgf_profile_collect(double *ms_out, long long *launches_out)
{
    if (!ms_out || !launches_out) return HGF_ERR_NULL;
    for (int kind = 0; kind < 2; ++kind) {
        double total = 0.0;
        long long n = 0;
        for (auto &pr : g_events[kind]) {
            float ms = 0.f;
            if (hipEventSynchronize(pr.second) == hipSuccess && hipEventElapsedTime(&ms, pr.first, pr.second) == hipSuccess) {
                total += ms;
                ++n;
            }
            g_event_pool.push_back(pr.first);
            g_event_pool.push_back(pr.second);
        }
        g_events[kind].clear();
        ms_out[kind] = total;
        launches_out[kind] = n;
    }
    return HGF_OK;
}

void hgf_set_single_launch(int level) { g_launch_level = level < 0 ? 0 : (level > 2 ? 2 : level); }

void hgf_set_wait_limit(int tries) { set_stack_wait_limit(tries); }

void hgf_set_stack_trace(void *device_buffer, size_t bytes, int first_phase)
{
    set_stack_trace(reinterpret_cast<unsigned long long *>(device_buffer), bytes, first_phase);
}

}  // extern "C"
