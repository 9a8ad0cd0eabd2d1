// A whole list of layers for a handful of tokens (M <= 4) in ONE persistent launch.
//
// Algorithm 1 of the HGF paper, steps 1-8, for every layer of a stack.  Launching each group
// of layers on its own leaves two thirds of the time in launch gaps and start-up latency
// (first touch of the activations, cold translation, kernel arguments).  Here the workgroups
// (one per compute unit) stay resident for the whole list and walk it phase by phase -- a
// phase is a group of up to four layers that read the same activations:
//
//   * two loader wavefronts stream the weight tiles into rings in LDS, phase after phase as
//     far ahead as the rings reach: weights do not depend on activations, so while a phase
//     waits for its input the memory system keeps delivering its tiles;
//   * eight contracting wavefronts (two per SIMD): wavefront w contracts the k-tiles w, w+8,
//     ... of every row-block, so it fetches and quantises exactly those columns of the tokens
//     itself; the eight meet once per phase, for the per-token absmax;
//   * the slice wavefront computes its slice of A x from the columns that slice needs,
//     collects all slices and puts SiLU of their sum into LDS;
//   * the unit wavefront finishes the units its workgroup owns (dequantise, B h, gate, store).
//   No wavefront takes part in a workgroup barrier after the first instruction: the roles
//   meet through counters in LDS.
//
// Activations pass from one phase to the next through the workspace: the unit wavefronts
// store every output both to the caller's slot and, with device scope, to an exchange
// region that holds a sentinel bit pattern (all ones) wherever nothing has been written;
// readers re-read with device scope until no word is the sentinel.  No flag, no fence, no
// grid barrier.  (An output that is NaN is stored as the canonical quiet NaN, which is not
// the sentinel.)  The partial sums of A x travel the same way.  Two sets of regions
// alternate from launch to launch by a counter in the workspace; each launch refills, in the
// other set, what the previous launch used.  Every wait is bounded; on expiry a sticky word
// is set in the workspace, the affected outputs are NaN and later waits are skipped.
#include "hgf_internal.h"


#include <type_traits>

namespace hgf {

namespace {

constexpr int kStream = 8;             // contracting wavefronts per workgroup (0..7): two per SIMD, so that one's
                                       // MFMAs overlap the other's unpacking of the 2-bit codes
constexpr int kLoaders = 2;            // loader wavefronts (8, 9): each feeds four contracting ones; 10, 11 serve
constexpr int kFeed = kStream / kLoaders;
constexpr int kUnitWaves = 4;          // unit wavefronts (11..14): unit i of a workgroup goes to number i mod 4
constexpr int kWaves = kStream + kLoaders + 1 + kUnitWaves;
constexpr int kWindow = 3;             // groups of kFeed weight tiles a loader keeps in flight
constexpr int kMinRing = 8;            // tiles per contracting wavefront the LDS ring must hold at least (> kWindow; even)
constexpr int kMaxRing = 48;
constexpr int kMaxUnits = 16;          // units per workgroup and phase at most
constexpr int kLdsPollsDefault = 1 << 22;   // bound of a wait on LDS (about a second)
constexpr int kMemPollsDefault = 1 << 18;   // bound of a wait on an exchange region (about a second)
constexpr unsigned kSentinel = 0xFFFFFFFFu;
constexpr int kHsStride = HGF_MAX_RANK;  // halves per (layer, token) row of SiLU(A x) in LDS
constexpr int kUN = 8;                 // 64-column steps of a slice of A x requested together
constexpr int kSplit = kFusedSplit;    // slices of d_in at most

typedef __attribute__((address_space(3))) void *lds_ptr_t;
typedef unsigned int v2u __attribute__((ext_vector_type(2)));

struct Control {                       // LDS words shared by the two sides; [2]: one set per phase parity
    alignas(16) int ready[kStream];    // weight tiles of the wavefront's ring that have landed in LDS, in all
    int consumed[kStream];             // ... and how many of them it has read
    int arrived[2][kMaxUnits];         // contracting wavefronts that have posted the unit (the unit wavefront resets it)
    int rowsum_part[2][kStream][kMaxFusedM];   // sums of the quantised columns each wavefront owns
    float amax_part[2][kStream][kMaxFusedM];   // absmax of those columns
    float sx[2][kMaxFusedM];
    int sync;                          // absmax parts posted, summed over the phases
    int svc_done[kUnitWaves];          // phases whose units each unit wavefront has finished
    int h_ready;                       // phases whose SiLU(A x) the slice wavefront has put into LDS
    int failed;                        // a wait of a loader, contracting or slice wavefront has expired
    unsigned long long stamps[kTraceRoles][kTracePhases][kTraceIds];   // time stamps (only with p.trace set)
};

// Notes the device-wide clock for (role, phase, id) when tracing is on and the phase is traced.
#define HGF_STAMP(role, ph, id)                                                                        \
    do {                                                                                               \
        if (p.trace != nullptr && (threadIdx.x & 63) == 0 && (unsigned)((ph)-p.trace_ph0) < (unsigned)kTracePhases) \
            ctl->stamps[role][(ph)-p.trace_ph0][id] = wall_clock64();                                  \
    } while (0)
__device__ __forceinline__ void trace_flush(const StackParams &p, Control *ctl, int c, int role)
{
    if (p.trace == nullptr) return;
    const unsigned long long *src = &ctl->stamps[role][0][0];
    unsigned long long *dst = p.trace + ((size_t)c * kTraceRoles + role) * kTracePhases * kTraceIds;
    for (int e = threadIdx.x & 63; e < kTracePhases * kTraceIds; e += 64) dst[e] = src[e];
}

__device__ __forceinline__ int lds_load(const int *p) { return __hip_atomic_load(p, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP); }
__device__ __forceinline__ v4u load16_agent(rsrc_t r, unsigned off, bool ok = true)
{
    return __builtin_bit_cast(v4u, __builtin_amdgcn_raw_buffer_load_b128(r, (int)(ok ? off : kOob), 0, 16));
}
__device__ __forceinline__ void store16_agent(rsrc_t r, unsigned off, v4u v)
{
    __builtin_amdgcn_raw_buffer_store_b128(v, r, (int)off, 0, 16);
}
__device__ __forceinline__ bool has_sentinel(v4u v)
{
    return v[0] == kSentinel || v[1] == kSentinel || v[2] == kSentinel || v[3] == kSentinel;
}
__device__ __forceinline__ float exp_fast(float v) { return __builtin_amdgcn_exp2f(v * 1.44269504088896340736f); }
__device__ __forceinline__ float silu_fast(float h) { return h * __builtin_amdgcn_rcpf(1.0f + exp_fast(-h)); }
__device__ __forceinline__ float tanh_fast(float a) { return 1.0f - 2.0f * __builtin_amdgcn_rcpf(1.0f + exp_fast(2.0f * a)); }
// Every unit wavefront has finished the phases before `n`.
__device__ __forceinline__ bool units_done(const Control *ctl, int n)
{
    bool ok = true;
#pragma unroll
    for (int u = 0; u < kUnitWaves; ++u) ok = ok && lds_load(&ctl->svc_done[u]) >= n;
    return ok;
}
// What both sides derive from a phase's entry in the kernel arguments (all wave-uniform).
struct PhaseShape {
    int K, Kp, KT, TPW, TPP, G, first; // TPW: k-tiles per contracting wavefront; TPP: pairs of them; first: the phase's first layer
    int units, nunits;                 // row-blocks of the phase; of this workgroup
    int us1, us2, us3;                 // running sums of the layers' row-blocks (0x7fffffff beyond G)
};
__device__ __forceinline__ PhaseShape shape_of(const StackParams &p, int ph, int c)
{
    PhaseShape s;
    const StackPhase &P = p.ph[ph];
    s.K = P.K;
    s.Kp = (s.K + kTileCols - 1) / kTileCols * kTileCols;
    s.KT = s.Kp / kTileCols;
    s.TPW = (s.KT + kStream - 1) / kStream;
    s.TPP = (s.TPW + 1) / 2;
    s.G = P.G;
    s.first = P.first_layer;
    const int r0 = (p.L[s.first].N + kTileRows - 1) / kTileRows;
    const int r1 = s.G > 1 ? (p.L[s.first + 1].N + kTileRows - 1) / kTileRows : 0;
    const int r2 = s.G > 2 ? (p.L[s.first + 2].N + kTileRows - 1) / kTileRows : 0;
    const int r3 = s.G > 3 ? (p.L[s.first + 3].N + kTileRows - 1) / kTileRows : 0;
    s.us1 = s.G > 1 ? r0 : 0x7fffffff;
    s.us2 = s.G > 2 ? r0 + r1 : 0x7fffffff;
    s.us3 = s.G > 3 ? r0 + r1 + r2 : 0x7fffffff;
    s.units = r0 + r1 + r2 + r3;
    s.nunits = c < s.units ? (s.units - c + p.nwg - 1) / p.nwg : 0;
    return s;
}
typedef _Float16 v2h __attribute__((ext_vector_type(2)));
// fp32 product of fp16 half H (0: low, 1: high) of `packed` and the fp32 `scale`, rounded once
// (an FMA whose addend is zero), without a conversion instruction of its own
template <int H>
__device__ __forceinline__ float scaled_half(uint32_t packed, float scale)
{
    float r;
    if (H == 0) asm("v_fma_mix_f32 %0, %1, %2, 0 op_sel_hi:[1,0,0]" : "=v"(r) : "v"(packed), "v"(scale));
    else asm("v_fma_mix_f32 %0, %1, %2, 0 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "=v"(r) : "v"(packed), "v"(scale));
    return r;
}

// ------------------------------------------------------------------ loaders and contracting wavefronts
// Per-token absmax int8 quantisation (Sec. 2.2.1) of the columns wavefront w contracts: the
// k-tiles w, w+8, ... (128 columns each).  The columns come from the caller's slot or, once
// no word of them is the sentinel, from the exchange region; they stay in registers between
// the two passes.  The eight wavefronts exchange their absmax parts through LDS and a counter
// (`sync_target`: its value once all eight have posted this phase's part); the quantised
// columns go to the token rows in LDS, where only this wavefront reads them.
template <int MT>
__device__ __forceinline__ void fetch_quantise(const StackParams &p, const PhaseShape &S, rsrc_t xr, bool ext,
                                               unsigned char *lds, Control *ctl, int w, int ph, int sync_target,
                                               bool &failed)
{
    const int l = threadIdx.x & 63, par = ph & 1;
    constexpr int XU = 3;               // 64 lanes x 3 pieces of 8 columns = 12 tiles of a token
    const int pc = l & 15;
    // what this phase shares with the unit wavefront was last used two phases ago; looked at
    // here, where the wavefront is about to wait for memory anyway, and waited for (rarely)
    // after the tokens have come
    bool unit_done = units_done(ctl, ph - 1);
    v4u v[MT][XU];
    int polls = 0;
    // Nothing of the layer before can be complete while this workgroup's own row-blocks of it
    // are not stored, and the lines of that layer's output are polled by every workgroup: the
    // time a poll takes grows with the polls queued on a line, so polls that cannot succeed only
    // delay the ones that can (measured: 3040 -> 3120 GB/s).
    if (!ext) {
        int spins = 0;
#pragma clang loop unroll(disable)
        while (!failed && !units_done(ctl, ph)) {
            if (++spins >= p.lds_polls) failed = true;
            __builtin_amdgcn_s_sleep(1);
        }
        unit_done = true;
    }
#pragma clang loop unroll(disable)
    while (true) {
        bool ready = true;
#pragma unroll
        for (int m = 0; m < MT; ++m) {
#pragma unroll
            for (int u = 0; u < XU; ++u) {
                const int j = (l >> 4) + 4 * u;
                const int col = (j * kStream + w) * kTileCols + pc * 8;
                v[m][u] = load16_agent(xr, (unsigned)(m * S.K + col) * 2u, m < p.M && j < S.TPW && col < S.K);
                ready = ready && !has_sentinel(v[m][u]);
            }
        }
        if (ext || failed || __builtin_amdgcn_ballot_w64(!ready) == 0) break;
        if (++polls >= p.mem_polls) {
            failed = true;
            break;
        }
        __builtin_amdgcn_s_sleep(1);
    }
    HGF_STAMP(w, ph, 1);
#pragma unroll
    for (int m = 0; m < MT; ++m) {
        // (the maximum of fp16 magnitudes is exact in fp16: two at a time, widened once at the end;
        //  the instruction by hand: the builtin adds a canonicalising maximum per operand)
        uint32_t mx = 0u;
#pragma unroll
        for (int u = 0; u < XU; ++u) {
            if (4 * u >= S.TPW) continue;           // (no k-turn that far in this phase: nothing was read)
#pragma unroll
            for (int d = 0; d < 4; ++d) asm("v_pk_max_f16 %0, %1, %2" : "=v"(mx) : "v"(mx), "v"(v[m][u][d] & 0x7fff7fffu));
        }
        const v2h mx2 = __builtin_bit_cast(v2h, mx);
        float amax = wave_max(fmaxf((float)mx2[0], (float)mx2[1]));
        if (l == 0) ctl->amax_part[par][w][m] = amax;
    }
    if (l == 0) __hip_atomic_fetch_add(&ctl->sync, 1, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
    polls = 0;
#pragma clang loop unroll(disable)
    while (!failed && lds_load(&ctl->sync) < sync_target) {
        if (++polls >= p.lds_polls) failed = true;
    }
    HGF_STAMP(w, ph, 2);
    polls = 0;
#pragma clang loop unroll(disable)
    while (!unit_done && !failed) {
        unit_done = units_done(ctl, ph - 1);
        if (++polls >= p.lds_polls) failed = true;
        __builtin_amdgcn_s_sleep(1);
    }
#pragma unroll
    for (int m = 0; m < MT; ++m) {
        float amax = ctl->amax_part[par][0][m];
#pragma unroll
        for (int i = 1; i < kStream; ++i) amax = fmaxf(amax, ctl->amax_part[par][i][m]);
        amax = fmaxf(amax, 1e-5f);
        const float inv = 127.0f / amax;
        int sum = 0;
#pragma unroll
        for (int u = 0; u < XU; ++u) {
            if (4 * u >= S.TPW) continue;
            const int j = (l >> 4) + 4 * u;
            const int kt = j * kStream + w;
            // (columns past d_in were read as zero)
            // round(x * inv) by adding 1.5 * 2^23 to the (separately rounded) product: the sum's
            // spacing is 1, so the addition rounds half to even and leaves the integer, in two's
            // complement, in the low mantissa bits -- its low byte is the code.  No clipping: |x| is
            // at most the token's absmax, so the product is at most 127 (1 + 2^-23).  Three byte
            // permutes gather four codes into a word, a dot product with ones adds them up.
            // The product comes from the mixed-precision FMA with a zero addend: it widens the fp16
            // operand itself and rounds once, which is the fp32 product, in one instruction instead of two.
            uint32_t rb[8];
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                rb[2 * d] = __builtin_bit_cast(uint32_t, __fadd_rn(scaled_half<0>(v[m][u][d], inv), 12582912.0f));
                rb[2 * d + 1] = __builtin_bit_cast(uint32_t, __fadd_rn(scaled_half<1>(v[m][u][d], inv), 12582912.0f));
            }
            uint32_t q2[2];
#pragma unroll
            for (int hw = 0; hw < 2; ++hw) {
                const uint32_t lo = __builtin_amdgcn_perm(rb[4 * hw + 1], rb[4 * hw + 0], 0x0c0c0400u);
                const uint32_t hi = __builtin_amdgcn_perm(rb[4 * hw + 3], rb[4 * hw + 2], 0x0c0c0400u);
                q2[hw] = __builtin_amdgcn_perm(hi, lo, 0x05040100u);
                sum = __builtin_amdgcn_sdot4((int)q2[hw], 0x01010101, sum, false);
            }
            // The tile's 128 codes are stored in the order the contraction reads them: column
            // 32 t + 16 h + 4 s + b of the tile at byte (4 h + s) 16 + 4 t + b, so that the sixteen
            // columns one MFMA operand register set needs for shift s (all t, all b) are contiguous.
            // The lane's eight columns are t = pc / 4, h = (pc / 2) % 2, s = 2 (pc % 2) and s + 1.
            if (m < p.M && j < S.TPW && kt < S.KT) {
                unsigned char *at = lds + m * p.xstride + kt * kTileCols + (((pc >> 1) & 1) * 4 + (pc & 1) * 2) * 16 + (pc >> 2) * 4;
                *reinterpret_cast<uint32_t *>(at) = q2[0];
                *reinterpret_cast<uint32_t *>(at + 16) = q2[1];
            }
        }
        sum = wave_sum(sum);
        if (l == 0 && m < p.M) {
            ctl->rowsum_part[par][w][m] = sum;
            if (w == 0) ctl->sx[par][m] = amax / 127.0f;
        }
    }
}

// LDS accesses the compiler must not see: around LDS-direct loads it orders every LDS access it
// knows of behind all outstanding memory operations, which would empty the loader's window.
__device__ __forceinline__ unsigned lds_offset(const void *q)
{
    return (unsigned)reinterpret_cast<size_t>((__attribute__((address_space(3))) const void *)q);
}
__device__ __forceinline__ int lds_peek(unsigned at)
{
    int v;
    asm volatile("ds_read_b32 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(v) : "v"(at) : "memory");
    return v;
}
__device__ __forceinline__ void lds_poke(unsigned at, int v)
{
    asm volatile("ds_write_b32 %0, %1\n\ts_waitcnt lgkmcnt(0)" ::"v"(at), "v"(v) : "memory");
}

// ---- a loader wavefront: streams the weight tiles of kFeed contracting wavefronts (a = kFeed*ld
//      and the following) into their rings in LDS with LDS-direct loads, in the order those will
//      read them: phase by phase, row-block by row-block, k-turn by k-turn.  Weights do not
//      depend on activations, so it runs ahead of the phases as far as the rings reach; it keeps
//      kWindow groups of requests in flight (enough to cover the memory's latency, few enough
//      that the queues stay short for the other wavefronts' exchanges) and publishes a group once
//      kWindow younger ones have been issued and the wait count says it has landed.
__device__ __forceinline__ void loader_wave(const StackParams &p, unsigned char *lds, Control *ctl, int c, int ld)
{
    const int l = threadIdx.x & 63;
    const int a = kFeed * ld;
    unsigned char *ring = lds + p.ring_off + (size_t)a * p.ring_slots * kTileBytes;
    const unsigned ready_at = lds_offset(&ctl->ready[a]), cons_at = lds_offset(&ctl->consumed[a]);
    const unsigned failed_at = lds_offset(&ctl->failed);
    // (one 16-byte write for the four readers, not waited for: LDS takes a wavefront's requests in order)
    static_assert(kFeed == 4 && offsetof(Control, ready) % 16 == 0, "the four counters are written as one piece");
    auto publish = [&](int n) __attribute__((always_inline)) {
        const v4i four = {n, n, n, n};
        asm volatile("ds_write_b128 %0, %1" ::"v"(ready_at), "v"(four) : "memory");
    };
    // waits until at most k of the groups requested are still on their way
    auto landed_but = [](int k) __attribute__((always_inline)) {
        static_assert(kWindow <= 5, "one case per group of the window");
        switch (k) {
            case 0: asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); break;
            case 1: asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kFeed * 1) : "memory"); break;
            case 2: asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kFeed * 2) : "memory"); break;
            case 3: asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kFeed * 3) : "memory"); break;
            case 4: asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kFeed * 4) : "memory"); break;
            default: asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kFeed * 5) : "memory"); break;
        }
    };
    // groups issued; ring slot of the next; groups published; groups all readers are known to have read
    int n = 0, slot = 0, pub = 0, freed = 0;
    bool failed = false;
    for (int ph = 0; ph < p.nphases; ++ph) {
        const PhaseShape S = shape_of(p, ph, c);
        const StackLayer *L = p.L + S.first;
        if (ld == 0) HGF_STAMP(kStream + 2, ph, 0);
        if (ld == 0 && p.trace != nullptr && l == 0 && (unsigned)(ph - p.trace_ph0) < (unsigned)kTracePhases)
            ctl->stamps[kStream + 2][ph - p.trace_ph0][2] = clock64();
        for (int i = 0; i < S.nunits; ++i) {
            const int u = c + i * p.nwg;
            int g = 0, first = 0;
            if (u >= S.us1) { g = 1; first = S.us1; }
            if (u >= S.us2) { g = 2; first = S.us2; }
            if (u >= S.us3) { g = 3; first = S.us3; }
            const unsigned rows = (unsigned)((L[g].N + kTileRows - 1) / kTileRows);
            const rsrc_t wr = make_rsrc(L[g].packed, rows * S.KT * kTileBytes);
            const unsigned row = (unsigned)(u - first) * S.KT;
            for (int j = 0; j < 2 * S.TPP; ++j) {   // (an odd count is padded with a void tile: the contraction goes in pairs)
                // room in the rings?  While there is none, the groups on their way are published one
                // by one as they land (the readers may be waiting for exactly those), and the next
                // request goes out as soon as the readers have freed a slot: the readers free slots
                // two at a time while they contract, and a loader that let everything land before
                // it looked again would then request one group per trip to memory.
                if (n - freed >= p.ring_slots) {
                    int spins = 0;
#pragma clang loop unroll(disable)
                    while (!failed) {
                        freed = lds_peek(cons_at);
#pragma unroll
                        for (int f = 1; f < kFeed; ++f) freed = min(freed, lds_peek(cons_at + 4u * f));
                        if (n - freed < p.ring_slots) break;
                        if (pub < n) {
                            landed_but(n - pub - 1);
                            publish(++pub);
                        } else {
                            if (++spins >= p.lds_polls || lds_peek(failed_at) != 0) failed = true;
                            __builtin_amdgcn_s_sleep(2);
                        }
                    }
                }
#pragma unroll
                for (int f = 0; f < kFeed; ++f) {
                    const int kt = j * kStream + a + f;
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(
                        wr, (lds_ptr_t)(ring + ((size_t)f * p.ring_slots + slot) * kTileBytes), 16,
                        (int)(kt < S.KT ? (row + kt) * kTileBytes + l * 16 : kOob), 0, 0, 2);
                }
                ++n;
                slot = slot + 1 == p.ring_slots ? 0 : slot + 1;
                if (n - pub > kWindow) {
                    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kFeed * kWindow) : "memory");
                    pub = n - kWindow;
                    publish(pub);
                }
            }
        }
        if (ld == 0) HGF_STAMP(kStream + 2, ph, 1);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    publish(n);
    if (ld == 0) trace_flush(p, ctl, c, kStream + 2);
    if (failed && l == 0) {
        lds_poke(failed_at, 1);
        __hip_atomic_store(p.flags + 2, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// ---- a contracting wavefront: quantises its columns of the phase's tokens, then contracts the
//      k-tiles w, w+8, ... of every row-block of the workgroup with them (Alg. 1 steps 2-3),
//      reading the tiles from its ring in LDS as the loader publishes them
__device__ __forceinline__ void contract_wave(const StackParams &p, unsigned char *lds, Control *ctl, int c)
{
    const int tid = threadIdx.x, l = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);

    const unsigned epoch = (unsigned)__hip_atomic_load(p.flags + 4, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const unsigned char *mine = p.xchg + (size_t)(epoch & 1u) * kStackSetBytes;
    bool failed = false;
    int sync_target = 0;
    int gs = 0, slot = 0, known = 0;    // tiles read so far; ring slot of the next; tiles known to have landed
    for (int ph = 0; ph < p.nphases; ++ph) {
        const PhaseShape S = shape_of(p, ph, c);
        const int par = ph & 1;
        if (S.nunits == 0) continue;
        {
            const StackPhase &P = p.ph[ph];
            const bool ext = P.x_ext != nullptr;
            const rsrc_t xr = make_rsrc(ext ? reinterpret_cast<const unsigned char *>(P.x_ext) : mine + P.src_off,
                                        (unsigned)p.M * S.K * 2u);
            sync_target += kStream;
            if (lds_load(&ctl->failed) != 0) failed = true;
            const bool was = failed;
            HGF_STAMP(w, ph, 0);
            if (p.M == 1) fetch_quantise<1>(p, S, xr, ext, lds, ctl, w, ph, sync_target, failed);
            else if (p.M == 2) fetch_quantise<2>(p, S, xr, ext, lds, ctl, w, ph, sync_target, failed);
            else fetch_quantise<4>(p, S, xr, ext, lds, ctl, w, ph, sync_target, failed);
            if (failed && !was && l == 0) {
                __hip_atomic_store(&ctl->failed, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                __hip_atomic_store(p.flags + 2, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            HGF_STAMP(w, ph, 3);
        }

        // ---- contraction with the 16x16x64 MFMA, two k-tiles to a step.  The tokens (at most
        //      four) are rows of A, sixteen weight rows the columns of B.  A packed tile keeps, for
        //      weight row r and k-half h, sixteen bytes (lane r + 32 h of the 32x32x32 layout) whose
        //      dword t holds the codes of columns 32 t + 16 h + 4 s + b at bits 8 b + 2 s.  Lane
        //      (n = l%16, kq = l/16) reads exactly those sixteen bytes, of tile kq/2 of the pair and
        //      k-half kq%2, with one conflict-free 16-byte LDS read per row half nb; masking them
        //      with 0x03030303 << 2 s leaves, in place, the sixteen codes of shift s times 4^s:
        //      an operand of an MFMA whose k-index runs over (tile, h, t, b) -- no shifts.  (For
        //      s = 3 the dword is shifted right once first, so that 2 << 6 does not overflow int8:
        //      scale 32.)  Each shift has accumulators of its own; at the end of a unit they are
        //      divided by their scales -- exactly: every term is a multiple -- and added.  The
        //      tokens' image in LDS is stored in the matching order (fetch_quantise), so the A
        //      operand of shift s is one 16-byte read as well.  20 vector instructions unpack a
        //      tile where shift-and-mask of single dwords took 28, and the reads of the tile are
        //      two instead of four conflicting ones: the step is bound by instruction issue.
        //      A wavefront issues its MFMAs and its other vector instructions one after the other
        //      (the other contracting wavefront of the SIMD fills the gaps), so everything that is
        //      not contraction is kept out of the step: scalar conditions, no branches but the
        //      rare waits, ring bookkeeping every other step.  The operands of the next step are
        //      read from LDS while this step computes.
        int *tiles = reinterpret_cast<int *>(lds + p.tile_off) + par * p.tile_par;
        const int n16 = l & 15, kq = l >> 4;
        const unsigned char *tlane = lds + p.ring_off + (size_t)w * p.ring_slots * kTileBytes + (kq >> 1) * kTileBytes +
                                     (n16 + 32 * (kq & 1)) * 16;
        // this lane's token row, at its tile of the pair and its k-half; and 128 bytes of zeros
        const int xbase = (n16 < p.M ? n16 : 0) * p.xstride + ((kq >> 1) * kStream + w) * kTileCols + (kq & 1) * 64;
        const int zbase = p.jx_off + kMaxFusedM * 1024 + (kq & 1) * 64;
        const int total = S.nunits * S.TPP;             // steps: pairs of tiles
        const unsigned long long token_rows = __builtin_amdgcn_ballot_w64(n16 < p.M);
        unsigned long long exec_save;
        const unsigned cons_at = lds_offset(&ctl->consumed[w]);
        struct Ops {
            v4u t[2];                   // [nb]: the lane's sixteen bytes of codes of row half nb
            v4i x[4];                   // [s]: the lane's token's sixteen columns of shift s
        };
        Ops o0, o1;
        // requests the operands of step `st` (pair jp of its row-block): the tiles' bytes from the
        // ring (waiting, if the contraction has caught up with the loader, until both tiles have
        // landed) and the tokens' columns -- zeros where the row-block has no k-tile for this
        // wavefront (the second tile of its last pair, or a void turn), so that the MFMAs need no
        // condition.  Past the phase's last step the requests still go out, to addresses that are
        // valid and hold nothing of interest: requests under a condition would make every wait on
        // LDS a wait for all.
        auto operands = [&](Ops &o, int jp, int st) __attribute__((always_inline)) {
            const bool real = st < total;
            if (__builtin_expect(real && known < gs + 2 * st + 2, 0)) {
                const bool traced = p.trace != nullptr && (unsigned)(ph - p.trace_ph0) < (unsigned)kTracePhases;
                const unsigned long long since = traced ? wall_clock64() : 0ull;
                int spins = 0;
#pragma clang loop unroll(disable)
                do {
                    known = __builtin_amdgcn_readfirstlane(lds_load(&ctl->ready[w]));
                    if (++spins >= p.lds_polls) failed = true;
                } while (known < gs + 2 * st + 2 && !failed);
                if (traced && l == 0) {     // ids 6, 7: clock ticks spent waiting for tiles to land, and the waits
                    ctl->stamps[w][ph - p.trace_ph0][6] += wall_clock64() - since;
                    ctl->stamps[w][ph - p.trace_ph0][7] += 1;
                }
            }
            const unsigned char *ta = tlane + slot * kTileBytes;        // (the ring holds an even number of tiles)
            o.t[0] = *reinterpret_cast<const v4u *>(ta);
            o.t[1] = *reinterpret_cast<const v4u *>(ta + 256);
            const int next = slot + 2 == p.ring_slots ? 0 : slot + 2;
            slot = real ? next : slot;
            const int kt = (2 * jp + (kq >> 1)) * kStream + w;           // this lane's tile of the pair
            const int xa = kt < S.KT ? xbase + 2 * jp * kStream * kTileCols : zbase;
            // Only the lanes of the tokens' rows read: a read by all 64 lanes costs LDS 16 times
            // the bandwidth, and LDS is what the eight contracting wavefronts share.  The lanes are
            // switched off around the reads by hand: a branch would make the compiler wait here for
            // the requests just made.  It does not see these reads, so the step waits for them itself.
            // The same lanes tell the loader what it may overwrite: the tiles of the step before
            // this request's are in registers by now (the caller has waited for them).
            asm volatile("s_mov_b64 %[save], exec\n\t"
                         "s_mov_b64 exec, %[rows]\n\t"
                         "ds_read_b128 %[a], %[at]\n\t"
                         "ds_read_b128 %[b], %[at] offset:16\n\t"
                         "ds_read_b128 %[c], %[at] offset:32\n\t"
                         "ds_read_b128 %[d], %[at] offset:48\n\t"
                         "ds_write_b32 %[cons], %[done]\n\t"
                         "s_mov_b64 exec, %[save]"
                         : [a] "=&v"(o.x[0]), [b] "=&v"(o.x[1]), [c] "=&v"(o.x[2]), [d] "=&v"(o.x[3]), [save] "=&s"(exec_save)
                         : [at] "v"(lds_offset(lds + xa)), [rows] "s"(token_rows), [cons] "v"(cons_at),
                           [done] "v"(gs + 2 * min(st, total))
                         : "memory");
        };
        auto masked = [](const v4u t, unsigned m) __attribute__((always_inline)) {
            return (v4i){(int)(t[0] & m), (int)(t[1] & m), (int)(t[2] & m), (int)(t[3] & m)};
        };
        int ci = 0, cj = 0;
        const unsigned arrived_at = lds_offset(&ctl->arrived[par][0]);
        // [nb][s]: weight rows 0..15 and 16..31 of the unit, shift s (scale 1, 4, 16, 32); element m: token m
        v4i acc[2][4];
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
            for (int sh = 0; sh < 4; ++sh) acc[nb][sh] = (v4i){0, 0, 0, 0};
        // one step: request the next step's operands into the other register set, then contract
        // this step's (two named sets, taken in turn: copying one set into the other would wait
        // for the requests just made and undo the overlap)
        auto step = [&](const Ops &oc, Ops &on, int st) __attribute__((always_inline)) {
            const int nj = cj + 1 == S.TPP ? 0 : cj + 1;
            __builtin_amdgcn_s_waitcnt(0xC07F);     // lgkmcnt(0): this step's operands, requested a step ago
            __builtin_amdgcn_sched_barrier(0);
            // The two contracting wavefronts of a SIMD (w and w + 4) share its matrix core.  Left
            // alone, the older one always wins the issue arbitration and the younger one's steps take
            // half as long again.  The younger one raises its issue priority for the part of the step
            // that feeds the matrix core and lowers it for the rest: the two then take turns
            // (measured on the whole kernel: 2843 -> 3025 GB/s; both wavefronts toggling between 1
            // and 0, either way round: 2950; a whole step at one priority, alternating: 2855; the level
            // it raises to matters little: 1, 2 and 3 within 0.6 %, 3 ahead).
            if (w >= kStream / 2) __builtin_amdgcn_s_setprio(3);
#pragma unroll
            for (int nb = 0; nb < 2; ++nb) {
                // the next step's requests go out between the two halves: the matrix core works on
                // the first half's products while the wavefront issues them
                if (nb == 1) {
                    __builtin_amdgcn_sched_barrier(0);
                    operands(on, nj, st + 1);
                    __builtin_amdgcn_sched_barrier(0);
                }
                const v4u t = oc.t[nb];
                const v4u t3 = {t[0] >> 1, t[1] >> 1, t[2] >> 1, t[3] >> 1};
                acc[nb][0] = __builtin_amdgcn_mfma_i32_16x16x64_i8(oc.x[0], masked(t, 0x03030303u), acc[nb][0], 0, 0, 0);
                acc[nb][1] = __builtin_amdgcn_mfma_i32_16x16x64_i8(oc.x[1], masked(t, 0x0C0C0C0Cu), acc[nb][1], 0, 0, 0);
                acc[nb][2] = __builtin_amdgcn_mfma_i32_16x16x64_i8(oc.x[2], masked(t, 0x30303030u), acc[nb][2], 0, 0, 0);
                acc[nb][3] = __builtin_amdgcn_mfma_i32_16x16x64_i8(oc.x[3], masked(t3, 0x60606060u), acc[nb][3], 0, 0, 0);
            }
            __builtin_amdgcn_s_setprio(0);
            cj = nj;
            if (nj == 0) {
                if (l < 16) {           // lanes 0..15 hold tokens 0..3 of weight rows l (nb 0) and 16 + l (nb 1)
#pragma unroll
                    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
                        for (int m = 0; m < kMaxFusedM; ++m)
                            if (m < p.M) {
                                const int sum = acc[nb][0][m] + (acc[nb][1][m] >> 2) + (acc[nb][2][m] >> 4) + (acc[nb][3][m] >> 5);
                                __hip_atomic_fetch_add(tiles + (ci * kMaxFusedM + m) * kTileRows + 16 * nb + l, sum, __ATOMIC_RELAXED,
                                                       __HIP_MEMORY_SCOPE_WORKGROUP);
                            }
                }
                // (LDS takes a wavefront's requests in order: the count follows the sums without a wait,
                //  which would be one for the operands just requested as well)
                if (l == 0) asm volatile("ds_add_u32 %0, %1" ::"v"(arrived_at + 4u * (unsigned)ci), "v"(1) : "memory");
                if (ci == 0) HGF_STAMP(w, ph, 4);
                if (ci == S.nunits - 1) HGF_STAMP(w, ph, 5);
                // the next unit starts from zero in the tokens' elements; the others are never read
#pragma unroll
                for (int nb = 0; nb < 2; ++nb)
#pragma unroll
                    for (int sh = 0; sh < 4; ++sh) acc[nb][sh][0] = 0;
                if (p.M > 1) {
#pragma unroll
                    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
                        for (int sh = 0; sh < 4; ++sh) acc[nb][sh][1] = acc[nb][sh][2] = acc[nb][sh][3] = 0;
                }
                ++ci;
            }
        };
        operands(o0, 0, 0);
        for (int st = 0; st < total; st += 2) {
            step(o0, o1, st);
            if (st + 1 < total) step(o1, o0, st + 1);
        }
        gs += 2 * total;

    }
    trace_flush(p, ctl, c, w);
}

// ------------------------------------------------------------------ slice and unit wavefronts
struct JobRegs {
    v8h a[kUN][2];
};
// Requests the rows of A for one batch of a slice: lane (i = l%16, kb = l/16) holds
// A[rt*16+i][k] for k = 64*kp + 16*kb + 0..7 and + 8..15.
__device__ __forceinline__ void job_load(JobRegs &r, const _Float16 *A, int rank, int K, int rt, int kpb, int kp1)
{
    const int l = threadIdx.x & 63, i = l & 15, kb = l >> 4;
    const int j = rt * 16 + i;
    const rsrc_t ar = make_rsrc(A, (unsigned)rank * K * 2u);
#pragma unroll
    for (int u = 0; u < kUN; ++u) {
        const int k0 = (kpb + u) * 64 + kb * 16;
        const bool ok = (kpb + u) < kp1 && j < rank;
        r.a[u][0] = buf_load8h<true>(ar, (unsigned)j * K + k0, K - k0, ok);
        r.a[u][1] = buf_load8h<true>(ar, (unsigned)j * K + k0 + 8, K - k0 - 8, ok);
    }
}
// The tokens' side of the same batch: 512 columns per token, one 16-byte piece per lane, read
// from the caller's slot or, once no word is the sentinel, from the exchange region (one
// request per token and try, so that a try costs little more than the memory's latency).
// The pieces are left in 1 KiB of LDS per token, from where the products read them in the
// operand layout: lane (i, kb) takes token i's 16 columns at 64*kp + 16*kb.
template <int MT>
__device__ __forceinline__ void job_xfetch(unsigned char *jxl, rsrc_t xr, bool ext, int M, int K, int kpb,
                                           int kp1, int mem_polls, bool &failed)
{
    const int l = threadIdx.x & 63;
    const int col = kpb * 64 + l * 8;
    const bool mine = kpb + (l >> 3) < kp1 && col < K;
    v4u v[MT];
    int polls = 0;
#pragma clang loop unroll(disable)
    while (true) {
        bool ready = true;
#pragma unroll
        for (int m = 0; m < MT; ++m) {
            v[m] = load16_agent(xr, (unsigned)(m * K + col) * 2u, mine && m < M);
            ready = ready && !has_sentinel(v[m]);
        }
        if (ext || failed || __builtin_amdgcn_ballot_w64(!ready) == 0) break;
        if (++polls >= mem_polls) {
            failed = true;
            break;
        }
        __builtin_amdgcn_s_sleep(1);
    }
#pragma unroll
    for (int m = 0; m < MT; ++m) *reinterpret_cast<v4u *>(jxl + m * 1024 + l * 16) = v[m];
}
// The products of one batch, the tokens' operands read from LDS half a batch at a time (the
// rows of A already fill half of the wavefront's registers).
__device__ __forceinline__ v4f job_mfma(const JobRegs &r, const unsigned char *jxl, int M, v4f acc)
{
    const int l = threadIdx.x & 63, i = l & 15, kb = l >> 4;
    const v4u zero = {0u, 0u, 0u, 0u};
    const unsigned char *row = jxl + i * 1024 + kb * 32;
#pragma unroll
    for (int u0 = 0; u0 < kUN; u0 += kUN / 2) {
        v4u b[kUN / 2][2];
#pragma unroll
        for (int u = 0; u < kUN / 2; ++u) {
            b[u][0] = i < M ? *reinterpret_cast<const v4u *>(row + (u0 + u) * 128) : zero;
            b[u][1] = i < M ? *reinterpret_cast<const v4u *>(row + (u0 + u) * 128 + 16) : zero;
        }
#pragma unroll
        for (int u = 0; u < kUN / 2; ++u) {
            acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(r.a[u0 + u][0], __builtin_bit_cast(v8h, b[u][0]), acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(r.a[u0 + u][1], __builtin_bit_cast(v8h, b[u][1]), acc, 0, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
    }
    return acc;
}

// Requests the epilogue operands of a unit into LDS (see hgf_fused.hip: B rows as 16-byte
// pieces in column-major order, then the 32 gate parameters).
__device__ __forceinline__ void stage_unit(const StackParams &p, const StackLayer &L, int n0, unsigned char *dst)
{
    const int l = threadIdx.x & 63, r = l & 31;
    if (L.rank == 0) return;
    const int hstride = h_stride(L.rank);
    const rsrc_t br = make_rsrc(L.B, (unsigned)L.N * L.rank * 2u);
    const rsrc_t ar = make_rsrc(L.alpha, ((unsigned)L.N * 2u + 3u) & ~3u);
    const int ninstr = hstride / 16;
    for (int k = 0; k < ninstr; ++k) {
        const int cp = 2 * k + (l >> 5);
        const bool ok = cp * 8 < L.rank && n0 + r < L.N;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(br, (lds_ptr_t)(dst + k * 1024), 16,
                                                 (int)(ok ? (unsigned)((n0 + r) * L.rank + cp * 8) * 2u : kOob), 0, 0, 0);
    }
    __builtin_amdgcn_raw_ptr_buffer_load_lds(ar, (lds_ptr_t)(dst + p.unit_alpha), 4,
                                             (int)(l < 16 && n0 + 2 * l < L.N ? (unsigned)(n0 * 2 + l * 4) : kOob), 0, 0, 0);
}

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

// unit of a phase -> (layer within the phase, first row)
__device__ __forceinline__ void unit_decode(const PhaseShape &S, int u, int &g, int &n0)
{
    g = 0;
    int first = 0;
    if (u >= S.us1) { g = 1; first = S.us1; }
    if (u >= S.us2) { g = 2; first = S.us2; }
    if (u >= S.us3) { g = 3; first = S.us3; }
    n0 = (u - first) * kTileRows;
}

// ---- the slice wavefront: its slices of A x (step 5), then SiLU of the sum of all slices
//      (step 6) into LDS for the unit wavefront
__device__ __forceinline__ void slice_wave(const StackParams &p, unsigned char *lds, Control *ctl, int c)
{
    const int l = threadIdx.x & 63;
    bool failed = false;
    const unsigned epoch = (unsigned)__hip_atomic_load(p.flags + 4, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const unsigned char *mine = p.xchg + (size_t)(epoch & 1u) * kStackSetBytes;
    const rsrc_t mail = make_rsrc(mine + kStackActBytes, (unsigned)(kStackSetBytes - kStackActBytes));
    unsigned char *jxl = lds + p.jx_off;

    // ---- the phase's slices of A x and the one this workgroup starts with.  The rows of A for
    //      it are requested a phase ahead, right after the previous phase's SiLU(A x): they come
    //      from HBM through queues the weight stream keeps full, and loads return in order, so
    //      requested just before the tokens they would hold the tokens back by microseconds.
    int pairs = 0, pps = 0, Sn = 0, rk0 = 0, rk1 = 0, rk2 = 0, rk3 = 0, hs0 = 32, hs1 = 32, hs2 = 32, hs3 = 32;
    int jb1 = 0, jb2 = 0, jb3 = 0, njobs = 0, jK = 0;
    unsigned mo0 = 0, mo1 = 0, mo2 = 0, mo3 = 0;
    int jfirst = 0;                     // (an index, not a pointer into the arguments: a pointer carried
    int job = 0;                        //  from phase to phase makes the compiler copy them to private memory)
    JobRegs jr;
    int g = 0, rt = 0, sp = 0, kp0 = 0, kp1 = 0, jrank = 0, jhs = 0;
    unsigned jmo = 0;
    const _Float16 *jA = nullptr;
    auto job_decode = [&]() __attribute__((always_inline)) {
        g = 0;
        int first = 0;
        jrank = rk0; jhs = hs0; jmo = mo0;
        if (job >= jb1) { g = 1; first = jb1; jrank = rk1; jhs = hs1; jmo = mo1; }
        if (job >= jb2) { g = 2; first = jb2; jrank = rk2; jhs = hs2; jmo = mo2; }
        if (job >= jb3) { g = 3; first = jb3; jrank = rk3; jhs = hs3; jmo = mo3; }
        jA = p.L[jfirst + g].A;
        rt = (job - first) / Sn;
        sp = (job - first) % Sn;
        kp0 = sp * pps;
        kp1 = min(kp0 + pps, pairs);
    };
    auto plan_phase = [&](int ph) __attribute__((always_inline)) {
        const StackPhase &P = p.ph[ph];
        jfirst = P.first_layer;
        const StackLayer *JL = p.L + jfirst;
        jK = P.K;
        // slices of 512 columns each, at most kSplit and 64 (slice, token) rows
        pairs = (jK + 63) / 64;
        int nsl = (pairs + 7) / 8;
        if (nsl > kSplit) nsl = kSplit;
        if (nsl > 64 / p.M) nsl = 64 / p.M;
        pps = (pairs + nsl - 1) / nsl;
        Sn = (pairs + pps - 1) / pps;
        rk0 = JL[0].rank;
        rk1 = P.G > 1 ? JL[1].rank : 0;
        rk2 = P.G > 2 ? JL[2].rank : 0;
        rk3 = P.G > 3 ? JL[3].rank : 0;
        hs0 = h_stride(rk0);
        hs1 = h_stride(rk1);
        hs2 = h_stride(rk2);
        hs3 = h_stride(rk3);
        jb1 = (rk0 + 15) / 16 * Sn;
        jb2 = jb1 + (rk1 + 15) / 16 * Sn;
        jb3 = jb2 + (rk2 + 15) / 16 * Sn;
        njobs = jb3 + (rk3 + 15) / 16 * Sn;
        // byte offsets of the layers' partial sums inside the phase's region: [slice][token][hstride] fp32
        mo0 = P.mail_off;
        mo1 = mo0 + (unsigned)(rk0 > 0 ? Sn * p.M * hs0 * 4 : 0);
        mo2 = mo1 + (unsigned)(rk1 > 0 ? Sn * p.M * hs1 * 4 : 0);
        mo3 = mo2 + (unsigned)(rk2 > 0 ? Sn * p.M * hs2 * 4 : 0);
        job = p.nwg - 1 - c;            // the highest workgroups, which own the fewest units, come first
        job_decode();                   // (without a branch: no job, no columns, and every request is void)
        job_load(jr, jA, jrank, jK, rt, kp0, job < njobs ? kp1 : kp0);
    };
    plan_phase(0);
    int gather_target = 0;

    for (int ph = 0; ph < p.nphases; ++ph) {
        const PhaseShape S = shape_of(p, ph, c);
        const StackPhase &P = p.ph[ph];
        _Float16 *hs = reinterpret_cast<_Float16 *>(lds + p.h_off + (ph & 1) * p.h_par);
        HGF_STAMP(kStream, ph, 0);

        // ---- my slices of A x (step 5): needs only the columns of the slice, so it starts as
        //      soon as the row-blocks of the previous layer that cover them have been stored
        const bool ext = P.x_ext != nullptr;
        const rsrc_t xr = make_rsrc(ext ? reinterpret_cast<const unsigned char *>(P.x_ext) : mine + P.src_off,
                                    (unsigned)p.M * S.K * 2u);
        while (job < njobs) {
            v4f acc = {0.f, 0.f, 0.f, 0.f};
            for (int kpb = kp0; kpb < kp1; kpb += kUN) {
                if (kpb > kp0) job_load(jr, jA, jrank, S.K, rt, kpb, kp1);
                if (p.M == 1) job_xfetch<1>(jxl, xr, ext, p.M, S.K, kpb, kp1, p.mem_polls, failed);
                else if (p.M == 2) job_xfetch<2>(jxl, xr, ext, p.M, S.K, kpb, kp1, p.mem_polls, failed);
                else job_xfetch<4>(jxl, xr, ext, p.M, S.K, kpb, kp1, p.mem_polls, failed);
                acc = job_mfma(jr, jxl, p.M, acc);
                HGF_STAMP(kStream, ph, 3);
            }
            // acc[v]: rank index rt*16 + 4*kb + v of token i  ->  [sp][i][hstride] of the layer
            const int i = l & 15, kb = l >> 4;
            store16_agent(mail, i < p.M ? jmo + (unsigned)(((sp * p.M + i) * jhs + rt * 16 + 4 * kb) * 4) : kOob,
                          __builtin_bit_cast(v4u, acc));
            job += p.nwg;
            if (job < njobs) {
                job_decode();
                job_load(jr, jA, jrank, S.K, rt, kp0, kp1);
            }
        }

        HGF_STAMP(kStream, ph, 1);
        if (S.nunits > 0) {
            // this parity's rows were last read by the unit wavefront two phases ago
            int spins = 0;
#pragma clang loop unroll(disable)
            while (!failed && !units_done(ctl, ph - 1)) {
                if (++spins >= p.lds_polls) failed = true;
                __builtin_amdgcn_s_sleep(1);
            }
            // the other workgroups' slices cannot be there before the tokens are, and their lines are
            // polled by every workgroup: hold the polls until this workgroup's contracting
            // wavefronts have all of their tokens (measured: 3120 -> 3240 GB/s)
            gather_target += kStream;
            spins = 0;
#pragma clang loop unroll(disable)
            while (!failed && lds_load(&ctl->sync) < gather_target) {
                if (++spins >= p.lds_polls) failed = true;
                __builtin_amdgcn_s_sleep(1);
            }
            // ---- collect every slice: h[g][m][j] = SiLU(sum_sp partial) (step 6); a lane takes four
            //      consecutive ranks of one (layer, token); one batch of loads usually covers all
            const int ge0 = rk0 > 0 ? p.M * hs0 / 4 : 0;
            const int ge1 = ge0 + (rk1 > 0 ? p.M * hs1 / 4 : 0);
            const int ge2 = ge1 + (rk2 > 0 ? p.M * hs2 / 4 : 0);
            const int ge3 = ge2 + (rk3 > 0 ? p.M * hs3 / 4 : 0);
            // With few sums to collect, 2 or 4 lanes share one and take every 2nd or 4th slice each,
            // so that more slices fit one batch of requests (a batch costs a trip to memory).
            const int Q = ge3 <= 16 ? 4 : (ge3 <= 32 ? 2 : 1);
            const int fl = 64 / Q, q = l / fl;
            for (int f0 = 0; f0 < ge3; f0 += fl) {
                const int f = f0 + (l & (fl - 1));
                // per-lane layer: arithmetic on the comparison results (a chain of selects between
                // these scalars gets turned into a table in private memory)
                const int b0 = f >= ge0, b1 = f >= ge1, b2 = f >= ge2;
                const int gg = b0 + b1 + b2;
                const int first = b0 * ge0 + b1 * (ge1 - ge0) + b2 * (ge2 - ge1);
                const int rank = rk0 + b0 * (rk1 - rk0) + b1 * (rk2 - rk1) + b2 * (rk3 - rk2);
                const int hstride = hs0 + b0 * (hs1 - hs0) + b1 * (hs2 - hs1) + b2 * (hs3 - hs2);
                const unsigned mo = mo0 + (unsigned)b0 * (mo1 - mo0) + (unsigned)b1 * (mo2 - mo1) + (unsigned)b2 * (mo3 - mo2);
                const bool inside = f < ge3;
                const int idx = f - first;
                const int j = (idx * 4) % hstride;
                const bool wanted = inside && j < (rank + 15) / 16 * 16;
                const unsigned at = mo + (unsigned)idx * 16u;
                const unsigned step = (unsigned)p.M * hstride * 4u;
                v4f h = {0.f, 0.f, 0.f, 0.f};
                // the slices of the lane's four sums, eight to a batch of requests (a try costs as
                // many requests and comparisons as the batch is long); each lane adds its slices in
                // order, then the lanes that share a sum add theirs
                for (int sb = 0; sb < Sn; sb += 8 * Q) {
                    const int s0 = sb + q;
                    v4f part[8];
                    int polls = 0;
#pragma clang loop unroll(disable)
                    while (true) {
                        bool ready = true;
#pragma unroll
                        for (int sl = 0; sl < 8; ++sl) {
                            const v4u raw = load16_agent(mail, at + (unsigned)(s0 + sl * Q) * step, wanted && s0 + sl * Q < Sn);
                            ready = ready && !has_sentinel(raw);
                            part[sl] = __builtin_bit_cast(v4f, raw);
                        }
                        if (failed || __builtin_amdgcn_ballot_w64(!ready) == 0) break;
                        if (++polls >= p.mem_polls) {
                            failed = true;
                            break;
                        }
                        __builtin_amdgcn_s_sleep(1);
                    }
#pragma unroll
                    for (int sl = 0; sl < 8; ++sl) h += part[sl];   // (slices past the last one were read as zero)
                }
                if (Q > 1) {
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        h[v] += __shfl_xor(h[v], 32, 64);
                        if (Q > 2) h[v] += __shfl_xor(h[v], 16, 64);
                    }
                }
                if (inside && q == 0) {
                    v4h o;
#pragma unroll
                    for (int v = 0; v < 4; ++v) o[v] = (j + v < rank) ? (_Float16)silu_fast(h[v]) : (_Float16)0.0f;
                    *reinterpret_cast<v4h *>(hs + (gg * p.M + idx * 4 / hstride) * kHsStride + j) = o;
                }
            }

        }
        if (failed && l == 0) {
            __hip_atomic_store(&ctl->failed, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            __hip_atomic_store(p.flags + 2, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        if (l == 0) __hip_atomic_store(&ctl->h_ready, ph + 1, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
        HGF_STAMP(kStream, ph, 2);
        if (ph + 1 < p.nphases) plan_phase(ph + 1);
    }
    trace_flush(p, ctl, c, kStream);
}

// ---- the unit wavefront: finishes the row-blocks this workgroup owns (steps 4, 7, 8) and
//      hands their outputs on
__device__ __forceinline__ void unit_wave(const StackParams &p, unsigned char *lds, Control *ctl, int c, int uw)
{
    const int l = threadIdx.x & 63, jl = l & 31, hf = l >> 5;
    bool failed = false;

    // ---- which set of exchange regions this launch uses; what the previous launch used in the other
    const unsigned epoch = (unsigned)__hip_atomic_load(p.flags + 4, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const unsigned prev_act = (unsigned)__hip_atomic_load(p.flags + 6, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const unsigned prev_mail = (unsigned)__hip_atomic_load(p.flags + 7, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    unsigned char *mine = p.xchg + (size_t)(epoch & 1u) * kStackSetBytes;
    unsigned char *other = p.xchg + (size_t)((epoch & 1u) ^ 1u) * kStackSetBytes;
    const rsrc_t act = make_rsrc(mine, (unsigned)kStackActBytes);

    unsigned char *ustage = lds + p.unit_off;
    int *tiles_all = reinterpret_cast<int *>(lds + p.tile_off);

    for (int ph = 0; ph < p.nphases; ++ph) {
        const PhaseShape S = shape_of(p, ph, c);
        const StackLayer *L = p.L + S.first;
        const int par = ph & 1;
        int *tiles = tiles_all + par * p.tile_par;
        const _Float16 *hs = reinterpret_cast<const _Float16 *>(lds + p.h_off + par * p.h_par);

        HGF_STAMP(kStream + 1, ph, 0);
        // ---- requests that do not depend on the tokens: epilogue operands of my units
        //      (LDS-direct) and the weight scales
        for (int i = uw; i < S.nunits; i += kUnitWaves) {
            int g2, n0;
            unit_decode(S, c + i * p.nwg, g2, n0);
            stage_unit(p, L[g2], n0, ustage + i * p.unit_stride);
        }
        const unsigned swb0 = buf_load4(make_rsrc(L[0].s_w, 4u), 0u);
        const unsigned swb1 = buf_load4(make_rsrc(S.G > 1 ? L[1].s_w : nullptr, S.G > 1 ? 4u : 0u), 0u);
        const unsigned swb2 = buf_load4(make_rsrc(S.G > 2 ? L[2].s_w : nullptr, S.G > 2 ? 4u : 0u), 0u);
        const unsigned swb3 = buf_load4(make_rsrc(S.G > 3 ? L[3].s_w : nullptr, S.G > 3 ? 4u : 0u), 0u);
        const int hs0 = h_stride(L[0].rank), hs1 = h_stride(S.G > 1 ? L[1].rank : 0),
                  hs2 = h_stride(S.G > 2 ? L[2].rank : 0), hs3 = h_stride(S.G > 3 ? L[3].rank : 0);

        if (S.nunits > uw) {
            // ---- SiLU(A x) of the phase is in LDS once the slice wavefront says so
            int spins = 0;
#pragma clang loop unroll(disable)
            while (!failed && lds_load(&ctl->h_ready) < ph + 1) {
                if (++spins >= p.lds_polls) failed = true;
                __builtin_amdgcn_s_sleep(1);
            }
            HGF_STAMP(kStream + 1, ph, 1);
            // ---- per unit: lane n < 32 owns output row n of the unit for every token
            int rs[kMaxFusedM] = {0, 0, 0, 0};
            float sxv[kMaxFusedM] = {0.f, 0.f, 0.f, 0.f};
            for (int i = uw; i < S.nunits; i += kUnitWaves) {
                const unsigned char *op = ustage + i * p.unit_stride;
                int gg, n0;
                unit_decode(S, c + i * p.nwg, gg, n0);
                const StackLayer &Lg = L[gg];
                const unsigned swb = gg == 0 ? swb0 : (gg == 1 ? swb1 : (gg == 2 ? swb2 : swb3));
                const int hstride = gg == 0 ? hs0 : (gg == 1 ? hs1 : (gg == 2 ? hs2 : hs3));
                // the correction term needs only SiLU(A x) and the staged operands: it is computed
                // before the wait for the contraction, so that after the last unit's contraction
                // only the sums, one multiply-add per output and the stores remain
                v16f corr = (v16f){};
                float gate = 0.f;
                if (Lg.rank > 0) {
                    gate = tanh_fast((float)*reinterpret_cast<const _Float16 *>(op + p.unit_alpha + jl * 2));
                    const _Float16 *hrow = hs + (gg * p.M + jl) * kHsStride + hf * 8;
                    const unsigned char *brow = op + (hf * 32 + jl) * 16;
                    switch (hstride / 16) {
                        case 2: corr = corr_unit<2>(hrow, brow, jl < p.M); break;
                        case 4: corr = corr_unit<4>(hrow, brow, jl < p.M); break;
                        default: corr = corr_unit<8>(hrow, brow, jl < p.M); break;
                    }
                }
                if (i == 0) HGF_STAMP(kStream + 1, ph, 5);
                int polls = 0;
#pragma clang loop unroll(disable)
                while (!failed && lds_load(&ctl->arrived[par][i]) < kStream) {
                    if (++polls >= p.lds_polls) {
                        failed = true;
                        break;
                    }
                    __builtin_amdgcn_s_sleep(1);
                }
                if (i == 0) HGF_STAMP(kStream + 1, ph, 2);
                if (i == S.nunits - 1) HGF_STAMP(kStream + 1, ph, 3);
                // the unit's sums (and whether a wait of another wavefront has expired), then this
                // parity's words are ready for the phase after next
                const int others_failed = __hip_atomic_load(&ctl->failed, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                int a[kMaxFusedM];
#pragma unroll
                for (int m = 0; m < kMaxFusedM; ++m) a[m] = tiles[(i * kMaxFusedM + m) * kTileRows + jl];
                if (others_failed != 0) failed = true;
                if (i == uw) {          // every contracting wavefront has posted: so are the tokens' sums and scales
#pragma unroll
                    for (int m = 0; m < kMaxFusedM; ++m) {
                        rs[m] = 0;
#pragma unroll
                        for (int ww = 0; ww < kStream; ++ww) rs[m] += ctl->rowsum_part[par][ww][m];
                        sxv[m] = ctl->sx[par][m];
                    }
                }
#pragma unroll
                for (int m = 0; m < kMaxFusedM; ++m)
                    if (l < 32) tiles[(i * kMaxFusedM + m) * kTileRows + l] = 0;
                if (l == 0) ctl->arrived[par][i] = 0;
                const int n = n0 + l;
                const float s_w = __builtin_bit_cast(float, swb);
                const int Npad = (Lg.N + 7) & ~7;         // row pitch of the exchange copy (16-byte rows)
#pragma unroll
                for (int m = 0; m < kMaxFusedM; ++m) {
                    if (m < p.M) {
                        _Float16 o = (_Float16)((float)(a[m] - rs[m]) * (sxv[m] * s_w) + gate * corr[m]);
                        if (o != o || failed) o = __builtin_bit_cast(_Float16, (unsigned short)0x7e00);
                        if (l < 32 && n < Lg.N) Lg.y[(size_t)m * Lg.N + n] = o;
                        // exchange copy: 32 lanes x 2 bytes gathered into 16 lanes x 4 bytes, padding
                        // columns written as zero so that no sentinel remains in the row
                        const unsigned lo = (unsigned)__builtin_bit_cast(unsigned short, o);
                        const unsigned nb = (unsigned)dpp_move<0xB1>((int)lo);   // (lane l ^ 1: the right neighbour of an even lane)
                        const unsigned pairw = (n < Lg.N ? lo : 0u) | ((n + 1 < Lg.N ? nb : 0u) << 16);
                        const bool writer = l < 32 && (l & 1) == 0 && n < Npad;
                        __builtin_amdgcn_raw_buffer_store_b32(pairw, act,
                                                              (int)(writer ? Lg.act_off + (unsigned)(m * Npad + n) * 2u : kOob), 0, 16);
                    }
                }
            }
        }
        HGF_STAMP(kStream + 1, ph, 4);
        // the other wavefronts may now reuse this parity's words (two phases from here)
        if (l == 0) __hip_atomic_store(&ctl->svc_done[uw], ph + 1, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);

        // ---- my share of the sentinels for the launch after this one (once, in the first phase)
        if (ph == 0 && uw == 0) {
            const rsrc_t oa = make_rsrc(other, prev_act);
            const rsrc_t om = make_rsrc(other + kStackActBytes, prev_mail);
            const v4u s4 = {kSentinel, kSentinel, kSentinel, kSentinel};
            for (unsigned v = (unsigned)c * 64u + l; v < (prev_act + 15u) / 16u; v += (unsigned)p.nwg * 64u)
                store16_agent(oa, v * 16u, s4);
            for (unsigned v = (unsigned)c * 64u + l; v < (prev_mail + 15u) / 16u; v += (unsigned)p.nwg * 64u)
                store16_agent(om, v * 16u, s4);
        }
    }

    if (failed && l == 0) __hip_atomic_store(p.flags + 2, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (uw != 0) return;
    // (the stamps of all unit wavefronts: the others finish their last phase no later than a few polls from here)
    trace_flush(p, ctl, c, kStream + 1);
    // ---- the last workgroup to get here advances the launch counter and records what was used
    if (l == 0) {
        const int done = __hip_atomic_fetch_add(p.flags + 5, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (done == p.nwg - 1) {
            __hip_atomic_store(p.flags + 5, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(p.flags + 6, (int)p.act_used, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(p.flags + 7, (int)p.mail_used, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(p.flags + 4, (int)(epoch + 1u), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

// The launch description travels by value in the kernel arguments.  (Behind a pointer to
// device memory every field costs a scalar load from memory, which measured 12 % slower; but
// watch the code object when changing this kernel: indexing the arguments at run-time
// offsets can make the compiler copy all 4 KiB of them into private memory -- it does with
// a ring of more than 8 tiles -- and the kernel then crawls.)
__global__ __launch_bounds__(64 * kWaves) void stack_kernel(const StackParams p)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    __shared__ Control ctl;
    const int c = blockIdx.x;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // everything the roles add into or count with starts at zero; afterwards the unit
    // wavefront resets what it has consumed
    int *tiles = reinterpret_cast<int *>(lds + p.tile_off);
    for (int e = threadIdx.x; e < 2 * p.tile_par; e += 64 * kWaves) tiles[e] = 0;
    for (int e = threadIdx.x; e < (int)(sizeof(Control) / sizeof(int)); e += 64 * kWaves) reinterpret_cast<int *>(&ctl)[e] = 0;
    if (threadIdx.x < 32) reinterpret_cast<int *>(lds + p.jx_off + kMaxFusedM * 1024)[threadIdx.x] = 0;
    __syncthreads();
    if (w < kStream) {
        contract_wave(p, lds, &ctl, c);
    } else if (w < kStream + kLoaders) {
        __builtin_amdgcn_s_setprio(3);
        loader_wave(p, lds, &ctl, c, w - kStream);
    } else {
        // the two serving wavefronts share their SIMDs with contracting ones and are the ones
        // every other workgroup waits for: they issue first
        if (w == kStream + kLoaders) {
            __builtin_amdgcn_s_setprio(3);
            slice_wave(p, lds, &ctl, c);
        } else {
            __builtin_amdgcn_s_setprio(3);
            unit_wave(p, lds, &ctl, c, w - (kStream + kLoaders + 1));
        }
    }
}

int g_num_cus = 0, g_device = -1;
int g_wait_limit = 0;                  // 0: the default bounds
unsigned long long *g_trace = nullptr; // time-stamp buffer of the measurement aid (null: off)
size_t g_trace_bytes = 0;
int g_trace_ph0 = 0;
constexpr size_t kStackLdsMax = 156 * 1024;   // (the compute unit has 160 KiB; the control words are static)
static_assert(sizeof(Control) <= 160 * 1024 - kStackLdsMax, "the control words must fit beside the dynamic part");

}  // namespace

// Plans one launch over `n` phases starting at `phases[0]`.  The caller has filled M, the
// phases (x_ext/src_off, K, first_layer, G) and the layers (pointers, N, rank); this fills
// the exchange offsets, the launch shape and the LDS layout.  False: does not fit this path.
bool plan_stack(StackParams &p, size_t *lds_bytes)
{
    // The workgroups of this kernel wait for each other, so all of them must be resident at
    // once: the launch is sized to what the occupancy query says one compute unit holds of this
    // kernel at its largest LDS request, times the compute units (asked once per device).
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) {
        (void)hipGetLastError();
        return false;
    }
    if (g_num_cus == 0 || dev != g_device) {
        int n = 0, per_cu = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
            hipFuncSetAttribute(reinterpret_cast<const void *>(stack_kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)kStackLdsMax) != hipSuccess ||
            hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, stack_kernel, 64 * kWaves, kStackLdsMax) !=
                hipSuccess ||
            per_cu < 1) {
            (void)hipGetLastError();
            return false;
        }
        g_num_cus = n > 0 ? n : 1;              // (one workgroup per compute unit even where two would fit:
        g_device = dev;                         //  a workgroup is sized to use a whole unit's LDS)
    }
    p.trace = nullptr;
    p.trace_ph0 = g_trace_ph0;
    p.mem_polls = g_wait_limit > 0 ? g_wait_limit : kMemPollsDefault;
    p.lds_polls = g_wait_limit > 0 ? g_wait_limit : kLdsPollsDefault;
    const int M = p.M;
    int kmax = 0, units_max = 0, jobs_max = 0, hstride_max = 32, gmax = 1;
    size_t mail = 0;
    for (int ph = 0; ph < p.nphases; ++ph) {
        StackPhase &P = p.ph[ph];
        if (P.K > kmax) kmax = P.K;
        if (P.G > gmax) gmax = P.G;
        const int pairs = (P.K + 63) / 64;
        int nsl = (pairs + 7) / 8;
        if (nsl > kSplit) nsl = kSplit;
        if (nsl > 64 / M) nsl = 64 / M;
        const int pps = (pairs + nsl - 1) / nsl;
        const int Sn = (pairs + pps - 1) / pps;
        int units = 0, jobs = 0;
        P.mail_off = (unsigned)mail;
        for (int g = 0; g < P.G; ++g) {
            const StackLayer &L = p.L[P.first_layer + g];
            units += (L.N + kTileRows - 1) / kTileRows;
            if (L.rank > 0) {
                const int hs = h_stride(L.rank);
                if (hs > hstride_max) hstride_max = hs;
                jobs += (L.rank + 15) / 16 * Sn;
                mail += (size_t)Sn * M * hs * 4;
            }
        }
        if (units > units_max) units_max = units;
        if (jobs > jobs_max) jobs_max = jobs;
    }
    if (mail > kStackSetBytes - kStackActBytes) return false;
    p.mail_used = (unsigned)mail;
    int nwg = units_max > jobs_max ? units_max : jobs_max;
    if (nwg > g_num_cus) nwg = g_num_cus;
    p.nwg = nwg;
    const int per_wg = (units_max + nwg - 1) / nwg;
    if (per_wg > kMaxUnits) return false;
    if (g_trace && g_trace_bytes >= (size_t)nwg * kTraceRoles * kTracePhases * kTraceIds * sizeof(unsigned long long))
        p.trace = g_trace;

    const int kp = round_up(kmax, kTileCols);
    p.xstride = kp + 16;
    size_t off = ((size_t)M * p.xstride + 15) & ~size_t(15);     // quantised tokens at offset 0
    p.tile_off = (int)off;
    p.tile_par = per_wg * kMaxFusedM * kTileRows;                 // the units' [token][row] sums, per phase parity
    off += (size_t)2 * p.tile_par * sizeof(int);
    p.h_off = (int)off;                                           // one set of rows per phase parity
    p.h_par = (int)((size_t)gmax * M * kHsStride * sizeof(_Float16));
    off += (size_t)2 * p.h_par;
    off = (off + 1023) & ~size_t(1023);
    p.jx_off = (int)off;                                          // the slice wavefront's pieces of the tokens
    off += (size_t)kMaxFusedM * 1024 + 1024;                      // ... and 128 bytes of zeros (kept 1 KiB aligned)
    p.unit_off = (int)off;
    p.unit_alpha = 64 * hstride_max;
    p.unit_stride = p.unit_alpha + 256;
    off += (size_t)per_wg * p.unit_stride;
    // the rest holds the rings of weight tiles: the deeper, the longer the loaders keep the
    // memory busy while a phase waits for its tokens
    if (off + (size_t)kStream * kMinRing * kTileBytes > kStackLdsMax) return false;
    int slots = (int)((kStackLdsMax - off) / ((size_t)kStream * kTileBytes));
    if (slots > kMaxRing) slots = kMaxRing;
    slots &= ~1;                                                  // the contraction takes the tiles in pairs
    p.ring_off = (int)off;
    p.ring_slots = slots;
    off += (size_t)kStream * slots * kTileBytes;
    *lds_bytes = off;
    return true;
}

void set_stack_wait_limit(int tries) { g_wait_limit = tries > 0 ? tries : 0; }

void set_stack_trace(unsigned long long *buf, size_t bytes, int first_phase)
{
    g_trace = buf;
    g_trace_bytes = buf ? bytes : 0;
    g_trace_ph0 = first_phase > 0 ? first_phase : 0;
}

hipError_t launch_stack(const StackParams &p, size_t lds_bytes, hipStream_t st)
{
    hipLaunchKernelGGL(stack_kernel, dim3(p.nwg), dim3(64 * kWaves), lds_bytes, st, p);
    return hipGetLastError();
}

}  // namespace hgf

