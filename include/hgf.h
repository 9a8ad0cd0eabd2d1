/*
 * hgf.h -- C ABI of the MI355X (gfx950) HGF linear-layer library.
 *
 * The library computes the inference forward pass of one Hybrid Gated Flow linear
 * layer (Algorithm 1, "HGF 1.0 Forward Pass, Inference Mode"):
 *
 *     y[m, n] = s_x[m] * s_w * sum_k T[n, k] * x_q[m, k]
 *             + tanh(alpha[n]) * sum_j B[n, j] * SiLU( sum_k A[j, k] * x[m, k] )
 *
 * with T in {-1, 0, +1} the absmean-ternarised weights (2 bits each, packed),
 * x_q the per-token absmax int8 quantisation of the fp16 activations x, and A, B,
 * alpha the fp16 low-rank correction path and its gate.
 *
 * Conventions for every entry point
 *   - Every data pointer is a DEVICE pointer owned by the caller unless it is
 *     marked "host".  The library never allocates, frees or keeps a pointer (the one
 *     exception, a measurement aid that is no part of the layer, says so where it is declared).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  A call
 *     only enqueues kernels on that stream: no synchronisation, no host read-back.
 *   - Arguments are validated on the host before anything is enqueued; on error
 *     nothing has been launched and a non-zero hgf_status is returned.
 *   - Matrices are row-major.  fp16 tensors are IEEE binary16, passed as void*.
 *   - Limits: 1 <= d_in, d_out <= 65536; rank in {0} u [1, 128]; M >= 1 with
 *     M * max(d_in, d_out) < 2^31; packed weights, x_q, x and y 16-byte aligned.
 */
#ifndef HGF_H
#define HGF_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    HGF_OK = 0,
    HGF_ERR_NULL = 1,        /* a required pointer is NULL                          */
    HGF_ERR_SHAPE = 2,       /* a dimension is out of the supported range           */
    HGF_ERR_ALIGN = 3,       /* a buffer is not 16-byte aligned                     */
    HGF_ERR_UNSUPPORTED = 4, /* valid request this build does not implement         */
    HGF_ERR_WORKSPACE = 5,   /* workspace missing or smaller than hgf_workspace_bytes */
    HGF_ERR_DEVICE = 6       /* the HIP runtime refused a launch                    */
} hgf_status;

#define HGF_MAX_RANK 128
#define HGF_MAX_DIM 65536

/* Human-readable name of a status code (static storage, host). */
const char *hgf_status_string(int status);
/* Library version, major*10000 + minor*100 + patch. */
int hgf_version(void);

/* ---------------------------------------------------------------- sizes (host only) */

/* d_in rounded up to the packing granule (128).  Rows of x_q have this many bytes;
 * the padding bytes are written as 0 by hgf_quantize_activations. */
int hgf_padded_k(int d_in);
/* Bytes of the packed 2-bit weight buffer of a [d_out, d_in] matrix (d_out padded to
 * 32, d_in to 128; padding decodes to 0).  0 on invalid sizes. */
size_t hgf_packed_weight_bytes(int d_out, int d_in);
/* Bytes of workspace that any call with M <= M_max, d_in <= d_in_max,
 * d_out <= d_out_max, rank <= rank_max needs.  0 on invalid sizes. */
size_t hgf_workspace_bytes(int M_max, int d_in_max, int d_out_max, int rank_max);

/* Prepares a workspace.  Must be called once (and again after any call that returned
 * HGF_ERR_DEVICE) before the workspace is used: the few-token path keeps a launch counter, an
 * arrival count and a sticky error word at the start of the workspace (zeroed here) and two
 * exchange buffers that hold a sentinel bit pattern between launches (filled here).  The
 * error word (int32 at byte offset 8) becomes nonzero if a bounded in-kernel wait ever runs
 * out; the outputs of that launch are then NaN.  A workspace serves one call at a time:
 * calls that share one must be ordered on a single stream. */
hgf_status hgf_workspace_init(void *workspace, size_t workspace_bytes, void *stream);

/* ---------------------------------------------------------------- weights (offline)
 *
 * Absmean ternarisation (Sec. 2.2, weight-quantisation definition; the paper's own
 * implementation fixes the details): gamma_W = max(mean |W|, 1e-5), the mean taken in
 * fp64 and rounded once to fp32; T = clip(round_half_even(W * (1/gamma_W)), -1, 1) in
 * fp32.  Writes the packed codes and the scalar s_w = gamma_W.
 *
 *   W          fp32 [d_out, d_in]
 *   packed_out hgf_packed_weight_bytes(d_out, d_in) bytes
 *   s_w_out    one fp32
 *
 * Packed layout: tiles of 32 rows x 128 columns, 1 KiB each, ordered row-block major
 * then along d_in, so one row-block's tiles are contiguous and a wavefront reads a tile
 * with one 16-byte load per lane.  Within a tile, bytes 16*l + 4*t .. +3 (l = 0..63,
 * t = 0..3) are a little-endian 32-bit word holding the 16 codes of row (l mod 32),
 * columns 32*t + 16*(l div 32) + 0..15; column offset 4*s + b sits at bits
 * [8*b + 2*s, 8*b + 2*s + 1] (so a shift by 2*s and a mask give the four int8 of one
 * register of a 32x32x32 int8 MFMA operand).  A code is T + 1 (0, 1 or 2; 3 never
 * occurs); padding rows and columns hold code 1.
 */
hgf_status hgf_quantize_pack_weights(const float *W, int d_out, int d_in, void *packed_out,
                                     float *s_w_out, void *workspace, size_t workspace_bytes,
                                     void *stream);

/* Inverse of the packed layout: T_out int8 [d_out, d_in] with values -1, 0, +1. */
hgf_status hgf_unpack_weights(const void *packed, int d_out, int d_in, int8_t *T_out,
                              void *stream);

/* ---------------------------------------------------------------- activations
 *
 * Per-token absmax int8 quantisation (Sec. 2.2.1; Algorithm 1, steps 1-2):
 * amax = max(max_k |x[m, k]|, 1e-5); x_q = clip(round_half_even(x * (127/amax)), -127,
 * 127) in fp32; s_x[m] = amax / 127.
 *
 *   x_f16      fp16 [M, d_in]
 *   xq_out     int8 [M, hgf_padded_k(d_in)]   (padding columns = 0)
 *   s_x_out    fp32 [M]
 *   rowsum_out int32 [M] = sum_k x_q[m, k]; may be NULL
 */
hgf_status hgf_quantize_activations(const void *x_f16, int M, int d_in, int8_t *xq_out,
                                    float *s_x_out, int32_t *rowsum_out, void *stream);

/* The same quantiser behind a LayerNorm, fused (appendix implementation, BitLinear forward):
 * v = ((x - mu) * rstd) * gamma + beta with mu = mean_k x and rstd = 1/sqrt(mean_k (x-mu)^2 + eps),
 * the two reductions in fp64 rounded once to fp32, the elementwise part in fp32 in the order
 * written; then amax, x_q, s_x and rowsum of v exactly as above.  The normalised row is never
 * stored.  ln_gamma fp32 [d_in]; ln_beta fp32 [d_in] or NULL (zero). */
hgf_status hgf_layernorm_quantize_activations(const void *x_f16, int M, int d_in, const float *ln_gamma,
                                              const float *ln_beta, float ln_eps, int8_t *xq_out,
                                              float *s_x_out, int32_t *rowsum_out, void *stream);

/* ---------------------------------------------------------------- one layer */

typedef struct {
    int d_in, d_out;
    int rank;               /* 0: no correction path (A, B, alpha ignored): a pure ternary layer */
    const void *W_packed;   /* from hgf_quantize_pack_weights                                     */
    const float *s_w;       /* device scalar gamma_W                                              */
    const void *A_f16;      /* fp16 [rank, d_in]   down-projection                                */
    const void *B_f16;      /* fp16 [d_out, rank]  up-projection                                  */
    const void *alpha_f16;  /* fp16 [d_out]        gate parameter, g = tanh(alpha)                */
    int src_slot, dst_slot; /* used only by hgf_stack_forward                                     */
    /* Optional LayerNorm in front of the backbone's quantiser (appendix implementation, BitLinear
     * forward: the ternary path quantises layernorm(x) while the correction path reads x itself).
     * ln_gamma == NULL: none (Algorithm 1 as printed).  Otherwise fp32 [d_in] scale and shift
     * (ln_beta may be NULL: zero) and the epsilon added to the variance. */
    const float *ln_gamma;
    const float *ln_beta;
    float ln_eps;
} hgf_layer;

/* Algorithm 1, steps 1-8, for one layer.
 *
 *   x_f16     fp16 [M, d_in]
 *   L         host pointer to the layer description (its pointers are device pointers)
 *   y_f16     fp16 [M, d_out], written
 *   acc_debug int32 [M, d_out] or NULL: receives the exact integer accumulators
 *             sum_k T[n,k] x_q[m,k] of step 3 (for parity tests)
 *
 * M <= 40 (and up to 64 for layers of few rows) runs the bandwidth-bound decode kernels (weights streamed once); larger M
 * runs the int8 MFMA prefill kernel.  Both give the same integers.  A layer with ln_gamma set
 * takes the fused LayerNorm quantiser as its prologue (one more launch than a layer without;
 * layers with a LayerNorm of their own never share a quantisation in hgf_stack_forward). */
hgf_status hgf_linear_forward(const void *x_f16, int M, const hgf_layer *L, void *y_f16,
                              int32_t *acc_debug, void *workspace, size_t workspace_bytes,
                              void *stream);

/* The gated pair of the paper's MLP (appendix implementation, block forward:
 * x + w3(SiLU(w1(n2 x)) * w2(n2 x)); w1, w2, w3 are HGF linears): both projections of one input
 * and their product in one pass,
 *
 *     z[m, n] = SiLU(y_gate[m, n]) * y_up[m, n],      SiLU(v) = v * sigmoid(v),
 *
 * with y_gate and y_up the outputs of Algorithm 1 for the layers `gate` (w1) and `up` (w2) on
 * the same x: one activation quantisation serves both, each workgroup contracts the same rows of
 * both weight matrices, and the two fp32 results meet in registers or LDS -- neither y is
 * rounded to fp16 or written to memory; z is rounded to fp16 once.  z is the input of the
 * down projection (w3), an ordinary hgf_linear_forward.
 *
 *   x_f16           fp16 [M, d_in]
 *   gate, up        host pointers; same d_in and d_out; ranks may differ (for M > 40 they must
 *                   pad to the same multiple-of-32 width, else HGF_ERR_UNSUPPORTED)
 *   z_f16           fp16 [M, d_out], written
 *   amax_out        fp32 [M] or NULL: per-token max_n |z[m, n]| of the stored fp16 values -- the
 *                   gamma_x of Algorithm 1 step 1 for the layer that reads z
 *   acc_debug_gate, acc_debug_up   int32 [M, d_out] or NULL: the exact accumulators of step 3
 */
hgf_status hgf_swiglu_forward(const void *x_f16, int M, const hgf_layer *gate, const hgf_layer *up,
                              void *z_f16, float *amax_out, int32_t *acc_debug_gate,
                              int32_t *acc_debug_up, void *workspace, size_t workspace_bytes,
                              void *stream);

/* ---------------------------------------------------------------- differential attention, one decode step
 *
 * The block that consumes the q, k, v projections (Sec. 2.4, Def. "Differential Attention"):
 *     O = (softmax(Q1 K1^T / sqrt(d_h)) - lambda * softmax(Q2 K2^T / sqrt(d_h))) V,
 * with the details the appendix implementation fixes: q and k hold 2 n_heads heads of d_h columns
 * (heads 0 .. n_heads-1 are branch 1, the rest branch 2), v holds n_heads heads of d_h columns
 * (V: d -> d/2), head h of both branches reads head h of v, and the difference is multiplied by 0.5.
 * One decode step: for each sequence b the newest token's q attends to the cached positions
 * 0 .. lens[b]-1 (its own k and v already appended by the caller).
 *
 *   q_f16        fp16 [B, 2 n_heads, d_h]
 *   k_cache_f16  fp16 [B, L_max, 2 n_heads, d_h]      v_cache_f16  fp16 [B, L_max, n_heads, d_h]
 *   lens         int32 [B] (device), 1 <= lens[b] <= L_max (0: that sequence's output is zero)
 *   lambda       the scalar of the definition (its initial value there: 0.8 - 0.6 exp(-0.3 d))
 *   out_f16      fp16 [B, n_heads, d_h], written
 *   workspace    hgf_diff_attention_workspace_bytes(B, L_max, n_heads, d_h) bytes, 16-byte aligned
 * d_h a power of two in 8 .. 128.  fp32 arithmetic; the caches are read once. */
size_t hgf_diff_attention_workspace_bytes(int B, int L_max, int n_heads, int d_h);
hgf_status hgf_diff_attention_decode(const void *q_f16, const void *k_cache_f16, const void *v_cache_f16,
                                     const int32_t *lens, int B, int L_max, int n_heads, int d_h,
                                     float lambda, void *out_f16, void *workspace, size_t workspace_bytes,
                                     void *stream);

/* ---------------------------------------------------------------- base-3 packing (1.6 bits per weight)
 *
 * The paper counts its backbone at log2 3 = 1.58 bits per weight (Sec. 4.1, Def. "Effective
 * Bit-Width").  This alternative layout stores five ternary weights per byte (3^5 = 243 <= 256):
 * 20 % fewer bytes to stream than the 2-bit layout, for the few-token decode where the weights are
 * nearly all the traffic.  Same ternarisation as hgf_quantize_pack_weights (same s_w, same T).
 *
 * Layout: row n of the matrix is ceil(d_in / 5) bytes padded to a multiple of 16 (rows start
 * 16-byte aligned; a lane's 16-byte load is 80 weights of one row); byte g of a row is
 * sum_{i<5} (T[n, 5g+i] + 1) * 3^i, columns past d_in counting as T = 0 (padding bytes: 121).
 *
 * hgf_linear_forward_b3 is Algorithm 1 for one layer whose W_packed is such a buffer, for
 * M <= 4 tokens and d_in <= 20480 (HGF_ERR_UNSUPPORTED beyond; layers with ln_gamma likewise):
 * the same integers as hgf_linear_forward, outputs within the same tolerance. */
size_t hgf_packed_weight_bytes_b3(int d_out, int d_in);
hgf_status hgf_quantize_pack_weights_b3(const float *W, int d_out, int d_in, void *packed_out,
                                        float *s_w_out, void *workspace, size_t workspace_bytes,
                                        void *stream);
hgf_status hgf_unpack_weights_b3(const void *packed, int d_out, int d_in, int8_t *T_out, void *stream);
hgf_status hgf_linear_forward_b3(const void *x_f16, int M, const hgf_layer *L, void *y_f16,
                                 int32_t *acc_debug, void *workspace, size_t workspace_bytes,
                                 void *stream);

/* hgf_linear_forward for callers that cannot allocate device memory and have no workspace to
 * pass: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same arguments, same kernels and same results as hgf_linear_forward, but what the workspace
 * holds there (launch counter, exchange buffers, x_q, token scales, SiLU(A x), partial sums)
 * lives in a fixed array inside the library's device image: hgf_static_scratch_bytes() bytes
 * (8 MiB) on every GPU the library runs on, held until the process ends.  The call allocates
 * and frees nothing (no hipMalloc, no hipFree, no allocating library routine).
 *
 * Limit: hgf_static_scratch_needed(M, d_in, d_out, rank) <= hgf_static_scratch_bytes(), roughly
 * M * pad128(d_in) + 1 KiB * M (+ 16 KiB * M for M <= 64) + 0.3 MiB: e.g. any d_in at
 * M <= 64, or d_in <= 3072 at M = 2048.  Beyond it: HGF_ERR_WORKSPACE, nothing enqueued.
 * The first call on a GPU (with that GPU current) looks up the array's address there and
 * enqueues two small fill kernels on `stream` that prepare it, as hgf_workspace_init does for a
 * workspace.  Every call on a GPU shares that GPU's array, which keeps what the last call left:
 * each call rewrites what it reads, and the launch counter and exchange buffers are handed on
 * in a consistent state -- provided calls on one GPU do not overlap.  Calls must be ordered
 * (one stream, or events between streams); concurrent calls on one GPU race on the array.
 * Other entry points and other workspaces are not affected. */
size_t hgf_static_scratch_bytes(void);
size_t hgf_static_scratch_needed(int M, int d_in, int d_out, int rank);   /* 0 on invalid sizes */
hgf_status hgf_linear_forward_static(const void *x_f16, int M, const hgf_layer *L, void *y_f16,
                                     int32_t *acc_debug, void *stream);

/* Algorithm 1 over a list of layers, run in order on one stream.  The paper's blocks apply
 * several HGF linears to one input: the attention of Sec. 2.4 (Def. "HGF Attention
 * Projections": Q, K and V are each Phi_HGF of the same X; the appendix implementation's
 * attention forward calls the three projections on the same tensor) and its MLP (appendix
 * implementation, block forward: w1 and w2 both read the normalised block input, w3 reads
 * their product).  Layer i reads slots[src_slot] (fp16 [M, d_in]) and writes slots[dst_slot]
 * (fp16 [M, d_out]); consecutive layers with the same src_slot and d_in share one
 * activation quantisation (steps 1-2 of Algorithm 1 run once for the group).
 *
 *   layers  host array of n_layers descriptions
 *   slots   host array of n_slots device pointers
 *
 * For M <= 4 runs of layers execute as persistent launches whose workgroups hand activations
 * to each other inside the launch.  Such a launch is sized to what an occupancy query says
 * the device holds at once, and needs the device to itself while it runs: kernels of other
 * streams that occupy compute units can starve its workgroups, whose bounded waits then run
 * out (NaN outputs, error word set -- see hgf_workspace_init).  The call cannot see that:
 * after synchronising, read the int32 at byte offset 8 of the workspace; nonzero means the
 * outputs of some launch since the last hgf_workspace_init are void.  HGF_ERR_DEVICE is
 * returned when the runtime refuses a launch (layers enqueued before it have run).
 */
hgf_status hgf_stack_forward(const hgf_layer *layers, int n_layers, void *const *slots,
                             int n_slots, int M, void *workspace, size_t workspace_bytes,
                             void *stream);

/* Profiling aid (host state, not thread-safe, not for use under graph capture).  While
 * enabled, hgf_linear_forward and hgf_stack_forward bracket every main-kernel launch
 * (the decode or the prefill kernel, not the quantiser or the down-projection) with a
 * pair of HIP events on the call's stream.  hgf_profile_collect waits for the recorded
 * events, then writes the summed elapsed milliseconds and the launch count per kind:
 * index 0 = decode kernel, index 1 = prefill kernel (both arrays: 2 host elements), and
 * forgets the recorded pairs. */
void hgf_profile_enable(int on);
hgf_status hgf_profile_collect(double *ms_out, long long *launches_out);

/* Measurement aid: the int8 rate the matrix cores sustain on a loop of nothing but the MFMA of
 * the prefill kernel (operands in registers, no memory traffic, two workgroups of four
 * wavefronts per compute unit, ten timed launches of `iters` x 32 MFMAs per wavefront after ten
 * untimed ones), for operand values of kind 0 = all ones, 1 = codes 0..2 against random int8
 * (this layer's operands), 2 = random int8 on both sides.  The chip lowers its clock under the
 * matrix cores' switching power, so the rate depends on the values.  Writes tera-operations per
 * second (2 per multiply-add) and the shader clock in GHz seen by one workgroup (host
 * pointers).  Allocates and frees its own small device buffers; synchronises the stream.
 * HGF_ERR_SHAPE for a kind outside 0..2 or iters outside 1..2^20. */
hgf_status hgf_probe_mfma_rate(int operand_kind, int iters, double *tops_out, double *ghz_out, void *stream);

/* Tuning hook (host state, not thread-safe) for calls with at most 4 tokens, d_in % 8 == 0 and
 * d_in <= 12288.  level 2 (default): hgf_stack_forward runs whole runs of groups of layers as
 * one persistent launch (activations handed from layer to layer inside the launch), and
 * single groups as level 1; level 1: each group of layers is one persistent launch;
 * level 0: the two-launch path that serves 5..64 tokens.  Results agree bit for bit in the
 * integers; the fp16 outputs may differ in the last place (different split of A x). */
void hgf_set_single_launch(int level);

/* Test hook (host state, not thread-safe) for the whole-stack launch of hgf_stack_forward, in
 * which workgroups wait for each other's results: every such wait gives up after a bounded
 * number of tries (by default about a second), sets the sticky error word of the workspace
 * (byte offset 8, cleared by hgf_workspace_init), turns the affected outputs into NaN and lets
 * the kernel run to its end.  tries > 0 replaces the bound of every wait by that many tries, so
 * that a test can see the give-up path without anything having to go wrong; 0 restores the
 * default.  Never needed in production. */
void hgf_set_wait_limit(int tries);

/* Measurement aid (host state, not thread-safe): time stamps from inside the whole-stack launch
 * of hgf_stack_forward.  With a device buffer set, every later launch whose workgroups fit it
 * writes, per workgroup, 11 roles x 4 phases x 8 words: stamps of the device-wide 100 MHz clock
 * (uint64; 0 = not reached): roles 0..7 the contracting wavefronts (0 phase entered, 1 tokens
 * complete, 2 absmax agreed, 3 tokens quantised, 4 first unit contracted, 5 last unit contracted;
 * 6 is no stamp but the ticks the wavefront waited for weight tiles to land, 7 its number of such waits), 8 the
 * slice wavefront (0 phase entered, 1 own slices of A x stored, 2 SiLU(A x) in LDS), 9 the unit
 * wavefront (0 phase entered, 1 SiLU(A x) seen, 2 first unit's sums complete, 3 last unit's sums
 * complete, 4 last unit stored), 10 the first loader (0 first weight tile of the phase
 * requested), for the phases first_phase .. first_phase + 3 of the launch.  bytes must cover
 * 256 workgroups (256 * 11 * 4 * 8 * 8).  NULL switches it off.  bench.py --timeline prints the
 * medians. */
void hgf_set_stack_trace(void *device_buffer, size_t bytes, int first_phase);

#ifdef __cplusplus
}
#endif
#endif /* HGF_H */
