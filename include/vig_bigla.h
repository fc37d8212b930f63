/*
 * vig_bigla.h -- C ABI of the MI355X (gfx950) BiGLA token mixer and 2D gating locality
 * injection: the forward hot path of the ViG block (Sections 4.2.1 and 4.2.2 of the paper).
 *
 * Conventions for every entry point
 *   - All tensor pointers are DEVICE pointers owned by the caller.  The library never
 *     allocates or frees device memory and never synchronises; work is enqueued on `stream`
 *     (a hipStream_t passed as void*, NULL = the default stream) and the call returns at once.
 *     The one exception is the measurement aid at the end of this header: vig_timing_enable(1)
 *     creates a pool of HIP events, and vig_timing_collect waits for them.
 *   - Tensors are dense, row-major, innermost index = feature.  All tensors of one call
 *     share `dtype` (vig_dtype).  VIG_BF16: bf16 in, fp32 accumulate, bf16 out rounded to
 *     nearest even.  VIG_F32: fp32 throughout.
 *   - Every tensor pointer must be 16-byte aligned; outputs must not alias inputs.
 *   - Return value: a vig_status.  Arguments are validated on the host before anything is
 *     launched; nothing aborts or throws across this boundary.  After VIG_ERR_HIP the raw
 *     hipError_t is available from vig_last_hip_error().
 */
#ifndef VIG_BIGLA_H
#define VIG_BIGLA_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    VIG_OK = 0,
    VIG_ERR_NULL = -1,        /* a required pointer is NULL                              */
    VIG_ERR_SHAPE = -2,       /* a size is <= 0 or the product of sizes overflows        */
    VIG_ERR_DTYPE = -3,       /* dtype is not a vig_dtype                                */
    VIG_ERR_UNSUPPORTED = -4, /* dk or dv outside {16, 32, 64}; D not a multiple of 32;
                                 a plan the shape does not admit                         */
    VIG_ERR_ALIGN = -5,       /* a pointer is not 16-byte aligned                        */
    VIG_ERR_WORKSPACE = -6,   /* workspace NULL or smaller than bigla_workspace_bytes()  */
    VIG_ERR_HIP = -7,         /* a HIP call failed; see vig_last_hip_error()             */
    VIG_ERR_LAYOUT = -8,      /* layout is not a vig_layout                              */
    VIG_ERR_SCRATCH_LIMIT = -9 /* bigla_fwd_static_scratch: the problem needs more scratch
                                 than VIG_STATIC_SCRATCH_BYTES                           */
} vig_status;

typedef enum { VIG_F32 = 0, VIG_BF16 = 1 } vig_dtype;

/*
 * Placement of heads and tokens in the activations.  VIG_LAYOUT_BHLD, [B, H, L, d], is what
 * bigla_fwd / locality_gate_fwd take.  VIG_LAYOUT_BLHD, [B, L, H, d] (token-major: a token's H*d
 * features are contiguous, the form in which the projections of a block emit q, k, v and the
 * gates, so that no transpose is needed around the token mixer -- Section 4.2.1 treats heads as
 * independent slices of the feature dimension), is accepted by the *_layout entry points.
 */
typedef enum { VIG_LAYOUT_BHLD = 0, VIG_LAYOUT_BLHD = 1 } vig_layout;

/*
 * Bytes of device scratch that bigla_fwd needs for this problem (0 if none).  The scratch
 * holds the boundary states of the chunkwise evaluation (per segment and per chunk), or the
 * forward partial outputs of the fp32-arithmetic recurrence on bf16 storage; its contents
 * before the call are ignored and after the call are unspecified.  Returns 0 for invalid
 * sizes (bigla_fwd reports those).
 */
size_t bigla_workspace_bytes(int B, int H, int L, int dk, int dv, int dtype);

/*
 * BiGLA forward -- Section 4.2.1, Eq. (BiGLA).  For every batch b and head h, with
 * alpha_fwd = exp(g_fwd), alpha_bwd = exp(g_bwd) (per key dimension):
 *     S_fwd_t = diag(alpha_fwd_t) S_fwd_{t-1} + k_t^T v_t ,   S_fwd_{-1} = 0
 *     S_bwd_t = diag(alpha_bwd_t) S_bwd_{t+1} + k_t^T v_t ,   S_bwd_{L}  = 0
 *     out_t   = ( q_t S_fwd_t + q_t S_bwd_t ) / 2
 * Both directions are evaluated in the same launches; no reversed copy of the sequence
 * is ever written.  No scaling of q is applied.
 *
 *   q, k         [B, H, L, dk]   in
 *   v            [B, H, L, dv]   in
 *   g_fwd, g_bwd [B, H, L, dk]   in   LOG forget gates, log(alpha) <= 0
 *                                     (log alpha = logsigmoid(.)/tau for the paper's gate);
 *                                     positive or NaN values are outside the contract
 *   out          [B, H, L, dv]   out
 *   L >= 1 is arbitrary (ragged final chunk handled inside); dk, dv in {16, 32, 64}.  On the
 *   chunkwise path (below) L must stay below 2^24 (VIG_ERR_SHAPE otherwise).
 *   workspace / workspace_bytes: device scratch of at least bigla_workspace_bytes(...);
 *   may be NULL/0 when that function returns 0.
 *
 * Numerics: VIG_BF16 with dv = 64, dk = 64 or 32 and L >= 32 runs the chunkwise MFMA path (bf16
 * operands, fp32 accumulation, fp32 carried state; dk = 32 is widened to 64 key channels with zeros
 * inside the kernels).  Where some channel of a 64-token chunk decays by more than 16 nats (a quarter
 * of a nat per step), the operands of every token's nearest products are kept to 16 bits: at full
 * speed up to 60 nats per chunk where the eight-wave kernels run (see bigla_fwd_plan),
 * otherwise in a range-safe form, several times slower, that treats per-step log gates below -8
 * as -8 (alpha < 3.4e-4 acts as a hard reset either way; the difference is far below the bf16
 * tolerance).  Every other case runs the exact recurrence in fp32 arithmetic.
 */
int bigla_fwd(const void *q, const void *k, const void *v, const void *g_fwd, const void *g_bwd,
              void *out, int B, int H, int L, int dk, int dv, int dtype, void *workspace,
              size_t workspace_bytes, void *stream);

/*
 * bigla_fwd with the activations q, k, v, g_fwd, g_bwd and out all in `layout` (a vig_layout);
 * everything else as for bigla_fwd (same workspace size).  With VIG_LAYOUT_BLHD, L * H * max(dk, dv)
 * must stay below 2^31 and L below 2^24 (VIG_ERR_SHAPE otherwise).
 */
int bigla_fwd_layout(const void *q, const void *k, const void *v, const void *g_fwd, const void *g_bwd,
                     void *out, int B, int H, int L, int dk, int dv, int dtype, int layout,
                     void *workspace, size_t workspace_bytes, void *stream);

/*
 * bigla_fwd_layout with a choice among the kernels that evaluate the chunkwise form (Section 4.2.1,
 * Eq. (BiGLA); a measurement and testing aid: the result is the same up to operand rounding).
 *   VIG_FWD_AUTO              what bigla_fwd_layout runs: the eight-wave kernels where they apply,
 *                             the four-wave kernels elsewhere;
 *   VIG_FWD_FOUR_WAVE         workgroups of four waves, each wave walking the whole chain of a chunk
 *                             step for its 16 tokens;
 *   VIG_FWD_WAVE_SPECIALISED  workgroups of eight waves: producer waves (gate scans, exponentials, scaled
 *                             keys, score tiles, P.V) and consumer waves (state readouts, output rows,
 *                             state update) on the same SIMDs, one chunk apart.  VIG_BF16 with dv = 64,
 *                             dk = 64 or 32 and at least two chunks, except short sequences in many slabs
 *                             (VIG_ERR_UNSUPPORTED otherwise).  A (slab, segment) unit whose gates are
 *                             outside the fast form's range is evaluated by the general four-wave code
 *                             inside the same launches.
 *   VIG_FWD_SLAB_SWEEP        the four-wave code with one workgroup per (batch, head) slab that sweeps the
 *                             whole sequence twice in one launch (right to left for the backward states,
 *                             left to right for the outputs): no segments, so k, v and the gates are read
 *                             from memory once when the second sweep finds them in cache, at the price of
 *                             B * H workgroups only.  What VIG_FWD_AUTO runs for short sequences in many
 *                             slabs; selectable here for any shape of the chunkwise path.
 * Workspace as for bigla_fwd_layout.  Unknown plan: VIG_ERR_UNSUPPORTED.
 */
typedef enum {
    VIG_FWD_AUTO = 0,
    VIG_FWD_FOUR_WAVE = 1,
    VIG_FWD_WAVE_SPECIALISED = 2,
    VIG_FWD_SLAB_SWEEP = 3
} vig_fwd_plan;
int bigla_fwd_plan(const void *q, const void *k, const void *v, const void *g_fwd, const void *g_bwd,
                   void *out, int B, int H, int L, int dk, int dv, int dtype, int layout, int plan,
                   void *workspace, size_t workspace_bytes, void *stream);

/*
 * bigla_fwd_layout for callers that cannot allocate device memory or pass a workspace: code that
 * runs under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The scratch
 * that bigla_fwd_layout takes from the caller lives here in an array that is part of the library
 * itself (VIG_STATIC_SCRATCH_BYTES bytes per GPU, held from the first call on that GPU until the
 * process ends); inputs and the output are still the caller's.  The call allocates and frees
 * nothing, neither directly nor through another library.  The first call on a GPU looks up the
 * array's address on that GPU (make it outside a capture).
 *   - Arguments, numerics, results and errors as for bigla_fwd_layout (bit-identical results).
 *   - A problem for which bigla_workspace_bytes(...) exceeds VIG_STATIC_SCRATCH_BYTES is rejected
 *     with VIG_ERR_SCRATCH_LIMIT before anything is launched.  The limit holds each of the five
 *     benchmark configurations (the largest, B=8, H=6, L=4096, needs 42 MB).
 *   - Every call on one GPU uses that GPU's one array, whose contents are unspecified between
 *     calls (nothing in it has to start at zero: each call writes what it later reads).  Calls
 *     that overlap in time on one GPU -- on different streams or from different threads -- race on
 *     it; order them on one stream or with events.
 */
#define VIG_STATIC_SCRATCH_BYTES (48u << 20)
int bigla_fwd_static_scratch(const void *q, const void *k, const void *v, const void *g_fwd, const void *g_bwd,
                             void *out, int B, int H, int L, int dk, int dv, int dtype, int layout,
                             void *stream);

/*
 * BiGLA backward -- the gradient of bigla_fwd (Section 4.2.1, Eq. (BiGLA); the paper trains
 * through the token mixer, Section 5, and prints no gradient formulas, so this is the chain rule
 * on the two recurrences).  Given d_out = dLoss/d_out it returns dLoss/d(q, k, v, g_fwd, g_bwd):
 * with do_t = d_out_t / 2 and, per direction, the adjoint of the state
 *     A_t = q_t^T do_t + diag(alpha_{t+1}) A_{t+1}   (forward direction; mirrored for backward),
 *     dq_t = S_t do_t^T ,  dk_t = A_t v_t^T ,  dv_t = k_t A_t     (summed over both directions),
 *     dg_fwd_t = alpha_fwd_t * sum_j A_fwd_t[., j] S_fwd_{t-1}[., j]   (likewise dg_bwd with t+1).
 *
 *   q, k, v, g_fwd, g_bwd   as for bigla_fwd_layout            in
 *   d_out                   [B, H, L, dv]                      in
 *   dq, dk, dg_fwd, dg_bwd  [B, H, L, dk]                      out
 *   dv                      [B, H, L, dv]                      out
 *   (all in `layout`; dk, dv in {16, 32, 64}; any L >= 1)
 *   workspace: at least bigla_bwd_workspace_bytes(...) bytes (fp32 partial gradients; for bf16 with
 *   dv = 64 and dk = 64 or 32 also four 64 x 64 bf16 state matrices per 64-token chunk).
 * Two sets of kernels.  bigla_bwd_plan with VIG_BWD_RECURRENT runs the exact ones: fp32 arithmetic
 * token by token for either dtype (bf16 in and out, rounded to nearest even), the gate gradients
 * formed as running sums of q * dq - k * dk per direction, which is the same quantity.
 * VIG_BWD_AUTO (what bigla_bwd runs) takes, for VIG_BF16 with dv = 64 and dk = 64 or 32, the chunkwise
 * matrix-core kernels (operands rounded to bf16, fp32 accumulation, the counterpart of the
 * forward's chunkwise path; L below 2^24 and a slab addressable with 32-bit byte offsets, else
 * VIG_ERR_SHAPE) and leaves to the exact kernels, inside the same call, only the (b, h) slabs in
 * which some 64-token chunk decays by more than 60 nats in a channel; for every other dtype or
 * head shape it is the exact kernels.  Unknown plan: VIG_ERR_UNSUPPORTED.
 */
size_t bigla_bwd_workspace_bytes(int B, int H, int L, int dk, int dv, int dtype);
int bigla_bwd(const void *q, const void *k, const void *v, const void *g_fwd, const void *g_bwd,
              const void *d_out, void *dq, void *dk, void *dv, void *dg_fwd, void *dg_bwd, int B, int H,
              int L, int dk_, int dv_, int dtype, int layout, void *workspace, size_t workspace_bytes,
              void *stream);
typedef enum { VIG_BWD_AUTO = 0, VIG_BWD_RECURRENT = 1 } vig_bwd_plan;
int bigla_bwd_plan(const void *q, const void *k, const void *v, const void *g_fwd, const void *g_bwd,
                   const void *d_out, void *dq, void *dk, void *dv, void *dg_fwd, void *dg_bwd, int B, int H,
                   int L, int dk_, int dv_, int dtype, int layout, int plan, void *workspace,
                   size_t workspace_bytes, void *stream);

/*
 * 2D gating locality injection forward -- Section 4.2.2.  Token t of the flattened
 * sequence is patch (y, xp) of the Hg x Wg grid, t = y*Wg + xp; channel c = h*dv + j.
 *     O_local[y,xp,c] = bias[c] + sum_{dy,dx in {-1,0,1}} w[c,dy+1,dx+1] * x[y+dy, xp+dx, c]
 *                       (stride 1, zero padding, cross-correlation)
 *     G   = sigmoid(gate_logits)
 *     out = G * O_local + (1 - G) * o_global
 *
 *   x, gate_logits, o_global  [B, H, Hg*Wg, dv]   in
 *   w                         [H*dv, 3, 3]        in
 *   bias                      [H*dv] or NULL      in
 *   out                       [B, H, Hg*Wg, dv]   out
 *   dv in {16, 32, 64}.  One (batch element, head) slab must stay below 4 GiB (VIG_ERR_SHAPE).
 */
int locality_gate_fwd(const void *x, const void *w, const void *bias, const void *gate_logits,
                      const void *o_global, void *out, int B, int H, int Hg, int Wg, int dv,
                      int dtype, void *stream);

/*
 * locality_gate_fwd with x, gate_logits, o_global and out in `layout` (a vig_layout): with
 * VIG_LAYOUT_BLHD they are [B, Hg*Wg, H, dv], i.e. channel c = h*dv + j of a pixel is contiguous.
 * w and bias as for locality_gate_fwd.  With VIG_LAYOUT_BLHD one batch element must stay below 4 GiB.
 */
int locality_gate_fwd_layout(const void *x, const void *w, const void *bias, const void *gate_logits,
                             const void *o_global, void *out, int B, int H, int Hg, int Wg, int dv,
                             int dtype, int layout, void *stream);

/*
 * The two steps above as one call -- Section 4.2.2, Eq. (2D gating), lines 2 and 4, with the
 * gate logits given:
 *     out = G * DWConv3x3(x) + (1 - G) * BiGLA(q, k, v, g_fwd, g_bwd),   G = sigmoid(gate_logits)
 * for L = Hg * Wg tokens in raster order.  Arguments as for bigla_fwd_layout and
 * locality_gate_fwd_layout (all activations in `layout`; Hg * Wg below 2^24).  `plan` (a vig_plan):
 *   VIG_PLAN_TWO_LAUNCHES     the token mixer writes its output into the workspace and the locality
 *                             kernel reads it back (any supported shape and dtype);
 *   VIG_PLAN_FUSED_EPILOGUE   the output pass of the chunkwise path applies the blend to each chunk's
 *                             rows before writing them, so the token mixer's output (rounded to bf16
 *                             as bigla_fwd would store it) never goes through memory: a sixth fewer
 *                             bytes per step and no intermediate tensor, at about the speed of two
 *                             launches where the eight-wave kernels carry it (grids under 65 columns,
 *                             the shapes of VIG_FWD_WAVE_SPECIALISED) and slower elsewhere.
 *                             VIG_BF16 with dv = 64, dk = 64 or 32 and at least 32 tokens only,
 *                             the cases in which bigla_fwd runs the chunkwise path
 *                             (VIG_ERR_UNSUPPORTED otherwise);
 *   VIG_PLAN_AUTO             two launches (the output pass is bound by its vector arithmetic, and
 *                             the blend's arithmetic costs there what the second pass over memory
 *                             costs): the fused plan is for callers who cannot afford the
 *                             intermediate tensor.
 * The two-launch plan returns bit for bit what bigla_fwd_layout followed by locality_gate_fwd_layout
 * returns; the fused plan may differ from it by a bf16 step of an output here and there (it sums the
 * conv's taps in pairs, and for some shapes evaluates the token mixer with another set of kernels).
 * workspace: at least bigla_locality_workspace_bytes(B, H, Hg*Wg, dk, dv, dtype, plan) bytes
 * (that function returns 0 for invalid or unsupported arguments).
 */
typedef enum { VIG_PLAN_AUTO = 0, VIG_PLAN_TWO_LAUNCHES = 1, VIG_PLAN_FUSED_EPILOGUE = 2 } vig_plan;
size_t bigla_locality_workspace_bytes(int B, int H, int L, int dk, int dv, int dtype, int plan);
int bigla_locality_fwd(const void *q, const void *k, const void *v, const void *g_fwd, const void *g_bwd,
                       const void *x, const void *w, const void *bias, const void *gate_logits, void *out,
                       int B, int H, int Hg, int Wg, int dk, int dv, int dtype, int layout, int plan,
                       void *workspace, size_t workspace_bytes, void *stream);

/*
 * Direction-wise forget gates -- Section 3 (low-rank gate, temperature tau) and the first two
 * lines of Eq. (BiGLA), Section 4.2.1.  For every token t of every batch element, with x_t the
 * block input of width D:
 *     z_t     = (x_t W1) W2 + b                in R^{2*H*dk}     (W1: D x 16, W2: 16 x 2*H*dk)
 *     alpha_t = sigmoid(z_t)^(1/tau)
 *     entries [0, H*dk) of alpha_t are the forward gates, [H*dk, 2*H*dk) the backward gates;
 *     inside each half head h owns entries [h*dk, (h+1)*dk)
 * and the outputs are the LOG gates log(alpha) = log(sigmoid(z)) / tau (<= 0, finite for every
 * finite z) in the form bigla_fwd takes.
 *
 *   x            [B, L, D]            in    D a multiple of 32; VIG_BF16: one of 32, 64, ..., 256,
 *                                           320, 384, 512, 576, 640, 768, 1024
 *   w1           [16, D]              in    W1 transposed (how a linear layer D -> 16 stores its weight)
 *   w2           [2*H*dk, 16]         in    W2 transposed (linear layer 16 -> 2*H*dk)
 *   bias         [2*H*dk] or NULL     in
 *   g_fwd, g_bwd [B, H, L, dk] (VIG_LAYOUT_BHLD) or [B, L, H, dk] (VIG_LAYOUT_BLHD)   out
 *   dk in {16, 32, 64}; tau > 0 (16 in the paper); layout a vig_layout (of the outputs).
 * VIG_BF16: both products on the matrix cores with fp32 accumulation (x W1 rounded to bf16 in
 * between), fp32 log-sigmoid, bf16 out.  VIG_F32: fp32 throughout.
 */
int gate_producer_fwd(const void *x, const void *w1, const void *w2, const void *bias, void *g_fwd,
                      void *g_bwd, int B, int H, int L, int D, int dk, float tau, int dtype, int layout,
                      void *stream);

/*
 * The gate producer and the token mixer as one call -- Section 3 (gate) and all of Eq. (BiGLA),
 * Section 4.2.1: gate_producer_fwd(x, w1, w2, bias -> g_fwd, g_bwd) followed by
 * bigla_fwd_layout(q, k, v, g_fwd, g_bwd -> out).  g_fwd and g_bwd are OUTPUTS here as well: the log gates
 * are returned (the mixer's gradient needs them), in `layout` like q, k, v and out.  Arguments as for those
 * two functions.
 *   VIG_GATES_SEPARATE       the two launches one after the other (every shape and dtype they support);
 *   VIG_GATES_IN_STATE_PASS  x W1 alone in a small launch (32 bytes per token, in the workspace); the state
 *                            pass of the chunkwise mixer then makes each chunk's gates itself from it, writes
 *                            them to g_fwd / g_bwd for the output pass and never reads them back: the gates
 *                            cross memory twice (written, read by the output pass) instead of three times.
 *                            Same arithmetic as gate_producer_fwd, bit for bit.  VIG_BF16, dv = 64,
 *                            where bigla_fwd_plan admits VIG_FWD_WAVE_SPECIALISED (VIG_ERR_UNSUPPORTED
 *                            otherwise, and while vig_measure_alias_slabs is on);
 *   VIG_GATES_AUTO           VIG_GATES_IN_STATE_PASS where it applies, else VIG_GATES_SEPARATE.
 * workspace: at least gated_bigla_workspace_bytes(B, H, L, dk, dv, dtype) bytes (0 for invalid or unsupported
 * arguments; it covers every plan).
 */
typedef enum { VIG_GATES_AUTO = 0, VIG_GATES_SEPARATE = 1, VIG_GATES_IN_STATE_PASS = 2 } vig_gates_plan;
size_t gated_bigla_workspace_bytes(int B, int H, int L, int dk, int dv, int dtype);
int gated_bigla_fwd(const void *x, const void *w1, const void *w2, const void *bias, const void *q, const void *k,
                    const void *v, void *g_fwd, void *g_bwd, void *out, int B, int H, int L, int D, int dk, int dv,
                    float tau, int dtype, int layout, int plan, void *workspace, size_t workspace_bytes,
                    void *stream);

/*
 * Measurement aid (no part of the method): per-kernel timing with HIP events recorded on the
 * stream each kernel is launched on.  vig_timing_enable(1) clears the records and makes every
 * later launch of this library from the calling thread record a start/stop event pair;
 * vig_timing_enable(0) stops recording.  vig_timing_collect waits for the recorded events of one
 * kernel (a vig_kernel id) and returns their summed duration in milliseconds and their count.
 * Host pointers; VIG_ERR_SHAPE for an unknown id.
 */
typedef enum {
    VIG_KERNEL_SEGMENT_STATE = 0, /* chunkwise path, launch 1: segment end states + stash     */
    VIG_KERNEL_GATE_LOWRANK = 1,  /* x W1 alone, for the gate producer inside the state pass   */
    VIG_KERNEL_SEGMENT_OUT = 2,   /* chunkwise path, launch 2: output pass                    */
    VIG_KERNEL_RECURRENT = 3,     /* exact fp32 recurrence                                    */
    VIG_KERNEL_LOCALITY_GATE = 4, /* depthwise conv + gate                                    */
    VIG_KERNEL_SEGMENT_OUT_GENERAL = 5, /* chunkwise path, output pass of single-chunk sequences */
    VIG_KERNEL_GATE_PRODUCER = 6, /* forget-gate producer                                     */
    VIG_KERNEL_SLAB = 7,          /* chunkwise path, one-segment plans: both passes, one launch */
    VIG_KERNEL_BACKWARD = 8       /* all launches of one bigla_bwd call together               */
} vig_kernel;
int vig_timing_enable(int on);
int vig_timing_collect(int kernel, double *total_ms, long *launches);

/*
 * Measurement aid (no part of the method): vig_measure_alias_slabs(1) makes the chunkwise kernels of
 * bigla_fwd read the q, k, v and gates of the first (batch, head) slab for every slab, so that those
 * inputs stay cache-resident and the kernels' contractions can be timed without the stream from memory
 * (outputs, and the workspace, are still written per slab; results are meaningless).  0 restores normal
 * operation.  The call synchronises the device (it copies a flag into the kernels' constant state) and
 * applies to every later call from any thread.
 */
int vig_measure_alias_slabs(int on);

/* Human-readable name of a vig_status (static storage, never NULL). */
const char *vig_status_str(int status);

/* The hipError_t of the most recent VIG_ERR_HIP on this thread (0 if none). */
int vig_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* VIG_BIGLA_H */
