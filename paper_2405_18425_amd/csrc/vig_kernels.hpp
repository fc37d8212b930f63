// Internal launch interface between the C-ABI layer and the kernel translation units.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>

namespace vig {

// Tensor layouts.  Head-major [B, H, L, d] is the default.  Token-major [B, L, H, d] (what the
// projection GEMMs of a block emit) is passed to the BiGLA launches as `heads_token_major` = H
// (0 selects head-major) and to the locality launch as a flag.

// ---- exact fp32 recurrence (any supported head shape, both dtypes) --------------------------
size_t bigla_recurrent_workspace_bytes(long BH, int L, int dv, bool is_bf16);
hipError_t bigla_recurrent_launch(const void *q, const void *k, const void *v, const void *g_fwd,
                                  const void *g_bwd, void *out, long BH, int L, int dk, int dv, bool is_bf16,
                                  int heads_token_major, void *workspace, hipStream_t stream);

// ---- chunkwise bf16 MFMA path (dv = 64, dk = 64 or 32) ----------------------------------------
bool bigla_chunk_supported(int dk, int dv, bool is_bf16);
size_t bigla_chunk_workspace_bytes(long BH, int L);
// Inputs of the 2D gating locality injection when the chunkwise output pass applies it to its rows
// before writing them (x and gate_logits in the activations' layout, L = Hg * Wg).
struct LocalityFusion {
    const void *x, *w, *bias /* may be null */, *gate_logits;
    int H, Hg, Wg;
};
// fusion == nullptr: out receives the token mixer's output; otherwise the block output.
// kernels: 0 = the faster set of kernels for the shape, 1 = the four-wave kernels, 2 = the eight-wave
// producer/consumer kernels (bigla_chunk_ws_selectable says where they apply; never with a fusion).
bool bigla_chunk_ws_selectable(long BH, int L, int dk);
// measurement aid: every slab of the chunkwise forward kernels reads slab 0's q, k, v and gates (synchronous)
hipError_t bigla_chunk_set_alias(int on);
hipError_t bigla_chunk_launch(const void *q, const void *k, const void *v, const void *g_fwd, const void *g_bwd,
                              void *out, long BH, int L, int dk, int heads_token_major, const LocalityFusion *fusion,
                              int kernels, void *workspace, hipStream_t stream);

// The eight-wave kernels with the state pass making the gates from the gate producer's low-rank half
// (lowrank [B][L][16] bf16); g_fwd, g_bwd are written.  bf16, dv = 64, dk = 64 or 32; not while slabs are aliased.
bool bigla_chunk_gated_selectable(long BH, int L, int dk);
hipError_t bigla_chunk_gated_launch(const void *q, const void *k, const void *v, void *g_fwd, void *g_bwd, void *out,
                                    long BH, int L, int dk, int n_heads, int heads_token_major, const void *lowrank,
                                    const void *w2, const void *bias, float tau, void *workspace, hipStream_t stream);

// ---- gradient of the token mixer -----------------------------------------------------------------
// Exact fp32 recurrences for any supported head shape and both dtypes; for bf16 with dv = 64 and dk = 64 or 32 the
// chunkwise matrix-core kernels run first and leave to the exact ones only the slabs they mark
// (gates beyond their range).  recurrent_only: the exact kernels take everything.
size_t bigla_bwd_workspace_bytes(long BH, int L, int dk, int dv, bool is_bf16);
hipError_t bigla_bwd_launch(const void *q, const void *k, const void *v, const void *g_fwd, const void *g_bwd,
                            const void *d_out, void *dq, void *dk, void *dv, void *dg_fwd, void *dg_bwd, long BH, int L,
                            int dk_, int dv_, bool is_bf16, int heads_token_major, bool recurrent_only, void *workspace,
                            hipStream_t stream);
bool bigla_bwd_chunk_supported(int dk, int dv, bool is_bf16);
size_t bigla_bwd_chunk_workspace_bytes(long BH, int L);
// the per-slab marks inside a chunkwise workspace (device memory, valid after the launch below)
const int *bigla_bwd_chunk_marks(void *workspace, long BH, int L);
hipError_t bigla_bwd_chunk_launch(const void *q, const void *k, const void *v, const void *g_fwd, const void *g_bwd,
                                  const void *d_out, void *dq, void *dk, void *dv, void *dg_fwd, void *dg_bwd, long BH,
                                  int L, int dk_, int heads_token_major, void *workspace, hipStream_t stream);

// ---- depthwise 3x3 conv + sigmoid-gated blend -------------------------------------------------
hipError_t locality_gate_launch(const void *x, const void *w, const void *bias, const void *gate_logits,
                                const void *o_global, void *out, int B, int H, int Hg, int Wg, int dv,
                                bool is_bf16, int token_major, hipStream_t stream);

// ---- direction-wise forget-gate producer (low-rank projection + log-sigmoid / tau) -----------
bool gate_producer_width_ok(int D, bool is_bf16);
hipError_t gate_producer_launch(const void *x, const void *w1, const void *w2, const void *bias, void *g_fwd,
                                void *g_bwd, int B, int H, int L, int D, int dk, float tau, bool is_bf16,
                                int token_major, hipStream_t stream);
// x W1 alone, bf16: lowrank [B][L][16]
hipError_t gate_lowrank_launch(const void *x, const void *w1, void *lowrank, int B, int L, int D, hipStream_t stream);

}  // namespace vig
