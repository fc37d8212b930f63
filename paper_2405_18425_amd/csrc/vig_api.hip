// C-ABI entry points (declared in include/vig_bigla.h): host-side validation and dispatch only.
// Every step of the path runs in the kernels of the other translation units.
#include <stdint.h>

#include <atomic>

#include "../../include/vig_bigla.h"
#include "vig_kernels.hpp"

namespace {

thread_local int g_last_hip_error = 0;

bool head_dim_ok(int d) { return d == 16 || d == 32 || d == 64; }

// Sequences shorter than half a chunk run the exact recurrence even where the chunkwise kernels apply:
// a slab of a few tokens is a handful of query-key products that can all be small at once, and the bf16
// rounding of the chunkwise form's scaled operands is then large against the slab's own outputs.
constexpr int kChunkwiseMinTokens = 32;
bool chunkwise_fwd(int L, int dk, int dv, bool bf16) { return vig::bigla_chunk_supported(dk, dv, bf16) && L >= kChunkwiseMinTokens; }
bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// B*H*L*d elements must stay addressable with a comfortable margin
bool sizes_ok(long a, long b, long c, long d)
{
    const long lim = 1L << 40;
    long n = a;
    if (n > lim / b) return false;
    n *= b;
    if (n > lim / c) return false;
    n *= c;
    if (n > lim / d) return false;
    return true;
}

// rows of 64 bf16 values, pitch 128 bytes (times H when token-major), L + 64 of them
bool chunk_offsets_ok(int L, int H, int layout)
{
    const long pitch = 128L * (layout == VIG_LAYOUT_BLHD ? H : 1);
    return L < (1 << 24) && (long(L) + 64) * pitch <= 0xfffffff0L;
}

int hip_status(hipError_t e)
{
    if (e == hipSuccess) return VIG_OK;
    g_last_hip_error = int(e);
    return VIG_ERR_HIP;
}

// The launch functions report hipGetLastError() after their launches.  That call returns the
// thread's sticky error, which an unrelated earlier HIP call of the caller may have left behind:
// it is cleared before anything is launched so that only this call's own error is reported.
void clear_stale_hip_error() { (void)hipGetLastError(); }

// ---- scratch of the entry point that allocates nothing ----------------------------------------
// The workspace of bigla_fwd_static_scratch: one array per GPU, part of the library's code object,
// held from the first use on that GPU until the process ends.  In host code the array's name is
// only a handle for hipGetSymbolAddress; the device address it yields (one per device) is what the
// kernels receive, exactly as they receive the caller's workspace in bigla_fwd_layout.
static __device__ __align__(256) unsigned char scratch[VIG_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
std::atomic<void *> g_scratch_ptr[kMaxDevices];

// The device address of `scratch` on the current device (looked up once per device), or nullptr
// with the HIP error recorded.
void *static_scratch()
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess && (dev < 0 || dev >= kMaxDevices)) e = hipErrorInvalidDevice;
    if (e != hipSuccess) {
        g_last_hip_error = int(e);
        return nullptr;
    }
    void *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (p) return p;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) {
        g_last_hip_error = int(e != hipSuccess ? e : hipErrorInvalidSymbol);
        return nullptr;
    }
    g_scratch_ptr[dev].store(p, std::memory_order_release);  // concurrent first calls store the same address
    return p;
}

}  // namespace

extern "C" {

size_t bigla_workspace_bytes(int B, int H, int L, int dk, int dv, int dtype)
{
    if (B <= 0 || H <= 0 || L <= 0 || !head_dim_ok(dk) || !head_dim_ok(dv)) return 0;
    if (dtype != VIG_F32 && dtype != VIG_BF16) return 0;
    const bool bf16 = dtype == VIG_BF16;
    if (!sizes_ok(B, H, L, dk > dv ? dk : dv)) return 0;
    const long BH = long(B) * H;
    if (chunkwise_fwd(L, dk, dv, bf16)) return vig::bigla_chunk_workspace_bytes(BH, L);
    return vig::bigla_recurrent_workspace_bytes(BH, L, dv, bf16);
}

int bigla_fwd(const void *q, const void *k, const void *v, const void *g_fwd, const void *g_bwd, void *out,
              int B, int H, int L, int dk, int dv, int dtype, void *workspace, size_t workspace_bytes,
              void *stream)
{
    return bigla_fwd_layout(q, k, v, g_fwd, g_bwd, out, B, H, L, dk, dv, dtype, VIG_LAYOUT_BHLD, workspace,
                            workspace_bytes, stream);
}

int bigla_fwd_layout(const void *q, const void *k, const void *v, const void *g_fwd, const void *g_bwd, void *out,
                     int B, int H, int L, int dk, int dv, int dtype, int layout, void *workspace,
                     size_t workspace_bytes, void *stream)
{
    return bigla_fwd_plan(q, k, v, g_fwd, g_bwd, out, B, H, L, dk, dv, dtype, layout, VIG_FWD_AUTO, workspace,
                          workspace_bytes, stream);
}

int bigla_fwd_plan(const void *q, const void *k, const void *v, const void *g_fwd, const void *g_bwd, void *out,
                   int B, int H, int L, int dk, int dv, int dtype, int layout, int plan, void *workspace,
                   size_t workspace_bytes, void *stream)
{
    if (!q || !k || !v || !g_fwd || !g_bwd || !out) return VIG_ERR_NULL;
    if (layout != VIG_LAYOUT_BHLD && layout != VIG_LAYOUT_BLHD) return VIG_ERR_LAYOUT;
    if (plan != VIG_FWD_AUTO && plan != VIG_FWD_FOUR_WAVE && plan != VIG_FWD_WAVE_SPECIALISED &&
        plan != VIG_FWD_SLAB_SWEEP)
        return VIG_ERR_UNSUPPORTED;
    if (B <= 0 || H <= 0 || L <= 0 || dk <= 0 || dv <= 0) return VIG_ERR_SHAPE;
    if (dtype != VIG_F32 && dtype != VIG_BF16) return VIG_ERR_DTYPE;
    if (!head_dim_ok(dk) || !head_dim_ok(dv)) return VIG_ERR_UNSUPPORTED;
    if (!sizes_ok(B, H, L, dk > dv ? dk : dv) || long(B) * H > 0x7fffffffL) return VIG_ERR_SHAPE;
    // token-major offsets inside one batch element are formed in 32 bits (24-bit factors)
    if (layout == VIG_LAYOUT_BLHD &&
        (L >= (1 << 24) || long(H) * 64 >= (1 << 24) || long(L) * H * (dk > dv ? dk : dv) >= (1L << 31)))
        return VIG_ERR_SHAPE;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(g_fwd) || !aligned16(g_bwd) ||
        !aligned16(out) || !aligned16(workspace))
        return VIG_ERR_ALIGN;
    const size_t need = bigla_workspace_bytes(B, H, L, dk, dv, dtype);
    if (need > 0 && (!workspace || workspace_bytes < need)) return VIG_ERR_WORKSPACE;

    const bool bf16 = dtype == VIG_BF16;
    const long BH = long(B) * H;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int heads_token_major = layout == VIG_LAYOUT_BLHD ? H : 0;
    // the chunkwise kernels address the rows of a slab (token-major: of a batch element) with 32-bit
    // byte offsets, up to one chunk past the sequence
    const bool chunkwise = chunkwise_fwd(L, dk, dv, bf16);
    if (chunkwise && !chunk_offsets_ok(L, H, layout)) return VIG_ERR_SHAPE;
    const bool ws = plan == VIG_FWD_WAVE_SPECIALISED;
    if (ws && !(chunkwise && vig::bigla_chunk_ws_selectable(BH, L, dk))) return VIG_ERR_UNSUPPORTED;
    clear_stale_hip_error();
    if (chunkwise)
        return hip_status(
            vig::bigla_chunk_launch(q, k, v, g_fwd, g_bwd, out, BH, L, dk, heads_token_major, nullptr, plan, workspace, s));
    return hip_status(vig::bigla_recurrent_launch(q, k, v, g_fwd, g_bwd, out, BH, L, dk, dv, bf16,
                                                  heads_token_major, workspace, s));
}

int bigla_fwd_static_scratch(const void *q, const void *k, const void *v, const void *g_fwd, const void *g_bwd,
                             void *out, int B, int H, int L, int dk, int dv, int dtype, int layout, void *stream)
{
    // sizes first: an invalid problem reports its own error, a valid one that is too large the limit
    if (B <= 0 || H <= 0 || L <= 0 || dk <= 0 || dv <= 0) return VIG_ERR_SHAPE;
    if (dtype != VIG_F32 && dtype != VIG_BF16) return VIG_ERR_DTYPE;
    if (!head_dim_ok(dk) || !head_dim_ok(dv)) return VIG_ERR_UNSUPPORTED;
    if (!sizes_ok(B, H, L, dk > dv ? dk : dv)) return VIG_ERR_SHAPE;
    if (bigla_workspace_bytes(B, H, L, dk, dv, dtype) > size_t(VIG_STATIC_SCRATCH_BYTES)) return VIG_ERR_SCRATCH_LIMIT;
    void *ws = static_scratch();
    if (!ws) return VIG_ERR_HIP;
    return bigla_fwd_layout(q, k, v, g_fwd, g_bwd, out, B, H, L, dk, dv, dtype, layout, ws,
                            size_t(VIG_STATIC_SCRATCH_BYTES), stream);
}

size_t bigla_bwd_workspace_bytes(int B, int H, int L, int dk, int dv, int dtype)
{
    if (B <= 0 || H <= 0 || L <= 0 || !head_dim_ok(dk) || !head_dim_ok(dv)) return 0;
    if (dtype != VIG_F32 && dtype != VIG_BF16) return 0;
    if (!sizes_ok(B, H, L, 3L * dk + dv)) return 0;
    return vig::bigla_bwd_workspace_bytes(long(B) * H, L, dk, dv, dtype == VIG_BF16);
}

int bigla_bwd(const void *q, const void *k, const void *v, const void *g_fwd, const void *g_bwd, const void *d_out,
              void *dq, void *dk, void *dv, void *dg_fwd, void *dg_bwd, int B, int H, int L, int dk_, int dv_,
              int dtype, int layout, void *workspace, size_t workspace_bytes, void *stream)
{
    return bigla_bwd_plan(q, k, v, g_fwd, g_bwd, d_out, dq, dk, dv, dg_fwd, dg_bwd, B, H, L, dk_, dv_, dtype, layout,
                          VIG_BWD_AUTO, workspace, workspace_bytes, stream);
}

int bigla_bwd_plan(const void *q, const void *k, const void *v, const void *g_fwd, const void *g_bwd,
                   const void *d_out, void *dq, void *dk, void *dv, void *dg_fwd, void *dg_bwd, int B, int H, int L,
                   int dk_, int dv_, int dtype, int layout, int plan, void *workspace, size_t workspace_bytes,
                   void *stream)
{
    if (!q || !k || !v || !g_fwd || !g_bwd || !d_out || !dq || !dk || !dv || !dg_fwd || !dg_bwd) return VIG_ERR_NULL;
    if (layout != VIG_LAYOUT_BHLD && layout != VIG_LAYOUT_BLHD) return VIG_ERR_LAYOUT;
    if (B <= 0 || H <= 0 || L <= 0 || dk_ <= 0 || dv_ <= 0) return VIG_ERR_SHAPE;
    if (dtype != VIG_F32 && dtype != VIG_BF16) return VIG_ERR_DTYPE;
    if (!head_dim_ok(dk_) || !head_dim_ok(dv_)) return VIG_ERR_UNSUPPORTED;
    if (plan != VIG_BWD_AUTO && plan != VIG_BWD_RECURRENT) return VIG_ERR_UNSUPPORTED;
    if (!sizes_ok(B, H, L, 3L * dk_ + dv_) || long(B) * H * 4 > 0x7fffffffL) return VIG_ERR_SHAPE;
    const bool chunkwise = plan == VIG_BWD_AUTO && vig::bigla_bwd_chunk_supported(dk_, dv_, dtype == VIG_BF16);
    if (chunkwise && !chunk_offsets_ok(L, H, layout)) return VIG_ERR_SHAPE;
    if (chunkwise && long(B) * H * ((long(L) + 63) / 64) > 0x7fffffffL) return VIG_ERR_SHAPE;  // a workgroup per chunk
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(g_fwd) || !aligned16(g_bwd) ||
        !aligned16(d_out) || !aligned16(dq) || !aligned16(dk) || !aligned16(dv) || !aligned16(dg_fwd) ||
        !aligned16(dg_bwd) || !aligned16(workspace))
        return VIG_ERR_ALIGN;
    const size_t need = bigla_bwd_workspace_bytes(B, H, L, dk_, dv_, dtype);
    if (!workspace || workspace_bytes < need) return VIG_ERR_WORKSPACE;
    clear_stale_hip_error();
    return hip_status(vig::bigla_bwd_launch(q, k, v, g_fwd, g_bwd, d_out, dq, dk, dv, dg_fwd, dg_bwd, long(B) * H, L,
                                            dk_, dv_, dtype == VIG_BF16, layout == VIG_LAYOUT_BLHD ? H : 0,
                                            plan == VIG_BWD_RECURRENT, workspace, static_cast<hipStream_t>(stream)));
}

int locality_gate_fwd(const void *x, const void *w, const void *bias, const void *gate_logits,
                      const void *o_global, void *out, int B, int H, int Hg, int Wg, int dv, int dtype,
                      void *stream)
{
    return locality_gate_fwd_layout(x, w, bias, gate_logits, o_global, out, B, H, Hg, Wg, dv, dtype,
                                    VIG_LAYOUT_BHLD, stream);
}

int locality_gate_fwd_layout(const void *x, const void *w, const void *bias, const void *gate_logits,
                             const void *o_global, void *out, int B, int H, int Hg, int Wg, int dv, int dtype,
                             int layout, void *stream)
{
    if (!x || !w || !gate_logits || !o_global || !out) return VIG_ERR_NULL;
    if (layout != VIG_LAYOUT_BHLD && layout != VIG_LAYOUT_BLHD) return VIG_ERR_LAYOUT;
    if (B <= 0 || H <= 0 || Hg <= 0 || Wg <= 0 || dv <= 0) return VIG_ERR_SHAPE;
    if (dtype != VIG_F32 && dtype != VIG_BF16) return VIG_ERR_DTYPE;
    if (!head_dim_ok(dv)) return VIG_ERR_UNSUPPORTED;
    if (!sizes_ok(B, H, Hg, long(Wg) * dv) || long(Hg) * Wg > 0x7fffffffL) return VIG_ERR_SHAPE;
    // the pixels of one slab (token-major: of one batch element) are addressed with 32-bit byte offsets
    if (long(Hg) * Wg * (layout == VIG_LAYOUT_BLHD ? H : 1) * dv * (dtype == VIG_BF16 ? 2 : 4) >= 0xffffff00L)
        return VIG_ERR_SHAPE;
    if (!aligned16(x) || !aligned16(w) || !aligned16(bias) || !aligned16(gate_logits) || !aligned16(o_global) ||
        !aligned16(out))
        return VIG_ERR_ALIGN;
    clear_stale_hip_error();
    return hip_status(vig::locality_gate_launch(x, w, bias, gate_logits, o_global, out, B, H, Hg, Wg, dv,
                                                dtype == VIG_BF16, layout == VIG_LAYOUT_BLHD ? 1 : 0,
                                                static_cast<hipStream_t>(stream)));
}

namespace {
size_t align256(size_t n) { return (n + 255) / 256 * 256; }
}  // namespace

size_t bigla_locality_workspace_bytes(int B, int H, int L, int dk, int dv, int dtype, int plan)
{
    if (B <= 0 || H <= 0 || L <= 0 || !head_dim_ok(dk) || !head_dim_ok(dv)) return 0;
    if (dtype != VIG_F32 && dtype != VIG_BF16) return 0;
    if (plan != VIG_PLAN_AUTO && plan != VIG_PLAN_TWO_LAUNCHES && plan != VIG_PLAN_FUSED_EPILOGUE) return 0;
    const size_t mixer = bigla_workspace_bytes(B, H, L, dk, dv, dtype);
    if (plan == VIG_PLAN_FUSED_EPILOGUE)
        return chunkwise_fwd(L, dk, dv, dtype == VIG_BF16) ? vig::bigla_chunk_workspace_bytes(long(B) * H, L) : 0;
    if (!sizes_ok(B, H, L, dv)) return 0;
    // the token mixer's output goes through the workspace
    return align256(mixer) + size_t(B) * H * L * dv * (dtype == VIG_BF16 ? 2 : 4);
}

int bigla_locality_fwd(const void *q, const void *k, const void *v, const void *g_fwd, const void *g_bwd,
                       const void *x, const void *w, const void *bias, const void *gate_logits, void *out, int B,
                       int H, int Hg, int Wg, int dk, int dv, int dtype, int layout, int plan, void *workspace,
                       size_t workspace_bytes, void *stream)
{
    if (!q || !k || !v || !g_fwd || !g_bwd || !x || !w || !gate_logits || !out) return VIG_ERR_NULL;
    if (layout != VIG_LAYOUT_BHLD && layout != VIG_LAYOUT_BLHD) return VIG_ERR_LAYOUT;
    if (plan != VIG_PLAN_AUTO && plan != VIG_PLAN_TWO_LAUNCHES && plan != VIG_PLAN_FUSED_EPILOGUE)
        return VIG_ERR_UNSUPPORTED;
    if (B <= 0 || H <= 0 || Hg <= 0 || Wg <= 0 || dk <= 0 || dv <= 0) return VIG_ERR_SHAPE;
    if (long(Hg) * Wg >= (1L << 24)) return VIG_ERR_SHAPE;
    const int L = Hg * Wg;
    if (dtype != VIG_F32 && dtype != VIG_BF16) return VIG_ERR_DTYPE;
    if (!head_dim_ok(dk) || !head_dim_ok(dv)) return VIG_ERR_UNSUPPORTED;
    const bool bf16 = dtype == VIG_BF16;
    if (plan != VIG_PLAN_FUSED_EPILOGUE) {
        // the token mixer into the workspace, then the locality kernel (both validate their arguments)
        const size_t mixer = align256(bigla_workspace_bytes(B, H, L, dk, dv, dtype));
        const size_t need = bigla_locality_workspace_bytes(B, H, L, dk, dv, dtype, plan);
        if (need == 0) return VIG_ERR_SHAPE;
        if (!workspace || workspace_bytes < need) return VIG_ERR_WORKSPACE;
        if (!aligned16(workspace)) return VIG_ERR_ALIGN;
        void *o_global = static_cast<unsigned char *>(workspace) + mixer;
        const int st = bigla_fwd_layout(q, k, v, g_fwd, g_bwd, o_global, B, H, L, dk, dv, dtype, layout, workspace,
                                        mixer, stream);
        if (st != VIG_OK) return st;
        return locality_gate_fwd_layout(x, w, bias, gate_logits, o_global, out, B, H, Hg, Wg, dv, dtype, layout,
                                        stream);
    }
    // the epilogue lives in the chunkwise kernels; shorter sequences are left to the exact recurrence
    if (!chunkwise_fwd(L, dk, dv, bf16)) return VIG_ERR_UNSUPPORTED;
    if (!sizes_ok(B, H, L, dk > dv ? dk : dv) || long(B) * H > 0x7fffffffL) return VIG_ERR_SHAPE;
    if (!chunk_offsets_ok(L, H, layout)) return VIG_ERR_SHAPE;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(g_fwd) || !aligned16(g_bwd) ||
        !aligned16(x) || !aligned16(w) || !aligned16(bias) || !aligned16(gate_logits) || !aligned16(out) ||
        !aligned16(workspace))
        return VIG_ERR_ALIGN;
    const size_t need = vig::bigla_chunk_workspace_bytes(long(B) * H, L);
    if (need > 0 && (!workspace || workspace_bytes < need)) return VIG_ERR_WORKSPACE;
    const vig::LocalityFusion fusion = {x, w, bias, gate_logits, H, Hg, Wg};
    clear_stale_hip_error();
    return hip_status(vig::bigla_chunk_launch(q, k, v, g_fwd, g_bwd, out, long(B) * H, L, dk,
                                              layout == VIG_LAYOUT_BLHD ? H : 0, &fusion, VIG_FWD_AUTO, workspace,
                                              static_cast<hipStream_t>(stream)));
}

int gate_producer_fwd(const void *x, const void *w1, const void *w2, const void *bias, void *g_fwd, void *g_bwd,
                      int B, int H, int L, int D, int dk, float tau, int dtype, int layout, void *stream)
{
    if (!x || !w1 || !w2 || !g_fwd || !g_bwd) return VIG_ERR_NULL;
    if (layout != VIG_LAYOUT_BHLD && layout != VIG_LAYOUT_BLHD) return VIG_ERR_LAYOUT;
    if (B <= 0 || H <= 0 || L <= 0 || D <= 0 || dk <= 0 || !(tau > 0.f)) return VIG_ERR_SHAPE;
    if (dtype != VIG_F32 && dtype != VIG_BF16) return VIG_ERR_DTYPE;
    if (!head_dim_ok(dk) || !vig::gate_producer_width_ok(D, dtype == VIG_BF16)) return VIG_ERR_UNSUPPORTED;
    if (!sizes_ok(B, L, D, 1) || !sizes_ok(B, L, H, 2 * dk) || long(H) * dk > (1 << 20)) return VIG_ERR_SHAPE;
    if (!aligned16(x) || !aligned16(w1) || !aligned16(w2) || !aligned16(bias) || !aligned16(g_fwd) ||
        !aligned16(g_bwd))
        return VIG_ERR_ALIGN;
    clear_stale_hip_error();
    return hip_status(vig::gate_producer_launch(x, w1, w2, bias, g_fwd, g_bwd, B, H, L, D, dk, tau,
                                                dtype == VIG_BF16, layout == VIG_LAYOUT_BLHD ? 1 : 0,
                                                static_cast<hipStream_t>(stream)));
}

namespace {
size_t round256(size_t n) { return (n + 255) / 256 * 256; }
}  // namespace

size_t gated_bigla_workspace_bytes(int B, int H, int L, int dk, int dv, int dtype)
{
    if (B <= 0 || H <= 0 || L <= 0 || !head_dim_ok(dk) || !head_dim_ok(dv)) return 0;
    if (dtype != VIG_F32 && dtype != VIG_BF16) return 0;
    // the mixer's workspace, then the low-rank product (bf16 [B][L][16])
    return round256(bigla_workspace_bytes(B, H, L, dk, dv, dtype)) + round256(size_t(B) * L * 16 * 2);
}

int gated_bigla_fwd(const void *x, const void *w1, const void *w2, const void *bias, const void *q, const void *k,
                    const void *v, void *g_fwd, void *g_bwd, void *out, int B, int H, int L, int D, int dk, int dv,
                    float tau, int dtype, int layout, int plan, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!x || !w1 || !w2 || !q || !k || !v || !g_fwd || !g_bwd || !out) return VIG_ERR_NULL;
    if (layout != VIG_LAYOUT_BHLD && layout != VIG_LAYOUT_BLHD) return VIG_ERR_LAYOUT;
    if (plan != VIG_GATES_AUTO && plan != VIG_GATES_SEPARATE && plan != VIG_GATES_IN_STATE_PASS) return VIG_ERR_UNSUPPORTED;
    if (B <= 0 || H <= 0 || L <= 0 || D <= 0 || dk <= 0 || dv <= 0 || !(tau > 0.f)) return VIG_ERR_SHAPE;
    if (dtype != VIG_F32 && dtype != VIG_BF16) return VIG_ERR_DTYPE;
    if (!head_dim_ok(dk) || !head_dim_ok(dv) || !vig::gate_producer_width_ok(D, dtype == VIG_BF16)) return VIG_ERR_UNSUPPORTED;
    if (!sizes_ok(B, L, D, 1) || !sizes_ok(B, L, H, 2 * dk) || !sizes_ok(B, H, L, dk > dv ? dk : dv) ||
        long(H) * dk > (1 << 20))
        return VIG_ERR_SHAPE;
    const size_t need = gated_bigla_workspace_bytes(B, H, L, dk, dv, dtype);
    if (!workspace || workspace_bytes < need) return VIG_ERR_WORKSPACE;
    if (!aligned16(workspace)) return VIG_ERR_ALIGN;
    const bool bf16 = dtype == VIG_BF16;
    const long BH = long(B) * H;
    const bool fusable = chunkwise_fwd(L, dk, dv, bf16) && vig::bigla_chunk_gated_selectable(BH, L, dk) &&
                         chunk_offsets_ok(L, H, layout);
    if (plan == VIG_GATES_IN_STATE_PASS && !fusable) return VIG_ERR_UNSUPPORTED;
    const size_t mixer_bytes = round256(bigla_workspace_bytes(B, H, L, dk, dv, dtype));
    if (plan == VIG_GATES_SEPARATE || !fusable) {
        const int st = gate_producer_fwd(x, w1, w2, bias, g_fwd, g_bwd, B, H, L, D, dk, tau, dtype, layout, stream);
        if (st != VIG_OK) return st;
        return bigla_fwd_layout(q, k, v, g_fwd, g_bwd, out, B, H, L, dk, dv, dtype, layout, workspace, mixer_bytes, stream);
    }
    // the checks the two separate entry points make
    if (layout == VIG_LAYOUT_BLHD &&
        (L >= (1 << 24) || long(H) * 64 >= (1 << 24) || long(L) * H * (dk > dv ? dk : dv) >= (1L << 31)))
        return VIG_ERR_SHAPE;
    if (!aligned16(x) || !aligned16(w1) || !aligned16(w2) || !aligned16(bias) || !aligned16(q) || !aligned16(k) ||
        !aligned16(v) || !aligned16(g_fwd) || !aligned16(g_bwd) || !aligned16(out))
        return VIG_ERR_ALIGN;
    hipStream_t s = static_cast<hipStream_t>(stream);
    void *lowrank = static_cast<unsigned char *>(workspace) + mixer_bytes;
    clear_stale_hip_error();
    const hipError_t e = vig::gate_lowrank_launch(x, w1, lowrank, B, L, D, s);
    if (e != hipSuccess) return hip_status(e);
    return hip_status(vig::bigla_chunk_gated_launch(q, k, v, g_fwd, g_bwd, out, BH, L, dk, H,
                                                    layout == VIG_LAYOUT_BLHD ? H : 0, lowrank, w2, bias, tau, workspace, s));
}

const char *vig_status_str(int status)
{
    switch (status) {
        case VIG_OK: return "VIG_OK";
        case VIG_ERR_NULL: return "VIG_ERR_NULL: a required pointer is NULL";
        case VIG_ERR_SHAPE: return "VIG_ERR_SHAPE: a size is <= 0 or too large";
        case VIG_ERR_DTYPE: return "VIG_ERR_DTYPE: dtype is not VIG_F32 or VIG_BF16";
        case VIG_ERR_UNSUPPORTED:
            return "VIG_ERR_UNSUPPORTED: head widths must be 16, 32 or 64 (model width a multiple of 32); plan a vig_plan "
                   "the shape admits";
        case VIG_ERR_ALIGN: return "VIG_ERR_ALIGN: a pointer is not 16-byte aligned";
        case VIG_ERR_WORKSPACE: return "VIG_ERR_WORKSPACE: workspace missing or too small";
        case VIG_ERR_HIP: return "VIG_ERR_HIP: a HIP call failed (see vig_last_hip_error)";
        case VIG_ERR_LAYOUT: return "VIG_ERR_LAYOUT: layout is not a vig_layout";
        case VIG_ERR_SCRATCH_LIMIT:
            return "VIG_ERR_SCRATCH_LIMIT: the problem needs more scratch than the library's static buffer "
                   "(VIG_STATIC_SCRATCH_BYTES) holds";
    }
    return "unknown vig_status";
}

int vig_last_hip_error(void) { return g_last_hip_error; }

}  // extern "C"
