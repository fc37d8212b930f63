// Chunkwise bf16 MFMA evaluation of BiGLA (Section 4.2.1, Eq. (BiGLA)) for dk = dv = 64.
//
// The recurrence S_t = diag(alpha_t) S_{t-1} + k_t^T v_t, o_t = q_t S_t is regrouped exactly
// (no approximation beyond bf16 operand rounding) over chunks of 64 tokens.  With b_t the
// cumulative log-gate inside a chunk,
//   o_t = sum_{i<=t, same chunk} (sum_c q_tc k_ic exp(b_tc - b_ic)) v_i   (intra-chunk, masked)
//       + (q_t * exp(b_t)) S_in                                           (inter-chunk readout)
//   S_out = diag(exp(b_end)) S_in + sum_i (k_i * exp(b_end - b_i))^T v_i  (state passing)
// and the backward direction is the mirror image (suffix sums, keys to the right).  Every
// contraction runs on v_mfma_f32_16x16x32_bf16 with fp32 accumulation; the carried state stays
// fp32 in accumulator registers and only its readout copy is rounded to bf16.
//
// Numerical range -- two evaluations of a chunk, chosen per chunk from the gates themselves.
//   FAST.  With b_t the cumulative log-gate since the chunk edge, queries are scaled by
//   exp(b_t) and keys by exp(-b_i); one key tile then serves the masked scores AND the state
//   update, S_out = diag(exp(b_end)) (S_in + sum_i (k_i exp(-b_i))^T v_i), and one query tile
//   serves the scores AND the readout.  exp(-b_i) grows with the decay accumulated over the
//   chunk, so this form is used only when the chunk's total log-decay provably stays within
//   60 nats in every channel (the sum over its four 16-token sub-blocks of the largest
//   per-channel sub-block total is checked).  Gates of the paper's form, sigmoid(z)^(1/16),
//   stay far inside: 64 steps reach 60 nats only for z < -15 throughout.
//   RANGE-SAFE.  Otherwise cumulative gates stay local to a sub-block: off-diagonal 16x16 tiles
//   scale keys by the decay to the END of the key's own sub-block and queries by the decay from
//   the START of the query's sub-block times the whole-sub-block factors in between, so every
//   factor is <= 1 and underflow to 0 is the correct limit.  The diagonal tile refers both
//   sides to the MIDDLE of the sub-block, so its factors span at most 8 steps in either sense;
//   the per-step log-gate is floored at -8 there (alpha >= 3.4e-4; anything smaller is a hard
//   reset whose leak is far below the bf16 tolerance), which keeps them within e^(+-64).
// Masking is by select, never by multiplying with 0.
//
// Parallel decomposition.  A sequence is cut into segments of kSegChunks chunks.
//   1. bigla_segment_state_kernel : one workgroup per (slab, segment) computes, for BOTH
//      directions in one pass over k, v, g, the segment's local end state and total decay.
//   2. bigla_state_scan_kernel    : per state element, the sequential scan over segments in
//      both directions turns local states into the states ENTERING each segment (in place).
//   3. bigla_segment_out_kernel   : one workgroup per (slab, segment) sweeps its chunks
//      left-to-right for the forward direction and right-to-left for the backward direction,
//      holding the fp32 output tiles in registers between the sweeps, and writes
//      (o_fwd + o_bwd)/2 once.  Sequences of at most one segment need only this launch.
// Nothing is reversed or copied in HBM; both directions read the same q, k, v.
//
// Wavefront mapping (256 threads = 4 waves).  Wave w owns tokens [16w, 16w+16) of the chunk;
// lane (r = lane%16, g = lane/16) holds 16 channels of token 16w + r.  Slot n = 4*ct + e of the
// lane is channel 16*ct + 4g + e: that is the accumulator layout in which the cumulative gates
// leave the matrix cores (below), and slots 8kk..8kk+7 are the lane's k-slots of K-step kk of
// every contraction over channels (A and B operands of the 16x16x32 MFMA only have to agree on
// the channel of each k-slot).  LDS tiles of scaled keys and states keep channels in that
// operand order (position 32kk + 8g + slot%8), as does the segment-state workspace; only the
// global loads of q and k see the permutation.  Contractions over tokens (P.V, the state
// update, the gate scan) take their token-major operands from row-major LDS tiles through
// ds_read_b64_tr_b16.
//
// Cumulative gates on the matrix cores.  The chunk-level cumulative log-gate is a product with
// a triangular 0/1 matrix, B^T[c][t] = sum_i g[i][c] * [i <= t] (or [i >= t] backward), which
// is exact in bf16 x bf16 -> fp32.  Two K-steps of the MFMA per 16-channel tile replace the
// wavefront prefix scans, the cross-sub-block offsets and every unpack of g on the vector
// ALUs, which are the scarce unit on this path; a second product with the all-ones matrix gives
// every lane the chunk totals of its channels (state decay, choice of the form).  The
// range-safe form still scans its sub-block-local, floored gates with DPP row operations.
#include "vig_common.hpp"
#include "vig_kernels.hpp"
#include "vig_timing.hpp"

namespace vig {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) short s16x4;

constexpr int kC = 64;          // chunk length (tokens)
constexpr int kD = 64;          // dk = dv
constexpr int kPitch = 72;      // LDS row pitch in bf16 elements (64 + 8: 16-byte aligned, bank-staggered)
constexpr int kSegChunks = 4;   // chunks per segment (ring of output tiles held in registers)
constexpr int kThreads = 256;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kGateFloorLog2 = -8.0f * kLog2e;  // per-step floor of the log-gate (range-safe form), log2 domain
constexpr float kFastRange = 60.0f;  // largest chunk log-decay (nats, any channel) the fast form accepts

// ---- small device helpers ------------------------------------------------------------------

template <int CTRL>
__device__ __forceinline__ float dpp_or_zero(float x)
{
    // lanes whose DPP source falls outside the 16-lane row receive 0
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xf, 0xf, false));
}

// Inclusive scan over the 16 lanes of a DPP row: prefix (DIR 0) or suffix (DIR 1).
template <int DIR>
__device__ __forceinline__ float row_scan(float x)
{
    if (DIR == 0) {
        x += dpp_or_zero<0x111>(x);  // row_shr:1
        x += dpp_or_zero<0x112>(x);
        x += dpp_or_zero<0x114>(x);
        x += dpp_or_zero<0x118>(x);
    } else {
        x += dpp_or_zero<0x101>(x);  // row_shl:1
        x += dpp_or_zero<0x102>(x);
        x += dpp_or_zero<0x104>(x);
        x += dpp_or_zero<0x108>(x);
    }
    return x;
}

// Row-wide broadcasts (row_newbcast:n).  In scan order the far-edge lane holds the sub-block
// total (lane 15 for the prefix scan, lane 0 for the suffix scan); the middle lane is the last
// lane of the first half in scan order (lane 7 / lane 8).
template <int DIR>
__device__ __forceinline__ float bcast_far(float x)
{
    return DIR == 0 ? dpp_or_zero<0x15f>(x) : dpp_or_zero<0x150>(x);
}
template <int DIR>
__device__ __forceinline__ float bcast_mid(float x)
{
    return DIR == 0 ? dpp_or_zero<0x157>(x) : dpp_or_zero<0x158>(x);
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ uint32_t pack2(float lo, float hi)
{
    f32x2 a = {lo, hi};
    bf16x2 b = __builtin_convertvector(a, bf16x2);  // v_cvt_pk_bf16_f32, round to nearest even
    return __builtin_bit_cast(uint32_t, b);
}

__device__ __forceinline__ bf16x8 pack8(const float *f)
{
    uint4 u;
    u.x = pack2(f[0], f[1]);
    u.y = pack2(f[2], f[3]);
    u.z = pack2(f[4], f[5]);
    u.w = pack2(f[6], f[7]);
    return __builtin_bit_cast(bf16x8, u);
}

__device__ __forceinline__ void unpack8(const uint4 &u, float *f)
{
    f[0] = bf16_lo_to_f32(u.x); f[1] = bf16_hi_to_f32(u.x);
    f[2] = bf16_lo_to_f32(u.y); f[3] = bf16_hi_to_f32(u.y);
    f[4] = bf16_lo_to_f32(u.z); f[5] = bf16_hi_to_f32(u.z);
    f[6] = bf16_lo_to_f32(u.w); f[7] = bf16_hi_to_f32(u.w);
}

__device__ __forceinline__ f32x4 mfma(bf16x8 a, bf16x8 b, f32x4 c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}

// Transposing LDS read: the 16 lanes of a row fetch a 4 (tokens) x 16 (columns) bf16 patch of a
// row-major tile; lane n of the row receives the 4 tokens of column n.  Lane n supplies the
// address of token n/4, columns 4*(n%4).. of the patch.
__device__ __forceinline__ s16x4 lds_read_tr(const uint16_t *p)
{
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3))) *)(p));
}

__device__ __forceinline__ bf16x8 join(s16x4 lo, s16x4 hi)
{
    typedef __attribute__((ext_vector_type(8))) short s16x8;
    s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, v);
}

// 16 bf16 values of one token held by a lane, packed two per dword
struct Row16 {
    uint4 p[2];
};

// Natural order: two 16-byte pieces at channel offsets 8g and 32+8g (tiles that are only staged)
__device__ __forceinline__ Row16 load_row_natural(const uint16_t *slab_base, long token, bool valid, int g)
{
    Row16 r;
    if (valid) {
        const uint4 *p = reinterpret_cast<const uint4 *>(slab_base + token * kD + 8 * g);
        r.p[0] = p[0];
        r.p[1] = p[4];  // +32 elements
    } else {
        r.p[0] = make_uint4(0, 0, 0, 0);
        r.p[1] = make_uint4(0, 0, 0, 0);
    }
    return r;
}

// Operand order: slot n = 4*ct + e holds channel 16*ct + 4g + e (four 8-byte pieces)
__device__ __forceinline__ Row16 load_row_operand(const uint16_t *slab_base, long token, bool valid, int g)
{
    Row16 r;
    if (valid) {
        const uint2 *p = reinterpret_cast<const uint2 *>(slab_base + token * kD + 4 * g);
        const uint2 a = p[0], b = p[4], c = p[8], d = p[12];  // +16 elements each
        r.p[0] = make_uint4(a.x, a.y, b.x, b.y);
        r.p[1] = make_uint4(c.x, c.y, d.x, d.y);
    } else {
        r.p[0] = make_uint4(0, 0, 0, 0);
        r.p[1] = make_uint4(0, 0, 0, 0);
    }
    return r;
}

// The same 16 slots of one token out of a natural-order LDS tile
__device__ __forceinline__ Row16 lds_row_operand(const uint16_t (*tile)[kPitch], int row, int g)
{
    const uint2 a = *reinterpret_cast<const uint2 *>(&tile[row][4 * g]);
    const uint2 b = *reinterpret_cast<const uint2 *>(&tile[row][16 + 4 * g]);
    const uint2 c = *reinterpret_cast<const uint2 *>(&tile[row][32 + 4 * g]);
    const uint2 d = *reinterpret_cast<const uint2 *>(&tile[row][48 + 4 * g]);
    Row16 r;
    r.p[0] = make_uint4(a.x, a.y, b.x, b.y);
    r.p[1] = make_uint4(c.x, c.y, d.x, d.y);
    return r;
}

__device__ __forceinline__ void unpack16(const Row16 &r, float (&f)[16])
{
    unpack8(r.p[0], f);
    unpack8(r.p[1], f + 8);
}

__device__ __forceinline__ void store_row16(uint16_t (*tile)[kPitch], int row, int g, const float (&f)[16])
{
    uint4 a, b;
    a.x = pack2(f[0], f[1]); a.y = pack2(f[2], f[3]); a.z = pack2(f[4], f[5]); a.w = pack2(f[6], f[7]);
    b.x = pack2(f[8], f[9]); b.y = pack2(f[10], f[11]); b.z = pack2(f[12], f[13]); b.w = pack2(f[14], f[15]);
    *reinterpret_cast<uint4 *>(&tile[row][8 * g]) = a;
    *reinterpret_cast<uint4 *>(&tile[row][32 + 8 * g]) = b;
}

__device__ __forceinline__ void store_row16_raw(uint16_t (*tile)[kPitch], int row, int g, const Row16 &r)
{
    *reinterpret_cast<uint4 *>(&tile[row][8 * g]) = r.p[0];
    *reinterpret_cast<uint4 *>(&tile[row][32 + 8 * g]) = r.p[1];
}

// the lane's 16 channels of a per-channel fp32 vector in LDS
__device__ __forceinline__ void load_chan16(const float *vec, int g, float (&f)[16])
{
    const float4 *a = reinterpret_cast<const float4 *>(vec + 8 * g);
    const float4 *b = reinterpret_cast<const float4 *>(vec + 32 + 8 * g);
    float4 t;
    t = a[0]; f[0] = t.x; f[1] = t.y; f[2] = t.z; f[3] = t.w;
    t = a[1]; f[4] = t.x; f[5] = t.y; f[6] = t.z; f[7] = t.w;
    t = b[0]; f[8] = t.x; f[9] = t.y; f[10] = t.z; f[11] = t.w;
    t = b[1]; f[12] = t.x; f[13] = t.y; f[14] = t.z; f[15] = t.w;
}

__device__ __forceinline__ void store_chan16(float *vec, int g, const float (&f)[16])
{
    float4 *a = reinterpret_cast<float4 *>(vec + 8 * g);
    float4 *b = reinterpret_cast<float4 *>(vec + 32 + 8 * g);
    a[0] = make_float4(f[0], f[1], f[2], f[3]);
    a[1] = make_float4(f[4], f[5], f[6], f[7]);
    b[0] = make_float4(f[8], f[9], f[10], f[11]);
    b[1] = make_float4(f[12], f[13], f[14], f[15]);
}

// Logical order of the four sub-blocks as seen from sub-block w in direction DIR:
// slot 0 = w itself, slots 1..nb = the sub-blocks whose keys w's queries see (nearest first),
// remaining slots = the sub-blocks after w (nearest first).
template <int DIR>
struct SubOrder {
    int w, nb;
    __device__ __forceinline__ explicit SubOrder(int w_) : w(w_), nb(DIR == 0 ? w_ : 3 - w_) {}
    __device__ __forceinline__ int before(int d) const { return DIR == 0 ? w - d : w + d; }  // 1 <= d <= nb
    __device__ __forceinline__ int after(int a) const { return DIR == 0 ? w + a : w - a; }   // 1 <= a <= 3-nb
    __device__ __forceinline__ int slot(int s) const { return s == 0 ? w : (s <= nb ? before(s) : after(s - nb)); }
};

// Range-safe form: cumulative log2-gates of the lane's 16 channels inside its sub-block,
// inclusive of the lane's own token, in scan order (prefix for DIR 0, suffix for DIR 1); every
// step floored at kGateFloorLog2 and capped at 0 (alpha <= 1).
template <int DIR>
__device__ __forceinline__ void gate_scan(const Row16 &graw, float (&b)[16])
{
    unpack16(graw, b);
#pragma unroll
    for (int e = 0; e < 16; ++e)
        b[e] = row_scan<DIR>(__builtin_amdgcn_fmed3f(b[e] * kLog2e, kGateFloorLog2, 0.f));
}

// Gate factors of the output sweep for the lane's token t and 16 channels, with B_mid the
// cumulative gate at the middle lane and B_tot the sub-block total:
//   X    = exp(b_t - B_mid)      Y = 1/X = exp(B_mid - b_t)       (diagonal tile: q*X, k*Y)
//   F    = exp(B_tot - b_t)      decay from t (exclusive) to the far edge      (keys, <= 1)
//   Emid = exp(B_mid)            so that exp(b_t) = X * Emid                    (queries, <= 1)
//   EB   = exp(B_tot)            whole-sub-block decay
// Two transcendentals per element: the middle lane's own Y is 1 by definition, so its slot of
// the second exp2 evaluates Emid instead, which a row broadcast then hands to every lane.
template <int DIR>
__device__ __forceinline__ void gate_factors(const Row16 &graw, int r, float (&X)[16], float (&Y)[16],
                                             float (&F)[16], float (&Emid)[16], float (&EB)[16])
{
    float b[16];
    gate_scan<DIR>(graw, b);
    const bool is_mid = r == (DIR == 0 ? 7 : 8);
#pragma unroll
    for (int e = 0; e < 16; ++e) {
        const float xa = b[e] - bcast_mid<DIR>(b[e]);
        X[e] = fast_exp2(xa);
        const float yraw = fast_exp2(is_mid ? b[e] : -xa);
        Emid[e] = bcast_mid<DIR>(yraw);
        Y[e] = is_mid ? 1.f : yraw;
        const float xfar = bcast_far<DIR>(X[e]);
        F[e] = Y[e] * xfar;
        EB[e] = Emid[e] * xfar;
    }
}

// Gate factors of the state pass: F and EB only.
template <int DIR>
__device__ __forceinline__ void gate_factors_state(const Row16 &graw, float (&F)[16], float (&EB)[16])
{
    float b[16];
    gate_scan<DIR>(graw, b);
#pragma unroll
    for (int e = 0; e < 16; ++e) {
        const float btot = bcast_far<DIR>(b[e]);
        F[e] = fast_exp2(btot - b[e]);
        EB[e] = fast_exp2(btot);
    }
}

// ---- shared memory ---------------------------------------------------------------------------

struct __align__(16) OutLds {
    uint16_t kt[kC][kPitch];   // scaled keys                  [token][channel, operand order]
    uint16_t ks[kC][kPitch];   // range-safe form only: keys scaled for the state update, same layout
    uint16_t g[kC][kPitch];    // raw log-gates of the sweep's direction [token][channel, natural order]
    uint16_t v[kC][kPitch];    // values                       [token][column]
    uint16_t st[kD][kPitch];   // carried state, bf16 copy     [column][channel, operand order]
    float tot[kD];             // chunk total log-gate per channel (fast form), operand order
    float eb[4][kD];           // whole-sub-block decay factors per channel (range-safe form)
};

struct __align__(16) StateLds {
    uint16_t ks[2][kC][kPitch];
    uint16_t g[2][kC][kPitch];
    uint16_t v[kC][kPitch];
    float tot[2][kD];
    float eb[2][4][kD];
};

// Workspace layout per (slab, segment): two fp32 64x64 states then two fp32 decay vectors.
constexpr size_t kSegStateFloats = 2 * size_t(kD) * kD;
constexpr size_t kSegFloats = kSegStateFloats + 2 * kD;

// Token-major MFMA operands of a 64-token tile for contractions over tokens.  k-slot layout:
// slots 0..3 = tokens 4g..4g+3 of sub-block s0, slots 4..7 = the same tokens of sub-block s1.
__device__ __forceinline__ bf16x8 token_operand(const uint16_t (*tile)[kPitch], int s0, int s1, int col0, int r,
                                                int g)
{
    const int tr_row = 4 * g + (r >> 2), tr_col = col0 + 4 * (r & 3);
    return join(lds_read_tr(&tile[16 * s0 + tr_row][tr_col]), lds_read_tr(&tile[16 * s1 + tr_row][tr_col]));
}

__device__ __forceinline__ uint2 pack4(const f32x4 &p) { return make_uint2(pack2(p[0], p[1]), pack2(p[2], p[3])); }

// The lane's column of the triangular 0/1 matrix of the gate scan, as the B operand of the two
// K-steps over the chunk's tokens: slot s of step p is token i = 16*(2p + s/4) + 4g + s%4 and
// holds 1 when token i contributes to the cumulative gate of the lane's own token t = 16w + r,
// i.e. i <= t forward, i >= t backward.
template <int DIR>
__device__ __forceinline__ void scan_triangle(int w, int r, int g, bf16x8 (&tri)[2])
{
    const int t = 16 * w + r;
#pragma unroll
    for (int p = 0; p < 2; ++p) {
        uint32_t word[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            uint32_t bits = 0;
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                const int slot = 2 * j + half;
                const int i = 16 * (2 * p + slot / 4) + 4 * g + slot % 4;
                const bool one = DIR == 0 ? (i <= t) : (i >= t);
                bits |= (one ? 0x3F80u : 0u) << (16 * half);
            }
            word[j] = bits;
        }
        tri[p] = __builtin_bit_cast(bf16x8, make_uint4(word[0], word[1], word[2], word[3]));
    }
}

// Cumulative log-gates of the chunk on the matrix cores (natural-log units): B[ct][e] is the
// inclusive cumulative gate, since the chunk edge of the direction, of channel 16ct + 4g + e
// (slot 4ct + e) at the lane's own token; T[ct][e] is the chunk total of the same channel.
__device__ __forceinline__ void chunk_gate_scan(const uint16_t (*gtile)[kPitch], const bf16x8 (&tri)[2], int r, int g,
                                                f32x4 (&B)[4], f32x4 (&T)[4])
{
    const bf16x8 ones = __builtin_bit_cast(bf16x8, make_uint4(0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u));
#pragma unroll
    for (int ct = 0; ct < 4; ++ct) {
        const bf16x8 a0 = token_operand(gtile, 0, 1, 16 * ct, r, g);
        const bf16x8 a1 = token_operand(gtile, 2, 3, 16 * ct, r, g);
        const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
        B[ct] = mfma(a1, tri[1], mfma(a0, tri[0], zero));
        T[ct] = mfma(a1, ones, mfma(a0, ones, zero));
    }
}

// Largest chunk log-decay (nats) over all 64 channels, identical in every lane of the wave: the
// four lanes 0, 16, 32, 48 together hold the totals of every channel.
__device__ __forceinline__ float chunk_decay_max(const f32x4 (&T)[4])
{
    float m = 0.f;
#pragma unroll
    for (int ct = 0; ct < 4; ++ct)
#pragma unroll
        for (int e = 0; e < 4; ++e) m = fminf(m, T[ct][e]);
    const float m0 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(m), 0));
    const float m1 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(m), 16));
    const float m2 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(m), 32));
    const float m3 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(m), 48));
    return -fminf(fminf(m0, m1), fminf(m2, m3));
}

// Diagonal 16x16 score tile, transposed (lane: keys 4g..4g+3, query r): keep key <= query for
// the forward direction, key >= query for the backward one (own token in both).
template <int DIR>
__device__ __forceinline__ uint2 masked_diag(f32x4 p, int r, int g)
{
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const int i = 4 * g + e;
        const bool keep = DIR == 0 ? (i <= r) : (i >= r);
        p[e] = keep ? p[e] : 0.f;
    }
    return pack4(p);
}

// O^T += V^T.P^T over the visible sub-blocks, then the readout S^T.q^T of the incoming state.
// Computed transposed so that the accumulators are token-per-lane: lane (r, g) ends up with
// columns 16*jt + 4g .. +3 of its own token 16w + r.
__device__ __forceinline__ void accumulate_output(const OutLds &sm, const uint2 (&pk)[4], bool second_pair,
                                                  const bf16x8 (&vop)[2][4], bf16x8 qr0, bf16x8 qr1, int r, int g,
                                                  f32x4 (&O)[4])
{
    const bf16x8 pa0 = __builtin_bit_cast(bf16x8, make_uint4(pk[0].x, pk[0].y, pk[1].x, pk[1].y));
#pragma unroll
    for (int jt = 0; jt < 4; ++jt) O[jt] = mfma(vop[0][jt], pa0, O[jt]);
    if (second_pair) {
        const bf16x8 pa1 = __builtin_bit_cast(bf16x8, make_uint4(pk[2].x, pk[2].y, pk[3].x, pk[3].y));
#pragma unroll
        for (int jt = 0; jt < 4; ++jt) O[jt] = mfma(vop[1][jt], pa1, O[jt]);
    }
#pragma unroll
    for (int jt = 0; jt < 4; ++jt) {
        const bf16x8 b0 = *reinterpret_cast<const bf16x8 *>(&sm.st[16 * jt + r][8 * g]);
        const bf16x8 b1 = *reinterpret_cast<const bf16x8 *>(&sm.st[16 * jt + r][32 + 8 * g]);
        O[jt] = mfma(b0, qr0, O[jt]);
        O[jt] = mfma(b1, qr1, O[jt]);
    }
}

// bf16 copy of the carried state for the next readout, [column][channel]
__device__ __forceinline__ void publish_state(OutLds &sm, int w, int r, int g, const f32x4 (&S)[4])
{
#pragma unroll
    for (int jt = 0; jt < 4; ++jt)
        *reinterpret_cast<uint2 *>(&sm.st[16 * jt + r][16 * w + 4 * g]) = pack4(S[jt]);
}

// ---- kernel 3: per-segment output sweep -------------------------------------------------------

// FAST form of one chunk of one direction (see the header).  B / T are the lane's cumulative and
// total log-gates from chunk_gate_scan; sm.v holds the chunk's values.
template <int DIR>
__device__ __forceinline__ void out_chunk_fast(OutLds &sm, const SubOrder<DIR> &ord, const int w, const int r,
                                               const int g, const f32x4 (&B)[4], const f32x4 (&T)[4],
                                               const Row16 &qraw, const Row16 &kraw, f32x4 (&O)[4], f32x4 (&S)[4])
{
    const int row = 16 * w + r;
    if (r == 0) {  // chunk totals per channel, operand order, for the state decay below
        float t[16];
#pragma unroll
        for (int n = 0; n < 16; ++n) t[n] = T[n >> 2][n & 3];
        store_chan16(sm.tot, g, t);
    }
    float qf[16], kf[16];
    unpack16(qraw, qf);
    unpack16(kraw, kf);
#pragma unroll
    for (int n = 0; n < 16; ++n) {
        const float x = B[n >> 2][n & 3] * kLog2e;
        qf[n] *= fast_exp2(x);   // q * exp(b_t)
        kf[n] *= fast_exp2(-x);  // k * exp(-b_i)
    }
    const bf16x8 q0 = pack8(qf), q1 = pack8(qf + 8);
    const bf16x8 k0 = pack8(kf), k1 = pack8(kf + 8);
    *reinterpret_cast<bf16x8 *>(&sm.kt[row][8 * g]) = k0;
    *reinterpret_cast<bf16x8 *>(&sm.kt[row][32 + 8 * g]) = k1;

    __syncthreads();  // kt, tot visible

    // intra-chunk scores, transposed: P^T[i][t] = sum_c kt[i][c] * qt[t][c]
    uint2 pk[4];
    {
        f32x4 p = {0.f, 0.f, 0.f, 0.f};
        p = mfma(k0, q0, p);
        p = mfma(k1, q1, p);
        pk[0] = masked_diag<DIR>(p, r, g);
    }
#pragma unroll
    for (int d = 1; d <= 3; ++d) {
        if (d <= ord.nb) {
            const int kb = ord.before(d);
            const bf16x8 a0 = *reinterpret_cast<const bf16x8 *>(&sm.kt[16 * kb + r][8 * g]);
            const bf16x8 a1 = *reinterpret_cast<const bf16x8 *>(&sm.kt[16 * kb + r][32 + 8 * g]);
            f32x4 p = {0.f, 0.f, 0.f, 0.f};
            p = mfma(a0, q0, p);
            p = mfma(a1, q1, p);
            pk[d] = pack4(p);
        } else {
            pk[d] = make_uint2(0u, 0u);
        }
    }
    bf16x8 vop[2][4];
#pragma unroll
    for (int p = 0; p < 2; ++p)
#pragma unroll
        for (int jt = 0; jt < 4; ++jt) vop[p][jt] = token_operand(sm.v, ord.slot(2 * p), ord.slot(2 * p + 1), 16 * jt, r, g);

    accumulate_output(sm, pk, ord.nb >= 2, vop, q0, q1, r, g, O);

    // state: S = diag(exp(b_end)) (S + kt^T V), rows at LDS positions 16w + 4g + e
    {
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            const bf16x8 a = token_operand(sm.kt, ord.slot(2 * p), ord.slot(2 * p + 1), 16 * w, r, g);
#pragma unroll
            for (int jt = 0; jt < 4; ++jt) S[jt] = mfma(a, vop[p][jt], S[jt]);
        }
        const float4 t = *reinterpret_cast<const float4 *>(&sm.tot[16 * w + 4 * g]);
        const float dx = fast_exp2(t.x * kLog2e), dy = fast_exp2(t.y * kLog2e);
        const float dz = fast_exp2(t.z * kLog2e), dw = fast_exp2(t.w * kLog2e);
#pragma unroll
        for (int jt = 0; jt < 4; ++jt) {
            S[jt][0] *= dx; S[jt][1] *= dy; S[jt][2] *= dz; S[jt][3] *= dw;
        }
    }

    __syncthreads();  // every read of st / kt / v / g / tot of this step is done
    publish_state(sm, w, r, g, S);
}

// RANGE-SAFE form of one chunk of one direction (see the header); scans the sub-block-local,
// floored gates itself.  sm.g / sm.v hold the chunk's raw gates and values.
template <int DIR>
__device__ __forceinline__ void out_chunk_safe(OutLds &sm, const SubOrder<DIR> &ord, const int w, const int r,
                                               const int g, const Row16 &qraw, const Row16 &kraw, f32x4 (&O)[4],
                                               f32x4 (&S)[4])
{
    const int row = 16 * w + r;
    const Row16 graw = lds_row_operand(sm.g, row, g);

    float X[16], Y[16], F[16], Emid[16], EB[16];
    gate_factors<DIR>(graw, r, X, Y, F, Emid, EB);
    if (r == 0) store_chan16(sm.eb[w], g, EB);  // whole-sub-block decay exp(B_w)

    float qf[16], kf[16];
    unpack16(qraw, qf);
    unpack16(kraw, kf);
    float khat[16], tmp[16], cum[16];
#pragma unroll
    for (int e = 0; e < 16; ++e) khat[e] = kf[e] * F[e];
    store_row16(sm.kt, row, g, khat);
    // diagonal tile operands, both referred to the middle of the sub-block
#pragma unroll
    for (int e = 0; e < 16; ++e) tmp[e] = kf[e] * Y[e];
    const bf16x8 kd0 = pack8(tmp), kd1 = pack8(tmp + 8);
#pragma unroll
    for (int e = 0; e < 16; ++e) cum[e] = qf[e] * X[e];
    const bf16x8 qd0 = pack8(cum), qd1 = pack8(cum + 8);

    __syncthreads();  // eb, kt visible

    // query variants: qv[d] pairs with the keys of before(d+1); readout uses the full product.
    // q * exp(b_t) = (q * X) * Emid is the decay since the near edge of the query's sub-block.
#pragma unroll
    for (int e = 0; e < 16; ++e) cum[e] *= Emid[e];
    bf16x8 qv[3][2];
    qv[0][0] = pack8(cum);
    qv[0][1] = pack8(cum + 8);
#pragma unroll
    for (int d = 1; d <= 3; ++d) {
        if (d <= ord.nb) {
            load_chan16(sm.eb[ord.before(d)], g, tmp);
#pragma unroll
            for (int e = 0; e < 16; ++e) cum[e] *= tmp[e];
            if (d < 3) {
                qv[d][0] = pack8(cum);
                qv[d][1] = pack8(cum + 8);
            }
        }
    }
    const bf16x8 qr0 = pack8(cum), qr1 = pack8(cum + 8);  // readout queries: q * exp(decay since chunk edge)

    // state-update keys: khat times the whole sub-blocks after this one
#pragma unroll
    for (int a = 1; a <= 3; ++a) {
        if (a <= 3 - ord.nb) {
            load_chan16(sm.eb[ord.after(a)], g, tmp);
#pragma unroll
            for (int e = 0; e < 16; ++e) khat[e] *= tmp[e];
        }
    }
    store_row16(sm.ks, row, g, khat);

    __syncthreads();  // ks visible

    // intra-chunk scores, transposed: P^T[i][t] = sum_c khat[i][c] * qv[t][c]
    uint2 pk[4];
    {
        f32x4 p = {0.f, 0.f, 0.f, 0.f};
        p = mfma(kd0, qd0, p);
        p = mfma(kd1, qd1, p);
        pk[0] = masked_diag<DIR>(p, r, g);
    }
#pragma unroll
    for (int d = 1; d <= 3; ++d) {
        if (d <= ord.nb) {
            const int kb = ord.before(d);
            const bf16x8 a0 = *reinterpret_cast<const bf16x8 *>(&sm.kt[16 * kb + r][8 * g]);
            const bf16x8 a1 = *reinterpret_cast<const bf16x8 *>(&sm.kt[16 * kb + r][32 + 8 * g]);
            f32x4 p = {0.f, 0.f, 0.f, 0.f};
            p = mfma(a0, qv[d - 1][0], p);
            p = mfma(a1, qv[d - 1][1], p);
            pk[d] = pack4(p);
        } else {
            pk[d] = make_uint2(0u, 0u);
        }
    }
    bf16x8 vop[2][4];
#pragma unroll
    for (int p = 0; p < 2; ++p)
#pragma unroll
        for (int jt = 0; jt < 4; ++jt) vop[p][jt] = token_operand(sm.v, ord.slot(2 * p), ord.slot(2 * p + 1), 16 * jt, r, g);

    accumulate_output(sm, pk, ord.nb >= 2, vop, qr0, qr1, r, g, O);

    // state update: S = diag(chunk decay) S + ks^T V  (rows c = 16w + 4g + e)
    {
        float4 dch = *reinterpret_cast<const float4 *>(&sm.eb[0][16 * w + 4 * g]);
#pragma unroll
        for (int sb = 1; sb < 4; ++sb) {
            const float4 t = *reinterpret_cast<const float4 *>(&sm.eb[sb][16 * w + 4 * g]);
            dch.x *= t.x; dch.y *= t.y; dch.z *= t.z; dch.w *= t.w;
        }
#pragma unroll
        for (int jt = 0; jt < 4; ++jt) {
            S[jt][0] *= dch.x; S[jt][1] *= dch.y; S[jt][2] *= dch.z; S[jt][3] *= dch.w;
        }
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            const bf16x8 a = token_operand(sm.ks, ord.slot(2 * p), ord.slot(2 * p + 1), 16 * w, r, g);
#pragma unroll
            for (int jt = 0; jt < 4; ++jt) S[jt] = mfma(a, vop[p][jt], S[jt]);
        }
    }

    __syncthreads();  // every read of st / kt / ks / v / eb of this step is done
    publish_state(sm, w, r, g, S);
}

// One chunk of one direction.  O accumulates this chunk's output tile, token-per-lane (token
// 16w + r, columns 16*jt + 4g + e); S is this wave's 16 rows of the carried fp32 state (rows at
// LDS positions 16w + 4g + e, column 16*jt + r).  graw / vraw are natural-order rows that are
// only staged; qraw / kraw are in operand order.
template <int DIR>
__device__ __forceinline__ void out_chunk_step(OutLds &sm, const bf16x8 (&tri)[2], const int w, const int r,
                                               const int g, const Row16 &qraw, const Row16 &kraw, const Row16 &graw,
                                               const Row16 &vraw, f32x4 (&O)[4], f32x4 (&S)[4])
{
    const SubOrder<DIR> ord(w);
    store_row16_raw(sm.g, 16 * w + r, g, graw);
    store_row16_raw(sm.v, 16 * w + r, g, vraw);

    __syncthreads();  // g, v visible

    f32x4 B[4], T[4];
    chunk_gate_scan(sm.g, tri, r, g, B, T);
    if (chunk_decay_max(T) <= kFastRange)  // same totals in every wave: uniform over the workgroup
        out_chunk_fast<DIR>(sm, ord, w, r, g, B, T, qraw, kraw, O, S);
    else
        out_chunk_safe<DIR>(sm, ord, w, r, g, qraw, kraw, O, S);
}

__device__ __forceinline__ void load_state(const float *src, bool zero, int w, int r, int g, f32x4 (&S)[4])
{
#pragma unroll
    for (int jt = 0; jt < 4; ++jt)
#pragma unroll
        for (int e = 0; e < 4; ++e) S[jt][e] = zero ? 0.f : src[(16 * w + 4 * g + e) * kD + 16 * jt + r];
}

__global__ __launch_bounds__(kThreads, 2) void bigla_segment_out_kernel(
    const uint16_t *__restrict__ q, const uint16_t *__restrict__ k, const uint16_t *__restrict__ v,
    const uint16_t *__restrict__ g_fwd, const uint16_t *__restrict__ g_bwd, uint16_t *__restrict__ out,
    const float *__restrict__ seg_states /* states entering each segment, or nullptr when one segment */, int L,
    int n_seg)
{
    __shared__ OutLds sm;
    const int tid = threadIdx.x;
    const int w = tid >> 6, lane = tid & 63, r = lane & 15, g = lane >> 4;
    const long slab = blockIdx.x / n_seg;
    const int seg = blockIdx.x % n_seg;
    const long base = slab * L * kD;
    q += base; k += base; v += base; g_fwd += base; g_bwd += base; out += base;

    const int chunk0 = seg * kSegChunks;
    const int n_chunks_total = (L + kC - 1) / kC;
    const int nch = min(kSegChunks, n_chunks_total - chunk0);
    const float *st_in = seg_states ? seg_states + (slab * n_seg + seg) * kSegFloats : nullptr;

    // forward-direction output tiles of the segment's chunks, parked between the two sweeps
    f32x4 parked[kSegChunks][4];
    auto park = [&](int m, const f32x4 (&O)[4]) {
#pragma unroll
        for (int p = 0; p < kSegChunks; ++p)
            if (p == m) {
#pragma unroll
                for (int jt = 0; jt < 4; ++jt) parked[p][jt] = O[jt];
            }
    };
    auto unpark = [&](int m, f32x4 (&O)[4]) {
#pragma unroll
        for (int p = 0; p < kSegChunks; ++p)
            if (p == m) {
#pragma unroll
                for (int jt = 0; jt < 4; ++jt) O[jt] = parked[p][jt];
            }
    };

    f32x4 S[4];

    // rows of the next chunk are fetched while the current chunk is being processed
    struct ChunkRows {
        Row16 q, k, g, v;
    };
    auto fetch = [&](int m, const uint16_t *gate) {
        const long tok = long(chunk0 + m) * kC + 16 * w + r;
        const bool valid = tok < L;
        ChunkRows c;
        c.q = load_row_operand(q, tok, valid, g);
        c.k = load_row_operand(k, tok, valid, g);
        c.g = load_row_natural(gate, tok, valid, g);
        c.v = load_row_natural(v, tok, valid, g);
        return c;
    };
    bf16x8 tri[2];

    // ---------------- forward sweep: chunks ascending ----------------
    ChunkRows next = fetch(0, g_fwd);
    scan_triangle<0>(w, r, g, tri);
    load_state(st_in, st_in == nullptr, w, r, g, S);
    publish_state(sm, w, r, g, S);  // made visible by the first barrier inside the step
    for (int m = 0; m < nch; ++m) {
        const ChunkRows cur = next;
        next = m + 1 < nch ? fetch(m + 1, g_fwd) : fetch(nch - 1, g_bwd);
        f32x4 O[4];
#pragma unroll
        for (int jt = 0; jt < 4; ++jt) O[jt] = f32x4{0.f, 0.f, 0.f, 0.f};
        out_chunk_step<0>(sm, tri, w, r, g, cur.q, cur.k, cur.g, cur.v, O, S);
        park(m, O);
    }

    // ---------------- backward sweep: chunks descending ----------------
    __syncthreads();  // the forward sweep's last state copy is no longer read
    load_state(st_in ? st_in + size_t(kD) * kD : nullptr, st_in == nullptr, w, r, g, S);
    publish_state(sm, w, r, g, S);
    scan_triangle<1>(w, r, g, tri);
    for (int m = nch - 1; m >= 0; --m) {
        // the parked tile comes back before the next prefetch is issued: vector-memory results
        // return in order, so a later wait for it must not sit behind the prefetch
        f32x4 O[4];
        unpark(m, O);
        const ChunkRows cur = next;
        if (m > 0) next = fetch(m - 1, g_bwd);
        out_chunk_step<1>(sm, tri, w, r, g, cur.q, cur.k, cur.g, cur.v, O, S);
        // o_t = (o_fwd_t + o_bwd_t) / 2 for token 16w + r, columns 16*jt + 4g .. +3
        const long tok = long(chunk0 + m) * kC + 16 * w + r;
        if (tok < L) {
#pragma unroll
            for (int jt = 0; jt < 4; ++jt) {
                const f32x4 o = O[jt];
                *reinterpret_cast<uint2 *>(out + tok * kD + 16 * jt + 4 * g) =
                    make_uint2(pack2(0.5f * o[0], 0.5f * o[1]), pack2(0.5f * o[2], 0.5f * o[3]));
            }
        }
    }
}

// ---- kernel 1: per-segment local end states, both directions in one pass ----------------------

__global__ __launch_bounds__(kThreads, 2) void bigla_segment_state_kernel(
    const uint16_t *__restrict__ k, const uint16_t *__restrict__ v, const uint16_t *__restrict__ g_fwd,
    const uint16_t *__restrict__ g_bwd, float *__restrict__ seg_states, int L, int n_seg)
{
    __shared__ StateLds sm;
    const int tid = threadIdx.x;
    const int w = tid >> 6, lane = tid & 63, r = lane & 15, g = lane >> 4;
    const long slab = blockIdx.x / n_seg;
    const int seg = blockIdx.x % n_seg;
    const long base = slab * L * kD;
    k += base; v += base; g_fwd += base; g_bwd += base;
    float *dst = seg_states + (slab * n_seg + seg) * kSegFloats;

    const int chunk0 = seg * kSegChunks;
    const int n_chunks_total = (L + kC - 1) / kC;
    const int nch = min(kSegChunks, n_chunks_total - chunk0);
    const int row = 16 * w + r;

    f32x4 Sf[4], Sb[4];
#pragma unroll
    for (int jt = 0; jt < 4; ++jt) {
        Sf[jt] = f32x4{0.f, 0.f, 0.f, 0.f};
        Sb[jt] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    // Total decay of the chunks seen so far, rows 16w + 4g + e.  The backward state is walked left
    // to right: the state at the segment's LEFT edge is sum_n (decay of the chunks left of n) *
    // (chunk n's state at its own left edge), so chunk n's contribution is scaled by the running
    // product once and nothing accumulated ever decays again.
    float4 dtot_f = make_float4(1.f, 1.f, 1.f, 1.f), dtot_b = dtot_f;

    // rows of the next chunk are fetched while the current chunk is being processed
    struct ChunkRows {
        Row16 k, v, gf, gb;
    };
    auto fetch = [&](int m) {
        const long tok = long(chunk0 + m) * kC + row;
        const bool valid = tok < L;
        ChunkRows c;
        c.k = load_row_operand(k, tok, valid, g);
        c.v = load_row_natural(v, tok, valid, g);
        c.gf = load_row_natural(g_fwd, tok, valid, g);
        c.gb = load_row_natural(g_bwd, tok, valid, g);
        return c;
    };
    ChunkRows next = fetch(0);
    bf16x8 tri_f[2], tri_b[2];
    scan_triangle<0>(w, r, g, tri_f);
    scan_triangle<1>(w, r, g, tri_b);

    for (int m = 0; m < nch; ++m) {
        const ChunkRows cur = next;
        if (m + 1 < nch) next = fetch(m + 1);

        store_row16_raw(sm.g[0], row, g, cur.gf);
        store_row16_raw(sm.g[1], row, g, cur.gb);
        store_row16_raw(sm.v, row, g, cur.v);
        __syncthreads();  // g, v visible

        float kf[16];
        unpack16(cur.k, kf);
        f32x4 Bf[4], Bb[4];
        float max_f, max_b;
        {
            f32x4 T[4];
            float t[16];
            chunk_gate_scan(sm.g[0], tri_f, r, g, Bf, T);
            max_f = chunk_decay_max(T);
#pragma unroll
            for (int n = 0; n < 16; ++n) t[n] = T[n >> 2][n & 3];
            if (r == 0) store_chan16(sm.tot[0], g, t);  // chunk totals per channel, operand order
            chunk_gate_scan(sm.g[1], tri_b, r, g, Bb, T);
            max_b = chunk_decay_max(T);
#pragma unroll
            for (int n = 0; n < 16; ++n) t[n] = T[n >> 2][n & 3];
            if (r == 0) store_chan16(sm.tot[1], g, t);
        }
        const bool fast = fmaxf(max_f, max_b) <= kFastRange;  // uniform over the workgroup
        float4 df, db;  // this chunk's decay, rows at LDS positions 16w + 4g + e
        float tmp[16];
        if (fast) {
            // keys k * exp(-b_i), b_i cumulative since the chunk edge of each direction
            float kb[16];
#pragma unroll
            for (int n = 0; n < 16; ++n) {
                kb[n] = kf[n] * fast_exp2(-kLog2e * Bb[n >> 2][n & 3]);
                kf[n] = kf[n] * fast_exp2(-kLog2e * Bf[n >> 2][n & 3]);
            }
            store_row16(sm.ks[0], row, g, kf);
            store_row16(sm.ks[1], row, g, kb);
            __syncthreads();  // ks, tot visible
            const float4 tf = *reinterpret_cast<const float4 *>(&sm.tot[0][16 * w + 4 * g]);
            const float4 tb = *reinterpret_cast<const float4 *>(&sm.tot[1][16 * w + 4 * g]);
            df = make_float4(fast_exp2(tf.x * kLog2e), fast_exp2(tf.y * kLog2e), fast_exp2(tf.z * kLog2e),
                             fast_exp2(tf.w * kLog2e));
            db = make_float4(fast_exp2(tb.x * kLog2e), fast_exp2(tb.y * kLog2e), fast_exp2(tb.z * kLog2e),
                             fast_exp2(tb.w * kLog2e));
        } else {
            // range-safe keys: decay from the token to the chunk edge, every factor <= 1
            float EB[16], Ff[16], Fb[16];
            gate_factors_state<0>(lds_row_operand(sm.g[0], row, g), Ff, EB);
            if (r == 0) store_chan16(sm.eb[0][w], g, EB);
            gate_factors_state<1>(lds_row_operand(sm.g[1], row, g), Fb, EB);
            if (r == 0) store_chan16(sm.eb[1][w], g, EB);
            __syncthreads();  // eb visible
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                Ff[e] *= kf[e];
                Fb[e] *= kf[e];
            }
#pragma unroll
            for (int sb = 0; sb < 4; ++sb) {
                if (sb > w) {  // forward: the sub-blocks to the right
                    load_chan16(sm.eb[0][sb], g, tmp);
#pragma unroll
                    for (int e = 0; e < 16; ++e) Ff[e] *= tmp[e];
                }
                if (sb < w) {  // backward: the sub-blocks to the left
                    load_chan16(sm.eb[1][sb], g, tmp);
#pragma unroll
                    for (int e = 0; e < 16; ++e) Fb[e] *= tmp[e];
                }
            }
            store_row16(sm.ks[0], row, g, Ff);
            store_row16(sm.ks[1], row, g, Fb);
            df = *reinterpret_cast<const float4 *>(&sm.eb[0][0][16 * w + 4 * g]);
            db = *reinterpret_cast<const float4 *>(&sm.eb[1][0][16 * w + 4 * g]);
#pragma unroll
            for (int sb = 1; sb < 4; ++sb) {
                const float4 a = *reinterpret_cast<const float4 *>(&sm.eb[0][sb][16 * w + 4 * g]);
                const float4 b = *reinterpret_cast<const float4 *>(&sm.eb[1][sb][16 * w + 4 * g]);
                df.x *= a.x; df.y *= a.y; df.z *= a.z; df.w *= a.w;
                db.x *= b.x; db.y *= b.y; db.z *= b.z; db.w *= b.w;
            }
            __syncthreads();  // ks visible
        }

        // chunk contributions K^T V of both directions, rows c = 16w + 4g + e
        f32x4 Cf[4], Cb[4];
#pragma unroll
        for (int jt = 0; jt < 4; ++jt) {
            // fast: S_f = df * (S_f + Kf^T V) accumulates onto the state; safe: S_f = df * S_f + Kf^T V
            Cf[jt] = fast ? Sf[jt] : f32x4{0.f, 0.f, 0.f, 0.f};
            Cb[jt] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            const bf16x8 af = token_operand(sm.ks[0], 2 * p, 2 * p + 1, 16 * w, r, g);
            const bf16x8 ab = token_operand(sm.ks[1], 2 * p, 2 * p + 1, 16 * w, r, g);
#pragma unroll
            for (int jt = 0; jt < 4; ++jt) {
                const bf16x8 vb = token_operand(sm.v, 2 * p, 2 * p + 1, 16 * jt, r, g);
                Cf[jt] = mfma(af, vb, Cf[jt]);
                Cb[jt] = mfma(ab, vb, Cb[jt]);
            }
        }
        // backward: chunk state at its own left edge is db * Cb (fast) or Cb (safe); scale by the
        // decay of the chunks to its left
        const float4 sb4 = fast ? make_float4(dtot_b.x * db.x, dtot_b.y * db.y, dtot_b.z * db.z, dtot_b.w * db.w) : dtot_b;
#pragma unroll
        for (int jt = 0; jt < 4; ++jt) {
            if (fast) {
                Sf[jt][0] = Cf[jt][0] * df.x; Sf[jt][1] = Cf[jt][1] * df.y;
                Sf[jt][2] = Cf[jt][2] * df.z; Sf[jt][3] = Cf[jt][3] * df.w;
            } else {
                Sf[jt][0] = fmaf(Sf[jt][0], df.x, Cf[jt][0]); Sf[jt][1] = fmaf(Sf[jt][1], df.y, Cf[jt][1]);
                Sf[jt][2] = fmaf(Sf[jt][2], df.z, Cf[jt][2]); Sf[jt][3] = fmaf(Sf[jt][3], df.w, Cf[jt][3]);
            }
            Sb[jt][0] = fmaf(Cb[jt][0], sb4.x, Sb[jt][0]); Sb[jt][1] = fmaf(Cb[jt][1], sb4.y, Sb[jt][1]);
            Sb[jt][2] = fmaf(Cb[jt][2], sb4.z, Sb[jt][2]); Sb[jt][3] = fmaf(Cb[jt][3], sb4.w, Sb[jt][3]);
        }
        dtot_f.x *= df.x; dtot_f.y *= df.y; dtot_f.z *= df.z; dtot_f.w *= df.w;
        dtot_b.x *= db.x; dtot_b.y *= db.y; dtot_b.z *= db.z; dtot_b.w *= db.w;
        __syncthreads();  // every read of this chunk's LDS tiles is done
    }

#pragma unroll
    for (int jt = 0; jt < 4; ++jt)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int idx = (16 * w + 4 * g + e) * kD + 16 * jt + r;
            dst[idx] = Sf[jt][e];
            dst[size_t(kD) * kD + idx] = Sb[jt][e];
        }
    if (r == 0) {
        *reinterpret_cast<float4 *>(dst + kSegStateFloats + 16 * w + 4 * g) = dtot_f;
        *reinterpret_cast<float4 *>(dst + kSegStateFloats + kD + 16 * w + 4 * g) = dtot_b;
    }
}

// ---- kernel 2: scan of segment states, in place ------------------------------------------------
// On entry seg_states[slab][n] holds segment n's local end states and decays; on exit it holds the
// states ENTERING segment n: from the left for the forward direction, from the right for the
// backward direction.  One thread per (slab, direction, state element).
__global__ __launch_bounds__(kThreads) void bigla_state_scan_kernel(float *__restrict__ seg_states, int n_seg)
{
    constexpr int kBlocksPerState = kD * kD / kThreads;
    const int elem = (blockIdx.x % kBlocksPerState) * kThreads + threadIdx.x;  // 0 .. 4095
    const int dir = (blockIdx.x / kBlocksPerState) & 1;
    const long slab = blockIdx.x / (2 * kBlocksPerState);
    float *base = seg_states + slab * n_seg * kSegFloats;
    const int c = elem / kD;
    float run = 0.f;
    for (int i = 0; i < n_seg; ++i) {
        const int n = dir == 0 ? i : n_seg - 1 - i;
        float *s = base + n * kSegFloats;
        const float local = s[dir * kD * kD + elem];
        const float decay = s[kSegStateFloats + dir * kD + c];
        s[dir * kD * kD + elem] = run;
        run = fmaf(run, decay, local);
    }
}

}  // namespace

bool bigla_chunk_supported(int dk, int dv, bool is_bf16) { return is_bf16 && dk == kD && dv == kD; }

size_t bigla_chunk_workspace_bytes(long BH, int L)
{
    const long n_chunks = (L + kC - 1) / kC;
    const long n_seg = (n_chunks + kSegChunks - 1) / kSegChunks;
    // always non-zero so that callers can size one buffer per problem; unused when n_seg == 1
    return size_t(BH) * n_seg * kSegFloats * sizeof(float);
}

hipError_t bigla_chunk_launch(const void *q, const void *k, const void *v, const void *g_fwd, const void *g_bwd,
                              void *out, long BH, int L, void *workspace, hipStream_t stream)
{
    const long n_chunks = (L + kC - 1) / kC;
    const int n_seg = int((n_chunks + kSegChunks - 1) / kSegChunks);
    const long blocks = BH * n_seg;
    if (blocks > 0x7fffffffL || BH * 2 * (kD * kD / kThreads) > 0x7fffffffL) return hipErrorInvalidValue;
    const uint16_t *qq = static_cast<const uint16_t *>(q), *kk = static_cast<const uint16_t *>(k);
    const uint16_t *vv = static_cast<const uint16_t *>(v);
    const uint16_t *gf = static_cast<const uint16_t *>(g_fwd), *gb = static_cast<const uint16_t *>(g_bwd);
    float *ws = static_cast<float *>(workspace);
    if (n_seg > 1) {
        {
            LaunchTimer timer(kKernelSegmentState, stream);
            hipLaunchKernelGGL(bigla_segment_state_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, stream, kk, vv,
                               gf, gb, ws, L, n_seg);
        }
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        {
            LaunchTimer timer(kKernelStateScan, stream);
            hipLaunchKernelGGL(bigla_state_scan_kernel, dim3((unsigned)(BH * 2 * (kD * kD / kThreads))),
                               dim3(kThreads), 0, stream, ws, n_seg);
        }
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    {
        LaunchTimer timer(kKernelSegmentOut, stream);
        hipLaunchKernelGGL(bigla_segment_out_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, stream, qq, kk, vv, gf,
                           gb, static_cast<uint16_t *>(out), n_seg > 1 ? ws : nullptr, L, n_seg);
    }
    return hipGetLastError();
}

}  // namespace vig
