// Chunkwise bf16 MFMA evaluation of BiGLA (Section 4.2.1, Eq. (BiGLA)) for dv = 64 and dk = 64
// (or 32, widened to 64 with zero channels).
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
//   16 nats in every channel (the sum over its four 16-token sub-blocks of the largest
//   per-channel sub-block total is checked): far inside fp32's range, and slow enough a decay
//   that an output sums over enough tokens for the rounding of the scaled operands to stay
//   within the stated tolerance.  Gates of the paper's form, sigmoid(z)^(1/16), stay inside:
//   64 steps reach 16 nats only for z < -4 throughout.  (The eight-wave kernels of
//   bigla_chunk_ws.hpp keep the fast form up to 60 nats, with split operands for the diagonal
//   score tiles beyond 16.)
//   RANGE-SAFE.  Otherwise cumulative gates stay local to a sub-block: off-diagonal 16x16 tiles
//   scale keys by the decay to the END of the key's own sub-block and queries by the decay from
//   the START of the query's sub-block times the whole-sub-block factors in between, so every
//   factor is <= 1 and underflow to 0 is the correct limit.  The diagonal tile refers both
//   sides to the MIDDLE of the sub-block, so its factors span at most 8 steps in either sense
//   (its operands are split into bf16 pairs hi + lo and multiplied as hi.hi + hi.lo + lo.hi);
//   the per-step log-gate is floored at -8 there (alpha >= 3.4e-4; anything smaller is a hard
//   reset whose leak is far below the bf16 tolerance), which keeps them within e^(+-64).
// Masking is by select, never by multiplying with 0.
//
// Parallel decomposition.  A sequence is cut into segments of consecutive chunks (the segment
// length is chosen at launch so that the workgroups about fill the chip once).
//   1. bigla_segment_state_kernel : one workgroup per (slab, segment) walks its chunks right to
//      left, once, for BOTH directions: it carries the backward state and, before each chunk,
//      stashes it (bf16, state entering the chunk from the right, local to the segment)
//      together with the decay from that chunk's right edge to the segment's right edge; it
//      also accumulates the segment's forward end state, the backward state at the segment's
//      left edge and both total decays.
//   2. bigla_segment_out_kernel   : one workgroup per (slab, segment).  It first folds the
//      segment-local end states and decays of the slab's other segments into the two states
//      ENTERING its own segment (forward from the left, backward from the right: a short
//      sequential scan per state element, E <- D_n E + S_n, whose operands sit in the L2 of the
//      XCD that all segments of a slab are assigned to), then walks its chunks left to
//      right, once.  Each chunk is finished in a single step for both directions: one merged
//      64x64 score tile (lower triangle forward, upper triangle backward, the diagonal from
//      both), ONE P.V contraction, the forward state readout from the state carried in
//      registers, ONE backward readout from the stash tile to which the segment's entering
//      state (scaled per channel by the stashed decay) has been added, then the forward state
//      update.  out = (o_fwd + o_bwd)/2 is written once; q, k, v, g_fwd, g_bwd are read once
//      here.  Segments the state kernel flagged as mild run fast-form-only code inlined in the
//      kernel; the others call the general code (both forms) as a separate function.
//   When a plan has one segment per slab, bigla_slab_kernel runs both passes in a single launch
//   (a workgroup per slab; no segment states, no flags).
// Nothing is reversed or copied in HBM; both directions read the same q, k, v.
//
// Wavefront mapping (256 threads = 4 waves).  Wave w owns tokens [16w, 16w+16) of the chunk;
// lane (r = lane%16, g = lane/16) holds 16 channels of token 16w + r: slot n of the lane is
// channel 32*(n/8) + 8g + n%8, i.e. two 16-byte pieces of the token row, and slots 8kk..8kk+7
// are the lane's k-slots of K-step kk of every contraction over channels.  The cumulative
// gates leave the matrix cores (below) in accumulator layout, lane (r, g) holding rows
// 4g..4g+3 of each 16-row tile; the staged gate tiles therefore keep their columns permuted
// (channel 32kk + 8g + 4h + e at column 16(2kk+h) + 4g + e) so that tile ct, row 4g+e is the
// lane's slot 4ct + e.  Every row tensor moves between HBM and the chip in fully contiguous
// wave accesses, 8 whole 128-byte rows per instruction; q, k and out change between row order
// and operand order through the wave's own rows of an idle LDS tile.  Contractions over tokens
// (P.V, the state update, the gate scan) take their token-major operands from row-major LDS
// tiles through ds_read_b64_tr_b16.
//
// Cumulative gates on the matrix cores.  The chunk-level cumulative log-gate is a product with
// a triangular 0/1 matrix, B^T[c][t] = sum_i g[i][c] * [i <= t] (or [i >= t] backward), which
// is exact in bf16 x bf16 -> fp32.  Two K-steps of the MFMA per 16-channel tile replace the
// wavefront prefix scans, the cross-sub-block offsets and every unpack of g on the vector
// ALUs, which are the scarce unit on this path; a second product with the all-ones matrix gives
// every lane the chunk totals of its channels (state decay, choice of the form).  The
// range-safe form still scans its sub-block-local, floored gates with DPP row operations.
#include <type_traits>

#include "bigla_chunk_tiles.hpp"
#include "vig_common.hpp"
#include "vig_kernels.hpp"
#include "vig_timing.hpp"

namespace vig {

namespace {

// ---- kernel 3: per-segment output pass --------------------------------------------------------

// What the first half of a chunk step (scores) hands to the second half (finish_chunk)
struct ChunkOperands {
    uint2 pk[4], pl[4];                // merged masked score tile per key sub-block as bf16 pairs: p = pk + pl
    bf16x8 qf0, qf1, qb0, qb1;  // readout queries: forward, backward
};

struct ChunkFlags {
    bool stash;  // a backward state stashed for this chunk exists (not the segment's last chunk)
    bool seg;    // a backward state enters the segment from the right
};

// One slab's inputs of the fused 2D gating locality injection (Section 4.2.2): the conv input and
// the gate logits as buffer resources whose rows sit at the activations' token pitch.  Taps that
// fall off the grid, and rows past the sequence, are requested at kOffGrid, which is beyond the
// resource's extent: the bounds check of the load returns zeros for them, the conv's zero padding.
struct LocalitySlab {
    __amdgpu_buffer_rsrc_t x, z;
    int Hg, Wg;
};
constexpr unsigned kOffGrid = 0xfffffff0u;

// Everything after the score tiles, common to both forms: O^T = V^T P^T + the three readouts,
// out = O (the score and readout queries carry the 1/2 of the average), then the forward state
// update with the keys in `ktile`.
// fast_update: S = d (S + K^T V) with d = exp(tot); otherwise S = d S + K^T V with d = prod(eb).
// kKs = 1 (32-wide head, fast-form code only): state rows 32..63 are identically zero, so the waves
// that own them (w >= 2) skip the state update and nobody reads the upper K-step of a state tile.
// kLoc: the locality blend is applied to the chunk's rows before they are written (below).
template <bool kTm, int kKs, bool kLoc, class Prefetch>
__device__ __forceinline__ void finish_chunk(OutLds &sm, const uint16_t (*ktile)[kPitch], const ChunkOperands &op,
                                             const ChunkFlags fl, const bool fast_update, const int w, const int r,
                                             const int g, __amdgpu_buffer_rsrc_t out_rows, const LaneRows &vr,
                                             const unsigned chunk_token0, f32x4 (&S)[4], const LocalitySlab &ls,
                                             Prefetch &&prefetch)
{
    const uint2(&pk)[4] = op.pk;
    const uint2(&pl)[4] = op.pl;
    bf16x8 vop[2][4];
#pragma unroll
    for (int p = 0; p < 2; ++p)
#pragma unroll
        for (int jt = 0; jt < 4; ++jt) vop[p][jt] = token_operand(sm.v, 2 * p, 2 * p + 1, 16 * jt, r, g);
    prefetch(0);

    // token-per-lane accumulators: lane (r, g) gets columns 16*jt + 4g .. +3 of its own token
    f32x4 O[4];
    {
        // the score tile enters as hi + lo, so that its own rounding to bf16 does not reach the output
        const bf16x8 pa0 = operand(pk[0], pk[1]), pa1 = operand(pk[2], pk[3]);
        const bf16x8 pb0 = operand(pl[0], pl[1]), pb1 = operand(pl[2], pl[3]);
        const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int jt = 0; jt < 4; ++jt)
            O[jt] = mfma(vop[1][jt], pa1, mfma(vop[0][jt], pa0, mfma(vop[1][jt], pb1, mfma(vop[0][jt], pb0, zero))));
    }
    prefetch(1);
    readout<kKs>(sm.st, op.qf0, op.qf1, r, g, O);
    prefetch(2);
    if (fl.stash || fl.seg) readout<kKs>(sm.sb, op.qb0, op.qb1, r, g, O);
    prefetch(3);
    const int lane = 16 * g + r;
    {  // o_t = (o_fwd_t + o_bwd_t) / 2 (the queries arrive halved), turned into whole rows through the wave's own rows of the
       // forward gate tile (last read before the score tiles), then written 8 rows per store
#pragma unroll
        for (int jt = 0; jt < 4; ++jt)
            *reinterpret_cast<uint2 *>(&sm.gf[16 * w + r][16 * jt + 4 * g]) =
                make_uint2(pack2(O[jt][0], O[jt][1]), pack2(O[jt][2], O[jt][3]));
        wave_lds_fence();
        if (!kLoc) {
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const int rr = 16 * w + 8 * t + (lane >> 3);
                const uint4 o = *reinterpret_cast<const uint4 *>(&sm.gf[rr][8 * (lane & 7)]);
                __builtin_amdgcn_raw_buffer_store_b128(u32x4{o.x, o.y, o.z, o.w}, out_rows,
                                                       vr.off[t] + chunk_token0 * vr.pitch, 0, 0);
            }
        }
    }

    // forward state, rows at LDS positions 16w + 4g + e
    const bool owns_rows = kKs > 1 || w < 2;
    float4 d = make_float4(1.f, 1.f, 1.f, 1.f);
    if (!owns_rows) {
        // nothing to update
    } else if (fast_update) {
        const float4 t = *reinterpret_cast<const float4 *>(&sm.tot[16 * w + 4 * g]);
        d = make_float4(fast_exp2(t.x * kLog2e), fast_exp2(t.y * kLog2e), fast_exp2(t.z * kLog2e),
                        fast_exp2(t.w * kLog2e));
    } else {
        d = *reinterpret_cast<const float4 *>(&sm.eb[0][0][16 * w + 4 * g]);
#pragma unroll
        for (int sb = 1; sb < 4; ++sb) {
            const float4 t = *reinterpret_cast<const float4 *>(&sm.eb[0][sb][16 * w + 4 * g]);
            d.x *= t.x; d.y *= t.y; d.z *= t.z; d.w *= t.w;
        }
#pragma unroll
        for (int jt = 0; jt < 4; ++jt) {
            S[jt][0] *= d.x; S[jt][1] *= d.y; S[jt][2] *= d.z; S[jt][3] *= d.w;
        }
    }
    if (owns_rows) {
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            const bf16x8 a = token_operand(ktile, 2 * p, 2 * p + 1, 16 * w, r, g);
#pragma unroll
            for (int jt = 0; jt < 4; ++jt) S[jt] = mfma(a, vop[p][jt], S[jt]);
        }
    }
    if (fast_update && owns_rows) {
#pragma unroll
        for (int jt = 0; jt < 4; ++jt) {
            S[jt][0] *= d.x; S[jt][1] *= d.y; S[jt][2] *= d.z; S[jt][3] *= d.w;
        }
    }

    __syncthreads();  // every LDS read of this step is done
    if (owns_rows) publish_state(sm.st, w, r, g, S);

    if (kLoc) {
        // out = G * (bias + sum_taps w * x) + (1 - G) * o, G = sigmoid(z): the arithmetic (fp32,
        // taps in row-major order) of the stand-alone locality kernel, on the o rounded to bf16.
        // One token row at a time (the lane's piece, 8 channels, of its 3x3 neighbourhood is ten
        // 16-byte loads); o is still in the wave's rows of the gate tile.
        const int c0 = 8 * (lane & 7);
        const unsigned pitch_b = vr.pitch;
#pragma unroll 1
        for (int t = 0; t < 2; ++t) {
            const int rr = 16 * w + 8 * t + (lane >> 3);
            const int tok = int(chunk_token0) + rr;
            const unsigned own = vr.off[t] + chunk_token0 * vr.pitch;
            const int y = tok / ls.Wg, xp = tok - y * ls.Wg;
            u32x4 x_nb[9];
#pragma unroll
            for (int ky = -1; ky <= 1; ++ky)
#pragma unroll
                for (int kx = -1; kx <= 1; ++kx) {
                    const bool in = unsigned(y + ky) < unsigned(ls.Hg) && unsigned(xp + kx) < unsigned(ls.Wg);
                    const unsigned off = own + unsigned(ky * ls.Wg + kx) * pitch_b;
                    x_nb[3 * (ky + 1) + kx + 1] = __builtin_amdgcn_raw_buffer_load_b128(ls.x, in ? off : kOffGrid, 0, 0);
                }
            const u32x4 z_row = __builtin_amdgcn_raw_buffer_load_b128(ls.z, own, 0, 0);
            float acc[8];
            {
                const float4 b0 = *reinterpret_cast<const float4 *>(&sm.cb[c0]);
                const float4 b1 = *reinterpret_cast<const float4 *>(&sm.cb[c0 + 4]);
                acc[0] = b0.x; acc[1] = b0.y; acc[2] = b0.z; acc[3] = b0.w;
                acc[4] = b1.x; acc[5] = b1.y; acc[6] = b1.z; acc[7] = b1.w;
            }
#pragma unroll
            for (int tap = 0; tap < 9; ++tap) {
                const float4 w0 = *reinterpret_cast<const float4 *>(&sm.cw[tap][c0]);
                const float4 w1 = *reinterpret_cast<const float4 *>(&sm.cw[tap][c0 + 4]);
                const float wt[8] = {w0.x, w0.y, w0.z, w0.w, w1.x, w1.y, w1.z, w1.w};
                float xf[8];
                unpack8(make_uint4(x_nb[tap].x, x_nb[tap].y, x_nb[tap].z, x_nb[tap].w), xf);
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[e] = fmaf(wt[e], xf[e], acc[e]);
            }
            float zf[8], of[8];
            unpack8(make_uint4(z_row.x, z_row.y, z_row.z, z_row.w), zf);
            unpack8(*reinterpret_cast<const uint4 *>(&sm.gf[rr][c0]), of);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float gate = __builtin_amdgcn_rcpf(1.f + __expf(-zf[e]));
                acc[e] = fmaf(gate, acc[e] - of[e], of[e]);
            }
            __builtin_amdgcn_raw_buffer_store_b128(
                u32x4{pack2(acc[0], acc[1]), pack2(acc[2], acc[3]), pack2(acc[4], acc[5]), pack2(acc[6], acc[7])},
                out_rows, own, 0, 0);
        }
    }
}

// Merged score tiles of the fast form and the readout queries, from this lane's scaled operands
// and the key tiles in LDS.
template <int kKs = 2>
__device__ __forceinline__ void score_tiles(OutLds &sm, const int w, const int r, const int g, const bf16x8 qf0,
                                            const bf16x8 qf1, const bf16x8 qb0, const bf16x8 qb1, const bf16x8 kf0,
                                            const bf16x8 kf1, const bf16x8 kb0, const bf16x8 kb1, ChunkOperands &op)
{
    // merged score tile, transposed: P^T[i][t]; key sub-block I < w forward, I > w backward,
    // I = w the masked sum of both (own token counted by both directions)
#pragma unroll
    for (int I = 0; I < 4; ++I) {
        const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
        if (I == w) {
            f32x4 pf = mfma(kf0, qf0, zero), pb = mfma(kb0, qb0, zero);
            if (kKs > 1) {
                pf = mfma(kf1, qf1, pf);
                pb = mfma(kb1, qb1, pb);
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int i = 4 * g + e;
                pf[e] = (i <= r ? pf[e] : 0.f) + (i >= r ? pb[e] : 0.f);
            }
            split4(pf, op.pk[I], op.pl[I]);
        } else if (I < w) {
            const bf16x8 a0 = *reinterpret_cast<const bf16x8 *>(&sm.kf[16 * I + r][8 * g]);
            f32x4 p = mfma(a0, qf0, zero);
            if (kKs > 1) p = mfma(*reinterpret_cast<const bf16x8 *>(&sm.kf[16 * I + r][32 + 8 * g]), qf1, p);
            split4(p, op.pk[I], op.pl[I]);
        } else {
            const bf16x8 a0 = *reinterpret_cast<const bf16x8 *>(&sm.kb[16 * I + r][8 * g]);
            f32x4 p = mfma(a0, qb0, zero);
            if (kKs > 1) p = mfma(*reinterpret_cast<const bf16x8 *>(&sm.kb[16 * I + r][32 + 8 * g]), qb1, p);
            split4(p, op.pk[I], op.pl[I]);
        }
    }
    op.qf0 = qf0; op.qf1 = qf1; op.qb0 = qb0; op.qb1 = qb1;
}

// FAST form of one chunk, both directions (see the header).  Bf / Bb are the lane's cumulative
// log-gates of the two directions, Tf the forward chunk totals.
template <class Prefetch>
__device__ __forceinline__ void out_chunk_fast(OutLds &sm, const int w, const int r, const int g, const f32x4 (&Bf)[4],
                                               const f32x4 (&Bb)[4], const f32x4 (&Tf)[4], const Row16 &qraw,
                                               const Row16 &kraw, const ChunkFlags /*fl*/, ChunkOperands &op,
                                               Prefetch &&prefetch_first)
{
    const int row = 16 * w + r;
    if (r == 0) {  // forward chunk totals per channel, operand order, for the state decay
        float t[16];
#pragma unroll
        for (int n = 0; n < 16; ++n) t[n] = Tf[n >> 2][n & 3];
        store_chan16(sm.tot, g, t);
    }
    float qf[16], kf[16], qb[16], kb[16];
    unpack16(qraw, qf);
    unpack16(kraw, kf);
#pragma unroll
    for (int n = 0; n < 16; ++n) {
        const float xf = Bf[n >> 2][n & 3] * kLog2e, xb = Bb[n >> 2][n & 3] * kLog2e;
        qb[n] = qf[n] * fast_exp2(xb - 1.f);  // q * exp(c_t) / 2   backward
        kb[n] = kf[n] * fast_exp2(-xb);       // k * exp(-c_i)
        qf[n] *= fast_exp2(xf - 1.f);         // q * exp(b_t) / 2   forward
        kf[n] *= fast_exp2(-xf);              // k * exp(-b_i)
    }
    const bf16x8 qf0 = pack8(qf), qf1 = pack8(qf + 8), qb0 = pack8(qb), qb1 = pack8(qb + 8);
    const bf16x8 kf0 = pack8(kf), kf1 = pack8(kf + 8), kb0 = pack8(kb), kb1 = pack8(kb + 8);
    *reinterpret_cast<bf16x8 *>(&sm.kf[row][8 * g]) = kf0;
    *reinterpret_cast<bf16x8 *>(&sm.kf[row][32 + 8 * g]) = kf1;
    *reinterpret_cast<bf16x8 *>(&sm.kb[row][8 * g]) = kb0;
    *reinterpret_cast<bf16x8 *>(&sm.kb[row][32 + 8 * g]) = kb1;
    __syncthreads();  // kf, kb, tot visible
    prefetch_first();

    score_tiles(sm, w, r, g, qf0, qf1, qb0, qb1, kf0, kf1, kb0, kb1, op);
}

// FAST form with the gate scans folded in, for the kernel that runs nothing else: per 16-channel
// tile the two directions' cumulative gates come off the matrix cores and are consumed by the
// exponentials and scalings of that tile's four slots right away, so that the vector ALU work
// of one tile can overlap the LDS reads and MFMAs of the next (one basic block, no branch
// between the scan and its use).  The forward chunk totals are the cumulative gates of the
// chunk's last token (wave 3, r = 15).
template <int kKs, class Prefetch>
__device__ __forceinline__ void out_chunk_fast_fused(OutLds &sm, const bf16x8 (&tri_f)[2], const bf16x8 (&tri_b)[2],
                                                     const int w, const int r, const int g, const Row16 &qraw,
                                                     const Row16 &kraw, ChunkOperands &op, Prefetch &&prefetch_first)
{
    const int row = 16 * w + r;
    constexpr int kCt = 2 * kKs;  // 16-channel tiles that carry data
    float qf[16], kf[16], qb[16], kb[16], tot[16];
    unpack16(qraw, qf);
    unpack16(kraw, kf);
#pragma unroll
    for (int n = 4 * kCt; n < 16; ++n) qf[n] = kf[n] = qb[n] = kb[n] = tot[n] = 0.f;
#pragma unroll
    for (int ct = 0; ct < kCt; ++ct) {
        const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
        const bf16x8 f0 = token_operand(sm.gf, 0, 1, 16 * ct, r, g), f1 = token_operand(sm.gf, 2, 3, 16 * ct, r, g);
        const bf16x8 b0 = token_operand(sm.gb, 0, 1, 16 * ct, r, g), b1 = token_operand(sm.gb, 2, 3, 16 * ct, r, g);
        const f32x4 Bf = mfma(f1, tri_f[1], mfma(f0, tri_f[0], zero));
        const f32x4 Bb = mfma(b1, tri_b[1], mfma(b0, tri_b[0], zero));
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int n = 4 * ct + e;
            const float xf = Bf[e] * kLog2e, xb = Bb[e] * kLog2e;
            tot[n] = Bf[e];
            qb[n] = qf[n] * fast_exp2(xb - 1.f);  // q * exp(c_t) / 2   backward
            kb[n] = kf[n] * fast_exp2(-xb);       // k * exp(-c_i)
            qf[n] *= fast_exp2(xf - 1.f);         // q * exp(b_t) / 2   forward
            kf[n] *= fast_exp2(-xf);              // k * exp(-b_i)
        }
    }
    const bf16x8 qf0 = pack8(qf), qf1 = pack8(qf + 8), qb0 = pack8(qb), qb1 = pack8(qb + 8);
    const bf16x8 kf0 = pack8(kf), kf1 = pack8(kf + 8), kb0 = pack8(kb), kb1 = pack8(kb + 8);
    *reinterpret_cast<bf16x8 *>(&sm.kf[row][8 * g]) = kf0;
    *reinterpret_cast<bf16x8 *>(&sm.kb[row][8 * g]) = kb0;
    if (kKs > 1) {  // the upper K-step of the key tiles is never read otherwise
        *reinterpret_cast<bf16x8 *>(&sm.kf[row][32 + 8 * g]) = kf1;
        *reinterpret_cast<bf16x8 *>(&sm.kb[row][32 + 8 * g]) = kb1;
    }
    if (w == 3 && r == 15) store_chan16(sm.tot, g, tot);  // for the state decay

    __syncthreads();  // kf, kb, tot visible
    prefetch_first();
    score_tiles<kKs>(sm, w, r, g, qf0, qf1, qb0, qb1, kf0, kf1, kb0, kb1, op);
}

// RANGE-SAFE form of one chunk, both directions (see the header); scans the sub-block-local,
// floored gates itself from the staged raw gates.
template <class Prefetch>
__device__ __forceinline__ void out_chunk_safe(OutLds &sm, const int w, const int r, const int g, const Row16 &qraw,
                                               const Row16 &kraw, const ChunkFlags /*fl*/, ChunkOperands &op,
                                               Prefetch &&prefetch_first)
{
    const int row = 16 * w + r;
    float qf[16], kf[16], tmp[16];
    unpack16(qraw, qf);
    unpack16(kraw, kf);
#pragma unroll
    for (int e = 0; e < 16; ++e) qf[e] *= 0.5f;  // the 1/2 of the output, carried by every query variant

    // per direction: diagonal-tile operands (referred to the middle of the sub-block), the keys
    // for off-diagonal tiles (decay to the far edge of their sub-block) and the running query
    // (each as hi + lo: a token's products with itself and its nearest neighbours carry the output where the
    // decay is fast, which is where this form runs, so their operands keep 16 bits)
    bf16x8 kd[2][2], qd[2][2], kdl[2][2], qdl[2][2];
    float cum[2][16], khat_f[16];
    {
        float X[16], Y[16], F[16], Emid[16], EB[16];
        gate_factors<0>(lds_row_operand(sm.gf, row, g), r, X, Y, F, Emid, EB);
        if (r == 0) store_chan16(sm.eb[0][w], g, EB);
#pragma unroll
        for (int e = 0; e < 16; ++e) khat_f[e] = kf[e] * F[e];
        store_row16(sm.kf, row, g, khat_f);
#pragma unroll
        for (int e = 0; e < 16; ++e) tmp[e] = kf[e] * Y[e];
        pack8_split(tmp, kd[0][0], kdl[0][0]);
        pack8_split(tmp + 8, kd[0][1], kdl[0][1]);
#pragma unroll
        for (int e = 0; e < 16; ++e) tmp[e] = qf[e] * X[e];
        pack8_split(tmp, qd[0][0], qdl[0][0]);
        pack8_split(tmp + 8, qd[0][1], qdl[0][1]);
#pragma unroll
        for (int e = 0; e < 16; ++e) cum[0][e] = tmp[e] * Emid[e];  // q * exp(decay since the sub-block's near edge)
    }
    {
        float X[16], Y[16], F[16], Emid[16], EB[16];
        gate_factors<1>(lds_row_operand(sm.gb, row, g), r, X, Y, F, Emid, EB);
        if (r == 0) store_chan16(sm.eb[1][w], g, EB);
#pragma unroll
        for (int e = 0; e < 16; ++e) tmp[e] = kf[e] * F[e];
        store_row16(sm.kb, row, g, tmp);
#pragma unroll
        for (int e = 0; e < 16; ++e) tmp[e] = kf[e] * Y[e];
        pack8_split(tmp, kd[1][0], kdl[1][0]);
        pack8_split(tmp + 8, kd[1][1], kdl[1][1]);
#pragma unroll
        for (int e = 0; e < 16; ++e) tmp[e] = qf[e] * X[e];
        pack8_split(tmp, qd[1][0], qdl[1][0]);
        pack8_split(tmp + 8, qd[1][1], qdl[1][1]);
#pragma unroll
        for (int e = 0; e < 16; ++e) cum[1][e] = tmp[e] * Emid[e];
    }

    __syncthreads();  // eb, kf, kb visible; the raw gate tiles are no longer read
    prefetch_first();

    // query variants: qv[dir][d] pairs with the keys d+1 sub-blocks away in that direction's
    // past; after the last one the running query is the readout query (decay since the chunk edge)
    bf16x8 qv[2][3][2];
#pragma unroll
    for (int dir = 0; dir < 2; ++dir) {
        const int nb = dir == 0 ? w : 3 - w;
        qv[dir][0][0] = pack8(cum[dir]);
        qv[dir][0][1] = pack8(cum[dir] + 8);
#pragma unroll
        for (int d = 1; d <= 3; ++d) {
            if (d <= nb) {
                load_chan16(sm.eb[dir][dir == 0 ? w - d : w + d], g, tmp);
#pragma unroll
                for (int e = 0; e < 16; ++e) cum[dir][e] *= tmp[e];
                if (d < 3) {
                    qv[dir][d][0] = pack8(cum[dir]);
                    qv[dir][d][1] = pack8(cum[dir] + 8);
                }
            }
        }
    }
    const bf16x8 qf0 = pack8(cum[0]), qf1 = pack8(cum[0] + 8), qb0 = pack8(cum[1]), qb1 = pack8(cum[1] + 8);
    // forward state-update keys: decay to the chunk's right edge = khat times the sub-blocks to
    // the right; they take the place of the raw backward gates in LDS
#pragma unroll
    for (int sb = 1; sb < 4; ++sb) {
        if (sb > w) {
            load_chan16(sm.eb[0][sb], g, tmp);
#pragma unroll
            for (int e = 0; e < 16; ++e) khat_f[e] *= tmp[e];
        }
    }
    store_row16(sm.gb, row, g, khat_f);

    __syncthreads();  // state-update keys visible

#pragma unroll
    for (int I = 0; I < 4; ++I) {
        const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
        if (I == w) {
            f32x4 pf = zero, pb = zero;
#pragma unroll
            for (int kk = 0; kk < 2; ++kk) {  // small terms first
                pf = mfma(kdl[0][kk], qd[0][kk], mfma(kd[0][kk], qdl[0][kk], pf));
                pb = mfma(kdl[1][kk], qd[1][kk], mfma(kd[1][kk], qdl[1][kk], pb));
            }
#pragma unroll
            for (int kk = 0; kk < 2; ++kk) {
                pf = mfma(kd[0][kk], qd[0][kk], pf);
                pb = mfma(kd[1][kk], qd[1][kk], pb);
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int i = 4 * g + e;
                pf[e] = (i <= r ? pf[e] : 0.f) + (i >= r ? pb[e] : 0.f);
            }
            split4(pf, op.pk[I], op.pl[I]);
        } else {
            const bool fwd = I < w;
            const uint16_t(*kt)[kPitch] = fwd ? sm.kf : sm.kb;
            const bf16x8 a0 = *reinterpret_cast<const bf16x8 *>(&kt[16 * I + r][8 * g]);
            const bf16x8 a1 = *reinterpret_cast<const bf16x8 *>(&kt[16 * I + r][32 + 8 * g]);
            f32x4 p = zero;
#pragma unroll
            for (int d = 1; d <= 3; ++d) {
                if ((fwd ? w - I : I - w) == d) {
                    const int dir = fwd ? 0 : 1;
                    // compile-time variant index, uniform run-time choice of the direction
                    const bf16x8 b0 = dir == 0 ? qv[0][d - 1][0] : qv[1][d - 1][0];
                    const bf16x8 b1 = dir == 0 ? qv[0][d - 1][1] : qv[1][d - 1][1];
                    p = mfma(a1, b1, mfma(a0, b0, zero));
                }
            }
            split4(p, op.pk[I], op.pl[I]);
        }
    }
    op.qf0 = qf0; op.qf1 = qf1; op.qb0 = qb0; op.qb1 = qb1;
}

// kFastOnly = true : handles the segments the state kernel has flagged as entirely within the
//                     fast form's range, and contains no range-safe code (whose register
//                     footprint would otherwise spill into the fast path); other segments exit.
// kFastOnly = false: handles the remaining segments (all of them when seg_mild is nullptr), each
//                     chunk choosing its form.
// The kernels' LDS, at namespace scope so that the inlined fast-form code and the separately
// compiled general code address the same allocation as LDS (not through a generic reference).
// The state pass and the output pass use it one after the other (the single-launch kernel for
// one-segment plans runs both).
// Measurement aid: when set (vig_measure_alias_slabs), every slab reads the inputs of slab 0, so that q, k,
// v and the gates stay cache-resident while outputs and workspace are still written per slab.
__device__ int g_alias_inputs = 0;

union PathLds {
    OutLds out;
    StateLds state;
};
__shared__ PathLds g_lds;

// The LDS of a unit function: the four-wave kernels' own allocation, or, when the eight-wave kernels call
// the general code for a unit outside the fast form's range (kInWs), the front of THEIR allocation.
template <bool kInWs>
__device__ __forceinline__ PathLds &path_lds();
template <>
__device__ __forceinline__ PathLds &path_lds<false>()
{
    return g_lds;
}

// kLoc: the 2D gating locality injection of `lf` is applied to every chunk's rows before they are
// written, so that `out_all` receives the block output instead of the token mixer's.
template <bool kFastOnly, int kDk, bool kTm, bool kLoc, bool kInWs = false>
__device__ __forceinline__ void out_unit(
    const uint16_t *__restrict__ q_all, const uint16_t *__restrict__ k_all, const uint16_t *__restrict__ v_all,
    const uint16_t *__restrict__ gf_all, const uint16_t *__restrict__ gb_all, uint16_t *__restrict__ out_all,
    const float *__restrict__ seg_states, const unsigned char *__restrict__ stash_all, int L, int n_chunks,
    int seg_chunks, int n_seg, const long unit, int heads, const LocalityFusion &lf)
{
    OutLds &sm = path_lds<kInWs>().out;
    const int tid = threadIdx.x;
    const int w = tid >> 6, lane = tid & 63, r = lane & 15, g = lane >> 4;
    // The fast-form code of a 32-wide head skips the zero half of the key dimension: one K-step per
    // contraction over channels, no state rows (and no stash) for the waves that would own rows
    // 32..63.  The general code keeps the widened form throughout.
    constexpr int kKs = (kFastOnly && kDk == kD / 2) ? 1 : 2;
    const bool owns_rows = kKs > 1 || w < 2;
    long slab;
    int seg;
    unit_slab_segment(unit, n_seg, slab, seg);
    // first row of the slab and distance between its tokens, in rows of the tensor
    const long row0 = kTm ? (slab / heads) * L * heads + slab % heads : slab * L;
    const long row0_in = g_alias_inputs ? 0 : row0;
    const long base = row0 * kD, in_base = row0_in * kD, key_base = row0_in * kDk;
    // bytes between consecutive tokens of the slab, and the slab's extent from its first row
    const unsigned key_pitch = unsigned(heads) * kDk * 2u, val_pitch = unsigned(heads) * kD * 2u;
    const unsigned key_extent = unsigned(L - 1) * key_pitch + kDk * 2u, val_extent = unsigned(L - 1) * val_pitch + kD * 2u;
    const __amdgpu_buffer_rsrc_t q = slab_resource(q_all + key_base, key_extent);
    const __amdgpu_buffer_rsrc_t k = slab_resource(k_all + key_base, key_extent);
    const __amdgpu_buffer_rsrc_t g_fwd = slab_resource(gf_all + key_base, key_extent);
    const __amdgpu_buffer_rsrc_t g_bwd = slab_resource(gb_all + key_base, key_extent);
    const __amdgpu_buffer_rsrc_t v = slab_resource(v_all + in_base, val_extent);
    const __amdgpu_buffer_rsrc_t out = slab_resource(out_all + base, val_extent);
    const unsigned char *stash = stash_all + size_t(slab) * n_chunks * kStashBytes;

    const int chunk0 = seg * seg_chunks;
    const int nch = min(seg_chunks, n_chunks - chunk0);
    const bool seg_in = seg_states != nullptr && seg + 1 < n_seg;  // the last segment's entering backward state is zero
    const int row = 16 * w + r;

    LocalitySlab ls;
    if (kLoc) {
        // the head's taps and bias as fp32 in LDS (read after the first barrier of the first step)
        const int head = int(slab % lf.H);
        const uint16_t *taps = static_cast<const uint16_t *>(lf.w) + size_t(head) * kD * 9;
        for (int i = tid; i < kD * 9; i += kThreads) sm.cw[i % 9][i / 9] = bf16_lo_to_f32(taps[i]);
        if (tid < kD)
            sm.cb[tid] = lf.bias ? bf16_lo_to_f32(static_cast<const uint16_t *>(lf.bias)[head * kD + tid]) : 0.f;
        ls.x = slab_resource(static_cast<const uint16_t *>(lf.x) + base, val_extent);
        ls.z = slab_resource(static_cast<const uint16_t *>(lf.gate_logits) + base, val_extent);
        ls.Hg = lf.Hg;
        ls.Wg = lf.Wg;
    }

    // rows of the next chunk are fetched while the current chunk is being processed
    struct ChunkRows {
        Row16 sb;
        float4 dr;  // decay of the lane's state rows from the chunk's right edge to the segment's
        StagedRows q, k, gf, gb, v;
    };
    // The rows of the next chunk are requested a tile at a time between the phases of a step (a
    // burst of all thirteen loads would stall the wave at issue while the memory pipeline is
    // full).  m may run one past the segment: clamped, the rows are then unused.
    const LaneRows kr = lane_rows<kDk>(w, lane, key_pitch), vr = lane_rows<kD>(w, lane, val_pitch);
    auto chunk_token0 = [&](int m) { return unsigned(chunk0 + min(m, nch - 1)) * kC; };
    auto fetch_stash = [&](ChunkRows &c, int m) {
        // this lane's 16 values of the chunk's stashed state (unwritten, and unused, for the
        // segment's last chunk) and the decay of its rows
        // (waves without state rows read their first row's values instead: same cache lines, unused)
        const unsigned char *base = stash + size_t(chunk0 + min(m, nch - 1)) * kStashBytes;
        const uint4 *p = reinterpret_cast<const uint4 *>(base) + (owns_rows ? tid : (tid & 127));
        c.sb.p[0] = p[0];
        c.sb.p[1] = p[kThreads];
        c.dr = *reinterpret_cast<const float4 *>(base + size_t(kD) * kD * sizeof(uint16_t) +
                                                 (16 * (owns_rows ? w : (w & 1)) + 4 * g) * sizeof(float));
    };
    // part 0..5: q, k, g_fwd, g_bwd, v, stash
    auto fetch_part = [&](ChunkRows &c, int m, int part) {
        const unsigned t0 = chunk_token0(m);
        if (part == 0) c.q = load_rows(q, kr, t0);
        if (part == 1) c.k = load_rows(k, kr, t0);
        if (part == 2) c.gf = load_rows(g_fwd, kr, t0);
        if (part == 3) c.gb = load_rows(g_bwd, kr, t0);
        if (part == 4) c.v = load_rows(v, vr, t0);
        if (part == 5) fetch_stash(c, m);
    };
    // The general code, short of registers, fetches a chunk's rows at the start of its step
    // instead of one step ahead (measured faster there).
    ChunkRows next;
    if (kFastOnly) {
#pragma unroll
        for (int part = 0; part < 6; ++part) fetch_part(next, 0, part);
    }

    // States entering the segment, folded here from the segments' LOCAL end states and decays that
    // the state pass left in the workspace: forward from the left, E <- D_n * E + S_n over the
    // segments n < seg; backward from the right over n > seg (kept in registers: each step adds
    // its decayed copy to the chunk's stashed state, so that one readout serves both).  The loads
    // of up to four segments are in flight together.
    f32x4 S[4], Sseg[4];
#pragma unroll
    for (int jt = 0; jt < 4; ++jt) S[jt] = Sseg[jt] = f32x4{0.f, 0.f, 0.f, 0.f};
    if (seg_states != nullptr && owns_rows) {
        const float *slab_states = seg_states + slab * n_seg * kSegFloats;
        auto fold = [&](f32x4 (&E)[4], int dir, int first, int count, int step) {
            constexpr int kBatch = 4;
            for (int i0 = 0; i0 < count; i0 += kBatch) {
                f32x4 local[kBatch][4];
                float4 decay[kBatch];
#pragma unroll
                for (int u = 0; u < kBatch; ++u) {
                    const float *sp = slab_states + size_t(first + step * min(i0 + u, count - 1)) * kSegFloats;
#pragma unroll
                    for (int jt = 0; jt < 4; ++jt)
                        local[u][jt] = reinterpret_cast<const f32x4 *>(sp + dir * kD * kD)[kThreads * jt + tid];
                    decay[u] = *reinterpret_cast<const float4 *>(sp + kSegStateFloats + dir * kD + 16 * w + 4 * g);
                }
#pragma unroll
                for (int u = 0; u < kBatch; ++u) {
                    if (i0 + u < count) {
#pragma unroll
                        for (int jt = 0; jt < 4; ++jt) {
                            E[jt][0] = fmaf(E[jt][0], decay[u].x, local[u][jt][0]);
                            E[jt][1] = fmaf(E[jt][1], decay[u].y, local[u][jt][1]);
                            E[jt][2] = fmaf(E[jt][2], decay[u].z, local[u][jt][2]);
                            E[jt][3] = fmaf(E[jt][3], decay[u].w, local[u][jt][3]);
                        }
                    }
                }
            }
        };
        fold(S, 0, 0, seg, 1);
        fold(Sseg, 1, n_seg - 1, n_seg - 1 - seg, -1);
    }
    if (owns_rows) publish_state(sm.st, w, r, g, S);  // made visible by the first barrier of the first step
    bf16x8 tri_f[2], tri_b[2];
    scan_triangle<0>(w, r, g, tri_f);
    scan_triangle<1>(w, r, g, tri_b);

    for (int m = 0; m < nch; ++m) {
        if (!kFastOnly) {
#pragma unroll
            for (int part = 0; part < 6; ++part) fetch_part(next, m, part);
        }
        ChunkRows cur = next;
        zero_widened_half<kDk>(cur.q, lane);
        zero_widened_half<kDk>(cur.k, lane);
        zero_widened_half<kDk>(cur.gf, lane);
        zero_widened_half<kDk>(cur.gb, lane);
        ChunkFlags fl;
        fl.stash = m + 1 < nch;
        fl.seg = seg_in;

        // kf / kb are idle until this step's scaled keys are written: the wave's own rows of
        // them carry q and k from row order into operand order
        bounce_store(sm.kf, w, lane, cur.q);
        bounce_store(sm.kb, w, lane, cur.k);
        stage_gates(sm.gf, w, lane, cur.gf);
        stage_gates(sm.gb, w, lane, cur.gb);
        stage_values(sm.v, w, lane, cur.v);
        wave_lds_fence();
        const Row16 q_row = bounce_load(sm.kf, row, g), k_row = bounce_load(sm.kb, row, g);
        if ((fl.stash || fl.seg) && owns_rows) {
            // backward state entering the chunk from the right: the stash (accumulator order, zero
            // for the segment's last chunk) plus the segment's entering state decayed from the
            // segment's right edge to the chunk's; stored as a [column][channel] tile
            uint2 t[4] = {make_uint2(cur.sb.p[0].x, cur.sb.p[0].y), make_uint2(cur.sb.p[0].z, cur.sb.p[0].w),
                          make_uint2(cur.sb.p[1].x, cur.sb.p[1].y), make_uint2(cur.sb.p[1].z, cur.sb.p[1].w)};
            if (fl.seg) {
#pragma unroll
                for (int jt = 0; jt < 4; ++jt) {
                    f32x4 x = {0.f, 0.f, 0.f, 0.f};
                    if (fl.stash)
                        x = f32x4{bf16_lo_to_f32(t[jt].x), bf16_hi_to_f32(t[jt].x), bf16_lo_to_f32(t[jt].y),
                                  bf16_hi_to_f32(t[jt].y)};
                    x[0] = fmaf(cur.dr.x, Sseg[jt][0], x[0]);
                    x[1] = fmaf(cur.dr.y, Sseg[jt][1], x[1]);
                    x[2] = fmaf(cur.dr.z, Sseg[jt][2], x[2]);
                    x[3] = fmaf(cur.dr.w, Sseg[jt][3], x[3]);
                    t[jt] = pack4(x);
                }
            }
#pragma unroll
            for (int jt = 0; jt < 4; ++jt) *reinterpret_cast<uint2 *>(&sm.sb[16 * jt + r][16 * w + 4 * g]) = t[jt];
        }
        __syncthreads();  // staged tiles visible

        f32x4 Bf[4], Tf[4], Bb[4];
        ChunkOperands op;
        bool fast = true;
        // fast code: q and k after the barrier of the first half, both gates after the score
        // tiles, v and the stash after the readouts (finer splits measured slower)
        auto prefetch_first = [&]() {
            if (kFastOnly) {
                fetch_part(next, m + 1, 0);
                fetch_part(next, m + 1, 1);
            }
        };
        auto prefetch_second_half = [&](int point) {
            if (kFastOnly && point == 3) {
                fetch_part(next, m + 1, 4);
                fetch_part(next, m + 1, 5);
            }
        };
        if (kFastOnly) {
            out_chunk_fast_fused<kKs>(sm, tri_f, tri_b, w, r, g, q_row, k_row, op, prefetch_first);
        } else {
            f32x4 Tb[4];
            chunk_gate_scan(sm.gf, tri_f, r, g, Bf, Tf);
            chunk_gate_scan(sm.gb, tri_b, r, g, Bb, Tb);
            // same totals in every wave: the choice is uniform over the workgroup
            fast = fmaxf(chunk_decay_max(Tf), chunk_decay_max(Tb)) <= kMildRange;
            if (fast)
                out_chunk_fast(sm, w, r, g, Bf, Bb, Tf, q_row, k_row, fl, op, prefetch_first);
            else
                out_chunk_safe(sm, w, r, g, q_row, k_row, fl, op, prefetch_first);
        }
        if (kFastOnly) {
            fetch_part(next, m + 1, 2);
            fetch_part(next, m + 1, 3);
        }
        finish_chunk<kTm, kKs, kLoc>(sm, fast ? sm.kf : sm.gb, op, fl, fast, w, r, g, out, vr, unsigned(chunk0 + m) * kC,
                                     S, ls, prefetch_second_half);
    }
}

template <int kDk, bool kTm, bool kLoc, bool kInWs = false>
__device__ __attribute__((noinline)) void out_unit_general(
    const uint16_t *q_all, const uint16_t *k_all, const uint16_t *v_all, const uint16_t *gf_all, const uint16_t *gb_all,
    uint16_t *out_all, const float *seg_states, const unsigned char *stash_all, int L, int n_chunks, int seg_chunks,
    int n_seg, const long unit, int heads, const LocalityFusion &lf)
{
    out_unit<false, kDk, kTm, kLoc, kInWs>(q_all, k_all, v_all, gf_all, gb_all, out_all, seg_states, stash_all, L,
                                           n_chunks, seg_chunks, n_seg, unit, heads, lf);
}

// One workgroup per (slab, segment) unit.  kByFlag: units the state kernel flagged as mild run the
// fast-form code inline; the others call the general code as a real function, so that its
// register appetite (spilled to its own stack frame) does not touch the fast path's allocation
// and one launch serves both.  !kByFlag (single-chunk sequences, no flags): general code only.
template <bool kByFlag, int kDk, bool kTm, bool kLoc>
__global__ __launch_bounds__(kThreads, 2) void bigla_segment_out_kernel(
    const uint16_t *__restrict__ q_all, const uint16_t *__restrict__ k_all, const uint16_t *__restrict__ v_all,
    const uint16_t *__restrict__ gf_all, const uint16_t *__restrict__ gb_all, uint16_t *__restrict__ out_all,
    const float *__restrict__ seg_states /* states entering each segment, nullptr when one segment */,
    const int *__restrict__ seg_mild /* per unit: every chunk admits the fast form (kByFlag) */,
    const unsigned char *__restrict__ stash_all, int L, int n_chunks, int seg_chunks, int n_seg,
    int heads /* used when kTm: activations are [B,L,H,d] */, const LocalityFusion lf /* used when kLoc */)
{
    const long unit = blockIdx.x;
    if (kByFlag && seg_mild[unit] != 0)  // uniform over the workgroup
        out_unit<true, kDk, kTm, kLoc>(q_all, k_all, v_all, gf_all, gb_all, out_all, seg_states, stash_all, L,
                                       n_chunks, seg_chunks, n_seg, unit, heads, lf);
    else
        out_unit_general<kDk, kTm, kLoc>(q_all, k_all, v_all, gf_all, gb_all, out_all, seg_states, stash_all, L,
                                         n_chunks, seg_chunks, n_seg, unit, heads, lf);
}

// ---- kernel 1: per-segment end states and per-chunk backward stash -----------------------------

// One (slab, segment) unit of the state pass.  Returns whether every chunk admitted the fast form.
// seg_states == nullptr (one segment per slab): the end states are not needed and not stored.
// kFwd = false (only with seg_states == nullptr): nothing reads the forward end state, so the fast
// form skips the forward direction altogether (its cumulative gates, scaled keys and K^T V); the
// forward chunk totals are still formed, for the choice of the form.
template <int kDk, bool kTm, bool kFwd = true, bool kInWs = false>
__device__ __forceinline__ bool state_unit(
    const uint16_t *__restrict__ k_all, const uint16_t *__restrict__ v_all, const uint16_t *__restrict__ gf_all,
    const uint16_t *__restrict__ gb_all, float *__restrict__ seg_states, unsigned char *__restrict__ stash, int L,
    int n_chunks, int seg_chunks, int n_seg, const long unit, int heads)
{
    StateLds &sm = path_lds<kInWs>().state;
    const int tid = threadIdx.x;
    const int w = tid >> 6, lane = tid & 63, r = lane & 15, g = lane >> 4;
    long slab;
    int seg;
    unit_slab_segment(unit, n_seg, slab, seg);
    const long row0 = g_alias_inputs ? 0 : (kTm ? (slab / heads) * L * heads + slab % heads : slab * L);
    // bytes between consecutive tokens of the slab, and the slab's extent from its first row
    const unsigned key_pitch = unsigned(heads) * kDk * 2u, val_pitch = unsigned(heads) * kD * 2u;
    const unsigned key_extent = unsigned(L - 1) * key_pitch + kDk * 2u, val_extent = unsigned(L - 1) * val_pitch + kD * 2u;
    const __amdgpu_buffer_rsrc_t k = slab_resource(k_all + row0 * kDk, key_extent);
    const __amdgpu_buffer_rsrc_t g_fwd = slab_resource(gf_all + row0 * kDk, key_extent);
    const __amdgpu_buffer_rsrc_t g_bwd = slab_resource(gb_all + row0 * kDk, key_extent);
    const __amdgpu_buffer_rsrc_t v = slab_resource(v_all + row0 * kD, val_extent);
    float *dst = seg_states ? seg_states + (slab * n_seg + seg) * kSegFloats : nullptr;
    stash += size_t(slab) * n_chunks * kStashBytes;

    const int chunk0 = seg * seg_chunks;
    const int nch = min(seg_chunks, n_chunks - chunk0);
    const int row = 16 * w + r;

    // Sb: backward state, carried right to left (plain recurrence).  Sf: forward state at the
    // segment's RIGHT edge = sum_n (decay of the chunks right of n) * (chunk n's state at its own
    // right edge); walking right to left, chunk n's contribution is scaled once by the running
    // product rf and nothing accumulated ever decays again.  rf / rb: decay of the chunks seen
    // so far (rows at positions 16w + 4g + e).
    f32x4 Sf[4], Sb[4];
#pragma unroll
    for (int jt = 0; jt < 4; ++jt) {
        Sf[jt] = f32x4{0.f, 0.f, 0.f, 0.f};
        Sb[jt] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    float4 rf = make_float4(1.f, 1.f, 1.f, 1.f), rb = rf;
    bool all_fast = true;  // every chunk of the segment within the fast form's range

    struct ChunkRows {
        StagedRows k, v, gf, gb;
    };
    const LaneRows kr = lane_rows<kDk>(w, lane, key_pitch), vr = lane_rows<kD>(w, lane, val_pitch);
    auto fetch = [&](int m) {  // m may run one before the segment: clamped, the rows are then unused
        ChunkRows c;
        const unsigned t0 = unsigned(chunk0 + max(m, 0)) * kC;
        c.k = load_rows(k, kr, t0);
        c.v = load_rows(v, vr, t0);
        c.gf = load_rows(g_fwd, kr, t0);
        c.gb = load_rows(g_bwd, kr, t0);
        return c;
    };
    ChunkRows next = fetch(nch - 1);
    bf16x8 tri_f[2], tri_b[2];
    scan_triangle<0>(w, r, g, tri_f);
    scan_triangle<1>(w, r, g, tri_b);
    // A 32-wide head: channels 32..63 are zero padding.  The fast form skips them (half the
    // channel tiles in the scans, half the slots in the scalings, no K^T V for the waves that
    // own state rows 32..63, which stay zero); the range-safe form keeps the widened arithmetic.
    constexpr int kCt = kDk / 16, kSlots = kDk / 4;
    const bool owns_rows = 16 * w < kDk;

    for (int m = nch - 1; m >= 0; --m) {
        ChunkRows cur = next;
        zero_widened_half<kDk>(cur.k, lane);
        zero_widened_half<kDk>(cur.gf, lane);
        zero_widened_half<kDk>(cur.gb, lane);
        // the rows of chunk m-1 are requested a tile at a time between the phases of this step:
        // a burst of all of them would stall this wave at issue while the memory pipeline is full
        const unsigned far_token0 = unsigned(chunk0 + max(m - 1, 0)) * kC;
        next.k = load_rows(k, kr, far_token0);

        // stash for chunk m: the backward state entering it from the right (zero, and not
        // stored, for the segment's last chunk) and the decay from its right edge to the
        // segment's right edge
        {
            unsigned char *dstm = stash + size_t(chunk0 + m) * kStashBytes;
            if (m + 1 < nch) {  // accumulator order, two halves of 4 KB, each store contiguous over the wave
                uint4 *sdst = reinterpret_cast<uint4 *>(dstm) + tid;
                const uint2 a = pack4(Sb[0]), b = pack4(Sb[1]), c = pack4(Sb[2]), d = pack4(Sb[3]);
                sdst[0] = make_uint4(a.x, a.y, b.x, b.y);
                sdst[kThreads] = make_uint4(c.x, c.y, d.x, d.y);
            }
            if (r == 0)
                *reinterpret_cast<float4 *>(dstm + size_t(kD) * kD * sizeof(uint16_t) + (16 * w + 4 * g) * sizeof(float)) = rb;
        }

        // ks[0] is idle until this step's scaled keys are written: the wave's own rows of it
        // carry k from row order into operand order
        bounce_store(sm.ks[0], w, lane, cur.k);
        stage_gates(sm.g[0], w, lane, cur.gf);
        stage_gates(sm.g[1], w, lane, cur.gb);
        stage_values(sm.v, w, lane, cur.v);
        wave_lds_fence();
        float kf[16];
        unpack16(bounce_load(sm.ks[0], row, g), kf);
        __syncthreads();  // g, v visible
        next.v = load_rows(v, vr, far_token0);

        f32x4 Bf[4], Bb[4];
        float max_f, max_b;
        {
            f32x4 T[4];
            float t[16];
            if (kFwd) {
                chunk_gate_scan<kCt>(sm.g[0], tri_f, r, g, Bf, T);
            } else {
                chunk_gate_totals<kCt>(sm.g[0], r, g, T);
            }
            max_f = chunk_decay_max(T);
#pragma unroll
            for (int n = 0; n < 16; ++n) t[n] = T[n >> 2][n & 3];
            if (kFwd && r == 0) store_chan16(sm.tot[0], g, t);  // chunk totals per channel, operand order
            chunk_gate_scan<kCt>(sm.g[1], tri_b, r, g, Bb, T);
            max_b = chunk_decay_max(T);
#pragma unroll
            for (int n = 0; n < 16; ++n) t[n] = T[n >> 2][n & 3];
            if (r == 0) store_chan16(sm.tot[1], g, t);
        }
        const bool fast = fmaxf(max_f, max_b) <= kMildRange;  // uniform over the workgroup
        all_fast = all_fast && fast;
        next.gf = load_rows(g_fwd, kr, far_token0);
        float4 df, db;  // this chunk's decay, rows at LDS positions 16w + 4g + e
        float tmp[16];
        if (fast) {
            // keys k * exp(-b_i), b_i cumulative since the chunk edge of each direction
            float kb[16];
#pragma unroll
            for (int n = kSlots; n < 16; ++n) kb[n] = kf[n] = 0.f;
#pragma unroll
            for (int n = 0; n < kSlots; ++n) {
                kb[n] = kf[n] * fast_exp2(-kLog2e * Bb[n >> 2][n & 3]);
                if (kFwd) kf[n] = kf[n] * fast_exp2(-kLog2e * Bf[n >> 2][n & 3]);
            }
            if (kFwd) store_row16(sm.ks[0], row, g, kf);
            store_row16(sm.ks[1], row, g, kb);
            __syncthreads();  // ks, tot visible
            const float4 tb = *reinterpret_cast<const float4 *>(&sm.tot[1][16 * w + 4 * g]);
            df = make_float4(1.f, 1.f, 1.f, 1.f);
            if (kFwd) {
                const float4 tf = *reinterpret_cast<const float4 *>(&sm.tot[0][16 * w + 4 * g]);
                df = make_float4(fast_exp2(tf.x * kLog2e), fast_exp2(tf.y * kLog2e), fast_exp2(tf.z * kLog2e),
                                 fast_exp2(tf.w * kLog2e));
            }
            db = make_float4(fast_exp2(tb.x * kLog2e), fast_exp2(tb.y * kLog2e), fast_exp2(tb.z * kLog2e),
                             fast_exp2(tb.w * kLog2e));
        } else {
            // range-safe keys: decay from the token to the chunk edge, every factor <= 1.  One
            // direction at a time (this form is rare; fewer live registers matter more than a barrier)
            float F[16], EB[16];
            gate_factors_state<0>(lds_row_operand(sm.g[0], row, g), F, EB);
            if (r == 0) store_chan16(sm.eb[0][w], g, EB);
            __syncthreads();  // eb[0] visible
#pragma unroll
            for (int e = 0; e < 16; ++e) F[e] *= kf[e];
#pragma unroll
            for (int sb = 1; sb < 4; ++sb) {
                if (sb > w) {  // forward: the sub-blocks to the right
                    load_chan16(sm.eb[0][sb], g, tmp);
#pragma unroll
                    for (int e = 0; e < 16; ++e) F[e] *= tmp[e];
                }
            }
            store_row16(sm.ks[0], row, g, F);
            gate_factors_state<1>(lds_row_operand(sm.g[1], row, g), F, EB);
            if (r == 0) store_chan16(sm.eb[1][w], g, EB);
            __syncthreads();  // eb[1] visible
#pragma unroll
            for (int e = 0; e < 16; ++e) F[e] *= kf[e];
#pragma unroll
            for (int sb = 0; sb < 3; ++sb) {
                if (sb < w) {  // backward: the sub-blocks to the left
                    load_chan16(sm.eb[1][sb], g, tmp);
#pragma unroll
                    for (int e = 0; e < 16; ++e) F[e] *= tmp[e];
                }
            }
            store_row16(sm.ks[1], row, g, F);
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

        next.gb = load_rows(g_bwd, kr, far_token0);
        // chunk contributions K^T V of both directions, rows at positions 16w + 4g + e
        f32x4 Cf[4], Cb[4];
#pragma unroll
        for (int jt = 0; jt < 4; ++jt) {
            Cf[jt] = f32x4{0.f, 0.f, 0.f, 0.f};
            // fast: S_b = db * (S_b + Kb^T V) accumulates onto the state; safe: S_b = db * S_b + Kb^T V
            Cb[jt] = fast ? Sb[jt] : f32x4{0.f, 0.f, 0.f, 0.f};
        }
        if (owns_rows) {
#pragma unroll
            for (int p = 0; p < 2; ++p) {
                const bf16x8 ab = token_operand(sm.ks[1], 2 * p, 2 * p + 1, 16 * w, r, g);
                bf16x8 af = ab;
                if (kFwd) af = token_operand(sm.ks[0], 2 * p, 2 * p + 1, 16 * w, r, g);
#pragma unroll
                for (int jt = 0; jt < 4; ++jt) {
                    const bf16x8 vb = token_operand(sm.v, 2 * p, 2 * p + 1, 16 * jt, r, g);
                    if (kFwd) Cf[jt] = mfma(af, vb, Cf[jt]);
                    Cb[jt] = mfma(ab, vb, Cb[jt]);
                }
            }
        }
        // forward: chunk state at its own right edge is df * Cf (fast) or Cf (safe); scale by the
        // decay of the chunks to its right
        const float4 sf4 = fast ? make_float4(rf.x * df.x, rf.y * df.y, rf.z * df.z, rf.w * df.w) : rf;
#pragma unroll
        for (int jt = 0; jt < 4; ++jt) {
            if (fast) {
                Sb[jt][0] = Cb[jt][0] * db.x; Sb[jt][1] = Cb[jt][1] * db.y;
                Sb[jt][2] = Cb[jt][2] * db.z; Sb[jt][3] = Cb[jt][3] * db.w;
            } else {
                Sb[jt][0] = fmaf(Sb[jt][0], db.x, Cb[jt][0]); Sb[jt][1] = fmaf(Sb[jt][1], db.y, Cb[jt][1]);
                Sb[jt][2] = fmaf(Sb[jt][2], db.z, Cb[jt][2]); Sb[jt][3] = fmaf(Sb[jt][3], db.w, Cb[jt][3]);
            }
            if (kFwd) {
                Sf[jt][0] = fmaf(Cf[jt][0], sf4.x, Sf[jt][0]); Sf[jt][1] = fmaf(Cf[jt][1], sf4.y, Sf[jt][1]);
                Sf[jt][2] = fmaf(Cf[jt][2], sf4.z, Sf[jt][2]); Sf[jt][3] = fmaf(Cf[jt][3], sf4.w, Sf[jt][3]);
            }
        }
        if (kFwd) {
            rf.x *= df.x; rf.y *= df.y; rf.z *= df.z; rf.w *= df.w;
        }
        rb.x *= db.x; rb.y *= db.y; rb.z *= db.z; rb.w *= db.w;
        __syncthreads();  // every read of this chunk's LDS tiles is done
    }

    if (seg_states) {
#pragma unroll
        for (int jt = 0; jt < 4; ++jt) {
            reinterpret_cast<f32x4 *>(dst)[kThreads * jt + tid] = Sf[jt];
            reinterpret_cast<f32x4 *>(dst + size_t(kD) * kD)[kThreads * jt + tid] = Sb[jt];
        }
        if (r == 0) {
            *reinterpret_cast<float4 *>(dst + kSegStateFloats + 16 * w + 4 * g) = rf;
            *reinterpret_cast<float4 *>(dst + kSegStateFloats + kD + 16 * w + 4 * g) = rb;
        }
    }
    return all_fast;
}

template <int kDk, bool kTm>
__global__ __launch_bounds__(kThreads, 2) void bigla_segment_state_kernel(
    const uint16_t *__restrict__ k, const uint16_t *__restrict__ v, const uint16_t *__restrict__ g_fwd,
    const uint16_t *__restrict__ g_bwd, float *__restrict__ seg_states, int *__restrict__ seg_mild,
    unsigned char *__restrict__ stash, int L, int n_chunks, int seg_chunks, int n_seg,
    int heads /* used when kTm: activations are [B,L,H,d] */)
{
    const bool all_fast =
        state_unit<kDk, kTm>(k, v, g_fwd, g_bwd, seg_states, stash, L, n_chunks, seg_chunks, n_seg, blockIdx.x, heads);
    if (threadIdx.x == 0) seg_mild[blockIdx.x] = all_fast ? 1 : 0;
}

// One-segment plans (a workgroup per slab): state pass and output pass in ONE launch.  The stash
// the state pass writes is read back by the same workgroup (the barrier between the passes orders
// the global writes before the reads), no segment states or flags go through memory, and the
// second read of k, v and the gates finds them in L2.
template <int kDk, bool kTm, bool kLoc>
__global__ __launch_bounds__(kThreads, 2) void bigla_slab_kernel(
    const uint16_t *__restrict__ q, const uint16_t *__restrict__ k, const uint16_t *__restrict__ v,
    const uint16_t *__restrict__ g_fwd, const uint16_t *__restrict__ g_bwd, uint16_t *__restrict__ out,
    unsigned char *__restrict__ stash, int L, int n_chunks, int heads, const LocalityFusion lf)
{
    const long unit = blockIdx.x;
    const bool all_fast =
        state_unit<kDk, kTm, false>(k, v, g_fwd, g_bwd, nullptr, stash, L, n_chunks, n_chunks, 1, unit, heads);
    __syncthreads();  // stash written (and complete), the state pass's LDS no longer read
    if (all_fast)     // uniform over the workgroup
        out_unit<true, kDk, kTm, kLoc>(q, k, v, g_fwd, g_bwd, out, nullptr, stash, L, n_chunks, n_chunks, 1, unit,
                                       heads, lf);
    else
        out_unit_general<kDk, kTm, kLoc>(q, k, v, g_fwd, g_bwd, out, nullptr, stash, L, n_chunks, n_chunks, 1, unit,
                                         heads, lf);
}

}  // namespace

}  // namespace vig

#include "bigla_chunk_ws.hpp"

namespace vig {

bool bigla_chunk_supported(int dk, int dv, bool is_bf16) { return is_bf16 && dv == kD && (dk == kD || dk == kD / 2); }

namespace {
size_t seg_region_bytes(long BH, const Plan &p) { return size_t(BH) * p.n_seg * kSegFloats * sizeof(float); }
size_t flag_region_bytes(long BH, const Plan &p) { return (size_t(BH) * p.n_seg * sizeof(int) + 15) / 16 * 16; }
}  // namespace

namespace {
size_t four_wave_bytes(long BH, int L)
{
    const Plan p = make_plan(BH, L);
    return seg_region_bytes(BH, p) + flag_region_bytes(BH, p) + size_t(BH) * p.n_chunks * kStashBytes;
}
}  // namespace

// either set of kernels may run a call: the workspace holds the larger of the two layouts
size_t bigla_chunk_workspace_bytes(long BH, int L)
{
    const size_t a = four_wave_bytes(BH, L), b = bigla_chunk_ws_workspace_bytes(BH, L);
    return a > b ? a : b;
}

namespace {
template <int kDk, bool kTm, bool kLoc>
hipError_t chunk_launch(const void *q, const void *k, const void *v, const void *g_fwd, const void *g_bwd, void *out,
                        long BH, int L, int heads_token_major, const LocalityFusion &lf, bool slab_sweep,
                        void *workspace, hipStream_t stream)
{
    Plan p = make_plan(BH, L);
    if (slab_sweep) {  // one segment per slab whatever the shape (needs no more workspace than the plan's own)
        p.seg_chunks = p.n_chunks;
        p.n_seg = 1;
    }
    const long blocks = BH * p.n_seg;
    if (blocks > 0x7fffffffL) return hipErrorInvalidValue;
    const uint16_t *qq = static_cast<const uint16_t *>(q), *kk = static_cast<const uint16_t *>(k);
    const uint16_t *vv = static_cast<const uint16_t *>(v);
    const uint16_t *gf = static_cast<const uint16_t *>(g_fwd), *gb = static_cast<const uint16_t *>(g_bwd);
    float *seg_states = static_cast<float *>(workspace);
    int *seg_mild = reinterpret_cast<int *>(static_cast<unsigned char *>(workspace) + seg_region_bytes(BH, p));
    unsigned char *stash = reinterpret_cast<unsigned char *>(seg_mild) + flag_region_bytes(BH, p);
    hipError_t e = hipSuccess;
    uint16_t *oo = static_cast<uint16_t *>(out);
    if (p.n_seg == 1 && p.n_chunks > 1) {  // one workgroup per slab does both passes in one launch
        LaunchTimer timer(kKernelSlab, stream);
        hipLaunchKernelGGL((bigla_slab_kernel<kDk, kTm, kLoc>), dim3((unsigned)blocks), dim3(kThreads), 0, stream, qq,
                           kk, vv, gf, gb, oo, stash, L, p.n_chunks, heads_token_major, lf);
        return hipGetLastError();
    }
    if (p.n_chunks > 1) {  // a single chunk has neither a stash nor entering states
        {
            LaunchTimer timer(kKernelSegmentState, stream);
            hipLaunchKernelGGL((bigla_segment_state_kernel<kDk, kTm>), dim3((unsigned)blocks), dim3(kThreads), 0, stream, kk, vv,
                               gf, gb, seg_states, seg_mild, stash, L, p.n_chunks, p.seg_chunks, p.n_seg,
                               heads_token_major);
        }
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    const float *seg_in = p.n_seg > 1 ? seg_states : nullptr;
    const int *flags = p.n_chunks > 1 ? seg_mild : nullptr;
    {
        LaunchTimer timer(flags ? kKernelSegmentOut : kKernelSegmentOutGeneral, stream);
        if (flags)
            hipLaunchKernelGGL((bigla_segment_out_kernel<true, kDk, kTm, kLoc>), dim3((unsigned)blocks),
                               dim3(kThreads), 0, stream, qq, kk, vv, gf, gb, oo, seg_in, flags, stash, L, p.n_chunks,
                               p.seg_chunks, p.n_seg, heads_token_major, lf);
        else  // a single chunk per sequence: no state kernel has run, no flags exist
            hipLaunchKernelGGL((bigla_segment_out_kernel<false, kDk, kTm, kLoc>), dim3((unsigned)blocks),
                               dim3(kThreads), 0, stream, qq, kk, vv, gf, gb, oo, seg_in, flags, stash, L, p.n_chunks,
                               p.seg_chunks, p.n_seg, heads_token_major, lf);
    }
    return hipGetLastError();
}
}  // namespace

namespace {
bool g_alias_on = false;  // host copy of g_alias_inputs
}

hipError_t bigla_chunk_set_alias(int on)
{
    g_alias_on = on != 0;
    return hipMemcpyToSymbol(HIP_SYMBOL(g_alias_inputs), &on, sizeof(int));
}

bool bigla_chunk_gated_selectable(long BH, int L, int dk) { return !g_alias_on && bigla_chunk_ws_applicable(BH, L, dk); }

// bigla_chunk_launch with the eight-wave kernels, the state pass making the gates from the gate producer's
// low-rank half (and writing them to g_fwd, g_bwd, which the output pass then reads).
hipError_t bigla_chunk_gated_launch(const void *q, const void *k, const void *v, void *g_fwd, void *g_bwd, void *out,
                                    long BH, int L, int dk, int n_heads, int heads_token_major, const void *lowrank,
                                    const void *w2, const void *bias, float tau, void *workspace, hipStream_t stream)
{
    if (!bigla_chunk_ws_applicable(BH, L, dk) || n_heads <= 0 || BH % n_heads != 0) return hipErrorInvalidValue;
    if (g_alias_on) return hipErrorInvalidValue;  // aliased slabs would all write the first slab's gates
    GateSource gs;
    gs.lowrank = static_cast<const uint16_t *>(lowrank);
    gs.w2 = static_cast<const uint16_t *>(w2);
    gs.bias = static_cast<const uint16_t *>(bias);
    gs.inv_tau = 1.f / tau;
    gs.n_heads = n_heads;
    return bigla_chunk_ws_launch(q, k, v, g_fwd, g_bwd, out, BH, L, dk, heads_token_major, workspace, stream, &gs);
}

bool bigla_chunk_ws_selectable(long BH, int L, int dk) { return bigla_chunk_ws_applicable(BH, L, dk); }

hipError_t bigla_chunk_launch(const void *q, const void *k, const void *v, const void *g_fwd, const void *g_bwd,
                              void *out, long BH, int L, int dk, int heads_token_major, const LocalityFusion *fusion,
                              int kernels, void *workspace, hipStream_t stream)
{
    const bool tm = heads_token_major > 0;
    const int heads = tm ? heads_token_major : 1;
    if (dk != kD && dk != kD / 2) return hipErrorInvalidValue;
    const LocalityFusion none = {};
    // (key width, layout, fused epilogue) pick the instantiation
    // kernels: 0 = the faster set for the shape (the eight-wave kernels where they apply), 1 = four-wave,
    // 2 = eight-wave (an error where they do not apply), 3 = four-wave with one workgroup per slab
    // (with a fusion: grids narrow enough for the eight-wave epilogue's ring of conv-input rows)
    const bool ws_ok = bigla_chunk_ws_applicable(BH, L, dk) && (!fusion || (fusion->Wg < kXHalo && L < (1 << 22)));
    if (kernels == 2 && !ws_ok) return hipErrorInvalidValue;
    if (kernels == 2 || (kernels == 0 && ws_ok)) {
        return bigla_chunk_ws_launch(q, k, v, g_fwd, g_bwd, out, BH, L, dk, heads_token_major, workspace, stream,
                                     nullptr, fusion);
    }
    auto go = [&](auto dk_c, auto tm_c, auto loc_c) {
        return chunk_launch<decltype(dk_c)::value, decltype(tm_c)::value, decltype(loc_c)::value>(
            q, k, v, g_fwd, g_bwd, out, BH, L, heads, fusion ? *fusion : none, kernels == 3, workspace, stream);
    };
    using std::integral_constant;
    using std::true_type;
    using std::false_type;
    typedef integral_constant<int, kD> wide;
    typedef integral_constant<int, kD / 2> half;
    if (fusion) {
        if (dk == kD) return tm ? go(wide{}, true_type{}, true_type{}) : go(wide{}, false_type{}, true_type{});
        return tm ? go(half{}, true_type{}, true_type{}) : go(half{}, false_type{}, true_type{});
    }
    if (dk == kD) return tm ? go(wide{}, true_type{}, false_type{}) : go(wide{}, false_type{}, false_type{});
    return tm ? go(half{}, true_type{}, false_type{}) : go(half{}, false_type{}, false_type{});
}

}  // namespace vig
