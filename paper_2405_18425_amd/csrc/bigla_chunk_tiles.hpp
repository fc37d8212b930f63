// Tiles, lane layouts and matrix-core building blocks shared by the chunkwise BiGLA forward
// kernels (Section 4.2.1, Eq. (BiGLA)): the four-wave kernels of bigla_chunk.hip and the
// wave-specialised kernels of bigla_chunk_ws.hip.  The algebra of the chunkwise regrouping and the
// wavefront mapping are described at the head of bigla_chunk.hip.
#pragma once

#include "vig_common.hpp"

namespace vig {

namespace {

constexpr int kC = 64;          // chunk length (tokens)
constexpr int kD = 64;          // dk = dv
constexpr int kPitch = 72;      // LDS row pitch in bf16 elements (64 + 8: 16-byte aligned, bank-staggered)
constexpr int kTargetWorkgroups = 512;  // segments are sized so that about this many workgroups are launched
constexpr int kThreads = 256;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kGateFloorLog2 = -8.0f * kLog2e;  // per-step floor of the log-gate (range-safe form), log2 domain
// Chunk log-decays (nats, largest over the channels) that bound the forms of a chunk's evaluation.
//   kFastRange: beyond it the factors exp(-b) of the fast form leave the range in which fp32 products of
//     them are safe; such chunks take the range-safe form.
//   kMildRange: the faster the decay, the fewer tokens an output sums over, and the rounding of the exp-scaled
//     operands of a token's nearest few products then stands against a smaller output (emulated on the CPU:
//     from 0.2 to 0.5 nats per step the worst element of 400 000 sits at 0.55-0.8 of a bound of 2 % of
//     |value| + slab rms with bf16 operands and at 0.2-0.4 with the diagonal tile exact; a random case at
//     0.48 nats per step reached 1.13).  Beyond a quarter of a nat per step the operands of the diagonal score
//     tile are split into two bf16 terms: the eight-wave kernels do that inside the fast form, the four-wave
//     kernels take the range-safe form (which splits them always).  Gates of the paper's form at the
//     benchmark's statistics stay under 11 nats per chunk.
constexpr float kFastRange = 60.0f;
constexpr float kMildRange = 16.0f;

// ---- small device helpers ------------------------------------------------------------------

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

__device__ __forceinline__ bf16x8 pack8(const float *f)
{
    uint4 u;
    u.x = pack2(f[0], f[1]);
    u.y = pack2(f[2], f[3]);
    u.z = pack2(f[4], f[5]);
    u.w = pack2(f[6], f[7]);
    return __builtin_bit_cast(bf16x8, u);
}

// f = hi + lo with both parts bf16: the pair carries 16 significant bits of every value
__device__ __forceinline__ void pack8_split(const float *f, bf16x8 &hi, bf16x8 &lo)
{
    uint4 h, l;
    uint32_t *hp = &h.x, *lp = &l.x;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        hp[i] = pack2(f[2 * i], f[2 * i + 1]);
        lp[i] = pack2(f[2 * i] - bf16_lo_to_f32(hp[i]), f[2 * i + 1] - bf16_hi_to_f32(hp[i]));
    }
    hi = __builtin_bit_cast(bf16x8, h);
    lo = __builtin_bit_cast(bf16x8, l);
}

__device__ __forceinline__ void unpack8(const uint4 &u, float *f)
{
    f[0] = bf16_lo_to_f32(u.x); f[1] = bf16_hi_to_f32(u.x);
    f[2] = bf16_lo_to_f32(u.y); f[3] = bf16_hi_to_f32(u.y);
    f[4] = bf16_lo_to_f32(u.z); f[5] = bf16_hi_to_f32(u.z);
    f[6] = bf16_lo_to_f32(u.w); f[7] = bf16_hi_to_f32(u.w);
}

// 16 bf16 values of one token held by a lane, packed two per dword
struct Row16 {
    uint4 p[2];
};

// Every global row access is a fully contiguous wave access, 8 whole 128-byte rows per instruction:
// lane i of wave w takes 16-byte piece i%8 of rows 16w + i/8 and 16w + 8 + i/8 of the chunk.
struct StagedRows {
    uint4 p[2];
};

// Byte offsets of a lane's two pieces inside a chunk, for rows of kRow elements `pitch` bytes apart
// (head-major [B, H, L, d]: pitch = 2 * kRow; token-major [B, L, H, d]: pitch = 2 * H * kRow).
// Rows of 32 (keys, queries and gates of a 32-wide head) are widened to the kernels' 64 channels
// with zeros: channels 32..63 then carry q = k = 0 and log-gate 0 through every later step, which
// leaves the result unchanged.  The lanes of the zero half repeat the addresses of the other half
// (the instruction still touches whole rows) and are cleared by zero_widened_half when the rows
// are consumed.
struct LaneRows {
    unsigned off[2];
    unsigned pitch;
};

template <int kRow>
__device__ __forceinline__ LaneRows lane_rows(int w, int lane, unsigned pitch)
{
    static_assert(kRow == kD || kRow == kD / 2, "row length");
    constexpr int kPieces = kRow / 8;
    LaneRows r;
    r.pitch = pitch;
#pragma unroll
    for (int t = 0; t < 2; ++t) r.off[t] = unsigned(16 * w + 8 * t + (lane >> 3)) * pitch + 16u * ((lane & 7) % kPieces);
    return r;
}

// The lane's pieces of the chunk that starts at token chunk_token0 (below 2^24)
__device__ __forceinline__ StagedRows load_rows(__amdgpu_buffer_rsrc_t rows, const LaneRows &lr, unsigned chunk_token0)
{
    const unsigned chunk_off = chunk_token0 * lr.pitch;
    StagedRows s;
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rows, lr.off[t] + chunk_off, 0, 0);
        s.p[t] = make_uint4(v.x, v.y, v.z, v.w);
    }
    return s;
}

// The zero half of a widened 32-wide row, applied when the rows are consumed (a select right
// after the load would make the wave wait for it at once).
template <int kRow>
__device__ __forceinline__ void zero_widened_half(StagedRows &s, int lane)
{
    if (kRow < kD && (lane & 7) >= kRow / 8) s.p[0] = s.p[1] = make_uint4(0, 0, 0, 0);
}

// Orders this wave's earlier LDS writes before its later LDS reads of what other lanes of the
// same wave wrote (the LDS executes one wave's accesses in order; this keeps the compiler from
// moving them across each other).
__device__ __forceinline__ void wave_lds_fence()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Operand rows (q, k) arrive as contiguous rows too; the wave turns its own 16 rows into the
// operand layout through 16 tile rows that no other wave touches at that point.
__device__ __forceinline__ void bounce_store(uint16_t (*tile)[kPitch], int w, int lane, const StagedRows &s)
{
#pragma unroll
    for (int t = 0; t < 2; ++t)
        *reinterpret_cast<uint4 *>(&tile[16 * w + 8 * t + (lane >> 3)][8 * (lane & 7)]) = s.p[t];
}

__device__ __forceinline__ Row16 bounce_load(const uint16_t (*tile)[kPitch], int row, int g)
{
    Row16 r;
    r.p[0] = *reinterpret_cast<const uint4 *>(&tile[row][8 * g]);
    r.p[1] = *reinterpret_cast<const uint4 *>(&tile[row][32 + 8 * g]);
    return r;
}

// values: natural column order
__device__ __forceinline__ void stage_values(uint16_t (*tile)[kPitch], int w, int lane, const StagedRows &s)
{
#pragma unroll
    for (int t = 0; t < 2; ++t)
        *reinterpret_cast<uint4 *>(&tile[16 * w + 8 * t + (lane >> 3)][8 * (lane & 7)]) = s.p[t];
}

// log-gates: columns permuted so that the gate scan's 16-channel tiles come out in operand
// order.  Channel 32kk + 8g + 4h + e is stored at column 16*(2kk + h) + 4g + e: the piece with
// channels 8p..8p+7 (p = 4kk + g) is split into its two 8-byte halves.
__device__ __forceinline__ void stage_gates(uint16_t (*tile)[kPitch], int w, int lane, const StagedRows &s)
{
    const int piece = lane & 7, kk = piece >> 2, gg = piece & 3;
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        const int row = 16 * w + 8 * t + (lane >> 3);
        *reinterpret_cast<uint2 *>(&tile[row][32 * kk + 4 * gg]) = make_uint2(s.p[t].x, s.p[t].y);
        *reinterpret_cast<uint2 *>(&tile[row][32 * kk + 16 + 4 * gg]) = make_uint2(s.p[t].z, s.p[t].w);
    }
}

// The lane's 16 slots of one token out of a staged gate tile (column order of stage_gates)
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
    uint16_t kf[kC][kPitch];    // forward-scaled keys           [token][channel, operand order]
    uint16_t kb[kC][kPitch];    // backward-scaled keys          [token][channel, operand order]
    uint16_t gf[kC][kPitch];    // raw forward log-gates         [token][channel, natural order]
    uint16_t gb[kC][kPitch];    // raw backward log-gates        [token][channel, natural order];
                                // the range-safe form reuses it for the forward state-update keys
    uint16_t v[kC][kPitch];     // values                        [token][column]
    uint16_t st[kD][kPitch];    // forward state, bf16 copy      [column][channel, operand order]
    uint16_t sb[kD][kPitch];    // stashed backward state entering the chunk, same layout
    float tot[kD];              // forward chunk total log-gate per channel (fast form), operand order
    float eb[2][4][kD];         // whole-sub-block decay factors per channel (range-safe form)
    float cw[9][kD];            // fused locality epilogue: the head's 3x3 taps, [tap][channel]
    float cb[kD];               //                          and its conv bias
};

struct __align__(16) StateLds {
    uint16_t ks[2][kC][kPitch];
    uint16_t g[2][kC][kPitch];
    uint16_t v[kC][kPitch];
    float tot[2][kD];
    float eb[2][4][kD];
};

// Workspace: [segment region][segment flags][stash region].
//   segment region, per (slab, segment): two fp32 64x64 states (forward, backward) in
//     accumulator order (float4 number 256*jt + t belongs to thread t of the workgroup:
//     column 16*jt + r of rows 16w + 4g + e), then two fp32 decay vectors indexed by row: the
//     segment's LOCAL end states (forward at its right edge, backward at its left edge, both
//     from a zero start) and total decays, written by the state pass, folded by the output pass.
//   segment flags, per (slab, segment): one int, non-zero when every chunk of the segment
//     admits the fast form (written by the state kernel); padded to a multiple of 16 bytes.
//   stash region, per (slab, chunk): one bf16 64x64 state in accumulator order (thread t of
//     the workgroup owns 16 consecutive values: columns 16*jt + r of rows 16w + 4g + e), then
//     one fp32 decay vector.
constexpr size_t kSegStateFloats = 2 * size_t(kD) * kD;
constexpr size_t kSegFloats = kSegStateFloats + 2 * kD;
constexpr size_t kStashBytes = size_t(kD) * kD * sizeof(uint16_t) + kD * sizeof(float);

struct Plan {
    int n_chunks, seg_chunks, n_seg;
};

inline Plan make_plan(long BH, int L)
{
    Plan p;
    p.n_chunks = (L + kC - 1) / kC;
    long want = kTargetWorkgroups / (BH > 0 ? BH : 1);
    if (want < 1) want = 1;
    if (want > p.n_chunks) want = p.n_chunks;
    // short sequences with at least half a chip of slabs: one segment per slab saves the scan
    // launch and the segment states, which outweighs the longer walk (measured at L = 196)
    if (BH >= 128 && p.n_chunks <= 4) want = 1;
    p.seg_chunks = int((p.n_chunks + want - 1) / want);
    p.n_seg = (p.n_chunks + p.seg_chunks - 1) / p.seg_chunks;
    return p;
}

// Token-major MFMA operands of a 64-token tile for contractions over tokens.  k-slot layout:
// slots 0..3 = tokens 4g..4g+3 of sub-block s0, slots 4..7 = the same tokens of sub-block s1.
__device__ __forceinline__ bf16x8 token_operand(const uint16_t (*tile)[kPitch], int s0, int s1, int col0, int r,
                                                int g)
{
    const int tr_row = 4 * g + (r >> 2), tr_col = col0 + 4 * (r & 3);
    return join(lds_read_tr(&tile[16 * s0 + tr_row][tr_col]), lds_read_tr(&tile[16 * s1 + tr_row][tr_col]));
}

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
// kCt < 4: only the first kCt channel tiles carry data (a 32-wide head), the others are zero.
template <int kCt = 4>
__device__ __forceinline__ void chunk_gate_scan(const uint16_t (*gtile)[kPitch], const bf16x8 (&tri)[2], int r, int g,
                                                f32x4 (&B)[4], f32x4 (&T)[4])
{
    const bf16x8 ones = __builtin_bit_cast(bf16x8, make_uint4(0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u));
#pragma unroll
    for (int ct = kCt; ct < 4; ++ct) B[ct] = T[ct] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ct = 0; ct < kCt; ++ct) {
        const bf16x8 a0 = token_operand(gtile, 0, 1, 16 * ct, r, g);
        const bf16x8 a1 = token_operand(gtile, 2, 3, 16 * ct, r, g);
        const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
        B[ct] = mfma(a1, tri[1], mfma(a0, tri[0], zero));
        T[ct] = mfma(a1, ones, mfma(a0, ones, zero));
    }
}

// Largest chunk log-decay (nats) over all 64 channels, identical in every lane of the wave: the
// four lanes 0, 16, 32, 48 together hold the totals of every channel.
// Chunk totals alone (where the cumulative gates of a direction are not needed)
template <int kCt = 4>
__device__ __forceinline__ void chunk_gate_totals(const uint16_t (*gtile)[kPitch], int r, int g, f32x4 (&T)[4])
{
    const bf16x8 ones = __builtin_bit_cast(bf16x8, make_uint4(0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u));
#pragma unroll
    for (int ct = kCt; ct < 4; ++ct) T[ct] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ct = 0; ct < kCt; ++ct) {
        const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
        T[ct] = mfma(token_operand(gtile, 2, 3, 16 * ct, r, g), ones,
                     mfma(token_operand(gtile, 0, 1, 16 * ct, r, g), ones, zero));
    }
}

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

// bf16 copy of an fp32 state tile held in accumulator layout (rows at positions 16w + 4g + e,
// column 16*jt + r) into a [column][channel] tile
__device__ __forceinline__ void publish_state(uint16_t (*tile)[kPitch], int w, int r, int g, const f32x4 (&S)[4])
{
#pragma unroll
    for (int jt = 0; jt < 4; ++jt) *reinterpret_cast<uint2 *>(&tile[16 * jt + r][16 * w + 4 * g]) = pack4(S[jt]);
}

__device__ __forceinline__ void load_state(const float *src, bool zero, int tid, f32x4 (&S)[4])
{
#pragma unroll
    for (int jt = 0; jt < 4; ++jt) {
        S[jt] = f32x4{0.f, 0.f, 0.f, 0.f};
        if (!zero) S[jt] = reinterpret_cast<const f32x4 *>(src)[kThreads * jt + tid];
    }
}

// O^T += S^T q^T for one [column][channel] state tile (readout of a state by scaled queries)
// kKs = 1: only channels 0..31 carry data (a 32-wide head widened with zeros), the second K-step
// is skipped.
template <int kKs = 2>
__device__ __forceinline__ void readout(const uint16_t (*tile)[kPitch], bf16x8 q0, bf16x8 q1, int r, int g,
                                        f32x4 (&O)[4])
{
#pragma unroll
    for (int jt = 0; jt < 4; ++jt) {
        const bf16x8 s0 = *reinterpret_cast<const bf16x8 *>(&tile[16 * jt + r][8 * g]);
        O[jt] = mfma(s0, q0, O[jt]);
        if (kKs > 1) {
            const bf16x8 s1 = *reinterpret_cast<const bf16x8 *>(&tile[16 * jt + r][32 + 8 * g]);
            O[jt] = mfma(s1, q1, O[jt]);
        }
    }
}

// x = hi + lo with both halves bf16 (hi = bf16(x), lo = bf16(x - hi))
__device__ __forceinline__ void split4(const f32x4 &x, uint2 &hi, uint2 &lo)
{
    hi = pack4(x);
    const f32x4 h = unpack4(hi);
    lo = pack4(f32x4{x[0] - h[0], x[1] - h[1], x[2] - h[2], x[3] - h[3]});
}

__device__ __forceinline__ bf16x8 operand(const uint2 &a, const uint2 &b)
{
    return __builtin_bit_cast(bf16x8, make_uint4(a.x, a.y, b.x, b.y));
}

// Which (slab, segment) a workgroup handles.  Workgroups go to the eight XCDs round-robin by index
// and each XCD has an L2 of its own: when the slab count divides by eight, all segments of a slab
// are given to workgroups of one XCD, so that the segment states the state pass leaves behind are
// found in that L2 when the output pass folds them (and the stash of a chunk is read where it was
// written in either case: both passes use the same mapping).
__device__ __forceinline__ void unit_slab_segment(long unit, int n_seg, long &slab, int &seg)
{
    const long n_slabs = gridDim.x / unsigned(n_seg);
    if (n_slabs % 8 == 0) {
        const long j = unit / 8;
        slab = unit % 8 + 8 * (j / n_seg);
        seg = int(j % n_seg);
    } else {
        slab = unit / n_seg;
        seg = int(unit % n_seg);
    }
}

}  // namespace

}  // namespace vig
