// Wave-specialised chunkwise BiGLA forward (Section 4.2.1, Eq. (BiGLA)) for bf16, dv = 64, dk = 64 or 32:
// the same two passes, workspace layout and arithmetic as the four-wave kernels of
// bigla_chunk.hip (whose header has the algebra of the regrouping over 64-token chunks), with the
// work of a chunk step divided between two sets of waves that run on the same SIMDs.
//
// Why.  A chunk step is a chain: gate scan (matrix cores) -> 64 exponentials per lane and the
// scalings (vector ALU) -> scaled keys through LDS -> score tiles (matrix cores) -> P.V, two state
// readouts and the state update (matrix cores, LDS operands).  With every wave walking that chain
// on its own, and two waves per SIMD, the vector ALU, the LDS and the matrix cores were busy one
// after the other: their busy times added up to the step time.  Here a workgroup has eight waves,
// one producer and one consumer per SIMD:
//   producers (waves 0-3, wave w owns tokens 16w..16w+15 of the chunk): cumulative gates, the
//     exponentials and scalings, the scaled key tiles, the score tiles of the wave's tokens, their
//     mask, and P.V (whose operands the producer holds in registers already);
//   consumers (waves 4-7, wave 4+w owns the same tokens for the output and rows 16w..16w+15 of
//     the carried state): the two state readouts, the output rows, the state update, the state
//     tiles for the next chunk, the stash.
// The consumers work one chunk behind the producers; what a producer made for its 16 tokens (the
// fp32 accumulators of P.V and the scaled queries for the readouts) goes to the consumer of the
// same tokens through lane-private LDS slots (lane i of wave w writes, lane i of wave 4+w reads:
// contiguous 16-byte pieces, no layout change), so the vector work of chunk n+1 and the LDS-fed
// matrix work of chunk n share a SIMD at the same time.  Synchronisation is by workgroup barriers
// only (two per step in the output pass, one in the state pass), executed by every wave the same
// number of times.
//
// The score tile enters P.V as bf16 pairs hi + lo (x = hi + lo to 16 bits), so that of the operand
// roundings of the chunkwise form only those of the scaled queries and keys and of the bf16 state
// tiles remain.
//
// Range.  The eight-wave code evaluates the FAST form only (queries q exp(b), keys k exp(-b), see
// bigla_chunk.hip).  The state pass checks every chunk's total log-decay while it works and leaves
// a flag per (slab, segment) unit.  A unit in which some chunk decays by more than kMildRange is
// evaluated with the operands of the diagonal score tiles split into bf16 pairs hi + lo (three
// products instead of one for those tiles: with fast decay an output is little more than its
// token's nearest products, and their operands then need the bits).  A unit in which some chunk
// is outside the fast form's range altogether (kFastRange) is redone on the spot by the general
// four-wave code of bigla_chunk.hip on four of the workgroup's eight waves (the other four have
// left: a workgroup barrier waits for the surviving waves only), and the output pass runs the
// general code for it in the same way.  Nothing else changes: both codes read and write the same
// workspace layout.
//
// This file is part of the translation unit of bigla_chunk.hip (included by it, after the four-wave
// device code it calls).
#pragma once

// Phase markers for a timing build (a harness defines WS_MARK to record the cycle counter); inert here.
#ifndef WS_MARK
#define WS_MARK(slot)
#endif

namespace vig {

namespace {

constexpr int kWsThreads = 512;           // 4 producer + 4 consumer waves
// Rows of the conv input that the locality epilogue keeps in LDS: the 3x3 neighbourhoods of a chunk's 64 tokens
// span the chunk and kXHalo tokens on either side (a grid row and one token: grids up to kXHalo - 1 columns
// wide); the 64 rows that the next chunk adds are staged once every wave is through with the current chunk's.
constexpr int kXHalo = 65;
constexpr int kXRing = 256;  // >= 64 + 2 * kXHalo, and a power of two: row of token t is t mod kXRing

// c + a.lo * b.lo + a.hi * b.hi on bf16 pairs, fp32 result
__device__ __forceinline__ float dot2(uint32_t a, uint32_t b, float c)
{
    typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, a), __builtin_bit_cast(bf16x2, b), c, false);
}
constexpr int kWsTargetWorkgroups = 256;  // one workgroup per CU (LDS-limited)

struct __align__(16) WsStateLds {
    uint16_t g[2][2][kC][kPitch];   // [buffer][direction] raw log-gates, columns permuted as by stage_gates
    uint16_t ks[2][2][kC][kPitch];  // [buffer][direction] scaled keys k exp(-b)  [token][channel, operand order]
    uint16_t v[2][kC][kPitch];      // [buffer] values [token][column]
    float tot[2][2][kD];            // [buffer][direction] chunk total log-gate per channel, operand order
    int not_fast;                   // some chunk of the unit is outside the fast form's range
    int strong;                     // some chunk of the unit decays by more than kMildRange
};

struct __align__(16) WsOutLds {
    uint16_t g[2][kC][kPitch];   // [direction] raw log-gates of the chunk the producers work on
    uint16_t kf[2][kC][kPitch];  // [buffer] forward-scaled keys (scores now, state update one step later)
    uint16_t kb[kC][kPitch];     // backward-scaled keys
    uint16_t v[2][kC][kPitch];   // [buffer] values (P.V now, state update one step later)
    uint16_t st[kD][kPitch];     // forward state entering the consumers' chunk, bf16  [column][channel]
    uint16_t sb[kD][kPitch];     // backward state entering the consumers' chunk, bf16
    uint16_t ob[kC][kPitch];     // the consumers' output rows on their way from accumulator to row order
    uint4 hand_o[4][256];        // producer -> consumer: fp32 accumulators of P.V (lane-private slots)
    uint4 hand_q[4][256];        // producer -> consumer: readout queries qf0, qf1, qb0, qb1
    float tot[2][kD];            // [buffer] forward chunk total log-gate per channel, operand order
};

union WsLds {
    WsStateLds state;
    WsOutLds out;
    PathLds general;  // the general four-wave code, for a unit outside the fast form's range
};
__shared__ WsLds g_ws_lds;
// locality epilogue: the rows of the conv input around the consumers' chunk, a ring indexed by token, and one row
// of zeros (taps beside the grid).  An object of its own: only the kernels with the epilogue allocate it.
__shared__ __align__(16) uint16_t g_ws_xr[kXRing + 1][kD];

template <>
__device__ __forceinline__ PathLds &path_lds<true>()
{
    return g_ws_lds.general;
}

// Plan of the wave-specialised path: about one workgroup per CU.
inline Plan make_ws_plan(long BH, int L)
{
    Plan p;
    p.n_chunks = (L + kC - 1) / kC;
    long want = kWsTargetWorkgroups / (BH > 0 ? BH : 1);
    if (want < 1) want = 1;
    if (want > p.n_chunks) want = p.n_chunks;
    p.seg_chunks = int((p.n_chunks + want - 1) / want);
    p.n_seg = (p.n_chunks + p.seg_chunks - 1) / p.seg_chunks;
    return p;
}

// One slab's row tensors.  kDk: width of the q, k and gate rows (64, or 32: the rows are then widened to the
// kernels' 64 channels with zeros as they are taken out of the registers they were loaded into, and the code
// skips the zero half: two of the four 16-channel tiles, one of the two K-steps of every contraction over
// channels, state rows 32..63).
template <bool kTm, int kDk = kD>
struct SlabIo {
    __amdgpu_buffer_rsrc_t q, k, gf, gb, v, out;
    unsigned pitch;      // bytes between consecutive tokens of v and out
    unsigned key_pitch;  // of q, k and the gates
    __device__ __forceinline__ SlabIo(const uint16_t *q_all, const uint16_t *k_all, const uint16_t *v_all,
                                      const uint16_t *gf_all, const uint16_t *gb_all, uint16_t *out_all, long slab,
                                      int L, int heads)
    {
        const long row0 = kTm ? (slab / heads) * L * heads + slab % heads : slab * L;
        const long in0 = g_alias_inputs ? 0 : row0;
        pitch = unsigned(kTm ? heads : 1) * kD * 2u;
        key_pitch = unsigned(kTm ? heads : 1) * kDk * 2u;
        const unsigned extent = unsigned(L - 1) * pitch + kD * 2u;
        const unsigned key_extent = unsigned(L - 1) * key_pitch + kDk * 2u;
        q = slab_resource(q_all ? q_all + in0 * kDk : nullptr, q_all ? key_extent : 0u);
        k = slab_resource(k_all + in0 * kDk, key_extent);
        gf = slab_resource(gf_all + in0 * kDk, key_extent);
        gb = slab_resource(gb_all + in0 * kDk, key_extent);
        v = slab_resource(v_all + in0 * kD, extent);
        out = slab_resource(out_all ? out_all + row0 * kD : nullptr, out_all ? extent : 0u);
    }
};

// Where the log forget gates come from when the state pass makes them itself (kGates): the low-rank half
// x W1 of the gate producer (Section 3; Eq. (BiGLA), lines 1-2), bf16 [B][L][16], and the producer's second
// weight matrix w2 [2*H*dk][16] and bias [2*H*dk] (may be null).
struct GateSource {
    const uint16_t *lowrank, *w2, *bias;
    float inv_tau;
    int n_heads;
};

// ---- state pass ------------------------------------------------------------------------------------
// One (slab, segment) unit per workgroup, chunks right to left.  Step s: the producers scale the keys
// of chunk nch-1-s, the consumers fold chunk nch-s into the carried states.  What is written to the
// workspace is what bigla_segment_state_kernel writes.
//
// kGates: g_fwd and g_bwd are OUTPUTS.  One step ahead of the scans that read them, the waves make the gates
// of a chunk, log sigmoid((x W1) w2^T + b) / tau with the arithmetic of gate_producer_bf16_kernel bit for bit
// (the wave of tokens 16w..16w+15 does what that kernel's wave does for 16 tokens, for the 64 channels of its
// head in one direction), put them into the gate tiles in LDS, and write them to memory for the output pass;
// no gates are loaded.
template <bool kTm, bool kGates = false, int kDk = kD>
__global__ __launch_bounds__(kWsThreads) void bigla_ws_state_kernel(
    const uint16_t *__restrict__ k_all, const uint16_t *__restrict__ v_all, const uint16_t *gf_all,
    const uint16_t *gb_all, float *__restrict__ seg_states, int *__restrict__ seg_mild,
    unsigned char *__restrict__ stash, int L, int n_chunks, int seg_chunks, int n_seg, int heads, GateSource gs)
{
    WsStateLds &sm = g_ws_lds.state;
    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63, r = lane & 15, g = lane >> 4;
    const bool producer = wave < 4;
    const int w = wave & 3;
    const int tid4 = tid & 255;  // index among the four waves of the role
    long slab;
    int seg;
    unit_slab_segment(blockIdx.x, n_seg, slab, seg);
    constexpr int kCt = kDk / 16;       // 16-channel tiles that carry data
    const bool owns_rows = 16 * w < kDk;  // consumer wave w carries state rows 16w .. 16w+15
    const SlabIo<kTm, kDk> io(nullptr, k_all, v_all, gf_all, gb_all, nullptr, slab, L, heads);
    const int chunk0 = seg * seg_chunks;
    const int nch = min(seg_chunks, n_chunks - chunk0);
    const int row = 16 * w + r;
    const LaneRows lr = lane_rows<kD>(w, lane, io.pitch), lrk = lane_rows<kDk>(w, lane, io.key_pitch);
    auto token0 = [&](int m) { return unsigned(chunk0 + max(m, 0)) * kC; };  // m may run before the segment: clamped, unused
    auto load_keys = [&](__amdgpu_buffer_rsrc_t rows, int m) {
        StagedRows s = load_rows(rows, lrk, token0(m));
        return s;
    };

    if (tid == 0) sm.not_fast = sm.strong = 0;

    // kGates: lane (r, g) of wave w makes the gates of channels 16g..16g+15 of token 16w + r of a chunk, the
    // consumer waves those of the forward direction, the producer waves those of the backward direction (the
    // two roles share a SIMD's vector ALU; split like this neither role's step grows by the whole job).  A
    // operands (w2 rows of the head, arranged as in gate_producer_bf16_kernel so that the four tiles leave the
    // lane 16 consecutive channels) and the bias stay in registers.
    const int gdir = producer ? 1 : 0;
    s16x4 gate_a[4];
    f32x4 gate_bias[4];  // element e of tile i: channel 16g + 4i + e (the accumulators' initial value)
    const uint16_t *lowrank_rows = nullptr;
    if (kGates) {
        const int head = int(slab % gs.n_heads);
        lowrank_rows = gs.lowrank + size_t(slab / gs.n_heads) * L * 16;
        // (a 32-wide head has channels for the lanes g = 0, 1 only; the others repeat those rows and make zeros)
        const int arow = (16 * (r >> 2)) % kDk + (r & 3);
        const int base = (gdir * gs.n_heads + head) * kDk;
#pragma unroll
        for (int i = 0; i < 4; ++i)
            gate_a[i] = __builtin_bit_cast(s16x4, *reinterpret_cast<const uint2 *>(gs.w2 + size_t(base + arow + 4 * i) * 16 + 4 * g));
        uint4 braw[2];
#pragma unroll
        for (int hh = 0; hh < 2; ++hh)
            braw[hh] = gs.bias ? *reinterpret_cast<const uint4 *>(gs.bias + base + (16 * g) % kDk + 8 * hh) : make_uint4(0u, 0u, 0u, 0u);
        const uint32_t b[8] = {braw[0].x, braw[0].y, braw[0].z, braw[0].w, braw[1].x, braw[1].y, braw[1].z, braw[1].w};
#pragma unroll
        for (int i = 0; i < 4; ++i)
            gate_bias[i] = f32x4{bf16_lo_to_f32(b[2 * i]), bf16_hi_to_f32(b[2 * i]), bf16_lo_to_f32(b[2 * i + 1]),
                                 bf16_hi_to_f32(b[2 * i + 1])};
    }
    // the low-rank row of the lane's token in chunk m of the segment (zeros past the sequence or the segment)
    auto fetch_lowrank = [&](int m) {
        const long t = long(chunk0 + m) * kC + row;
        uint2 h = make_uint2(0u, 0u);
        if (kGates && m >= 0 && t < L) h = *reinterpret_cast<const uint2 *>(lowrank_rows + t * 16 + 4 * g);
        return h;
    };
    // this role's gates of chunk m from its low-rank rows: into gate tile buffer `buf` and out to memory.  Rows
    // past the sequence get log-gate 0 in LDS (they must not decay anything) and their stores are dropped by the
    // bounds check of the slab's buffer resource.
    auto make_gates = [&](const uint2 lowrank_row, int m, int buf) {
        const s16x4 hop = __builtin_bit_cast(s16x4, lowrank_row);
        const bool live = long(chunk0 + m) * kC + row < L && 16 * g < kDk;
        // (lanes without channels of their own store nowhere: an offset beyond the slab's extent, also 16 bytes on)
        const unsigned off = 16 * g < kDk ? (unsigned(chunk0 + m) * kC + unsigned(row)) * io.key_pitch + 32u * unsigned(g) : 0xf0000000u;
        uint32_t packed[8];
#pragma unroll
        for (int i = 0; i < 4; ++i) {  // channels 16g + 4i .. + 3
            const f32x4 z = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(gate_a[i], hop, gate_bias[i], 0, 0, 0);
            const float o0 = log_sigmoid(z[0]) * gs.inv_tau, o1 = log_sigmoid(z[1]) * gs.inv_tau;
            const float o2 = log_sigmoid(z[2]) * gs.inv_tau, o3 = log_sigmoid(z[3]) * gs.inv_tau;
            packed[2 * i] = live ? pack2(o0, o1) : 0u;
            packed[2 * i + 1] = live ? pack2(o2, o3) : 0u;
        }
        // column order of stage_gates: channels 16g + 8p + 4h + e at column 32 (g / 2) + 16 h + 4 (2 (g % 2) + p) + e
        uint16_t(*tile)[kPitch] = sm.g[buf][gdir];
        const int c0 = 32 * (g >> 1) + 8 * (g & 1);
        *reinterpret_cast<uint2 *>(&tile[row][c0]) = make_uint2(packed[0], packed[1]);
        *reinterpret_cast<uint2 *>(&tile[row][c0 + 16]) = make_uint2(packed[2], packed[3]);
        *reinterpret_cast<uint2 *>(&tile[row][c0 + 4]) = make_uint2(packed[4], packed[5]);
        *reinterpret_cast<uint2 *>(&tile[row][c0 + 20]) = make_uint2(packed[6], packed[7]);
        const __amdgpu_buffer_rsrc_t dst = gdir == 0 ? io.gf : io.gb;
        __builtin_amdgcn_raw_buffer_store_b128(u32x4{packed[0], packed[1], packed[2], packed[3]}, dst, off, 0, 0);
        __builtin_amdgcn_raw_buffer_store_b128(u32x4{packed[4], packed[5], packed[6], packed[7]}, dst, off + 16u, 0, 0);
    };
    uint2 rlow = make_uint2(0u, 0u);
    if (kGates) {
        make_gates(fetch_lowrank(nch - 1), nch - 1, 0);
        rlow = fetch_lowrank(nch - 2);
    }

    if (producer) {
        bf16x8 tri_f[2], tri_b[2];
        scan_triangle<0>(w, r, g, tri_f);
        scan_triangle<1>(w, r, g, tri_b);
        StagedRows rk = load_keys(io.k, nch - 1);
        StagedRows rgf, rgb;
        if (!kGates) {
            StagedRows gf = load_keys(io.gf, nch - 1), gb = load_keys(io.gb, nch - 1);
            zero_widened_half<kDk>(gf, lane);
            zero_widened_half<kDk>(gb, lane);
            stage_gates(sm.g[0][0], w, lane, gf);
            stage_gates(sm.g[0][1], w, lane, gb);
            rgf = load_keys(io.gf, nch - 2);
            rgb = load_keys(io.gb, nch - 2);
        }
        __syncthreads();
        for (int s = 0; s <= nch; ++s) {
            WS_MARK(0);
            if (s < nch) {
                const int m = nch - 1 - s, b = s & 1;
                // the wave's own rows of the key tile carry k from row order into operand order
                zero_widened_half<kDk>(rk, lane);
                bounce_store(sm.ks[b][0], w, lane, rk);
                wave_lds_fence();
                float kf[16], kb[16], totf[16], totb[16];
                unpack16(bounce_load(sm.ks[b][0], row, g), kf);
                rk = load_keys(io.k, m - 1);
#pragma unroll
                for (int n = 4 * kCt; n < 16; ++n) kb[n] = totf[n] = totb[n] = 0.f;  // (kf is zero there already)
#pragma unroll
                for (int ct = 0; ct < kCt; ++ct) {
                    const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
                    const bf16x8 f0 = token_operand(sm.g[b][0], 0, 1, 16 * ct, r, g), f1 = token_operand(sm.g[b][0], 2, 3, 16 * ct, r, g);
                    const bf16x8 b0 = token_operand(sm.g[b][1], 0, 1, 16 * ct, r, g), b1 = token_operand(sm.g[b][1], 2, 3, 16 * ct, r, g);
                    const f32x4 Bf = mfma(f1, tri_f[1], mfma(f0, tri_f[0], zero));
                    const f32x4 Bb = mfma(b1, tri_b[1], mfma(b0, tri_b[0], zero));
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int n = 4 * ct + e;
                        totf[n] = Bf[e];
                        totb[n] = Bb[e];
                        kb[n] = kf[n] * fast_exp2(-kLog2e * Bb[e]);  // k * exp(-c_i)
                        kf[n] = kf[n] * fast_exp2(-kLog2e * Bf[e]);  // k * exp(-b_i)
                    }
                }
                store_row16(sm.ks[b][0], row, g, kf);
                store_row16(sm.ks[b][1], row, g, kb);
                // chunk totals: the forward cumulative gate of the chunk's last token, the backward one of its
                // first token; outside the fast form's range the unit is marked
                if (w == 3 && r == 15) {
                    store_chan16(sm.tot[b][0], g, totf);
                    float mn = 0.f;
#pragma unroll
                    for (int n = 0; n < 16; ++n) mn = fminf(mn, totf[n]);
                    if (!(mn >= -kFastRange)) sm.not_fast = 1;
                    if (!(mn >= -kMildRange)) sm.strong = 1;
                }
                if (w == 0 && r == 0) {
                    store_chan16(sm.tot[b][1], g, totb);
                    float mn = 0.f;
#pragma unroll
                    for (int n = 0; n < 16; ++n) mn = fminf(mn, totb[n]);
                    if (!(mn >= -kFastRange)) sm.not_fast = 1;
                    if (!(mn >= -kMildRange)) sm.strong = 1;
                }
                if (!kGates) {  // the gates of chunk m-1 go to the other buffer (last read one step ago)
                    zero_widened_half<kDk>(rgf, lane);
                    zero_widened_half<kDk>(rgb, lane);
                    stage_gates(sm.g[b ^ 1][0], w, lane, rgf);
                    stage_gates(sm.g[b ^ 1][1], w, lane, rgb);
                    rgf = load_keys(io.gf, m - 2);
                    rgb = load_keys(io.gb, m - 2);
                } else if (m >= 1) {  // the backward gates of chunk m-1
                    make_gates(rlow, m - 1, b ^ 1);
                    rlow = fetch_lowrank(m - 2);
                }
            }
            WS_MARK(5);
            __syncthreads();
            WS_MARK(6);
        }
    } else {
        // Sb: backward state, carried right to left.  Sf: forward state at the segment's right edge, each
        // chunk's contribution scaled once by the decay rf of the chunks to its right.
        f32x4 Sf[4], Sb[4];
#pragma unroll
        for (int jt = 0; jt < 4; ++jt) Sf[jt] = Sb[jt] = f32x4{0.f, 0.f, 0.f, 0.f};
        float4 rf = make_float4(1.f, 1.f, 1.f, 1.f), rb = rf;
        unsigned char *stash_slab = stash + size_t(slab) * n_chunks * kStashBytes;
        StagedRows rv = load_rows(io.v, lr, token0(nch - 1));

        __syncthreads();
        for (int s = 0; s <= nch; ++s) {
            WS_MARK(0);
            if (kGates && s + 1 < nch) {  // the forward gates of the chunk the producers take in the next step
                make_gates(rlow, nch - 2 - s, (s + 1) & 1);
                rlow = fetch_lowrank(nch - 3 - s);
            }
            if (s >= 1) {
                const int m = nch - s, b = (s - 1) & 1;
                {  // stash for chunk m: the backward state entering it from the right and the decay to the segment's edge
                    unsigned char *dstm = stash_slab + size_t(chunk0 + m) * kStashBytes;
                    // (a 32-wide head: the state rows 32..63 are zero, and neither stored here nor fetched by the
                    // output pass; a unit redone by the general code gets its whole stash from that code)
                    if (m + 1 < nch && owns_rows) {
                        uint4 *sdst = reinterpret_cast<uint4 *>(dstm) + tid4;
                        const uint2 a = pack4(Sb[0]), bb = pack4(Sb[1]), c = pack4(Sb[2]), d = pack4(Sb[3]);
                        sdst[0] = make_uint4(a.x, a.y, bb.x, bb.y);
                        sdst[256] = make_uint4(c.x, c.y, d.x, d.y);
                    }
                    if (r == 0 && owns_rows)
                        *reinterpret_cast<float4 *>(dstm + size_t(kD) * kD * sizeof(uint16_t) + (16 * w + 4 * g) * sizeof(float)) = rb;
                }
              if (owns_rows) {
                f32x4 Cf[4];
#pragma unroll
                for (int jt = 0; jt < 4; ++jt) Cf[jt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int p = 0; p < 2; ++p) {
                    const bf16x8 af = token_operand(sm.ks[b][0], 2 * p, 2 * p + 1, 16 * w, r, g);
                    const bf16x8 ab = token_operand(sm.ks[b][1], 2 * p, 2 * p + 1, 16 * w, r, g);
#pragma unroll
                    for (int jt = 0; jt < 4; ++jt) {
                        const bf16x8 vb = token_operand(sm.v[b], 2 * p, 2 * p + 1, 16 * jt, r, g);
                        Cf[jt] = mfma(af, vb, Cf[jt]);
                        Sb[jt] = mfma(ab, vb, Sb[jt]);  // S_b = db * (S_b + Kb^T V)
                    }
                }
                const float4 tf = *reinterpret_cast<const float4 *>(&sm.tot[b][0][16 * w + 4 * g]);
                const float4 tb = *reinterpret_cast<const float4 *>(&sm.tot[b][1][16 * w + 4 * g]);
                const float4 df = make_float4(fast_exp2(tf.x * kLog2e), fast_exp2(tf.y * kLog2e), fast_exp2(tf.z * kLog2e), fast_exp2(tf.w * kLog2e));
                const float4 db = make_float4(fast_exp2(tb.x * kLog2e), fast_exp2(tb.y * kLog2e), fast_exp2(tb.z * kLog2e), fast_exp2(tb.w * kLog2e));
                const float4 sf4 = make_float4(rf.x * df.x, rf.y * df.y, rf.z * df.z, rf.w * df.w);
#pragma unroll
                for (int jt = 0; jt < 4; ++jt) {
                    Sb[jt][0] *= db.x; Sb[jt][1] *= db.y; Sb[jt][2] *= db.z; Sb[jt][3] *= db.w;
                    Sf[jt][0] = fmaf(Cf[jt][0], sf4.x, Sf[jt][0]); Sf[jt][1] = fmaf(Cf[jt][1], sf4.y, Sf[jt][1]);
                    Sf[jt][2] = fmaf(Cf[jt][2], sf4.z, Sf[jt][2]); Sf[jt][3] = fmaf(Cf[jt][3], sf4.w, Sf[jt][3]);
                }
                rf = sf4;
                rb.x *= db.x; rb.y *= db.y; rb.z *= db.z; rb.w *= db.w;
              }
            }
            if (s < nch) {  // values of the chunk the consumers take in the next step, into the buffer not in use
                stage_values(sm.v[s & 1], w, lane, rv);
                rv = load_rows(io.v, lr, token0(nch - 2 - s));
            }
            WS_MARK(5);
            __syncthreads();
            WS_MARK(6);
        }
        if (seg_states && sm.not_fast == 0) {  // (a unit outside the fast form's range is redone below)
            float *dst = seg_states + (slab * n_seg + seg) * kSegFloats;
#pragma unroll
            for (int jt = 0; jt < 4; ++jt) {
                reinterpret_cast<f32x4 *>(dst)[256 * jt + tid4] = Sf[jt];
                reinterpret_cast<f32x4 *>(dst + size_t(kD) * kD)[256 * jt + tid4] = Sb[jt];
            }
            if (r == 0) {
                *reinterpret_cast<float4 *>(dst + kSegStateFloats + 16 * w + 4 * g) = rf;
                *reinterpret_cast<float4 *>(dst + kSegStateFloats + kD + 16 * w + 4 * g) = rb;
            }
        }
    }
    // (every write of not_fast precedes the loops' last barrier)
    // the unit's flag for the output pass: 0 general code, 1 fast form, 2 fast form with split diagonal operands
    const bool redo = sm.not_fast != 0;
    if (tid == 0) seg_mild[blockIdx.x] = redo ? 0 : (sm.strong != 0 ? 2 : 1);
    if (redo) {
        // some chunk is outside the fast form's range: the general code redoes the unit on four waves
        // (it overwrites everything the walk above has written for this unit)
        if (wave >= 4) {
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");  // this wave's stash stores are out before it leaves
            return;
        }
        __syncthreads();  // waits for the four waves that stay (and for the others to have left)
        if (kGates) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");  // the gates the other waves wrote are read below
        state_unit<kDk, kTm, true, true>(k_all, v_all, gf_all, gb_all, seg_states, stash, L, n_chunks, seg_chunks, n_seg,
                                         blockIdx.x, heads);
    }
}

// kernel argument of the output pass without the locality epilogue: converts to an all-zero LocalityFusion
struct NoFusion {
    __host__ __device__ operator LocalityFusion() const { return LocalityFusion{nullptr, nullptr, nullptr, nullptr, 0, 0, 0}; }
};

// ---- output pass -----------------------------------------------------------------------------------
// One (slab, segment) unit per workgroup, chunks left to right.  Step m:
//   producers, chunk m: before the mid-step barrier the scalings (gate scan, exponentials, scaled key
//     tiles); after it the score tiles of the wave's tokens, their mask and hi + lo split, and P.V,
//     whose accumulators go to the consumer of the same tokens together with the readout queries;
//   consumers, chunk m-1: before the barrier the two state readouts on top of what the producer
//     left, and the output rows; after it the forward state update with chunk m-1's keys and values
//     and the state tiles for chunk m.
//
// kLoc: the 2D gating locality injection of `lf` (Section 4.2.2) is applied to the output rows before they are
// written: out = G * (bias + sum_taps w * x) + (1 - G) * o as in the stand-alone kernel (fp32, o rounded to
// bf16 first), the taps summed two at a time by v_dot2c_f32_bf16.  The conv input's rows around the chunk sit in an
// LDS ring that the consumers fill one chunk ahead (every row of x is read from memory once per segment, plus
// the halo at the segment's ends); rows outside the sequence read as zeros through the buffer bounds check,
// taps beside the grid are pointed at a row of zeros.  Needs Wg < kXHalo.
//
// split_diag (a compile-time copy of the walk for either value, so that the common one carries nothing of the
// other): fast decay somewhere in the unit, the operands of the diagonal score tiles keep 16 bits (hi + lo).
template <bool kTm, bool kLoc, bool split_diag, int kDk>
__device__ __forceinline__ void ws_out_unit(
    const uint16_t *__restrict__ q_all, const uint16_t *__restrict__ k_all, const uint16_t *__restrict__ v_all,
    const uint16_t *__restrict__ gf_all, const uint16_t *__restrict__ gb_all, uint16_t *__restrict__ out_all,
    const float *__restrict__ seg_states, const unsigned char *__restrict__ stash_all, int L, int n_chunks,
    int seg_chunks, int n_seg, int heads, const LocalityFusion &lf)
{
    WsOutLds &sm = g_ws_lds.out;
    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63, r = lane & 15, g = lane >> 4;
    const bool producer = wave < 4;
    const int w = wave & 3;
    const int tid4 = tid & 255;
    long slab;
    int seg;
    unit_slab_segment(blockIdx.x, n_seg, slab, seg);
    constexpr int kCt = kDk / 16;   // 16-channel tiles that carry data
    constexpr int kKs = kDk / 32;   // K-steps of a contraction over channels
    const bool owns_rows = 16 * w < kDk;  // consumer wave w carries state rows 16w .. 16w+15
    const SlabIo<kTm, kDk> io(q_all, k_all, v_all, gf_all, gb_all, out_all, slab, L, heads);
    const int chunk0 = seg * seg_chunks;
    const int nch = min(seg_chunks, n_chunks - chunk0);
    const int row = 16 * w + r;
    const LaneRows lr = lane_rows<kD>(w, lane, io.pitch), lrk = lane_rows<kDk>(w, lane, io.key_pitch);
    auto token0 = [&](int m) { return unsigned(chunk0 + min(m, nch - 1)) * kC; };  // m may run past the segment: clamped, unused

    // ---- locality epilogue (kLoc): what both roles need.  A lane writes 8 channels of two of its wave's 16 output
    // rows; the consumer waves blend the first of the two in their first half-step, the producer waves the second
    // in their second half-step (after the mid-step barrier the rounded rows are in the bounce tile), so that
    // neither role's half grows by the whole job.
    const int c0 = 8 * (lane & 7);  // the lane's channels of the rows it writes
    uint32_t wp[8][5];
    float cbias[8];
    __amdgpu_buffer_rsrc_t rz = io.v;
    const float inv_wg = 1.f / float(lf.Wg > 0 ? lf.Wg : 1);
    auto ring_slot = [&](int tok) { return tok & (kXRing - 1); };
    if (kLoc) {
        const int head = int(slab % lf.H);
        // taps [channel][9] bf16: the lane's 8 channels are 72 consecutive values.  Kept as bf16 pairs of
        // taps (0,1) (2,3) (4,5) (6,7) (8,-): a pair meets the same two taps of the input in one
        // v_dot2c_f32_bf16 (exact products, fp32 sum).
        const uint16_t *tp = static_cast<const uint16_t *>(lf.w) + size_t(head * kD + c0) * 9;
        uint4 raw[9];
#pragma unroll
        for (int i = 0; i < 9; ++i) raw[i] = reinterpret_cast<const uint4 *>(tp)[i];
        const uint32_t *rw = reinterpret_cast<const uint32_t *>(raw);
        auto tap = [&](int e, int k) { const int i = 9 * e + k; return (rw[i >> 1] >> (16 * (i & 1))) & 0xffffu; };
#pragma unroll
        for (int e = 0; e < 8; ++e) {
#pragma unroll
            for (int pr = 0; pr < 4; ++pr) wp[e][pr] = tap(e, 2 * pr) | (tap(e, 2 * pr + 1) << 16);
            wp[e][4] = tap(e, 8);
        }
        if (lf.bias) {
            unpack8(*reinterpret_cast<const uint4 *>(static_cast<const uint16_t *>(lf.bias) + head * kD + c0), cbias);
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) cbias[e] = 0.f;
        }
        const long row0 = kTm ? (slab / heads) * long(L) * heads + slab % heads : slab * long(L);
        rz = slab_resource(static_cast<const uint16_t *>(lf.gate_logits) + row0 * kD, unsigned(L - 1) * io.pitch + kD * 2u);
    }
    // the lane's gate logits of row t (of its two) of chunk c of the segment
    auto load_z = [&](int c, int t) {
        const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rz, lr.off[t] + unsigned(chunk0 + min(c, nch - 1)) * kC * lr.pitch, 0, 0);
        return make_uint4(v.x, v.y, v.z, v.w);
    };
    // out = G * (bias + conv) + (1 - G) * o for row t of chunk c, from the rounded row in the bounce tile; stored
    auto blend_row = [&](int c, int t, const uint4 zrow) {
        const int rr = 16 * w + 8 * t + (lane >> 3);
        uint4 o = *reinterpret_cast<const uint4 *>(&sm.ob[rr][c0]);
        if (kLoc) {
            const int tok = (chunk0 + c) * kC + rr;
            // grid column of the token (tok < 2^22, checked at launch: the float quotient is off by one at most)
            int xp = tok - int(float(tok) * inv_wg) * lf.Wg;
            xp += xp < 0 ? lf.Wg : 0;
            xp -= xp >= lf.Wg ? lf.Wg : 0;
            const bool left = xp > 0, right = xp + 1 < lf.Wg;
            float acc[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[e] = cbias[e];
            // the nine neighbours' rows (8 channels each); rows above and below the grid are rows outside
            // the sequence: zeros in the ring
            uint4 xn[9];
#pragma unroll
            for (int ky = -1; ky <= 1; ++ky)
#pragma unroll
                for (int kx = -1; kx <= 1; ++kx) {
                    const bool in = kx < 0 ? left : (kx > 0 ? right : true);
                    const int slot = in ? ring_slot(tok + ky * lf.Wg + kx) : kXRing;
                    xn[3 * (ky + 1) + kx + 1] = *reinterpret_cast<const uint4 *>(&g_ws_xr[slot][c0]);
                }
#pragma unroll
            for (int j = 0; j < 4; ++j) {  // channels 2j, 2j+1 of the lane's eight
                auto dword = [&](int k) { const uint4 &v = xn[k]; return j == 0 ? v.x : (j == 1 ? v.y : (j == 2 ? v.z : v.w)); };
#pragma unroll
                for (int pr = 0; pr < 4; ++pr) {
                    const uint32_t a = dword(2 * pr), b2 = dword(2 * pr + 1);
                    acc[2 * j] = dot2(__builtin_amdgcn_perm(b2, a, 0x05040100u), wp[2 * j][pr], acc[2 * j]);
                    acc[2 * j + 1] = dot2(__builtin_amdgcn_perm(b2, a, 0x07060302u), wp[2 * j + 1][pr], acc[2 * j + 1]);
                }
                acc[2 * j] = dot2(dword(8) & 0xffffu, wp[2 * j][4], acc[2 * j]);
                acc[2 * j + 1] = dot2(dword(8) >> 16, wp[2 * j + 1][4], acc[2 * j + 1]);
            }
            float zf[8], of[8];
            unpack8(zrow, zf);
            unpack8(o, of);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float gate = __builtin_amdgcn_rcpf(1.f + __expf(-zf[e]));
                acc[e] = fmaf(gate, acc[e] - of[e], of[e]);
            }
            o = make_uint4(pack2(acc[0], acc[1]), pack2(acc[2], acc[3]), pack2(acc[4], acc[5]), pack2(acc[6], acc[7]));
        }
        __builtin_amdgcn_raw_buffer_store_b128(u32x4{o.x, o.y, o.z, o.w}, io.out, lr.off[t] + unsigned(chunk0 + c) * kC * lr.pitch, 0, 0);
    };

    // a contraction over the channels that carry data: one K-step for a 32-wide head, two otherwise
    auto dotk = [](bf16x8 a0, bf16x8 a1, bf16x8 b0, bf16x8 b1, f32x4 acc) {
        acc = mfma(a0, b0, acc);
        if (kKs > 1) acc = mfma(a1, b1, acc);
        return acc;
    };

    if (producer) {
        bf16x8 tri_f[2], tri_b[2];
        scan_triangle<0>(w, r, g, tri_f);
        scan_triangle<1>(w, r, g, tri_b);
        StagedRows rq = load_rows(io.q, lrk, token0(0)), rk = load_rows(io.k, lrk, token0(0)), rv = load_rows(io.v, lr, token0(0));
        {
            StagedRows gf = load_rows(io.gf, lrk, token0(0)), gb = load_rows(io.gb, lrk, token0(0));
            zero_widened_half<kDk>(gf, lane);
            zero_widened_half<kDk>(gb, lane);
            stage_gates(sm.g[0], w, lane, gf);
            stage_gates(sm.g[1], w, lane, gb);
        }
        StagedRows rgf = load_rows(io.gf, lrk, token0(1)), rgb = load_rows(io.gb, lrk, token0(1));
        uint4 rz1 = make_uint4(0u, 0u, 0u, 0u);
        __syncthreads();
        for (int m = 0; m <= nch; ++m) {
            bf16x8 qf0 = {}, qf1 = {}, qb0 = {}, qb1 = {}, kf0 = {}, kf1 = {}, kb0 = {}, kb1 = {};
            bf16x8 lo[8] = {};  // split_diag: the low halves of the eight operands above, in that order
            const int b = m & 1;
            WS_MARK(0);
            if (m < nch) {
                // the wave's own rows of the key tiles carry q and k from row order into operand order
                zero_widened_half<kDk>(rq, lane);
                zero_widened_half<kDk>(rk, lane);
                bounce_store(sm.kf[b], w, lane, rq);
                bounce_store(sm.kb, w, lane, rk);
                stage_values(sm.v[b], w, lane, rv);
                wave_lds_fence();
                float qf[16], kf[16], qb[16], kb[16], tot[16];
                unpack16(bounce_load(sm.kf[b], row, g), qf);
                unpack16(bounce_load(sm.kb, row, g), kf);
                rq = load_rows(io.q, lrk, token0(m + 1));
                rk = load_rows(io.k, lrk, token0(m + 1));
                rv = load_rows(io.v, lr, token0(m + 1));
#pragma unroll
                for (int n = 4 * kCt; n < 16; ++n) qb[n] = kb[n] = tot[n] = 0.f;  // (qf and kf are zero there already)
#pragma unroll
                for (int ct = 0; ct < kCt; ++ct) {
                    const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
                    const bf16x8 f0 = token_operand(sm.g[0], 0, 1, 16 * ct, r, g), f1 = token_operand(sm.g[0], 2, 3, 16 * ct, r, g);
                    const bf16x8 b0 = token_operand(sm.g[1], 0, 1, 16 * ct, r, g), b1 = token_operand(sm.g[1], 2, 3, 16 * ct, r, g);
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
                if (split_diag) {
                    pack8_split(qf, qf0, lo[0]); pack8_split(qb, qb0, lo[2]);
                    pack8_split(kf, kf0, lo[4]); pack8_split(kb, kb0, lo[6]);
                    if (kKs > 1) {
                        pack8_split(qf + 8, qf1, lo[1]); pack8_split(qb + 8, qb1, lo[3]);
                        pack8_split(kf + 8, kf1, lo[5]); pack8_split(kb + 8, kb1, lo[7]);
                    }
                } else {
                    qf0 = pack8(qf); qb0 = pack8(qb); kf0 = pack8(kf); kb0 = pack8(kb);
                    if (kKs > 1) {
                        qf1 = pack8(qf + 8); qb1 = pack8(qb + 8); kf1 = pack8(kf + 8); kb1 = pack8(kb + 8);
                    }
                }
                *reinterpret_cast<bf16x8 *>(&sm.kf[b][row][8 * g]) = kf0;
                *reinterpret_cast<bf16x8 *>(&sm.kb[row][8 * g]) = kb0;
                if (kKs > 1) {  // (the upper K-step of the key tiles is never read otherwise)
                    *reinterpret_cast<bf16x8 *>(&sm.kf[b][row][32 + 8 * g]) = kf1;
                    *reinterpret_cast<bf16x8 *>(&sm.kb[row][32 + 8 * g]) = kb1;
                }
                if (w == 3 && r == 15) store_chan16(sm.tot[b], g, tot);  // for the state decay
            }
            WS_MARK(1);
            __syncthreads();  // mid-step: scaled keys and values visible
            WS_MARK(2);
            // locality epilogue: the second row of the lane's two of chunk m-1, which the consumers have left rounded
            // in the bounce tile before the barrier (they overwrite it after the end-of-step barrier)
            if (kLoc) {
                if (m >= 1) blend_row(m - 1, 1, rz1);
                rz1 = load_z(m, 1);  // gate logits of the row blended a step from now
            }
            if (m < nch) {
                // merged masked score tile, transposed (P^T[i][t]): key sub-block I < w forward, I > w backward,
                // I = w both (key <= query of the forward piece, key >= query of the backward one; own token in
                // both); lane: keys 4g..4g+3, query r.  It enters P.V as bf16 pairs hi + lo.
                uint2 ph[4], pl[4];
                const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int I = 0; I < 4; ++I) {
                    f32x4 p;
                    if (I == w) {
                        f32x4 pb = zero;
                        p = zero;
                        if (split_diag) {  // hi.lo + lo.hi first (the small terms), then hi.hi
                            p = dotk(lo[4], lo[5], qf0, qf1, dotk(kf0, kf1, lo[0], lo[1], p));
                            pb = dotk(lo[6], lo[7], qb0, qb1, dotk(kb0, kb1, lo[2], lo[3], pb));
                        }
                        p = dotk(kf0, kf1, qf0, qf1, p);
                        pb = dotk(kb0, kb1, qb0, qb1, pb);
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const int i = 4 * g + e;
                            p[e] = (i <= r ? p[e] : 0.f) + (i >= r ? pb[e] : 0.f);
                        }
                    } else if (I < w) {
                        p = mfma(*reinterpret_cast<const bf16x8 *>(&sm.kf[b][16 * I + r][8 * g]), qf0, zero);
                        if (kKs > 1) p = mfma(*reinterpret_cast<const bf16x8 *>(&sm.kf[b][16 * I + r][32 + 8 * g]), qf1, p);
                    } else {
                        p = mfma(*reinterpret_cast<const bf16x8 *>(&sm.kb[16 * I + r][8 * g]), qb0, zero);
                        if (kKs > 1) p = mfma(*reinterpret_cast<const bf16x8 *>(&sm.kb[16 * I + r][32 + 8 * g]), qb1, p);
                    }
                    split4(p, ph[I], pl[I]);
                }
                // O^T = V^T P^T, token-per-lane accumulators: lane (r, g) gets columns 16*jt + 4g .. +3 of its own token
                f32x4 O[4];
                {
                    const bf16x8 h0 = operand(ph[0], ph[1]), h1 = operand(ph[2], ph[3]);
                    const bf16x8 l0 = operand(pl[0], pl[1]), l1 = operand(pl[2], pl[3]);
#pragma unroll
                    for (int jt = 0; jt < 4; ++jt) {
                        const bf16x8 v0 = token_operand(sm.v[b], 0, 1, 16 * jt, r, g), v1 = token_operand(sm.v[b], 2, 3, 16 * jt, r, g);
                        O[jt] = mfma(v1, h1, mfma(v0, h0, mfma(v1, l1, mfma(v0, l0, zero))));
                    }
                }
#pragma unroll
                for (int jt = 0; jt < 4; ++jt) sm.hand_o[jt][tid4] = __builtin_bit_cast(uint4, O[jt]);
                sm.hand_q[0][tid4] = __builtin_bit_cast(uint4, qf0);
                sm.hand_q[2][tid4] = __builtin_bit_cast(uint4, qb0);
                if (kKs > 1) {
                    sm.hand_q[1][tid4] = __builtin_bit_cast(uint4, qf1);
                    sm.hand_q[3][tid4] = __builtin_bit_cast(uint4, qb1);
                }
                // the gates of chunk m+1 (the tiles were last read before the mid-step barrier)
                zero_widened_half<kDk>(rgf, lane);
                zero_widened_half<kDk>(rgb, lane);
                stage_gates(sm.g[0], w, lane, rgf);
                stage_gates(sm.g[1], w, lane, rgb);
                rgf = load_rows(io.gf, lrk, token0(m + 2));
                rgb = load_rows(io.gb, lrk, token0(m + 2));
            }
            WS_MARK(3);
            __syncthreads();  // end of step
            WS_MARK(4);
        }
    } else {
        const unsigned char *stash = stash_all + size_t(slab) * n_chunks * kStashBytes;
        const bool seg_in = seg_states != nullptr && seg + 1 < n_seg;  // the last segment's entering backward state is zero
        struct StashRows {
            uint4 p[2];
            float4 dr;  // decay of the lane's state rows from the chunk's right edge to the segment's
        };
        auto fetch_stash = [&](int m) {
            StashRows c = {};
            if (!owns_rows) return c;  // (a 32-wide head: state rows 32..63 are zero and not stored)
            const unsigned char *base = stash + size_t(chunk0 + min(m, nch - 1)) * kStashBytes;
            const uint4 *p = reinterpret_cast<const uint4 *>(base) + tid4;
            c.p[0] = p[0];
            c.p[1] = p[256];
            c.dr = *reinterpret_cast<const float4 *>(base + size_t(kD) * kD * sizeof(uint16_t) + (16 * w + 4 * g) * sizeof(float));
            return c;
        };
        StashRows rs = fetch_stash(0);

        // States entering the segment, folded from the segments' local end states and decays that the state
        // pass left: forward from the left, E <- D_n * E + S_n over the segments n < seg; backward from the
        // right over n > seg (kept in registers; each chunk adds its decayed copy to the stashed state).
        f32x4 S[4], Sseg[4];
#pragma unroll
        for (int jt = 0; jt < 4; ++jt) S[jt] = Sseg[jt] = f32x4{0.f, 0.f, 0.f, 0.f};
        auto fold = [&](f32x4 (&E)[4], int dir, int first, int count, int step) {
            const float *slab_states = seg_states + slab * n_seg * kSegFloats;
            constexpr int kBatch = 4;
            for (int i0 = 0; i0 < count; i0 += kBatch) {
                f32x4 local[kBatch][4];
                float4 decay[kBatch];
#pragma unroll
                for (int u = 0; u < kBatch; ++u) {
                    const float *sp = slab_states + size_t(first + step * min(i0 + u, count - 1)) * kSegFloats;
#pragma unroll
                    for (int jt = 0; jt < 4; ++jt)
                        local[u][jt] = reinterpret_cast<const f32x4 *>(sp + dir * kD * kD)[256 * jt + tid4];
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
        // state tiles for chunk m: the forward state, and the backward state entering the chunk = its stashed
        // state (zero for the segment's last chunk) + the segment's entering state decayed to the chunk's edge
        auto publish = [&](const StashRows &c, int m) {
            const bool has_stash = m + 1 < nch;
            uint2 t[4] = {make_uint2(c.p[0].x, c.p[0].y), make_uint2(c.p[0].z, c.p[0].w),
                          make_uint2(c.p[1].x, c.p[1].y), make_uint2(c.p[1].z, c.p[1].w)};
#pragma unroll
            for (int jt = 0; jt < 4; ++jt) {
                *reinterpret_cast<uint2 *>(&sm.st[16 * jt + r][16 * w + 4 * g]) = pack4(S[jt]);
                if (seg_in) {
                    f32x4 x = has_stash ? unpack4(t[jt]) : f32x4{0.f, 0.f, 0.f, 0.f};
                    x[0] = fmaf(c.dr.x, Sseg[jt][0], x[0]);
                    x[1] = fmaf(c.dr.y, Sseg[jt][1], x[1]);
                    x[2] = fmaf(c.dr.z, Sseg[jt][2], x[2]);
                    x[3] = fmaf(c.dr.w, Sseg[jt][3], x[3]);
                    t[jt] = pack4(x);
                } else if (!has_stash) {
                    t[jt] = make_uint2(0u, 0u);
                }
                *reinterpret_cast<uint2 *>(&sm.sb[16 * jt + r][16 * w + 4 * g]) = t[jt];
            }
        };

        // ---- locality epilogue, consumer side: the ring of conv-input rows and prefetch registers
        auto group_token0 = [&](int j) { return (chunk0 + j - 1) * kC + kXHalo; };
        // group j: the 64 tokens that become needed with chunk j of the segment (their first: kXHalo past its start)
        auto stage_group = [&](const StagedRows &s, int j) {
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const int slot = ring_slot(group_token0(j) + 16 * w + 8 * t + (lane >> 3));
                *reinterpret_cast<uint4 *>(&g_ws_xr[slot][c0]) = s.p[t];
            }
        };
        __amdgpu_buffer_rsrc_t rx = io.v;
        StagedRows rxg;
        uint4 rz0 = make_uint4(0u, 0u, 0u, 0u);
        if (kLoc) {
            const long row0 = kTm ? (slab / heads) * long(L) * heads + slab % heads : slab * long(L);
            const unsigned extent = unsigned(L - 1) * io.pitch + kD * 2u;
            rx = slab_resource(static_cast<const uint16_t *>(lf.x) + row0 * kD, extent);
            if (tid4 < 8) *reinterpret_cast<uint4 *>(&g_ws_xr[kXRing][8 * tid4]) = make_uint4(0u, 0u, 0u, 0u);
            // what the first chunk needs: groups -2 .. 1 (tokens -127 .. 128 around the segment's start)
            StagedRows first[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) first[j] = load_rows(rx, lr, unsigned(group_token0(j - 2)));
#pragma unroll
            for (int j = 0; j < 4; ++j) stage_group(first[j], j - 2);
            rxg = load_rows(rx, lr, unsigned(group_token0(2)));
            rz0 = load_z(0, 0);
        }

        if (seg_states != nullptr && owns_rows) {
            fold(S, 0, 0, seg, 1);
            fold(Sseg, 1, n_seg - 1, n_seg - 1 - seg, -1);
        }
        __syncthreads();  // (the producers' prologue barrier)
        for (int m = 0; m <= nch; ++m) {
            const int c = m - 1, b = c & 1;
            WS_MARK(0);
            if (m >= 1) {
                // what the producer of the same tokens left: P.V of the chunk and the readout queries
                f32x4 O[4];
#pragma unroll
                for (int jt = 0; jt < 4; ++jt) O[jt] = __builtin_bit_cast(f32x4, sm.hand_o[jt][tid4]);
                const bf16x8 qf0 = __builtin_bit_cast(bf16x8, sm.hand_q[0][tid4]), qb0 = __builtin_bit_cast(bf16x8, sm.hand_q[2][tid4]);
                bf16x8 qf1 = {}, qb1 = {};
                if (kKs > 1) {
                    qf1 = __builtin_bit_cast(bf16x8, sm.hand_q[1][tid4]);
                    qb1 = __builtin_bit_cast(bf16x8, sm.hand_q[3][tid4]);
                }
                readout<kKs>(sm.st, qf0, qf1, r, g, O);
                if (c + 1 < nch || seg_in) readout<kKs>(sm.sb, qb0, qb1, r, g, O);
                // o_t = (o_fwd_t + o_bwd_t) / 2 (the queries arrive halved), turned into whole rows through the wave's
                // own rows of the bounce tile, then written 8 rows per store
#pragma unroll
                for (int jt = 0; jt < 4; ++jt)
                    *reinterpret_cast<uint2 *>(&sm.ob[16 * w + r][16 * jt + 4 * g]) = pack4(O[jt]);
                wave_lds_fence();
                if (kLoc) {
                    // (the producer of the same tokens writes the second of the lane's two rows)
                    blend_row(c, 0, rz0);
                    rz0 = load_z(m, 0);  // the next chunk's gate logits
                } else {
#pragma unroll
                    for (int t = 0; t < 2; ++t) {
                        const int rr = 16 * w + 8 * t + (lane >> 3);
                        const uint4 o = *reinterpret_cast<const uint4 *>(&sm.ob[rr][8 * (lane & 7)]);
                        __builtin_amdgcn_raw_buffer_store_b128(u32x4{o.x, o.y, o.z, o.w}, io.out,
                                                               lr.off[t] + unsigned(chunk0 + c) * kC * lr.pitch, 0, 0);
                    }
                }
            }
            WS_MARK(1);
            __syncthreads();  // mid-step
            WS_MARK(2);
            if (m >= 1) {
                if (kLoc) {
                    // the rows that the next chunk's neighbourhoods add: every wave is through with this chunk's, and
                    // the ring slots they take hold rows that no later chunk needs
                    stage_group(rxg, m + 1);
                    rxg = load_rows(rx, lr, unsigned(group_token0(m + 2)));
                }
              if (owns_rows) {
                // forward state update: S = d (S + K^T V), d = exp(chunk total)
                const float4 t = *reinterpret_cast<const float4 *>(&sm.tot[b][16 * w + 4 * g]);
                const float4 d = make_float4(fast_exp2(t.x * kLog2e), fast_exp2(t.y * kLog2e), fast_exp2(t.z * kLog2e), fast_exp2(t.w * kLog2e));
#pragma unroll
                for (int p = 0; p < 2; ++p) {
                    const bf16x8 a = token_operand(sm.kf[b], 2 * p, 2 * p + 1, 16 * w, r, g);
#pragma unroll
                    for (int jt = 0; jt < 4; ++jt) S[jt] = mfma(a, token_operand(sm.v[b], 2 * p, 2 * p + 1, 16 * jt, r, g), S[jt]);
                }
#pragma unroll
                for (int jt = 0; jt < 4; ++jt) {
                    S[jt][0] *= d.x; S[jt][1] *= d.y; S[jt][2] *= d.z; S[jt][3] *= d.w;
                }
              }
            }
            if (m < nch && owns_rows) {
                // tiles for chunk m, which the consumers take in the next step
                publish(rs, m);
                rs = fetch_stash(m + 1);
            }
            WS_MARK(3);
            __syncthreads();  // end of step
            WS_MARK(4);
        }
    }
}

template <bool kTm, bool kLoc = false, int kDk = kD>
__global__ __launch_bounds__(kWsThreads) void bigla_ws_out_kernel(
    const uint16_t *__restrict__ q_all, const uint16_t *__restrict__ k_all, const uint16_t *__restrict__ v_all,
    const uint16_t *__restrict__ gf_all, const uint16_t *__restrict__ gb_all, uint16_t *__restrict__ out_all,
    const float *__restrict__ seg_states /* nullptr when one segment per slab */, const int *__restrict__ seg_mild,
    const unsigned char *__restrict__ stash_all, int L, int n_chunks, int seg_chunks, int n_seg, int heads,
    const typename std::conditional<kLoc, LocalityFusion, NoFusion>::type lf_arg)
{
    const LocalityFusion lf = lf_arg;
    const int unit_flag = seg_mild[blockIdx.x];  // what the state pass found: uniform over the workgroup
    if (unit_flag == 0) {
        // a unit outside the fast form's range: the general four-wave code, on four waves
        if (threadIdx.x >= 256) return;
        out_unit_general<kDk, kTm, kLoc, true>(q_all, k_all, v_all, gf_all, gb_all, out_all, seg_states, stash_all, L,
                                               n_chunks, seg_chunks, n_seg, blockIdx.x, heads, lf);
    } else if (unit_flag == 2) {
        ws_out_unit<kTm, kLoc, true, kDk>(q_all, k_all, v_all, gf_all, gb_all, out_all, seg_states, stash_all, L,
                                          n_chunks, seg_chunks, n_seg, heads, lf);
    } else {
        ws_out_unit<kTm, kLoc, false, kDk>(q_all, k_all, v_all, gf_all, gb_all, out_all, seg_states, stash_all, L,
                                           n_chunks, seg_chunks, n_seg, heads, lf);
    }
}

// ---- host side ---------------------------------------------------------------------------------------

bool bigla_chunk_ws_applicable(long BH, int L, int dk)
{
    const Plan p = make_ws_plan(BH, L);
    // short sequences with at least half a chip of slabs stay with the single-launch slab kernel
    if (BH >= 128 && p.n_chunks <= 4) return false;
    return (dk == kD || dk == kD / 2) && p.n_chunks > 1;
}

// [segment states][unit flags][stash], as in the four-wave path, for this path's own plan
size_t bigla_chunk_ws_workspace_bytes(long BH, int L)
{
    const Plan p = make_ws_plan(BH, L);
    return size_t(BH) * p.n_seg * kSegFloats * sizeof(float) + (size_t(BH) * p.n_seg * sizeof(int) + 15) / 16 * 16 +
           size_t(BH) * p.n_chunks * kStashBytes;
}

// gates: null when g_fwd and g_bwd are inputs; otherwise the state pass makes them (and writes them there)
hipError_t bigla_chunk_ws_launch(const void *q, const void *k, const void *v, const void *g_fwd, const void *g_bwd,
                                 void *out, long BH, int L, int dk, int heads_token_major, void *workspace,
                                 hipStream_t stream, const GateSource *gates = nullptr,
                                 const LocalityFusion *fusion = nullptr)
{
    const Plan p = make_ws_plan(BH, L);
    const long blocks = BH * p.n_seg;
    if (blocks > 0x7fffffffL) return hipErrorInvalidValue;
    const uint16_t *qq = static_cast<const uint16_t *>(q), *kk = static_cast<const uint16_t *>(k);
    const uint16_t *vv = static_cast<const uint16_t *>(v);
    const uint16_t *gf = static_cast<const uint16_t *>(g_fwd), *gb = static_cast<const uint16_t *>(g_bwd);
    uint16_t *oo = static_cast<uint16_t *>(out);
    float *seg_states = static_cast<float *>(workspace);
    const size_t seg_bytes = size_t(BH) * p.n_seg * kSegFloats * sizeof(float);
    int *seg_mild = reinterpret_cast<int *>(static_cast<unsigned char *>(workspace) + seg_bytes);
    unsigned char *stash = reinterpret_cast<unsigned char *>(seg_mild) + (size_t(blocks) * sizeof(int) + 15) / 16 * 16;
    const bool tm = heads_token_major > 0;
    const int heads = tm ? heads_token_major : 1;
    float *seg_out = p.n_seg > 1 ? seg_states : nullptr;
    const dim3 grid((unsigned)blocks), block(kWsThreads);
    using std::integral_constant;
    typedef integral_constant<bool, true> yes;
    typedef integral_constant<bool, false> no;
    typedef integral_constant<int, kD> wide;
    typedef integral_constant<int, kD / 2> half;
    {
        LaunchTimer timer(kKernelSegmentState, stream);
        const GateSource none = {};
        auto go = [&](auto tm_c, auto gates_c, auto dk_c) {
            hipLaunchKernelGGL((bigla_ws_state_kernel<decltype(tm_c)::value, decltype(gates_c)::value, decltype(dk_c)::value>),
                               grid, block, 0, stream, kk, vv, gf, gb, seg_out, seg_mild, stash, L, p.n_chunks,
                               p.seg_chunks, p.n_seg, heads, gates ? *gates : none);
        };
        if (gates && dk == kD) {
            if (tm) go(yes{}, yes{}, wide{}); else go(no{}, yes{}, wide{});
        } else if (gates) {
            if (tm) go(yes{}, yes{}, half{}); else go(no{}, yes{}, half{});
        } else if (dk == kD) {
            if (tm) go(yes{}, no{}, wide{}); else go(no{}, no{}, wide{});
        } else {
            if (tm) go(yes{}, no{}, half{}); else go(no{}, no{}, half{});
        }
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    {
        LaunchTimer timer(kKernelSegmentOut, stream);
        auto go = [&](auto tm_c, auto loc_c, auto dk_c) {
            typename std::conditional<decltype(loc_c)::value, LocalityFusion, NoFusion>::type arg = {};
            if constexpr (decltype(loc_c)::value) arg = *fusion;
            hipLaunchKernelGGL((bigla_ws_out_kernel<decltype(tm_c)::value, decltype(loc_c)::value, decltype(dk_c)::value>),
                               grid, block, 0, stream, qq, kk, vv, gf, gb, oo, seg_out, seg_mild, stash, L, p.n_chunks,
                               p.seg_chunks, p.n_seg, heads, arg);
        };
        if (dk == kD) {
            if (fusion) { if (tm) go(yes{}, yes{}, wide{}); else go(no{}, yes{}, wide{}); }
            else { if (tm) go(yes{}, no{}, wide{}); else go(no{}, no{}, wide{}); }
        } else {
            if (fusion) { if (tm) go(yes{}, yes{}, half{}); else go(no{}, yes{}, half{}); }
            else { if (tm) go(yes{}, no{}, half{}); else go(no{}, no{}, half{}); }
        }
    }
    return hipGetLastError();
}

}  // namespace

}  // namespace vig
