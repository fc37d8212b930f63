// Chunkwise bf16 MFMA evaluation of the gradient of the BiGLA token mixer (Section 4.2.1,
// Eq. (BiGLA); the paper trains through it, Section 5, and prints no gradient formulas) for
// dv = 64 and dk = 64 (or 32, widened to 64 with zero channels) in bf16: the counterpart of the
// chunkwise forward kernels.
//
// One direction, forward (the backward one is its mirror image: suffix sums, keys to the right).
// Inside a chunk of 64 tokens let b_t be the inclusive cumulative log-gate since the chunk's left
// edge, E+ = exp(b), E- = exp(-b), q~ = q * E+, k~ = k * E-, do' = d_out / 2.  With
//   S_in : the state entering the chunk (after the previous chunk's last token), [dk][dv]
//   A'   : diag(exp(b_end)) times the adjoint of the chunk's end state due to all later chunks
// the regrouped chain rule is, with the masks s <= t,
//   P  = mask(q~ k~^T)             dP = mask(do' v^T)                          [t][s]
//   X  = dP k~ + do' S_in^T        dq = E+ * X
//   Yi = dP^T q~   Ye = v A'^T     dk = E- * (Yi + Ye)
//   dv = P^T do' + k~ A'
//   dg_u = sum_{t >= u} (q~ * X - k~ * Yi)_t + sum_{t < u} (k~ * Ye)_t + rowsum(S_in * A')
// (the three parts of dg are the token pairs (s, t), s < u <= t, that straddle u: both inside the
// chunk or s before it; s inside and t after it; s before and t after).  Every sum of dg runs over
// at most one chunk, so no long-range cancellation enters it; its two prefix/suffix sums are fp32
// scans over the wave's tokens (DPP row operations) plus the other waves' totals.
// States come from two small launches before the main one:
//   1. bigla_bwd_chunk_local_kernel (workgroup per chunk): the chunk's own contributions
//      U = (k * exp(b_end - b))^T v and W = q~^T do' for both directions, and the chunk totals of
//      the log-gates;
//   2. bigla_bwd_chunk_scan_kernel (elementwise over the 64x64 matrices, sequential over the
//      chunks of a slab): S_in(c+1) = d_c S_in(c) + U_c and A'_c = d_c (W_{c+1} + A'_{c+1}), in
//      place, fp32 running values, bf16 storage; it also marks the slabs in which some chunk's
//      total log-decay exceeds 60 nats in some channel;
//   3. bigla_bwd_chunk_main_kernel (workgroup per chunk): everything above for both directions,
//      dq, dk, dv accumulated in registers and written once.
// exp(-b) grows with the decay accumulated over a chunk, so marked slabs are left to the exact
// token-by-token kernels (which skip every other slab); gates of the paper's form,
// sigmoid(z)^(1/16), reach 60 nats in 64 steps only for z < -15 throughout.
//
// Wavefront mapping (256 threads = 4 waves): wave w owns tokens 16w..16w+15 of the chunk; results
// are produced transposed, so that lane (r = lane%16, g = lane/16) holds, for token 16w + r,
// channels 16ct + 4g + e (ct, e = 0..3) -- four 8-byte pieces of the token's row.  All tiles are
// row-major bf16 in LDS; an operand whose contraction index runs along the tile's rows is read
// with ds_read_b64_tr_b16.  Tokens past the sequence are read as zeros (q = k = v = do = 0,
// log-gate 0: a no-op) and their stores are dropped, both by the bounds check of the buffer
// resource that spans the slab.
#include <type_traits>

#include "vig_common.hpp"
#include "vig_kernels.hpp"
#include "vig_timing.hpp"

namespace vig {

namespace {

constexpr int kC = 64;       // chunk length (tokens)
constexpr int kD = 64;       // dk = dv
constexpr int kPitch = 72;   // LDS row pitch in bf16 elements
constexpr int kThreads = 256;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kFastRange = 60.0f;  // largest chunk log-decay (nats, any channel) this path accepts
constexpr size_t kMat = size_t(kD) * kD;  // elements of one state matrix

typedef uint16_t Tile[kC][kPitch];

template <int SUFFIX>
__device__ __forceinline__ float row_total(float scanned)
{
    return SUFFIX == 0 ? dpp_or_zero<0x15f>(scanned) : dpp_or_zero<0x150>(scanned);  // row_newbcast:15 / :0
}

// MFMA operand whose 16 rows (A) or columns (B) are tile rows row0..row0+15 and whose contraction
// index runs along the tile's columns: k-slot j of K-step kk is column 32kk + 8g + j.
__device__ __forceinline__ bf16x8 row_frag(const Tile &tile, int row0, int kk, int r, int g)
{
    return *reinterpret_cast<const bf16x8 *>(&tile[row0 + r][32 * kk + 8 * g]);
}

// MFMA operand whose 16 rows (A) or columns (B) are tile columns col0..col0+15 and whose contraction
// index runs along the tile's rows: k-slot j of K-step kk is row 32kk + 8g + j.
__device__ __forceinline__ bf16x8 col_frag(const Tile &tile, int col0, int kk, int r, int g)
{
    const int row = 32 * kk + 8 * g + (r >> 2), col = col0 + 4 * (r & 3);
    return join(lds_read_tr(&tile[row][col]), lds_read_tr(&tile[row + 4][col]));
}

// MFMA A operand whose 16 rows are tile columns col0..col0+15, contracted over the tile's rows
// (tokens) in accumulator order: k-slots 0..3 of K-step kk are rows 32kk + 4g + e, slots 4..7 rows
// 32kk + 16 + 4g + e, which is where a lane's accumulators of two stacked 16x16 tiles sit.
__device__ __forceinline__ bf16x8 token_frag(const Tile &tile, int col0, int kk, int r, int g)
{
    const int row = 32 * kk + 4 * g + (r >> 2), col = col0 + 4 * (r & 3);
    return join(lds_read_tr(&tile[row][col]), lds_read_tr(&tile[row + 16][col]));
}

// B operand of a contraction over the chunk's tokens with a 0/1 triangle: k-slot j of K-step kk is
// token s = 32kk + 8g + j, the lane's column is token u; 1 where s REL u holds.
enum Rel { kLe = 0, kGe = 1 };
template <int REL>
__device__ __forceinline__ bf16x8 tri_frag(int kk, int g, int u)
{
    uint32_t word[4];
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) {
        uint32_t bits = 0;
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            const int s = 32 * kk + 8 * g + 2 * jj + half;
            const bool one = REL == kLe ? s <= u : s >= u;
            bits |= (one ? 0x3F80u : 0u) << (16 * half);
        }
        word[jj] = bits;
    }
    return __builtin_bit_cast(bf16x8, make_uint4(word[0], word[1], word[2], word[3]));
}

// One slab's rows of a [.., width] bf16 tensor (width 64, or 32 for the queries, keys and gates of
// a 32-wide head) behind a buffer resource that ends with the slab's last token (loads beyond it
// return zeros, stores beyond it are dropped).  Rows of 32 are widened to the kernels' 64 channels
// with zeros: channels 32..63 then carry q = k = 0 and log-gate 0 through every step and their
// results are not stored; the pieces of the missing half are requested, and stored, at an offset
// beyond the extent.
struct SlabRows {
    __amdgpu_buffer_rsrc_t rsrc;
    unsigned pitch;   // bytes between consecutive tokens
    unsigned pieces;  // 16-byte pieces per row: 8 or 4
};
constexpr unsigned kBeyond = 0xfffffff0u;

__device__ __forceinline__ SlabRows slab_rows(const void *base, long slab, int L, int heads_token_major, int width = kD)
{
    const size_t first = heads_token_major
                             ? size_t(slab / heads_token_major) * size_t(L) * heads_token_major + slab % heads_token_major
                             : size_t(slab) * L;
    const unsigned pitch = 2u * unsigned(width) * unsigned(heads_token_major ? heads_token_major : 1);
    const unsigned extent = unsigned(L - 1) * pitch + 2u * unsigned(width);
    SlabRows s;
    s.rsrc = slab_resource(static_cast<const char *>(base) + first * (2 * size_t(width)), extent);
    s.pitch = pitch;
    s.pieces = unsigned(width) / 8u;
    return s;
}

// Whole rows of a chunk: lane i of wave w takes 16-byte piece i%8 of rows 16w + i/8 and 16w + 8 + i/8.
// Requested first (all of a phase's tensors together), put into a tile when they are needed.
struct ChunkRows {
    u32x4 p[2];
};

__device__ __forceinline__ ChunkRows fetch_rows(const SlabRows &rows, unsigned t0, int w, int lane)
{
    ChunkRows c;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const unsigned off = (t0 + 16 * w + 8 * h + (lane >> 3)) * rows.pitch + 16u * (lane & 7);
        c.p[h] = __builtin_amdgcn_raw_buffer_load_b128(rows.rsrc, unsigned(lane & 7) < rows.pieces ? off : kBeyond, 0, 0);
    }
    return c;
}

// kHalf: the values are halved on the way (exact in bf16).
template <bool kHalf>
__device__ __forceinline__ void put_rows(Tile &tile, const ChunkRows &c, int w, int lane)
{
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        u32x4 x = c.p[h];
        if (kHalf) {
#pragma unroll
            for (int i = 0; i < 4; ++i) x[i] = pack2(0.5f * bf16_lo_to_f32(x[i]), 0.5f * bf16_hi_to_f32(x[i]));
        }
        *reinterpret_cast<uint4 *>(&tile[16 * w + 8 * h + (lane >> 3)][8 * (lane & 7)]) = make_uint4(x[0], x[1], x[2], x[3]);
    }
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

// The lane's own four pieces of a token row (channels 16ct + 4g .. + 3 of token 16w + r) out of
// rows the wave has staged itself: rows 16w..16w+15 of a tile belong to wave w alone.
__device__ __forceinline__ void take_own(const Tile &tile, int w, int r, int g, uint2 (&x)[4])
{
    wave_lds_fence();
#pragma unroll
    for (int ct = 0; ct < 4; ++ct) x[ct] = *reinterpret_cast<const uint2 *>(&tile[16 * w + r][16 * ct + 4 * g]);
}

// The wave's 16 result rows, held as the lanes' own pieces, to global memory as whole rows: through
// the wave's rows of a tile that nobody reads at that point, then 16 bytes per lane, 8 lanes a row.
__device__ __forceinline__ void store_own(Tile &tile, const SlabRows &rows, unsigned t0, int w, int lane, int r, int g,
                                          const f32x4 (&x)[4])
{
#pragma unroll
    for (int ct = 0; ct < 4; ++ct) *reinterpret_cast<uint2 *>(&tile[16 * w + r][16 * ct + 4 * g]) = pack4(x[ct]);
    wave_lds_fence();
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int row = 16 * w + 8 * h + (lane >> 3);
        const uint4 v = *reinterpret_cast<const uint4 *>(&tile[row][8 * (lane & 7)]);
        const unsigned off = (t0 + row) * rows.pitch + 16u * (lane & 7);
        __builtin_amdgcn_raw_buffer_store_b128(u32x4{v.x, v.y, v.z, v.w}, rows.rsrc,
                                               unsigned(lane & 7) < rows.pieces ? off : kBeyond, 0, 0);
    }
    wave_lds_fence();  // the rows may be reused by this wave right away
}

// the lane's piece of tile row 16w + r
__device__ __forceinline__ void put_own(Tile &tile, int w, int r, int g, int ct, const f32x4 &x)
{
    *reinterpret_cast<uint2 *>(&tile[16 * w + r][16 * ct + 4 * g]) = pack4(x);
}

// Inclusive cumulative log-gates of the chunk on the matrix cores (a product with a 0/1 triangle is
// exact in bf16 x bf16 -> fp32): b[ct][e] for the lane's token and channel 16ct + 4g + e, prefix
// sums for DIR 0, suffix sums for DIR 1.
template <int DIR, int kCt>
__device__ __forceinline__ void gate_scan(const Tile &gates, int w, int r, int g, f32x4 (&b)[4])
{
    const bf16x8 t0 = tri_frag<DIR == 0 ? kLe : kGe>(0, g, 16 * w + r);
    const bf16x8 t1 = tri_frag<DIR == 0 ? kLe : kGe>(1, g, 16 * w + r);
#pragma unroll
    for (int ct = 0; ct < 4; ++ct) {
        const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
        b[ct] = zero;
        if (ct < kCt) b[ct] = mfma(col_frag(gates, 16 * ct, 1, r, g), t1, mfma(col_frag(gates, 16 * ct, 0, r, g), t0, zero));
    }
}

// ---- workspace ---------------------------------------------------------------------------------
// [states][log-decays][slab marks]
//   states, per (slab, chunk): four bf16 64x64 matrices, row-major [key channel][value column]:
//     0: forward  state entering the chunk from the left      (pass 1 leaves U there)
//     1: forward  A' of the chunk (decayed adjoint from the right)     (pass 1: W)
//     2: backward state entering the chunk from the right
//     3: backward A' of the chunk (decayed adjoint from the left)
//   log-decays, per (slab, chunk, direction): the chunk's total log-gate per channel, fp32
//   slab marks: one int per slab, non-zero when the slab is left to the exact kernels
struct Workspace {
    uint16_t *states;
    float *logdec;
    int *marks;
};

inline size_t align256(size_t n) { return (n + 255) / 256 * 256; }

inline int chunks_of(int L) { return (L + kC - 1) / kC; }

inline size_t states_bytes(long BH, int L) { return align256(size_t(BH) * chunks_of(L) * 4 * kMat * sizeof(uint16_t)); }
inline size_t logdec_bytes(long BH, int L) { return align256(size_t(BH) * chunks_of(L) * 2 * kD * sizeof(float)); }
inline size_t marks_bytes(long BH) { return align256(size_t(BH) * sizeof(int)); }

struct LocalLds {
    Tile v, dout, gates, qt, kh;
};

// ---- pass 1: the chunk's own contributions to the states ----------------------------------------
// kCt: channel tiles of 16 that carry data (4; 2 for a 32-wide head, whose channels 32..63 are zero
// in q, k and the gates: their rows of the matrices are neither computed, stored nor read anywhere).
template <int kCt>
__global__ __launch_bounds__(kThreads, 2) void bigla_bwd_chunk_local_kernel(
    const void *__restrict__ q_all, const void *__restrict__ k_all, const void *__restrict__ v_all,
    const void *__restrict__ gf_all, const void *__restrict__ gb_all, const void *__restrict__ do_all,
    uint16_t *__restrict__ states, float *__restrict__ logdec, int L, int heads_token_major, int n_chunks, int dk)
{
    __shared__ __align__(16) LocalLds sm;
    const long unit = blockIdx.x;
    const long slab = unit / n_chunks;
    const int chunk = int(unit % n_chunks);
    const unsigned t0 = unsigned(chunk) * kC;
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, r = lane & 15, g = lane >> 4;

    const SlabRows q = slab_rows(q_all, slab, L, heads_token_major, dk), k = slab_rows(k_all, slab, L, heads_token_major, dk);
    const SlabRows v = slab_rows(v_all, slab, L, heads_token_major), dout = slab_rows(do_all, slab, L, heads_token_major);
    const SlabRows gf = slab_rows(gf_all, slab, L, heads_token_major, dk), gb = slab_rows(gb_all, slab, L, heads_token_major, dk);

    uint2 qr[4], kr[4];
    {
        const ChunkRows cq = fetch_rows(q, t0, w, lane), ck = fetch_rows(k, t0, w, lane);
        const ChunkRows cv = fetch_rows(v, t0, w, lane), cd = fetch_rows(dout, t0, w, lane);
        put_rows<false>(sm.qt, cq, w, lane);
        put_rows<false>(sm.kh, ck, w, lane);
        put_rows<false>(sm.v, cv, w, lane);
        put_rows<true>(sm.dout, cd, w, lane);
    }
    ChunkRows cg[2] = {fetch_rows(gf, t0, w, lane), fetch_rows(gb, t0, w, lane)};
    take_own(sm.qt, w, r, g, qr);
    take_own(sm.kh, w, r, g, kr);

    uint16_t *mats = states + size_t(unit) * 4 * kMat;
    const bf16x8 ones = __builtin_bit_cast(bf16x8, make_uint4(0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u));

#pragma unroll
    for (int dir = 0; dir < 2; ++dir) {
        if (dir == 1) __syncthreads();  // the first direction's products have read the tiles
        put_rows<false>(sm.gates, cg[dir], w, lane);
        __syncthreads();
        f32x4 b[4], T[4];
        if (dir == 0)
            gate_scan<0, kCt>(sm.gates, w, r, g, b);
        else
            gate_scan<1, kCt>(sm.gates, w, r, g, b);
#pragma unroll
        for (int ct = 0; ct < 4; ++ct) {
            const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
            if (ct >= kCt) {  // no data: total log-gate 0 (the scan of the marks reads every channel)
                if (w == 0 && r == 0) *reinterpret_cast<f32x4 *>(&logdec[(size_t(unit) * 2 + dir) * kD + 16 * ct + 4 * g]) = zero;
                continue;
            }
            T[ct] = mfma(col_frag(sm.gates, 16 * ct, 1, r, g), ones, mfma(col_frag(sm.gates, 16 * ct, 0, r, g), ones, zero));
            const f32x4 qv = unpack4(qr[ct]), kv = unpack4(kr[ct]);
            f32x4 qs, ks;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                qs[e] = qv[e] * fast_exp2(b[ct][e] * kLog2e);
                ks[e] = kv[e] * fast_exp2((T[ct][e] - b[ct][e]) * kLog2e);
            }
            put_own(sm.qt, w, r, g, ct, qs);
            put_own(sm.kh, w, r, g, ct, ks);
            if (w == 0 && r == 0)
                *reinterpret_cast<f32x4 *>(&logdec[(size_t(unit) * 2 + dir) * kD + 16 * ct + 4 * g]) = T[ct];
        }
        __syncthreads();
        // U^T[j][i] = sum_t v[t][j] kh[t][i],  W^T[j][i] = sum_t do'[t][j] q~[t][i]: a wave takes 16 rows
        // i (and, with two row tiles only, half of the column tiles), the lane ends up with four
        // consecutive columns j of its row
        uint16_t *U = mats + size_t(2 * dir) * kMat, *W = U + kMat;
        const int it = kCt == 4 ? w : (w & 1);          // row tile
        const int mt0 = kCt == 4 ? 0 : 2 * (w >> 1);    // first column tile
#pragma unroll
        for (int mi = 0; mi < kCt; ++mi) {
            const int mt = mt0 + mi;
            f32x4 u = {0.f, 0.f, 0.f, 0.f}, x = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kk = 0; kk < 2; ++kk) {
                u = mfma(col_frag(sm.v, 16 * mt, kk, r, g), col_frag(sm.kh, 16 * it, kk, r, g), u);
                x = mfma(col_frag(sm.dout, 16 * mt, kk, r, g), col_frag(sm.qt, 16 * it, kk, r, g), x);
            }
            *reinterpret_cast<uint2 *>(&U[(16 * it + r) * kD + 16 * mt + 4 * g]) = pack4(u);
            *reinterpret_cast<uint2 *>(&W[(16 * it + r) * kD + 16 * mt + 4 * g]) = pack4(x);
        }
    }
}

// ---- pass 2: the chunk-to-chunk recurrences, elementwise ------------------------------------------
// grid: 16 workgroups per slab = 4 matrices x 4 quarters; a thread owns 4 consecutive elements of a
// row and walks the slab's chunks in the matrix's direction, its loads requested kScanAhead chunks
// ahead (the walk is a chain of dependent fp32 operations, but the addresses are known; measured at
// 64 chunks per slab: 69 / 66 / 62 / 56 us for 4 / 8 / 16 / 32 chunks ahead; with 4 chunks per slab
// the deep version only pays for its longer prologue, 25 us against 17 us).
constexpr int kScanThreads = 256;

template <int kScanAhead, int kCt>
__global__ __launch_bounds__(kScanThreads) void bigla_bwd_chunk_scan_kernel(uint16_t *__restrict__ states,
                                                                       const float *__restrict__ logdec,
                                                                       int *__restrict__ marks, int n_chunks)
{
    constexpr int kScanParts = kCt * 256 / kScanThreads;  // workgroups per matrix: 16 * kCt rows of 16 pieces
    const long slab = blockIdx.x / (4 * kScanParts);
    const int kind = (blockIdx.x / kScanParts) & 3, part = blockIdx.x % kScanParts;
    const int tid = threadIdx.x;
    const int piece = part * kScanThreads + tid;  // 0 .. 256 * kCt - 1
    const int row = piece >> 4;
    const int dir = kind >> 1;
    const bool adjoint = (kind & 1) != 0;
    const bool ascending = kind == 0 || kind == 3;

    if (kind == 0 && part == 0) {
        // mark the slab when some chunk decays by more than the fast form can carry
        __shared__ float lowest[kScanThreads];
        float m = 0.f;
        const float *ld = logdec + size_t(slab) * n_chunks * 2 * kD;
        for (long i = tid; i < long(n_chunks) * 2 * kD; i += kScanThreads) m = fminf(m, ld[i]);
        lowest[tid] = m;
        __syncthreads();
        for (int s = kScanThreads / 2; s > 0; s >>= 1) {
            if (tid < s) lowest[tid] = fminf(lowest[tid], lowest[tid + s]);
            __syncthreads();
        }
        // (a NaN gate total compares false and leaves the slab to this path, whose outputs are then NaN too)
        if (tid == 0) marks[slab] = (-lowest[0] > kFastRange) ? 1 : 0;
    }

    uint16_t *mat = states + (size_t(slab) * n_chunks * 4 + kind) * kMat + size_t(piece) * 4;
    const float *ld = logdec + (size_t(slab) * n_chunks * 2 + dir) * kD + row;
    struct Item {
        uint2 x;
        float logd;
    };
    auto fetch = [&](int n) {
        Item it;
        it.x = make_uint2(0u, 0u);
        it.logd = 0.f;
        if (n < n_chunks) {
            const int c = ascending ? n : n_chunks - 1 - n;
            it.x = *reinterpret_cast<const uint2 *>(mat + size_t(c) * 4 * kMat);
            it.logd = ld[size_t(c) * 2 * kD];
        }
        return it;
    };
    f32x4 s = {0.f, 0.f, 0.f, 0.f};
    Item ahead[kScanAhead];
#pragma unroll
    for (int j = 0; j < kScanAhead; ++j) ahead[j] = fetch(j);
    for (int n0 = 0; n0 < n_chunks; n0 += kScanAhead) {
#pragma unroll
        for (int j = 0; j < kScanAhead; ++j) {
            const int n = n0 + j;
            if (n < n_chunks) {
                const Item cur = ahead[j];
                ahead[j] = fetch(n + kScanAhead);
                const int c = ascending ? n : n_chunks - 1 - n;
                const float d = fast_exp2(cur.logd * kLog2e);
                const f32x4 u = unpack4(cur.x);
                f32x4 o;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    if (adjoint) {
                        o[e] = d * s[e];     // A' of this chunk
                        s[e] = u[e] + o[e];  // adjoint of the previous chunk's end state
                    } else {
                        o[e] = s[e];         // state entering this chunk
                        s[e] = d * s[e] + u[e];
                    }
                }
                *reinterpret_cast<uint2 *>(mat + size_t(c) * 4 * kMat) = pack4(o);
            }
        }
    }
}

// ---- pass 3: the gradients of one chunk ------------------------------------------------------------

struct MainLds {
    Tile v;      // values                                   [token][column]
    Tile dout;   // d_out / 2                                [token][column]
    Tile gp;     // log-gates                                [token][channel]
    Tile qt;     // q~                                       [token][channel]
    Tile kt;     // k~
    Tile st;     // S_in                                     [channel][column]
    Tile ad;     // A'
    float R[kD]; // rowsum(S_in * A') per channel
    float tot[2][4][kD];  // per wave and channel: the wave's sums of the two kinds of dg summands
};

struct Grads {
    f32x4 dq[4], dk[4], dv[4];  // token 16w + r, channels / columns 16ct + 4g + e
};

// What one direction reads beside q, k, v, do: its log-gates and its two state matrices.  Requested
// ahead of the phase that needs them (the global latency then overlaps other work).
struct DirInputs {
    ChunkRows gates;
    uint4 st[2], ad[2];
};

template <int DIR, int kCt>
__device__ __forceinline__ DirInputs fetch_dir(const SlabRows &gates, const uint16_t *mats, unsigned t0, int tid, int w,
                                               int lane)
{
    DirInputs in;
    in.gates = fetch_rows(gates, t0, w, lane);
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        in.st[h] = in.ad[h] = make_uint4(0u, 0u, 0u, 0u);
        if (2 * h < kCt) {  // piece tid + 256 h lies in rows 32h .. 32h + 31
            in.st[h] = reinterpret_cast<const uint4 *>(mats + size_t(2 * DIR) * kMat)[tid + kThreads * h];
            in.ad[h] = reinterpret_cast<const uint4 *>(mats + size_t(2 * DIR + 1) * kMat)[tid + kThreads * h];
        }
    }
    return in;
}

__device__ __forceinline__ void put_matrix(Tile &tile, const uint4 (&x)[2], int tid)
{
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int p = tid + kThreads * h;
        *reinterpret_cast<uint4 *>(&tile[p >> 3][8 * (p & 7)]) = x[h];
    }
}

// `in`: this direction's inputs, already requested; `next`: called once the contractions are done,
// to request the other direction's.
template <int DIR, int kCt, class Next>
__device__ __forceinline__ void chunk_direction(MainLds &sm, const DirInputs &in, const SlabRows &dg_rows, unsigned t0,
                                                int tid, int w, int lane, int r, int g, const uint2 (&qr)[4],
                                                const uint2 (&kr)[4], Grads &acc, Next next)
{
    const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
    if (DIR == 1) __syncthreads();  // the first direction's last reads of the tiles are done
    put_rows<false>(sm.gp, in.gates, w, lane);
    put_matrix(sm.st, in.st, tid);
    put_matrix(sm.ad, in.ad, tid);
    __syncthreads();

    // cumulative gates, scaled queries and keys (kept as rounded: the gate gradient below must use
    // exactly the operands of the contractions, see there)
    f32x4 Ep[4];
    {
        f32x4 b[4];
        gate_scan<DIR, kCt>(sm.gp, w, r, g, b);
#pragma unroll
        for (int ct = 0; ct < kCt; ++ct) {
            const f32x4 qv = unpack4(qr[ct]), kv = unpack4(kr[ct]);
            f32x4 qs, ks;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float x = b[ct][e] * kLog2e;
                Ep[ct][e] = fast_exp2(x);
                qs[e] = qv[e] * Ep[ct][e];
                ks[e] = kv[e] * fast_exp2(-x);
            }
            put_own(sm.qt, w, r, g, ct, qs);
            put_own(sm.kt, w, r, g, ct, ks);
        }
    }
    // rowsum(S_in * A'): four threads per row, 16 columns each
    if ((tid >> 2) < 16 * kCt) {
        const int row = tid >> 2, c0 = 16 * (tid & 3);
        float sum = 0.f;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const uint4 a = *reinterpret_cast<const uint4 *>(&sm.st[row][c0 + 8 * h]);
            const uint4 b = *reinterpret_cast<const uint4 *>(&sm.ad[row][c0 + 8 * h]);
            sum += bf16_lo_to_f32(a.x) * bf16_lo_to_f32(b.x) + bf16_hi_to_f32(a.x) * bf16_hi_to_f32(b.x);
            sum += bf16_lo_to_f32(a.y) * bf16_lo_to_f32(b.y) + bf16_hi_to_f32(a.y) * bf16_hi_to_f32(b.y);
            sum += bf16_lo_to_f32(a.z) * bf16_lo_to_f32(b.z) + bf16_hi_to_f32(a.z) * bf16_hi_to_f32(b.z);
            sum += bf16_lo_to_f32(a.w) * bf16_lo_to_f32(b.w) + bf16_hi_to_f32(a.w) * bf16_hi_to_f32(b.w);
        }
        sum += __shfl_xor(sum, 1);
        sum += __shfl_xor(sum, 2);
        if ((tid & 3) == 0) sm.R[row] = sum;
    }
    __syncthreads();  // q~, k~ complete; every wave is done with the gates

    // The wave's strips of the masked score matrices, straight from the accumulators into the B
    // operands of the contractions over tokens (no trip through LDS): the row strip of dP for X
    // (keys 16m + 4g + e, query 16w + r) and the column strips of dP and P for Yi and dv (queries
    // 16m + 4g + e, key 16w + r).  A lane's accumulators of tiles m = 2kk, 2kk + 1 are exactly its
    // k-slots of K-step kk when slots 0..3 are tokens 32kk + 4g + e and slots 4..7 tokens
    // 32kk + 16 + 4g + e; the A operands (token_frag) use the same order.
    const bf16x8 own_k[2] = {row_frag(sm.kt, 16 * w, 0, r, g), row_frag(sm.kt, 16 * w, 1, r, g)};
    const bf16x8 own_d[2] = {row_frag(sm.dout, 16 * w, 0, r, g), row_frag(sm.dout, 16 * w, 1, r, g)};
    const bf16x8 own_v[2] = {row_frag(sm.v, 16 * w, 0, r, g), row_frag(sm.v, 16 * w, 1, r, g)};
    // Each strip is split into two bf16 halves (value = hi + lo to 16 bits): the scores then enter
    // the second contraction unrounded, for one more MFMA per product and no further LDS traffic.
    bf16x8 bX[2], bY[2], bP[2], bXl[2], bYl[2], bPl[2];
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) {
        uint2 x[2], y[2], p[2], xl[2], yl[2], pl[2];
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            const int m = 2 * kk + half;
            f32x4 dr = zero, dc = zero, pc = zero;
#pragma unroll
            for (int k2 = 0; k2 < 2; ++k2) {
                dr = mfma(row_frag(sm.v, 16 * m, k2, r, g), own_d[k2], dr);     // dP[t own][s]
                dc = mfma(row_frag(sm.dout, 16 * m, k2, r, g), own_v[k2], dc);  // dP[t][s own]
                if (2 * k2 < kCt) pc = mfma(row_frag(sm.qt, 16 * m, k2, r, g), own_k[k2], pc);  // P[t][s own]
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int far = 16 * m + 4 * g + e, own = 16 * w + r;
                // row strip: far is the key, own the query; column strips: the other way round
                const bool keep_row = DIR == 0 ? far <= own : far >= own;
                const bool keep_col = DIR == 0 ? own <= far : own >= far;
                dr[e] = keep_row ? dr[e] : 0.f;
                dc[e] = keep_col ? dc[e] : 0.f;
                pc[e] = keep_col ? pc[e] : 0.f;
            }
            x[half] = pack4(dr);
            y[half] = pack4(dc);
            p[half] = pack4(pc);
            const f32x4 xh = unpack4(x[half]), yh = unpack4(y[half]), ph = unpack4(p[half]);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                dr[e] -= xh[e];
                dc[e] -= yh[e];
                pc[e] -= ph[e];
            }
            xl[half] = pack4(dr);
            yl[half] = pack4(dc);
            pl[half] = pack4(pc);
        }
        bX[kk] = __builtin_bit_cast(bf16x8, make_uint4(x[0].x, x[0].y, x[1].x, x[1].y));
        bY[kk] = __builtin_bit_cast(bf16x8, make_uint4(y[0].x, y[0].y, y[1].x, y[1].y));
        bP[kk] = __builtin_bit_cast(bf16x8, make_uint4(p[0].x, p[0].y, p[1].x, p[1].y));
        bXl[kk] = __builtin_bit_cast(bf16x8, make_uint4(xl[0].x, xl[0].y, xl[1].x, xl[1].y));
        bYl[kk] = __builtin_bit_cast(bf16x8, make_uint4(yl[0].x, yl[0].y, yl[1].x, yl[1].y));
        bPl[kk] = __builtin_bit_cast(bf16x8, make_uint4(pl[0].x, pl[0].y, pl[1].x, pl[1].y));
    }

    f32x4 E1[4], E2[4];
#pragma unroll
    for (int ct = 0; ct < 4; ++ct) {
        f32x4 X = zero, Yi = zero, Ye = zero, V = zero;
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
            if (ct < kCt) {
                // X^T[c][t] = sum_s k~[s][c] dP[t][s] + sum_j S_in[c][j] do'[t][j]
                const bf16x8 ak = token_frag(sm.kt, 16 * ct, kk, r, g);
                X = mfma(ak, bXl[kk], X);
                X = mfma(ak, bX[kk], X);
                X = mfma(row_frag(sm.st, 16 * ct, kk, r, g), own_d[kk], X);
                // Yi^T[c][s] = sum_t q~[t][c] dP[t][s],  Ye^T[c][s] = sum_j A'[c][j] v[s][j]
                const bf16x8 aq = token_frag(sm.qt, 16 * ct, kk, r, g);
                Yi = mfma(aq, bYl[kk], Yi);
                Yi = mfma(aq, bY[kk], Yi);
                Ye = mfma(row_frag(sm.ad, 16 * ct, kk, r, g), own_v[kk], Ye);
            }
            // dv^T[j][s] = sum_t do'[t][j] P[t][s] + sum_i A'[i][j] k~[s][i]   (column tile j = ct)
            const bf16x8 ad = token_frag(sm.dout, 16 * ct, kk, r, g);
            V = mfma(ad, bPl[kk], V);
            V = mfma(ad, bP[kk], V);
            if (2 * kk < kCt) V = mfma(col_frag(sm.ad, 16 * ct, kk, r, g), own_k[kk], V);
        }
        if (ct >= kCt) {
#pragma unroll
            for (int e = 0; e < 4; ++e) acc.dv[ct][e] += V[e];
            continue;
        }
        // The summands of the gate gradient take q~ and k~ as the contractions saw them (rounded to
        // bf16): sum_{t>=u} q~ * X - sum_{s>=u} k~ * Yi is then, term by term, the sum over the pairs
        // s < u <= t of q~_t dP_ts k~_s, and the rounding of the operands perturbs each pair once
        // instead of leaving the difference of two long sums that no longer cancel.
        const f32x4 qv = unpack4(*reinterpret_cast<const uint2 *>(&sm.qt[16 * w + r][16 * ct + 4 * g]));
        const f32x4 kv = unpack4(*reinterpret_cast<const uint2 *>(&sm.kt[16 * w + r][16 * ct + 4 * g]));
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            acc.dq[ct][e] += Ep[ct][e] * X[e];
            acc.dk[ct][e] += __builtin_amdgcn_rcpf(Ep[ct][e]) * (Yi[e] + Ye[e]);
            acc.dv[ct][e] += V[e];
            E1[ct][e] = qv[e] * X[e] - kv[e] * Yi[e];
            E2[ct][e] = kv[e] * Ye[e];
        }
    }
    next();
    // dg_u = sum_{t >= u} E1_t + sum_{t < u} E2_t + rowsum(S_in * A')   (forward; mirrored backward):
    // scans over the wave's 16 tokens with DPP row operations, in fp32, then the other waves' totals
    {
        constexpr int kFar = DIR == 0 ? 1 : 0;  // E1 accumulates from the far side of the direction
        f32x4 dg[4];
#pragma unroll
        for (int ct = kCt; ct < 4; ++ct) dg[ct] = zero;
#pragma unroll
        for (int ct = 0; ct < kCt; ++ct) {
            f32x4 t1, t2;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float a = row_scan<kFar>(E1[ct][e]);
                const float b = row_scan<1 - kFar>(E2[ct][e]);
                dg[ct][e] = a + (b - E2[ct][e]);
                t1[e] = row_total<kFar>(a);
                t2[e] = row_total<1 - kFar>(b);
            }
            if (r == 0) {
                *reinterpret_cast<f32x4 *>(&sm.tot[0][w][16 * ct + 4 * g]) = t1;
                *reinterpret_cast<f32x4 *>(&sm.tot[1][w][16 * ct + 4 * g]) = t2;
            }
        }
        __syncthreads();  // totals visible; every wave is done with S_in, whose tile carries dg out
#pragma unroll
        for (int ct = 0; ct < kCt; ++ct) {
            f32x4 s = *reinterpret_cast<const f32x4 *>(&sm.R[16 * ct + 4 * g]);
#pragma unroll
            for (int w2 = 0; w2 < 4; ++w2) {
                if (w2 == w) continue;
                const bool far = DIR == 0 ? w2 > w : w2 < w;
                const f32x4 t = *reinterpret_cast<const f32x4 *>(&sm.tot[far ? 0 : 1][w2][16 * ct + 4 * g]);
#pragma unroll
                for (int e = 0; e < 4; ++e) s[e] += t[e];
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) dg[ct][e] += s[e];
        }
        store_own(sm.st, dg_rows, t0, w, lane, r, g, dg);
    }
}

template <int kCt>
__global__ __launch_bounds__(kThreads, 2) void bigla_bwd_chunk_main_kernel(
    const void *__restrict__ q_all, const void *__restrict__ k_all, const void *__restrict__ v_all,
    const void *__restrict__ gf_all, const void *__restrict__ gb_all, const void *__restrict__ do_all,
    void *__restrict__ dq_all, void *__restrict__ dk_all, void *__restrict__ dv_all, void *__restrict__ dgf_all,
    void *__restrict__ dgb_all, const uint16_t *__restrict__ states, const int *__restrict__ marks, int L,
    int heads_token_major, int n_chunks, int dk)
{
    __shared__ __align__(16) MainLds sm;
    const long unit = blockIdx.x;
    const long slab = unit / n_chunks;
    if (marks[slab] != 0) return;  // left to the exact kernels
    const int chunk = int(unit % n_chunks);
    const unsigned t0 = unsigned(chunk) * kC;
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, r = lane & 15, g = lane >> 4;

    const SlabRows q = slab_rows(q_all, slab, L, heads_token_major, dk), k = slab_rows(k_all, slab, L, heads_token_major, dk);
    const SlabRows v = slab_rows(v_all, slab, L, heads_token_major), dout = slab_rows(do_all, slab, L, heads_token_major);
    const SlabRows gf = slab_rows(gf_all, slab, L, heads_token_major, dk), gb = slab_rows(gb_all, slab, L, heads_token_major, dk);
    const SlabRows dgf = slab_rows(dgf_all, slab, L, heads_token_major, dk), dgb = slab_rows(dgb_all, slab, L, heads_token_major, dk);

    uint2 qr[4], kr[4];
    const uint16_t *mats = states + size_t(unit) * 4 * kMat;
    {
        const ChunkRows cq = fetch_rows(q, t0, w, lane), ck = fetch_rows(k, t0, w, lane);
        const ChunkRows cv = fetch_rows(v, t0, w, lane), cd = fetch_rows(dout, t0, w, lane);
        put_rows<false>(sm.qt, cq, w, lane);
        put_rows<false>(sm.kt, ck, w, lane);
        put_rows<false>(sm.v, cv, w, lane);
        put_rows<true>(sm.dout, cd, w, lane);
    }
    const DirInputs in_f = fetch_dir<0, kCt>(gf, mats, t0, tid, w, lane);
    take_own(sm.qt, w, r, g, qr);
    take_own(sm.kt, w, r, g, kr);

    Grads acc;
#pragma unroll
    for (int ct = 0; ct < 4; ++ct) acc.dq[ct] = acc.dk[ct] = acc.dv[ct] = f32x4{0.f, 0.f, 0.f, 0.f};
    DirInputs in_b;
    chunk_direction<0, kCt>(sm, in_f, dgf, t0, tid, w, lane, r, g, qr, kr, acc,
                            [&]() { in_b = fetch_dir<1, kCt>(gb, mats, t0, tid, w, lane); });
    chunk_direction<1, kCt>(sm, in_b, dgb, t0, tid, w, lane, r, g, qr, kr, acc, []() {});

    store_own(sm.st, slab_rows(dq_all, slab, L, heads_token_major, dk), t0, w, lane, r, g, acc.dq);
    store_own(sm.ad, slab_rows(dk_all, slab, L, heads_token_major, dk), t0, w, lane, r, g, acc.dk);
    store_own(sm.v, slab_rows(dv_all, slab, L, heads_token_major), t0, w, lane, r, g, acc.dv);
}

}  // namespace

bool bigla_bwd_chunk_supported(int dk, int dv, bool is_bf16) { return is_bf16 && (dk == kD || dk == kD / 2) && dv == kD; }

size_t bigla_bwd_chunk_workspace_bytes(long BH, int L)
{
    return states_bytes(BH, L) + logdec_bytes(BH, L) + marks_bytes(BH);
}

const int *bigla_bwd_chunk_marks(void *workspace, long BH, int L)
{
    return reinterpret_cast<const int *>(static_cast<char *>(workspace) + states_bytes(BH, L) + logdec_bytes(BH, L));
}

hipError_t bigla_bwd_chunk_launch(const void *q, const void *k, const void *v, const void *g_fwd, const void *g_bwd,
                                  const void *d_out, void *dq, void *dk, void *dv, void *dg_fwd, void *dg_bwd, long BH,
                                  int L, int dk_, int heads_token_major, void *workspace, hipStream_t stream)
{
    const int n_chunks = chunks_of(L);
    const long units = BH * n_chunks;
    if (units > 0x7fffffffL || BH * 16 > 0x7fffffffL) return hipErrorInvalidValue;
    Workspace ws;
    char *base = static_cast<char *>(workspace);
    ws.states = reinterpret_cast<uint16_t *>(base);
    ws.logdec = reinterpret_cast<float *>(base + states_bytes(BH, L));
    ws.marks = reinterpret_cast<int *>(base + states_bytes(BH, L) + logdec_bytes(BH, L));
    auto launch = [&](auto ct) {
        constexpr int kCt = decltype(ct)::value;
        const dim3 scan_grid((unsigned)(BH * 4 * (kCt * 256 / kScanThreads)));
        hipLaunchKernelGGL(bigla_bwd_chunk_local_kernel<kCt>, dim3((unsigned)units), dim3(kThreads), 0, stream, q, k, v,
                           g_fwd, g_bwd, d_out, ws.states, ws.logdec, L, heads_token_major, n_chunks, dk_);
        if (n_chunks > 16)
            hipLaunchKernelGGL((bigla_bwd_chunk_scan_kernel<32, kCt>), scan_grid, dim3(kScanThreads), 0, stream, ws.states,
                               ws.logdec, ws.marks, n_chunks);
        else
            hipLaunchKernelGGL((bigla_bwd_chunk_scan_kernel<8, kCt>), scan_grid, dim3(kScanThreads), 0, stream, ws.states,
                               ws.logdec, ws.marks, n_chunks);
        hipLaunchKernelGGL(bigla_bwd_chunk_main_kernel<kCt>, dim3((unsigned)units), dim3(kThreads), 0, stream, q, k, v,
                           g_fwd, g_bwd, d_out, dq, dk, dv, dg_fwd, dg_bwd, ws.states, ws.marks, L, heads_token_major,
                           n_chunks, dk_);
    };
    if (dk_ == kD)
        launch(std::integral_constant<int, 4>{});
    else
        launch(std::integral_constant<int, 2>{});
    return hipGetLastError();
}

}  // namespace vig
