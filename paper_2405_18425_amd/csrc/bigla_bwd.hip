// Gradient of the BiGLA token mixer (Section 4.2.1, Eq. (BiGLA); the paper trains through it,
// Section 5, and prints no gradient formulas), evaluated token by token in fp32 arithmetic.
//
// With do_t = d_out_t / 2 and, per direction, the state S_t = diag(alpha_t) S_{t-/+1} + k_t^T v_t
// and its adjoint A_t = q_t^T do_t + diag(alpha_{t+/-1}) A_{t+/-1} (running against the state),
//     dq_t = S_t do_t^T ,   dk_t = A_t v_t^T ,   dv_t = k_t A_t ,
// each summed over the two directions, and the log-gates of a direction enter the output only
// through differences of their cumulative sums b, so that dLoss/db_t = q_t * dq_t - k_t * dk_t
// (that direction's parts, elementwise) and
//     dg_fwd_s = sum_{t >= s} (q_t * dq^f_t - k_t * dk^f_t) ,
//     dg_bwd_s = sum_{t <= s} (q_t * dq^b_t - k_t * dk^b_t) .
// A state needs the forward order of its direction, an adjoint the reverse one, so every quantity
// takes two sweeps over the sequence (one per direction); the first sweep's part is parked in the
// fp32 workspace and the second sweep adds its own and writes the result.
//
// Two launches (dq and dv together, then dk with the gate gradients), a workgroup per (slab,
// block of 16 rows or columns of the dk x dv matrices); the matrix lives in registers, 16 lanes
// share a row (or column), a tile of 16 tokens is staged through LDS (requested two tiles ahead)
// and its 16 products are reduced over the sharing lanes in one butterfly:
//   dq : state rows          (ascending sweep with g_fwd, descending with g_bwd); keeps dq^f, dq^b
//   dv : adjoint columns     (descending with g_fwd, ascending with g_bwd)
//   dk : adjoint rows, and the running sums that are dg_fwd (descending sweep) and dg_bwd
//        (ascending); reads dq^f, dq^b, so it runs after the first launch.
// This is the exact-arithmetic path for every head shape and both dtypes (bf16 storage, fp32
// arithmetic).  For bf16 with 64-wide heads the chunkwise matrix-core kernels run first and these
// kernels then take only the slabs marked for them (gates beyond the chunkwise range).
#include "vig_common.hpp"
#include "vig_kernels.hpp"
#include "vig_timing.hpp"

namespace vig {

namespace {

constexpr int kTile = 16;     // tokens staged per LDS tile
constexpr int kShare = 16;    // lanes sharing one row (or column) of the matrix
constexpr int kBlock = 16;    // rows (or columns) per workgroup
constexpr int kThreads = kShare * kBlock;

enum Role { kRoleDq = 0, kRoleDk = 1, kRoleDv = 2 };

// Sums of 16 values over the 16 lanes that share a row: on entry every lane holds its partial sum
// for each of 16 tokens, on exit lane s holds the complete sum of token s (a butterfly that halves
// the values kept per lane at every step: 15 shuffles instead of 64 for 16 separate reductions).
template <int kHalf>
__device__ __forceinline__ void share_sum_step(float (&x)[kTile], int s)
{
    const bool upper = (s & kHalf) != 0;
#pragma unroll
    for (int j = 0; j < kHalf; ++j) {
        const float keep = upper ? x[j + kHalf] : x[j];
        const float send = upper ? x[j] : x[j + kHalf];
        x[j] = keep + __shfl_xor(send, kHalf);
    }
}

__device__ __forceinline__ float share_sum_scatter(float (&x)[kTile], int s)
{
    share_sum_step<8>(x, s);
    share_sum_step<4>(x, s);
    share_sum_step<2>(x, s);
    share_sum_step<1>(x, s);
    return x[0];
}

// Inclusive prefix sum over the 16 lanes that share a row
__device__ __forceinline__ float share_scan(float x, int s)
{
#pragma unroll
    for (int d = 1; d < kShare; d <<= 1) {
        const float y = __shfl_up(x, d, kShare);
        if (s >= d) x += y;
    }
    return x;
}

// A [16 tokens][NC columns] piece of a row tensor moves as 16-byte chunks, one per thread:
// chunk = (token, 16-byte part of the token's NC columns); tokens past the sequence repeat the last
// one (always a valid address) and are replaced by `pad` when the piece is put into LDS.
template <typename E, int NC>
struct Piece {
    static constexpr int kVals = 16 / int(sizeof(E));   // values per chunk
    static constexpr int kPerRow = NC / kVals;           // chunks per token
    static constexpr int kChunks = kTile * kPerRow;      // <= 256 for NC <= 64
    static_assert(NC % kVals == 0 && kChunks <= kShare * kBlock, "piece fits one chunk per thread");

    static __device__ __forceinline__ uint4 load(const E *base, size_t pitch, int t0, int col0, int L, int tid)
    {
        uint4 r = make_uint4(0u, 0u, 0u, 0u);
        if (tid < kChunks) {
            const int tok = min(t0 + tid / kPerRow, L - 1);
            r = *reinterpret_cast<const uint4 *>(base + size_t(tok) * pitch + col0 + (tid % kPerRow) * kVals);
        }
        return r;
    }

    // dst[token][column] = f(value) (f: scale, or exp for log-gates), `pad` for tokens >= n
    template <bool kExp>
    static __device__ __forceinline__ void put(float (*dst)[NC], const uint4 &raw, int n, float scale, float pad, int tid)
    {
        if (tid >= kChunks) return;
        const int tt = tid / kPerRow, c = (tid % kPerRow) * kVals;
        float f[kVals];
        if (sizeof(E) == 2) {
            f[0] = bf16_lo_to_f32(raw.x); f[1] = bf16_hi_to_f32(raw.x);
            f[2 % kVals] = bf16_lo_to_f32(raw.y); f[3 % kVals] = bf16_hi_to_f32(raw.y);
            f[4 % kVals] = bf16_lo_to_f32(raw.z); f[5 % kVals] = bf16_hi_to_f32(raw.z);
            f[6 % kVals] = bf16_lo_to_f32(raw.w); f[7 % kVals] = bf16_hi_to_f32(raw.w);
        } else {
            f[0] = __uint_as_float(raw.x); f[1] = __uint_as_float(raw.y);
            f[2] = __uint_as_float(raw.z); f[3] = __uint_as_float(raw.w);
        }
#pragma unroll
        for (int j = 0; j < kVals; ++j) {
            const float x = kExp ? __expf(f[j]) : scale * f[j];
            dst[tt][c + j] = tt < n ? x : pad;
        }
    }
};

// Rows of one slab of a tensor: element (t, c) of a [.., L, D] slab sits at base[t * pitch + c]
template <typename T>
struct Rows {
    const T *base;
    size_t pitch;
    __device__ __forceinline__ float at(int t, int c) const { return io<T>::load(base + size_t(t) * pitch + c); }
};

// One workgroup's share of one of the three quantities: `block` = slab * parts + part.
template <typename T, int DK, int DV, int ROLE>
__device__ __forceinline__ void bwd_block(
    const T *__restrict__ q_all, const T *__restrict__ k_all, const T *__restrict__ v_all,
    const T *__restrict__ gf_all, const T *__restrict__ gb_all, const T *__restrict__ do_all, T *__restrict__ dq_all,
    T *__restrict__ dk_all, T *__restrict__ dv_all, T *__restrict__ dgf_all, T *__restrict__ dgb_all,
    float *__restrict__ ws_dq /* [2][slabs][L][DK]: dq^f, dq^b */, float *__restrict__ ws_part /* [slabs][L][D]: first sweep */,
    int L, int heads_token_major /* 0: [B,H,L,d]; H: [B,L,H,d] */, long n_slabs, long block,
    const int *__restrict__ only_marked /* null: every slab; else only slabs whose entry is non-zero */)
{
    constexpr bool kRowsRole = ROLE != kRoleDv;     // the workgroup owns rows (channels) of the matrix
    constexpr int D_OWN = kRowsRole ? DK : DV;      // the dimension the workgroup's block lies in
    constexpr int D_SPLIT = kRowsRole ? DV : DK;    // the dimension shared among the 16 lanes
    constexpr int kParts = D_OWN / kBlock;
    constexpr int E = D_SPLIT / kShare;             // matrix elements per thread
    static_assert(D_OWN % kBlock == 0 && D_SPLIT % kShare == 0, "head widths are multiples of 16");

    const int tid = threadIdx.x, own = tid / kShare, s = tid % kShare;
    const long slab = block / kParts;
    if (only_marked && only_marked[slab] == 0) return;  // the chunkwise kernels have taken this slab
    const int i0 = int(block % kParts) * kBlock;  // first row (column) of the block
    const int idx = i0 + own;                          // this thread's row (column)
    const int e0 = s * E;                              // its first element along the shared dimension
    const size_t row0 = heads_token_major
                            ? size_t(slab / heads_token_major) * size_t(L) * heads_token_major + slab % heads_token_major
                            : size_t(slab) * L;
    const size_t step = heads_token_major ? heads_token_major : 1;
    const Rows<T> q = {q_all + row0 * DK, step * DK}, k = {k_all + row0 * DK, step * DK};
    const Rows<T> gf = {gf_all + row0 * DK, step * DK}, gb = {gb_all + row0 * DK, step * DK};
    const Rows<T> v = {v_all + row0 * DV, step * DV}, dout = {do_all + row0 * DV, step * DV};
    float *dqf = ws_dq + size_t(slab) * L * DK, *dqb = ws_dq + (size_t(n_slabs) + slab) * L * DK;
    float *part = ws_part + size_t(slab) * L * D_OWN;

    // per token of the tile: the block's 16 entries of the operand that scales the update (k for the
    // state, q for the adjoint), of the gate, (dk launch) of k and dq^dir, and of the first sweep's
    // result; whole rows of the operands along the shared dimension
    __shared__ float s_own[kTile][kBlock], s_alpha[kTile][kBlock], s_k[kTile][kBlock], s_dq[kTile][kBlock],
        s_first[kTile][kBlock];
    __shared__ __align__(16) float s_a[kTile][D_SPLIT], s_b[kTile][D_SPLIT], s_gate[kRowsRole ? 1 : kTile][D_SPLIT];

    for (int sweep = 0; sweep < 2; ++sweep) {
        if (sweep == 1) {
            // the second sweep starts on the tile the first one ended on and reads, through other
            // threads, what that sweep has just parked in global memory
            __threadfence();
            __syncthreads();
        }
        // first sweep: the forward direction's part (gates g_fwd), second: the backward direction's
        // (g_bwd); the state of a direction is walked with it, its adjoint against it
        const Rows<T> &g = sweep == 0 ? gf : gb;
        const bool ascending = ROLE == kRoleDq ? sweep == 0 : sweep == 1;
        float M[E];       // the thread's elements of S (dq) or A (dk, dv)
        float decay[E];   // dv launch: gate of the previously visited token, per element (rows differ)
        float decay_own = 0.f;  // row launches: the row's gate at the previously visited token
        float G = 0.f;    // dk launch: running sum that is dg
#pragma unroll
        for (int e = 0; e < E; ++e) M[e] = decay[e] = 0.f;

        // A tile's operands are requested one tile ahead, all loads issued together from clamped
        // (always valid) addresses, and put into LDS (zeroed past the sequence) when their turn comes.
        struct TileRegs {
            uint4 own, gate_own, k, dq, first, a, b, gate;
        };
        typedef Piece<T, kBlock> Own;        // the block's 16 columns of a row tensor
        typedef Piece<float, kBlock> OwnF;   // ... of an fp32 workspace array
        typedef Piece<T, D_SPLIT> Full;      // whole rows along the shared dimension
        auto fetch = [&](int tile) {
            TileRegs r;
            const int t0 = tile * kTile;
            r.gate_own = r.k = r.dq = r.first = r.gate = make_uint4(0u, 0u, 0u, 0u);
            if (kRowsRole) {
                r.own = Own::load((ROLE == kRoleDq ? k : q).base, k.pitch, t0, i0, L, tid);
                r.gate_own = Own::load(g.base, g.pitch, t0, i0, L, tid);
                if (ROLE == kRoleDk) {
                    r.k = Own::load(k.base, k.pitch, t0, i0, L, tid);
                    r.dq = OwnF::load(sweep == 0 ? dqf : dqb, DK, t0, i0, L, tid);
                }
            } else {
                r.own = Own::load(dout.base, dout.pitch, t0, i0, L, tid);
            }
            if (sweep == 1) r.first = OwnF::load(ROLE == kRoleDq ? dqf : part, D_OWN, t0, i0, L, tid);
            if (ROLE == kRoleDq) {
                r.a = Full::load(v.base, v.pitch, t0, 0, L, tid);
                r.b = Full::load(dout.base, dout.pitch, t0, 0, L, tid);
            } else if (ROLE == kRoleDk) {
                r.a = Full::load(dout.base, dout.pitch, t0, 0, L, tid);
                r.b = Full::load(v.base, v.pitch, t0, 0, L, tid);
            } else {
                r.a = Full::load(q.base, q.pitch, t0, 0, L, tid);
                r.b = Full::load(k.base, k.pitch, t0, 0, L, tid);
                r.gate = Full::load(g.base, g.pitch, t0, 0, L, tid);
            }
            return r;
        };
        // rows past the sequence are zero (a gate of 1 there is harmless: an ascending sweep visits
        // nothing after them, a descending sweep meets them first, with a zero matrix)
        auto stash = [&](const TileRegs &r, int n) {
            if (kRowsRole) {
                Own::template put<false>(s_own, r.own, n, 1.f, 0.f, tid);
                Own::template put<true>(s_alpha, r.gate_own, n, 1.f, 1.f, tid);
                if (ROLE == kRoleDk) {
                    Own::template put<false>(s_k, r.k, n, 1.f, 0.f, tid);
                    OwnF::template put<false>(s_dq, r.dq, n, 1.f, 0.f, tid);
                }
            } else {
                Own::template put<false>(s_own, r.own, n, 0.5f, 0.f, tid);  // do of the block's columns
            }
            if (sweep == 1) OwnF::template put<false>(s_first, r.first, n, 1.f, 0.f, tid);
            if (ROLE == kRoleDq) {
                Full::template put<false>(s_a, r.a, n, 1.f, 0.f, tid);
                Full::template put<false>(s_b, r.b, n, 0.5f, 0.f, tid);
            } else if (ROLE == kRoleDk) {
                Full::template put<false>(s_a, r.a, n, 0.5f, 0.f, tid);
                Full::template put<false>(s_b, r.b, n, 1.f, 0.f, tid);
            } else {
                Full::template put<false>(s_a, r.a, n, 1.f, 0.f, tid);
                Full::template put<false>(s_b, r.b, n, 1.f, 0.f, tid);
                Full::template put<true>(s_gate, r.gate, n, 1.f, 1.f, tid);
            }
        };

        const int ntiles = (L + kTile - 1) / kTile;
        auto visited = [&](int it) { return ascending ? min(it, ntiles - 1) : max(ntiles - 1 - it, 0); };
        TileRegs next = fetch(visited(0)), next2 = fetch(visited(1));  // two tiles in flight
        for (int it = 0; it < ntiles; ++it) {
            const int tile = visited(it);
            const int t0 = tile * kTile;
            const int n = min(kTile, L - t0);
            __syncthreads();  // the previous tile's LDS reads are done
            stash(next, n);
            __syncthreads();
            next = next2;
            next2 = fetch(visited(it + 2));  // (clamped past the end: loaded, never used)

            // the 16 tokens of the tile in visiting order: the matrix recurrence is sequential, the
            // partial sums of the products are kept and reduced over the sharing lanes in one go
            float acc[kTile];
#pragma unroll
            for (int i = 0; i < kTile; ++i) {
                const int tt = ascending ? i : kTile - 1 - i;
                float a = 0.f;
                if (ROLE == kRoleDq) {
                    // S_t = alpha_t S_prev + k_t^T v_t ;  dq_t = S_t do_t^T
                    const float al = s_alpha[tt][own], kk = s_own[tt][own];
#pragma unroll
                    for (int e = 0; e < E; ++e) {
                        M[e] = fmaf(al, M[e], kk * s_a[tt][e0 + e]);
                        a = fmaf(M[e], s_b[tt][e0 + e], a);
                    }
                } else if (ROLE == kRoleDk) {
                    // A_t = alpha_prev A_prev + q_t^T do_t ;  dk_t = A_t v_t^T
                    const float qq = s_own[tt][own];
#pragma unroll
                    for (int e = 0; e < E; ++e) {
                        M[e] = fmaf(decay_own, M[e], qq * s_a[tt][e0 + e]);
                        a = fmaf(M[e], s_b[tt][e0 + e], a);
                    }
                    decay_own = s_alpha[tt][own];
                } else {
                    // A_t = alpha_prev A_prev + q_t^T do_t ;  dv_t = k_t A_t   (this thread: rows e0.., column idx)
                    const float dd = s_own[tt][own];
#pragma unroll
                    for (int e = 0; e < E; ++e) {
                        M[e] = fmaf(decay[e], M[e], s_a[tt][e0 + e] * dd);
                        a = fmaf(s_b[tt][e0 + e], M[e], a);
                        decay[e] = s_gate[tt][e0 + e];
                    }
                }
                acc[i] = a;
            }
            // lane s now finishes the token visited s-th
            const float total = share_sum_scatter(acc, s);
            const int tt = ascending ? s : kTile - 1 - s;
            const bool live = tt < n;
            const size_t t = size_t(t0 + tt);
            if (ROLE == kRoleDq) {
                if (live) {
                    (sweep == 0 ? dqf : dqb)[t * DK + idx] = total;
                    if (sweep == 1) io<T>::store(dq_all + row0 * DK + t * step * DK + idx, s_first[tt][own] + total);
                }
            } else if (ROLE == kRoleDk) {
                // dg = running sum (in visiting order) of q dq - k dk of this direction
                const float term = live ? s_own[tt][own] * s_dq[tt][own] - s_k[tt][own] * total : 0.f;
                const float run = G + share_scan(term, s);
                G = __shfl(run, kShare - 1, kShare);
                if (live) {
                    io<T>::store((sweep == 0 ? dgf_all : dgb_all) + row0 * DK + t * step * DK + idx, run);
                    if (sweep == 0)
                        part[t * DK + idx] = total;
                    else
                        io<T>::store(dk_all + row0 * DK + t * step * DK + idx, s_first[tt][own] + total);
                }
            } else {
                if (live) {
                    if (sweep == 0)
                        part[t * DV + idx] = total;
                    else
                        io<T>::store(dv_all + row0 * DV + t * step * DV + idx, s_first[tt][own] + total);
                }
            }
        }
    }
}

// dq and dv do not depend on each other: one launch, the first n_slabs * DK / 16 workgroups take dq
template <typename T, int DK, int DV>
__global__ __launch_bounds__(kThreads) void bigla_bwd_dq_dv_kernel(
    const T *__restrict__ q, const T *__restrict__ k, const T *__restrict__ v, const T *__restrict__ gf,
    const T *__restrict__ gb, const T *__restrict__ d_out, T *__restrict__ dq, T *__restrict__ dv,
    float *__restrict__ ws_dq, float *__restrict__ ws_dv, int L, int heads_token_major, long n_slabs,
    const int *__restrict__ only_marked)
{
    const long dq_blocks = n_slabs * (DK / kBlock);
    if (long(blockIdx.x) < dq_blocks)
        bwd_block<T, DK, DV, kRoleDq>(q, k, v, gf, gb, d_out, dq, nullptr, nullptr, nullptr, nullptr, ws_dq, nullptr, L,
                                      heads_token_major, n_slabs, blockIdx.x, only_marked);
    else
        bwd_block<T, DK, DV, kRoleDv>(q, k, v, gf, gb, d_out, nullptr, nullptr, dv, nullptr, nullptr, ws_dq, ws_dv, L,
                                      heads_token_major, n_slabs, long(blockIdx.x) - dq_blocks, only_marked);
}

// dk and both gate gradients (reads dq^f, dq^b from the workspace)
template <typename T, int DK, int DV>
__global__ __launch_bounds__(kThreads) void bigla_bwd_dk_dg_kernel(
    const T *__restrict__ q, const T *__restrict__ k, const T *__restrict__ v, const T *__restrict__ gf,
    const T *__restrict__ gb, const T *__restrict__ d_out, T *__restrict__ dk, T *__restrict__ dgf,
    T *__restrict__ dgb, float *__restrict__ ws_dq, float *__restrict__ ws_dk, int L, int heads_token_major,
    long n_slabs, const int *__restrict__ only_marked)
{
    bwd_block<T, DK, DV, kRoleDk>(q, k, v, gf, gb, d_out, nullptr, dk, nullptr, dgf, dgb, ws_dq, ws_dk, L,
                                  heads_token_major, n_slabs, blockIdx.x, only_marked);
}

template <typename T, int DK, int DV>
hipError_t launch(const void *q, const void *k, const void *v, const void *gf, const void *gb, const void *d_out,
                  void *dq, void *dk, void *dv, void *dgf, void *dgb, long BH, int L, int heads_token_major,
                  float *ws, const int *only_marked, hipStream_t stream)
{
    float *ws_dq = ws;                                // dq^f, dq^b
    float *ws_dk = ws + size_t(2) * BH * L * DK;      // dk of the first sweep
    float *ws_dv = ws_dk + size_t(BH) * L * DK;       // dv of the first sweep
    const long dq_blocks = BH * (DK / kBlock), dv_blocks = BH * (DV / kBlock);
    if (dq_blocks + dv_blocks > 0x7fffffffL) return hipErrorInvalidValue;
    const T *qq = static_cast<const T *>(q), *kk = static_cast<const T *>(k), *vv = static_cast<const T *>(v);
    const T *f = static_cast<const T *>(gf), *b = static_cast<const T *>(gb), *dd = static_cast<const T *>(d_out);
    hipLaunchKernelGGL((bigla_bwd_dq_dv_kernel<T, DK, DV>), dim3((unsigned)(dq_blocks + dv_blocks)), dim3(kThreads), 0,
                       stream, qq, kk, vv, f, b, dd, static_cast<T *>(dq), static_cast<T *>(dv), ws_dq, ws_dv, L,
                       heads_token_major, BH, only_marked);
    hipLaunchKernelGGL((bigla_bwd_dk_dg_kernel<T, DK, DV>), dim3((unsigned)dq_blocks), dim3(kThreads), 0, stream, qq, kk,
                       vv, f, b, dd, static_cast<T *>(dk), static_cast<T *>(dgf), static_cast<T *>(dgb), ws_dq, ws_dk, L,
                       heads_token_major, BH, only_marked);
    return hipGetLastError();
}

template <typename T, int DK>
hipError_t launch_dv(int dv_, const void *q, const void *k, const void *v, const void *gf, const void *gb,
                     const void *d_out, void *dq, void *dk, void *dv, void *dgf, void *dgb, long BH, int L,
                     int heads_token_major, float *ws, const int *only_marked, hipStream_t stream)
{
    switch (dv_) {
        case 16: return launch<T, DK, 16>(q, k, v, gf, gb, d_out, dq, dk, dv, dgf, dgb, BH, L, heads_token_major, ws, only_marked, stream);
        case 32: return launch<T, DK, 32>(q, k, v, gf, gb, d_out, dq, dk, dv, dgf, dgb, BH, L, heads_token_major, ws, only_marked, stream);
        case 64: return launch<T, DK, 64>(q, k, v, gf, gb, d_out, dq, dk, dv, dgf, dgb, BH, L, heads_token_major, ws, only_marked, stream);
    }
    return hipErrorInvalidValue;
}

template <typename T>
hipError_t launch_dk(int dk_, int dv_, const void *q, const void *k, const void *v, const void *gf, const void *gb,
                     const void *d_out, void *dq, void *dk, void *dv, void *dgf, void *dgb, long BH, int L,
                     int heads_token_major, float *ws, const int *only_marked, hipStream_t stream)
{
    switch (dk_) {
        case 16: return launch_dv<T, 16>(dv_, q, k, v, gf, gb, d_out, dq, dk, dv, dgf, dgb, BH, L, heads_token_major, ws, only_marked, stream);
        case 32: return launch_dv<T, 32>(dv_, q, k, v, gf, gb, d_out, dq, dk, dv, dgf, dgb, BH, L, heads_token_major, ws, only_marked, stream);
        case 64: return launch_dv<T, 64>(dv_, q, k, v, gf, gb, d_out, dq, dk, dv, dgf, dgb, BH, L, heads_token_major, ws, only_marked, stream);
    }
    return hipErrorInvalidValue;
}

}  // namespace

size_t bigla_bwd_workspace_bytes(long BH, int L, int dk, int dv, bool is_bf16)
{
    const size_t exact = size_t(BH) * L * (size_t(3) * dk + dv) * sizeof(float);
    return exact + (bigla_bwd_chunk_supported(dk, dv, is_bf16) ? bigla_bwd_chunk_workspace_bytes(BH, L) : 0);
}

constexpr int kChunkwiseMinTokens = 32;

hipError_t bigla_bwd_launch(const void *q, const void *k, const void *v, const void *g_fwd, const void *g_bwd,
                            const void *d_out, void *dq, void *dk, void *dv, void *dg_fwd, void *dg_bwd, long BH, int L,
                            int dk_, int dv_, bool is_bf16, int heads_token_major, bool recurrent_only, void *workspace,
                            hipStream_t stream)
{
    LaunchTimer timer(kKernelBackward, stream);
    char *base = static_cast<char *>(workspace);
    const int *only_marked = nullptr;
    if (bigla_bwd_chunk_supported(dk_, dv_, is_bf16)) {
        // The chunkwise kernels take every slab whose gates they can carry and mark the others.  Sequences
        // shorter than half a chunk go to the exact kernels altogether: a slab of a few tokens has only a
        // handful of score entries, all of which can be small at once, and the bf16 rounding of the scaled
        // queries and keys (relative to the summands of those entries) is then large against the slab's own
        // gradients -- reproduced on the CPU from the operand roundings alone.
        if (!recurrent_only && L >= kChunkwiseMinTokens) {
            const hipError_t e = bigla_bwd_chunk_launch(q, k, v, g_fwd, g_bwd, d_out, dq, dk, dv, dg_fwd, dg_bwd, BH, L,
                                                        dk_, heads_token_major, base, stream);
            if (e != hipSuccess) return e;
            only_marked = bigla_bwd_chunk_marks(base, BH, L);
        }
        base += bigla_bwd_chunk_workspace_bytes(BH, L);
    }
    float *ws = reinterpret_cast<float *>(base);
    if (is_bf16)
        return launch_dk<bf16_t>(dk_, dv_, q, k, v, g_fwd, g_bwd, d_out, dq, dk, dv, dg_fwd, dg_bwd, BH, L,
                                 heads_token_major, ws, only_marked, stream);
    return launch_dk<float>(dk_, dv_, q, k, v, g_fwd, g_bwd, d_out, dq, dk, dv, dg_fwd, dg_bwd, BH, L,
                            heads_token_major, ws, only_marked, stream);
}

}  // namespace vig
