// Direction-wise forget gates of BiGLA (Section 3: low-rank gate with temperature tau; Eq. (BiGLA),
// Section 4.2.1, lines 1-2: one gate vector of width 2*dk per token, split into a forward and a
// backward half), written as the LOG gates bigla_fwd takes:
//     z_t = (x_t W1) W2 + b            in R^{2*H*dk}
//     g   = log(sigmoid(z)^(1/tau)) = log(sigmoid(z)) / tau
// entries [0, H*dk) of z are the forward gates, [H*dk, 2*H*dk) the backward gates; inside each
// half head h owns entries [h*dk, (h+1)*dk).
//
// Weights arrive in the "out-features major" form a linear layer stores them in, w1 [16, D] and
// w2 [2*H*dk, 16]: exactly the operand layouts the matrix cores want, so nothing is staged or
// transposed.  The step is bound by its HBM traffic (D values read, 2*H*dk written per token)
// and by two transcendentals per output.
//
// bf16: one wave per 16 tokens.
//   GEMM 1  H1^T[rank][token] = w1[rank][:] . x[token][:]   v_mfma_f32_16x16x32_bf16, K = D
//           A = w1 rows (lane: rank l%16, 8 consecutive inputs), B = x rows (lane: token l%16,
//           the same 8 inputs); the accumulator leaves lane (token l%16, ranks 4g..4g+3)
//   GEMM 2  Z^T[channel][token] = w2[channel][:] . H1^T[:][token]   v_mfma_f32_16x16x16_bf16, K = 16
//           B is the bf16 copy of GEMM 1's accumulator as it stands (lane: token l%16, ranks
//           4g..4g+3), A = w2 rows (lane: one channel, ranks 4g..4g+3); the result leaves lane
//           (token l%16, the channels of A rows 4g..4g+3).  The A rows of four consecutive tiles
//           are chosen so that the lane ends up with 16 consecutive channels: whole-row stores.
// fp32: plain fp32 FMAs, one workgroup per 16 tokens (low-rank products through LDS).
#include "vig_common.hpp"
#include "vig_kernels.hpp"
#include "vig_timing.hpp"

namespace vig {

namespace {

constexpr int kRank = 16;  // width of the low-rank bottleneck (Section 3)
constexpr int kThreads = 256;
constexpr int kTokensPerWave = 16;
constexpr int kPersistentBlocks = 768;  // three workgroups per CU walk the token tiles


// Copy w2 ([width][16] bf16, 2 x 16 bytes per row) and the bias into LDS, eight loads in flight per
// thread and batch (a load-store-load-store loop would pay one memory round trip per 16 bytes).
__device__ __forceinline__ void stage_weights(const uint16_t *w2, const uint16_t *bias, uint16_t *s_w2,
                                              uint16_t *s_bias, int width)
{
    const uint4 *src = reinterpret_cast<const uint4 *>(w2);
    uint4 *dst = reinterpret_cast<uint4 *>(s_w2);
    const int n = width * 2;
    for (int i0 = threadIdx.x; i0 < n; i0 += 8 * kThreads) {
        uint4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = src[min(i0 + u * kThreads, n - 1)];
#pragma unroll
        for (int u = 0; u < 8; ++u)
            if (i0 + u * kThreads < n) dst[i0 + u * kThreads] = v[u];
    }
    for (int i = threadIdx.x; i < width / 8; i += kThreads)
        reinterpret_cast<uint4 *>(s_bias)[i] = bias ? reinterpret_cast<const uint4 *>(bias)[i] : make_uint4(0u, 0u, 0u, 0u);
}

// Persistent workgroups: w2 and the bias are copied into LDS once (rows of 32 bytes, read back 8
// bytes per lane, so that the loop over channel tiles waits on LDS, not on global memory), each
// wave keeps its A operands of GEMM 1 (all of w1) in registers, and then walks token tiles with a
// grid stride.  The x rows of a wave's NEXT tile are requested as soon as GEMM 1 has consumed the
// current ones, so they travel during the long channel loop.
// kSteps = D / 32 (every load of the low-rank product is unrolled); kLdsW2 = false reads w2 and
// the bias from global memory (when they do not fit the LDS budget).
template <int kSteps, bool kLdsW2>
__global__ __launch_bounds__(kThreads) void gate_producer_bf16_kernel(
    const uint16_t *__restrict__ x, const uint16_t *__restrict__ w1, const uint16_t *__restrict__ w2,
    const uint16_t *__restrict__ bias, uint16_t *__restrict__ g_fwd, uint16_t *__restrict__ g_bwd, long tokens,
    int H, int L, int D, int dk, float inv_tau, int token_major)
{
    extern __shared__ __align__(16) unsigned char dyn_lds[];
    const int width = 2 * H * dk, half = H * dk;
    uint16_t *s_w2 = reinterpret_cast<uint16_t *>(dyn_lds);       // [width][16]
    uint16_t *s_bias = s_w2 + size_t(width) * kRank;              // [width] (zeros when there is no bias)
    const int lane = threadIdx.x & 63, r = lane & 15, g = lane >> 4;
    const long n_tiles = (tokens + kTokensPerWave - 1) / kTokensPerWave;
    const long tile_step = long(gridDim.x) * (kThreads / 64);
    long tile = long(blockIdx.x) * (kThreads / 64) + (threadIdx.x >> 6);

    // lane (r, g): A operand = w1 row r (rank), B operand = x row of token r; 16 bytes at 32kk + 8g
    auto x_row = [&](long t) {
        const long tok = t * kTokensPerWave + r;
        return reinterpret_cast<const uint4 *>(x + size_t(tok < tokens ? tok : tokens - 1) * D) + g;
    };
    uint4 wa[kSteps], xa[kSteps];
    {
        const uint4 *wrow = reinterpret_cast<const uint4 *>(w1 + size_t(r) * D) + g;
        const uint4 *xrow = x_row(tile < n_tiles ? tile : n_tiles - 1);
#pragma unroll
        for (int kk = 0; kk < kSteps; ++kk) {
            xa[kk] = xrow[4 * kk];
            wa[kk] = wrow[4 * kk];
        }
    }
    if (kLdsW2) {
        stage_weights(w2, bias, s_w2, s_bias, width);
        __syncthreads();
    }
    const uint16_t *w2src = kLdsW2 ? s_w2 : w2;
    const uint16_t *bsrc = kLdsW2 ? s_bias : bias;
    const int dk_shift = dk == 64 ? 6 : (dk == 32 ? 5 : 4);
    const int arow = 16 * (r >> 2) + (r & 3);  // channel of this lane's A row inside a group, tile 0

    for (; tile < n_tiles; tile += tile_step) {
        // ---- GEMM 1: H1^T = w1 . x^T, two accumulators so that consecutive MFMAs do not wait on each other
        f32x4 acc[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
#pragma unroll
        for (int kk = 0; kk < kSteps; ++kk)
            acc[kk & 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, wa[kk]),
                                                                  __builtin_bit_cast(bf16x8, xa[kk]), acc[kk & 1], 0, 0, 0);
        // lane (token r, ranks 4g..4g+3) -> bf16 B operand of the K = 16 MFMA
        const uint2 hb = make_uint2(pack2(acc[0][0] + acc[1][0], acc[0][1] + acc[1][1]),
                                    pack2(acc[0][2] + acc[1][2], acc[0][3] + acc[1][3]));
        const s16x4 hop = __builtin_bit_cast(s16x4, hb);
        {  // the next tile's rows (clamped past the end: loaded, never used)
            const long next = tile + tile_step;
            const uint4 *xrow = x_row(next < n_tiles ? next : n_tiles - 1);
#pragma unroll
            for (int kk = 0; kk < kSteps; ++kk) xa[kk] = xrow[4 * kk];
        }

        // ---- GEMM 2 in groups of 64 channels (four MFMA tiles), then bias, log-sigmoid, 1/tau, store.
        // Row 4g'+e of tile i of a group is given channel 16g' + 4i + e, so that after the four tiles
        // lane (r, g) holds the 16 CONSECUTIVE channels 16g .. 16g+15 of its token: 32 contiguous
        // bytes per lane, whole 128-byte rows per store instruction.  Those 16 channels lie inside
        // one head of one direction (dk is 16, 32 or 64: shifts, no division).
        const long tok = tile * kTokensPerWave + r;
        const long tok_c = tok < tokens ? tok : tokens - 1;
        const long b_idx = tok_c / L;
        const int t_idx = int(tok_c % L);
        for (int cb = 0; cb < width; cb += 64) {
            const int c = min(cb + 16 * g, width - 16);  // first of this lane's 16 channels (a ragged last group: unused)
            // the bias enters as the accumulator's initial value: element e of tile i is channel c + 4i + e
            f32x4 z[4];
            if (bsrc) {
                const uint4 b0 = *reinterpret_cast<const uint4 *>(bsrc + c), b1 = *reinterpret_cast<const uint4 *>(bsrc + c + 8);
                const uint32_t raw[8] = {b0.x, b0.y, b0.z, b0.w, b1.x, b1.y, b1.z, b1.w};
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    z[i] = f32x4{bf16_lo_to_f32(raw[2 * i]), bf16_hi_to_f32(raw[2 * i]), bf16_lo_to_f32(raw[2 * i + 1]),
                                 bf16_hi_to_f32(raw[2 * i + 1])};
            } else {
#pragma unroll
                for (int i = 0; i < 4; ++i) z[i] = f32x4{0.f, 0.f, 0.f, 0.f};
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int ch = min(cb + arow + 4 * i, width - 1);  // a ragged last group repeats a row, unused
                const uint2 a2 = *reinterpret_cast<const uint2 *>(w2src + size_t(ch) * kRank + 4 * g);
                z[i] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(s16x4, a2), hop, z[i], 0, 0, 0);
            }
            if (cb + 16 * g >= width) continue;
            uint32_t packed[8];
#pragma unroll
            for (int i = 0; i < 4; ++i) {  // channel c + 4i + e
                const float o0 = log_sigmoid(z[i][0]) * inv_tau, o1 = log_sigmoid(z[i][1]) * inv_tau;
                const float o2 = log_sigmoid(z[i][2]) * inv_tau, o3 = log_sigmoid(z[i][3]) * inv_tau;
                packed[2 * i] = pack2(o0, o1);
                packed[2 * i + 1] = pack2(o2, o3);
            }
            if (tok < tokens) {
                const bool bwd = c >= half;
                const int cc = bwd ? c - half : c;
                const int h = cc >> dk_shift, j = cc & (dk - 1);
                const size_t row = token_major ? (size_t(b_idx) * L + t_idx) * H + h : (size_t(b_idx) * H + h) * L + t_idx;
                uint4 *dst = reinterpret_cast<uint4 *>((bwd ? g_bwd : g_fwd) + row * dk + j);
                // streaming stores (nothing here reads the gates back): measured 2 us faster
                __builtin_nontemporal_store(u32x4{packed[0], packed[1], packed[2], packed[3]},
                                            reinterpret_cast<u32x4 *>(dst));
                __builtin_nontemporal_store(u32x4{packed[4], packed[5], packed[6], packed[7]},
                                            reinterpret_cast<u32x4 *>(dst) + 1);
            }
        }
    }
}

// The low-rank half alone, for the token mixer's state pass when it makes the gates itself: GEMM 1 exactly as
// above (same operands, same order of accumulation), the bf16 B operand of GEMM 2 written out instead of used:
// lowrank[token][16], 32 bytes per token.  One wave per 16 tokens.
template <int kSteps>
__global__ __launch_bounds__(kThreads) void gate_lowrank_bf16_kernel(const uint16_t *__restrict__ x,
                                                                     const uint16_t *__restrict__ w1,
                                                                     uint16_t *__restrict__ lowrank, long tokens, int D)
{
    const int lane = threadIdx.x & 63, r = lane & 15, g = lane >> 4;
    const long tile = long(blockIdx.x) * (kThreads / 64) + (threadIdx.x >> 6);
    const long tok = tile * kTokensPerWave + r;
    if (tile * kTokensPerWave >= tokens) return;
    const uint4 *wrow = reinterpret_cast<const uint4 *>(w1 + size_t(r) * D) + g;
    const uint4 *xrow = reinterpret_cast<const uint4 *>(x + size_t(tok < tokens ? tok : tokens - 1) * D) + g;
    uint4 wa[kSteps], xa[kSteps];
#pragma unroll
    for (int kk = 0; kk < kSteps; ++kk) {
        xa[kk] = xrow[4 * kk];
        wa[kk] = wrow[4 * kk];
    }
    f32x4 acc[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
#pragma unroll
    for (int kk = 0; kk < kSteps; ++kk)
        acc[kk & 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, wa[kk]),
                                                              __builtin_bit_cast(bf16x8, xa[kk]), acc[kk & 1], 0, 0, 0);
    const uint2 hb = make_uint2(pack2(acc[0][0] + acc[1][0], acc[0][1] + acc[1][1]),
                                pack2(acc[0][2] + acc[1][2], acc[0][3] + acc[1][3]));
    if (tok < tokens) *reinterpret_cast<uint2 *>(lowrank + size_t(tok) * kRank + 4 * g) = hb;
}

// fp32: one workgroup per 16 tokens; thread (t, rank) forms the low-rank product, then the threads
// sweep the gate channels.
__global__ __launch_bounds__(kThreads) void gate_producer_f32_kernel(
    const float *__restrict__ x, const float *__restrict__ w1, const float *__restrict__ w2,
    const float *__restrict__ bias, float *__restrict__ g_fwd, float *__restrict__ g_bwd, long tokens, int H, int L,
    int D, int dk, float inv_tau, int token_major)
{
    __shared__ float low[kTokensPerWave][kRank];
    const long tok0 = long(blockIdx.x) * kTokensPerWave;
    {
        const int t = threadIdx.x / kRank, rk = threadIdx.x % kRank;
        const long tok = tok0 + t;
        float acc = 0.f;
        if (tok < tokens) {
            const float *xr = x + size_t(tok) * D, *wr = w1 + size_t(rk) * D;
            for (int i = 0; i < D; ++i) acc = fmaf(xr[i], wr[i], acc);
        }
        low[t][rk] = acc;
    }
    __syncthreads();
    const int width = 2 * H * dk, half = H * dk;
    for (int c = threadIdx.x; c < width; c += kThreads) {
        float wv[kRank];
#pragma unroll
        for (int rk = 0; rk < kRank; ++rk) wv[rk] = w2[size_t(c) * kRank + rk];
        const float bc = bias ? bias[c] : 0.f;
        float *gbase = c < half ? g_fwd : g_bwd;
        const int cc = c < half ? c : c - half;
        const int h = cc / dk, j = cc % dk;
        for (int t = 0; t < kTokensPerWave; ++t) {
            const long tok = tok0 + t;
            if (tok >= tokens) break;
            float z = bc;
#pragma unroll
            for (int rk = 0; rk < kRank; ++rk) z = fmaf(low[t][rk], wv[rk], z);
            const long b = tok / L;
            const int tt = int(tok % L);
            const size_t row = token_major ? (size_t(b) * L + tt) * H + h : (size_t(b) * H + h) * L + tt;
            // accurate logf/expf here: the fp32 path is held to 1e-4 and is not a benchmark line
            gbase[row * dk + j] = (fminf(z, 0.f) - log1pf(expf(-fabsf(z)))) * inv_tau;
        }
    }
}

}  // namespace

bool gate_producer_width_ok(int D, bool is_bf16)
{
    if (D <= 0 || D % 32 != 0) return false;
    if (!is_bf16) return true;
    switch (D / 32) {  // the unrolled instantiations of the bf16 kernel
        case 1: case 2: case 3: case 4: case 5: case 6: case 7: case 8: case 10: case 12: case 16: case 18: case 20:
        case 24: case 32: return true;
    }
    return false;
}

hipError_t gate_producer_launch(const void *x, const void *w1, const void *w2, const void *bias, void *g_fwd,
                                void *g_bwd, int B, int H, int L, int D, int dk, float tau, bool is_bf16,
                                int token_major, hipStream_t stream)
{
    const long tokens = long(B) * L;
    const float inv_tau = 1.f / tau;
    LaunchTimer timer(kKernelGateProducer, stream);
    if (is_bf16) {
        const long tiles = (tokens + kTokensPerWave - 1) / kTokensPerWave;
        long blocks = (tiles + kThreads / 64 - 1) / (kThreads / 64);
        if (blocks > kPersistentBlocks) blocks = kPersistentBlocks;
        const size_t w2_bytes = size_t(2) * H * dk * (kRank + 1) * sizeof(uint16_t);  // w2 and the bias
        const bool lds = w2_bytes <= 52 * 1024;
#define VIG_GP_LAUNCH(KS, LDS)                                                                                     \
    hipLaunchKernelGGL((gate_producer_bf16_kernel<KS, LDS>), dim3((unsigned)blocks), dim3(kThreads),               \
                       (LDS) ? w2_bytes : 0, stream, static_cast<const uint16_t *>(x),                            \
                       static_cast<const uint16_t *>(w1), static_cast<const uint16_t *>(w2),                      \
                       static_cast<const uint16_t *>(bias), static_cast<uint16_t *>(g_fwd),                       \
                       static_cast<uint16_t *>(g_bwd), tokens, H, L, D, dk, inv_tau, token_major)
#define VIG_GP_CASE(KS)                                                                                            \
    case KS:                                                                                                       \
        if (lds)                                                                                                   \
            VIG_GP_LAUNCH(KS, true);                                                                               \
        else                                                                                                       \
            VIG_GP_LAUNCH(KS, false);                                                                              \
        break
        switch (D / 32) {  // model widths 32 .. 1024 in steps of 32 up to 256, then the common larger ones
            VIG_GP_CASE(1); VIG_GP_CASE(2); VIG_GP_CASE(3); VIG_GP_CASE(4); VIG_GP_CASE(5); VIG_GP_CASE(6);
            VIG_GP_CASE(7); VIG_GP_CASE(8); VIG_GP_CASE(10); VIG_GP_CASE(12); VIG_GP_CASE(16); VIG_GP_CASE(18);
            VIG_GP_CASE(20); VIG_GP_CASE(24); VIG_GP_CASE(32);
            default: return hipErrorInvalidValue;
        }
#undef VIG_GP_CASE
#undef VIG_GP_LAUNCH
    } else {
        const long blocks = (tokens + kTokensPerWave - 1) / kTokensPerWave;
        if (blocks > 0x7fffffffL) return hipErrorInvalidValue;
        hipLaunchKernelGGL(gate_producer_f32_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, stream,
                           static_cast<const float *>(x), static_cast<const float *>(w1),
                           static_cast<const float *>(w2), static_cast<const float *>(bias),
                           static_cast<float *>(g_fwd), static_cast<float *>(g_bwd), tokens, H, L, D, dk, inv_tau,
                           token_major);
    }
    return hipGetLastError();
}

hipError_t gate_lowrank_launch(const void *x, const void *w1, void *lowrank, int B, int L, int D, hipStream_t stream)
{
    const long tokens = long(B) * L;
    const long tiles = (tokens + kTokensPerWave - 1) / kTokensPerWave;
    const long blocks = (tiles + kThreads / 64 - 1) / (kThreads / 64);
    if (blocks > 0x7fffffffL) return hipErrorInvalidValue;
    LaunchTimer timer(kKernelGateLowrank, stream);
#define VIG_LR_CASE(KS)                                                                                            \
    case KS:                                                                                                       \
        hipLaunchKernelGGL((gate_lowrank_bf16_kernel<KS>), dim3((unsigned)blocks), dim3(kThreads), 0, stream,      \
                           static_cast<const uint16_t *>(x), static_cast<const uint16_t *>(w1),                    \
                           static_cast<uint16_t *>(lowrank), tokens, D);                                           \
        break
    switch (D / 32) {
        VIG_LR_CASE(1); VIG_LR_CASE(2); VIG_LR_CASE(3); VIG_LR_CASE(4); VIG_LR_CASE(5); VIG_LR_CASE(6);
        VIG_LR_CASE(7); VIG_LR_CASE(8); VIG_LR_CASE(10); VIG_LR_CASE(12); VIG_LR_CASE(16); VIG_LR_CASE(18);
        VIG_LR_CASE(20); VIG_LR_CASE(24); VIG_LR_CASE(32);
        default: return hipErrorInvalidValue;
    }
#undef VIG_LR_CASE
    return hipGetLastError();
}

}  // namespace vig
