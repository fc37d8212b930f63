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
//           4g..4g+3), A = w2 rows (lane: channel l%16 of the tile, ranks 4g..4g+3); the result
//           leaves lane (token l%16, channels 4g..4g+3 of the tile): 8 bytes per lane to store.
// fp32: plain fp32 FMAs, one workgroup per 16 tokens (low-rank products through LDS).
#include "vig_common.hpp"
#include "vig_kernels.hpp"
#include "vig_timing.hpp"

namespace vig {

namespace {

constexpr int kRank = 16;  // width of the low-rank bottleneck (Section 3)
constexpr int kThreads = 256;
constexpr int kTokensPerWave = 16;

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;

// log(sigmoid(z)) = min(z, 0) - log(1 + exp(-|z|)), finite for every finite z
__device__ __forceinline__ float log_sigmoid(float z)
{
    return fminf(z, 0.f) - __logf(1.f + __expf(-fabsf(z)));
}

__device__ __forceinline__ uint32_t pack2(float lo, float hi)
{
    f32x2 a = {lo, hi};
    bf16x2 b = __builtin_convertvector(a, bf16x2);  // v_cvt_pk_bf16_f32, round to nearest even
    return __builtin_bit_cast(uint32_t, b);
}

template <int kDummy = 0>
__global__ __launch_bounds__(kThreads) void gate_producer_bf16_kernel(
    const uint16_t *__restrict__ x, const uint16_t *__restrict__ w1, const uint16_t *__restrict__ w2,
    const uint16_t *__restrict__ bias, uint16_t *__restrict__ g_fwd, uint16_t *__restrict__ g_bwd, long tokens,
    int H, int L, int D, int dk, float inv_tau, int token_major)
{
    const int lane = threadIdx.x & 63, r = lane & 15, g = lane >> 4;
    const long tile = long(blockIdx.x) * (kThreads / 64) + (threadIdx.x >> 6);
    const long tok0 = tile * kTokensPerWave;
    if (tok0 >= tokens) return;  // whole wave
    const long tok = tok0 + r;
    const long tok_c = tok < tokens ? tok : tokens - 1;  // rows past the end repeat the last one, not stored

    // ---- GEMM 1: H1^T = w1 . x^T, two accumulators so that consecutive MFMAs do not wait on each other
    f32x4 acc[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
    const uint4 *xrow = reinterpret_cast<const uint4 *>(x + size_t(tok_c) * D) + g;
    const uint4 *wrow = reinterpret_cast<const uint4 *>(w1 + size_t(r) * D) + g;
    const int ksteps = D / 32;
#pragma unroll 4
    for (int kk = 0; kk < ksteps; ++kk) {
        const bf16x8 a = __builtin_bit_cast(bf16x8, wrow[4 * kk]);
        const bf16x8 b = __builtin_bit_cast(bf16x8, xrow[4 * kk]);
        acc[kk & 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc[kk & 1], 0, 0, 0);
    }
    // lane (token r, ranks 4g..4g+3) -> bf16 B operand of the K = 16 MFMA
    const uint2 hb = make_uint2(pack2(acc[0][0] + acc[1][0], acc[0][1] + acc[1][1]),
                                pack2(acc[0][2] + acc[1][2], acc[0][3] + acc[1][3]));
    const s16x4 hop = __builtin_bit_cast(s16x4, hb);

    // ---- GEMM 2 per 16-channel tile, then bias, log-sigmoid, 1/tau, store
    const int width = 2 * H * dk, half = H * dk;
    const long b_idx = tok_c / L;
    const int t_idx = int(tok_c % L);
    for (int c0 = 0; c0 < width; c0 += 16) {
        const uint2 wa = *reinterpret_cast<const uint2 *>(w2 + size_t(c0 + r) * kRank + 4 * g);
        f32x4 z = {0.f, 0.f, 0.f, 0.f};
        z = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(s16x4, wa), hop, z, 0, 0, 0);
        float bv[4] = {0.f, 0.f, 0.f, 0.f};
        if (bias) {
            const uint2 braw = *reinterpret_cast<const uint2 *>(bias + c0 + 4 * g);
            bv[0] = bf16_lo_to_f32(braw.x); bv[1] = bf16_hi_to_f32(braw.x);
            bv[2] = bf16_lo_to_f32(braw.y); bv[3] = bf16_hi_to_f32(braw.y);
        }
        float o[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] = log_sigmoid(z[e] + bv[e]) * inv_tau;
        if (tok < tokens) {
            // a 16-channel tile lies inside one head of one direction (dk is a multiple of 16)
            uint16_t *gbase = c0 < half ? g_fwd : g_bwd;
            const int cc = (c0 < half ? c0 : c0 - half) + 4 * g;
            const int h = cc / dk, j = cc % dk;
            const size_t row = token_major ? (size_t(b_idx) * L + t_idx) * H + h : (size_t(b_idx) * H + h) * L + t_idx;
            *reinterpret_cast<uint2 *>(gbase + row * dk + j) = make_uint2(pack2(o[0], o[1]), pack2(o[2], o[3]));
        }
    }
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

hipError_t gate_producer_launch(const void *x, const void *w1, const void *w2, const void *bias, void *g_fwd,
                                void *g_bwd, int B, int H, int L, int D, int dk, float tau, bool is_bf16,
                                int token_major, hipStream_t stream)
{
    const long tokens = long(B) * L;
    const float inv_tau = 1.f / tau;
    LaunchTimer timer(kKernelGateProducer, stream);
    if (is_bf16) {
        const long tiles = (tokens + kTokensPerWave - 1) / kTokensPerWave;
        const long blocks = (tiles + kThreads / 64 - 1) / (kThreads / 64);
        if (blocks > 0x7fffffffL) return hipErrorInvalidValue;
        hipLaunchKernelGGL(gate_producer_bf16_kernel<0>, dim3((unsigned)blocks), dim3(kThreads), 0, stream,
                           static_cast<const uint16_t *>(x), static_cast<const uint16_t *>(w1),
                           static_cast<const uint16_t *>(w2), static_cast<const uint16_t *>(bias),
                           static_cast<uint16_t *>(g_fwd), static_cast<uint16_t *>(g_bwd), tokens, H, L, D, dk,
                           inv_tau, token_major);
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

}  // namespace vig
