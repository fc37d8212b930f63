// Exact fp32 evaluation of the BiGLA recurrences (Section 4.2.1, Eq. (BiGLA)), token by token.
//
// This is the fp32 path of the library and the path for every head shape the chunkwise MFMA
// kernels do not cover.  One workgroup owns one (batch, head) slab and runs both directions in
// the same launch: a forward sweep that stores o_fwd as fp32, then a backward sweep that reads
// it back and writes (o_fwd + o_bwd)/2.  The dk x dv state lives in registers: thread
// (j, s) holds rows [s*DK/4, (s+1)*DK/4) of column j, so a token costs DK/4 fused
// decay-update-readout steps per thread plus a 4-lane reduction.  Tokens are staged through LDS
// 16 at a time with coalesced loads; alpha = exp(log-gate) is evaluated once per element there.
#include "vig_common.hpp"
#include "vig_kernels.hpp"
#include "vig_timing.hpp"

namespace vig {

namespace {

constexpr int kSplit = 4;   // threads sharing one state column
constexpr int kTile = 16;   // tokens staged per LDS tile

template <typename T, int DK, int DV>
__global__ __launch_bounds__(DV *kSplit) void bigla_recurrent_kernel(
    const T *__restrict__ q, const T *__restrict__ k, const T *__restrict__ v, const T *__restrict__ g_fwd,
    const T *__restrict__ g_bwd, T *out, float *o_fwd /* may alias out (fp32) */, int L,
    int heads_token_major /* 0: [B,H,L,d]; H: [B,L,H,d] */, bool o_fwd_in_out)
{
    constexpr int R = DK / kSplit;
    constexpr int NT = DV * kSplit;
    __shared__ float sq[kTile][DK], sk[kTile][DK], sa[kTile][DK], sv[kTile][DV];

    const int tid = threadIdx.x;
    const int j = tid / kSplit, s = tid % kSplit, c0 = s * R;
    const size_t slab = blockIdx.x;
    // first row of the slab and distance between its tokens, in rows of the tensor
    const size_t row0 = heads_token_major
                            ? (slab / heads_token_major) * size_t(L) * heads_token_major + slab % heads_token_major
                            : slab * size_t(L);
    const size_t step = heads_token_major ? heads_token_major : 1;
    q += row0 * DK;
    k += row0 * DK;
    g_fwd += row0 * DK;
    g_bwd += row0 * DK;
    v += row0 * DV;
    out += row0 * DV;
    // the fp32 side buffer is dense [slab][L][DV]; when the partial sums live in `out` they follow it
    o_fwd += (o_fwd_in_out ? row0 : slab * size_t(L)) * DV;
    const size_t fwd_step = o_fwd_in_out ? step : 1;

    float S[R];

    for (int dir = 0; dir < 2; ++dir) {
        const T *g = dir == 0 ? g_fwd : g_bwd;
#pragma unroll
        for (int r = 0; r < R; ++r) S[r] = 0.f;
        const int ntiles = (L + kTile - 1) / kTile;
        for (int it = 0; it < ntiles; ++it) {
            const int tile = dir == 0 ? it : ntiles - 1 - it;
            const int t0 = tile * kTile;
            const int n = min(kTile, L - t0);
            __syncthreads();
            for (int e = tid; e < n * DK; e += NT) {
                const int tt = e / DK, c = e % DK;
                const size_t off = size_t(t0 + tt) * step * DK + c;
                sq[tt][c] = io<T>::load(q + off);
                sk[tt][c] = io<T>::load(k + off);
                sa[tt][c] = expf(io<T>::load(g + off));
            }
            for (int e = tid; e < n * DV; e += NT) {
                const int tt = e / DV, c = e % DV;
                sv[tt][c] = io<T>::load(v + size_t(t0 + tt) * step * DV + c);
            }
            __syncthreads();
            for (int i = 0; i < n; ++i) {
                const int tt = dir == 0 ? i : n - 1 - i;
                const float vj = sv[tt][j];
                float acc = 0.f;
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    // S_t = diag(alpha_t) S_{t -/+ 1} + k_t^T v_t ;  o_t = q_t S_t
                    S[r] = fmaf(sa[tt][c0 + r], S[r], sk[tt][c0 + r] * vj);
                    acc = fmaf(sq[tt][c0 + r], S[r], acc);
                }
                acc += __shfl_xor(acc, 1);
                acc += __shfl_xor(acc, 2);
                if (s == 0) {
                    const size_t o = size_t(t0 + tt) * step * DV + j, of = size_t(t0 + tt) * fwd_step * DV + j;
                    if (dir == 0)
                        o_fwd[of] = acc;
                    else
                        io<T>::store(out + o, 0.5f * (o_fwd[of] + acc));
                }
            }
        }
    }
}

template <typename T, int DK, int DV>
hipError_t launch(const void *q, const void *k, const void *v, const void *gf, const void *gb, void *out,
                  float *o_fwd, int BH, int L, int heads_token_major, hipStream_t stream)
{
    LaunchTimer timer(kKernelRecurrent, stream);
    hipLaunchKernelGGL((bigla_recurrent_kernel<T, DK, DV>), dim3(BH), dim3(DV * kSplit), 0, stream,
                       static_cast<const T *>(q), static_cast<const T *>(k), static_cast<const T *>(v),
                       static_cast<const T *>(gf), static_cast<const T *>(gb), static_cast<T *>(out), o_fwd, L,
                       heads_token_major, static_cast<void *>(o_fwd) == out);
    return hipGetLastError();
}

template <typename T, int DK>
hipError_t launch_dv(int dv, const void *q, const void *k, const void *v, const void *gf, const void *gb,
                     void *out, float *o_fwd, int BH, int L, int heads_token_major, hipStream_t stream)
{
    switch (dv) {
        case 16: return launch<T, DK, 16>(q, k, v, gf, gb, out, o_fwd, BH, L, heads_token_major, stream);
        case 32: return launch<T, DK, 32>(q, k, v, gf, gb, out, o_fwd, BH, L, heads_token_major, stream);
        case 64: return launch<T, DK, 64>(q, k, v, gf, gb, out, o_fwd, BH, L, heads_token_major, stream);
    }
    return hipErrorInvalidValue;
}

template <typename T>
hipError_t launch_dk(int dk, int dv, const void *q, const void *k, const void *v, const void *gf,
                     const void *gb, void *out, float *o_fwd, int BH, int L, int heads_token_major, hipStream_t stream)
{
    switch (dk) {
        case 16: return launch_dv<T, 16>(dv, q, k, v, gf, gb, out, o_fwd, BH, L, heads_token_major, stream);
        case 32: return launch_dv<T, 32>(dv, q, k, v, gf, gb, out, o_fwd, BH, L, heads_token_major, stream);
        case 64: return launch_dv<T, 64>(dv, q, k, v, gf, gb, out, o_fwd, BH, L, heads_token_major, stream);
    }
    return hipErrorInvalidValue;
}

}  // namespace

size_t bigla_recurrent_workspace_bytes(long BH, int L, int dv, bool is_bf16)
{
    // fp32 runs keep o_fwd in `out` itself; bf16 runs need an fp32 side buffer
    return is_bf16 ? size_t(BH) * L * dv * sizeof(float) : 0;
}

hipError_t bigla_recurrent_launch(const void *q, const void *k, const void *v, const void *g_fwd,
                                  const void *g_bwd, void *out, long BH, int L, int dk, int dv, bool is_bf16,
                                  int heads_token_major, void *workspace, hipStream_t stream)
{
    if (is_bf16)
        return launch_dk<bf16_t>(dk, dv, q, k, v, g_fwd, g_bwd, out, static_cast<float *>(workspace), int(BH), L,
                                 heads_token_major, stream);
    return launch_dk<float>(dk, dv, q, k, v, g_fwd, g_bwd, out, static_cast<float *>(out), int(BH), L,
                            heads_token_major, stream);
}

}  // namespace vig
