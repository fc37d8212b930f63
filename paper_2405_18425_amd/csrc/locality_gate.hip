// 2D gating locality injection (Section 4.2.2): depthwise 3x3 convolution on the patch grid
// blended with the global branch through a sigmoid gate,
//     out = sigmoid(z) * DWConv3x3(x) + (1 - sigmoid(z)) * o_global .
//
// The step is pure bandwidth (about 25 flops per element against 4 element transfers), so the
// kernel is organised around memory: a thread owns 4 consecutive channels of one grid column and
// walks down a strip of rows keeping a 3x3 window of fp32 values in registers, so that each
// input row costs three vector loads (left, centre, right neighbour -- two of them come from
// cache lines the neighbouring threads fetch anyway) instead of nine.  Consecutive
// threads cover consecutive channel groups and then consecutive columns, i.e. one contiguous
// row of the [.., y, x, channel] tensor per wavefront load.  Arithmetic is fp32 on either dtype.
#include "vig_common.hpp"
#include "vig_kernels.hpp"
#include "vig_timing.hpp"

namespace vig {

namespace {

// A thread's slice of one pixel: 4 consecutive channels (8 bytes of bf16, 16 bytes of fp32),
// widened to fp32 lanes.  Four channels keep the 3x3 window plus the 36 filter taps near 100
// registers, i.e. 4-5 resident waves per SIMD to cover HBM latency.
template <typename T>
struct vec4;

template <>
struct vec4<float> {
    static constexpr int N = 4;
    typedef float4 raw_t;
    static __device__ __forceinline__ raw_t zero() { return make_float4(0.f, 0.f, 0.f, 0.f); }
    static __device__ __forceinline__ void widen(const raw_t &r, float (&f)[N])
    {
        f[0] = r.x; f[1] = r.y; f[2] = r.z; f[3] = r.w;
    }
    static __device__ __forceinline__ void load(const float *p, float (&f)[N])
    {
        const float4 r = *reinterpret_cast<const float4 *>(p);
        f[0] = r.x; f[1] = r.y; f[2] = r.z; f[3] = r.w;
    }
    static __device__ __forceinline__ void store(float *p, const float (&f)[N])
    {
        *reinterpret_cast<float4 *>(p) = make_float4(f[0], f[1], f[2], f[3]);
    }
};

template <>
struct vec4<bf16_t> {
    static constexpr int N = 4;
    typedef uint2 raw_t;
    static __device__ __forceinline__ raw_t zero() { return make_uint2(0u, 0u); }
    static __device__ __forceinline__ void widen(const raw_t &r, float (&f)[N])
    {
        f[0] = bf16_lo_to_f32(r.x); f[1] = bf16_hi_to_f32(r.x);
        f[2] = bf16_lo_to_f32(r.y); f[3] = bf16_hi_to_f32(r.y);
    }
    static __device__ __forceinline__ void load(const bf16_t *p, float (&f)[N])
    {
        const uint2 r = *reinterpret_cast<const uint2 *>(p);
        f[0] = bf16_lo_to_f32(r.x); f[1] = bf16_hi_to_f32(r.x);
        f[2] = bf16_lo_to_f32(r.y); f[3] = bf16_hi_to_f32(r.y);
    }
    static __device__ __forceinline__ void store(bf16_t *p, const float (&f)[N])
    {
        *reinterpret_cast<uint2 *>(p) = make_uint2(pack_bf16x2(f[0], f[1]), pack_bf16x2(f[2], f[3]));
    }
};

constexpr int kThreads = 256;

template <typename T, int DV, int RS, bool kTm /* [B,L,H,dv] instead of [B,H,L,dv] */>
__global__ __launch_bounds__(kThreads) void locality_gate_kernel(
    const T *__restrict__ x, const T *__restrict__ w, const T *__restrict__ bias, const T *__restrict__ z,
    const T *__restrict__ og, T *__restrict__ out, int H, int Hg, int Wg, int n_strips, long total_threads)
{
    using V = vec4<T>;
    using raw_t = typename V::raw_t;
    constexpr int N = V::N;
    constexpr int CG = DV / N;

    const long gid = long(blockIdx.x) * kThreads + threadIdx.x;
    if (gid >= total_threads) return;
    const int cg = int(gid % CG);
    long rest = gid / CG;
    const int xp = int(rest % Wg);
    rest /= Wg;
    const int strip = int(rest % n_strips);
    const long slab = rest / n_strips;
    const int h = int(slab % H);
    const int c0 = h * DV + cg * N;
    // first pixel of the slab and distance between pixels, in rows of DV channels
    const size_t row0 = kTm ? size_t(slab / H) * Hg * Wg * H + h : size_t(slab) * Hg * Wg;
    const size_t px = kTm ? size_t(H) * DV : size_t(DV);
    const size_t slab_off = row0 * DV + size_t(cg) * N;
    const int y0 = strip * RS;

    // ---- every load of the strip is issued before any arithmetic: (RS+2)*3 input vectors (rows
    // y0-1 .. y0+RS, columns xp-1 .. xp+1; out-of-grid taps are zero), 2*RS gate/global vectors
    // and the 9 tap vectors, so that one wave keeps several hundred bytes per lane in flight ----
    raw_t xr[RS + 2][3], zr[RS], gr[RS], wr[9];
#pragma unroll
    for (int i = 0; i < RS + 2; ++i) {
        const int yy = y0 - 1 + i;
#pragma unroll
        for (int kx = 0; kx < 3; ++kx) {
            const int xx = xp + kx - 1;
            const bool in = yy >= 0 && yy < Hg && xx >= 0 && xx < Wg;
            xr[i][kx] = in ? *reinterpret_cast<const raw_t *>(x + slab_off + (size_t(yy) * Wg + xx) * px) : V::zero();
        }
    }
#pragma unroll
    for (int i = 0; i < RS; ++i) {
        const bool in = y0 + i < Hg;
        const size_t o = slab_off + (size_t(y0 + i) * Wg + xp) * px;
        zr[i] = in ? *reinterpret_cast<const raw_t *>(z + o) : V::zero();
        gr[i] = in ? *reinterpret_cast<const raw_t *>(og + o) : V::zero();
    }
#pragma unroll
    for (int i = 0; i < 9; ++i) wr[i] = *reinterpret_cast<const raw_t *>(w + size_t(c0) * 9 + i * N);

    // filter taps and bias of this thread's N channels, fp32: the 9*N taps are contiguous in w
    float wt[N][9], b[N];
    {
        float flat[9 * N];
#pragma unroll
        for (int i = 0; i < 9; ++i) {
            float piece[N];
            V::widen(wr[i], piece);
#pragma unroll
            for (int e = 0; e < N; ++e) flat[i * N + e] = piece[e];
        }
#pragma unroll
        for (int e = 0; e < N; ++e)
#pragma unroll
            for (int tap = 0; tap < 9; ++tap) wt[e][tap] = flat[e * 9 + tap];
        if (bias) {
            V::load(bias + c0, b);
        } else {
#pragma unroll
            for (int e = 0; e < N; ++e) b[e] = 0.f;
        }
    }

#pragma unroll
    for (int i = 0; i < RS; ++i) {
        if (y0 + i < Hg) {
            float zf[N], gf[N], res[N];
            V::widen(zr[i], zf);
            V::widen(gr[i], gf);
#pragma unroll
            for (int e = 0; e < N; ++e) res[e] = b[e];
#pragma unroll
            for (int ky = 0; ky < 3; ++ky)
#pragma unroll
                for (int kx = 0; kx < 3; ++kx) {
                    float xv[N];
                    V::widen(xr[i + ky][kx], xv);
#pragma unroll
                    for (int e = 0; e < N; ++e) res[e] = fmaf(wt[e][ky * 3 + kx], xv[e], res[e]);
                }
#pragma unroll
            for (int e = 0; e < N; ++e) {
                const float gate = __builtin_amdgcn_rcpf(1.f + __expf(-zf[e]));
                // G * O_local + (1 - G) * O_global
                res[e] = fmaf(gate, res[e] - gf[e], gf[e]);
            }
            V::store(out + slab_off + (size_t(y0 + i) * Wg + xp) * px, res);
        }
    }
}

template <typename T, int DV, int RS>
hipError_t launch_rs(const void *x, const void *w, const void *bias, const void *z, const void *og, void *out,
                     long slabs, int H, int Hg, int Wg, int token_major, hipStream_t stream)
{
    constexpr int CG = DV / vec4<T>::N;
    const int n_strips = (Hg + RS - 1) / RS;
    const long total = slabs * n_strips * Wg * CG;
    const long blocks = (total + kThreads - 1) / kThreads;
    if (blocks > 0x7fffffffL) return hipErrorInvalidValue;
    LaunchTimer timer(kKernelLocalityGate, stream);
    if (token_major)
        hipLaunchKernelGGL((locality_gate_kernel<T, DV, RS, true>), dim3((unsigned)blocks), dim3(kThreads), 0, stream,
                           static_cast<const T *>(x), static_cast<const T *>(w), static_cast<const T *>(bias),
                           static_cast<const T *>(z), static_cast<const T *>(og), static_cast<T *>(out), H, Hg, Wg,
                           n_strips, total);
    else
        hipLaunchKernelGGL((locality_gate_kernel<T, DV, RS, false>), dim3((unsigned)blocks), dim3(kThreads), 0,
                           stream, static_cast<const T *>(x), static_cast<const T *>(w),
                           static_cast<const T *>(bias), static_cast<const T *>(z), static_cast<const T *>(og),
                           static_cast<T *>(out), H, Hg, Wg, n_strips, total);
    return hipGetLastError();
}

template <typename T, int DV>
hipError_t launch(const void *x, const void *w, const void *bias, const void *z, const void *og, void *out, int B,
                  int H, int Hg, int Wg, int token_major, hipStream_t stream)
{
    constexpr int CG = DV / vec4<T>::N;
    // strips of 4 rows (1.5x input reads, the halo rows come from L2) when that still fills the
    // chip several times over, else strips of 2 rows
    const long slabs = long(B) * H;
    const long blocks4 = (slabs * ((Hg + 3) / 4) * Wg * CG + kThreads - 1) / kThreads;
    if (blocks4 >= 2048) return launch_rs<T, DV, 4>(x, w, bias, z, og, out, slabs, H, Hg, Wg, token_major, stream);
    return launch_rs<T, DV, 2>(x, w, bias, z, og, out, slabs, H, Hg, Wg, token_major, stream);
}

template <typename T>
hipError_t launch_dv(int dv, const void *x, const void *w, const void *bias, const void *z, const void *og,
                     void *out, int B, int H, int Hg, int Wg, int token_major, hipStream_t stream)
{
    switch (dv) {
        case 16: return launch<T, 16>(x, w, bias, z, og, out, B, H, Hg, Wg, token_major, stream);
        case 32: return launch<T, 32>(x, w, bias, z, og, out, B, H, Hg, Wg, token_major, stream);
        case 64: return launch<T, 64>(x, w, bias, z, og, out, B, H, Hg, Wg, token_major, stream);
    }
    return hipErrorInvalidValue;
}

}  // namespace

hipError_t locality_gate_launch(const void *x, const void *w, const void *bias, const void *gate_logits,
                                const void *o_global, void *out, int B, int H, int Hg, int Wg, int dv,
                                bool is_bf16, int token_major, hipStream_t stream)
{
    if (is_bf16) return launch_dv<bf16_t>(dv, x, w, bias, gate_logits, o_global, out, B, H, Hg, Wg, token_major, stream);
    return launch_dv<float>(dv, x, w, bias, gate_logits, o_global, out, B, H, Hg, Wg, token_major, stream);
}

}  // namespace vig
