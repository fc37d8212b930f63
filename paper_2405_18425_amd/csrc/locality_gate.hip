// 2D gating locality injection (Section 4.2.2): depthwise 3x3 convolution on the patch grid
// blended with the global branch through a sigmoid gate,
//     out = sigmoid(z) * DWConv3x3(x) + (1 - sigmoid(z)) * o_global .
//
// The step is pure bandwidth (about 25 flops per element against 4 element transfers), so the
// kernel is organised around memory: a thread owns 16 bytes of channels (8 bf16 / 4 fp32) of one
// grid column and walks down a strip of rows keeping a 3x3 window of fp32 values in registers, so
// that each input row costs three 16-byte loads (left, centre, right neighbour -- the last two
// come from cache lines the neighbouring threads fetch anyway) instead of nine.  Consecutive
// threads cover consecutive channel groups and then consecutive columns, i.e. one contiguous
// row of the [.., y, x, channel] tensor per wavefront load.  Arithmetic is fp32 on either dtype.
#include "vig_common.hpp"
#include "vig_kernels.hpp"
#include "vig_timing.hpp"

namespace vig {

namespace {

template <typename T>
struct vec16;  // 16-byte vector of T, widened to fp32 lanes

template <>
struct vec16<float> {
    static constexpr int N = 4;
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
struct vec16<bf16_t> {
    static constexpr int N = 8;
    static __device__ __forceinline__ void load(const bf16_t *p, float (&f)[N])
    {
        const uint4 r = *reinterpret_cast<const uint4 *>(p);
        f[0] = bf16_lo_to_f32(r.x); f[1] = bf16_hi_to_f32(r.x);
        f[2] = bf16_lo_to_f32(r.y); f[3] = bf16_hi_to_f32(r.y);
        f[4] = bf16_lo_to_f32(r.z); f[5] = bf16_hi_to_f32(r.z);
        f[6] = bf16_lo_to_f32(r.w); f[7] = bf16_hi_to_f32(r.w);
    }
    static __device__ __forceinline__ void store(bf16_t *p, const float (&f)[N])
    {
        uint4 r;
        r.x = pack_bf16x2(f[0], f[1]);
        r.y = pack_bf16x2(f[2], f[3]);
        r.z = pack_bf16x2(f[4], f[5]);
        r.w = pack_bf16x2(f[6], f[7]);
        *reinterpret_cast<uint4 *>(p) = r;
    }
};

constexpr int kThreads = 256;

template <typename T, int DV>
__global__ __launch_bounds__(kThreads) void locality_gate_kernel(
    const T *__restrict__ x, const T *__restrict__ w, const T *__restrict__ bias, const T *__restrict__ z,
    const T *__restrict__ og, T *__restrict__ out, int H, int Hg, int Wg, int rows_per_strip, int n_strips,
    long total_threads)
{
    using V = vec16<T>;
    constexpr int N = V::N;
    constexpr int CG = DV / N;

    const long gid = long(blockIdx.x) * kThreads + threadIdx.x;
    if (gid >= total_threads) return;
    const int cg = int(gid % CG);
    long r = gid / CG;
    const int xp = int(r % Wg);
    r /= Wg;
    const int strip = int(r % n_strips);
    const long slab = r / n_strips;
    const int h = int(slab % H);
    const int c0 = h * DV + cg * N;

    // filter taps and bias of this thread's N channels, fp32
    float wt[N][9];
    float b[N];
#pragma unroll
    for (int e = 0; e < N; ++e) {
#pragma unroll
        for (int tap = 0; tap < 9; ++tap) wt[e][tap] = io<T>::load(w + size_t(c0 + e) * 9 + tap);
        b[e] = bias ? io<T>::load(bias + c0 + e) : 0.f;
    }

    const size_t slab_off = size_t(slab) * Hg * Wg * DV + size_t(cg) * N;
    const T *xs = x + slab_off;
    const int y0 = strip * rows_per_strip;
    const int y1 = min(Hg, y0 + rows_per_strip);

    // win[ky][kx] = x[y + ky - 1][xp + kx - 1]; out-of-grid taps are zero (zero padding)
    float win[3][3][N];
    auto load_row = [&](int yy, float (&row)[3][N]) {
#pragma unroll
        for (int kx = 0; kx < 3; ++kx) {
            const int xx = xp + kx - 1;
            if (yy >= 0 && yy < Hg && xx >= 0 && xx < Wg) {
                V::load(xs + (size_t(yy) * Wg + xx) * DV, row[kx]);
            } else {
#pragma unroll
                for (int e = 0; e < N; ++e) row[kx][e] = 0.f;
            }
        }
    };
    load_row(y0 - 1, win[0]);
    load_row(y0, win[1]);

    for (int y = y0; y < y1; ++y) {
        load_row(y + 1, win[2]);
        const size_t o = slab_off + (size_t(y) * Wg + xp) * DV;
        float zf[N], gf[N], res[N];
        V::load(z + o, zf);
        V::load(og + o, gf);
#pragma unroll
        for (int e = 0; e < N; ++e) {
            float local = b[e];
#pragma unroll
            for (int ky = 0; ky < 3; ++ky)
#pragma unroll
                for (int kx = 0; kx < 3; ++kx) local = fmaf(wt[e][ky * 3 + kx], win[ky][kx][e], local);
            const float gate = 1.f / (1.f + expf(-zf[e]));
            // G * O_local + (1 - G) * O_global
            res[e] = fmaf(gate, local - gf[e], gf[e]);
        }
        V::store(out + o, res);
#pragma unroll
        for (int kx = 0; kx < 3; ++kx)
#pragma unroll
            for (int e = 0; e < N; ++e) {
                win[0][kx][e] = win[1][kx][e];
                win[1][kx][e] = win[2][kx][e];
            }
    }
}

template <typename T, int DV>
hipError_t launch(const void *x, const void *w, const void *bias, const void *z, const void *og, void *out, int B,
                  int H, int Hg, int Wg, hipStream_t stream)
{
    constexpr int CG = DV / vec16<T>::N;
    // strips of 8 rows when that still yields a few thousand workgroups, else 4 (more halo, more waves)
    const long slabs = long(B) * H;
    int rows = 8;
    auto blocks_for = [&](int rps) {
        const long strips = (Hg + rps - 1) / rps;
        return (slabs * strips * Wg * CG + kThreads - 1) / kThreads;
    };
    if (blocks_for(rows) < 2048) rows = 4;
    if (blocks_for(rows) < 1024) rows = 2;
    const int n_strips = (Hg + rows - 1) / rows;
    const long total = slabs * n_strips * Wg * CG;
    const long blocks = (total + kThreads - 1) / kThreads;
    if (blocks > 0x7fffffffL) return hipErrorInvalidValue;
    LaunchTimer timer(kKernelLocalityGate, stream);
    hipLaunchKernelGGL((locality_gate_kernel<T, DV>), dim3((unsigned)blocks), dim3(kThreads), 0, stream,
                       static_cast<const T *>(x), static_cast<const T *>(w), static_cast<const T *>(bias),
                       static_cast<const T *>(z), static_cast<const T *>(og), static_cast<T *>(out), H, Hg, Wg, rows,
                       n_strips, total);
    return hipGetLastError();
}

template <typename T>
hipError_t launch_dv(int dv, const void *x, const void *w, const void *bias, const void *z, const void *og,
                     void *out, int B, int H, int Hg, int Wg, hipStream_t stream)
{
    switch (dv) {
        case 16: return launch<T, 16>(x, w, bias, z, og, out, B, H, Hg, Wg, stream);
        case 32: return launch<T, 32>(x, w, bias, z, og, out, B, H, Hg, Wg, stream);
        case 64: return launch<T, 64>(x, w, bias, z, og, out, B, H, Hg, Wg, stream);
    }
    return hipErrorInvalidValue;
}

}  // namespace

hipError_t locality_gate_launch(const void *x, const void *w, const void *bias, const void *gate_logits,
                                const void *o_global, void *out, int B, int H, int Hg, int Wg, int dv,
                                bool is_bf16, hipStream_t stream)
{
    if (is_bf16) return launch_dv<bf16_t>(dv, x, w, bias, gate_logits, o_global, out, B, H, Hg, Wg, stream);
    return launch_dv<float>(dv, x, w, bias, gate_logits, o_global, out, B, H, Hg, Wg, stream);
}

}  // namespace vig
