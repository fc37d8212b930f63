// 2D gating locality injection (Section 4.2.2): depthwise 3x3 convolution on the patch grid
// blended with the global branch through a sigmoid gate,
//     out = sigmoid(z) * DWConv3x3(x) + (1 - sigmoid(z)) * o_global .
//
// The step moves 4 element transfers per output for about 25 flops, and at four channels per
// thread its vector instructions (unpacking bf16, address arithmetic, bounds selects) would cost
// nearly as much time as its memory traffic, so the kernel is organised to keep both down: a thread
// owns 4 consecutive channels of one grid column and a strip of rows; every load of the strip is a
// buffer load through a per-slab resource with a 32-bit offset, and taps off the grid are
// requested beyond the resource's extent, where the hardware's bounds check returns the zero
// padding without a branch or a select on the data; each input row is widened to fp32 once and
// added into the (up to three) output rows it touches.  Consecutive threads cover consecutive
// channel groups and then consecutive columns, i.e. one contiguous row of the [.., y, x, channel]
// tensor per wavefront load.  Arithmetic is fp32 on either dtype.
#include "vig_common.hpp"
#include "vig_kernels.hpp"
#include "vig_timing.hpp"

namespace vig {

namespace {

// A thread's slice of one pixel: 4 consecutive channels (8 bytes of bf16, 16 bytes of fp32),
// widened to fp32 lanes.

template <typename T>
struct vec4;

template <>
struct vec4<float> {
    static constexpr int N = 4;
    typedef u32x4 raw_t;
    static __device__ __forceinline__ raw_t load(__amdgpu_buffer_rsrc_t r, unsigned off)
    {
        return __builtin_amdgcn_raw_buffer_load_b128(r, off, 0, 0);
    }
    static __device__ __forceinline__ void widen(const raw_t &r, float (&f)[N])
    {
        f[0] = __uint_as_float(r.x); f[1] = __uint_as_float(r.y);
        f[2] = __uint_as_float(r.z); f[3] = __uint_as_float(r.w);
    }
    static __device__ __forceinline__ void store(__amdgpu_buffer_rsrc_t r, unsigned off, const float (&f)[N])
    {
        const raw_t v = {__float_as_uint(f[0]), __float_as_uint(f[1]), __float_as_uint(f[2]), __float_as_uint(f[3])};
        __builtin_amdgcn_raw_buffer_store_b128(v, r, off, 0, 0);
    }
};

template <>
struct vec4<bf16_t> {
    static constexpr int N = 4;
    typedef u32x2 raw_t;
    static __device__ __forceinline__ raw_t load(__amdgpu_buffer_rsrc_t r, unsigned off)
    {
        return __builtin_amdgcn_raw_buffer_load_b64(r, off, 0, 0);
    }
    static __device__ __forceinline__ void widen(const raw_t &r, float (&f)[N])
    {
        f[0] = bf16_lo_to_f32(r.x); f[1] = bf16_hi_to_f32(r.x);
        f[2] = bf16_lo_to_f32(r.y); f[3] = bf16_hi_to_f32(r.y);
    }
    static __device__ __forceinline__ void store(__amdgpu_buffer_rsrc_t r, unsigned off, const float (&f)[N])
    {
        const raw_t v = {pack_bf16x2(f[0], f[1]), pack_bf16x2(f[2], f[3])};
        __builtin_amdgcn_raw_buffer_store_b64(v, r, off, 0, 0);
    }
};

constexpr int kThreads = 256;
// offset of a tap off the grid (or a row past it): beyond every resource's extent, so the load
// returns zeros and the store is dropped
constexpr unsigned kOffGrid = 0xfffffff0u;

// One slab (batch element, head) per group of `blocks_per_slab` consecutive workgroups, so that
// everything that depends on the slab is uniform over a workgroup.
template <typename T, int DV, int RS, bool kTm /* [B,L,H,dv] instead of [B,H,L,dv] */>
__global__ __launch_bounds__(kThreads) void locality_gate_kernel(
    const T *__restrict__ x, const T *__restrict__ w, const T *__restrict__ bias, const T *__restrict__ z,
    const T *__restrict__ og, T *__restrict__ out, int H, int Hg, int Wg, unsigned threads_per_slab,
    unsigned blocks_per_slab)
{
    using V = vec4<T>;
    using raw_t = typename V::raw_t;
    constexpr int N = V::N;
    constexpr int CG = DV / N;

    const unsigned slab = blockIdx.x / blocks_per_slab;
    const unsigned lid = (blockIdx.x % blocks_per_slab) * kThreads + threadIdx.x;
    if (lid >= threads_per_slab) return;
    const int cg = int(lid % CG);
    const unsigned rest = lid / CG;
    const int xp = int(rest % unsigned(Wg));
    const int y0 = int(rest / unsigned(Wg)) * RS;
    const int h = int(slab % unsigned(H));
    const int c0 = h * DV + cg * N;
    // first pixel of the slab (in elements) and distance between pixels (in bytes)
    const size_t first = (kTm ? size_t(slab / unsigned(H)) * Hg * Wg * H + h : size_t(slab) * Hg * Wg) * DV;
    const unsigned px = unsigned(kTm ? H * DV : DV) * unsigned(sizeof(T));
    const unsigned extent = unsigned(Hg * Wg - 1) * px + unsigned(DV * sizeof(T));
    const __amdgpu_buffer_rsrc_t rx = slab_resource(x + first, extent), rz = slab_resource(z + first, extent);
    const __amdgpu_buffer_rsrc_t rg = slab_resource(og + first, extent), ro = slab_resource(out + first, extent);
    const unsigned own = unsigned(y0 * Wg + xp) * px + unsigned(cg * N * sizeof(T));  // pixel (y0, xp)
    const unsigned row = unsigned(Wg) * px;

    // ---- every load of the strip is issued before any arithmetic: (RS+2)*3 input vectors (rows
    // y0-1 .. y0+RS, columns xp-1 .. xp+1), 2*RS gate/global vectors and the 9 tap vectors, so
    // that one wave keeps several hundred bytes per lane in flight ----
    raw_t xr[RS + 2][3], zr[RS], gr[RS];
    const bool col_in[3] = {xp > 0, true, xp + 1 < Wg};
#pragma unroll
    for (int i = 0; i < RS + 2; ++i) {
        const int yy = y0 - 1 + i;
        const bool row_in = yy >= 0 && yy < Hg;
#pragma unroll
        for (int kx = 0; kx < 3; ++kx) {
            const unsigned off = own + unsigned(i - 1) * row + unsigned(kx - 1) * px;  // wraps consistently
            xr[i][kx] = V::load(rx, row_in && col_in[kx] ? off : kOffGrid);
        }
    }
#pragma unroll
    for (int i = 0; i < RS; ++i) {
        const unsigned off = y0 + i < Hg ? own + unsigned(i) * row : kOffGrid;
        zr[i] = V::load(rz, off);
        gr[i] = V::load(rg, off);
    }

    // filter taps and bias of this thread's N channels, fp32: the 9*N taps are contiguous in w
    float wt[N][9], acc[RS][N];
    {
        float flat[9 * N];
        if (sizeof(T) == 2) {
            const uint2 *wp = reinterpret_cast<const uint2 *>(w + size_t(c0) * 9);
#pragma unroll
            for (int i = 0; i < 9; ++i) {
                const uint2 r = wp[i];
                flat[i * N + 0] = bf16_lo_to_f32(r.x); flat[i * N + 1] = bf16_hi_to_f32(r.x);
                flat[i * N + 2] = bf16_lo_to_f32(r.y); flat[i * N + 3] = bf16_hi_to_f32(r.y);
            }
        } else {
            const float4 *wp = reinterpret_cast<const float4 *>(w + size_t(c0) * 9);
#pragma unroll
            for (int i = 0; i < 9; ++i) {
                const float4 r = wp[i];
                flat[i * N + 0] = r.x; flat[i * N + 1] = r.y; flat[i * N + 2] = r.z; flat[i * N + 3] = r.w;
            }
        }
#pragma unroll
        for (int e = 0; e < N; ++e)
#pragma unroll
            for (int tap = 0; tap < 9; ++tap) wt[e][tap] = flat[e * 9 + tap];
#pragma unroll
        for (int e = 0; e < N; ++e) {
            const float b = bias ? io<T>::load(bias + c0 + e) : 0.f;
#pragma unroll
            for (int i = 0; i < RS; ++i) acc[i][e] = b;
        }
    }

    // input row y0-1+i, widened once, goes into output rows i-2 .. i with filter rows 2 .. 0: every
    // output still accumulates bias, then its taps in row-major order
#pragma unroll
    for (int i = 0; i < RS + 2; ++i) {
        float xv[3][N];
#pragma unroll
        for (int kx = 0; kx < 3; ++kx) V::widen(xr[i][kx], xv[kx]);
#pragma unroll
        for (int ky = 2; ky >= 0; --ky) {
            const int o = i - ky;
            if (o < 0 || o >= RS) continue;
#pragma unroll
            for (int kx = 0; kx < 3; ++kx)
#pragma unroll
                for (int e = 0; e < N; ++e) acc[o][e] = fmaf(wt[e][ky * 3 + kx], xv[kx][e], acc[o][e]);
        }
    }

#pragma unroll
    for (int i = 0; i < RS; ++i) {
        float zf[N], gf[N];
        V::widen(zr[i], zf);
        V::widen(gr[i], gf);
#pragma unroll
        for (int e = 0; e < N; ++e) {
            const float gate = __builtin_amdgcn_rcpf(1.f + __expf(-zf[e]));
            // G * O_local + (1 - G) * O_global
            acc[i][e] = fmaf(gate, acc[i][e] - gf[e], gf[e]);
        }
        V::store(ro, y0 + i < Hg ? own + unsigned(i) * row : kOffGrid, acc[i]);
    }
}

template <typename T, int DV, int RS>
hipError_t launch_rs(const void *x, const void *w, const void *bias, const void *z, const void *og, void *out,
                     long slabs, int H, int Hg, int Wg, int token_major, hipStream_t stream)
{
    constexpr int CG = DV / vec4<T>::N;
    const long per_slab = long((Hg + RS - 1) / RS) * Wg * CG;
    const long blocks_per_slab = (per_slab + kThreads - 1) / kThreads;
    const long blocks = slabs * blocks_per_slab;
    if (per_slab > 0x7fffffffL || blocks > 0x7fffffffL) return hipErrorInvalidValue;
    LaunchTimer timer(kKernelLocalityGate, stream);
    if (token_major)
        hipLaunchKernelGGL((locality_gate_kernel<T, DV, RS, true>), dim3((unsigned)blocks), dim3(kThreads), 0, stream,
                           static_cast<const T *>(x), static_cast<const T *>(w), static_cast<const T *>(bias),
                           static_cast<const T *>(z), static_cast<const T *>(og), static_cast<T *>(out), H, Hg, Wg,
                           unsigned(per_slab), unsigned(blocks_per_slab));
    else
        hipLaunchKernelGGL((locality_gate_kernel<T, DV, RS, false>), dim3((unsigned)blocks), dim3(kThreads), 0,
                           stream, static_cast<const T *>(x), static_cast<const T *>(w),
                           static_cast<const T *>(bias), static_cast<const T *>(z), static_cast<const T *>(og),
                           static_cast<T *>(out), H, Hg, Wg, unsigned(per_slab), unsigned(blocks_per_slab));
    return hipGetLastError();
}

template <typename T, int DV>
hipError_t launch(const void *x, const void *w, const void *bias, const void *z, const void *og, void *out, int B,
                  int H, int Hg, int Wg, int token_major, hipStream_t stream)
{
    constexpr int CG = DV / vec4<T>::N;
    // Taller strips re-read less (a strip of RS rows reads RS + 2 input rows) but mean fewer threads and
    // more registers per thread: 8 rows while that still leaves about four workgroups per compute
    // unit (measured at 48 slabs of 64 x 64: 21.9 us against 22.5 us with 4 rows, 27.4 us with 2),
    // then 4 rows, and 2 rows for small problems.
    const long slabs = long(B) * H;
    auto blocks = [&](int rs) { return slabs * ((long((Hg + rs - 1) / rs) * Wg * CG + kThreads - 1) / kThreads); };
    if (blocks(8) >= 1024) return launch_rs<T, DV, 8>(x, w, bias, z, og, out, slabs, H, Hg, Wg, token_major, stream);
    if (blocks(4) >= 2048) return launch_rs<T, DV, 4>(x, w, bias, z, og, out, slabs, H, Hg, Wg, token_major, stream);
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
