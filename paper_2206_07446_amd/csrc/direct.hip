// Direct convolution and depthwise convolution: the kernel alternatives that run from
// raw (or trivially repacked) weights, i.e. with a free weight transformation and the
// slowest execution (Table 2 rows "3x3s1", "general"; Fig. 5 depthwise kernels).
//
// Both are plain vector-ALU kernels.  direct: one thread owns one output pixel and KB
// output channels; the filter taps it needs are wave-uniform, so they come through
// scalar loads, and x is read along W (coalesced).  depthwise: HBM-bound, one thread per
// output pixel of one channel plane, taps of the channel from the packed
// [C/32][9][32] layout.
#include "nnv_internal.h"

namespace nnv {

struct DirectParams {
    int N, C, H, W, K, R, S, sh, sw, ph, pw, P, Q, Cg, Kg;
};

template <typename T> __device__ static inline float ld(const T *p, size_t i);
template <> __device__ inline float ld<float>(const float *p, size_t i) { return p[i]; }
template <> __device__ inline float ld<__half>(const __half *p, size_t i) { return __half2float(p[i]); }
template <typename T> __device__ static inline void st(T *p, size_t i, float v);
template <> __device__ inline void st<float>(float *p, size_t i, float v) { p[i] = v; }
template <> __device__ inline void st<__half>(__half *p, size_t i, float v) { p[i] = __float2half_rn(v); }

template <typename T, int KB>
__global__ __launch_bounds__(256) void direct_conv_kernel(const T *__restrict__ x, const float *__restrict__ w,
                                                          const float *__restrict__ bias, T *__restrict__ y,
                                                          const DirectParams d) {
    const int pq = blockIdx.x * 256 + threadIdx.x;
    const int k0 = blockIdx.y * KB;
    const int img = blockIdx.z;
    const bool live = pq < d.P * d.Q;
    const int p = live ? pq / d.Q : 0, q = live ? pq - p * d.Q : 0;
    const int grp = k0 / d.Kg;
    const int ih0 = p * d.sh - d.ph, iw0 = q * d.sw - d.pw;
    float acc[KB];
#pragma unroll
    for (int j = 0; j < KB; ++j) acc[j] = bias ? bias[k0 + j] : 0.f;
    const T *xb = x + ((size_t)img * d.C + (size_t)grp * d.Cg) * d.H * d.W;
    const size_t wk = (size_t)d.Cg * d.R * d.S;
    for (int c = 0; c < d.Cg; ++c) {
        const T *xc = xb + (size_t)c * d.H * d.W;
        const float *wc = w + (size_t)k0 * wk + (size_t)c * d.R * d.S;
        for (int r = 0; r < d.R; ++r) {
            const int ih = ih0 + r;
            const bool rok = live && ih >= 0 && ih < d.H;
            for (int s = 0; s < d.S; ++s) {
                const int iw = iw0 + s;
                const bool ok = rok && iw >= 0 && iw < d.W;
                const float xv = ok ? ld<T>(xc, (size_t)ih * d.W + iw) : 0.f;
#pragma unroll
                for (int j = 0; j < KB; ++j) acc[j] = fmaf(xv, wc[j * wk + r * d.S + s], acc[j]);
            }
        }
    }
    if (live) {
#pragma unroll
        for (int j = 0; j < KB; ++j) st<T>(y, ((size_t)img * d.K + k0 + j) * d.P * d.Q + pq, acc[j]);
    }
}

template <typename T>
static hipError_t launch_direct_t(const Geo &g, const T *x, const float *w, const float *bias, T *y, hipStream_t st_) {
    DirectParams d{g.n, g.c, g.h, g.w, g.k, g.r, g.s, g.sh, g.sw, g.ph, g.pw, g.p, g.q, g.cg, g.kg};
    const int pq_blocks = ceil_div(g.p * g.q, 256);
    int kb = 1;
    if (g.kg % 8 == 0) kb = 8;
    else if (g.kg % 4 == 0) kb = 4;
    else if (g.kg % 2 == 0) kb = 2;
    // keep the grid large enough to occupy the chip on small layers
    while (kb > 1 && (long)pq_blocks * (g.k / kb) * g.n < 1024) kb /= 2;
    dim3 grid(pq_blocks, g.k / kb, g.n);
    switch (kb) {
        case 8: hipLaunchKernelGGL((direct_conv_kernel<T, 8>), grid, dim3(256), 0, st_, x, w, bias, y, d); break;
        case 4: hipLaunchKernelGGL((direct_conv_kernel<T, 4>), grid, dim3(256), 0, st_, x, w, bias, y, d); break;
        case 2: hipLaunchKernelGGL((direct_conv_kernel<T, 2>), grid, dim3(256), 0, st_, x, w, bias, y, d); break;
        default: hipLaunchKernelGGL((direct_conv_kernel<T, 1>), grid, dim3(256), 0, st_, x, w, bias, y, d); break;
    }
    return hipGetLastError();
}

hipError_t launch_direct(const Geo &g, const void *x, const float *w, const float *bias, void *y, hipStream_t st_) {
    if (g.dtype == NNV_F16)
        return launch_direct_t<__half>(g, static_cast<const __half *>(x), w, bias, static_cast<__half *>(y), st_);
    return launch_direct_t<float>(g, static_cast<const float *>(x), w, bias, static_cast<float *>(y), st_);
}

// ------------------------------------------------------------------ depthwise 3x3

struct DwParams {
    int N, C, H, W, st, ph, pw, P, Q;
};

template <typename T>
__global__ __launch_bounds__(256) void depthwise_kernel(const T *__restrict__ x, const T *__restrict__ wp,
                                                        const float *__restrict__ bias, T *__restrict__ y,
                                                        const DwParams d) {
    const int pq = blockIdx.x * 256 + threadIdx.x;
    const int c = blockIdx.y, img = blockIdx.z;
    if (pq >= d.P * d.Q) return;
    const int p = pq / d.Q, q = pq - p * d.Q;
    const T *wc = wp + (size_t)(c >> 5) * 288 + (c & 31);
    const T *xc = x + ((size_t)img * d.C + c) * d.H * d.W;
    const int ih0 = p * d.st - d.ph, iw0 = q * d.st - d.pw;
    float acc = bias ? bias[c] : 0.f;
#pragma unroll
    for (int r = 0; r < 3; ++r) {
        const int ih = ih0 + r;
        const bool rok = ih >= 0 && ih < d.H;
#pragma unroll
        for (int s = 0; s < 3; ++s) {
            const int iw = iw0 + s;
            const bool ok = rok && iw >= 0 && iw < d.W;
            const float xv = ok ? ld<T>(xc, (size_t)ih * d.W + iw) : 0.f;
            acc = fmaf(xv, ld<T>(wc, (r * 3 + s) * 32), acc);
        }
    }
    st<T>(y, ((size_t)img * d.C + c) * d.P * d.Q + pq, acc);
}

hipError_t launch_depthwise(const Geo &g, const void *x, const void *w, const float *bias, void *y, hipStream_t st_) {
    if (g.c > 65535) return hipErrorInvalidValue;
    DwParams d{g.n, g.c, g.h, g.w, g.sh, g.ph, g.pw, g.p, g.q};
    dim3 grid(ceil_div(g.p * g.q, 256), g.c, g.n);
    if (g.dtype == NNV_F16)
        hipLaunchKernelGGL(depthwise_kernel<__half>, grid, dim3(256), 0, st_, static_cast<const __half *>(x),
                           static_cast<const __half *>(w), bias, static_cast<__half *>(y), d);
    else
        hipLaunchKernelGGL(depthwise_kernel<float>, grid, dim3(256), 0, st_, static_cast<const float *>(x),
                           static_cast<const float *>(w), bias, static_cast<float *>(y), d);
    return hipGetLastError();
}

}  // namespace nnv
