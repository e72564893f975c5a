// Implicit im2col GEMM convolution on the matrix cores (the "sgemm" kernel family of
// Table 2 / Fig. 5, including 1x1 pointwise layers):
//     y[k, n] = sum_kk Wp[k, kk] * col[kk, n],  n = (img, p, q),  kk = (c, r, s)
// The col matrix is never materialised: every wavefront gathers its B fragments
// straight from x with per-lane validity masks for the zero padding.
//
// float32: v_mfma_f32_16x16x4_f32.  One k-step = 4 channels at one filter tap (r,s);
//   lane l holds row/column l%16 and channel slot l/16, so the packed weight fragment
//   of a step is 64 consecutive floats (one coalesced 256 B load) and the B fragment is
//   x[c0 + l/16][ih][iw + l%16...] (contiguous along W for stride 1).
// float16: v_mfma_f32_16x16x32_f16.  One k-step = 32 channels at one tap; lane l holds
//   8 consecutive channels (slot group l/16), so x is first copied to a channel-last
//   [N][H][W][Cpad32] half buffer in the workspace and both fragments are 16-byte loads.
// A workgroup is 4 wavefronts side by side along n; a wavefront owns TM x TN 16x16
// accumulator blocks.  Loads run D k-steps ahead of the MFMAs in registers.  Layers
// with few output tiles but a long reduction split the k-steps over blockIdx.z into
// float32 partial sums in the workspace, summed in fixed order by a second kernel.
#include "nnv_internal.h"

namespace nnv {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef _Float16 half8 __attribute__((ext_vector_type(8)));

struct GemmParams {
    const void *x;       // float32 NCHW, or half channel-last copy
    const void *wp;      // packed panels
    const float *bias;
    void *y;
    float *partial;      // [splits][K16*16][npix_pad] when splits > 1
    int N, C, H, W, K, R, S, sh, sw, ph, pw, P, Q;
    int npix, npix16;    // N*P*Q and its 16-blocks
    int K16;
    int nsteps;          // k-steps in total
    int steps_per_split, splits;
    int cpad;            // channel stride of the half channel-last copy
    int half_out;
};

template <bool HALF> struct FragT {
    typedef float type;
    __device__ static inline float zero() { return 0.f; }
};
template <> struct FragT<true> {
    typedef half8 type;
    __device__ static inline half8 zero() { return half8{0, 0, 0, 0, 0, 0, 0, 0}; }
};

template <bool HALF, int TM, int TN, int D>
__global__ __launch_bounds__(256) void im2col_gemm_kernel(const GemmParams g) {
    typedef typename FragT<HALF>::type frag_t;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int col = lane & 15, slot = lane >> 4;
    const int mb0 = blockIdx.y * TM;
    const int nb0 = (blockIdx.x * 4 + wave) * TN;
    const int HW = g.H * g.W, PQ = g.P * g.Q, RS = g.R * g.S;

    // per-lane pixel state of each of the TN column blocks
    int xoff[TN];
    uint32_t rmask[TN], smask[TN];
#pragma unroll
    for (int t = 0; t < TN; ++t) {
        const int n = (nb0 + t) * 16 + col;
        rmask[t] = smask[t] = 0;
        xoff[t] = 0;
        if (n < g.npix) {
            const int img = n / PQ, pq = n - img * PQ;
            const int p = pq / g.Q, q = pq - p * g.Q;
            const int ih0 = p * g.sh - g.ph, iw0 = q * g.sw - g.pw;
            for (int r = 0; r < g.R; ++r)
                if (ih0 + r >= 0 && ih0 + r < g.H) rmask[t] |= 1u << r;
            for (int s = 0; s < g.S; ++s)
                if (iw0 + s >= 0 && iw0 + s < g.W) smask[t] |= 1u << s;
            if (HALF) xoff[t] = ((img * g.H + ih0) * g.W + iw0) * g.cpad + slot * 8;
            else xoff[t] = ((img * g.C + slot) * g.H + ih0) * g.W + iw0;
        }
    }

    const int s_begin = blockIdx.z * g.steps_per_split;
    const int s_end = min(g.nsteps, s_begin + g.steps_per_split);
    // (channel block, r, s) of the next step to load
    int cb = s_begin / RS;
    int rs0 = s_begin - cb * RS;
    int lr = rs0 / g.S, ls = rs0 - lr * g.S;
    int lstep = s_begin;

    const frag_t *wfrag = static_cast<const frag_t *>(g.wp);
    frag_t a[2][D][TM], b[2][D][TN];

    auto load_chunk = [&](int buf) {
#pragma unroll
        for (int d = 0; d < D; ++d) {
            const bool live = lstep < s_end;
#pragma unroll
            for (int m = 0; m < TM; ++m) {
                frag_t v = FragT<HALF>::zero();
                if (live && mb0 + m < g.K16) v = wfrag[((size_t)(mb0 + m) * g.nsteps + lstep) * 64 + lane];
                a[buf][d][m] = v;
            }
#pragma unroll
            for (int t = 0; t < TN; ++t) {
                frag_t v = FragT<HALF>::zero();
                bool ok = live && ((rmask[t] >> lr) & (smask[t] >> ls) & 1u);
                if (HALF) {
                    if (ok) v = *reinterpret_cast<const frag_t *>(static_cast<const _Float16 *>(g.x) + xoff[t] +
                                                                  (lr * g.W + ls) * g.cpad + cb * 32);
                } else {
                    ok = ok && (cb * 4 + slot < g.C);
                    if (ok) v = *reinterpret_cast<const frag_t *>(static_cast<const float *>(g.x) + xoff[t] +
                                                                  cb * 4 * HW + lr * g.W + ls);
                }
                b[buf][d][t] = v;
            }
            ++lstep;
            if (++ls == g.S) { ls = 0; if (++lr == g.R) { lr = 0; ++cb; } }
        }
    };

    floatx4 acc[TM][TN];
#pragma unroll
    for (int m = 0; m < TM; ++m)
#pragma unroll
        for (int t = 0; t < TN; ++t) acc[m][t] = floatx4{0.f, 0.f, 0.f, 0.f};

    auto compute = [&](int buf) {
#pragma unroll
        for (int d = 0; d < D; ++d)
#pragma unroll
            for (int m = 0; m < TM; ++m)
#pragma unroll
                for (int t = 0; t < TN; ++t) {
                    if constexpr (HALF)
                        acc[m][t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[buf][d][m], b[buf][d][t], acc[m][t], 0, 0, 0);
                    else
                        acc[m][t] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[buf][d][m], b[buf][d][t], acc[m][t], 0, 0, 0);
                }
    };

    load_chunk(0);
    for (int base = s_begin; base < s_end; base += 2 * D) {
        load_chunk(1);
        compute(0);
        load_chunk(0);
        if (base + D < s_end) compute(1);
    }

    // epilogue: lane holds rows 4*slot + j, column col of each block
#pragma unroll
    for (int t = 0; t < TN; ++t) {
        const int n = (nb0 + t) * 16 + col;
#pragma unroll
        for (int m = 0; m < TM; ++m) {
            if (mb0 + m >= g.K16) continue;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int k = (mb0 + m) * 16 + slot * 4 + j;
                const float v = acc[m][t][j];
                if (g.splits > 1) {
                    if (n < g.npix16 * 16)
                        g.partial[((size_t)blockIdx.z * g.K16 * 16 + k) * ((size_t)g.npix16 * 16) + n] = v;
                } else if (k < g.K && n < g.npix) {
                    const int img = n / PQ, pq = n - img * PQ;
                    const size_t o = ((size_t)img * g.K + k) * PQ + pq;
                    const float r = v + (g.bias ? g.bias[k] : 0.f);
                    if (g.half_out) static_cast<__half *>(g.y)[o] = __float2half_rn(r);
                    else static_cast<float *>(g.y)[o] = r;
                }
            }
        }
    }
}

// y[k, n] = bias[k] + sum_z partial[z][k][n], fixed summation order.
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const GemmParams g) {
    const int n = blockIdx.x * 256 + threadIdx.x;
    const int k = blockIdx.y;
    if (n >= g.npix) return;
    const size_t npad = (size_t)g.npix16 * 16;
    const size_t zstride = (size_t)g.K16 * 16 * npad;
    const float *p = g.partial + (size_t)k * npad + n;
    float acc = g.bias ? g.bias[k] : 0.f;
    for (int z = 0; z < g.splits; ++z) acc += p[z * zstride];
    const int PQ = g.P * g.Q;
    const int img = n / PQ, pq = n - img * PQ;
    const size_t o = ((size_t)img * g.K + k) * PQ + pq;
    if (g.half_out) static_cast<__half *>(g.y)[o] = __float2half_rn(acc);
    else static_cast<float *>(g.y)[o] = acc;
}

// half NCHW -> half [N][H][W][cpad] (channels last, zero padded to a multiple of 32).
__global__ __launch_bounds__(256) void to_channels_last_kernel(const __half *__restrict__ x, __half *__restrict__ xt,
                                                               int C, int HW, int cpad) {
    const int pix = blockIdx.x * 256 + threadIdx.x;
    const int oct = blockIdx.y, img = blockIdx.z;
    if (pix >= HW) return;
    __half v[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const int c = oct * 8 + j;
        v[j] = (c < C) ? x[((size_t)img * C + c) * HW + pix] : __float2half(0.f);
    }
    *reinterpret_cast<uint4 *>(xt + ((size_t)img * HW + pix) * cpad + oct * 8) = *reinterpret_cast<uint4 *>(v);
}

// ---------------------------------------------------------------- host side

struct GemmPlan {
    int tm, tn, splits, steps_per_split;
    size_t xt_bytes, partial_bytes;
};

static GemmPlan plan_im2col(const Geo &g) {
    GemmPlan pl{};
    const bool half = g.dtype == NNV_F16;
    const int K16 = ceil_div(g.k, 16);
    const int npix16 = ceil_div(g.n * g.p * g.q, 16);
    const int nsteps = (half ? ceil_div(g.c, 32) : ceil_div(g.c, 4)) * g.r * g.s;
    auto waves = [&](int tm, int tn) { return (long)ceil_div(K16, tm) * ceil_div(npix16, tn); };
    const long target = 1024;   // one wavefront per SIMD
    if (waves(2, 2) >= target) { pl.tm = 2; pl.tn = 2; }
    else if (waves(2, 1) >= target) { pl.tm = 2; pl.tn = 1; }
    else { pl.tm = 1; pl.tn = 1; }
    long wv = waves(pl.tm, pl.tn);
    int splits = 1;
    if (wv < target / 2) {
        splits = (int)((target + wv - 1) / wv);
        const int max_splits = nsteps / 16 > 0 ? nsteps / 16 : 1;   // at least 16 k-steps each
        if (splits > max_splits) splits = max_splits;
        if (splits > 64) splits = 64;
    }
    pl.steps_per_split = ceil_div(nsteps, splits);
    pl.splits = ceil_div(nsteps, pl.steps_per_split);
    pl.xt_bytes = half ? align_up((size_t)g.n * g.h * g.w * ceil_div(g.c, 32) * 32 * sizeof(__half), 256) : 0;
    pl.partial_bytes = pl.splits > 1 ? (size_t)pl.splits * K16 * 16 * npix16 * 16 * sizeof(float) : 0;
    return pl;
}

size_t im2col_workspace_bytes(const Geo &g) {
    const GemmPlan pl = plan_im2col(g);
    return pl.xt_bytes + pl.partial_bytes;
}

template <bool HALF>
static void launch_gemm_variant(const GemmPlan &pl, const GemmParams &gp, dim3 grid, hipStream_t st) {
    constexpr int D = HALF ? 2 : 4;
    if (pl.tm == 2 && pl.tn == 2)
        hipLaunchKernelGGL((im2col_gemm_kernel<HALF, 2, 2, D>), grid, dim3(256), 0, st, gp);
    else if (pl.tm == 2 && pl.tn == 1)
        hipLaunchKernelGGL((im2col_gemm_kernel<HALF, 2, 1, D>), grid, dim3(256), 0, st, gp);
    else
        hipLaunchKernelGGL((im2col_gemm_kernel<HALF, 1, 1, D>), grid, dim3(256), 0, st, gp);
}

hipError_t launch_im2col(const Geo &g, const void *x, const void *w, const float *bias, void *y, void *ws, hipStream_t st) {
    const GemmPlan pl = plan_im2col(g);
    const bool half = g.dtype == NNV_F16;
    GemmParams gp{};
    gp.x = x; gp.wp = w; gp.bias = bias; gp.y = y;
    gp.N = g.n; gp.C = g.c; gp.H = g.h; gp.W = g.w; gp.K = g.k; gp.R = g.r; gp.S = g.s;
    gp.sh = g.sh; gp.sw = g.sw; gp.ph = g.ph; gp.pw = g.pw; gp.P = g.p; gp.Q = g.q;
    gp.npix = g.n * g.p * g.q;
    gp.npix16 = ceil_div(gp.npix, 16);
    gp.K16 = ceil_div(g.k, 16);
    gp.cpad = ceil_div(g.c, 32) * 32;
    gp.nsteps = (half ? ceil_div(g.c, 32) : ceil_div(g.c, 4)) * g.r * g.s;
    gp.steps_per_split = pl.steps_per_split;
    gp.splits = pl.splits;
    gp.half_out = half;
    char *wsp = static_cast<char *>(ws);
    if (half) {
        __half *xt = reinterpret_cast<__half *>(wsp);
        dim3 grid(ceil_div(g.h * g.w, 256), gp.cpad / 8, g.n);
        hipLaunchKernelGGL(to_channels_last_kernel, grid, dim3(256), 0, st, static_cast<const __half *>(x), xt, g.c,
                           g.h * g.w, gp.cpad);
        gp.x = xt;
        wsp += pl.xt_bytes;
    }
    gp.partial = pl.splits > 1 ? reinterpret_cast<float *>(wsp) : nullptr;
    dim3 grid(ceil_div(gp.npix16, 4 * pl.tn), ceil_div(gp.K16, pl.tm), pl.splits);
    if (half) launch_gemm_variant<true>(pl, gp, grid, st);
    else launch_gemm_variant<false>(pl, gp, grid, st);
    if (pl.splits > 1) {
        dim3 rgrid(ceil_div(gp.npix, 256), g.k, 1);
        hipLaunchKernelGGL(splitk_reduce_kernel, rgrid, dim3(256), 0, st, gp);
    }
    return hipGetLastError();
}

}  // namespace nnv
