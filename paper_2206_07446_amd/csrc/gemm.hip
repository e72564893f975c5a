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
// A wavefront owns TM x TN 16x16 accumulator blocks; loads run D k-steps ahead of the
// MFMAs in registers (no LDS on the operand path: at 32 cycles per float32 MFMA the L1/L2
// path feeds fragments fast enough, what matters is enough loads in flight).  Batch-1
// layers have few output tiles but long reductions, so KS wavefronts of a workgroup share
// one output tile and split its k-steps; their partial sums meet in LDS and are added in
// fixed order.  A workgroup holds 4/KS tiles side by side along n when KS < 4.
#include <cstdio>
#include <cstdlib>
#include "nnv_internal.h"
#include "buf.h"

namespace nnv {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef half8_t half8;

struct GemmParams {
    const void *x;       // float32 NCHW, or half channel-last copy
    const void *wp;      // packed panels
    const float *bias;
    void *y;
    int N, C, H, W, K, R, S, sh, sw, ph, pw, P, Q;
    int npix, npix16;    // N*P*Q and its 16-blocks
    int K16;
    int nsteps;          // k-steps in total
    int ks_shift;        // wavefronts sharing one output tile = 1 << ks_shift
    int cpad;            // channel stride of the half channel-last copy
    uint32_t x_bytes, w_bytes;   // sizes of the x and wp buffers (range-checked loads)
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
__global__ __launch_bounds__(1024) void im2col_gemm_kernel(const GemmParams g) {
    typedef typename FragT<HALF>::type frag_t;
    extern __shared__ __align__(16) float red[];
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave index as a scalar
    const int col = lane & 15, slot = lane >> 4;
    const int KS = 1 << g.ks_shift;
    const int ks = wave & (KS - 1), nt = wave >> g.ks_shift;       // k-split index, tile within the workgroup
    const int tiles_per_wg = (blockDim.x >> 6) >> g.ks_shift;
    const int mb0 = blockIdx.y * TM;
    const int nb0 = (blockIdx.x * tiles_per_wg + nt) * TN;
    const int HW = g.H * g.W, PQ = g.P * g.Q, RS = g.R * g.S;

    // per-lane pixel state of each of the TN column blocks: byte offset of the patch origin
    // in x and the validity masks of its rows and columns (zero padding)
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
            if (HALF) xoff[t] = (((img * g.H + ih0) * g.W + iw0) * g.cpad + slot * 8) * 2;
            else xoff[t] = (((img * g.C + slot) * g.H + ih0) * g.W + iw0) * 4;
        }
    }

    const int per_wave = (g.nsteps + KS - 1) >> g.ks_shift;
    const int s_begin = min(g.nsteps, ks * per_wave);
    const int s_end = min(g.nsteps, s_begin + per_wave);
    // (channel block, r, s) of the next step to load
    int cb = s_begin / RS;
    int rs0 = s_begin - cb * RS;
    int lr = rs0 / g.S, ls = rs0 - lr * g.S;
    int lstep = s_begin;

    const __amdgpu_buffer_rsrc_t wres = make_rsrc(g.wp, g.w_bytes);
    const __amdgpu_buffer_rsrc_t xres = make_rsrc(g.x, g.x_bytes);
    constexpr uint32_t FB = sizeof(frag_t);          // bytes per lane of one fragment
    const uint32_t a_lane = lane * FB;
    frag_t a[2][D][TM], b[2][D][TN];

    // all loads of a chunk are unconditional buffer loads: masked lanes read beyond the buffer -> 0
    auto load_chunk = [&](int buf) {
#pragma unroll
        for (int d = 0; d < D; ++d) {
            const bool live = lstep < s_end;
#pragma unroll
            for (int m = 0; m < TM; ++m) {
                const bool ok = live && mb0 + m < g.K16;
                a[buf][d][m] = buf_load<frag_t>(wres, ok ? a_lane : kOobOffset,
                                                ok ? (uint32_t)((mb0 + m) * g.nsteps + lstep) * (64 * FB) : 0u);
            }
            // uniform part of the B offset for this step
            const int step_off = HALF ? ((lr * g.W + ls) * g.cpad + cb * 32) * 2 : (cb * 4 * HW + lr * g.W + ls) * 4;
#pragma unroll
            for (int t = 0; t < TN; ++t) {
                bool ok = live && ((rmask[t] >> lr) & (smask[t] >> ls) & 1u);
                if (!HALF) ok = ok && (cb * 4 + slot < g.C);
                b[buf][d][t] = buf_load<frag_t>(xres, ok ? (uint32_t)(xoff[t] + step_off) : kOobOffset, 0u);
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

    // sum the KS partial tiles through LDS: red[((nt * KS + ks) * NREG + reg) * 64 + lane]
    constexpr int NREG = TM * TN * 4;
    if (KS > 1) {
#pragma unroll
        for (int m = 0; m < TM; ++m)
#pragma unroll
            for (int t = 0; t < TN; ++t)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    red[((nt * KS + ks) * NREG + (m * TN + t) * 4 + j) * 64 + lane] = acc[m][t][j];
        __syncthreads();
    }
    // epilogue: lane holds rows 4*slot + j, column col of each block; wave ks finishes the
    // accumulator registers reg = ks, ks + KS, ...
#pragma unroll
    for (int m = 0; m < TM; ++m) {
#pragma unroll
        for (int t = 0; t < TN; ++t) {
            const int n = (nb0 + t) * 16 + col;
            const int img = n / PQ, pq = n - img * PQ;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int reg = (m * TN + t) * 4 + j;
                if ((reg & (KS - 1)) != ks) continue;
                float v = acc[m][t][j];
                if (KS > 1) {
                    v = 0.f;
                    for (int z = 0; z < KS; ++z) v += red[((nt * KS + z) * NREG + reg) * 64 + lane];
                }
                const int k = (mb0 + m) * 16 + slot * 4 + j;
                if (k < g.K && n < g.npix) {
                    const size_t o = ((size_t)img * g.K + k) * PQ + pq;
                    const float r = v + (g.bias ? g.bias[k] : 0.f);
                    if (g.half_out) static_cast<__half *>(g.y)[o] = __float2half_rn(r);
                    else static_cast<float *>(g.y)[o] = r;
                }
            }
        }
    }
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
    int tm, tn, ks_shift, d;
    size_t xt_bytes;
};

static GemmPlan plan_im2col(const Geo &g) {
    GemmPlan pl{};
    const bool half = g.dtype == NNV_F16;
    const int K16 = ceil_div(g.k, 16);
    const int npix16 = ceil_div(g.n * g.p * g.q, 16);
    const int nsteps = (half ? ceil_div(g.c, 32) : ceil_div(g.c, 4)) * g.r * g.s;
    auto tiles = [&](int tm, int tn) { return (long)ceil_div(K16, tm) * ceil_div(npix16, tn); };
    // Batch-1 layers are latency-bound: what pays is many wavefronts with a short reduction each.
    // Split the k-steps over KS wavefronts until about 1.5 wavefronts per SIMD exist, keeping at
    // least 12 k-steps per wavefront; take the 32x16 tile if that still gives enough wavefronts,
    // the 32x32 tile only for layers with thousands of tiles.
    auto split_for = [&](long t) {
        int shift = 0;
        while (shift < 4 && (t << shift) < 1536 && (nsteps >> (shift + 1)) >= 12) ++shift;
        return shift;
    };
    if (tiles(2, 2) >= 4096) { pl.tm = 2; pl.tn = 2; }
    else if ((tiles(2, 1) << split_for(tiles(2, 1))) >= 1536) { pl.tm = 2; pl.tn = 1; }
    else { pl.tm = 1; pl.tn = 1; }
    pl.ks_shift = split_for(tiles(pl.tm, pl.tn));
    pl.d = 4;
    if (const char *e = getenv("NNV_GEMM_PLAN")) {   // tm,tn,ks_shift,d
        int a, b, c, d;
        if (sscanf(e, "%d,%d,%d,%d", &a, &b, &c, &d) == 4) { pl.tm = a; pl.tn = b; pl.ks_shift = c; pl.d = d; }
    }
    pl.xt_bytes = half ? align_up((size_t)g.n * g.h * g.w * ceil_div(g.c, 32) * 32 * sizeof(__half), 256) : 0;
    return pl;
}

size_t im2col_workspace_bytes(const Geo &g) { return plan_im2col(g).xt_bytes; }

template <bool HALF, int TM, int TN>
static void launch_gemm_d(const GemmPlan &pl, const GemmParams &gp, dim3 grid, dim3 block, size_t lds, hipStream_t st) {
    if (HALF) {
        hipLaunchKernelGGL((im2col_gemm_kernel<HALF, TM, TN, 2>), grid, block, lds, st, gp);
        return;
    }
    if (pl.d == 4) hipLaunchKernelGGL((im2col_gemm_kernel<HALF, TM, TN, 4>), grid, block, lds, st, gp);
    else if (pl.d == 16 && TM * TN == 1) hipLaunchKernelGGL((im2col_gemm_kernel<HALF, TM, TN, 16>), grid, block, lds, st, gp);
    else hipLaunchKernelGGL((im2col_gemm_kernel<HALF, TM, TN, 8>), grid, block, lds, st, gp);
}

template <bool HALF>
static void launch_gemm_variant(const GemmPlan &pl, const GemmParams &gp, dim3 grid, dim3 block, size_t lds, hipStream_t st) {
    if (pl.tm == 2 && pl.tn == 2) launch_gemm_d<HALF, 2, 2>(pl, gp, grid, block, lds, st);
    else if (pl.tm == 2 && pl.tn == 1) launch_gemm_d<HALF, 2, 1>(pl, gp, grid, block, lds, st);
    else launch_gemm_d<HALF, 1, 1>(pl, gp, grid, block, lds, st);
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
    gp.ks_shift = pl.ks_shift;
    gp.half_out = half;
    gp.x_bytes = half ? (uint32_t)((size_t)g.n * g.h * g.w * gp.cpad * 2) : (uint32_t)((size_t)g.n * g.c * g.h * g.w * 4);
    gp.w_bytes = (uint32_t)((size_t)gp.K16 * gp.nsteps * 64 * (half ? 16 : 4));
    if (half) {
        __half *xt = static_cast<__half *>(ws);
        dim3 grid(ceil_div(g.h * g.w, 256), gp.cpad / 8, g.n);
        hipLaunchKernelGGL(to_channels_last_kernel, grid, dim3(256), 0, st, static_cast<const __half *>(x), xt, g.c,
                           g.h * g.w, gp.cpad);
        gp.x = xt;
    }
    const int KS = 1 << pl.ks_shift;
    const int waves = KS < 4 ? 4 : KS;
    const int tiles_per_wg = waves / KS;
    dim3 grid(ceil_div(ceil_div(gp.npix16, pl.tn), tiles_per_wg), ceil_div(gp.K16, pl.tm), 1);
    const size_t lds = KS > 1 ? (size_t)waves * pl.tm * pl.tn * 4 * 64 * sizeof(float) : 0;
    if (half) launch_gemm_variant<true>(pl, gp, grid, dim3(64 * waves), lds, st);
    else launch_gemm_variant<false>(pl, gp, grid, dim3(64 * waves), lds, st);
    return hipGetLastError();
}

}  // namespace nnv
