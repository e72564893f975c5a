// Direct convolution and depthwise convolution: the kernel alternatives that run from
// raw (or trivially repacked) weights, i.e. with a free weight transformation and the
// slowest execution (Table 2 rows "3x3s1", "general"; Fig. 5 depthwise kernels).
//
// Both are plain vector-ALU kernels.  direct: one thread owns one output pixel and KB
// output channels; the filter taps it needs are wave-uniform, so they come through
// scalar loads, and x is read along W (coalesced).  depthwise: HBM-bound, one thread per
// output pixel of one channel plane, taps of the channel (3x3 or 5x5) from the packed
// [C/32][taps][32] layout.
#include <algorithm>
#include <climits>
#include <type_traits>
#include "nnv_internal.h"
#include "buf.h"

namespace nnv {

struct DirectParams {
    int N, C, H, W, K, R, S, sh, sw, ph, pw, P, Q, Cg, Kg;
    int grid_nx, grid_ny;   // scalar-weight kernel: pixel groups, output-channel groups (logical grid)
    int k_major;            // 1: consecutive logical blocks walk the pixels first (an XCD keeps few filters)
    int relu;               // outputs clamped at zero before the store
};

__device__ static inline float act(float v, int relu) { return relu ? fmaxf(v, 0.f) : v; }

template <typename T> __device__ static inline float ld(const T *p, size_t i);
template <> __device__ inline float ld<float>(const float *p, size_t i) { return p[i]; }
template <> __device__ inline float ld<__half>(const __half *p, size_t i) { return __half2float(p[i]); }
template <typename T> __device__ static inline void st(T *p, size_t i, float v);
template <> __device__ inline void st<float>(float *p, size_t i, float v) { p[i] = v; }
template <> __device__ inline void st<__half>(__half *p, size_t i, float v) { p[i] = __float2half_rn(v); }

// Fallback for channel counts the tiled kernel does not cover (few output channels per group).
template <typename T, int KB>
__global__ __launch_bounds__(256) void direct_conv_simple_kernel(const T *__restrict__ x, const float *__restrict__ w,
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
        for (int j = 0; j < KB; ++j) st<T>(y, ((size_t)img * d.K + k0 + j) * d.P * d.Q + pq, act(acc[j], d.relu));
    }
}

// Tiled direct convolution.  A thread owns TP consecutive output pixels x TK output channels;
// the CS wavefronts of a block share those outputs and split the input channels between them
// (summed through LDS at the end, fixed order), which is what keeps 1024 SIMDs busy on a
// batch-1 layer.  The block's filter taps are staged in LDS per chunk of CC channels as
// [c][r][s][TK] and read back as wave-uniform broadcasts.  FS = filter size when square and
// known at compile time (1, 3), else 0.
template <typename T, int TK, int TP, int FS>
__global__ __launch_bounds__(1024) void direct_conv_tiled_kernel(const T *__restrict__ x, const float *__restrict__ w,
                                                                 const float *__restrict__ bias, T *__restrict__ y,
                                                                 const DirectParams d, const int CC) {
    extern __shared__ __align__(16) float lds[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int CS = blockDim.x >> 6;
    const int R = FS ? FS : d.R, S = FS ? FS : d.S, RS = R * S;
    const int PQ = d.P * d.Q, HW = d.H * d.W;
    const int k0 = blockIdx.y * TK, img = blockIdx.z;
    const int grp = k0 / d.Kg;
    int ih0[TP], iw0[TP];
    bool live[TP];
#pragma unroll
    for (int t = 0; t < TP; ++t) {
        const int pix = (blockIdx.x * 64 + lane) * TP + t;
        live[t] = pix < PQ;
        const int p = live[t] ? pix / d.Q : 0, q = live[t] ? pix - p * d.Q : 0;
        ih0[t] = p * d.sh - d.ph;
        iw0[t] = q * d.sw - d.pw;
    }
    float acc[TP][TK];
#pragma unroll
    for (int t = 0; t < TP; ++t)
#pragma unroll
        for (int j = 0; j < TK; ++j) acc[t][j] = 0.f;
    const T *xb = x + ((size_t)img * d.C + (size_t)grp * d.Cg) * HW;
    const size_t wk = (size_t)d.Cg * RS;
    for (int c0 = 0; c0 < d.Cg; c0 += CC) {
        const int ccn = min(CC, d.Cg - c0);
        __syncthreads();
        // stage taps: element i -> (idx = i / TK, j = i % TK), lds[idx * TK + j] = w[k0 + j][c0*RS + idx]
        const float *wb = w + (size_t)k0 * wk + (size_t)c0 * RS;
        for (int i = threadIdx.x; i < ccn * RS * TK; i += blockDim.x) lds[i] = wb[(size_t)(i % TK) * wk + i / TK];
        __syncthreads();
        for (int cc = wave; cc < ccn; cc += CS) {
            const T *xc = xb + (size_t)(c0 + cc) * HW;
            const float *wl = lds + cc * RS * TK;
#pragma unroll 1
            for (int r = 0; r < R; ++r) {
#pragma unroll
                for (int s = 0; s < S; ++s) {
                    float xv[TP];
#pragma unroll
                    for (int t = 0; t < TP; ++t) {
                        const int ih = ih0[t] + r, iw = iw0[t] + s;
                        const bool ok = live[t] && ih >= 0 && ih < d.H && iw >= 0 && iw < d.W;
                        xv[t] = ok ? ld<T>(xc, (size_t)ih * d.W + iw) : 0.f;
                    }
                    const float4 *w4 = reinterpret_cast<const float4 *>(wl + (r * S + s) * TK);
#pragma unroll
                    for (int j4 = 0; j4 < TK / 4; ++j4) {
                        const float4 wv = w4[j4];
#pragma unroll
                        for (int t = 0; t < TP; ++t) {
                            acc[t][j4 * 4 + 0] = fmaf(xv[t], wv.x, acc[t][j4 * 4 + 0]);
                            acc[t][j4 * 4 + 1] = fmaf(xv[t], wv.y, acc[t][j4 * 4 + 1]);
                            acc[t][j4 * 4 + 2] = fmaf(xv[t], wv.z, acc[t][j4 * 4 + 2]);
                            acc[t][j4 * 4 + 3] = fmaf(xv[t], wv.w, acc[t][j4 * 4 + 3]);
                        }
                    }
                }
            }
        }
    }
    // sum the CS partial tiles: red[(wave * TP*TK + o) * 64 + lane]
    __syncthreads();
    if (CS > 1) {
#pragma unroll
        for (int t = 0; t < TP; ++t)
#pragma unroll
            for (int j = 0; j < TK; ++j) lds[((wave * TP + t) * TK + j) * 64 + lane] = acc[t][j];
        __syncthreads();
    }
    for (int o = wave; o < TP * TK; o += CS) {
        const int t = o / TK, j = o - t * TK;
        float v = 0.f;
        if (CS > 1) {
            for (int ws = 0; ws < CS; ++ws) v += lds[(ws * TP * TK + o) * 64 + lane];
        } else {
            // single wavefront: pick acc[t][j] without dynamic register indexing
#pragma unroll
            for (int tt = 0; tt < TP; ++tt)
#pragma unroll
                for (int jj = 0; jj < TK; ++jj)
                    if (tt == t && jj == j) v = acc[tt][jj];
        }
        const int pix = (blockIdx.x * 64 + lane) * TP + t;
        if (pix < PQ) st<T>(y, ((size_t)img * d.K + k0 + j) * PQ + pix, act(v + (bias ? bias[k0 + j] : 0.f), d.relu));
    }
}

// Direct convolution, lean form for groups == 1 and 3x3 / 1x1 filters: a lane owns one output
// pixel and TK output channels; the CS wavefronts of a block split the input channels.  The
// filter taps of a wavefront are uniform, so they are read straight from the raw OIHW tensor
// into scalar registers (scalar cache; nine consecutive floats per output and input channel)
// and feed the FMAs as scalar operands: no LDS staging, no barrier in the channel loop.  x comes
// through buffer loads with one hoisted byte offset per tap (out of range in the zero padding).
//
// GRID8 (3x3, stride 1, input planes up to 7x7: the last stage of an ImageNet CNN).  There the
// nine pixel loads per channel, not the FMAs, set the time (measured: the kernel with its FMAs
// cut to a ninth runs as long as the full one).  The 64 lanes form an 8x8 grid that holds the
// whole plane, fetched by ONE load per channel, and every lane takes its eight neighbours from
// the other lanes with ds_bpermute (a register crossbar, no memory).  Row 7 and column 7 of the
// grid hold zeros, and because lane indices wrap modulo 64 they serve as the zero padding on
// all four sides.  (Cutting larger planes into 6x6-output tiles with an 8x8 halo patch was
// measured too and loses: 36 useful lanes of 64 cost more than the loads save.)
// lblk: the workgroup's logical block (image, pixel group, output-channel group); CS: its wavefronts
template <typename T, int TK, int FS, bool GRID8 = false>
__device__ __forceinline__ void direct_slane_block(const T *__restrict__ x, const float *__restrict__ w,
                                                   const float *__restrict__ bias, T *__restrict__ y,
                                                   const DirectParams &d, const int lblk, const int CS, float *lds) {
    constexpr int ESZ = sizeof(T);
    constexpr int RS = FS * FS;
    const int lane = threadIdx.x & 63;
    const int wave = CS == 1 ? 0 : __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // CS == 1: the wavefront works alone, wherever it sits in the workgroup
    const int PQ = d.P * d.Q, HW = d.H * d.W;
    const int img = lblk / (d.grid_nx * d.grid_ny), l2 = lblk - img * (d.grid_nx * d.grid_ny);
    const int bx = d.k_major ? l2 % d.grid_nx : l2 / d.grid_ny;
    const int by = d.k_major ? l2 / d.grid_nx : l2 % d.grid_ny;
    const int k0 = by * TK;
    int pix;
    bool live;
    uint32_t voff[GRID8 ? 1 : RS];
    int nb[GRID8 ? RS : 1];       // GRID8: byte index (lane * 4) of the lane that holds tap (r, s)
    if constexpr (GRID8) {
        // lane (gy, gx) holds x[gy][gx] (zero beyond the plane) and computes output (gy, gx); tap
        // (r, s) of that output is x[gy - pad_h + r][gx - pad_w + s], i.e. the lane 8 (r - pad_h) +
        // (s - pad_w) further on, modulo 64
        const int gy = lane >> 3, gx = lane & 7;
        const bool ok = gy < d.H && gx < d.W;
        voff[0] = ok ? (uint32_t)((gy * d.W + gx) * ESZ) : kOobOffset;
#pragma unroll
        for (int rs = 0; rs < RS; ++rs) nb[rs] = ((lane + (rs / 3 - d.ph) * 8 + rs % 3 - d.pw) & 63) * 4;
        live = gy < d.P && gx < d.Q;
        pix = gy * d.Q + gx;
    } else {
        pix = bx * 64 + lane;
        live = pix < PQ;
        const int p = live ? pix / d.Q : 0, q = live ? pix - p * d.Q : 0;
#pragma unroll
        for (int r = 0; r < FS; ++r)
#pragma unroll
            for (int s2 = 0; s2 < FS; ++s2) {
                const int ih = p * d.sh - d.ph + r, iw = q * d.sw - d.pw + s2;
                const bool ok = live && (unsigned)ih < (unsigned)d.H && (unsigned)iw < (unsigned)d.W;
                voff[r * FS + s2] = ok ? (uint32_t)((ih * d.W + iw) * ESZ) : kOobOffset;
            }
    }
    const __amdgpu_buffer_rsrc_t xres = make_rsrc(x + (size_t)img * d.C * HW, (uint32_t)((size_t)d.C * HW * ESZ));
    const uint32_t plane = (uint32_t)(HW * ESZ);
    const size_t wk = (size_t)d.C * RS;
    // The taps are wave-uniform and nothing in this kernel writes them: reading them through the
    // constant address space makes them scalar loads whatever the compiler can prove about
    // aliasing (in the many-layer kernel the pointers come out of a table, and it proves nothing).
    typedef const __attribute__((address_space(4))) float *ConstFloatPtr;
    const ConstFloatPtr wrow = (ConstFloatPtr)(uintptr_t)(w + (size_t)k0 * wk);
    float acc[TK];
#pragma unroll
    for (int j = 0; j < TK; ++j) acc[j] = 0.f;
    int c = wave;
    if (FS == 1 && (d.C & 7) == 0) {
        // 1x1 filter: the taps of eight consecutive input channels are contiguous, one
        // eight-dword scalar load per output channel; a wavefront takes channel blocks of 8
        for (int cb = wave * 8; cb < d.C; cb += CS * 8) {
            float xa[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) xa[i] = buf_load_x<T>(xres, voff[0], (uint32_t)(cb + i) * plane);
#pragma unroll
            for (int j = 0; j < TK; ++j)
#pragma unroll
                for (int i = 0; i < 8; ++i) acc[j] = fmaf(xa[i], wrow[j * wk + cb + i], acc[j]);
        }
        c = d.C;
    }
    // two channels per iteration: the loads of both are issued before the FMAs of the first
    // (large filters: one channel at a time, their taps alone fill the registers)
    // pixels of the RS taps of channel cc: RS loads, or one load and RS - 1 lane exchanges
    auto load_pixels = [&](float (&xv)[RS], int cc) __attribute__((always_inline)) {
        if constexpr (GRID8) {
            const float own = buf_load_x<T>(xres, voff[0], (uint32_t)cc * plane);
#pragma unroll
            for (int i = 0; i < RS; ++i)
                xv[i] = __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute(nb[i], __builtin_bit_cast(int, own)));
        } else {
#pragma unroll
            for (int i = 0; i < RS; ++i) xv[i] = buf_load_x<T>(xres, voff[i], (uint32_t)cc * plane);
        }
    };
    for (; FS <= 3 && c + CS < d.C; c += 2 * CS) {
        float xa[RS], xb[RS];
        load_pixels(xa, c);
        load_pixels(xb, c + CS);
        const ConstFloatPtr wa = wrow + (size_t)c * RS, wb = wrow + (size_t)(c + CS) * RS;
#pragma unroll
        for (int j = 0; j < TK; ++j)
#pragma unroll
            for (int i = 0; i < RS; ++i) acc[j] = fmaf(xa[i], wa[j * wk + i], acc[j]);
#pragma unroll
        for (int j = 0; j < TK; ++j)
#pragma unroll
            for (int i = 0; i < RS; ++i) acc[j] = fmaf(xb[i], wb[j * wk + i], acc[j]);
    }
    for (; c < d.C; c += CS) {
        float xa[RS];
        load_pixels(xa, c);
        const ConstFloatPtr wa = wrow + (size_t)c * RS;
#pragma unroll
        for (int j = 0; j < TK; ++j)
#pragma unroll
            for (int i = 0; i < RS; ++i) acc[j] = fmaf(xa[i], wa[j * wk + i], acc[j]);
    }
    // sum the CS partial results: red[(wave * TK + j) * 64 + lane], fixed order
    if (CS > 1) {
#pragma unroll
        for (int j = 0; j < TK; ++j) lds[(wave * TK + j) * 64 + lane] = acc[j];
        __syncthreads();
    }
    for (int j = wave; j < TK; j += CS) {
        float v = 0.f;
        if (CS > 1) {
            for (int ws = 0; ws < CS; ++ws) v += lds[(ws * TK + j) * 64 + lane];
        } else {
#pragma unroll
            for (int jj = 0; jj < TK; ++jj)
                if (jj == j) v = acc[jj];
        }
        if (live) st<T>(y, ((size_t)img * d.K + k0 + j) * PQ + pix, act(v + (bias ? bias[k0 + j] : 0.f), d.relu));
    }
}

template <typename T, int TK, int FS, bool GRID8 = false>
__global__ __launch_bounds__(1024) void direct_conv_slane_kernel(const T *__restrict__ x, const float *__restrict__ w,
                                                                 const float *__restrict__ bias, T *__restrict__ y,
                                                                 const DirectParams d) {
    extern __shared__ __align__(16) float lds[];
    // XCD-aware block order: an XCD gets a contiguous range of output-channel groups (deep layers,
    // filters dominate the traffic) or of pixel groups (shallow layers, x dominates)
    const int lblk = xcd_logical_tile(d.grid_nx * d.grid_ny * d.N);
    if (lblk < 0) return;
    direct_slane_block<T, TK, FS, GRID8>(x, w, bias, y, d, lblk, blockDim.x >> 6, lds);
}

// ---- 3x3 and 1x1 (stride 1 or 2) and 7x7 (stride 2) layers with the lanes along the output channels
// (float32 arithmetic; x and y in float32 or float16, the weights are the raw float32 tensor)
//
// lane = output channel (64 per wavefront), tile = TR output rows x TW columns held as TR * TW
// accumulators per lane.  The two operands swap roles against the kernel above.
//
// Pixels.  Every lane needs the same pixels, so they must arrive as uniform operands.  The patch of
// a tile (NR rows x NPX columns of one channel) is fetched by vector loads with the lanes along
// the patch (flattened over ceil(NR NPX / 64) loads, zero outside the plane through the range
// check of the buffer), written to an LDS slot of the wavefront and read back with uniform
// addresses, 16 bytes at a time: every lane then holds the same four pixels in vector registers.
// The LDS pipe runs beside the vector ALU (sixteen such reads next to 48 FMAs cost nothing,
// measured) and a wavefront's LDS operations complete in order, so there is no barrier in the
// channel loop.  Ways of feeding the pixels that were measured and dropped: through the scalar
// cache as FMA scalar operands (rows of 16 by scalar loads: fine for deep layers, but on planes
// of 56 x 56 and more every row load misses the scalar cache and the wavefronts mostly wait;
// 525 against 421 us on a VGG-16-shaped stack, 84 against 77 us on a ResNet-18-shaped one; at
// stride 2 a scalar row load pays for at most 36 FMAs), held once per quad of lanes and
// broadcast by a DPP operand on the FMA (DPP FMAs issue at about half rate), and v_readlane into
// scalar registers (one v_readlane costs the issue time of four FMAs).
//
// Taps.  A lane needs the taps of its own output channel, and the 64 filters of a block lie
// C * FS * FS * 4 bytes apart: fetched per lane, every load instruction touches 64 cache lines, and
// with such loads the deep layers are bound by the address path of the CU.  3x3: the wavefront
// fetches the taps of two channels (72 contiguous bytes per filter) as they lie in memory, 8 bytes
// per lane and 7 filters per instruction, copies them to its LDS region as they come (filter k at
// byte 72 k) and every lane reads its filter back: ten loads that touch some ten lines each
// instead of five that touch 64.  The fetch for the next pair of channels is issued before this
// pair is computed, the copy to LDS sits between its two channels, the read after them.  7x7 layers with at most four
// input channels (a stem): the 64 whole filters of the workgroup are staged once in LDS, row
// stride odd, and read back a channel at a time.
//
// The cs wavefronts of a tile split the channels; partial sums meet in LDS, one output row of the
// tile per pass, in a fixed order, and the store runs with the columns fastest over the lanes.
constexpr int kKlWaves = 8;                 // wavefronts per workgroup (16, with a 16-way channel split for the deepest layers, was measured: slower on every stack)
constexpr int kTapRegion = 64 * 20;         // LDS floats of a wavefront's tap staging area: 3x3: 64 filters x 2 channels x 9 taps and the overrun of the last copy (1264); 1x1: 64 filters x 16 channels, row stride 20
constexpr int kKlStagedMaxC = 4;            // whole filters are staged in LDS up to this many input channels
typedef float kl_f4 __attribute__((ext_vector_type(4)));
typedef float kl_f2 __attribute__((ext_vector_type(2)));

struct KLaneLayer {
    const void *x;      // float32 or float16 activations (the kernel's storage type T)
    const float *w, *bias;
    void *y;
    int N, C, H, W, K, P, Q, ph, pw, fs, st;
    int staged;   // 1: whole filters in LDS (7x7, C <= kKlStagedMaxC), 0: taps of two (3x3, C a multiple of 4) or sixteen (1x1, C a multiple of 16) channels at a time
    int tw;       // tile width: 14, or 7 for a 3x3 layer whose Q is an odd multiple of 7 (the last tile of a row may be ragged)
    int tr;       // tile rows: 2 at stride 1, 1 at stride 2
    int nseg;     // ceil(Q / tw)
    int ntile;    // nseg * ceil(P / tr)
    int cs;       // wavefronts per tile (1, 2, 4 or 8): each takes C / cs channels, a multiple of 4 (3x3) or 16 (1x1); staged: 1
    int wgt;      // workgroups per (image, block of 64 output channels) = ceil(ntile / (kKlWaves / cs))
    int ts;       // staged: row stride (floats) of the filters in LDS, odd
    int relu;
};
// tile geometry of a layer (the same arithmetic sizes the launch on the host and places a workgroup on the device)
__host__ __device__ static inline void klane_geometry(KLaneLayer &L) {
    L.staged = L.fs == 7;
    L.tw = (L.fs <= 3 && L.Q % 7 == 0 && L.Q % 14 != 0) ? 7 : 14;
    // two output rows per tile at stride 1: a tap then feeds twice the FMAs.  (One-row tiles for the
    // 512-channel layers on 7 x 7 planes, whose 256 long wavefronts end a launch of small layers, were
    // measured: 82 against 76 us; two pairs of taps in flight instead of one changed nothing.)
    L.tr = L.st == 1 ? 2 : 1;
    L.nseg = (L.Q + L.tw - 1) / L.tw;
    L.ntile = L.nseg * ((L.P + L.tr - 1) / L.tr);
    int cs = 1;
    if (!L.staged) {
        // 3x3: about 32 channels per wavefront (measured against 16 and 64 at stride 1, 8 and 64 at stride 2); 1x1: 128
        cs = L.C / (L.fs == 3 ? 32 : 128);
        cs = cs >= 8 ? 8 : cs >= 4 ? 4 : cs >= 2 ? 2 : 1;
        while (cs > 1 && L.C % ((L.fs == 3 ? 4 : 16) * cs) != 0) cs >>= 1;
    }
    L.cs = cs;
    L.wgt = (L.ntile + kKlWaves / cs - 1) / (kKlWaves / cs);
    L.ts = (L.C * L.fs * L.fs) | 1;
}
__host__ __device__ static inline int klane_blocks(const KLaneLayer &L) { return L.wgt * (L.K / 64) * L.N; }
// LDS floats in front of the output rows (the staged filters)
__host__ __device__ static inline int klane_filter_floats(const KLaneLayer &L) { return L.staged ? 64 * L.ts : 0; }
// LDS floats of a workgroup: staged: [filters][output rows, 14 x 65 per wavefront][pixel slots]; else
// [a region of kTapRegion floats per wavefront: its tap staging area in the channel loop, its output rows afterwards][pixel slots];
// two pixel slots of 256 floats per wavefront
__host__ __device__ static inline int klane_lds_floats(const KLaneLayer &L) {
    return L.staged ? klane_filter_floats(L) + kKlWaves * (14 * 65 + 256) : kKlWaves * (kTapRegion + 512);
}

// One channel of a tile: the wavefront's patch (NR rows x NPX columns, flat index f = row * NPX +
// column) lies in its LDS slot; it is read back kKlChunk pixels at a time with uniform addresses and
// each pixel feeds the FMAs of the outputs it belongs to:
// acc[orow][q] += pixel(orow * ST + dr, q * ST + sx) * t[dr][sx].
// The chunks rotate over kKlSets register sets and the reads run up to kKlDepth chunks ahead of the
// FMAs: a wavefront alternates between few FMAs and an LDS round trip, and with one chunk in flight
// a chunk took as long as the round trip whatever its FMAs.
// PAR: the set of this channel's first chunk (a constant once the caller's loop is unrolled).  PRE:
// the first klane_depth chunks are in their registers already (the previous channel fetched them
// from `slot`); next: where the next channel's patch lies, or null -- its first chunks are then
// fetched beside the last FMAs of this channel.
constexpr int kKlChunk = 8, kKlSets = 4, kKlDepth = 3;
template <int FS, int ST, int TW, int TR> constexpr int klane_chunks() { return (((TR - 1) * ST + FS) * ((TW - 1) * ST + FS) + kKlChunk - 1) / kKlChunk; }
template <int FS, int ST, int TW, int TR> constexpr int klane_depth() { return klane_chunks<FS, ST, TW, TR>() < kKlDepth ? klane_chunks<FS, ST, TW, TR>() : kKlDepth; }
typedef kl_f4 KlPixels[kKlSets][kKlChunk / 4];
template <int FS, int ST, int TW, int TR>
__device__ __forceinline__ void klane_read_chunk(const float *from, const int ch, const int set, KlPixels &px) {
    constexpr int NF = ((TR - 1) * ST + FS) * ((TW - 1) * ST + FS);
#pragma unroll
    for (int m = 0; m < kKlChunk / 4; ++m)
        if (kKlChunk * ch + 4 * m < NF) px[set][m] = *reinterpret_cast<const kl_f4 *>(from + kKlChunk * ch + 4 * m);
}
// the first chunks of the first channel of a loop (sets 0 ..)
template <int FS, int ST, int TW, int TR>
__device__ __forceinline__ void klane_preload(const float *slot, KlPixels &px) {
#pragma unroll
    for (int d = 0; d < klane_depth<FS, ST, TW, TR>(); ++d) klane_read_chunk<FS, ST, TW, TR>(slot, d, d, px);
}
template <int FS, int ST, int TW, int TR, bool PRE>
__device__ __forceinline__ void klane_channel(const float *slot, const float *next, const float (&t)[FS * FS], float (&acc)[TR * TW],
                                              KlPixels &px, const int PAR) {
    constexpr int NR = (TR - 1) * ST + FS, NPX = (TW - 1) * ST + FS, NF = NR * NPX;
    constexpr int CP = kKlChunk, NCH = klane_chunks<FS, ST, TW, TR>(), D = klane_depth<FS, ST, TW, TR>();
    static_assert(D + 1 <= kKlSets, "the chunk in use and the chunks in flight have a register set each");
    if (!PRE) {
#pragma unroll
        for (int d = 0; d < D; ++d) klane_read_chunk<FS, ST, TW, TR>(slot, d, (PAR + d) % kKlSets, px);
    }
#pragma unroll
    for (int ch = 0; ch < NCH; ++ch) {
        const int cur = (PAR + ch) % kKlSets, nx = ch + D;
        if (nx < NCH) klane_read_chunk<FS, ST, TW, TR>(slot, nx, (PAR + nx) % kKlSets, px);
        else if (next) klane_read_chunk<FS, ST, TW, TR>(next, nx - NCH, (PAR + nx) % kKlSets, px);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int e = 0; e < CP; ++e) {
            const int f = CP * ch + e;
            if (f >= NF) continue;
            const int r = f / NPX, i = f - r * NPX;
            const float v = px[cur][e >> 2][e & 3];
#pragma unroll
            for (int dr = 0; dr < FS; ++dr) {
                const int ro = r - dr;
                if (ro < 0 || ro % ST != 0 || ro / ST >= TR) continue;
#pragma unroll
                for (int sx = 0; sx < FS; ++sx) {
                    const int d = i - sx;
                    if (d < 0 || d % ST != 0 || d / ST >= TW) continue;
                    acc[(ro / ST) * TW + d / ST] = fmaf(v, t[dr * FS + sx], acc[(ro / ST) * TW + d / ST]);
                }
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    }
}

template <typename T, int FS, int ST, int TW, int TR, bool STAGED>
__device__ __forceinline__ void klane_tile(const KLaneLayer &L, const int lblk, float *lds) {
    constexpr int ESZ = sizeof(T);
    static_assert(STAGED || FS == 3 || FS == 1, "taps of a few channels at a time: 3x3 and 1x1");
    constexpr int NR = (TR - 1) * ST + FS, NPX = (TW - 1) * ST + FS, NF = NR * NPX, NLD = (NF + 63) / 64;
    static_assert(NLD * 64 <= 256, "pixel slot");
    KlPixels px;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int KB = L.K >> 6;
    // (the divisions run on the vector unit: the results are uniform and go back to scalar registers)
    const int tg = lblk % L.wgt, rest = lblk / L.wgt;
    const int img = __builtin_amdgcn_readfirstlane(rest / KB), kb = rest - img * KB;
    const int tile = __builtin_amdgcn_readfirstlane(tg * (kKlWaves / L.cs) + wave / L.cs);
    const int cw = __builtin_amdgcn_readfirstlane(wave % L.cs), w0 = wave - cw;
    const bool live = tile < L.ntile;
    const int rp = __builtin_amdgcn_readfirstlane(tile / L.nseg), seg = tile - rp * L.nseg;
    const int p0 = rp * TR, q0 = seg * TW;
    const int HW = L.H * L.W;
    constexpr int OWS = STAGED ? 14 * 65 : kTapRegion;       // floats from one wavefront's output rows to the next one's
    float *out = lds + klane_filter_floats(L);
    float *slot = out + kKlWaves * OWS + wave * (STAGED ? 256 : 512);      // two pixel slots of 256 floats: this channel's patch and the next one's
    // the lane's pixels in the NLD loads of a channel (1x1: a load holds two channels, 32 lanes each)
    constexpr int LPC = FS == 1 ? 32 : 64;
    static_assert(FS != 1 || NF <= 32, "two channels per pixel load");
    uint32_t voff[NLD];
#pragma unroll
    for (int j = 0; j < NLD; ++j) {
        const int f = j * 64 + (lane & (LPC - 1));
        const int r = f / NPX, i = f - r * NPX;
        const int ih = ST * p0 - L.ph + r, iw = ST * q0 - L.pw + i;
        const bool ok = live && f < NF && ih >= 0 && ih < L.H && iw >= 0 && iw < L.W;
        voff[j] = ok ? (uint32_t)(((lane / LPC) * HW + ih * L.W + iw) * ESZ) : kOobOffset;
    }
    const __amdgpu_buffer_rsrc_t xres = make_rsrc(static_cast<const T *>(L.x) + (size_t)img * L.C * HW, (uint32_t)((size_t)L.C * HW * ESZ));
    const uint32_t plane = (uint32_t)(HW * ESZ);
    float acc[TR * TW];
#pragma unroll
    for (int q = 0; q < TR * TW; ++q) acc[q] = 0.f;
    if constexpr (!STAGED && FS == 1) {
        if (live) {
            // taps of 16 channels (64 contiguous bytes per filter) at a time: 16 bytes per lane, 16 filters
            // per instruction, copied to LDS with a row stride of 20 floats (the 16-byte reads of
            // eight neighbouring lanes then cover all banks), read back by the filter's lane
            const uint32_t rowbytes = (uint32_t)L.C * 4u;
            const __amdgpu_buffer_rsrc_t wres = make_rsrc(L.w, (uint32_t)((size_t)L.K * rowbytes));
            const uint32_t tvoff = (uint32_t)(kb * 64 + (lane >> 2)) * rowbytes + (uint32_t)(lane & 3) * 16u;
            float *stage = out + wave * OWS;
            auto tap_fetch = [&](kl_f4 (&tmp)[4], uint32_t c) __attribute__((always_inline)) {
#pragma unroll
                for (int it = 0; it < 4; ++it)
                    tmp[it] = __builtin_bit_cast(kl_f4, __builtin_amdgcn_raw_buffer_load_b128(wres, tvoff, c * 4u + (uint32_t)(it * 16) * rowbytes, 0));
            };
            auto tap_copy = [&](const kl_f4 (&tmp)[4]) __attribute__((always_inline)) {
#pragma unroll
                for (int it = 0; it < 4; ++it) *reinterpret_cast<kl_f4 *>(stage + (it * 16 + (lane >> 2)) * 20 + (lane & 3) * 4) = tmp[it];
            };
            auto tap_take = [&](float (&t)[16]) __attribute__((always_inline)) {
#pragma unroll
                for (int m = 0; m < 4; ++m) {
                    const kl_f4 v = *reinterpret_cast<const kl_f4 *>(stage + lane * 20 + 4 * m);
                    t[4 * m] = v.x; t[4 * m + 1] = v.y; t[4 * m + 2] = v.z; t[4 * m + 3] = v.w;
                }
            };
            const uint32_t per = (uint32_t)(L.C / L.cs), cbeg = (uint32_t)cw * per, cendx = cbeg + per;
            // pixels of four channel pairs in flight (register j: channels c16 + 2 j and + 1; the eight pairs
            // of a group alternate over the registers); requests in a pinned order as below
            kl_f4 tmp[4];
            float t[16];
            tap_fetch(tmp, cbeg);
            float R[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                __builtin_amdgcn_sched_barrier(0);
                R[j] = buf_load_x<T>(xres, voff[0], (cbeg + 2 * j) * plane);
            }
            __builtin_amdgcn_sched_barrier(0);
            tap_copy(tmp);
            tap_take(t);
            // A pair's pixels go to LDS one pair ahead (two slots of 64 floats alternate) and a channel's
            // first chunk is read beside the last FMAs of the channel before it.
            constexpr int NCH = klane_chunks<1, ST, TW, TR>();
            static_assert((2 * NCH) % kKlSets == 0, "every pair starts with register set 0");
            slot[lane] = R[0];
            R[0] = buf_load_x<T>(xres, voff[0], min(cbeg + 8, cendx - 2) * plane);
            klane_preload<1, ST, TW, TR>(slot, px);
            for (uint32_t c16 = cbeg; c16 < cendx; c16 += 16) {
                // (the last group fetches itself again: in range, never used)
                tap_fetch(tmp, min(c16 + 16, cendx - 16));
#pragma unroll
                for (int jp = 0; jp < 8; ++jp) {
                    const int jn = (jp + 1) & 3;
                    float *cur = slot + (jp & 1) * 64, *nslot = slot + ((jp + 1) & 1) * 64;
                    nslot[lane] = R[jn];                     // the next pair (past the end: the last pair again)
                    const uint32_t cn = min(c16 + 2 * jp + 10, cendx - 2);
                    R[jn] = buf_load_x<T>(xres, voff[0], cn * plane);
                    const float t0[1] = {t[2 * jp]}, t1[1] = {t[2 * jp + 1]};
                    klane_channel<1, ST, TW, TR, true>(cur, cur + 32, t0, acc, px, 0);
                    klane_channel<1, ST, TW, TR, true>(cur + 32, nslot, t1, acc, px, NCH % kKlSets);
                    // (the accumulators are pinned here: left alone, the compiler sinks the FMAs of many
                    // channels below their LDS reads and parks the pixels in scratch memory meanwhile)
#pragma unroll
                    for (int q = 0; q < TR * TW; ++q) asm volatile("" : "+v"(acc[q]));
                    if (jp == 3) tap_copy(tmp);
                }
                tap_take(t);
            }
        }
    } else if constexpr (!STAGED) {
        if (live) {
            const uint32_t rowbytes = (uint32_t)L.C * 36u;
            const __amdgpu_buffer_rsrc_t wres = make_rsrc(L.w, (uint32_t)((size_t)L.K * rowbytes));
            const uint32_t fbase = (uint32_t)(kb * 64) * rowbytes;
            // lane -> (filter lane / 9 of the seven an instruction fetches, 8-byte piece lane % 9); lane 63 idle
            const uint32_t tvoff = lane < 63 ? fbase + (uint32_t)(lane / 9) * rowbytes + (uint32_t)(lane % 9) * 8u : kOobOffset;
            const uint32_t tvoff_last = lane < 9 ? fbase + (uint32_t)lane * 8u : kOobOffset;     // filter 63
            kl_f2 *stage = reinterpret_cast<kl_f2 *>(out + wave * OWS);
            // (the scalar offset is not part of the range check of a buffer load: it stays inside the tensor)
            auto tap_fetch = [&](kl_f2 (&tmp)[10], uint32_t c) __attribute__((always_inline)) {
#pragma unroll
                for (int it = 0; it < 9; ++it)
                    tmp[it] = __builtin_bit_cast(kl_f2, __builtin_amdgcn_raw_buffer_load_b64(wres, tvoff, c * 36u + (uint32_t)(it * 7) * rowbytes, 0));
                tmp[9] = __builtin_bit_cast(kl_f2, __builtin_amdgcn_raw_buffer_load_b64(wres, tvoff_last, c * 36u + 63u * rowbytes, 0));
            };
            // (no lane is masked: lane 63 of a copy writes what lane 0 of the next one overwrites, LDS
            // operations of a wavefront complete in order, and the last copy runs 55 pairs past filter 63)
            auto tap_copy = [&](const kl_f2 (&tmp)[10]) __attribute__((always_inline)) {
#pragma unroll
                for (int it = 0; it < 10; ++it) stage[it * 63 + lane] = tmp[it];
            };
            auto tap_take = [&](float (&t)[18]) __attribute__((always_inline)) {
#pragma unroll
                for (int m = 0; m < 9; ++m) {
                    const kl_f2 v = stage[lane * 9 + m];
                    t[2 * m] = v.x;
                    t[2 * m + 1] = v.y;
                }
            };
            const uint32_t per = (uint32_t)(L.C / L.cs), cbeg = (uint32_t)cw * per, cendx = cbeg + per;
            // pixels of four channels in flight: slot j holds channel c4 + j, refilled with channel
            // c4 + j + 4 once it has gone to LDS (channels past the end re-read the last one: unused).
            // The order of the requests is pinned: the wait in front of a channel's first use then
            // leaves the younger requests in flight.
            kl_f2 tmp[10];
            float t[18];
            tap_fetch(tmp, cbeg);
            float R[4][NLD];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int l = 0; l < NLD; ++l) R[j][l] = buf_load_x<T>(xres, voff[l], (cbeg + j) * plane);
            }
            __builtin_amdgcn_sched_barrier(0);
            tap_copy(tmp);
            tap_take(t);
            // The patch of a channel goes to LDS one channel ahead (the two slots alternate) and its first
            // chunk is read beside the last FMAs of the channel before it.  Slot j & 1 holds channel c4 + j.
            constexpr int NCH = klane_chunks<3, ST, TW, TR>();
#pragma unroll
            for (int l = 0; l < NLD; ++l) slot[l * 64 + lane] = R[0][l];
#pragma unroll
            for (int l = 0; l < NLD; ++l) R[0][l] = buf_load_x<T>(xres, voff[l], min(cbeg + 4, cendx - 1) * plane);
            klane_preload<3, ST, TW, TR>(slot, px);
            for (uint32_t c4 = cbeg; c4 < cendx; c4 += 4) {
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    // (the last pair fetches itself again: in range, never used)
                    tap_fetch(tmp, min(c4 + 2 * h + 2, cendx - 2));
#pragma unroll
                    for (int jj = 0; jj < 2; ++jj) {
                        const int j = 2 * h + jj, jn = (j + 1) & 3;
                        // the next channel's patch (slot jn holds channel c4 + j + 1; past the end: the last channel again)
                        float *nslot = slot + ((j + 1) & 1) * 256;
#pragma unroll
                        for (int l = 0; l < NLD; ++l) nslot[l * 64 + lane] = R[jn][l];
                        const uint32_t cn = min(c4 + j + 5, cendx - 1);
#pragma unroll
                        for (int l = 0; l < NLD; ++l) R[jn][l] = buf_load_x<T>(xres, voff[l], cn * plane);
                        float tj[9];
#pragma unroll
                        for (int i = 0; i < 9; ++i) tj[i] = t[jj * 9 + i];
                        klane_channel<3, ST, TW, TR, true>(slot + (j & 1) * 256, nslot, tj, acc, px, (j * NCH) % kKlSets);
                        // the next pair's taps go to LDS between the two channels (the staging area
                        // holds nothing that is still needed: this pair's taps are in registers)
                        if (jj == 0) tap_copy(tmp);
                    }
                    tap_take(t);
                }
            }
        }
    } else {
        // the workgroup's 64 filters: read as they lie in memory, written with an odd row stride
        // (six requests in flight per thread; filter and position within it advance without a division)
        const int flen = L.C * FS * FS, total = 64 * flen;
        const float *wb = L.w + (size_t)kb * total;
        constexpr int NT = 64 * kKlWaves, UN = 6;
        const int dk = NT / flen, dr = NT - dk * flen;
        int k = threadIdx.x / flen, rem = threadIdx.x - k * flen;
        for (int e0 = threadIdx.x; e0 < total; e0 += NT * UN) {
            float v[UN];
#pragma unroll
            for (int u = 0; u < UN; ++u) v[u] = e0 + u * NT < total ? wb[e0 + u * NT] : 0.f;
#pragma unroll
            for (int u = 0; u < UN; ++u) {
                if (e0 + u * NT < total) lds[k * L.ts + rem] = v[u];
                k += dk;
                rem += dr;
                if (rem >= flen) { rem -= flen; ++k; }
            }
        }
        __syncthreads();
        if (live) {
            const float *mine = lds + lane * L.ts;
            float cur[NLD], nxt[NLD];
#pragma unroll
            for (int l = 0; l < NLD; ++l) nxt[l] = buf_load_x<T>(xres, voff[l], 0u);
            for (int c = 0; c < L.C; ++c) {
#pragma unroll
                for (int l = 0; l < NLD; ++l) cur[l] = nxt[l];
                const uint32_t cn = (uint32_t)min(c + 1, L.C - 1);
#pragma unroll
                for (int l = 0; l < NLD; ++l) nxt[l] = buf_load_x<T>(xres, voff[l], cn * plane);
#pragma unroll
                for (int l = 0; l < NLD; ++l) slot[l * 64 + lane] = cur[l];
                float tc[FS * FS];
#pragma unroll
                for (int i = 0; i < FS * FS; ++i) tc[i] = mine[c * FS * FS + i];
                klane_channel<FS, ST, TW, TR, false>(slot, nullptr, tc, acc, px, 0);
            }
        }
    }
    // Sum over the cs wavefronts of the tile and store, one output row of the tile per pass.  Every
    // wavefront leaves its row as out[wave * OWS + q * 65 + lane]; then the tile's wavefronts share its
    // 64 x TW outputs with the columns running fastest over the lanes, so that a store covers runs of
    // TW consecutive floats of y instead of 64 separate rows (row stride 65: the transposed reads
    // spread over the banks).  Fixed summation order.
    const size_t ybase = ((size_t)img * L.K + (size_t)kb * 64) * L.P * L.Q;
#pragma unroll
    for (int r = 0; r < TR; ++r) {
#pragma unroll
        for (int q = 0; q < TW; ++q) out[wave * OWS + q * 65 + lane] = acc[r * TW + q];
        __syncthreads();
        if (live && p0 + r < L.P) {
            for (int o = cw * 64 + lane; o < 64 * TW; o += L.cs * 64) {
                const int k = o / TW, q = o - k * TW;
                if (q0 + q >= L.Q) continue;
                float v = 0.f;
                for (int ws = 0; ws < L.cs; ++ws) v += out[(w0 + ws) * OWS + q * 65 + k];
                const float b = L.bias ? L.bias[kb * 64 + k] : 0.f;
                st<T>(static_cast<T *>(L.y), ybase + ((size_t)k * L.P + p0 + r) * L.Q + q0 + q, act(v + b, L.relu));
            }
        }
        if (TR > 1) __syncthreads();
    }
}

// ---- many direct-convolution layers (groups 1, square 1x1 / 3x3 / 5x5 / 7x7 filter) in one launch
// of four-wavefront workgroups: a workgroup finds its layer by counting the entries of a prefix
// array it has reached and then runs that layer's block.
struct DirectLayer {
    const void *x;
    const float *w, *bias;
    void *y;
    DirectParams d;
    int variant;        // 8 * (index of the filter size in {1, 3, 5, 7}) + 4 * (8 channels per lane) + 2 * (lane grid), + 32: a block per wavefront; 64: output-channel lanes
};
struct DirectTable {
    DirectLayer layer[kMaxDirectLayers];
    int block0[kMaxDirectLayers];     // first workgroup of each layer, INT_MAX beyond the last
    int nblocks;
};
static_assert(sizeof(DirectTable) <= 4096, "the table is passed by value as the kernel argument");
typedef const __attribute__((address_space(4))) DirectTable *DirectTablePtr;
// A launch runs workgroups of 4 or 16 wavefronts (the wavefronts of a workgroup split the input
// channels): deep layers have few blocks with long channel loops and need the wider split.

// Finds the layer of logical block b in the table and copies its record; returns the index of the block within the layer.
__device__ __forceinline__ int direct_many_lookup(const DirectTablePtr tbl, const int b, DirectLayer &L) {
    int first;
    const int li = table_find<kMaxDirectLayers>(&tbl->block0[0], b, first);
    static_assert(sizeof(DirectLayer) % 4 == 0, "copied word by word");
    const __attribute__((address_space(4))) uint32_t *src = (const __attribute__((address_space(4))) uint32_t *)&tbl->layer[li];
    uint32_t *dst = reinterpret_cast<uint32_t *>(&L);
#pragma unroll
    for (int k = 0; k < (int)(sizeof(DirectLayer) / 4); ++k) dst[k] = src[k];
    return b - first;
}
// groups of 8 consecutive blocks (neighbouring pixel or channel groups of a layer) go to one XCD
__device__ __forceinline__ int direct_many_block() {
    const int i = blockIdx.x, xcd = i & 7, j = i >> 3;
    return ((j >> 3) * 8 + xcd) * 8 + (j & 7);
}

// Layers with the lanes along the pixels.  (Held to 64 registers so that two workgroups of 16
// wavefronts fit a CU, the launch takes as long: every wavefront then takes twice the time.  The
// filters of the deep layers are a stream of scalar-cache misses, and that path is the limit.)
template <typename T>
__global__ __launch_bounds__(1024) void direct_conv_many_kernel(const DirectTable tbl_arg) {
    extern __shared__ __align__(16) float lds[];      // waves x 8 outputs x 64 lanes
    const int waves = blockDim.x >> 6;
    const DirectTablePtr tbl = (DirectTablePtr)__builtin_amdgcn_kernarg_segment_ptr();
    const int b = direct_many_block();
    if (b >= tbl->nblocks) return;
    DirectLayer L;
    int lblk = direct_many_lookup(tbl, b, L);
    const T *x = static_cast<const T *>(L.x);
    T *y = static_cast<T *>(L.y);
    int cs = waves;
    if (L.variant & 32) {
        // a layer with fewer input channels than wavefronts: nothing to split, every wavefront takes a block of its own
        lblk = lblk * waves + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
        cs = 1;
        if (lblk >= L.d.grid_nx * L.d.grid_ny * L.d.N) return;
    }
    switch (L.variant & 31) {
        case 0: direct_slane_block<T, 4, 1>(x, L.w, L.bias, y, L.d, lblk, cs, lds); break;
        case 4: direct_slane_block<T, 8, 1>(x, L.w, L.bias, y, L.d, lblk, cs, lds); break;
        case 8: direct_slane_block<T, 4, 3>(x, L.w, L.bias, y, L.d, lblk, cs, lds); break;
        case 10: direct_slane_block<T, 4, 3, true>(x, L.w, L.bias, y, L.d, lblk, cs, lds); break;
        case 12: direct_slane_block<T, 8, 3>(x, L.w, L.bias, y, L.d, lblk, cs, lds); break;
        case 14: direct_slane_block<T, 8, 3, true>(x, L.w, L.bias, y, L.d, lblk, cs, lds); break;
        case 16: direct_slane_block<T, 4, 5>(x, L.w, L.bias, y, L.d, lblk, cs, lds); break;
        default: direct_slane_block<T, 4, 7>(x, L.w, L.bias, y, L.d, lblk, cs, lds); break;
    }
}

// Output-channel-lane layers (variant 64), kKlWaves wavefronts per workgroup; T: storage type of x and y.
template <typename T>
__global__ __launch_bounds__(1024) void direct_conv_many_klane_kernel(const DirectTable tbl_arg) {
    extern __shared__ __align__(16) float lds[];      // klane_lds_floats of the launch's largest layer
    const DirectTablePtr tbl = (DirectTablePtr)__builtin_amdgcn_kernarg_segment_ptr();
    const int b = direct_many_block();
    if (b >= tbl->nblocks) return;
    DirectLayer L;
    const int lblk = direct_many_lookup(tbl, b, L);
    KLaneLayer K{L.x, L.w, L.bias, L.y, L.d.N, L.d.C, L.d.H, L.d.W, L.d.K,
                 L.d.P, L.d.Q, L.d.ph, L.d.pw, L.d.R, L.d.sh, 0, 0, 0, 0, 0, 0, 0, 0, L.d.relu};
    klane_geometry(K);
    if (K.fs == 7) klane_tile<T, 7, 2, 14, 1, true>(K, lblk, lds);      // (a 7-wide tile of a 7x7 filter would not pay: 19 pixels for 7 outputs)
    else if (K.fs == 1 && K.st == 1 && K.tw == 7) klane_tile<T, 1, 1, 7, 2, false>(K, lblk, lds);
    else if (K.fs == 1 && K.st == 1) klane_tile<T, 1, 1, 14, 2, false>(K, lblk, lds);
    else if (K.fs == 1 && K.tw == 7) klane_tile<T, 1, 2, 7, 1, false>(K, lblk, lds);
    else if (K.fs == 1) klane_tile<T, 1, 2, 14, 1, false>(K, lblk, lds);
    else if (K.st == 1 && K.tw == 7) klane_tile<T, 3, 1, 7, 2, false>(K, lblk, lds);
    else if (K.st == 1) klane_tile<T, 3, 1, 14, 2, false>(K, lblk, lds);
    else if (K.tw == 7) klane_tile<T, 3, 2, 7, 1, false>(K, lblk, lds);
    else klane_tile<T, 3, 2, 14, 1, false>(K, lblk, lds);
}

struct DirectPlan {
    int tk, tp, cs, cc;   // tk == 0: simple kernel
    size_t lds;
};

static DirectPlan plan_direct(const Geo &g) {
    DirectPlan pl{0, 1, 1, 0, 0};
    if (g.kg % 8 != 0) return pl;
    const int RS = g.r * g.s;
    const long PQ = (long)g.p * g.q;
    const int opt[3][2] = {{16, 2}, {16, 1}, {8, 1}};
    long best_waves = -1;
    for (int i = 0; i < 3; ++i) {
        const int tk = opt[i][0], tp = opt[i][1];
        if (g.kg % tk) continue;
        int cs_max = 128 / (tk * tp);
        while (cs_max > 1 && cs_max > g.cg) cs_max /= 2;
        const long base = ((PQ + 64 * tp - 1) / (64 * tp)) * (g.k / tk) * g.n;
        int cs = 1;
        while (cs < cs_max && base * cs < 1024) cs *= 2;
        const long waves = base * cs;
        if (waves >= 1024 || waves > best_waves) {
            pl.tk = tk; pl.tp = tp; pl.cs = cs;
            best_waves = waves;
            if (waves >= 1024) break;
        }
    }
    // channels staged per chunk: a multiple of cs, about 16 KB of taps
    int cc = (4096 / (RS * pl.tk)) / pl.cs * pl.cs;
    if (cc < pl.cs) cc = pl.cs;
    if (cc > g.cg) cc = g.cg;
    pl.cc = cc;
    const size_t wbytes = (size_t)cc * RS * pl.tk * sizeof(float);
    const size_t rbytes = pl.cs > 1 ? (size_t)pl.cs * pl.tp * pl.tk * 64 * sizeof(float) : 0;
    pl.lds = wbytes > rbytes ? wbytes : rbytes;
    // a large filter (e.g. 15x15) does not fit its staged taps into the 64 KiB a workgroup gets
    // without opting in to more: such layers take the plain kernel
    if (pl.lds > 64 * 1024) pl = DirectPlan{0, 1, 1, 0, 0};
    return pl;
}

template <typename T, int TK, int TP>
static void launch_tiled(const Geo &g, const DirectPlan &pl, const DirectParams &d, const T *x, const float *w,
                         const float *bias, T *y, hipStream_t st_) {
    dim3 grid(ceil_div(g.p * g.q, 64 * TP), g.k / TK, g.n);
    dim3 block(64 * pl.cs);
    if (g.r == 3 && g.s == 3)
        hipLaunchKernelGGL((direct_conv_tiled_kernel<T, TK, TP, 3>), grid, block, pl.lds, st_, x, w, bias, y, d, pl.cc);
    else if (g.r == 1 && g.s == 1)
        hipLaunchKernelGGL((direct_conv_tiled_kernel<T, TK, TP, 1>), grid, block, pl.lds, st_, x, w, bias, y, d, pl.cc);
    else
        hipLaunchKernelGGL((direct_conv_tiled_kernel<T, TK, TP, 0>), grid, block, pl.lds, st_, x, w, bias, y, d, pl.cc);
}

// lean scalar-weight kernel: groups 1, square 1x1 / 3x3 / 5x5 / 7x7 filter, K a multiple of 4
static bool slane_supported(const Geo &g) {
    return g.groups == 1 && g.r == g.s && (g.r == 3 || g.r == 1 || g.r == 5 || g.r == 7) && g.k % 4 == 0;
}

template <typename T>
static void launch_slane(const Geo &g, DirectParams d, const T *x, const float *w, const float *bias, T *y,
                         hipStream_t st_) {
    // 3x3 stride-1 layers on planes up to 7x7 take the 8x8 lane grid (one pixel load per channel
    // instead of nine; needs a zero row and column, and pads <= 1 so that taps wrap into them)
    const bool grid8 = g.r == 3 && g.sh == 1 && g.sw == 1 && g.h <= 7 && g.w <= 7 && g.ph <= 1 && g.pw <= 1;
    const long pixw = grid8 ? 1 : ceil_div(g.p * g.q, 64);
    // 8 output channels per lane while that leaves enough blocks, else 4; channel split until about
    // two wavefronts per SIMD exist (measured on ResNet-18-shaped layers)
    int tk = (g.k % 8 == 0 && pixw * (g.k / 8) * g.n >= 160 && g.r <= 3) ? 8 : 4;
    const long base = pixw * (g.k / tk) * g.n;
    int cs = 1;
    while (cs < 16 && base * cs < 2048 && cs * 2 <= g.c) cs *= 2;
    const size_t lds = cs > 1 ? (size_t)cs * tk * 64 * sizeof(float) : 0;
    d.grid_nx = (int)pixw;
    d.grid_ny = g.k / tk;
    d.k_major = (size_t)g.k * g.c * g.r * g.s * 4 >= (size_t)g.c * g.h * g.w * sizeof(T);
    dim3 grid(xcd_grid(d.grid_nx * d.grid_ny * g.n), 1, 1);
    dim3 block(64 * cs);
    if (g.r == 3 && grid8) {
        if (tk == 8) hipLaunchKernelGGL((direct_conv_slane_kernel<T, 8, 3, true>), grid, block, lds, st_, x, w, bias, y, d);
        else hipLaunchKernelGGL((direct_conv_slane_kernel<T, 4, 3, true>), grid, block, lds, st_, x, w, bias, y, d);
    } else if (g.r == 3) {
        if (tk == 8) hipLaunchKernelGGL((direct_conv_slane_kernel<T, 8, 3>), grid, block, lds, st_, x, w, bias, y, d);
        else hipLaunchKernelGGL((direct_conv_slane_kernel<T, 4, 3>), grid, block, lds, st_, x, w, bias, y, d);
    } else if (g.r == 1) {
        if (tk == 8) hipLaunchKernelGGL((direct_conv_slane_kernel<T, 8, 1>), grid, block, lds, st_, x, w, bias, y, d);
        else hipLaunchKernelGGL((direct_conv_slane_kernel<T, 4, 1>), grid, block, lds, st_, x, w, bias, y, d);
    } else if (g.r == 5) {
        hipLaunchKernelGGL((direct_conv_slane_kernel<T, 4, 5>), grid, block, lds, st_, x, w, bias, y, d);
    } else {
        hipLaunchKernelGGL((direct_conv_slane_kernel<T, 4, 7>), grid, block, lds, st_, x, w, bias, y, d);
    }
}

template <typename T>
static hipError_t launch_direct_t(const Geo &g, const T *x, const float *w, const float *bias, T *y, hipStream_t st_) {
    DirectParams d{g.n, g.c, g.h, g.w, g.k, g.r, g.s, g.sh, g.sw, g.ph, g.pw, g.p, g.q, g.cg, g.kg, 0, 0, 0, g.relu};
    if (slane_supported(g)) {
        launch_slane<T>(g, d, x, w, bias, y, st_);
        return hipGetLastError();
    }
    const DirectPlan pl = plan_direct(g);
    if (pl.tk == 16 && pl.tp == 2) launch_tiled<T, 16, 2>(g, pl, d, x, w, bias, y, st_);
    else if (pl.tk == 16) launch_tiled<T, 16, 1>(g, pl, d, x, w, bias, y, st_);
    else if (pl.tk == 8) launch_tiled<T, 8, 1>(g, pl, d, x, w, bias, y, st_);
    else {
        const int pq_blocks = ceil_div(g.p * g.q, 256);
        int kb = 1;
        if (g.kg % 4 == 0) kb = 4;
        else if (g.kg % 2 == 0) kb = 2;
        dim3 grid(pq_blocks, g.k / kb, g.n);
        switch (kb) {
            case 4: hipLaunchKernelGGL((direct_conv_simple_kernel<T, 4>), grid, dim3(256), 0, st_, x, w, bias, y, d); break;
            case 2: hipLaunchKernelGGL((direct_conv_simple_kernel<T, 2>), grid, dim3(256), 0, st_, x, w, bias, y, d); break;
            default: hipLaunchKernelGGL((direct_conv_simple_kernel<T, 1>), grid, dim3(256), 0, st_, x, w, bias, y, d); break;
        }
    }
    return hipGetLastError();
}

bool direct_many_supported(const Geo &g) { return slane_supported(g); }

// groups 1, K a multiple of 64; 3x3 at stride 1 or 2 with C a multiple of 4; 1x1 with C a multiple of 16; 7x7 at stride 2
// with at most kKlStagedMaxC channels.  (A 3x3 first layer with three channels through the staged
// path was measured: its 1792 short tiles lengthen the launch of a VGG-16-shaped stack by more
// than the 19 us the layer takes with the lanes along the pixels.)
static bool klane_supported(const Geo &g) {
    if (!(g.groups == 1 && g.r == g.s && g.sh == g.sw && g.k % 64 == 0)) return false;
    if ((size_t)g.c * g.h * g.w * 4 >= (1u << 31) || (size_t)g.k * g.c * g.r * g.s * 4 >= (1ull << 32)) return false;
    if (g.r == 3) return (g.sh == 1 || g.sh == 2) && g.c % 4 == 0;
    if (g.r == 1) return (g.sh == 1 || g.sh == 2) && g.c % 16 == 0;
    return g.r == 7 && g.sh == 2 && g.c <= kKlStagedMaxC;
}
static KLaneLayer klane_layer(const Geo &g) {
    KLaneLayer K{nullptr, nullptr, nullptr, nullptr, g.n, g.c, g.h, g.w, g.k, g.p, g.q, g.ph, g.pw, g.r, g.sh, 0, 0, 0, 0, 0, 0, 0, 0, 0};
    klane_geometry(K);
    return K;
}

// Layers [0, n) (one storage type, n <= kMaxDirectLayers, each direct_many_supported): one launch of
// 8-wavefront workgroups for the layers the output-channel-lane kernel covers and, for the others,
// one launch of 16-wavefront workgroups (the wavefronts of a workgroup split the input channels: a
// deep layer is a chain of scalar-load round trips per wavefront, the wide split shortens it; layers
// with fewer channels than wavefronts run a block per wavefront).  A call without output-channel-lane
// layers splits the others by depth into a launch of 16- and one of 4-wavefront workgroups.  Within
// a launch the longest wavefronts come first.  (All in one launch, dealt out alternately, was
// measured: slower.)
hipError_t launch_direct_many(int n, const Geo *geos, const void *const *x, const void *const *w, const float *const *bias,
                              void *const *y, hipStream_t st_) {
    if (n <= 0) return hipSuccess;
    if (n > kMaxDirectLayers) return hipErrorInvalidValue;
    const bool half = geos[0].dtype == NNV_F16;
    bool any_klane = false;
    for (int i = 0; i < n; ++i) {
        if ((geos[i].dtype == NNV_F16) != half || !slane_supported(geos[i])) return hipErrorInvalidValue;
        any_klane = any_klane || klane_supported(geos[i]);
    }
    // pass 0 / 1: workgroups of 16 / 4 wavefronts; pass 2: output-channel-lane layers, 8 wavefronts
    for (int pass = 0; pass < 3; ++pass) {
        const int waves = pass == 0 ? 16 : pass == 1 ? 4 : kKlWaves;
        int order[kMaxDirectLayers], m = 0;
        long weight[kMaxDirectLayers];        // sort key: about the FMAs of one wavefront
        for (int i = 0; i < n; ++i) {
            const Geo &g = geos[i];
            int p;
            if (klane_supported(g)) p = 2;
            else if (any_klane) p = 0;      // what is left are few layers of short work: one launch, and the wide channel split shortens their chains
            else p = g.c > 128 ? 0 : 1;
            if (p != pass) continue;
            order[m++] = i;
            if (klane_supported(g)) {
                const KLaneLayer K = klane_layer(g);
                weight[i] = K.staged ? 0 : (long)(g.c / K.cs) * g.r * g.r * K.tw * K.tr;
            } else {
                weight[i] = (long)(g.c < waves ? g.c : ceil_div(g.c, waves)) * g.r * g.s * ((g.k % 8 == 0 && g.r <= 3) ? 8 : 4);
            }
        }
        if (m == 0) continue;
        std::stable_sort(order, order + m, [&](int a, int b) { return weight[a] > weight[b]; });
        DirectTable tbl{};
        long blocks = 0;
        size_t klane_lds = 0;       // output-channel-lane launch: LDS floats of its largest layout
        for (int o = 0; o < m; ++o) {
            const Geo &g = geos[order[o]];
            const int i = order[o];
            DirectLayer &L = tbl.layer[o];
            L.x = x[i]; L.w = static_cast<const float *>(w[i]); L.bias = bias ? bias[i] : nullptr; L.y = y[i];
            L.d = DirectParams{g.n, g.c, g.h, g.w, g.k, g.r, g.s, g.sh, g.sw, g.ph, g.pw, g.p, g.q, g.cg, g.kg, 0, 0, 0, g.relu};
            tbl.block0[o] = (int)blocks;
            if (pass == 2) {
                const KLaneLayer K = klane_layer(g);
                L.variant = 64;
                blocks += klane_blocks(K);
                klane_lds = std::max<size_t>(klane_lds, (size_t)klane_lds_floats(K));
            } else {
                const bool grid8 = g.r == 3 && g.sh == 1 && g.sw == 1 && g.h <= 7 && g.w <= 7 && g.ph <= 1 && g.pw <= 1;
                const int tk = (g.k % 8 == 0 && g.r <= 3) ? 8 : 4;      // the launch holds plenty of blocks: 8 outputs per loaded pixel
                L.d.grid_nx = grid8 ? 1 : ceil_div(g.p * g.q, 64);
                L.d.grid_ny = g.k / tk;
                L.d.k_major = (size_t)g.k * g.c * g.r * g.s * 4 >= (size_t)g.c * g.h * g.w * (half ? 2 : 4);
                const int fs_index = g.r == 1 ? 0 : g.r == 3 ? 1 : g.r == 5 ? 2 : 3;
                L.variant = 8 * fs_index + 4 * (tk == 8) + 2 * (grid8 ? 1 : 0);
                const long lb = (long)L.d.grid_nx * L.d.grid_ny * g.n;
                if (g.c < waves) {
                    L.variant |= 32;
                    blocks += (lb + waves - 1) / waves;
                } else {
                    blocks += lb;
                }
            }
            if (blocks >= (1L << 30)) return hipErrorInvalidValue;
        }
        for (int o = m; o < kMaxDirectLayers; ++o) tbl.block0[o] = INT_MAX;
        tbl.nblocks = (int)blocks;
        const int per_xcd = ceil_div(ceil_div((int)blocks, 8), 8) * 8;
        const size_t lds = pass == 2 ? klane_lds * sizeof(float) : (size_t)waves * 8 * 64 * sizeof(float);
        if (lds > 64 * 1024) {
            const void *fn = half ? reinterpret_cast<const void *>(direct_conv_many_klane_kernel<__half>) : reinterpret_cast<const void *>(direct_conv_many_klane_kernel<float>);
            hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
        }
        if (pass == 2 && half) hipLaunchKernelGGL(direct_conv_many_klane_kernel<__half>, dim3(per_xcd * 8), dim3(64 * waves), lds, st_, tbl);
        else if (pass == 2) hipLaunchKernelGGL(direct_conv_many_klane_kernel<float>, dim3(per_xcd * 8), dim3(64 * waves), lds, st_, tbl);
        else if (half) hipLaunchKernelGGL(direct_conv_many_kernel<__half>, dim3(per_xcd * 8), dim3(64 * waves), lds, st_, tbl);
        else hipLaunchKernelGGL(direct_conv_many_kernel<float>, dim3(per_xcd * 8), dim3(64 * waves), lds, st_, tbl);
    }
    return hipGetLastError();
}

hipError_t launch_direct(const Geo &g, const void *x, const float *w, const float *bias, void *y, hipStream_t st_) {
    // A layer big enough to fill the chip with output-channel-lane wavefronts runs that kernel by itself
    // (a table of one layer): measured on VGG-16-shaped layers, 1792 wavefronts and more reach 47-56
    // against 36-46 TFLOP/s.  With 448 and fewer (512 channels at 14 x 14, every ResNet-18-shaped layer)
    // the launch lasts as long as one long wavefront, and the lanes along the pixels with the wide
    // channel split are 1.5 to 4 times faster.
    constexpr long min_waves = 1024;
    if (klane_supported(g) && (long)klane_blocks(klane_layer(g)) * kKlWaves >= min_waves) {
        const void *xs[1] = {x}, *ws[1] = {w};
        const float *bs[1] = {bias};
        void *ys[1] = {y};
        return launch_direct_many(1, &g, xs, ws, bias ? bs : nullptr, ys, st_);
    }
    if (g.dtype == NNV_F16)
        return launch_direct_t<__half>(g, static_cast<const __half *>(x), w, bias, static_cast<__half *>(y), st_);
    return launch_direct_t<float>(g, static_cast<const float *>(x), w, bias, static_cast<float *>(y), st_);
}

// ------------------------------------------------------------------ depthwise 3x3 / 5x5

struct DwParams {
    int N, C, H, W, st, ph, pw, P, Q, relu;
};

template <typename T, int FS>
__device__ __forceinline__ void depthwise_block(const T *__restrict__ x, const T *__restrict__ wp,
                                                const float *__restrict__ bias, T *__restrict__ y, const DwParams &d,
                                                const int pqb, const int c, const int img) {
    const int pq = pqb * 256 + threadIdx.x;
    if (pq >= d.P * d.Q) return;
    const int p = pq / d.Q, q = pq - p * d.Q;
    // the channel's taps are uniform over the workgroup: constant address space = scalar loads
    typedef typename std::conditional<sizeof(T) == 2, unsigned short, float>::type Raw;
    typedef const __attribute__((address_space(4))) Raw *ConstTapPtr;
    const ConstTapPtr wc = (ConstTapPtr)(uintptr_t)(wp + (size_t)(c >> 5) * (FS * FS * 32) + (c & 31));
    auto tap = [&](int i) -> float {
        if constexpr (sizeof(T) == 2) return (float)__builtin_bit_cast(_Float16, (unsigned short)wc[i]);
        else return wc[i];
    };
    const T *xc = x + ((size_t)img * d.C + c) * d.H * d.W;
    const int ih0 = p * d.st - d.ph, iw0 = q * d.st - d.pw;
    float acc = bias ? bias[c] : 0.f;
#pragma unroll
    for (int r = 0; r < FS; ++r) {
        const int ih = ih0 + r;
        const bool rok = ih >= 0 && ih < d.H;
#pragma unroll
        for (int s = 0; s < FS; ++s) {
            const int iw = iw0 + s;
            const bool ok = rok && iw >= 0 && iw < d.W;
            const float xv = ok ? ld<T>(xc, (size_t)ih * d.W + iw) : 0.f;
            acc = fmaf(xv, tap((r * FS + s) * 32), acc);
        }
    }
    st<T>(y, ((size_t)img * d.C + c) * d.P * d.Q + pq, act(acc, d.relu));
}

template <typename T, int FS>
__global__ __launch_bounds__(256) void depthwise_kernel(const T *__restrict__ x, const T *__restrict__ wp,
                                                        const float *__restrict__ bias, T *__restrict__ y,
                                                        const DwParams d) {
    depthwise_block<T, FS>(x, wp, bias, y, d, blockIdx.x, blockIdx.y, blockIdx.z);
}

// ---- many depthwise layers in one launch (a MobileNet-style network has 13-17 of them, each a few
// microseconds of work).  y of a layer is one contiguous [N*C][P*Q] array: a thread owns
// kDwPerThread outputs of that flat array (stride 256, so every store of a wavefront is one
// contiguous run whatever the plane size: 7x7 planes fill the lanes like 112x112 ones), finds
// channel and pixel by division, and reads the channel's taps with ordinary (cached) loads.
// Two outputs per thread for 3x3 and one for 5x5 keep the kernel at 8 wavefronts per SIMD: what
// bounds these small layers is how many loads the chip has in flight, not a thread's own pace.
__host__ __device__ constexpr int dw_per_thread(int fs) { return fs == 3 ? 2 : 1; }
struct DwLayer {
    const void *x, *w;
    const float *bias;
    void *y;
    DwParams d;
    int fs;
    int raw;        // w holds the untransformed float32 filters [c][fs * fs] (a depthwise layer run by the direct kind)
};
struct DwTable {
    DwLayer layer[kMaxDwLayers];
    int block0[kMaxDwLayers];     // first workgroup of each layer, INT_MAX beyond the last
    int nblocks;
};
static_assert(sizeof(DwTable) <= 4096, "the table is passed by value as the kernel argument");
typedef const __attribute__((address_space(4))) DwTable *DwTablePtr;

template <typename T, int FS, bool RAW>
__device__ __forceinline__ void depthwise_flat_block(const T *__restrict__ x, const void *__restrict__ wv,
                                                     const float *__restrict__ bias, T *__restrict__ y,
                                                     const DwParams &d, const int blk) {
    constexpr int kDwPerThread = dw_per_thread(FS);
    const int PQ = d.P * d.Q, total = d.N * d.C * PQ;
    int o[kDwPerThread], pq[kDwPerThread], c[kDwPerThread], plane[kDwPerThread];
    float acc[kDwPerThread];
#pragma unroll
    for (int i = 0; i < kDwPerThread; ++i) {
        o[i] = (blk * kDwPerThread + i) * 256 + threadIdx.x;
        const int oo = o[i] < total ? o[i] : 0;
        plane[i] = oo / PQ;                        // image * C + channel
        pq[i] = oo - plane[i] * PQ;
        c[i] = d.N == 1 ? plane[i] : plane[i] % d.C;
        acc[i] = bias ? bias[c[i]] : 0.f;
    }
#pragma unroll
    for (int i = 0; i < kDwPerThread; ++i) {
        const int p = pq[i] / d.Q, q = pq[i] - p * d.Q;
        const T *wc = static_cast<const T *>(wv) + (size_t)(c[i] >> 5) * (FS * FS * 32) + (c[i] & 31);
        const float *wr = static_cast<const float *>(wv) + (size_t)c[i] * (FS * FS);
        const T *xc = x + (size_t)plane[i] * d.H * d.W;
        const int ih0 = p * d.st - d.ph, iw0 = q * d.st - d.pw;
#pragma unroll
        for (int r = 0; r < FS; ++r) {
            const int ih = ih0 + r;
            const bool rok = ih >= 0 && ih < d.H;
#pragma unroll
            for (int s2 = 0; s2 < FS; ++s2) {
                const int iw = iw0 + s2;
                const bool ok = rok && iw >= 0 && iw < d.W;
                const float xv = ok ? ld<T>(xc, (size_t)ih * d.W + iw) : 0.f;
                acc[i] = fmaf(xv, RAW ? wr[r * FS + s2] : ld<T>(wc, (r * FS + s2) * 32), acc[i]);
            }
        }
    }
#pragma unroll
    for (int i = 0; i < kDwPerThread; ++i)
        if (o[i] < total) st<T>(y, (size_t)o[i], act(acc[i], d.relu));
}

template <typename T>
__global__ __launch_bounds__(256) void depthwise_many_kernel(const DwTable tbl_arg) {
    const DwTablePtr tbl = (DwTablePtr)__builtin_amdgcn_kernarg_segment_ptr();
    const int b = blockIdx.x;
    int first;
    const int li = table_find<kMaxDwLayers>(&tbl->block0[0], b, first);
    DwLayer L;
    {
        static_assert(sizeof(DwLayer) % 4 == 0, "copied word by word");
        const __attribute__((address_space(4))) uint32_t *src = (const __attribute__((address_space(4))) uint32_t *)&tbl->layer[li];
        uint32_t *dst = reinterpret_cast<uint32_t *>(&L);
#pragma unroll
        for (int k = 0; k < (int)(sizeof(DwLayer) / 4); ++k) dst[k] = src[k];
    }
    const T *x = static_cast<const T *>(L.x);
    T *y = static_cast<T *>(L.y);
    if (L.raw) {
        if (L.fs == 5) depthwise_flat_block<T, 5, true>(x, L.w, L.bias, y, L.d, b - first);
        else depthwise_flat_block<T, 3, true>(x, L.w, L.bias, y, L.d, b - first);
    } else {
        if (L.fs == 5) depthwise_flat_block<T, 5, false>(x, L.w, L.bias, y, L.d, b - first);
        else depthwise_flat_block<T, 3, false>(x, L.w, L.bias, y, L.d, b - first);
    }
}

hipError_t launch_depthwise_many(int n, const Geo *geos, const void *const *x, const void *const *w, const float *const *bias,
                                 void *const *y, bool raw, hipStream_t st_) {
    if (n <= 0) return hipSuccess;
    if (n > kMaxDwLayers) return hipErrorInvalidValue;
    const bool half = geos[0].dtype == NNV_F16;
    DwTable tbl{};
    long blocks = 0;
    for (int i = 0; i < n; ++i) {
        const Geo &g = geos[i];
        if ((g.dtype == NNV_F16) != half) return hipErrorInvalidValue;
        DwLayer &L = tbl.layer[i];
        L.x = x[i]; L.w = w[i]; L.bias = bias ? bias[i] : nullptr; L.y = y[i];
        L.d = DwParams{g.n, g.c, g.h, g.w, g.sh, g.ph, g.pw, g.p, g.q, g.relu};
        L.fs = g.r;
        L.raw = raw ? 1 : 0;
        tbl.block0[i] = (int)blocks;
        blocks += ((long)g.n * g.c * g.p * g.q + 256 * dw_per_thread(g.r) - 1) / (256 * dw_per_thread(g.r));
        if (blocks >= (1L << 30)) return hipErrorInvalidValue;
    }
    for (int i = n; i < kMaxDwLayers; ++i) tbl.block0[i] = INT_MAX;
    tbl.nblocks = (int)blocks;
    if (half) hipLaunchKernelGGL(depthwise_many_kernel<__half>, dim3((unsigned)blocks), dim3(256), 0, st_, tbl);
    else hipLaunchKernelGGL(depthwise_many_kernel<float>, dim3((unsigned)blocks), dim3(256), 0, st_, tbl);
    return hipGetLastError();
}

hipError_t launch_depthwise(const Geo &g, const void *x, const void *w, const float *bias, void *y, hipStream_t st_) {
    if (g.c > 65535) return hipErrorInvalidValue;
    DwParams d{g.n, g.c, g.h, g.w, g.sh, g.ph, g.pw, g.p, g.q, g.relu};
    dim3 grid(ceil_div(g.p * g.q, 256), g.c, g.n);
    const bool five = g.r == 5;
    if (g.dtype == NNV_F16) {
        auto k = five ? depthwise_kernel<__half, 5> : depthwise_kernel<__half, 3>;
        hipLaunchKernelGGL(k, grid, dim3(256), 0, st_, static_cast<const __half *>(x), static_cast<const __half *>(w), bias,
                           static_cast<__half *>(y), d);
    } else {
        auto k = five ? depthwise_kernel<float, 5> : depthwise_kernel<float, 3>;
        hipLaunchKernelGGL(k, grid, dim3(256), 0, st_, static_cast<const float *>(x), static_cast<const float *>(w), bias,
                           static_cast<float *>(y), d);
    }
    return hipGetLastError();
}

}  // namespace nnv
