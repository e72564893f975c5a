// Implicit im2col GEMM convolution on the matrix cores (the "sgemm" kernel family of
// Table 2 / Fig. 5, including 1x1 pointwise layers):
//     y[k, n] = sum_kk Wp[k, kk] * col[kk, n],  n = (img, p, q),  kk = (c, r, s)
// The col matrix is never materialised: every wavefront gathers its B fragments
// straight from x.
//
// float32: v_mfma_f32_16x16x4_f32.  One k-step = 4 channels at one filter tap (r,s);
//   lane l holds row/column l%16 and channel slot l/16, so the packed weight fragment
//   of a step is 64 consecutive floats (one coalesced 256 B load) and the B fragment is
//   x[c0 + l/16][ih][iw + l%16...] (contiguous along W for stride 1).
// float16: v_mfma_f32_16x16x32_f16.  One k-step = 32 channels at one tap; lane l holds
//   8 consecutive channels (slot group l/16).  For filters larger than 1x1, x is first copied
//   to a channel-last [N][H][W][Cpad32] half buffer in the workspace and both fragments are
//   16-byte loads.  For 1x1 filters (most layers of the bottleneck and inverted-residual
//   networks) that copy would cost a launch of its own, as long as the layer itself: there a
//   lane gathers its 8 channels straight from NCHW with eight 2-byte loads per fragment.
//
// Batch-1 layers put one or two wavefronts on a SIMD, and a lone wavefront issues one
// instruction every four cycles: the k-loop must be almost nothing but loads and MFMAs.
// So all addressing is hoisted: operands come through buffer loads whose hardware range
// check returns 0 for an out-of-range offset; each lane keeps one byte offset per filter
// tap, already set beyond the buffer where the tap falls into the zero padding; the
// channel advance is a scalar offset; fragments of consecutive steps use immediate
// offsets.  A chunk (one channel block x all taps, or 8 channel blocks for 1x1) is loaded
// one chunk ahead of the MFMAs (register ping-pong).  KS wavefronts of a workgroup share one
// output tile and split the channel blocks; partial sums meet in LDS, fixed order.
#include <algorithm>
#include <climits>
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
    int npix;            // N*P*Q
    int K16;             // 16-row panels in all: groups * kg16
    int kg16, Kg, Cg;    // per group: 16-row panels, output channels, input channels (groups == 1: the whole layer)
    int cblocks;         // channel blocks (of 4 float32 / 32 half channels) of one group
    int c_rem;           // float32: C % 4, float16 1x1: C % 32 (channels of the last, partial block; 0 = full)
    uint32_t plane_bytes;   // float16 1x1: bytes of one channel plane of x (H*W*2)
    int ks_shift;        // wavefronts sharing one output tile = 1 << ks_shift
    int cpad;            // channel stride of the half channel-last copy
    uint32_t x_bytes, w_bytes;   // sizes of the x and wp buffers (range-checked loads)
    uint32_t cb_stride;  // bytes between channel blocks in x
    int half_out;
    int relu;              // outputs clamped at zero before the store
    int grid_nx, grid_ny;  // logical grid: tile groups along n, along m
    int m_major;           // 1: consecutive logical tiles walk n first (an XCD keeps few weight panels),
                           // 0: they walk m first (an XCD keeps a pixel range of x)
};

template <bool HALF> struct FragT { typedef float type; };
template <> struct FragT<true> { typedef half8 type; };

// MODE: how the k-steps of a wavefront are grouped into chunks (a chunk is what is loaded ahead)
//   1  1x1 filter: a unit is a channel block, a chunk is 8 units (2 in half precision)
//   3  3x3 filter, float32: a unit = chunk = one channel block, 9 taps, tap offsets loop-invariant
//      3x3 filter, half: row mode (fragments are four registers wide, nine steps do not fit)
//   5,7  filters with S = 5 / 7 (float32): row mode, a unit = chunk = one filter row of a channel block
//   0  anything else: a unit = chunk = one k-step
template <bool HALF, int MODE> struct ModeT {
    static constexpr bool ROW = MODE == 5 || MODE == 7 || (MODE == 3 && HALF);
    static constexpr bool WHOLE3 = MODE == 3 && !HALF;
    static constexpr int UNITS = MODE == 1 ? (HALF ? 2 : 8) : 1;                           // units per chunk
    static constexpr int STEPS = MODE == 0 ? 1 : MODE == 1 ? UNITS : WHOLE3 ? 9 : MODE;    // k-steps per chunk
    static constexpr int NVOFF = (MODE == 0 || MODE == 1) ? 1 : STEPS;                     // tap offsets kept per lane
};

// Output pixels of a wavefront's tile columns: image, position in the P x Q plane, inside the problem or not.
template <int TN> struct PixState {
    int img[TN], pq[TN];
    bool valid[TN];
};

// The k-loop of one wavefront: TM x TN blocks of 16 x 16 outputs (panels mb0.., 16-pixel blocks
// nb0..), summed over the ks-th of nsplit equal ranges of the layer's units.
template <bool HALF, int TM, int TN, int MODE, int NBUF>
__device__ __forceinline__ void gemm_accumulate(const GemmParams &g, const int mb0, const int nb0, const int ks,
                                                const int nsplit, const int lane, floatx4 (&acc)[TM][TN],
                                                PixState<TN> &px) {
    typedef typename FragT<HALF>::type frag_t;
    typedef ModeT<HALF, MODE> MT;
    constexpr int STEPS = MT::STEPS, UNITS = MT::UNITS, NVOFF = MT::NVOFF;
    constexpr bool ROW = MT::ROW, WHOLE3 = MT::WHOLE3;
    constexpr uint32_t FB = sizeof(frag_t);            // bytes per lane of one fragment
    constexpr uint32_t FRAG = 64 * FB;                 // bytes of one fragment
    const int col = lane & 15, slot = lane >> 4;
    const int grp = mb0 / g.kg16;
    const int cbase = grp * g.Cg;                         // first input channel of the group
    const int PQ = g.P * g.Q, RS = g.R * g.S;

    // ---- per-lane pixel state: origin of the patch in x (bytes, may be negative) and tap offsets
    int xbase[TN], ih0[TN], iw0[TN];
    int (&pix_img)[TN] = px.img, (&pix_pq)[TN] = px.pq;
    bool (&pvalid)[TN] = px.valid;
#pragma unroll
    for (int t = 0; t < TN; ++t) {
        const int n = (nb0 + t) * 16 + col;
        pvalid[t] = n < g.npix;
        const int nn = pvalid[t] ? n : 0;
        const int img = g.N == 1 ? 0 : nn / PQ;
        const int pq = nn - img * PQ;
        const int p = pq / g.Q, q = pq - p * g.Q;
        pix_img[t] = img; pix_pq[t] = pq;
        ih0[t] = p * g.sh - g.ph;
        iw0[t] = q * g.sw - g.pw;
        if (HALF && MODE == 1) xbase[t] = (((img * g.C + cbase + slot * 8) * g.H + ih0[t]) * g.W + iw0[t]) * 2;   // NCHW
        else if (HALF) xbase[t] = (((img * g.H + ih0[t]) * g.W + iw0[t]) * g.cpad + cbase + slot * 8) * 2;
        else xbase[t] = (((img * g.C + cbase + slot) * g.H + ih0[t]) * g.W + iw0[t]) * 4;
    }
    const int tap_w = HALF ? g.cpad * 2 : 4;             // bytes per step along s
    const int tap_h = g.W * tap_w;                       // bytes per step along r
    auto tap_off = [&](int t, int r, int s) -> uint32_t {
        const bool ok = pvalid[t] && (unsigned)(ih0[t] + r) < (unsigned)g.H && (unsigned)(iw0[t] + s) < (unsigned)g.W;
        return ok ? (uint32_t)(xbase[t] + r * tap_h + s * tap_w) : kOobOffset;
    };
    // row mode: the column part of the tap offsets (origin + s, or out of range) does not change
    // from chunk to chunk; a chunk's offsets are that plus its row, or out of range for a row in
    // the padding
    uint32_t colv[TN][ROW ? NVOFF : 1];
    if (ROW) {
#pragma unroll
        for (int t = 0; t < TN; ++t)
#pragma unroll
            for (int sx = 0; sx < NVOFF; ++sx)
                colv[t][sx] = (pvalid[t] && (unsigned)(iw0[t] + sx) < (unsigned)g.W) ? (uint32_t)(xbase[t] + sx * tap_w) : kOobOffset;
    }
    // byte offset per tap of the current chunk; loop-invariant for MODE 1 and 3
    uint32_t voff[TN][NVOFF];
    if (MODE == 1) {
#pragma unroll
        for (int t = 0; t < TN; ++t) voff[t][0] = tap_off(t, 0, 0);
    } else if (WHOLE3) {
#pragma unroll
        for (int t = 0; t < TN; ++t)
#pragma unroll
            for (int rs = 0; rs < NVOFF; ++rs) voff[t][rs] = tap_off(t, rs / 3, rs % 3);
    }
    // ---- this wavefront's range of units
    const int nunits = MODE == 0 ? g.cblocks * RS : ROW ? g.cblocks * g.R : g.cblocks;
    const int per_wave = (nunits + nsplit - 1) / nsplit;
    const int u_begin = min(nunits, ks * per_wave);
    const int u_end = min(nunits, u_begin + per_wave);
    const int steps_per_unit = MODE == 0 ? 1 : ROW ? MODE : RS;   // MODE 1: RS == 1
    const uint32_t nsteps_total = (uint32_t)g.cblocks * RS;

    const __amdgpu_buffer_rsrc_t xres = make_rsrc(g.x, g.x_bytes);
    const uint32_t a_lane = lane * FB;
    frag_t a[NBUF][STEPS][TM], b[NBUF][STEPS][TN];

    // Load the chunk starting at unit u (clamped into the range: a chunk past the end re-reads
    // valid data that is never used).  Straight-line code, no branches between the loads.
    // The weight fragments of a chunk are consecutive in memory: they are read through a
    // resource window that starts at the chunk (immediate offsets per step) and ends at the end
    // of the buffer, so a read past this wavefront's range or past the last panel returns
    // data that is not used, or zero, but never faults.
    auto load_chunk = [&](int buf, int u) {
        u = max(min(u, u_end - 1), 0);
#pragma unroll
        for (int m = 0; m < TM; ++m) {
            uint32_t off = ((uint32_t)(mb0 + m) * nsteps_total + (uint32_t)u * steps_per_unit) * FRAG;
            off = min(off, g.w_bytes);        // panels beyond K: empty window, all zeros
            const __amdgpu_buffer_rsrc_t win = make_rsrc(static_cast<const char *>(g.wp) + off, g.w_bytes - off);
#pragma unroll
            for (int j = 0; j < STEPS; ++j) a[buf][j][m] = buf_load<frag_t>(win, a_lane + j * FRAG, 0u);
        }
        if constexpr (MODE == 1 && HALF) {
            // x is NCHW: the lane's 8 channels are 8 planes apart; channels past C (last block)
            // read as zero through an out-of-range offset
#pragma unroll
            for (int j = 0; j < STEPS; ++j) {
                const int cb = min(u + j, u_end - 1);
                const bool part = g.c_rem != 0 && cb == g.cblocks - 1;   // uniform
#pragma unroll
                for (int t = 0; t < TN; ++t) {
                    half8 v;
#pragma unroll
                    for (int i = 0; i < 8; ++i) {
                        uint32_t vo = voff[t][0];
                        if (part) vo = slot * 8 + i < g.c_rem ? vo : kOobOffset;
                        const unsigned short h = __builtin_amdgcn_raw_buffer_load_b16(
                            xres, vo, (uint32_t)cb * g.cb_stride + (uint32_t)i * g.plane_bytes, 0);
                        v[i] = __builtin_bit_cast(_Float16, h);
                    }
                    b[buf][j][t] = v;
                }
            }
        } else if (MODE == 1) {
#pragma unroll
            for (int j = 0; j < STEPS; ++j) {
                const int cb = min(u + j, u_end - 1);
#pragma unroll
                for (int t = 0; t < TN; ++t) b[buf][j][t] = buf_load<frag_t>(xres, voff[t][0], (uint32_t)cb * g.cb_stride);
            }
        } else {
            int cb, r0 = 0, s0 = 0;
            if (WHOLE3) cb = u;
            else if (MODE == 0) { cb = u / RS; const int rs = u - cb * RS; r0 = rs / g.S; s0 = rs - r0 * g.S; }
            else { cb = u / g.R; r0 = u - cb * g.R; }
            if (ROW) {
#pragma unroll
                for (int t = 0; t < TN; ++t) {
                    const bool rok = (unsigned)(ih0[t] + r0) < (unsigned)g.H;
                    const uint32_t radd = (uint32_t)(r0 * tap_h);
#pragma unroll
                    for (int s = 0; s < NVOFF; ++s) voff[t][s] = rok ? colv[t][s] + radd : kOobOffset;   // 2^31 + anything below 2^31 stays out of range
                }
            } else if (MODE == 0) {
#pragma unroll
                for (int t = 0; t < TN; ++t) voff[t][0] = tap_off(t, r0, s0);
            }
            const bool partial = !HALF && g.c_rem != 0 && cb == g.cblocks - 1;   // uniform
            const uint32_t b_soff = (uint32_t)cb * g.cb_stride;
#pragma unroll
            for (int j = 0; j < STEPS; ++j) {
#pragma unroll
                for (int t = 0; t < TN; ++t) {
                    uint32_t vo = voff[t][j < NVOFF ? j : 0];
                    if (partial) vo = slot < g.c_rem ? vo : kOobOffset;
                    b[buf][j][t] = buf_load<frag_t>(xres, vo, b_soff);
                }
            }
        }
    };

#pragma unroll
    for (int m = 0; m < TM; ++m)
#pragma unroll
        for (int t = 0; t < TN; ++t) acc[m][t] = floatx4{0.f, 0.f, 0.f, 0.f};

    auto mfma_step = [&](int buf, int j) {
#pragma unroll
        for (int m = 0; m < TM; ++m)
#pragma unroll
            for (int t = 0; t < TN; ++t) {
                if constexpr (HALF)
                    acc[m][t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[buf][j][m], b[buf][j][t], acc[m][t], 0, 0, 0);
                else
                    acc[m][t] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[buf][j][m], b[buf][j][t], acc[m][t], 0, 0, 0);
            }
    };
    // MFMAs of the chunk starting at unit u: all of it, or (MODE 1 tail) only its valid units
    auto compute = [&](int buf, int u) {
        if (UNITS == 1 || u + UNITS <= u_end) {
#pragma unroll
            for (int j = 0; j < STEPS; ++j) mfma_step(buf, j);
        } else {
#pragma unroll
            for (int j = 0; j < STEPS; ++j)
                if (u + j < u_end) mfma_step(buf, j);
        }
    };

    // ring of NBUF register sets: loads run NBUF-1 chunks ahead of the MFMAs
    if (u_begin < u_end) {
#pragma unroll
        for (int i = 0; i < NBUF - 1; ++i) load_chunk(i, u_begin + i * UNITS);
        __builtin_amdgcn_s_setprio(0);
        // The scheduling barriers keep the loads of a later chunk in front of the MFMAs of the
        // current one: left alone, the compiler sinks them behind the MFMAs to save registers,
        // which puts every load's latency in front of the instruction that needs it.
        __builtin_amdgcn_sched_barrier(0);
        for (int u = u_begin; u < u_end; u += NBUF * UNITS) {
#pragma unroll
            for (int i = 0; i < NBUF; ++i) {
                load_chunk((i + NBUF - 1) % NBUF, u + (i + NBUF - 1) * UNITS);
                __builtin_amdgcn_sched_barrier(0);
                if (i == 0 || u + i * UNITS < u_end) compute(i, u + i * UNITS);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    }

}

// ---- the k-loops of the work-item kernel for float32 3x3 and 1x1 filters, TM = 1, 2 or 4 panels per tile.
// What bounds the 32 x 32 tile on a busy chip is the vector memory path of a CU (address unit and
// data return are 60-70 % busy, measured), not the matrix pipe: every MFMA needs one operand
// fragment through it.  A 64 x 32 tile needs 0.75.  To keep the register count where four
// wavefronts still fit on a SIMD, a chunk is one filter row (3 k-steps) and three chunks form the
// ring, so loads run two chunks (48 MFMAs) ahead; the buffer of a chunk is the filter row it
// belongs to, which makes every index in the unrolled loop a constant.
template <int TN>
__device__ __forceinline__ void gemm_pixels(const GemmParams &g, const int mb0, const int nb0, const int lane,
                                            PixState<TN> &px, int (&ih0)[TN], int (&iw0)[TN], int (&xbase)[TN]) {
    const int col = lane & 15, slot = lane >> 4;
    const int cbase = (mb0 / g.kg16) * g.Cg;              // first input channel of the tile's group
    const int PQ = g.P * g.Q;
#pragma unroll
    for (int t = 0; t < TN; ++t) {
        const int n = (nb0 + t) * 16 + col;
        px.valid[t] = n < g.npix;
        const int nn = px.valid[t] ? n : 0;
        const int img = g.N == 1 ? 0 : nn / PQ;
        const int pq = nn - img * PQ;
        const int p = pq / g.Q, q = pq - p * g.Q;
        px.img[t] = img; px.pq[t] = pq;
        ih0[t] = p * g.sh - g.ph;
        iw0[t] = q * g.sw - g.pw;
        xbase[t] = (((img * g.C + cbase + slot) * g.H + ih0[t]) * g.W + iw0[t]) * 4;
    }
}

template <int TM, int TN>
__device__ __forceinline__ void gemm_accumulate_3x3(const GemmParams &g, const int mb0, const int nb0, const int ks,
                                                    const int nsplit, const int lane, floatx4 (&acc)[TM][TN],
                                                    PixState<TN> &px) {
    const int slot = lane >> 4;
    int ih0[TN], iw0[TN], xbase[TN];
    gemm_pixels<TN>(g, mb0, nb0, lane, px, ih0, iw0, xbase);
    uint32_t voff[TN][9];
    const int tap_h = g.W * 4;
#pragma unroll
    for (int t = 0; t < TN; ++t)
#pragma unroll
        for (int r = 0; r < 3; ++r) {
            const bool rok = px.valid[t] && (unsigned)(ih0[t] + r) < (unsigned)g.H;
#pragma unroll
            for (int sx = 0; sx < 3; ++sx)
                voff[t][r * 3 + sx] = (rok && (unsigned)(iw0[t] + sx) < (unsigned)g.W) ? (uint32_t)(xbase[t] + r * tap_h + sx * 4) : kOobOffset;
        }
    const int cblocks = g.cblocks;
    const int per = (cblocks + nsplit - 1) / nsplit;
    const int cb_begin = min(cblocks, ks * per), cb_end = min(cblocks, cb_begin + per);
    const __amdgpu_buffer_rsrc_t xres = make_rsrc(g.x, g.x_bytes);
    const __amdgpu_buffer_rsrc_t wres = make_rsrc(g.wp, g.w_bytes);
    uint32_t a_voff[TM], a_base[TM];      // per-lane offset (out of range for panels beyond K), scalar fragment index of the panel
#pragma unroll
    for (int m = 0; m < TM; ++m) {
        const bool ok = mb0 + m < g.K16;
        a_voff[m] = ok ? (uint32_t)lane * 4u : kOobOffset;
        a_base[m] = ok ? (uint32_t)(mb0 + m) * (uint32_t)cblocks * 9u : 0u;
    }
    float a[3][3][TM], b[3][3][TN];
    auto load_row = [&](const int r, int cb) __attribute__((always_inline)) {
        cb = max(min(cb, cb_end - 1), 0);          // past the range: re-read valid data that is not used
        const bool partial = g.c_rem != 0 && cb == cblocks - 1;     // uniform
#pragma unroll
        for (int m = 0; m < TM; ++m) {
            const uint32_t soff = (a_base[m] + (uint32_t)cb * 9u + (uint32_t)r * 3u) * 256u;
#pragma unroll
            for (int sx = 0; sx < 3; ++sx) a[r][sx][m] = buf_load<float>(wres, a_voff[m] + sx * 256u, soff);
        }
        const uint32_t b_soff = (uint32_t)cb * g.cb_stride;
#pragma unroll
        for (int sx = 0; sx < 3; ++sx)
#pragma unroll
            for (int t = 0; t < TN; ++t) {
                uint32_t vo = voff[t][r * 3 + sx];
                if (partial) vo = slot < g.c_rem ? vo : kOobOffset;
                b[r][sx][t] = buf_load<float>(xres, vo, b_soff);
            }
    };
    auto compute_row = [&](const int r) __attribute__((always_inline)) {
#pragma unroll
        for (int sx = 0; sx < 3; ++sx)
#pragma unroll
            for (int m = 0; m < TM; ++m)
#pragma unroll
                for (int t = 0; t < TN; ++t)
                    acc[m][t] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[r][sx][m], b[r][sx][t], acc[m][t], 0, 0, 0);
    };
#pragma unroll
    for (int m = 0; m < TM; ++m)
#pragma unroll
        for (int t = 0; t < TN; ++t) acc[m][t] = floatx4{0.f, 0.f, 0.f, 0.f};
    if (cb_begin < cb_end) {
        load_row(0, cb_begin);
        load_row(1, cb_begin);
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_setprio(0);
        for (int cb = cb_begin; cb < cb_end; ++cb) {
            load_row(2, cb);
            __builtin_amdgcn_sched_barrier(0);
            compute_row(0);
            __builtin_amdgcn_sched_barrier(0);
            load_row(0, cb + 1);
            __builtin_amdgcn_sched_barrier(0);
            compute_row(1);
            __builtin_amdgcn_sched_barrier(0);
            load_row(1, cb + 1);
            __builtin_amdgcn_sched_barrier(0);
            compute_row(2);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
}

// 1x1 filters: a chunk is four channel blocks, three chunks form the ring.
template <int TM, int TN>
__device__ __forceinline__ void gemm_accumulate_1x1(const GemmParams &g, const int mb0, const int nb0, const int ks,
                                                    const int nsplit, const int lane, floatx4 (&acc)[TM][TN],
                                                    PixState<TN> &px) {
    constexpr int CH = 4;
    int ih0[TN], iw0[TN], xbase[TN];
    gemm_pixels<TN>(g, mb0, nb0, lane, px, ih0, iw0, xbase);
    uint32_t voff[TN];
#pragma unroll
    for (int t = 0; t < TN; ++t)
        voff[t] = (px.valid[t] && (unsigned)ih0[t] < (unsigned)g.H && (unsigned)iw0[t] < (unsigned)g.W) ? (uint32_t)xbase[t] : kOobOffset;
    const int cblocks = g.cblocks;
    const int nchunks = (cblocks + CH - 1) / CH;
    const int per = (nchunks + nsplit - 1) / nsplit;
    const int q_begin = min(nchunks, ks * per), q_end = min(nchunks, q_begin + per);
    const __amdgpu_buffer_rsrc_t xres = make_rsrc(g.x, g.x_bytes);
    const __amdgpu_buffer_rsrc_t wres = make_rsrc(g.wp, g.w_bytes);
    uint32_t a_voff[TM], a_base[TM];
#pragma unroll
    for (int m = 0; m < TM; ++m) {
        const bool ok = mb0 + m < g.K16;
        a_voff[m] = ok ? (uint32_t)lane * 4u : kOobOffset;
        a_base[m] = ok ? (uint32_t)(mb0 + m) * (uint32_t)cblocks : 0u;
    }
    // Chunks past the range and blocks past C are read through an empty resource (every load
    // returns 0), so the MFMAs need no condition and the unrolled loop keeps one accumulator set.
    const __amdgpu_buffer_rsrc_t zres = make_rsrc(g.x, 0u);
    float a[3][CH][TM], b[3][CH][TN];
    auto load_chunk = [&](const int buf, const int q) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < CH; ++j) {
            const int cbj = q * CH + j;
            const bool ok = q < q_end && cbj < cblocks;          // uniform
            const int cb = ok ? cbj : 0;
            const __amdgpu_buffer_rsrc_t wsel = ok ? wres : zres, xsel = ok ? xres : zres;
#pragma unroll
            for (int m = 0; m < TM; ++m) a[buf][j][m] = buf_load<float>(wsel, a_voff[m], (a_base[m] + (uint32_t)cb) * 256u);
#pragma unroll
            for (int t = 0; t < TN; ++t) b[buf][j][t] = buf_load<float>(xsel, voff[t], (uint32_t)cb * g.cb_stride);
        }
    };
    auto compute = [&](const int buf) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < CH; ++j)
#pragma unroll
            for (int m = 0; m < TM; ++m)
#pragma unroll
                for (int t = 0; t < TN; ++t)
                    acc[m][t] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[buf][j][m], b[buf][j][t], acc[m][t], 0, 0, 0);
    };
#pragma unroll
    for (int m = 0; m < TM; ++m)
#pragma unroll
        for (int t = 0; t < TN; ++t) acc[m][t] = floatx4{0.f, 0.f, 0.f, 0.f};
    if (q_begin < q_end) {
        load_chunk(0, q_begin);
        load_chunk(1, q_begin + 1);
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_setprio(0);
        for (int q = q_begin; q < q_end; q += 3) {
            load_chunk(2, q + 2);
            __builtin_amdgcn_sched_barrier(0);
            compute(0);
            __builtin_amdgcn_sched_barrier(0);
            load_chunk(0, q + 3);
            __builtin_amdgcn_sched_barrier(0);
            compute(1);
            __builtin_amdgcn_sched_barrier(0);
            load_chunk(1, q + 4);
            __builtin_amdgcn_sched_barrier(0);
            compute(2);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
}

// Row state of a lane's outputs: for each of its 4 * TM rows the element offset of the row in y
// (k * P * Q, or out of range) and the bias value.
template <int TM> struct RowState {
    uint32_t off[TM][4];      // byte offset of (image 0, row k, pixel 0), kOobOffset for rows beyond K
    float bias[TM][4];
};

template <int TM>
__device__ __forceinline__ void gemm_rows(const GemmParams &g, const int mb0, const int slot, RowState<TM> &rs) {
    const int PQ = g.P * g.Q, Kg = g.Kg, kg16 = g.kg16;
    const uint32_t esz = g.half_out ? 2u : 4u;
    const float *bias = g.bias;
    const int grp = mb0 / kg16, mbl = mb0 - grp * kg16;
    const __amdgpu_buffer_rsrc_t bres = make_rsrc(bias, bias ? (uint32_t)g.K * 4u : 0u);   // no bias: every load reads 0
#pragma unroll
    for (int m = 0; m < TM; ++m)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int kl = (mbl + m) * 16 + slot * 4 + j;         // row within the group
            const int k = grp * Kg + kl;
            const bool ok = kl < Kg && mbl + m < kg16;
            rs.off[m][j] = ok ? (uint32_t)(k * PQ) * esz : kOobOffset;
            rs.bias[m][j] = buf_load<float>(bres, ok ? (uint32_t)k * 4u : kOobOffset, 0u);
        }
}

// One finished output: bias, optional clamp at zero, one rounding to the storage type; the store is
// range-checked, so rows beyond K and pixels beyond the layer (offset out of range) write nothing.
__device__ __forceinline__ void gemm_store(const __amdgpu_buffer_rsrc_t yres, const bool relu, const bool half,
                                           const uint32_t off, const float bias, const float v) {
    float r = v + bias;
    if (relu) r = fmaxf(r, 0.f);
    if (half) {
        const _Float16 h = (_Float16)r;      // round to nearest even
        __builtin_amdgcn_raw_buffer_store_b16(__builtin_bit_cast(unsigned short, h), yres, off, 0u, 0);
    } else {
        __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(uint32_t, r), yres, off, 0u, 0);
    }
}

// Byte offset of pixel (img, pq) within its row of y, or out of range.
__device__ __forceinline__ uint32_t gemm_pixel_offset(const GemmParams &g, const int img, const int pq, const bool valid) {
    const uint32_t esz = g.half_out ? 2u : 4u;
    return valid ? ((uint32_t)img * (uint32_t)(g.K * g.P * g.Q) + (uint32_t)pq) * esz : kOobOffset;
}

__device__ __forceinline__ __amdgpu_buffer_rsrc_t gemm_y_rsrc(const GemmParams &g) {
    return make_rsrc(g.y, (uint32_t)g.N * (uint32_t)(g.K * g.P * g.Q) * (g.half_out ? 2u : 4u));
}

// One layer per launch: a workgroup of KS wavefronts owns one output tile, the wavefronts split
// the channel blocks and add their partial sums through LDS in fixed order.
// (the 32 x 32 tile is launched as one wavefront per workgroup only, and needs more than the 128
// registers a 16-wavefront workgroup leaves each lane)
template <bool HALF, int TM, int TN, int MODE, int NBUF>
__global__ __launch_bounds__(TM * TN == 4 ? 64 : 1024) void im2col_gemm_kernel(const GemmParams g) {
    extern __shared__ __align__(16) float red[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // scalar
    const int slot = lane >> 4;
    const int KS = 1 << g.ks_shift;
    const int ks = wave & (KS - 1), nt = wave >> g.ks_shift;             // k-split index, tile within the workgroup
    const int tiles_per_wg = (blockDim.x >> 6) >> g.ks_shift;
    const int ltile = xcd_logical_tile(g.grid_nx * g.grid_ny);
    if (ltile < 0) return;                                               // whole workgroup: grid padding
    const int bx = g.m_major ? ltile % g.grid_nx : ltile / g.grid_ny;
    const int by = g.m_major ? ltile / g.grid_nx : ltile % g.grid_ny;
    const int mb0 = by * TM;                              // panel index over all groups; TM panels stay in one group
    const int nb0 = (bx * tiles_per_wg + nt) * TN;
    floatx4 acc[TM][TN];
    PixState<TN> px;
    gemm_accumulate<HALF, TM, TN, MODE, NBUF>(g, mb0, nb0, ks, KS, lane, acc, px);

    // ---- sum the KS partial tiles through LDS: red[((nt * KS + ks) * NREG + reg) * 64 + lane]
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
    // epilogue: lane holds rows 4*slot + j, column col of each block; wavefront ks finishes the
    // accumulator registers reg = ks, ks + KS, ...
    RowState<TM> rs;
    gemm_rows<TM>(g, mb0, slot, rs);
    const __amdgpu_buffer_rsrc_t yres = gemm_y_rsrc(g);
    const bool relu = g.relu, half_out = g.half_out;
    uint32_t pixoff[TN];
#pragma unroll
    for (int t = 0; t < TN; ++t) pixoff[t] = gemm_pixel_offset(g, px.img[t], px.pq[t], px.valid[t]);
#pragma unroll
    for (int m = 0; m < TM; ++m) {
#pragma unroll
        for (int t = 0; t < TN; ++t) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int reg = (m * TN + t) * 4 + j;
                if ((reg & (KS - 1)) != ks) continue;
                float v = acc[m][t][j];
                if (KS > 1) {
                    v = 0.f;
                    for (int z = 0; z < KS; ++z) v += red[((nt * KS + z) * NREG + reg) * 64 + lane];
                }
                // either offset may be the out-of-range constant 2^31; both at once would wrap to a small sum
                const uint32_t off = rs.off[m][j] == kOobOffset ? kOobOffset : rs.off[m][j] + pixoff[t];
                gemm_store(yres, relu, half_out, off, rs.bias[m][j], v);
            }
        }
    }
}

// ---------------------------------------------------------------- many layers in one launch
// A batch-1 layer neither fills 256 CUs nor runs long enough to hide its launch, its first loads
// and its epilogue.  Independent layers (what the decision stage profiles, and what a model's
// parallel branches are) therefore go into ONE launch of single-wavefront workgroups, one per
// work item: an item is one output tile (TM x 2 blocks of 16 x 16) of one layer over one of the
// nsplit ranges its reduction is cut into, the ranges sized so that items of different layers
// take about the same time.  The chip's dispatcher balances the items over the CUs; two to four
// items are resident per SIMD, so one item's addressing and first loads run under another's
// MFMAs.  A split layer's items store partial tiles, which a second launch adds in fixed order.
struct GemmItemLayer {
    GemmParams g;
    float *part;        // partial tiles of a split layer (workspace): [tile][split][reg][lane]
    int ntn;            // tiles along the pixels
    int nsplit;         // ranges of the reduction (1: the item stores y itself)
    int mode, tm;       // chunking mode (ModeT); 16-row panels per tile (1 or 2)
};
struct GemmItemTable {
    GemmItemLayer layer[kMaxGemmLayers];
    // first item / first reduction workgroup of each layer, INT_MAX beyond the last layer: a
    // workgroup finds its layer by counting the entries it has reached (table_find)
    int item0[kMaxGemmLayers], red0[kMaxGemmLayers];
    int nlayers, nitems;
    int group;          // consecutive items handed to one XCD
    int nred;           // workgroups of the reduction launch
};
static_assert(sizeof(GemmItemTable) <= 4096, "the table is passed by value as the kernel argument");

template <bool HALF, int TM, int MODE, int NBUF = 2>
__device__ __forceinline__ void gemm_item(const GemmItemLayer &L, const int local, const int lane) {
    constexpr int TN = 2;
    const int nb = local % L.ntn, rest = local / L.ntn;
    const int ks = rest % L.nsplit, mt = rest / L.nsplit;       // order: tile row, range, tile column (fastest)
    floatx4 acc[TM][TN];
    PixState<TN> px;
    if constexpr (!HALF && MODE == 3) gemm_accumulate_3x3<TM, TN>(L.g, mt * TM, nb * TN, ks, L.nsplit, lane, acc, px);
    else if constexpr (!HALF && MODE == 1) gemm_accumulate_1x1<TM, TN>(L.g, mt * TM, nb * TN, ks, L.nsplit, lane, acc, px);
    else gemm_accumulate<HALF, TM, TN, MODE, NBUF>(L.g, mt * TM, nb * TN, ks, L.nsplit, lane, acc, px);
    __builtin_amdgcn_s_setprio(3);
    if (L.nsplit == 1) {
        RowState<TM> rs;
        gemm_rows<TM>(L.g, mt * TM, lane >> 4, rs);
        const __amdgpu_buffer_rsrc_t yres = gemm_y_rsrc(L.g);
        const bool relu = L.g.relu, half_out = L.g.half_out;
        uint32_t pixoff[TN];
#pragma unroll
        for (int t = 0; t < TN; ++t) pixoff[t] = gemm_pixel_offset(L.g, px.img[t], px.pq[t], px.valid[t]);
        __builtin_amdgcn_sched_barrier(0);      // parameters and bias values first, then nothing but stores
#pragma unroll
        for (int m = 0; m < TM; ++m)
#pragma unroll
            for (int t = 0; t < TN; ++t)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const uint32_t off = rs.off[m][j] == kOobOffset ? kOobOffset : rs.off[m][j] + pixoff[t];
                    gemm_store(yres, relu, half_out, off, rs.bias[m][j], acc[m][t][j]);
                }
    } else {
        constexpr int NREG = TM * TN * 4;
        float *o = L.part + ((size_t)(mt * L.ntn + nb) * L.nsplit + ks) * (NREG * 64) + lane;
#pragma unroll
        for (int m = 0; m < TM; ++m)
#pragma unroll
            for (int t = 0; t < TN; ++t)
#pragma unroll
                for (int j = 0; j < 4; ++j) o[((m * TN + t) * 4 + j) * 64] = acc[m][t][j];
    }
}

// The table is the kernel argument; the kernel reads it through the kernel-argument segment
// pointer (constant address space, scalar loads at computed offsets).  Indexing the by-value
// parameter itself with a run-time layer number makes the compiler copy all 4 KB of it to
// scratch memory first, in every wavefront.
typedef const __attribute__((address_space(4))) GemmItemTable *GemmItemTablePtr;

__device__ __forceinline__ void load_item_layer(GemmItemLayer &dst, const GemmItemTablePtr tbl, const int li) {
    static_assert(sizeof(GemmItemLayer) % 4 == 0, "copied word by word");
    const __attribute__((address_space(4))) uint32_t *src = (const __attribute__((address_space(4))) uint32_t *)&tbl->layer[li];
    uint32_t *d = reinterpret_cast<uint32_t *>(&dst);
#pragma unroll
    for (int i = 0; i < (int)(sizeof(GemmItemLayer) / 4); ++i) d[i] = src[i];
}

constexpr int kItemWaves = 4;      // items per workgroup (one wavefront each)

template <bool HALF, int NBUF = 2>
__global__ __launch_bounds__(64 * kItemWaves, 3) void gemm_items_kernel(const GemmItemTable tbl_arg) {
    const GemmItemTablePtr tbl = (GemmItemTablePtr)__builtin_amdgcn_kernarg_segment_ptr();
    // Workgroup i runs on XCD i % 8.  Groups of `group` consecutive items (neighbouring tiles of
    // one layer: they share a weight panel) are dealt to the XCDs in turn, so every XCD sees the
    // same mix of layers in the same order and a panel is fetched into one L2.
    // An item's addressing competes for issue slots with the MFMA loops of the other wavefronts on
    // its SIMD, which always have an instruction ready: without a higher priority it is served
    // last and takes several microseconds.  The k-loop drops back to the default priority.
    __builtin_amdgcn_s_setprio(3);
    // The wavefronts of a workgroup take consecutive items (neighbouring tiles along the pixels:
    // the same weight fragments at about the same time, so three of four reads of them hit in
    // the CU's L1); they share nothing else and never wait for one another.
    const int G = tbl->group;
    const int i = blockIdx.x, xcd = i & 7, j = i >> 3;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int item = (((j / G) * 8 + xcd) * G + j % G) * kItemWaves + wave;
    if (item >= tbl->nitems) return;
    int first;
    const int li = table_find<kMaxGemmLayers>(&tbl->item0[0], item, first);
    GemmItemLayer L;
    load_item_layer(L, tbl, li);                     // one batch of scalar loads
    const int local = item - first;
    const int lane = threadIdx.x & 63;
    if (L.tm == 4) {
        if constexpr (!HALF) {
            if (L.mode == 3) gemm_item<false, 4, 3, NBUF>(L, local, lane);
            else gemm_item<false, 4, 1, NBUF>(L, local, lane);
        }
    } else if (L.tm == 2) {
        switch (L.mode) {
            case 1: gemm_item<HALF, 2, 1, NBUF>(L, local, lane); break;
            case 3: gemm_item<HALF, 2, 3, NBUF>(L, local, lane); break;
            case 5: if constexpr (!HALF) gemm_item<HALF, 2, 5, NBUF>(L, local, lane); break;
            case 7: if constexpr (!HALF) gemm_item<HALF, 2, 7, NBUF>(L, local, lane); break;
            default: gemm_item<HALF, 2, 0, NBUF>(L, local, lane); break;
        }
    } else {
        switch (L.mode) {
            case 1: gemm_item<HALF, 1, 1, NBUF>(L, local, lane); break;
            case 3: gemm_item<HALF, 1, 3, NBUF>(L, local, lane); break;
            case 5: if constexpr (!HALF) gemm_item<HALF, 1, 5, NBUF>(L, local, lane); break;
            case 7: if constexpr (!HALF) gemm_item<HALF, 1, 7, NBUF>(L, local, lane); break;
            default: gemm_item<HALF, 1, 0, NBUF>(L, local, lane); break;
        }
    }
}

__device__ static inline int ceil_div_dev(int a, int b) { return (a + b - 1) / b; }

// Adds the nsplit partial tiles of every split layer in the order of the ranges and stores y.
// A thread owns four consecutive lanes of one accumulator register (16-byte loads); the loads of
// twelve ranges are in flight at once, the additions keep the order of the ranges.
__global__ __launch_bounds__(256) void gemm_reduce_kernel(const GemmItemTable tbl_arg) {
    const GemmItemTablePtr tbl = (GemmItemTablePtr)__builtin_amdgcn_kernarg_segment_ptr();
    const int b = blockIdx.x;
    int first;
    const int li = table_find<kMaxGemmLayers>(&tbl->red0[0], b, first);      // the last layer that starts at or before b
    GemmItemLayer L;
    load_item_layer(L, tbl, li);
    const int nreg = L.tm * 8;                                   // accumulator registers per lane: TM x 2 blocks x 4
    const int per_tile = nreg * 64;
    const int e = ((b - first) * 256 + threadIdx.x) * 4;          // over [tile][reg][lane]
    const int tile = e / per_tile, rl = e - tile * per_tile;
    const int reg = rl >> 6, lane0 = rl & 63;
    if (tile >= ceil_div_dev(L.g.K16, L.tm) * L.ntn) return;     // second half of the last workgroup of an odd tile count
    const float4 *src = reinterpret_cast<const float4 *>(L.part + (size_t)tile * L.nsplit * per_tile + rl);
    const size_t zs = (size_t)per_tile / 4;
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    constexpr int kInFlight = 12;
    for (int z = 0; z < L.nsplit; z += kInFlight) {
        // (ranges past the last one load the last one again and are not added)
        float4 p[kInFlight];
#pragma unroll
        for (int i = 0; i < kInFlight; ++i) p[i] = src[(size_t)min(z + i, L.nsplit - 1) * zs];
#pragma unroll
        for (int i = 0; i < kInFlight; ++i)
            if (z + i < L.nsplit) { v.x += p[i].x; v.y += p[i].y; v.z += p[i].z; v.w += p[i].w; }
    }
    // the four values are rows (lane0 / 16) * 4 + jj of panel m, pixels (lane0 % 16) .. + 3 of block t
    const int mt = tile / L.ntn, nb = tile - mt * L.ntn;
    const int m = reg >> 3, t = (reg >> 2) & 1, jj = reg & 3;
    const int PQ = L.g.P * L.g.Q, Kg = L.g.Kg, kg16 = L.g.kg16, npix = L.g.npix;
    const bool relu = L.g.relu, half_out = L.g.half_out;
    const float *bias = L.g.bias;
    const __amdgpu_buffer_rsrc_t yres = gemm_y_rsrc(L.g);
    const int mb0 = mt * L.tm, grp = mb0 / kg16, mbl = mb0 - grp * kg16;
    const int kl = (mbl + m) * 16 + (lane0 >> 4) * 4 + jj;
    const int k = grp * Kg + kl;
    const bool rok = kl < Kg && mbl + m < kg16;
    const float bv = (bias && rok) ? bias[k] : 0.f;
    const uint32_t esz = half_out ? 2u : 4u;
    const float vv[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int n = (nb * 2 + t) * 16 + (lane0 & 15) + i;
        const bool valid = rok && n < npix;
        const int nn = valid ? n : 0;
        const int img = nn / PQ;
        const uint32_t off = valid ? ((uint32_t)(img * L.g.K + k) * (uint32_t)PQ + (uint32_t)(nn - img * PQ)) * esz : kOobOffset;
        gemm_store(yres, relu, half_out, off, bv, vv[i]);
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

// The same conversion for several layers in one launch: a workgroup finds its layer by its index,
// as the item kernel does, then converts 256 pixels of 32 channels of one image.
struct ChannelsLastTable {
    const __half *x[kMaxGemmLayers];
    __half *xt[kMaxGemmLayers];
    int C[kMaxGemmLayers], HW[kMaxGemmLayers], cpad[kMaxGemmLayers];
    int block0[kMaxGemmLayers];      // first workgroup of each layer, INT_MAX beyond the last one
    int nblocks;
};
typedef const __attribute__((address_space(4))) ChannelsLastTable *ChannelsLastTablePtr;

__global__ __launch_bounds__(256) void to_channels_last_many_kernel(const ChannelsLastTable tbl_arg) {
    const ChannelsLastTablePtr tbl = (ChannelsLastTablePtr)__builtin_amdgcn_kernarg_segment_ptr();
    const int b = blockIdx.x;
    if (b >= tbl->nblocks) return;
    int first;
    const int li = table_find<kMaxGemmLayers>(&tbl->block0[0], b, first);
    const int C = tbl->C[li], HW = tbl->HW[li], cpad = tbl->cpad[li];
    const __half *x = tbl->x[li];
    __half *xt = tbl->xt[li];
    const int npb = (HW + 255) / 256, nblk = cpad / 32;
    const int local = b - first;
    const int pb = local % npb, rest = local / npb;
    const int cb = rest % nblk, img = rest / nblk;
    const int pix = pb * 256 + threadIdx.x;
    if (pix >= HW) return;
    // (a thread writes the 64 contiguous bytes of its pixel's 32 channels; 8 channels per thread, or
    // two pixels per thread with 4-byte loads, took the same 10-11 us on the ResNet-18-shaped stack)
    __half v[32];
#pragma unroll
    for (int j = 0; j < 32; ++j) {
        const int c = cb * 32 + j;
        v[j] = (c < C) ? x[((size_t)img * C + c) * HW + pix] : __float2half(0.f);
    }
    uint4 *dst = reinterpret_cast<uint4 *>(xt + ((size_t)img * HW + pix) * cpad + cb * 32);
#pragma unroll
    for (int q = 0; q < 4; ++q) dst[q] = reinterpret_cast<const uint4 *>(v)[q];
}

// ---------------------------------------------------------------- host side

struct GemmPlan {
    int tm, tn, ks_shift, mode, nbuf;
    size_t xt_bytes;
};

static GemmPlan plan_im2col(const Geo &g) {
    GemmPlan pl{};
    const bool half = g.dtype == NNV_F16;
    const int kg16 = ceil_div(g.kg, 16);
    const int K16 = g.groups * kg16;
    const int npix16 = ceil_div(g.n * g.p * g.q, 16);
    const int cblocks = half ? ceil_div(g.cg, 32) : ceil_div(g.cg, 4);
    const bool partial = !half && (g.cg % 4) != 0;
    if (g.r == 1 && g.s == 1 && !partial) pl.mode = 1;
    else if (g.r == 3 && g.s == 3) pl.mode = 3;
    else if (g.s == 7 && !half) pl.mode = 7;
    else if (g.s == 5 && !half) pl.mode = 5;
    else pl.mode = 0;
    const bool row = pl.mode == 5 || pl.mode == 7 || (pl.mode == 3 && half);
    const int nunits = pl.mode == 0 ? cblocks * g.r * g.s : row ? cblocks * g.r : cblocks;
    const int unit_steps = pl.mode == 0 ? 1 : row ? pl.mode : g.r * g.s;
    auto tiles = [&](int tm, int tn) { return (long)ceil_div(K16, tm) * ceil_div(npix16, tn); };
    // Batch-1 layers are latency-bound.  What pays (measured on ResNet-18-shaped layers): the
    // 32x32 tile only with thousands of tiles; the 32x16 tile while it still leaves >= 160 tiles,
    // its units split over KS wavefronts up to ~2048 wavefronts; else the 16x16 tile with a
    // moderate split (>= 768 wavefronts) and a deeper register ring, because its few workgroups
    // stream the weights from HBM and each CU keeps only so many misses in flight.
    auto split_for = [&](long t, long target) {
        int shift = 0;
        while (shift < 4 && (t << shift) < target && (nunits >> (shift + 1)) >= 1 &&
               (((long)nunits * unit_steps) >> (shift + 1)) >= 9)
            ++shift;
        return shift;
    };
    // (the float16 1x1 gather keeps eight loads per fragment in flight: no room for the 32x32 tile)
    if (tiles(2, 2) >= 4096 && !(half && pl.mode == 1)) { pl.tm = 2; pl.tn = 2; pl.ks_shift = 0; }
    else if (tiles(2, 1) >= 160) { pl.tm = 2; pl.tn = 1; pl.ks_shift = split_for(tiles(2, 1), 2048); }
    else { pl.tm = 1; pl.tn = 1; pl.ks_shift = split_for(tiles(1, 1), 768); }
    if (g.groups > 1 && kg16 % pl.tm != 0) {       // a wavefront's panels must belong to one group
        pl.tm = 1; pl.tn = 1;
        pl.ks_shift = split_for(tiles(1, 1), 2048);
    }
    // depth of the register ring: never more sets than the wavefront has chunks to load
    const int units_per_wave = ceil_div(nunits, 1 << pl.ks_shift);
    const int chunk_units = pl.mode == 1 ? (half ? 2 : 8) : 1;
    const int chunks = ceil_div(units_per_wave, chunk_units);
    pl.nbuf = 2;
    if (pl.tm == 1 && chunks >= 6) pl.nbuf = 4;
    else if (pl.tm * pl.tn <= 2 && chunks >= 3) pl.nbuf = 3;
    if (half || pl.tm * pl.tn == 4) pl.nbuf = 2;
    // float16 needs the channel-last copy of x, except for 1x1 filters (gathered from NCHW)
    pl.xt_bytes = (half && pl.mode != 1) ? align_up((size_t)g.n * g.h * g.w * ceil_div(g.c, 32) * 32 * sizeof(__half), 256) : 0;
    return pl;
}

size_t im2col_workspace_bytes(const Geo &g) { return plan_im2col(g).xt_bytes; }

template <bool HALF, int TM, int TN, int NBUF>
static void launch_gemm_mode(int mode, const GemmParams &gp, dim3 grid, dim3 block, size_t lds, hipStream_t st) {
    switch (mode) {
        case 1: hipLaunchKernelGGL((im2col_gemm_kernel<HALF, TM, TN, 1, NBUF>), grid, block, lds, st, gp); break;
        case 3: hipLaunchKernelGGL((im2col_gemm_kernel<HALF, TM, TN, 3, NBUF>), grid, block, lds, st, gp); break;
        case 5: if constexpr (!HALF) { hipLaunchKernelGGL((im2col_gemm_kernel<HALF, TM, TN, 5, NBUF>), grid, block, lds, st, gp); } break;
        case 7: if constexpr (!HALF) { hipLaunchKernelGGL((im2col_gemm_kernel<HALF, TM, TN, 7, NBUF>), grid, block, lds, st, gp); } break;
        default: hipLaunchKernelGGL((im2col_gemm_kernel<HALF, TM, TN, 0, NBUF>), grid, block, lds, st, gp); break;
    }
}

template <bool HALF>
static void launch_gemm_variant(const GemmPlan &pl, const GemmParams &gp, dim3 grid, dim3 block, size_t lds, hipStream_t st) {
    if (pl.tm == 2 && pl.tn == 2) launch_gemm_mode<HALF, 2, 2, 2>(pl.mode, gp, grid, block, lds, st);
    else if (pl.tm == 2 && pl.tn == 1) {
        if (!HALF && pl.nbuf >= 3) launch_gemm_mode<HALF, 2, 1, 3>(pl.mode, gp, grid, block, lds, st);
        else launch_gemm_mode<HALF, 2, 1, 2>(pl.mode, gp, grid, block, lds, st);
    } else {
        if (!HALF && pl.nbuf >= 4) launch_gemm_mode<HALF, 1, 1, 4>(pl.mode, gp, grid, block, lds, st);
        else if (!HALF && pl.nbuf == 3) launch_gemm_mode<HALF, 1, 1, 3>(pl.mode, gp, grid, block, lds, st);
        else launch_gemm_mode<HALF, 1, 1, 2>(pl.mode, gp, grid, block, lds, st);
    }
}

// Kernel parameters of a layer apart from the tile plan.
static GemmParams gemm_params(const Geo &g, int mode, const void *x, const void *w, const float *bias, void *y) {
    const bool half = g.dtype == NNV_F16;
    GemmParams gp{};
    gp.x = x; gp.wp = w; gp.bias = bias; gp.y = y;
    gp.N = g.n; gp.C = g.c; gp.H = g.h; gp.W = g.w; gp.K = g.k; gp.R = g.r; gp.S = g.s;
    gp.sh = g.sh; gp.sw = g.sw; gp.ph = g.ph; gp.pw = g.pw; gp.P = g.p; gp.Q = g.q;
    gp.npix = g.n * g.p * g.q;
    gp.kg16 = ceil_div(g.kg, 16);
    gp.K16 = g.groups * gp.kg16;
    gp.Kg = g.kg; gp.Cg = g.cg;
    gp.cpad = ceil_div(g.c, 32) * 32;
    gp.cblocks = half ? ceil_div(g.cg, 32) : ceil_div(g.cg, 4);
    const bool gather = half && mode == 1;      // float16 1x1: B fragments gathered from NCHW
    gp.c_rem = gather ? g.cg % 32 : half ? 0 : g.cg % 4;
    gp.plane_bytes = (uint32_t)(g.h * g.w * 2);
    gp.half_out = half;
    gp.relu = g.relu;
    gp.x_bytes = gather ? (uint32_t)((size_t)g.n * g.c * g.h * g.w * 2)
                 : half ? (uint32_t)((size_t)g.n * g.h * g.w * gp.cpad * 2) : (uint32_t)((size_t)g.n * g.c * g.h * g.w * 4);
    gp.w_bytes = (uint32_t)((size_t)gp.K16 * gp.cblocks * g.r * g.s * 64 * (half ? 16 : 4));
    gp.cb_stride = gather ? 32u * gp.plane_bytes : half ? 64u : (uint32_t)(4 * g.h * g.w * 4);
    return gp;
}

// float16 layers with a filter larger than 1x1 read x from a channel-last copy in the workspace.
static void launch_channels_last(const Geo &g, const GemmParams &gp, const void *x, void *xt, hipStream_t st) {
    dim3 grid(ceil_div(g.h * g.w, 256), gp.cpad / 8, g.n);
    hipLaunchKernelGGL(to_channels_last_kernel, grid, dim3(256), 0, st, static_cast<const __half *>(x),
                       static_cast<__half *>(xt), g.c, g.h * g.w, gp.cpad);
}

hipError_t launch_im2col(const Geo &g, const void *x, const void *w, const float *bias, void *y, void *ws, hipStream_t st) {
    const GemmPlan pl = plan_im2col(g);
    const bool half = g.dtype == NNV_F16;
    GemmParams gp = gemm_params(g, pl.mode, x, w, bias, y);
    gp.ks_shift = pl.ks_shift;
    if (half && pl.mode != 1) {
        launch_channels_last(g, gp, x, ws, st);
        gp.x = ws;
    }
    const int KS = 1 << pl.ks_shift;
    const int waves = KS;
    const int tiles_per_wg = waves / KS;
    const int npix16 = ceil_div(gp.npix, 16);
    gp.grid_nx = ceil_div(ceil_div(npix16, pl.tn), tiles_per_wg);
    gp.grid_ny = ceil_div(gp.K16, pl.tm);
    gp.m_major = gp.w_bytes >= gp.x_bytes;
    dim3 grid(xcd_grid(gp.grid_nx * gp.grid_ny), 1, 1);
    const size_t lds = KS > 1 ? (size_t)waves * pl.tm * pl.tn * 4 * 64 * sizeof(float) : 0;
    if (half) launch_gemm_variant<true>(pl, gp, grid, dim3(64 * waves), lds, st);
    else launch_gemm_variant<false>(pl, gp, grid, dim3(64 * waves), lds, st);
    return hipGetLastError();
}

// ---- many layers in one launch: item plan of one layer
struct ItemPlan {
    int mode, tm, nmt, ntn, nsplit;
    int steps;              // k-steps of the whole reduction
    size_t part_bytes;      // partial tiles (0 if the layer is not split)
    size_t xt_bytes;        // channel-last float16 copy of x (0 if not needed)
};

// k-steps (one MFMA per 16 x 16 block each) a work item aims at: long enough to amortise an
// item's addressing, first loads and store, short enough that the chip's last round of items
// stays small against the whole launch.
constexpr int kItemSteps = 144;

static ItemPlan plan_items(const Geo &g, const int item_steps) {
    ItemPlan ip{};
    const GemmPlan pl = plan_im2col(g);
    const bool half = g.dtype == NNV_F16;
    ip.mode = pl.mode;
    ip.xt_bytes = pl.xt_bytes;
    const int kg16 = ceil_div(g.kg, 16);
    const int K16 = g.groups * kg16;
    // two panels per tile unless that leaves a third or more of the tile rows empty
    // (a tile's panels must belong to one group)
    ip.tm = (kg16 % 2 == 0 || (g.groups == 1 && kg16 >= 5)) ? 2 : 1;
    // float32 3x3 and 1x1 layers with at least 64 output channels: four panels per tile
    if (!half && g.groups == 1 && (pl.mode == 3 || pl.mode == 1) && (kg16 % 4 == 0 || kg16 >= 12)) ip.tm = 4;
    ip.nmt = ceil_div(K16, ip.tm);
    ip.ntn = ceil_div(ceil_div(g.n * g.p * g.q, 16), 2);
    const int cblocks = half ? ceil_div(g.cg, 32) : ceil_div(g.cg, 4);
    const bool row = pl.mode == 5 || pl.mode == 7 || (pl.mode == 3 && half);
    int nunits = pl.mode == 0 ? cblocks * g.r * g.s : row ? cblocks * g.r : cblocks;
    int unit_steps = pl.mode == 0 ? 1 : row ? pl.mode : g.r * g.s;
    int chunk_units = pl.mode == 1 ? (half ? 2 : 8) : 1;
    int target = item_steps;
    if (ip.tm == 4) {
        // a wide item does twice the MFMAs per k-step: somewhat fewer steps per item
        target = std::max(9, item_steps * 3 / 4);
    }
    if (!half && pl.mode == 1) { nunits = ceil_div(cblocks, 4); unit_steps = 4; chunk_units = 1; }   // float32 1x1: the kernel splits whole chunks of 4 blocks
    const long steps = (long)nunits * unit_steps;
    ip.steps = (int)steps;
    long nsplit = (steps + target / 2) / target;
    const long most = std::max(1, nunits / chunk_units);          // every range holds at least one chunk
    nsplit = std::max(1L, std::min(nsplit, most));
    // ranges are ceil(nunits / nsplit) units long: drop ranges that would come out empty
    const int per = ceil_div(nunits, (int)nsplit);
    ip.nsplit = ceil_div(nunits, per);
    ip.part_bytes = ip.nsplit > 1 ? (size_t)ip.nmt * ip.ntn * ip.nsplit * (ip.tm * 8) * 64 * sizeof(float) : 0;
    return ip;
}

// Item length of a launch of these layers.
// float16 items of a call that fills the chip fewer than three times over are a quarter as long:
// such a launch ends with its longest items (a 512-channel 3x3 layer is one item of 144 steps per tile
// otherwise), and a float16 step moves eight times the channels of a float32 one.  Measured on
// the ResNet-18-, ResNet-50- and VGG-16-shaped stacks: 75 -> 61, 129 -> 123 and (the long items
// kept) 184 us against 201 us with the short ones.
// float32: a launch whose items all fit the chip at once (kItemsResident, less a sixteenth: a launch
// that fills every slot was measured slower than one that leaves a few free) takes the shortest
// item length, in steps of 12 down to kItemStepsMin, with which they still do: the launch lasts as
// long as an item, and the free slots would stay idle.  Measured (us, one call): SqueezeNet-shaped
// stack 84 -> 64, GoogLeNet 131 -> 101, AlexNet 80 -> 51, MobileNetV2 66 -> 55, ResNet-50 170 -> 159;
// the ResNet-18-shaped stack (2882 items of 144 steps) keeps its items.
constexpr int kItemStepsShortHalf = 36, kItemStepsMin = 48;
constexpr int kItemsResident = 256 * 3 * kItemWaves;

int im2col_items_target(int n, const Geo *geos) {
    auto total_at = [&](int t) {
        long tot = 0;
        for (int i = 0; i < n; ++i) {
            const ItemPlan p = plan_items(geos[i], t);
            tot += (long)p.nmt * p.ntn * p.nsplit;
        }
        return tot;
    };
    const long total = total_at(kItemSteps);
    if (geos[0].dtype == NNV_F16) return total < 3L * kItemsResident ? kItemStepsShortHalf : kItemSteps;
    constexpr long fit = (long)kItemsResident * 15 / 16;
    int best = kItemSteps;
    if (total <= fit)
        for (int t = kItemSteps - 12; t >= kItemStepsMin; t -= 12) {
            if (total_at(t) > fit) break;
            best = t;
        }
    return best;
}

size_t im2col_items_workspace_bytes(const Geo &g, int target) {
    const ItemPlan ip = plan_items(g, target);
    return align_up(ip.part_bytes, 256) + align_up(ip.xt_bytes, 256);
}

// Launches layers [0, n) (all of one storage type, n <= kMaxGemmLayers) as one item launch plus,
// if any layer is split, one reduction launch.  ws[i] is layer i's own workspace region of
// im2col_items_workspace_bytes(geos[i], im2col_items_target(n, geos)).
hipError_t launch_im2col_items(int n, const Geo *geos, const void *const *x, const void *const *w, const float *const *bias,
                               void *const *y, void *const *ws, hipStream_t st) {
    if (n <= 0) return hipSuccess;
    if (n > kMaxGemmLayers) return hipErrorInvalidValue;
    const bool half = geos[0].dtype == NNV_F16;
    // Order: layers with the longest items first, so that the chip's last round of items is made
    // of the short ones.
    ItemPlan plans[kMaxGemmLayers];
    int order[kMaxGemmLayers];
    for (int i = 0; i < n; ++i)
        if ((geos[i].dtype == NNV_F16) != half) return hipErrorInvalidValue;
    const int target = im2col_items_target(n, geos);
    for (int i = 0; i < n; ++i) {
        plans[i] = plan_items(geos[i], target);
        order[i] = i;
    }
    auto item_len = [&](int i) { return ceil_div(plans[i].steps, plans[i].nsplit) * plans[i].tm; };
    std::stable_sort(order, order + n, [&](int a, int b) { return item_len(a) > item_len(b); });
    GemmItemTable tbl{};
    ChannelsLastTable cl{};
    int items = 0, red = 0, ncl = 0, clblocks = 0;
    for (int o = 0; o < n; ++o) {
        const int i = order[o];
        const Geo &g = geos[i];
        const ItemPlan &ip = plans[i];
        GemmItemLayer &L = tbl.layer[o];
        L.g = gemm_params(g, ip.mode, x[i], w[i], bias ? bias[i] : nullptr, y[i]);
        char *region = static_cast<char *>(ws[i]);
        if (ip.xt_bytes) {
            // all channel-last copies of the call are made by one launch in front of the item launch
            void *xt = region + align_up(ip.part_bytes, 256);
            cl.x[ncl] = static_cast<const __half *>(x[i]);
            cl.xt[ncl] = static_cast<__half *>(xt);
            cl.C[ncl] = g.c;
            cl.HW[ncl] = g.h * g.w;
            cl.cpad[ncl] = L.g.cpad;
            cl.block0[ncl] = clblocks;
            clblocks += ceil_div(g.h * g.w, 256) * (L.g.cpad / 32) * g.n;
            ++ncl;
            L.g.x = xt;
        }
        L.part = ip.nsplit > 1 ? reinterpret_cast<float *>(region) : nullptr;
        tbl.item0[o] = items;
        tbl.red0[o] = red;
        L.ntn = ip.ntn;
        L.nsplit = ip.nsplit;
        L.mode = ip.mode;
        L.tm = ip.tm;
        items += ip.nmt * ip.ntn * ip.nsplit;
        if (ip.nsplit > 1) red += ceil_div(ip.nmt * ip.ntn * (ip.tm * 8), 16);     // 1024 values per workgroup
    }
    for (int i = n; i < kMaxGemmLayers; ++i) tbl.item0[i] = tbl.red0[i] = INT_MAX;
    tbl.nlayers = n;
    tbl.nitems = items;
    tbl.group = 2;       // workgroups (of kItemWaves items) handed to one XCD in a row
    tbl.nred = red;
    if (ncl > 0) {
        for (int i = ncl; i < kMaxGemmLayers; ++i) cl.block0[i] = INT_MAX;
        cl.nblocks = clblocks;
        hipLaunchKernelGGL(to_channels_last_many_kernel, dim3(clblocks), dim3(256), 0, st, cl);
    }
    const int wgs = ceil_div(items, kItemWaves);
    const int per_xcd = ceil_div(ceil_div(wgs, tbl.group), 8) * tbl.group;
    if (half) hipLaunchKernelGGL(gemm_items_kernel<true>, dim3(per_xcd * 8), dim3(64 * kItemWaves), 0, st, tbl);
    else hipLaunchKernelGGL(gemm_items_kernel<false>, dim3(per_xcd * 8), dim3(64 * kItemWaves), 0, st, tbl);
    if (red > 0) hipLaunchKernelGGL(gemm_reduce_kernel, dim3(red), dim3(256), 0, st, tbl);
    return hipGetLastError();
}

}  // namespace nnv
