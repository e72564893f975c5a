// Winograd F(2x2,3x3) / F(4x4,3x3) / F(6x6,3x3) convolution from transformed weights (the fastest
// executing, most expensive to prepare kernel family of Table 2).  Three kernels:
//   1. input transform   V[xi][tile block][c][16 tiles] = (B^T d B)[xi]   (vector ALU)
//   2. batched tile GEMM M[xi] = U[xi] (K x C) * V[xi] (C x T), alpha^2 independent
//      products on the matrix cores; U and V are stored as ready-made 16-row operand
//      fragments, so both are read with one coalesced load per fragment and no LDS;
//      deep layers with few tiles split the channels over the wavefronts of a workgroup
//      and add the partial sums through LDS in fixed order
//   3. output transform  Y = A^T M A, clipped to P x Q, plus bias        (vector ALU)
// V and M live in the caller's workspace.  float16 storage keeps U, V and y in half
// precision; the transforms and the accumulation are float32.
// float32 F(2x2) / F(4x4) layers with many tiles and few channels run instead as ONE kernel
// (wino_fused_kernel below) that keeps V and M in registers and needs no workspace.
#include <climits>
#include <type_traits>
#include "nnv_internal.h"
#include "buf.h"
#include "wino_consts.h"

namespace nnv {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef half8_t half8;

struct WinoParams {
    const void *x;
    const void *U;
    void *V;
    float *M;
    const float *bias;
    void *y;
    int N, C, H, W, K, ph, pw, P, Q;
    int th, tw, T, T16;     // tiles per image (rows, cols), total tiles, 16-blocks of tiles
    int K16, cpad, csteps;  // cpad: channels padded to 4 (float32) / 32 (float16); csteps = cpad / that
    int ks_shift;           // wavefronts sharing one output tile (splitting the channels) = 1 << ks_shift
    int ntb;                // tile-block groups per frequency: ceil(T16 / TN)
    uint32_t u_bytes, v_bytes;   // sizes of U and V (range-checked loads)
    uint32_t x_bytes;            // size of x
    int relu;                    // outputs clamped at zero before the store
    int gemm_wgs_per_xi;         // workgroups per frequency in the tile GEMM
    int alpha2;                  // number of frequencies
};

// out[i][j] = sum_k L[i][k] * in[k][j] with a compile-time matrix L (zeros skipped).
#define NNV_MATMUL_LEFT(L, ROWS, INNER, COLS, in, out)                                  \
    _Pragma("unroll") for (int i_ = 0; i_ < ROWS; ++i_) _Pragma("unroll") for (int j_ = 0; j_ < COLS; ++j_) { \
        float acc_ = 0.f;                                                               \
        _Pragma("unroll") for (int k_ = 0; k_ < INNER; ++k_) if (L[i_][k_] != 0.f) acc_ += L[i_][k_] * in[k_][j_]; \
        out[i_][j_] = acc_;                                                             \
    }
// out[i][j] = sum_k in[i][k] * Rm[j][k]   (right-multiply by Rm^T)
#define NNV_MATMUL_RIGHT_T(Rm, ROWS, INNER, COLS, in, out)                              \
    _Pragma("unroll") for (int i_ = 0; i_ < ROWS; ++i_) _Pragma("unroll") for (int j_ = 0; j_ < COLS; ++j_) { \
        float acc_ = 0.f;                                                               \
        _Pragma("unroll") for (int k_ = 0; k_ < INNER; ++k_) if (Rm[j_][k_] != 0.f) acc_ += in[i_][k_] * Rm[j_][k_]; \
        out[i_][j_] = acc_;                                                             \
    }

// ---- 1. input transform.  Block = 16 tiles x 16 channels (float32: x blockDim/16 channels, so
// that small layers can be spread over more, smaller workgroups).
// (tb, by): tile block and channel group of the workgroup; bdim: its threads
template <int SET, bool HALF>
__device__ __forceinline__ void wino_input_block(const WinoParams &w, const int tb, const int by, const int bdim) {
    using Wm = WinoMat<SET>;
    constexpr int A = Wm::A, M = Wm::M;
    typedef typename std::conditional<HALF, __half, float>::type T;
    int t_in, c;
    if (HALF) {   // lanes: 8 channels fastest, then tiles -> 128 B contiguous half stores
        t_in = (threadIdx.x >> 3) & 15;
        c = by * 16 + (threadIdx.x >> 7) * 8 + (threadIdx.x & 7);
    } else {      // lanes: 16 tiles fastest, then channels -> 256 B contiguous stores
        t_in = threadIdx.x & 15;
        c = (by * bdim + threadIdx.x) >> 4;
    }
    if (c >= w.cpad) return;
    const int t = tb * 16 + t_in;
    // The alpha x alpha patch, all loads in flight at once: elements in the zero padding, of
    // tiles past the end and of padding channels get an out-of-range offset and read as zero.
    float d[A][A];
    {
        const bool live = t < w.T && c < w.C;
        const int tt = live ? t : 0, cc = live ? c : 0;
        const int per = w.th * w.tw;
        const int img = tt / per, rem = tt - img * per;
        const int ti = rem / w.tw, tj = rem - ti * w.tw;
        const int ih0 = ti * M - w.ph, iw0 = tj * M - w.pw;
        const int base = (img * w.C + cc) * w.H * w.W;
        const __amdgpu_buffer_rsrc_t xres = make_rsrc(w.x, w.x_bytes);
#pragma unroll
        for (int u = 0; u < A; ++u) {
            const int ih = ih0 + u;
            const bool rok = live && (unsigned)ih < (unsigned)w.H;
#pragma unroll
            for (int v = 0; v < A; ++v) {
                const int iw = iw0 + v;
                const bool ok = rok && (unsigned)iw < (unsigned)w.W;
                d[u][v] = buf_load_x<T>(xres, ok ? (uint32_t)(base + ih * w.W + iw) * (uint32_t)sizeof(T) : kOobOffset, 0u);
            }
        }
    }
    float tmp[A][A], V[A][A];
    NNV_MATMUL_LEFT(Wm::BT, A, A, A, d, tmp)
    NNV_MATMUL_RIGHT_T(Wm::BT, A, A, A, tmp, V)
    if (HALF) {
        __half *o = static_cast<__half *>(w.V) + ((size_t)tb * w.csteps + c / 32) * 512 + ((c % 32) / 8) * 128 + t_in * 8 + (c & 7);
        const size_t xs = (size_t)w.T16 * w.csteps * 512;
#pragma unroll
        for (int u = 0; u < A; ++u)
#pragma unroll
            for (int v = 0; v < A; ++v) o[(u * A + v) * xs] = __float2half_rn(V[u][v]);
    } else {
        float *o = static_cast<float *>(w.V) + ((size_t)tb * w.cpad + c) * 16 + t_in;
        const size_t xs = (size_t)w.T16 * w.cpad * 16;
#pragma unroll
        for (int u = 0; u < A; ++u)
#pragma unroll
            for (int v = 0; v < A; ++v) o[(u * A + v) * xs] = V[u][v];
    }
}

template <int SET, bool HALF>
__global__ __launch_bounds__(256) void wino_input_kernel(const WinoParams w) {
    wino_input_block<SET, HALF>(w, blockIdx.x, blockIdx.y, blockDim.x);
}

// ---- 2. batched tile GEMM.  grid = (tile-block groups, k-block groups, alpha^2).
template <bool HALF> struct WFrag {
    typedef float type;
    __device__ static inline float zero() { return 0.f; }
};
template <> struct WFrag<true> {
    typedef half8 type;
    __device__ static inline half8 zero() { return half8{0, 0, 0, 0, 0, 0, 0, 0}; }
};

// The k-loop is kept to loads and MFMAs: a lone wavefront on a SIMD issues one instruction
// every four cycles, so every select or address computation in the loop costs as much as a
// quarter of a float32 MFMA.  Offsets are a per-lane constant (or an out-of-range constant
// for fragments outside the problem) plus a scalar that advances by one fragment per step.
// One wavefront's tile of one frequency: TM x TN blocks of 16 x 16, summed over the ks-th of KS
// ranges of the channel steps; `red` is the workgroup's LDS (used if KS > 1), nt the wavefront's
// tile slot in it.
template <bool HALF, int TM, int TN, int D>
__device__ __forceinline__ void wino_gemm_tile(const WinoParams &w, const int xi, const int kb0, const int tb0,
                                               const int ks, const int KS, const int ks_shift, const int nt,
                                               const int lane, float *red) {
    typedef typename WFrag<HALF>::type frag_t;
    const __amdgpu_buffer_rsrc_t ures = make_rsrc(w.U, w.u_bytes);
    const __amdgpu_buffer_rsrc_t vres = make_rsrc(w.V, w.v_bytes);
    constexpr uint32_t FB = sizeof(frag_t), FRAG = 64 * FB;
    uint32_t a_voff[TM], b_voff[TN];
    uint32_t a_base[TM], b_base[TN];     // fragment index of step 0 (scalars)
#pragma unroll
    for (int m = 0; m < TM; ++m) {
        const bool ok = kb0 + m < w.K16;
        a_voff[m] = ok ? lane * FB : kOobOffset;
        a_base[m] = ok ? ((uint32_t)xi * w.K16 + kb0 + m) * w.csteps : 0u;
    }
#pragma unroll
    for (int t = 0; t < TN; ++t) {
        const bool ok = kb0 < w.K16 && tb0 + t < w.T16;
        b_voff[t] = ok ? lane * FB : kOobOffset;
        b_base[t] = ok ? ((uint32_t)xi * w.T16 + tb0 + t) * w.csteps : 0u;
    }
    const int per_wave = (w.csteps + KS - 1) >> ks_shift;
    const int s_begin = min(w.csteps, ks * per_wave);
    const int s_end = min(w.csteps, s_begin + per_wave);

    frag_t a[2][D][TM], b[2][D][TN];
    // chunk of D steps starting at step s0; steps past the end re-read the last valid step (unused)
    auto load_chunk = [&](int buf, int s0) {
#pragma unroll
        for (int d = 0; d < D; ++d) {
            const int st = max(min(s0 + d, s_end - 1), 0);
#pragma unroll
            for (int m = 0; m < TM; ++m) a[buf][d][m] = buf_load<frag_t>(ures, a_voff[m], (a_base[m] + st) * FRAG);
#pragma unroll
            for (int t = 0; t < TN; ++t) b[buf][d][t] = buf_load<frag_t>(vres, b_voff[t], (b_base[t] + st) * FRAG);
        }
    };
    floatx4 acc[TM][TN];
#pragma unroll
    for (int m = 0; m < TM; ++m)
#pragma unroll
        for (int t = 0; t < TN; ++t) acc[m][t] = floatx4{0.f, 0.f, 0.f, 0.f};
    auto mfma_step = [&](int buf, int d) {
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
    auto compute = [&](int buf, int s0) {
        if (s0 + D <= s_end) {
#pragma unroll
            for (int d = 0; d < D; ++d) mfma_step(buf, d);
        } else {
#pragma unroll
            for (int d = 0; d < D; ++d)
                if (s0 + d < s_end) mfma_step(buf, d);
        }
    };
    // (scheduling barriers: the loads of the next chunk stay in front of this chunk's MFMAs)
    if (s_begin < s_end) {
        load_chunk(0, s_begin);
        __builtin_amdgcn_sched_barrier(0);
        for (int s0 = s_begin; s0 < s_end; s0 += 2 * D) {
            load_chunk(1, s0 + D);
            __builtin_amdgcn_sched_barrier(0);
            compute(0, s0);
            __builtin_amdgcn_sched_barrier(0);
            load_chunk(0, s0 + 2 * D);
            __builtin_amdgcn_sched_barrier(0);
            if (s0 + D < s_end) compute(1, s0 + D);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
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
    // M[xi][kb][tb][16 k][16 t]: lane holds rows 4*(lane/16)+j, column lane%16
    const int col = lane & 15, slot = lane >> 4;
#pragma unroll
    for (int m = 0; m < TM; ++m) {
#pragma unroll
        for (int t = 0; t < TN; ++t) {
            const bool inb = kb0 + m < w.K16 && tb0 + t < w.T16;
            float *o = w.M + (((size_t)xi * w.K16 + kb0 + m) * w.T16 + tb0 + t) * 256 + slot * 64 + col;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int reg = (m * TN + t) * 4 + j;
                if ((reg & (KS - 1)) != ks) continue;
                float v = acc[m][t][j];
                if (KS > 1) {
                    v = 0.f;
                    for (int z = 0; z < KS; ++z) v += red[((nt * KS + z) * NREG + reg) * 64 + lane];
                }
                if (inb) o[j * 16] = v;
            }
        }
    }
}

template <bool HALF, int TM, int TN, int D>
__global__ __launch_bounds__(1024) void wino_gemm_kernel(const WinoParams w) {
    extern __shared__ __align__(16) float red[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // scalar
    const int KS = 1 << w.ks_shift;
    const int ks = wave & (KS - 1), nt = wave >> w.ks_shift;
    const int tiles_per_wg = (blockDim.x >> 6) >> w.ks_shift;
    // logical workgroup order: frequency slowest, so an XCD works on a few frequencies and keeps
    // their U and V panels in its own L2
    const int lwg = xcd_logical_tile(w.gemm_wgs_per_xi * w.alpha2);
    if (lwg < 0) return;
    const int xi = lwg / w.gemm_wgs_per_xi;
    const int tile = (lwg - xi * w.gemm_wgs_per_xi) * tiles_per_wg + nt;   // flattened (k-block group, tile-block group)
    const int kbt = tile / w.ntb, tbt = tile - kbt * w.ntb;
    wino_gemm_tile<HALF, TM, TN, D>(w, xi, kbt * TM, tbt * TN, ks, KS, w.ks_shift, nt, lane, red);   // kb0 >= K16 for surplus wavefronts
}

// Bias, optional clamp at zero and store of the M x M outputs of tile t, channel k, clipped to P x Q.
template <int M, bool HALF>
__device__ __forceinline__ void wino_store_tile(const WinoParams &w, float (&Y)[M][M], int t, int k) {
    const float bv = w.bias ? w.bias[k] : 0.f;
#pragma unroll
    for (int a = 0; a < M; ++a)
#pragma unroll
        for (int b = 0; b < M; ++b) {
            Y[a][b] += bv;
            if (w.relu) Y[a][b] = fmaxf(Y[a][b], 0.f);
        }
    const int per = w.th * w.tw;
    const int img = t / per, rem = t - img * per;
    const int ti = rem / w.tw, tj = rem - ti * w.tw;
    const size_t base = ((size_t)img * w.K + k) * w.P * w.Q;
    // Rows of a tile are stored VW elements at a time where Q is a multiple of VW (every group
    // of VW columns is then entirely inside the image and aligned): adjacent lanes hold
    // adjacent tiles, so a wavefront writes contiguous runs instead of 4-byte pieces.
    constexpr int VW = M % 4 == 0 ? 4 : 2;
    const bool vec = w.Q % VW == 0;
#pragma unroll
    for (int a = 0; a < M; ++a) {
        const int p = ti * M + a;
        if (p >= w.P) continue;
        if (vec) {
#pragma unroll
            for (int b = 0; b < M; b += VW) {
                const int q = tj * M + b;
                if (q >= w.Q) continue;
                const size_t o = base + (size_t)p * w.Q + q;
                if constexpr (HALF) {
                    uint32_t pk[VW / 2];
#pragma unroll
                    for (int i = 0; i < VW / 2; ++i) {
                        __half2 h = __floats2half2_rn(Y[a][b + 2 * i], Y[a][b + 2 * i + 1]);
                        pk[i] = *reinterpret_cast<uint32_t *>(&h);
                    }
                    if constexpr (VW == 4) *reinterpret_cast<uint2 *>(static_cast<__half *>(w.y) + o) = make_uint2(pk[0], pk[1]);
                    else *reinterpret_cast<uint32_t *>(static_cast<__half *>(w.y) + o) = pk[0];
                } else {
                    if constexpr (VW == 4)
                        *reinterpret_cast<float4 *>(static_cast<float *>(w.y) + o) =
                            make_float4(Y[a][b], Y[a][b + 1], Y[a][b + 2], Y[a][b + 3]);
                    else
                        *reinterpret_cast<float2 *>(static_cast<float *>(w.y) + o) = make_float2(Y[a][b], Y[a][b + 1]);
                }
            }
        } else {
#pragma unroll
            for (int b = 0; b < M; ++b) {
                const int q = tj * M + b;
                if (q >= w.Q) continue;
                const float v = Y[a][b];
                if (HALF) static_cast<__half *>(w.y)[base + (size_t)p * w.Q + q] = __float2half_rn(v);
                else static_cast<float *>(w.y)[base + (size_t)p * w.Q + q] = v;
            }
        }
    }
}

// ---- 3. output transform.  Block = 16 tiles x blockDim/16 output channels.
template <int SET, bool HALF>
__device__ __forceinline__ void wino_output_block(const WinoParams &w, const int tb, const int by, const int bdim) {
    using Wm = WinoMat<SET>;
    constexpr int A = Wm::A, M = Wm::M;
    const int t_in = threadIdx.x & 15;
    const int k = (by * bdim + threadIdx.x) >> 4, kb = k >> 4, k_in = k & 15;
    const int t = tb * 16 + t_in;
    if (t >= w.T || k >= w.K) return;
    const float *mp = w.M + ((size_t)kb * w.T16 + tb) * 256 + k_in * 16 + t_in;
    const size_t xs = (size_t)w.K16 * w.T16 * 256;
    float m[A][A];
#pragma unroll
    for (int u = 0; u < A; ++u)
#pragma unroll
        for (int v = 0; v < A; ++v) m[u][v] = mp[(u * A + v) * xs];
    float tmp[M][A], Y[M][M];
    NNV_MATMUL_LEFT(Wm::AT, M, A, A, m, tmp)
    NNV_MATMUL_RIGHT_T(Wm::AT, M, A, M, tmp, Y)
    wino_store_tile<M, HALF>(w, Y, t, k);
}

template <int SET, bool HALF>
__global__ __launch_bounds__(256) void wino_output_kernel(const WinoParams w) {
    wino_output_block<SET, HALF>(w, blockIdx.x, blockIdx.y, blockDim.x);
}

// ---- many layers of one Winograd variant and storage type in three launches (input transforms,
// tile GEMMs, output transforms of all of them), for the same reason as the implicit GEMM's
// work-item launch: a batch-1 layer fills neither the chip nor the time its launch takes.
// A workgroup finds its layer by counting the entries of a prefix array it has reached.
constexpr int kWinoItemWaves = 4;
struct WinoTable {
    WinoParams layer[kMaxWinoLayers];
    int in0[kMaxWinoLayers];      // first workgroup of each layer: input transform,
    int gemm0[kMaxWinoLayers];    //   tile GEMM (workgroups of work items: frequency x tile),
    int out0[kMaxWinoLayers];     //   output transform; INT_MAX beyond the last layer
    int in_by[kMaxWinoLayers], out_by[kMaxWinoLayers];     // channel groups per tile block (the "y" extent of the single launches)
    int tm[kMaxWinoLayers], tn[kMaxWinoLayers];            // tile of the GEMM items
    int n_in, n_gemm, n_out;
    int gemm_waves;               // wavefronts per tile-GEMM workgroup: 1 or kWinoItemWaves
};
static_assert(sizeof(WinoTable) <= 4096, "the table is passed by value as the kernel argument");
typedef const __attribute__((address_space(4))) WinoTable *WinoTablePtr;

__device__ __forceinline__ void load_wino_layer(WinoParams &dst, const WinoTablePtr tbl, const int li) {
    static_assert(sizeof(WinoParams) % 4 == 0, "copied word by word");
    const __attribute__((address_space(4))) uint32_t *src = (const __attribute__((address_space(4))) uint32_t *)&tbl->layer[li];
    uint32_t *d = reinterpret_cast<uint32_t *>(&dst);
#pragma unroll
    for (int i = 0; i < (int)(sizeof(WinoParams) / 4); ++i) d[i] = src[i];
}

#define NNV_FIND_LAYER(prefix, b, li, first) \
    int first;                               \
    const int li = table_find<kMaxWinoLayers>(&tbl->prefix[0], (b), first);

template <int SET, bool HALF>
__global__ __launch_bounds__(256) void wino_input_many_kernel(const WinoTable tbl_arg) {
    const WinoTablePtr tbl = (WinoTablePtr)__builtin_amdgcn_kernarg_segment_ptr();
    const int b = blockIdx.x;
    NNV_FIND_LAYER(in0, b, li, first)
    WinoParams w;
    load_wino_layer(w, tbl, li);
    const int local = b - first, by_n = tbl->in_by[li];
    wino_input_block<SET, HALF>(w, local / by_n, local % by_n, 256);
}

template <int SET, bool HALF>
__global__ __launch_bounds__(256) void wino_output_many_kernel(const WinoTable tbl_arg) {
    const WinoTablePtr tbl = (WinoTablePtr)__builtin_amdgcn_kernarg_segment_ptr();
    const int b = blockIdx.x;
    NNV_FIND_LAYER(out0, b, li, first)
    WinoParams w;
    load_wino_layer(w, tbl, li);
    const int local = b - first, by_n = tbl->out_by[li];
    wino_output_block<SET, HALF>(w, local / by_n, local % by_n, 256);
}

// Tile GEMM work items (frequency x tile).  A launch of many items runs one item per one-wavefront
// workgroup.  A launch of few items uses workgroups of kWinoItemWaves wavefronts, and a layer with
// many channel steps gives each item to 2 or 4 of them that split the steps (summed through LDS in
// a fixed order): a lone wavefront streams its U panel at the pace of the few loads it keeps in
// flight, and the 128-step items of a 512-channel layer took 35 us each, as long as the rest of
// the launch; the wavefronts of a workgroup otherwise take consecutive items.  Items of a layer
// are ordered frequency slowest; groups of 8 consecutive workgroups go to one XCD.
template <bool HALF>
__global__ __launch_bounds__(64 * kWinoItemWaves) void wino_gemm_many_kernel(const WinoTable tbl_arg) {
    extern __shared__ __align__(16) float red[];      // kWinoItemWaves x 16 accumulator registers x 64 lanes
    const WinoTablePtr tbl = (WinoTablePtr)__builtin_amdgcn_kernarg_segment_ptr();
    constexpr int G = 8;
    const int i = blockIdx.x, xcd = i & 7, j = i >> 3;
    const int wg = ((j / G) * 8 + xcd) * G + j % G;
    if (wg >= tbl->n_gemm) return;
    NNV_FIND_LAYER(gemm0, wg, li, first)
    WinoParams w;
    load_wino_layer(w, tbl, li);
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int KS = 1 << w.ks_shift, ks = wave & (KS - 1), nt = wave >> w.ks_shift;
    const int local = (wg - first) * ((int)(blockDim.x >> 6) >> w.ks_shift) + nt;
    const int tm = tbl->tm[li], tn = tbl->tn[li];
    const int per_xi = w.gemm_wgs_per_xi;                 // tiles per frequency
    const bool surplus = local >= per_xi * w.alpha2;      // the last workgroup of a layer may hold fewer items
    const int xi = surplus ? 0 : local / per_xi, tile = local - xi * per_xi;
    const int kbt = surplus ? w.K16 : tile / w.ntb, tbt = surplus ? 0 : tile - kbt * w.ntb;   // kb0 >= K16: nothing loaded, nothing stored
    constexpr int D = HALF ? 2 : 4;     // float32: a ring of 4 steps keeps the kernel at 71 registers (7 wavefronts per SIMD); 8 steps and 4 wavefronts were measured: 8-11 % slower on small stacks
    if (tm == 2 && tn == 2) wino_gemm_tile<HALF, 2, 2, D>(w, xi, kbt * 2, tbt * 2, ks, KS, w.ks_shift, nt, lane, red);
    else if (tm == 2) wino_gemm_tile<HALF, 2, 1, D>(w, xi, kbt * 2, tbt, ks, KS, w.ks_shift, nt, lane, red);
    else wino_gemm_tile<HALF, 1, 1, D>(w, xi, kbt, tbt, ks, KS, w.ks_shift, nt, lane, red);
}

// ---- fused variant (float32, F(2x2) and F(4x4)): all three steps in one kernel, no workspace.
// On layers with many tiles and few output channels the three-kernel route spends most of its
// time writing and re-reading V and M.  Here a wavefront owns 16 tiles x 16 output channels.
// Per step of 4 input channels every lane transforms the patch of one (tile, channel) pair in
// registers: lane (tile l%16, channel l/16) then holds, for every frequency, exactly its element
// of the B operand of the 16x16x4 MFMA.  The alpha^2 accumulators stay in registers and the
// output transform is applied to them in place (accumulator register j of lane l is output
// channel 4*(l/16)+j of tile l%16).  The input transform is repeated by every 16-channel block
// of K, which is what restricts this route to layers with few output channels.
template <int SET>
__global__ __launch_bounds__(256) void wino_fused_kernel(const WinoParams w) {
    using Wm = WinoMat<SET>;
    constexpr int A = Wm::A, M = Wm::M, AA = A * A;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // logical order: tile blocks fastest, so neighbouring workgroups share U; the four
    // wavefronts of a workgroup share the patches (same tiles, four blocks of output channels)
    const int lwg = xcd_logical_tile(w.gemm_wgs_per_xi);
    if (lwg < 0) return;
    const int kbg = lwg / w.T16, tb = lwg - kbg * w.T16;
    const int kb = kbg * 4 + wave;
    if (kb >= w.K16) return;
    const int col = lane & 15, slot = lane >> 4;
    const int t = tb * 16 + col;
    const bool live = t < w.T;
    const __amdgpu_buffer_rsrc_t xres = make_rsrc(w.x, w.x_bytes);
    const __amdgpu_buffer_rsrc_t ures = make_rsrc(w.U, w.u_bytes);
    const uint32_t plane4 = (uint32_t)(w.H * w.W) * 16u;     // bytes of 4 channel planes
    // per-lane byte offsets of the patch rows and columns in channel `slot`; a step adds its
    // channel base as the scalar offset.  Rows and columns in the zero padding (and every row of
    // a surplus tile) carry 2^30 instead, which puts the sum beyond the end of x (x is smaller
    // than 2^30 bytes on this route), so those elements read as zero.
    constexpr uint32_t kOut = 0x40000000u;
    uint32_t rowoff[A], coloff[A];
    {
        const int tt = live ? t : 0;
        const int per = w.th * w.tw;
        const int img = tt / per, rem = tt - img * per;
        const int ti = rem / w.tw, tj = rem - ti * w.tw;
        const int ih0 = ti * M - w.ph, iw0 = tj * M - w.pw;
        const int base = (img * w.C + slot) * w.H * w.W;
#pragma unroll
        for (int u = 0; u < A; ++u) {
            const int ih = ih0 + u;
            rowoff[u] = (live && (unsigned)ih < (unsigned)w.H) ? (uint32_t)(base + ih * w.W) * 4u : kOut;
        }
#pragma unroll
        for (int v = 0; v < A; ++v) {
            const int iw = iw0 + v;
            coloff[v] = (unsigned)iw < (unsigned)w.W ? (uint32_t)iw * 4u : kOut;
        }
    }
    const uint32_t a_voff = lane * 4u;
    const uint32_t a_base = (uint32_t)kb * w.csteps;          // fragment index at frequency 0, step 0
    const uint32_t a_xi = (uint32_t)w.K16 * w.csteps;         // fragments per frequency
    floatx4 acc[AA];
#pragma unroll
    for (int i = 0; i < AA; ++i) acc[i] = floatx4{0.f, 0.f, 0.f, 0.f};
    // Everything a step needs is requested one step earlier.  Patches alternate between two
    // register sets; the U fragment of frequency i is re-requested for the next step right
    // after the MFMA that consumed it, into the same register.  Loads complete in order, and
    // the order of issue is patch(s), U(s), patch(s+1), U(s+1), ..., so waiting for one of
    // them never waits for anything requested later.  The scheduling barriers keep that order.
    float d[2][A][A], a[AA];
    const int full = w.C >> 2;                                // steps whose 4 channels all exist
    const int last = w.csteps - 1;
    auto load_patch = [&](int buf, int s) __attribute__((always_inline)) {
        const uint32_t soff = (uint32_t)s * plane4;
#pragma unroll
        for (int u = 0; u < A; ++u)
#pragma unroll
            for (int v = 0; v < A; ++v) d[buf][u][v] = buf_load<float>(xres, rowoff[u] + coloff[v], soff);
        __builtin_amdgcn_sched_barrier(0);
    };
    auto load_a = [&](int i, int s) __attribute__((always_inline)) {
        a[i] = buf_load<float>(ures, a_voff, (a_base + (uint32_t)i * a_xi + s) * 256u);
    };
    auto step = [&](int buf, int s) __attribute__((always_inline)) {
        float tmp[A][A], V[A][A];
        NNV_MATMUL_LEFT(Wm::BT, A, A, A, d[buf], tmp)
        NNV_MATMUL_RIGHT_T(Wm::BT, A, A, A, tmp, V)
        const int sn = min(s + 1, last);
#pragma unroll
        for (int i = 0; i < AA; ++i) {
            acc[i] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[i], V[i / A][i % A], acc[i], 0, 0, 0);
            load_a(i, sn);
        }
        __builtin_amdgcn_sched_barrier(0);
    };
    if (full > 0) load_patch(0, 0);
#pragma unroll
    for (int i = 0; i < AA; ++i) load_a(i, 0);
    __builtin_amdgcn_sched_barrier(0);
    if (full > 0) {
        int s = 0;
        for (; s + 2 <= full; s += 2) {
            load_patch(1, s + 1);
            step(0, s);
            load_patch(0, min(s + 2, full - 1));
            step(1, s + 1);
        }
        if (s < full) step(0, s);
    }
    if (w.C & 3) {
        // last step of a channel count that is not a multiple of 4: lanes of missing channels read zero
        const bool cok = full * 4 + slot < w.C;
        const uint32_t soff = (uint32_t)full * plane4;
#pragma unroll
        for (int u = 0; u < A; ++u)
#pragma unroll
            for (int v = 0; v < A; ++v) d[0][u][v] = buf_load<float>(xres, cok ? rowoff[u] + coloff[v] : kOobOffset, soff);
        __builtin_amdgcn_sched_barrier(0);
        step(0, full);
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int k = kb * 16 + slot * 4 + j;
        if (!live || k >= w.K) continue;
        float m[A][A], tmp[M][A], Y[M][M];
#pragma unroll
        for (int u = 0; u < A; ++u)
#pragma unroll
            for (int v = 0; v < A; ++v) m[u][v] = acc[u * A + v][j];
        NNV_MATMUL_LEFT(Wm::AT, M, A, A, m, tmp)
        NNV_MATMUL_RIGHT_T(Wm::AT, M, A, M, tmp, Y)
        wino_store_tile<M, false>(w, Y, t, k);
    }
}

// ---------------------------------------------------------------- host side

struct WinoPlan {
    int m, alpha, th, tw, T, T16, K16, cpad, csteps;
    size_t v_bytes, m_bytes;
};

static WinoPlan plan_wino(const Geo &g, int kind) {
    WinoPlan p{};
    const bool half = g.dtype == NNV_F16;
    p.m = wino_m(kind);
    p.alpha = p.m + 2;
    p.th = ceil_div(g.p, p.m);
    p.tw = ceil_div(g.q, p.m);
    p.T = g.n * p.th * p.tw;
    p.T16 = ceil_div(p.T, 16);
    p.K16 = ceil_div(g.k, 16);
    const int cb = half ? 32 : 4;
    p.csteps = ceil_div(g.c, cb);
    p.cpad = p.csteps * cb;
    const size_t aa = (size_t)p.alpha * p.alpha;
    p.v_bytes = align_up(aa * p.T16 * 16 * p.cpad * (half ? 2 : 4), 256);
    p.m_bytes = align_up(aa * p.K16 * p.T16 * 256 * sizeof(float), 256);
    return p;
}

// The fused kernel repeats the input transform (and the strided patch loads, which dominate its
// time) once per 16 output channels and runs one or two wavefronts per SIMD, so it pays only
// where the three-kernel route is dominated by launch floors and by its V and M round trips.
// The choice compares two estimates fitted to a sweep over 48..224-pixel planes, 4..64 input
// and 16..128 output channels (they pick the faster route, or one within 5 %, at every point):
//   fused = 4 us + y / 2.3 TB/s + channel steps x time per step x max(1, workgroups / 256);
//           a step takes 0.47 us (F(2x2)) or 1.9 us (F(4x4)) for a lone wavefront on a CU and
//           0.16 / 0.5 us more for each further wavefront of the workgroup
//   three = 8 us + 2 (V + M) / 3 TB/s
// e.g. 3 -> 64 channels at 224x224, F(4x4): 11 us fused against 32 us; 64 -> 64 at 56x56,
// F(2x2): 21 us fused against 13 us.  Outside the swept range the three kernels are kept.
static bool wino_fused(const Geo &g, int kind, const WinoPlan &p) {
    if (g.dtype != NNV_F32 || (kind != NNV_WINO_F2 && kind != NNV_WINO_F4)) return false;
    const size_t x_bytes = (size_t)g.n * g.c * g.h * g.w * 4;
    if (p.T16 < 32 || p.K16 > 8 || p.csteps > 16 || x_bytes >= ((size_t)1 << 30)) return false;
    const double wgs = (double)p.T16 * ceil_div(p.K16, 4);
    const double rounds = wgs > 256.0 ? wgs / 256.0 : 1.0;
    const int waves = p.K16 < 4 ? p.K16 : 4;
    const double step_us = kind == NNV_WINO_F2 ? 0.47 + 0.16 * (waves - 1) : 1.9 + 0.5 * (waves - 1);
    const double y_mb = (double)g.n * g.k * g.p * g.q * 4e-6;
    const double fused_us = 4.0 + y_mb / 2.3 + p.csteps * step_us * rounds;
    const double three_us = 8.0 + 2.0 * (double)(p.v_bytes + p.m_bytes) * 1e-6 / 3.0;
    return fused_us < three_us;
}

size_t wino_workspace_bytes(const Geo &g, int kind) {
    const WinoPlan p = plan_wino(g, kind);
    if (wino_fused(g, kind, p)) return 0;
    return p.v_bytes + p.m_bytes;
}

template <int SET>
static hipError_t launch_wino_fused(const WinoPlan &p, WinoParams &w, hipStream_t st) {
    w.u_bytes = (uint32_t)((size_t)p.alpha * p.alpha * p.K16 * p.csteps * 256);
    w.gemm_wgs_per_xi = p.T16 * ceil_div(p.K16, 4);
    hipLaunchKernelGGL((wino_fused_kernel<SET>), dim3(xcd_grid(w.gemm_wgs_per_xi)), dim3(256), 0, st, w);
    return hipGetLastError();
}

template <int SET, bool HALF>
static hipError_t launch_wino_t(const Geo &g, const WinoPlan &p, WinoParams &w, hipStream_t st) {
    {
        // one wavefront per workgroup (16 tiles x 4 channels) while that keeps the launch small:
        // a batch-1 layer then occupies four times as many CUs
        const int bt = (!HALF && (long)p.T16 * ceil_div(p.cpad, 16) < 4096) ? 64 : 256;
        dim3 grid(p.T16, HALF ? ceil_div(p.cpad, 16) : ceil_div(p.cpad * 16, bt), 1);
        hipLaunchKernelGGL((wino_input_kernel<SET, HALF>), grid, dim3(bt), 0, st, w);
    }
    {
        // wavefront tile, channel split and workgroup shape: cover >= 1024 wavefronts if possible
        const long aa = (long)p.alpha * p.alpha;
        // latency-bound at batch 1 (measured on ResNet-18-shaped layers): the largest wavefront
        // tile that still leaves >= 768 wavefronts; then split the channel steps over the
        // wavefronts of a workgroup towards ~4 per SIMD, keeping >= 16 steps each
        int tm = 1, tn = 1;
        if (p.T16 >= 2 && aa * ceil_div(p.K16, 2) * ceil_div(p.T16, 2) >= 768) { tm = 2; tn = 2; }
        else if (aa * ceil_div(p.K16, 2) * p.T16 >= 768) { tm = 2; }
        int shift = 0;
        const long tiles = (long)ceil_div(p.K16, tm) * ceil_div(p.T16, tn);
        while (shift < 4 && ((aa * tiles) << shift) < 4096 && (p.csteps >> (shift + 1)) >= (HALF ? 4 : 16)) ++shift;
        const int d = HALF ? 2 : 8;
        w.ks_shift = shift;
        w.ntb = ceil_div(p.T16, tn);
        w.u_bytes = (uint32_t)((size_t)aa * p.K16 * p.csteps * 64 * (HALF ? 16 : 4));
        w.v_bytes = (uint32_t)((size_t)aa * p.T16 * p.csteps * 64 * (HALF ? 16 : 4));
        const int KS = 1 << shift;
        const int waves = KS;
        const int tiles_per_wg = waves / KS;
        const long ntiles = (long)ceil_div(p.K16, tm) * w.ntb;
        w.gemm_wgs_per_xi = ceil_div((int)ntiles, tiles_per_wg);
        w.alpha2 = (int)aa;
        dim3 grid(xcd_grid(w.gemm_wgs_per_xi * (int)aa), 1, 1);
        dim3 block(64 * waves);
        const size_t lds = KS > 1 ? (size_t)waves * tm * tn * 4 * 64 * sizeof(float) : 0;
        if constexpr (HALF) {
            if (tm == 2 && tn == 2) hipLaunchKernelGGL((wino_gemm_kernel<HALF, 2, 2, 2>), grid, block, lds, st, w);
            else if (tm == 2 && tn == 1) hipLaunchKernelGGL((wino_gemm_kernel<HALF, 2, 1, 2>), grid, block, lds, st, w);
            else hipLaunchKernelGGL((wino_gemm_kernel<HALF, 1, 1, 2>), grid, block, lds, st, w);
        } else if (d == 4) {
            if (tm == 2 && tn == 2) hipLaunchKernelGGL((wino_gemm_kernel<false, 2, 2, 4>), grid, block, lds, st, w);
            else if (tm == 2 && tn == 1) hipLaunchKernelGGL((wino_gemm_kernel<false, 2, 1, 4>), grid, block, lds, st, w);
            else hipLaunchKernelGGL((wino_gemm_kernel<false, 1, 1, 4>), grid, block, lds, st, w);
        } else {
            if (tm == 2 && tn == 2) hipLaunchKernelGGL((wino_gemm_kernel<false, 2, 2, 8>), grid, block, lds, st, w);
            else if (tm == 2 && tn == 1) hipLaunchKernelGGL((wino_gemm_kernel<false, 2, 1, 8>), grid, block, lds, st, w);
            else hipLaunchKernelGGL((wino_gemm_kernel<false, 1, 1, 8>), grid, block, lds, st, w);
        }
    }
    {
        const int bt = (long)p.T16 * p.K16 < 4096 ? 64 : 256;
        dim3 grid(p.T16, p.K16 * (256 / bt), 1);
        hipLaunchKernelGGL((wino_output_kernel<SET, HALF>), grid, dim3(bt), 0, st, w);
    }
    return hipGetLastError();
}

static WinoParams wino_params(const Geo &g, const WinoPlan &p, const void *x, const void *U, const float *bias, void *y,
                              void *ws) {
    const bool half = g.dtype == NNV_F16;
    WinoParams w{};
    w.x = x; w.U = U; w.bias = bias; w.y = y;
    w.V = ws;
    w.M = reinterpret_cast<float *>(static_cast<char *>(ws) + p.v_bytes);
    w.N = g.n; w.C = g.c; w.H = g.h; w.W = g.w; w.K = g.k; w.ph = g.ph; w.pw = g.pw; w.P = g.p; w.Q = g.q;
    w.x_bytes = (uint32_t)((size_t)g.n * g.c * g.h * g.w * (half ? 2 : 4));
    w.relu = g.relu;
    w.th = p.th; w.tw = p.tw; w.T = p.T; w.T16 = p.T16; w.K16 = p.K16; w.cpad = p.cpad; w.csteps = p.csteps;
    const size_t aa = (size_t)p.alpha * p.alpha;
    w.u_bytes = (uint32_t)(aa * p.K16 * p.csteps * 64 * (half ? 16 : 4));
    w.v_bytes = (uint32_t)(aa * p.T16 * p.csteps * 64 * (half ? 16 : 4));
    w.alpha2 = (int)aa;
    return w;
}

bool wino_many_supported(const Geo &g, int kind) {
    const WinoPlan p = plan_wino(g, kind);
    return !wino_fused(g, kind, p) && p.T16 <= (1 << 20) && p.K16 <= 65535;
}

template <int SET, bool HALF>
static void launch_wino_many_t(const WinoTable &tbl, hipStream_t st) {
    hipLaunchKernelGGL((wino_input_many_kernel<SET, HALF>), dim3(tbl.n_in), dim3(256), 0, st, tbl);
    const int per_xcd = ceil_div(ceil_div(tbl.n_gemm, 8), 8) * 8;
    hipLaunchKernelGGL((wino_gemm_many_kernel<HALF>), dim3(per_xcd * 8), dim3(64 * tbl.gemm_waves),
                       (size_t)tbl.gemm_waves * 16 * 64 * sizeof(float), st, tbl);
    hipLaunchKernelGGL((wino_output_many_kernel<SET, HALF>), dim3(tbl.n_out), dim3(256), 0, st, tbl);
}

// Layers [0, n) of one Winograd kind and storage type (n <= kMaxWinoLayers, none of them on the
// fused route) in three launches; ws[i] is layer i's own region of wino_workspace_bytes.
hipError_t launch_wino_many(int n, const Geo *geos, int kind, const void *const *x, const void *const *U,
                            const float *const *bias, void *const *y, void *const *ws, hipStream_t st) {
    if (n <= 0) return hipSuccess;
    if (n > kMaxWinoLayers) return hipErrorInvalidValue;
    const bool half = geos[0].dtype == NNV_F16;
    WinoTable tbl{};
    long n_in = 0, n_gemm = 0, n_out = 0;
    // a launch of few items (less than two rounds of the chip's wavefront slots) ends with its longest
    // items: there the items of layers with many channel steps are split over 2 or 4 wavefronts
    long items = 0;
    for (int i = 0; i < n; ++i) {
        const WinoPlan p = plan_wino(geos[i], kind);
        const int tm = p.K16 >= 2 ? 2 : 1, tn = (tm == 2 && p.T16 >= 2) ? 2 : 1;
        items += (long)p.alpha * p.alpha * ceil_div(p.K16, tm) * ceil_div(p.T16, tn);
    }
    const bool split = items < 8192;
    tbl.gemm_waves = split ? kWinoItemWaves : 1;
    for (int i = 0; i < n; ++i) {
        const Geo &g = geos[i];
        if ((g.dtype == NNV_F16) != half || !wino_many_supported(g, kind)) return hipErrorInvalidValue;
        const WinoPlan p = plan_wino(g, kind);
        WinoParams &w = tbl.layer[i];
        w = wino_params(g, p, x[i], U[i], bias ? bias[i] : nullptr, y[i], ws[i]);
        // tile of a GEMM item: as large as the layer allows (the launch holds thousands of items)
        const int tm = p.K16 >= 2 ? 2 : 1, tn = (tm == 2 && p.T16 >= 2) ? 2 : 1;
        // then at most about 32 channel steps per wavefront
        w.ks_shift = !split ? 0 : p.csteps > 64 ? 2 : p.csteps > 32 ? 1 : 0;
        w.ntb = ceil_div(p.T16, tn);
        w.gemm_wgs_per_xi = ceil_div(p.K16, tm) * w.ntb;
        tbl.tm[i] = tm; tbl.tn[i] = tn;
        tbl.in_by[i] = half ? p.cpad / 16 : ceil_div(p.cpad * 16, 256);
        tbl.out_by[i] = p.K16;
        tbl.in0[i] = (int)n_in; tbl.gemm0[i] = (int)n_gemm; tbl.out0[i] = (int)n_out;
        n_in += (long)p.T16 * tbl.in_by[i];
        n_gemm += ceil_div(w.alpha2 * w.gemm_wgs_per_xi, tbl.gemm_waves >> w.ks_shift);
        n_out += (long)p.T16 * tbl.out_by[i];
        if (n_in >= (1L << 30) || n_gemm >= (1L << 30) || n_out >= (1L << 30)) return hipErrorInvalidValue;
    }
    for (int i = n; i < kMaxWinoLayers; ++i) tbl.in0[i] = tbl.gemm0[i] = tbl.out0[i] = INT_MAX;
    tbl.n_in = (int)n_in; tbl.n_gemm = (int)n_gemm; tbl.n_out = (int)n_out;
    const int set = wino_set(kind, geos[0].dtype);
    if (set == WS_F2) { if (half) launch_wino_many_t<0, true>(tbl, st); else launch_wino_many_t<0, false>(tbl, st); }
    else if (set == WS_F4) launch_wino_many_t<1, false>(tbl, st);
    else if (set == WS_F6) launch_wino_many_t<3, false>(tbl, st);
    else launch_wino_many_t<2, true>(tbl, st);
    return hipGetLastError();
}

hipError_t launch_wino(const Geo &g, int kind, const void *x, const void *U, const float *bias, void *y, void *ws,
                       hipStream_t st) {
    const WinoPlan p = plan_wino(g, kind);
    if (p.T16 > 65535 * 16 || p.K16 > 65535) return hipErrorInvalidValue;
    WinoParams w{};
    w.x = x; w.U = U; w.bias = bias; w.y = y;
    w.V = ws;
    w.M = reinterpret_cast<float *>(static_cast<char *>(ws) + p.v_bytes);
    w.N = g.n; w.C = g.c; w.H = g.h; w.W = g.w; w.K = g.k; w.ph = g.ph; w.pw = g.pw; w.P = g.p; w.Q = g.q;
    w.x_bytes = (uint32_t)((size_t)g.n * g.c * g.h * g.w * (g.dtype == NNV_F16 ? 2 : 4));
    w.relu = g.relu;
    w.th = p.th; w.tw = p.tw; w.T = p.T; w.T16 = p.T16; w.K16 = p.K16; w.cpad = p.cpad; w.csteps = p.csteps;
    const int set = wino_set(kind, g.dtype);
    if (wino_fused(g, kind, p)) {
        if (set == WS_F2) return launch_wino_fused<0>(p, w, st);
        return launch_wino_fused<1>(p, w, st);
    }
    if (set == WS_F2) {
        if (g.dtype == NNV_F16) return launch_wino_t<0, true>(g, p, w, st);
        return launch_wino_t<0, false>(g, p, w, st);
    }
    if (set == WS_F4) return launch_wino_t<1, false>(g, p, w, st);
    if (set == WS_F6) return launch_wino_t<3, false>(g, p, w, st);
    return launch_wino_t<2, true>(g, p, w, st);
}

}  // namespace nnv
