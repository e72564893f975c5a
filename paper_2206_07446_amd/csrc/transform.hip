// Weight-transformation kernels: raw OIHW float32 -> the layout a kernel executes from
// (the operation w_i of Section 3.2; Section 2 "weights transformation", Fig. 3).
//
// All of them are bandwidth-bound permutations (plus the tiny G g G^T product for
// Winograd), so the design goal is full-width coalesced reads and writes:
//   * a block owns 16 output channels (one fragment row group) and a chunk of input
//     channels; it stages the 16 contiguous row segments of the raw tensor in LDS with
//     coalesced (float4 when aligned) loads,
//   * threads then read their filter taps from LDS with the k-index fastest, so every
//     wavefront store is one contiguous 256 B .. 1 KB piece of the output fragment.
// One launch can carry many layers (a job table passed by value as kernel argument),
// because single layers of a batch-1 CNN are far too small to fill 256 CUs.
#include <climits>
#include "nnv_internal.h"
#include "wino_consts.h"
#include "buf.h"

namespace nnv {

static constexpr int kRows = 16;   // output channels per block / fragment

__host__ __device__ static inline int lds_row_stride(int rowlen) {
    // multiple of 64 plus 4: 16 rows x odd tap strides map to distinct LDS banks
    return ((rowlen + 63) / 64) * 64 + 4;
}

// Stage rows k0..k0+15, columns [col0, col0+len_valid) of a (K x rowstride) float matrix
// into lds[row * ROW + col], zero-filling up to len_fill and for rows >= K.
__device__ static inline void stage_rows(const float *__restrict__ src, float *lds, int ROW, int k0, int K,
                                         size_t rowstride, size_t col0, int len_valid, int len_fill) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const bool vec = ((rowstride & 3) == 0) && ((col0 & 3) == 0) && ((len_valid & 3) == 0);
    const int fill4 = (len_fill + 3) >> 2;
    for (int rr = 0; rr < kRows / 4; ++rr) {
        const int row = wave * (kRows / 4) + rr;
        const int k = k0 + row;
        const float *rp = src + (size_t)k * rowstride + col0;
        float *lp = lds + row * ROW;
        if (vec) {
            const int valid4 = (k < K) ? (len_valid >> 2) : 0;
            for (int i = lane; i < fill4; i += 64) {
                float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
                if (i < valid4) v = reinterpret_cast<const float4 *>(rp)[i];
                reinterpret_cast<float4 *>(lp)[i] = v;
            }
        } else {
            const int valid = (k < K) ? len_valid : 0;
            for (int i = lane; i < fill4 * 4; i += 64) {
                float v = 0.f;
                if (i < valid) v = rp[i];
                lp[i] = v;
            }
        }
    }
    __syncthreads();
}

// Transformed weights are written once and not read again by this kernel: non-temporal stores
// keep them from displacing the raw weights (which several jobs of a launch share) in L2.
typedef uint32_t uint2v __attribute__((ext_vector_type(2)));
typedef uint32_t uint4v __attribute__((ext_vector_type(4)));
template <typename V> __device__ static inline void nt_store(V *p, V v) { __builtin_nontemporal_store(v, p); }

__device__ static inline uint32_t pack_half2(float a, float b) {
    __half2 h = __floats2half2_rn(a, b);
    return *reinterpret_cast<uint32_t *>(&h);
}

// Channels per block of a Winograd job: 32 in float32 (21 KB of LDS per block, seven blocks per CU;
// measured 4 % faster than 64), 64 in float16 (a wavefront packs 8 channels per lane pair).
__host__ __device__ constexpr int wino_chunk(bool half) { return half ? 64 : 32; }

// Winograd weight transformation of one block: 16 output channels x up to wino_chunk channels.
template <int SET, bool HALF>
__device__ static inline void wino_block(const TransformJob &job, int local_block, float *lds) {
    using W = WinoMat<SET>;
    constexpr int AA = W::A * W::A;
    const int kb = local_block / job.nchunks, chunk = local_block % job.nchunks;
    const int K16 = (job.K + 15) / 16;
    const int cpad = HALF ? ((job.C + 31) / 32) * 32 : ((job.C + 3) / 4) * 4;
    constexpr int CH = wino_chunk(HALF);
    const int c0 = chunk * CH;
    const int cfill = min(CH, cpad - c0);
    const int cvalid = max(0, min(CH, job.C - c0));
    const int ROW = lds_row_stride(CH * 9);
    stage_rows(job.src, lds, ROW, kb * 16, job.K, (size_t)job.C * 9, (size_t)c0 * 9, cvalid * 9, cfill * 9);
    if (!HALF) {
        float *dst = static_cast<float *>(job.dst);
        const int k_in = threadIdx.x & 15, csub = threadIdx.x >> 4;
#pragma unroll 1
        for (int j = 0; j < CH / 16; ++j) {
            const int cl = j * 16 + csub;
            if (cl >= cfill) break;
            float g[9];
#pragma unroll
            for (int i = 0; i < 9; ++i) g[i] = lds[k_in * ROW + cl * 9 + i];
            // U = G g G^T one row at a time, each row stored as soon as it exists: one live output
            // pointer and one row of values instead of alpha^2 of each keeps the registers low
            // (16-byte stores by threads that own four filters were measured too: slower)
            float *o = dst + ((size_t)kb * cpad + c0 + cl) * 16 + k_in;
            const size_t xi_stride = (size_t)K16 * cpad * 16;
#pragma unroll
            for (int a = 0; a < W::A; ++a) {
                float t[3];
#pragma unroll
                for (int s2 = 0; s2 < 3; ++s2) {
                    float acc = 0.f;
#pragma unroll
                    for (int r = 0; r < 3; ++r)
                        if (W::G[a][r] != 0.f) acc += W::G[a][r] * g[r * 3 + s2];
                    t[s2] = acc;
                }
#pragma unroll
                for (int b = 0; b < W::A; ++b) {
                    float acc = 0.f;
#pragma unroll
                    for (int s2 = 0; s2 < 3; ++s2)
                        if (W::G[b][s2] != 0.f) acc += t[s2] * W::G[b][s2];
                    nt_store(o, acc);
                    o += xi_stride;
                }
            }
        }
    } else {
        __half *dst = static_cast<__half *>(job.dst);
        const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
        const int oct = wave * 2 + (lane >> 5), hq = lane & 1, k_in = (lane >> 1) & 15;
        if (oct * 8 < cfill) {
            // four filters per thread (channels cl .. cl + 3 of its 8-channel lane pair), U row by row
            float g[4][9];
            const int cl = oct * 8 + hq * 4;
#pragma unroll
            for (int f = 0; f < 4; ++f)
#pragma unroll
                for (int i = 0; i < 9; ++i) g[f][i] = lds[k_in * ROW + (cl + f) * 9 + i];
            const int cabs = c0 + oct * 8;
            const int c32n = cpad / 32;
            __half *o = dst + ((size_t)kb * c32n + cabs / 32) * 512 + ((cabs % 32) / 8) * 128 + k_in * 8 + hq * 4;
            const size_t xi_stride = (size_t)K16 * c32n * 512;
#pragma unroll
            for (int a = 0; a < W::A; ++a) {
                float t[4][3];
#pragma unroll
                for (int f = 0; f < 4; ++f)
#pragma unroll
                    for (int s2 = 0; s2 < 3; ++s2) {
                        float acc = 0.f;
#pragma unroll
                        for (int r = 0; r < 3; ++r)
                            if (W::G[a][r] != 0.f) acc += W::G[a][r] * g[f][r * 3 + s2];
                        t[f][s2] = acc;
                    }
#pragma unroll
                for (int b = 0; b < W::A; ++b) {
                    float u[4];
#pragma unroll
                    for (int f = 0; f < 4; ++f) {
                        float acc = 0.f;
#pragma unroll
                        for (int s2 = 0; s2 < 3; ++s2)
                            if (W::G[b][s2] != 0.f) acc += t[f][s2] * W::G[b][s2];
                        u[f] = acc;
                    }
                    nt_store(reinterpret_cast<uint2v *>(o), uint2v{pack_half2(u[0], u[1]), pack_half2(u[2], u[3])});
                    o += xi_stride;
                }
            }
        }
    }
}

// GEMM panel pack of one block: 16 output channels x job.cchunk channels x RS taps.
template <bool HALF>
__device__ static inline void gemm_block(const TransformJob &job, int local_block, float *lds) {
    const int kb = local_block / job.nchunks, chunk = local_block % job.nchunks;
    const int RS = job.RS;
    const int cpad = HALF ? ((job.C + 31) / 32) * 32 : ((job.C + 3) / 4) * 4;
    const int c0 = chunk * job.cchunk;
    const int cfill = min(job.cchunk, cpad - c0);
    const int cvalid = max(0, min(job.cchunk, job.C - c0));
    const int ROW = lds_row_stride(min(job.cchunk, cpad) * RS);
    stage_rows(job.src, lds, ROW, kb * 16, job.K, (size_t)job.C * RS, (size_t)c0 * RS, cvalid * RS, cfill * RS);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int k_in = lane & 15, grp = lane >> 4;
    if (!HALF) {
        float *dst = static_cast<float *>(job.dst) + ((size_t)kb * (cpad / 4) + c0 / 4) * RS * 64;
        const int nfrag = (cfill / 4) * RS;
        int cb = 0, rs = wave;
        while (rs >= RS) { rs -= RS; ++cb; }
        for (int f = wave; f < nfrag; f += 4) {
            const float v = lds[k_in * ROW + (cb * 4 + grp) * RS + rs];
            nt_store(&dst[(size_t)f * 64 + lane], v);
            rs += 4;
            while (rs >= RS) { rs -= RS; ++cb; }
        }
    } else {
        __half *dst = static_cast<__half *>(job.dst) + ((size_t)kb * (cpad / 32) + c0 / 32) * RS * 512;
        const int nfrag = (cfill / 32) * RS;
        int cb = 0, rs = wave;
        while (rs >= RS) { rs -= RS; ++cb; }
        for (int f = wave; f < nfrag; f += 4) {
            const float *lp = lds + k_in * ROW + (cb * 32 + grp * 8) * RS + rs;
            uint4 v;
            v.x = pack_half2(lp[0], lp[RS]);
            v.y = pack_half2(lp[2 * RS], lp[3 * RS]);
            v.z = pack_half2(lp[4 * RS], lp[5 * RS]);
            v.w = pack_half2(lp[6 * RS], lp[7 * RS]);
            nt_store(reinterpret_cast<uint4v *>(dst + (size_t)f * 512 + lane * 8), uint4v{v.x, v.y, v.z, v.w});
            rs += 4;
            while (rs >= RS) { rs -= RS; ++cb; }
        }
    }
}

// Depthwise repack (C,1,R,S) -> [C/32][R*S taps][32 channels]; 256 outputs per block.
template <bool HALF>
__device__ static inline void dw_block(const TransformJob &job, int local_block) {
    const int per = job.RS * 32;
    const int total = ((job.C + 31) / 32) * per;
    const int o = local_block * 256 + threadIdx.x;
    if (o >= total) return;
    const int cb = o / per, rem = o - cb * per, tap = rem >> 5, ci = rem & 31;
    const int c = cb * 32 + ci;
    const float v = (c < job.C) ? job.src[(size_t)c * job.RS + tap] : 0.f;
    if (HALF) static_cast<__half *>(job.dst)[o] = __float2half_rn(v);
    else static_cast<float *>(job.dst)[o] = v;
}

// F6: the launch holds F(6x6) jobs.  Their 64 outputs per filter take more registers than
// any other job, so launches without them run an instantiation that leaves that branch out
// and keeps four wavefronts per SIMD.
// The table is read through the kernel-argument segment pointer (constant address space, scalar
// loads); a block's job is found by counting, the job's record is loaded in one batch.
typedef const __attribute__((address_space(4))) JobTable *JobTablePtr;

template <bool F6>
__global__ __launch_bounds__(256) void transform_kernel(const JobTable tbl_arg) {
    extern __shared__ __align__(16) float lds[];
    const JobTablePtr tbl = (JobTablePtr)__builtin_amdgcn_kernarg_segment_ptr();
    const int b = blockIdx.x;
    int first_unused;
    const int j = table_find<kMaxJobs>(&tbl->first_block[0], b, first_unused);
    TransformJob job;
    {
        static_assert(sizeof(TransformJob) % 4 == 0, "copied word by word");
        const __attribute__((address_space(4))) uint32_t *src = (const __attribute__((address_space(4))) uint32_t *)&tbl->job[j];
        uint32_t *dst = reinterpret_cast<uint32_t *>(&job);
#pragma unroll
        for (int k = 0; k < (int)(sizeof(TransformJob) / 4); ++k) dst[k] = src[k];
    }
    const int lb = b - job.block0;
    if (job.type == JOB_WINO) {
        if (job.wset == WS_F2) {
            if (job.half) wino_block<0, true>(job, lb, lds); else wino_block<0, false>(job, lb, lds);
        } else if (job.wset == WS_F4) {
            wino_block<1, false>(job, lb, lds);
        } else if (job.wset == WS_F6) {
            if constexpr (F6) wino_block<3, false>(job, lb, lds);
        } else {
            wino_block<2, true>(job, lb, lds);
        }
    } else if (job.type == JOB_GEMM) {
        if (job.half) gemm_block<true>(job, lb, lds); else gemm_block<false>(job, lb, lds);
    } else {
        if (job.half) dw_block<true>(job, lb); else dw_block<false>(job, lb);
    }
}

// ---------------------------------------------------------------- host side

int fill_transform_job(const Geo &g, int kind, const float *src, void *dst, TransformJob *job) {
    job->src = src;
    job->dst = dst;
    job->half = g.dtype == NNV_F16;
    job->K = g.k;
    job->C = g.cg;
    job->RS = g.r * g.s;
    job->wset = 0;
    job->block0 = 0;
    const int k16 = ceil_div(g.k, 16);
    if (is_wino(kind)) {
        job->type = JOB_WINO;
        job->wset = wino_set(kind, g.dtype);
        const int cpad = job->half ? ceil_div(g.cg, 32) * 32 : ceil_div(g.cg, 4) * 4;
        job->cchunk = wino_chunk(job->half);
        job->nchunks = ceil_div(cpad, job->cchunk);
        job->nblocks = k16 * job->nchunks;
    } else if (kind == NNV_IM2COL_GEMM) {
        job->type = JOB_GEMM;
        const int cpad = job->half ? ceil_div(g.cg, 32) * 32 : ceil_div(g.cg, 4) * 4;
        // about 18 KB of LDS per block (as many resident blocks as the Winograd jobs of the
        // same launch allow): about 288 floats per row, in whole fragments' worth of channels
        // (float32: 4, so that even an 11x11 filter stages only 31 KB; float16: 32, twice the row)
        const int unit = job->half ? 32 : 4;
        int cc = ((job->half ? 576 : 288) / job->RS) / unit * unit;
        if (cc < unit) cc = unit;
        if (cc > 32 && !job->half) cc = cc / 32 * 32;
        job->cchunk = cc;
        job->nchunks = ceil_div(cpad, cc);
        job->nblocks = k16 * job->nchunks;
    } else if (kind == NNV_DEPTHWISE) {
        job->type = JOB_DW;
        job->cchunk = 32;
        job->nchunks = 1;
        job->nblocks = ceil_div(ceil_div(g.c, 32) * g.r * g.s * 32, 256);
        job->C = g.c;
    } else {
        return -1;
    }
    return 0;
}

size_t transform_job_lds_bytes(const TransformJob &job) {
    if (job.type == JOB_WINO) return (size_t)kRows * lds_row_stride(wino_chunk(job.half) * 9) * sizeof(float);
    if (job.type == JOB_GEMM) {
        const int cpad = job.half ? ceil_div(job.C, 32) * 32 : ceil_div(job.C, 4) * 4;
        const int cc = job.cchunk < cpad ? job.cchunk : cpad;
        return (size_t)kRows * lds_row_stride(cc * job.RS) * sizeof(float);
    }
    return 0;
}

hipError_t launch_transform_jobs(const JobTable &table, int total_blocks, size_t lds, hipStream_t st) {
    if (total_blocks <= 0) return hipSuccess;
    JobTable tbl = table;
    for (int j = 0; j < kMaxJobs; ++j) tbl.first_block[j] = j < tbl.njobs ? tbl.job[j].block0 : INT_MAX;
    bool f6 = false;
    for (int j = 0; j < tbl.njobs; ++j) f6 = f6 || (tbl.job[j].type == JOB_WINO && tbl.job[j].wset == WS_F6);
    if (lds > 64 * 1024) {
        const void *fn = f6 ? reinterpret_cast<const void *>(transform_kernel<true>)
                            : reinterpret_cast<const void *>(transform_kernel<false>);
        hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    if (f6) hipLaunchKernelGGL(transform_kernel<true>, dim3(total_blocks), dim3(256), lds, st, tbl);
    else hipLaunchKernelGGL(transform_kernel<false>, dim3(total_blocks), dim3(256), lds, st, tbl);
    return hipGetLastError();
}

__global__ __launch_bounds__(256) void copy_f32_kernel(const float *__restrict__ src, float *__restrict__ dst, size_t n) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) dst[i] = src[i];
}

hipError_t launch_copy_f32(const float *src, float *dst, size_t n, hipStream_t st) {
    if (n == 0) return hipSuccess;
    size_t blocks = (n + 255) / 256;
    if (blocks > 8192) blocks = 8192;
    hipLaunchKernelGGL(copy_f32_kernel, dim3((unsigned)blocks), dim3(256), 0, st, src, dst, n);
    return hipGetLastError();
}

__global__ __launch_bounds__(256) void fill_u32_kernel(uint4 *__restrict__ dst, size_t n4, uint32_t v) {
    const uint4 val = make_uint4(v, v, v, v);
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += (size_t)gridDim.x * 256) dst[i] = val;
}

// Overwrite n 32-bit words (n rounded down to a multiple of 4): the cache flush of nnv_time_layer.
hipError_t launch_fill_u32(uint32_t *dst, size_t n, uint32_t v, hipStream_t st) {
    const size_t n4 = n / 4;
    if (n4 == 0) return hipSuccess;
    size_t blocks = (n4 + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(fill_u32_kernel, dim3((unsigned)blocks), dim3(256), 0, st, reinterpret_cast<uint4 *>(dst), n4, v);
    return hipGetLastError();
}

}  // namespace nnv
