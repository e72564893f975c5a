// Internal declarations shared by the host dispatch and the HIP kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>
#include <stddef.h>
#include "nnv.h"

namespace nnv {

// Validated geometry of one conv layer (host side).
struct Geo {
    int n, c, h, w, k, r, s, sh, sw, ph, pw, groups, dtype;
    int p, q;      // output height / width
    int cg, kg;    // channels per group (input / output)
    int relu;      // clamp the outputs at zero before the store (not part of the descriptor)
};

static inline int ceil_div(int a, int b) { return (a + b - 1) / b; }
static inline bool is_wino(int kind) { return kind == NNV_WINO_F2 || kind == NNV_WINO_F4 || kind == NNV_WINO_F6; }
static inline int wino_m(int kind) { return kind == NNV_WINO_F2 ? 2 : kind == NNV_WINO_F4 ? 4 : 6; }
static inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Fewest input channels for which Winograd runs with float16 storage (see nnv_kind_supported).
constexpr int kWinoHalfMinChannels = 16;

// Winograd matrix sets (see wino_consts.h)
enum WinoSet { WS_F2 = 0, WS_F4 = 1, WS_F4H = 2, WS_F6 = 3 };
static inline int wino_set(int kind, int dtype) {
    if (kind == NNV_WINO_F2) return WS_F2;
    if (kind == NNV_WINO_F6) return WS_F6;
    return dtype == NNV_F16 ? WS_F4H : WS_F4;
}

// One weight-transformation job of a grouped launch.
enum JobType { JOB_WINO = 0, JOB_GEMM = 1, JOB_DW = 2 };
struct TransformJob {
    const float *src;
    void *dst;
    int type;        // JobType
    int wset;        // WinoSet (JOB_WINO)
    int half;        // output float16
    int K, C, RS;    // rows, channels per row, taps
    int cchunk;      // channels handled by one block
    int nchunks;     // blocks per 16-row group
    int block0;      // first block of this job in the launch
    int nblocks;
};
constexpr int kMaxJobs = 64;   // 64 jobs of 56 bytes + 64 block offsets: the table still fits the 4 KB of kernel arguments
struct JobTable {
    TransformJob job[kMaxJobs];
    int first_block[kMaxJobs];   // job[j].block0 again, INT_MAX beyond the last job: a block finds its job by
                                 // counting the entries it has reached (no chain of dependent loads)
    int njobs;
};
static_assert(sizeof(JobTable) <= 4096, "the job table is passed by value as the kernel argument");

// Records the text of a failed HIP call for nnv_last_hip_error and returns NNV_E_HIP.
int record_hip_error(hipError_t e);

int fill_transform_job(const Geo &g, int kind, const float *src, void *dst, TransformJob *job);
size_t transform_job_lds_bytes(const TransformJob &job);
hipError_t launch_transform_jobs(const JobTable &tbl, int total_blocks, size_t lds, hipStream_t st);
hipError_t launch_copy_f32(const float *src, float *dst, size_t n, hipStream_t st);
hipError_t launch_fill_u32(uint32_t *dst, size_t n, uint32_t v, hipStream_t st);

hipError_t launch_direct(const Geo &g, const void *x, const float *w, const float *bias, void *y, hipStream_t st);
hipError_t launch_depthwise(const Geo &g, const void *x, const void *w, const float *bias, void *y, hipStream_t st);

// Many layers in one launch: direct convolution (layers for which direct_many_supported holds) and
// depthwise convolution; one storage type per call.
constexpr int kMaxDirectLayers = 32;
constexpr int kMaxDwLayers = 40;
bool direct_many_supported(const Geo &g);
hipError_t launch_direct_many(int n, const Geo *geos, const void *const *x, const void *const *w, const float *const *bias,
                              void *const *y, hipStream_t st);
// raw: w[i] are the untransformed float32 filters (depthwise layers run by the direct kind), else the
// channel-blocked tap-major ones of the depthwise kind.
hipError_t launch_depthwise_many(int n, const Geo *geos, const void *const *x, const void *const *w,
                                 const float *const *bias, void *const *y, bool raw, hipStream_t st);

size_t im2col_workspace_bytes(const Geo &g);
hipError_t launch_im2col(const Geo &g, const void *x, const void *w, const float *bias, void *y, void *ws, hipStream_t st);

// Many independent IM2COL_GEMM layers (one storage type, at most kMaxGemmLayers) in one launch of
// single-wavefront work items, plus one reduction launch if a layer's channels are split; ws[i] is
// layer i's own region of im2col_items_workspace_bytes(geos[i], im2col_items_target(n, geos)) bytes.
constexpr int kMaxGemmLayers = 20;
int im2col_items_target(int n, const Geo *geos);             // item length (k-steps) a launch of these layers uses
size_t im2col_items_workspace_bytes(const Geo &g, int target);
hipError_t launch_im2col_items(int n, const Geo *geos, const void *const *x, const void *const *w,
                               const float *const *bias, void *const *y, void *const *ws, hipStream_t st);

size_t wino_workspace_bytes(const Geo &g, int kind);
// Many layers of one Winograd kind and storage type in three launches (see winograd.hip).
constexpr int kMaxWinoLayers = 20;
bool wino_many_supported(const Geo &g, int kind);
hipError_t launch_wino_many(int n, const Geo *geos, int kind, const void *const *x, const void *const *U,
                            const float *const *bias, void *const *y, void *const *ws, hipStream_t st);
hipError_t launch_wino(const Geo &g, int kind, const void *x, const void *w, const float *bias, void *y, void *ws, hipStream_t st);

}  // namespace nnv
