/* nnv.h -- C ABI of the conv hot path behind NNV12-style cold inference on MI355X.
 *
 * The paper splits every operator of a cold inference into operations: reading
 * the weights, transforming them into the layout a kernel wants (w_i) and
 * executing the kernel (e_i); its scheduler chooses, per conv layer, which
 * kernel alternative to use from the measured cost of those operations
 * (Section 3.1.1 kernel selection, Table 2, Section 3.2, Algorithm 1's
 * profiling input).  This library is the w_i and e_i of a convolution for six
 * kernel alternatives, the per-operation timing the selection needs, and the
 * on-disk cache of transformed weights that lets a cold start skip w_i
 * (Section 3.1.2).
 *
 * All data pointers are DEVICE pointers unless a parameter says "host".  The
 * caller owns every buffer; the library allocates no device memory and keeps
 * no mutable global state (one exception, stated there: the pinned staging
 * buffer of nnv_cache_read).  Device buffers must be 16-byte aligned.  Work is
 * enqueued on the given HIP stream (a hipStream_t passed as void*, NULL = the
 * default stream) and the call returns without waiting, except nnv_time_layer.
 * Every function returns NNV_OK (0) or a negative nnv_status; none aborts or
 * throws.
 *
 * Tensors at the boundary: x is NCHW, y is NKPQ, raw weights are OIHW
 * (K, C/groups, R, S) and ALWAYS float32.  desc.dtype is the storage type of x,
 * y and the transformed weights; accumulation is float32 in both cases.
 * Convolution means zero-padded cross-correlation, dilation 1,
 * P = floor((H + 2*pad_h - R)/stride_h) + 1.
 */
#ifndef NNV_H
#define NNV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Kernel alternatives of the conv operator (Section 3.1.1, Fig. 5, Table 2 name
 * winograd, sgemm, direct and depthwise families). */
typedef enum {
    NNV_DIRECT = 0,      /* direct convolution from raw OIHW weights, no transformation       */
    NNV_IM2COL_GEMM = 1, /* implicit im2col GEMM from matrix-instruction-ordered weight panels */
    NNV_WINO_F2 = 2,     /* Winograd F(2x2,3x3): 4x4 tiles                                     */
    NNV_WINO_F4 = 3,     /* Winograd F(4x4,3x3): 6x6 tiles                                     */
    NNV_DEPTHWISE = 4,   /* 3x3 or 5x5 depthwise (groups = C = K) from channel-blocked tap-major weights */
    NNV_WINO_F6 = 5,     /* Winograd F(6x6,3x3): 8x8 tiles, the tile size of Fig. 3; float32 only */
    NNV_KIND_COUNT = 6
} nnv_kind;

typedef enum { NNV_F32 = 0, NNV_F16 = 1 } nnv_dtype;

typedef enum {
    NNV_OK = 0,
    NNV_E_NULL = -1,        /* a required pointer is NULL                                  */
    NNV_E_BAD_DESC = -2,    /* non-positive size, empty output, groups not dividing C or K */
    NNV_E_UNSUPPORTED = -3, /* this kind cannot run this layer (see nnv_kind_supported)     */
    NNV_E_WORKSPACE = -4,   /* workspace smaller than nnv_workspace_bytes                   */
    NNV_E_ALIGN = -5,       /* a device pointer is not 16-byte aligned                      */
    NNV_E_HIP = -6,         /* a HIP call failed; text via nnv_last_hip_error               */
    NNV_E_ARG = -7,         /* bad count / reps / enum value                                */
    NNV_E_IO = -8,          /* a cache file could not be opened, read or written (errno set) */
    NNV_E_CACHE = -9        /* a cache file does not hold what was asked for                 */
} nnv_status;

typedef struct {
    int32_t n, c, h, w;          /* input  N x C x H x W               */
    int32_t k;                   /* output channels                    */
    int32_t r, s;                /* filter height, width               */
    int32_t stride_h, stride_w;
    int32_t pad_h, pad_w;
    int32_t groups;              /* 1, or any divisor of C and K       */
    int32_t dtype;               /* nnv_dtype of x, y, transformed w   */
} nnv_conv_desc;

/* Result of nnv_time_layer: GPU time of the two operations of one (layer, kind)
 * and the algorithmic traffic/work they stand for. */
typedef struct {
    double transform_ms;       /* median GPU time of the weight transformation           */
    double forward_ms;         /* median GPU time of the convolution                      */
    double transform_bytes;    /* raw weights read + transformed weights written          */
    double forward_bytes;      /* x + transformed weights + y (workspace traffic excluded) */
    double forward_flops;      /* flops executed (Winograd: 2*alpha^2*K*C*tiles)           */
    double direct_equiv_flops; /* 2 * multiply-accumulates of the plain convolution        */
} nnv_timing;

/* Version of the transformed-weight layouts and of the Winograd matrix sets.
 * Version 1: 16-row fragments (float32: 16x4, float16: 16x32); Winograd points
 * {0,1,-1} (F2), {0,+-1,+-2} (F4 float32), {0,1,-1,2,-1/2} with G rows scaled by
 * (4,4,4,16,4,1) (F4 float16), {0,+-1,+-2,+-1/2} (F6 float32).  Cache files carry
 * this number and are refused under any other. */
int nnv_layout_version(void);

/* Static text for a status code (never NULL). */
const char *nnv_status_string(int status);

/* Text of the last HIP error seen by the calling thread ("" if none). */
const char *nnv_last_hip_error(void);

/* 1 if `kind` can run the layer, 0 if not, NNV_E_* if the descriptor is invalid.
 *   WINO_F2/F4   : R = S = 3, stride 1, groups 1; with dtype float16 also C >= 16 (with a
 *                  handful of channels the roundings of U and V to float16 put the error
 *                  above the float16 bound of this library, 5e-3 * max|y|: refused)
 *   WINO_F6      : the same, and dtype float32 (with U and V rounded to float16 its error
 *                  exceeds the float16 bound of this library, so that pairing is refused)
 *   DEPTHWISE    : groups = C = K, R = S in {3,5}, stride_h = stride_w in {1,2}
 *   IM2COL_GEMM  : R,S <= 32, R*S <= 128 (float16: <= 64); groups 1, or up to 64 groups
 *                  (float16 with a filter larger than 1x1: C/groups a multiple of 32)
 *   DIRECT       : any groups dividing C and K
 * (the paper's engine keys the usable kernels on filter size, stride and channel
 * divisibility in the same way, Fig. 5). */
int nnv_kind_supported(const nnv_conv_desc *desc, nnv_kind kind);

/* Bytes of the transformed-weight buffer of `kind` (0 if unsupported/invalid).
 * This is the size a post-transformed-weights cache would store and read back
 * (Section 3.1.2): alpha^2/9 of the raw size for Winograd up to padding. */
size_t nnv_transformed_bytes(const nnv_conv_desc *desc, nnv_kind kind);

/* Bytes of scratch nnv_conv_forward needs for `kind` (may be 0: DIRECT, DEPTHWISE, float32
 * IM2COL_GEMM, and float32 WINO_F2/F4 on layers that run as one fused kernel; the other
 * Winograd layers keep their transformed input V and the tile products M there). */
size_t nnv_workspace_bytes(const nnv_conv_desc *desc, nnv_kind kind);

/* Weight transformation w_i (Section 2 "weights transformation", Fig. 3, Table 2
 * column "Weights Trans."): raw OIHW float32 -> the layout `kind` executes from.
 *   w_raw : device, K*(C/groups)*R*S float32, read only
 *   w_tx  : device, nnv_transformed_bytes(desc, kind) bytes, fully overwritten
 *           (padding included).  For NNV_DIRECT the layout is the raw one: if
 *           w_tx == w_raw nothing is done, else the weights are copied.
 * Errors: NULL, BAD_DESC, UNSUPPORTED, ALIGN, HIP. */
int nnv_transform_weights(const nnv_conv_desc *desc, nnv_kind kind, const float *w_raw,
                          void *w_tx, void *hip_stream);

/* The same for n_layers layers in as few launches as possible (a whole model's
 * weights at cold start, Table 1 "weights transformation").  descs, kinds,
 * w_raw and w_tx are HOST arrays of length n_layers holding descriptors, kinds
 * and device pointers.  Layers are independent; outputs must not overlap. */
int nnv_transform_weights_grouped(int n_layers, const nnv_conv_desc *descs, const nnv_kind *kinds,
                                  const float *const *w_raw, void *const *w_tx, void *hip_stream);

/* Kernel execution e_i (Table 2 column "Execution") from transformed weights.
 *   x    : device, N*C*H*W elements of desc.dtype, read only
 *   w_tx : device, output of nnv_transform_weights for the same desc and kind
 *   bias : device, K float32, or NULL
 *   y    : device, N*K*P*Q elements of desc.dtype, fully overwritten
 *   workspace : device, >= nnv_workspace_bytes(desc, kind) bytes (may be NULL if 0)
 * Errors: NULL, BAD_DESC, UNSUPPORTED, WORKSPACE, ALIGN, HIP. */
int nnv_conv_forward(const nnv_conv_desc *desc, nnv_kind kind, const void *x, const void *w_tx,
                     const float *bias, void *y, void *workspace, size_t workspace_bytes,
                     void *hip_stream);

/* The same with the activation that follows almost every convolution of the paper's
 * networks fused into the store: y = max(conv + bias, 0), clamped in float32 before the
 * one rounding to desc.dtype.  Same arguments and errors as nnv_conv_forward. */
int nnv_conv_forward_relu(const nnv_conv_desc *desc, nnv_kind kind, const void *x, const void *w_tx,
                          const float *bias, void *y, void *workspace, size_t workspace_bytes,
                          void *hip_stream);

/* Kernel execution of n_layers INDEPENDENT layers (none reads what another writes) in as
 * few launches as possible.  The decision stage profiles every kernel candidate of every
 * layer (Algorithm 1's input, Section 3.3, Table 2), and a batch-1 layer alone neither fills
 * the GPU nor outlasts its own launch: IM2COL_GEMM layers of one storage type share one
 * launch of single-wavefront work items (output tile x range of the reduction) and one
 * reduction launch (float16 layers with filters larger than 1x1: one more, which makes the
 * channels-last copies of all their inputs); Winograd layers of one kind and storage type share three launches (all
 * input transforms, all tile GEMMs, all output transforms), except those nnv_conv_forward
 * runs as one fused kernel; DEPTHWISE layers of one storage type share one launch; DIRECT
 * layers with groups = 1 and a square 1x1, 3x3, 5x5 or 7x7 filter share up to three (one of
 * them for the layers that run with the lanes along the output channels: K a multiple of 64 and
 * a 3x3 filter with C a multiple of 4, a 1x1 filter with C a multiple of 16, each at stride 1 or
 * 2, or a 7x7 stride-2 filter with at most 4 channels); DIRECT layers of depthwise shape
 * (as the DEPTHWISE kind accepts) share one launch of the depthwise kernel, which reads the
 * untransformed filters.  The
 * remaining layers, and the layers of a kind of which the call holds only one or two (three
 * for IM2COL_GEMM: the shared launches are laid out to fill the GPU), are executed one after
 * the other as by nnv_conv_forward.  Results per layer are as nnv_conv_forward's up to the
 * order of the float32 summation over the channels (deterministic: fixed order).
 *   descs, kinds, x, w_tx, y : HOST arrays of length n_layers (descriptors, kinds, device
 *       pointers as for nnv_conv_forward); outputs must not overlap
 *   bias  : NULL, or a HOST array of n_layers device pointers (entries may be NULL)
 *   workspace : device, >= nnv_conv_forward_grouped_workspace_bytes(...) bytes
 *   flags : 0, or NNV_FORWARD_RELU for y = max(conv + bias, 0) on every layer
 * Errors: NULL, BAD_DESC, ARG, UNSUPPORTED, WORKSPACE, ALIGN, HIP; nothing is launched unless
 * every layer passes the checks. */
#define NNV_FORWARD_RELU 1u
size_t nnv_conv_forward_grouped_workspace_bytes(int n_layers, const nnv_conv_desc *descs, const nnv_kind *kinds);
int nnv_conv_forward_grouped(int n_layers, const nnv_conv_desc *descs, const nnv_kind *kinds,
                             const void *const *x, const void *const *w_tx, const float *const *bias,
                             void *const *y, void *workspace, size_t workspace_bytes, unsigned flags,
                             void *hip_stream);

/* nnv_conv_forward for callers that cannot allocate or pass device scratch (code under HIP
 * graph capture, tight serving loops, harnesses that forbid allocation): the workspace is
 * a static device array of NNV_STATIC_SCRATCH_BYTES that is part of the library's code
 * object (each GPU the library runs on holds its own copy until the process ends).  The
 * call allocates nothing.  The first call on a device looks the array's address up once
 * (make that call before starting a capture).  A layer whose nnv_workspace_bytes exceeds
 * NNV_STATIC_SCRATCH_BYTES is refused with NNV_E_WORKSPACE.  Every call on one GPU uses the
 * same array: nothing in it has to start at zero (each kernel overwrites what the next one
 * reads), but two calls that overlap in time on one GPU (different streams) race -- keep
 * them on one stream or order them with events.  Other arguments, results and errors as
 * nnv_conv_forward. */
#define NNV_STATIC_SCRATCH_BYTES ((size_t)64 << 20)
int nnv_conv_forward_static(const nnv_conv_desc *desc, nnv_kind kind, const void *x, const void *w_tx,
                            const float *bias, void *y, void *hip_stream);

/* Per-operation profiling (the latency table Algorithm 1 consumes; Section 3.3
 * re-profiles operations while planning).  Runs `warmup` untimed and `reps`
 * timed repetitions of the transformation and, separately, of the forward pass,
 * each bracketed by HIP events on `hip_stream`, and reports the medians.  If
 * flush is non-NULL, flush_bytes of it are overwritten before every timed
 * repetition so that weights and activations are not cache-resident ("cold")
 * and a repetition is one launch; without a flush buffer a repetition is a
 * queue of 8 back-to-back launches between one pair of events and its time
 * is their mean (a batch-1 layer runs for less than a pair of events costs).
 * Synchronises the stream.  `out` is a HOST pointer. */
int nnv_time_layer(const nnv_conv_desc *desc, nnv_kind kind, const float *w_raw, void *w_tx,
                   const void *x, void *y, void *workspace, size_t workspace_bytes,
                   void *flush, size_t flush_bytes, int warmup, int reps, void *hip_stream,
                   nnv_timing *out);

/* Cold pass over a list of layers with the two operations pipelined (Section 3.1.3:
 * the transformation of later layers overlaps the execution of earlier ones, layer
 * by layer).  The layers are cut into stages of `stage_layers` consecutive layers
 * (<= 0: one stage holding all).  Each stage's weights are transformed in one grouped
 * launch on stream_tx; each layer's convolution runs on stream_exec once its stage
 * is transformed.  With stream_tx == stream_exec the same launches are issued in
 * the same order on one stream: the unpipelined baseline.
 *   descs, kinds, w_raw, w_tx, x, y : HOST arrays of length n_layers (descriptors,
 *       kinds, device pointers); bias is not applied
 *   workspace : device, >= the largest nnv_workspace_bytes of the list, shared by
 *       all layers (their convolutions are serialised on stream_exec)
 * stream_tx first waits for the work already queued on stream_exec, and stream_exec
 * ends up waiting for everything issued on stream_tx, so the call may be captured
 * into a HIP graph from stream_exec; work the caller queues on either stream
 * afterwards is ordered after the whole pass.  Returns without waiting.
 * Errors: NULL, BAD_DESC, ARG, UNSUPPORTED, WORKSPACE, ALIGN, HIP. */
int nnv_cold_stack(int n_layers, const nnv_conv_desc *descs, const nnv_kind *kinds, const float *const *w_raw,
                   void *const *w_tx, const void *const *x, void *const *y, void *workspace,
                   size_t workspace_bytes, int stage_layers, void *stream_exec, void *stream_tx);

/* ---- cache of post-transformation weights on disk (Section 3.1.2, Table 2
 * columns "Read Raw" / "Read Cache"): the decision stage writes the transformed
 * weights of the kinds it picked, the cold start reads them back instead of
 * transforming.  A file of kind NNV_DIRECT holds the raw weights, so reading it
 * and transforming is the "Read Raw + Weights Trans." alternative.
 *
 * File: a 4096-byte header block (magic "NNVCACHE", format version, layout
 * version, kind, dtype, K, C, R, S, groups, payload bytes, payload checksum)
 * followed by the nnv_transformed_bytes(desc, kind) bytes of w_tx exactly as
 * they lie in device memory. */

/* What nnv_cache_read measured. */
typedef struct {
    double total_ms;   /* wall clock, open to last byte in device memory            */
    double file_ms;    /* of that, time inside the file reads                        */
    double bytes;      /* payload bytes                                              */
    int32_t direct_io; /* 1: read with O_DIRECT, bypassing the page cache; 0: the file
                        * system or the kernel refused that (no O_DIRECT, or no direct
                        * I/O into pinned memory), the file's cached pages were dropped
                        * with posix_fadvise first and buffered reads were used       */
} nnv_cache_io;

/* Copy w_tx (device) to host and write it to `path` (host string), replacing the
 * file.  Synchronises hip_stream first.  Errors: NULL, BAD_DESC, ARG,
 * UNSUPPORTED, HIP, IO. */
int nnv_cache_write(const char *path, const nnv_conv_desc *desc, nnv_kind kind, const void *w_tx,
                    void *hip_stream);

/* Read the file into w_tx (device, nnv_transformed_bytes bytes).  The header
 * must match desc's K, C, R, S, groups and dtype, `kind` and
 * nnv_layout_version(), else NNV_E_CACHE and w_tx is untouched; with verify != 0
 * the payload checksum is checked as well (NNV_E_CACHE after the copy if it
 * differs).  The file is read in 8 MiB pieces into two pinned host buffers and
 * copied to the device on hip_stream while the next piece is read; the call
 * returns after the last copy has finished.  The pinned buffers (16 MiB) are
 * allocated on the first call and kept until the process ends; calls are
 * serialised by a lock.  `io` (host, may be NULL) receives the timing.
 * Errors: NULL, BAD_DESC, ARG, UNSUPPORTED, ALIGN, HIP, IO, CACHE. */
int nnv_cache_read(const char *path, const nnv_conv_desc *desc, nnv_kind kind, void *w_tx, int verify,
                   void *hip_stream, nnv_cache_io *io);

#ifdef __cplusplus
}
#endif
#endif /* NNV_H */
