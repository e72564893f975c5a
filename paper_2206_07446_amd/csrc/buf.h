// Buffer-resource loads: the hardware range check turns an out-of-range offset into a
// zero result, so masked lanes (zero padding of the convolution, tails of a tile) need no
// branch: they get an offset beyond the buffer.  All loads of a pipeline stage then sit in
// straight-line code and can be kept in flight across the matrix instructions.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

namespace nnv {

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));

constexpr uint32_t kOobOffset = 0x80000000u;   // beyond any buffer (sizes are kept below 2 GiB); adding an
                                               // immediate offset to it cannot wrap around

__device__ static inline __amdgpu_buffer_rsrc_t make_rsrc(const void *p, uint32_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p), 0, bytes, 0x00020000);
}

template <typename F> __device__ static inline F buf_load(__amdgpu_buffer_rsrc_t r, uint32_t voff, uint32_t soff);
template <> __device__ inline float buf_load<float>(__amdgpu_buffer_rsrc_t r, uint32_t voff, uint32_t soff) {
    return __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(r, voff, soff, 0));
}
template <> __device__ inline half8_t buf_load<half8_t>(__amdgpu_buffer_rsrc_t r, uint32_t voff, uint32_t soff) {
    return __builtin_bit_cast(half8_t, __builtin_amdgcn_raw_buffer_load_b128(r, voff, soff, 0));
}

// One activation element (float32 or float16 storage) as float.
template <typename T> __device__ static inline float buf_load_x(__amdgpu_buffer_rsrc_t r, uint32_t voff, uint32_t soff);
template <> __device__ inline float buf_load_x<float>(__amdgpu_buffer_rsrc_t r, uint32_t voff, uint32_t soff) {
    return __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(r, voff, soff, 0));
}
template <> __device__ inline float buf_load_x<__half>(__amdgpu_buffer_rsrc_t r, uint32_t voff, uint32_t soff) {
    const unsigned short u = __builtin_amdgcn_raw_buffer_load_b16(r, voff, soff, 0);
    return (float)__builtin_bit_cast(_Float16, u);
}

// XCD-aware workgroup order.  The chip has 8 XCDs with one L2 each and hands consecutive
// workgroups of a launch to the XCDs round-robin, so workgroup i runs on XCD i % 8.  A 1-D grid
// of `total` logical tiles (rounded up to a multiple of 8 workgroups) is remapped so that XCD x
// works on the contiguous logical range [x * per, (x + 1) * per): tiles that share an operand
// panel then share an L2 instead of fetching the panel once per XCD.  Returns -1 for the padding.
__device__ static inline int xcd_logical_tile(int total) {
    const int per = (total + 7) >> 3;
    const int i = blockIdx.x;
    const int l = (i & 7) * per + (i >> 3);
    return l < total ? l : -1;
}
static inline unsigned xcd_grid(int total) { return (unsigned)(((total + 7) / 8) * 8); }

// Many-layer launches: a workgroup (or wavefront) finds its layer in an ascending table of first
// block numbers that lies in the kernel-argument segment (at most 64 entries, INT_MAX beyond the used
// ones, entry 0 is 0).  Lane l looks at entry l; the entries that b has reached are a prefix of the
// lanes, so one vector load and a ballot give the index.  (A chain of scalar comparisons over the
// table, the first version, took a wavefront 2 us on a busy chip: half the life of a depthwise
// wavefront.)  b must be uniform over the wavefront.  Returns the index; first = that entry.
template <int N>
__device__ static inline int table_find(const __attribute__((address_space(4))) int *table, const int b, int &first) {
    static_assert(N <= 64, "one table entry per lane");
    const int lane = threadIdx.x & 63;
    const int *t = reinterpret_cast<const int *>(reinterpret_cast<uintptr_t>(table));
    const int mine = lane < N ? t[lane] : 0x7fffffff;
    const int li = __builtin_popcountll(__ballot(b >= mine)) - 1;
    first = __builtin_amdgcn_readlane(mine, li);
    return li;
}

}  // namespace nnv
