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

}  // namespace nnv
