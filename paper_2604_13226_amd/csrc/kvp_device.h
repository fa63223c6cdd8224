// kvp_device.h -- small device helpers shared by this library's kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kvp_plan.h"

namespace kvp {

typedef uint16_t bf16_t;  // raw bfloat16 bits

__device__ __forceinline__ float bf16_to_f32(bf16_t h) { return __uint_as_float((uint32_t)h << 16); }

// round to nearest even; inputs finite by contract
__device__ __forceinline__ bf16_t f32_to_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}

__device__ __forceinline__ float ld_elem(const float *p) { return *p; }
__device__ __forceinline__ float ld_elem(const bf16_t *p) { return bf16_to_f32(*p); }
__device__ __forceinline__ void st_elem(float *p, float x) { *p = x; }
__device__ __forceinline__ void st_elem(bf16_t *p, float x) { *p = f32_to_bf16(x); }

// Element offset of cache row `row` of (request, layer, kv head).
__device__ __forceinline__ int64_t cache_row_off(const CacheView &c, int req, int layer, int head,
                                                 int row, int n_kv, int d)
{
    if (c.layout == 0) {
        return (int64_t)req * c.req_stride + (int64_t)layer * c.layer_stride +
               ((int64_t)head * c.t_cap + row) * d;
    }
    int blk = c.block_table[(int64_t)req * c.max_blocks + (row >> c.block_shift)];
    int slot = row & ((1 << c.block_shift) - 1);
    return (int64_t)layer * c.layer_stride +
           ((((int64_t)blk * n_kv + head) << c.block_shift) + slot) * d;
}

}  // namespace kvp
