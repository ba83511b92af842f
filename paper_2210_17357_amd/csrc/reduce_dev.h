// Per-layer sum of the quantization profile's tile partials, shared by the stand-alone reduction
// kernel and the Top-K scan kernel (which takes the reduction along as extra workgroups when both
// families are profiled in one call).
#pragma once

#include "common.h"

namespace lgreco {

struct ReduceCols {
    int32_t n;
    int32_t col[kMaxQuant];
};

// errors[l][c] = sum of the layer's tile partials in tile order (fixed tree -> reproducible); one
// 256-thread workgroup per layer; all columns together: per thread the same strided sums, then the
// same tree per column.
__device__ __forceinline__ void reduce_partials_block(const double* __restrict__ partials, int stride,
                                                      const ReduceCols& cols, const DevLayer* __restrict__ layers,
                                                      double* __restrict__ errors, int layer,
                                                      double (*s)[256]) {
    const DevLayer L = layers[layer];
    double a[kMaxQuant];
#pragma unroll
    for (int ci = 0; ci < kMaxQuant; ++ci) a[ci] = 0.0;
    for (int t = L.tile_begin + threadIdx.x; t < L.tile_end; t += 256) {
#pragma unroll
        for (int ci = 0; ci < kMaxQuant; ++ci)
            if (ci < cols.n) a[ci] += partials[(size_t)t * stride + cols.col[ci]];
    }
#pragma unroll
    for (int ci = 0; ci < kMaxQuant; ++ci) s[ci][threadIdx.x] = a[ci];
    __syncthreads();
    for (int o = 128; o > 0; o >>= 1) {
        if ((int)threadIdx.x < o) {
#pragma unroll
            for (int ci = 0; ci < kMaxQuant; ++ci)
                if (ci < cols.n) s[ci][threadIdx.x] += s[ci][threadIdx.x + o];
        }
        __syncthreads();
    }
    if ((int)threadIdx.x < cols.n) errors[(size_t)layer * stride + cols.col[threadIdx.x]] = s[threadIdx.x][0];
}

}  // namespace lgreco
