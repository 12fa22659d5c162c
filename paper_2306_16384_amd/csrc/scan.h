// Wave and workgroup prefix sums shared by the kernels that compact or scatter
// variable-length output (ID dedup, neighbour sampling).  Workgroups of 256.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace gids {

constexpr int SCAN_THREADS = 256;

__device__ __forceinline__ uint32_t lane_id() { return threadIdx.x & 63; }

__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t x) {
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        uint32_t y = __shfl_up(x, d);
        if (lane_id() >= (uint32_t)d) x += y;
    }
    return x;
}

// exclusive prefix of x over the 256 threads of the block; *total = block sum
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t x, uint32_t* total, uint32_t* smem /* >= 5 */) {
    const uint32_t incl = wave_inclusive_scan(x);
    const uint32_t wave = threadIdx.x >> 6;
    __syncthreads();                      // smem may still be read from a previous call
    if (lane_id() == 63) smem[wave] = incl;
    __syncthreads();
    uint32_t base = 0, sum = 0;
#pragma unroll
    for (int w = 0; w < SCAN_THREADS / 64; w++) {
        const uint32_t s = smem[w];
        if ((uint32_t)w < wave) base += s;
        sum += s;
    }
    *total = sum;
    return base + incl - x;
}

}  // namespace gids
