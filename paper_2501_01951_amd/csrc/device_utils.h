// Small device-side helpers: wave/block prefix sums for 256-thread blocks of 64-wide waves.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mixgcn {

constexpr int kBlock = 256;  // threads per block used by the integer kernels
constexpr int kWave = 64;

__device__ inline uint64_t wave_inclusive_scan_u64(uint64_t v)
{
    const int lane = threadIdx.x & (kWave - 1);
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) {
        unsigned long long t = __shfl_up((unsigned long long)v, o, kWave);
        if (lane >= o) v += t;
    }
    return v;
}

// Exclusive prefix sum over the 256 threads of a block; *total receives the block sum.
// lds must hold 4 uint64.  Contains two __syncthreads().
__device__ inline uint64_t block_exclusive_scan_u64(uint64_t v, uint64_t* total, uint64_t* lds)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int w = threadIdx.x >> 6;
    const uint64_t inc = wave_inclusive_scan_u64(v);
    if (lane == kWave - 1) lds[w] = inc;
    __syncthreads();
    uint64_t woff = 0, tot = 0;
#pragma unroll
    for (int i = 0; i < kBlock / kWave; ++i) {
        const uint64_t x = lds[i];
        if (i < w) woff += x;
        tot += x;
    }
    __syncthreads();
    *total = tot;
    return woff + inc - v;
}

}  // namespace mixgcn
