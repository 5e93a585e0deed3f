// A workgroup-wide exclusive prefix sum for 256-thread workgroups (device code only).
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace gp {

constexpr int kScanThreads = 256;
constexpr int kScanWaves = kScanThreads / 64;

// exclusive prefix of v over the workgroup's threads, in thread order; *total = the sum.  Every thread of the
// workgroup must call it (two barriers inside); wave_sums: kScanWaves + 1 words of LDS.
__device__ inline uint32_t block_exclusive(uint32_t v, uint32_t* wave_sums, uint32_t* total)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t incl = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t up = __shfl_up(incl, o, 64);
        if (lane >= o) incl += up;
    }
    __syncthreads();  // (wave_sums may still be read from the call before)
    if (lane == 63) wave_sums[wave] = incl;
    __syncthreads();
    uint32_t before = 0, all = 0;
#pragma unroll
    for (int w = 0; w < kScanWaves; ++w) {
        if (w < wave) before += wave_sums[w];
        all += wave_sums[w];
    }
    *total = all;
    return before + incl - v;
}

}  // namespace gp
