// Device helpers for order-preserving compaction with 64-lane wavefronts.
//
// A list is compacted in two launches with no waiting between workgroups: the first launch leaves one
// count per workgroup, the second lets every workgroup add up the counts of the workgroups before it
// (a few KB from L2) and then ranks its own elements with wavefront ballots.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

constexpr int FG_WAVE = 64;

__device__ __forceinline__ int fg_lane() { return threadIdx.x & (FG_WAVE - 1); }
__device__ __forceinline__ int fg_wave() { return threadIdx.x >> 6; }

// Number of lanes below this one for which `flag` holds; `total` = lanes of the wave for which it holds.
__device__ __forceinline__ int fg_wave_rank(bool flag, int& total) {
    const unsigned long long m = __ballot(flag);
    total = __popcll(m);
    return __popcll(m & ((1ull << fg_lane()) - 1ull));
}

// Exclusive rank of `flag` within a workgroup of up to 1024 threads (blockDim.x a multiple of 64) and the
// workgroup total. `lds` needs 17 ints and may be reused after the call returns.
__device__ __forceinline__ int fg_block_rank(bool flag, int& block_total, int* lds) {
    int wave_total;
    const int r = fg_wave_rank(flag, wave_total);
    const int nw = blockDim.x >> 6;
    __syncthreads();  // protects a previous use of lds
    if (fg_lane() == 0) lds[fg_wave()] = wave_total;
    __syncthreads();
    int before = 0, all = 0;
    for (int w = 0; w < nw; ++w) {
        const int t = lds[w];
        if (w < fg_wave()) before += t;
        all += t;
    }
    block_total = all;
    return before + r;
}

// Sum over the workgroup of a per-thread int64 value; every thread gets the result. `lds64` needs 16 entries.
__device__ __forceinline__ long long fg_block_sum(long long v, long long* lds64) {
    for (int off = FG_WAVE / 2; off > 0; off >>= 1) v += __shfl_down(v, off, FG_WAVE);
    const int nw = blockDim.x >> 6;
    __syncthreads();
    if (fg_lane() == 0) lds64[fg_wave()] = v;
    __syncthreads();
    long long s = 0;
    for (int w = 0; w < nw; ++w) s += lds64[w];
    return s;
}
