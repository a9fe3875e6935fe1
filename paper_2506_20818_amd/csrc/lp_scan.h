// Device-wide exclusive prefix sums over a functor, for 32- or 64-bit unsigned values: block sums, then every block
// adds up the sums of the blocks before it and applies (two launches; with more than kDirectBlocks blocks a
// one-block pass over the block sums comes in between).  Integer sums are associative, so the result does not
// depend on how the work is split.
// Everything here has internal linkage: each translation unit that includes this header gets its own kernels.
#pragma once

#include "lp_internal.h"

namespace lp_scan {
namespace {

constexpr int kThreads = 256;
constexpr int kItems = 8;
constexpr int kTile = kThreads * kItems;  // values per block

// words of block-sum workspace (of the value type) for a scan over n values
inline size_t block_sum_count(int64_t n) { return (size_t)(lp_ceil_div(n > 0 ? n : 1, kTile) + 8); }

// ------------------------------------------------------------------ block-wide exclusive prefix sum
template <class V>
__device__ inline V wave_inclusive_scan(V v) {
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        V o = __shfl_up(v, d, 64);
        if (lane >= d) v += o;
    }
    return v;
}

// 256 threads; returns the exclusive prefix of v over the block and the block total.
template <class V>
__device__ inline V block_exclusive_scan(V v, V *lds4, V &total) {
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    V inc = wave_inclusive_scan(v);
    __syncthreads();
    if (lane == 63) lds4[w] = inc;
    __syncthreads();
    V off = 0;
    V t = 0;
#pragma unroll
    for (int i = 0; i < kThreads / 64; ++i) {
        V s = lds4[i];
        if (i < w) off += s;
        t += s;
    }
    total = t;
    return off + inc - v;
}

// ------------------------------------------------------------------ device-wide exclusive scan of f(i), i < n
template <class V, class F>
__global__ __launch_bounds__(kThreads) void scan_reduce_kernel(F f, int64_t n, V *block_sums) {
    __shared__ V lds4[4];
    const int64_t base = (int64_t)blockIdx.x * kTile + (int64_t)threadIdx.x * kItems;
    V s = 0;
#pragma unroll
    for (int i = 0; i < kItems; ++i)
        if (base + i < n) s += f(base + i);
    V total;
    block_exclusive_scan(s, lds4, total);
    if (threadIdx.x == 0) block_sums[blockIdx.x] = total;
}

// one block: block_sums[i] <- exclusive prefix; *total <- sum
template <class V>
__global__ __launch_bounds__(kThreads) void scan_spine_kernel(V *block_sums, int64_t nb, V *total_out) {
    __shared__ V lds4[4];
    V carry = 0;
    for (int64_t base = 0; base < nb; base += kThreads) {
        int64_t i = base + threadIdx.x;
        V v = i < nb ? block_sums[i] : 0u;
        V total;
        V ex = block_exclusive_scan(v, lds4, total);
        if (i < nb) block_sums[i] = carry + ex;
        carry += total;
        __syncthreads();
    }
    if (threadIdx.x == 0 && total_out) *total_out = carry;
}

// sink(i, exclusive_prefix_of_i, f(i)) is called for every i < n.  DIRECT: block_sums holds the plain block sums and
// the block adds up those before it itself (the last block also writes the grand total); otherwise block_sums holds
// their exclusive prefix.
template <class V, class F, class S, bool DIRECT>
__global__ __launch_bounds__(kThreads) void scan_apply_kernel(F f, S sink, int64_t n, const V *block_sums, V *total_out) {
    __shared__ V lds4[4];
    const int64_t base = (int64_t)blockIdx.x * kTile + (int64_t)threadIdx.x * kItems;
    V v[kItems];
    V s = 0;
#pragma unroll
    for (int i = 0; i < kItems; ++i) {
        v[i] = (base + i < n) ? f(base + i) : 0u;
        s += v[i];
    }
    V before;
    if (DIRECT) {
        V mine = 0;
        for (int64_t i = threadIdx.x; i < (int64_t)blockIdx.x; i += kThreads) mine += block_sums[i];
        block_exclusive_scan(mine, lds4, before);
        __syncthreads();
    } else {
        before = block_sums[blockIdx.x];
    }
    V total;
    V run = before + block_exclusive_scan(s, lds4, total);
    if (DIRECT && total_out && blockIdx.x == gridDim.x - 1 && threadIdx.x == 0) *total_out = before + total;
#pragma unroll
    for (int i = 0; i < kItems; ++i) {
        if (base + i < n) sink(base + i, run, v[i]);
        run += v[i];
    }
}

constexpr int64_t kDirectBlocks = 4096;  // up to here every block reads the sums of all blocks before it

template <class V, class F, class S>
int device_exclusive_scan(F f, S sink, int64_t n, V *block_sums, V *total_out, hipStream_t st) {
    const int64_t nb = lp_ceil_div(n > 0 ? n : 1, kTile);
    hipLaunchKernelGGL((scan_reduce_kernel<V, F>), dim3((unsigned)nb), dim3(kThreads), 0, st, f, n, block_sums);
    if (nb <= kDirectBlocks) {
        hipLaunchKernelGGL((scan_apply_kernel<V, F, S, true>), dim3((unsigned)nb), dim3(kThreads), 0, st, f, sink, n, block_sums, total_out);
    } else {
        hipLaunchKernelGGL((scan_spine_kernel<V>), dim3(1), dim3(kThreads), 0, st, block_sums, nb, total_out);
        hipLaunchKernelGGL((scan_apply_kernel<V, F, S, false>), dim3((unsigned)nb), dim3(kThreads), 0, st, f, sink, n, block_sums, total_out);
    }
    return lp_after_launch();
}

}  // namespace
}  // namespace lp_scan
