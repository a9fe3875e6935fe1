// Hits@K, the accuracy metric of the paper's experiments ("Hyperparameters": Hits@100, the Open Graph Benchmark's
// link-prediction metric): the K-th largest score among the negative edges is the threshold, and a positive edge is
// a hit when its score is strictly greater.  Integer result: exactly one answer is correct for given scores.
//
// The negative scores are mapped to 32-bit keys that sort like the floats (sign bit flipped for non-negative values,
// all bits flipped for negative ones), sorted with the library's radix sort (four 8-bit passes) and the key at
// position n_neg - K is mapped back; the positives above it are counted with integer atomics.
#include "lp_internal.h"

namespace {

__device__ __forceinline__ uint32_t ordered_bits(float x) {
    const uint32_t u = __float_as_uint(x);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float from_ordered_bits(uint32_t k) {
    return __uint_as_float((k & 0x80000000u) ? (k & 0x7fffffffu) : ~k);
}

__global__ void score_keys_kernel(const float *__restrict__ s, int64_t n, uint64_t *__restrict__ keys) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) keys[i] = ordered_bits(s[i] + 0.0f);   // + 0.0f: -0.0 and +0.0 compare equal as floats, so as keys too
}

// hits <- 0, threshold <- K-th largest (or -inf when there are fewer than K keys)
__global__ void threshold_kernel(const uint64_t *__restrict__ sorted, int64_t n, int64_t K, float *__restrict__ thr_out,
                                 float *__restrict__ thr_ws, unsigned long long *__restrict__ hits) {
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        const float t = n >= K ? from_ordered_bits((uint32_t)sorted[n - K]) : -INFINITY;
        *thr_ws = t;
        if (thr_out) *thr_out = t;
        *hits = 0ull;
    }
}

__global__ __launch_bounds__(256) void count_hits_kernel(const float *__restrict__ pos, int64_t n, const float *__restrict__ thr,
                                                         unsigned long long *__restrict__ hits) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const bool hit = i < n && pos[i] > *thr;
    const unsigned long long b = __ballot(hit);
    if ((threadIdx.x & 63) == 0 && b) atomicAdd(hits, (unsigned long long)__popcll(b));
}

struct EvalWs {
    uint64_t *keys_a, *keys_b;
    uint32_t *hist;
    float *thr;
    size_t bytes;
};

EvalWs carve_eval(void *ws, int64_t n_neg) {
    char *p = static_cast<char *>(ws);
    size_t off = 0;
    auto take = [&](size_t bytes) { char *q = p ? p + off : nullptr; off += lp_align_up(bytes); return q; };
    EvalWs w;
    const size_t n = (size_t)(n_neg > 0 ? n_neg : 1);
    w.keys_a = reinterpret_cast<uint64_t *>(take(sizeof(uint64_t) * n));
    w.keys_b = reinterpret_cast<uint64_t *>(take(sizeof(uint64_t) * n));
    w.hist = reinterpret_cast<uint32_t *>(take(sizeof(uint32_t) * lp_radix_sort_hist_words((int64_t)n)));
    w.thr = reinterpret_cast<float *>(take(256));
    w.bytes = off;
    return w;
}

}  // namespace

extern "C" size_t lp_hits_at_k_workspace_bytes(int64_t n_neg) {
    if (n_neg < 0) return 0;
    return carve_eval(nullptr, n_neg).bytes;
}

extern "C" int lp_hits_at_k(const float *pos_scores, int64_t n_pos, const float *neg_scores, int64_t n_neg, int64_t K,
                            int64_t *hits, float *threshold, void *ws, size_t ws_bytes, void *stream) {
    if (n_pos < 0 || n_neg < 0 || K < 1 || !hits) return LP_ERR_INVALID_ARG;
    if ((n_pos > 0 && !pos_scores) || (n_neg > 0 && !neg_scores)) return LP_ERR_INVALID_ARG;
    if (n_neg >= ((int64_t)1 << 31) || n_pos >= ((int64_t)1 << 40)) return LP_ERR_OUT_OF_RANGE;
    if (!ws || ws_bytes < lp_hits_at_k_workspace_bytes(n_neg)) return LP_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const EvalWs w = carve_eval(ws, n_neg);
    const uint64_t *sorted = w.keys_a;
    if (n_neg > 0) {
        hipLaunchKernelGGL(score_keys_kernel, dim3((unsigned)lp_ceil_div(n_neg, 256)), dim3(256), 0, st, neg_scores, n_neg, w.keys_a);
        int status;
        sorted = lp_radix_sort(w.keys_a, w.keys_b, n_neg, 0, 32, w.hist, st, &status);
        LP_TRY(status);
    }
    hipLaunchKernelGGL(threshold_kernel, dim3(1), dim3(64), 0, st, sorted, n_neg, K, threshold, w.thr,
                       reinterpret_cast<unsigned long long *>(hits));
    if (n_pos > 0)
        hipLaunchKernelGGL(count_hits_kernel, dim3((unsigned)lp_ceil_div(n_pos, 256)), dim3(256), 0, st, pos_scores, n_pos, w.thr,
                           reinterpret_cast<unsigned long long *>(hits));
    return lp_after_launch();
}
