// lp_sample_neg: per-source uniform negative sampling (Sec. II-B of the paper; Algorithm 1, "Generate negative
// samples").  One thread per sample; the random stream is the counter-based Philox4x32-10 generator of Salmon,
// Moraes, Dror and Shaw (SC'11), so a sample's value depends only on (seed, step, sample index, attempt).
#include "lp_internal.h"
#include "lp_philox.h"

namespace {

__device__ inline bool row_contains(const int32_t *__restrict__ colidx, int32_t lo, int32_t hi, int32_t c) {
    const int32_t end = hi;
    while (lo < hi) {
        int32_t mid = lo + ((hi - lo) >> 1);
        if (colidx[mid] < c) lo = mid + 1; else hi = mid;
    }
    return lo < end && colidx[lo] == c;
}

__global__ __launch_bounds__(256) void sample_neg_kernel(const int32_t *__restrict__ rowptr, const int32_t *__restrict__ colidx,
                                                         int32_t n_nodes, const int32_t *__restrict__ pos_src, int64_t n_q,
                                                         int32_t k_neg, uint32_t n_space, uint32_t seed_lo, uint32_t seed_hi,
                                                         uint32_t step_lo, uint32_t step_hi, int32_t *__restrict__ neg_dst,
                                                         int32_t *__restrict__ neg_src, int32_t *__restrict__ n_failed) {
    const int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (q >= n_q) return;
    const int32_t u = pos_src[q / k_neg];
    int32_t lo = 0, hi = 0;
    if (u >= 0 && u < n_nodes) { lo = rowptr[u]; hi = rowptr[u + 1]; }
    int32_t c = 0;
    bool found = false;
    for (int blk = 0; blk < 4 && !found; ++blk) {
        const LpU4 r = lp_philox4x32_10(LpU4{(uint32_t)q, (uint32_t)blk, step_lo, step_hi}, seed_lo, seed_hi);
        const uint32_t word[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (!found) {
                c = (int32_t)(((uint64_t)word[i] * n_space) >> 32);
                found = (c != u) && !row_contains(colidx, lo, hi, c);
            }
        }
    }
    if (!found) {  // sixteen rejections: walk forward from the last candidate
        const int32_t last = c;
        for (uint32_t s = 0; s < n_space && !found; ++s) {
            c = c + 1 == (int32_t)n_space ? 0 : c + 1;
            found = (c != u) && !row_contains(colidx, lo, hi, c);
        }
        if (!found) {
            c = last;
            if (n_failed) atomicAdd(n_failed, 1);
        }
    }
    neg_dst[q] = c;
    if (neg_src) neg_src[q] = u;
}

}  // namespace

extern "C" int lp_sample_neg(const lp_csr *g, int64_t n_pos, const int32_t *pos_src, int32_t k_neg, int32_t n_space,
                             uint64_t seed, uint64_t step, int32_t *neg_dst, int32_t *neg_src, int32_t *n_failed,
                             void *stream) {
    if (!g || n_pos < 0 || k_neg < 0 || n_space <= 0 || g->n_nodes <= 0) return LP_ERR_INVALID_ARG;
    if (!g->rowptr || (g->nnz > 0 && !g->colidx)) return LP_ERR_INVALID_ARG;
    const int64_t n_q = n_pos * (int64_t)k_neg;
    if (n_pos > 0 && k_neg > 0 && n_pos > (((int64_t)1 << 31) - 1) / k_neg) return LP_ERR_OUT_OF_RANGE;
    if (n_q == 0) return LP_OK;
    if (!pos_src || !neg_dst) return LP_ERR_INVALID_ARG;
    LpTimedScope timed(LP_KC_SAMPLE, static_cast<hipStream_t>(stream));
    hipLaunchKernelGGL(sample_neg_kernel, dim3((unsigned)lp_ceil_div(n_q, 256)), dim3(256), 0,
                       static_cast<hipStream_t>(stream), g->rowptr, g->colidx, g->n_nodes, pos_src, n_q, k_neg,
                       (uint32_t)n_space, (uint32_t)seed, (uint32_t)(seed >> 32), (uint32_t)step, (uint32_t)(step >> 32),
                       neg_dst, neg_src, n_failed);
    return lp_after_launch();
}
