// lp_sparsify: the degree-based graph sparsifier of the paper (Algorithm 1, "Graph Sparsification"; Sec. IV-B).
// L edges are drawn independently, with replacement, from one partition's edge list, edge (u, v) with probability
// proportional to 1/d_u + 1/d_v (the degree bound on the effective resistance, Theorem 2); a drawn edge gets weight
// 1/(L p) and repeated draws add up, so the result is the set of distinct drawn edges, each with weight c/(L p).
//
// All decisions are taken in integer arithmetic, so every correct implementation returns the same edges:
//   q_e = floor(2^32/d_u) + floor(2^32/d_v),  Q = sum q_e,  p_e = q_e/Q;
//   draw l: r = 64 bits of Philox4x32-10(counter (l_lo, l_hi, 0, 0), key seed), t = floor(r Q / 2^64), and the
//   edge whose slice [cum_e, cum_e + q_e) of [0, Q) holds t (cum = running sum of q in input order).
// Pipeline: degree histogram (integer atomics) -> q -> 64-bit exclusive scan -> one thread per draw (binary
// search in cum, integer atomic count) -> compaction of the drawn edges in input order.
#include "lp_internal.h"
#include "lp_philox.h"
#include "lp_scan.h"

namespace {

using namespace lp_scan;

struct SparsifyWs {
    int32_t *deg;       // [n_nodes]
    uint64_t *q;        // [n_edges]
    uint64_t *cum;      // [n_edges + 1]
    int32_t *count;     // [n_edges]
    uint64_t *sums64;   // block sums of the 64-bit scan
    uint32_t *sums32;   // block sums of the 32-bit scan
    uint32_t *scalars;  // [0] = n_kept, [1] = range-error flag
    size_t bytes;
};

SparsifyWs carve(void *ws, int32_t n_nodes, int64_t n_edges) {
    char *p = static_cast<char *>(ws);
    size_t off = 0;
    auto take = [&](size_t bytes) { char *q = p ? p + off : nullptr; off += lp_align_up(bytes); return q; };
    SparsifyWs w;
    w.deg = reinterpret_cast<int32_t *>(take(sizeof(int32_t) * (size_t)n_nodes));
    w.q = reinterpret_cast<uint64_t *>(take(sizeof(uint64_t) * (size_t)n_edges));
    w.cum = reinterpret_cast<uint64_t *>(take(sizeof(uint64_t) * (size_t)(n_edges + 1)));
    w.count = reinterpret_cast<int32_t *>(take(sizeof(int32_t) * (size_t)n_edges));
    w.sums64 = reinterpret_cast<uint64_t *>(take(sizeof(uint64_t) * block_sum_count(n_edges + 1)));
    w.sums32 = reinterpret_cast<uint32_t *>(take(sizeof(uint32_t) * block_sum_count(n_edges)));
    w.scalars = reinterpret_cast<uint32_t *>(take(256));
    w.bytes = off;
    return w;
}

__global__ void degree_kernel(const int32_t *__restrict__ eu, const int32_t *__restrict__ ev, int64_t n_edges, int32_t n_nodes,
                              int32_t *__restrict__ deg, uint32_t *__restrict__ err) {
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= n_edges) return;
    const int32_t u = eu[e], v = ev[e];
    if (u < 0 || u >= n_nodes || v < 0 || v >= n_nodes) {
        atomicOr(err, 1u);
        return;
    }
    atomicAdd(&deg[u], 1);
    atomicAdd(&deg[v], 1);
}

__global__ void weight_kernel(const int32_t *__restrict__ eu, const int32_t *__restrict__ ev, int64_t n_edges, int32_t n_nodes,
                              const int32_t *__restrict__ deg, uint64_t *__restrict__ q) {
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= n_edges) return;
    const int32_t u = eu[e], v = ev[e];
    uint64_t x = 0;
    if (u >= 0 && u < n_nodes && v >= 0 && v < n_nodes)  // a listed edge gives both ends a degree of at least one
        x = ((uint64_t)1 << 32) / (uint64_t)deg[u] + ((uint64_t)1 << 32) / (uint64_t)deg[v];
    q[e] = x;
}

__global__ void draw_kernel(const uint64_t *__restrict__ cum, int64_t n_edges, int64_t n_draws, uint32_t seed_lo, uint32_t seed_hi,
                            int32_t *__restrict__ count) {
    const int64_t l = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (l >= n_draws) return;
    const uint64_t total = cum[n_edges];
    if (total == 0) return;
    const LpU4 w = lp_philox4x32_10(LpU4{(uint32_t)l, (uint32_t)((uint64_t)l >> 32), 0u, 0u}, seed_lo, seed_hi);
    const uint64_t r = ((uint64_t)w.x << 32) | w.y;
    const uint64_t t = __umul64hi(r, total);
    int64_t lo = 0, hi = n_edges;  // cum[lo] <= t < cum[hi]
    while (hi - lo > 1) {
        const int64_t mid = (lo + hi) >> 1;
        if (cum[mid] <= t) lo = mid; else hi = mid;
    }
    atomicAdd(&count[lo], 1);
}

}  // namespace

extern "C" size_t lp_sparsify_workspace_bytes(int32_t n_nodes, int64_t n_edges) {
    if (n_nodes <= 0 || n_edges < 0) return 0;
    return carve(nullptr, n_nodes, n_edges).bytes;
}

extern "C" int lp_sparsify(int32_t n_nodes, int64_t n_edges, const int32_t *eu, const int32_t *ev, int64_t n_draws, uint64_t seed,
                           int32_t *kept_edge, int32_t *kept_u, int32_t *kept_v, int32_t *kept_count, float *kept_weight,
                           int64_t *n_kept_out, void *ws, size_t ws_bytes, void *stream) {
    if (n_nodes <= 0 || n_edges < 0 || n_draws < 0 || !n_kept_out) return LP_ERR_INVALID_ARG;
    if (n_edges >= ((int64_t)1 << 31)) return LP_ERR_OUT_OF_RANGE;
    *n_kept_out = 0;
    if (n_edges == 0 || n_draws == 0) return LP_OK;
    if (!eu || !ev || !kept_edge || !kept_weight) return LP_ERR_INVALID_ARG;
    if (!ws || ws_bytes < lp_sparsify_workspace_bytes(n_nodes, n_edges)) return LP_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    SparsifyWs w = carve(ws, n_nodes, n_edges);
    const unsigned ge = (unsigned)lp_ceil_div(n_edges, 256);

    LP_TRY(lp_launch_zero(reinterpret_cast<float *>(w.deg), n_nodes, st));
    LP_TRY(lp_launch_zero(reinterpret_cast<float *>(w.count), n_edges, st));
    LP_TRY(lp_launch_zero(reinterpret_cast<float *>(w.scalars), 64, st));
    hipLaunchKernelGGL(degree_kernel, dim3(ge), dim3(256), 0, st, eu, ev, n_edges, n_nodes, w.deg, w.scalars + 1);
    hipLaunchKernelGGL(weight_kernel, dim3(ge), dim3(256), 0, st, eu, ev, n_edges, n_nodes, w.deg, w.q);
    LP_TRY(lp_after_launch());
    {   // cum[i] = q[0] + ... + q[i-1] for i = 0 .. n_edges (the scan runs over one extra, empty, element)
        const uint64_t *q = w.q;
        uint64_t *cum = w.cum;
        auto load = [q, n_edges] __device__(int64_t i) { return i < n_edges ? q[i] : (uint64_t)0; };
        auto store = [cum] __device__(int64_t i, uint64_t ex, uint64_t) { cum[i] = ex; };
        LP_TRY(device_exclusive_scan<uint64_t>(load, store, n_edges + 1, w.sums64, static_cast<uint64_t *>(nullptr), st));
    }
    hipLaunchKernelGGL(draw_kernel, dim3((unsigned)lp_ceil_div(n_draws, 256)), dim3(256), 0, st, w.cum, n_edges, n_draws,
                       (uint32_t)seed, (uint32_t)(seed >> 32), w.count);
    LP_TRY(lp_after_launch());
    {   // drawn edges, in input order
        const int32_t *count = w.count;
        const uint64_t *q = w.q, *cum = w.cum;
        const double draws = (double)n_draws;
        auto drawn = [count] __device__(int64_t e) { return (uint32_t)(count[e] > 0); };
        auto emit = [=] __device__(int64_t e, uint32_t pos, uint32_t flag) {
            if (!flag) return;
            kept_edge[pos] = (int32_t)e;
            if (kept_u) kept_u[pos] = eu[e];
            if (kept_v) kept_v[pos] = ev[e];
            if (kept_count) kept_count[pos] = count[e];
            // c / (L p) with p = q / Q
            kept_weight[pos] = (float)((double)count[e] * (double)cum[n_edges] / (draws * (double)q[e]));
        };
        LP_TRY(device_exclusive_scan<uint32_t>(drawn, emit, n_edges, w.sums32, w.scalars, st));
    }
    uint32_t host_scalars[2] = {0, 0};
    LP_HIP_TRY(hipMemcpyAsync(host_scalars, w.scalars, sizeof(host_scalars), hipMemcpyDeviceToHost, st));
    LP_HIP_TRY(hipStreamSynchronize(st));
    if (host_scalars[1]) return LP_ERR_OUT_OF_RANGE;
    *n_kept_out = (int64_t)host_scalars[0];
    return LP_OK;
}
