// Sampled-neighbourhood form of the training step: the per-mini-batch computational graph of the paper (Sec. II-B,
// last paragraph; Fig. 1b; "Hyperparameters": 25, 10 and 5 sampled neighbours for the first, second and third hop).
//
// lp_sample_blocks builds, for one batch of scored edges, the K bipartite blocks of that graph:
//   frontier K  = the end points of the scored edges, ascending;
//   hop h = 1..K (layer k = K+1-h): every node of frontier k draws min(degree, fanout[h-1]) distinct neighbours
//   uniformly without replacement; frontier k-1 = frontier k followed by the drawn nodes that are new, ascending.
// Every frontier is therefore a prefix of one node list, and a node keeps its position through all layers.
// The draw is a partial Fisher-Yates shuffle over the positions of the (sorted) neighbour list: swap t exchanges
// position t with t + floor(word * (d - t) / 2^32), word = word (t mod 4) of Philox4x32-10 with counter
// (node, hop * 2^16 + t div 4, step_lo, step_hi) and key (seed_lo, seed_hi); a node whose degree fits takes all its
// neighbours in list order.  Everything here is integer work and has exactly one correct result.
// lp_sage_forward_blocks / lp_backward_blocks evaluate Eq. (1) and its gradient on those blocks with the same
// aggregation and MFMA kernels as the full-graph calls; row counts live on the device, grids are sized by bounds.
#include "lp_internal.h"
#include "lp_philox.h"
#include "lp_scan.h"

namespace {

using namespace lp_scan;

// ---------------------------------------------------------------------------------------------- bounds
struct Bounds {
    int32_t cap[LP_MAX_LAYERS + 1];
    int64_t cap_entries[LP_MAX_LAYERS];
    int64_t max_entries;
};

int compute_bounds(int32_t n_nodes, int64_t nnz, int64_t B, int32_t K, const int32_t *fanout, Bounds &b) {
    if (n_nodes <= 0 || nnz < 0 || B < 0 || K < 1 || K > LP_MAX_LAYERS || !fanout) return LP_ERR_INVALID_ARG;
    if (B >= ((int64_t)1 << 30) || nnz >= ((int64_t)1 << 31)) return LP_ERR_OUT_OF_RANGE;
    for (int h = 0; h < K; ++h)
        if (fanout[h] != LP_FANOUT_ALL && (fanout[h] < 1 || fanout[h] > LP_MAX_FANOUT)) return LP_ERR_UNSUPPORTED;
    int64_t c = 2 * B < n_nodes ? 2 * B : n_nodes;
    b.cap[K] = (int32_t)c;
    b.max_entries = 1;
    for (int k = K; k >= 1; --k) {
        const int64_t f = fanout[K - k] == LP_FANOUT_ALL ? nnz + 1 : fanout[K - k];   // all neighbours: only nnz and N bound it
        int64_t e = c * f < nnz ? c * f : nnz;
        b.cap_entries[k - 1] = e;
        b.max_entries = e > b.max_entries ? e : b.max_entries;
        c = c * (1 + f) < n_nodes ? c * (1 + f) : n_nodes;
        b.cap[k - 1] = (int32_t)c;
    }
    return LP_OK;
}

// ---------------------------------------------------------------------------------------------- sampling kernels
__global__ void mark_endpoints_kernel(const int32_t *__restrict__ e_src, const int32_t *__restrict__ e_dst, int64_t B,
                                      int32_t n_nodes, int32_t *__restrict__ mark) {
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= B) return;
    const int32_t u = e_src[e], v = e_dst[e];
    if (u >= 0 && u < n_nodes) mark[u] = 1;  // every writer stores the same value
    if (v >= 0 && v < n_nodes) mark[v] = 1;
}

__global__ void edge_positions_kernel(const int32_t *__restrict__ e_src, const int32_t *__restrict__ e_dst, int64_t B,
                                      int32_t n_nodes, const int32_t *__restrict__ index, int32_t *__restrict__ ps,
                                      int32_t *__restrict__ pd) {
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= B) return;
    const int32_t u = e_src[e], v = e_dst[e];
    ps[e] = (u >= 0 && u < n_nodes) ? index[u] : -1;
    pd[e] = (v >= 0 && v < n_nodes) ? index[v] : -1;
}

__global__ void set_scalar_kernel(int32_t *dst, const int32_t *a, const uint32_t *b) {
    if (blockIdx.x == 0 && threadIdx.x == 0) *dst = (a ? *a : 0) + (int32_t)*b;
}

// G lanes per node of the frontier (G >= fan): its sample, in draw order, as global ids.  The partial Fisher-Yates
// shuffle runs over the virtual array a[p] = p; the positions written so far are remembered one per lane (in the order
// they were written), so "the current value at position r" is a ballot over the group and the latest matching lane.
// Lane q of a group computes Philox block q (the words of swaps 4q .. 4q+3) once, before the swaps.
template <int G>
__global__ __launch_bounds__(256) void sample_rows_kernel(const int32_t *__restrict__ rowptr, const int32_t *__restrict__ colidx,
                                                          const int32_t *__restrict__ nodes, const int32_t *__restrict__ n_rows_dev,
                                                          int32_t fan, uint32_t hop, uint32_t seed_lo, uint32_t seed_hi,
                                                          uint32_t step_lo, uint32_t step_hi, const int32_t *__restrict__ ptr,
                                                          int32_t *__restrict__ col_global, int32_t *__restrict__ row_of_entry,
                                                          const int32_t *__restrict__ index, int32_t *__restrict__ mark) {
    const int lane = threadIdx.x & 63, sub = lane % G, gbase = lane - sub;
    const int64_t i = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) / G;
    const bool live = i < *n_rows_dev;
    int32_t v = 0, lo = 0, d = 0, base = 0;
    if (live) {
        v = nodes[i];
        lo = rowptr[v];
        d = rowptr[v + 1] - lo;
        base = ptr[i];
    }
    const bool drawn = d > fan;          // same for all lanes of a group
    int32_t position = sub;              // a node with d <= fan takes all its neighbours in list order
    if (__any(drawn)) {
        LpU4 w = {0u, 0u, 0u, 0u};
        if (drawn && 4 * sub < fan) w = lp_philox4x32_10(LpU4{(uint32_t)v, (hop << 16) + (uint32_t)sub, step_lo, step_hi}, seed_lo, seed_hi);
        const uint64_t gmask = G == 64 ? ~0ull : ((1ull << (G & 63)) - 1ull);
        int32_t mpos = -1, mval = 0;     // remembered write number `sub` of this group
        int nm = 0;                      // writes remembered so far
        for (int t = 0; t < fan; ++t) {  // every lane of the wavefront runs the same trip count
            const uint32_t mine = (t & 3) == 0 ? w.x : (t & 3) == 1 ? w.y : (t & 3) == 2 ? w.z : w.w;
            const uint32_t word = (uint32_t)__shfl((int)mine, gbase + (t >> 2));
            const int32_t r = t + (int32_t)(((uint64_t)word * (uint32_t)(drawn ? d - t : 1)) >> 32);
            const uint64_t hit_r = (__ballot(sub < nm && mpos == r) >> gbase) & gmask;
            const uint64_t hit_t = (__ballot(sub < nm && mpos == t) >> gbase) & gmask;
            const int32_t from_r = __shfl(mval, gbase + (hit_r ? 63 - __clzll((long long)hit_r) : 0));
            const int32_t from_t = __shfl(mval, gbase + (hit_t ? 63 - __clzll((long long)hit_t) : 0));
            const int32_t val_r = hit_r ? from_r : r, val_t = hit_t ? from_t : t;
            if (r != t) {
                if (sub == nm) { mpos = r; mval = val_t; }
                ++nm;
            }
            if (drawn && sub == t) position = val_r;
        }
    }
    const int32_t take = d < fan ? d : fan;
    if (live && sub < take) {
        const int32_t u = colidx[lo + position];
        col_global[base + sub] = u;
        row_of_entry[base + sub] = (int32_t)i;
        if (index[u] < 0) mark[u] = 1;  // joins the next frontier; every writer stores the same value
    }
}

// Full-neighbourhood hop: a 64-lane group per node of the frontier copies the node's whole list, in list order.
__global__ __launch_bounds__(256) void take_all_rows_kernel(const int32_t *__restrict__ rowptr, const int32_t *__restrict__ colidx,
                                                            const int32_t *__restrict__ nodes, const int32_t *__restrict__ n_rows_dev,
                                                            const int32_t *__restrict__ ptr, int32_t *__restrict__ col_global,
                                                            int32_t *__restrict__ row_of_entry, const int32_t *__restrict__ index,
                                                            int32_t *__restrict__ mark) {
    const int lane = threadIdx.x & 63;
    const int64_t i = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    if (i >= *n_rows_dev) return;
    const int32_t v = nodes[i];
    const int32_t lo = rowptr[v], d = rowptr[v + 1] - lo, base = ptr[i];
    for (int32_t t = lane; t < d; t += 64) {
        const int32_t u = colidx[lo + t];
        col_global[base + t] = u;
        row_of_entry[base + t] = (int32_t)i;
        if (index[u] < 0) mark[u] = 1;  // joins the next frontier; every writer stores the same value
    }
}

__global__ void node_inv_deg_kernel(const int32_t *__restrict__ nodes, const int32_t *__restrict__ n_dev, const float *__restrict__ inv_deg,
                                    float *__restrict__ out) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < *n_dev) out[i] = inv_deg[nodes[i]];
}

// Local column of every entry, its sort key (column, position), and the entry count as a device scalar: the sort and
// the row offsets of the transposed block run over the entries actually drawn, not over the capacity.
__global__ void translate_kernel(const int32_t *__restrict__ col_global, const int32_t *__restrict__ ptr,
                                 const int32_t *__restrict__ n_rows_dev, int64_t cap_entries, const int32_t *__restrict__ index,
                                 int32_t *__restrict__ col, uint64_t *__restrict__ keys, uint32_t *__restrict__ n_entries_out) {
    const int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int32_t n_entries = ptr[*n_rows_dev];
    if (p == 0) *n_entries_out = (uint32_t)n_entries;
    if (p >= cap_entries || p >= n_entries) return;
    const int32_t c = index[col_global[p]];
    col[p] = c;
    keys[p] = ((uint64_t)(uint32_t)c << 32) | (uint32_t)p;
}

__global__ void transposed_cols_kernel(const uint64_t *__restrict__ sorted, const int32_t *__restrict__ ptr,
                                       const int32_t *__restrict__ n_rows_dev, int64_t cap_entries,
                                       const int32_t *__restrict__ row_of_entry, int32_t *__restrict__ t_col) {
    const int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= cap_entries || p >= ptr[*n_rows_dev]) return;
    t_col[p] = row_of_entry[(uint32_t)sorted[p]];
}

template <typename T>
__global__ void gather_rows_kernel(const T *__restrict__ in, const int32_t *__restrict__ rows, const int32_t *__restrict__ n_rows_dev,
                                   int FV, T *__restrict__ out) {
    constexpr int VE = LpVec<T>::N;
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t i = idx / FV;
    const int c = (int)(idx % FV);
    if (i >= *n_rows_dev) return;
    float x[VE];
    LpVec<T>::load(in + ((int64_t)rows[i] * FV + c) * VE, x);
    LpVec<T>::store(out + (i * FV + c) * VE, x);
}

struct SampleWs {
    int32_t *mark;          // [n_nodes]
    int32_t *col_global;    // [max entries]
    int32_t *row_of_entry;  // [max entries]
    uint64_t *keys_a, *keys_b;
    uint32_t *hist;
    uint32_t *sums;         // block sums of the scans
    uint32_t *total;        // scalar
    size_t bytes;
};

SampleWs carve_sample(void *ws, int32_t n_nodes, const Bounds &b) {
    char *p = static_cast<char *>(ws);
    size_t off = 0;
    auto take = [&](size_t bytes) { char *q = p ? p + off : nullptr; off += lp_align_up(bytes); return q; };
    SampleWs w;
    const size_t me = (size_t)b.max_entries;
    w.mark = reinterpret_cast<int32_t *>(take(sizeof(int32_t) * (size_t)n_nodes));
    w.col_global = reinterpret_cast<int32_t *>(take(sizeof(int32_t) * me));
    w.row_of_entry = reinterpret_cast<int32_t *>(take(sizeof(int32_t) * me));
    w.keys_a = reinterpret_cast<uint64_t *>(take(sizeof(uint64_t) * (me + 1)));
    w.keys_b = reinterpret_cast<uint64_t *>(take(sizeof(uint64_t) * (me + 1)));
    w.hist = reinterpret_cast<uint32_t *>(take(sizeof(uint32_t) * lp_radix_sort_hist_words((int64_t)me + 1)));
    w.sums = reinterpret_cast<uint32_t *>(take(sizeof(uint32_t) * block_sum_count((int64_t)n_nodes + 1)));
    w.total = reinterpret_cast<uint32_t *>(take(256));
    w.bytes = off;
    return w;
}

int check_blocks(const lp_blocks *b, bool need_transposed) {
    if (!b || b->n_layers < 1 || b->n_layers > LP_MAX_LAYERS || b->n_graph_nodes <= 0) return LP_ERR_INVALID_ARG;
    if (!b->n || !b->nodes || !b->index || !b->e_src_pos || !b->e_dst_pos || !b->node_inv_deg) return LP_ERR_INVALID_ARG;
    for (int k = 0; k <= b->n_layers; ++k)
        if (b->cap[k] < 0 || (k < b->n_layers && b->cap[k] < b->cap[k + 1])) return LP_ERR_INVALID_ARG;
    for (int k = 0; k < b->n_layers; ++k) {
        if (b->cap_entries[k] < 0 || b->cap_entries[k] >= ((int64_t)1 << 31)) return LP_ERR_INVALID_ARG;
        if (!b->ptr[k] || !b->inv_cnt[k] || (b->cap_entries[k] > 0 && !b->col[k])) return LP_ERR_INVALID_ARG;
        if (need_transposed && (!b->t_ptr[k] || (b->cap_entries[k] > 0 && !b->t_col[k]))) return LP_ERR_INVALID_ARG;
    }
    return LP_OK;
}

int check_block_model(const lp_model *m, const lp_blocks *b) {
    if (!m || m->n_layers != b->n_layers) return LP_ERR_INVALID_ARG;
    if (m->dtype != LP_F32 && m->dtype != LP_BF16) return LP_ERR_UNSUPPORTED;
    if (m->layer_type != LP_LAYER_SAGE_MEAN && m->layer_type != LP_LAYER_GCN) return LP_ERR_UNSUPPORTED;
    if (!lp_valid_fp32_products(m->fp32_products) || m->reserved_ != 0) return LP_ERR_INVALID_ARG;
    const bool gcn = m->layer_type == LP_LAYER_GCN;   // a single weight matrix (W_neigh) per layer
    for (int k = 0; k <= m->n_layers; ++k) {
        if (m->dims[k] <= 0) return LP_ERR_INVALID_ARG;
        if ((m->dims[k] % lp_vec_elems(m->dtype)) || m->dims[k] > 1024) return LP_ERR_UNSUPPORTED;
    }
    for (int k = 0; k < m->n_layers; ++k) {
        if ((!gcn && !m->W_self[k]) || !m->W_neigh[k] || !m->bias[k]) return LP_ERR_INVALID_ARG;
        if ((!gcn && !lp_aligned16(m->W_self[k])) || !lp_aligned16(m->W_neigh[k])) return LP_ERR_INVALID_ARG;
    }
    return LP_OK;
}

size_t transposed_weight_bytes(const lp_model *m) {
    size_t n = 0;
    for (int k = 0; k < m->n_layers; ++k) n += 2 * lp_align_up((size_t)m->dims[k] * m->dims[k + 1], 64);
    return lp_align_up(n * (size_t)lp_elem_bytes(m->dtype));
}

int max_dim(const lp_model *m) {
    int d = 0;
    for (int k = 0; k <= m->n_layers; ++k) d = m->dims[k] > d ? m->dims[k] : d;
    return d;
}

struct BlockBackwardWs {
    void *buf[3];
    float *tn_partials, *colsum_partials;
    BatchGroupWs group;
    int32_t *bptr, *bcol;
    float *bw;
    int32_t *long_queue;
    size_t bytes;
};

BlockBackwardWs carve_block_backward(void *ws, const lp_model *m, const lp_blocks *b) {
    char *p = static_cast<char *>(ws);
    size_t off = 0;
    auto take = [&](size_t bytes) { char *q = p ? p + off : nullptr; off += lp_align_up(bytes); return q; };
    BlockBackwardWs w;
    const int K = m->n_layers;
    // gradient matrices of layer k have cap[k] rows; the widest of them all bounds the three rotating buffers
    size_t big = 0;
    for (int k = 1; k <= K; ++k) {
        const size_t a = (size_t)b->cap[k] * m->dims[k], c = (size_t)b->cap[k - 1] * m->dims[k - 1];
        big = a > big ? a : big;
        big = c > big ? c : big;
    }
    big *= (size_t)lp_elem_bytes(m->dtype);
    for (int i = 0; i < 3; ++i) w.buf[i] = take(big);
    size_t tn = 0, cs = 0;
    for (int k = 1; k <= K; ++k) {
        const size_t t = lp_weight_grads_partials_bytes(m->dtype, b->cap[k] > 0 ? b->cap[k] : 1,
                                                        m->layer_type == LP_LAYER_GCN ? 0 : m->dims[k - 1], m->dims[k - 1], m->dims[k]);
        tn = t > tn ? t : tn;
        const size_t c = lp_colsum_partials_bytes(b->cap[k], m->dims[k]);
        cs = c > cs ? c : cs;
    }
    w.tn_partials = reinterpret_cast<float *>(take(tn));
    w.colsum_partials = reinterpret_cast<float *>(take(cs));
    const size_t n2 = (size_t)(2 * (b->n_edges > 0 ? b->n_edges : 0) + 1);
    w.group.keys_a = reinterpret_cast<uint64_t *>(take(sizeof(uint64_t) * n2));
    w.group.keys_b = reinterpret_cast<uint64_t *>(take(sizeof(uint64_t) * n2));
    w.group.hist = reinterpret_cast<uint32_t *>(take(sizeof(uint32_t) * lp_radix_sort_hist_words((int64_t)n2)));
    w.bptr = reinterpret_cast<int32_t *>(take(sizeof(int32_t) * ((size_t)b->cap[K] + 1)));
    w.bcol = reinterpret_cast<int32_t *>(take(sizeof(int32_t) * n2));
    w.bw = reinterpret_cast<float *>(take(sizeof(float) * n2));
    w.long_queue = reinterpret_cast<int32_t *>(take(lp_spmm_queue_bytes(b->cap[0], max_dim(m))));
    w.bytes = off;
    return w;
}

}  // namespace

extern "C" int lp_blocks_bounds(int32_t n_nodes, int64_t nnz, int64_t B, int32_t K, const int32_t *fanout, int32_t *cap,
                                int64_t *cap_entries) {
    Bounds b;
    LP_TRY(compute_bounds(n_nodes, nnz, B, K, fanout, b));
    if (!cap || !cap_entries) return LP_ERR_INVALID_ARG;
    for (int k = 0; k <= K; ++k) cap[k] = b.cap[k];
    for (int k = 0; k < K; ++k) cap_entries[k] = b.cap_entries[k];
    return LP_OK;
}

extern "C" size_t lp_sample_blocks_workspace_bytes(int32_t n_nodes, int64_t nnz, int64_t B, int32_t K, const int32_t *fanout) {
    Bounds b;
    if (compute_bounds(n_nodes, nnz, B, K, fanout, b) != LP_OK) return 0;
    return carve_sample(nullptr, n_nodes, b).bytes;
}

extern "C" int lp_sample_blocks(const lp_csr *g, int64_t B, const int32_t *e_src, const int32_t *e_dst, int32_t K,
                                const int32_t *fanout, uint64_t seed, uint64_t step, lp_blocks *out, void *ws, size_t ws_bytes,
                                void *stream) {
    if (!g || g->n_nodes <= 0 || g->nnz < 0 || !g->rowptr || (g->nnz > 0 && !g->colidx) || !g->inv_deg || !out) return LP_ERR_INVALID_ARG;
    Bounds bd;
    LP_TRY(compute_bounds(g->n_nodes, g->nnz, B, K, fanout, bd));
    if (B > 0 && (!e_src || !e_dst)) return LP_ERR_INVALID_ARG;
    LP_TRY(check_blocks(out, true));
    if (out->n_layers != K || out->n_graph_nodes != g->n_nodes || out->n_edges != B) return LP_ERR_INVALID_ARG;
    for (int k = 0; k <= K; ++k)
        if (out->cap[k] < bd.cap[k]) return LP_ERR_INVALID_ARG;
    for (int k = 0; k < K; ++k)
        if (out->cap_entries[k] < bd.cap_entries[k]) return LP_ERR_INVALID_ARG;
    if (!ws || ws_bytes < lp_sample_blocks_workspace_bytes(g->n_nodes, g->nnz, B, K, fanout)) return LP_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const SampleWs w = carve_sample(ws, g->n_nodes, bd);
    const int32_t N = g->n_nodes;
    LpTimedScope timed(LP_KC_SAMPLE, st);

    // frontier K: the end points of the scored edges, ascending
    LP_TRY(lp_launch_zero(reinterpret_cast<float *>(w.mark), N, st));
    if (B > 0) hipLaunchKernelGGL(mark_endpoints_kernel, dim3((unsigned)lp_ceil_div(B, 256)), dim3(256), 0, st, e_src, e_dst, B, N, w.mark);
    {
        const int32_t *mark = w.mark;
        int32_t *nodes = out->nodes, *index = out->index;
        auto flagged = [mark] __device__(int64_t v) { return (uint32_t)mark[v]; };
        auto place = [nodes, index] __device__(int64_t v, uint32_t pos, uint32_t flag) {
            index[v] = flag ? (int32_t)pos : -1;
            if (flag) nodes[pos] = (int32_t)v;
        };
        LP_TRY(device_exclusive_scan<uint32_t>(flagged, place, (int64_t)N, w.sums, w.total, st));
        hipLaunchKernelGGL(set_scalar_kernel, dim3(1), dim3(64), 0, st, out->n + K, static_cast<const int32_t *>(nullptr), w.total);
    }
    if (B > 0)
        hipLaunchKernelGGL(edge_positions_kernel, dim3((unsigned)lp_ceil_div(B, 256)), dim3(256), 0, st, e_src, e_dst, B, N, out->index,
                           out->e_src_pos, out->e_dst_pos);
    LP_TRY(lp_after_launch());

    for (int k = K; k >= 1; --k) {
        const bool take_all = fanout[K - k] == LP_FANOUT_ALL;
        const int32_t fan = take_all ? 0x7fffffff : fanout[K - k];
        const uint32_t hop = (uint32_t)(K + 1 - k);
        const int32_t cap_k = out->cap[k] < bd.cap[k] ? out->cap[k] : bd.cap[k];
        const int64_t cap_e = bd.cap_entries[k - 1];
        const int32_t *n_k = out->n + k;
        int32_t *ptr = out->ptr[k - 1];
        float *inv_cnt = out->inv_cnt[k - 1];
        {   // ptr[i] = entries of the rows before i; the scan runs one element further so that ptr[n_k] is the total
            const int32_t *rowptr = g->rowptr, *nodes = out->nodes;
            auto count = [rowptr, nodes, n_k, fan] __device__(int64_t i) {
                if (i >= *n_k) return (uint32_t)0;
                const int32_t v = nodes[i];
                const int32_t d = rowptr[v + 1] - rowptr[v];
                return (uint32_t)(d < fan ? d : fan);
            };
            auto store = [ptr, inv_cnt, n_k] __device__(int64_t i, uint32_t ex, uint32_t c) {
                ptr[i] = (int32_t)ex;
                if (i < *n_k) inv_cnt[i] = c ? 1.0f / (float)c : 0.0f;
            };
            LP_TRY(device_exclusive_scan<uint32_t>(count, store, (int64_t)cap_k + 1, w.sums, static_cast<uint32_t *>(nullptr), st));
        }
        LP_TRY(lp_launch_zero(reinterpret_cast<float *>(w.mark), N, st));
        if (cap_k <= 0) {
            // nothing to draw from
        } else if (take_all) {
            hipLaunchKernelGGL(take_all_rows_kernel, dim3((unsigned)lp_ceil_div((int64_t)cap_k * 64, 256)), dim3(256), 0, st, g->rowptr, g->colidx,
                               out->nodes, n_k, ptr, w.col_global, w.row_of_entry, out->index, w.mark);
        } else {
            const int G = fan <= 16 ? 16 : 64;
            const dim3 sgrid((unsigned)lp_ceil_div((int64_t)cap_k * G, 256));
            if (G == 16)
                hipLaunchKernelGGL(sample_rows_kernel<16>, sgrid, dim3(256), 0, st, g->rowptr, g->colidx, out->nodes, n_k, fan, hop, (uint32_t)seed,
                                   (uint32_t)(seed >> 32), (uint32_t)step, (uint32_t)(step >> 32), ptr, w.col_global, w.row_of_entry, out->index,
                                   w.mark);
            else
                hipLaunchKernelGGL(sample_rows_kernel<64>, sgrid, dim3(256), 0, st, g->rowptr, g->colidx, out->nodes, n_k, fan, hop, (uint32_t)seed,
                                   (uint32_t)(seed >> 32), (uint32_t)step, (uint32_t)(step >> 32), ptr, w.col_global, w.row_of_entry, out->index,
                                   w.mark);
        }
        {   // the drawn nodes that are new join the node list, ascending
            const int32_t *mark = w.mark;
            int32_t *nodes = out->nodes, *index = out->index;
            auto flagged = [mark] __device__(int64_t v) { return (uint32_t)mark[v]; };
            auto place = [nodes, index, n_k] __device__(int64_t v, uint32_t pos, uint32_t flag) {
                if (flag) {
                    const int32_t at = *n_k + (int32_t)pos;
                    nodes[at] = (int32_t)v;
                    index[v] = at;
                }
            };
            LP_TRY(device_exclusive_scan<uint32_t>(flagged, place, (int64_t)N, w.sums, w.total, st));
            hipLaunchKernelGGL(set_scalar_kernel, dim3(1), dim3(64), 0, st, out->n + (k - 1), n_k, w.total);
        }
        if (cap_e > 0) {
            const unsigned ge = (unsigned)lp_ceil_div(cap_e, 256);
            uint32_t *n_entries = w.total + 8;   // its own word of the scalar area
            hipLaunchKernelGGL(translate_kernel, dim3(ge), dim3(256), 0, st, w.col_global, ptr, n_k, cap_e, out->index, out->col[k - 1],
                               w.keys_a, n_entries);
            int status;
            const uint64_t *sorted = lp_radix_sort(w.keys_a, w.keys_b, cap_e, 32, lp_bits_for((int64_t)out->cap[k - 1] + 1), w.hist, st, &status,
                                                   n_entries);
            LP_TRY(status);
            LP_TRY(lp_launch_row_offsets(sorted, cap_e, n_entries, out->cap[k - 1], 32, out->t_ptr[k - 1], st));
            hipLaunchKernelGGL(transposed_cols_kernel, dim3(ge), dim3(256), 0, st, sorted, ptr, n_k, cap_e, w.row_of_entry, out->t_col[k - 1]);
        } else {
            LP_TRY(lp_launch_zero(reinterpret_cast<float *>(out->t_ptr[k - 1]), (int64_t)out->cap[k - 1] + 1, st));
        }
        LP_TRY(lp_after_launch());
    }
    // 1/|N(v)| of every node of the computational graph (the GCN layers normalise with the full graph's degrees)
    if (out->cap[0] > 0) {
        hipLaunchKernelGGL(node_inv_deg_kernel, dim3((unsigned)lp_ceil_div(out->cap[0], 256)), dim3(256), 0, st, out->nodes, out->n, g->inv_deg,
                           out->node_inv_deg);
        LP_TRY(lp_after_launch());
    }
    return LP_OK;
}

extern "C" size_t lp_forward_blocks_workspace_bytes(const lp_model *m, const lp_blocks *b) {
    if (check_blocks(b, false) != LP_OK || check_block_model(m, b) != LP_OK) return 0;
    return transposed_weight_bytes(m);
}

extern "C" int lp_sage_forward_blocks(const lp_blocks *b, const lp_model *m, const void *X, void *X_frontier, lp_acts *saved,
                                      void *ws, size_t ws_bytes, void *stream) {
    LP_TRY(check_blocks(b, false));
    LP_TRY(check_block_model(m, b));
    if (!X || !lp_aligned16(X) || !X_frontier || !lp_aligned16(X_frontier) || !saved) return LP_ERR_INVALID_ARG;
    const int K = m->n_layers;
    for (int k = 0; k < K; ++k)
        if (!saved->A[k] || !saved->H[k] || !lp_aligned16(saved->A[k]) || !lp_aligned16(saved->H[k])) return LP_ERR_INVALID_ARG;
    if (!ws || ws_bytes < lp_forward_blocks_workspace_bytes(m, b)) return LP_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int dt = m->dtype;
    const size_t eb = (size_t)lp_elem_bytes(dt);
    char *wt = static_cast<char *>(ws);

    if (b->cap[0] > 0) {  // h^(0) of the outermost frontier: the feature rows of its nodes
        LpTimedScope timed(LP_KC_OTHER, st);
        const int FV = m->dims[0] / lp_vec_elems(dt);
        const unsigned grid = (unsigned)lp_ceil_div((int64_t)b->cap[0] * FV, 256);
        if (dt == LP_BF16)
            hipLaunchKernelGGL((gather_rows_kernel<lp_bf16_t>), dim3(grid), dim3(256), 0, st, static_cast<const lp_bf16_t *>(X), b->nodes, b->n,
                               FV, static_cast<lp_bf16_t *>(X_frontier));
        else
            hipLaunchKernelGGL((gather_rows_kernel<float>), dim3(grid), dim3(256), 0, st, static_cast<const float *>(X), b->nodes, b->n, FV,
                               static_cast<float *>(X_frontier));
        LP_TRY(lp_after_launch());
    }
    const void *Hprev = X_frontier;
    const bool gcn = m->layer_type == LP_LAYER_GCN;
    LP_TRY(lp_launch_transpose_weights(m, wt, st));   // every W^T, in one launch
    for (int k = 1; k <= K; ++k) {
        const int Fi = m->dims[k - 1], Fo = m->dims[k];
        SpmmArgs sp;
        sp.dtype = dt;
        sp.n_rows = b->cap[k]; sp.n_rows_dev = b->n + k;
        sp.F = Fi;
        sp.rowptr = b->ptr[k - 1]; sp.colidx = b->col[k - 1];
        if (gcn) {   // (d_v / |S(v)|) sum h_u / sqrt(d_v d_u), d = degrees of the graph the blocks were sampled from
            sp.inv_deg = b->node_inv_deg; sp.sym_norm = true; sp.sym_row_cnt = b->inv_cnt[k - 1];
        } else {
            sp.inv_deg = b->inv_cnt[k - 1];
        }
        sp.n_entries = b->cap_entries[k - 1];
        sp.in = Hprev; sp.out = saved->A[k - 1];
        LP_TRY(lp_launch_spmm(sp, st));
        const size_t wbytes = lp_align_up((size_t)Fi * Fo, 64) * eb;
        void *WsT = wt, *WnT = wt + wbytes;
        wt += 2 * wbytes;
        GemmNtArgs ge;
        ge.dtype = dt;
        ge.fp32_products = m->fp32_products;
        ge.M = b->cap[k]; ge.m_dev = b->n + k;
        ge.N = Fo; ge.n_split = Fo;
        ge.A[0] = Hprev; ge.A[1] = saved->A[k - 1];   // a frontier is a prefix of the one before: row i is node i in both
        ge.lda[0] = ge.lda[1] = Fi;
        ge.K[0] = gcn ? 0 : Fi; ge.K[1] = Fi;
        ge.Bt[0][0] = WsT; ge.Bt[1][0] = WnT;
        ge.ldb[0] = ge.ldb[1] = Fi;
        ge.bias = static_cast<const float *>(m->bias[k - 1]);
        ge.relu = k < K;
        ge.C[0] = saved->H[k - 1]; ge.ldc[0] = Fo;
        LP_TRY(lp_launch_gemm_nt(ge, st));
        Hprev = saved->H[k - 1];
    }
    return LP_OK;
}

extern "C" size_t lp_backward_blocks_workspace_bytes(const lp_model *m, const lp_blocks *b) {
    if (check_blocks(b, true) != LP_OK || check_block_model(m, b) != LP_OK) return 0;
    return carve_block_backward(nullptr, m, b).bytes;
}

namespace {
// dL/dH^K is seeded either from dscore (dot-product scorer) or from edge_grad (per-edge gradient rows of another
// scorer); exactly one of the two is given.
int backward_blocks_impl(const lp_blocks *b, const lp_model *m, const void *X_frontier, const lp_acts *saved, const float *dscore,
                         const void *edge_grad, lp_grads *out, void *ws, size_t ws_bytes, void *stream) {
    LP_TRY(check_blocks(b, true));
    LP_TRY(check_block_model(m, b));
    if (!X_frontier || !lp_aligned16(X_frontier) || !saved || !out) return LP_ERR_INVALID_ARG;
    const int K = m->n_layers;
    const int64_t B = b->n_edges;
    const bool gcn = m->layer_type == LP_LAYER_GCN;   // one weight matrix per layer: its gradient goes to dW_neigh
    if (B < 0 || (B > 0 && !dscore && !edge_grad)) return LP_ERR_INVALID_ARG;
    if (edge_grad && !lp_aligned16(edge_grad)) return LP_ERR_INVALID_ARG;
    for (int k = 0; k < K; ++k) {
        if (!saved->A[k] || !saved->H[k]) return LP_ERR_INVALID_ARG;
        if ((!gcn && !out->dW_self[k]) || !out->dW_neigh[k] || !out->dbias[k]) return LP_ERR_INVALID_ARG;
    }
    if (!ws || ws_bytes < lp_backward_blocks_workspace_bytes(m, b)) return LP_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int dt = m->dtype;
    if (B == 0 || b->cap[K] == 0) {  // an empty batch has a zero loss: every gradient is zero
        for (int k = 0; k < K; ++k) {
            const int64_t nw = (int64_t)m->dims[k] * m->dims[k + 1];
            if (!gcn) LP_TRY(lp_launch_zero(out->dW_self[k], nw, st));
            LP_TRY(lp_launch_zero(out->dW_neigh[k], nw, st));
            LP_TRY(lp_launch_zero(out->dbias[k], m->dims[k + 1], st));
        }
        return LP_OK;
    }
    const BlockBackwardWs w = carve_block_backward(ws, m, b);
    void *dZ = w.buf[0], *Q = w.buf[1], *R = w.buf[2];
    {   // dL/dH^K on frontier K: every position there is an end point of some scored edge
        {
            LpTimedScope timed(LP_KC_SCATTER, st);
            LP_TRY(lp_group_batch_by_row(b->e_src_pos, b->e_dst_pos, dscore, B, b->cap[K], w.group, w.bptr, w.bcol, w.bw, st));
        }
        SpmmArgs sc;
        sc.dtype = dt;
        sc.n_rows = b->cap[K]; sc.n_rows_dev = b->n + K; sc.F = m->dims[K];
        sc.rowptr = w.bptr; sc.colidx = w.bcol;
        if (dscore) sc.w = w.bw;
        else { sc.entry_rows = edge_grad; sc.entry_row_index = reinterpret_cast<const int32_t *>(w.bw); }
        sc.n_entries = 2 * B; sc.long_queue = w.long_queue;
        sc.in = saved->H[K - 1]; sc.out = dZ;
        sc.timing_class = LP_KC_SCATTER;
        LP_TRY(lp_launch_spmm(sc, st));
    }
    for (int k = K; k >= 1; --k) {
        const int Fi = m->dims[k - 1], Fo = m->dims[k];
        const void *Hin = k > 1 ? saved->H[k - 2] : X_frontier;
        const int32_t rows = b->cap[k];
        const int32_t *rows_dev = b->n + k;
        WeightGradArgs wg;
        wg.dtype = dt;
        wg.fp32_products = m->fp32_products;
        wg.Kn = rows; wg.kn_dev = rows_dev;
        if (!gcn) { wg.At[0] = Hin; wg.Mw[0] = Fi; wg.lda[0] = Fi; wg.C[0] = out->dW_self[k - 1]; }   // rows 0..n_k-1 of the wider frontier are the same nodes
        wg.At[1] = saved->A[k - 1]; wg.Mw[1] = Fi; wg.lda[1] = Fi; wg.C[1] = out->dW_neigh[k - 1];
        wg.B = dZ; wg.Nw = Fo; wg.ldb = Fo;
        wg.dbias = out->dbias[k - 1];
        wg.partials = w.tn_partials; wg.colsum_partials = w.colsum_partials;
        LP_TRY(lp_launch_weight_grads(wg, st));
        if (k == 1) break;
        GemmNtArgs ge;
        ge.dtype = dt;
        ge.fp32_products = m->fp32_products;
        ge.M = rows; ge.m_dev = rows_dev;
        ge.A[0] = dZ; ge.lda[0] = Fo; ge.K[0] = Fo;
        ge.ldb[0] = Fo;
        if (gcn) {   // dZ W^T -> R; the normalisation is applied by the aggregation that follows
            ge.N = Fi; ge.n_split = Fi;
            ge.Bt[0][0] = m->W_neigh[k - 1];
            ge.C[0] = R; ge.ldc[0] = Fi;
        } else {
            ge.N = 2 * Fi; ge.n_split = Fi;
            ge.Bt[0][0] = m->W_self[k - 1];
            ge.Bt[0][1] = m->W_neigh[k - 1];
            ge.rowscale = b->inv_cnt[k - 1];
            ge.C[0] = Q; ge.C[1] = R;
            ge.ldc[0] = ge.ldc[1] = Fi;
        }
        LP_TRY(lp_launch_gemm_nt(ge, st));
        // gradient on frontier k-1: the self path for its first n_k rows plus the transposed block, gated by the ReLU
        SpmmArgs sp;
        sp.dtype = dt;
        sp.n_rows = b->cap[k - 1]; sp.n_rows_dev = b->n + (k - 1); sp.F = Fi;
        sp.rowptr = b->t_ptr[k - 1]; sp.colidx = b->t_col[k - 1];
        sp.n_entries = b->cap_entries[k - 1]; sp.long_queue = w.long_queue;   // a popular node can be drawn by thousands of rows
        sp.in = R;
        if (gcn) {   // entry (u <- v) weighs (1/|S(v)|) / sqrt(1/d_v), row u is scaled by sqrt(1/d_u); no separate self path
            sp.inv_deg = b->node_inv_deg; sp.sym_norm = true; sp.sym_col_cnt = b->inv_cnt[k - 1];
        } else {
            sp.addend = Q; sp.addend_rows_dev = rows_dev;
        }
        sp.gate = Hin;
        sp.out = dZ;   // dZ of layer k is finished: its buffer takes the gradient of layer k-1
        LP_TRY(lp_launch_spmm(sp, st));
    }
    return LP_OK;
}
}  // namespace

extern "C" int lp_backward_blocks(const lp_blocks *b, const lp_model *m, const void *X_frontier, const lp_acts *saved,
                                  const float *dscore, lp_grads *out, void *ws, size_t ws_bytes, void *stream) {
    if (b && b->n_edges > 0 && !dscore) return LP_ERR_INVALID_ARG;
    return backward_blocks_impl(b, m, X_frontier, saved, dscore, nullptr, out, ws, ws_bytes, stream);
}

extern "C" int lp_backward_blocks_edge_grads(const lp_blocks *b, const lp_model *m, const void *X_frontier, const lp_acts *saved,
                                             const void *edge_grad, lp_grads *out, void *ws, size_t ws_bytes, void *stream) {
    if (b && b->n_edges > 0 && !edge_grad) return LP_ERR_INVALID_ARG;
    return backward_blocks_impl(b, m, X_frontier, saved, nullptr, edge_grad, out, ws, ws_bytes, stream);
}
