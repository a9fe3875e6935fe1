// lp_sage_forward, lp_sage_forward_edges and lp_backward: the K GraphSAGE-mean layers (Eq. 1 of the paper with the mean
// aggregator and two linear maps per layer) over every visible node, the same pass with the last layer evaluated only
// where the loss of a training step reads it (the end points of the scored edges), and the reverse walk through the
// layers (Algorithm 1, "Compute the gradient").  Host-side orchestration only; the work is done by the kernels in
// spmm_mean.hip and gemm_mfma.hip plus the small batch kernels below (end-point flags and list, row copies, the
// edge-gradient grouping).
#include "lp_internal.h"
#include "lp_scan.h"

namespace {

int check_model(const lp_model *m) {
    if (!m || m->n_layers < 1 || m->n_layers > LP_MAX_LAYERS) return LP_ERR_INVALID_ARG;
    if (m->dtype != LP_F32 && m->dtype != LP_BF16) return LP_ERR_UNSUPPORTED;
    if (m->layer_type != LP_LAYER_SAGE_MEAN && m->layer_type != LP_LAYER_GCN) return LP_ERR_UNSUPPORTED;
    if (!lp_valid_fp32_products(m->fp32_products) || m->reserved_ != 0) return LP_ERR_INVALID_ARG;
    const bool has_self = m->layer_type == LP_LAYER_SAGE_MEAN;
    for (int k = 0; k <= m->n_layers; ++k) {
        if (m->dims[k] <= 0) return LP_ERR_INVALID_ARG;
        if ((m->dims[k] % lp_vec_elems(m->dtype)) || m->dims[k] > 1024) return LP_ERR_UNSUPPORTED;
    }
    for (int k = 0; k < m->n_layers; ++k) {
        if ((has_self && !m->W_self[k]) || !m->W_neigh[k] || !m->bias[k]) return LP_ERR_INVALID_ARG;
        if ((has_self && !lp_aligned16(m->W_self[k])) || !lp_aligned16(m->W_neigh[k])) return LP_ERR_INVALID_ARG;
    }
    return LP_OK;
}

int check_graph(const lp_csr *g, bool need_transpose) {
    if (!g || g->n_nodes <= 0 || g->nnz < 0 || !g->rowptr || !g->inv_deg) return LP_ERR_INVALID_ARG;
    if (g->nnz >= ((int64_t)1 << 31)) return LP_ERR_OUT_OF_RANGE;
    if (g->nnz > 0 && !g->colidx) return LP_ERR_INVALID_ARG;
    if (need_transpose && (!g->t_rowptr || (g->nnz > 0 && !g->t_colidx))) return LP_ERR_INVALID_ARG;
    return LP_OK;
}

int check_acts(const lp_model *m, const lp_acts *a) {
    if (!a) return LP_ERR_INVALID_ARG;
    for (int k = 0; k < m->n_layers; ++k)
        if (!a->A[k] || !a->H[k] || !lp_aligned16(a->A[k]) || !lp_aligned16(a->H[k])) return LP_ERR_INVALID_ARG;
    return LP_OK;
}

size_t transposed_weight_elems(const lp_model *m) {
    size_t n = 0;
    for (int k = 0; k < m->n_layers; ++k) n += 2 * lp_align_up((size_t)m->dims[k] * m->dims[k + 1], 64);
    return n;
}

int max_dim(const lp_model *m) {
    int d = 0;
    for (int k = 0; k <= m->n_layers; ++k) d = m->dims[k] > d ? m->dims[k] : d;
    return d;
}

// dL/dH^K: every scored edge (u, v) with weight g = dL/ds adds g*h_v to row u and g*h_u to row v.
// Instead of atomic adds, the 2B (node, other endpoint, g) entries are grouped by node with a stable radix
// sort and each row is then summed by one wavefront in a fixed order: the result does not depend on scheduling,
// and rows no edge touches are written as zeros by the same pass.
__global__ void batch_keys_kernel(const int32_t *__restrict__ e_src, const int32_t *__restrict__ e_dst, int64_t B,
                                  int32_t n_nodes, uint64_t *__restrict__ keys) {
    const int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= 2 * B) return;
    const int64_t e = j < B ? j : j - B;
    const int32_t u = e_src[e], v = e_dst[e];
    const bool ok = u >= 0 && u < n_nodes && v >= 0 && v < n_nodes;
    const int32_t node = ok ? (j < B ? u : v) : n_nodes;  // edges with a bad id are parked behind the last row
    keys[j] = ((uint64_t)(uint32_t)node << 32) | (uint32_t)j;
}

__global__ void batch_entries_kernel(const uint64_t *__restrict__ sorted, int64_t B, const int32_t *__restrict__ e_src,
                                     const int32_t *__restrict__ e_dst, const float *__restrict__ dscore, int32_t n_nodes,
                                     int32_t *__restrict__ col, float *__restrict__ w) {
    const int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= 2 * B) return;
    const uint64_t k = sorted[p];
    const int64_t j = (int64_t)(uint32_t)k;
    const int64_t e = j < B ? j : j - B;
    const bool parked = (int32_t)(k >> 32) >= n_nodes;
    col[p] = parked ? 0 : (j < B ? e_dst[e] : e_src[e]);
    if (dscore) w[p] = parked ? 0.f : dscore[e];
    else reinterpret_cast<int32_t *>(w)[p] = (int32_t)e;   // which scored edge the entry belongs to
}

// ---- the training forward pass evaluates its last layer only for the end points of the scored edges
// flag[v] = 1 for every node that is an end point of a scored edge (ids outside the graph are skipped); racing
// stores all write the same value
__global__ void mark_endpoints_kernel(const int32_t *__restrict__ e_src, const int32_t *__restrict__ e_dst, int64_t B,
                                      int32_t n_nodes, uint32_t *__restrict__ flag) {
    const int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= 2 * B) return;
    const int64_t e = j < B ? j : j - B;
    const int32_t u = e_src[e], v = e_dst[e];
    if (u < 0 || u >= n_nodes || v < 0 || v >= n_nodes) return;
    flag[j < B ? u : v] = 1u;
}

// 16-byte vectors of rows: dst[r] = src[list[r]] (GATHER) or dst[list[r]] = src[r], for r < *n_listed; up to two
// matrices with the same row length in one launch
template <bool GATHER>
__global__ void copy_listed_rows_kernel(const int32_t *__restrict__ list, const int32_t *__restrict__ n_listed, int32_t cap,
                                        int32_t row_vecs, const uint4 *__restrict__ src0, uint4 *__restrict__ dst0,
                                        const uint4 *__restrict__ src1, uint4 *__restrict__ dst1) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t r = i / row_vecs;
    const int32_t c = (int32_t)(i - r * row_vecs);
    const int32_t n = *n_listed < cap ? *n_listed : cap;
    if (r >= n) return;
    const int64_t v = list[r];
    const int64_t from = (GATHER ? v : r) * row_vecs + c, to = (GATHER ? r : v) * row_vecs + c;
    if (src0) dst0[to] = src0[from];
    if (src1) dst1[to] = src1[from];
}

struct ForwardWs {
    char *wt;                 // transposed weights
    int32_t *long_queue;
    uint32_t *flag;           // [n_nodes]
    int32_t *list, *n_listed; // end points of the scored edges, ascending; their number
    uint32_t *scan_ws;
    void *rows[3];            // [cap, widest layer] each: gathered h^(K-1) rows, gathered aggregates, h^(K) rows
    size_t bytes;
};

struct BackwardWs {
    void *buf[3];  // [n_nodes, max width] in the model's storage type
    float *tn_partials;
    float *colsum_partials;
    uint64_t *keys_a, *keys_b;
    uint32_t *hist;
    int32_t *bptr, *bcol;
    float *bw;
    int32_t *long_queue;
    int32_t *touched, *touched_index, *touched_ptr, *n_touched;  // rows of dL/dH^K that receive anything
    void *compact_ws;
    size_t bytes;
};

// At most this many nodes can be an endpoint of one of B scored edges.
int32_t touched_cap(int32_t n_nodes, int64_t B) {
    const int64_t two_b = 2 * (B > 0 ? B : 0);
    return (int32_t)(two_b < n_nodes ? two_b : n_nodes);
}

BackwardWs carve_backward(void *ws, const lp_model *m, int32_t n_nodes, int64_t B) {
    char *p = static_cast<char *>(ws);
    size_t off = 0;
    auto take = [&](size_t bytes) { char *q = p ? p + off : nullptr; off += lp_align_up(bytes); return reinterpret_cast<float *>(q); };
    BackwardWs w;
    const size_t big = (size_t)lp_elem_bytes(m->dtype) * (size_t)n_nodes * (size_t)max_dim(m);
    for (int i = 0; i < 3; ++i) w.buf[i] = take(big);
    size_t tn = 0, cs = 0;
    for (int k = 0; k < m->n_layers; ++k) {
        size_t t = lp_weight_grads_partials_bytes(m->dtype, n_nodes, m->layer_type == LP_LAYER_GCN ? 0 : m->dims[k], m->dims[k], m->dims[k + 1]);
        tn = t > tn ? t : tn;
        size_t c = lp_colsum_partials_bytes(n_nodes, m->dims[k + 1]);
        cs = c > cs ? c : cs;
    }
    w.tn_partials = take(tn);
    w.colsum_partials = take(cs);
    const size_t n2 = (size_t)(2 * (B > 0 ? B : 0) + 1);
    w.keys_a = reinterpret_cast<uint64_t *>(take(sizeof(uint64_t) * n2));
    w.keys_b = reinterpret_cast<uint64_t *>(take(sizeof(uint64_t) * n2));
    w.hist = reinterpret_cast<uint32_t *>(take(sizeof(uint32_t) * lp_radix_sort_hist_words((int64_t)n2)));
    w.bptr = reinterpret_cast<int32_t *>(take(sizeof(int32_t) * ((size_t)n_nodes + 1)));
    w.bcol = reinterpret_cast<int32_t *>(take(sizeof(int32_t) * n2));
    w.bw = take(sizeof(float) * n2);
    w.long_queue = reinterpret_cast<int32_t *>(take(lp_spmm_queue_bytes(n_nodes, max_dim(m))));
    const size_t cap = (size_t)touched_cap(n_nodes, B);
    w.touched = reinterpret_cast<int32_t *>(take(sizeof(int32_t) * (cap + 1)));
    w.touched_index = reinterpret_cast<int32_t *>(take(sizeof(int32_t) * (size_t)n_nodes));
    w.touched_ptr = reinterpret_cast<int32_t *>(take(sizeof(int32_t) * (cap + 1)));
    w.n_touched = reinterpret_cast<int32_t *>(take(256));
    w.compact_ws = take(lp_compact_rows_ws_bytes(n_nodes));
    w.bytes = off;
    return w;
}


// Whether the training forward lists the rows of its last layer.  Listing pays when the batch touches a small part of
// the graph; near 2B = N the list building and the row copies cost what the rows left out save (measured change of the
// step: -10 % at 2B = 0.18 N, -4 % at 0.73 N, 0 at 0.98 N, +2 % at 1.1 N and 1.2 N), so from 2B = 0.75 N on every
// node is evaluated.  B < 0: the plain forward pass.
bool lists_rows(int32_t n_nodes, int64_t B) { return B >= 0 && 8 * B < 3 * (int64_t)n_nodes; }

ForwardWs carve_forward(void *ws, const lp_model *m, int32_t n_nodes, int64_t B) {
    char *p = static_cast<char *>(ws);
    size_t off = 0;
    auto take = [&](size_t bytes) { char *q = p ? p + off : nullptr; off += lp_align_up(bytes); return q; };
    ForwardWs w{};
    w.wt = take((size_t)lp_elem_bytes(m->dtype) * transposed_weight_elems(m));
    w.long_queue = reinterpret_cast<int32_t *>(take(lp_spmm_queue_bytes(n_nodes, max_dim(m))));
    if (lists_rows(n_nodes, B)) {
        const size_t cap = (size_t)touched_cap(n_nodes, B);
        w.flag = reinterpret_cast<uint32_t *>(take(sizeof(uint32_t) * (size_t)n_nodes));
        w.list = reinterpret_cast<int32_t *>(take(sizeof(int32_t) * (cap + 1)));
        w.n_listed = reinterpret_cast<int32_t *>(take(256));
        w.scan_ws = reinterpret_cast<uint32_t *>(take(sizeof(uint32_t) * lp_scan::block_sum_count(n_nodes)));
        for (int i = 0; i < 3; ++i) w.rows[i] = take((size_t)lp_elem_bytes(m->dtype) * cap * (size_t)max_dim(m));
    }
    w.bytes = off;
    return w;
}

}  // namespace

int lp_group_batch_by_row(const int32_t *e_src, const int32_t *e_dst, const float *dscore, int64_t B, int32_t n_rows,
                          const BatchGroupWs &ws, int32_t *ptr, int32_t *col, float *w, hipStream_t st) {
    const int64_t n2 = 2 * B;
    const unsigned g2 = (unsigned)lp_ceil_div(n2, 256);
    hipLaunchKernelGGL(batch_keys_kernel, dim3(g2), dim3(256), 0, st, e_src, e_dst, B, n_rows, ws.keys_a);
    int status;
    const uint64_t *sorted = lp_radix_sort(ws.keys_a, ws.keys_b, n2, 32, lp_bits_for((int64_t)n_rows + 1), ws.hist, st, &status);
    LP_TRY(status);
    LP_TRY(lp_launch_row_offsets(sorted, n2, nullptr, n_rows, 32, ptr, st));
    hipLaunchKernelGGL(batch_entries_kernel, dim3(g2), dim3(256), 0, st, sorted, B, e_src, e_dst, dscore, n_rows, col, w);
    return lp_after_launch();
}

// One layer of the forward pass.  rows == nullptr: every node.  Otherwise only the nodes list[0 .. *n_listed) (at most
// cap of them): their aggregates and outputs land in the same rows of A and H as in the full pass, all other rows of
// A and H are left alone; the dense product runs on gathered copies of the listed rows.
static int forward_layer(const lp_csr *g, const lp_model *m, int k, const void *Hprev, void *A, void *H, const void *WsT,
                         const void *WnT, const ForwardWs &w, bool listed, int32_t cap, hipStream_t st) {
    const int K = m->n_layers, dt = m->dtype;
    const bool gcn = m->layer_type == LP_LAYER_GCN;
    const int Fi = m->dims[k - 1], Fo = m->dims[k];
    SpmmArgs sp;
    sp.dtype = dt;
    sp.n_rows = listed ? cap : g->n_nodes;
    sp.n_rows_dev = listed ? w.n_listed : nullptr;
    sp.F = Fi;
    sp.rowptr = g->rowptr;
    sp.colidx = g->colidx;
    sp.row_order = listed ? w.list : g->row_order;
    sp.inv_deg = g->inv_deg;
    sp.sym_norm = gcn;   // 1/sqrt(d_v d_u) per entry instead of 1/d_v per row
    sp.n_entries = g->nnz;
    sp.long_queue = w.long_queue;
    sp.in = Hprev;
    sp.out = A;
    LP_TRY(lp_launch_spmm(sp, st));
    const void *Hin = Hprev, *Ain = A;
    void *Hout = H;
    if (listed) {
        LpTimedScope timed(LP_KC_SCATTER, st);
        const int32_t vecs = Fi * lp_elem_bytes(dt) / 16;
        hipLaunchKernelGGL((copy_listed_rows_kernel<true>), dim3((unsigned)lp_ceil_div((int64_t)cap * vecs, 256)), dim3(256), 0, st,
                           w.list, w.n_listed, cap, vecs, gcn ? nullptr : static_cast<const uint4 *>(Hprev),
                           static_cast<uint4 *>(w.rows[0]), static_cast<const uint4 *>(A), static_cast<uint4 *>(w.rows[1]));
        LP_TRY(lp_after_launch());
        Hin = w.rows[0]; Ain = w.rows[1]; Hout = w.rows[2];
    }
    GemmNtArgs ge;
    ge.dtype = dt;
    ge.fp32_products = m->fp32_products;
    ge.M = listed ? cap : g->n_nodes;
    ge.m_dev = listed ? w.n_listed : nullptr;
    ge.N = Fo;
    ge.n_split = Fo;
    ge.A[0] = Hin; ge.A[1] = Ain;
    ge.lda[0] = ge.lda[1] = Fi;
    ge.K[0] = gcn ? 0 : Fi;   // no self path in a GCN layer
    ge.K[1] = Fi;
    ge.Bt[0][0] = WsT; ge.Bt[1][0] = WnT;
    ge.ldb[0] = ge.ldb[1] = Fi;
    ge.bias = static_cast<const float *>(m->bias[k - 1]);
    ge.relu = k < K;
    ge.C[0] = Hout;
    ge.ldc[0] = Fo;
    LP_TRY(lp_launch_gemm_nt(ge, st));
    if (listed) {
        LpTimedScope timed(LP_KC_SCATTER, st);
        const int32_t vecs = Fo * lp_elem_bytes(dt) / 16;
        hipLaunchKernelGGL((copy_listed_rows_kernel<false>), dim3((unsigned)lp_ceil_div((int64_t)cap * vecs, 256)), dim3(256), 0, st,
                           w.list, w.n_listed, cap, vecs, static_cast<const uint4 *>(Hout), static_cast<uint4 *>(H),
                           static_cast<const uint4 *>(nullptr), static_cast<uint4 *>(nullptr));
        LP_TRY(lp_after_launch());
    }
    return LP_OK;
}

// B < 0: every layer for every node.  B >= 0: the last layer only for the end points of the B scored edges, if
// those can only be a small part of the nodes.
static int forward_impl(const lp_csr *g, const lp_model *m, const void *X, int64_t B, const int32_t *e_src, const int32_t *e_dst,
                        lp_acts *saved, void *ws, size_t ws_bytes, void *stream) {
    LP_TRY(check_model(m));
    LP_TRY(check_graph(g, false));
    LP_TRY(check_acts(m, saved));
    if (!X || !lp_aligned16(X)) return LP_ERR_INVALID_ARG;
    if (B > 0 && (!e_src || !e_dst)) return LP_ERR_INVALID_ARG;
    if (B >= ((int64_t)1 << 31)) return LP_ERR_OUT_OF_RANGE;
    if (!ws || ws_bytes < carve_forward(nullptr, m, g->n_nodes, B).bytes) return LP_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const ForwardWs w = carve_forward(ws, m, g->n_nodes, B);
    const size_t eb = (size_t)lp_elem_bytes(m->dtype);
    const int K = m->n_layers;
    const int32_t N = g->n_nodes;
    const bool list_rows = lists_rows(N, B);
    const int32_t cap = list_rows ? touched_cap(N, B) : 0;
    // the NT products want the reduction index contiguous: every W^T ([Fo, Fi]) is written up front, in one launch
    LP_TRY(lp_launch_transpose_weights(m, w.wt, st));
    if (cap > 0) {   // the end points of the scored edges, ascending: flags, then a prefix sum over the flags
        LpTimedScope timed(LP_KC_SCATTER, st);
        LP_TRY(lp_launch_zero(reinterpret_cast<float *>(w.flag), N, st));
        hipLaunchKernelGGL(mark_endpoints_kernel, dim3((unsigned)lp_ceil_div(2 * B, 256)), dim3(256), 0, st, e_src, e_dst, B, N, w.flag);
        LP_TRY(lp_after_launch());
        const uint32_t *flag = w.flag;
        int32_t *list = w.list;
        auto is_end = [flag] __device__(int64_t v) { return flag[v]; };
        auto emit = [list] __device__(int64_t v, uint32_t pos, uint32_t f) { if (f) list[pos] = (int32_t)v; };
        LP_TRY(lp_scan::device_exclusive_scan<uint32_t>(is_end, emit, (int64_t)N, w.scan_ws, reinterpret_cast<uint32_t *>(w.n_listed), st));
    }
    const void *Hprev = X;
    char *wt = w.wt;
    for (int k = 1; k <= K; ++k) {
        const size_t wbytes = lp_align_up((size_t)m->dims[k - 1] * m->dims[k], 64) * eb;
        const bool listed = list_rows && k == K;
        if (!listed || cap > 0)
            LP_TRY(forward_layer(g, m, k, Hprev, saved->A[k - 1], saved->H[k - 1], wt, wt + wbytes, w, listed, cap, st));
        wt += 2 * wbytes;
        Hprev = saved->H[k - 1];
    }
    return LP_OK;
}

extern "C" size_t lp_sage_forward_workspace_bytes(const lp_model *m, int32_t n_nodes) {
    if (check_model(m) != LP_OK || n_nodes <= 0) return 0;
    return carve_forward(nullptr, m, n_nodes, -1).bytes;
}

extern "C" int lp_sage_forward(const lp_csr *g, const lp_model *m, const void *X, lp_acts *saved, void *ws, size_t ws_bytes,
                               void *stream) {
    return forward_impl(g, m, X, -1, nullptr, nullptr, saved, ws, ws_bytes, stream);
}

extern "C" size_t lp_sage_forward_edges_workspace_bytes(const lp_model *m, int32_t n_nodes, int64_t B) {
    if (check_model(m) != LP_OK || n_nodes <= 0 || B < 0 || B >= ((int64_t)1 << 31)) return 0;
    return carve_forward(nullptr, m, n_nodes, B).bytes;
}

extern "C" int lp_sage_forward_edges(const lp_csr *g, const lp_model *m, const void *X, int64_t B, const int32_t *e_src,
                                     const int32_t *e_dst, lp_acts *saved, void *ws, size_t ws_bytes, void *stream) {
    if (B < 0) return LP_ERR_INVALID_ARG;
    return forward_impl(g, m, X, B, e_src, e_dst, saved, ws, ws_bytes, stream);
}

extern "C" size_t lp_backward_workspace_bytes(const lp_model *m, int32_t n_nodes, int64_t B) {
    if (check_model(m) != LP_OK || n_nodes <= 0 || B < 0) return 0;
    return carve_backward(nullptr, m, n_nodes, B).bytes;
}

// dscore (one scalar per scored edge, dot-product scorer) or edge_grad (one row dL/d(h_u * h_v) per scored edge,
// any scorer that works on the element-wise product) seeds dL/dH^K; everything after that is common.
static int backward_impl(const lp_csr *g, const lp_model *m, const void *X, const lp_acts *saved, int64_t B,
                         const int32_t *e_src, const int32_t *e_dst, const float *dscore, const void *edge_grad, lp_grads *out,
                         void *ws, size_t ws_bytes, void *stream) {
    LP_TRY(check_model(m));
    LP_TRY(check_graph(g, true));
    LP_TRY(check_acts(m, saved));
    if (!X || !lp_aligned16(X) || !out || B < 0) return LP_ERR_INVALID_ARG;
    if (B > 0 && (!e_src || !e_dst || (!dscore && !edge_grad))) return LP_ERR_INVALID_ARG;
    if (edge_grad && !lp_aligned16(edge_grad)) return LP_ERR_INVALID_ARG;
    if (B >= ((int64_t)1 << 31)) return LP_ERR_OUT_OF_RANGE;
    const int K = m->n_layers;
    const bool gcn = m->layer_type == LP_LAYER_GCN;
    for (int k = 0; k < K; ++k)
        if ((!gcn && !out->dW_self[k]) || !out->dW_neigh[k] || !out->dbias[k]) return LP_ERR_INVALID_ARG;
    if (out->dX && !lp_aligned16(out->dX)) return LP_ERR_INVALID_ARG;
    if (!ws || ws_bytes < lp_backward_workspace_bytes(m, g->n_nodes, B)) return LP_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    BackwardWs w = carve_backward(ws, m, g->n_nodes, B);
    const int32_t N = g->n_nodes;

    const int dt = m->dtype;
    void *dZ = w.buf[0], *Q = w.buf[1], *R = w.buf[2];
    const void *HK = saved->H[K - 1];
    if (B == 0) {  // an empty batch has a zero loss: every gradient is zero
        for (int k = 0; k < K; ++k) {
            const int64_t nw = (int64_t)m->dims[k] * m->dims[k + 1];
            if (!gcn) LP_TRY(lp_launch_zero(out->dW_self[k], nw, st));
            LP_TRY(lp_launch_zero(out->dW_neigh[k], nw, st));
            LP_TRY(lp_launch_zero(out->dbias[k], m->dims[k + 1], st));
        }
        if (out->dX) LP_TRY(lp_launch_zero(static_cast<float *>(out->dX), (int64_t)N * m->dims[0] * lp_elem_bytes(dt) / 4, st));
        return LP_OK;
    }

    // dL/dH^K is non-zero only on rows that are an endpoint of a scored edge.  Those rows are listed (ascending) and
    // the whole last layer works on that list: its gradient matrix, both weight-gradient products and the input-
    // gradient product have one row per listed node, and only the aggregation that follows widens back to all nodes.
    const int32_t cap = touched_cap(N, B);
    {
        const int64_t n2 = 2 * B;
        {
            LpTimedScope timed(LP_KC_SCATTER, st);
            BatchGroupWs gw{w.keys_a, w.keys_b, w.hist};
            LP_TRY(lp_group_batch_by_row(e_src, e_dst, dscore, B, N, gw, w.bptr, w.bcol, w.bw, st));
            LP_TRY(lp_launch_compact_rows(w.bptr, N, w.touched, w.touched_index, w.touched_ptr, w.n_touched, w.compact_ws, st));
        }
        SpmmArgs sc;
        sc.dtype = dt;
        sc.n_rows = cap; sc.n_rows_dev = w.n_touched; sc.F = m->dims[K];
        sc.rowptr = w.touched_ptr; sc.colidx = w.bcol;
        if (dscore) sc.w = w.bw;
        else { sc.entry_rows = edge_grad; sc.entry_row_index = reinterpret_cast<const int32_t *>(w.bw); }
        sc.n_entries = n2; sc.long_queue = w.long_queue;
        sc.in = HK; sc.out = dZ;
        sc.timing_class = LP_KC_SCATTER;
        LP_TRY(lp_launch_spmm(sc, st));
    }

    for (int k = K; k >= 1; --k) {
        const int Fi = m->dims[k - 1], Fo = m->dims[k];
        const void *Hin = k > 1 ? saved->H[k - 2] : X;
        const void *Ak = saved->A[k - 1];
        const bool listed = k == K;               // dZ holds one row per listed node instead of one per node
        const int32_t rows = listed ? cap : N;    // host-side bound; the exact count is read on the device
        const int32_t *rows_dev = listed ? w.n_touched : nullptr;
        const int32_t *row_of = listed ? w.touched : nullptr;
        WeightGradArgs wg;
        wg.dtype = dt;
        wg.fp32_products = m->fp32_products;
        wg.Kn = rows; wg.kn_dev = rows_dev; wg.at_index = row_of;
        if (!gcn) { wg.At[0] = Hin; wg.Mw[0] = Fi; wg.lda[0] = Fi; wg.C[0] = out->dW_self[k - 1]; }
        wg.At[1] = Ak; wg.Mw[1] = Fi; wg.lda[1] = Fi; wg.C[1] = out->dW_neigh[k - 1];
        wg.B = dZ; wg.Nw = Fo; wg.ldb = Fo;
        wg.dbias = out->dbias[k - 1];
        wg.partials = w.tn_partials; wg.colsum_partials = w.colsum_partials;
        LP_TRY(lp_launch_weight_grads(wg, st));
        if (k == 1 && !out->dX) break;
        // Input gradient G^{k-1} = gate . (dZ W_self^T + M^T(dZ W_neigh^T)), M^T the adjoint of the mean.  The adjoint
        // commutes with the linear map, so where the layer does not widen the aggregation (F_k <= F_{k-1}) and dZ has a
        // row per node, dZ is aggregated FIRST (entries weighted by the 1/deg of their source row) and ONE product
        // [dZ | M^T dZ] [W_self^T ; W_neigh^T] follows, gated in its epilogue: nothing like Q and R below is written and
        // read back, and the aggregation reads no addend and no gate rows (fp32 storage; the bf16 path keeps the
        // order whose stored matrices its parity bound is stated for).
        if (!gcn && !listed && dt == LP_F32 && Fo <= Fi && k > 1) {
            SpmmArgs sp;
            sp.dtype = dt;
            sp.n_rows = N; sp.F = Fo;
            sp.rowptr = g->t_rowptr; sp.colidx = g->t_colidx; sp.row_order = g->t_row_order;
            sp.n_entries = g->nnz; sp.long_queue = w.long_queue;
            if (g->t_entry_scale) sp.w = g->t_entry_scale;   // in entry order: no scattered 4-byte read per entry
            else sp.col_w = g->inv_deg;
            sp.in = dZ; sp.out = R;
            LP_TRY(lp_launch_spmm(sp, st));
            GemmNtArgs ge;
            ge.dtype = dt;
            ge.fp32_products = m->fp32_products;
            ge.M = N;
            ge.N = Fi; ge.n_split = Fi;
            ge.A[0] = dZ; ge.A[1] = R;
            ge.lda[0] = ge.lda[1] = Fo;
            ge.K[0] = ge.K[1] = Fo;
            ge.Bt[0][0] = m->W_self[k - 1]; ge.Bt[1][0] = m->W_neigh[k - 1];
            ge.ldb[0] = ge.ldb[1] = Fo;
            ge.C[0] = Q; ge.ldc[0] = Fi;
            ge.gate = static_cast<const float *>(Hin); ge.ldgate = Fi;
            LP_TRY(lp_launch_gemm_nt(ge, st));
            void *t = dZ; dZ = Q; Q = t;
            continue;
        }
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
        } else {     // [dZ W_self^T | diag(inv_deg) dZ W_neigh^T] -> Q, R
            ge.N = 2 * Fi; ge.n_split = Fi;
            ge.Bt[0][0] = m->W_self[k - 1];
            ge.Bt[0][1] = m->W_neigh[k - 1];
            ge.rowscale = g->inv_deg; ge.rowscale_index = row_of;
            ge.C[0] = Q; ge.C[1] = R;
            ge.ldc[0] = ge.ldc[1] = Fi;
        }
        LP_TRY(lp_launch_gemm_nt(ge, st));
        // G^{k-1} = (Q + sum over the transposed CSR of R) gated by relu'(z^{k-1}) = [h^{k-1} > 0]
        SpmmArgs sp;
        sp.dtype = dt;
        sp.n_rows = N; sp.F = Fi;
        sp.rowptr = g->t_rowptr; sp.colidx = g->t_colidx; sp.row_order = g->t_row_order;
        sp.n_entries = g->nnz; sp.long_queue = w.long_queue;
        sp.in = R; sp.addend = gcn ? nullptr : Q;
        if (gcn) { sp.inv_deg = g->inv_deg; sp.sym_norm = true; }
        sp.in_index = listed ? w.touched_index : nullptr;
        sp.gate = k > 1 ? Hin : nullptr;
        if (listed) {
            // Q and R hold listed rows only; the result has every row and replaces the (finished) listed dZ
            sp.out = k > 1 ? dZ : static_cast<void *>(out->dX);
            LP_TRY(lp_launch_spmm(sp, st));
        } else {
            sp.out = k > 1 ? Q : static_cast<void *>(out->dX);
            LP_TRY(lp_launch_spmm(sp, st));
            void *t = dZ; dZ = Q; Q = t;
        }
    }
    return LP_OK;
}

extern "C" int lp_backward(const lp_csr *g, const lp_model *m, const void *X, const lp_acts *saved, int64_t B,
                           const int32_t *e_src, const int32_t *e_dst, const float *dscore, lp_grads *out, void *ws,
                           size_t ws_bytes, void *stream) {
    if (B > 0 && !dscore) return LP_ERR_INVALID_ARG;
    return backward_impl(g, m, X, saved, B, e_src, e_dst, dscore, nullptr, out, ws, ws_bytes, stream);
}

extern "C" int lp_backward_edge_grads(const lp_csr *g, const lp_model *m, const void *X, const lp_acts *saved, int64_t B,
                                      const int32_t *e_src, const int32_t *e_dst, const void *edge_grad, lp_grads *out, void *ws,
                                      size_t ws_bytes, void *stream) {
    if (B > 0 && !edge_grad) return LP_ERR_INVALID_ARG;
    return backward_impl(g, m, X, saved, B, e_src, e_dst, nullptr, edge_grad, out, ws, ws_bytes, stream);
}
