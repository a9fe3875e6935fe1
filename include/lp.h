/*
 * lp.h - C ABI of the MI355X (gfx950) link-prediction training-step library.
 *
 * One worker's training step of distributed GNN link prediction (the body of
 * the per-worker loop in the paper's Algorithm 1, "Distributed Model
 * Training"): K GraphSAGE-mean layers over the worker's visible graph
 * (Eq. 1), per-source uniform negative sampling (Sec. II-B), dot-product edge
 * scores (Eq. 2), binary cross-entropy averaged over the batch (Sec. IV-B,
 * last paragraph), and the gradient of that loss with respect to every model
 * weight.
 *
 * Conventions shared by every call
 * --------------------------------
 *  - Every pointer marked "device" is HIP device memory of the current device,
 *    allocated and owned by the caller.  The library never allocates, frees or
 *    keeps device memory: outputs and scratch space ("ws") come from the
 *    caller, and the size of the scratch space is given by the matching
 *    *_workspace_bytes() function, which is pure host arithmetic.
 *  - Matrices are row-major and node-major: row v of a [N, F] matrix is the
 *    vector of node v.  Feature, activation and weight pointers must be
 *    16-byte aligned and every layer width must be a multiple of 4 (of 8 with
 *    LP_BF16, where those matrices hold bfloat16 and everything is still
 *    accumulated in fp32; biases, scores, loss and gradients stay fp32).
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    Work is enqueued on it and, except for lp_build_csr, the call returns
 *    without waiting.
 *  - Apart from the benchmark instrumentation at the end of this file (and
 *    the fixed scratch array of lp_score_loss_noalloc) the library keeps no
 *    state between calls.
 *  - Return value: LP_OK or a negative LP_ERR_* code.  Arguments are checked on
 *    the host before anything is launched; a call that returns an error other
 *    than LP_ERR_HIP has launched nothing.  No exception crosses this ABI.
 *  - Node ids, row pointers and column indices are int32; the number of
 *    directed entries (nnz) must stay below 2^31.
 */
#ifndef LP_H_
#define LP_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define LP_MAX_LAYERS 8
#define LP_MAX_MLP_LAYERS 4 /* linear layers of the MLP edge predictor */
#define LP_MAX_FANOUT 64 /* most neighbours one node may draw per hop in lp_sample_blocks */
#define LP_FANOUT_ALL 0  /* fan-out value that stands for "all neighbours" (no draw) */

enum {
    LP_OK = 0,
    LP_ERR_INVALID_ARG = -1,  /* null pointer, negative size, misaligned matrix, bad layer count */
    LP_ERR_OUT_OF_RANGE = -2, /* node id outside [0, n_nodes), or sizes beyond int32 indexing */
    LP_ERR_WORKSPACE = -3,    /* ws is NULL or smaller than *_workspace_bytes() */
    LP_ERR_UNSUPPORTED = -4,  /* unknown dtype, or a width that is not a multiple of 4 (8 for LP_BF16) */
    LP_ERR_HIP = -5           /* the HIP runtime reported an error (no device, failed launch) */
};

enum {
    LP_F32 = 0, /* fp32 storage */
    LP_BF16 = 1 /* bfloat16 storage (features, weights, activations), fp32 accumulation, fp32 gradients */
};

/* How the dense products of an fp32 model are formed (Eq. 1's UPDATE and its
 * gradients; the paper fixes no arithmetic): the `fp32_products` field of
 * lp_model and lp_mlp, a property of each call.  Storage, accumulation and every
 * result are fp32 in both modes; models with bf16 storage ignore the field.
 *   LP_FP32_PRODUCTS_NATIVE (0, what a zero-initialised struct selects): the
 *     fp32 matrix instructions; IEEE behaviour for every input.
 *   LP_FP32_PRODUCTS_BF16X6: each fp32 operand value is written as the exact sum
 *     of three bfloat16 terms and a product is taken as the six largest of the
 *     nine term products on the bf16 matrix cores, accumulated in fp32.  What is
 *     left out is below 2^-26 of each product, a quarter of one fp32 rounding;
 *     measured against fp64 the results are as close as those of the fp32
 *     matrix instructions, at 6/16 of their issue time.  Contract of this mode:
 *     every finite fp32 input is split exactly (magnitudes in the last half
 *     bfloat16 step below the fp32 maximum included); a non-finite input makes
 *     every result that depends on it non-finite (NaN where the fp32
 *     instructions might give an infinity); term products below the smallest
 *     normal fp32 (1.2e-38) are flushed to zero, so products smaller than about
 *     1e-33 lose the accuracy of their small terms.  Products whose shape the
 *     bf16-term kernels do not take (an inner dimension that is not a multiple
 *     of 16, outputs narrower than 65 columns, fused weight gradients below
 *     192 x 192) use the fp32 matrix instructions in this mode too.
 * Another value is rejected with LP_ERR_INVALID_ARG by every call that takes the
 * struct. */
#define LP_FP32_PRODUCTS_NATIVE 0
#define LP_FP32_PRODUCTS_BF16X6 1

/* layer types of lp_model */
enum {
    LP_LAYER_SAGE_MEAN = 0, /* z_v = h_v W_self + mean_{u in N(v)} h_u W_neigh + b */
    LP_LAYER_GCN = 1        /* z_v = sum_{u in N(v)} h_u / sqrt(|N(v)| |N(u)|) W_neigh + b; W_self is not used */
};

/* flags of lp_build_csr */
#define LP_SYMMETRIZE 1u /* every input pair (r, c) also counts as (c, r) */

/* Visible graph of one worker in canonical CSR form, plus its transpose.
 * Row v lists N(v), the nodes v aggregates from (Eq. 1), ascending and without
 * repeats.  Row u of the transposed CSR lists the nodes v with u in N(v). */
typedef struct lp_csr {
    int32_t n_nodes;
    int32_t reserved_;
    int64_t nnz;               /* entries of colidx and of t_colidx */
    const int32_t *rowptr;     /* device [n_nodes + 1] */
    const int32_t *colidx;     /* device [nnz] */
    const int32_t *t_rowptr;   /* device [n_nodes + 1] */
    const int32_t *t_colidx;   /* device [nnz] */
    const float *inv_deg;      /* device [n_nodes]: 1/|N(v)|, 0 when N(v) is empty */
    const int32_t *row_order;  /* device [n_nodes] or NULL: a permutation of the rows, the order the aggregation visits
                                  them in (lp_build_csr: rows with |N(v)| >= 64 by decreasing floor(log2 |N(v)|), then
                                  all others, ids ascending inside a class); any permutation gives the same results */
    const int32_t *t_row_order;/* device [n_nodes] or NULL: same for the transposed CSR */
    const float *t_entry_scale;/* device [nnz] or NULL: inv_deg[t_colidx[p]] for every entry p of the transposed CSR, i.e.
                                  the weight 1/|N(v)| with which row v's gradient reaches its neighbour (the adjoint of
                                  the mean); NULL: the backward pass looks the weights up in inv_deg entry by entry */
} lp_csr;

/* K-layer model.  Layer k = 1..K maps width dims[k-1] to dims[k]:
 *   LP_LAYER_SAGE_MEAN (GraphSAGE with mean aggregator, the model of the benchmark configurations):
 *     z_v = h_v W_self[k-1] + mean_{u in N(v)} h_u W_neigh[k-1] + bias[k-1]
 *   LP_LAYER_GCN (the paper's second representative model, "Hyperparameters"; the graph convolution of Kipf and
 *   Welling): z_v = sum_{u in N(v)} h_u / sqrt(|N(v)| |N(u)|) W_neigh[k-1] + bias[k-1], on a CSR that already
 *     contains the self-pair (v, v) of every node (append them to the pair list given to lp_build_csr), so that
 *     |N(v)| is the degree plus one.  W_self and dW_self are ignored and may be NULL.
 *   h'_v = max(z_v, 0) for k < K and z_v for k = K. */
typedef struct lp_model {
    int32_t n_layers;                     /* K, 1..LP_MAX_LAYERS */
    int32_t dtype;                        /* LP_F32 or LP_BF16: storage of X, W_self, W_neigh, A and H */
    int32_t dims[LP_MAX_LAYERS + 1];      /* F_0 .. F_K */
    int32_t layer_type;                   /* LP_LAYER_SAGE_MEAN or LP_LAYER_GCN */
    int32_t fp32_products;                /* LP_FP32_PRODUCTS_*: how an LP_F32 model multiplies (ignored with LP_BF16) */
    int32_t reserved_;                    /* must be 0 */
    const void *W_self[LP_MAX_LAYERS];    /* device [F_{k-1}, F_k] */
    const void *W_neigh[LP_MAX_LAYERS];   /* device [F_{k-1}, F_k] */
    const void *bias[LP_MAX_LAYERS];      /* device [F_k], always fp32 */
} lp_model;

/* Activations written by lp_sage_forward and read by lp_backward. */
typedef struct lp_acts {
    void *A[LP_MAX_LAYERS]; /* A[k-1]: device [n_nodes, F_{k-1}], neighbourhood mean of layer k's input */
    void *H[LP_MAX_LAYERS]; /* H[k-1]: device [n_nodes, F_k], output of layer k; H[K-1] are the embeddings */
} lp_acts;

/* Gradients written (overwritten, not accumulated) by lp_backward.  Weight and bias gradients are always fp32. */
typedef struct lp_grads {
    float *dW_self[LP_MAX_LAYERS];  /* device [F_{k-1}, F_k] */
    float *dW_neigh[LP_MAX_LAYERS]; /* device [F_{k-1}, F_k] */
    float *dbias[LP_MAX_LAYERS];    /* device [F_k] */
    void *dX;                       /* device [n_nodes, F_0] in the model's storage type, or NULL to skip it */
} lp_grads;

/* The computational graph of one mini-batch with sampled neighbourhoods (Sec. II-B, last paragraph; Fig. 1b), as K
 * bipartite blocks over ONE node list: frontier k = the first n[k] entries of `nodes`, n[K] <= ... <= n[0]; frontier
 * K holds the end points of the scored edges.  Block k (arrays with index k-1) lists, for every node of frontier k,
 * the positions (in frontier k-1) of its sampled neighbours.  All arrays are caller-allocated device memory, sized
 * by the host-side bounds cap / cap_entries that lp_blocks_bounds computes; the exact sizes n[] live on the device. */
typedef struct lp_blocks {
    int32_t n_layers;                       /* K */
    int32_t n_graph_nodes;                  /* nodes of the graph the blocks are sampled from */
    int64_t n_edges;                        /* B, scored edges of the batch */
    int32_t cap[LP_MAX_LAYERS + 1];         /* cap[k] >= n[k] */
    int32_t reserved_;
    int64_t cap_entries[LP_MAX_LAYERS];     /* cap_entries[k-1] >= entries of block k */
    int32_t *n;                             /* device [K+1] */
    int32_t *nodes;                         /* device [cap[0]]: graph ids */
    int32_t *index;                         /* device [n_graph_nodes]: position of a node in `nodes`, or -1 */
    int32_t *ptr[LP_MAX_LAYERS];            /* device [cap[k]+1]: row pointers of block k */
    int32_t *col[LP_MAX_LAYERS];            /* device [cap_entries[k-1]]: positions in frontier k-1, draw order */
    float *inv_cnt[LP_MAX_LAYERS];          /* device [cap[k]]: 1/(sampled neighbours), 0 for none */
    int32_t *t_ptr[LP_MAX_LAYERS];          /* device [cap[k-1]+1]: transposed block, rows = positions in frontier k-1 */
    int32_t *t_col[LP_MAX_LAYERS];          /* device [cap_entries[k-1]]: positions in frontier k, by entry index */
    int32_t *e_src_pos, *e_dst_pos;         /* device [B]: the scored edges in positions of frontier K (-1: id out of range) */
    float *node_inv_deg;                    /* device [cap[0]]: inv_deg (of the graph sampled from) of nodes[i] */
} lp_blocks;

/* MLP edge predictor: x_e = h_u * h_v (element-wise), u^j = relu(u^(j-1) W[j-1] + bias[j-1]) for j < L,
 * s_e = u^(L-1) W[L-1] + bias[L-1].  dims[0] = width of the embeddings, dims[L] = 1. */
typedef struct lp_mlp {
    int32_t n_layers;                       /* L, 1..LP_MAX_MLP_LAYERS */
    int32_t dtype;                          /* LP_F32 or LP_BF16: storage of W, of the products and of the hidden layers */
    int32_t dims[LP_MAX_MLP_LAYERS + 1];
    int32_t fp32_products;                  /* LP_FP32_PRODUCTS_*: as in lp_model */
    const void *W[LP_MAX_MLP_LAYERS];       /* device [dims[j], dims[j+1]] */
    const float *bias[LP_MAX_MLP_LAYERS];   /* device [dims[j+1]], fp32 */
} lp_mlp;

/* Written by lp_mlp_score_loss, read by lp_mlp_backward. */
typedef struct lp_mlp_acts {
    void *X;                                /* device [B, dims[0]]: products of the end-point embeddings */
    void *U[LP_MAX_MLP_LAYERS];             /* U[j-1]: device [B, dims[j]], hidden layer j = 1..L-1 */
} lp_mlp_acts;

typedef struct lp_mlp_grads {
    float *dW[LP_MAX_MLP_LAYERS];           /* device [dims[j], dims[j+1]], fp32 */
    float *dbias[LP_MAX_MLP_LAYERS];        /* device [dims[j+1]], fp32 */
} lp_mlp_grads;

/* Adam moments, one fp32 array per parameter tensor, same shapes as lp_grads; the caller zeroes them before the
 * first lp_adam_step. */
typedef struct lp_opt_state {
    float *m_W_self[LP_MAX_LAYERS], *m_W_neigh[LP_MAX_LAYERS], *m_bias[LP_MAX_LAYERS];
    float *v_W_self[LP_MAX_LAYERS], *v_W_neigh[LP_MAX_LAYERS], *v_bias[LP_MAX_LAYERS];
} lp_opt_state;

/* Text for a status code (static storage, never NULL). */
const char *lp_strerror(int status);

/* Version of this header's structs and signatures, bumped with every change to them.  lp_abi_version() returns the
 * value the library was built with: a caller (or binding) that was written against another one must not go on. */
#define LP_ABI_VERSION 5
int lp_abi_version(void);

/* ---------------------------------------------------------------------------
 * lp_build_csr - canonical CSR of the visible edge set (Sec. II-A: the graph
 * is a node set with a set of node pairs; Sec. IV-A: undirected, unweighted,
 * degree d_v = number of neighbours).  Done once per graph, not per step.
 *
 * rows/cols: device [n_in], the pair (rows[i], cols[i]) puts cols[i] into
 * N(rows[i]).  Repeated pairs collapse; a pair with rows[i] == cols[i] is kept
 * as an ordinary entry.  With LP_SYMMETRIZE each pair also counts reversed.
 * Outputs (device): rowptr, t_rowptr [n_nodes+1]; colidx, t_colidx with room
 * for n_in entries (2*n_in with LP_SYMMETRIZE); inv_deg [n_nodes]; row_order
 * and t_row_order [n_nodes] (both may be NULL); t_entry_scale, as many floats
 * as t_colidx has room for (may be NULL).  *nnz_out (HOST pointer)
 * receives the number of entries.  There is exactly one correct output.
 *
 * This call waits for the stream before it returns (it reads nnz back).
 * Errors: LP_ERR_OUT_OF_RANGE if an id lies outside [0, n_nodes) - detected
 * on the device without any out-of-bounds access; outputs are then undefined.
 */
size_t lp_build_csr_workspace_bytes(int32_t n_nodes, int64_t n_in, uint32_t flags);
int lp_build_csr(int32_t n_nodes, int64_t n_in, const int32_t *rows, const int32_t *cols, uint32_t flags,
                 int32_t *rowptr, int32_t *colidx, int32_t *t_rowptr, int32_t *t_colidx, float *inv_deg,
                 int32_t *row_order, int32_t *t_row_order, float *t_entry_scale, int64_t *nnz_out, void *ws,
                 size_t ws_bytes, void *stream);

/* ---------------------------------------------------------------------------
 * lp_sage_forward - the K aggregation layers of Eq. (1) for every visible
 * node (Algorithm 1, the loop "for k = 1 to K compute h_v^(k)"), with h^(0) = x.
 * X: device [n_nodes, F_0].  Fills saved->A[k-1] and saved->H[k-1] for
 * k = 1..K; the embeddings are saved->H[K-1].  A node without neighbours
 * aggregates the zero vector.
 */
size_t lp_sage_forward_workspace_bytes(const lp_model *m, int32_t n_nodes);
int lp_sage_forward(const lp_csr *g, const lp_model *m, const void *X, lp_acts *saved, void *ws,
                    size_t ws_bytes, void *stream);

/* ---------------------------------------------------------------------------
 * lp_sage_forward_edges - the forward pass of a TRAINING step (Algorithm 1:
 * the layers of Eq. (1), of which the loss of Eq. (2) reads only the
 * embeddings of the end points of the scored edges).  Layers 1..K-1 are
 * evaluated for every visible node as in lp_sage_forward; layer K only for the
 * nodes that are e_src[i] or e_dst[i] of one of the B scored edges (device
 * [B] each; an edge with an id outside [0, n_nodes) lists nothing).  Rows of
 * saved->A[K-1] and saved->H[K-1] that belong to other nodes are unspecified
 * afterwards: when 8*B < 3*n_nodes they are neither read nor written and keep
 * whatever they held; a larger batch can touch so much of the graph that
 * listing does not pay, and every row is evaluated.  lp_score_loss / lp_mlp_score_loss
 * and lp_backward / lp_backward_edge_grads on the SAME edges read only rows
 * that were written, and give what they give after lp_sage_forward up to the
 * order of fp32 sums.  B = 0 evaluates layers 1..K-1 only.  Embeddings of all
 * nodes (evaluation, inference) need lp_sage_forward.
 * Errors as lp_sage_forward; B < 0 or B > 0 with a NULL id array is
 * LP_ERR_INVALID_ARG, B >= 2^31 LP_ERR_OUT_OF_RANGE.
 */
size_t lp_sage_forward_edges_workspace_bytes(const lp_model *m, int32_t n_nodes, int64_t B);
int lp_sage_forward_edges(const lp_csr *g, const lp_model *m, const void *X, int64_t B, const int32_t *e_src,
                          const int32_t *e_dst, lp_acts *saved, void *ws, size_t ws_bytes, void *stream);

/* ---------------------------------------------------------------------------
 * lp_sample_neg - per-source uniform negative sampling (Sec. II-B; Algorithm 1,
 * "Generate negative samples"): sample q = i*k_neg + j keeps the source
 * u = pos_src[i] and receives a destination drawn uniformly from [0, n_space)
 * that is neither u nor a member of N(u).
 *
 * Random stream: attempt t of sample q uses 32-bit word (t mod 4) of
 * Philox4x32-10 with counter (q, t div 4, step_lo, step_hi) and key
 * (seed_lo, seed_hi); the candidate is floor(word * n_space / 2^32).  The
 * first valid candidate of attempts 0..15 is taken; after sixteen rejections
 * the nodes following the last candidate (mod n_space) are tried in order.  If
 * no node is valid, the last candidate is written and *n_failed incremented.
 * The result is a pure function of (graph, pos_src, k_neg, n_space, seed, step).
 *
 * pos_src: device [n_pos].  neg_dst: device [n_pos*k_neg].  neg_src: device
 * [n_pos*k_neg] or NULL; receives the kept source of each sample.  n_failed:
 * device int32 or NULL; the caller zeroes it.  n_pos*k_neg must be < 2^31.
 * Sources must lie in [0, g->n_nodes); a source outside is treated as having
 * no neighbours.
 */
int lp_sample_neg(const lp_csr *g, int64_t n_pos, const int32_t *pos_src, int32_t k_neg, int32_t n_space,
                  uint64_t seed, uint64_t step, int32_t *neg_dst, int32_t *neg_src, int32_t *n_failed,
                  void *stream);

/* ---------------------------------------------------------------------------
 * lp_score_loss - edge scores, loss and its derivative (Eq. 2 with the dot
 * product; Algorithm 1, the per-edge loop and "Compute L^i"):
 *   s_e = <H[e_src[e]], H[e_dst[e]]>,  y_e = 1 for e < n_pos_edges else 0,
 *   l_e = -[y ln sigma(s) + (1-y) ln(1-sigma(s))],  loss = (1/B) sum_e l_e,
 *   dscore_e = (sigma(s_e) - y_e) / B.
 * HK: device [n_nodes, F].  e_src, e_dst: device [B], ids in [0, n_nodes).
 * An edge with an id outside that range is never dereferenced: it is scored 0,
 * gets dscore 0, adds nothing to the loss sum and still counts in B, so a batch
 * that contains such edges trains on a loss that is too small.  n_invalid:
 * device int32 or NULL; the caller zeroes it and it receives the number of such
 * edges, so that a corrupted batch does not go unnoticed (check it whenever the
 * edge list does not come from lp_sample_neg on the same graph).
 * scores: device [B].  loss: device float.  dscore: device [B] or NULL.
 * The loss is summed in a fixed order, so repeated calls give the same bits.
 */
size_t lp_score_loss_workspace_bytes(int64_t B);
int lp_score_loss(const void *HK, int32_t n_nodes, int32_t F, int32_t dtype, int64_t B, int64_t n_pos_edges,
                  const int32_t *e_src, const int32_t *e_dst, float *scores, float *loss, float *dscore,
                  int32_t *n_invalid, void *ws, size_t ws_bytes, void *stream);

/* ---------------------------------------------------------------------------
 * lp_score_loss_noalloc - lp_score_loss for callers that cannot allocate or hand
 * over a workspace: code under HIP graph capture, tight serving loops that score
 * candidate edges, harnesses that forbid hipMalloc.  Same arguments without
 * ws/ws_bytes, same kernels, same results bit for bit.  The per-block partial
 * sums of the loss (the only scratch of this call, 2 048 floats = 8 KiB whatever
 * B is) live in a device array inside the library, of which every GPU the
 * library runs on holds one copy until the process ends; the call allocates and
 * frees nothing.  The array's device address is looked up on the first call on
 * each device (make that call outside a graph capture).
 * Limits: B <= LP_SCORE_LOSS_NOALLOC_MAX_EDGES, else LP_ERR_OUT_OF_RANGE (the
 * block count, and with it the scratch, stays fixed; edges beyond the first
 * few thousand per block are walked in a loop).  Every call on one GPU shares
 * that GPU's array: calls that overlap in time on one GPU (two streams, two
 * threads) race on it and must be ordered by the caller; calls one after the
 * other on a stream need nothing, every entry that is read was written by the
 * same call.  LP_ERR_HIP if the address cannot be obtained.
 */
#define LP_SCORE_LOSS_NOALLOC_MAX_EDGES ((int64_t)1 << 28)
int lp_score_loss_noalloc(const void *HK, int32_t n_nodes, int32_t F, int32_t dtype, int64_t B, int64_t n_pos_edges,
                          const int32_t *e_src, const int32_t *e_dst, float *scores, float *loss, float *dscore,
                          int32_t *n_invalid, void *stream);

/* ---------------------------------------------------------------------------
 * lp_backward - gradient of the batch loss with respect to all weights
 * (Algorithm 1, "Compute the gradient"): scatters dscore through the dot
 * product into dL/dH^K, then walks the layers K..1 through the ReLU, the two
 * linear maps and the adjoint of the mean aggregation (transposed CSR).
 * X and `saved` are the input and result of the lp_sage_forward (or
 * lp_sage_forward_edges, with the same e_src/e_dst) call for the same graph
 * and model: of saved->A[K-1] and saved->H[K-1] only the rows of the end
 * points of the scored edges are read.  e_src/e_dst/dscore as in
 * lp_score_loss (an edge with an id outside [0, n_nodes) contributes
 * nothing).  All sums are taken in a fixed order: repeated calls give the
 * same bits.
 */
size_t lp_backward_workspace_bytes(const lp_model *m, int32_t n_nodes, int64_t B);
int lp_backward(const lp_csr *g, const lp_model *m, const void *X, const lp_acts *saved, int64_t B,
                const int32_t *e_src, const int32_t *e_dst, const float *dscore, lp_grads *out, void *ws,
                size_t ws_bytes, void *stream);

/* ---------------------------------------------------------------------------
 * lp_sparsify - the degree-based graph sparsifier (Algorithm 1, "Graph
 * Sparsification"; Sec. IV-B, second paragraph; Theorems 1 and 2): n_draws edges
 * are drawn independently and with replacement from one partition's edge list,
 * edge (u, v) with probability p proportional to 1/d_u + 1/d_v, where d is the
 * number of listed edges at a node; a drawn edge carries weight 1/(n_draws p)
 * and repeated draws add up.  Done once per partition, before training.
 *
 * So that every implementation draws the same edges, all decisions are taken
 * on integers: q_e = floor(2^32/d_u) + floor(2^32/d_v), Q = sum of q_e,
 * p_e = q_e/Q; draw l forms r = word0 * 2^32 + word1 of Philox4x32-10 with
 * counter (l_lo, l_hi, 0, 0) and key (seed_lo, seed_hi), t = floor(r Q / 2^64),
 * and takes the edge e with cum_e <= t < cum_e + q_e (cum = running sum of q in
 * input order).
 *
 * eu, ev: device [n_edges], the undirected edges, each listed once, no
 * self-pairs (an edge listed twice counts twice towards the degrees and can be
 * drawn under either index).  Outputs (device), each with room for
 * min(n_edges, n_draws) entries: kept_edge = indices of the distinct drawn
 * edges, ascending; kept_u / kept_v (may be NULL) = their end points as listed;
 * kept_count (may be NULL) = times drawn; kept_weight = count / (n_draws p).
 * *n_kept_out (HOST pointer) receives their number.
 *
 * This call waits for the stream before it returns.  Errors:
 * LP_ERR_OUT_OF_RANGE if an id lies outside [0, n_nodes) (detected on the
 * device without any out-of-bounds access; outputs are then undefined) or if
 * n_edges >= 2^31.
 */
size_t lp_sparsify_workspace_bytes(int32_t n_nodes, int64_t n_edges);
int lp_sparsify(int32_t n_nodes, int64_t n_edges, const int32_t *eu, const int32_t *ev, int64_t n_draws, uint64_t seed,
                int32_t *kept_edge, int32_t *kept_u, int32_t *kept_v, int32_t *kept_count, float *kept_weight,
                int64_t *n_kept_out, void *ws, size_t ws_bytes, void *stream);

/* ---------------------------------------------------------------------------
 * lp_sgd_step, lp_adam_step - the weight update that ends a training step
 * (Algorithm 1, "Update W <- W - eta grad L(W)"; "Hyperparameters": Adam,
 * learning rate 0.001).  Both update every parameter tensor of the model IN
 * PLACE (the weights that lp_model points at are written, although the struct
 * declares them const for the other calls) from the gradients in `g`, in one
 * kernel launch, and return without waiting.
 *   sgd:  w <- w - lr g
 *   adam: m <- beta1 m + (1-beta1) g;  v <- beta2 v + (1-beta2) g^2;
 *         w <- w - lr (m / (1-beta1^t)) / (sqrt(v / (1-beta2^t)) + eps),   t = t_step = 1, 2, ...
 * Arithmetic is fp32.  With LP_BF16 the weight matrices are widened, updated
 * and rounded back to bfloat16 (nearest even); biases, gradients and moments
 * are fp32 throughout.  Averaging gradients over workers, where there are
 * several, is the caller's business and comes before this call.
 * Errors: LP_ERR_INVALID_ARG for a NULL tensor, t_step < 1, beta outside [0,1),
 * a negative eps or a non-finite learning rate.
 */
int lp_sgd_step(const lp_model *m, const lp_grads *g, float lr, void *stream);
/* The same two updates for one tensor of n elements (dtype = storage of w; grad, m, v fp32): for parameters that
 * live outside lp_model, such as the MLP edge predictor's. */
int lp_sgd_update_tensor(void *w, int32_t dtype, const float *grad, int64_t n, float lr, void *stream);
int lp_adam_update_tensor(void *w, int32_t dtype, const float *grad, float *m, float *v, int64_t n, int64_t t_step, float lr,
                          float beta1, float beta2, float eps, void *stream);
int lp_adam_step(const lp_model *m, const lp_grads *g, const lp_opt_state *s, int64_t t_step, float lr, float beta1,
                 float beta2, float eps, void *stream);

/* ---------------------------------------------------------------------------
 * lp_hits_at_k - the accuracy metric of the paper's experiments
 * ("Hyperparameters": Hits@100, the metric of the Open Graph Benchmark's link
 * prediction tasks).  The K-th largest of the n_neg negative-edge scores is the
 * threshold; *hits (device int64) receives the number of the n_pos positive
 * scores that are strictly greater; Hits@K = *hits / n_pos.  With n_neg < K
 * the threshold is -infinity and every positive is a hit.  threshold: optional
 * device float that receives the threshold.  Scores are device fp32 arrays
 * (e.g. the `scores` output of lp_score_loss or lp_mlp_score_loss on the test
 * edges); they must not contain NaN.  Integer result: bit-exact.
 * Errors: LP_ERR_INVALID_ARG (K < 1, negative counts, NULL arrays or hits),
 * LP_ERR_OUT_OF_RANGE (n_neg >= 2^31), LP_ERR_WORKSPACE.
 */
size_t lp_hits_at_k_workspace_bytes(int64_t n_neg);
int lp_hits_at_k(const float *pos_scores, int64_t n_pos, const float *neg_scores, int64_t n_neg, int64_t K, int64_t *hits,
                 float *threshold, void *ws, size_t ws_bytes, void *stream);

/* ---------------------------------------------------------------------------
 * Sampled-neighbourhood training step (the paper's mini-batch mode: Sec. II-B,
 * last paragraph; Fig. 1b; "Hyperparameters": 25, 10, 5 neighbours for the
 * first, second, third hop).
 *
 * lp_blocks_bounds: pure host arithmetic; cap [K+1] and cap_entries [K] for a
 * graph of n_nodes / nnz entries, B scored edges and fan-outs fanout[0..K-1]
 * (fanout[0] = first hop = layer K; each in 1..LP_MAX_FANOUT, or LP_FANOUT_ALL
 * for a full-neighbourhood hop: every node of the frontier takes its whole
 * list, in list order).
 *
 * lp_sample_blocks: fills `out` (whose arrays and cap fields the caller set up
 * from the bounds) for the batch e_src/e_dst (device [B]; ids outside the graph
 * are ignored and get position -1).  Frontier K = the distinct end points,
 * ascending.  At hop h = 1..K (layer k = K+1-h) every node v of frontier k
 * draws min(|N(v)|, fanout[h-1]) distinct neighbours uniformly without
 * replacement: a partial Fisher-Yates shuffle of the positions 0..d-1 of its
 * sorted neighbour list, swap t exchanging position t with position
 * t + floor(word * (d-t) / 2^32), word = word (t mod 4) of Philox4x32-10 with
 * counter (v, hop*2^16 + t div 4, step_lo, step_hi) and key (seed_lo, seed_hi);
 * the sample is positions 0..f-1 in that order; a node with d <= f takes its
 * whole list in order.  Frontier k-1 = frontier k followed by the drawn nodes
 * that are new, ascending.  The transposed block lists, for every position of
 * frontier k-1, the rows that drew it, ordered by entry index.  Exactly one
 * result is correct.  Returns without waiting for the stream.
 *
 * lp_sage_forward_blocks: Eq. (1) on the blocks.  X: device [n_graph_nodes, F_0];
 * X_frontier: device [cap[0], F_0], receives the feature rows of frontier 0;
 * saved->A[k-1]: device [cap[k], F_{k-1}], saved->H[k-1]: device [cap[k], F_k];
 * row i belongs to nodes[i].  The embeddings of the batch end points are the
 * first n[K] rows of saved->H[K-1]; score them with lp_score_loss(H, cap[K],
 * ..., e_src_pos, e_dst_pos, ...).  With layer_type = LP_LAYER_GCN the layer is
 * the graph convolution of the full graph restricted to the blocks, with the
 * full graph's degrees in the normalisation:
 *   a_v = (d_v / |S(v)|) sum_{u in S(v)} h_u / sqrt(d_v d_u),  z_v = a_v W_neigh + b
 * (d = row lengths of the CSR the blocks were sampled from, which holds the
 * self-pairs; the factor d_v / |S(v)| is 1 for a full-neighbourhood hop, for
 * which the result equals lp_sage_forward's GCN on the computational graph).
 *
 * lp_backward_blocks: weight and bias gradients of the batch loss through the
 * blocks (dscore from lp_score_loss); out->dX is ignored.  Fixed summation
 * order: repeated calls give the same bits.
 *
 * lp_backward_blocks_edge_grads: the same with dL/dH^K seeded from edge_grad
 * (device [n_edges, F_K], storage type, from lp_mlp_backward on the frontier
 * positions: Eq. 2 with the MLP scorer): row e_src_pos[e] receives
 * edge_grad_e * h_v, row e_dst_pos[e] receives edge_grad_e * h_u.
 */
int lp_blocks_bounds(int32_t n_nodes, int64_t nnz, int64_t B, int32_t K, const int32_t *fanout, int32_t *cap,
                     int64_t *cap_entries);
size_t lp_sample_blocks_workspace_bytes(int32_t n_nodes, int64_t nnz, int64_t B, int32_t K, const int32_t *fanout);
int lp_sample_blocks(const lp_csr *g, int64_t B, const int32_t *e_src, const int32_t *e_dst, int32_t K, const int32_t *fanout,
                     uint64_t seed, uint64_t step, lp_blocks *out, void *ws, size_t ws_bytes, void *stream);
size_t lp_forward_blocks_workspace_bytes(const lp_model *m, const lp_blocks *b);
int lp_sage_forward_blocks(const lp_blocks *b, const lp_model *m, const void *X, void *X_frontier, lp_acts *saved, void *ws,
                           size_t ws_bytes, void *stream);
size_t lp_backward_blocks_workspace_bytes(const lp_model *m, const lp_blocks *b);
int lp_backward_blocks(const lp_blocks *b, const lp_model *m, const void *X_frontier, const lp_acts *saved, const float *dscore,
                       lp_grads *out, void *ws, size_t ws_bytes, void *stream);
int lp_backward_blocks_edge_grads(const lp_blocks *b, const lp_model *m, const void *X_frontier, const lp_acts *saved,
                                  const void *edge_grad, lp_grads *out, void *ws, size_t ws_bytes, void *stream);

/* ---------------------------------------------------------------------------
 * MLP edge predictor (Eq. 2 with the MLP the paper's experiments use, see
 * "Hyperparameters": a 3-layer MLP, hidden width 256) in place of the dot
 * product.  The two end-point embeddings are combined by their element-wise
 * product (the dot product is the special case of one layer of ones).
 *
 * lp_mlp_score_loss: scores, loss and dscore as lp_score_loss, but
 * s_e = MLP(H[e_src[e]] * H[e_dst[e]]); HK has the storage type p->dtype and
 * width p->dims[0].  Fills `saved`.  An edge with an id outside [0, n_nodes)
 * is scored 0, gets dscore 0 and adds nothing to the loss sum.
 *
 * lp_mlp_backward: gradients of the predictor's weights and biases, and
 * edge_grad (device [B, dims[0]], storage type) = dL/d(h_u * h_v) per scored edge.
 *
 * lp_backward_edge_grads: lp_backward with dL/dH^K seeded from edge_grad
 * (row u receives edge_grad_e * h_v, row v receives edge_grad_e * h_u) instead
 * of from dscore; everything else is identical.
 */
size_t lp_mlp_score_loss_workspace_bytes(const lp_mlp *p, int64_t B);
int lp_mlp_score_loss(const void *HK, int32_t n_nodes, int64_t B, int64_t n_pos_edges, const int32_t *e_src, const int32_t *e_dst,
                      const lp_mlp *p, lp_mlp_acts *saved, float *scores, float *loss, float *dscore, void *ws, size_t ws_bytes,
                      void *stream);
size_t lp_mlp_backward_workspace_bytes(const lp_mlp *p, int64_t B);
int lp_mlp_backward(const lp_mlp *p, const lp_mlp_acts *saved, int64_t B, const float *dscore, lp_mlp_grads *out, void *edge_grad,
                    void *ws, size_t ws_bytes, void *stream);
int lp_backward_edge_grads(const lp_csr *g, const lp_model *m, const void *X, const lp_acts *saved, int64_t B,
                           const int32_t *e_src, const int32_t *e_dst, const void *edge_grad, lp_grads *out, void *ws,
                           size_t ws_bytes, void *stream);

/* ---------------------------------------------------------------------------
 * Instrumentation for benchmarks (not part of the method).  While enabled, each
 * kernel launch made by the calls above is bracketed by two HIP events on the
 * launch stream (lp_timing_enable(1): all classes but LP_KC_OTHER, whose small
 * launches would pay more for the events than they take; lp_timing_enable(2):
 * every launch; 0: off).  lp_timing_collect waits for the recorded events, writes the
 * summed milliseconds and launch counts per kernel class (arrays of at least
 * LP_KC_COUNT entries) and forgets them.  Off by default.  Process-wide state
 * (the only switch the library keeps), guarded by a mutex.
 */
enum {
    LP_KC_SPMM = 0,     /* CSR mean aggregation, forward and transposed */
    LP_KC_GEMM_NT = 1,  /* layer transform and input-gradient transform */
    LP_KC_GEMM_TN = 2,  /* weight gradients (incl. the partial-sum reduction) */
    LP_KC_SCATTER = 3,  /* edge gradient scatter */
    LP_KC_SCORE = 4,    /* edge scores and loss */
    LP_KC_SAMPLE = 5,   /* negative sampler */
    LP_KC_OTHER = 6,    /* fills, bias gradients, weight transposes */
    LP_KC_COUNT = 7
};
int lp_timing_enable(int on);
int lp_timing_collect(double *ms_by_class, int64_t *launches_by_class, int32_t n_classes);

#ifdef __cplusplus
}
#endif
#endif /* LP_H_ */
