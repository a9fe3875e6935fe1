// MLP edge predictor (Eq. 2 of the paper with "MLP" as the predictor; the experiments use a 3-layer MLP, see
// "Hyperparameters"): the embeddings of the two end points are combined by the element-wise product and sent through
// L linear layers with ReLU between them and a single output,
//     x_e = h_u * h_v,  u^0 = x_e,  u^j = relu(u^(j-1) W_j + c_j) (j < L),  s_e = u^(L-1) W_L + c_L,
// followed by the same binary cross-entropy and batch mean as the dot-product path.  The hidden layers run on the
// MFMA kernels of gemm_mfma.hip over the B scored edges; the output layer, the loss and the element-wise pieces
// are small kernels here.  lp_mlp_backward returns dL/dx_e per scored edge, which lp_backward_edge_grads scatters
// into dL/dH^K.
#include "lp_internal.h"

namespace {

constexpr int kThreads = 256;
constexpr int kMaxLossBlocks = 2048;

int check_mlp(const lp_mlp *p) {
    if (!p || p->n_layers < 1 || p->n_layers > LP_MAX_MLP_LAYERS) return LP_ERR_INVALID_ARG;
    if (p->dtype != LP_F32 && p->dtype != LP_BF16) return LP_ERR_UNSUPPORTED;
    if (!lp_valid_fp32_products(p->fp32_products)) return LP_ERR_INVALID_ARG;
    const int L = p->n_layers;
    if (p->dims[L] != 1) return LP_ERR_INVALID_ARG;
    for (int j = 0; j < L; ++j) {
        if (p->dims[j] <= 0) return LP_ERR_INVALID_ARG;
        if ((p->dims[j] % lp_vec_elems(p->dtype)) || p->dims[j] > 1024) return LP_ERR_UNSUPPORTED;
        if (!p->W[j] || !p->bias[j] || !lp_aligned16(p->W[j])) return LP_ERR_INVALID_ARG;
    }
    return LP_OK;
}

int max_width(const lp_mlp *p) {
    int d = 0;
    for (int j = 0; j < p->n_layers; ++j) d = p->dims[j] > d ? p->dims[j] : d;
    return d;
}

size_t transposed_bytes(const lp_mlp *p) {
    size_t n = 0;
    for (int j = 1; j < p->n_layers; ++j) n += lp_align_up((size_t)p->dims[j - 1] * p->dims[j], 64);
    return lp_align_up(n * (size_t)lp_elem_bytes(p->dtype));
}

template <int G>
__device__ inline float group_sum(float v) {
#pragma unroll
    for (int d = G >> 1; d >= 1; d >>= 1) v += __shfl_xor(v, d, 64);
    return v;
}

// X[e, :] = H[u_e, :] * H[v_e, :], zero for an edge with an id outside the graph
template <typename T>
__global__ void edge_product_kernel(const T *__restrict__ H, int32_t n_nodes, int FV, int64_t B, const int32_t *__restrict__ e_src,
                                    const int32_t *__restrict__ e_dst, T *__restrict__ X) {
    constexpr int VE = LpVec<T>::N;
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t e = idx / FV;
    const int c = (int)(idx % FV);
    if (e >= B) return;
    const int32_t u = e_src[e], v = e_dst[e];
    float x[VE];
#pragma unroll
    for (int i = 0; i < VE; ++i) x[i] = 0.f;
    if (u >= 0 && u < n_nodes && v >= 0 && v < n_nodes) {
        float a[VE], b[VE];
        LpVec<T>::load(H + ((int64_t)u * FV + c) * VE, a);
        LpVec<T>::load(H + ((int64_t)v * FV + c) * VE, b);
#pragma unroll
        for (int i = 0; i < VE; ++i) x[i] = a[i] * b[i];
    }
    LpVec<T>::store(X + (e * FV + c) * VE, x);
}

// s_e = <U[e, :], w> + c, loss and dL/ds; a group of G lanes per edge, block sums in a fixed order
template <typename T, int G>
__global__ __launch_bounds__(kThreads) void mlp_out_loss_kernel(const T *__restrict__ U, const T *__restrict__ w, const float *__restrict__ c,
                                                                int32_t n_nodes, int32_t F, int64_t B, int64_t n_pos,
                                                                const int32_t *__restrict__ e_src, const int32_t *__restrict__ e_dst,
                                                                float *__restrict__ scores, float *__restrict__ dscore,
                                                                float *__restrict__ partial) {
    __shared__ float red[kThreads / 64];
    constexpr int VE = LpVec<T>::N;
    const int sub = threadIdx.x % G;
    const int64_t groups_per_block = kThreads / G;
    const int64_t gid = (int64_t)blockIdx.x * groups_per_block + threadIdx.x / G;
    const int64_t n_groups = (int64_t)gridDim.x * groups_per_block;
    const float invB = 1.0f / (float)B;
    const int FV = F / VE;
    const float c0 = c[0];
    float acc = 0.0f;
    for (int64_t e = gid; e < B; e += n_groups) {
        const int32_t u = e_src[e], v = e_dst[e];
        const bool ok = u >= 0 && u < n_nodes && v >= 0 && v < n_nodes;
        float s = 0.0f;
        if (ok) {
            for (int j = sub; j < FV; j += G) {
                float a[VE], b[VE];
                LpVec<T>::load(U + e * F + j * VE, a);
                LpVec<T>::load(w + j * VE, b);
#pragma unroll
                for (int i = 0; i < VE; ++i) s += a[i] * b[i];
            }
        }
        s = group_sum<G>(s);
        if (sub == 0) {
            s = ok ? s + c0 : 0.0f;
            const float y = e < n_pos ? 1.0f : 0.0f;
            const float ex = expf(-fabsf(s));
            const float ell = fmaxf(s, 0.0f) - y * s + log1pf(ex);
            const float sig = s >= 0.0f ? 1.0f / (1.0f + ex) : ex / (1.0f + ex);
            scores[e] = s;
            if (dscore) dscore[e] = ok ? (sig - y) * invB : 0.0f;
            if (ok) acc += ell;
        }
    }
    acc = group_sum<64>(acc);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) partial[blockIdx.x] = (red[0] + red[1]) + (red[2] + red[3]);
}

__global__ __launch_bounds__(kThreads) void mean_finish_kernel(const float *__restrict__ partial, int n, int64_t B, float *__restrict__ loss) {
    __shared__ double red[kThreads];
    double s = 0.0;
    for (int i = threadIdx.x; i < n; i += kThreads) s += (double)partial[i];
    red[threadIdx.x] = s;
    __syncthreads();
    for (int d = kThreads / 2; d >= 1; d >>= 1) {
        if (threadIdx.x < d) red[threadIdx.x] += red[threadIdx.x + d];
        __syncthreads();
    }
    if (threadIdx.x == 0) *loss = B > 0 ? (float)(red[0] / (double)B) : 0.0f;
}

// Output layer, backward.  P[e, j] = ds_e * U[e, j] for j < F and P[e, F] = ds_e (the column sums of P are the
// gradients of the output weights and of the output bias); dU[e, j] = ds_e * w_j, zeroed where the hidden unit is
// not active (gate_on), in the storage type.
template <typename T>
__global__ void mlp_out_backward_kernel(const T *__restrict__ U, const T *__restrict__ w, const float *__restrict__ ds, int FV,
                                        int64_t B, bool gate_on, float *__restrict__ P, T *__restrict__ dU) {
    constexpr int VE = LpVec<T>::N;
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t e = idx / FV;
    const int c = (int)(idx % FV);
    if (e >= B) return;
    const int F = FV * VE;
    const float g = ds[e];
    float u[VE], ww[VE], d[VE];
    LpVec<T>::load(U + (e * FV + c) * VE, u);
    LpVec<T>::load(w + c * VE, ww);
    float *prow = P + e * (F + 4) + c * VE;
#pragma unroll
    for (int i = 0; i < VE; ++i) {
        prow[i] = g * u[i];
        d[i] = (!gate_on || u[i] > 0.f) ? g * ww[i] : 0.f;
    }
    LpVec<T>::store(dU + (e * FV + c) * VE, d);
    if (c == 0) {
        float *tail = P + e * (F + 4) + F;
        tail[0] = g; tail[1] = 0.f; tail[2] = 0.f; tail[3] = 0.f;
    }
}

// y = gate > 0 ? y : 0, element-wise, in place
template <typename T>
__global__ void relu_gate_kernel(T *__restrict__ y, const T *__restrict__ gate, int64_t n_vec) {
    constexpr int VE = LpVec<T>::N;
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_vec) return;
    float a[VE], g[VE];
    LpVec<T>::load(y + i * VE, a);
    LpVec<T>::load(gate + i * VE, g);
#pragma unroll
    for (int k = 0; k < VE; ++k) a[k] = g[k] > 0.f ? a[k] : 0.f;
    LpVec<T>::store(y + i * VE, a);
}

int loss_blocks(int64_t B, int G) {
    const int64_t groups_per_block = kThreads / G;
    int64_t nb = lp_ceil_div(B, groups_per_block * 4);
    if (nb < 1) nb = 1;
    if (nb > kMaxLossBlocks) nb = kMaxLossBlocks;
    return (int)nb;
}

int group_lanes(int F, int vec) {
    int g = 8;
    while (g < 64 && g * vec < F) g <<= 1;
    return g;
}

template <typename T>
void launch_out_loss(int G, int nb, hipStream_t st, const void *U, const void *w, const float *c, int32_t n_nodes, int32_t F, int64_t B,
                     int64_t n_pos, const int32_t *e_src, const int32_t *e_dst, float *scores, float *dscore, float *partial) {
    const T *u = static_cast<const T *>(U), *ww = static_cast<const T *>(w);
    switch (G) {
        case 8: hipLaunchKernelGGL((mlp_out_loss_kernel<T, 8>), dim3(nb), dim3(kThreads), 0, st, u, ww, c, n_nodes, F, B, n_pos, e_src, e_dst, scores, dscore, partial); break;
        case 16: hipLaunchKernelGGL((mlp_out_loss_kernel<T, 16>), dim3(nb), dim3(kThreads), 0, st, u, ww, c, n_nodes, F, B, n_pos, e_src, e_dst, scores, dscore, partial); break;
        case 32: hipLaunchKernelGGL((mlp_out_loss_kernel<T, 32>), dim3(nb), dim3(kThreads), 0, st, u, ww, c, n_nodes, F, B, n_pos, e_src, e_dst, scores, dscore, partial); break;
        default: hipLaunchKernelGGL((mlp_out_loss_kernel<T, 64>), dim3(nb), dim3(kThreads), 0, st, u, ww, c, n_nodes, F, B, n_pos, e_src, e_dst, scores, dscore, partial);
    }
}

struct MlpBackwardWs {
    float *P;             // [B, widest + 4]
    float *sums;          // [widest + 4]
    void *buf[2];         // [B, widest] in the storage type
    float *tn_partials, *colsum_partials;
    size_t bytes;
};

MlpBackwardWs carve_backward(void *ws, const lp_mlp *p, int64_t B) {
    char *q = static_cast<char *>(ws);
    size_t off = 0;
    auto take = [&](size_t bytes) { char *r = q ? q + off : nullptr; off += lp_align_up(bytes); return r; };
    MlpBackwardWs w;
    const size_t rows = (size_t)(B > 0 ? B : 1);
    const int wmax = max_width(p);
    w.P = reinterpret_cast<float *>(take(sizeof(float) * rows * (size_t)(wmax + 4)));
    w.sums = reinterpret_cast<float *>(take(sizeof(float) * (size_t)(wmax + 4)));
    for (int i = 0; i < 2; ++i) w.buf[i] = take((size_t)lp_elem_bytes(p->dtype) * rows * (size_t)wmax);
    size_t tn = 0, cs = lp_colsum_partials_bytes((int64_t)rows, wmax + 4);
    for (int j = 1; j < p->n_layers; ++j) {
        const size_t t = lp_weight_grads_partials_bytes(p->dtype, (int32_t)rows, 0, p->dims[j - 1], p->dims[j]);
        tn = t > tn ? t : tn;
    }
    w.tn_partials = reinterpret_cast<float *>(take(tn));
    w.colsum_partials = reinterpret_cast<float *>(take(cs));
    w.bytes = off;
    return w;
}

}  // namespace

extern "C" size_t lp_mlp_score_loss_workspace_bytes(const lp_mlp *p, int64_t B) {
    (void)B;
    if (check_mlp(p) != LP_OK) return 0;
    return lp_align_up(sizeof(float) * kMaxLossBlocks) + transposed_bytes(p);
}

extern "C" int lp_mlp_score_loss(const void *HK, int32_t n_nodes, int64_t B, int64_t n_pos_edges, const int32_t *e_src,
                                 const int32_t *e_dst, const lp_mlp *p, lp_mlp_acts *saved, float *scores, float *loss, float *dscore,
                                 void *ws, size_t ws_bytes, void *stream) {
    LP_TRY(check_mlp(p));
    if (!HK || !lp_aligned16(HK) || n_nodes <= 0 || B < 0 || n_pos_edges < 0 || n_pos_edges > B || !loss || !saved) return LP_ERR_INVALID_ARG;
    if (B >= ((int64_t)1 << 31)) return LP_ERR_OUT_OF_RANGE;
    if (B > 0 && (!e_src || !e_dst || !scores)) return LP_ERR_INVALID_ARG;
    const int L = p->n_layers;
    if (B > 0) {
        if (!saved->X || !lp_aligned16(saved->X)) return LP_ERR_INVALID_ARG;
        for (int j = 1; j < L; ++j)
            if (!saved->U[j - 1] || !lp_aligned16(saved->U[j - 1])) return LP_ERR_INVALID_ARG;
    }
    if (!ws || ws_bytes < lp_mlp_score_loss_workspace_bytes(p, B)) return LP_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int dt = p->dtype;
    float *partial = static_cast<float *>(ws);
    char *wt = static_cast<char *>(ws) + lp_align_up(sizeof(float) * kMaxLossBlocks);
    if (B > 0) {
        LpTimedScope timed(LP_KC_SCORE, st);
        const int FV = p->dims[0] / lp_vec_elems(dt);
        const unsigned grid = (unsigned)lp_ceil_div(B * FV, 256);
        if (dt == LP_BF16)
            hipLaunchKernelGGL((edge_product_kernel<lp_bf16_t>), dim3(grid), dim3(256), 0, st, static_cast<const lp_bf16_t *>(HK), n_nodes, FV,
                               B, e_src, e_dst, static_cast<lp_bf16_t *>(saved->X));
        else
            hipLaunchKernelGGL((edge_product_kernel<float>), dim3(grid), dim3(256), 0, st, static_cast<const float *>(HK), n_nodes, FV, B,
                               e_src, e_dst, static_cast<float *>(saved->X));
        LP_TRY(lp_after_launch());
    }
    const void *Uprev = saved->X;
    for (int j = 1; j < L && B > 0; ++j) {
        const int Fi = p->dims[j - 1], Fo = p->dims[j];
        void *WT = wt;
        wt += lp_align_up((size_t)Fi * Fo, 64) * (size_t)lp_elem_bytes(dt);
        LP_TRY(lp_launch_transpose(p->W[j - 1], Fi, Fo, WT, dt, st));
        GemmNtArgs ge;
        ge.dtype = dt;
        ge.fp32_products = p->fp32_products;
        ge.M = (int32_t)B; ge.N = Fo; ge.n_split = Fo;
        ge.A[0] = Uprev; ge.lda[0] = Fi; ge.K[0] = Fi;
        ge.Bt[0][0] = WT; ge.ldb[0] = Fi;
        ge.bias = p->bias[j - 1];
        ge.relu = true;
        ge.C[0] = saved->U[j - 1]; ge.ldc[0] = Fo;
        LP_TRY(lp_launch_gemm_nt(ge, st));
        Uprev = saved->U[j - 1];
    }
    const int F = p->dims[L - 1];
    const int G = group_lanes(F, lp_vec_elems(dt));
    const int nb = loss_blocks(B, G);
    LpTimedScope timed(LP_KC_SCORE, st);   // opened after the products, which time themselves
    if (dt == LP_BF16) launch_out_loss<lp_bf16_t>(G, nb, st, Uprev, p->W[L - 1], p->bias[L - 1], n_nodes, F, B, n_pos_edges, e_src, e_dst, scores, dscore, partial);
    else launch_out_loss<float>(G, nb, st, Uprev, p->W[L - 1], p->bias[L - 1], n_nodes, F, B, n_pos_edges, e_src, e_dst, scores, dscore, partial);
    hipLaunchKernelGGL(mean_finish_kernel, dim3(1), dim3(kThreads), 0, st, partial, nb, B, loss);
    return lp_after_launch();
}

extern "C" size_t lp_mlp_backward_workspace_bytes(const lp_mlp *p, int64_t B) {
    if (check_mlp(p) != LP_OK || B < 0) return 0;
    return carve_backward(nullptr, p, B).bytes;
}

extern "C" int lp_mlp_backward(const lp_mlp *p, const lp_mlp_acts *saved, int64_t B, const float *dscore, lp_mlp_grads *out,
                               void *edge_grad, void *ws, size_t ws_bytes, void *stream) {
    LP_TRY(check_mlp(p));
    if (!saved || !out || B < 0) return LP_ERR_INVALID_ARG;
    if (B >= ((int64_t)1 << 31)) return LP_ERR_OUT_OF_RANGE;
    const int L = p->n_layers;
    for (int j = 0; j < L; ++j)
        if (!out->dW[j] || !out->dbias[j]) return LP_ERR_INVALID_ARG;
    if (B > 0) {
        if (!dscore || !edge_grad || !lp_aligned16(edge_grad) || !saved->X) return LP_ERR_INVALID_ARG;
        for (int j = 1; j < L; ++j)
            if (!saved->U[j - 1]) return LP_ERR_INVALID_ARG;
    }
    if (!ws || ws_bytes < lp_mlp_backward_workspace_bytes(p, B)) return LP_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int dt = p->dtype;
    if (B == 0) {
        for (int j = 0; j < L; ++j) {
            LP_TRY(lp_launch_zero(out->dW[j], (int64_t)p->dims[j] * p->dims[j + 1], st));
            LP_TRY(lp_launch_zero(out->dbias[j], p->dims[j + 1], st));
        }
        return LP_OK;
    }
    const MlpBackwardWs w = carve_backward(ws, p, B);
    // output layer
    const int Fl = p->dims[L - 1];
    const void *Ul = L > 1 ? saved->U[L - 2] : saved->X;
    void *dZ = L > 1 ? w.buf[0] : edge_grad;   // with a single layer dL/dx is ds * w itself
    {
        LpTimedScope timed(LP_KC_OTHER, st);
        const int FV = Fl / lp_vec_elems(dt);
        const unsigned grid = (unsigned)lp_ceil_div(B * FV, 256);
        if (dt == LP_BF16)
            hipLaunchKernelGGL((mlp_out_backward_kernel<lp_bf16_t>), dim3(grid), dim3(256), 0, st, static_cast<const lp_bf16_t *>(Ul),
                               static_cast<const lp_bf16_t *>(p->W[L - 1]), dscore, FV, B, L > 1, w.P, static_cast<lp_bf16_t *>(dZ));
        else
            hipLaunchKernelGGL((mlp_out_backward_kernel<float>), dim3(grid), dim3(256), 0, st, static_cast<const float *>(Ul),
                               static_cast<const float *>(p->W[L - 1]), dscore, FV, B, L > 1, w.P, static_cast<float *>(dZ));
        LP_TRY(lp_after_launch());
    }
    // column sums of P: Fl output-weight gradients, then the output-bias gradient (and three zero columns)
    LP_TRY(lp_launch_colsum(w.P, LP_F32, B, Fl + 4, w.sums, w.colsum_partials, st));
    LP_HIP_TRY(hipMemcpyAsync(out->dW[L - 1], w.sums, sizeof(float) * (size_t)Fl, hipMemcpyDeviceToDevice, st));
    LP_HIP_TRY(hipMemcpyAsync(out->dbias[L - 1], w.sums + Fl, sizeof(float), hipMemcpyDeviceToDevice, st));
    // hidden layers, last to first
    void *other = w.buf[1];
    for (int j = L - 1; j >= 1; --j) {
        const int Fi = p->dims[j - 1], Fo = p->dims[j];
        const void *Uin = j > 1 ? saved->U[j - 2] : saved->X;
        WeightGradArgs wg;   // dW_j = U_{j-1}^T dZ and db_j = column sums of dZ in one pass
        wg.dtype = dt;
        wg.fp32_products = p->fp32_products;
        wg.Kn = (int32_t)B;
        wg.At[1] = Uin; wg.Mw[1] = Fi; wg.lda[1] = Fi; wg.C[1] = out->dW[j - 1];
        wg.B = dZ; wg.Nw = Fo; wg.ldb = Fo;
        wg.dbias = out->dbias[j - 1];
        wg.partials = w.tn_partials; wg.colsum_partials = w.colsum_partials;
        LP_TRY(lp_launch_weight_grads(wg, st));
        void *dst = j > 1 ? other : edge_grad;
        GemmNtArgs ge;
        ge.dtype = dt;
        ge.fp32_products = p->fp32_products;
        ge.M = (int32_t)B; ge.N = Fi; ge.n_split = Fi;
        ge.A[0] = dZ; ge.lda[0] = Fo; ge.K[0] = Fo;
        ge.Bt[0][0] = p->W[j - 1]; ge.ldb[0] = Fo;   // W_j is [Fi, Fo]: row n of it is the n-th row of W_j^T's transpose operand
        ge.C[0] = dst; ge.ldc[0] = Fi;
        LP_TRY(lp_launch_gemm_nt(ge, st));
        if (j > 1) {
            LpTimedScope timed(LP_KC_OTHER, st);
            const int64_t n_vec = B * (Fi / lp_vec_elems(dt));
            const unsigned grid = (unsigned)lp_ceil_div(n_vec, 256);
            if (dt == LP_BF16)
                hipLaunchKernelGGL((relu_gate_kernel<lp_bf16_t>), dim3(grid), dim3(256), 0, st, static_cast<lp_bf16_t *>(dst),
                                   static_cast<const lp_bf16_t *>(Uin), n_vec);
            else
                hipLaunchKernelGGL((relu_gate_kernel<float>), dim3(grid), dim3(256), 0, st, static_cast<float *>(dst),
                                   static_cast<const float *>(Uin), n_vec);
            LP_TRY(lp_after_launch());
            other = dZ;
            dZ = dst;
        }
    }
    return LP_OK;
}
