// lp_sgd_step / lp_adam_step: the weight update that closes a training step (Algorithm 1, "Update W <- W - eta
// grad L(W)"; the experiments use Adam with learning rate 0.001, see "Hyperparameters").  All 3K parameter tensors
// of the model (W_self, W_neigh, bias per layer) are updated by ONE launch: blockIdx.y picks the tensor, the x
// dimension strides over its elements.  Arithmetic is fp32; bf16 weights are widened, updated and rounded back
// (nearest even), their moments stay fp32.
#include "lp_internal.h"

#include <cmath>

namespace {

constexpr int kMaxTensors = 3 * LP_MAX_LAYERS;

struct TensorTable {
    void *w[kMaxTensors];         // weights, storage type `bf16[i] ? bfloat16 : float`
    const float *g[kMaxTensors];  // gradients
    float *m[kMaxTensors];        // first moments (Adam)
    float *v[kMaxTensors];        // second moments (Adam)
    int64_t n[kMaxTensors];
    uint8_t bf16[kMaxTensors];
    int count;
};

__device__ __forceinline__ float load_w(const void *w, bool bf16, int64_t i) {
    return bf16 ? lp_bf16_to_f32(static_cast<const lp_bf16_t *>(w)[i]) : static_cast<const float *>(w)[i];
}
__device__ __forceinline__ void store_w(void *w, bool bf16, int64_t i, float x) {
    if (bf16) static_cast<lp_bf16_t *>(w)[i] = lp_f32_to_bf16(x);
    else static_cast<float *>(w)[i] = x;
}

__global__ __launch_bounds__(256) void sgd_kernel(TensorTable t, float lr) {
    const int k = blockIdx.y;
    const int64_t n = t.n[k];
    const bool bf = t.bf16[k] != 0;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x)
        store_w(t.w[k], bf, i, load_w(t.w[k], bf, i) - lr * t.g[k][i]);
}

// c1 = 1/(1 - beta1^t), c2 = 1/(1 - beta2^t), computed on the host in double
__global__ __launch_bounds__(256) void adam_kernel(TensorTable t, float lr, float beta1, float beta2, float eps, float c1, float c2) {
    const int k = blockIdx.y;
    const int64_t n = t.n[k];
    const bool bf = t.bf16[k] != 0;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) {
        const float g = t.g[k][i];
        const float m = beta1 * t.m[k][i] + (1.f - beta1) * g;
        const float v = beta2 * t.v[k][i] + (1.f - beta2) * g * g;
        t.m[k][i] = m;
        t.v[k][i] = v;
        const float step = lr * (m * c1) / (sqrtf(v * c2) + eps);
        store_w(t.w[k], bf, i, load_w(t.w[k], bf, i) - step);
    }
}

int fill_table(const lp_model *m, const lp_grads *g, const lp_opt_state *s, bool need_state, TensorTable &t, int64_t &n_max) {
    if (!m || !g || m->n_layers < 1 || m->n_layers > LP_MAX_LAYERS) return LP_ERR_INVALID_ARG;
    if (m->dtype != LP_F32 && m->dtype != LP_BF16) return LP_ERR_UNSUPPORTED;
    if (m->layer_type != LP_LAYER_SAGE_MEAN && m->layer_type != LP_LAYER_GCN) return LP_ERR_UNSUPPORTED;
    if (!lp_valid_fp32_products(m->fp32_products) || m->reserved_ != 0) return LP_ERR_INVALID_ARG;
    if (need_state && !s) return LP_ERR_INVALID_ARG;
    t.count = 0;
    n_max = 0;
    for (int k = 0; k < m->n_layers; ++k) {
        if (m->dims[k] <= 0 || m->dims[k + 1] <= 0) return LP_ERR_INVALID_ARG;
        const int64_t nw = (int64_t)m->dims[k] * m->dims[k + 1], nb = m->dims[k + 1];
        const void *w[3] = {m->W_self[k], m->W_neigh[k], m->bias[k]};
        const float *gr[3] = {g->dW_self[k], g->dW_neigh[k], g->dbias[k]};
        float *mo[3] = {s ? s->m_W_self[k] : nullptr, s ? s->m_W_neigh[k] : nullptr, s ? s->m_bias[k] : nullptr};
        float *ve[3] = {s ? s->v_W_self[k] : nullptr, s ? s->v_W_neigh[k] : nullptr, s ? s->v_bias[k] : nullptr};
        for (int j = 0; j < 3; ++j) {
            if (j == 0 && m->layer_type == LP_LAYER_GCN) continue;  // a GCN layer has no self weight
            if (!w[j] || !gr[j] || (need_state && (!mo[j] || !ve[j]))) return LP_ERR_INVALID_ARG;
            const int i = t.count++;
            t.w[i] = const_cast<void *>(w[j]);
            t.g[i] = gr[j];
            t.m[i] = mo[j];
            t.v[i] = ve[j];
            t.n[i] = j == 2 ? nb : nw;
            t.bf16[i] = (j != 2 && m->dtype == LP_BF16) ? 1 : 0;  // biases are always fp32
            n_max = t.n[i] > n_max ? t.n[i] : n_max;
        }
    }
    return LP_OK;
}

dim3 grid_for(int64_t n_max, int count) {
    int64_t bx = lp_ceil_div(n_max, 256);
    if (bx > 1024) bx = 1024;
    return dim3((unsigned)bx, (unsigned)count);
}

}  // namespace

// one tensor at a time: parameters that live outside lp_model (the MLP edge predictor's)
extern "C" int lp_adam_update_tensor(void *w, int32_t dtype, const float *grad, float *m, float *v, int64_t n, int64_t t_step, float lr,
                                     float beta1, float beta2, float eps, void *stream) {
    if (!w || !grad || !m || !v || n < 0) return LP_ERR_INVALID_ARG;
    if (dtype != LP_F32 && dtype != LP_BF16) return LP_ERR_UNSUPPORTED;
    if (t_step < 1 || !std::isfinite(lr) || !(beta1 >= 0.f && beta1 < 1.f) || !(beta2 >= 0.f && beta2 < 1.f) || !(eps >= 0.f))
        return LP_ERR_INVALID_ARG;
    if (n == 0) return LP_OK;
    TensorTable t;
    t.count = 1;
    t.w[0] = w; t.g[0] = grad; t.m[0] = m; t.v[0] = v; t.n[0] = n; t.bf16[0] = dtype == LP_BF16 ? 1 : 0;
    const float c1 = (float)(1.0 / (1.0 - std::pow((double)beta1, (double)t_step)));
    const float c2 = (float)(1.0 / (1.0 - std::pow((double)beta2, (double)t_step)));
    hipStream_t st = static_cast<hipStream_t>(stream);
    LpTimedScope timed(LP_KC_OTHER, st);
    hipLaunchKernelGGL(adam_kernel, grid_for(n, 1), dim3(256), 0, st, t, lr, beta1, beta2, eps, c1, c2);
    return lp_after_launch();
}

extern "C" int lp_sgd_update_tensor(void *w, int32_t dtype, const float *grad, int64_t n, float lr, void *stream) {
    if (!w || !grad || n < 0 || !std::isfinite(lr)) return LP_ERR_INVALID_ARG;
    if (dtype != LP_F32 && dtype != LP_BF16) return LP_ERR_UNSUPPORTED;
    if (n == 0) return LP_OK;
    TensorTable t;
    t.count = 1;
    t.w[0] = w; t.g[0] = grad; t.m[0] = nullptr; t.v[0] = nullptr; t.n[0] = n; t.bf16[0] = dtype == LP_BF16 ? 1 : 0;
    hipStream_t st = static_cast<hipStream_t>(stream);
    LpTimedScope timed(LP_KC_OTHER, st);
    hipLaunchKernelGGL(sgd_kernel, grid_for(n, 1), dim3(256), 0, st, t, lr);
    return lp_after_launch();
}

extern "C" int lp_sgd_step(const lp_model *m, const lp_grads *g, float lr, void *stream) {
    TensorTable t;
    int64_t n_max;
    LP_TRY(fill_table(m, g, nullptr, false, t, n_max));
    if (!std::isfinite(lr)) return LP_ERR_INVALID_ARG;
    hipStream_t st = static_cast<hipStream_t>(stream);
    LpTimedScope timed(LP_KC_OTHER, st);
    hipLaunchKernelGGL(sgd_kernel, grid_for(n_max, t.count), dim3(256), 0, st, t, lr);
    return lp_after_launch();
}

extern "C" int lp_adam_step(const lp_model *m, const lp_grads *g, const lp_opt_state *s, int64_t t_step, float lr, float beta1,
                            float beta2, float eps, void *stream) {
    TensorTable t;
    int64_t n_max;
    LP_TRY(fill_table(m, g, s, true, t, n_max));
    if (t_step < 1 || !std::isfinite(lr) || !(beta1 >= 0.f && beta1 < 1.f) || !(beta2 >= 0.f && beta2 < 1.f) || !(eps >= 0.f))
        return LP_ERR_INVALID_ARG;
    const float c1 = (float)(1.0 / (1.0 - std::pow((double)beta1, (double)t_step)));
    const float c2 = (float)(1.0 / (1.0 - std::pow((double)beta2, (double)t_step)));
    hipStream_t st = static_cast<hipStream_t>(stream);
    LpTimedScope timed(LP_KC_OTHER, st);
    hipLaunchKernelGGL(adam_kernel, grid_for(n_max, t.count), dim3(256), 0, st, t, lr, beta1, beta2, eps, c1, c2);
    return lp_after_launch();
}
