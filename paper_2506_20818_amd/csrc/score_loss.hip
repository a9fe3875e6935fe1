// lp_score_loss: dot-product edge scores (Eq. 2 of the paper), binary cross-entropy with labels 1/0 and the
// batch mean (Algorithm 1, per-edge loop and "Compute L^i"; Sec. IV-B last paragraph), plus dL/ds.
//
// A group of G lanes (power of two, at most a wavefront) owns one edge: each lane loads 16 bytes (4 floats or
// 8 bfloat16) of both
// endpoint rows, and the products are summed across the group with xor-shuffles (a segmented reduction inside
// the wavefront).  The loss is reduced block by block and then by one block, always in the same order.
#include "lp_internal.h"

#include <mutex>

constexpr int kThreads = 256;
constexpr int kMaxLossBlocks = 2048;

// Scratch of lp_score_loss_noalloc: the per-block partial sums of the loss, one float per block (8 KiB).  Each GPU
// that the library runs on holds its own copy of this array at its own address until the process ends.  In host
// code the name below is only a stand-in for the symbol, not a device address: the address is looked up once per
// device with hipGetSymbolAddress and only that pointer is ever handed to a kernel.
static __device__ __align__(256) float scratch[kMaxLossBlocks];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
float *g_scratch_ptr[kMaxDevices] = {};

// Device address of `scratch` on the current device (looked up on the first call per device); nullptr on failure.
float *scratch_of_current_device() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        float *p = nullptr;
        if (hipGetSymbolAddress(reinterpret_cast<void **>(&p), HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
        g_scratch_ptr[dev] = p;
    }
    return g_scratch_ptr[dev];
}

template <int G>
__device__ inline float group_sum(float v) {
#pragma unroll
    for (int d = G >> 1; d >= 1; d >>= 1) v += __shfl_xor(v, d, 64);
    return v;
}

template <typename T, int G>
__global__ __launch_bounds__(kThreads) void score_loss_kernel(const T *__restrict__ H, int32_t n_nodes, int32_t F,
                                                              int64_t B, int64_t n_pos, const int32_t *__restrict__ e_src,
                                                              const int32_t *__restrict__ e_dst, float *__restrict__ scores,
                                                              float *__restrict__ dscore, float *__restrict__ partial,
                                                              int32_t *__restrict__ n_invalid) {
    __shared__ float red[kThreads / 64];
    const int sub = threadIdx.x % G;
    const int64_t groups_per_block = kThreads / G;
    const int64_t gid = (int64_t)blockIdx.x * groups_per_block + threadIdx.x / G;
    const int64_t n_groups = (int64_t)gridDim.x * groups_per_block;
    const float invB = 1.0f / (float)B;
    constexpr int VE = LpVec<T>::N;
    const int FV = F / VE;
    float acc = 0.0f;
    for (int64_t e = gid; e < B; e += n_groups) {
        const int32_t u = e_src[e], v = e_dst[e];
        const bool ok = u >= 0 && u < n_nodes && v >= 0 && v < n_nodes;
        float s = 0.0f;
        if (ok) {
            const T *hu = H + (int64_t)u * F, *hv = H + (int64_t)v * F;
            for (int j = sub; j < FV; j += G) {
                float a[VE], b[VE];
                LpVec<T>::load(hu + j * VE, a);
                LpVec<T>::load(hv + j * VE, b);
#pragma unroll
                for (int e = 0; e < VE; ++e) s += a[e] * b[e];
            }
        }
        s = group_sum<G>(s);
        if (sub == 0) {
            const float y = e < n_pos ? 1.0f : 0.0f;
            const float ex = expf(-fabsf(s));
            const float ell = fmaxf(s, 0.0f) - y * s + log1pf(ex);
            const float sig = s >= 0.0f ? 1.0f / (1.0f + ex) : ex / (1.0f + ex);
            scores[e] = s;
            if (dscore) dscore[e] = ok ? (sig - y) * invB : 0.0f;
            if (ok) acc += ell;
            else if (n_invalid) atomicAdd(n_invalid, 1);   // an integer count: the same on every run
        }
    }
    // block sum in a fixed order
    acc = group_sum<64>(acc);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) partial[blockIdx.x] = (red[0] + red[1]) + (red[2] + red[3]);
}

__global__ __launch_bounds__(kThreads) void loss_finish_kernel(const float *__restrict__ partial, int n, int64_t B,
                                                               float *__restrict__ loss) {
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

int loss_blocks(int64_t B, int G) {
    const int64_t groups_per_block = kThreads / G;
    int64_t nb = lp_ceil_div(B, groups_per_block * 4);  // about four edges per group
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
void launch_score(int G, int nb, hipStream_t st, const void *HK, int32_t n_nodes, int32_t F, int64_t B, int64_t n_pos,
                  const int32_t *e_src, const int32_t *e_dst, float *scores, float *dscore, float *partial, int32_t *n_invalid) {
    const T *H = static_cast<const T *>(HK);
    switch (G) {
        case 8: hipLaunchKernelGGL((score_loss_kernel<T, 8>), dim3(nb), dim3(kThreads), 0, st, H, n_nodes, F, B, n_pos, e_src, e_dst, scores, dscore, partial, n_invalid); break;
        case 16: hipLaunchKernelGGL((score_loss_kernel<T, 16>), dim3(nb), dim3(kThreads), 0, st, H, n_nodes, F, B, n_pos, e_src, e_dst, scores, dscore, partial, n_invalid); break;
        case 32: hipLaunchKernelGGL((score_loss_kernel<T, 32>), dim3(nb), dim3(kThreads), 0, st, H, n_nodes, F, B, n_pos, e_src, e_dst, scores, dscore, partial, n_invalid); break;
        default: hipLaunchKernelGGL((score_loss_kernel<T, 64>), dim3(nb), dim3(kThreads), 0, st, H, n_nodes, F, B, n_pos, e_src, e_dst, scores, dscore, partial, n_invalid);
    }
}

}  // namespace

extern "C" size_t lp_score_loss_workspace_bytes(int64_t B) {
    (void)B;
    return sizeof(float) * kMaxLossBlocks;
}

namespace {

int check_score_args(const void *HK, int32_t n_nodes, int32_t F, int32_t dtype, int64_t B, int64_t n_pos_edges,
                     const int32_t *e_src, const int32_t *e_dst, const float *scores, const float *loss) {
    if (!HK || n_nodes <= 0 || F <= 0 || B < 0 || n_pos_edges < 0 || n_pos_edges > B || !loss) return LP_ERR_INVALID_ARG;
    if (B > 0 && (!e_src || !e_dst || !scores)) return LP_ERR_INVALID_ARG;
    if ((dtype != LP_F32 && dtype != LP_BF16) || F % lp_vec_elems(dtype)) return LP_ERR_UNSUPPORTED;
    if (!lp_aligned16(HK)) return LP_ERR_INVALID_ARG;
    if (B >= ((int64_t)1 << 31)) return LP_ERR_OUT_OF_RANGE;
    return LP_OK;
}

// Both entry points: `partial` holds at least kMaxLossBlocks floats; the first `nb` are overwritten by the scoring
// kernel (every block writes its sum) and only those are read by the finishing kernel, so nothing needs clearing.
int run_score_loss(const void *HK, int32_t n_nodes, int32_t F, int32_t dtype, int64_t B, int64_t n_pos_edges,
                   const int32_t *e_src, const int32_t *e_dst, float *scores, float *loss, float *dscore, int32_t *n_invalid,
                   float *partial, hipStream_t st) {
    const int G = group_lanes(F, lp_vec_elems(dtype));
    const int nb = loss_blocks(B, G);
    LpTimedScope timed(LP_KC_SCORE, st);
    if (dtype == LP_BF16) launch_score<lp_bf16_t>(G, nb, st, HK, n_nodes, F, B, n_pos_edges, e_src, e_dst, scores, dscore, partial, n_invalid);
    else launch_score<float>(G, nb, st, HK, n_nodes, F, B, n_pos_edges, e_src, e_dst, scores, dscore, partial, n_invalid);
    hipLaunchKernelGGL(loss_finish_kernel, dim3(1), dim3(kThreads), 0, st, partial, nb, B, loss);
    return lp_after_launch();
}

}  // namespace

extern "C" int lp_score_loss(const void *HK, int32_t n_nodes, int32_t F, int32_t dtype, int64_t B, int64_t n_pos_edges,
                             const int32_t *e_src, const int32_t *e_dst, float *scores, float *loss, float *dscore,
                             int32_t *n_invalid, void *ws, size_t ws_bytes, void *stream) {
    LP_TRY(check_score_args(HK, n_nodes, F, dtype, B, n_pos_edges, e_src, e_dst, scores, loss));
    if (!ws || ws_bytes < lp_score_loss_workspace_bytes(B)) return LP_ERR_WORKSPACE;
    return run_score_loss(HK, n_nodes, F, dtype, B, n_pos_edges, e_src, e_dst, scores, loss, dscore, n_invalid,
                          static_cast<float *>(ws), static_cast<hipStream_t>(stream));
}

extern "C" int lp_score_loss_noalloc(const void *HK, int32_t n_nodes, int32_t F, int32_t dtype, int64_t B,
                                     int64_t n_pos_edges, const int32_t *e_src, const int32_t *e_dst, float *scores,
                                     float *loss, float *dscore, int32_t *n_invalid, void *stream) {
    LP_TRY(check_score_args(HK, n_nodes, F, dtype, B, n_pos_edges, e_src, e_dst, scores, loss));
    if (B > LP_SCORE_LOSS_NOALLOC_MAX_EDGES) return LP_ERR_OUT_OF_RANGE;
    float *partial = scratch_of_current_device();   // the device address, never the array's name
    if (!partial) return LP_ERR_HIP;
    return run_score_loss(HK, n_nodes, F, dtype, B, n_pos_edges, e_src, e_dst, scores, loss, dscore, n_invalid, partial,
                          static_cast<hipStream_t>(stream));
}
