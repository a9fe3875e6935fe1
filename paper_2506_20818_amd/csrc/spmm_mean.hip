// Sparse neighbourhood aggregation over CSR (the AGG of Eq. 1 of the paper with the mean aggregator, and its
// adjoint over the transposed CSR in the backward pass).
//
//   out[v, :] = rowscale(v) * sum_{p in row v} w[p] * in[colidx[p], :]   (+ addend[v, :])   (zeroed where gate <= 0)
//
// One wavefront owns one output row.  A neighbour row is read by G lanes with one 16-byte load each (4 floats or
// 8 bfloat16; fully coalesced: 64 lanes cover 1 KiB); when G < 64 the wavefront reads 64/G neighbours at once and
// folds the partial sums with xor-shuffles at the end.  Neighbour ids are fetched 64 at a time (coalesced) and
// handed to the lanes that need them through the LDS crossbar (ds_bpermute), four rows in flight per lane.
// Rows are visited in `row_order` (longest first) when given, so that hub rows start early and never form the tail.
// Sums are always accumulated in fp32, whatever the storage type.
#include "lp_internal.h"

namespace {

constexpr int kThreads = 256;
constexpr int kUnroll = 4;

// T: storage type, G: lanes per neighbour row (8..64), C: 16-byte chunks per lane (C > 1 only when G == 64),
// W: per-entry weights
template <typename T, int G, int C, bool W>
__global__ __launch_bounds__(kThreads) void spmm_rows_kernel(SpmmArgs a) {
    constexpr int P = 64 / G;  // neighbours read per step
    constexpr int VE = LpVec<T>::N;
    const int lane = threadIdx.x & 63;
    const int64_t r = (int64_t)blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);
    if (r >= a.n_rows) return;
    const int32_t v = a.row_order ? a.row_order[r] : (int32_t)r;
    const int sub = lane / G, fl = lane % G;
    const int FV = a.F / VE;           // 16-byte vectors per row
    const bool lane_on = fl < FV;      // F/VE need not be a power of two
    const T *__restrict__ in = static_cast<const T *>(a.in);
    const int32_t lo = a.rowptr[v], hi = a.rowptr[v + 1];

    float acc[C][VE];
#pragma unroll
    for (int c = 0; c < C; ++c)
#pragma unroll
        for (int e = 0; e < VE; ++e) acc[c][e] = 0.f;

    for (int32_t base = lo; base < hi; base += 64) {
        const int cnt = min(64, hi - base);
        const int32_t mine = lane < cnt ? a.colidx[base + lane] : 0;
        float mine_w = 1.f;
        if (W) mine_w = lane < cnt ? a.w[base + lane] : 0.f;
        for (int j0 = 0; j0 < cnt; j0 += P * kUnroll) {
            float x[kUnroll][C][VE];
            float wj[kUnroll];
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                const int j = j0 + u * P + sub;
                const int32_t nb = __shfl(mine, j & 63, 64);
                wj[u] = W ? __shfl(mine_w, j & 63, 64) : 1.f;
                const bool on = lane_on && j < cnt;
#pragma unroll
                for (int c = 0; c < C; ++c) {
#pragma unroll
                    for (int e = 0; e < VE; ++e) x[u][c][e] = 0.f;
                    if (on && (C == 1 || fl + 64 * c < FV)) LpVec<T>::load(in + ((int64_t)nb * FV + fl + 64 * c) * VE, x[u][c]);
                }
            }
#pragma unroll
            for (int u = 0; u < kUnroll; ++u)
#pragma unroll
                for (int c = 0; c < C; ++c)
#pragma unroll
                    for (int e = 0; e < VE; ++e) {
                        if (W) acc[c][e] += wj[u] * x[u][c][e];
                        else acc[c][e] += x[u][c][e];
                    }
        }
    }
#pragma unroll
    for (int d = G; d < 64; d <<= 1)
#pragma unroll
        for (int c = 0; c < C; ++c)
#pragma unroll
            for (int e = 0; e < VE; ++e) acc[c][e] += __shfl_xor(acc[c][e], d, 64);
    if (sub != 0 || !lane_on) return;
    const float scale = a.inv_deg ? a.inv_deg[v] : 1.0f;
#pragma unroll
    for (int c = 0; c < C; ++c) {
        const int colv = fl + 64 * c;
        if (C > 1 && colv >= FV) break;
        const int64_t o = ((int64_t)v * FV + colv) * VE;
        float y[VE];
#pragma unroll
        for (int e = 0; e < VE; ++e) y[e] = acc[c][e] * scale;
        if (a.addend) {
            float t[VE];
            LpVec<T>::load(static_cast<const T *>(a.addend) + o, t);
#pragma unroll
            for (int e = 0; e < VE; ++e) y[e] += t[e];
        }
        if (a.gate) {
            float gt[VE];
            LpVec<T>::load(static_cast<const T *>(a.gate) + o, gt);
#pragma unroll
            for (int e = 0; e < VE; ++e) y[e] = gt[e] > 0.f ? y[e] : 0.f;
        }
        LpVec<T>::store(static_cast<T *>(a.out) + o, y);
    }
}

template <typename T, int G, int C>
int launch(const SpmmArgs &a, hipStream_t st) {
    const unsigned grid = (unsigned)lp_ceil_div(a.n_rows, kThreads / 64);
    if (a.w) hipLaunchKernelGGL((spmm_rows_kernel<T, G, C, true>), dim3(grid), dim3(kThreads), 0, st, a);
    else hipLaunchKernelGGL((spmm_rows_kernel<T, G, C, false>), dim3(grid), dim3(kThreads), 0, st, a);
    return lp_after_launch();
}

template <typename T>
int dispatch(const SpmmArgs &a, hipStream_t st) {
    const int FV = a.F / LpVec<T>::N;
    if (FV <= 8) return launch<T, 8, 1>(a, st);
    if (FV <= 16) return launch<T, 16, 1>(a, st);
    if (FV <= 32) return launch<T, 32, 1>(a, st);
    if (FV <= 64) return launch<T, 64, 1>(a, st);
    if (FV <= 128) return launch<T, 64, 2>(a, st);
    if (FV <= 256) return launch<T, 64, 4>(a, st);
    return LP_ERR_UNSUPPORTED;  // rows wider than 4 KiB
}

}  // namespace

int lp_launch_spmm(const SpmmArgs &a, hipStream_t st) {
    if (a.n_rows <= 0) return LP_OK;
    if (a.F <= 0 || a.F % lp_vec_elems(a.dtype)) return LP_ERR_UNSUPPORTED;
    LpTimedScope timed(a.timing_class, st);
    if (a.dtype == LP_BF16) return dispatch<lp_bf16_t>(a, st);
    if (a.dtype == LP_F32) return dispatch<float>(a, st);
    return LP_ERR_UNSUPPORTED;
}
