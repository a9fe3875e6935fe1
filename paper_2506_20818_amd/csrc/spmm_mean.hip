// Sparse neighbourhood aggregation over CSR (the AGG of Eq. 1 of the paper with the mean aggregator, and its
// adjoint over the transposed CSR in the backward pass).
//
//   out[v, :] = rowscale(v) * sum_{u in row v} in[u, :]   (+ addend[v, :])   (zeroed where gate[v, :] <= 0)
//
// One wavefront owns one output row.  A neighbour row of F floats is read by G = F/4 lanes with one 16-byte
// load each (fully coalesced: 64 lanes cover 1 KiB); when G < 64 the wavefront reads 64/G neighbours at once
// and folds the partial sums with xor-shuffles at the end.  Neighbour ids are fetched 64 at a time (coalesced)
// and handed to the lanes that need them through the LDS crossbar (ds_bpermute), four rows in flight per lane.
// Rows are visited in `row_order` (longest first) when given, so that hub rows start early and never form the tail.
#include "lp_internal.h"

namespace {

constexpr int kThreads = 256;
constexpr int kUnroll = 4;

__device__ inline float4 f4_add(float4 a, float4 b) { return make_float4(a.x + b.x, a.y + b.y, a.z + b.z, a.w + b.w); }

// G: lanes per neighbour row (8..64), C: 16-byte chunks per lane (C > 1 only when G == 64 and F > 256)
template <int G, int C, bool W>
__global__ __launch_bounds__(kThreads) void spmm_rows_kernel(SpmmArgs a) {
    constexpr int P = 64 / G;  // neighbours read per step
    const int lane = threadIdx.x & 63;
    const int64_t r = (int64_t)blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);
    if (r >= a.n_rows) return;
    const int32_t v = a.row_order ? a.row_order[r] : (int32_t)r;
    const int sub = lane / G, fl = lane % G;
    const int F4 = a.F >> 2;
    const bool lane_on = fl < F4;  // F/4 need not be a power of two
    const float4 *__restrict__ in4 = reinterpret_cast<const float4 *>(a.in);
    const int32_t lo = a.rowptr[v], hi = a.rowptr[v + 1];

    float4 acc[C];
#pragma unroll
    for (int c = 0; c < C; ++c) acc[c] = make_float4(0.f, 0.f, 0.f, 0.f);

    for (int32_t base = lo; base < hi; base += 64) {
        const int cnt = min(64, hi - base);
        const int32_t mine = lane < cnt ? a.colidx[base + lane] : 0;
        float mine_w = 1.f;
        if (W) mine_w = lane < cnt ? a.w[base + lane] : 0.f;
        for (int j0 = 0; j0 < cnt; j0 += P * kUnroll) {
            float4 x[kUnroll][C];
            float wj[kUnroll];
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                const int j = j0 + u * P + sub;
                const int32_t nb = __shfl(mine, j & 63, 64);
                wj[u] = W ? __shfl(mine_w, j & 63, 64) : 1.f;
                const bool on = lane_on && j < cnt;
#pragma unroll
                for (int c = 0; c < C; ++c) {
                    x[u][c] = make_float4(0.f, 0.f, 0.f, 0.f);
                    if (on && (C == 1 || fl + 64 * c < F4)) x[u][c] = in4[(int64_t)nb * F4 + fl + 64 * c];
                }
            }
#pragma unroll
            for (int u = 0; u < kUnroll; ++u)
#pragma unroll
                for (int c = 0; c < C; ++c) {
                    if (W) {
                        acc[c].x += wj[u] * x[u][c].x;
                        acc[c].y += wj[u] * x[u][c].y;
                        acc[c].z += wj[u] * x[u][c].z;
                        acc[c].w += wj[u] * x[u][c].w;
                    } else {
                        acc[c] = f4_add(acc[c], x[u][c]);
                    }
                }
        }
    }
#pragma unroll
    for (int d = G; d < 64; d <<= 1) {
#pragma unroll
        for (int c = 0; c < C; ++c) {
            acc[c].x += __shfl_xor(acc[c].x, d, 64);
            acc[c].y += __shfl_xor(acc[c].y, d, 64);
            acc[c].z += __shfl_xor(acc[c].z, d, 64);
            acc[c].w += __shfl_xor(acc[c].w, d, 64);
        }
    }
    if (sub != 0 || !lane_on) return;
    const float scale = a.inv_deg ? a.inv_deg[v] : 1.0f;
#pragma unroll
    for (int c = 0; c < C; ++c) {
        const int col4 = fl + 64 * c;
        if (C > 1 && col4 >= F4) break;
        const int64_t o = (int64_t)v * F4 + col4;
        float4 y = make_float4(acc[c].x * scale, acc[c].y * scale, acc[c].z * scale, acc[c].w * scale);
        if (a.addend) y = f4_add(y, reinterpret_cast<const float4 *>(a.addend)[o]);
        if (a.gate) {
            const float4 g = reinterpret_cast<const float4 *>(a.gate)[o];
            y.x = g.x > 0.f ? y.x : 0.f;
            y.y = g.y > 0.f ? y.y : 0.f;
            y.z = g.z > 0.f ? y.z : 0.f;
            y.w = g.w > 0.f ? y.w : 0.f;
        }
        reinterpret_cast<float4 *>(a.out)[o] = y;
    }
}

template <int G, int C>
int launch(const SpmmArgs &a, hipStream_t st) {
    const unsigned grid = (unsigned)lp_ceil_div(a.n_rows, kThreads / 64);
    if (a.w) hipLaunchKernelGGL((spmm_rows_kernel<G, C, true>), dim3(grid), dim3(kThreads), 0, st, a);
    else hipLaunchKernelGGL((spmm_rows_kernel<G, C, false>), dim3(grid), dim3(kThreads), 0, st, a);
    return lp_after_launch();
}

}  // namespace

int lp_launch_spmm(const SpmmArgs &a, hipStream_t st) {
    if (a.n_rows <= 0) return LP_OK;
    if (a.F <= 0 || (a.F & 3)) return LP_ERR_UNSUPPORTED;
    LpTimedScope timed(a.timing_class, st);
    const int F4 = a.F >> 2;
    if (F4 <= 8) return launch<8, 1>(a, st);
    if (F4 <= 16) return launch<16, 1>(a, st);
    if (F4 <= 32) return launch<32, 1>(a, st);
    if (F4 <= 64) return launch<64, 1>(a, st);
    if (F4 <= 128) return launch<64, 2>(a, st);
    if (F4 <= 256) return launch<64, 4>(a, st);
    return LP_ERR_UNSUPPORTED;  // rows wider than 1024 floats
}
