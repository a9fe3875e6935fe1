// Sparse neighbourhood aggregation over CSR (the AGG of Eq. 1 of the paper with the mean aggregator, and its
// adjoint over the transposed CSR in the backward pass).
//
//   out[v, :] = rowscale(v) * sum_{p in row v} w[p] * in[colidx[p], :]   (+ addend[v, :])   (zeroed where gate <= 0)
//
// Ordinary rows: one wavefront owns one output row.  A neighbour row is read by G lanes with one 16-byte load each
// (4 floats or 8 bfloat16; fully coalesced: 64 lanes cover 1 KiB); when G < 64 the wavefront reads 64/G neighbours
// at once and folds the partial sums with xor-shuffles at the end.  Neighbour ids are fetched 64 at a time
// (coalesced) and handed to the lanes that need them through the LDS crossbar (ds_bpermute), several rows in flight
// per lane.  Rows are visited in `row_order` (longest first) when given, so that long rows start early.
//
// Hub rows: a single wavefront keeps only a few KiB in flight, so a row with thousands of neighbours would take
// longer than the rest of the launch together (power-law graphs have such rows).  When the caller supplies a queue,
// a wavefront that meets a row of at least kLongRow neighbours appends it to the queue instead, and a second launch
// gives every queued row to a whole workgroup of sixteen wavefronts: wavefront w takes the 64-neighbour blocks
// w, w+16, ... and the sixteen partial sums are added in wavefront order through LDS.  Which workgroup serves which
// queued row depends on scheduling; the value computed for a row does not.
// Sums are always accumulated in fp32, whatever the storage type.
#include "lp_internal.h"

namespace {

constexpr int kThreads = 256;
constexpr int kLongThreads = 1024;
constexpr int kLongWaves = kLongThreads / 64;

// Accumulates the 64-neighbour blocks first, first + stride, ... (< hi) of one CSR row into acc.
// T: storage type, G: lanes per neighbour row (8..64), C: 16-byte chunks per lane (C > 1 only when G == 64),
// W: 0 = no weights, 1 = one scalar per entry, 2 = one row of `entry_rows` per entry (multiplied element-wise),
// U: neighbour rows in flight per lane.
template <typename T, int G, int C, int W, int U>
__device__ __forceinline__ void accumulate_blocks(const SpmmArgs &a, const T *__restrict__ in, int32_t first, int32_t hi,
                                                  int32_t stride, int lane, float (&acc)[C][LpVec<T>::N]) {
    constexpr int P = 64 / G;  // neighbours read per step
    constexpr int VE = LpVec<T>::N;
    const int sub = lane / G, fl = lane % G;
    const int FV = a.F / VE;           // 16-byte vectors per row
    const bool lane_on = fl < FV;      // F/VE need not be a power of two
    for (int32_t base = first; base < hi; base += stride) {
        const int cnt = min(64, hi - base);
        int32_t mine = lane < cnt ? a.colidx[base + lane] : 0;
        float mine_w = 1.f;
        if (W == 1) {
            mine_w = 0.f;
            if (lane < cnt) {
                if (!a.sym_norm) mine_w = a.w[base + lane];
                else if (a.sym_col_cnt) mine_w = a.sym_col_cnt[mine] / sqrtf(a.inv_deg[mine]);   // the column has this entry: inv_deg > 0
                else mine_w = sqrtf(a.inv_deg[mine]);
            }
        }
        int32_t mine_row = 0;
        if (W == 2) mine_row = lane < cnt ? a.entry_row_index[base + lane] : 0;
        if (a.in_index) mine = lane < cnt ? a.in_index[mine] : -1;  // row of `in` that holds the neighbour, < 0: a zero row
        for (int j0 = 0; j0 < cnt; j0 += P * U) {
            float x[U][C][VE];
            float rw[W == 2 ? U : 1][C][VE];
            float wj[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int j = j0 + u * P + sub;
                const int32_t nb = __shfl(mine, j & 63, 64);
                wj[u] = W == 1 ? __shfl(mine_w, j & 63, 64) : 1.f;
                const int32_t er = W == 2 ? __shfl(mine_row, j & 63, 64) : 0;
                const bool on = lane_on && j < cnt && nb >= 0;
#pragma unroll
                for (int c = 0; c < C; ++c) {
#pragma unroll
                    for (int e = 0; e < VE; ++e) x[u][c][e] = 0.f;
                    if (W == 2) {
#pragma unroll
                        for (int e = 0; e < VE; ++e) rw[u][c][e] = 0.f;
                    }
                    if (on && (C == 1 || fl + 64 * c < FV)) {
                        LpVec<T>::load(in + ((int64_t)nb * FV + fl + 64 * c) * VE, x[u][c]);
                        if (W == 2) LpVec<T>::load(static_cast<const T *>(a.entry_rows) + ((int64_t)er * FV + fl + 64 * c) * VE, rw[u][c]);
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int c = 0; c < C; ++c)
#pragma unroll
                    for (int e = 0; e < VE; ++e) {
                        if (W == 1) acc[c][e] += wj[u] * x[u][c][e];
                        else if (W == 2) acc[c][e] += rw[u][c][e] * x[u][c][e];
                        else acc[c][e] += x[u][c][e];
                    }
        }
    }
}

// Lanes with the same position inside their group of G add up their partial sums (all lanes end with the total).
template <int G, int C, int VE>
__device__ __forceinline__ void fold_groups(float (&acc)[C][VE]) {
#pragma unroll
    for (int d = G; d < 64; d <<= 1)
#pragma unroll
        for (int c = 0; c < C; ++c)
#pragma unroll
            for (int e = 0; e < VE; ++e) acc[c][e] += __shfl_xor(acc[c][e], d, 64);
}

// What the sum of row v is multiplied by: 1/deg (mean), sqrt(1/deg) (symmetric normalisation), or, for a sampled
// subset of the neighbours, (1/|S|) / sqrt(1/deg).
__device__ __forceinline__ float row_scale(const SpmmArgs &a, int32_t v) {
    if (!a.inv_deg) return 1.0f;
    const float id = a.inv_deg[v];
    if (!a.sym_norm) return id;
    if (a.sym_row_cnt) return id > 0.f ? a.sym_row_cnt[v] / sqrtf(id) : 0.f;
    return sqrtf(id);
}

// Scale, optional addend, optional gate, store: 16 bytes of output row v starting at vector column colv.
template <typename T>
__device__ __forceinline__ void finish_vector(const SpmmArgs &a, int32_t v, int FV, int colv, float scale,
                                              const float (&sum)[LpVec<T>::N]) {
    constexpr int VE = LpVec<T>::N;
    const int64_t o = ((int64_t)v * FV + colv) * VE;
    float y[VE];
#pragma unroll
    for (int e = 0; e < VE; ++e) y[e] = sum[e] * scale;
    if (a.addend) {
        int32_t ar = a.in_index ? a.in_index[v] : v;
        if (a.addend_rows_dev && v >= *a.addend_rows_dev) ar = -1;
        if (ar >= 0) {
            float t[VE];
            LpVec<T>::load(static_cast<const T *>(a.addend) + ((int64_t)ar * FV + colv) * VE, t);
#pragma unroll
            for (int e = 0; e < VE; ++e) y[e] += t[e];
        }
    }
    if (a.gate) {
        float gt[VE];
        LpVec<T>::load(static_cast<const T *>(a.gate) + o, gt);
#pragma unroll
        for (int e = 0; e < VE; ++e) y[e] = gt[e] > 0.f ? y[e] : 0.f;
    }
    LpVec<T>::store_streaming(static_cast<T *>(a.out) + o, y);   // written once, read by a later kernel: leave the caches to the gathered rows
}

template <typename T, int G, int C, int W>
__global__ __launch_bounds__(kThreads) void spmm_rows_kernel(SpmmArgs a) {
    constexpr int VE = LpVec<T>::N;
    const int lane = threadIdx.x & 63;
    const int64_t r = (int64_t)blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);
    if (r >= a.n_rows || (a.n_rows_dev && r >= *a.n_rows_dev)) return;
    const int32_t v = a.row_order ? a.row_order[r] : (int32_t)r;
    const int sub = lane / G, fl = lane % G;
    const int FV = a.F / VE;
    const int32_t lo = a.rowptr[v], hi = a.rowptr[v + 1];
    if (a.long_queue && hi - lo >= a.long_threshold) {  // a hub: leave it to a whole workgroup of the second launch
        if (lane == 0) a.long_queue[1 + atomicAdd(a.long_queue, 1)] = v;
        return;
    }

    float acc[C][VE];
#pragma unroll
    for (int c = 0; c < C; ++c)
#pragma unroll
        for (int e = 0; e < VE; ++e) acc[c][e] = 0.f;
    const float scale = row_scale(a, v);   // requested before the gathers, not after them: one memory latency less per row
    accumulate_blocks<T, G, C, W, 4>(a, static_cast<const T *>(a.in), lo, hi, 64, lane, acc);
    fold_groups<G, C, VE>(acc);
    if (sub != 0 || fl >= FV) return;
#pragma unroll
    for (int c = 0; c < C; ++c) {
        const int colv = fl + 64 * c;
        if (C > 1 && colv >= FV) break;
        finish_vector<T>(a, v, FV, colv, scale, acc[c]);
    }
}

// One workgroup of sixteen wavefronts per queued row; workgroup b serves queue entries b, b + gridDim.x, ...
template <typename T, int G, int C, int W>
__global__ __launch_bounds__(kLongThreads) void spmm_long_rows_kernel(SpmmArgs a) {
    constexpr int VE = LpVec<T>::N;
    constexpr int U = C == 1 ? 8 : 4;
    __shared__ float red[kLongWaves][G][VE];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int sub = lane / G, fl = lane % G;
    const int FV = a.F / VE;
    const int32_t n_queued = a.long_queue[0];
    for (int32_t i = blockIdx.x; i < n_queued; i += gridDim.x) {  // uniform over the workgroup
        const int32_t v = a.long_queue[1 + i];
        const int32_t lo = a.rowptr[v], hi = a.rowptr[v + 1];
        float acc[C][VE];
#pragma unroll
        for (int c = 0; c < C; ++c)
#pragma unroll
            for (int e = 0; e < VE; ++e) acc[c][e] = 0.f;
        accumulate_blocks<T, G, C, W, U>(a, static_cast<const T *>(a.in), lo + 64 * wave, hi, 64 * kLongWaves, lane, acc);
        fold_groups<G, C, VE>(acc);
        const float scale = row_scale(a, v);
#pragma unroll
        for (int c = 0; c < C; ++c) {
            if (sub == 0) {
#pragma unroll
                for (int e = 0; e < VE; ++e) red[wave][fl][e] = acc[c][e];
            }
            __syncthreads();
            const int colv = fl + 64 * c;
            if (wave == 0 && sub == 0 && colv < FV) {
                float sum[VE];
#pragma unroll
                for (int e = 0; e < VE; ++e) sum[e] = red[0][fl][e];
#pragma unroll
                for (int w = 1; w < kLongWaves; ++w)
#pragma unroll
                    for (int e = 0; e < VE; ++e) sum[e] += red[w][fl][e];
                finish_vector<T>(a, v, FV, colv, scale, sum);
            }
            __syncthreads();
        }
    }
}

template <typename T, int G, int C>
int launch(const SpmmArgs &a, hipStream_t st) {
    const unsigned grid = (unsigned)lp_ceil_div(a.n_rows, kThreads / 64);
    const int mode = a.entry_rows ? 2 : ((a.w || a.sym_norm) ? 1 : 0);
    if (mode == 2) hipLaunchKernelGGL((spmm_rows_kernel<T, G, C, 2>), dim3(grid), dim3(kThreads), 0, st, a);
    else if (mode == 1) hipLaunchKernelGGL((spmm_rows_kernel<T, G, C, 1>), dim3(grid), dim3(kThreads), 0, st, a);
    else hipLaunchKernelGGL((spmm_rows_kernel<T, G, C, 0>), dim3(grid), dim3(kThreads), 0, st, a);
    if (a.long_queue) {
        // no more rows can be queued than fit the entry count; two workgroups per compute unit walk the queue
        const int64_t most = a.n_entries / a.long_threshold;
        const int64_t slots = 2 * (int64_t)lp_compute_units();
        const unsigned lgrid = (unsigned)(most < slots ? most : slots);
        if (lgrid > 0) {
            if (mode == 2) hipLaunchKernelGGL((spmm_long_rows_kernel<T, G, C, 2>), dim3(lgrid), dim3(kLongThreads), 0, st, a);
            else if (mode == 1) hipLaunchKernelGGL((spmm_long_rows_kernel<T, G, C, 1>), dim3(lgrid), dim3(kLongThreads), 0, st, a);
            else hipLaunchKernelGGL((spmm_long_rows_kernel<T, G, C, 0>), dim3(lgrid), dim3(kLongThreads), 0, st, a);
        }
    }
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

size_t lp_spmm_queue_bytes(int32_t n_rows) { return lp_align_up(sizeof(int32_t) * ((size_t)(n_rows > 0 ? n_rows : 0) + 1)); }

int lp_launch_spmm(const SpmmArgs &args, hipStream_t st) {
    if (args.n_rows <= 0) return LP_OK;
    if (args.F <= 0 || args.F % lp_vec_elems(args.dtype)) return LP_ERR_UNSUPPORTED;
    if (args.sym_norm && !args.inv_deg) return LP_ERR_INVALID_ARG;
    if (args.entry_rows && !args.entry_row_index) return LP_ERR_INVALID_ARG;
    SpmmArgs a = args;
    a.long_threshold = kSpmmLongRow;
    if (a.n_entries < a.long_threshold) a.long_queue = nullptr;  // no row can be that long
    if (a.long_queue) LP_TRY(lp_launch_zero(reinterpret_cast<float *>(a.long_queue), 1, st));  // queue length
    LpTimedScope timed(a.timing_class, st);
    if (a.dtype == LP_BF16) return dispatch<lp_bf16_t>(a, st);
    if (a.dtype == LP_F32) return dispatch<float>(a, st);
    return LP_ERR_UNSUPPORTED;
}
