// Sparse neighbourhood aggregation over CSR (the AGG of Eq. 1 of the paper with the mean aggregator, and its
// adjoint over the transposed CSR in the backward pass).
//
//   out[v, :] = rowscale(v) * sum_{p in row v} w[p] * in[colidx[p], :]   (+ addend[v, :])   (zeroed where gate <= 0)
//
// Ordinary rows: one wavefront owns one output row.  A neighbour row is read by G lanes with one 16-byte load each
// (4 floats or 8 bfloat16; fully coalesced: 64 lanes cover 1 KiB); when G < 64 the wavefront reads 64/G neighbours
// at once and folds the partial sums with xor-shuffles at the end.  Neighbour ids are fetched 64 at a time
// (coalesced) and handed to the lanes that need them through the LDS crossbar (ds_bpermute), several rows in flight
// per lane.  Rows are visited in `row_order` when given (lp_build_csr lists rows of 64 and more entries first, by
// decreasing size class, then all others by ascending id), so that long rows start early.
//
// Hub rows: a single wavefront keeps only a few KiB in flight, so a row with thousands of neighbours would take
// longer than the rest of the launch together (power-law graphs have such rows).  When the caller supplies a queue,
// a wavefront that meets a row of at least kLongRow neighbours appends it to the queue instead.  The queued rows are
// then cut into tasks of at most `seg` entries (a multiple of 1024 chosen so that about two thousand tasks result:
// a row of fifteen thousand entries served by one workgroup would otherwise still be running long after everything
// else has finished, every workgroup getting the same small share of the memory system).  A task goes to a workgroup
// of sixteen wavefronts: wavefront w takes the 64-neighbour blocks w, w+16, ... of the task and the sixteen partial
// sums are added in wavefront order through LDS.  A row that is a single task is finished there; the tasks of a longer
// row leave fp32 partial rows in scratch memory and a last small kernel adds them in task order and finishes the
// row.  The plan depends only on the row lengths and on the order in which rows were queued; the latter changes which
// scratch slot a row uses, never the order of any sum, so results are the same bits on every run.
// Sums are always accumulated in fp32, whatever the storage type.
#include "lp_internal.h"

namespace {

constexpr int kThreads = 256;
// Rows per workgroup of the row kernel.  One (64 threads) where row lengths vary: the wavefronts of a larger workgroup
// hold their slots until its longest row is done, which cost 1-8 % on graphs whose neighbouring rows differ much in
// length (measured with 128 and 256 threads).  Four (256 threads) where the caller passes no queue for long rows,
// i.e. knows its rows to be short (sampled neighbourhoods, at most the fan-out): there the workgroup launches
// themselves are the cost (+12 % on the sampled step's aggregations with one row per workgroup).
constexpr int kRowThreads = 64;
constexpr int kShortRowThreads = 256;
constexpr int kLongThreads = 1024;
constexpr int kLongWaves = kLongThreads / 64;
constexpr int kLongHeader = 64;                        // words ahead of the queued rows (count, seg, tasks, slots)
constexpr int kLongTargetTasks = 2048;                 // aimed-at number of tasks of one launch
constexpr int kLongSlots = 2 * kLongTargetTasks;       // partial rows that can be live: see plan_long_rows_kernel

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
                if (!a.sym_norm) mine_w = a.col_w ? a.col_w[mine] : a.w[base + lane];
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

template <typename T, int G, int C, int W, int RT>
__global__ __launch_bounds__(RT) void spmm_rows_kernel(SpmmArgs a) {
    constexpr int VE = LpVec<T>::N;
    const int lane = threadIdx.x & 63;
    const int64_t r = (int64_t)blockIdx.x * (RT / 64) + (threadIdx.x >> 6);
    if (r >= a.n_rows || (a.n_rows_dev && r >= *a.n_rows_dev)) return;
    const int32_t v = a.row_order ? a.row_order[r] : (int32_t)r;
    const int sub = lane / G, fl = lane % G;
    const int FV = a.F / VE;
    const int32_t lo = a.rowptr[v], hi = a.rowptr[v + 1];
    if (a.long_queue && hi - lo >= a.long_threshold) {  // a hub: leave it to whole workgroups of the later launches
        if (lane == 0) a.long_queue[kLongHeader + atomicAdd(a.long_queue, 1)] = v;
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

// ---- queued rows.  Layout of the queue workspace (int32 words): [0] number of queued rows, [1] seg, [2] number of
// tasks, [3] number of scratch slots in use, [4] tasks handed out so far; then rows [cap], task_base [cap + 1], slot_base [cap], each padded to a
// multiple of 64 words, cap = n_rows; then the scratch slots (kLongSlots x F floats).

struct LongQueue {
    int32_t *head, *rows, *task_base, *slot_base;
    float *slots;
};
__host__ __device__ inline size_t long_words(int32_t cap) { return ((size_t)cap + 1 + 63) / 64 * 64; }
__host__ __device__ inline LongQueue long_queue_of(int32_t *q, int32_t cap) {
    LongQueue l;
    l.head = q;
    l.rows = q + kLongHeader;
    l.task_base = l.rows + long_words(cap);
    l.slot_base = l.task_base + long_words(cap);
    l.slots = reinterpret_cast<float *>(l.slot_base + long_words(cap));
    return l;
}

// One workgroup: seg from the total length of the queued rows, then the running task and slot counts in queue order.
// Rows of more than seg entries number at most total / seg <= kLongTargetTasks and have at most total / seg + their
// number <= 2 kLongTargetTasks tasks together: kLongSlots slots always suffice.
__global__ __launch_bounds__(1024) void plan_long_rows_kernel(const int32_t *__restrict__ rowptr, int32_t *q, int32_t cap) {
    __shared__ long long red[1024];
    const LongQueue l = long_queue_of(q, cap);
    const int32_t n = l.head[0];
    long long total = 0;
    for (int32_t i = threadIdx.x; i < n; i += 1024) {
        const int32_t v = l.rows[i];
        total += rowptr[v + 1] - rowptr[v];
    }
    red[threadIdx.x] = total;
    __syncthreads();
    for (int d = 512; d >= 1; d >>= 1) {
        if ((int)threadIdx.x < d) red[threadIdx.x] += red[threadIdx.x + d];
        __syncthreads();
    }
    total = red[0];
    __syncthreads();
    long long want = (total + kLongTargetTasks - 1) / kLongTargetTasks;
    const int32_t seg = (int32_t)((want < 1024 ? 1024 : (want + 1023) / 1024 * 1024));
    // thread t owns the queue entries [t * per, (t + 1) * per): its own totals, one scan over the 1024 threads, then
    // the running counts of its entries
    int32_t *cnt = reinterpret_cast<int32_t *>(red);          // [0..1023] tasks, [1024..2047] slots per thread
    const int32_t per = (n + 1023) / 1024;
    const int32_t first = (int32_t)threadIdx.x * per;
    const int32_t last = min(n, first + per);
    int32_t tasks = 0, slots = 0;
    for (int32_t i = first; i < last; ++i) {
        const int32_t v = l.rows[i];
        const int32_t t = (rowptr[v + 1] - rowptr[v] + seg - 1) / seg;
        tasks += t;
        slots += t > 1 ? t : 0;
    }
    cnt[threadIdx.x] = tasks;
    cnt[1024 + threadIdx.x] = slots;
    __syncthreads();
    for (int d = 1; d < 1024; d <<= 1) {                     // inclusive scans of both counts
        const int32_t a = (int)threadIdx.x >= d ? cnt[threadIdx.x - d] : 0;
        const int32_t b = (int)threadIdx.x >= d ? cnt[1024 + threadIdx.x - d] : 0;
        __syncthreads();
        cnt[threadIdx.x] += a;
        cnt[1024 + threadIdx.x] += b;
        __syncthreads();
    }
    int32_t tb = cnt[threadIdx.x] - tasks, sb = cnt[1024 + threadIdx.x] - slots;
    for (int32_t i = first; i < last; ++i) {
        const int32_t v = l.rows[i];
        const int32_t t = (rowptr[v + 1] - rowptr[v] + seg - 1) / seg;
        l.task_base[i] = tb;
        l.slot_base[i] = sb;
        tb += t;
        sb += t > 1 ? t : 0;
    }
    if (threadIdx.x == 1023) {
        l.task_base[n] = cnt[1023];
        l.head[1] = seg;
        l.head[2] = cnt[1023];
        l.head[3] = cnt[2047];
        l.head[4] = 0;          // the task counter of spmm_long_rows_kernel
    }
}

// One workgroup of sixteen wavefronts per task.
template <typename T, int G, int C, int W>
__global__ __launch_bounds__(kLongThreads) void spmm_long_rows_kernel(SpmmArgs a) {
    constexpr int VE = LpVec<T>::N;
    constexpr int U = C == 1 ? 8 : 4;
    __shared__ float red[kLongWaves][G][VE];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int sub = lane / G, fl = lane % G;
    const int FV = a.F / VE;
    const LongQueue l = long_queue_of(a.long_queue, a.n_rows);
    const int32_t n_queued = l.head[0], seg = l.head[1], n_tasks = l.head[2];
    // Tasks differ in length (a row of 512 entries is one task, so is a piece of seg entries), so a workgroup takes
    // the next task from a counter when it is done with the last one.  Which workgroup serves a task changes
    // nothing in the result: every task owns its output row or its scratch slot.
    __shared__ int32_t next_task;
    for (;;) {
        if (threadIdx.x == 0) next_task = atomicAdd(&l.head[4], 1);
        __syncthreads();
        const int32_t t = next_task;                              // uniform over the workgroup
        __syncthreads();
        if (t >= n_tasks) break;
        int32_t lo_i = 0, hi_i = n_queued;                        // last queue entry i with task_base[i] <= t
        while (hi_i - lo_i > 1) {
            const int32_t mid = (lo_i + hi_i) >> 1;
            if (l.task_base[mid] <= t) lo_i = mid; else hi_i = mid;
        }
        const int32_t v = l.rows[lo_i];
        const int32_t part = t - l.task_base[lo_i];
        const int32_t row_lo = a.rowptr[v], row_hi = a.rowptr[v + 1];
        const bool whole = row_hi - row_lo <= seg;                // the row is this one task
        const int32_t lo = row_lo + part * seg;
        const int32_t hi = min(row_hi, lo + seg);
        float acc[C][VE];
#pragma unroll
        for (int c = 0; c < C; ++c)
#pragma unroll
            for (int e = 0; e < VE; ++e) acc[c][e] = 0.f;
        accumulate_blocks<T, G, C, W, U>(a, static_cast<const T *>(a.in), lo + 64 * wave, hi, 64 * kLongWaves, lane, acc);
        fold_groups<G, C, VE>(acc);
        const float scale = whole ? row_scale(a, v) : 1.f;
        float *slot = whole ? nullptr : l.slots + (size_t)(l.slot_base[lo_i] + part) * a.F;
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
                if (whole) {
                    finish_vector<T>(a, v, FV, colv, scale, sum);
                } else {
#pragma unroll
                    for (int e = 0; e < VE; ++e) slot[colv * VE + e] = sum[e];
                }
            }
            __syncthreads();
        }
    }
}

// The rows that were cut into several tasks: one wavefront per queue entry adds the partial rows in task order.
template <typename T>
__global__ __launch_bounds__(kThreads) void spmm_long_rows_finish_kernel(SpmmArgs a) {
    constexpr int VE = LpVec<T>::N;
    const int lane = threadIdx.x & 63;
    const LongQueue l = long_queue_of(a.long_queue, a.n_rows);
    const int32_t n_queued = l.head[0], seg = l.head[1];
    const int FV = a.F / VE;
    for (int32_t i = blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6); i < n_queued; i += gridDim.x * (kThreads / 64)) {
        const int32_t v = l.rows[i];
        const int32_t len = a.rowptr[v + 1] - a.rowptr[v];
        if (len <= seg) continue;
        const int32_t parts = (len + seg - 1) / seg;
        const float *slot = l.slots + (size_t)l.slot_base[i] * a.F;
        const float scale = row_scale(a, v);
        for (int colv = lane; colv < FV; colv += 64) {
            float sum[VE];
#pragma unroll
            for (int e = 0; e < VE; ++e) sum[e] = 0.f;
            for (int32_t p = 0; p < parts; ++p)
#pragma unroll
                for (int e = 0; e < VE; ++e) sum[e] += slot[(size_t)p * a.F + colv * VE + e];
            finish_vector<T>(a, v, FV, colv, scale, sum);
        }
    }
}

template <typename T, int G, int C>
int launch(const SpmmArgs &a, hipStream_t st) {
    const int mode = a.entry_rows ? 2 : ((a.w || a.col_w || a.sym_norm) ? 1 : 0);
    if (a.long_queue) {
        const unsigned grid = (unsigned)lp_ceil_div(a.n_rows, kRowThreads / 64);
        if (mode == 2) hipLaunchKernelGGL((spmm_rows_kernel<T, G, C, 2, kRowThreads>), dim3(grid), dim3(kRowThreads), 0, st, a);
        else if (mode == 1) hipLaunchKernelGGL((spmm_rows_kernel<T, G, C, 1, kRowThreads>), dim3(grid), dim3(kRowThreads), 0, st, a);
        else hipLaunchKernelGGL((spmm_rows_kernel<T, G, C, 0, kRowThreads>), dim3(grid), dim3(kRowThreads), 0, st, a);
    } else {
        const unsigned grid = (unsigned)lp_ceil_div(a.n_rows, kShortRowThreads / 64);
        if (mode == 2) hipLaunchKernelGGL((spmm_rows_kernel<T, G, C, 2, kShortRowThreads>), dim3(grid), dim3(kShortRowThreads), 0, st, a);
        else if (mode == 1) hipLaunchKernelGGL((spmm_rows_kernel<T, G, C, 1, kShortRowThreads>), dim3(grid), dim3(kShortRowThreads), 0, st, a);
        else hipLaunchKernelGGL((spmm_rows_kernel<T, G, C, 0, kShortRowThreads>), dim3(grid), dim3(kShortRowThreads), 0, st, a);
    }
    if (a.long_queue) {
        // no more rows can be queued than fit the entry count, and a row of at least 512 entries is at most two tasks
        // per 1024 entries; two workgroups per compute unit walk the tasks
        const int64_t most_rows = a.n_entries / a.long_threshold;
        const int64_t most_tasks = most_rows + kLongSlots;
        const int64_t slots = 2 * (int64_t)lp_compute_units();
        const unsigned lgrid = (unsigned)(most_tasks < slots ? most_tasks : slots);
        if (most_rows > 0) {
            hipLaunchKernelGGL(plan_long_rows_kernel, dim3(1), dim3(1024), 0, st, a.rowptr, a.long_queue, a.n_rows);
            if (mode == 2) hipLaunchKernelGGL((spmm_long_rows_kernel<T, G, C, 2>), dim3(lgrid), dim3(kLongThreads), 0, st, a);
            else if (mode == 1) hipLaunchKernelGGL((spmm_long_rows_kernel<T, G, C, 1>), dim3(lgrid), dim3(kLongThreads), 0, st, a);
            else hipLaunchKernelGGL((spmm_long_rows_kernel<T, G, C, 0>), dim3(lgrid), dim3(kLongThreads), 0, st, a);
            // rows cut into several tasks are at most kLongTargetTasks; the grid also never needs more wavefronts than rows
            const int64_t fin_rows = most_rows < 4 * slots ? most_rows : 4 * slots;
            hipLaunchKernelGGL((spmm_long_rows_finish_kernel<T>), dim3((unsigned)lp_ceil_div(fin_rows, kThreads / 64)), dim3(kThreads), 0, st, a);
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

size_t lp_spmm_queue_bytes(int32_t n_rows, int32_t max_width) {
    const int32_t cap = n_rows > 0 ? n_rows : 0;
    return lp_align_up(sizeof(int32_t) * (kLongHeader + 3 * long_words(cap)) + sizeof(float) * (size_t)kLongSlots * (size_t)(max_width > 0 ? max_width : 0));
}

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
