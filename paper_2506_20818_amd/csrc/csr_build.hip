// lp_build_csr: canonical CSR (+ transpose, inverse degrees, degree-ordered row lists) of a pair list.
//
// Pipeline, all on the device:
//   pack (row, col) into one 64-bit key  ->  least-significant-digit radix sort, 8 or 9 bits per pass, only over
//   the bits a node id can occupy  ->  flag first occurrences, prefix-sum, compact (repeated pairs collapse)
//   ->  row pointers by binary search of each row's first key  ->  the same on swapped keys for the transpose.
// The graph definition this realises: Sec. II-A (edge set over node pairs) and Sec. IV-A (neighbour sets,
// degrees) of the paper.  Any correct sort yields the same bytes because the output is sorted and unique.
#include "lp_internal.h"
#include "lp_scan.h"

namespace {

using namespace lp_scan;
constexpr int kWaveChunk = 64 * kItems;   // keys per wavefront

// ------------------------------------------------------------------ radix sort of 64-bit keys, one digit of 8 or 9 bits per pass
// (nine when that saves a pass: node ids below 2^18 sort in two passes instead of three)
template <int BITS>
__global__ __launch_bounds__(kThreads) void rs_hist_kernel(const uint64_t *__restrict__ keys, int64_t n, const uint32_t *__restrict__ n_dev,
                                                           int shift, uint32_t *__restrict__ hist, int64_t nb) {
    constexpr int BINS = 1 << BITS;
    __shared__ uint32_t h[BINS];
    if (n_dev) n = min(n, (int64_t)*n_dev);   // keys actually present (blocks past them still write their zero counts)
#pragma unroll
    for (int j = threadIdx.x; j < BINS; j += kThreads) h[j] = 0;
    __syncthreads();
    const int64_t base = (int64_t)blockIdx.x * kTile;
#pragma unroll
    for (int i = 0; i < kItems; ++i) {
        int64_t idx = base + i * kThreads + threadIdx.x;
        if (idx < n) atomicAdd(&h[(keys[idx] >> shift) & (uint32_t)(BINS - 1)], 1u);
    }
    __syncthreads();
#pragma unroll
    for (int j = threadIdx.x; j < BINS; j += kThreads) hist[(int64_t)j * nb + blockIdx.x] = h[j];  // digit-major, so one scan orders everything
}

// Stable scatter.  Keys of a block are taken in index order: wavefront w owns keys [w*512, w*512+512) of the
// tile and walks them 64 at a time; inside such a group the rank among equal digits comes from one ballot per bit.
template <int BITS>
__global__ __launch_bounds__(kThreads) void rs_scatter_kernel(const uint64_t *__restrict__ in, uint64_t *__restrict__ out,
                                                              int64_t n, const uint32_t *__restrict__ n_dev, int shift,
                                                              const uint32_t *__restrict__ gbase, int64_t nb) {
    constexpr int BINS = 1 << BITS;
    __shared__ uint32_t cnt[4][BINS];
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
    if (n_dev) n = min(n, (int64_t)*n_dev);
    if ((int64_t)blockIdx.x * kTile >= n) return;   // the whole workgroup: nothing of this tile is present
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = tid; j < BINS; j += kThreads) cnt[i][j] = 0;
    __syncthreads();
    const int64_t wbase = (int64_t)blockIdx.x * kTile + (int64_t)w * kWaveChunk;
    uint64_t k[kItems];
    bool valid[kItems];
#pragma unroll
    for (int r = 0; r < kItems; ++r) {
        int64_t idx = wbase + r * 64 + lane;
        valid[r] = idx < n;
        k[r] = valid[r] ? in[idx] : 0ull;
        if (valid[r]) atomicAdd(&cnt[w][(k[r] >> shift) & (uint32_t)(BINS - 1)], 1u);
    }
    __syncthreads();
#pragma unroll
    for (int j = tid; j < BINS; j += kThreads) {
        uint32_t run = gbase[(int64_t)j * nb + blockIdx.x];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            uint32_t c = cnt[i][j];
            cnt[i][j] = run;
            run += c;
        }
    }
    __syncthreads();
    volatile uint32_t *my = cnt[w];
#pragma unroll
    for (int r = 0; r < kItems; ++r) {
        const uint32_t d = (uint32_t)(k[r] >> shift) & (uint32_t)(BINS - 1);
        unsigned long long peers = __ballot(valid[r]);
#pragma unroll
        for (int b = 0; b < BITS; ++b) {
            const bool bit = (d >> b) & 1u;
            unsigned long long bb = __ballot(valid[r] && bit);
            peers &= bit ? bb : ~bb;
        }
        uint32_t base = 0;
        if (valid[r]) base = my[d];
        const uint32_t rank = __popcll(peers & ((1ull << lane) - 1ull));
        if (valid[r]) {
            out[base + rank] = k[r];
            if (lane == 63 - __clzll(peers)) my[d] = base + (uint32_t)__popcll(peers);
        }
        __builtin_amdgcn_wave_barrier();
    }
}

// Sorts keys on bits [first_bit, first_bit + n_bits).  `a` holds the input, `b` is a buffer of the same size; returns the
// buffer that holds the result.  hist: radix_hist_words(n) uint32.  With n_dev (a device count, at most n) only the
// first *n_dev keys are sorted; what lies behind them in the returned buffer is unspecified.
uint64_t *radix_sort(uint64_t *a, uint64_t *b, int64_t n, int first_bit, int n_bits, uint32_t *hist, hipStream_t st,
                     int *status, const uint32_t *n_dev = nullptr) {
    *status = LP_OK;
    if (n <= 1) return a;
    const int64_t nb = lp_ceil_div(n, kTile);
    const int digit = (n_bits + 8) / 9 < (n_bits + 7) / 8 ? 9 : 8;   // bits per pass
    const int64_t bins = (int64_t)1 << digit;
    uint32_t *spine = hist + bins * nb;
    for (int shift = first_bit; shift < first_bit + n_bits; shift += digit) {
        if (digit == 9) hipLaunchKernelGGL(rs_hist_kernel<9>, dim3((unsigned)nb), dim3(kThreads), 0, st, a, n, n_dev, shift, hist, nb);
        else hipLaunchKernelGGL(rs_hist_kernel<8>, dim3((unsigned)nb), dim3(kThreads), 0, st, a, n, n_dev, shift, hist, nb);
        auto load = [hist] __device__(int64_t i) { return hist[i]; };
        auto store = [hist] __device__(int64_t i, uint32_t ex, uint32_t) { hist[i] = ex; };
        int s = device_exclusive_scan<uint32_t>(load, store, bins * nb, spine, nullptr, st);
        if (s != LP_OK) { *status = s; return a; }
        if (digit == 9) hipLaunchKernelGGL(rs_scatter_kernel<9>, dim3((unsigned)nb), dim3(kThreads), 0, st, a, b, n, n_dev, shift, hist, nb);
        else hipLaunchKernelGGL(rs_scatter_kernel<8>, dim3((unsigned)nb), dim3(kThreads), 0, st, a, b, n, n_dev, shift, hist, nb);
        uint64_t *t = a; a = b; b = t;
    }
    *status = lp_after_launch();
    return a;
}

size_t radix_hist_words(int64_t n) {   // enough for either digit width
    const int64_t nb = lp_ceil_div(n > 0 ? n : 1, kTile);
    return (size_t)(512 * nb + lp_ceil_div(512 * nb, kTile) + 8);
}

// ------------------------------------------------------------------ CSR specific kernels
__global__ void pack_keys_kernel(const int32_t *__restrict__ rows, const int32_t *__restrict__ cols, int64_t n_in,
                                 int32_t n_nodes, int bits, bool symmetrize, uint64_t *__restrict__ keys,
                                 uint32_t *__restrict__ err) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_in) return;
    int32_t r = rows[i], c = cols[i];
    if (r < 0 || r >= n_nodes || c < 0 || c >= n_nodes) {
        atomicOr(err, 1u);
        r = 0;
        c = 0;
    }
    keys[i] = ((uint64_t)(uint32_t)r << bits) | (uint32_t)c;
    if (symmetrize) keys[n_in + i] = ((uint64_t)(uint32_t)c << bits) | (uint32_t)r;
}

__global__ void swap_keys_kernel(const uint64_t *__restrict__ in, const uint32_t *__restrict__ nnz_dev, int bits,
                                 uint64_t *__restrict__ out) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (int64_t)*nnz_dev) return;
    const uint64_t mask = (1ull << bits) - 1ull;
    uint64_t k = in[i];
    out[i] = ((k & mask) << bits) | (k >> bits);
}

__global__ void split_cols_kernel(const uint64_t *__restrict__ keys, int64_t n, int bits, int32_t *__restrict__ colidx) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) colidx[i] = (int32_t)(keys[i] & ((1ull << bits) - 1ull));
}

// rowptr[r] = number of keys whose row is < r = first position with key >= (r << bits)
__global__ void rowptr_kernel(const uint64_t *__restrict__ ukeys, int64_t n_host, const uint32_t *__restrict__ nnz_dev,
                              int32_t n_nodes, int bits, int32_t *__restrict__ rowptr) {
    int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (r > n_nodes) return;
    const uint64_t target = (uint64_t)r << bits;
    int64_t lo = 0, hi = nnz_dev ? (int64_t)*nnz_dev : n_host;
    while (lo < hi) {
        int64_t mid = (lo + hi) >> 1;
        if (ukeys[mid] < target) lo = mid + 1; else hi = mid;
    }
    rowptr[r] = (int32_t)lo;
}

__global__ void inv_deg_kernel(const int32_t *__restrict__ rowptr, int32_t n_nodes, float *__restrict__ inv_deg) {
    int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (r >= n_nodes) return;
    int32_t d = rowptr[r + 1] - rowptr[r];
    inv_deg[r] = d > 0 ? 1.0f / (float)d : 0.0f;
}

// key = (class << 32) | row, so that an ascending stable sort on the class byte lists rows of 64 and more entries by
// decreasing size class (floor(log2) of the length) and then every shorter row, ids ascending inside a class.  Long
// rows go first so that none of them starts late; the short rows stay in id order, which keeps the reads of rowptr and
// colidx and the writes of the output rows sequential and was 5-8 % faster at 2.9 M rows than a full order by class.
__global__ void degree_class_keys_kernel(const int32_t *__restrict__ rowptr, int32_t n_nodes, uint64_t *__restrict__ keys) {
    int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (r >= n_nodes) return;
    uint32_t d = (uint32_t)(rowptr[r + 1] - rowptr[r]);
    uint32_t cls = d >= 64u ? (uint32_t)__clz(d) : 26u;      // 0 (huge) .. 25 (64-127 entries), 26 (all shorter rows)
    keys[r] = ((uint64_t)cls << 32) | (uint32_t)r;
}

__global__ void low_words_kernel(const uint64_t *__restrict__ keys, int64_t n, int32_t *__restrict__ out) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) out[i] = (int32_t)(uint32_t)keys[i];
}

inline int bits_for(int32_t n_nodes) { return lp_bits_for(n_nodes); }

struct BuildWs {
    uint64_t *keys_a, *keys_b, *ukeys;
    uint32_t *hist, *scan_sums, *scalars;  // scalars[0] = nnz, scalars[1] = error flag
    size_t bytes;
};

BuildWs carve(void *ws, int32_t n_nodes, int64_t n_in, uint32_t flags) {
    const int64_t cap = (flags & LP_SYMMETRIZE) ? 2 * n_in : n_in;
    const int64_t sort_n = cap > n_nodes ? cap : n_nodes;
    char *p = static_cast<char *>(ws);
    size_t off = 0;
    auto take = [&](size_t bytes) { char *q = p ? p + off : nullptr; off += lp_align_up(bytes); return q; };
    BuildWs w;
    w.keys_a = reinterpret_cast<uint64_t *>(take(sizeof(uint64_t) * (size_t)(sort_n + 1)));
    w.keys_b = reinterpret_cast<uint64_t *>(take(sizeof(uint64_t) * (size_t)(sort_n + 1)));
    w.ukeys = reinterpret_cast<uint64_t *>(take(sizeof(uint64_t) * (size_t)(cap + 1)));
    w.hist = reinterpret_cast<uint32_t *>(take(sizeof(uint32_t) * radix_hist_words(sort_n)));
    w.scan_sums = reinterpret_cast<uint32_t *>(take(sizeof(uint32_t) * (size_t)(lp_ceil_div(sort_n + 1, kTile) + 8)));
    w.scalars = reinterpret_cast<uint32_t *>(take(256));
    w.bytes = off;
    return w;
}

int order_rows(const int32_t *rowptr, int32_t n_nodes, int32_t *order, BuildWs &w, hipStream_t st) {
    const unsigned g = (unsigned)lp_ceil_div(n_nodes, 256);
    hipLaunchKernelGGL(degree_class_keys_kernel, dim3(g), dim3(256), 0, st, rowptr, n_nodes, w.keys_a);
    int status;
    uint64_t *sorted = radix_sort(w.keys_a, w.keys_b, n_nodes, 32, 8, w.hist, st, &status);
    LP_TRY(status);
    hipLaunchKernelGGL(low_words_kernel, dim3(g), dim3(256), 0, st, sorted, (int64_t)n_nodes, order);
    return lp_after_launch();
}

}  // namespace

int lp_bits_for(int64_t n_values) {
    int b = 1;
    while (((int64_t)1 << b) < n_values) ++b;
    return b;
}

size_t lp_radix_sort_hist_words(int64_t n) { return radix_hist_words(n); }

uint64_t *lp_radix_sort(uint64_t *a, uint64_t *b, int64_t n, int first_bit, int n_bits, uint32_t *hist, hipStream_t st,
                        int *status, const uint32_t *n_dev) {
    return radix_sort(a, b, n, first_bit, n_bits, hist, st, status, n_dev);
}

int lp_launch_row_offsets(const uint64_t *sorted, int64_t n_host, const uint32_t *n_dev, int32_t n_rows, int shift,
                          int32_t *offsets, hipStream_t st) {
    hipLaunchKernelGGL(rowptr_kernel, dim3((unsigned)lp_ceil_div((int64_t)n_rows + 1, 256)), dim3(256), 0, st, sorted, n_host,
                       n_dev, n_rows, shift, offsets);
    return lp_after_launch();
}

__global__ void compact_tail_kernel(const int32_t *__restrict__ offsets, int32_t n_rows, const int32_t *__restrict__ count,
                                    int32_t *__restrict__ ptr) {
    if (blockIdx.x == 0 && threadIdx.x == 0) ptr[*count] = offsets[n_rows];
}

size_t lp_compact_rows_ws_bytes(int32_t n_rows) {
    return lp_align_up(sizeof(uint32_t) * (size_t)(lp_ceil_div((int64_t)(n_rows > 0 ? n_rows : 1), kTile) + 8));
}

int lp_launch_compact_rows(const int32_t *offsets, int32_t n_rows, int32_t *list, int32_t *index, int32_t *ptr,
                           int32_t *count_dev, void *scan_ws, hipStream_t st) {
    if (n_rows <= 0) return LP_OK;
    auto occupied = [offsets] __device__(int64_t v) { return (uint32_t)(offsets[v + 1] > offsets[v]); };
    auto emit = [offsets, list, index, ptr] __device__(int64_t v, uint32_t pos, uint32_t flag) {
        index[v] = flag ? (int32_t)pos : -1;
        if (flag) {
            list[pos] = (int32_t)v;
            ptr[pos] = offsets[v];
        }
    };
    LP_TRY(device_exclusive_scan<uint32_t>(occupied, emit, (int64_t)n_rows, static_cast<uint32_t *>(scan_ws),
                                 reinterpret_cast<uint32_t *>(count_dev), st));
    hipLaunchKernelGGL(compact_tail_kernel, dim3(1), dim3(64), 0, st, offsets, n_rows, count_dev, ptr);
    return lp_after_launch();
}

extern "C" size_t lp_build_csr_workspace_bytes(int32_t n_nodes, int64_t n_in, uint32_t flags) {
    if (n_nodes <= 0 || n_in < 0) return 0;
    return carve(nullptr, n_nodes, n_in, flags).bytes;
}

// scale[p] = inv_deg[col[p]]: the per-node factor of every entry, laid out in entry order
__global__ void entry_scale_kernel(const int32_t *__restrict__ col, int64_t n, const float *__restrict__ inv_deg,
                                   float *__restrict__ scale) {
    const int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (p < n) scale[p] = inv_deg[col[p]];
}

extern "C" int lp_build_csr(int32_t n_nodes, int64_t n_in, const int32_t *rows, const int32_t *cols, uint32_t flags,
                            int32_t *rowptr, int32_t *colidx, int32_t *t_rowptr, int32_t *t_colidx, float *inv_deg,
                            int32_t *row_order, int32_t *t_row_order, float *t_entry_scale, int64_t *nnz_out, void *ws,
                            size_t ws_bytes, void *stream) {
    if (n_nodes <= 0 || n_in < 0 || (flags & ~LP_SYMMETRIZE)) return LP_ERR_INVALID_ARG;
    if (!rowptr || !t_rowptr || !inv_deg || !nnz_out) return LP_ERR_INVALID_ARG;
    if (n_in > 0 && (!rows || !cols || !colidx || !t_colidx)) return LP_ERR_INVALID_ARG;
    const bool sym = (flags & LP_SYMMETRIZE) != 0;
    const int64_t cap = sym ? 2 * n_in : n_in;
    if (cap >= ((int64_t)1 << 31)) return LP_ERR_OUT_OF_RANGE;
    if (!ws || ws_bytes < lp_build_csr_workspace_bytes(n_nodes, n_in, flags)) return LP_ERR_WORKSPACE;

    hipStream_t st = static_cast<hipStream_t>(stream);
    BuildWs w = carve(ws, n_nodes, n_in, flags);
    const int bits = bits_for(n_nodes);
    const unsigned g_nodes1 = (unsigned)lp_ceil_div((int64_t)n_nodes + 1, 256);
    const unsigned g_nodes = (unsigned)lp_ceil_div(n_nodes, 256);

    LP_TRY(lp_launch_zero(reinterpret_cast<float *>(w.scalars), 64, st));
    uint32_t host_scalars[2] = {0, 0};
    if (cap > 0) {
        hipLaunchKernelGGL(pack_keys_kernel, dim3((unsigned)lp_ceil_div(n_in, 256)), dim3(256), 0, st, rows, cols, n_in,
                           n_nodes, bits, sym, w.keys_a, w.scalars + 1);
        int status;
        const uint64_t *sorted = radix_sort(w.keys_a, w.keys_b, cap, 0, 2 * bits, w.hist, st, &status);
        LP_TRY(status);
        // first occurrences -> compacted unique keys and column indices
        uint64_t *ukeys = w.ukeys;
        const int mbits = bits;
        auto is_first = [sorted] __device__(int64_t i) { return (uint32_t)(i == 0 || sorted[i] != sorted[i - 1]); };
        auto emit = [sorted, ukeys, colidx, mbits] __device__(int64_t i, uint32_t pos, uint32_t flag) {
            if (flag) {
                uint64_t k = sorted[i];
                ukeys[pos] = k;
                colidx[pos] = (int32_t)(k & ((1ull << mbits) - 1ull));
            }
        };
        LP_TRY(device_exclusive_scan<uint32_t>(is_first, emit, cap, w.scan_sums, w.scalars, st));
    }
    hipLaunchKernelGGL(rowptr_kernel, dim3(g_nodes1), dim3(256), 0, st, w.ukeys, (int64_t)0, w.scalars, n_nodes, bits, rowptr);
    hipLaunchKernelGGL(inv_deg_kernel, dim3(g_nodes), dim3(256), 0, st, rowptr, n_nodes, inv_deg);
    LP_TRY(lp_after_launch());

    // nnz and the range-error flag are needed on the host: the transpose is sorted at its exact size
    LP_HIP_TRY(hipMemcpyAsync(host_scalars, w.scalars, sizeof(host_scalars), hipMemcpyDeviceToHost, st));
    LP_HIP_TRY(hipStreamSynchronize(st));
    if (host_scalars[1]) return LP_ERR_OUT_OF_RANGE;
    const int64_t nnz = host_scalars[0];
    *nnz_out = nnz;

    if (sym) {
        // a symmetric pair set is its own transpose
        LP_HIP_TRY(hipMemcpyAsync(t_rowptr, rowptr, sizeof(int32_t) * ((size_t)n_nodes + 1), hipMemcpyDeviceToDevice, st));
        if (nnz) LP_HIP_TRY(hipMemcpyAsync(t_colidx, colidx, sizeof(int32_t) * (size_t)nnz, hipMemcpyDeviceToDevice, st));
    } else {
        const uint64_t *tsorted = w.keys_a;
        if (nnz) {
            hipLaunchKernelGGL(swap_keys_kernel, dim3((unsigned)lp_ceil_div(nnz, 256)), dim3(256), 0, st, w.ukeys,
                               w.scalars, bits, w.keys_a);
            int status;
            tsorted = radix_sort(w.keys_a, w.keys_b, nnz, 0, 2 * bits, w.hist, st, &status);
            LP_TRY(status);
            hipLaunchKernelGGL(split_cols_kernel, dim3((unsigned)lp_ceil_div(nnz, 256)), dim3(256), 0, st, tsorted, nnz,
                               bits, t_colidx);
        }
        hipLaunchKernelGGL(rowptr_kernel, dim3(g_nodes1), dim3(256), 0, st, tsorted, (int64_t)0, w.scalars, n_nodes, bits, t_rowptr);
        LP_TRY(lp_after_launch());
    }
    if (t_entry_scale && nnz) {
        hipLaunchKernelGGL(entry_scale_kernel, dim3((unsigned)lp_ceil_div(nnz, 256)), dim3(256), 0, st, t_colidx, nnz, inv_deg,
                           t_entry_scale);
        LP_TRY(lp_after_launch());
    }
    if (row_order) LP_TRY(order_rows(rowptr, n_nodes, row_order, w, st));
    if (t_row_order) {
        if (sym && row_order) {
            LP_HIP_TRY(hipMemcpyAsync(t_row_order, row_order, sizeof(int32_t) * (size_t)n_nodes, hipMemcpyDeviceToDevice, st));
        } else {
            LP_TRY(order_rows(t_rowptr, n_nodes, t_row_order, w, st));
        }
    }
    LP_HIP_TRY(hipStreamSynchronize(st));
    return LP_OK;
}
