// Internal declarations shared by the HIP translation units of the library.
// Nothing here is part of the public ABI (that is include/lp.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "lp.h"

#define LP_TRY(expr)                         \
    do {                                     \
        int lp_status_ = (expr);             \
        if (lp_status_ != LP_OK) return lp_status_; \
    } while (0)

#define LP_HIP_TRY(expr)                              \
    do {                                              \
        if ((expr) != hipSuccess) return LP_ERR_HIP;  \
    } while (0)

static inline int lp_after_launch() { return hipGetLastError() == hipSuccess ? LP_OK : LP_ERR_HIP; }

static inline int64_t lp_ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
static inline size_t lp_align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }
static inline bool lp_aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
static inline bool lp_valid_fp32_products(int32_t v) { return v == LP_FP32_PRODUCTS_NATIVE || v == LP_FP32_PRODUCTS_BF16X6; }

// ---------------------------------------------------------------- instrumentation (lp_timing.hip)
// Kernel classes of lp_timing_collect, in the order of LP_KC_* in lp.h.
class LpTimedScope {
public:
    LpTimedScope(int cls, hipStream_t st);
    ~LpTimedScope();
    LpTimedScope(const LpTimedScope &) = delete;
    LpTimedScope &operator=(const LpTimedScope &) = delete;

private:
    int cls_;
    hipStream_t st_;
    void *beg_;
};

// ---------------------------------------------------------------- sparse aggregation (spmm_mean.hip)
// out[v, :] = rowscale(v) * sum_{p in row v} w[p] * in[colidx[p], :]  (+ addend[v, :])  (* [gate[v, :] > 0])
//   w[p] = 1 when w == nullptr (or col_w[colidx[p]] when col_w is given)
//   rowscale(v) = inv_deg[v] when inv_deg != nullptr, else 1
// With `in_index`, `in` and `addend` hold only some rows: node u lives in row in_index[u], and a negative entry
// stands for an all-zero row.  With `n_rows_dev` the number of output rows is read on the device (at most n_rows).
// All matrices are [n_rows, F] in the storage type `dtype` with contiguous rows; F is a multiple of 4 (fp32) or 8 (bf16).
struct SpmmArgs {
    int32_t dtype = LP_F32;              // storage of in, addend, gate and out
    int32_t n_rows = 0;
    int32_t F = 0;
    const int32_t *rowptr = nullptr;
    const int32_t *colidx = nullptr;
    const int32_t *row_order = nullptr;  // optional processing order
    const float *inv_deg = nullptr;      // optional per-output-row scale
    const float *w = nullptr;            // optional per-entry weight (parallel to colidx)
    const float *col_w = nullptr;        // optional per-node weight: entry p weighs col_w[colidx[p]] (instead of w)
    const void *entry_rows = nullptr;    // optional matrix with rows of F values (storage type): entry p is multiplied
    const int32_t *entry_row_index = nullptr;  // element-wise by its row entry_row_index[p] (instead of a scalar weight)
    bool sym_norm = false;               // symmetric normalisation: entry p weighs sqrt(inv_deg[colidx[p]]), row v is
                                         // scaled by sqrt(inv_deg[v]) (inv_deg required, w unused)
    // with sym_norm, for a sampled subset of the neighbours (inverse counts 1/|S| of the sampled rows): a row v with
    // sym_row_cnt is scaled by sym_row_cnt[v] / sqrt(inv_deg[v]) instead; an entry with column c and sym_col_cnt
    // weighs sym_col_cnt[c] / sqrt(inv_deg[c]) instead (the transposed pass)
    const float *sym_row_cnt = nullptr;
    const float *sym_col_cnt = nullptr;
    const void *in = nullptr;
    const void *addend = nullptr;        // optional [n_rows, F]
    const int32_t *in_index = nullptr;   // optional [number of nodes]: row of `in` / `addend` that holds a node, or < 0
    const int32_t *n_rows_dev = nullptr; // optional device scalar: rows actually present (<= n_rows)
    const int32_t *addend_rows_dev = nullptr;  // optional device scalar: only rows below it have an addend row
    const void *gate = nullptr;          // optional [n_rows, F]: output is zeroed where gate <= 0
    void *out = nullptr;
    int64_t n_entries = 0;               // entries of colidx (bounds how many rows can be long)
    int32_t *long_queue = nullptr;       // optional workspace of lp_spmm_queue_bytes(n_rows, F): rows of at least
                                         // kSpmmLongRow entries are served by whole workgroups
    int32_t long_threshold = 0;          // set by the launcher
    int timing_class = LP_KC_SPMM;       // class the launch is booked under by the instrumentation
};
constexpr int32_t kSpmmLongRow = 512;
size_t lp_spmm_queue_bytes(int32_t n_rows, int32_t max_width);   // max_width: the widest F the queue will be used with
int lp_launch_spmm(const SpmmArgs &a, hipStream_t stream);

// ---------------------------------------------------------------- dense products (gemm_mfma.hip)
// C[M, N] = sum_{s<2} A[s][M, K[s]] * Bt[s][.]^T, operands with the reduction index contiguous ("NT"):
//   A[s] is [M, K[s]] row-major (leading dimension lda[s]);
//   the B operand of K-part s is given transposed: column n of the product reads row n of
//   Bt[s][0] when n < n_split, else row (n - n_split) of Bt[s][1]; rows have K[s] contiguous floats (ldb[s]).
// Epilogue: + bias[n] (optional), max(.,0) (optional); columns n >= n_split are multiplied by
// rowscale[m] (optional) and go to C[1] (leading dimension ldc[1]) at column n - n_split, the others to C[0];
// with a gate matrix (fp32 storage, unsplit output) results are zeroed where the gate is not positive.
struct GemmNtArgs {
    int32_t dtype = LP_F32;              // storage of A, Bt and C (bias and rowscale are always fp32)
    int32_t fp32_products = LP_FP32_PRODUCTS_NATIVE;   // LP_F32 only: fp32 matrix instructions or bfloat16 terms
    int32_t M = 0, N = 0;
    int32_t n_split = 0;                 // == N when the output is not split
    const void *A[2] = {nullptr, nullptr};
    int32_t lda[2] = {0, 0};
    int32_t K[2] = {0, 0};
    const void *Bt[2][2] = {{nullptr, nullptr}, {nullptr, nullptr}};
    int32_t ldb[2] = {0, 0};
    const float *bias = nullptr;
    bool relu = false;
    const float *rowscale = nullptr;
    const int32_t *rowscale_index = nullptr;  // optional [M]: row m is scaled by rowscale[rowscale_index[m]]
    const int32_t *m_dev = nullptr;           // optional device scalar: rows actually present (<= M)
    void *C[2] = {nullptr, nullptr};
    int32_t ldc[2] = {0, 0};
    const float *gate = nullptr;              // optional [M, N] fp32 (LP_F32, one output only): C[m, n] = 0 where gate[m, n] <= 0
    int32_t ldgate = 0;
};
int lp_launch_gemm_nt(const GemmNtArgs &a, hipStream_t stream);

// dW[Mw, Nw] = At[Kn, Mw]^T * B[Kn, Nw], the reduction index (nodes) is the slow one on both operands ("TN").
// Also accumulates nothing else; partial sums of the row chunks go to `partials` and are then added up in a
// fixed order, so the result does not depend on scheduling.
struct GemmTnArgs {
    int32_t dtype = LP_F32;              // storage of At and B; C and the partial sums are fp32
    int32_t Kn = 0;                      // reduction length (number of nodes)
    int32_t Mw = 0, Nw = 0;              // output shape
    const void *At = nullptr;            // [Kn, Mw], leading dimension lda
    int32_t lda = 0;
    const int32_t *at_index = nullptr;   // optional [Kn]: reduction step k reads row at_index[k] of At (B stays direct)
    const int32_t *kn_dev = nullptr;     // optional device scalar: reduction length actually present (<= Kn)
    const void *B = nullptr;             // [Kn, Nw], leading dimension ldb
    int32_t ldb = 0;
    float *C = nullptr;                  // [Mw, Nw] contiguous
    float *partials = nullptr;           // workspace, lp_gemm_tn_partials_bytes()
};
size_t lp_gemm_tn_partials_bytes(int32_t Kn, int32_t Mw, int32_t Nw);
int lp_launch_gemm_tn(const GemmTnArgs &a, hipStream_t stream);

// Weight and bias gradients of one layer in one pass over the nodes:
//   C[0] = At[0]^T B,  C[1] = At[1]^T B,  dbias = column sums of B,
// At[s]: [Kn, Mw[s]] (Mw[0] may be 0), B: [Kn, Nw]; at_index / kn_dev as in GemmTnArgs.  fp32 layers of the usual
// widths take a fused kernel (B is read once, 256 x 256 tiles); everything else goes through lp_launch_gemm_tn and
// lp_launch_colsum.  Sums are taken in a fixed order.
struct WeightGradArgs {
    int32_t dtype = LP_F32;
    int32_t fp32_products = LP_FP32_PRODUCTS_NATIVE;   // LP_F32 only, as in GemmNtArgs
    int32_t Kn = 0;
    const int32_t *kn_dev = nullptr;
    const int32_t *at_index = nullptr;
    const void *At[2] = {nullptr, nullptr};
    int32_t Mw[2] = {0, 0};
    int32_t lda[2] = {0, 0};
    const void *B = nullptr;
    int32_t Nw = 0, ldb = 0;
    float *C[2] = {nullptr, nullptr};    // [Mw[s], Nw] contiguous
    float *dbias = nullptr;              // [Nw] or null
    float *partials = nullptr;           // lp_weight_grads_partials_bytes()
    float *colsum_partials = nullptr;    // lp_colsum_partials_bytes(Kn, Nw); used by the unfused path
};
size_t lp_weight_grads_partials_bytes(int32_t dtype, int32_t Kn, int32_t Mw0, int32_t Mw1, int32_t Nw);
int lp_launch_weight_grads(const WeightGradArgs &a, hipStream_t stream);

// out[c, r] = in[r, c] for a small [rows, cols] matrix (weights) of 4-byte or 2-byte elements.
int lp_launch_transpose(const void *in, int32_t rows, int32_t cols, void *out, int dtype, hipStream_t stream);
// the same for up to 16 matrices of one storage type in a single launch (out[i] = in[i]^T)
struct TransposeBatch {
    int n = 0;
    const void *in[16];
    void *out[16];
    int32_t rows[16], cols[16];
};
int lp_launch_transpose_batch(const TransposeBatch &b, int dtype, hipStream_t stream);
// all weight matrices of a model transposed into consecutive areas of `wt` (layer k: W_self^T, then W_neigh^T, each
// lp_align_up(F_{k-1} F_k, 64) elements; a NULL W_self leaves its area unwritten): one launch
int lp_launch_transpose_weights(const lp_model *m, void *wt, hipStream_t stream);
// out[n] = sum_m in[m, n] for a contiguous [M, N] matrix stored as `dtype` (N a multiple of its vector width);
// fp32 sums in a fixed order; partials: lp_colsum_partials_bytes()
size_t lp_colsum_partials_bytes(int64_t M, int64_t N);
int lp_launch_colsum(const void *in, int dtype, int64_t M, int64_t N, float *out, float *partials, hipStream_t stream,
                     const int32_t *m_dev = nullptr);  // m_dev: optional device scalar, rows actually present (<= M)
// fill n floats with zero (a kernel, so that callers may capture it); n floats = 2n bfloat16
int lp_launch_zero(float *p, int64_t n, hipStream_t stream);

// ---------------------------------------------------------------- sorting (csr_build.hip)
// Stable least-significant-digit radix sort of 64-bit keys on bits [first_bit, first_bit + n_bits), 8 or 9 bits per
// pass.  `a` holds the input, `b` is a second buffer of n keys, `hist` has lp_radix_sort_hist_words(n) words.
// Returns the buffer that holds the sorted keys (a or b).  With n_dev (a device count, at most n) only the first
// *n_dev keys are sorted and what lies behind them in the returned buffer is unspecified.
size_t lp_radix_sort_hist_words(int64_t n);
uint64_t *lp_radix_sort(uint64_t *a, uint64_t *b, int64_t n, int first_bit, int n_bits, uint32_t *hist, hipStream_t stream,
                        int *status, const uint32_t *n_dev = nullptr);
// offsets[r] = number of sorted keys below (r << shift), r = 0..n_rows; the key count is *n_dev when n_dev is
// given, else n_host.
int lp_launch_row_offsets(const uint64_t *sorted, int64_t n_host, const uint32_t *n_dev, int32_t n_rows, int shift,
                          int32_t *offsets, hipStream_t stream);
int lp_bits_for(int64_t n_values);
// Rows of a CSR row-pointer array that are not empty: list[i] = i-th such row (ascending), index[v] = position of
// row v in the list or -1, ptr[i] = offsets[list[i]] for i < count and ptr[count] = offsets[n_rows], *count_dev =
// their number.  list and ptr have room for cap + 1 entries, where the caller guarantees count <= cap;
// scan_ws: lp_compact_rows_ws_bytes(n_rows).
size_t lp_compact_rows_ws_bytes(int32_t n_rows);
int lp_launch_compact_rows(const int32_t *offsets, int32_t n_rows, int32_t *list, int32_t *index, int32_t *ptr,
                           int32_t *count_dev, void *scan_ws, hipStream_t stream);

// ---------------------------------------------------------------- scored edges grouped by end point (sage_layers.hip)
// Every scored edge (u, v) with weight g = dL/ds sends g*h_v to row u and g*h_u to row v.  The 2B (row, other end,
// g) entries are grouped by row with a stable radix sort: ptr [n_rows + 1], col / w [2B] in row order.  Edges with
// an end outside [0, n_rows) are left out.
struct BatchGroupWs {
    uint64_t *keys_a, *keys_b;  // [2B + 1] each
    uint32_t *hist;             // lp_radix_sort_hist_words(2B + 1)
};
// With dscore == nullptr the per-entry output is the index of the scored edge (as int32 in the storage of `w`)
// instead of its weight.
int lp_group_batch_by_row(const int32_t *e_src, const int32_t *e_dst, const float *dscore, int64_t B, int32_t n_rows,
                          const BatchGroupWs &ws, int32_t *ptr, int32_t *col, float *w, hipStream_t stream);

// ---------------------------------------------------------------- storage types
// LP_F32 matrices hold floats; LP_BF16 matrices hold raw bfloat16 bit patterns (uint16_t).  All arithmetic is fp32.
typedef uint16_t lp_bf16_t;

#if defined(__HIPCC__)
__device__ __forceinline__ float lp_bf16_to_f32(lp_bf16_t b) { return __uint_as_float((uint32_t)b << 16); }
// fp32 -> bfloat16, round to nearest, ties to even: the hardware pair conversion (v_cvt_pk_bf16_f32); `lo` lands in
// the low half of the word
__device__ __forceinline__ uint32_t lp_f32x2_to_bf16x2(float lo, float hi) {
    typedef __bf16 lp_bf2 __attribute__((ext_vector_type(2)));
    typedef float lp_f2 __attribute__((ext_vector_type(2)));
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(lp_f2{lo, hi}, lp_bf2));
}
__device__ __forceinline__ lp_bf16_t lp_f32_to_bf16(float x) { return (lp_bf16_t)(lp_f32x2_to_bf16x2(x, 0.f) & 0xffffu); }

// One 16-byte vector of a matrix row: 4 floats or 8 bfloat16 values, handled as fp32 in registers.
template <typename T> struct LpVec;
template <> struct LpVec<float> {
    static constexpr int N = 4;
    static __device__ __forceinline__ void load(const float *p, float (&v)[4]) {
        const float4 x = *reinterpret_cast<const float4 *>(p);
        v[0] = x.x; v[1] = x.y; v[2] = x.z; v[3] = x.w;
    }
    static __device__ __forceinline__ void store(float *p, const float (&v)[4]) {
        *reinterpret_cast<float4 *>(p) = make_float4(v[0], v[1], v[2], v[3]);
    }
    // streaming store: the line is not kept in the caches for this kernel's own later reads
    static __device__ __forceinline__ void store_streaming(float *p, const float (&v)[4]) {
        typedef float lp_v4f __attribute__((ext_vector_type(4)));
        __builtin_nontemporal_store(lp_v4f{v[0], v[1], v[2], v[3]}, reinterpret_cast<lp_v4f *>(p));
    }
};
template <> struct LpVec<lp_bf16_t> {
    static constexpr int N = 8;
    static __device__ __forceinline__ void load(const lp_bf16_t *p, float (&v)[8]) {
        const uint4 x = *reinterpret_cast<const uint4 *>(p);
        const uint32_t w[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            v[2 * i] = __uint_as_float(w[i] << 16);
            v[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
        }
    }
    static __device__ __forceinline__ void store(lp_bf16_t *p, const float (&v)[8]) {
        uint32_t w[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) w[i] = lp_f32x2_to_bf16x2(v[2 * i], v[2 * i + 1]);
        *reinterpret_cast<uint4 *>(p) = make_uint4(w[0], w[1], w[2], w[3]);
    }
    static __device__ __forceinline__ void store_streaming(lp_bf16_t *p, const float (&v)[8]) {
        typedef uint32_t lp_v4u __attribute__((ext_vector_type(4)));
        uint32_t w[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) w[i] = lp_f32x2_to_bf16x2(v[2 * i], v[2 * i + 1]);
        __builtin_nontemporal_store(lp_v4u{w[0], w[1], w[2], w[3]}, reinterpret_cast<lp_v4u *>(p));
    }
};
#endif

// number of compute units of the current device (cached)
int lp_compute_units();

static inline int lp_elem_bytes(int dtype) { return dtype == LP_BF16 ? 2 : 4; }
static inline int lp_vec_elems(int dtype) { return dtype == LP_BF16 ? 8 : 4; }
