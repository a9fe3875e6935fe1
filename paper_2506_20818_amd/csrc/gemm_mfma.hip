// Dense products of the layer update (the UPDATE of Eq. 1 of the paper as two linear maps plus bias) and of its
// backward pass, on the fp32 matrix cores of gfx950 (v_mfma_f32_32x32x2_f32, wavefront of 64 lanes).
//
// NT kernel (forward transform, input-gradient transform): both operands have the reduction index contiguous.
//   Workgroup: 256 threads = 2x2 wavefronts, tile 128 x BN (BN = 128 or 64), K step 32.
//   LDS: A tile [128][32+4] and B tile [BN][32+4] floats.  The +4 padding makes the 16-byte operand reads
//   conflict free: eight consecutive rows start in eight different groups of four banks.
//   One MFMA consumes k = {h, h'} for lane halves h = 0/1.  Since a sum over k may be taken in any order, lane
//   half h reads the four consecutive k values 4h..4h+3 of each group of eight with a single 16-byte LDS load
//   and feeds them to four successive MFMAs; A and B use the same assignment, so every k meets its partner.
// TN kernel (weight gradients): the reduction index (nodes) is the slow index of both operands; tiles are
//   copied to LDS as they are and read 4 bytes per lane (consecutive lanes, consecutive banks).  The node range
//   is split over the grid; partial tiles are written out and summed in a fixed order by a second kernel.
#include "lp_internal.h"

#include <atomic>
#include <type_traits>
#include <algorithm>

namespace {

typedef float v16f __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;
constexpr int BM = 128;
constexpr int BK = 32;
constexpr int LDS_LD = BK + 4;

__device__ inline v16f mfma32(float a, float b, v16f c) { return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0); }

// ------------------------------------------------------------------------------------------------ NT
template <int NB>  // 32-column blocks per wavefront: BN = 64 * NB
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(2))) void gemm_nt_kernel(GemmNtArgs g) {
    constexpr int BN = 64 * NB;
    constexpr int WN = 32 * NB;                 // columns per wavefront
    constexpr int A_LOADS = BM * BK / 4 / kThreads;  // float4 per thread: 4
    constexpr int B_LOADS = BN * BK / 4 / kThreads;  // 4 or 2
    __shared__ float As[BM * LDS_LD];
    __shared__ float Bs[BN * LDS_LD];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int i32 = lane & 31, h = lane >> 5;
    const int M_ = g.m_dev ? min(*g.m_dev, g.M) : g.M;  // rows actually present
    // Workgroups are handed to the eight XCDs round-robin by linear id.  The column tiles of one row tile get ids
    // that are 8 apart, so they run on the same XCD back to back and the second one finds the A rows in that L2.
    const int col_tiles = (g.N + BN - 1) / BN;
    const int slot = blockIdx.x >> 3;
    const int64_t row_tile = (int64_t)(slot / col_tiles) * 8 + (blockIdx.x & 7);
    if (row_tile * BM >= M_) return;
    const int64_t m0 = row_tile * BM;
    const int n0 = (slot % col_tiles) * BN;
    const int tiles0 = (g.K[0] + BK - 1) / BK, tiles1 = (g.K[1] + BK - 1) / BK;
    const int n_tiles = tiles0 + tiles1;

    v16f acc[2][NB];
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
        for (int cb = 0; cb < NB; ++cb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[rb][cb][r] = 0.f;

    float4 ra[A_LOADS], rbv[B_LOADS];
    auto fetch = [&](int t) {
        const int s = t < tiles0 ? 0 : 1;
        const int k0 = (s ? t - tiles0 : t) * BK;
        const float *__restrict__ A = static_cast<const float *>(s ? g.A[1] : g.A[0]);  // explicit selects keep the argument block in SGPRs
        const int K = s ? g.K[1] : g.K[0];
        const int lda = s ? g.lda[1] : g.lda[0];
        const int ldb = s ? g.ldb[1] : g.ldb[0];
        const float *__restrict__ Bt0 = static_cast<const float *>(s ? g.Bt[1][0] : g.Bt[0][0]);
        const float *__restrict__ Bt1 = static_cast<const float *>(s ? g.Bt[1][1] : g.Bt[0][1]);
        // out-of-range rows and k are read from a clamped (valid) address and then zeroed: no branches
#pragma unroll
        for (int p = 0; p < A_LOADS; ++p) {
            const int idx = p * kThreads + tid;
            const int row = idx >> 3, k = k0 + ((idx & 7) << 2);
            const int64_t m = m0 + row;
            const bool ok = m < M_ && k < K;
            const float4 v = *reinterpret_cast<const float4 *>(A + (m < M_ ? m : M_ - 1) * lda + (k < K ? k : K - 4));
            ra[p] = make_float4(ok ? v.x : 0.f, ok ? v.y : 0.f, ok ? v.z : 0.f, ok ? v.w : 0.f);
        }
#pragma unroll
        for (int p = 0; p < B_LOADS; ++p) {
            const int idx = p * kThreads + tid;
            const int row = idx >> 3, k = k0 + ((idx & 7) << 2);
            const int n = n0 + row;
            const int nn = n < g.N ? n : g.N - 1;
            const bool ok = n < g.N && k < K;
            const float *__restrict__ brow = nn < g.n_split ? Bt0 + (int64_t)nn * ldb : Bt1 + (int64_t)(nn - g.n_split) * ldb;
            const float4 v = *reinterpret_cast<const float4 *>(brow + (k < K ? k : K - 4));
            rbv[p] = make_float4(ok ? v.x : 0.f, ok ? v.y : 0.f, ok ? v.z : 0.f, ok ? v.w : 0.f);
        }
    };
    auto stash = [&]() {
#pragma unroll
        for (int p = 0; p < A_LOADS; ++p) {
            const int idx = p * kThreads + tid;
            *reinterpret_cast<float4 *>(&As[(idx >> 3) * LDS_LD + ((idx & 7) << 2)]) = ra[p];
        }
#pragma unroll
        for (int p = 0; p < B_LOADS; ++p) {
            const int idx = p * kThreads + tid;
            *reinterpret_cast<float4 *>(&Bs[(idx >> 3) * LDS_LD + ((idx & 7) << 2)]) = rbv[p];
        }
    };

    if (n_tiles > 0) fetch(0);
    for (int t = 0; t < n_tiles; ++t) {
        __syncthreads();  // previous tile fully consumed
        stash();
        __syncthreads();
        if (t + 1 < n_tiles) fetch(t + 1);  // global loads overlap the MFMAs below
#pragma unroll
        for (int kk = 0; kk < BK / 8; ++kk) {
            float4 a[2], b[NB];
#pragma unroll
            for (int rb = 0; rb < 2; ++rb)
                a[rb] = *reinterpret_cast<const float4 *>(&As[(wm * 64 + rb * 32 + i32) * LDS_LD + kk * 8 + 4 * h]);
#pragma unroll
            for (int cb = 0; cb < NB; ++cb)
                b[cb] = *reinterpret_cast<const float4 *>(&Bs[(wn * WN + cb * 32 + i32) * LDS_LD + kk * 8 + 4 * h]);
            // k-major order: consecutive MFMAs write different accumulators
#pragma unroll
            for (int rb = 0; rb < 2; ++rb)
#pragma unroll
                for (int cb = 0; cb < NB; ++cb) acc[rb][cb] = mfma32(a[rb].x, b[cb].x, acc[rb][cb]);
#pragma unroll
            for (int rb = 0; rb < 2; ++rb)
#pragma unroll
                for (int cb = 0; cb < NB; ++cb) acc[rb][cb] = mfma32(a[rb].y, b[cb].y, acc[rb][cb]);
#pragma unroll
            for (int rb = 0; rb < 2; ++rb)
#pragma unroll
                for (int cb = 0; cb < NB; ++cb) acc[rb][cb] = mfma32(a[rb].z, b[cb].z, acc[rb][cb]);
#pragma unroll
            for (int rb = 0; rb < 2; ++rb)
#pragma unroll
                for (int cb = 0; cb < NB; ++cb) acc[rb][cb] = mfma32(a[rb].w, b[cb].w, acc[rb][cb]);
        }
    }

    // epilogue: accumulator register r of lane (j = lane % 32, h = lane / 32) is row 8*(r/4) + 4*h + r%4, column j.
    // Row scales are fetched up front so that the stores that follow need no waits between them.
    float rs[2][16];
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
        for (int r = 0; r < 16; ++r) rs[rb][r] = 1.f;
    if (g.rowscale) {
#pragma unroll
        for (int rb = 0; rb < 2; ++rb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int64_t m = m0 + wm * 64 + rb * 32 + 8 * (r >> 2) + 4 * h + (r & 3);
                { const int64_t mm = m < M_ ? m : M_ - 1; rs[rb][r] = g.rowscale[g.rowscale_index ? g.rowscale_index[mm] : mm]; }
            }
    }
#pragma unroll
    for (int cb = 0; cb < NB; ++cb) {
        const int n = n0 + wn * WN + cb * 32 + i32;
        const bool n_ok = n < g.N;
        const float bias = (g.bias && n_ok) ? g.bias[n] : 0.f;
        const bool second = n >= g.n_split;
        float *__restrict__ C = static_cast<float *>(second ? g.C[1] : g.C[0]);
        const int64_t ldc = second ? g.ldc[1] : g.ldc[0];
        C += second ? n - g.n_split : n;
#pragma unroll
        for (int rb = 0; rb < 2; ++rb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int64_t m = m0 + wm * 64 + rb * 32 + 8 * (r >> 2) + 4 * h + (r & 3);
                float y = acc[rb][cb][r] + bias;
                if (g.relu) y = fmaxf(y, 0.f);
                y *= second ? rs[rb][r] : 1.f;
                if (n_ok && m < M_) {
                    if (g.gate && !(g.gate[m * g.ldgate + n] > 0.f)) y = 0.f;
                    C[m * ldc] = y;
                }
            }
    }
}

// ------------------------------------------------------------------------------------------------ NT, fast path
// Same product as gemm_nt_kernel for shapes whose K parts are whole K steps and whose column tiles do not
// straddle n_split, for fp32 and for bfloat16 storage.  What makes it faster:
//  * persistent workgroups: a workgroup walks over row tiles b, b+G, b+2G, ... and, for each, over all column
//    tiles, as ONE software pipeline.  The loads of the next tile's first K steps are already in flight while the
//    current tile's results are stored, so only the very first tile pays the load latency, and the second column
//    tile of a row tile finds the A rows in the XCD's L2;
//  * two LDS stages and one barrier per K step: while the MFMAs of step u run from stage u&1, step u+1 (already
//    in registers) is written to the other stage and the loads of step u+2 are issued;
//  * addresses are a wavefront-uniform base plus a per-thread 32-bit byte offset that is set once per K part; rows
//    and columns past the edge are clamped to the last valid one (their products land in outputs never stored);
//  * LDS rows are padded by 16 bytes, so consecutive rows start in different groups of four banks.
// Everything is laid out in bytes: a K step covers KSB bytes of every operand row (KSB/4 fp32 or KSB/2 bfloat16
// values), and a 32-byte group of a row feeds four fp32 MFMAs (k pairs) or one bf16 MFMA (sixteen k), with lane
// half h owning bytes 16h..16h+15 of the group for both operands.
// The weight tile is the row operand of the MFMAs, so each 32x32 accumulator block is the TRANSPOSE of the output
// block: lane (j = lane % 32, h = lane / 32) holds output row j and, in registers 4q..4q+3, the four consecutive
// columns 8q + 4h .. + 3.  Every lane therefore stores whole 16-byte (fp32) or 8-byte (bfloat16) pieces and needs
// a single row scale.
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef int v4i __attribute__((ext_vector_type(4)));

template <typename T> struct NtElem;
template <> struct NtElem<float> {
    static constexpr int STEPS = 4;  // MFMAs per 32-byte group: one per fp32 value of the lane's 16 bytes
    static __device__ __forceinline__ void mfma_step(v16f &acc, const v4i &w, const v4i &x, int s) {
        acc = mfma32(__builtin_bit_cast(v4f, w)[s], __builtin_bit_cast(v4f, x)[s], acc);
    }
    static __device__ __forceinline__ void store4(float *p, const float (&y)[4]) {
        *reinterpret_cast<v4f *>(p) = v4f{y[0], y[1], y[2], y[3]};
    }
};
template <> struct NtElem<lp_bf16_t> {
    static constexpr int STEPS = 1;
    static __device__ __forceinline__ void mfma_step(v16f &acc, const v4i &w, const v4i &x, int) {
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, w), __builtin_bit_cast(v8bf, x), acc, 0, 0, 0);
    }
    static __device__ __forceinline__ void store4(lp_bf16_t *p, const float (&y)[4]) {
        *reinterpret_cast<uint2 *>(p) = make_uint2(lp_f32x2_to_bf16x2(y[0], y[1]), lp_f32x2_to_bf16x2(y[2], y[3]));
    }
};

// f(std::integral_constant<int, 0>{}), ..., f(std::integral_constant<int, N - 1>{}): a loop whose index is a constant
// expression inside the body
template <int N, int I = 0, class F>
__device__ __forceinline__ void lp_unrolled(F &&f) {
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        lp_unrolled<N, I + 1>(f);
    }
}

// fp32 values as sums of three bfloat16 terms (SPLIT variant of the kernel below).  t0 = bf16(x), t1 = bf16(x - t0),
// t2 = bf16(x - t0 - t1), every rounding to nearest: the remainders are exact in fp32 and the last one fits in eight
// bits, so t0 + t1 + t2 == x for every finite x whose last term is not subnormal.  (Rounding the few values within
// half a bfloat16 step of the fp32 maximum would give an infinite t0 and with it NaN terms; t0 is therefore held at
// the largest finite bfloat16, which leaves an exactly representable remainder.  Non-finite x still yield non-finite
// terms: infinity - t0 and NaN - t0 propagate through t1.)  A product x*y is then the sum of
// nine exact bf16 products, of which the three smallest (t1*u2, t2*u1, t2*u2: below 2^-26 of |x*y|) are left out; the
// other six run on the bf16 matrix cores with fp32 accumulation.  Measured against fp64, the result is as close as
// the fp32 MFMA's (both are dominated by the fp32 accumulation), at 6/16 of its issue time.
// Magnitudes of a bfloat16 pair held at the largest finite value 0x7f7f (signs kept).
__device__ __forceinline__ uint32_t lp_finite_bf16x2(uint32_t p) {
    typedef unsigned short lp_us2 __attribute__((ext_vector_type(2)));
    const lp_us2 mag = __builtin_bit_cast(lp_us2, p & 0x7fff7fffu);
    const lp_us2 cap = __builtin_elementwise_min(mag, lp_us2{0x7f7f, 0x7f7f});
    return (p & 0x80008000u) | __builtin_bit_cast(uint32_t, cap);
}

// Four consecutive values of a row -> the 8-byte pieces of the three term planes.
__device__ __forceinline__ void lp_split3(const v4i &v, uint2 &t0, uint2 &t1, uint2 &t2) {
    const v4f x = __builtin_bit_cast(v4f, v);
    float r[4];
    t0 = make_uint2(lp_finite_bf16x2(lp_f32x2_to_bf16x2(x[0], x[1])), lp_finite_bf16x2(lp_f32x2_to_bf16x2(x[2], x[3])));
    r[0] = x[0] - __uint_as_float(t0.x << 16);
    r[1] = x[1] - __uint_as_float(t0.x & 0xffff0000u);
    r[2] = x[2] - __uint_as_float(t0.y << 16);
    r[3] = x[3] - __uint_as_float(t0.y & 0xffff0000u);
    t1 = make_uint2(lp_f32x2_to_bf16x2(r[0], r[1]), lp_f32x2_to_bf16x2(r[2], r[3]));
    r[0] -= __uint_as_float(t1.x << 16);
    r[1] -= __uint_as_float(t1.x & 0xffff0000u);
    r[2] -= __uint_as_float(t1.y << 16);
    r[3] -= __uint_as_float(t1.y & 0xffff0000u);
    t2 = make_uint2(lp_f32x2_to_bf16x2(r[0], r[1]), lp_f32x2_to_bf16x2(r[2], r[3]));
}

// T: storage type; NB: 32-column blocks per wavefront (tile width 64*NB); MW: wavefronts along M (tile height 64*MW,
// 128*MW threads); KSB: bytes of every operand row consumed per K step (64 or 128).
// SPLIT (fp32 only, KSB = 64): the tile copy turns the sixteen fp32 values of a row into three planes of sixteen
// bfloat16 terms (an LDS row is plane 0 | plane 1 | plane 2 | 16 bytes of padding = 112 bytes = 28 banks: sixteen
// consecutive rows start in sixteen different groups of four banks), and a K step is six bf16 MFMAs per accumulator
// block instead of eight fp32 ones.
// GATE (fp32 only): results are zeroed where the gate matrix is not positive; a wavefront requests the gate values of a
// store pass (one 16-byte vector per store instruction) before it lays the pass out in LDS, so they arrive meanwhile.
template <typename T, int NB, int MW, int KSB, bool SPLIT = false, bool GATE = false>
__global__ __launch_bounds__(128 * MW) __attribute__((amdgpu_waves_per_eu(2))) void gemm_nt_fast_kernel(GemmNtArgs g) {
    static_assert(!SPLIT || (sizeof(T) == 4 && KSB == 64), "the split product is defined for fp32 rows, sixteen values per step");
    static_assert(!GATE || sizeof(T) == 4, "the gated epilogue is written for fp32 storage");
    constexpr int ES = (int)sizeof(T);
    constexpr int TH = 128 * MW;
    constexpr int BMt = 64 * MW;
    constexpr int BN = 64 * NB;
    constexpr int WN = 32 * NB;
    constexpr int ROWB = SPLIT ? 3 * (KSB / 2) + 16 : KSB + 16;   // bytes per LDS row
    constexpr int KQ = KSB / 16;                     // 16-byte vectors per tile row
    constexpr int A_LOADS = BMt * KQ / TH;
    constexpr int B_LOADS = BN * KQ / TH;
    constexpr int EPB = MW == 4 ? 256 : 128;         // bytes of an output row segment per store pass of a wavefront
    constexpr int EROW = EPB + 16;                   // its LDS pitch
    constexpr int EPC = EPB / ES;                    // columns per pass
    constexpr int CBP = EPC / 32;                    // 32-column accumulator blocks per pass
    constexpr int TILEB = (BMt + BN) * ROWB;         // bytes of the two operand tiles
    constexpr int STAGEB = (TH / 64) * 32 * EROW;    // bytes of the store staging of all wavefronts
    constexpr int STAGE = TILEB > STAGEB ? TILEB : STAGEB;   // bytes per LDS stage
    static_assert(CBP >= 1 && NB % CBP == 0, "a pass covers whole accumulator blocks");
    __shared__ __attribute__((aligned(16))) char lds[2 * STAGE];
    __shared__ __attribute__((aligned(16))) char bias_lds[(TH / 64) * WN * 4];  // per wavefront: bias of its columns

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int i32 = lane & 31, h = lane >> 5;
    const int M_ = g.m_dev ? min(*g.m_dev, g.M) : g.M;  // rows actually present
    const int col_tiles = (g.N + BN - 1) / BN;
    const int row_tiles = M_ > 0 ? (M_ - 1) / BMt + 1 : 0;
    const int tiles0 = g.K[0] * ES / KSB, tiles1 = g.K[1] * ES / KSB;
    const int n_tiles = tiles0 + tiles1;
    if ((int)blockIdx.x >= row_tiles || n_tiles == 0) return;
    const int my_rows = (row_tiles - (int)blockIdx.x + (int)gridDim.x - 1) / (int)gridDim.x;
    const int n_steps = my_rows * col_tiles * n_tiles;  // the launcher keeps this below 2^31

    v16f acc[2][NB];
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
        for (int cb = 0; cb < NB; ++cb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[rb][cb][r] = 0.f;

    // Load cursor: the K steps of one part of one output tile form a segment, inside which both operand pointers
    // just advance by KSB; what a new segment needs (pointers, pitches, row clamps, the next tile's bias) is worked
    // out only when the count of steps left in the segment reaches zero.  Offsets are formed per load (clamped row
    // * pitch + column bytes) instead of being kept in registers.  The loads themselves are unconditional (a cursor
    // past its end repeats its last step): with a fixed number of loads per step the compiler can wait for the
    // older ones by count and leave the younger ones in flight.  (Keeping two steps of A rows in flight was tried
    // for the short bfloat16 steps and measured no faster.)
    constexpr int RP = TH / KQ;                      // tile rows covered by one load of every thread
    const int r0 = tid / KQ, c16 = (tid % KQ) << 4;
    int rowF = blockIdx.x, colF = 0, partF = 0;      // the segment that begins next: row tile, column tile, K part
    int seg_left = 0;                                // K steps left in the current segment
    int kstep = KSB;                                 // pointer advance per step; 0 once the cursor is past its end
    const char *abase = nullptr, *bbase = nullptr;
    uint32_t pitchA = 0, pitchB = 0;
    int rmaxA = 0, rmaxB = 0;
    v4i ra[A_LOADS], rbv[B_LOADS];  // plain vector registers: a struct copy would go through private memory
    // Bias of this wavefront's columns: requested when the first segment of a tile begins (two steps before that
    // tile's first MFMA), parked in LDS when the tile before it has been stored.
    const char *bias_src = reinterpret_cast<const char *>(g.bias ? g.bias : static_cast<const float *>(tiles0 > 0 ? g.Bt[0][0] : g.Bt[1][0]));
    char *bias_w = bias_lds + wave * (WN * 4);
    v4f rbias = {0.f, 0.f, 0.f, 0.f};

#define LP_BEGIN_SEGMENT()                                                                                             \
    if (rowF >= row_tiles) {   /* nothing left: keep repeating the last step */                                        \
        abase -= KSB;                                                                                                  \
        bbase -= KSB;                                                                                                  \
        kstep = 0;                                                                                                     \
        seg_left = 0x7fffffff;                                                                                         \
    } else {                                                                                                           \
        const int part = (partF == 0 && tiles0 > 0) ? 0 : 1;                                                           \
        const int64_t m0f = (int64_t)rowF * BMt;                                                                       \
        pitchA = (uint32_t)g.lda[part] * ES;                                                                           \
        abase = static_cast<const char *>(g.A[part]) + m0f * (int64_t)pitchA;                                          \
        rmaxA = (int)(M_ - 1 - m0f < BMt - 1 ? M_ - 1 - m0f : BMt - 1);                                                \
        const int n0f = colF * BN;                                                                                     \
        const bool secondf = n0f >= g.n_split;                                                                         \
        const int n_endf = secondf ? g.N : (g.n_split < g.N ? g.n_split : g.N);                                        \
        pitchB = (uint32_t)g.ldb[part] * ES;                                                                           \
        bbase = static_cast<const char *>(g.Bt[part][secondf ? 1 : 0]) +                                               \
                (int64_t)(secondf ? n0f - g.n_split : n0f) * (int64_t)pitchB;                                          \
        rmaxB = n_endf - 1 - n0f < BN - 1 ? n_endf - 1 - n0f : BN - 1;                                                 \
        seg_left = part == 0 ? tiles0 : tiles1;                                                                        \
        if (partF == 0) {   /* first segment of a tile */                                                              \
            const int nb_ = g.bias ? min(n0f + wn * WN + 4 * (lane % (WN / 4)), g.N - 4) : 0;                          \
            rbias = *reinterpret_cast<const v4f *>(bias_src + 4 * nb_);                                                \
        }                                                                                                              \
        if (part == 0 && tiles1 > 0) {                                                                                 \
            partF = 1;                                                                                                 \
        } else {                                                                                                       \
            partF = 0;                                                                                                 \
            if (++colF == col_tiles) {                                                                                 \
                colF = 0;                                                                                              \
                rowF += gridDim.x;                                                                                     \
            }                                                                                                          \
        }                                                                                                              \
    }
    // loads of the next K step in pipeline order (possibly the first step of the next output tile)
#define LP_CURSOR()                                                                                                    \
    if (seg_left == 0) { LP_BEGIN_SEGMENT() }
#define LP_FETCH()                                                                                                     \
    LP_CURSOR()                                                                                                        \
    LP_LOADS()
#define LP_LOADS()                                                                                                     \
    _Pragma("unroll") for (int p = 0; p < B_LOADS; ++p)                                                                \
        rbv[p] = *reinterpret_cast<const v4i *>(bbase + ((uint32_t)min(r0 + p * RP, rmaxB) * pitchB + c16));           \
    _Pragma("unroll") for (int p = 0; p < A_LOADS; ++p)                                                                \
        ra[p] = *reinterpret_cast<const v4i *>(abase + ((uint32_t)min(r0 + p * RP, rmaxA) * pitchA + c16));            \
    abase += kstep;                                                                                                    \
    bbase += kstep;                                                                                                    \
    --seg_left;
    // SPLIT: vector j of the step's fetch (A vectors first, then the weight vectors): its copy into a stage, and its
    // reload for the step after next (the cursor's pointers move once per step, in LP_ADVANCE)
#define LP_MOVE_ONE(stage, j)                                                                                          \
    {                                                                                                                  \
        char *As_ = lds + (stage) * STAGE;                                                                             \
        char *Bs_ = As_ + BMt * ROWB;                                                                                  \
        if ((j) < A_LOADS) {                                                                                           \
            LP_STASH_ONE(As_, (j) * TH + tid, ra[(j) < A_LOADS ? (j) : 0])                                             \
            ra[(j) < A_LOADS ? (j) : 0] = *reinterpret_cast<const v4i *>(abase + ((uint32_t)min(r0 + (j) * RP, rmaxA) * pitchA + c16)); \
        } else {                                                                                                       \
            LP_STASH_ONE(Bs_, ((j) - A_LOADS) * TH + tid, rbv[(j) >= A_LOADS ? (j) - A_LOADS : 0])                     \
            rbv[(j) >= A_LOADS ? (j) - A_LOADS : 0] =                                                                  \
                *reinterpret_cast<const v4i *>(bbase + ((uint32_t)min(r0 + ((j) - A_LOADS) * RP, rmaxB) * pitchB + c16)); \
        }                                                                                                              \
    }
#define LP_ADVANCE()                                                                                                   \
    abase += kstep;                                                                                                    \
    bbase += kstep;                                                                                                    \
    --seg_left;
#define LP_PUT_BIAS()                                                                                                  \
    if (lane < WN / 4) *reinterpret_cast<v4f *>(bias_w + 16 * lane) = rbias;
#define LP_STASH_ONE(base_, idx_, v_)                                                                                  \
    if constexpr (SPLIT) {                                                                                             \
        uint2 t0_, t1_, t2_;                                                                                           \
        lp_split3(v_, t0_, t1_, t2_);                                                                                  \
        char *d_ = (base_) + ((idx_) / KQ) * ROWB + (((idx_) % KQ) << 3);                                              \
        *reinterpret_cast<uint2 *>(d_) = t0_;                                                                          \
        *reinterpret_cast<uint2 *>(d_ + KSB / 2) = t1_;                                                                \
        *reinterpret_cast<uint2 *>(d_ + KSB) = t2_;                                                                    \
    } else {                                                                                                           \
        *reinterpret_cast<v4i *>((base_) + ((idx_) / KQ) * ROWB + (((idx_) % KQ) << 4)) = v_;                          \
    }
#define LP_STASH(stage)                                                                                                \
    {                                                                                                                  \
        char *As_ = lds + (stage) * STAGE;                                                                             \
        char *Bs_ = As_ + BMt * ROWB;                                                                                  \
        _Pragma("unroll") for (int p = 0; p < A_LOADS; ++p) { LP_STASH_ONE(As_, p * TH + tid, ra[p]) }                 \
        _Pragma("unroll") for (int p = 0; p < B_LOADS; ++p) { LP_STASH_ONE(Bs_, p * TH + tid, rbv[p]) }                \
    }
    // SPLIT: the three term planes of the K step: two row blocks of the A tile, NB column blocks of the weight tile
#define LP_LOAD_PLANES(stage, a_, b_)                                                                                  \
    {                                                                                                                  \
        const char *As_ = lds + (stage) * STAGE;                                                                       \
        const char *Bs_ = As_ + BMt * ROWB;                                                                            \
        _Pragma("unroll") for (int t = 0; t < 3; ++t) {                                                                \
            _Pragma("unroll") for (int rb = 0; rb < 2; ++rb)                                                           \
                a_[t][rb] = *reinterpret_cast<const v4i *>(As_ + (wm * 64 + rb * 32 + i32) * ROWB + t * (KSB / 2) + 16 * h); \
            _Pragma("unroll") for (int cb = 0; cb < NB; ++cb)                                                          \
                b_[t][cb] = *reinterpret_cast<const v4i *>(Bs_ + (wn * WN + cb * 32 + i32) * ROWB + t * (KSB / 2) + 16 * h); \
        }                                                                                                              \
    }
#define LP_LOAD_PLANE_A(stage, a_, t)                                                                                  \
    {                                                                                                                  \
        const char *As_ = lds + (stage) * STAGE;                                                                       \
        _Pragma("unroll") for (int rb = 0; rb < 2; ++rb)                                                               \
            a_[t][rb] = *reinterpret_cast<const v4i *>(As_ + (wm * 64 + rb * 32 + i32) * ROWB + (t) * (KSB / 2) + 16 * h); \
    }
#define LP_LOAD_PLANE_B(stage, b_, t)                                                                                  \
    {                                                                                                                  \
        const char *Bs_ = lds + (stage) * STAGE + BMt * ROWB;                                                          \
        _Pragma("unroll") for (int cb = 0; cb < NB; ++cb)                                                              \
            b_[t][cb] = *reinterpret_cast<const v4i *>(Bs_ + (wn * WN + cb * 32 + i32) * ROWB + (t) * (KSB / 2) + 16 * h); \
    }
    // one pair of term planes: weight term tb times row term ta, into every accumulator block
#define LP_MFMA_TERM(a_, b_, ta, tb)                                                                                   \
    {                                                                                                                  \
        _Pragma("unroll") for (int rb = 0; rb < 2; ++rb)                                                               \
            _Pragma("unroll") for (int cb = 0; cb < NB; ++cb)                                                          \
                acc[rb][cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, b_[tb][cb]),            \
                                                                      __builtin_bit_cast(v8bf, a_[ta][rb]), acc[rb][cb], 0, 0, 0); \
    }
    // operands of one 32-byte group of the K step: two row blocks of the A tile, NB column blocks of the weight tile
#define LP_LOAD_OPS(stage, kk, a_, b_)                                                                                 \
    {                                                                                                                  \
        const char *As_ = lds + (stage) * STAGE;                                                                       \
        const char *Bs_ = As_ + BMt * ROWB;                                                                            \
        _Pragma("unroll") for (int rb = 0; rb < 2; ++rb)                                                               \
            a_[rb] = *reinterpret_cast<const v4i *>(As_ + (wm * 64 + rb * 32 + i32) * ROWB + (kk) * 32 + 16 * h);      \
        _Pragma("unroll") for (int cb = 0; cb < NB; ++cb)                                                              \
            b_[cb] = *reinterpret_cast<const v4i *>(Bs_ + (wn * WN + cb * 32 + i32) * ROWB + (kk) * 32 + 16 * h);      \
    }
    // k-major order: consecutive MFMAs write different accumulators
#define LP_MFMA_OPS(a_, b_)                                                                                            \
    {                                                                                                                  \
        _Pragma("unroll") for (int s_ = 0; s_ < NtElem<T>::STEPS; ++s_)                                                \
            _Pragma("unroll") for (int rb = 0; rb < 2; ++rb)                                                           \
                _Pragma("unroll") for (int cb = 0; cb < NB; ++cb) NtElem<T>::mfma_step(acc[rb][cb], b_[cb], a_[rb], s_); \
    }
    // the LDS reads of the next group are issued before the MFMAs of the current one (two operand register sets)
#define LP_ORDER() __builtin_amdgcn_sched_barrier(0)

    // One K step: MFMAs on LDS stage `cur`, while the registers of step u+1 go to the other stage and the loads of
    // step u+2 are requested.
    // SPLIT: one K step.  The LDS pipe is shared by eight wavefronts and a wavefront starts a matrix instruction only
    // every 64 clocks, so the term planes are read one term pair ahead of their use instead of all at once behind the
    // barrier, and the tile copy is spread over the last four pairs, a quarter of the fetched vectors under each (a
    // vector is reloaded for the step after next right after its copy, which gives every load a whole step).  In a
    // loop of the same shape without global memory traffic this order kept the matrix pipes 84 % busy against 75 %
    // for "all reads, two pairs, the whole copy, four pairs".  The fences keep the compiler from regrouping.
#define LP_STEP_SPLIT(u_)                                                                                              \
    {                                                                                                                  \
        const int cur = (u_) & 1;                                                                                      \
        LP_CURSOR()   /* the only branch of the step */                                                                \
        LP_LOAD_PLANE_A(cur, sa, 2)                                                                                    \
        LP_LOAD_PLANE_B(cur, sb, 0)                                                                                    \
        LP_LOAD_PLANE_A(cur, sa, 0)                                                                                    \
        LP_ORDER();                                                                                                    \
        LP_MFMA_TERM(sa, sb, 2, 0)                                                                                     \
        LP_LOAD_PLANE_B(cur, sb, 2)                                                                                    \
        LP_ORDER();                                                                                                    \
        LP_MFMA_TERM(sa, sb, 0, 0)                                                                                     \
        LP_LOAD_PLANE_A(cur, sa, 1)                                                                                    \
        lp_unrolled<NV / 4>([&](auto q_) { LP_MOVE_ONE(cur ^ 1, decltype(q_)::value) });                               \
        LP_ORDER();                                                                                                    \
        LP_MFMA_TERM(sa, sb, 0, 2)                                                                                     \
        LP_LOAD_PLANE_B(cur, sb, 1)                                                                                    \
        lp_unrolled<NV / 2 - NV / 4>([&](auto q_) { LP_MOVE_ONE(cur ^ 1, NV / 4 + decltype(q_)::value) });             \
        LP_ORDER();                                                                                                    \
        LP_MFMA_TERM(sa, sb, 1, 0)                                                                                     \
        lp_unrolled<3 * NV / 4 - NV / 2>([&](auto q_) { LP_MOVE_ONE(cur ^ 1, NV / 2 + decltype(q_)::value) });         \
        LP_ORDER();                                                                                                    \
        LP_MFMA_TERM(sa, sb, 0, 1)                                                                                     \
        lp_unrolled<NV - 3 * NV / 4>([&](auto q_) { LP_MOVE_ONE(cur ^ 1, 3 * NV / 4 + decltype(q_)::value) });         \
        LP_ADVANCE()                                                                                                   \
        LP_ORDER();                                                                                                    \
        LP_MFMA_TERM(sa, sb, 1, 1)                                                                                     \
        __syncthreads();                                                                                               \
        if (++ct == n_tiles) {                                                                                         \
            ct = 0;                                                                                                    \
            store_tile(cur);                                                                                           \
        }                                                                                                              \
    }
    // Four-group step (KSB = 128) with the tile copy spread over the groups, a quarter of the fetched vectors under
    // each, every vector reloaded right after its copy (the order that paid in the SPLIT step)
#define LP_STEP_SPREAD(u_)                                                                                             \
    {                                                                                                                  \
        const int cur = (u_) & 1;                                                                                      \
        LP_CURSOR()                                                                                                    \
        LP_LOAD_OPS(cur, 0, a0, b0)                                                                                    \
        LP_LOAD_OPS(cur, 1, a1, b1)                                                                                    \
        LP_ORDER();                                                                                                    \
        LP_MFMA_OPS(a0, b0)                                                                                            \
        lp_unrolled<NV / 4>([&](auto q_) { LP_MOVE_ONE(cur ^ 1, decltype(q_)::value) });                               \
        LP_ORDER();                                                                                                    \
        LP_LOAD_OPS(cur, 2, a0, b0)                                                                                    \
        LP_ORDER();                                                                                                    \
        LP_MFMA_OPS(a1, b1)                                                                                            \
        lp_unrolled<NV / 2 - NV / 4>([&](auto q_) { LP_MOVE_ONE(cur ^ 1, NV / 4 + decltype(q_)::value) });             \
        LP_ORDER();                                                                                                    \
        LP_LOAD_OPS(cur, 3, a1, b1)                                                                                    \
        LP_ORDER();                                                                                                    \
        LP_MFMA_OPS(a0, b0)                                                                                            \
        lp_unrolled<3 * NV / 4 - NV / 2>([&](auto q_) { LP_MOVE_ONE(cur ^ 1, NV / 2 + decltype(q_)::value) });         \
        LP_ORDER();                                                                                                    \
        LP_MFMA_OPS(a1, b1)                                                                                            \
        lp_unrolled<NV - 3 * NV / 4>([&](auto q_) { LP_MOVE_ONE(cur ^ 1, 3 * NV / 4 + decltype(q_)::value) });         \
        LP_ADVANCE()                                                                                                   \
        __syncthreads();                                                                                               \
        if (++ct == n_tiles) {                                                                                         \
            ct = 0;                                                                                                    \
            store_tile(cur);                                                                                           \
        }                                                                                                              \
    }
#define LP_STEP(u_)                                                                                                    \
    {                                                                                                                  \
        const int cur = (u_) & 1;                                                                                      \
        LP_LOAD_OPS(cur, 0, a0, b0)                                                                                    \
        LP_LOAD_OPS(cur, 1, a1, b1)                                                                                    \
        LP_ORDER();                                                                                                    \
        LP_MFMA_OPS(a0, b0)                                                                                            \
        if (KSB == 128) {                                                                                              \
            LP_ORDER();                                                                                                \
            LP_LOAD_OPS(cur, 2, a0, b0)                                                                                \
            LP_ORDER();                                                                                                \
            LP_MFMA_OPS(a1, b1)                                                                                        \
        }                                                                                                              \
        LP_ORDER();                                                                                                    \
        LP_STASH(cur ^ 1)                                                                                              \
        LP_FETCH()                                                                                                     \
        LP_ORDER();                                                                                                    \
        if (KSB == 128) {                                                                                              \
            LP_LOAD_OPS(cur, 3, a1, b1)                                                                                \
            LP_ORDER();                                                                                                \
            LP_MFMA_OPS(a0, b0)                                                                                        \
            LP_ORDER();                                                                                                \
        }                                                                                                              \
        LP_MFMA_OPS(a1, b1)                                                                                            \
        __syncthreads();                                                                                               \
        if (++ct == n_tiles) {                                                                                         \
            ct = 0;                                                                                                    \
            store_tile(cur);                                                                                           \
        }                                                                                                              \
    }

    int rowC = blockIdx.x, colC = 0;  // output tile being accumulated
    int ct = 0;                       // its K step
    // ---- an output tile is complete.  Every wavefront turns its accumulators into stored values, lays them out
    // row-major in a private piece of the LDS stage that was just consumed, and reads them back so that one store
    // instruction writes whole row segments of EPB bytes (LDS operations of one wavefront execute in order; the
    // fences only keep the compiler from reordering them).  The closing barrier keeps the next step's tile copy out
    // of that stage until every wavefront has left it.
    auto store_tile = [&](int stage) __attribute__((always_inline)) {
        const int64_t m0 = (int64_t)rowC * BMt + wm * 64;
        const int n0 = colC * BN;
        if (++colC == col_tiles) {
            colC = 0;
            rowC += gridDim.x;
        }
        const bool second = n0 >= g.n_split;
        const bool scaled = g.rowscale && second;
        char *__restrict__ Cb = static_cast<char *>(second ? g.C[1] : g.C[0]);
        const int64_t pitchC = (int64_t)(second ? g.ldc[1] : g.ldc[0]) * ES;
        const int nw0 = n0 + wn * WN;                      // first column of this wavefront
        const int nshift = second ? g.n_split : 0;
        float rs[2];
#pragma unroll
        for (int rb = 0; rb < 2; ++rb) {
            const int64_t m = m0 + rb * 32 + i32;
            rs[rb] = (scaled && m < M_) ? g.rowscale[g.rowscale_index ? g.rowscale_index[m] : m] : 1.f;
        }
        char *reg = lds + stage * STAGE + wave * (32 * EROW);
        constexpr int LPR = EPB / 16;                      // lanes per row segment
        constexpr int RPI = 64 / LPR;                      // rows per store instruction
#pragma unroll
        for (int rb = 0; rb < 2; ++rb)
#pragma unroll
            for (int pass = 0; pass < NB / CBP; ++pass) {
                v4f gv[GATE ? 32 / RPI : 1];
                if constexpr (GATE) {
#pragma unroll
                    for (int j = 0; j < 32 / RPI; ++j) {
                        const int64_t m = m0 + rb * 32 + j * RPI + lane / LPR;
                        const int n = nw0 + pass * EPC + (lane % LPR) * (16 / ES);
                        gv[j] = v4f{1.f, 1.f, 1.f, 1.f};
                        if (m < M_ && n < g.N) gv[j] = *reinterpret_cast<const v4f *>(g.gate + m * (int64_t)g.ldgate + n);
                    }
                }
#pragma unroll
                for (int cbl = 0; cbl < CBP; ++cbl) {
                    const int cb = pass * CBP + cbl;
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        v4f bias = {0.f, 0.f, 0.f, 0.f};
                        if (g.bias) bias = *reinterpret_cast<const v4f *>(bias_w + 16 * (cb * 8 + 2 * q + h));
                        float y[4];
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            float t = acc[rb][cb][4 * q + e] + bias[e];
                            if (g.relu) t = fmaxf(t, 0.f);
                            y[e] = t * rs[rb];
                            acc[rb][cb][4 * q + e] = 0.f;
                        }
                        NtElem<T>::store4(reinterpret_cast<T *>(reg + i32 * EROW) + cbl * 32 + 8 * q + 4 * h, y);
                    }
                }
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
                for (int j = 0; j < 32 / RPI; ++j) {
                    const int row = j * RPI + lane / LPR, chunk = lane % LPR;
                    v4i v = *reinterpret_cast<const v4i *>(reg + row * EROW + 16 * chunk);
                    if constexpr (GATE) {
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (!(gv[j][e] > 0.f)) v[e] = 0;
                    }
                    const int64_t m = m0 + rb * 32 + row;
                    const int n = nw0 + pass * EPC + chunk * (16 / ES);
                    if (m < M_ && n < g.N) *reinterpret_cast<v4i *>(Cb + m * pitchC + (int64_t)(n - nshift) * ES) = v;
                }
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            }
        LP_PUT_BIAS()   // the next tile's bias (requested two steps ago) replaces the one just used
        __syncthreads();
    };

    LP_FETCH()
    LP_PUT_BIAS()       // first tile
    LP_STASH(0)
    LP_FETCH()
    __syncthreads();
    if constexpr (SPLIT) {
        constexpr int NV = A_LOADS + B_LOADS;   // vectors a thread fetches per step
        v4i sa[3][2], sb[3][NB];
        for (int u = 0; u < n_steps; ++u) LP_STEP_SPLIT(u)
    } else if constexpr (KSB == 128) {
        constexpr int NV = A_LOADS + B_LOADS;
        v4i a0[2], b0[NB], a1[2], b1[NB];
        for (int u = 0; u < n_steps; ++u) LP_STEP_SPREAD(u)
    } else {
        v4i a0[2], b0[NB], a1[2], b1[NB];
        for (int u = 0; u < n_steps; ++u) LP_STEP(u)
    }
#undef LP_STEP
#undef LP_STEP_SPLIT
#undef LP_STEP_SPREAD
#undef LP_STASH_ONE
#undef LP_MOVE_ONE
#undef LP_ADVANCE
#undef LP_LOAD_PLANE_A
#undef LP_LOAD_PLANE_B
#undef LP_LOAD_PLANES
#undef LP_MFMA_TERM
#undef LP_FETCH
#undef LP_CURSOR
#undef LP_LOADS
#undef LP_BEGIN_SEGMENT
#undef LP_STASH
#undef LP_PUT_BIAS
#undef LP_LOAD_OPS
#undef LP_MFMA_OPS
#undef LP_ORDER
}

// ------------------------------------------------------------------------------------------------ NT, bfloat16
// Same product with bfloat16 operands and fp32 accumulation (v_mfma_f32_32x32x16_bf16: lane half h supplies the
// eight consecutive k values 8h..8h+7 of a 16-wide step, i.e. one 16-byte LDS read).  K step 64; LDS rows hold
// 64 + 8 elements (144 bytes = 36 banks: eight consecutive rows start in eight different groups of four banks).
// The weight tile is the row operand of the MFMA, so an accumulator block is the transposed output block and a
// lane owns four consecutive columns of one output row: results are rounded to bfloat16 and stored 8 bytes at a time.
constexpr int HK = 64;
constexpr int H_LD = HK + 8;

template <int NB>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(2))) void gemm_nt_bf16_kernel(GemmNtArgs g) {
    constexpr int BN = 64 * NB;
    constexpr int WN = 32 * NB;
    constexpr int A_LOADS = BM * HK / 8 / kThreads;  // 16-byte vectors per thread: 4
    constexpr int B_LOADS = BN * HK / 8 / kThreads;  // NB * 2
    __shared__ lp_bf16_t As[BM * H_LD];
    __shared__ lp_bf16_t Bs[BN * H_LD];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int i32 = lane & 31, h = lane >> 5;
    const int M_ = g.m_dev ? min(*g.m_dev, g.M) : g.M;  // rows actually present
    const int col_tiles = (g.N + BN - 1) / BN;
    const int slot = blockIdx.x >> 3;
    const int64_t row_tile = (int64_t)(slot / col_tiles) * 8 + (blockIdx.x & 7);
    if (row_tile * BM >= M_) return;
    const int64_t m0 = row_tile * BM;
    const int n0 = (slot % col_tiles) * BN;
    const int tiles0 = (g.K[0] + HK - 1) / HK, tiles1 = (g.K[1] + HK - 1) / HK;
    const int n_tiles = tiles0 + tiles1;

    v16f acc[2][NB];
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
        for (int cb = 0; cb < NB; ++cb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[rb][cb][r] = 0.f;

    v4i ra[A_LOADS], rbv[B_LOADS];
    const v4i zero = {0, 0, 0, 0};
    for (int t = 0; t <= n_tiles; ++t) {
        if (t > 0) {
            __syncthreads();  // previous tile fully consumed
#pragma unroll
            for (int p = 0; p < A_LOADS; ++p) {
                const int idx = p * kThreads + tid;
                *reinterpret_cast<v4i *>(&As[(idx >> 3) * H_LD + ((idx & 7) << 3)]) = ra[p];
            }
#pragma unroll
            for (int p = 0; p < B_LOADS; ++p) {
                const int idx = p * kThreads + tid;
                *reinterpret_cast<v4i *>(&Bs[(idx >> 3) * H_LD + ((idx & 7) << 3)]) = rbv[p];
            }
            __syncthreads();
        }
        if (t < n_tiles) {  // global loads of tile t overlap the MFMAs of tile t-1 below
            const int part = t < tiles0 ? 0 : 1;
            const int k0 = (part ? t - tiles0 : t) * HK;
            const lp_bf16_t *__restrict__ A = static_cast<const lp_bf16_t *>(part ? g.A[1] : g.A[0]);
            const int K = part ? g.K[1] : g.K[0];
            const int64_t lda = part ? g.lda[1] : g.lda[0];
            const int64_t ldb = part ? g.ldb[1] : g.ldb[0];
            const lp_bf16_t *__restrict__ Bt0 = static_cast<const lp_bf16_t *>(part ? g.Bt[1][0] : g.Bt[0][0]);
            const lp_bf16_t *__restrict__ Bt1 = static_cast<const lp_bf16_t *>(part ? g.Bt[1][1] : g.Bt[0][1]);
#pragma unroll
            for (int p = 0; p < A_LOADS; ++p) {
                const int idx = p * kThreads + tid;
                const int k = k0 + ((idx & 7) << 3);
                int64_t m = m0 + (idx >> 3);
                m = m < M_ ? m : M_ - 1;  // rows past the edge only feed outputs that are never stored
                const v4i v = *reinterpret_cast<const v4i *>(A + m * lda + (k < K ? k : K - 8));
                ra[p] = k < K ? v : zero;
            }
#pragma unroll
            for (int p = 0; p < B_LOADS; ++p) {
                const int idx = p * kThreads + tid;
                const int k = k0 + ((idx & 7) << 3);
                int n = n0 + (idx >> 3);
                n = n < g.N ? n : g.N - 1;
                const lp_bf16_t *__restrict__ brow = n < g.n_split ? Bt0 + (int64_t)n * ldb : Bt1 + (int64_t)(n - g.n_split) * ldb;
                const v4i v = *reinterpret_cast<const v4i *>(brow + (k < K ? k : K - 8));
                rbv[p] = k < K ? v : zero;
            }
        }
        if (t == 0) continue;
#pragma unroll
        for (int kk = 0; kk < HK / 16; ++kk) {
            v4i a[2], b[NB];
#pragma unroll
            for (int rb = 0; rb < 2; ++rb)
                a[rb] = *reinterpret_cast<const v4i *>(&As[(wm * 64 + rb * 32 + i32) * H_LD + kk * 16 + 8 * h]);
#pragma unroll
            for (int cb = 0; cb < NB; ++cb)
                b[cb] = *reinterpret_cast<const v4i *>(&Bs[(wn * WN + cb * 32 + i32) * H_LD + kk * 16 + 8 * h]);
#pragma unroll
            for (int rb = 0; rb < 2; ++rb)
#pragma unroll
                for (int cb = 0; cb < NB; ++cb)
                    acc[rb][cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, b[cb]), __builtin_bit_cast(v8bf, a[rb]),
                                                                          acc[rb][cb], 0, 0, 0);
        }
    }

    // transposed accumulator blocks: lane (j = lane % 32, h) holds output row j, columns 8q + 4h .. + 3 in registers 4q..4q+3
#pragma unroll
    for (int rb = 0; rb < 2; ++rb) {
        const int64_t m = m0 + wm * 64 + rb * 32 + i32;
        const bool m_ok = m < M_;
        const float rs_row = (g.rowscale && m_ok) ? g.rowscale[g.rowscale_index ? g.rowscale_index[m] : m] : 1.f;
#pragma unroll
        for (int cb = 0; cb < NB; ++cb)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int n = n0 + wn * WN + cb * 32 + 8 * q + 4 * h;
                const bool n_ok = n < g.N;
                const bool second = n >= g.n_split;
                v4f bias = {0.f, 0.f, 0.f, 0.f};
                if (g.bias && n_ok) bias = *reinterpret_cast<const v4f *>(g.bias + n);
                const float rs = second ? rs_row : 1.f;
                uint32_t packed[2];
#pragma unroll
                for (int e = 0; e < 2; ++e) {
                    float t0 = acc[rb][cb][4 * q + 2 * e] + bias[2 * e], t1 = acc[rb][cb][4 * q + 2 * e + 1] + bias[2 * e + 1];
                    if (g.relu) { t0 = fmaxf(t0, 0.f); t1 = fmaxf(t1, 0.f); }
                    packed[e] = lp_f32x2_to_bf16x2(t0 * rs, t1 * rs);
                }
                if (m_ok && n_ok) {
                    lp_bf16_t *__restrict__ C = static_cast<lp_bf16_t *>(second ? g.C[1] : g.C[0]);
                    const int64_t ldc = second ? g.ldc[1] : g.ldc[0];
                    *reinterpret_cast<uint2 *>(C + m * ldc + (second ? n - g.n_split : n)) = make_uint2(packed[0], packed[1]);
                }
            }
    }
}

// ------------------------------------------------------------------------------------------------ TN
constexpr int TN_LD = 128 + 4;

template <typename T, int MB, int NBk>  // storage type; 32-row / 32-column blocks per wavefront: tile (64*MB) x (64*NBk)
__global__ __launch_bounds__(kThreads) void gemm_tn_kernel(GemmTnArgs g, int chunk) {
    constexpr int TM = 64 * MB, TNn = 64 * NBk;
    constexpr int VE = LpVec<T>::N;  // elements per 16-byte load; bfloat16 is widened to fp32 on its way into LDS
    __shared__ float As[BK * TN_LD];
    __shared__ float Bs[BK * TN_LD];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int i32 = lane & 31, h = lane >> 5;
    const int tiles_n = (g.Nw + TNn - 1) / TNn;
    const int m0 = (blockIdx.x / tiles_n) * TM, n0 = (blockIdx.x % tiles_n) * TNn;
    int64_t Kn_ = g.Kn;
    if (g.kn_dev) {  // reduction length read on the device: share what is really there evenly among the splits
        Kn_ = min((int64_t)*g.kn_dev, (int64_t)g.Kn);
        chunk = (int)(((Kn_ + gridDim.y - 1) / gridDim.y + BK - 1) / BK * BK);
    }
    const int64_t kbeg = (int64_t)blockIdx.y * chunk;
    const int64_t kend = kbeg + chunk < Kn_ ? kbeg + chunk : Kn_;
    const T *__restrict__ At = static_cast<const T *>(g.At);
    const T *__restrict__ Bm = static_cast<const T *>(g.B);

    v16f acc[MB][NBk];
#pragma unroll
    for (int rb = 0; rb < MB; ++rb)
#pragma unroll
        for (int cb = 0; cb < NBk; ++cb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[rb][cb][r] = 0.f;

    constexpr int A_LOADS = BK * TM / VE / kThreads;
    constexpr int B_LOADS = BK * TNn / VE / kThreads;
    float ra[A_LOADS][VE], rbv[B_LOADS][VE];
    int64_t arow[A_LOADS];  // rows of At for the next fetch, looked up one step ahead so that a fetch is one round trip
    auto lookup = [&](int64_t k0) {
#pragma unroll
        for (int p = 0; p < A_LOADS; ++p) {
            const int64_t k = k0 + (p * kThreads + tid) / (TM / VE);
            arow[p] = (g.at_index && k < kend) ? (int64_t)g.at_index[k] : k;
        }
    };
    auto fetch = [&](int64_t k0) {
#pragma unroll
        for (int p = 0; p < A_LOADS; ++p) {
            const int idx = p * kThreads + tid;
            const int kr = idx / (TM / VE), c = (idx % (TM / VE)) * VE;
            const int64_t k = k0 + kr;
#pragma unroll
            for (int e = 0; e < VE; ++e) ra[p][e] = 0.f;
            if (k < kend && m0 + c < g.Mw) LpVec<T>::load(At + arow[p] * g.lda + m0 + c, ra[p]);
        }
#pragma unroll
        for (int p = 0; p < B_LOADS; ++p) {
            const int idx = p * kThreads + tid;
            const int kr = idx / (TNn / VE), c = (idx % (TNn / VE)) * VE;
            const int64_t k = k0 + kr;
#pragma unroll
            for (int e = 0; e < VE; ++e) rbv[p][e] = 0.f;
            if (k < kend && n0 + c < g.Nw) LpVec<T>::load(Bm + k * g.ldb + n0 + c, rbv[p]);
        }
        lookup(k0 + BK);
    };
    auto stash = [&]() {
#pragma unroll
        for (int p = 0; p < A_LOADS; ++p) {
            const int idx = p * kThreads + tid;
            float *dst = &As[(idx / (TM / VE)) * TN_LD + (idx % (TM / VE)) * VE];
#pragma unroll
            for (int e = 0; e < VE; e += 4) *reinterpret_cast<float4 *>(dst + e) = make_float4(ra[p][e], ra[p][e + 1], ra[p][e + 2], ra[p][e + 3]);
        }
#pragma unroll
        for (int p = 0; p < B_LOADS; ++p) {
            const int idx = p * kThreads + tid;
            float *dst = &Bs[(idx / (TNn / VE)) * TN_LD + (idx % (TNn / VE)) * VE];
#pragma unroll
            for (int e = 0; e < VE; e += 4) *reinterpret_cast<float4 *>(dst + e) = make_float4(rbv[p][e], rbv[p][e + 1], rbv[p][e + 2], rbv[p][e + 3]);
        }
    };

    lookup(kbeg);
    if (kbeg < kend) fetch(kbeg);
    for (int64_t k0 = kbeg; k0 < kend; k0 += BK) {
        __syncthreads();
        stash();
        __syncthreads();
        if (k0 + BK < kend) fetch(k0 + BK);
#pragma unroll
        for (int kp = 0; kp < BK / 2; ++kp) {
            float a[MB], b[NBk];
#pragma unroll
            for (int rb = 0; rb < MB; ++rb) a[rb] = As[(kp * 2 + h) * TN_LD + wm * 32 * MB + rb * 32 + i32];
#pragma unroll
            for (int cb = 0; cb < NBk; ++cb) b[cb] = Bs[(kp * 2 + h) * TN_LD + wn * 32 * NBk + cb * 32 + i32];
#pragma unroll
            for (int rb = 0; rb < MB; ++rb)
#pragma unroll
                for (int cb = 0; cb < NBk; ++cb) acc[rb][cb] = mfma32(a[rb], b[cb], acc[rb][cb]);
        }
    }
    float *__restrict__ P = g.partials + (int64_t)blockIdx.y * g.Mw * g.Nw;
#pragma unroll
    for (int cb = 0; cb < NBk; ++cb) {
        const int n = n0 + wn * 32 * NBk + cb * 32 + i32;
        if (n >= g.Nw) continue;
#pragma unroll
        for (int rb = 0; rb < MB; ++rb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int m = m0 + wm * 32 * MB + rb * 32 + 8 * (r >> 2) + 4 * h + (r & 3);
                if (m < g.Mw) P[(int64_t)m * g.Nw + n] = acc[rb][cb][r];
            }
    }
}

// ------------------------------------------------------------------------------------------------ TN, bfloat16
// Weight gradients from bfloat16 operands on the bf16 matrix cores (v_mfma_f32_32x32x16_bf16, fp32 accumulation):
// the products of bfloat16 values are exact in fp32, so this computes the same sums as widening to fp32 first.
// The MFMA wants, per lane, eight consecutive values of the reduction index (nodes) for one fixed column, while
// memory holds node-major rows.  Each loader thread therefore fetches an 8 (nodes) x 8 (columns) block as eight
// 16-byte row pieces, transposes it in registers (byte permutes) and writes eight 16-byte column pieces to an LDS
// tile laid out [column][node]; lanes are assigned so that eight neighbouring lanes write 128 contiguous bytes.
// Workgroups are numbered so that all tiles of one node chunk run on the same XCD and share its L2.
constexpr int TK = 64;          // nodes per step
constexpr int T_LD = TK + 8;    // LDS row: 64 nodes + 8 of padding (144 bytes)

template <int MB, int NBk>  // 32-row / 32-column blocks per wavefront: tile (64*MB) x (64*NBk)
__global__ __launch_bounds__(kThreads) void gemm_tn_bf16_kernel(GemmTnArgs g, int chunk, int splits) {
    constexpr int TM = 64 * MB, TNn = 64 * NBk;
    static_assert(TM + TNn <= kThreads, "one loader task per thread");
    __shared__ lp_bf16_t As[TM * T_LD];
    __shared__ lp_bf16_t Bs[TNn * T_LD];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int i32 = lane & 31, h = lane >> 5;
    const int tiles_n = (g.Nw + TNn - 1) / TNn;
    const int tiles = ((g.Mw + TM - 1) / TM) * tiles_n;
    // linear workgroup ids go round-robin over the eight XCDs: id % 8 picks the XCD, and with it the node chunk
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int tile = slot % tiles;
    const int split = (slot / tiles) * 8 + xcd;
    if (split >= splits) return;
    const int m0 = (tile / tiles_n) * TM, n0 = (tile % tiles_n) * TNn;
    int64_t Kn_ = g.Kn;
    if (g.kn_dev) {  // reduction length read on the device: share what is really there evenly among the splits
        Kn_ = min((int64_t)*g.kn_dev, (int64_t)g.Kn);
        chunk = (int)(((Kn_ + splits - 1) / splits + TK - 1) / TK * TK);
    }
    const int64_t kbeg = (int64_t)split * chunk;
    const int64_t kend = kbeg + chunk < Kn_ ? kbeg + chunk : Kn_;

    // loader task of this thread: threads [0, TM) serve At, threads [TM, TM + TNn) serve B
    const bool loads_a = tid < TM;
    const int task = loads_a ? tid : tid - TM;
    const bool has_task = tid < TM + TNn;
    const int q = task & 7, c = task >> 3;                       // node chunk (8 nodes), column chunk (8 columns)
    const lp_bf16_t *__restrict__ src = static_cast<const lp_bf16_t *>(loads_a ? g.At : g.B);
    const int64_t ld = loads_a ? g.lda : g.ldb;
    const int32_t *__restrict__ row_of = loads_a ? g.at_index : nullptr;
    const int col = (loads_a ? m0 : n0) + 8 * c;
    const bool col_ok = has_task && col < (loads_a ? g.Mw : g.Nw);
    lp_bf16_t *__restrict__ dst = (loads_a ? As : Bs) + (8 * c) * T_LD + 8 * q;

    v16f acc[MB][NBk];
#pragma unroll
    for (int rb = 0; rb < MB; ++rb)
#pragma unroll
        for (int cb = 0; cb < NBk; ++cb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[rb][cb][r] = 0.f;

    v4i rows[8];
    const v4i zero = {0, 0, 0, 0};
    int64_t srow[8];  // source rows of the next fetch, looked up one step ahead so that a fetch is one round trip
    auto lookup = [&](int64_t k0) {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int64_t k = k0 + 8 * q + e;
            srow[e] = (row_of && col_ok && k < kend) ? (int64_t)row_of[k] : k;
        }
    };
    auto fetch = [&](int64_t k0) {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int64_t k = k0 + 8 * q + e;
            rows[e] = zero;
            if (col_ok && k < kend) rows[e] = *reinterpret_cast<const v4i *>(src + srow[e] * ld + col);
        }
        lookup(k0 + TK);
    };
    auto stash = [&]() {
        if (!has_task) return;
#pragma unroll
        for (int j = 0; j < 8; ++j) {  // column j of the block: nodes 0..7, two per 32-bit word
            v4i o;
#pragma unroll
            for (int d = 0; d < 4; ++d)
                o[d] = (int)__builtin_amdgcn_perm((uint32_t)rows[2 * d + 1][j >> 1], (uint32_t)rows[2 * d][j >> 1],
                                                  (j & 1) ? 0x07060302u : 0x05040100u);
            *reinterpret_cast<v4i *>(dst + j * T_LD) = o;
        }
    };

    lookup(kbeg);
    if (kbeg < kend) fetch(kbeg);
    for (int64_t k0 = kbeg; k0 < kend; k0 += TK) {
        __syncthreads();
        stash();
        __syncthreads();
        if (k0 + TK < kend) fetch(k0 + TK);
#pragma unroll
        for (int kk = 0; kk < TK / 16; ++kk) {
            v4i a[MB], b[NBk];
#pragma unroll
            for (int rb = 0; rb < MB; ++rb)
                a[rb] = *reinterpret_cast<const v4i *>(&As[(wm * 32 * MB + rb * 32 + i32) * T_LD + kk * 16 + 8 * h]);
#pragma unroll
            for (int cb = 0; cb < NBk; ++cb)
                b[cb] = *reinterpret_cast<const v4i *>(&Bs[(wn * 32 * NBk + cb * 32 + i32) * T_LD + kk * 16 + 8 * h]);
#pragma unroll
            for (int rb = 0; rb < MB; ++rb)
#pragma unroll
                for (int cb = 0; cb < NBk; ++cb)
                    acc[rb][cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, a[rb]), __builtin_bit_cast(v8bf, b[cb]),
                                                                          acc[rb][cb], 0, 0, 0);
        }
    }
    float *__restrict__ P = g.partials + (int64_t)split * g.Mw * g.Nw;
#pragma unroll
    for (int cb = 0; cb < NBk; ++cb) {
        const int n = n0 + wn * 32 * NBk + cb * 32 + i32;
        if (n >= g.Nw) continue;
#pragma unroll
        for (int rb = 0; rb < MB; ++rb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int m = m0 + wm * 32 * MB + rb * 32 + 8 * (r >> 2) + 4 * h + (r & 3);
                if (m < g.Mw) P[(int64_t)m * g.Nw + n] = acc[rb][cb][r];
            }
    }
}

struct TnPlan {
    int tm, tn, tiles, splits, chunk;
};

TnPlan plan_tn(int32_t Kn, int32_t Mw, int32_t Nw) {
    TnPlan p;
    p.tm = Mw > 64 ? 128 : 64;
    p.tn = Nw > 64 ? 128 : 64;
    p.tiles = (int)(lp_ceil_div(Mw, p.tm) * lp_ceil_div(Nw, p.tn));
    int64_t want = lp_ceil_div(512, p.tiles);           // about two workgroups per compute unit
    int64_t max_by_len = lp_ceil_div(Kn, 8 * BK);       // at least 256 nodes per workgroup
    int64_t s = want < max_by_len ? want : max_by_len;
    if (s < 1) s = 1;
    p.chunk = (int)(lp_ceil_div(lp_ceil_div(Kn, s), 64) * 64);
    p.splits = (int)lp_ceil_div(Kn, p.chunk);
    return p;
}

// ------------------------------------------------------------------------------------------------ fused weight gradients
// [At0 | At1]^T B and the column sums of B for fp32 storage.  256 x 256 output tile, eight wavefronts of 64 x 128,
// 32 nodes per step, two LDS stages with one barrier per step; the reduction over nodes is split across the grid
// and the partial tiles (and partial column sums, written by the workgroups of the first tile row) are folded
// afterwards in a fixed order.
// A loader thread fetches a 4 x 4 block of each operand (four nodes, sixteen bytes of each) and writes it transposed
// (a renaming of registers) into an LDS tile laid out [column][node], pitch 32 nodes + 16 bytes: the layout of the NT
// kernel's stage, so that one 16-byte LDS read per operand block feeds four MFMAs (lane half h supplies nodes
// 4h .. 4h+3 of a group of eight).  The B loaders also add up their blocks for the column sums.
// Loads are unconditional: a node beyond the end of the chunk reads the last valid row and is replaced by zeros.
constexpr int WG_BK = 32;
constexpr int WG_ROWB = WG_BK * 4 + 16;   // bytes per LDS row (one column of an operand tile)
constexpr int WG_THREADS = 512;

template <bool INDEXED>  // rows of At taken through at_index
__global__ __launch_bounds__(WG_THREADS) __attribute__((amdgpu_waves_per_eu(2))) void weight_grads_kernel(WeightGradArgs g, int chunk, int splits,
                                                                                                         int tiles_n, int tiles) {
    constexpr int STAGE = 512 * WG_ROWB;  // 256 columns of each operand
    __shared__ __attribute__((aligned(16))) char lds[2 * STAGE];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int i32 = lane & 31, h = lane >> 5;
    // the tiles of one node chunk get linear ids that are 8 apart: same XCD, so the chunk of B is fetched into one L2
    const int L = blockIdx.x;
    const int s = (L & 7) + 8 * ((L >> 3) / tiles);
    const int t = (L >> 3) % tiles;
    if (s >= splits) return;
    const int m0 = (t / tiles_n) * 256, n0 = (t % tiles_n) * 256;
    const int Mtot = g.Mw[0] + g.Mw[1];
    int64_t Kn_ = g.Kn;
    if (g.kn_dev) {
        Kn_ = min((int64_t)*g.kn_dev, (int64_t)g.Kn);
        chunk = (int)(((Kn_ + splits - 1) / splits + WG_BK - 1) / WG_BK * WG_BK);
    }
    const int64_t kbeg = (int64_t)s * chunk;
    const int64_t kend = kbeg + chunk < Kn_ ? kbeg + chunk : Kn_;

    v16f acc[2][4];
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
        for (int cb = 0; cb < 4; ++cb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[rb][cb][r] = 0.f;
    const bool do_bias = g.dbias != nullptr && m0 == 0;
    const int ng = tid & 7, cg = tid >> 3;     // loader task: nodes 4 ng .. + 3, tile columns 4 cg .. + 3 of both operands
    v4f bsum = {0.f, 0.f, 0.f, 0.f};           // column sums of this thread's B columns over its nodes

    if (kbeg < kend) {
        const int c = 4 * cg;
        const int ma = m0 + c, nb = n0 + c;
        // a thread whose columns lie outside the operands still loads (column 0 of At[1] / B) and drops the values
        const bool a_ok = ma < Mtot, b_ok = nb < g.Nw;
        const float *abase = static_cast<const float *>(g.At[1]);
        int64_t pitch_a = g.lda[1];
        if (ma < g.Mw[0]) { abase = static_cast<const float *>(g.At[0]) + ma; pitch_a = g.lda[0]; }
        else if (a_ok) abase += ma - g.Mw[0];
        const float *bbase = static_cast<const float *>(g.B) + (b_ok ? nb : 0);
        const int64_t klast = Kn_ - 1;
        v4f ra[4], rbv[4];
        int64_t arow[4];
        auto lookup = [&](int64_t k0) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int64_t k = min(k0 + 4 * ng + i, klast);
                arow[i] = INDEXED ? (int64_t)g.at_index[k] : k;
            }
        };
        auto fetch = [&](int64_t k0) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int64_t k = k0 + 4 * ng + i;
                const bool live = k < kend;
                const v4f va = *reinterpret_cast<const v4f *>(abase + arow[i] * pitch_a);
                const v4f vb = *reinterpret_cast<const v4f *>(bbase + min(k, klast) * g.ldb);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    ra[i][e] = (live && a_ok) ? va[e] : 0.f;
                    rbv[i][e] = (live && b_ok) ? vb[e] : 0.f;
                }
            }
        };
        auto stash = [&](int stage) {
            char *As = lds + stage * STAGE, *Bs = As + 256 * WG_ROWB;
#pragma unroll
            for (int j = 0; j < 4; ++j) {   // column j of the block: its four nodes
                *reinterpret_cast<v4f *>(As + (c + j) * WG_ROWB + 16 * ng) = v4f{ra[0][j], ra[1][j], ra[2][j], ra[3][j]};
                *reinterpret_cast<v4f *>(Bs + (c + j) * WG_ROWB + 16 * ng) = v4f{rbv[0][j], rbv[1][j], rbv[2][j], rbv[3][j]};
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) bsum += rbv[i];
        };
        auto compute = [&](int stage, int kk0) {
            const char *As = lds + stage * STAGE, *Bs = As + 256 * WG_ROWB;
#pragma unroll
            for (int kk = kk0; kk < kk0 + 2; ++kk) {   // a group of eight nodes: 32 bytes of every row
                v4f a[2], b[4];
#pragma unroll
                for (int rb = 0; rb < 2; ++rb) a[rb] = *reinterpret_cast<const v4f *>(As + (wm * 64 + rb * 32 + i32) * WG_ROWB + kk * 32 + 16 * h);
#pragma unroll
                for (int cb = 0; cb < 4; ++cb) b[cb] = *reinterpret_cast<const v4f *>(Bs + (wn * 128 + cb * 32 + i32) * WG_ROWB + kk * 32 + 16 * h);
#pragma unroll
                for (int e = 0; e < 4; ++e)
#pragma unroll
                    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
                        for (int cb = 0; cb < 4; ++cb) acc[rb][cb] = mfma32(a[rb][e], b[cb][e], acc[rb][cb]);
            }
        };

        lookup(kbeg);
        fetch(kbeg);
        lookup(kbeg + WG_BK);
        stash(0);
        fetch(kbeg + WG_BK);
        lookup(kbeg + 2 * WG_BK);
        __syncthreads();
        int cur = 0;
        for (int64_t k0 = kbeg; k0 < kend; k0 += WG_BK, cur ^= 1) {
            compute(cur, 0);
            stash(cur ^ 1);                 // registers hold step k0 + 32 (zeros past the end)
            fetch(k0 + 2 * WG_BK);
            lookup(k0 + 3 * WG_BK);
            compute(cur, 2);
            __syncthreads();
        }
    }

    const int64_t ptot = (int64_t)Mtot * g.Nw + g.Nw;
    float *__restrict__ P = g.partials + (int64_t)s * ptot;
#pragma unroll
    for (int cb = 0; cb < 4; ++cb) {
        const int n = n0 + wn * 128 + cb * 32 + i32;
        if (n >= g.Nw) continue;
#pragma unroll
        for (int rb = 0; rb < 2; ++rb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int m = m0 + wm * 64 + rb * 32 + 8 * (r >> 2) + 4 * h + (r & 3);
                if (m < Mtot) P[(int64_t)m * g.Nw + n] = acc[rb][cb][r];
            }
    }
    if (do_bias) {  // the eight node groups of a column meet in LDS and are added in a fixed order
        float *red = reinterpret_cast<float *>(lds);
        __syncthreads();
        *reinterpret_cast<v4f *>(red + ng * 256 + 4 * cg) = bsum;
        __syncthreads();
        if (tid < 256 && n0 + tid < g.Nw) {
            float sum = 0.f;
#pragma unroll
            for (int q = 0; q < 8; ++q) sum += red[q * 256 + tid];
            P[(int64_t)Mtot * g.Nw + n0 + tid] = sum;
        }
    }
}

// The same for fp32 storage with every product formed from bfloat16 terms (see lp_split3): sixteen nodes per step, an
// LDS row (one column of an operand tile) holds the three term planes of its sixteen nodes (112 bytes with padding, the
// layout of the SPLIT NT kernel), and a step is six bf16 MFMAs per accumulator block.  Wavefronts 0-3 load the
// [At0 | At1] tile, wavefronts 4-7 the B tile: a loader thread fetches a 4 x 4 block (four nodes, sixteen bytes of
// each), and for each of its four columns splits the four nodes' values and writes 8 bytes to each plane.  The B
// loaders of every tile add up their blocks for the column sums (kept by the first tile row only).
constexpr int WS_BK = 16;
constexpr int WS_ROWB = 3 * (WS_BK * 2) + 16;

template <bool INDEXED>
__global__ __launch_bounds__(WG_THREADS) __attribute__((amdgpu_waves_per_eu(2))) void weight_grads_split_kernel(WeightGradArgs g, int chunk,
                                                                                                               int splits, int tiles_n, int tiles) {
    constexpr int STAGE = 512 * WS_ROWB;  // 256 columns of each operand
    __shared__ __attribute__((aligned(16))) char lds[2 * STAGE];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int i32 = lane & 31, h = lane >> 5;
    const int L = blockIdx.x;
    const int s = (L & 7) + 8 * ((L >> 3) / tiles);
    const int t = (L >> 3) % tiles;
    if (s >= splits) return;
    const int m0 = (t / tiles_n) * 256, n0 = (t % tiles_n) * 256;
    const int Mtot = g.Mw[0] + g.Mw[1];
    int64_t Kn_ = g.Kn;
    if (g.kn_dev) {
        Kn_ = min((int64_t)*g.kn_dev, (int64_t)g.Kn);
        chunk = (int)(((Kn_ + splits - 1) / splits + WS_BK - 1) / WS_BK * WS_BK);
    }
    const int64_t kbeg = (int64_t)s * chunk;
    const int64_t kend = kbeg + chunk < Kn_ ? kbeg + chunk : Kn_;

    v16f acc[2][4];
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
        for (int cb = 0; cb < 4; ++cb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[rb][cb][r] = 0.f;
    const bool do_bias = g.dbias != nullptr && m0 == 0;
    const bool is_b = tid >= 256;                 // wavefront-uniform: which operand this thread loads
    const int ng = tid & 3, cg = (tid & 255) >> 2;   // loader task: nodes 4 ng .. + 3, tile columns 4 cg .. + 3
    v4f bsum = {0.f, 0.f, 0.f, 0.f};

    if (kbeg < kend) {
        const int c = 4 * cg;
        const int ma = m0 + c, nb = n0 + c;
        // a thread whose columns lie outside its operand still loads (column 0 of At[1] / B) and drops the values
        const bool ok = is_b ? nb < g.Nw : ma < Mtot;
        const float *base;
        int64_t pitch;
        if (is_b) {
            base = static_cast<const float *>(g.B) + (ok ? nb : 0);
            pitch = g.ldb;
        } else if (ma < g.Mw[0]) {
            base = static_cast<const float *>(g.At[0]) + ma;
            pitch = g.lda[0];
        } else {
            base = static_cast<const float *>(g.At[1]) + (ok ? ma - g.Mw[0] : 0);
            pitch = g.lda[1];
        }
        const int64_t klast = Kn_ - 1;
        v4f rv[4];
        int64_t row[4];
        const bool through_list = INDEXED && !is_b;   // wavefront-uniform
        auto lookup = [&](int64_t k0) {   // rows taken through the list are looked up one step ahead of their fetch
            if (!through_list) return;
#pragma unroll
            for (int i = 0; i < 4; ++i) row[i] = (int64_t)g.at_index[min(k0 + 4 * ng + i, klast)];
        };
        auto fetch = [&](int64_t k0) {   // values are used as loaded: see stash_half
            if (through_list) {
#pragma unroll
                for (int i = 0; i < 4; ++i) rv[i] = *reinterpret_cast<const v4f *>(base + row[i] * pitch);
            } else if (k0 + WS_BK <= kend) {   // a whole step inside the chunk (the same for every thread): consecutive rows, no clamp
                const float *p = base + (k0 + 4 * ng) * pitch;
#pragma unroll
                for (int i = 0; i < 4; ++i) rv[i] = *reinterpret_cast<const v4f *>(p + i * pitch);
            } else {
#pragma unroll
                for (int i = 0; i < 4; ++i) rv[i] = *reinterpret_cast<const v4f *>(base + min(k0 + 4 * ng + i, klast) * pitch);
            }
        };
        // columns j0, j0 + 1 of the block (four nodes each, fetched for the step that starts at node k0) into a stage;
        // nodes beyond the end of the chunk and columns outside the operand count as zeros (decided here, not at the
        // load, so that nothing waits for the loads before this point); the second half also adds up the block
        auto stash_half = [&](int stage, int j0, int64_t k0) {
            char *dst = lds + stage * STAGE + (is_b ? 256 * WS_ROWB : 0) + c * WS_ROWB + 8 * ng;
            if (j0 == 0 && !(ok && k0 + WS_BK <= kend)) {   // (a whole step of an operand column that exists needs no masking)
                bool live[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) live[i] = ok && k0 + 4 * ng + i < kend;
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int e = 0; e < 4; ++e) rv[i][e] = live[i] ? rv[i][e] : 0.f;
            }
#pragma unroll
            for (int j = j0; j < j0 + 2; ++j) {
                uint2 t0, t1, t2;
                lp_split3(__builtin_bit_cast(v4i, v4f{rv[0][j], rv[1][j], rv[2][j], rv[3][j]}), t0, t1, t2);
                *reinterpret_cast<uint2 *>(dst + j * WS_ROWB) = t0;
                *reinterpret_cast<uint2 *>(dst + j * WS_ROWB + 2 * WS_BK) = t1;
                *reinterpret_cast<uint2 *>(dst + j * WS_ROWB + 4 * WS_BK) = t2;
            }
            if (j0 == 2) {
#pragma unroll
                for (int i = 0; i < 4; ++i) bsum += rv[i];
            }
        };
        auto stash = [&](int stage, int64_t k0) {
            stash_half(stage, 0, k0);
            stash_half(stage, 2, k0);
        };
        v4i sa[3][2], sb[3][4];
        auto plane_a = [&](int stage, int tt) {
            const char *As = lds + stage * STAGE;
#pragma unroll
            for (int rb = 0; rb < 2; ++rb)
                sa[tt][rb] = *reinterpret_cast<const v4i *>(As + (wm * 64 + rb * 32 + i32) * WS_ROWB + tt * (2 * WS_BK) + 16 * h);
        };
        auto plane_b = [&](int stage, int tt) {
            const char *Bs = lds + stage * STAGE + 256 * WS_ROWB;
#pragma unroll
            for (int cb = 0; cb < 4; ++cb)
                sb[tt][cb] = *reinterpret_cast<const v4i *>(Bs + (wn * 128 + cb * 32 + i32) * WS_ROWB + tt * (2 * WS_BK) + 16 * h);
        };
        auto term = [&](int ta, int tb) {
#pragma unroll
            for (int rb = 0; rb < 2; ++rb)
#pragma unroll
                for (int cb = 0; cb < 4; ++cb)
                    acc[rb][cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, sa[ta][rb]), __builtin_bit_cast(v8bf, sb[tb][cb]),
                                                                          acc[rb][cb], 0, 0, 0);
        };

        lookup(kbeg);
        fetch(kbeg);
        lookup(kbeg + WS_BK);
        stash(0, kbeg);
        fetch(kbeg + WS_BK);
        lookup(kbeg + 2 * WS_BK);
        __syncthreads();
        int cur = 0;
        // One step, in the order of the SPLIT NT kernel's: term planes read one term pair ahead of their use, the tile
        // copy (registers hold step k0 + 16, zeros past the end) in two halves under the second and third pair, then
        // the loads of step k0 + 32, which so have most of a step to arrive.
        for (int64_t k0 = kbeg; k0 < kend; k0 += WS_BK, cur ^= 1) {
            plane_a(cur, 2);
            plane_b(cur, 0);
            plane_a(cur, 0);
            __builtin_amdgcn_sched_barrier(0);
            term(2, 0);
            plane_b(cur, 2);
            __builtin_amdgcn_sched_barrier(0);
            term(0, 0);
            plane_a(cur, 1);
            stash_half(cur ^ 1, 0, k0 + WS_BK);
            __builtin_amdgcn_sched_barrier(0);
            term(0, 2);
            plane_b(cur, 1);
            stash_half(cur ^ 1, 2, k0 + WS_BK);
            fetch(k0 + 2 * WS_BK);
            lookup(k0 + 3 * WS_BK);
            __builtin_amdgcn_sched_barrier(0);
            term(1, 0);
            term(0, 1);
            term(1, 1);
            __syncthreads();
        }
    }

    const int64_t ptot = (int64_t)Mtot * g.Nw + g.Nw;
    float *__restrict__ P = g.partials + (int64_t)s * ptot;
#pragma unroll
    for (int cb = 0; cb < 4; ++cb) {
        const int n = n0 + wn * 128 + cb * 32 + i32;
        if (n >= g.Nw) continue;
#pragma unroll
        for (int rb = 0; rb < 2; ++rb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int m = m0 + wm * 64 + rb * 32 + 8 * (r >> 2) + 4 * h + (r & 3);
                if (m < Mtot) P[(int64_t)m * g.Nw + n] = acc[rb][cb][r];
            }
    }
    if (do_bias) {  // the four node groups of a column meet in LDS and are added in a fixed order
        float *red = reinterpret_cast<float *>(lds);
        __syncthreads();
        if (is_b) *reinterpret_cast<v4f *>(red + ng * 256 + 4 * cg) = bsum;
        __syncthreads();
        if (tid < 256 && n0 + tid < g.Nw) {
            float sum = 0.f;
#pragma unroll
            for (int q = 0; q < 4; ++q) sum += red[q * 256 + tid];
            P[(int64_t)Mtot * g.Nw + n0 + tid] = sum;
        }
    }
}

// The same for bfloat16 storage.  The MFMA (v_mfma_f32_32x32x16_bf16) takes eight consecutive nodes per lane while
// memory is node-major, so a loader thread fetches an 8 x 8 block (eight nodes, sixteen bytes of each), transposes it
// in registers and writes eight 16-byte pieces to an LDS tile laid out [column][node] (pitch 64 + 8 nodes).  256 x 256
// output tile, eight wavefronts of 64 x 128, 64 nodes per step, two LDS stages, one barrier per step; wavefronts 0-3
// load the [At0 | At1] tile, wavefronts 4-7 the B tile.  The column sums of B are not taken here.
template <bool INDEXED>
__global__ __launch_bounds__(WG_THREADS) __attribute__((amdgpu_waves_per_eu(2))) void weight_grads_bf16_kernel(WeightGradArgs g, int chunk,
                                                                                                              int splits, int tiles_n, int tiles) {
    constexpr int STAGE = 512 * T_LD;  // elements per LDS stage: 256 columns of each operand
    __shared__ __attribute__((aligned(16))) lp_bf16_t lds[2 * STAGE];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int i32 = lane & 31, h = lane >> 5;
    const int L = blockIdx.x;
    const int s = (L & 7) + 8 * ((L >> 3) / tiles);
    const int t = (L >> 3) % tiles;
    if (s >= splits) return;
    const int m0 = (t / tiles_n) * 256, n0 = (t % tiles_n) * 256;
    const int Mtot = g.Mw[0] + g.Mw[1];
    int64_t Kn_ = g.Kn;
    if (g.kn_dev) {
        Kn_ = min((int64_t)*g.kn_dev, (int64_t)g.Kn);
        chunk = (int)(((Kn_ + splits - 1) / splits + TK - 1) / TK * TK);
    }
    const int64_t kbeg = (int64_t)s * chunk;
    const int64_t kend = kbeg + chunk < Kn_ ? kbeg + chunk : Kn_;

    v16f acc[2][4];
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
        for (int cb = 0; cb < 4; ++cb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[rb][cb][r] = 0.f;
    // column sums of B: the workgroups of the first tile row add up what their B loaders pass on, per thread for
    // its eight columns and its node chunk (fp32 sums of the transposed node pairs)
    const bool do_bias = g.dbias != nullptr && m0 == 0;
    float bsum[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

    if (kbeg < kend) {
        // loader task: node chunk q (8 nodes) and column chunk c (8 columns) of one operand tile
        const bool loads_a = tid < 256;
        const int task = tid & 255;
        const int q = task & 7, c = task >> 3;
        const int col = (loads_a ? m0 : n0) + 8 * c;
        const bool col_ok = col < (loads_a ? Mtot : g.Nw);
        // a thread whose columns lie outside the operand still loads (column 0) and drops the values
        const lp_bf16_t *src;
        int64_t pitch;
        if (!loads_a) { src = static_cast<const lp_bf16_t *>(g.B) + (col_ok ? col : 0); pitch = g.ldb; }
        else if (col < g.Mw[0]) { src = static_cast<const lp_bf16_t *>(g.At[0]) + col; pitch = g.lda[0]; }
        else { src = static_cast<const lp_bf16_t *>(g.At[1]) + (col_ok ? col - g.Mw[0] : 0); pitch = g.lda[1]; }
        const bool indexed = INDEXED && loads_a;
        const int dst_off = (loads_a ? 0 : 256 * T_LD) + (8 * c) * T_LD + 8 * q;
        const int64_t klast = Kn_ - 1;
        v4i rows[8];
        int64_t srow[8];
        auto lookup = [&](int64_t k0) {   // rows taken through the list are looked up one step ahead of their fetch
            if (!indexed) return;
#pragma unroll
            for (int e = 0; e < 8; ++e) srow[e] = (int64_t)g.at_index[min(k0 + 8 * q + e, klast)];
        };
        auto fetch = [&](int64_t k0) {
            if (k0 + TK <= kend) {   // the whole step lies inside the chunk (the same for every thread): nothing to clamp or mask
                if (indexed) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) rows[e] = *reinterpret_cast<const v4i *>(src + srow[e] * pitch);
                } else {
                    const lp_bf16_t *p = src + (k0 + 8 * q) * pitch;
#pragma unroll
                    for (int e = 0; e < 8; ++e) rows[e] = *reinterpret_cast<const v4i *>(p + e * pitch);
                }
                if (!col_ok) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) rows[e] = v4i{0, 0, 0, 0};
                }
                return;
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const bool live = col_ok && k0 + 8 * q + e < kend;
                const int64_t row = indexed ? srow[e] : min(k0 + 8 * q + e, klast);
                const v4i v = *reinterpret_cast<const v4i *>(src + row * pitch);
#pragma unroll
                for (int d = 0; d < 4; ++d) rows[e][d] = live ? v[d] : 0;
            }
        };
        auto stash = [&](int stage) {
            lp_bf16_t *dst = lds + stage * STAGE + dst_off;
#pragma unroll
            for (int j = 0; j < 8; ++j) {  // column j of the block: nodes 0..7, two per 32-bit word
                v4i o;
#pragma unroll
                for (int d = 0; d < 4; ++d)
                    o[d] = (int)__builtin_amdgcn_perm((uint32_t)rows[2 * d + 1][j >> 1], (uint32_t)rows[2 * d][j >> 1],
                                                      (j & 1) ? 0x07060302u : 0x05040100u);
                *reinterpret_cast<v4i *>(dst + j * T_LD) = o;
                if (do_bias && !loads_a) {
#pragma unroll
                    for (int d = 0; d < 4; ++d)
                        bsum[j] += __uint_as_float((uint32_t)o[d] << 16) + __uint_as_float((uint32_t)o[d] & 0xffff0000u);
                }
            }
        };
        auto compute = [&](int stage, int kk0) {
            const lp_bf16_t *As = lds + stage * STAGE, *Bs = As + 256 * T_LD;
#pragma unroll
            for (int kk = kk0; kk < kk0 + TK / 32; ++kk) {
                v4i a[2], b[4];
#pragma unroll
                for (int rb = 0; rb < 2; ++rb) a[rb] = *reinterpret_cast<const v4i *>(&As[(wm * 64 + rb * 32 + i32) * T_LD + kk * 16 + 8 * h]);
#pragma unroll
                for (int cb = 0; cb < 4; ++cb) b[cb] = *reinterpret_cast<const v4i *>(&Bs[(wn * 128 + cb * 32 + i32) * T_LD + kk * 16 + 8 * h]);
#pragma unroll
                for (int rb = 0; rb < 2; ++rb)
#pragma unroll
                    for (int cb = 0; cb < 4; ++cb)
                        acc[rb][cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, a[rb]), __builtin_bit_cast(v8bf, b[cb]),
                                                                              acc[rb][cb], 0, 0, 0);
            }
        };

        lookup(kbeg);
        fetch(kbeg);
        lookup(kbeg + TK);
        stash(0);
        fetch(kbeg + TK);
        lookup(kbeg + 2 * TK);
        __syncthreads();
        int cur = 0;
        for (int64_t k0 = kbeg; k0 < kend; k0 += TK, cur ^= 1) {
            compute(cur, 0);
            stash(cur ^ 1);                 // registers hold step k0 + 64 (zeros past the end)
            fetch(k0 + 2 * TK);
            lookup(k0 + 3 * TK);
            compute(cur, TK / 32);
            __syncthreads();
        }
    }

    const int64_t ptot = (int64_t)Mtot * g.Nw + g.Nw;
    float *__restrict__ P = g.partials + (int64_t)s * ptot;
#pragma unroll
    for (int cb = 0; cb < 4; ++cb) {
        const int n = n0 + wn * 128 + cb * 32 + i32;
        if (n >= g.Nw) continue;
#pragma unroll
        for (int rb = 0; rb < 2; ++rb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int m = m0 + wm * 64 + rb * 32 + 8 * (r >> 2) + 4 * h + (r & 3);
                if (m < Mtot) P[(int64_t)m * g.Nw + n] = acc[rb][cb][r];
            }
    }
    if (do_bias) {  // the eight node chunks of a column meet in LDS and are added in a fixed order
        float *red = reinterpret_cast<float *>(lds);
        __syncthreads();
        if (tid >= 256) {
            const int task = tid & 255;
#pragma unroll
            for (int j = 0; j < 8; ++j) red[(task & 7) * 256 + 8 * (task >> 3) + j] = bsum[j];
        }
        __syncthreads();
        if (tid < 256 && n0 + tid < g.Nw) {
            float sum = 0.f;
#pragma unroll
            for (int qq = 0; qq < 8; ++qq) sum += red[qq * 256 + tid];
            P[(int64_t)Mtot * g.Nw + n0 + tid] = sum;
        }
    }
}

// out = sum over the `rows` partial rows of P[rows, n0 + n1 + n2], columns routed to three outputs.  Same order of
// additions as colsum_partial_kernel.
__global__ __launch_bounds__(kThreads) void weight_grads_fold_kernel(const float *__restrict__ P, int rows, int64_t row_len, int64_t n0,
                                                                      int64_t n1, int64_t n2, float *__restrict__ o0, float *__restrict__ o1,
                                                                      float *__restrict__ o2) {
    __shared__ float red[4][64][4];
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    const int64_t NV = row_len / 4;            // pitch of a partial row in 16-byte pieces
    const int64_t NC = (n0 + n1 + n2) / 4;     // pieces that are summed
    const int64_t cv = (int64_t)blockIdx.x * 64 + tx;
    v4f a0 = {0.f, 0.f, 0.f, 0.f}, a1 = a0;
    if (cv < NC) {
        int r = ty;
        for (; r + 12 < rows; r += 16) {
            const v4f x0 = *reinterpret_cast<const v4f *>(P + ((int64_t)r * NV + cv) * 4);
            const v4f x1 = *reinterpret_cast<const v4f *>(P + ((int64_t)(r + 4) * NV + cv) * 4);
            const v4f x2 = *reinterpret_cast<const v4f *>(P + ((int64_t)(r + 8) * NV + cv) * 4);
            const v4f x3 = *reinterpret_cast<const v4f *>(P + ((int64_t)(r + 12) * NV + cv) * 4);
            a0 += x0;
            a1 += x1;
            a0 += x2;
            a1 += x3;
        }
        for (; r < rows; r += 4) a0 += *reinterpret_cast<const v4f *>(P + ((int64_t)r * NV + cv) * 4);
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) red[ty][tx][e] = a0[e] + a1[e];
    __syncthreads();
    if (ty == 0 && cv < NC) {
        const int64_t col = cv * 4;
        float *dst = col < n0 ? o0 + col : (col < n0 + n1 ? o1 + (col - n0) : o2 + (col - n0 - n1));
#pragma unroll
        for (int e = 0; e < 4; ++e) dst[e] = (red[0][tx][e] + red[1][tx][e]) + (red[2][tx][e] + red[3][tx][e]);
    }
}

// ------------------------------------------------------------------------------------------------ small helpers
template <typename T>
__global__ void transpose_kernel(const T *__restrict__ in, int rows, int cols, T *__restrict__ out) {
    __shared__ T tile[32][33];
    const int c = blockIdx.x * 32 + threadIdx.x, r0 = blockIdx.y * 32;
    for (int i = threadIdx.y; i < 32; i += blockDim.y)
        if (r0 + i < rows && c < cols) tile[i][threadIdx.x] = in[(int64_t)(r0 + i) * cols + c];
    __syncthreads();
    const int orow0 = blockIdx.x * 32, ocol = r0 + threadIdx.x;
    for (int i = threadIdx.y; i < 32; i += blockDim.y)
        if (orow0 + i < cols && ocol < rows) out[(int64_t)(orow0 + i) * rows + ocol] = tile[threadIdx.x][i];
}

template <typename T>
__global__ void transpose_batch_kernel(TransposeBatch b) {
    __shared__ T tile[32][33];
    const int z = blockIdx.z;
    const int rows = b.rows[z], cols = b.cols[z];
    const int c = blockIdx.x * 32 + threadIdx.x, r0 = blockIdx.y * 32;
    if (blockIdx.x * 32 >= cols || r0 >= rows) return;   // the grid covers the largest matrix of the batch
    const T *__restrict__ in = static_cast<const T *>(b.in[z]);
    T *__restrict__ out = static_cast<T *>(b.out[z]);
    for (int i = threadIdx.y; i < 32; i += blockDim.y)
        if (r0 + i < rows && c < cols) tile[i][threadIdx.x] = in[(int64_t)(r0 + i) * cols + c];
    __syncthreads();
    const int orow0 = blockIdx.x * 32, ocol = r0 + threadIdx.x;
    for (int i = threadIdx.y; i < 32; i += blockDim.y)
        if (orow0 + i < cols && ocol < rows) out[(int64_t)(orow0 + i) * rows + ocol] = tile[threadIdx.x][i];
}

constexpr int kColsumRows = 256;  // rows folded by one workgroup

// partials[chunk, c] = sum of in[r, c] over the rows r of the chunk, rows taken in a fixed order, summed in fp32.
// Workgroup: 64 column vectors (16 bytes each) x 4 row lanes; grid (column groups, row chunks).
template <typename T>
__global__ __launch_bounds__(kThreads) void colsum_partial_kernel(const T *__restrict__ in, int64_t M, int64_t NV,
                                                                  float *__restrict__ partials, const int32_t *__restrict__ m_dev) {
    if (m_dev) M = *m_dev < M ? *m_dev : M;  // rows actually present
    constexpr int VE = LpVec<T>::N;
    __shared__ float red[4][64][VE];
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    const int64_t cv = (int64_t)blockIdx.x * 64 + tx;
    const int64_t r0 = (int64_t)blockIdx.y * kColsumRows;
    const int64_t r1 = r0 + kColsumRows < M ? r0 + kColsumRows : M;
    float acc0[VE], acc1[VE];
#pragma unroll
    for (int e = 0; e < VE; ++e) acc0[e] = acc1[e] = 0.f;
    if (cv < NV) {
        int64_t r = r0 + ty;
        for (; r + 12 < r1; r += 16) {
            float x0[VE], x1[VE], x2[VE], x3[VE];
            LpVec<T>::load(in + (r * NV + cv) * VE, x0);
            LpVec<T>::load(in + ((r + 4) * NV + cv) * VE, x1);
            LpVec<T>::load(in + ((r + 8) * NV + cv) * VE, x2);
            LpVec<T>::load(in + ((r + 12) * NV + cv) * VE, x3);
#pragma unroll
            for (int e = 0; e < VE; ++e) {
                acc0[e] += x0[e];
                acc1[e] += x1[e];
                acc0[e] += x2[e];
                acc1[e] += x3[e];
            }
        }
        for (; r < r1; r += 4) {
            float x0[VE];
            LpVec<T>::load(in + (r * NV + cv) * VE, x0);
#pragma unroll
            for (int e = 0; e < VE; ++e) acc0[e] += x0[e];
        }
    }
#pragma unroll
    for (int e = 0; e < VE; ++e) red[ty][tx][e] = acc0[e] + acc1[e];
    __syncthreads();
    if (ty == 0 && cv < NV) {
#pragma unroll
        for (int e = 0; e < VE; ++e)
            partials[((int64_t)blockIdx.y * NV + cv) * VE + e] = (red[0][tx][e] + red[1][tx][e]) + (red[2][tx][e] + red[3][tx][e]);
    }
}

__global__ void zero_kernel(float4 *__restrict__ p4, int64_t n4, float *__restrict__ tail, int n_tail) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n4) p4[i] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (i < n_tail) tail[i] = 0.f;
}

}  // namespace

int lp_compute_units() {
    static int cus = 0;
    if (cus == 0) {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) == hipSuccess && hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0)
            cus = n;
        else
            cus = 256;
    }
    return cus;
}

int lp_launch_gemm_nt(const GemmNtArgs &a, hipStream_t st) {
    if (a.M <= 0 || a.N <= 0) return LP_OK;
    for (int s = 0; s < 2; ++s) {
        if (a.K[s] <= 0) continue;
        const int ve = lp_vec_elems(a.dtype);
        if ((a.K[s] % ve) || (a.lda[s] % ve) || (a.ldb[s] % ve)) return LP_ERR_UNSUPPORTED;
        if (!a.A[s] || !a.Bt[s][0] || !lp_aligned16(a.A[s]) || !lp_aligned16(a.Bt[s][0])) return LP_ERR_INVALID_ARG;
        if (a.n_split < a.N && (!a.Bt[s][1] || !lp_aligned16(a.Bt[s][1]))) return LP_ERR_INVALID_ARG;
    }
    if (!a.C[0] || (a.n_split < a.N && !a.C[1])) return LP_ERR_INVALID_ARG;
    if (a.dtype != LP_F32 && a.dtype != LP_BF16) return LP_ERR_UNSUPPORTED;
    if (a.gate) {   // fp32 storage, one output, gate rows in whole 16-byte vectors
        if (a.dtype != LP_F32 || a.n_split < a.N) return LP_ERR_UNSUPPORTED;
        if (!lp_aligned16(a.gate) || (a.ldgate & 3) || a.ldgate < a.N) return LP_ERR_INVALID_ARG;
    }
    LpTimedScope timed(LP_KC_GEMM_NT, st);
    const bool bf16 = a.dtype == LP_BF16;
    if (bf16 && ((a.N & 3) || (a.n_split & 3) || (a.ldc[0] & 3) || (a.n_split < a.N && (a.ldc[1] & 3)))) return LP_ERR_UNSUPPORTED;
    // fast path: K parts in whole steps (64 bytes of a row, 128 for the widest tile), no column tile straddling the
    // output split
    const int es = lp_elem_bytes(a.dtype);
    const int fast_bn = a.N > 128 ? 256 : 128;
    const int ve16 = 16 / es;
    // (at least two K steps per output tile: the bias of a tile is requested while the tile before it is finishing)
    const bool fast_ok = a.N > 64 && (a.K[0] * es % 64 == 0) && (a.K[1] * es % 64 == 0) && (int64_t)(a.K[0] + a.K[1]) * es >= 128 &&
                         (a.n_split >= a.N || a.n_split % fast_bn == 0) &&
                         // whole 16-byte pieces of output rows
                         a.N % ve16 == 0 && a.ldc[0] % ve16 == 0 && lp_aligned16(a.C[0]) && (!a.bias || lp_aligned16(a.bias)) &&
                         (a.n_split >= a.N || (a.ldc[1] % ve16 == 0 && lp_aligned16(a.C[1]))) &&
                         // row offsets inside a tile are formed in 32 bits
                         (int64_t)std::max(std::max(a.lda[0], a.lda[1]), std::max(a.ldb[0], a.ldb[1])) * es * 256 < ((int64_t)1 << 32);
    auto grid_for = [&](int bn) {
        const int64_t row_tiles8 = lp_ceil_div(lp_ceil_div(a.M, BM), 8) * 8;
        return dim3((unsigned)(row_tiles8 * lp_ceil_div(a.N, bn)));
    };
    if (fast_ok) {
        // persistent workgroups filling every compute unit; the widest tile (256 x 256, eight wavefronts, 128-byte
        // K step, one workgroup per compute unit) when K allows
        // (with fewer 256-row tiles than compute units, 128-row tiles spread the same work over twice as many of them)
        const bool big = fast_bn == 256 && (a.K[0] * es % 128 == 0) && (a.K[1] * es % 128 == 0) && (int64_t)(a.K[0] + a.K[1]) * es >= 256 &&
                         lp_ceil_div(a.M, 256) >= (int64_t)lp_compute_units();
        const int bm = big ? 256 : 128;
        const int64_t row_tiles = lp_ceil_div(a.M, bm);
        const int64_t slots = (big ? 1 : 2) * (int64_t)lp_compute_units();
        const dim3 pgrid((unsigned)(row_tiles < slots ? row_tiles : slots));
        const int64_t steps_per_wg = lp_ceil_div(row_tiles, (int64_t)pgrid.x) * lp_ceil_div(a.N, fast_bn) *
                                     ((int64_t)(a.K[0] + a.K[1]) * es / 64);
        if (steps_per_wg >= (int64_t)1 << 31) return LP_ERR_UNSUPPORTED;  // the kernels count K steps in 32 bits
#define LP_NT_FAST(T, GATED)                                                                                                  \
        if (big) hipLaunchKernelGGL((gemm_nt_fast_kernel<T, 4, 4, 128, false, GATED>), pgrid, dim3(512), 0, st, a);               \
        else if (fast_bn == 256) hipLaunchKernelGGL((gemm_nt_fast_kernel<T, 4, 2, 64, false, GATED>), pgrid, dim3(256), 0, st, a); \
        else hipLaunchKernelGGL((gemm_nt_fast_kernel<T, 2, 2, 64, false, GATED>), pgrid, dim3(256), 0, st, a);
#define LP_NT_SPLIT(GATED)                                                                                                    \
        if (fast_bn == 256 && lp_ceil_div(a.M, 256) >= (int64_t)lp_compute_units()) {                                         \
            /* sixteen values of a row per K step; 256-row tiles once they fill every compute unit */                         \
            const int64_t rt = lp_ceil_div(a.M, 256);                                                                         \
            const dim3 sgrid((unsigned)(rt < lp_compute_units() ? rt : lp_compute_units()));                                  \
            hipLaunchKernelGGL((gemm_nt_fast_kernel<float, 4, 4, 64, true, GATED>), sgrid, dim3(512), 0, st, a);              \
        } else {                                                                                                              \
            const int64_t rt = lp_ceil_div(a.M, 128);                                                                         \
            const int64_t sl = (fast_bn == 256 ? 1 : 2) * (int64_t)lp_compute_units();   /* resident workgroups (LDS) */      \
            const dim3 sgrid((unsigned)(rt < sl ? rt : sl));                                                                  \
            if (fast_bn == 256) hipLaunchKernelGGL((gemm_nt_fast_kernel<float, 4, 2, 64, true, GATED>), sgrid, dim3(256), 0, st, a); \
            else hipLaunchKernelGGL((gemm_nt_fast_kernel<float, 2, 2, 64, true, GATED>), sgrid, dim3(256), 0, st, a);         \
        }
        if (bf16) {
            LP_NT_FAST(lp_bf16_t, false)
        } else if (a.fp32_products == LP_FP32_PRODUCTS_BF16X6) {
            if (a.gate) { LP_NT_SPLIT(true) } else { LP_NT_SPLIT(false) }
        } else if (a.gate) {
            LP_NT_FAST(float, true)
        } else {
            LP_NT_FAST(float, false)
        }
#undef LP_NT_FAST
#undef LP_NT_SPLIT
    } else if (bf16) {
        const int bn = a.N > 128 ? 256 : (a.N > 64 ? 128 : 64);
        if (bn == 256) hipLaunchKernelGGL((gemm_nt_bf16_kernel<4>), grid_for(256), dim3(kThreads), 0, st, a);
        else if (bn == 128) hipLaunchKernelGGL((gemm_nt_bf16_kernel<2>), grid_for(128), dim3(kThreads), 0, st, a);
        else hipLaunchKernelGGL((gemm_nt_bf16_kernel<1>), grid_for(64), dim3(kThreads), 0, st, a);
    } else if (a.N > 128) {
        hipLaunchKernelGGL((gemm_nt_kernel<4>), grid_for(256), dim3(kThreads), 0, st, a);
    } else if (a.N > 64) {
        hipLaunchKernelGGL((gemm_nt_kernel<2>), grid_for(128), dim3(kThreads), 0, st, a);
    } else {
        hipLaunchKernelGGL((gemm_nt_kernel<1>), grid_for(64), dim3(kThreads), 0, st, a);
    }
    return lp_after_launch();
}

size_t lp_gemm_tn_partials_bytes(int32_t Kn, int32_t Mw, int32_t Nw) {
    if (Kn <= 0 || Mw <= 0 || Nw <= 0) return 0;
    const TnPlan p = plan_tn(Kn, Mw, Nw);
    return lp_align_up(sizeof(float) * (size_t)p.splits * Mw * Nw) + lp_colsum_partials_bytes(p.splits, (int64_t)Mw * Nw);
}

int lp_launch_gemm_tn(const GemmTnArgs &a, hipStream_t st) {
    if (a.Mw <= 0 || a.Nw <= 0) return LP_OK;
    const int ve = lp_vec_elems(a.dtype);
    if ((a.dtype != LP_F32 && a.dtype != LP_BF16) || (a.Mw % ve) || (a.Nw % ve) || (a.lda % ve) || (a.ldb % ve)) return LP_ERR_UNSUPPORTED;
    if (!a.C || !a.partials) return LP_ERR_INVALID_ARG;
    if (a.Kn <= 0) return lp_launch_zero(a.C, (int64_t)a.Mw * a.Nw, st);
    if (!a.At || !a.B || !lp_aligned16(a.At) || !lp_aligned16(a.B)) return LP_ERR_INVALID_ARG;
    LpTimedScope timed(LP_KC_GEMM_TN, st);
    const TnPlan p = plan_tn(a.Kn, a.Mw, a.Nw);
    const dim3 grid(p.tiles, p.splits);
#define LP_TN_LAUNCH(T)                                                                                                   \
    if (p.tm == 128 && p.tn == 128) hipLaunchKernelGGL((gemm_tn_kernel<T, 2, 2>), grid, dim3(kThreads), 0, st, a, p.chunk); \
    else if (p.tm == 128) hipLaunchKernelGGL((gemm_tn_kernel<T, 2, 1>), grid, dim3(kThreads), 0, st, a, p.chunk);           \
    else if (p.tn == 128) hipLaunchKernelGGL((gemm_tn_kernel<T, 1, 2>), grid, dim3(kThreads), 0, st, a, p.chunk);           \
    else hipLaunchKernelGGL((gemm_tn_kernel<T, 1, 1>), grid, dim3(kThreads), 0, st, a, p.chunk);
    if (a.dtype == LP_BF16) {
        const dim3 bgrid((unsigned)(p.tiles * lp_ceil_div(p.splits, 8) * 8));
        if (p.tm == 128 && p.tn == 128) hipLaunchKernelGGL((gemm_tn_bf16_kernel<2, 2>), bgrid, dim3(kThreads), 0, st, a, p.chunk, p.splits);
        else if (p.tm == 128) hipLaunchKernelGGL((gemm_tn_bf16_kernel<2, 1>), bgrid, dim3(kThreads), 0, st, a, p.chunk, p.splits);
        else if (p.tn == 128) hipLaunchKernelGGL((gemm_tn_bf16_kernel<1, 2>), bgrid, dim3(kThreads), 0, st, a, p.chunk, p.splits);
        else hipLaunchKernelGGL((gemm_tn_bf16_kernel<1, 1>), bgrid, dim3(kThreads), 0, st, a, p.chunk, p.splits);
    } else {
        LP_TN_LAUNCH(float)
    }
#undef LP_TN_LAUNCH
    LP_TRY(lp_after_launch());
    // fold the partial tiles: a column sum of the [splits, Mw*Nw] matrix
    const int64_t n = (int64_t)a.Mw * a.Nw;
    return lp_launch_colsum(a.partials, LP_F32, p.splits, n, a.C, a.partials + lp_align_up(sizeof(float) * (size_t)p.splits * n) / sizeof(float), st);
}

namespace {
struct WgPlan {
    bool fused = false;
    int tiles_m = 0, tiles_n = 0, tiles = 0, splits = 0, chunk = 0;
};
WgPlan plan_weight_grads(int32_t dtype, int32_t Kn, int32_t Mw0, int32_t Mw1, int32_t Nw) {
    WgPlan p;
    const int Mtot = Mw0 + Mw1;
    // fused path: fp32, 16-byte pieces never straddle the two operands, tiles reasonably full
    const int ve = lp_vec_elems(dtype);
    p.fused = (dtype == LP_F32 || dtype == LP_BF16) && Kn > 0 && Mw1 > 0 && (Mw0 % ve) == 0 && (Mw1 % ve) == 0 && (Nw % ve) == 0 &&
              Mtot >= 192 && Nw >= 192 && (Mtot % 256 == 0 || Mtot % 256 >= 128) && (Nw % 256 == 0 || Nw % 256 >= 128);
    if (!p.fused) return p;
    const int step = dtype == LP_BF16 ? TK : WG_BK;   // nodes per step
    p.tiles_m = (int)lp_ceil_div(Mtot, 256);
    p.tiles_n = (int)lp_ceil_div(Nw, 256);
    p.tiles = p.tiles_m * p.tiles_n;
    int64_t want = lp_ceil_div(lp_compute_units(), p.tiles);   // one workgroup per compute unit
    const int64_t max_by_len = lp_ceil_div(Kn, 256);           // at least 256 nodes per workgroup
    int64_t s = want < max_by_len ? want : max_by_len;
    if (s < 1) s = 1;
    p.chunk = (int)(lp_ceil_div(lp_ceil_div(Kn, s), step) * step);
    p.splits = (int)lp_ceil_div(Kn, p.chunk);
    return p;
}
}  // namespace

size_t lp_weight_grads_partials_bytes(int32_t dtype, int32_t Kn, int32_t Mw0, int32_t Mw1, int32_t Nw) {
    if (Kn <= 0 || Nw <= 0) return 0;
    const WgPlan p = plan_weight_grads(dtype, Kn, Mw0, Mw1, Nw);
    if (p.fused) return lp_align_up(sizeof(float) * (size_t)p.splits * ((size_t)(Mw0 + Mw1) * Nw + Nw));
    const size_t a = Mw0 > 0 ? lp_gemm_tn_partials_bytes(Kn, Mw0, Nw) : 0, b = Mw1 > 0 ? lp_gemm_tn_partials_bytes(Kn, Mw1, Nw) : 0;
    return a > b ? a : b;
}

int lp_launch_weight_grads(const WeightGradArgs &a, hipStream_t st) {
    if (a.Nw <= 0) return LP_OK;
    const WgPlan p = plan_weight_grads(a.dtype, a.Kn, a.Mw[0], a.Mw[1], a.Nw);
    const int ve = lp_vec_elems(a.dtype);
    const bool aligned = lp_aligned16(a.At[0]) && lp_aligned16(a.At[1]) && lp_aligned16(a.B) && (a.lda[0] % ve) == 0 && (a.lda[1] % ve) == 0 &&
                         (a.ldb % ve) == 0 && lp_aligned16(a.C[0]) && lp_aligned16(a.C[1]) && (!a.dbias || lp_aligned16(a.dbias));
    if (p.fused && aligned && (a.Mw[0] == 0 || (a.At[0] && a.C[0])) && a.At[1] && a.B && a.C[1] && a.partials) {
        const bool bf16 = a.dtype == LP_BF16;
        LpTimedScope timed(LP_KC_GEMM_TN, st);
        const unsigned grid = (unsigned)(p.tiles * lp_ceil_div(p.splits, 8) * 8);
        if (bf16) {
            if (a.at_index) hipLaunchKernelGGL(weight_grads_bf16_kernel<true>, dim3(grid), dim3(WG_THREADS), 0, st, a, p.chunk, p.splits, p.tiles_n, p.tiles);
            else hipLaunchKernelGGL(weight_grads_bf16_kernel<false>, dim3(grid), dim3(WG_THREADS), 0, st, a, p.chunk, p.splits, p.tiles_n, p.tiles);
        } else if (a.fp32_products == LP_FP32_PRODUCTS_BF16X6) {
            if (a.at_index) hipLaunchKernelGGL(weight_grads_split_kernel<true>, dim3(grid), dim3(WG_THREADS), 0, st, a, p.chunk, p.splits, p.tiles_n, p.tiles);
            else hipLaunchKernelGGL(weight_grads_split_kernel<false>, dim3(grid), dim3(WG_THREADS), 0, st, a, p.chunk, p.splits, p.tiles_n, p.tiles);
        } else {
            if (a.at_index) hipLaunchKernelGGL(weight_grads_kernel<true>, dim3(grid), dim3(WG_THREADS), 0, st, a, p.chunk, p.splits, p.tiles_n, p.tiles);
            else hipLaunchKernelGGL(weight_grads_kernel<false>, dim3(grid), dim3(WG_THREADS), 0, st, a, p.chunk, p.splits, p.tiles_n, p.tiles);
        }
        LP_TRY(lp_after_launch());
        const int64_t n0 = (int64_t)a.Mw[0] * a.Nw, n1 = (int64_t)a.Mw[1] * a.Nw, n2 = a.dbias ? a.Nw : 0;
        hipLaunchKernelGGL(weight_grads_fold_kernel, dim3((unsigned)lp_ceil_div((n0 + n1 + n2) / 4, 64)), dim3(kThreads), 0, st, a.partials,
                           p.splits, n0 + n1 + a.Nw, n0, n1, n2, a.C[0], a.C[1], a.dbias);
        return lp_after_launch();
    }
    if (a.dbias) LP_TRY(lp_launch_colsum(a.B, a.dtype, a.Kn, a.Nw, a.dbias, a.colsum_partials, st, a.kn_dev));
    for (int s = 0; s < 2; ++s) {
        if (a.Mw[s] <= 0) continue;
        GemmTnArgs tn;
        tn.dtype = a.dtype;
        tn.Kn = a.Kn; tn.kn_dev = a.kn_dev; tn.at_index = a.at_index;
        tn.Mw = a.Mw[s]; tn.Nw = a.Nw;
        tn.At = a.At[s]; tn.lda = a.lda[s];
        tn.B = a.B; tn.ldb = a.ldb;
        tn.C = a.C[s];
        tn.partials = a.partials;
        LP_TRY(lp_launch_gemm_tn(tn, st));
    }
    return LP_OK;
}

int lp_launch_transpose(const void *in, int32_t rows, int32_t cols, void *out, int dtype, hipStream_t st) {
    if (rows <= 0 || cols <= 0) return LP_OK;
    LpTimedScope timed(LP_KC_OTHER, st);
    const dim3 grid((unsigned)lp_ceil_div(cols, 32), (unsigned)lp_ceil_div(rows, 32));
    if (dtype == LP_BF16)
        hipLaunchKernelGGL((transpose_kernel<lp_bf16_t>), grid, dim3(32, 8), 0, st, static_cast<const lp_bf16_t *>(in), rows, cols,
                           static_cast<lp_bf16_t *>(out));
    else
        hipLaunchKernelGGL((transpose_kernel<float>), grid, dim3(32, 8), 0, st, static_cast<const float *>(in), rows, cols,
                           static_cast<float *>(out));
    return lp_after_launch();
}

int lp_launch_transpose_batch(const TransposeBatch &b, int dtype, hipStream_t st) {
    if (b.n <= 0) return LP_OK;
    if (b.n > 16) return LP_ERR_INVALID_ARG;
    int32_t max_rows = 0, max_cols = 0;
    for (int i = 0; i < b.n; ++i) {
        if (!b.in[i] || !b.out[i] || b.rows[i] <= 0 || b.cols[i] <= 0) return LP_ERR_INVALID_ARG;
        max_rows = std::max(max_rows, b.rows[i]);
        max_cols = std::max(max_cols, b.cols[i]);
    }
    LpTimedScope timed(LP_KC_OTHER, st);
    const dim3 grid((unsigned)lp_ceil_div(max_cols, 32), (unsigned)lp_ceil_div(max_rows, 32), (unsigned)b.n);
    if (dtype == LP_BF16) hipLaunchKernelGGL((transpose_batch_kernel<lp_bf16_t>), grid, dim3(32, 8), 0, st, b);
    else hipLaunchKernelGGL((transpose_batch_kernel<float>), grid, dim3(32, 8), 0, st, b);
    return lp_after_launch();
}

int lp_launch_transpose_weights(const lp_model *m, void *wt, hipStream_t st) {
    TransposeBatch b;
    char *p = static_cast<char *>(wt);
    const size_t eb = (size_t)lp_elem_bytes(m->dtype);
    for (int k = 1; k <= m->n_layers; ++k) {
        const int Fi = m->dims[k - 1], Fo = m->dims[k];
        const size_t wbytes = lp_align_up((size_t)Fi * Fo, 64) * eb;
        const void *src[2] = {m->W_self[k - 1], m->W_neigh[k - 1]};
        for (int s = 0; s < 2; ++s) {
            if (src[s]) {
                b.in[b.n] = src[s]; b.out[b.n] = p + s * wbytes; b.rows[b.n] = Fi; b.cols[b.n] = Fo;
                ++b.n;
            }
        }
        p += 2 * wbytes;
    }
    return lp_launch_transpose_batch(b, m->dtype, st);
}

size_t lp_colsum_partials_bytes(int64_t M, int64_t N) {
    // level sizes shrink by kColsumRows each time; two ping-pong areas of the first level's size are enough
    const int64_t chunks = lp_ceil_div(M > 0 ? M : 1, kColsumRows);
    return 2 * lp_align_up(sizeof(float) * (size_t)chunks * (size_t)(N > 0 ? N : 1));
}

int lp_launch_colsum(const void *in, int dtype, int64_t M, int64_t N, float *out, float *partials, hipStream_t st,
                     const int32_t *m_dev) {
    if (N <= 0) return LP_OK;
    if (N % lp_vec_elems(dtype)) return LP_ERR_UNSUPPORTED;
    if (M <= 0) return lp_launch_zero(out, N, st);
    LpTimedScope timed(LP_KC_OTHER, st);
    const size_t area = lp_align_up(sizeof(float) * (size_t)lp_ceil_div(M, kColsumRows) * (size_t)N) / sizeof(float);
    const void *src = in;
    int src_dtype = dtype;
    int64_t rows = M;
    int level = 0;
    while (true) {
        const int64_t chunks = lp_ceil_div(rows, kColsumRows);
        float *dst = chunks == 1 ? out : partials + (level & 1) * area;
        const int64_t NV = N / lp_vec_elems(src_dtype);
        const dim3 grid((unsigned)lp_ceil_div(NV, 64), (unsigned)chunks);
        if (src_dtype == LP_BF16)
            hipLaunchKernelGGL((colsum_partial_kernel<lp_bf16_t>), grid, dim3(kThreads), 0, st, static_cast<const lp_bf16_t *>(src), rows, NV, dst,
                               level == 0 ? m_dev : nullptr);
        else
            hipLaunchKernelGGL((colsum_partial_kernel<float>), grid, dim3(kThreads), 0, st, static_cast<const float *>(src), rows, NV, dst,
                               level == 0 ? m_dev : nullptr);
        if (chunks == 1) break;
        src = dst;
        src_dtype = LP_F32;  // the partial sums are fp32
        rows = chunks;
        ++level;
    }
    return lp_after_launch();
}

int lp_launch_zero(float *p, int64_t n, hipStream_t st) {
    if (n <= 0) return LP_OK;
    LpTimedScope timed(LP_KC_OTHER, st);
    const int head = (int)((16 - (reinterpret_cast<uintptr_t>(p) & 15u)) & 15u) / 4;  // floats before 16-byte alignment
    const int64_t h = head < n ? head : n;
    const int64_t n4 = (n - h) / 4;
    const int n_tail = (int)(n - h - 4 * n4);
    if (h) hipLaunchKernelGGL(zero_kernel, dim3(1), dim3(64), 0, st, nullptr, 0, p, (int)h);
    if (n4 || n_tail)
        hipLaunchKernelGGL(zero_kernel, dim3((unsigned)lp_ceil_div(n4 > 0 ? n4 : 1, 256)), dim3(256), 0, st,
                           reinterpret_cast<float4 *>(p + h), n4, p + h + 4 * n4, n_tail);
    return lp_after_launch();
}
