// Host-side checks of the C ABI under AddressSanitizer and UndefinedBehaviorSanitizer, with every kernel launch
// stubbed out.  Built and run by tests/test_abi_sanitized.py (no GPU needed, and none is touched when there is one):
// this file defines the HIP runtime entry points the library's host code uses, so the library's calls land here
// instead of in the runtime.  A "launch" only counts itself; armed, it reports hipErrorLaunchFailure the way the runtime
// would, which every entry point must turn into LP_ERR_HIP.  Device pointers are fake non-null addresses: host code
// must never read through them, and the sanitizers would catch it if it did.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstring>

#include "lp.h"

static int g_launches = 0;
static bool g_fail_launch = false;
static bool g_fail_symbol = false;
static hipError_t g_last = hipSuccess;
static dim3 g_grid, g_block;
static size_t g_shm;
static hipStream_t g_stream;

extern "C" hipError_t __hipPushCallConfiguration(dim3 grid, dim3 block, size_t shm, hipStream_t st) {
    g_grid = grid; g_block = block; g_shm = shm; g_stream = st;
    return hipSuccess;
}
extern "C" hipError_t __hipPopCallConfiguration(dim3 *grid, dim3 *block, size_t *shm, hipStream_t *st) {
    *grid = g_grid; *block = g_block; *shm = g_shm; *st = g_stream;
    return hipSuccess;
}
extern "C" hipError_t hipLaunchKernel(const void *, dim3 grid, dim3 block, void **, size_t, hipStream_t) {
    ++g_launches;
    if (grid.x == 0 || grid.y == 0 || grid.z == 0 || block.x == 0 || block.x * block.y * block.z > 1024) {
        std::printf("launch %d with an invalid configuration: grid (%u, %u, %u), block (%u, %u, %u)\n", g_launches, grid.x, grid.y,
                    grid.z, block.x, block.y, block.z);
        g_last = hipErrorInvalidConfiguration;
    }
    if (g_fail_launch) g_last = hipErrorLaunchFailure;
    return g_last;
}
extern "C" hipError_t hipGetLastError(void) {
    const hipError_t e = g_last;
    g_last = hipSuccess;
    return e;
}
static int g_copies = 0;
extern "C" hipError_t hipMemcpyAsync(void *, const void *, size_t, hipMemcpyKind kind, hipStream_t) {
    ++g_copies;   // only device-to-device copies are reached here (fake pointers: nothing is moved)
    return kind == hipMemcpyDeviceToDevice && !g_fail_launch ? hipSuccess : hipErrorInvalidValue;
}
extern "C" hipError_t hipGetDevice(int *dev) { *dev = 0; return hipSuccess; }
extern "C" hipError_t hipDeviceGetAttribute(int *value, hipDeviceAttribute_t, int) { *value = 256; return hipSuccess; }
extern "C" hipError_t hipGetSymbolAddress(void **p, const void *) {
    if (g_fail_symbol) return hipErrorInvalidSymbol;
    *p = reinterpret_cast<void *>(0x7000);
    return hipSuccess;
}

static int g_failed = 0;
#define CHECK(cond)                                                          \
    do {                                                                     \
        if (!(cond)) {                                                       \
            std::printf("FAILED line %d: %s\n", __LINE__, #cond);            \
            ++g_failed;                                                      \
        }                                                                    \
    } while (0)

template <typename T> static T *fake(uintptr_t a = 0x1000) { return reinterpret_cast<T *>(a); }

static lp_model model_of(std::initializer_list<int> dims, int dtype = LP_F32, int products = LP_FP32_PRODUCTS_NATIVE) {
    lp_model m;
    std::memset(&m, 0, sizeof m);
    m.n_layers = (int)dims.size() - 1;
    m.dtype = dtype;
    m.fp32_products = products;
    int i = 0;
    for (int d : dims) m.dims[i++] = d;
    for (int k = 0; k < m.n_layers; ++k) {
        m.W_self[k] = fake<void>();
        m.W_neigh[k] = fake<void>();
        m.bias[k] = fake<void>();
    }
    return m;
}

int main(int argc, char **argv) {
    if (argc > 1 && std::strcmp(argv[1], "no-symbol") == 0) {
        // a runtime that cannot give the scratch array's address (the address is cached per device after the first
        // success, hence a process of its own): LP_ERR_HIP, nothing launched
        g_fail_symbol = true;
        float *q = reinterpret_cast<float *>(0x1000);
        const int32_t *e = reinterpret_cast<const int32_t *>(0x1000);
        const int r = lp_score_loss_noalloc(q, 5000, 256, LP_F32, 1000, 400, e, e, q, q, q, nullptr, nullptr);
        std::printf("no-symbol: status %d, %d launches\n", r, g_launches);
        return (r == LP_ERR_HIP && g_launches == 0) ? 0 : 1;
    }
    lp_csr g;
    std::memset(&g, 0, sizeof g);
    g.n_nodes = 5000;
    g.nnz = 40000;
    g.rowptr = g.colidx = g.t_rowptr = g.t_colidx = fake<const int32_t>();
    g.inv_deg = fake<const float>();
    const int32_t *ip = fake<const int32_t>();
    int32_t *op = fake<int32_t>();
    float *fp = fake<float>();

    // ---- status texts
    for (int c = 0; c >= -5; --c) CHECK(lp_strerror(c) != nullptr && std::strlen(lp_strerror(c)) > 0);

    // ---- lp_sample_neg: validation, one launch, and a failing launch
    CHECK(lp_sample_neg(nullptr, 4, ip, 1, 10, 1, 1, op, nullptr, nullptr, nullptr) == LP_ERR_INVALID_ARG);
    CHECK(lp_sample_neg(&g, -1, ip, 1, 10, 1, 1, op, nullptr, nullptr, nullptr) == LP_ERR_INVALID_ARG);
    CHECK(lp_sample_neg(&g, (int64_t)1 << 30, ip, 4, 10, 1, 1, op, nullptr, nullptr, nullptr) == LP_ERR_OUT_OF_RANGE);
    CHECK(g_launches == 0);
    CHECK(lp_sample_neg(&g, 1000, ip, 3, 5000, 1, 1, op, op, op, nullptr) == LP_OK && g_launches == 1);
    g_fail_launch = true;
    CHECK(lp_sample_neg(&g, 1000, ip, 3, 5000, 1, 1, op, op, op, nullptr) == LP_ERR_HIP);
    g_fail_launch = false;

    // ---- lp_score_loss and the variant without a workspace
    const size_t sws = lp_score_loss_workspace_bytes(1000);
    CHECK(sws > 0);
    CHECK(lp_score_loss(fp, 5000, 256, LP_F32, 1000, 400, ip, ip, fp, fp, fp, op, fp, sws, nullptr) == LP_OK);
    CHECK(lp_score_loss(fp, 5000, 256, LP_F32, 1000, 400, ip, ip, fp, fp, fp, op, fp, sws - 1, nullptr) == LP_ERR_WORKSPACE);
    CHECK(lp_score_loss(fp, 5000, 254, LP_F32, 1000, 400, ip, ip, fp, fp, fp, op, fp, sws, nullptr) == LP_ERR_UNSUPPORTED);
    CHECK(lp_score_loss(fp, 5000, 256, LP_F32, 1000, 1001, ip, ip, fp, fp, fp, op, fp, sws, nullptr) == LP_ERR_INVALID_ARG);
    int before = g_launches;
    CHECK(lp_score_loss_noalloc(fp, 5000, 256, LP_BF16, 1000, 400, ip, ip, fp, fp, nullptr, nullptr, nullptr) == LP_OK);
    CHECK(g_launches == before + 2);
    CHECK(lp_score_loss_noalloc(fp, 5000, 256, LP_F32, LP_SCORE_LOSS_NOALLOC_MAX_EDGES + 1, 0, ip, ip, fp, fp, fp, op, nullptr) == LP_ERR_OUT_OF_RANGE);
    g_fail_launch = true;
    CHECK(lp_score_loss_noalloc(fp, 5000, 256, LP_F32, 1000, 400, ip, ip, fp, fp, fp, op, nullptr) == LP_ERR_HIP);
    CHECK(lp_score_loss(fp, 5000, 256, LP_F32, 1000, 400, ip, ip, fp, fp, fp, op, fp, sws, nullptr) == LP_ERR_HIP);
    g_fail_launch = false;

    // ---- lp_sage_forward / lp_backward: the whole host-side orchestration of a three-layer model, both storage
    // types and both ways of forming fp32 products, with nothing launched for real
    for (int variant = 0; variant < 3; ++variant) {
        lp_model m = variant == 2 ? model_of({128, 512, 512, 512}, LP_BF16)
                                  : model_of({128, 256, 256, 256}, LP_F32, variant ? LP_FP32_PRODUCTS_BF16X6 : LP_FP32_PRODUCTS_NATIVE);
        lp_acts acts;
        lp_grads grads;
        std::memset(&acts, 0, sizeof acts);
        std::memset(&grads, 0, sizeof grads);
        for (int k = 0; k < 3; ++k) {
            acts.A[k] = acts.H[k] = fake<void>();
            grads.dW_self[k] = grads.dW_neigh[k] = grads.dbias[k] = fp;
        }
        const size_t fws = lp_sage_forward_workspace_bytes(&m, g.n_nodes), bws = lp_backward_workspace_bytes(&m, g.n_nodes, 2000);
        CHECK(fws > 0 && bws > 0);
        before = g_launches;
        CHECK(lp_sage_forward(&g, &m, fp, &acts, fake<void>(0x100000), fws, nullptr) == LP_OK);
        CHECK(g_launches >= before + 6);   // three aggregations and three products at least
        CHECK(lp_sage_forward(&g, &m, fp, &acts, fake<void>(0x100000), fws - 1, nullptr) == LP_ERR_WORKSPACE);
        // the training forward: a batch small enough to list the rows of the last layer (more launches than the full
        // pass: flags, prefix sums, row copies), one too large for that, and an empty one
        {
            const int64_t few = g.n_nodes / 4 - 1, many = g.n_nodes;
            const size_t ews = lp_sage_forward_edges_workspace_bytes(&m, g.n_nodes, few);
            const size_t mws = lp_sage_forward_edges_workspace_bytes(&m, g.n_nodes, many);
            CHECK(ews > fws && mws == fws);
            long b0 = g_launches;
            CHECK(lp_sage_forward(&g, &m, fp, &acts, fake<void>(0x100000), fws, nullptr) == LP_OK);
            const long full_launches = g_launches - b0;
            b0 = g_launches;
            CHECK(lp_sage_forward_edges(&g, &m, fp, few, ip, ip, &acts, fake<void>(0x100000), ews, nullptr) == LP_OK);
            CHECK(g_launches - b0 > full_launches);
            b0 = g_launches;
            CHECK(lp_sage_forward_edges(&g, &m, fp, many, ip, ip, &acts, fake<void>(0x100000), mws, nullptr) == LP_OK);
            CHECK(g_launches - b0 == full_launches);
            b0 = g_launches;
            CHECK(lp_sage_forward_edges(&g, &m, fp, 0, nullptr, nullptr, &acts, fake<void>(0x100000),
                                        lp_sage_forward_edges_workspace_bytes(&m, g.n_nodes, 0), nullptr) == LP_OK);
            CHECK(g_launches - b0 < full_launches);   // the last layer is left out
            CHECK(lp_sage_forward_edges(&g, &m, fp, few, ip, ip, &acts, fake<void>(0x100000), ews - 1, nullptr) == LP_ERR_WORKSPACE);
            CHECK(lp_sage_forward_edges(&g, &m, fp, few, nullptr, ip, &acts, fake<void>(0x100000), ews, nullptr) == LP_ERR_INVALID_ARG);
            g_fail_launch = true;
            CHECK(lp_sage_forward_edges(&g, &m, fp, few, ip, ip, &acts, fake<void>(0x100000), ews, nullptr) == LP_ERR_HIP);
            g_fail_launch = false;
        }
        CHECK(lp_backward(&g, &m, fp, &acts, 2000, ip, ip, fp, &grads, fake<void>(0x100000), bws, nullptr) == LP_OK);
        grads.dX = fake<void>();
        CHECK(lp_backward(&g, &m, fp, &acts, 2000, ip, ip, fp, &grads, fake<void>(0x100000), bws, nullptr) == LP_OK);
        CHECK(lp_backward(&g, &m, fp, &acts, 2000, ip, ip, fp, &grads, fake<void>(0x100000), bws / 2, nullptr) == LP_ERR_WORKSPACE);
        g_fail_launch = true;
        CHECK(lp_sage_forward(&g, &m, fp, &acts, fake<void>(0x100000), fws, nullptr) == LP_ERR_HIP);
        CHECK(lp_backward(&g, &m, fp, &acts, 2000, ip, ip, fp, &grads, fake<void>(0x100000), bws, nullptr) == LP_ERR_HIP);
        g_fail_launch = false;
        lp_model bad = m;
        bad.fp32_products = 2;
        CHECK(lp_sage_forward(&g, &bad, fp, &acts, fake<void>(0x100000), fws, nullptr) == LP_ERR_INVALID_ARG);
        bad = m;
        bad.dims[1] = 250;
        CHECK(lp_sage_forward(&g, &bad, fp, &acts, fake<void>(0x100000), fws, nullptr) == LP_ERR_UNSUPPORTED);
        // weight update in one launch
        lp_opt_state st;
        std::memset(&st, 0, sizeof st);
        for (int k = 0; k < 3; ++k) st.m_W_self[k] = st.m_W_neigh[k] = st.m_bias[k] = st.v_W_self[k] = st.v_W_neigh[k] = st.v_bias[k] = fp;
        CHECK(lp_sgd_step(&m, &grads, 1e-3f, nullptr) == LP_OK);
        CHECK(lp_adam_step(&m, &grads, &st, 1, 1e-3f, 0.9f, 0.999f, 1e-8f, nullptr) == LP_OK);
        CHECK(lp_adam_step(&m, &grads, &st, 0, 1e-3f, 0.9f, 0.999f, 1e-8f, nullptr) == LP_ERR_INVALID_ARG);
    }

    // ---- MLP edge predictor
    {
        lp_mlp p;
        std::memset(&p, 0, sizeof p);
        p.n_layers = 3;
        p.dtype = LP_F32;
        p.fp32_products = LP_FP32_PRODUCTS_BF16X6;
        p.dims[0] = p.dims[1] = p.dims[2] = 256;
        p.dims[3] = 1;
        lp_mlp_acts ma;
        lp_mlp_grads mg;
        std::memset(&ma, 0, sizeof ma);
        std::memset(&mg, 0, sizeof mg);
        ma.X = fake<void>();
        for (int j = 0; j < 3; ++j) {
            p.W[j] = fake<void>();
            p.bias[j] = fp;
            ma.U[j] = fake<void>();
            mg.dW[j] = mg.dbias[j] = fp;
        }
        const size_t w1 = lp_mlp_score_loss_workspace_bytes(&p, 3000), w2 = lp_mlp_backward_workspace_bytes(&p, 3000);
        CHECK(w1 > 0 && w2 > 0);
        CHECK(lp_mlp_score_loss(fp, 5000, 3000, 1000, ip, ip, &p, &ma, fp, fp, fp, fake<void>(0x100000), w1, nullptr) == LP_OK);
        CHECK(lp_mlp_backward(&p, &ma, 3000, fp, &mg, fake<void>(), fake<void>(0x100000), w2, nullptr) == LP_OK);
        p.fp32_products = -3;
        CHECK(lp_mlp_score_loss(fp, 5000, 3000, 1000, ip, ip, &p, &ma, fp, fp, fp, fake<void>(0x100000), w1, nullptr) == LP_ERR_INVALID_ARG);
    }

    // ---- calls that read a result back on the host are only checked up to their argument validation
    int64_t nnz = 0;
    CHECK(lp_build_csr(0, 4, ip, ip, 0, op, op, op, op, fp, op, op, fp, &nnz, fake<void>(), 1 << 20, nullptr) == LP_ERR_INVALID_ARG);
    CHECK(lp_build_csr(100, 4, ip, ip, 0, op, op, op, op, fp, op, op, fp, &nnz, fake<void>(), 8, nullptr) == LP_ERR_WORKSPACE);
    CHECK(lp_hits_at_k(fp, 10, fp, 100, 0, fake<int64_t>(), nullptr, fake<void>(), 1 << 20, nullptr) == LP_ERR_INVALID_ARG);

    std::printf("%d launches stubbed, %d checks failed\n", g_launches, g_failed);
    return g_failed == 0 ? 0 : 1;
}
