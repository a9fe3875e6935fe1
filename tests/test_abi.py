"""Host-only checks of the C ABI: the library loads, exports every function the header declares, and rejects
bad arguments on the host before anything is launched (so these run without a GPU)."""
import ctypes as C
import os
import re

import pytest

import paper_2506_20818_amd.binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "lp.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(lp_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_function():
    lib = B.load_library()
    names = declared_functions()
    assert set(names) == set(B.EXPORTS), (names, sorted(B.EXPORTS))
    for n in names:
        assert getattr(lib, n) is not None


def test_library_and_header_agree_on_the_abi_version():
    text = open(os.path.join(ROOT, "include", "lp.h")).read()
    assert int(re.search(r"#define\s+LP_ABI_VERSION\s+(\d+)", text).group(1)) == B.load_library().lp_abi_version()


def test_strerror_covers_all_codes():
    texts = {B.lp_strerror(c) for c in (0, -1, -2, -3, -4, -5)}
    assert len(texts) == 6 and B.lp_strerror(-99) == "unknown status"


def _model(dims, dtype=0, null_w=False, products=0):
    m = B._ModelStruct()
    m.n_layers, m.dtype, m.fp32_products = len(dims) - 1, dtype, products
    for i, d in enumerate(dims):
        m.dims[i] = d
    for k in range(len(dims) - 1):
        m.W_self[k] = None if null_w else 0x1000
        m.W_neigh[k] = 0x1000
        m.bias[k] = 0x1000
    return m


def _csr(n=10, nnz=5):
    g = B._CsrStruct()
    g.n_nodes, g.nnz = n, nnz
    for f in ("rowptr", "colidx", "t_rowptr", "t_colidx", "inv_deg"):
        setattr(g, f, 0x1000)
    return g


def test_workspace_queries_are_host_arithmetic():
    lib = B.load_library()
    a = lib.lp_build_csr_workspace_bytes(1000, 5000, 1)
    b = lib.lp_build_csr_workspace_bytes(1000, 50000, 1)
    assert 0 < a < b
    assert lib.lp_build_csr_workspace_bytes(0, 5, 0) == 0
    m = _model([128, 256, 256, 256])
    f1 = lib.lp_sage_forward_workspace_bytes(C.byref(m), 1000)
    assert f1 >= 4 * 2 * (128 * 256 + 2 * 256 * 256)
    b1 = lib.lp_backward_workspace_bytes(C.byref(m), 1000, 100)
    b2 = lib.lp_backward_workspace_bytes(C.byref(m), 2000, 100)
    b3 = lib.lp_backward_workspace_bytes(C.byref(m), 2000, 100000)
    assert 3 * 1000 * 256 * 4 <= b1 < b2 < b3
    assert lib.lp_backward_workspace_bytes(C.byref(_model([128, 255])), 1000, 10) == 0
    assert lib.lp_score_loss_workspace_bytes(10) > 0


def test_build_csr_rejects_bad_arguments_on_the_host():
    lib = B.load_library()
    nnz = C.c_int64(0)
    p = C.c_void_p(0x1000)
    args = lambda **kw: [kw.get("n", 10), kw.get("n_in", 4), kw.get("rows", p), p, kw.get("flags", 0), p, p, p, p, p,
                         None, None, None, C.byref(nnz), kw.get("ws", p), kw.get("ws_bytes", 1 << 30), None]
    assert lib.lp_build_csr(*args(n=0)) == -1
    assert lib.lp_build_csr(*args(n_in=-1)) == -1
    assert lib.lp_build_csr(*args(rows=None)) == -1
    assert lib.lp_build_csr(*args(flags=8)) == -1
    assert lib.lp_build_csr(*args(n_in=1 << 31)) == -2
    assert lib.lp_build_csr(*args(ws=None)) == -3
    assert lib.lp_build_csr(*args(ws_bytes=16)) == -3


def test_forward_backward_reject_bad_arguments_on_the_host():
    lib = B.load_library()
    g, acts, grads = _csr(), B._ActsStruct(), B._GradsStruct()
    for k in range(3):
        acts.A[k] = acts.H[k] = 0x1000
        grads.dW_self[k] = grads.dW_neigh[k] = grads.dbias[k] = 0x1000
    p = C.c_void_p(0x1000)
    good = _model([128, 256, 256, 256])
    fwd = lambda m=good, graph=g, x=p, ws=p, wsb=1 << 40: lib.lp_sage_forward(
        C.byref(graph), C.byref(m), x, C.byref(acts), ws, wsb, None)
    assert fwd(m=_model([128, 256], dtype=7)) == -4
    assert fwd(m=_model([128, 254])) == -4            # width not a multiple of 4
    assert fwd(m=_model([128, 2048])) == -4
    assert fwd(m=_model([128, 256], null_w=True)) == -1
    # the way of forming fp32 products is a field of the model, checked on every call
    assert fwd(m=_model([128, 256], products=2)) == -1 and fwd(m=_model([128, 256], products=-1)) == -1
    assert fwd(m=_model([128, 256], dtype=1, products=7)) == -1          # checked for bf16 models too
    nonzero_reserved = _model([128, 256])
    nonzero_reserved.reserved_ = 1
    assert fwd(m=nonzero_reserved) == -1
    assert lib.lp_sage_forward_workspace_bytes(C.byref(_model([128, 256], products=3)), 1000) == 0
    assert fwd(x=None) == -1
    assert fwd(x=C.c_void_p(0x1004)) == -1            # misaligned features
    assert fwd(ws=None) == -3
    assert fwd(wsb=8) == -3
    bad_g = _csr()
    bad_g.rowptr = None
    assert fwd(graph=bad_g) == -1
    big = _csr(nnz=1 << 31)
    assert fwd(graph=big) == -2
    zero_layers = _model([128])
    assert fwd(m=zero_layers) == -1
    # the training forward: the same checks (shared code), plus those on the batch
    fwe = lambda B_=4, es=p, ed=p, m=good, ws=p, wsb=1 << 40: lib.lp_sage_forward_edges(
        C.byref(g), C.byref(m), p, B_, es, ed, C.byref(acts), ws, wsb, None)
    assert fwe(B_=-1) == -1
    assert fwe(es=None) == -1 and fwe(ed=None) == -1
    assert fwe(B_=1 << 31) == -2
    assert fwe(ws=None) == -3 and fwe(wsb=8) == -3
    assert fwe(m=_model([128, 256], products=2)) == -1
    n_graph = g.n_nodes
    few, many = n_graph // 4 - 1, n_graph
    w0 = lib.lp_sage_forward_workspace_bytes(C.byref(good), n_graph)
    w_few = lib.lp_sage_forward_edges_workspace_bytes(C.byref(good), n_graph, few)
    assert w_few > w0 > 0                                   # the list, its flags and three matrices of listed rows
    assert lib.lp_sage_forward_edges_workspace_bytes(C.byref(good), n_graph, -1) == 0
    assert lib.lp_sage_forward_edges_workspace_bytes(C.byref(good), n_graph, 1 << 31) == 0
    assert lib.lp_sage_forward_edges_workspace_bytes(C.byref(good), n_graph, many) == w0     # too many to list: the plain pass
    assert fwe(B_=few, wsb=w_few - 1) == -3
    bwd = lambda B_=4, es=p, ws=p, wsb=1 << 40, gr=grads: lib.lp_backward(
        C.byref(g), C.byref(good), p, C.byref(acts), B_, es, p, p, C.byref(gr), ws, wsb, None)
    assert bwd(B_=-1) == -1
    assert bwd(es=None) == -1
    assert bwd(ws=None) == -3
    assert bwd(wsb=100) == -3
    assert bwd(B_=1 << 31) == -2
    assert bwd(gr=B._GradsStruct()) == -1


def test_sampler_and_loss_reject_bad_arguments_on_the_host():
    lib = B.load_library()
    g = _csr()
    p = C.c_void_p(0x1000)
    s = lambda n_pos=4, k=1, space=10, src=p: lib.lp_sample_neg(C.byref(g), n_pos, src, k, space, 1, 2, p, None, None, None)
    assert s(n_pos=-1) == -1
    assert s(space=0) == -1
    assert s(src=None) == -1
    assert s(n_pos=1 << 30, k=4) == -2
    assert s(n_pos=0) == 0                             # nothing to do: no launch, no error
    sl = lambda F=64, dt=0, B_=4, npos=2, H=p, ws=p, wsb=1 << 20, loss=p: lib.lp_score_loss(
        H, 10, F, dt, B_, npos, p, p, p, loss, p, None, ws, wsb, None)
    assert sl(F=6) == -4
    assert sl(dt=3) == -4
    assert sl(npos=5) == -1
    assert sl(H=None) == -1
    assert sl(loss=None) == -1
    assert sl(ws=None) == -3
    assert sl(B_=1 << 31, npos=0) == -2


def test_sparsify_rejects_bad_arguments_on_the_host():
    lib = B.load_library()
    n_kept = C.c_int64(-1)
    p = C.c_void_p(0x1000)
    sp = lambda n=10, m=4, L=3, eu=p, kept=p, out=C.byref(n_kept), ws=p, wsb=1 << 30: lib.lp_sparsify(
        n, m, eu, p, L, 7, kept, None, None, None, p, out, ws, wsb, None)
    assert sp(n=0) == -1
    assert sp(m=-1) == -1
    assert sp(L=-1) == -1
    assert sp(out=None) == -1
    assert sp(m=1 << 31) == -2
    assert sp(eu=None) == -1
    assert sp(kept=None) == -1
    assert sp(ws=None) == -3
    assert sp(wsb=64) == -3
    assert sp(m=0) == 0 and n_kept.value == 0          # nothing to draw from: no launch, no error
    n_kept.value = -1
    assert sp(L=0) == 0 and n_kept.value == 0
    a, b = lib.lp_sparsify_workspace_bytes(1000, 5000), lib.lp_sparsify_workspace_bytes(1000, 50000)
    assert 0 < a < b and lib.lp_sparsify_workspace_bytes(0, 5) == 0


def test_optimizer_steps_reject_bad_arguments_on_the_host():
    lib = B.load_library()
    good = _model([128, 256, 256])
    grads, state = B._GradsStruct(), B._OptStateStruct()
    for k in range(2):
        grads.dW_self[k] = grads.dW_neigh[k] = grads.dbias[k] = 0x1000
        for name in ("m_W_self", "m_W_neigh", "m_bias", "v_W_self", "v_W_neigh", "v_bias"):
            getattr(state, name)[k] = 0x1000
    sgd = lambda m=good, g=grads, lr=0.1: lib.lp_sgd_step(C.byref(m), C.byref(g), lr, None)
    assert sgd(m=_model([128, 256], null_w=True)) == -1
    assert sgd(g=B._GradsStruct()) == -1
    assert sgd(lr=float("nan")) == -1
    assert sgd(m=_model([128, 256], dtype=5)) == -4
    adam = lambda m=good, g=grads, s=state, t=1, lr=1e-3, b1=0.9, b2=0.999, eps=1e-8: lib.lp_adam_step(
        C.byref(m), C.byref(g), C.byref(s), t, lr, b1, b2, eps, None)
    assert adam(t=0) == -1
    assert adam(b1=1.0) == -1
    assert adam(b2=-0.1) == -1
    assert adam(eps=-1.0) == -1
    assert adam(s=B._OptStateStruct()) == -1
    assert adam(g=B._GradsStruct()) == -1


def _blocks(K=3, n_graph=1000, n_edges=64, fan=(25, 10, 5), nnz=5000):
    lib = B.load_library()
    b = B._BlocksStruct()
    b.n_layers, b.n_graph_nodes, b.n_edges = K, n_graph, n_edges
    cap = (C.c_int32 * (K + 1))()
    cap_e = (C.c_int64 * K)()
    fan_c = (C.c_int32 * K)(*fan)
    assert lib.lp_blocks_bounds(n_graph, nnz, n_edges, K, fan_c, cap, cap_e) == 0
    for k in range(K + 1):
        b.cap[k] = cap[k]
    for k in range(K):
        b.cap_entries[k] = cap_e[k]
        b.ptr[k] = b.col[k] = b.inv_cnt[k] = b.t_ptr[k] = b.t_col[k] = 0x1000
    b.n = b.nodes = b.index = b.e_src_pos = b.e_dst_pos = b.node_inv_deg = 0x1000
    return b, fan_c


def test_blocks_bounds_and_argument_checks_on_the_host():
    lib = B.load_library()
    cap = (C.c_int32 * 4)()
    cap_e = (C.c_int64 * 3)()
    fan = (C.c_int32 * 3)(25, 10, 5)
    assert lib.lp_blocks_bounds(1000, 5000, 8, 3, fan, cap, cap_e) == 0
    assert list(cap) == [1000, 1000, 416, 16] and list(cap_e) == [5000, 4160, 400]      # min(N, c(1+f)), min(nnz, c f)
    assert lib.lp_blocks_bounds(1000, 5000, 8, 0, fan, cap, cap_e) == -1
    assert lib.lp_blocks_bounds(0, 5000, 8, 3, fan, cap, cap_e) == -1
    assert lib.lp_blocks_bounds(1000, 5000, 8, 3, (C.c_int32 * 3)(25, -1, 5), cap, cap_e) == -4
    assert lib.lp_blocks_bounds(1000, 5000, 8, 3, (C.c_int32 * 3)(0, 10, 5), cap, cap_e) == 0          # 0: all neighbours
    assert list(cap) == [1000, 1000, 1000, 16] and list(cap_e) == [5000, 5000, 5000]
    assert lib.lp_blocks_bounds(1000, 5000, 8, 3, (C.c_int32 * 3)(25, 65, 5), cap, cap_e) == -4
    assert lib.lp_blocks_bounds(1000, 5000, 1 << 30, 3, fan, cap, cap_e) == -2
    assert lib.lp_sample_blocks_workspace_bytes(1000, 5000, 8, 3, fan) > 0
    g = _csr(n=1000, nnz=5000)
    b, fan_c = _blocks()
    p = C.c_void_p(0x1000)
    sb = lambda graph=g, B_=64, es=p, blk=b, ws=p, wsb=1 << 40, K=3: lib.lp_sample_blocks(
        C.byref(graph), B_, es, p, K, fan_c, 1, 2, C.byref(blk), ws, wsb, None)
    assert sb(es=None) == -1
    assert sb(B_=32) == -1                                 # the blocks were sized for another batch
    assert sb(K=2) == -1
    assert sb(ws=None) == -3
    assert sb(wsb=64) == -3
    small, _ = _blocks()
    small.cap[0] = 10                                      # below the bound (and below cap[1])
    assert sb(blk=small) == -1
    no_ptr, _ = _blocks()
    no_ptr.ptr[1] = None
    assert sb(blk=no_ptr) == -1
    m = _model([128, 256, 256, 256])
    acts, grads = B._ActsStruct(), B._GradsStruct()
    for k in range(3):
        acts.A[k] = acts.H[k] = 0x1000
        grads.dW_self[k] = grads.dW_neigh[k] = grads.dbias[k] = 0x1000
    fwd = lambda model=m, blk=b, x=p, xf=p, ws=p, wsb=1 << 40: lib.lp_sage_forward_blocks(
        C.byref(blk), C.byref(model), x, xf, C.byref(acts), ws, wsb, None)
    assert fwd(model=_model([128, 256, 256])) == -1        # layer count differs from the blocks'
    assert fwd(model=_model([128, 256, 256, 250])) == -4
    assert fwd(x=None) == -1
    assert fwd(xf=C.c_void_p(0x1004)) == -1
    assert fwd(ws=None) == -3
    bwd = lambda blk=b, ds=p, gr=grads, ws=p, wsb=1 << 40: lib.lp_backward_blocks(
        C.byref(blk), C.byref(m), p, C.byref(acts), ds, C.byref(gr), ws, wsb, None)
    assert bwd(ds=None) == -1
    assert bwd(gr=B._GradsStruct()) == -1
    assert bwd(ws=None) == -3
    assert bwd(wsb=128) == -3
    assert lib.lp_backward_blocks_workspace_bytes(C.byref(m), C.byref(b)) > 0
    bwd_eg = lambda eg=p, gr=grads, ws=p, wsb=1 << 40: lib.lp_backward_blocks_edge_grads(
        C.byref(b), C.byref(m), p, C.byref(acts), eg, C.byref(gr), ws, wsb, None)
    assert bwd_eg(eg=None) == -1
    assert bwd_eg(eg=C.c_void_p(0x1004)) == -1            # not 16-byte aligned
    assert bwd_eg(gr=B._GradsStruct()) == -1
    assert bwd_eg(ws=None) == -3
    assert lib.lp_forward_blocks_workspace_bytes(C.byref(_model([128, 256])), C.byref(b)) == 0


def test_mlp_predictor_and_tensor_updates_reject_bad_arguments_on_the_host():
    lib = B.load_library()
    p = C.c_void_p(0x1000)

    def mlp(dims=(256, 256, 256, 1), dtype=0, null_w=False):
        s = B._MlpStruct()
        s.n_layers, s.dtype = len(dims) - 1, dtype
        for j, d in enumerate(dims):
            s.dims[j] = d
        for j in range(len(dims) - 1):
            s.W[j] = None if null_w else 0x1000
            s.bias[j] = 0x1000
        return s

    acts, grads = B._MlpActsStruct(), B._MlpGradsStruct()
    acts.X = 0x1000
    for j in range(3):
        acts.U[j] = 0x1000
        grads.dW[j] = grads.dbias[j] = 0x1000
    sl = lambda m=mlp(), H=p, B_=4, npos=2, ws=p, wsb=1 << 30, loss=p: lib.lp_mlp_score_loss(
        H, 10, B_, npos, p, p, C.byref(m), C.byref(acts), p, loss, p, ws, wsb, None)
    assert sl(m=mlp(dims=(256, 256, 2))) == -1           # the last layer must have one output
    assert sl(m=mlp(dims=(256, 250, 1))) == -4
    assert sl(m=mlp(dtype=9)) == -4
    assert sl(m=mlp(null_w=True)) == -1
    assert sl(H=None) == -1
    assert sl(npos=5) == -1
    assert sl(loss=None) == -1
    assert sl(ws=None) == -3
    assert sl(wsb=16) == -3
    bw = lambda m=mlp(), B_=4, ds=p, gr=grads, eg=p, ws=p, wsb=1 << 30: lib.lp_mlp_backward(
        C.byref(m), C.byref(acts), B_, ds, C.byref(gr), eg, ws, wsb, None)
    assert bw(ds=None) == -1
    assert bw(eg=None) == -1
    assert bw(gr=B._MlpGradsStruct()) == -1
    assert bw(ws=None) == -3
    assert bw(B_=-1) == -1
    assert lib.lp_mlp_backward_workspace_bytes(C.byref(mlp()), 1000) > lib.lp_mlp_backward_workspace_bytes(C.byref(mlp()), 10) > 0
    assert lib.lp_adam_update_tensor(None, 0, p, p, p, 10, 1, 1e-3, 0.9, 0.999, 1e-8, None) == -1
    assert lib.lp_adam_update_tensor(p, 0, p, p, p, 10, 0, 1e-3, 0.9, 0.999, 1e-8, None) == -1
    assert lib.lp_adam_update_tensor(p, 3, p, p, p, 10, 1, 1e-3, 0.9, 0.999, 1e-8, None) == -4
    assert lib.lp_adam_update_tensor(p, 0, p, p, p, 0, 1, 1e-3, 0.9, 0.999, 1e-8, None) == 0
    assert lib.lp_sgd_update_tensor(p, 0, None, 10, 0.1, None) == -1
    assert lib.lp_sgd_update_tensor(p, 0, p, 0, 0.1, None) == 0
    # lp_backward_edge_grads shares lp_backward's checks
    g, acts3, gr3 = _csr(), B._ActsStruct(), B._GradsStruct()
    for k in range(3):
        acts3.A[k] = acts3.H[k] = 0x1000
        gr3.dW_self[k] = gr3.dW_neigh[k] = gr3.dbias[k] = 0x1000
    good = _model([128, 256, 256, 256])
    eg = lambda B_=4, e=p, ws=p, wsb=1 << 40: lib.lp_backward_edge_grads(
        C.byref(g), C.byref(good), p, C.byref(acts3), B_, p, p, e, C.byref(gr3), ws, wsb, None)
    assert eg(e=None) == -1
    assert eg(e=C.c_void_p(0x1004)) == -1
    assert eg(ws=None) == -3


def test_hits_at_k_rejects_bad_arguments_on_the_host():
    lib = B.load_library()
    p = C.c_void_p(0x1000)
    call = lambda pos=p, n_pos=10, neg=p, n_neg=20, K=5, hits=p, ws=p, wsb=1 << 30: lib.lp_hits_at_k(
        pos, n_pos, neg, n_neg, K, hits, None, ws, wsb, None)
    assert call(K=0) == -1
    assert call(n_pos=-1) == -1
    assert call(pos=None) == -1
    assert call(neg=None) == -1
    assert call(hits=None) == -1
    assert call(n_neg=1 << 31) == -2
    assert call(ws=None) == -3
    assert call(wsb=64) == -3
    assert lib.lp_hits_at_k_workspace_bytes(1000) > 16000
    assert lib.lp_hits_at_k_workspace_bytes(-1) == 0


def test_model_struct_layout_matches_the_header():
    """The ctypes mirror of lp_model / lp_mlp has the fields of include/lp.h in the header's order (a stale mirror
    would shift every pointer)."""
    text = open(os.path.join(ROOT, "include", "lp.h")).read()
    for cname, mirror in (("lp_model", B._ModelStruct), ("lp_mlp", B._MlpStruct), ("lp_csr", B._CsrStruct),
                          ("lp_grads", B._GradsStruct), ("lp_acts", B._ActsStruct)):
        body = re.search(r"typedef struct %s \{(.*?)\} %s;" % (cname, cname), text, re.S).group(1)
        body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
        names = []
        for decl in body.split(";"):
            for part in decl.split(","):
                m = re.search(r"(\w+)\s*(\[[^\]]*\])?\s*$", part.strip())
                if m and part.strip():
                    names.append(m.group(1))
        assert names == [f[0] for f in mirror._fields_], (cname, names)
    assert B._ModelStruct.W_self.offset == 56 and B._ModelStruct.fp32_products.offset == 48
