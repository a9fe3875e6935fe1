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
    return sorted(set(re.findall(r"\b(lp_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_function():
    lib = B.load_library()
    names = declared_functions()
    assert set(names) == set(B.EXPORTS), (names, sorted(B.EXPORTS))
    for n in names:
        assert getattr(lib, n) is not None


def test_strerror_covers_all_codes():
    texts = {B.lp_strerror(c) for c in (0, -1, -2, -3, -4, -5)}
    assert len(texts) == 6 and B.lp_strerror(-99) == "unknown status"


def _model(dims, dtype=0, null_w=False):
    m = B._ModelStruct()
    m.n_layers, m.dtype = len(dims) - 1, dtype
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
                         None, None, C.byref(nnz), kw.get("ws", p), kw.get("ws_bytes", 1 << 30), None]
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
        H, 10, F, dt, B_, npos, p, p, p, loss, p, ws, wsb, None)
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
