"""ctypes binding of include/lp.h.  Argument marshalling only.

torch is used for device memory and the current HIP stream; no tensor arithmetic happens here.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional

import torch

LP_MAX_LAYERS = 8
LP_SYMMETRIZE = 1
LP_F32 = 0
LP_BF16 = 1
LP_LAYER_SAGE_MEAN = 0
LP_LAYER_GCN = 1
LP_FP32_PRODUCTS_NATIVE = 0
LP_FP32_PRODUCTS_BF16X6 = 1

_TORCH_OF = {LP_F32: torch.float32, LP_BF16: torch.bfloat16}
_LP_OF = {torch.float32: LP_F32, torch.bfloat16: LP_BF16}

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB = None


class LpError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s failed: %s (%d)" % (where, lp_strerror(status), status))


class _CsrStruct(C.Structure):
    _fields_ = [("n_nodes", C.c_int32), ("reserved_", C.c_int32), ("nnz", C.c_int64),
                ("rowptr", C.c_void_p), ("colidx", C.c_void_p), ("t_rowptr", C.c_void_p), ("t_colidx", C.c_void_p),
                ("inv_deg", C.c_void_p), ("row_order", C.c_void_p), ("t_row_order", C.c_void_p), ("t_entry_scale", C.c_void_p)]


class _ModelStruct(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("dtype", C.c_int32), ("dims", C.c_int32 * (LP_MAX_LAYERS + 1)),
                ("layer_type", C.c_int32), ("fp32_products", C.c_int32), ("reserved_", C.c_int32),
                ("W_self", C.c_void_p * LP_MAX_LAYERS), ("W_neigh", C.c_void_p * LP_MAX_LAYERS),
                ("bias", C.c_void_p * LP_MAX_LAYERS)]


class _ActsStruct(C.Structure):
    _fields_ = [("A", C.c_void_p * LP_MAX_LAYERS), ("H", C.c_void_p * LP_MAX_LAYERS)]


class _GradsStruct(C.Structure):
    _fields_ = [("dW_self", C.c_void_p * LP_MAX_LAYERS), ("dW_neigh", C.c_void_p * LP_MAX_LAYERS),
                ("dbias", C.c_void_p * LP_MAX_LAYERS), ("dX", C.c_void_p)]


LP_MAX_FANOUT = 64
LP_MAX_MLP_LAYERS = 4


class _MlpStruct(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("dtype", C.c_int32), ("dims", C.c_int32 * (LP_MAX_MLP_LAYERS + 1)),
                ("fp32_products", C.c_int32), ("W", C.c_void_p * LP_MAX_MLP_LAYERS), ("bias", C.c_void_p * LP_MAX_MLP_LAYERS)]


class _MlpActsStruct(C.Structure):
    _fields_ = [("X", C.c_void_p), ("U", C.c_void_p * LP_MAX_MLP_LAYERS)]


class _MlpGradsStruct(C.Structure):
    _fields_ = [("dW", C.c_void_p * LP_MAX_MLP_LAYERS), ("dbias", C.c_void_p * LP_MAX_MLP_LAYERS)]


class _BlocksStruct(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("n_graph_nodes", C.c_int32), ("n_edges", C.c_int64),
                ("cap", C.c_int32 * (LP_MAX_LAYERS + 1)), ("reserved_", C.c_int32),
                ("cap_entries", C.c_int64 * LP_MAX_LAYERS),
                ("n", C.c_void_p), ("nodes", C.c_void_p), ("index", C.c_void_p),
                ("ptr", C.c_void_p * LP_MAX_LAYERS), ("col", C.c_void_p * LP_MAX_LAYERS),
                ("inv_cnt", C.c_void_p * LP_MAX_LAYERS), ("t_ptr", C.c_void_p * LP_MAX_LAYERS),
                ("t_col", C.c_void_p * LP_MAX_LAYERS), ("e_src_pos", C.c_void_p), ("e_dst_pos", C.c_void_p),
                ("node_inv_deg", C.c_void_p)]


class _OptStateStruct(C.Structure):
    _fields_ = [(n, C.c_void_p * LP_MAX_LAYERS) for n in ("m_W_self", "m_W_neigh", "m_bias", "v_W_self", "v_W_neigh", "v_bias")]


EXPORTS = {
    "lp_strerror": (C.c_char_p, [C.c_int]),
    "lp_abi_version": (C.c_int, []),
    "lp_build_csr_workspace_bytes": (C.c_size_t, [C.c_int32, C.c_int64, C.c_uint32]),
    "lp_build_csr": (C.c_int, [C.c_int32, C.c_int64, C.c_void_p, C.c_void_p, C.c_uint32, C.c_void_p, C.c_void_p,
                               C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(C.c_int64),
                               C.c_void_p, C.c_size_t, C.c_void_p]),
    "lp_sage_forward_workspace_bytes": (C.c_size_t, [C.POINTER(_ModelStruct), C.c_int32]),
    "lp_sage_forward_edges_workspace_bytes": (C.c_size_t, [C.POINTER(_ModelStruct), C.c_int32, C.c_int64]),
    "lp_sage_forward_edges": (C.c_int, [C.POINTER(_CsrStruct), C.POINTER(_ModelStruct), C.c_void_p, C.c_int64, C.c_void_p,
                                        C.c_void_p, C.POINTER(_ActsStruct), C.c_void_p, C.c_size_t, C.c_void_p]),
    "lp_sage_forward": (C.c_int, [C.POINTER(_CsrStruct), C.POINTER(_ModelStruct), C.c_void_p, C.POINTER(_ActsStruct),
                                  C.c_void_p, C.c_size_t, C.c_void_p]),
    "lp_sample_neg": (C.c_int, [C.POINTER(_CsrStruct), C.c_int64, C.c_void_p, C.c_int32, C.c_int32, C.c_uint64,
                                C.c_uint64, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]),
    "lp_score_loss_workspace_bytes": (C.c_size_t, [C.c_int64]),
    "lp_score_loss": (C.c_int, [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int64, C.c_int64, C.c_void_p,
                                C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]),
    "lp_score_loss_noalloc": (C.c_int, [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int64, C.c_int64, C.c_void_p,
                                        C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]),
    "lp_backward_workspace_bytes": (C.c_size_t, [C.POINTER(_ModelStruct), C.c_int32, C.c_int64]),
    "lp_sparsify_workspace_bytes": (C.c_size_t, [C.c_int32, C.c_int64]),
    "lp_sparsify": (C.c_int, [C.c_int32, C.c_int64, C.c_void_p, C.c_void_p, C.c_int64, C.c_uint64, C.c_void_p, C.c_void_p,
                              C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(C.c_int64), C.c_void_p, C.c_size_t, C.c_void_p]),
    "lp_blocks_bounds": (C.c_int, [C.c_int32, C.c_int64, C.c_int64, C.c_int32, C.POINTER(C.c_int32), C.POINTER(C.c_int32),
                                   C.POINTER(C.c_int64)]),
    "lp_sample_blocks_workspace_bytes": (C.c_size_t, [C.c_int32, C.c_int64, C.c_int64, C.c_int32, C.POINTER(C.c_int32)]),
    "lp_sample_blocks": (C.c_int, [C.POINTER(_CsrStruct), C.c_int64, C.c_void_p, C.c_void_p, C.c_int32, C.POINTER(C.c_int32),
                                   C.c_uint64, C.c_uint64, C.POINTER(_BlocksStruct), C.c_void_p, C.c_size_t, C.c_void_p]),
    "lp_forward_blocks_workspace_bytes": (C.c_size_t, [C.POINTER(_ModelStruct), C.POINTER(_BlocksStruct)]),
    "lp_sage_forward_blocks": (C.c_int, [C.POINTER(_BlocksStruct), C.POINTER(_ModelStruct), C.c_void_p, C.c_void_p,
                                         C.POINTER(_ActsStruct), C.c_void_p, C.c_size_t, C.c_void_p]),
    "lp_backward_blocks_workspace_bytes": (C.c_size_t, [C.POINTER(_ModelStruct), C.POINTER(_BlocksStruct)]),
    "lp_backward_blocks": (C.c_int, [C.POINTER(_BlocksStruct), C.POINTER(_ModelStruct), C.c_void_p, C.POINTER(_ActsStruct),
                                     C.c_void_p, C.POINTER(_GradsStruct), C.c_void_p, C.c_size_t, C.c_void_p]),
    "lp_backward_blocks_edge_grads": (C.c_int, [C.POINTER(_BlocksStruct), C.POINTER(_ModelStruct), C.c_void_p, C.POINTER(_ActsStruct),
                                     C.c_void_p, C.POINTER(_GradsStruct), C.c_void_p, C.c_size_t, C.c_void_p]),
    "lp_hits_at_k_workspace_bytes": (C.c_size_t, [C.c_int64]),
    "lp_hits_at_k": (C.c_int, [C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t,
                               C.c_void_p]),
    "lp_mlp_score_loss_workspace_bytes": (C.c_size_t, [C.POINTER(_MlpStruct), C.c_int64]),
    "lp_mlp_score_loss": (C.c_int, [C.c_void_p, C.c_int32, C.c_int64, C.c_int64, C.c_void_p, C.c_void_p, C.POINTER(_MlpStruct),
                                    C.POINTER(_MlpActsStruct), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t,
                                    C.c_void_p]),
    "lp_mlp_backward_workspace_bytes": (C.c_size_t, [C.POINTER(_MlpStruct), C.c_int64]),
    "lp_mlp_backward": (C.c_int, [C.POINTER(_MlpStruct), C.POINTER(_MlpActsStruct), C.c_int64, C.c_void_p,
                                  C.POINTER(_MlpGradsStruct), C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]),
    "lp_backward_edge_grads": (C.c_int, [C.POINTER(_CsrStruct), C.POINTER(_ModelStruct), C.c_void_p, C.POINTER(_ActsStruct),
                                         C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(_GradsStruct), C.c_void_p,
                                         C.c_size_t, C.c_void_p]),
    "lp_sgd_update_tensor": (C.c_int, [C.c_void_p, C.c_int32, C.c_void_p, C.c_int64, C.c_float, C.c_void_p]),
    "lp_adam_update_tensor": (C.c_int, [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_int64,
                                        C.c_float, C.c_float, C.c_float, C.c_float, C.c_void_p]),
    "lp_sgd_step": (C.c_int, [C.POINTER(_ModelStruct), C.POINTER(_GradsStruct), C.c_float, C.c_void_p]),
    "lp_adam_step": (C.c_int, [C.POINTER(_ModelStruct), C.POINTER(_GradsStruct), C.POINTER(_OptStateStruct), C.c_int64,
                               C.c_float, C.c_float, C.c_float, C.c_float, C.c_void_p]),
    "lp_timing_enable": (C.c_int, [C.c_int]),
    "lp_timing_collect": (C.c_int, [C.POINTER(C.c_double), C.POINTER(C.c_int64), C.c_int32]),
    "lp_backward": (C.c_int, [C.POINTER(_CsrStruct), C.POINTER(_ModelStruct), C.c_void_p, C.POINTER(_ActsStruct),
                              C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(_GradsStruct), C.c_void_p,
                              C.c_size_t, C.c_void_p]),
}


def lib_path() -> str:
    return os.path.join(_PKG, "liblp_mi355x.so")


def load_library():
    """Load liblp_mi355x.so.  There is no fallback: a missing library is an error."""
    global _LIB
    if _LIB is None:
        path = lib_path()
        if not os.path.exists(path):
            raise RuntimeError("%s is not built; run `python -m paper_2506_20818_amd.build`" % path)
        lib = C.CDLL(path)
        for name, (res, args) in EXPORTS.items():
            fn = getattr(lib, name, None)
            if fn is None:
                raise RuntimeError("%s does not export %s: it was built from older sources; run "
                                   "`python -m paper_2506_20818_amd.build`" % (path, name))
            fn.restype = res
            fn.argtypes = args
        # a library built before the last change of include/lp.h would be called with the wrong struct layouts
        header = os.path.join(os.path.dirname(_PKG), "include", "lp.h")
        if os.path.exists(header):
            import re
            m = re.search(r"#define\s+LP_ABI_VERSION\s+(\d+)", open(header).read())
            if m and int(m.group(1)) != int(lib.lp_abi_version()):
                raise RuntimeError("%s was built for version %d of include/lp.h, the header is at version %s; run "
                                   "`python -m paper_2506_20818_amd.build`" % (path, lib.lp_abi_version(), m.group(1)))
        _LIB = lib
    return _LIB


def lp_strerror(status: int) -> str:
    return load_library().lp_strerror(int(status)).decode()


def _check(status: int, where: str):
    if status != 0:
        raise LpError(status, where)


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _need(t: torch.Tensor, dtype, name: str):
    if not (t.is_cuda and t.dtype == dtype and t.is_contiguous()):
        raise ValueError("%s must be a contiguous device tensor of %s" % (name, dtype))


def _ws(nbytes: int, device) -> torch.Tensor:
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


class Csr:
    """Device CSR of the visible graph, its transpose, inverse degrees and degree-ordered row lists."""

    def __init__(self, n_nodes, nnz, rowptr, colidx, t_rowptr, t_colidx, inv_deg, row_order, t_row_order, t_entry_scale=None):
        self.n_nodes, self.nnz = int(n_nodes), int(nnz)
        self.rowptr, self.colidx, self.t_rowptr, self.t_colidx = rowptr, colidx, t_rowptr, t_colidx
        self.inv_deg, self.row_order, self.t_row_order, self.t_entry_scale = inv_deg, row_order, t_row_order, t_entry_scale
        s = _CsrStruct()
        s.n_nodes, s.nnz = self.n_nodes, self.nnz
        s.rowptr, s.colidx = rowptr.data_ptr(), colidx.data_ptr()
        s.t_rowptr, s.t_colidx = t_rowptr.data_ptr(), t_colidx.data_ptr()
        s.inv_deg = inv_deg.data_ptr()
        s.row_order = row_order.data_ptr() if row_order is not None else None
        s.t_row_order = t_row_order.data_ptr() if t_row_order is not None else None
        s.t_entry_scale = t_entry_scale.data_ptr() if t_entry_scale is not None else None
        self.c = s


class Model:
    """Weights of the K layers: W_self[k], W_neigh[k] of shape [F_{k-1}, F_k] (float32 or bfloat16, which selects
    the storage type of the whole model) and bias[k] of shape [F_k] (always float32)."""

    def __init__(self, W_self: Optional[List[torch.Tensor]], W_neigh: List[torch.Tensor], bias: List[torch.Tensor],
                 layer_type: int = LP_LAYER_SAGE_MEAN, fp32_products: int = LP_FP32_PRODUCTS_BF16X6):
        """layer_type LP_LAYER_GCN: one weight matrix per layer (given as W_neigh), W_self is None.
        fp32_products: how a float32 model forms its dense products (the `fp32_products` field of lp_model; this
        binding fills in the bfloat16-term mode unless told otherwise, a zeroed C struct means the fp32 matrix
        instructions); ignored for bfloat16 models."""
        K = len(W_neigh)
        gcn = layer_type == LP_LAYER_GCN
        if W_self is None:
            W_self = [None] * K
        if not (1 <= K <= LP_MAX_LAYERS and len(W_self) == K and len(bias) == K):
            raise ValueError("bad layer count")
        self.layer_type = layer_type
        self.fp32_products = int(fp32_products)
        self.W_self, self.W_neigh, self.bias = list(W_self), list(W_neigh), list(bias)
        self.dims = [int(W_neigh[0].shape[0])] + [int(w.shape[1]) for w in W_neigh]
        self.torch_dtype = W_neigh[0].dtype
        if self.torch_dtype not in _LP_OF:
            raise ValueError("weights must be float32 or bfloat16")
        self.dtype = _LP_OF[self.torch_dtype]
        s = _ModelStruct()
        s.n_layers, s.dtype, s.layer_type, s.fp32_products = K, self.dtype, layer_type, self.fp32_products
        for k in range(K + 1):
            s.dims[k] = self.dims[k]
        for k in range(K):
            for t, nm in ((W_self[k], "W_self"), (W_neigh[k], "W_neigh")):
                if t is None and gcn and nm == "W_self":
                    continue
                _need(t, self.torch_dtype, nm)
                if tuple(t.shape) != (self.dims[k], self.dims[k + 1]):
                    raise ValueError("%s[%d] has the wrong shape" % (nm, k))
            _need(bias[k], torch.float32, "bias")
            s.W_self[k] = W_self[k].data_ptr() if W_self[k] is not None else None
            s.W_neigh[k], s.bias[k] = W_neigh[k].data_ptr(), bias[k].data_ptr()
        self.c = s

    def with_products(self, fp32_products: int) -> "Model":
        """The same weight tensors as a model that forms its fp32 products the other way."""
        return Model(self.W_self if self.layer_type != LP_LAYER_GCN else None, self.W_neigh, self.bias, self.layer_type, fp32_products)


class Acts:
    """Saved activations: A[k-1] = mean-aggregated input of layer k, H[k-1] = output of layer k."""

    def __init__(self, n_nodes: int, dims: List[int], device, dtype=torch.float32):
        K = len(dims) - 1
        self.A = [torch.empty((n_nodes, dims[k]), dtype=dtype, device=device) for k in range(K)]
        self.H = [torch.empty((n_nodes, dims[k + 1]), dtype=dtype, device=device) for k in range(K)]
        s = _ActsStruct()
        for k in range(K):
            s.A[k], s.H[k] = self.A[k].data_ptr(), self.H[k].data_ptr()
        self.c = s


class Grads:
    def __init__(self, n_nodes: int, dims: List[int], device, want_dX: bool = False, dtype=torch.float32):
        K = len(dims) - 1
        mk = lambda *shape: torch.empty(shape, dtype=torch.float32, device=device)
        self.dW_self = [mk(dims[k], dims[k + 1]) for k in range(K)]
        self.dW_neigh = [mk(dims[k], dims[k + 1]) for k in range(K)]
        self.dbias = [mk(dims[k + 1]) for k in range(K)]
        self.dX = torch.empty((n_nodes, dims[0]), dtype=dtype, device=device) if want_dX else None
        s = _GradsStruct()
        for k in range(K):
            s.dW_self[k], s.dW_neigh[k], s.dbias[k] = (self.dW_self[k].data_ptr(), self.dW_neigh[k].data_ptr(),
                                                       self.dbias[k].data_ptr())
        s.dX = self.dX.data_ptr() if want_dX else None
        self.c = s


# ----------------------------------------------------------------------------------------------------------
def lp_build_csr(n_nodes: int, rows: torch.Tensor, cols: torch.Tensor, symmetrize: bool,
                 with_row_order: bool = True, with_entry_scale: bool = True) -> Csr:
    lib = load_library()
    _need(rows, torch.int32, "rows")
    _need(cols, torch.int32, "cols")
    dev = rows.device
    n_in = int(rows.numel())
    flags = LP_SYMMETRIZE if symmetrize else 0
    cap = max(1, n_in * (2 if symmetrize else 1))
    i32 = lambda n: torch.empty(n, dtype=torch.int32, device=dev)
    rowptr, t_rowptr = i32(n_nodes + 1), i32(n_nodes + 1)
    colidx, t_colidx = i32(cap), i32(cap)
    inv_deg = torch.empty(n_nodes, dtype=torch.float32, device=dev)
    row_order = i32(n_nodes) if with_row_order else None
    t_row_order = i32(n_nodes) if with_row_order else None
    t_entry_scale = torch.empty(cap, dtype=torch.float32, device=dev) if with_entry_scale else None
    ws_bytes = lib.lp_build_csr_workspace_bytes(n_nodes, n_in, flags)
    ws = _ws(ws_bytes, dev)
    nnz = C.c_int64(0)
    _check(lib.lp_build_csr(n_nodes, n_in, _ptr(rows), _ptr(cols), flags, _ptr(rowptr), _ptr(colidx), _ptr(t_rowptr),
                            _ptr(t_colidx), _ptr(inv_deg), _ptr(row_order), _ptr(t_row_order), _ptr(t_entry_scale), C.byref(nnz),
                            _ptr(ws), ws.numel(), _stream()), "lp_build_csr")
    n = int(nnz.value)
    return Csr(n_nodes, n, rowptr, colidx[:n], t_rowptr, t_colidx[:n], inv_deg, row_order, t_row_order,
               t_entry_scale[:n] if t_entry_scale is not None else None)


def lp_sage_forward(g: Csr, m: Model, X: torch.Tensor, acts: Optional[Acts] = None, ws: Optional[torch.Tensor] = None) -> Acts:
    lib = load_library()
    _need(X, m.torch_dtype, "X")
    if tuple(X.shape) != (g.n_nodes, m.dims[0]):
        raise ValueError("X has the wrong shape")
    if acts is None:
        acts = Acts(g.n_nodes, m.dims, X.device, m.torch_dtype)
    if ws is None:
        ws = _ws(lib.lp_sage_forward_workspace_bytes(C.byref(m.c), g.n_nodes), X.device)
    _check(lib.lp_sage_forward(C.byref(g.c), C.byref(m.c), _ptr(X), C.byref(acts.c), _ptr(ws), ws.numel(), _stream()),
           "lp_sage_forward")
    return acts


def lp_sage_forward_edges(g: Csr, m: Model, X: torch.Tensor, e_src: torch.Tensor, e_dst: torch.Tensor,
                          acts: Optional[Acts] = None, ws: Optional[torch.Tensor] = None) -> Acts:
    """The forward pass of a training step: the last layer only for the end points of the scored edges (the other rows
    of acts.A[-1] and acts.H[-1] keep what they held)."""
    lib = load_library()
    _need(X, m.torch_dtype, "X")
    _need(e_src, torch.int32, "e_src")
    _need(e_dst, torch.int32, "e_dst")
    if tuple(X.shape) != (g.n_nodes, m.dims[0]):
        raise ValueError("X has the wrong shape")
    Bn = int(e_src.numel())
    if int(e_dst.numel()) != Bn:
        raise ValueError("e_src and e_dst differ in length")
    if acts is None:
        acts = Acts(g.n_nodes, m.dims, X.device, m.torch_dtype)
    if ws is None:
        ws = _ws(lib.lp_sage_forward_edges_workspace_bytes(C.byref(m.c), g.n_nodes, Bn), X.device)
    _check(lib.lp_sage_forward_edges(C.byref(g.c), C.byref(m.c), _ptr(X), Bn, _ptr(e_src), _ptr(e_dst), C.byref(acts.c),
                                     _ptr(ws), ws.numel(), _stream()), "lp_sage_forward_edges")
    return acts


def lp_sample_neg(g: Csr, pos_src: torch.Tensor, k_neg: int, n_space: int, seed: int, step: int,
                  neg_dst: Optional[torch.Tensor] = None, neg_src: Optional[torch.Tensor] = None,
                  n_failed: Optional[torch.Tensor] = None):
    lib = load_library()
    _need(pos_src, torch.int32, "pos_src")
    n_pos = int(pos_src.numel())
    if neg_dst is None:
        neg_dst = torch.empty(n_pos * k_neg, dtype=torch.int32, device=pos_src.device)
    _check(lib.lp_sample_neg(C.byref(g.c), n_pos, _ptr(pos_src), k_neg, n_space, seed, step, _ptr(neg_dst), _ptr(neg_src),
                             _ptr(n_failed), _stream()), "lp_sample_neg")
    return neg_dst


def lp_score_loss(HK: torch.Tensor, e_src: torch.Tensor, e_dst: torch.Tensor, n_pos_edges: int,
                  scores: Optional[torch.Tensor] = None, loss: Optional[torch.Tensor] = None,
                  dscore: Optional[torch.Tensor] = None, ws: Optional[torch.Tensor] = None,
                  n_invalid: Optional[torch.Tensor] = None):
    """n_invalid: optional int32 device scalar, zeroed by the caller; receives the number of edges with an id outside
    the node range (which are scored 0 and left out of the loss sum)."""
    lib = load_library()
    if HK.dtype not in _LP_OF:
        raise ValueError("HK must be float32 or bfloat16")
    _need(HK, HK.dtype, "HK")
    _need(e_src, torch.int32, "e_src")
    _need(e_dst, torch.int32, "e_dst")
    B = int(e_src.numel())
    dev = HK.device
    if scores is None:
        scores = torch.empty(B, dtype=torch.float32, device=dev)
    if loss is None:
        loss = torch.empty(1, dtype=torch.float32, device=dev)
    if dscore is None:
        dscore = torch.empty(B, dtype=torch.float32, device=dev)
    if ws is None:
        ws = _ws(lib.lp_score_loss_workspace_bytes(B), dev)
    _check(lib.lp_score_loss(_ptr(HK), HK.shape[0], HK.shape[1], _LP_OF[HK.dtype], B, n_pos_edges, _ptr(e_src), _ptr(e_dst),
                             _ptr(scores), _ptr(loss), _ptr(dscore), _ptr(n_invalid), _ptr(ws), ws.numel(), _stream()), "lp_score_loss")
    return scores, loss, dscore


def lp_score_loss_noalloc(HK: torch.Tensor, e_src: torch.Tensor, e_dst: torch.Tensor, n_pos_edges: int,
                          scores: torch.Tensor, loss: torch.Tensor, dscore: Optional[torch.Tensor] = None,
                          n_invalid: Optional[torch.Tensor] = None):
    """lp_score_loss without a workspace: the caller passes every output, nothing is allocated here or in the
    library (its scratch is a device array inside the library)."""
    lib = load_library()
    if HK.dtype not in _LP_OF:
        raise ValueError("HK must be float32 or bfloat16")
    _need(HK, HK.dtype, "HK")
    _need(e_src, torch.int32, "e_src")
    _need(e_dst, torch.int32, "e_dst")
    _need(scores, torch.float32, "scores")
    _need(loss, torch.float32, "loss")
    if dscore is not None:
        _need(dscore, torch.float32, "dscore")
    B = int(e_src.numel())
    if int(e_dst.numel()) != B or int(scores.numel()) < B or (dscore is not None and int(dscore.numel()) < B) or loss.numel() < 1:
        raise ValueError("e_dst, scores and dscore must hold one entry per edge of e_src")
    _check(lib.lp_score_loss_noalloc(_ptr(HK), HK.shape[0], HK.shape[1], _LP_OF[HK.dtype], B, n_pos_edges, _ptr(e_src),
                                     _ptr(e_dst), _ptr(scores), _ptr(loss), _ptr(dscore), _ptr(n_invalid), _stream()), "lp_score_loss_noalloc")
    return scores, loss, dscore


def lp_backward(g: Csr, m: Model, X: torch.Tensor, acts: Acts, e_src: torch.Tensor, e_dst: torch.Tensor,
                dscore: torch.Tensor, grads: Optional[Grads] = None, ws: Optional[torch.Tensor] = None,
                want_dX: bool = False) -> Grads:
    lib = load_library()
    _need(X, m.torch_dtype, "X")
    _need(dscore, torch.float32, "dscore")
    if grads is None:
        grads = Grads(g.n_nodes, m.dims, X.device, want_dX, m.torch_dtype)
    if ws is None:
        ws = _ws(lib.lp_backward_workspace_bytes(C.byref(m.c), g.n_nodes, int(e_src.numel())), X.device)
    _check(lib.lp_backward(C.byref(g.c), C.byref(m.c), _ptr(X), C.byref(acts.c), int(e_src.numel()), _ptr(e_src),
                           _ptr(e_dst), _ptr(dscore), C.byref(grads.c), _ptr(ws), ws.numel(), _stream()), "lp_backward")
    return grads


class Blocks:
    """Device arrays of one mini-batch's sampled computational graph (see lp_blocks in include/lp.h), sized by
    lp_blocks_bounds.  Reusable across batches of the same size on the same graph."""

    def __init__(self, g: Csr, B: int, fanout: List[int]):
        lib = load_library()
        K = len(fanout)
        self.K, self.B, self.fanout = K, int(B), [int(f) for f in fanout]
        self.fan_c = (C.c_int32 * K)(*self.fanout)
        cap = (C.c_int32 * (K + 1))()
        cap_e = (C.c_int64 * K)()
        _check(lib.lp_blocks_bounds(g.n_nodes, g.nnz, self.B, K, self.fan_c, cap, cap_e), "lp_blocks_bounds")
        self.cap, self.cap_entries = [int(x) for x in cap], [int(x) for x in cap_e]
        dev = g.rowptr.device
        i32 = lambda n: torch.empty(max(int(n), 1), dtype=torch.int32, device=dev)
        self.n = i32(K + 1)
        self.nodes, self.index = i32(self.cap[0]), i32(g.n_nodes)
        self.ptr = [i32(self.cap[k] + 1) for k in range(1, K + 1)]
        self.col = [i32(self.cap_entries[k - 1]) for k in range(1, K + 1)]
        self.inv_cnt = [torch.empty(max(self.cap[k], 1), dtype=torch.float32, device=dev) for k in range(1, K + 1)]
        self.t_ptr = [i32(self.cap[k - 1] + 1) for k in range(1, K + 1)]
        self.t_col = [i32(self.cap_entries[k - 1]) for k in range(1, K + 1)]
        self.e_src_pos, self.e_dst_pos = i32(self.B), i32(self.B)
        self.node_inv_deg = torch.empty(max(self.cap[0], 1), dtype=torch.float32, device=dev)
        s = _BlocksStruct()
        s.n_layers, s.n_graph_nodes, s.n_edges = K, g.n_nodes, self.B
        for k in range(K + 1):
            s.cap[k] = self.cap[k]
        for k in range(K):
            s.cap_entries[k] = self.cap_entries[k]
            s.ptr[k], s.col[k], s.inv_cnt[k] = self.ptr[k].data_ptr(), self.col[k].data_ptr(), self.inv_cnt[k].data_ptr()
            s.t_ptr[k], s.t_col[k] = self.t_ptr[k].data_ptr(), self.t_col[k].data_ptr()
        s.n, s.nodes, s.index = self.n.data_ptr(), self.nodes.data_ptr(), self.index.data_ptr()
        s.e_src_pos, s.e_dst_pos = self.e_src_pos.data_ptr(), self.e_dst_pos.data_ptr()
        s.node_inv_deg = self.node_inv_deg.data_ptr()
        self.c = s
        self.sample_ws = _ws(lib.lp_sample_blocks_workspace_bytes(g.n_nodes, g.nnz, self.B, K, self.fan_c), dev)


class BlockActs:
    """Activations of the sampled step: X_frontier [cap[0], F_0], A[k-1] [cap[k], F_{k-1}], H[k-1] [cap[k], F_k]."""

    def __init__(self, b: Blocks, dims: List[int], device, dtype=torch.float32):
        K = len(dims) - 1
        self.X_frontier = torch.empty((max(b.cap[0], 1), dims[0]), dtype=dtype, device=device)
        self.A = [torch.empty((max(b.cap[k + 1], 1), dims[k]), dtype=dtype, device=device) for k in range(K)]
        self.H = [torch.empty((max(b.cap[k + 1], 1), dims[k + 1]), dtype=dtype, device=device) for k in range(K)]
        s = _ActsStruct()
        for k in range(K):
            s.A[k], s.H[k] = self.A[k].data_ptr(), self.H[k].data_ptr()
        self.c = s


def lp_sample_blocks(g: Csr, e_src: torch.Tensor, e_dst: torch.Tensor, fanout: List[int], seed: int, step: int,
                     blocks: Optional[Blocks] = None) -> Blocks:
    _need(e_src, torch.int32, "e_src")
    _need(e_dst, torch.int32, "e_dst")
    if blocks is None:
        blocks = Blocks(g, int(e_src.numel()), fanout)
    _check(load_library().lp_sample_blocks(C.byref(g.c), blocks.B, _ptr(e_src), _ptr(e_dst), blocks.K, blocks.fan_c, seed, step,
                                           C.byref(blocks.c), _ptr(blocks.sample_ws), blocks.sample_ws.numel(), _stream()),
           "lp_sample_blocks")
    return blocks


def lp_sage_forward_blocks(b: Blocks, m: Model, X: torch.Tensor, acts: Optional[BlockActs] = None,
                           ws: Optional[torch.Tensor] = None) -> BlockActs:
    lib = load_library()
    _need(X, m.torch_dtype, "X")
    if acts is None:
        acts = BlockActs(b, m.dims, X.device, m.torch_dtype)
    if ws is None:
        ws = _ws(lib.lp_forward_blocks_workspace_bytes(C.byref(m.c), C.byref(b.c)), X.device)
    _check(lib.lp_sage_forward_blocks(C.byref(b.c), C.byref(m.c), _ptr(X), _ptr(acts.X_frontier), C.byref(acts.c), _ptr(ws),
                                      ws.numel(), _stream()), "lp_sage_forward_blocks")
    return acts


def lp_backward_blocks(b: Blocks, m: Model, acts: BlockActs, dscore: torch.Tensor, grads: Optional[Grads] = None,
                       ws: Optional[torch.Tensor] = None) -> Grads:
    lib = load_library()
    _need(dscore, torch.float32, "dscore")
    dev = dscore.device
    if grads is None:
        grads = Grads(1, m.dims, dev, False, m.torch_dtype)
    if ws is None:
        ws = _ws(lib.lp_backward_blocks_workspace_bytes(C.byref(m.c), C.byref(b.c)), dev)
    _check(lib.lp_backward_blocks(C.byref(b.c), C.byref(m.c), _ptr(acts.X_frontier), C.byref(acts.c), _ptr(dscore),
                                  C.byref(grads.c), _ptr(ws), ws.numel(), _stream()), "lp_backward_blocks")
    return grads


def lp_backward_blocks_edge_grads(b: Blocks, m: Model, acts: BlockActs, edge_grad: torch.Tensor, grads: Optional[Grads] = None,
                                  ws: Optional[torch.Tensor] = None) -> Grads:
    lib = load_library()
    _need(edge_grad, m.torch_dtype, "edge_grad")
    dev = edge_grad.device
    if grads is None:
        grads = Grads(1, m.dims, dev, False, m.torch_dtype)
    if ws is None:
        ws = _ws(lib.lp_backward_blocks_workspace_bytes(C.byref(m.c), C.byref(b.c)), dev)
    _check(lib.lp_backward_blocks_edge_grads(C.byref(b.c), C.byref(m.c), _ptr(acts.X_frontier), C.byref(acts.c), _ptr(edge_grad),
                                             C.byref(grads.c), _ptr(ws), ws.numel(), _stream()), "lp_backward_blocks_edge_grads")
    return grads


def lp_hits_at_k(pos_scores: torch.Tensor, neg_scores: torch.Tensor, K: int, ws: Optional[torch.Tensor] = None):
    """Returns (hits, threshold) as device tensors (int64 [1], float32 [1]); Hits@K = hits / pos_scores.numel()."""
    lib = load_library()
    _need(pos_scores, torch.float32, "pos_scores")
    _need(neg_scores, torch.float32, "neg_scores")
    dev = pos_scores.device
    hits = torch.zeros(1, dtype=torch.int64, device=dev)
    thr = torch.zeros(1, dtype=torch.float32, device=dev)
    if ws is None:
        ws = _ws(lib.lp_hits_at_k_workspace_bytes(int(neg_scores.numel())), dev)
    _check(lib.lp_hits_at_k(_ptr(pos_scores), int(pos_scores.numel()), _ptr(neg_scores), int(neg_scores.numel()), int(K), _ptr(hits),
                            _ptr(thr), _ptr(ws), ws.numel(), _stream()), "lp_hits_at_k")
    return hits, thr


def forward_blocks_workspace_bytes(m: Model, b: Blocks) -> int:
    return int(load_library().lp_forward_blocks_workspace_bytes(C.byref(m.c), C.byref(b.c)))


def backward_blocks_workspace_bytes(m: Model, b: Blocks) -> int:
    return int(load_library().lp_backward_blocks_workspace_bytes(C.byref(m.c), C.byref(b.c)))


class Mlp:
    """Weights of the MLP edge predictor: W[j] of shape [dims[j], dims[j+1]] (float32 or bfloat16), the last one
    [dims[L-1], 1]; bias[j] of shape [dims[j+1]] (float32)."""

    def __init__(self, W: List[torch.Tensor], bias: List[torch.Tensor], fp32_products: int = LP_FP32_PRODUCTS_BF16X6):
        L = len(W)
        if not (1 <= L <= LP_MAX_MLP_LAYERS and len(bias) == L):
            raise ValueError("bad layer count")
        self.W, self.bias = list(W), list(bias)
        self.dims = [int(W[0].shape[0])] + [int(w.shape[1]) for w in W]
        self.torch_dtype = W[0].dtype
        self.dtype = _LP_OF[self.torch_dtype]
        s = _MlpStruct()
        s.n_layers, s.dtype, s.fp32_products = L, self.dtype, int(fp32_products)
        for j in range(L + 1):
            s.dims[j] = self.dims[j]
        for j in range(L):
            _need(W[j], self.torch_dtype, "W")
            _need(bias[j], torch.float32, "bias")
            s.W[j], s.bias[j] = W[j].data_ptr(), bias[j].data_ptr()
        self.c = s


class MlpActs:
    def __init__(self, p: Mlp, B: int, device):
        L = len(p.W)
        self.X = torch.empty((max(B, 1), p.dims[0]), dtype=p.torch_dtype, device=device)
        self.U = [torch.empty((max(B, 1), p.dims[j]), dtype=p.torch_dtype, device=device) for j in range(1, L)]
        s = _MlpActsStruct()
        s.X = self.X.data_ptr()
        for j, t in enumerate(self.U):
            s.U[j] = t.data_ptr()
        self.c = s


class MlpGrads:
    def __init__(self, p: Mlp, device):
        L = len(p.W)
        self.dW = [torch.empty((p.dims[j], p.dims[j + 1]), dtype=torch.float32, device=device) for j in range(L)]
        self.dbias = [torch.empty(p.dims[j + 1], dtype=torch.float32, device=device) for j in range(L)]
        s = _MlpGradsStruct()
        for j in range(L):
            s.dW[j], s.dbias[j] = self.dW[j].data_ptr(), self.dbias[j].data_ptr()
        self.c = s


def lp_mlp_score_loss(HK: torch.Tensor, e_src: torch.Tensor, e_dst: torch.Tensor, n_pos_edges: int, p: Mlp,
                      acts: Optional[MlpActs] = None):
    lib = load_library()
    _need(HK, p.torch_dtype, "HK")
    _need(e_src, torch.int32, "e_src")
    _need(e_dst, torch.int32, "e_dst")
    B, dev = int(e_src.numel()), HK.device
    if acts is None:
        acts = MlpActs(p, B, dev)
    scores = torch.empty(B, dtype=torch.float32, device=dev)
    dscore = torch.empty(B, dtype=torch.float32, device=dev)
    loss = torch.empty(1, dtype=torch.float32, device=dev)
    ws = _ws(lib.lp_mlp_score_loss_workspace_bytes(C.byref(p.c), B), dev)
    _check(lib.lp_mlp_score_loss(_ptr(HK), HK.shape[0], B, n_pos_edges, _ptr(e_src), _ptr(e_dst), C.byref(p.c), C.byref(acts.c),
                                 _ptr(scores), _ptr(loss), _ptr(dscore), _ptr(ws), ws.numel(), _stream()), "lp_mlp_score_loss")
    return scores, loss, dscore, acts


def lp_mlp_backward(p: Mlp, acts: MlpActs, dscore: torch.Tensor, grads: Optional[MlpGrads] = None):
    """Returns (MlpGrads, edge_grad [B, dims[0]])."""
    lib = load_library()
    _need(dscore, torch.float32, "dscore")
    B, dev = int(dscore.numel()), dscore.device
    if grads is None:
        grads = MlpGrads(p, dev)
    edge_grad = torch.empty((max(B, 1), p.dims[0]), dtype=p.torch_dtype, device=dev)
    ws = _ws(lib.lp_mlp_backward_workspace_bytes(C.byref(p.c), B), dev)
    _check(lib.lp_mlp_backward(C.byref(p.c), C.byref(acts.c), B, _ptr(dscore), C.byref(grads.c), _ptr(edge_grad), _ptr(ws),
                               ws.numel(), _stream()), "lp_mlp_backward")
    return grads, edge_grad


def lp_backward_edge_grads(g: Csr, m: Model, X: torch.Tensor, acts: Acts, e_src: torch.Tensor, e_dst: torch.Tensor,
                           edge_grad: torch.Tensor, grads: Optional[Grads] = None, ws: Optional[torch.Tensor] = None,
                           want_dX: bool = False) -> Grads:
    lib = load_library()
    _need(X, m.torch_dtype, "X")
    _need(edge_grad, m.torch_dtype, "edge_grad")
    if grads is None:
        grads = Grads(g.n_nodes, m.dims, X.device, want_dX, m.torch_dtype)
    if ws is None:
        ws = _ws(lib.lp_backward_workspace_bytes(C.byref(m.c), g.n_nodes, int(e_src.numel())), X.device)
    _check(lib.lp_backward_edge_grads(C.byref(g.c), C.byref(m.c), _ptr(X), C.byref(acts.c), int(e_src.numel()), _ptr(e_src),
                                      _ptr(e_dst), _ptr(edge_grad), C.byref(grads.c), _ptr(ws), ws.numel(), _stream()),
           "lp_backward_edge_grads")
    return grads


class AdamState:
    """Zero-initialised first and second moments for every parameter tensor of a model."""

    def __init__(self, m: Model):
        z = lambda t: torch.zeros(t.shape if t is not None else (1,), dtype=torch.float32, device=m.bias[0].device)
        self.m_W_self, self.m_W_neigh, self.m_bias = [z(t) for t in m.W_self], [z(t) for t in m.W_neigh], [z(t) for t in m.bias]
        self.v_W_self, self.v_W_neigh, self.v_bias = [z(t) for t in m.W_self], [z(t) for t in m.W_neigh], [z(t) for t in m.bias]
        s = _OptStateStruct()
        for name in ("m_W_self", "m_W_neigh", "m_bias", "v_W_self", "v_W_neigh", "v_bias"):
            for k, t in enumerate(getattr(self, name)):
                getattr(s, name)[k] = t.data_ptr()
        self.c = s


def lp_adam_update_tensor(w: torch.Tensor, grad: torch.Tensor, m: torch.Tensor, v: torch.Tensor, t_step: int, lr: float = 1e-3,
                          beta1: float = 0.9, beta2: float = 0.999, eps: float = 1e-8) -> None:
    for t, nm in ((grad, "grad"), (m, "m"), (v, "v")):
        _need(t, torch.float32, nm)
    _need(w, w.dtype, "w")
    _check(load_library().lp_adam_update_tensor(_ptr(w), _LP_OF[w.dtype], _ptr(grad), _ptr(m), _ptr(v), int(w.numel()), int(t_step),
                                                lr, beta1, beta2, eps, _stream()), "lp_adam_update_tensor")


def lp_sgd_update_tensor(w: torch.Tensor, grad: torch.Tensor, lr: float) -> None:
    _need(grad, torch.float32, "grad")
    _need(w, w.dtype, "w")
    _check(load_library().lp_sgd_update_tensor(_ptr(w), _LP_OF[w.dtype], _ptr(grad), int(w.numel()), lr, _stream()),
           "lp_sgd_update_tensor")


def lp_sgd_step(m: Model, grads: Grads, lr: float) -> None:
    _check(load_library().lp_sgd_step(C.byref(m.c), C.byref(grads.c), lr, _stream()), "lp_sgd_step")


def lp_adam_step(m: Model, grads: Grads, state: AdamState, t_step: int, lr: float = 1e-3, beta1: float = 0.9,
                 beta2: float = 0.999, eps: float = 1e-8) -> None:
    _check(load_library().lp_adam_step(C.byref(m.c), C.byref(grads.c), C.byref(state.c), int(t_step), lr, beta1, beta2, eps,
                                       _stream()), "lp_adam_step")


class Sparsified:
    """Result of lp_sparsify: indices of the distinct drawn edges (ascending), their end points, how often each
    was drawn and its weight."""

    def __init__(self, kept_edge, kept_u, kept_v, count, weight):
        self.kept_edge, self.kept_u, self.kept_v, self.count, self.weight = kept_edge, kept_u, kept_v, count, weight


def lp_sparsify(n_nodes: int, eu: torch.Tensor, ev: torch.Tensor, n_draws: int, seed: int,
                ws: Optional[torch.Tensor] = None) -> Sparsified:
    lib = load_library()
    _need(eu, torch.int32, "eu")
    _need(ev, torch.int32, "ev")
    dev = eu.device
    m = int(eu.numel())
    cap = max(1, min(m, int(n_draws)))
    i32 = lambda: torch.empty(cap, dtype=torch.int32, device=dev)
    kept_edge, kept_u, kept_v, count = i32(), i32(), i32(), i32()
    weight = torch.empty(cap, dtype=torch.float32, device=dev)
    if ws is None:
        ws = _ws(lib.lp_sparsify_workspace_bytes(n_nodes, m), dev)
    n_kept = C.c_int64(0)
    _check(lib.lp_sparsify(n_nodes, m, _ptr(eu), _ptr(ev), int(n_draws), int(seed), _ptr(kept_edge), _ptr(kept_u),
                           _ptr(kept_v), _ptr(count), _ptr(weight), C.byref(n_kept), _ptr(ws), ws.numel(), _stream()),
           "lp_sparsify")
    n = int(n_kept.value)
    return Sparsified(kept_edge[:n], kept_u[:n], kept_v[:n], count[:n], weight[:n])


def sparsify_workspace_bytes(n_nodes: int, n_edges: int) -> int:
    return int(load_library().lp_sparsify_workspace_bytes(n_nodes, n_edges))


def backward_workspace_bytes(m: Model, n_nodes: int, B: int) -> int:
    return int(load_library().lp_backward_workspace_bytes(C.byref(m.c), n_nodes, B))


def forward_workspace_bytes(m: Model, n_nodes: int) -> int:
    return int(load_library().lp_sage_forward_workspace_bytes(C.byref(m.c), n_nodes))


def forward_edges_workspace_bytes(m: Model, n_nodes: int, B: int) -> int:
    return int(load_library().lp_sage_forward_edges_workspace_bytes(C.byref(m.c), n_nodes, B))


KERNEL_CLASSES = ["spmm", "gemm_nt", "gemm_tn", "scatter", "score", "sample", "other"]


def lp_timing_enable(level) -> None:
    """0/False: off; 1/True: the main kernel classes; 2: every launch."""
    _check(load_library().lp_timing_enable(int(level)), "lp_timing_enable")


def lp_timing_collect():
    """Returns {class: (milliseconds, launches)} for the launches since the last collect."""
    n = len(KERNEL_CLASSES)
    ms = (C.c_double * n)()
    cnt = (C.c_int64 * n)()
    _check(load_library().lp_timing_collect(ms, cnt, n), "lp_timing_collect")
    return {KERNEL_CLASSES[i]: (float(ms[i]), int(cnt[i])) for i in range(n)}
