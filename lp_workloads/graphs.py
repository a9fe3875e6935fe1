"""Seeded synthetic graphs and batches shaped like the paper's workloads.

The paper trains on nine public datasets (its Table I) that are not available
here; these generators only imitate their sizes and degree skew.  Everything is
drawn with ``numpy.random.default_rng(seed)`` on the host.

Nothing in this file belongs to the method itself: edges come out as an
unsorted list of undirected pairs, each once, with no self-pairs; building the
CSR, sampling negatives and all floating-point work are left to the code under
test.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional

import numpy as np

from .model_init import init_features, init_model


# --------------------------------------------------------------------------
# edge generators
# --------------------------------------------------------------------------
def _first_occurrence_unique_pairs(u: np.ndarray, v: np.ndarray, n: int):
    """Drop self-pairs and repeated unordered pairs, keeping draw order."""
    keep = u != v
    u, v = u[keep], v[keep]
    lo = np.minimum(u, v).astype(np.int64)
    hi = np.maximum(u, v).astype(np.int64)
    key = lo * np.int64(n) + hi
    _, first = np.unique(key, return_index=True)
    first.sort()
    return u[first], v[first]


def uniform_edges(n_nodes: int, m: int, seed: int):
    """``m`` distinct unordered pairs u != v, uniform over ``n_nodes`` nodes."""
    rng = np.random.default_rng(seed)
    u = np.empty(0, np.int64)
    v = np.empty(0, np.int64)
    while u.size < m:
        need = m - u.size
        du = rng.integers(0, n_nodes, size=need + need // 8 + 16)
        dv = rng.integers(0, n_nodes, size=du.size)
        u, v = _first_occurrence_unique_pairs(
            np.concatenate([u, du]), np.concatenate([v, dv]), n_nodes)
    return u[:m].astype(np.int32), v[:m].astype(np.int32)


def _chung_lu_weights(n_nodes: int, m: int, gamma: float, w_max: float):
    """Expected degrees w_i = c (i + i0)^(-1/(gamma-1)) with sum 2m and w_0 = w_max."""
    beta = 1.0 / (gamma - 1.0)
    idx = np.arange(n_nodes, dtype=np.float64)

    def w0(i0):
        raw = (idx + i0) ** (-beta)
        return 2.0 * m / raw.sum() * raw[0]

    lo, hi = 1e-9, 1e12          # w0 decreases as i0 grows
    for _ in range(200):
        mid = np.sqrt(lo * hi)
        if w0(mid) > w_max:
            lo = mid
        else:
            hi = mid
    i0 = np.sqrt(lo * hi)
    raw = (idx + i0) ** (-beta)
    return raw * (2.0 * m / raw.sum())


_EDGE_CACHE: Dict[tuple, tuple] = {}


def chung_lu_edges(n_nodes: int, m: int, gamma: float, seed: int, perm_seed: int,
                   w_max: Optional[float] = None):
    """Chung-Lu style power-law graph (the last few results are remembered per process: several workloads are
    views of the same graph, and drawing 15 M edges takes half a minute).  Callers get fresh copies."""
    key = (n_nodes, m, gamma, seed, perm_seed, w_max)
    if key not in _EDGE_CACHE:
        if len(_EDGE_CACHE) >= 2:
            _EDGE_CACHE.pop(next(iter(_EDGE_CACHE)))
        _EDGE_CACHE[key] = _chung_lu_edges(n_nodes, m, gamma, seed, perm_seed, w_max)
    u, v = _EDGE_CACHE[key]
    return u.copy(), v.copy()


def _chung_lu_edges(n_nodes: int, m: int, gamma: float, seed: int, perm_seed: int,
                    w_max: Optional[float] = None):
    """Chung-Lu style power-law graph.

    ``m`` endpoint pairs are drawn i.i.d. proportionally to the expected-degree
    weights (inverse CDF), self-pairs and repeated pairs are dropped, and node
    ids are shuffled so that degree carries no relation to id.  ``w_max`` caps
    the largest expected degree; by default it is sqrt(2m), the value above
    which two hubs would be joined with probability > 1.
    """
    if w_max is None:
        w_max = float(np.sqrt(2.0 * m))
    w = _chung_lu_weights(n_nodes, m, gamma, w_max)
    cdf = np.cumsum(w)
    cdf /= cdf[-1]
    rng = np.random.default_rng(seed)
    u = np.searchsorted(cdf, rng.random(m), side="right")
    v = np.searchsorted(cdf, rng.random(m), side="right")
    np.minimum(u, n_nodes - 1, out=u)
    np.minimum(v, n_nodes - 1, out=v)
    u, v = _first_occurrence_unique_pairs(u, v, n_nodes)
    perm = np.random.default_rng(perm_seed).permutation(n_nodes)
    return perm[u].astype(np.int32), perm[v].astype(np.int32)


def worker_view(u: np.ndarray, v: np.ndarray, n_nodes: int, parts: int, worker: int,
                keep_prob: float, part_seed: int, keep_seed: int):
    """One worker's visible graph under a random node partition.

    Nodes are assigned to ``parts`` workers uniformly at random.  The worker
    keeps every edge with both ends owned, and every edge with exactly one end
    owned independently with probability ``keep_prob`` (the stand-in for the
    sparsified remote view).  Owned nodes are relabelled first (ascending old
    id), then the remote nodes that kept at least one edge.  Kept edges are
    oriented with an owned node as the source.

    Returns (src, dst, n_visible, n_owned, old_id_of_new).
    """
    part = np.random.default_rng(part_seed).integers(0, parts, size=n_nodes)
    own_u = part[u] == worker
    own_v = part[v] == worker
    both = own_u & own_v
    one = own_u ^ own_v
    coin = np.random.default_rng(keep_seed).random(u.size) < keep_prob
    kept = both | (one & coin)
    ku, kv, kou = u[kept], v[kept], own_u[kept]
    src = np.where(kou, ku, kv)          # owned endpoint first
    dst = np.where(kou, kv, ku)
    owned = np.flatnonzero(part == worker)
    seen = np.zeros(n_nodes, bool)
    seen[dst] = True
    seen[owned] = False
    halo = np.flatnonzero(seen)
    old_of_new = np.concatenate([owned, halo])
    new_of_old = np.full(n_nodes, -1, np.int64)
    new_of_old[old_of_new] = np.arange(old_of_new.size)
    return (new_of_old[src].astype(np.int32), new_of_old[dst].astype(np.int32),
            int(old_of_new.size), int(owned.size), old_of_new)


def partition_edge_lists(u: np.ndarray, v: np.ndarray, n_nodes: int, parts: int, part_seed: int):
    """Uniform random node partition with the paper's halo rule (Sec. IV-B: cross-partition edges are kept in
    both partitions, so every owned node keeps its full neighbour list).

    Returns (part [n_nodes], edges) where edges[j] = (u_j, v_j) are the edges with at least one end in part j,
    in input order, node ids unchanged."""
    part = np.random.default_rng(part_seed).integers(0, parts, size=n_nodes)
    pu, pv = part[u], part[v]
    edges = []
    for j in range(parts):
        sel = (pu == j) | (pv == j)
        edges.append((u[sel].copy(), v[sel].copy()))
    return part, edges


# --------------------------------------------------------------------------
# workload table
# --------------------------------------------------------------------------
# Sizes follow the five benchmark configurations; seeds are fixed so that every
# consumer sees the same bytes.
CONFIGS: Dict[str, dict] = {
    # Cora/Citeseer scale
    "C1": dict(graph="uniform", n_nodes=2_000, m=10_000, dims=[64, 64, 64],
               n_pos=None, k_neg=1, dtype="f32",
               seeds=dict(graph=0, x=100, w=200, batch=300)),
    # Collab scale
    "C2": dict(graph="chung_lu", n_nodes=235_000, m=1_200_000, gamma=2.1,
               dims=[128, 256, 256, 256], n_pos=65_536, k_neg=1, dtype="f32",
               seeds=dict(graph=1, perm=11, x=101, w=201, batch=301)),
    # one of four workers on a 1M-node graph, cross edges kept w.p. 0.2
    "C3": dict(graph="chung_lu", n_nodes=1_000_000, m=10_000_000, gamma=2.1,
               view=dict(parts=4, worker=0, keep=0.2),
               dims=[128, 256, 256, 256], n_pos=65_536, k_neg=3, dtype="f32",
               seeds=dict(graph=2, perm=12, part=22, keep=32, x=102, w=202, batch=302)),
    # PPA edge count
    "C4": dict(graph="chung_lu", n_nodes=2_900_000, m=15_000_000, gamma=2.0, w_max=20_000.0,
               dims=[128, 256, 256, 256], n_pos=131_072, k_neg=1, dtype="f32",
               seeds=dict(graph=3, perm=13, x=103, w=203, batch=303)),
}
for _keep, _kseed in ((1.0, 33), (0.5, 34), (0.2, 35)):
    CONFIGS["C5_keep%g" % _keep] = dict(
        graph="chung_lu", n_nodes=2_900_000, m=15_000_000, gamma=2.0, w_max=20_000.0,
        view=dict(parts=4, worker=0, keep=_keep),
        dims=[128, 512, 512, 512], n_pos=131_072, k_neg=4, dtype="bf16",
        seeds=dict(graph=3, perm=13, part=23, keep=_kseed, x=103, w=204, batch=304))


@dataclass
class PartitionedInputs:
    """Inputs of one worker under the paper's own data layout: its partition in full, the other partitions as
    edge lists that the code under test has to sparsify (level alpha, one seed per partition), all nodes visible."""
    name: str
    n_nodes: int
    parts: int
    worker: int
    part: np.ndarray                     # int [n_nodes]: owner of each node
    edges: List[tuple]                   # edges[j] = (u, v) int32 arrays of partition j (halo edges included)
    alpha: float                         # draws per partition = floor(alpha * |E^j|)
    sparsify_seeds: List[int]
    dims: List[int]
    k_neg: int
    pos_src: np.ndarray                  # positives are edges of the worker's own partition
    pos_dst: np.ndarray
    sampler_seed: int
    sampler_step: int
    X: Optional[np.ndarray] = None
    W_self: List[np.ndarray] = field(default_factory=list)
    W_neigh: List[np.ndarray] = field(default_factory=list)
    bias: List[np.ndarray] = field(default_factory=list)

    def n_draws(self, j: int) -> int:
        return int(self.alpha * self.edges[j][0].size)

    def visible_edges(self, kept: List[tuple]):
        """Edge list of the worker's visible graph: its own partition plus the given sparsified remote edge
        lists (kept[j] = (u, v) for j != worker; entry `worker` is ignored).  Plain concatenation: pairs that
        occur more than once collapse when the CSR is built."""
        us = [self.edges[self.worker][0]] + [kept[j][0] for j in range(self.parts) if j != self.worker]
        vs = [self.edges[self.worker][1]] + [kept[j][1] for j in range(self.parts) if j != self.worker]
        return np.concatenate(us).astype(np.int32), np.concatenate(vs).astype(np.int32)


def make_partitioned(name: str = "C3", with_features: bool = True, scale: float = 1.0, alpha: float = 0.15) -> PartitionedInputs:
    """The graph of workload `name` split over its workers the paper's way (random node partition, halo edges in
    both partitions), with the sparsification left to the code under test."""
    cfg = CONFIGS[name]
    sd = cfg["seeds"]
    n = max(8, int(round(cfg["n_nodes"] * scale)))
    m = max(8, int(round(cfg["m"] * scale)))
    w_max = cfg.get("w_max")
    if w_max is not None and scale != 1.0:
        w_max = max(4.0, w_max * scale)
    u, v = chung_lu_edges(n, m, cfg["gamma"], sd["graph"], sd["perm"], w_max)
    vw = cfg["view"]
    part, edges = partition_edge_lists(u, v, n, vw["parts"], sd["part"])
    own_u, own_v = edges[vw["worker"]]
    n_pos = min(own_u.size, max(1, int(round(cfg["n_pos"] * scale))))
    pick = np.random.default_rng(sd["batch"]).permutation(own_u.size)[:n_pos]
    pin = PartitionedInputs(name=name + "s", n_nodes=n, parts=vw["parts"], worker=vw["worker"], part=part, edges=edges,
                            alpha=alpha, sparsify_seeds=[0x5A000000 + sd["keep"] * 16 + j for j in range(vw["parts"])],
                            dims=list(cfg["dims"]), k_neg=cfg["k_neg"], pos_src=own_u[pick].copy(), pos_dst=own_v[pick].copy(),
                            sampler_seed=0x5EED0000 + sd["batch"], sampler_step=7)
    pin.W_self, pin.W_neigh, pin.bias = init_model(pin.dims, sd["w"])
    if with_features:
        pin.X = init_features(n, pin.dims[0], sd["x"])
    return pin


@dataclass
class Workload:
    name: str
    n_nodes: int                 # nodes visible to the worker (N)
    n_owned: int                 # nodes the worker owns (== n_nodes without a partition)
    src: np.ndarray              # int32 [E], undirected edges, each once
    dst: np.ndarray              # int32 [E]
    dims: List[int]              # F_0 .. F_K
    k_neg: int
    n_space: int                 # negative destinations are drawn from [0, n_space)
    pos_src: np.ndarray          # int32 [n_pos]
    pos_dst: np.ndarray          # int32 [n_pos]
    sampler_seed: int
    sampler_step: int
    dtype: str
    X: Optional[np.ndarray] = None               # float32 [N, F_0]
    W_self: List[np.ndarray] = field(default_factory=list)    # [F_{k-1}, F_k]
    W_neigh: List[np.ndarray] = field(default_factory=list)
    bias: List[np.ndarray] = field(default_factory=list)

    @property
    def n_pos(self) -> int:
        return int(self.pos_src.size)

    @property
    def batch_edges(self) -> int:
        return self.n_pos * (1 + self.k_neg)


def make_workload(name: str, with_features: bool = True, scale: float = 1.0) -> Workload:
    """Build one of the named workloads.  ``scale`` < 1 shrinks node, edge and
    batch counts by that factor (used for bounded CPU timing samples)."""
    cfg = CONFIGS[name]
    sd = cfg["seeds"]
    n = max(8, int(round(cfg["n_nodes"] * scale)))
    m = max(8, int(round(cfg["m"] * scale)))
    if cfg["graph"] == "uniform":
        u, v = uniform_edges(n, m, sd["graph"])
    else:
        w_max = cfg.get("w_max")
        if w_max is not None and scale != 1.0:
            w_max = max(4.0, w_max * scale)
        u, v = chung_lu_edges(n, m, cfg["gamma"], sd["graph"], sd["perm"], w_max)
    n_vis, n_owned = n, n
    if "view" in cfg:
        vw = cfg["view"]
        u, v, n_vis, n_owned, _ = worker_view(u, v, n, vw["parts"], vw["worker"], vw["keep"],
                                              sd["part"], sd["keep"])
    rng = np.random.default_rng(sd["batch"])
    if cfg["n_pos"] is None:
        pick = np.arange(u.size)
    else:
        n_pos = min(u.size, max(1, int(round(cfg["n_pos"] * scale))))
        pick = rng.permutation(u.size)[:n_pos]
    wl = Workload(name=name, n_nodes=n_vis, n_owned=n_owned, src=u, dst=v,
                  dims=list(cfg["dims"]), k_neg=cfg["k_neg"], n_space=n_vis,
                  pos_src=u[pick].copy(), pos_dst=v[pick].copy(),
                  sampler_seed=0x5EED0000 + sd["batch"], sampler_step=7, dtype=cfg["dtype"])
    wl.W_self, wl.W_neigh, wl.bias = init_model(wl.dims, sd["w"])
    if with_features:
        wl.X = init_features(n_vis, wl.dims[0], sd["x"])
    return wl
