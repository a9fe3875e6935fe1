"""GPU parity of lp_sparsify against the sparsifier oracle: the drawn edges and their counts are integer results
and must match bit for bit; the weights (fp32 on the GPU, fp64 in the oracle) within 1e-6 relative."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

import paper_2506_20818_amd as lp
from lp_workloads import make_workload
from oracle import sparsify_oracle as S
from gpu_util import dev_i32, host


def say(msg):
    print("[case] " + msg, flush=True)


def check(n, eu, ev, L, seed):
    got = lp.lp_sparsify(n, dev_i32(eu), dev_i32(ev), L, seed)
    ref = S.sparsify(n, eu, ev, L, seed)
    assert np.array_equal(host(got.kept_edge), ref.kept_edge), "drawn edge set"
    assert np.array_equal(host(got.count), ref.count), "draw counts"
    assert np.array_equal(host(got.kept_u), eu[ref.kept_edge]) and np.array_equal(host(got.kept_v), ev[ref.kept_edge])
    np.testing.assert_allclose(host(got.weight), ref.weight, rtol=1e-6)
    return ref


def distinct_edges(rng, n, m):
    u = rng.integers(0, n, 3 * m)
    v = rng.integers(0, n, 3 * m)
    keep = u != v
    key = np.unique(np.minimum(u, v)[keep].astype(np.int64) * n + np.maximum(u, v)[keep])[:m]
    rng.shuffle(key)
    return (key // n).astype(np.int32), (key % n).astype(np.int32)


@pytest.mark.parametrize("seed", range(4))
def test_sparsify_small_random(seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(2, 4000))
    eu, ev = distinct_edges(rng, n, int(rng.integers(1, 9000)))
    L = int(rng.integers(1, 3 * eu.size + 2))           # from far fewer to more draws than edges
    say("sparsify random seed=%d n=%d m=%d L=%d" % (seed, n, eu.size, L))
    check(n, eu, ev, L, 1000 + seed)


def test_sparsify_edge_cases():
    say("sparsify single edge / star / one draw / huge seed / empty / out of range")
    one = np.array([0], np.int32), np.array([1], np.int32)
    r = check(2, one[0], one[1], 5, 3)
    assert r.kept_edge.tolist() == [0] and r.count.tolist() == [5] and abs(r.weight[0] - 1.0) < 1e-12
    n = 5000                                            # star: one hub of degree n-1, uniform probabilities
    check(n, np.zeros(n - 1, np.int32), np.arange(1, n, dtype=np.int32), 700, 11)
    rng = np.random.default_rng(2)
    eu, ev = distinct_edges(rng, 300, 2100)             # spans several scan tiles with a ragged tail
    check(300, eu, ev, 1, 5)
    check(300, eu, ev, 315, 2 ** 63 + 12345)
    z = np.zeros(0, np.int32)
    got = lp.lp_sparsify(10, dev_i32(z), dev_i32(z), 5, 1)
    assert got.kept_edge.numel() == 0
    got = lp.lp_sparsify(300, dev_i32(eu), dev_i32(ev), 0, 1)
    assert got.kept_edge.numel() == 0
    with pytest.raises(lp.LpError) as ei:
        lp.lp_sparsify(5, dev_i32([0, 1]), dev_i32([1, 5]), 3, 1)
    assert ei.value.status == -2


def test_sparsify_collab_scale_at_the_default_level():
    wl = make_workload("C2", with_features=False)
    L = int(0.15 * wl.src.size)                         # the paper's default sparsification level
    say("sparsify C2 n=%d m=%d L=%d" % (wl.n_nodes, wl.src.size, L))
    r = check(wl.n_nodes, wl.src, wl.dst, L, 42)
    # at level 0.15 at least 85 % of the edges are removed; repeated draws of low-degree edges remove a little more
    assert 0.5 * L < r.kept_edge.size <= L


def test_training_step_on_the_papers_worker_view():
    """One worker the paper's way (Sec. IV-A/B): its own partition in full (halo edges included), every other
    partition sparsified at level 0.15 by lp_sparsify, all nodes visible and in the negative sample space.  The
    sparsified edge lists must equal the oracle's bit for bit; the training step on the assembled graph is then
    compared with the oracle's step on the same graph.  One tenth of the C3 graph (100 000 nodes)."""
    from lp_workloads import Workload, make_partitioned
    from test_gpu_parity import run_whole_step
    pin = make_partitioned("C3", scale=0.1)
    say("paper view: N=%d parts=%d own edges=%d" % (pin.n_nodes, pin.parts, pin.edges[pin.worker][0].size))
    kept = [None] * pin.parts
    for j in range(pin.parts):
        if j == pin.worker:
            continue
        eu, ev = pin.edges[j]
        ref = check(pin.n_nodes, eu, ev, pin.n_draws(j), pin.sparsify_seeds[j])
        got = lp.lp_sparsify(pin.n_nodes, dev_i32(eu), dev_i32(ev), pin.n_draws(j), pin.sparsify_seeds[j])
        kept[j] = (host(got.kept_u), host(got.kept_v))           # the HIP path's own output feeds the HIP step
        assert np.array_equal(kept[j][0], eu[ref.kept_edge]) and np.array_equal(kept[j][1], ev[ref.kept_edge])
    u, v = pin.visible_edges(kept)
    wl = Workload(name=pin.name, n_nodes=pin.n_nodes, n_owned=int((pin.part == pin.worker).sum()), src=u, dst=v,
                  dims=pin.dims, k_neg=pin.k_neg, n_space=pin.n_nodes, pos_src=pin.pos_src, pos_dst=pin.pos_dst,
                  sampler_seed=pin.sampler_seed, sampler_step=pin.sampler_step, dtype="f32", X=pin.X,
                  W_self=pin.W_self, W_neigh=pin.W_neigh, bias=pin.bias)
    run_whole_step(wl)
