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
