"""The entry point that allocates nothing: lp_score_loss_noalloc against lp_score_loss.

Same kernels, scratch in a device array inside the library instead of a caller workspace, so the two must agree
bit for bit.  Two calls in a row, the second with a smaller batch (fewer blocks, so part of the scratch keeps the
first call's partial sums), in fp32 and bf16 storage; the size limit and the argument checks are exercised too.
"""
import ctypes as C

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

import paper_2506_20818_amd as lp
from paper_2506_20818_amd import binding as B_
from gpu_util import DEV, dev_f32, dev_i32, host


def both(H, es, ed, n_pos):
    s0, l0, d0 = lp.lp_score_loss(H, es, ed, n_pos)
    B = es.numel()
    s1 = torch.full((B,), 7.0, dtype=torch.float32, device=DEV)
    d1 = torch.full((B,), 7.0, dtype=torch.float32, device=DEV)
    l1 = torch.full((1,), 7.0, dtype=torch.float32, device=DEV)
    lp.lp_score_loss_noalloc(H, es, ed, n_pos, s1, l1, d1)
    assert host(s1).tobytes() == host(s0).tobytes(), "scores"
    assert host(d1).tobytes() == host(d0).tobytes(), "dscore"
    assert host(l1).tobytes() == host(l0).tobytes(), "loss"
    return float(host(l1)[0])


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_two_calls_in_a_row_second_smaller(dtype):
    print("[case] lp_score_loss_noalloc %s: B=70001 then B=901" % dtype, flush=True)
    rng = np.random.default_rng(11)
    n, F = 5000, 256
    H = dev_f32((rng.standard_normal((n, F)) * F ** -0.25).astype(np.float32)).to(dtype)
    es1, ed1 = dev_i32(rng.integers(0, n, 70001)), dev_i32(rng.integers(0, n, 70001))
    es2, ed2 = dev_i32(rng.integers(0, n, 901)), dev_i32(rng.integers(0, n, 901))
    big = both(H, es1, ed1, 30000)          # 2048 blocks: every entry of the scratch is written
    small = both(H, es2, ed2, 400)          # 15 blocks: the rest of the scratch still holds the first call's sums
    assert np.isfinite(big) and np.isfinite(small) and big != small
    big_again = both(H, es1, ed1, 30000)
    assert big_again == big
    # no dscore wanted, and an empty batch
    s = torch.empty(901, dtype=torch.float32, device=DEV)
    l = torch.empty(1, dtype=torch.float32, device=DEV)
    lp.lp_score_loss_noalloc(H, es2, ed2, 400, s, l, None)
    assert float(host(l)[0]) == small
    z = dev_i32(np.zeros(0, np.int32))
    lp.lp_score_loss_noalloc(H, z, z, 0, s, l, None)
    assert float(host(l)[0]) == 0.0


def test_limits_and_argument_checks():
    print("[case] lp_score_loss_noalloc: size limit and argument checks", flush=True)
    lib = B_.load_library()
    H = dev_f32(np.zeros((4, 8), np.float32))
    e = dev_i32(np.zeros(4, np.int32))
    s = torch.empty(4, dtype=torch.float32, device=DEV)
    l = torch.empty(1, dtype=torch.float32, device=DEV)
    p = lambda t: C.c_void_p(t.data_ptr())
    too_many = (1 << 28) + 1                 # beyond LP_SCORE_LOSS_NOALLOC_MAX_EDGES: rejected before any launch
    assert lib.lp_score_loss_noalloc(p(H), 4, 8, 0, too_many, 0, p(e), p(e), p(s), p(l), None, None, None) == -2
    assert lib.lp_score_loss_noalloc(None, 4, 8, 0, 4, 0, p(e), p(e), p(s), p(l), None, None, None) == -1
    assert lib.lp_score_loss_noalloc(p(H), 4, 6, 0, 4, 0, p(e), p(e), p(s), p(l), None, None, None) == -4
    assert lib.lp_score_loss_noalloc(p(H), 4, 8, 0, 4, 5, p(e), p(e), p(s), p(l), None, None, None) == -1
    assert lib.lp_score_loss_noalloc(p(H), 4, 8, 0, 4, 2, p(e), p(e), p(s), p(l), None, None, None) == 0
    torch.cuda.synchronize()
    assert abs(float(l.item()) - np.log(2.0)) < 1e-6
