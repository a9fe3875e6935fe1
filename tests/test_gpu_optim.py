"""GPU parity of lp_sgd_step / lp_adam_step with the optimizer oracle (fp32 on the GPU, fp64 in the oracle)."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

import paper_2506_20818_amd as lp
from oracle import optim_oracle as P
from gpu_util import DEV, assert_close, dev_f32, host


def say(msg):
    print("[case] " + msg, flush=True)


def setup(dims, bf16, seed):
    rng = np.random.default_rng(seed)
    K = len(dims) - 1
    tdt = torch.bfloat16 if bf16 else torch.float32
    Ws = [rng.standard_normal((dims[k], dims[k + 1])).astype(np.float32) for k in range(K)]
    Wn = [rng.standard_normal((dims[k], dims[k + 1])).astype(np.float32) for k in range(K)]
    b = [rng.standard_normal(dims[k + 1]).astype(np.float32) for k in range(K)]
    model = lp.Model([dev_f32(w).to(tdt) for w in Ws], [dev_f32(w).to(tdt) for w in Wn], [dev_f32(x) for x in b])
    # the oracle starts from what the device holds (bf16-rounded where stored as bf16)
    ref = {"W_self": [host(t.float()).astype(np.float64) for t in model.W_self],
           "W_neigh": [host(t.float()).astype(np.float64) for t in model.W_neigh],
           "bias": [host(t).astype(np.float64) for t in model.bias]}
    grads = lp.Grads(8, dims, DEV)
    return rng, model, ref, grads


def new_gradients(rng, grads, scale):
    out = {}
    for name, key in (("dW_self", "W_self"), ("dW_neigh", "W_neigh"), ("dbias", "bias")):
        out[key] = []
        for t in getattr(grads, name):
            g = (rng.standard_normal(tuple(t.shape)) * scale).astype(np.float32)
            g.flat[0] = 0.0                                   # an exactly zero gradient entry
            t.copy_(dev_f32(g))
            out[key].append(g.astype(np.float64))
    return out


def compare(model, ref, before, tol_update, bf16):
    for key in ("W_self", "W_neigh", "bias"):
        for k, t in enumerate(getattr(model, key)):
            got = host(t.float()).astype(np.float64)
            exp = ref[key][k]
            if bf16 and key != "bias":
                # stored as bfloat16: equal up to one rounding step where fp32 and fp64 sit on different sides of a tie
                assert np.all(np.abs(got - exp) <= np.abs(exp) * 2.0 ** -7), key
            else:
                # the update itself to tol_update of its size, plus one fp32 rounding of the stored weight
                upd_got, upd_exp = got - before[key][k], exp - before[key][k]
                err = np.abs(upd_got - upd_exp).max()
                bound = tol_update * np.abs(upd_exp).max() + 2.0 ** -23 * np.abs(exp).max()
                assert err <= bound, "%s[%d]: update error %.3e > %.3e" % (key, k, err, bound)


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("dims", [[8, 16, 8], [128, 256, 256, 256], [100, 132, 68]])
def test_adam_steps_match_oracle(dims, bf16):
    if bf16 and any(d % 8 for d in dims):
        pytest.skip("bf16 layers are multiples of 8 wide")
    say("adam dims=%s bf16=%s" % (dims, bf16))
    rng, model, ref, grads = setup(dims, bf16, 5 + len(dims))
    state = lp.AdamState(model)
    mom = {k: [np.zeros_like(x) for x in v] for k, v in ref.items()}
    vel = {k: [np.zeros_like(x) for x in v] for k, v in ref.items()}
    storage = "bf16" if bf16 else "f32"
    for t in range(1, 5):
        g = new_gradients(rng, grads, 10.0 ** (-t))
        before = {k: [x.copy() for x in v] for k, v in ref.items()}
        lp.lp_adam_step(model, grads, state, t, lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8)
        # the C ABI takes the hyper-parameters as floats: the oracle gets those same (float32-representable) numbers
        hp = dict(lr=float(np.float32(1e-3)), beta1=float(np.float32(0.9)), beta2=float(np.float32(0.999)),
                  eps=float(np.float32(1e-8)))
        for key in ref:
            for k in range(len(ref[key])):
                ref[key][k], mom[key][k], vel[key][k] = P.adam_step(
                    ref[key][k], g[key][k], mom[key][k], vel[key][k], t, storage="f32" if key == "bias" else storage, **hp)
        compare(model, ref, before, 1e-4, bf16)
        if bf16:                                              # keep both sides on the same stored weights
            for key in ("W_self", "W_neigh"):
                ref[key] = [host(x.float()).astype(np.float64) for x in getattr(model, key)]
    # per tensor, not per entry: a moment entry can be the small difference of two larger terms
    assert_close(host(state.m_W_self[0]), mom["W_self"][0], 1e-5, "first moment")
    assert_close(host(state.v_bias[-1]), vel["bias"][-1], 1e-5, "second moment")


@pytest.mark.parametrize("bf16", [False, True])
def test_sgd_step_matches_oracle(bf16):
    dims = [64, 128, 8]
    say("sgd dims=%s bf16=%s" % (dims, bf16))
    rng, model, ref, grads = setup(dims, bf16, 9)
    g = new_gradients(rng, grads, 0.5)
    before = {k: [x.copy() for x in v] for k, v in ref.items()}
    lp.lp_sgd_step(model, grads, 0.05)
    for key in ref:
        for k in range(len(ref[key])):
            ref[key][k] = P.sgd_step(ref[key][k], g[key][k], float(np.float32(0.05)), storage="bf16" if (bf16 and key != "bias") else "f32")
    compare(model, ref, before, 1e-6, bf16)


@pytest.mark.parametrize("bf16", [False, True])
def test_single_tensor_updates_match_oracle(bf16):
    say("adam/sgd single tensor bf16=%s" % bf16)
    rng = np.random.default_rng(21)
    tdt = torch.bfloat16 if bf16 else torch.float32
    w = dev_f32(rng.standard_normal((33, 8))).to(tdt)
    ref = host(w.float()).astype(np.float64)
    m, v = torch.zeros(33, 8, device=DEV), torch.zeros(33, 8, device=DEV)
    rm, rv = np.zeros_like(ref), np.zeros_like(ref)
    hp = dict(lr=float(np.float32(1e-2)), beta1=float(np.float32(0.9)), beta2=float(np.float32(0.999)), eps=float(np.float32(1e-8)))
    for t in range(1, 4):
        g = rng.standard_normal((33, 8)).astype(np.float32)
        lp.lp_adam_update_tensor(w, dev_f32(g), m, v, t, lr=1e-2)
        ref, rm, rv = P.adam_step(ref, g.astype(np.float64), rm, rv, t, storage="bf16" if bf16 else "f32", **hp)
        got = host(w.float()).astype(np.float64)
        assert np.all(np.abs(got - ref) <= np.abs(ref) * (2.0 ** -7 if bf16 else 2e-6) + 1e-7)
        ref = got.copy()
    g = rng.standard_normal((33, 8)).astype(np.float32)
    lp.lp_sgd_update_tensor(w, dev_f32(g), 0.05)
    ref = P.sgd_step(ref, g.astype(np.float64), float(np.float32(0.05)), storage="bf16" if bf16 else "f32")
    assert np.all(np.abs(host(w.float()) - ref) <= np.abs(ref) * (2.0 ** -7 if bf16 else 2e-6) + 1e-7)


def test_training_loop_follows_the_oracle_for_several_steps():
    """Algorithm 1's per-worker loop on a small graph: negatives (new Philox step each iteration), training forward, loss,
    backward, Adam update, five times, on the GPU and in the oracle (its own Adam on its own gradients).  The loss
    trajectories stay together, the loss goes down, and the accumulated weight change agrees per tensor."""
    from oracle import lp_oracle as O
    from gpu_util import HipStep, dev_i32, make_model
    rng = np.random.default_rng(2024)
    n, dims = 900, [16, 32, 24]
    K = len(dims) - 1
    src, dst = rng.integers(0, n, 3000).astype(np.int32), rng.integers(0, n, 3000).astype(np.int32)
    ref_csr = O.build_csr(n, src, dst, True)
    g = lp.lp_build_csr(n, dev_i32(src), dev_i32(dst), True)
    X = rng.standard_normal((n, dims[0])).astype(np.float32)
    Ws = [(rng.standard_normal((dims[k], dims[k + 1])) * 0.3).astype(np.float32) for k in range(K)]
    Wn = [(rng.standard_normal((dims[k], dims[k + 1])) * 0.3).astype(np.float32) for k in range(K)]
    b = [(rng.standard_normal(dims[k + 1]) * 0.1).astype(np.float32) for k in range(K)]
    pick = rng.choice(src.size, 70, replace=False)       # 210 scored edges: the training forward lists its last layer's rows
    pos_src, pos_dst = src[pick], dst[pick]
    model = make_model(Ws, Wn, b)
    state = lp.AdamState(model)
    Xd = dev_f32(X)
    ref = {"W_self": [w.astype(np.float64) for w in Ws], "W_neigh": [w.astype(np.float64) for w in Wn], "bias": [x.astype(np.float64) for x in b]}
    start = {k: [x.copy() for x in v] for k, v in ref.items()}
    mom = {k: [np.zeros_like(x) for x in v] for k, v in ref.items()}
    vel = {k: [np.zeros_like(x) for x in v] for k, v in ref.items()}
    hp = dict(lr=float(np.float32(1e-2)), beta1=float(np.float32(0.9)), beta2=float(np.float32(0.999)), eps=float(np.float32(1e-8)))
    losses_gpu, losses_ref = [], []
    for t in range(1, 6):
        say("training loop iteration %d" % t)
        got = HipStep(g, model, Xd, dev_i32(pos_src), dev_i32(pos_dst), 2, n, 99, t, want_dX=False, forward="edges")
        lp.lp_adam_step(model, got.grads, state, t, lr=1e-2, beta1=0.9, beta2=0.999, eps=1e-8)
        exp = O.train_step(ref_csr, ref["W_self"], ref["W_neigh"], ref["bias"], X, pos_src, pos_dst, 2, n, 99, t)
        assert np.array_equal(host(got.e_dst), exp.e_dst)                     # same negatives at every step
        losses_gpu.append(float(host(got.loss)[0]))
        losses_ref.append(float(exp.loss))
        gr = {"W_self": exp.grads.dW_self, "W_neigh": exp.grads.dW_neigh, "bias": exp.grads.dbias}
        for key in ref:
            for k in range(K):
                ref[key][k], mom[key][k], vel[key][k] = P.adam_step(ref[key][k], gr[key][k], mom[key][k], vel[key][k], t, **hp)
    torch.cuda.synchronize()
    assert np.allclose(losses_gpu, losses_ref, rtol=1e-3, atol=0), (losses_gpu, losses_ref)
    assert losses_ref[-1] < losses_ref[0] and losses_gpu[-1] < losses_gpu[0]
    for key in ("W_self", "W_neigh", "bias"):
        for k, tns in enumerate(getattr(model, key)):
            moved_gpu = host(tns.float()).astype(np.float64) - start[key][k]
            moved_ref = ref[key][k] - start[key][k]
            rel = np.linalg.norm(moved_gpu - moved_ref) / np.linalg.norm(moved_ref)
            assert rel < 2e-2, "%s[%d]: accumulated update differs by %.3e (relative L2)" % (key, k, rel)
