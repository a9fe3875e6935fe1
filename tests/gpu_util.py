"""Helpers for the GPU parity tests: run the HIP path through the C ABI and compare with the oracle."""
import numpy as np
import torch

import paper_2506_20818_amd as lp

DEV = "cuda:0"


def dev_i32(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(DEV)


def dev_f32(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(DEV)


def host(t):
    torch.cuda.synchronize()
    return t.detach().cpu().numpy()


def rel_err(got, ref):
    """Per-tensor relative errors: max-norm and 2-norm (per-element ratios are meaningless near zero)."""
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    if ref.size == 0:
        return 0.0, 0.0
    d = np.abs(got - ref)
    m = np.abs(ref).max()
    l2 = np.sqrt((ref * ref).sum())
    e_max = d.max() / m if m > 0 else d.max()
    e_l2 = np.sqrt((d * d).sum()) / l2 if l2 > 0 else np.sqrt((d * d).sum())
    return float(e_max), float(e_l2)


def assert_close(got, ref, tol, what):
    assert np.all(np.isfinite(got)), what + ": non-finite values"
    e_max, e_l2 = rel_err(got, ref)
    assert e_max <= tol and e_l2 <= tol, "%s: max-norm rel %.3e, 2-norm rel %.3e > %.1e" % (what, e_max, e_l2, tol)


def make_model(W_self, W_neigh, bias, products=lp.LP_FP32_PRODUCTS_BF16X6):
    return lp.Model([dev_f32(w) for w in W_self], [dev_f32(w) for w in W_neigh], [dev_f32(b) for b in bias],
                    fp32_products=products)


def nan_filled_acts(n_nodes, model, X):
    acts = lp.Acts(n_nodes, model.dims, X.device, model.torch_dtype)
    for t in acts.A + acts.H:
        t.fill_(float("nan"))
    return acts


class HipStep:
    """One training step through the five C-ABI calls, keeping every intermediate for comparison."""

    def __init__(self, g, model, X, pos_src, pos_dst, k_neg, n_space, seed, step, want_dX=True, forward="all"):
        n_pos = int(pos_src.numel())
        B = n_pos * (1 + k_neg)
        self.e_src = torch.empty(B, dtype=torch.int32, device=DEV)
        self.e_dst = torch.empty(B, dtype=torch.int32, device=DEV)
        self.e_src[:n_pos] = pos_src          # marshalling: positives first
        self.e_dst[:n_pos] = pos_dst
        self.n_failed = torch.zeros(1, dtype=torch.int32, device=DEV)
        lp.lp_sample_neg(g, pos_src, k_neg, n_space, seed, step, neg_dst=self.e_dst[n_pos:], neg_src=self.e_src[n_pos:],
                         n_failed=self.n_failed)
        if forward == "edges":   # the training forward: rows of the last layer that it must not touch hold NaN
            self.acts = nan_filled_acts(g.n_nodes, model, X)
            lp.lp_sage_forward_edges(g, model, X, self.e_src, self.e_dst, self.acts)
        else:
            self.acts = lp.lp_sage_forward(g, model, X)
        self.scores, self.loss, self.dscore = lp.lp_score_loss(self.acts.H[-1], self.e_src, self.e_dst, n_pos)
        self.grads = lp.lp_backward(g, model, X, self.acts, self.e_src, self.e_dst, self.dscore, want_dX=want_dX)
        torch.cuda.synchronize()
