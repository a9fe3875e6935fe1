"""The training step under HIP graph capture: the library allocates nothing, clears its scratch with kernels and keeps
no state between calls, so a step recorded once can be replayed.  Every replay must reproduce the eager result bit
for bit, also when other eager work and synchronisations run between the replays."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

import paper_2506_20818_amd as lp
from paper_2506_20818_amd import binding as B
from lp_workloads import make_workload
from gpu_util import DEV, dev_f32, dev_i32, make_model


def say(msg):
    print("[case] " + msg, flush=True)


class StepBuffers:
    """All outputs and workspaces of one step, allocated up front (graph capture must not allocate)."""

    def __init__(self, g, model, n_pos, k_neg, want_dX):
        Bn = n_pos * (1 + k_neg)
        u8 = lambda n: torch.empty(max(int(n), 16), dtype=torch.uint8, device=DEV)
        self.e_src = torch.zeros(Bn, dtype=torch.int32, device=DEV)
        self.e_dst = torch.zeros(Bn, dtype=torch.int32, device=DEV)
        self.acts = lp.Acts(g.n_nodes, model.dims, DEV, model.torch_dtype)
        for t in self.acts.A + self.acts.H:   # rows of the last layer that the training forward leaves alone compare equal
            t.zero_()
        self.grads = lp.Grads(g.n_nodes, model.dims, DEV, want_dX, model.torch_dtype)
        self.scores = torch.zeros(Bn, dtype=torch.float32, device=DEV)
        self.dscore = torch.zeros(Bn, dtype=torch.float32, device=DEV)
        self.loss = torch.zeros(1, dtype=torch.float32, device=DEV)
        self.ws_f = u8(B.forward_edges_workspace_bytes(model, g.n_nodes, Bn))
        self.ws_b = u8(B.backward_workspace_bytes(model, g.n_nodes, Bn))
        self.ws_l = u8(1 << 16)

    def tensors(self, K):
        out = [self.e_dst, self.scores, self.loss, self.dscore] + [self.acts.H[k] for k in range(K)]
        out += [self.grads.dW_self[k] for k in range(K)] + [self.grads.dW_neigh[k] for k in range(K)] + [self.grads.dbias[k] for k in range(K)]
        return out


def run_step(g, model, X, pos_src, pos_dst, k_neg, n_space, seed, step, buf):
    n_pos = int(pos_src.numel())
    buf.e_src[:n_pos].copy_(pos_src)
    buf.e_dst[:n_pos].copy_(pos_dst)
    lp.lp_sample_neg(g, pos_src, k_neg, n_space, seed, step, neg_dst=buf.e_dst[n_pos:], neg_src=buf.e_src[n_pos:])
    lp.lp_sage_forward_edges(g, model, X, buf.e_src, buf.e_dst, buf.acts, buf.ws_f)
    lp.lp_score_loss(buf.acts.H[-1], buf.e_src, buf.e_dst, n_pos, buf.scores, buf.loss, buf.dscore, buf.ws_l)
    lp.lp_backward(g, model, X, buf.acts, buf.e_src, buf.e_dst, buf.dscore, buf.grads, buf.ws_b)


@pytest.mark.parametrize("name,n_pos", [("C1", None), ("C2", None), ("C2", 8192)])
def test_captured_step_replays_bit_exactly(name, n_pos):
    """n_pos = 8192 of C2's positives: a batch small enough for the training forward to list the rows of its last layer
    (flags, prefix sums and row copies inside the captured graph, the number of listed rows read on the device)."""
    wl = make_workload(name)
    if n_pos is not None:
        wl.pos_src, wl.pos_dst = wl.pos_src[:n_pos], wl.pos_dst[:n_pos]
    n_pos = int(wl.pos_src.size)
    say("graph capture of the training step, %s, %d positives" % (name, n_pos))
    g = lp.lp_build_csr(wl.n_nodes, dev_i32(wl.src), dev_i32(wl.dst), True)
    model = make_model(wl.W_self, wl.W_neigh, wl.bias)
    X = dev_f32(wl.X)
    pos_src, pos_dst = dev_i32(wl.pos_src), dev_i32(wl.pos_dst)
    K = len(wl.dims) - 1
    eager = StepBuffers(g, model, n_pos, wl.k_neg, False)
    other = StepBuffers(g, model, n_pos, wl.k_neg, False)
    cap = StepBuffers(g, model, n_pos, wl.k_neg, False)
    run_step(g, model, X, pos_src, pos_dst, wl.k_neg, wl.n_space, wl.sampler_seed, 7, eager)
    torch.cuda.synchronize()
    expected = [t.clone() for t in eager.tensors(K)]

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                       # one eager pass on the capture stream first
        run_step(g, model, X, pos_src, pos_dst, wl.k_neg, wl.n_space, wl.sampler_seed, 7, cap)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        run_step(g, model, X, pos_src, pos_dst, wl.k_neg, wl.n_space, wl.sampler_seed, 7, cap)
    for replay in range(3):
        for t in cap.tensors(K):
            t.zero_()
        run_step(g, model, X, pos_src, pos_dst, wl.k_neg, wl.n_space, wl.sampler_seed, 100 + replay, other)   # eager work in between
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for i, (got, exp) in enumerate(zip(cap.tensors(K), expected)):
            assert torch.equal(got, exp), "replay %d: output %d differs from the eager step" % (replay, i)


def run_sampled_step(g, model, X, pos_src, pos_dst, k_neg, n_space, seed, step, fanout, buf):
    n_pos = int(pos_src.numel())
    buf["e_src"][:n_pos].copy_(pos_src)
    buf["e_dst"][:n_pos].copy_(pos_dst)
    lp.lp_sample_neg(g, pos_src, k_neg, n_space, seed, step, neg_dst=buf["e_dst"][n_pos:], neg_src=buf["e_src"][n_pos:])
    lp.lp_sample_blocks(g, buf["e_src"], buf["e_dst"], fanout, seed + 1, step, buf["blocks"])
    lp.lp_sage_forward_blocks(buf["blocks"], model, X, buf["acts"], buf["ws_f"])
    lp.lp_score_loss(buf["acts"].H[-1], buf["blocks"].e_src_pos, buf["blocks"].e_dst_pos, n_pos, buf["scores"], buf["loss"],
                     buf["dscore"], buf["ws_l"])
    lp.lp_backward_blocks(buf["blocks"], model, buf["acts"], buf["dscore"], buf["grads"], buf["ws_b"])


def sampled_buffers(g, model, Bn, fanout, dims):
    u8 = lambda n: torch.empty(max(int(n), 16), dtype=torch.uint8, device=DEV)
    blocks = lp.Blocks(g, Bn, fanout)
    return {"e_src": torch.zeros(Bn, dtype=torch.int32, device=DEV), "e_dst": torch.zeros(Bn, dtype=torch.int32, device=DEV),
            "blocks": blocks, "acts": lp.BlockActs(blocks, dims, DEV, model.torch_dtype),
            "grads": lp.Grads(1, dims, DEV, dtype=model.torch_dtype),
            "scores": torch.zeros(Bn, dtype=torch.float32, device=DEV), "dscore": torch.zeros(Bn, dtype=torch.float32, device=DEV),
            "loss": torch.zeros(1, dtype=torch.float32, device=DEV),
            "ws_f": u8(B.forward_blocks_workspace_bytes(model, blocks)), "ws_b": u8(B.backward_blocks_workspace_bytes(model, blocks)),
            "ws_l": u8(1 << 16)}


def sampled_outputs(buf, K):
    out = [buf["e_dst"], buf["blocks"].n, buf["blocks"].nodes, buf["scores"], buf["loss"], buf["dscore"]]
    out += [buf["grads"].dW_self[k] for k in range(K)] + [buf["grads"].dW_neigh[k] for k in range(K)] + [buf["grads"].dbias[k] for k in range(K)]
    return out


def test_captured_sampled_step_replays_bit_exactly():
    """The mini-batch mode (negatives, sampled blocks with device-side frontier sizes, forward, loss, backward) recorded
    as one HIP graph: grids are sized by host-side bounds and every count stays on the device, so the recording does not
    depend on the batch; three replays with eager work of other batches in between equal the eager step bit for bit."""
    wl = make_workload("C2")
    say("graph capture of the sampled-neighbourhood step, C2 graph")
    g = lp.lp_build_csr(wl.n_nodes, dev_i32(wl.src), dev_i32(wl.dst), True)
    model = make_model(wl.W_self, wl.W_neigh, wl.bias)
    X = dev_f32(wl.X)
    n_pos, fanout = 4096, [25, 10, 5]
    pos_src, pos_dst = dev_i32(wl.pos_src[:n_pos]), dev_i32(wl.pos_dst[:n_pos])
    Bn, K = n_pos * (1 + wl.k_neg), len(wl.dims) - 1
    eager, other, cap = (sampled_buffers(g, model, Bn, fanout, wl.dims) for _ in range(3))
    args = (g, model, X, pos_src, pos_dst, wl.k_neg, wl.n_space, wl.sampler_seed)
    run_sampled_step(*args, 7, fanout, eager)
    torch.cuda.synchronize()
    n_front = int(eager["blocks"].n[0].item())
    expected = [t.clone() for t in sampled_outputs(eager, K)]

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run_sampled_step(*args, 7, fanout, cap)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        run_sampled_step(*args, 7, fanout, cap)
    for replay in range(3):
        for t in sampled_outputs(cap, K):
            t.zero_()
        run_sampled_step(*args, 200 + replay, fanout, other)      # eager work of another batch in between
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for i, (got, exp) in enumerate(zip(sampled_outputs(cap, K), expected)):
            if i == 2:      # frontier node list: entries past the realised frontier size are unspecified
                got, exp = got[:n_front], exp[:n_front]
            assert torch.equal(got, exp), "replay %d: output %d differs from the eager step" % (replay, i)
