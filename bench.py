#!/usr/bin/env python3
"""Benchmark: one worker's link-prediction training step on one MI355X.

A step is one pass of the whole hot path over one minibatch: lp_sample_neg -> lp_sage_forward_edges (full-neighbour
layers over all visible nodes; the last layer at the end points of the scored edges, the only rows the loss reads) ->
lp_score_loss -> lp_backward, with every input already resident in HBM.  The workload is
by default the largest single-GPU configuration ("C4", the one the aggregation's HBM target is judged on): a power-law
graph with the paper's largest edge count, 2.9 M nodes, ~29 M directed CSR entries (feature matrices of 1.5-3 GB, far
beyond the 256 MB Infinity Cache), 128 -> 256 -> 256 -> 256 GraphSAGE-mean in fp32, 131 072 positives + 131 072
negatives per step; --workload selects the other configurations (C1, C2, C3, C5_keep1, C5_keep0.5, C5_keep0.2).
Run without --workload, the Collab-scale configuration C2 is measured after it and reported under "also" in the same
line.  Prints ONE JSON line.

The per-kernel numbers in "roofline" come from HIP events recorded by the library around each launch inside the
timed region (lp_timing_enable); "cpu_baseline" times the CPU oracle, as it stands, on a stated fraction of the
same workload.
"""
import argparse
import ctypes as C
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
MFMA_FP32_PEAK_TFLOPS = 157.3  # MI355X dense fp32 matrix


BF16_MFMA_PEAK_TFLOPS = 2500.0 # MI355X dense bf16 matrix
INFINITY_CACHE_BYTES = 256 << 20   # MI355X last-level cache in front of HBM

# fraction of each workload that the CPU oracle is timed on by default (about 10-30 s of host work)
CPU_SCALE = {"C1": 1.0, "C2": 1.0, "C3": 0.5, "C4": 0.2, "C5_keep1": 0.1, "C5_keep0.5": 0.1, "C5_keep0.2": 0.15}


def spmm_bytes(n, nnz, F, backward, eb=4):
    """Algorithmic bytes of one CSR aggregation launch: gathered rows + column ids + row pointers + output row,
    plus inverse degrees (forward) or the added/gating rows (backward).  eb = bytes per stored element."""
    b = nnz * (eb * F + 4) + (n + 1) * 4 + n * eb * F
    return b + (2 * n * eb * F if backward else n * 4)


def spmm_bytes_listed(n, nnz, F, n_t, nnz_t, eb=4):
    """The transposed aggregation of the last layer: its input has rows only for the n_t nodes that are an endpoint
    of a scored edge, so of the nnz entries only the nnz_t that point at such a node gather a row; every entry still
    reads its column id and its 4-byte slot of the node -> row table."""
    return nnz * 8 + nnz_t * eb * F + (n + 1) * 4 + n * 4 + 2 * n * eb * F + n_t * eb * F


def fp32_products_name(bf16, split):
    if bf16:
        return None
    return "bf16x6 (three bfloat16 terms per value, six term products, fp32 accumulation)" if split else "fp32 matrix instructions"


def spmm_bytes_rows(n_t, nnz_t, F, eb=4):
    """The last layer's forward aggregation: only the n_t rows of the end points of the scored edges (nnz_t entries
    in all): their list, row pointers, inverse degrees, column ids, gathered rows and output rows."""
    return n_t * 4 + 2 * n_t * 4 + n_t * 4 + nnz_t * (eb * F + 4) + n_t * eb * F


def lists_last_layer(n, B):
    """lp_sage_forward_edges evaluates its last layer only for the end points of the batch when 8 B < 3 N."""
    return 8 * B < 3 * n


def step_counts(n, nnz, dims, n_t, nnz_t, B, eb=4, paths=2):
    """(spmm algorithmic bytes, NT flops, TN flops) of one step.  The last layer's backward pass runs over the n_t end
    points of the scored edges only (every other row of dL/dH^K is exactly zero); so does its forward pass when the
    library lists them (no other row of h^(K) is read by the loss).  paths: weight matrices per layer (2 for
    GraphSAGE's self and neighbour paths, 1 for GCN)."""
    K = len(dims) - 1
    listed = lists_last_layer(n, B)
    sp = sum(spmm_bytes(n, nnz, dims[k - 1], False, eb) for k in range(1, K))
    sp += spmm_bytes_rows(n_t, nnz_t, dims[K - 1], eb) if listed else spmm_bytes(n, nnz, dims[K - 1], False, eb)
    for k in range(2, K):   # adjoint of layer k's aggregation, every row
        if paths == 2 and eb == 4 and dims[k] <= dims[k - 1]:
            # fp32 GraphSAGE layers that do not widen: dZ is aggregated before the product (entries weighted by a
            # per-node scale, 4 more bytes per entry), and the product adds the self path and applies the gate
            sp += nnz * (eb * dims[k] + 8) + (n + 1) * 4 + n * eb * dims[k]
        else:
            sp += spmm_bytes(n, nnz, dims[k - 1], True, eb)
    if K >= 2:
        sp += spmm_bytes_listed(n, nnz, dims[K - 1], n_t, nnz_t, eb)
    rows = lambda k: n_t if k == K else n
    frows = lambda k: n_t if (k == K and listed) else n
    nt = sum(2.0 * frows(k) * dims[k] * paths * dims[k - 1] for k in range(1, K + 1))     # forward
    nt += sum(2.0 * rows(k) * paths * dims[k - 1] * dims[k] for k in range(2, K + 1))     # input gradients
    tn = sum(2.0 * paths * rows(k) * dims[k - 1] * dims[k] for k in range(1, K + 1))      # dW_self, dW_neigh
    return sp, nt, tn


def cpu_baseline(workload, scale):
    """Time the CPU oracle, as it stands, on a `scale` fraction of `workload` (nodes, edges and batch all scaled by
    the same factor through the workload's own generator)."""
    from lp_workloads import make_workload, to_bf16_grid
    from oracle import lp_oracle as O
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    wl = make_workload(workload, scale=scale)
    storage = "bf16" if wl.dtype == "bf16" else "f32"
    if storage == "bf16":
        wl.X = to_bf16_grid(wl.X)
        wl.W_self, wl.W_neigh = [to_bf16_grid(w) for w in wl.W_self], [to_bf16_grid(w) for w in wl.W_neigh]
    g = O.build_csr(wl.n_nodes, wl.src, wl.dst, True)
    t0 = time.perf_counter()
    O.train_step(g, wl.W_self, wl.W_neigh, wl.bias, wl.X, wl.pos_src, wl.pos_dst, wl.k_neg, wl.n_space,
                 wl.sampler_seed, wl.sampler_step, storage=storage)
    dt = time.perf_counter() - t0
    return {"value": wl.batch_edges / dt, "unit": "edges/s", "cores": int(cores), "kind": "oracle",
            "seconds": round(dt, 3), "scale": scale,
            "sample": "one full oracle step (numpy fp64%s) on the %s generator at scale %.3g: %d nodes, %d directed "
                      "entries, %d scored edges; the dense products run on %d BLAS threads, the aggregation and its "
                      "adjoint are single-threaded loops over the rows"
                      % (", stored matrices rounded to bf16" if storage == "bf16" else "", workload, scale, wl.n_nodes,
                         g.nnz, wl.batch_edges, int(cores))}


def sparsify_task(args):
    """Second measurement: the sparsification pass of Algorithm 1 over all partitions of a partitioned graph
    (the paper's Table II times this step).  One "step" = sparsify every partition once at level alpha."""
    import numpy as np
    import torch

    import paper_2506_20818_amd as lp
    from paper_2506_20818_amd import binding as B
    from lp_workloads import make_partitioned

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    name = args.workload if args.workload in ("C3", "C5_keep1") else "C3"
    pin = make_partitioned(name, with_features=False, alpha=args.alpha)
    i32 = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(dev)
    parts = [(i32(u), i32(v)) for u, v in pin.edges]
    ws = [torch.empty(B.sparsify_workspace_bytes(pin.n_nodes, int(u.numel())), dtype=torch.uint8, device=dev) for u, _ in parts]
    total_edges = sum(int(u.numel()) for u, _ in parts)

    def step():
        kept = 0
        for j, (u, v) in enumerate(parts):
            kept += int(lp.lp_sparsify(pin.n_nodes, u, v, pin.n_draws(j), pin.sparsify_seeds[j], ws[j]).kept_edge.numel())
        return kept

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        kept = step()
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / max(args.steps, 1)
    # algorithmic traffic of one partition: edge list read twice (degrees, weights) + random degree reads, weights
    # written and scanned (8 B each way twice), ~log2(m) 8-byte probes per draw, counts zeroed/read, output
    out = {"metric": "sparsification pass over all partitions (Algorithm 1, sparsification loop): input edges/s",
           "value": round(total_edges / dt, 1), "unit": "edges/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
           "ms_per_step": round(dt * 1e3, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "u64", "data": "synthetic",
           "config": {"workload": "%s graph, %d nodes, %d-way random node partition with halo edges in both partitions, "
                                  "%d edges summed over partitions, level alpha=%.2f" % (name, pin.n_nodes, pin.parts, total_edges, pin.alpha),
                      "kept_edges": kept, "kept_fraction": round(kept / total_edges, 4)}}
    if not args.no_cpu_baseline:
        from oracle import sparsify_oracle as S
        t0 = time.perf_counter()
        j = 0
        r = S.sparsify(pin.n_nodes, pin.edges[j][0], pin.edges[j][1], pin.n_draws(j), pin.sparsify_seeds[j])
        cdt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": round(pin.edges[j][0].size / cdt, 1), "unit": "edges/s", "cores": 1, "kind": "oracle",
                               "seconds": round(cdt, 3),
                               "sample": "the numpy oracle on partition 0 only (%d edges, %d draws)" % (pin.edges[j][0].size, pin.n_draws(j))}
    print(json.dumps(out), flush=True)


def sampled_step_task(args):
    """Third measurement: the paper's own mini-batch mode.  One step = negatives, sampled computational graph
    (fan-outs 25/10/5), forward, loss, backward and an Adam update, for one batch of --n-pos positives."""
    import numpy as np
    import torch

    import paper_2506_20818_amd as lp
    from paper_2506_20818_amd import binding as B
    from lp_workloads import make_workload

    products = lp.LP_FP32_PRODUCTS_NATIVE if args.fp32_products == "native" else lp.LP_FP32_PRODUCTS_BF16X6
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    wl = make_workload(args.workload)
    i32 = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(dev)
    f32 = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(dev)
    g = lp.lp_build_csr(wl.n_nodes, i32(wl.src), i32(wl.dst), True)
    bf16 = wl.dtype == "bf16"
    split = (not bf16) and products == lp.LP_FP32_PRODUCTS_BF16X6
    tdt = torch.bfloat16 if bf16 else torch.float32
    st = (lambda a: f32(a).to(torch.bfloat16)) if bf16 else f32
    model = lp.Model([st(w) for w in wl.W_self], [st(w) for w in wl.W_neigh], [f32(b) for b in wl.bias], fp32_products=products)
    X = st(wl.X)
    n_pos = min(args.n_pos, wl.n_pos)
    k_neg = wl.k_neg
    Bn = n_pos * (1 + k_neg)
    fanout = [int(x) for x in args.fanout.split(",")]
    pos_src = i32(wl.pos_src[:n_pos])
    e_src = torch.empty(Bn, dtype=torch.int32, device=dev)
    e_dst = torch.empty(Bn, dtype=torch.int32, device=dev)
    e_src[:n_pos] = pos_src
    e_dst[:n_pos] = i32(wl.pos_dst[:n_pos])
    neg_src, neg_dst = e_src[n_pos:], e_dst[n_pos:]
    blocks = lp.Blocks(g, Bn, fanout)
    acts = lp.BlockActs(blocks, wl.dims, dev, tdt)
    grads = lp.Grads(1, wl.dims, dev, dtype=tdt)
    adam = lp.AdamState(model)
    ws_f = torch.empty(B.forward_blocks_workspace_bytes(model, blocks), dtype=torch.uint8, device=dev)
    ws_b = torch.empty(B.backward_blocks_workspace_bytes(model, blocks), dtype=torch.uint8, device=dev)
    ws_l = torch.empty(1 << 16, dtype=torch.uint8, device=dev)
    scores = torch.empty(Bn, dtype=torch.float32, device=dev)
    dscore = torch.empty(Bn, dtype=torch.float32, device=dev)
    loss = torch.zeros(1, dtype=torch.float32, device=dev)
    counter = [0]

    def step(i):
        counter[0] += 1
        lp.lp_sample_neg(g, pos_src, k_neg, wl.n_space, wl.sampler_seed, i, neg_dst=neg_dst, neg_src=neg_src)
        lp.lp_sample_blocks(g, e_src, e_dst, fanout, wl.sampler_seed + 1, i, blocks)
        lp.lp_sage_forward_blocks(blocks, model, X, acts, ws_f)
        lp.lp_score_loss(acts.H[-1], blocks.e_src_pos, blocks.e_dst_pos, n_pos, scores, loss, dscore, ws_l)
        lp.lp_backward_blocks(blocks, model, acts, dscore, grads, ws_b)
        lp.lp_adam_step(model, grads, adam, counter[0], lr=1e-3)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    first_loss = None
    lp.lp_timing_enable(True)
    lp.lp_timing_collect()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(1000 + i)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    classes = lp.lp_timing_collect()
    lp.lp_timing_enable(False)
    ms = dt * 1e3 / max(args.steps, 1)

    # The same step recorded once as a HIP graph and replayed (every replay repeats the recorded batch id and Adam
    # step count, so this is a timing of the launch overhead, not a training loop): informational.
    graph_ms = None
    try:
        cap = torch.cuda.Stream()
        cap.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(cap):
            step(1500)
        torch.cuda.current_stream().wait_stream(cap)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=cap):
            step(1500)
        graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - t0) * 1e3 / max(args.steps, 1)
    except RuntimeError as exc:
        sys.stderr.write("graph replay not measured: %s\n" % exc)

    # The same steps with the next batch's negatives and computational graph built on a second stream while the
    # current batch trains (they depend on the graph and the batch only, not on the weights): what a training loop
    # with a prefetching sampler sees.  Two sets of batch buffers; events order producer and consumer.
    sets = [(e_src, e_dst, blocks)]
    e_src2, e_dst2 = e_src.clone(), e_dst.clone()
    sets.append((e_src2, e_dst2, lp.Blocks(g, Bn, fanout)))
    side = torch.cuda.Stream()
    ready = [torch.cuda.Event(), torch.cuda.Event()]
    freed = [torch.cuda.Event(), torch.cuda.Event()]

    def produce(i, slot):
        es, ed, blk = sets[slot]
        with torch.cuda.stream(side):
            side.wait_event(freed[slot])
            lp.lp_sample_neg(g, pos_src, k_neg, wl.n_space, wl.sampler_seed, i, neg_dst=ed[n_pos:], neg_src=es[n_pos:])
            lp.lp_sample_blocks(g, es, ed, fanout, wl.sampler_seed + 1, i, blk)
            ready[slot].record(side)

    def consume(slot):
        counter[0] += 1
        blk = sets[slot][2]
        main = torch.cuda.current_stream()
        main.wait_event(ready[slot])
        lp.lp_sage_forward_blocks(blk, model, X, acts, ws_f)
        lp.lp_score_loss(acts.H[-1], blk.e_src_pos, blk.e_dst_pos, n_pos, scores, loss, dscore, ws_l)
        lp.lp_backward_blocks(blk, model, acts, dscore, grads, ws_b)
        lp.lp_adam_step(model, grads, adam, counter[0], lr=1e-3)
        freed[slot].record(main)

    torch.cuda.synchronize()
    for ev in freed:
        ev.record(torch.cuda.current_stream())
    produce(5000, 0)
    for i in range(2):                       # warm-up of the two-stream loop
        produce(5001 + i, (i + 1) % 2)
        consume(i % 2)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        produce(6001 + i, (i + 1) % 2)
        consume(i % 2)
    torch.cuda.synchronize()
    ms_prefetch = (time.perf_counter() - t0) * 1e3 / max(args.steps, 1)
    frontiers = [int(x) for x in blocks.n.cpu().tolist()]
    entries = [int(blocks.ptr[k][frontiers[k + 1]].item()) for k in range(len(fanout))]
    out = {"metric": "sampled-neighbourhood train-step edges/sec (pos+neg), Adam update included, on 1 MI355X",
           "value": round(Bn / (ms * 1e-3), 1), "unit": "edges/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
           "ms_per_step": round(ms, 4), "ms_per_step_graph_replay": round(graph_ms, 4) if graph_ms is not None else None,
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "bf16" if bf16 else "f32", "fp32_products": fp32_products_name(bf16, split), "data": "synthetic",
           "config": {"workload": "%s graph (%d nodes, %d directed entries), GraphSAGE-mean %s, %d positives + %d negatives per "
                                  "step, fan-outs %s (first hop first)" % (args.workload, wl.n_nodes, g.nnz, "->".join(map(str, wl.dims)),
                                                                           n_pos, n_pos * k_neg, fanout),
                      "frontier_sizes_layer0_to_K": frontiers, "block_entries_layer1_to_K": entries},
           "loss": round(float(loss.item()), 6),
           "kernel_ms_per_step": {k: round(v[0] / max(args.steps, 1), 4) for k, v in classes.items()},
           "with_prefetching_sampler": {"ms_per_step": round(ms_prefetch, 4), "value": round(Bn / (ms_prefetch * 1e-3), 1),
                                        "note": "negatives and blocks of batch t+1 built on a second stream during batch t"}}
    print(json.dumps(out), flush=True)


def run_train_step(args, workload, full=True):
    """One measurement of the training step on `workload`; returns the JSON object.  full=False (a secondary workload
    reported beside the headline) leaves out the graph replay, the other way of forming fp32 products and the oracle."""
    import numpy as np
    import torch

    import paper_2506_20818_amd as lp
    from paper_2506_20818_amd import binding as B
    from lp_workloads import make_workload

    products = lp.LP_FP32_PRODUCTS_NATIVE if args.fp32_products == "native" else lp.LP_FP32_PRODUCTS_BF16X6
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    wl = make_workload(workload)
    i32 = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(dev)
    f32 = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(dev)

    gcn, use_mlp = args.model == "gcn", args.predictor == "mlp"
    src_np, dst_np = wl.src, wl.dst
    if gcn:   # the GCN propagation runs over the graph with every self-pair present
        loop = np.arange(wl.n_nodes, dtype=np.int32)
        src_np, dst_np = np.concatenate([wl.src, loop]), np.concatenate([wl.dst, loop])
    rows, cols = i32(src_np), i32(dst_np)
    lp.lp_build_csr(wl.n_nodes, rows, cols, True)                     # warm-up of the setup path
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    g = lp.lp_build_csr(wl.n_nodes, rows, cols, True)
    torch.cuda.synchronize()
    build_s = time.perf_counter() - t0

    bf16 = wl.dtype == "bf16"
    split = (not bf16) and products == lp.LP_FP32_PRODUCTS_BF16X6
    tdt = torch.bfloat16 if bf16 else torch.float32
    st = (lambda a: f32(a).to(torch.bfloat16)) if bf16 else f32      # storage type of features and weights
    if gcn:
        model = lp.Model(None, [st(w) for w in wl.W_neigh], [f32(b) for b in wl.bias], layer_type=lp.LP_LAYER_GCN, fp32_products=products)
    else:
        model = lp.Model([st(w) for w in wl.W_self], [st(w) for w in wl.W_neigh], [f32(b) for b in wl.bias], fp32_products=products)
    models = {"timed": model}
    X = st(wl.X)
    n_pos, k_neg, Bn = wl.n_pos, wl.k_neg, wl.batch_edges
    pos_src = i32(wl.pos_src)
    mlp = None
    if use_mlp:   # "Hyperparameters": a 3-layer MLP edge predictor, hidden width 256 (here: the embedding width)
        rng = np.random.default_rng(777)
        F = wl.dims[-1]
        md = [F, F, F, 1]
        mlp = lp.Mlp([st((rng.standard_normal((md[j], md[j + 1])) / np.sqrt(md[j])).astype(np.float32)) for j in range(3)],
                     [f32(rng.uniform(-0.1, 0.1, md[j + 1]).astype(np.float32)) for j in range(3)], fp32_products=products)
        macts, mgrads = lp.MlpActs(mlp, Bn, dev), lp.MlpGrads(mlp, dev)
    e_src = torch.empty(Bn, dtype=torch.int32, device=dev)
    e_dst = torch.empty(Bn, dtype=torch.int32, device=dev)
    e_src[:n_pos] = pos_src
    e_dst[:n_pos] = i32(wl.pos_dst)
    neg_src, neg_dst = e_src[n_pos:], e_dst[n_pos:]
    acts = lp.Acts(wl.n_nodes, wl.dims, dev, tdt)
    grads = lp.Grads(wl.n_nodes, wl.dims, dev, dtype=tdt)
    ws_f = torch.empty(B.forward_edges_workspace_bytes(model, wl.n_nodes, Bn), dtype=torch.uint8, device=dev)
    ws_b = torch.empty(B.backward_workspace_bytes(model, wl.n_nodes, Bn), dtype=torch.uint8, device=dev)
    ws_l = torch.empty(1 << 16, dtype=torch.uint8, device=dev)
    scores = torch.empty(Bn, dtype=torch.float32, device=dev)
    dscore = torch.empty(Bn, dtype=torch.float32, device=dev)
    loss = torch.zeros(1, dtype=torch.float32, device=dev)

    def step(i, which="timed", every_row=False):
        model = models[which]
        lp.lp_sample_neg(g, pos_src, k_neg, wl.n_space, wl.sampler_seed, i, neg_dst=neg_dst, neg_src=neg_src)
        if every_row:   # for reference only: the last layer for every visible node
            lp.lp_sage_forward(g, model, X, acts, ws_f)
        else:           # the training forward: the last layer where the loss reads it
            lp.lp_sage_forward_edges(g, model, X, e_src, e_dst, acts, ws_f)
        if mlp is None:
            lp.lp_score_loss(acts.H[-1], e_src, e_dst, n_pos, scores, loss, dscore, ws_l)
            lp.lp_backward(g, model, X, acts, e_src, e_dst, dscore, grads, ws_b)
        else:   # the binding allocates scores, edge gradients and workspaces per call (torch's caching allocator)
            s_, l_, ds_, _ = lp.lp_mlp_score_loss(acts.H[-1], e_src, e_dst, n_pos, mlp, macts)
            _, eg = lp.lp_mlp_backward(mlp, macts, ds_, mgrads)
            lp.lp_backward_edge_grads(g, model, X, acts, e_src, e_dst, eg, grads, ws_b)
            loss.copy_(l_)

    if full and args.copy_calibration_mib > 0:
        a = torch.zeros(args.copy_calibration_mib << 18, dtype=torch.float32, device=dev)
        b = torch.empty_like(a)
        torch.cuda.synchronize()
        b.copy_(a)
        torch.cuda.synchronize()
        del a, b

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()

    # un-instrumented pass, for reference
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(1000 + i)
    torch.cuda.synchronize()
    plain_ms = (time.perf_counter() - t0) * 1e3 / max(args.steps, 1)

    # the same step recorded once as a HIP graph and replayed (the library allocates nothing and clears its scratch
    # with kernels, so a step can be captured); every replay draws the negatives of the recorded step id, which is why
    # this figure is informational and `value` comes from the eager steps
    graph_ms = None
    try:
        if not full:
            raise RuntimeError("not measured for a secondary workload")
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step(1500)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            step(1500)
        graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - t0) * 1e3 / max(args.steps, 1)
    except RuntimeError as exc:   # capture unsupported in this environment: report that, do not fail the benchmark
        if full:
            sys.stderr.write("graph replay not measured: %s\n" % exc)

    # timed region, with the library's per-launch HIP events switched on
    lp.lp_timing_enable(args.timing_level)
    lp.lp_timing_collect()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(2000 + i)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    classes = lp.lp_timing_collect()
    lp.lp_timing_enable(False)
    loss_val = float(loss.item())
    ms_per_step = dt * 1e3 / max(args.steps, 1)

    # for reference, the same steps with the other way of forming the fp32 products (outside the timed region)
    other_products = None
    if full and not bf16 and mlp is None:   # the same weight tensors as a second model with the other value of fp32_products
        models["other"] = model.with_products(lp.LP_FP32_PRODUCTS_NATIVE if split else lp.LP_FP32_PRODUCTS_BF16X6)
        for i in range(3):
            step(3000 + i, "other")
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            step(2000 + i, "other")      # the batches of the timed region: the last loss is comparable with "loss"
        torch.cuda.synchronize()
        oms = (time.perf_counter() - t0) * 1e3 / max(args.steps, 1)
        other_products = {"fp32_products": fp32_products_name(False, not split), "ms_per_step_without_events": round(oms, 4),
                          "value": round(Bn / (oms * 1e-3), 1), "loss": round(float(loss.item()), 6)}

    # for reference, the same steps with the embeddings of EVERY node computed by the last layer (lp_sage_forward), as
    # an evaluation pass needs them; the training step reads only those of the batch's end points
    every_row = None
    if full:
        for i in range(2):
            step(3000 + i, every_row=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            step(2000 + i, every_row=True)
        torch.cuda.synchronize()
        ems = (time.perf_counter() - t0) * 1e3 / max(args.steps, 1)
        every_row = {"ms_per_step_without_events": round(ems, 4), "value": round(Bn / (ems * 1e-3), 1), "loss": round(float(loss.item()), 6)}

    # accounting only (outside the timed region): how many nodes are an endpoint of a scored edge in the timed steps,
    # and how many CSR entries point at one of them
    deg = (g.rowptr[1:] - g.rowptr[:-1]).to(torch.int64)
    n_t_sum = nnz_t_sum = 0
    for i in range(args.steps):
        lp.lp_sample_neg(g, pos_src, k_neg, wl.n_space, wl.sampler_seed, 2000 + i, neg_dst=neg_dst, neg_src=neg_src)
        touched = torch.unique(torch.cat([e_src, e_dst]).to(torch.int64))
        n_t_sum += int(touched.numel())
        nnz_t_sum += int(deg[touched].sum().item())
    n_t, nnz_t = n_t_sum / max(args.steps, 1), nnz_t_sum / max(args.steps, 1)

    n, nnz = wl.n_nodes, g.nnz
    sp_bytes, nt_flops, tn_flops = step_counts(n, nnz, wl.dims, n_t, nnz_t, Bn, 2 if bf16 else 4, 1 if gcn else 2)
    if use_mlp:   # hidden layers of the predictor on Bn edge rows: forward, input gradients and weight gradients
        F = wl.dims[-1]
        nt_flops += 2 * 2.0 * Bn * F * F + 2 * 2.0 * Bn * F * F
        tn_flops += 2 * 2.0 * Bn * F * F
    per_step = {k: (ms / max(args.steps, 1), cnt // max(args.steps, 1)) for k, (ms, cnt) in classes.items()}

    es = 2 if bf16 else 4
    # whether the matrix the widest aggregation gathers from fits the Infinity Cache: if it does, "achieved" is
    # cache-assisted and must not be read as an HBM rate
    cache_resident = bool(n * max(wl.dims[:-1]) * es <= INFINITY_CACHE_BYTES)

    def hbm_line(cls, bytes_per_step):
        ms, cnt = per_step[cls]
        gbs = bytes_per_step / (ms * 1e-3) / 1e9 if ms > 0 else 0.0
        return {"bound": "hbm", "kernel": cls, "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(gbs / HBM_PEAK_GBS, 4), "traffic": None, "frac_counters": None, "cache_resident": cache_resident,
                "launches_per_step": cnt, "avg_launch_ms": round(ms / max(cnt, 1), 4),
                "algorithmic_bytes_per_launch": int(bytes_per_step / max(cnt, 1))}

    def mfma_line(cls, flops_per_step, peak=MFMA_FP32_PEAK_TFLOPS):
        ms, cnt = per_step[cls]
        tf = flops_per_step / (ms * 1e-3) / 1e12 if ms > 0 else 0.0
        return {"bound": "mfma", "kernel": cls, "achieved": round(tf, 2), "peak": peak, "unit": "TFLOP/s",
                "frac": round(tf / peak, 4), "traffic": None, "launches_per_step": cnt,
                "avg_launch_ms": round(ms / max(cnt, 1), 4), "flops_per_launch": int(flops_per_step / max(cnt, 1))}

    # HBM bytes per launch are NOT measured in this run (counter collection needs rocprofv3 around the process): they
    # are copied from the committed summary of two rocprofv3 --pmc runs of this same script (FETCH_SIZE, WRITE_SIZE,
    # each scaled by what a plain copy of known size reads), named in "traffic_source"; null when no summary covers
    # the workload and model variant.
    traffic = {}
    tpath = os.path.join(ROOT, "profiles", "traffic_%s.json" % workload)
    if os.path.exists(tpath) and not gcn and not use_mlp and (bf16 or split):
        with open(tpath) as fh:
            traffic = json.load(fh)

    # with bf16 storage both kinds of product run on the bf16 matrix cores (fp32 accumulation); so do fp32 models in
    # the default product mode, where one fp32 product costs six bf16 term products: the ceiling for algorithmic
    # fp32 flops is then a sixth of the bf16 peak
    mfma_peak = BF16_MFMA_PEAK_TFLOPS if bf16 else (round(BF16_MFMA_PEAK_TFLOPS / 6.0, 1) if split else MFMA_FP32_PEAK_TFLOPS)
    lines = {"spmm": hbm_line("spmm", sp_bytes),
             "gemm_nt": mfma_line("gemm_nt", nt_flops, mfma_peak),
             "gemm_tn": mfma_line("gemm_tn", tn_flops, mfma_peak)}
    if split:
        for cls in ("gemm_nt", "gemm_tn"):
            lines[cls]["peak_basis"] = "bf16 MFMA peak %.0f TFLOP/s / 6 term products per fp32 product" % BF16_MFMA_PEAK_TFLOPS
            lines[cls]["mfma_tflops_executed"] = round(6.0 * lines[cls]["achieved"], 1)
    # the two small steps of the metric's second half: scoring gathers two embedding rows per edge and writes a score
    # and a gradient scalar; the sampler is latency bound, so it is reported as samples per second
    score_bytes = Bn * (2.0 * wl.dims[-1] * es + 16.0)
    if use_mlp:   # the element-wise product of the two rows is written out, and the output layer reads the last hidden row
        score_bytes += Bn * 2.0 * wl.dims[-1] * es
    lines["score"] = hbm_line("score", score_bytes)
    lines["score"]["cache_resident"] = bool(n * wl.dims[-1] * es <= INFINITY_CACHE_BYTES)
    sample_ms = per_step["sample"][0]
    sample_line = {"bound": "latency", "kernel": "sample", "achieved": round(n_pos * k_neg / (sample_ms * 1e-3) / 1e9, 3) if sample_ms > 0 else 0.0,
                   "unit": "Gsamples/s", "launches_per_step": per_step["sample"][1], "avg_launch_ms": round(sample_ms / max(per_step["sample"][1], 1), 4),
                   "traffic": None, "counter_gbs": None}
    for cls in lines:
        t = traffic.get(cls + "_bytes_per_launch")
        lines[cls]["traffic"] = int(t) if t else None
        if t:
            lines[cls]["traffic_source"] = traffic.get("source", "profiles/traffic_%s.json" % workload)
            if lines[cls]["bound"] == "hbm" and lines[cls]["avg_launch_ms"] > 0:   # counter bytes / time / peak
                lines[cls]["frac_counters"] = round(t / (lines[cls]["avg_launch_ms"] * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)
    t = traffic.get("sample_bytes_per_launch")
    if t:
        sample_line["traffic"] = int(t)
        sample_line["traffic_source"] = traffic.get("source", "profiles/traffic_%s.json" % workload)
        if sample_line["avg_launch_ms"] > 0:
            sample_line["counter_gbs"] = round(t / (sample_line["avg_launch_ms"] * 1e-3) / 1e9, 1)
    score_line = lines.pop("score")
    dominant = max(lines, key=lambda c: per_step[c][0])

    out = {
        "metric": "train-step edges/sec (pos+neg) on 1 MI355X; SpMM achieved HBM GB/s",
        "value": round(Bn / (ms_per_step * 1e-3), 1),
        "unit": "edges/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "ms_per_step_without_events": round(plain_ms, 4),
        "ms_per_step_graph_replay": round(graph_ms, 4) if graph_ms is not None else None,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16" if bf16 else "f32",
        "fp32_products": fp32_products_name(bf16, split),
        "data": "synthetic",
        "config": {"workload": "%s: synthetic power-law graph, %d nodes, %d directed CSR entries, %s %s, %s, "
                               "%d positives + %d uniform negatives per step, full-neighbour aggregation"
                               % (workload, n, nnz, "GCN (self-pairs in the graph)" if gcn else "GraphSAGE-mean",
                                  "->".join(map(str, wl.dims)), "3-layer MLP edge predictor" if use_mlp else "dot-product scorer",
                                  n_pos, n_pos * k_neg),
                   "n_nodes": n, "nnz": nnz, "dims": wl.dims, "n_pos": n_pos, "k_neg": k_neg,
                   "batch_endpoint_nodes": round(n_t, 1),
                   "last_layer_rows": ("the end points of the batch (lp_sage_forward_edges lists them: 8 B < 3 N)" if lists_last_layer(n, Bn)
                                       else "every node (8 B >= 3 N: lp_sage_forward_edges does not list)")},
        "loss": round(loss_val, 6),
        "csr_build": {"seconds": round(build_s, 5), "input_edges_per_s": round(wl.src.size / build_s, 1)},
        "roofline": lines[dominant],
        "roofline_spmm": lines["spmm"],
        "roofline_gemm_nt": lines["gemm_nt"],
        "roofline_gemm_tn": lines["gemm_tn"],
        "roofline_score": score_line,
        "sampler": sample_line,
        "kernel_ms_per_step": {k: round(v[0], 4) for k, v in per_step.items() if k != "other" or args.timing_level > 1},
        "with_other_fp32_products": other_products,
        "with_last_layer_for_every_node": every_row,
    }
    if args.timing_level <= 1:   # the small launches (fills, transposes, column sums) are not bracketed: by difference
        out["kernel_ms_per_step"]["other_and_gaps"] = round(ms_per_step - sum(v[0] for k, v in per_step.items() if k != "other"), 4)
    if full and not args.no_cpu_baseline and not gcn and not use_mlp:   # the oracle leg times the headline step only
        out["cpu_baseline"] = cpu_baseline(workload, args.cpu_scale if args.cpu_scale else CPU_SCALE.get(workload, 0.1))
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default=None, help="default: C4 (train_step), C2 (sampled_step), C3 (sparsify)")
    ap.add_argument("--cpu-scale", type=float, default=None,
                    help="fraction of the workload the CPU oracle is timed on (default: per workload, 10-30 s of host work)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--also", default=None,
                    help="comma-separated workloads measured after the headline and reported under \"also\" (same step; no "
                         "oracle leg).  Default: C2 when --workload is not given, nothing otherwise")
    ap.add_argument("--timing-level", type=int, default=1, choices=[1, 2],
                    help="1: HIP events around the aggregation, GEMM, scatter, score and sampler launches; 2: around every launch")
    ap.add_argument("--task", default="train_step", choices=["train_step", "sparsify", "sampled_step"],
                    help="train_step: the headline metric; sparsify: the sparsification pass over all partitions; "
                         "sampled_step: the mini-batch mode with sampled neighbourhoods")
    ap.add_argument("--model", default="sage", choices=["sage", "gcn"],
                    help="--task train_step: GraphSAGE-mean layers (the headline) or GCN layers (self-pairs added to the graph)")
    ap.add_argument("--predictor", default="dot", choices=["dot", "mlp"],
                    help="--task train_step: dot-product scorer (the headline) or the 3-layer MLP edge predictor")
    ap.add_argument("--fp32-products", default="bf16x6", choices=["bf16x6", "native"],
                    help="how fp32 models form their dense products (the fp32_products field of lp_model in include/lp.h)")
    ap.add_argument("--n-pos", type=int, default=10240, help="positives per batch of --task sampled_step")
    ap.add_argument("--fanout", default="25,10,5", help="neighbours per hop of --task sampled_step, first hop first")
    ap.add_argument("--alpha", type=float, default=0.15, help="sparsification level (draws per edge) of --task sparsify")
    ap.add_argument("--copy-calibration-mib", type=int, default=0,
                    help="also run one plain device copy of this many MiB (a dispatch of known size for counter runs)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.stderr.write("bench.py measures one worker's step on ONE GPU; --gpus %d is not supported "
                         "(no collectives are part of this build)\n" % args.gpus)
        sys.exit(2)

    if args.task == "sparsify":
        return sparsify_task(args)
    if args.task == "sampled_step":
        args.workload = args.workload or "C2"
        return sampled_step_task(args)
    if args.also is None:
        args.also = "C2" if args.workload is None else ""
    args.workload = args.workload or "C4"

    out = run_train_step(args, args.workload, True)
    also = [w for w in args.also.split(",") if w and w != args.workload] if (args.model == "sage" and args.predictor == "dot") else []
    if also:   # e.g. the Collab-scale workload beside the headline: same step, same code, its own rooflines
        out["also"] = {}
        for w in also:
            import gc
            import torch
            gc.collect()
            torch.cuda.empty_cache()
            r = run_train_step(args, w, False)
            out["also"][w] = {k: r[k] for k in ("value", "unit", "ms_per_step", "ms_per_step_without_events", "dtype", "fp32_products",
                                                "config", "loss", "roofline_spmm", "roofline_gemm_nt", "roofline_gemm_tn",
                                                "roofline_score", "sampler", "kernel_ms_per_step")}
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
