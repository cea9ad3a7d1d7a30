#!/usr/bin/env python3
"""Benchmark of hard-routed FFF inference on one MI355X.

One "step" is one call of fff_forward_hard over a whole batch of synthetic
tokens (tree descent, bucketing, leaf networks, output rows), inputs already
resident in HBM.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config C4]

Beside the headline tokens/s the line carries: the roofline position of the
dominant kernel (algorithmic bytes per launch / its average duration measured
with HIP events recorded on the call's stream inside the library), the same
for every stage and for the whole path, the spread of the timing, the CPU
oracle timed on this host (all cores, and one core), an equal-training-width
dense feedforward on the same GPU for the speedup, the ceiling a plain
streaming copy reaches on this device ("copy_ceiling") with every fraction also
stated against it, and under "others" the remaining two of the three
bandwidth-bound workloads (C3, C4, C5) timed and checked the same way.

Other modes, each printing one JSON line of its own:
    --sweep depth     small-batch latency against tree depth (the paper's speed experiment)
    --sweep experts   the same with the mixture-of-experts lookup (one engaged expert) beside it
    --sweep widths    the paper's grid of small networks (training widths 16..128 x leaf sizes 1..8,
                      batch 2048) beside the dense feedforward network of the same width
    --soft            the soft pass (Forward_T, all leaves) of --config, against the MFMA roofline
    --block           the pre-norm residual layer with nodes of --node-size hidden neurons on the
                      shapes of --config
    --probe gather    the row-gather microbenchmark (random row fetches against table size)
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X HBM3E, published

MFMA_BF16_PEAK_TFLOPS = 2500.0   # MI355X dense bf16, published


def measured_traffic(workload, kernel_launch):
    """HBM-side bytes per launch from profiles/hbm_traffic.md: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
    runs (scaled by what the same counters read for a plain copy of known size), one row per
    workload and kernel, each with the launch it was measured on as the library describes it
    (fff_last_launch: kernel names with their tile parameters).  None unless the launch that has
    just been timed is that very one -- a figure measured on another kernel says nothing here."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.md")
    if not os.path.exists(path):
        return None
    for line in open(path):
        cells = [c.strip() for c in line.strip().strip("|").split("|")]
        if len(cells) >= 6 and cells[0] == workload and cells[1].strip("`") == kernel_launch:
            try:
                return {"bytes": float(cells[4]) * 1e6, "fetch_bytes": float(cells[2]) * 1e6,
                        "write_bytes": float(cells[3]) * 1e6, "source": cells[5].strip("`")}
            except ValueError:
                return None
    return None


_probe_lib = None


def probes():
    """The bench-only probe library (row gather, streaming copy); no part of the product ABI."""
    global _probe_lib
    if _probe_lib is None:
        import ctypes
        from paper_2308_14711_amd import build
        P = ctypes.CDLL(build.PROBE_LIB)
        vp, i32, i64 = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64
        P.fffb_gather.argtypes = [vp, i64, i64, i32, i64, i32, i32, vp, vp]
        P.fffb_copy.argtypes = [vp, vp, i64, i64, vp]
        _probe_lib = P
    return _probe_lib


def probe_gather(torch, table, row_bytes, rows_in_flight, blocks, iters, dependent, sink):
    """Launch the row-gather probe on torch's current stream; returns the bytes the launch reads."""
    rows = table.numel() * table.element_size() // row_bytes
    rc = probes().fffb_gather(table.data_ptr(), rows, row_bytes, rows_in_flight, blocks, iters, int(bool(dependent)),
                              sink.data_ptr(), torch.cuda.current_stream().cuda_stream or None)
    if rc != 0:
        raise RuntimeError("fffb_gather failed (%d)" % rc)
    return blocks * 32 * iters * rows_in_flight * row_bytes


def copy_ceiling(torch, mbytes=512, reps=10):
    """What a kernel that only moves rows reaches on this device: a plain streaming copy of
    `mbytes` MB (beyond the 256 MB last-level cache), bytes read plus bytes written over time."""
    n = mbytes << 20
    src = torch.zeros((n,), dtype=torch.uint8, device="cuda")
    dst = torch.empty_like(src)
    stream = torch.cuda.current_stream().cuda_stream or None
    best = {}
    for blocks in (1024, 2048, 4096, 8192):
        for _ in range(2):
            rc = probes().fffb_copy(dst.data_ptr(), src.data_ptr(), n, blocks, stream)
            if rc != 0:
                raise RuntimeError("fffb_copy failed (%d)" % rc)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            probes().fffb_copy(dst.data_ptr(), src.data_ptr(), n, blocks, stream)
        e1.record()
        torch.cuda.synchronize()
        best[blocks] = 2.0 * n * reps / (e0.elapsed_time(e1) * 1e-3) / 1e9
    for _ in range(2):
        dst.copy_(src)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        dst.copy_(src)
    e1.record()
    torch.cuda.synchronize()
    runtime_copy = 2.0 * n * reps / (e0.elapsed_time(e1) * 1e-3) / 1e9
    blocks = max(best, key=best.get)
    del src, dst
    return {"GBps": round(best[blocks], 1), "blocks_of_512": blocks, "MB": mbytes,
            "runtime_copy_GBps": round(runtime_copy, 1),
            "counts": "bytes read + bytes written"}


_ceiling = None


def copy_ceiling_once(torch):
    global _ceiling
    if _ceiling is None:
        _ceiling = copy_ceiling(torch)
    return _ceiling


def algorithmic_bytes(w, ref_idx):
    """Bytes the method itself must move: x once, out once, leaf_idx, and every
    node row / leaf block that some token actually touches, once."""
    import numpy as np
    s = 2 if w.dtype == 1 else 4
    T, D, O, L, d = w.T, w.D, w.O, w.leaf_width, w.depth
    leaves = np.unique(ref_idx)
    nodes = set()
    cur = leaves.astype(np.int64)
    for m in range(d - 1, -1, -1):           # parents of the touched leaves, level by level
        cur = np.unique(cur >> 1)
        nodes.update(((1 << m) - 1 + cur).tolist())
    u_node, u_leaf = len(nodes), int(leaves.size)
    counts = np.bincount(np.asarray(ref_idx, dtype=np.int64), minlength=1 << d)
    occupancy = {"leaves": 1 << d, "non_empty": u_leaf, "max_bucket": int(counts.max()),
                 "singletons": int((counts == 1).sum()), "mean_bucket_of_non_empty": round(T / max(u_leaf, 1), 2)}
    node_bytes = u_node * (D * s + s)
    leaf_bytes = u_leaf * (L * D * s + L * s + L * O * s + O * s)
    return {
        "u_node": u_node, "u_leaf": u_leaf, "occupancy": occupancy,
        "path": T * D * s + T * O * s + 4 * T + node_bytes + leaf_bytes,
        "descent": T * D * s + 4 * T + node_bytes,
        "bucketing": 4 * T + 4 * T,                     # leaf_idx in, perm out
        "leaf": T * D * s + T * O * s + 8 * T + leaf_bytes,
        # the tile path's two launches: token rows in, hidden activations out (bf16); those back in
        # with the output weights, output rows out; both read the grouped order and the slots' leaves
        "leaf_hidden": T * D * s + 8 * T + u_leaf * (L * D * s + L * s) + T * L * 2,
        "leaf_output": T * L * 2 + 8 * T + u_leaf * (L * O * s + O * s) + T * O * s,
        # the fused launch cut in two: token rows in, leaf ids and hidden activations (fp32) out; those
        # back in with the output weights and biases, output rows out
        "walk_hidden": T * D * s + 4 * T + node_bytes + u_leaf * (L * D * s + L * s) + 4 * T * L,
        "leaf_slices": 4 * T + 4 * T * L + u_leaf * (L * O * s + O * s) + T * O * s,
    }


def depth_sweep(args, np, torch, W, F, with_moe=False):
    """Time per call against tree depth for a small batch: inputs and outputs 768 wide, leaves of
    `--sweep-leaf-width` neurons, depth `--sweep-min-depth`..`--sweep-max-depth`, `--sweep-batch` tokens (the shape
    of the paper's inference-speed experiment, with synthetic inputs).  Three clocks per depth:
    calls issued back to back from Python (launch cost of the host loop included), the same calls
    replayed from a HIP graph holding 20 of them (per-call device time with launches amortised),
    and the CPU oracle.  The routing of every depth is checked against the oracle.

    with_moe: the paper's comparison of lookups -- a mixture of experts with one engaged expert and
    2^depth experts (the same leaf weights, a gating matrix of 2^depth rows instead of the tree) is
    timed and checked the same way; only the lookup differs between the two calls."""
    import oracle
    T, L, D, O = args.sweep_batch, args.sweep_leaf_width, 768, 768
    rows = []
    for d in range(args.sweep_min_depth, args.sweep_max_depth + 1):
        w = W.make_layer("depth_sweep", T, D, O, d, L, W.ACT_GELU, W.DTYPE_BF16, seed=d, keep_f32=False)
        dev = {}
        for k in W.TENSORS:
            a = np.ascontiguousarray(w.device_array(k))
            dev[k] = torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
        out = torch.empty((T, O), dtype=torch.bfloat16, device="cuda")
        idx = torch.empty((T,), dtype=torch.int32, device="cuda")
        F.fff_reserve_workspace(T, d)

        def call(stream=None):
            F.fff_forward_hard(dev["x"], dev["node_w"], dev["node_b"], dev["leaf_w1"], dev["leaf_b1"],
                               dev["leaf_w2"], dev["leaf_b2"], d, L, w.act, out, idx, stream)

        for _ in range(args.warmup):
            call()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            call()
        torch.cuda.synchronize()
        eager_us = (time.perf_counter() - t0) * 1e6 / args.steps
        per_graph = 20
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for _ in range(per_graph):
                call()
        for _ in range(3):
            g.replay()
        torch.cuda.synchronize()
        reps = max(1, args.steps // per_graph)
        t0 = time.perf_counter()
        for _ in range(reps):
            g.replay()
        torch.cuda.synchronize()
        graph_us = (time.perf_counter() - t0) * 1e6 / (reps * per_graph)
        ins = [np.ascontiguousarray(w.device_array(k)) for k in W.TENSORS]
        t0 = time.perf_counter()
        ref_out, ref_idx, margin = oracle.forward_hard(*ins, d, L, w.act)
        cpu_us = (time.perf_counter() - t0) * 1e6
        got_idx = idx.cpu().numpy()
        mism = np.nonzero(got_idx != ref_idx)[0]
        keep = got_idx == ref_idx
        got = out.float().cpu().numpy().astype(np.float64)
        scale = np.maximum(np.abs(ref_out[keep]).max(axis=1), 1e-30)
        rows.append({"depth": d, "us_per_call_python_loop": round(eager_us, 2), "us_per_call_graph": round(graph_us, 2),
                     "us_cpu_oracle": round(cpu_us, 1), "launch_path": int(F.fff_get_option("last_path")),
                     "idx_mismatch_outside_margin": int((margin[mism] >= 1e-4).sum()),
                     "max_rel_row_err": float((np.abs(got[keep] - ref_out[keep]).max(axis=1) / scale).max())})
        if with_moe:
            gw, gb = W.moe_gate(1 << d, D, W.DTYPE_BF16, seed=d)
            d_gw = torch.from_numpy(gw.view(np.int16)).cuda().view(torch.bfloat16)
            d_gb = torch.from_numpy(gb.view(np.int16)).cuda().view(torch.bfloat16)

            def moe_call():
                F.fff_moe_top1_forward(dev["x"], d_gw, d_gb, dev["leaf_w1"], dev["leaf_b1"], dev["leaf_w2"],
                                       dev["leaf_b2"], d, L, w.act, out, idx)

            for _ in range(args.warmup):
                moe_call()
            torch.cuda.synchronize()
            g2 = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g2):
                for _ in range(per_graph):
                    moe_call()
            for _ in range(3):
                g2.replay()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(reps):
                g2.replay()
            torch.cuda.synchronize()
            moe_us = (time.perf_counter() - t0) * 1e6 / (reps * per_graph)
            t0 = time.perf_counter()
            m_out, m_idx, m_margin = oracle.moe_top1(ins[0], gw, gb, *ins[3:], L, w.act)
            moe_cpu_us = (time.perf_counter() - t0) * 1e6
            g_idx = idx.cpu().numpy()
            mm = np.nonzero(g_idx != m_idx)[0]
            kp = g_idx == m_idx
            g_out = out.float().cpu().numpy().astype(np.float64)
            sc = np.maximum(np.abs(m_out[kp]).max(axis=1), 1e-30)
            rows[-1].update({"moe_us_per_call_graph": round(moe_us, 2), "moe_us_cpu_oracle": round(moe_cpu_us, 1),
                             "moe_experts": 1 << d, "moe_idx_mismatch_outside_margin": int((m_margin[mm] >= 1e-4).sum()),
                             "moe_max_rel_row_err": float((np.abs(g_out[kp] - m_out[kp]).max(axis=1) / sc).max()),
                             "moe_gating_bytes": int((1 << d) * (D + 1) * 2)})
            del d_gw, d_gb
        del dev, w, ins
    ds = np.array([r["depth"] for r in rows], dtype=np.float64)
    ys = np.array([r["us_per_call_graph"] for r in rows])
    slope, icpt = (np.polyfit(ds, ys, 1) if len(rows) > 1 else (0.0, ys[0]))
    resid = ys - (slope * ds + icpt)
    print(json.dumps({
        "metric": "fff_vs_moe_lookup_latency_vs_depth" if with_moe else "fff_hard_inference_latency_vs_depth",
        "unit": "us per call", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "higher_is_better": False, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "depth sweep: batch %d, D = O = 768, leaf width %d, GELU" % (T, L),
                   "options": args.opt, "cpu_oracle_cores": oracle.num_threads()},
        "linear_fit_graph": {"us_per_level": round(float(slope), 3), "us_at_depth_0": round(float(icpt), 2),
                             "max_abs_residual_us": round(float(np.abs(resid).max()), 2)},
        "sweep": rows}))


def width_sweep(args, np, torch, W, F):
    """The paper's small-network grid at its inference batch (section "Explorative evaluation",
    the table of training widths 16..128 against leaf sizes 1..8; testing batch 2048): MNIST-shaped
    inputs (784 features, 10 outputs, fp32, ReLU), for every training width w and leaf size l the
    FFF of depth log2(w / l) timed beside the dense feedforward network of width w (torch addmm +
    relu + addmm on the same GPU), both replayed from a HIP graph of 20 calls; every FFF cell is
    checked against the oracle."""
    import oracle
    T, D, O = args.sweep_batch if args.sweep_batch != 256 else 2048, 784, 10
    per_graph = 20
    reps = max(1, args.steps // per_graph)

    def graph_us(fn):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for _ in range(per_graph):
                fn()
        for _ in range(3):
            g.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            g.replay()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e6 / (reps * per_graph)

    rows = []
    for width in (16, 32, 64, 128):
        x32 = torch.randn((T, D), device="cuda")
        w1 = torch.randn((D, width), device="cuda") / 28.0
        b1 = torch.zeros((width,), device="cuda")
        w2 = torch.randn((width, O), device="cuda") / np.sqrt(width)
        b2 = torch.zeros((O,), device="cuda")
        ff_us = graph_us(lambda: torch.addmm(b2, torch.relu(torch.addmm(b1, x32, w1)), w2))
        for L in (8, 4, 2, 1):
            d = int(np.log2(width // L))
            w = W.make_layer("width_sweep", T, D, O, d, L, W.ACT_RELU, W.DTYPE_F32, seed=width + L,
                             x_dist="uniform01", node_b="centred0.1")
            dev = {k: torch.from_numpy(np.ascontiguousarray(w.device_array(k))).cuda() for k in W.TENSORS}
            out = torch.empty((T, O), dtype=torch.float32, device="cuda")
            idx = torch.empty((T,), dtype=torch.int32, device="cuda")
            F.fff_reserve_workspace(T, d)

            def call():
                F.fff_forward_hard(dev["x"], dev["node_w"] if d else None, dev["node_b"] if d else None,
                                   dev["leaf_w1"], dev["leaf_b1"], dev["leaf_w2"], dev["leaf_b2"], d, L, w.act, out, idx)

            us = graph_us(call)
            ins = [np.ascontiguousarray(w.device_array(k)) for k in W.TENSORS]
            ref_out, ref_idx, margin = oracle.forward_hard(*ins, d, L, w.act)
            got_idx = idx.cpu().numpy()
            mism = np.nonzero(got_idx != ref_idx)[0]
            keep = got_idx == ref_idx
            got = out.cpu().numpy().astype(np.float64)
            scale = np.maximum(np.abs(ref_out[keep]).max(axis=1), 1e-30)
            rows.append({"training_width": width, "leaf_size": L, "depth": d, "fff_us_per_call": round(us, 2),
                         "dense_ff_us_per_call": round(ff_us, 2), "speedup": round(ff_us / us, 2),
                         "launch_path": int(F.fff_get_option("last_path")),
                         "leaves_hit": int(np.unique(ref_idx).size),
                         "idx_mismatch_outside_margin": int((margin[mism] >= 1e-4).sum()),
                         "max_rel_row_err": float((np.abs(got[keep] - ref_out[keep]).max(axis=1) / scale).max())})
    print(json.dumps({"metric": "fff_vs_dense_ff_small_networks", "unit": "us per call", "n_gpus": 1,
                      "steps": args.steps, "warmup": args.warmup, "higher_is_better": False, "dtype": "f32",
                      "data": "synthetic",
                      "config": {"workload": "width sweep: batch %d, 784 inputs, 10 outputs, fp32, ReLU, training widths "
                                             "16..128 x leaf sizes 8..1" % T},
                      "sweep": rows}))


def soft_bench(args, np, torch, W, F):
    """Forward_T of the chosen workload: every token against every leaf.  One step = one call of
    fff_forward_soft (node scores, mixture weights, weighted hidden activations, output rows, per-node
    entropies).  The roofline is the matrix cores': flops of the three contractions over time."""
    import oracle
    w = W.config(args.config, keep_f32=False, T=args.tokens or None)
    assert w.dtype == W.DTYPE_BF16, "the soft pass runs on the bf16 matrix cores"
    NL, NN = 1 << w.depth, (1 << w.depth) - 1
    dev = {k: torch.from_numpy(np.ascontiguousarray(w.device_array(k)).view(np.int16)).cuda().view(torch.bfloat16)
           for k in W.TENSORS}
    out = torch.empty((w.T, w.O), dtype=torch.bfloat16, device="cuda")
    mix = torch.empty((w.T, NL), dtype=torch.float32, device="cuda")
    ent = torch.empty((max(NN, 1),), dtype=torch.float32, device="cuda")

    def step():
        F.fff_forward_soft(dev["x"], dev["node_w"] if w.depth else None, dev["node_b"] if w.depth else None,
                           dev["leaf_w1"], dev["leaf_b1"], dev["leaf_w2"], dev["leaf_b2"], w.depth, w.leaf_width,
                           w.act, out, mix, ent if w.depth else None)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    K2 = (NL * (w.leaf_width + 1) + 7) // 8 * 8
    flops = 2.0 * w.T * (w.D * NN + w.D * NL * w.leaf_width + K2 * w.O)
    tflops = flops / (ms * 1e-3) / 1e12
    # the oracle on a prefix of the batch: parity of those rows, and its rate
    n = min(w.T, 1024)
    ins = [np.ascontiguousarray(w.device_array(k)) for k in W.TENSORS]
    ins[0] = np.ascontiguousarray(ins[0][:n])
    t1 = time.perf_counter()
    ref_out, ref_mix = oracle.forward_soft(*ins, w.depth, w.leaf_width, w.act)
    cpu_s = time.perf_counter() - t1
    got = out[:n].float().cpu().numpy().astype(np.float64)
    err = np.abs(got - ref_out).max(axis=1) / np.maximum(np.abs(ref_out).max(axis=1), 1e-30)
    mix_err = float(np.abs(mix[:n].cpu().numpy().astype(np.float64) - ref_mix).max())
    print(json.dumps({
        "metric": "fff_soft_forward_tokens_per_s", "value": round(w.T / (ms * 1e-3), 1), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "%s: %s, soft pass over all %d leaves" % (w.name, w.note, NL), "T": w.T, "D": w.D,
                   "O": w.O, "depth": w.depth, "leaf_width": w.leaf_width, "seed": 0},
        "roofline": {"bound": "mfma", "achieved": round(tflops, 1), "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(tflops / MFMA_BF16_PEAK_TFLOPS, 4), "traffic": None, "flops": flops},
        "cpu_baseline": {"value": round(n / cpu_s, 1), "unit": "tokens/s", "cores": oracle.num_threads(),
                         "kind": "oracle", "sample": "first %d tokens of %s, one pass of Forward_T, fp64" % (n, w.name),
                         "seconds": round(cpu_s, 3)},
        "parity": {"rows_checked": n, "max_rel_row_err": float(err.max()), "max_mixture_err": mix_err}}))


def block_bench(args, np, torch, W, F):
    """Forward_I with nodes of --node-size hidden neurons as a pre-norm residual layer, on the shapes of
    the chosen workload (bf16 ones with O = D).  One step = one call of fff_forward_block = one kernel;
    its duration comes from events on the stream of the calls.  Roofline: HBM, every tensor once."""
    import oracle
    w = W.config(args.config, keep_f32=False, T=args.tokens or None)
    assert w.O == w.D, "the residual sum needs rows of one width"
    n, eps = args.node_size, 1e-5
    nodes = W.wide_nodes(w.depth, n, w.D, w.dtype)
    ln = W.layer_norm_params(w.D, w.dtype)
    leaves = [np.ascontiguousarray(w.device_array(k)) for k in ("leaf_w1", "leaf_b1", "leaf_w2", "leaf_b2")]
    x = np.ascontiguousarray(w.device_array("x"))

    def up(a):
        if a.dtype == np.uint16:
            return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
        return torch.from_numpy(a).cuda()

    d_ln, d_nodes, d_leaves = [up(a) for a in ln], [up(a) for a in nodes], [up(a) for a in leaves]
    sets = args.sets or 4            # rotate token and output buffers so that no step finds its rows cached
    xs = [up(x) for _ in range(sets)]
    outs = [torch.empty_like(xs[0]) for _ in range(sets)]
    idx = torch.empty((w.T,), dtype=torch.int32, device="cuda")

    def step(i):
        F.fff_forward_block(xs[i % sets], d_ln[0], d_ln[1], eps, *d_nodes, *d_leaves, w.depth, n, w.leaf_width,
                            w.act, True, outs[i % sets], idx)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for i in range(args.steps):
        step(i)
    e1.record()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    kernel_ms = e0.elapsed_time(e1) / args.steps
    launch = F.fff_last_launch()
    es = 2 if w.dtype == W.DTYPE_BF16 else 4
    # rows of up to 128 16-byte pieces take the 16-lanes-per-token kernel, longer ones a wave per token
    kernel = "block_group_kernel" if max(w.D, w.O) * es <= 128 * 16 else "block_kernel"
    # rows a token meets on its way: what the kernel asks of the caches per token
    row_bytes = es * (w.depth * n * w.D + w.leaf_width * (w.D + w.O))
    # the oracle on a prefix of the batch: parity of those rows, and its rate
    m = w.T
    step(0)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    cpu_passes = 0
    while cpu_passes < 1 or (time.perf_counter() - t1 < 5.0 and cpu_passes < 200):
        ref_out, ref_idx, margin = oracle.forward_block(x[:m], ln[0], ln[1], eps, *nodes, *leaves, w.depth, n,
                                                        w.leaf_width, w.act, True)
        cpu_passes += 1
    cpu_s = time.perf_counter() - t1
    got = outs[0][:m].float().cpu().numpy().astype(np.float64)
    gi = idx[:m].cpu().numpy()
    # algorithmic bytes: x, out and leaf_idx once, the layer-norm vectors, and every node network and
    # leaf block that some token touches, once
    touched = algorithmic_bytes(w, ref_idx)
    weight_bytes = es * (touched["u_node"] * (n * w.D + 2 * n + 1) + 2 * w.D +
                         touched["u_leaf"] * (w.leaf_width * (w.D + w.O + 1) + w.O))
    alg = es * w.T * (w.D + w.O) + 4 * w.T + weight_bytes
    gbs = alg / (kernel_ms * 1e-3) / 1e9
    same = gi == ref_idx
    assert (margin[~same] < 1e-4).all(), "routing differs outside the margin"
    err = (np.abs(got - ref_out).max(axis=1) / np.maximum(np.abs(ref_out).max(axis=1), 1e-30))[same]
    print(json.dumps({
        "metric": "fff_block_tokens_per_s", "value": round(w.T / (ms * 1e-3), 1), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if w.dtype == W.DTYPE_BF16 else "f32", "data": "synthetic",
        "config": {"workload": "%s shapes as a pre-norm residual layer, nodes of %d hidden neurons" % (w.name, n),
                   "T": w.T, "D": w.D, "O": w.O, "depth": w.depth, "node_size": n, "leaf_width": w.leaf_width,
                   "seed": 0, "buffer_sets": sets},
        "roofline": {"bound": "hbm", "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(gbs / HBM_PEAK_GBS, 4),
                     "traffic": (measured_traffic(w.name, launch) or {}).get("bytes") if not args.tokens else None,
                     "kernel_launch": launch,
                     "kernel": kernel,
                     "kernel_ms": round(kernel_ms, 5), "algorithmic_bytes": alg,
                     "weight_row_bytes_per_token": row_bytes},
        "cpu_baseline": {"value": round(m * cpu_passes / cpu_s, 1), "unit": "tokens/s", "cores": oracle.num_threads(),
                         "kind": "oracle", "sample": "the whole batch of %d tokens, %d passes, fp64" % (m, cpu_passes),
                         "seconds": round(cpu_s, 3)},
        "parity": {"rows_checked": int(same.sum()), "routed_differently_inside_margin": int((~same).sum()),
                   "max_rel_row_err": float(err.max())}}))


def gather_probe(args, np, torch, F):
    """The row-gather microbenchmark behind the roofline discussion (probe library, fffb_gather): random rows of
    --probe-row-bytes out of zero-filled tables from well inside one XCD's L2 to beyond the last-level
    cache, as a dependent chain with four rows in flight per 16 lanes.  One JSON line."""
    rb = args.probe_row_bytes
    sink = torch.zeros((4,), dtype=torch.int32, device="cuda")
    sizes = []
    for log_rows in range(8, 19):
        rows = 1 << log_rows
        if rows * rb > (1 << 30):
            break
        table = torch.zeros((rows * rb,), dtype=torch.uint8, device="cuda")
        blocks, iters = 512, 32
        res = {}
        for dep in (0, 1):
            for _ in range(2):
                nbytes = probe_gather(torch, table, rb, 4, blocks, iters, dep, sink)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(5):
                probe_gather(torch, table, rb, 4, blocks, iters, dep, sink)
            e1.record()
            torch.cuda.synchronize()
            res["dependent" if dep else "independent"] = round(nbytes * 5 / (e0.elapsed_time(e1) * 1e-3) / 1e12, 2)
        sizes.append({"table_MB": round(rows * rb / 1e6, 1), "rows": rows, "TBps": res})
        del table
    print(json.dumps({"metric": "row_gather_rate", "unit": "TB/s", "n_gpus": 1, "data": "synthetic",
                      "config": {"workload": "random %d-byte rows, 16 lanes per row, 4 rows in flight, %d blocks of 512"
                                 % (rb, 512)},
                      "tables": sizes}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", default="C4", help="workload: C1 C2 C2c C3 C4 C5")
    ap.add_argument("--tokens", type=int, default=0,
                    help="token count in place of the workload's own (same recipe; 0 = as defined)")
    ap.add_argument("--sets", type=int, default=0, help="distinct x/out buffer sets to rotate (0 = auto)")
    ap.add_argument("--opt", action="append", default=[], help="library option name=value (repeatable)")
    ap.add_argument("--force-top", type=int, default=0,
                    help="an experiment on the weights, not a workload: the biases of the top K nodes on the rightmost "
                         "path are set so that every token takes the right child there; the batch then lands in "
                         "1/2^K of the tree and the weight rows it gathers shrink by that factor (how much of a "
                         "launch's time is rows that no longer fit an L2)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-dense", action="store_true")
    ap.add_argument("--no-stage-timing", action="store_true")
    ap.add_argument("--no-others", dest="others", action="store_false",
                    help="time only --config (default: the other two of C3, C4, C5 are timed after it and "
                         "reported under \"others\")")
    ap.add_argument("--sweep", choices=["depth", "experts", "widths"], default=None,
                    help="depth: the small-batch latency sweep (time per call against tree depth) instead of a "
                         "workload; experts: the same sweep with the mixture-of-experts lookup (one engaged "
                         "expert) timed beside the tree lookup on the same leaves")
    ap.add_argument("--soft", action="store_true",
                    help="time the soft forward pass (Forward_T: all leaves, dense, MFMA-bound) of --config "
                         "instead of the hard one")
    ap.add_argument("--probe", choices=["gather"], default=None,
                    help="gather: the row-gather microbenchmark (rate of random row fetches against table size)")
    ap.add_argument("--probe-row-bytes", type=int, default=1536)
    ap.add_argument("--block", action="store_true",
                    help="time the pre-norm residual layer with nodes of --node-size hidden neurons "
                         "(fff_forward_block) on the shapes of --config")
    ap.add_argument("--node-size", type=int, default=4)
    ap.add_argument("--sweep-batch", type=int, default=256)
    ap.add_argument("--sweep-leaf-width", type=int, default=32)
    ap.add_argument("--sweep-min-depth", type=int, default=1)
    ap.add_argument("--sweep-max-depth", type=int, default=15)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding, no collectives); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import fff_workloads as W
    import paper_2308_14711_amd as F

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    F.lib()   # fail loudly here if the HIP library is missing
    for kv in args.opt:
        k, v = kv.split("=")
        try:
            F.fff_set_option(k, int(v))
        except F.FffError:
            F.fff_debug_option(k, int(v))      # an experiment switch of the kernels

    if args.sweep == "widths":
        width_sweep(args, np, torch, W, F)
        return

    if args.sweep in ("depth", "experts"):
        depth_sweep(args, np, torch, W, F, with_moe=args.sweep == "experts")
        return

    if args.probe == "gather":
        gather_probe(args, np, torch, F)
        return

    if args.soft:
        soft_bench(args, np, torch, W, F)
        return

    if args.block:
        block_bench(args, np, torch, W, F)
        return

    line = hard_bench(args.config, args, np, torch, W, F, headline=True)
    if args.others and not (args.tokens or args.opt or args.force_top):
        # the other two bandwidth-bound workloads, timed the same way (fewer extras): the default run
        # then covers all three configurations the bandwidth target is stated for
        line["others"] = {}
        for name in ("C3", "C4", "C5"):
            if name == args.config:
                continue
            o = hard_bench(name, args, np, torch, W, F, headline=False)
            line["others"][name] = {"ms_per_step": o["ms_per_step"], "tokens_per_s": o["value"],
                                    "launch_path": o["config"]["launch_path"], "kernels": o["config"]["kernels"],
                                    "alg_bytes": o["path"]["alg_bytes"], "path_frac": o["path"]["frac"],
                                    "path_frac_of_copy_ceiling": o["path"].get("frac_of_copy_ceiling"),
                                    "leaf_occupancy": o["leaf_occupancy"],
                                    "stages": o["stages"], "parity": o["parity"],
                                    "workload": o["config"]["workload"]}
    print(json.dumps(line))


def hard_bench(name, args, np, torch, W, F, headline=True):
    """Time fff_forward_hard on workload `name` and return the JSON line as a dict.  headline=False
    leaves out the CPU baseline legs, the dense comparator and the gather probe (the parity check and
    the per-stage durations stay)."""
    no_cpu = args.no_cpu_baseline or not headline
    no_dense = args.no_dense or not headline
    w = W.config(name, keep_f32=False, T=args.tokens or None)
    tdt = torch.bfloat16 if w.dtype == W.DTYPE_BF16 else torch.float32
    if args.force_top:          # concentrate the routing: a large bias on the top nodes of the rightmost path
        nb = np.array(w.device_array("node_b"), copy=True)
        node = 0
        for _ in range(min(args.force_top, w.depth)):
            nb[node] = 0x42C8 if nb.dtype == np.uint16 else 100.0      # 100.0 as bf16 bits / fp32
            node = 2 * node + 2
        if w.dtype == W.DTYPE_BF16:
            w.bits["node_b"] = nb
        else:
            w.f32["node_b"] = nb

    def up(a):
        a = np.ascontiguousarray(a)
        if a.dtype == np.uint16:
            return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
        return torch.from_numpy(a).cuda()

    dev = {k: up(w.device_array(k)) for k in W.TENSORS}
    nw = dev["node_w"] if w.depth else None
    nb = dev["node_b"] if w.depth else None

    # Rotate distinct x/out buffers so that a working set smaller than the 256 MB
    # last-level cache is not served from it: every set holds the same tokens.
    es = 2 if w.dtype == W.DTYPE_BF16 else 4
    per_set = w.T * (w.D + w.O) * es
    nsets = args.sets or max(1, min(8, int(np.ceil(1.2e9 / max(per_set, 1)))))
    xs = [dev["x"]] + [dev["x"].clone() for _ in range(nsets - 1)]
    outs = [torch.empty((w.T, w.O), dtype=tdt, device="cuda") for _ in range(nsets)]
    idx = torch.empty((w.T,), dtype=torch.int32, device="cuda")
    F.fff_reserve_workspace(w.T, w.depth)

    def step(i):
        j = i % nsets
        F.fff_forward_hard(xs[j], nw, nb, dev["leaf_w1"], dev["leaf_b1"], dev["leaf_w2"], dev["leaf_b2"],
                           w.depth, w.leaf_width, w.act, outs[j], idx)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    tokens_per_s = w.T * args.steps / (t1 - t0)
    kernels = F.fff_last_launch()     # what the timed calls launched, as the library names it

    # routing of the oracle: which nodes and leaves are touched (host side, for the byte model)
    import oracle
    ins = [np.ascontiguousarray(w.device_array(k)) for k in W.TENSORS]
    ref_out, ref_idx, margin = oracle.forward_hard(*ins, w.depth, w.leaf_width, w.act,
                                                   want_out=True)
    cpu_passes, cpu_s = 0, 0.0
    if not no_cpu:       # the oracle as it stands, whole batch, repeated for about 10 s
        t2 = time.perf_counter()
        while cpu_passes < 1 or (time.perf_counter() - t2 < 10.0 and cpu_passes < 400):
            oracle.forward_hard(*ins, w.depth, w.leaf_width, w.act)
            cpu_passes += 1
        cpu_s = time.perf_counter() - t2
    cpu_single = None
    if not no_cpu:       # and on one core, on a prefix of the batch (about a second)
        n1 = min(w.T, 8192)
        ins1 = [np.ascontiguousarray(ins[0][:n1])] + ins[1:]
        all_threads = oracle.num_threads()
        oracle.set_threads(1)
        try:
            t3 = time.perf_counter()
            oracle.forward_hard(*ins1, w.depth, w.leaf_width, w.act)
            cpu_single = {"value": round(n1 / (time.perf_counter() - t3), 1), "unit": "tokens/s", "cores": 1,
                          "sample": "first %d tokens of %s, one pass" % (n1, w.name)}
        finally:
            oracle.set_threads(all_threads)

    # spread of the timing: ten batches of steps / 10 calls, each bracketed by a synchronisation
    per_batch = max(1, args.steps // 10)
    batch_ms = []
    for b in range(10):
        torch.cuda.synchronize()
        tb = time.perf_counter()
        for i in range(per_batch):
            step(b * per_batch + i)
        torch.cuda.synchronize()
        batch_ms.append((time.perf_counter() - tb) * 1e3 / per_batch)
    timing_stats = {"batches": 10, "calls_per_batch": per_batch, "mean_ms": round(float(np.mean(batch_ms)), 5),
                    "std_ms": round(float(np.std(batch_ms)), 5), "median_ms": round(float(np.median(batch_ms)), 5)}

    alg = algorithmic_bytes(w, ref_idx)
    path_names = {1: "fused", 2: "staged", 3: "generic", 4: "token_block", 5: "split"}

    # per-stage durations: HIP events recorded by the library on the call's stream
    stages = {}
    if not args.no_stage_timing:
        F.fff_set_option("stage_timing", 1)
        for i in range(args.steps):
            step(i)
        torch.cuda.synchronize()
        d_ms, b_ms, l_ms, l2_ms, calls = F.fff_stage_times()
        F.fff_set_option("stage_timing", 0)
        single = F.fff_get_option("last_path") not in (2, 5)
        if F.fff_get_option("last_path") == 5:      # walk + hidden neurons per token, then output rows by column slices
            names = (("walk_hidden", d_ms), ("leaf_slices", l_ms))
        elif single:     # one launch did the whole path: it carries the whole path's bytes
            alg = dict(alg, walk_fused=alg["path"], token_block=alg["path"])
            names = ((("token_block" if F.fff_get_option("last_path") == 4 else "walk_fused"), d_ms),)
        elif F.fff_get_option("last_leaf_path") == 2:   # the leaf stage ran as two kernels
            names = (("descent", d_ms), ("bucketing", b_ms), ("leaf_hidden", l_ms), ("leaf_output", l2_ms))
        else:
            names = (("descent", d_ms), ("bucketing", b_ms), ("leaf", l_ms))
        for stage, ms in names:
            avg = ms / max(calls, 1)
            gbs = alg[stage] / (avg * 1e-3) / 1e9 if avg > 0 else 0.0
            stages[stage] = {"avg_ms": round(avg, 5), "alg_bytes": alg[stage], "GBps": round(gbs, 1),
                             "frac": round(gbs / HBM_PEAK_GBS, 4)}
    dom = max(stages, key=lambda k: stages[k]["avg_ms"]) if stages else None
    roofline = None
    if dom:
        # the dominant kernel as the library names it: the stage's position in the call's launches
        names_in_order = [k.strip() for k in kernels.split(" + ")]
        dom_kernel = kernels if len(stages) == 1 else None
        if dom_kernel is None:
            pos = {"descent": 0, "leaf_output": -1, "leaf_hidden": -2, "leaf": -1, "walk_hidden": 0, "leaf_slices": -1}.get(dom)
            dom_kernel = names_in_order[pos] if pos is not None and names_in_order else dom
        measured = None if args.tokens else measured_traffic(w.name, dom_kernel)
        ceiling = copy_ceiling_once(torch)
        roofline = {"bound": "hbm", "kernel": dom, "kernel_launch": dom_kernel, "achieved": stages[dom]["GBps"],
                    "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": stages[dom]["frac"],
                    "traffic": measured["bytes"] if measured else None,
                    "traffic_source": measured["source"] if measured else None,
                    "copy_ceiling_GBps": ceiling["GBps"],
                    "frac_of_copy_ceiling": round(stages[dom]["GBps"] / ceiling["GBps"], 4)}
    path_gbs = alg["path"] / (ms_per_step * 1e-3) / 1e9

    # the fused launch fetches weight rows per token; how fast such rows can come at all depends on
    # whether the weight table fits an L2: measure random row fetches over tables of the next smaller
    # and next larger power-of-two row count (the probe library's fffb_gather) and report the time the launch's
    # gathered rows alone would take at those rates
    if headline and roofline and dom in ("walk_fused", "walk_hidden") and w.O == w.D:
        es = 2 if w.dtype == W.DTYPE_BF16 else 4
        rb = w.D * es
        if rb % 16 == 0:
            top = F.fff_get_option("last_walk_top")
            leaf_rows = 2 * w.leaf_width + 1 if dom == "walk_fused" else w.leaf_width   # W1, W2, b2 / W1 alone
            rows_per_token = (w.depth - top) + leaf_rows                      # plus the node rows past LDS
            table_rows = max(1, alg["u_node"] - ((1 << top) - 1)) + alg["u_leaf"] * leaf_rows
            gathered = float(w.T) * rows_per_token * rb
            sink = torch.zeros((4,), dtype=torch.int32, device="cuda")
            bracket = []
            lo = 1 << max(0, int(np.floor(np.log2(table_rows))))
            for rows in (lo, 2 * lo):
                table = torch.zeros((rows * rb,), dtype=torch.uint8, device="cuda")
                for _ in range(2):
                    nbytes = probe_gather(torch, table, rb, 4, 512, 16, True, sink)
                torch.cuda.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for _ in range(5):
                    probe_gather(torch, table, rb, 4, 512, 16, True, sink)
                e1.record()
                torch.cuda.synchronize()
                rate = nbytes * 5 / (e0.elapsed_time(e1) * 1e-3)
                bracket.append({"table_MB": round(rows * rb / 1e6, 1), "TBps": round(rate / 1e12, 2),
                                "ms_for_gathered_rows": round(gathered / rate * 1e3, 4)})
                del table
            roofline["gather_bound"] = {"weight_rows_MB": round(table_rows * rb / 1e6, 1),
                                        "rows_per_token": rows_per_token, "gathered_bytes": gathered,
                                        "measured_on_tables": bracket}

    # parity spot check of the timed configuration against the oracle
    got_idx = idx.cpu().numpy()
    mism = np.nonzero(got_idx != ref_idx)[0]
    parity = {"idx_mismatch": int(mism.size),
              "idx_mismatch_outside_margin": int((margin[mism] >= 1e-4).sum()),
              "margin_tokens": int((margin < 1e-4).sum())}
    if ref_out is not None:
        got = outs[(args.steps - 1) % nsets].float().cpu().numpy().astype(np.float64)
        keep = got_idx == ref_idx
        scale = np.maximum(np.abs(ref_out[keep]).max(axis=1), 1e-30)
        parity["max_rel_row_err"] = float((np.abs(got[keep] - ref_out[keep]).max(axis=1) / scale).max())

    cpu = None
    if not no_cpu:
        cpu = {"value": round(w.T * cpu_passes / cpu_s, 1), "unit": "tokens/s", "cores": oracle.num_threads(),
               "kind": "oracle",
               "sample": "all %d tokens of %s, %d passes, fp64, OpenMP over tokens" % (w.T, w.name, cpu_passes),
               "seconds": round(cpu_s, 3)}

    dense = None
    if not no_dense and (1 << w.depth) * w.leaf_width <= 8192:
        H = (1 << w.depth) * w.leaf_width          # equal training width
        W1 = dev["leaf_w1"].reshape(H, w.D)
        B1 = dev["leaf_b1"].reshape(H)
        W2 = dev["leaf_w2"].reshape(H, w.O)
        B2 = dev["leaf_b2"][0]
        act = torch.nn.functional.gelu if w.act == W.ACT_GELU else torch.relu

        def dense_step(j):
            h = act(torch.addmm(B1, xs[j], W1.t()))
            torch.addmm(B2, h, W2, out=outs[j])

        for i in range(max(3, args.warmup // 4)):
            dense_step(i % nsets)
        torch.cuda.synchronize()
        n = max(10, args.steps // 4)
        t4 = time.perf_counter()
        for i in range(n):
            dense_step(i % nsets)
        torch.cuda.synchronize()
        dense_ms = (time.perf_counter() - t4) * 1e3 / n
        dense = {"hidden": H, "ms_per_step": round(dense_ms, 4), "speedup": round(dense_ms / ms_per_step, 2),
                 "impl": "torch addmm + activation + addmm, same dtype"}

    line = {
        "metric": "fff_hard_inference_tokens_per_s", "value": round(tokens_per_s, 1), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if w.dtype == W.DTYPE_BF16 else "f32", "data": "synthetic",
        "config": {"workload": "%s: %s" % (w.name, w.note), "T": w.T, "D": w.D, "O": w.O, "depth": w.depth,
                   "leaf_width": w.leaf_width, "act": "gelu" if w.act else "relu", "buffer_sets": nsets,
                   "seed": 0, "options": args.opt, "force_top": args.force_top,
                   "launch_path": path_names.get(F.fff_get_option("last_path"), "?"), "kernels": kernels},
        "roofline": roofline,
        "path": {"alg_bytes": alg["path"], "GBps": round(path_gbs, 1), "frac": round(path_gbs / HBM_PEAK_GBS, 4),
                 "frac_of_copy_ceiling": round(path_gbs / copy_ceiling_once(torch)["GBps"], 4),
                 "u_node": alg["u_node"], "u_leaf": alg["u_leaf"]},
        "leaf_occupancy": alg["occupancy"],
        "copy_ceiling": copy_ceiling_once(torch),
        "stages": stages,
        "timing_stats": timing_stats,
        "cpu_baseline": cpu,
        "cpu_baseline_one_core": cpu_single,
        "dense_ff": dense,
        "parity": parity,
    }
    del dev, xs, outs, idx
    torch.cuda.empty_cache()
    return line


if __name__ == "__main__":
    main()
