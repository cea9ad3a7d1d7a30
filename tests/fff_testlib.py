"""Shared helpers of the GPU parity tests: upload a workload, run the HIP
library through its C ABI, compare with the CPU oracle."""
import numpy as np

import fff_workloads as W
import oracle

ROUTING_MARGIN = 1e-4          # relative node-logit margin below which routing may differ
TOL = {W.DTYPE_F32: 1e-5, W.DTYPE_BF16: 2e-2}   # max row error / max |row| of the oracle


def to_device(w: W.Workload):
    import torch
    dev = {}
    for k in W.TENSORS:
        a = np.ascontiguousarray(w.device_array(k))
        t = torch.from_numpy(a.view(np.int16) if a.dtype == np.uint16 else a)
        t = t.cuda()
        dev[k] = t.view(torch.bfloat16) if a.dtype == np.uint16 else t
    return dev


def run_forward(w: W.Workload, dev=None, want_idx=True, stream=None):
    import torch
    import paper_2308_14711_amd as F
    dev = dev or to_device(w)
    out = torch.empty((w.T, w.O), dtype=dev["x"].dtype, device="cuda")
    out.fill_(float("nan"))
    idx = torch.full((w.T,), -7, dtype=torch.int32, device="cuda") if want_idx else None
    nw = dev["node_w"] if w.depth > 0 else None
    nb = dev["node_b"] if w.depth > 0 else None
    F.fff_forward_hard(dev["x"], nw, nb, dev["leaf_w1"], dev["leaf_b1"], dev["leaf_w2"], dev["leaf_b2"],
                       w.depth, w.leaf_width, w.act, out, idx, stream)
    torch.cuda.synchronize()
    return out, idx


def out_to_f64(out) -> np.ndarray:
    return out.float().cpu().numpy().astype(np.float64)


def oracle_inputs(w: W.Workload):
    return [np.ascontiguousarray(w.device_array(k)) for k in W.TENSORS]


def node_path_ok(w: W.Workload, t: int, leaf: int) -> bool:
    """Is `leaf` a legitimate destination of token t: at every node of its path the
    decision either agrees with the fp64 logit or that logit is inside the margin."""
    x = w.f32["x"][t].astype(np.float64)
    for m in range(w.depth):
        n = leaf >> (w.depth - m)
        row = (1 << m) - 1 + n
        terms = w.f32["node_w"][row].astype(np.float64) * x
        b = float(w.f32["node_b"][row])
        logit = terms.sum() + b
        bit = (leaf >> (w.depth - 1 - m)) & 1
        if (logit >= 0) != bool(bit):
            if abs(logit) >= ROUTING_MARGIN * (np.abs(terms).sum() + abs(b)):
                return False
    return True


def check_against_oracle(w: W.Workload, out_gpu, idx_gpu, ref=None):
    """Element-by-element parity.  Returns a dict of statistics; asserts the bar:
    leaf indices bit-exact outside the routing margin (inside it the GPU's leaf must
    still be a legitimate path), outputs within TOL of the oracle evaluated at the
    leaf the GPU took."""
    ins = oracle_inputs(w)
    if ref is None:
        ref = oracle.forward_hard(*ins, w.depth, w.leaf_width, w.act)
    ref_out, ref_idx, margin = ref
    got = out_to_f64(out_gpu)
    assert got.shape == ref_out.shape
    assert np.isfinite(got).all(), "output rows left unwritten or non-finite"
    stats = {"tokens": w.T, "margin_tokens": int((margin < ROUTING_MARGIN).sum()), "idx_mismatch": 0}
    if idx_gpu is not None:
        gi = idx_gpu.cpu().numpy()
        assert gi.dtype == np.int32 and gi.min(initial=0) >= 0 and gi.max(initial=0) < w.n_leaves
        diff = np.nonzero(gi != ref_idx)[0]
        stats["idx_mismatch"] = int(diff.size)
        bad = [int(t) for t in diff if margin[t] >= ROUTING_MARGIN]
        assert not bad, "routing differs outside the margin at tokens %s" % bad[:8]
        if diff.size:
            assert "node_w" in w.f32, "need fp32 copies to validate margin tokens"
            for t in diff:
                assert node_path_ok(w, int(t), int(gi[t])), "token %d took an illegitimate path" % t
            sub = [a[diff] if i == 0 else a for i, a in enumerate(ins)]
            redo = oracle.leaf_forward(sub[0], ins[3], ins[4], ins[5], ins[6], gi[diff], w.depth,
                                       w.leaf_width, w.act)
            ref_out = ref_out.copy()
            ref_out[diff] = redo
    else:
        # without leaf_idx from the GPU, margin tokens cannot be re-evaluated: compare the rest
        keep = margin >= ROUTING_MARGIN
        got, ref_out = got[keep], ref_out[keep]
    scale = np.maximum(np.abs(ref_out).max(axis=1), 1e-30)
    err = np.abs(got - ref_out).max(axis=1) / scale
    stats["max_rel_row_err"] = float(err.max(initial=0.0))
    stats["l2_rel_err"] = float(np.linalg.norm(got - ref_out) / max(np.linalg.norm(ref_out), 1e-30))
    tol = TOL[w.dtype]
    worst = int(np.argmax(err)) if err.size else -1
    assert stats["max_rel_row_err"] <= tol, "row %d off by %.3e (tolerance %.1e)" % (worst, err[worst], tol)
    return stats
