"""GPU parity of the mixture-of-experts comparator (one engaged expert, noiseless gating) against
the CPU oracle, through the C ABI: the gating index bit-exact outside the margin, inside it still
a near-maximal logit; output rows within the same tolerance as the FFF path."""
import numpy as np
import pytest

import fff_workloads as W
import oracle
from fff_testlib import TOL, ROUTING_MARGIN, out_to_f64, to_device

pytestmark = pytest.mark.gpu

CASES = [
    # name,            T,    D,   O,  log2 experts, L, bias
    ("latency_g2",     256,  768, 768, 1,  32, True),
    ("latency_g32",    256,  768, 768, 5,  32, False),
    ("latency_g512",   256,  768, 768, 9,  32, True),
    ("one_chunk",      70,   64,  16,  1,  2,  True),
    ("k_tail",         333,  200, 40,  7,  8,  True),
    ("ragged_experts", 100,  128, 64,  0,  4,  False),
    ("bucketed",       5000, 256, 128, 6,  4,  True),
    ("bucketed_wide",  9000, 768, 768, 3,  32, False),
    ("many_experts",   129,  96,  24,  12, 1,  True),
    # the end point of the paper's sweep (section "Inference speed comparison": 768-wide, experts of 32
    # neurons, batch 256, up to 2^15 experts), at full size
    ("sweep_end",      256,  768, 768, 15, 32, True),
]


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_moe_top1_against_the_oracle(case):
    import torch
    import paper_2308_14711_amd as F
    name, T, D, O, g, L, bias = case
    print("\n[case] moe %s T=%d D=%d O=%d experts=2^%d L=%d bias=%s seed 3" % (name, T, D, O, g, L, bias), flush=True)
    w = W.make_layer(name, T, D, O, g, L, W.ACT_GELU, W.DTYPE_BF16, seed=3, keep_f32=g < 14)
    gw, gb = W.moe_gate(1 << g, D, W.DTYPE_BF16, seed=3)
    dev = to_device(w)
    up = lambda a: torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    d_gw, d_gb = up(gw), (up(gb) if bias else None)
    out = torch.full((T, O), float("nan"), dtype=torch.bfloat16, device="cuda")
    idx = torch.full((T,), -5, dtype=torch.int32, device="cuda")
    F.fff_moe_top1_forward(dev["x"], d_gw, d_gb, dev["leaf_w1"], dev["leaf_b1"], dev["leaf_w2"], dev["leaf_b2"],
                           g, L, w.act, out, idx)
    torch.cuda.synchronize()
    took = F.fff_get_option("last_path")
    ins = [w.bits[k] for k in ("leaf_w1", "leaf_b1", "leaf_w2", "leaf_b2")]
    ref_out, ref_idx, margin = oracle.moe_top1(w.bits["x"], gw, gb if bias else None, *ins, L, w.act)
    gi = idx.cpu().numpy()
    assert gi.min() >= 0 and gi.max() < (1 << g)
    diff = np.nonzero(gi != ref_idx)[0]
    assert (margin[diff] < ROUTING_MARGIN).all(), "gating differs outside the margin at tokens %s" % diff[:5]
    if diff.size:        # inside the margin the expert taken must still have a near-maximal logit
        x64 = W.bf16_widen(w.bits["x"]).astype(np.float64)
        g64 = W.bf16_widen(gw).astype(np.float64)
        b64 = W.bf16_widen(gb).astype(np.float64) if bias else np.zeros(1 << g)
        for t in diff:
            logits = g64 @ x64[t] + b64
            scale = np.abs(g64[gi[t]] * x64[t]).sum() + abs(b64[gi[t]])
            assert logits.max() - logits[gi[t]] <= ROUTING_MARGIN * scale
    # rows against the oracle's expert networks evaluated at the experts the GPU took
    at_gpu = oracle.leaf_forward(w.bits["x"], *ins, gi, g, L, w.act)
    got = out_to_f64(out)
    assert np.isfinite(got).all()
    err = np.abs(got - at_gpu).max(axis=1) / np.maximum(np.abs(at_gpu).max(axis=1), 1e-30)
    assert err.max() <= TOL[W.DTYPE_BF16], "row error %.3e" % err.max()
    same = gi == ref_idx
    assert np.array_equal(at_gpu[same], ref_out[same])
    print("  moe %s: path %d, %d margin tokens, %d gated differently, max row error %.2e" % (
        name, took, int((margin < ROUTING_MARGIN).sum()), int(diff.size), err.max()), flush=True)


def test_moe_without_an_index_buffer_and_twice():
    """expert_idx is optional, and a second call with other sizes reuses the workspace."""
    import torch
    import paper_2308_14711_amd as F
    for T, g in ((300, 4), (200, 8)):
        w = W.make_layer("moe_noidx", T, 128, 64, g, 4, W.ACT_RELU, W.DTYPE_BF16, seed=4)
        gw, gb = W.moe_gate(1 << g, 128, W.DTYPE_BF16, seed=4)
        dev = to_device(w)
        up = lambda a: torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
        out = torch.full((T, 64), float("nan"), dtype=torch.bfloat16, device="cuda")
        F.fff_moe_top1_forward(dev["x"], up(gw), up(gb), dev["leaf_w1"], dev["leaf_b1"], dev["leaf_w2"],
                               dev["leaf_b2"], g, 4, w.act, out, None)
        torch.cuda.synchronize()
        ins = [w.bits[k] for k in ("leaf_w1", "leaf_b1", "leaf_w2", "leaf_b2")]
        ref_out, ref_idx, margin = oracle.moe_top1(w.bits["x"], gw, gb, *ins, 4, w.act)
        got = out_to_f64(out)
        safe = margin >= ROUTING_MARGIN
        err = np.abs(got[safe] - ref_out[safe]).max(axis=1) / np.maximum(np.abs(ref_out[safe]).max(axis=1), 1e-30)
        assert err.max() <= TOL[W.DTYPE_BF16]


def test_leaf_stage_alone_on_a_small_batch():
    """fff_leaf_forward on a small batch takes the one-block-per-token launch with given leaves."""
    import torch
    import paper_2308_14711_amd as F
    w = W.make_layer("leaf_small", 300, 256, 96, 5, 12, W.ACT_GELU, W.DTYPE_BF16, seed=6)
    dev = to_device(w)
    rng = np.random.default_rng(6)
    li = rng.integers(0, 32, w.T).astype(np.int32)
    out = torch.full((w.T, w.O), float("nan"), dtype=torch.bfloat16, device="cuda")
    F.fff_leaf_forward(dev["x"], dev["leaf_w1"], dev["leaf_b1"], dev["leaf_w2"], dev["leaf_b2"],
                       torch.from_numpy(li).cuda(), w.depth, w.leaf_width, w.act, out)
    torch.cuda.synchronize()
    ref = oracle.leaf_forward(w.bits["x"], w.bits["leaf_w1"], w.bits["leaf_b1"], w.bits["leaf_w2"], w.bits["leaf_b2"],
                              li, w.depth, w.leaf_width, w.act)
    got = out_to_f64(out)
    err = np.abs(got - ref).max(axis=1) / np.maximum(np.abs(ref).max(axis=1), 1e-30)
    assert err.max() <= TOL[W.DTYPE_BF16]
