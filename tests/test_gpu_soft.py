"""GPU parity of the soft forward pass (Forward_T of Algorithm 1) against the CPU oracle, through
the C ABI: output rows, the mixture weights over the leaves, and the batch mean entropy of the
node choice scores."""
import numpy as np
import pytest

import fff_workloads as W
import oracle
from fff_testlib import TOL, oracle_inputs, out_to_f64, to_device

pytestmark = pytest.mark.gpu

CASES = [
    # name,          T,    D,   O,   depth, L, act
    ("small",        300,  64,  48,  4, 3,  W.ACT_GELU),
    ("depth0",       130,  128, 136, 0, 5,  W.ACT_RELU),
    ("k_tail_deep",  200,  200, 24,  6, 2,  W.ACT_GELU),
    ("bert_rows",    65,   768, 768, 3, 8,  W.ACT_GELU),
    ("wide_leaves",  1000, 96,  40,  2, 32, W.ACT_RELU),
    ("one_token",    1,    64,  8,   5, 1,  W.ACT_GELU),
    ("odd_k2",       77,   72,  200, 1, 2,  W.ACT_GELU),      # 2 leaves x 3 columns = 6, padded to 8
    # batches of 2048 rows or more take the 128 x 256 tile: ragged in rows, columns and K; then whole tiles
    ("big_ragged",   2100, 200, 300, 7, 5,  W.ACT_GELU),
    ("big_whole",    2304, 128, 256, 8, 1,  W.ACT_RELU),
    ("big_shallow",  2200, 96,  24,  2, 4,  W.ACT_GELU),      # three nodes in the fused nodes + mixture launch
    ("big_deep",     2050, 64,  40,  9, 1,  W.ACT_RELU),      # 511 nodes: two column tiles, separate mixture kernel
    ("big_deeper",   2048, 64,  16,  11, 1, W.ACT_GELU),      # 2048 leaves: 64 KB of LDS in the mixture kernel
    ("per_leaf_mix", 300,  64,  16,  12, 1, W.ACT_RELU),      # 4096 leaves: the per-leaf mixture kernel
]


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_forward_soft_against_the_oracle(case):
    import torch
    import paper_2308_14711_amd as F
    name, T, D, O, depth, L, act = case
    print("\n[case] soft %s T=%d D=%d O=%d depth=%d L=%d act=%d seed 21" % (name, T, D, O, depth, L, act), flush=True)
    w = W.make_layer(name, T, D, O, depth, L, act, W.DTYPE_BF16, seed=21)
    dev = to_device(w)
    NL, NN = 1 << depth, (1 << depth) - 1
    out = torch.full((T, O), float("nan"), dtype=torch.bfloat16, device="cuda")
    mix = torch.full((T, NL), float("nan"), dtype=torch.float32, device="cuda")
    ent = torch.full((max(NN, 1),), float("nan"), dtype=torch.float32, device="cuda")
    nw = dev["node_w"] if depth else None
    nb = dev["node_b"] if depth else None
    for rep in range(2):        # twice: the second call reuses the workspace
        F.fff_forward_soft(dev["x"], nw, nb, dev["leaf_w1"], dev["leaf_b1"], dev["leaf_w2"], dev["leaf_b2"],
                           depth, L, act, out, mix, ent if depth else None)
        torch.cuda.synchronize()
    ref_out, ref_mix = oracle.forward_soft(*oracle_inputs(w), depth, L, act)
    got = out_to_f64(out)
    assert np.isfinite(got).all()
    err = np.abs(got - ref_out).max(axis=1) / np.maximum(np.abs(ref_out).max(axis=1), 1e-30)
    gm = mix.cpu().numpy().astype(np.float64)
    mix_err = np.abs(gm - ref_mix).max()
    assert mix_err <= 1e-4, "mixture weights off by %.3e" % mix_err
    assert np.allclose(gm.sum(axis=1), 1.0, atol=1e-4)
    assert err.max() <= TOL[W.DTYPE_BF16], "row error %.3e" % err.max()
    ent_err = 0.0
    if depth:
        ref_ent = oracle.node_entropy(w.bits["x"], w.bits["node_w"], w.bits["node_b"], depth)
        ent_err = np.abs(ent.cpu().numpy().astype(np.float64) - ref_ent).max()
        assert ent_err <= 1e-4, "entropies off by %.3e" % ent_err
    print("  soft %s: max row error %.2e, mixture %.1e, entropy %.1e" % (name, err.max(), mix_err, ent_err), flush=True)


def _random_soft_cases():
    rng = np.random.default_rng(2024)
    cases = []
    for i in range(8):
        depth = int(rng.integers(1, 10))
        L = int(rng.integers(1, 7))
        cases.append(("random%d" % i, int(rng.integers(2048, 3200)), 8 * int(rng.integers(2, 40)),
                      8 * int(rng.integers(1, 50)), depth, L, int(rng.integers(0, 2))))
    return cases


@pytest.mark.parametrize("case", _random_soft_cases(), ids=lambda c: c[0])
def test_forward_soft_on_seeded_random_shapes_that_take_the_large_tiles(case):
    """Batches of 2048 rows and more (the 128 x 256 tile wherever the widths fill it, the 64 x 128 tile
    elsewhere, the fused or the separate mixture launch by depth) against the oracle."""
    import torch
    import paper_2308_14711_amd as F
    name, T, D, O, depth, L, act = case
    print("\n[case] soft %s T=%d D=%d O=%d depth=%d L=%d act=%d seed 77" % (name, T, D, O, depth, L, act), flush=True)
    w = W.make_layer(name, T, D, O, depth, L, act, W.DTYPE_BF16, seed=77)
    dev = to_device(w)
    NL, NN = 1 << depth, (1 << depth) - 1
    out = torch.full((T, O), float("nan"), dtype=torch.bfloat16, device="cuda")
    mix = torch.full((T, NL), float("nan"), dtype=torch.float32, device="cuda")
    ent = torch.full((NN,), float("nan"), dtype=torch.float32, device="cuda")
    F.fff_forward_soft(dev["x"], dev["node_w"], dev["node_b"], dev["leaf_w1"], dev["leaf_b1"], dev["leaf_w2"],
                       dev["leaf_b2"], depth, L, act, out, mix, ent)
    torch.cuda.synchronize()
    launched = F.fff_last_launch()
    ref_out, ref_mix = oracle.forward_soft(*oracle_inputs(w), depth, L, act)
    got = out_to_f64(out)
    assert np.isfinite(got).all()
    err = np.abs(got - ref_out).max(axis=1) / np.maximum(np.abs(ref_out).max(axis=1), 1e-30)
    mix_err = np.abs(mix.cpu().numpy().astype(np.float64) - ref_mix).max()
    ref_ent = oracle.node_entropy(w.bits["x"], w.bits["node_w"], w.bits["node_b"], depth)
    ent_err = np.abs(ent.cpu().numpy().astype(np.float64) - ref_ent).max()
    print("  soft %s: %s: max row error %.2e, mixture %.1e, entropy %.1e" % (name, launched, err.max(), mix_err, ent_err),
          flush=True)
    assert mix_err <= 1e-4 and ent_err <= 1e-4
    assert err.max() <= TOL[W.DTYPE_BF16], "row error %.3e" % err.max()
    assert ("soft_nodes_mix_kernel" in launched) == (depth <= 8)


def test_mixture_weights_into_a_buffer_that_is_only_4_byte_aligned():
    """The fused nodes + mixture launch stores a lane's four weights as one 16-byte piece when the caller's
    matrix allows it; a matrix that starts 4 bytes into an allocation takes the scalar stores: same bits."""
    import torch
    import paper_2308_14711_amd as F
    T, D, O, depth, L = 2304, 64, 32, 8, 1
    w = W.make_layer("mix_align", T, D, O, depth, L, W.ACT_RELU, W.DTYPE_BF16, seed=5)
    dev = to_device(w)
    NL = 1 << depth
    out = torch.empty((T, O), dtype=torch.bfloat16, device="cuda")
    aligned = torch.full((T, NL), float("nan"), dtype=torch.float32, device="cuda")
    backing = torch.full((T * NL + 4,), float("nan"), dtype=torch.float32, device="cuda")
    shifted = backing[1:1 + T * NL].view(T, NL)
    assert shifted.data_ptr() % 16 == 4
    for mix in (aligned, shifted):
        F.fff_forward_soft(dev["x"], dev["node_w"], dev["node_b"], dev["leaf_w1"], dev["leaf_b1"], dev["leaf_w2"],
                           dev["leaf_b2"], depth, L, w.act, out, mix, None)
    torch.cuda.synchronize()
    assert "soft_nodes_mix_kernel" in F.fff_last_launch()
    assert bool(torch.isfinite(shifted).all())
    assert torch.equal(aligned, shifted)
    assert bool(torch.isnan(backing[0])) and bool(torch.isnan(backing[1 + T * NL:]).all())


def test_forward_soft_at_the_vit_block_size():
    """The soft pass at the full size of the ViT-block workload (50432 tokens against all 256 leaves), in
    the launch configuration the benchmark times: output rows and mixture weights on a strided sample of
    1024 tokens the oracle computes one by one, every row finite, the weights of every token a stochastic
    vector, and the per-node entropies (a mean over the whole batch) against the oracle over all tokens."""
    import torch
    import paper_2308_14711_amd as F
    w = W.config("C3", keep_f32=False)
    print("\n[case] soft C3 full size T=%d D=%d depth=%d L=%d" % (w.T, w.D, w.depth, w.leaf_width), flush=True)
    dev = to_device(w)
    NL, NN = 1 << w.depth, (1 << w.depth) - 1
    out = torch.full((w.T, w.O), float("nan"), dtype=torch.bfloat16, device="cuda")
    mix = torch.full((w.T, NL), float("nan"), dtype=torch.float32, device="cuda")
    ent = torch.full((NN,), float("nan"), dtype=torch.float32, device="cuda")
    F.fff_forward_soft(dev["x"], dev["node_w"], dev["node_b"], dev["leaf_w1"], dev["leaf_b1"], dev["leaf_w2"],
                       dev["leaf_b2"], w.depth, w.leaf_width, w.act, out, mix, ent)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(out.float()).all()) and bool(torch.isfinite(mix).all())
    sums = mix.sum(dim=1)
    assert float((sums - 1.0).abs().max()) <= 1e-4 and float(mix.min()) >= 0.0
    sel = np.arange(0, w.T, w.T // 1024)[:1024]
    ins = oracle_inputs(w)
    ins[0] = np.ascontiguousarray(ins[0][sel])
    ref_out, ref_mix = oracle.forward_soft(*ins, w.depth, w.leaf_width, w.act)
    tsel = torch.from_numpy(sel).cuda()
    got = out_to_f64(out[tsel])
    err = np.abs(got - ref_out).max(axis=1) / np.maximum(np.abs(ref_out).max(axis=1), 1e-30)
    mix_err = np.abs(mix[tsel].cpu().numpy().astype(np.float64) - ref_mix).max()
    assert mix_err <= 1e-4, "mixture weights off by %.3e" % mix_err
    assert err.max() <= TOL[W.DTYPE_BF16], "row error %.3e" % err.max()
    ref_ent = oracle.node_entropy(w.bits["x"], w.bits["node_w"], w.bits["node_b"], w.depth)
    ent_err = np.abs(ent.cpu().numpy().astype(np.float64) - ref_ent).max()
    assert ent_err <= 1e-4, "entropies off by %.3e" % ent_err
    print("  soft C3: max row error %.2e on %d sampled rows, mixture %.1e, entropy %.1e" % (
        err.max(), sel.size, mix_err, ent_err), flush=True)


def test_forward_soft_without_optional_outputs_and_after_hardening():
    """mix and entropy are optional; with node weights scaled up the soft pass approaches the hard one."""
    import torch
    import paper_2308_14711_amd as F
    w = W.make_layer("soft_hard", 400, 128, 64, 4, 4, W.ACT_GELU, W.DTYPE_BF16, seed=22)
    # harden: scale the node weights and biases by 2^10 (exact in bf16)
    for k in ("node_w", "node_b"):
        w.f32[k] = w.f32[k] * 1024.0
        w.bits[k] = W.bf16_round(w.f32[k])
    dev = to_device(w)
    out = torch.full((w.T, w.O), float("nan"), dtype=torch.bfloat16, device="cuda")
    F.fff_forward_soft(dev["x"], dev["node_w"], dev["node_b"], dev["leaf_w1"], dev["leaf_b1"], dev["leaf_w2"],
                       dev["leaf_b2"], w.depth, w.leaf_width, w.act, out)
    hard = torch.empty_like(out)
    F.fff_forward_hard(dev["x"], dev["node_w"], dev["node_b"], dev["leaf_w1"], dev["leaf_b1"], dev["leaf_w2"],
                       dev["leaf_b2"], w.depth, w.leaf_width, w.act, hard, None)
    torch.cuda.synchronize()
    ref_out, ref_mix = oracle.forward_soft(*oracle_inputs(w), w.depth, w.leaf_width, w.act)
    got = out_to_f64(out)
    err = np.abs(got - ref_out).max(axis=1) / np.maximum(np.abs(ref_out).max(axis=1), 1e-30)
    assert err.max() <= TOL[W.DTYPE_BF16]
    decided = ref_mix.max(axis=1) > 0.999999          # tokens whose every decision is saturated
    assert decided.sum() > w.T // 2
    h = out_to_f64(hard)
    gap = np.abs(got[decided] - h[decided]).max(axis=1) / np.maximum(np.abs(h[decided]).max(axis=1), 1e-30)
    assert gap.max() <= TOL[W.DTYPE_BF16]
