"""Pins of the oracle's mixture-of-experts function (one engaged expert, noiseless gating: the
configuration of the paper's inference speed comparison).  Each checks it against something other
than itself: a hand-worked example, scalar compares, the already pinned FFF forward pass, library
routines on tiny inputs, and the invariants the definition implies.  CPU only."""
import json
import os

import numpy as np

import oracle

HERE = os.path.dirname(os.path.abspath(__file__))


def _experts(rng, G, L, D, O):
    return (rng.normal(size=(G, L, D)), rng.normal(size=(G, L)), rng.normal(size=(G, L, O)), rng.normal(size=(G, O)))


def test_moe_hand_worked_example():
    g = json.load(open(os.path.join(HERE, "golden", "moe_hand_example.json")))
    a = {k: np.array(v, dtype=np.float64) for k, v in g.items() if not k.startswith("_")}
    out, idx, margin = oracle.moe_top1(a["x"], a["gate_w"], a["gate_b"], a["leaf_w1"], a["leaf_b1"], a["leaf_w2"],
                                       a["leaf_b2"], 1, oracle.ACT_RELU)
    assert idx.tolist() == g["expert_idx"]
    assert np.allclose(out, a["out"], rtol=0, atol=1e-15)
    assert np.allclose(margin, a["margin"], rtol=1e-15, atol=0)


def test_moe_one_hot_gates_pick_by_scalar_compares():
    """Gating row e is s_e times a unit vector: its logit is one product plus the bias, so the
    winner follows from scalar arithmetic alone (adding exact zeros changes nothing in fp64)."""
    rng = np.random.default_rng(21)
    T, D, O, G, L = 400, 12, 4, 9, 2
    x = rng.normal(size=(T, D))
    axis = rng.integers(0, D, G)
    s = rng.normal(size=G)
    gb = rng.normal(size=G)
    gw = np.zeros((G, D))
    gw[np.arange(G), axis] = s
    w1, b1, w2, b2 = _experts(rng, G, L, D, O)
    _, idx, _ = oracle.moe_top1(x, gw, gb, w1, b1, w2, b2, L, oracle.ACT_GELU, want_out=False)
    for t in range(T):
        logits = [gb[e] + s[e] * x[t, axis[e]] for e in range(G)]
        assert idx[t] == max(range(G), key=lambda e: (logits[e], -e))


def test_moe_with_two_experts_is_a_depth_one_fff():
    """Experts (0, 1) gated by logits (0, w.x + b) behave like the two leaves under one node
    with weights (w, b), except on the tie (a node sends logit 0 right, the argmax keeps the
    lower index): the FFF forward pass is pinned on its own."""
    rng = np.random.default_rng(22)
    T, D, O, L = 300, 10, 6, 3
    x = rng.normal(size=(T, D))
    w = rng.normal(size=(1, D))
    b = rng.normal(size=(1,))
    w1, b1, w2, b2 = _experts(rng, 2, L, D, O)
    ref_out, ref_idx, _ = oracle.forward_hard(x, w, b, w1, b1, w2, b2, 1, L, oracle.ACT_GELU)
    gw = np.concatenate([np.zeros((1, D)), w])
    gb = np.concatenate([np.zeros(1), b])
    out, idx, _ = oracle.moe_top1(x, gw, gb, w1, b1, w2, b2, L, oracle.ACT_GELU)
    clear = np.abs(x @ w[0] + b[0]) > 1e-9
    assert clear.sum() > T - 5
    assert np.array_equal(idx[clear], ref_idx[clear])
    assert np.array_equal(out[clear], ref_out[clear])      # same expert, same arithmetic: bit-equal


def test_moe_matches_library_argmax_and_dense_expert_on_tiny_inputs():
    rng = np.random.default_rng(23)
    T, D, O, G, L = 120, 7, 5, 13, 4
    x = rng.normal(size=(T, D))
    gw = rng.normal(size=(G, D))
    w1, b1, w2, b2 = _experts(rng, G, L, D, O)
    for gb in (None, rng.normal(size=G)):
        out, idx, margin = oracle.moe_top1(x, gw, gb, w1, b1, w2, b2, L, oracle.ACT_RELU)
        logits = x @ gw.T + (0.0 if gb is None else gb)
        srt = np.sort(logits, axis=1)
        clear = srt[:, -1] - srt[:, -2] > 1e-9
        assert np.array_equal(idx[clear], np.argmax(logits, axis=1)[clear])
        for t in range(T):
            e = idx[t]
            h = np.maximum(w1[e] @ x[t] + b1[e], 0.0)
            assert np.allclose(out[t], w2[e].T @ h + b2[e], rtol=1e-12, atol=1e-12)
        # the margin is the gap of the two largest logits over the larger row scale
        t = int(np.argmin(margin))
        order = np.argsort(logits[t])
        e1, e2 = order[-1], order[-2]
        sc = max(np.abs(gw[e] * x[t]).sum() + (0.0 if gb is None else abs(gb[e])) for e in (e1, e2))
        assert np.isclose(margin[t], (logits[t, e1] - logits[t, e2]) / sc, rtol=1e-9)


def test_moe_identical_experts_make_gating_irrelevant():
    rng = np.random.default_rng(24)
    T, D, O, G, L = 80, 9, 4, 6, 3
    x = rng.normal(size=(T, D))
    gw = rng.normal(size=(G, D))
    w1, b1, w2, b2 = _experts(rng, 1, L, D, O)
    rep = lambda a: np.repeat(a, G, axis=0)
    out, idx, _ = oracle.moe_top1(x, gw, None, rep(w1), rep(b1), rep(w2), rep(b2), L, oracle.ACT_GELU)
    assert len(set(idx.tolist())) > 1
    v = x @ w1[0].T + b1[0]
    from math import erf, sqrt
    h = 0.5 * v * (1.0 + np.vectorize(erf)(v / sqrt(2.0)))
    assert np.allclose(out, h @ w2[0] + b2[0], rtol=1e-12, atol=1e-12)


def test_moe_expert_permutation_permutes_the_indices_only():
    rng = np.random.default_rng(25)
    T, D, O, G, L = 150, 8, 3, 10, 2
    x = rng.normal(size=(T, D))
    gw = rng.normal(size=(G, D))
    gb = rng.normal(size=G)
    w1, b1, w2, b2 = _experts(rng, G, L, D, O)
    out, idx, _ = oracle.moe_top1(x, gw, gb, w1, b1, w2, b2, L, oracle.ACT_RELU)
    p = rng.permutation(G)                      # new expert i is old expert p[i]
    out2, idx2, _ = oracle.moe_top1(x, gw[p], gb[p], w1[p], b1[p], w2[p], b2[p], L, oracle.ACT_RELU)
    assert np.array_equal(p[idx2], idx)
    assert np.array_equal(out2, out)


def test_moe_ties_take_the_lowest_index_and_nan_never_wins():
    rng = np.random.default_rng(26)
    T, D, O, G, L = 40, 6, 3, 5, 2
    x = rng.normal(size=(T, D))
    row = rng.normal(size=D)
    gw = np.stack([row * 0.5, row, row, row * 0.5, row])       # experts 1, 2, 4 tie wherever row.x > 0
    w1, b1, w2, b2 = _experts(rng, G, L, D, O)
    _, idx, margin = oracle.moe_top1(x, gw, None, w1, b1, w2, b2, L, oracle.ACT_RELU, want_out=False)
    pos = x @ row > 0
    assert (idx[pos] == 1).all() and (idx[~pos] == 0).all()     # negative: 0.5 * row.x is the largest, experts 0 and 3
    assert (margin == 0).all()
    gb = np.array([0.0, np.nan, 0.0, 0.0, 0.0])
    _, idx, _ = oracle.moe_top1(x, gw, gb, w1, b1, w2, b2, L, oracle.ACT_RELU, want_out=False)
    assert (idx[pos] == 2).all()
    _, idx, _ = oracle.moe_top1(x, gw, np.full(G, np.nan), w1, b1, w2, b2, L, oracle.ACT_RELU, want_out=False)
    assert (idx == 0).all()


def test_moe_bf16_bits_are_widened_exactly():
    import fff_workloads as W
    rng = np.random.default_rng(27)
    T, D, O, G, L = 60, 16, 8, 8, 2
    arrs = [rng.normal(size=s).astype(np.float32) for s in ((T, D), (G, D), (G,), (G, L, D), (G, L), (G, L, O), (G, O))]
    bits = [W.bf16_round(a) for a in arrs]
    wide = [W.bf16_widen(b).astype(np.float64) for b in bits]
    a = oracle.moe_top1(*bits, L, oracle.ACT_GELU)
    b = oracle.moe_top1(*wide, L, oracle.ACT_GELU)
    for u, v in zip(a, b):
        assert np.array_equal(u, v)
