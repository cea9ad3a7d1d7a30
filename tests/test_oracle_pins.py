"""Pins for the CPU oracle: it is checked against what the paper and the
mathematics fix, never against itself or the HIP path.

Each test names the mistake it is meant to catch.
"""
import json
import os

import numpy as np
import pytest
from scipy.special import ndtr

import oracle
from oracle import ACT_GELU, ACT_RELU

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rand_layer(rng, T, D, O, depth, L, dtype=np.float64, node_bias=True):
    NN, NL = (1 << depth) - 1, 1 << depth
    x = rng.standard_normal((T, D)).astype(dtype)
    nw = rng.uniform(-1, 1, (NN, D)).astype(dtype)
    nb = (rng.uniform(-0.5, 0.5, (NN,)) if node_bias else np.zeros(NN)).astype(dtype)
    w1 = rng.uniform(-1, 1, (NL, L, D)).astype(dtype)
    b1 = rng.uniform(-1, 1, (NL, L)).astype(dtype)
    w2 = rng.uniform(-1, 1, (NL, L, O)).astype(dtype)
    b2 = rng.uniform(-1, 1, (NL, O)).astype(dtype)
    return x, nw, nb, w1, b1, w2, b2


def np_act(v, act):
    return np.maximum(v, 0.0) if act == ACT_RELU else v * ndtr(v)


def np_leaf(x, w1, b1, w2, b2, k, act):
    """One leaf network with library matmuls (independent of the oracle's loops)."""
    h = np_act(x @ w1[k].T + b1[k], act)
    return h @ w2[k] + b2[k]


# ---- printed values -------------------------------------------------------

def test_sizes_match_the_papers_table():
    """Catches a wrong size/width formula (e.g. 2^d nodes instead of 2^d - 1)."""
    g = json.load(open(os.path.join(GOLDEN, "vit_table_sizes.json")))
    n = g["node_size"]
    for r in g["rows"]:
        assert oracle.training_size(r["depth"], n, r["leaf"]) == r["training_size"]
        assert oracle.inference_size(r["depth"], n, r["leaf"]) == r["inference_size"]
        assert oracle.training_width(r["depth"], r["leaf"]) == r["training_width"]
        assert oracle.inference_width(r["depth"], r["leaf"]) == r["inference_width"]


def test_hand_worked_depth2_example():
    """Catches: wrong child on c >= 1/2, strict tie rule, root bit not the top
    bit, heap row of N_{1,1}, transposed W2, dropped bias."""
    g = json.load(open(os.path.join(GOLDEN, "hand_example_depth2.json")))
    a = lambda k: np.array(g[k], dtype=np.float64)
    x = np.array([t["x"] for t in g["tokens"]], dtype=np.float64)
    out, idx, _ = oracle.forward_hard(x, a("node_w"), a("node_b"), a("leaf_w1"), a("leaf_b1"),
                                      a("leaf_w2"), a("leaf_b2"), g["depth"], g["leaf_width"], ACT_RELU)
    assert idx.tolist() == [t["leaf"] for t in g["tokens"]]
    assert out.tolist() == [t["y"] for t in g["tokens"]]


def test_gelu_closed_form_points():
    """Catches a tanh-approximated or mis-scaled GELU."""
    g = json.load(open(os.path.join(GOLDEN, "gelu_closed_form.json")))
    one = np.ones((1, 1, 1))
    zero = np.zeros((1, 1))
    for v, want in g["points"]:
        out, idx, _ = oracle.forward_hard(np.array([[v]]), None, None, one, zero, one, zero, 0, 1, ACT_GELU)
        assert idx[0] == 0
        assert abs(out[0, 0] - want) < 1e-15
    w1 = np.array([[[1.0], [-1.0]]])
    out, _, _ = oracle.forward_hard(np.array([[1.0]]), None, None, w1, np.zeros((1, 2)),
                                    np.ones((1, 2, 1)), zero, 0, 2, ACT_GELU)
    assert abs(out[0, 0] - g["one_sigma"]) < 1e-15


# ---- saturated soft mixture = hard decision -------------------------------

@pytest.mark.parametrize("depth,D,L,O,act", [(1, 2, 1, 1, ACT_RELU), (2, 3, 2, 3, ACT_GELU),
                                             (3, 5, 3, 2, ACT_RELU), (4, 8, 2, 5, ACT_GELU)])
def test_saturated_soft_equals_hard(depth, D, L, O, act):
    """Forward_T with every node logit scaled by 1e6 puts weight exactly 1 on
    one leaf, and that must be Forward_I's leaf and output.  Catches any
    disagreement between the two recursions (child order, tie direction)."""
    rng = np.random.default_rng(100 + depth)
    lay = rand_layer(rng, 64, D, O, depth, L)
    hard, idx, margin = oracle.forward_hard(*lay, depth, L, act)
    soft, mix = oracle.forward_soft(*lay, depth, L, act, node_scale=1e6)
    ok = margin > 1e-4                       # sigmoid(1e6*logit) is exactly 0 or 1 there
    assert ok.sum() > 50
    assert np.array_equal(np.argmax(mix[ok], axis=1), idx[ok])
    assert np.all(np.sort(mix[ok], axis=1)[:, :-1] == 0.0) and np.all(mix[ok].max(axis=1) == 1.0)
    assert np.array_equal(soft[ok], hard[ok])        # exact: 1*y + 0*rest
    assert np.all((idx >= 0) & (idx < (1 << depth)))


def test_mixture_is_a_stochastic_vector():
    """Unsaturated Forward_T: leaf weights are positive and sum to 1, and the
    output is the weighted sum of all leaf outputs (library matmuls)."""
    rng = np.random.default_rng(7)
    depth, D, L, O = 3, 6, 2, 4
    lay = rand_layer(rng, 16, D, O, depth, L)
    x, nw, nb, w1, b1, w2, b2 = lay
    soft, mix = oracle.forward_soft(*lay, depth, L, ACT_GELU)
    assert np.all(mix > 0) and np.allclose(mix.sum(axis=1), 1.0, atol=1e-12)
    leaves = np.stack([np_leaf(x, w1, b1, w2, b2, k, ACT_GELU) for k in range(1 << depth)], axis=1)
    assert np.allclose(soft, np.einsum("tk,tko->to", mix, leaves), atol=1e-12)
    # the weight of leaf k is the product over its path of c (right) or 1 - c (left)
    for t in range(4):
        for k in range(1 << depth):
            wgt = 1.0
            for m in range(depth):
                n = k >> (depth - m)
                c = 1.0 / (1.0 + np.exp(-(nw[(1 << m) - 1 + n] @ x[t] + nb[(1 << m) - 1 + n])))
                wgt *= c if (k >> (depth - 1 - m)) & 1 else 1.0 - c
            assert abs(wgt - mix[t, k]) < 1e-13


def test_zero_node_weights_give_the_dense_ff():
    """All node weights 0: Forward_T is the plain feedforward layer over all
    2^d * l neurons with output weights scaled by 2^-d ("Size and width");
    Forward_I sends every token to the last leaf (c = 1/2 goes right)."""
    rng = np.random.default_rng(11)
    depth, D, L, O, T = 3, 5, 2, 4, 9
    x, nw, nb, w1, b1, w2, b2 = rand_layer(rng, T, D, O, depth, L)
    nw[:] = 0
    nb[:] = 0
    soft, mix = oracle.forward_soft(x, nw, nb, w1, b1, w2, b2, depth, L, ACT_RELU)
    assert np.allclose(mix, 2.0 ** -depth, atol=0, rtol=0)
    W1 = w1.reshape(-1, D)                       # [2^d*l, D]
    W2 = w2.reshape(-1, O) * 2.0 ** -depth
    dense = np.maximum(x @ W1.T + b1.reshape(-1), 0) @ W2 + b2.mean(axis=0)
    assert np.allclose(soft, dense, atol=1e-12)
    hard, idx, margin = oracle.forward_hard(x, nw, nb, w1, b1, w2, b2, depth, L, ACT_RELU)
    assert np.all(idx == (1 << depth) - 1)
    assert np.all(margin == 0.0)
    assert np.allclose(hard, np_leaf(x, w1, b1, w2, b2, (1 << depth) - 1, ACT_RELU), atol=1e-13)


@pytest.mark.parametrize("act", [ACT_RELU, ACT_GELU])
def test_depth_zero_is_a_plain_ff(act):
    """d = 0: no nodes, one leaf.  Non-square shapes catch a transposed W1/W2."""
    rng = np.random.default_rng(3)
    T, D, L, O = 7, 5, 3, 4
    x, _, _, w1, b1, w2, b2 = rand_layer(rng, T, D, O, 0, L)
    out, idx, margin = oracle.forward_hard(x, None, None, w1, b1, w2, b2, 0, L, act)
    assert np.all(idx == 0) and np.all(np.isinf(margin))
    assert np.allclose(out, np_leaf(x, w1, b1, w2, b2, 0, act), atol=1e-13)


# ---- routing ---------------------------------------------------------------

@pytest.mark.parametrize("depth", [1, 3, 6])
def test_bit_path_agrees_with_node_signs(depth):
    """From leaf_idx alone: the node visited at level m is position
    leaf_idx >> (d - m) and the sign of its logit (numpy dot) must be bit
    d-1-m of leaf_idx.  Catches heap-row and bit-order mistakes."""
    rng = np.random.default_rng(21 + depth)
    D, L, O, T = 9, 2, 3, 200
    x, nw, nb, w1, b1, w2, b2 = rand_layer(rng, T, D, O, depth, L)
    out, idx, margin = oracle.forward_hard(x, nw, nb, w1, b1, w2, b2, depth, L, ACT_RELU)
    assert len(set(idx.tolist())) > 1
    for t in range(T):
        mg = np.inf
        for m in range(depth):
            n = int(idx[t]) >> (depth - m)
            row = (1 << m) - 1 + n
            terms = nw[row] * x[t]
            logit = terms.sum() + nb[row]
            assert (logit >= 0) == bool((int(idx[t]) >> (depth - 1 - m)) & 1)
            mg = min(mg, abs(logit) / (np.abs(terms).sum() + abs(nb[row])))
        assert abs(mg - margin[t]) <= 1e-12 * max(mg, 1e-300) + 1e-15
        assert np.allclose(out[t], np_leaf(x[t:t + 1], w1, b1, w2, b2, int(idx[t]), ACT_RELU)[0], atol=1e-12)


def test_axis_aligned_nodes_route_like_a_kd_tree():
    """Node rows are unit vectors e_a with bias -tau: routing is decided by
    scalar compares x[a] >= tau alone, with no rounding at all."""
    rng = np.random.default_rng(5)
    depth, D, L, O, T = 5, 7, 1, 2, 500
    x, nw, nb, w1, b1, w2, b2 = rand_layer(rng, T, D, O, depth, L)
    NN = (1 << depth) - 1
    axis = rng.integers(0, D, NN)
    tau = rng.uniform(-0.7, 0.7, NN)
    nw[:] = 0
    nw[np.arange(NN), axis] = 1.0
    nb[:] = -tau
    x[0, :] = 0.0
    tau0 = tau.copy()
    _, idx, _ = oracle.forward_hard(x, nw, nb, w1, b1, w2, b2, depth, L, ACT_RELU, want_out=False)
    for t in range(T):
        i = 0
        for _ in range(depth):
            i = 2 * i + 1 + (1 if (x[t, axis[i]] - tau0[i]) >= 0 else 0)
        assert idx[t] == i - NN


def test_identical_leaves_make_routing_irrelevant():
    rng = np.random.default_rng(9)
    depth, D, L, O, T = 4, 6, 3, 5, 40
    x, nw, nb, w1, b1, w2, b2 = rand_layer(rng, T, D, O, depth, L)
    for a in (w1, b1, w2, b2):
        a[:] = a[0]
    out, idx, _ = oracle.forward_hard(x, nw, nb, w1, b1, w2, b2, depth, L, ACT_GELU)
    assert len(set(idx.tolist())) > 4
    assert np.allclose(out, np_leaf(x, w1, b1, w2, b2, 0, ACT_GELU), atol=1e-12)


def test_tokens_are_independent_and_permutable():
    rng = np.random.default_rng(13)
    depth, D, L, O, T = 4, 6, 2, 3, 50
    lay = list(rand_layer(rng, T, D, O, depth, L))
    out, idx, mg = oracle.forward_hard(*lay, depth, L, ACT_GELU)
    p = rng.permutation(T)
    lay2 = [lay[0][p]] + lay[1:]
    out2, idx2, mg2 = oracle.forward_hard(*lay2, depth, L, ACT_GELU)
    assert np.array_equal(out2, out[p]) and np.array_equal(idx2, idx[p]) and np.array_equal(mg2, mg[p])
    out3, idx3, _ = oracle.forward_hard(lay[0][17:18], *lay[1:], depth, L, ACT_GELU)
    assert np.array_equal(out3[0], out[17]) and idx3[0] == idx[17]


def test_leaf_forward_matches_forward_hard_and_library():
    rng = np.random.default_rng(17)
    depth, D, L, O, T = 3, 5, 2, 4, 30
    x, nw, nb, w1, b1, w2, b2 = rand_layer(rng, T, D, O, depth, L)
    out, idx, _ = oracle.forward_hard(x, nw, nb, w1, b1, w2, b2, depth, L, ACT_GELU)
    assert np.array_equal(oracle.leaf_forward(x, w1, b1, w2, b2, idx, depth, L, ACT_GELU), out)
    forced = (idx + 3) % (1 << depth)
    got = oracle.leaf_forward(x, w1, b1, w2, b2, forced, depth, L, ACT_GELU)
    for t in range(T):
        assert np.allclose(got[t], np_leaf(x[t:t + 1], w1, b1, w2, b2, int(forced[t]), ACT_GELU)[0], atol=1e-12)


# ---- element types ---------------------------------------------------------

def test_bf16_and_f32_inputs_are_widened_exactly():
    """bf16 bit patterns, the same values as fp32, and as fp64 give identical
    results: the oracle rounds nothing on the way in."""
    import fff_workloads as W
    rng = np.random.default_rng(19)
    depth, D, L, O, T = 3, 16, 2, 5, 20
    lay = rand_layer(rng, T, D, O, depth, L, dtype=np.float32)
    bits = [W.bf16_round(a) for a in lay]
    f32 = [W.bf16_widen(b) for b in bits]
    f64 = [a.astype(np.float64) for a in f32]
    r16 = oracle.forward_hard(*bits, depth, L, ACT_GELU)
    r32 = oracle.forward_hard(*f32, depth, L, ACT_GELU)
    r64 = oracle.forward_hard(*f64, depth, L, ACT_GELU)
    for a, b, c in zip(r16, r32, r64):
        assert np.array_equal(a, b) and np.array_equal(b, c)
    # bf16 rounding itself: ties to even on the 16 dropped bits
    probe = np.array([1.0, 1.00390625, 1.01171875, -1.00390625, 3.0e38, 1e-40], np.float32)
    want = np.array([1.0, 1.0, 1.015625, -1.0, 3.0e38, 1e-40], np.float32)
    got = W.bf16_widen(W.bf16_round(probe))
    assert got[0] == 1.0 and got[1] == 1.0 and got[2] == 1.015625 and got[3] == -1.0
    assert abs(got[4] - want[4]) / want[4] < 2 ** -8


# ---- bucketing --------------------------------------------------------------

@pytest.mark.parametrize("depth,T", [(0, 5), (3, 0), (3, 100), (8, 5000), (12, 3000)])
def test_bucket_against_library_sort(depth, T):
    rng = np.random.default_rng(23 + depth)
    NL = 1 << depth
    idx = (rng.zipf(1.3, T) % NL).astype(np.int32) if T else np.zeros(0, np.int32)
    count, offset, perm = oracle.bucket(idx, depth)
    assert np.array_equal(count, np.bincount(idx, minlength=NL))
    assert offset[0] == 0 and offset[-1] == T and np.array_equal(np.diff(offset), count)
    assert np.array_equal(perm, np.argsort(idx, kind="stable"))
    for j in range(NL):
        seg = perm[offset[j]:offset[j + 1]]
        assert np.all(idx[seg] == j) and np.all(np.diff(seg) > 0)


def test_node_entropy_closed_forms_and_library():
    """Batch mean entropy of the node choice scores (paragraph "Hardening"): ln 2 for undecided
    nodes, 0 for saturated ones, symmetric under a sign flip of the node, and equal to the
    textbook binary entropy of sigmoid(logits) computed with library routines."""
    rng = np.random.default_rng(31)
    T, D, depth = 200, 6, 3
    NN = (1 << depth) - 1
    x = rng.normal(size=(T, D))
    assert np.allclose(oracle.node_entropy(x, np.zeros((NN, D)), np.zeros(NN), depth), np.log(2.0), rtol=0, atol=1e-13)
    w = rng.normal(size=(NN, D))
    b = rng.normal(size=NN)
    assert np.all(oracle.node_entropy(x, 1e4 * w, 1e4 * b, depth) < 1e-6)
    e = oracle.node_entropy(x, w, b, depth)
    assert np.allclose(e, oracle.node_entropy(x, -w, -b, depth), rtol=1e-12)
    from scipy.special import expit, xlogy
    c = expit(x @ w.T + b)                                # [T, NN], heap order = row order of w
    ref = (-(xlogy(c, c) + xlogy(1 - c, 1 - c))).mean(axis=0)
    assert np.allclose(e, ref, rtol=1e-12, atol=1e-15)
    # only the node's own row matters: changing another node leaves its entropy alone
    w2 = w.copy()
    w2[4] *= 3.0
    e2 = oracle.node_entropy(x, w2, b, depth)
    assert np.array_equal(np.delete(e2, 4), np.delete(e, 4)) and e2[4] != e[4]
