"""Pins of the oracle's block function: Forward_I with nodes of size n >= 1 (the Definition's
<D, n, 1> node networks) on a layer-normalised input with a residual sum.  Each checks it against
something other than itself: a hand-worked example, the already pinned linear-node forward pass,
library routines (layer normalisation, matrix products) on tiny inputs, scalar compares, and the
invariants the definition implies.  CPU only."""
import json
import os

import numpy as np
import torch

import oracle

HERE = os.path.dirname(os.path.abspath(__file__))


def _fff(rng, depth, n, L, D, O):
    NN, NL = (1 << depth) - 1, 1 << depth
    return dict(node_w1=rng.normal(size=(NN, n, D)), node_b1=rng.normal(size=(NN, n)),
                node_w2=rng.normal(size=(NN, n)), node_b2=rng.normal(size=(NN,)),
                leaf_w1=rng.normal(size=(NL, L, D)), leaf_b1=rng.normal(size=(NL, L)),
                leaf_w2=rng.normal(size=(NL, L, O)), leaf_b2=rng.normal(size=(NL, O)))


def _run(x, w, depth, n, L, act, gamma=None, beta=None, eps=0.0, residual=False, want_out=True):
    return oracle.forward_block(x, gamma, beta, eps, w["node_w1"], w["node_b1"], w["node_w2"], w["node_b2"],
                                w["leaf_w1"], w["leaf_b1"], w["leaf_w2"], w["leaf_b2"], depth, n, L, act,
                                residual, want_out)


def test_block_hand_worked_example():
    g = json.load(open(os.path.join(HERE, "golden", "block_hand_example.json")))
    a = {k: np.array(v, dtype=np.float64) for k, v in g.items() if not k.startswith("_")}
    out, idx, margin = _run(a["x"], a, 1, 2, 1, oracle.ACT_RELU, a["ln_gamma"], a["ln_beta"], 0.0, True)
    assert idx.tolist() == g["leaf_idx"]
    assert np.allclose(out, a["out"], rtol=0, atol=1e-14)
    assert np.allclose(margin, a["margin"], rtol=1e-14, atol=0)
    out, idx, _ = _run(a["x"], a, 1, 2, 1, oracle.ACT_RELU, a["ln_gamma"], a["ln_beta"], 0.0, False)
    assert idx.tolist() == g["leaf_idx"]
    assert np.allclose(out, a["out_no_residual"], rtol=0, atol=1e-14)


def test_two_relu_neurons_make_the_linear_node():
    """Hidden neurons (w, b) and (-w, -b) with output weights (1, -1) and ReLU give
    relu(s) - relu(-s) = s exactly, so the node is the single linear neuron of the pinned
    forward pass; the output bias moves the threshold like the linear bias does."""
    rng = np.random.default_rng(31)
    T, D, O, depth, L = 500, 11, 5, 4, 3
    x = rng.normal(size=(T, D))
    w = _fff(rng, depth, 2, L, D, O)
    lin_w = rng.normal(size=((1 << depth) - 1, D))
    lin_b = rng.normal(size=((1 << depth) - 1,))
    w["node_w1"] = np.stack([lin_w, -lin_w], axis=1)
    w["node_b1"] = np.stack([lin_b, -lin_b], axis=1)
    w["node_w2"] = np.tile(np.array([1.0, -1.0]), ((1 << depth) - 1, 1))
    w["node_b2"] = np.zeros((1 << depth) - 1)
    ref_out, ref_idx, _ = oracle.forward_hard(x, lin_w, lin_b, w["leaf_w1"], w["leaf_b1"], w["leaf_w2"],
                                              w["leaf_b2"], depth, L, oracle.ACT_RELU)
    out, idx, _ = _run(x, w, depth, 2, L, oracle.ACT_RELU)
    assert np.array_equal(idx, ref_idx)
    assert np.array_equal(out, ref_out)
    assert len(set(idx.tolist())) > 8


def test_block_against_library_layer_norm_and_products():
    """Tiny inputs, torch's layer_norm and matrix products in fp64, the walk written with
    tensor operations per token."""
    rng = np.random.default_rng(32)
    T, D, depth, n, L = 60, 9, 3, 3, 2
    O = D
    x = rng.normal(size=(T, D)) * 2 + 0.5
    w = _fff(rng, depth, n, L, D, O)
    w["node_b2"] *= 0.1                      # keep the routing spread over the leaves
    gamma, beta, eps = rng.normal(size=D), 0.1 * rng.normal(size=D), 1e-3
    out, idx, _ = _run(x, w, depth, n, L, oracle.ACT_GELU, gamma, beta, eps, True)
    tw = {k: torch.from_numpy(v) for k, v in w.items()}
    z = torch.nn.functional.layer_norm(torch.from_numpy(x), (D,), torch.from_numpy(gamma), torch.from_numpy(beta), eps)
    gelu = torch.nn.GELU()
    for t in range(T):
        i = 0
        for _ in range(depth):
            logit = tw["node_w2"][i] @ gelu(tw["node_w1"][i] @ z[t] + tw["node_b1"][i]) + tw["node_b2"][i]
            i = 2 * i + (2 if logit >= 0 else 1)
        leaf = i - ((1 << depth) - 1)
        assert idx[t] == leaf
        y = gelu(tw["leaf_w1"][leaf] @ z[t] + tw["leaf_b1"][leaf]) @ tw["leaf_w2"][leaf] + tw["leaf_b2"][leaf]
        assert np.allclose(out[t], y.numpy() + x[t], rtol=1e-12, atol=1e-12)
    assert len(set(idx.tolist())) > 3


def test_layer_norm_is_numpy_standardisation_then_affine():
    """With the normalisation on, the block equals the same block without it applied to
    (x - mean) / sqrt(var + eps) * gamma + beta from numpy's mean and var (divisor D)."""
    rng = np.random.default_rng(33)
    T, D, O, depth, n, L = 200, 16, 7, 3, 2, 2
    x = rng.normal(size=(T, D)) * 3 - 1
    w = _fff(rng, depth, n, L, D, O)
    gamma, beta, eps = rng.normal(size=D), rng.normal(size=D), 0.25
    z = (x - x.mean(axis=1, keepdims=True)) / np.sqrt(x.var(axis=1, keepdims=True) + eps) * gamma + beta
    out, idx, _ = _run(x, w, depth, n, L, oracle.ACT_RELU, gamma, beta, eps)
    ref_out, ref_idx, margin = _run(z, w, depth, n, L, oracle.ACT_RELU)
    safe = margin > 1e-9
    assert safe.sum() > T - 5
    assert np.array_equal(idx[safe], ref_idx[safe])
    assert np.allclose(out[safe], ref_out[safe], rtol=1e-11, atol=1e-11)


def test_shift_and_scale_of_the_input_do_not_matter_under_layer_norm():
    """eps = 0: LayerNorm(a x + c) = LayerNorm(x) for a > 0, so only the residual term moves."""
    rng = np.random.default_rng(34)
    T, D, depth, n, L = 200, 12, 3, 2, 2
    x = rng.normal(size=(T, D))
    w = _fff(rng, depth, n, L, D, D)
    gamma, beta = rng.normal(size=D), rng.normal(size=D)
    out, idx, margin = _run(x, w, depth, n, L, oracle.ACT_GELU, gamma, beta, 0.0, True)
    x2 = 3.5 * x + 7.0
    out2, idx2, _ = _run(x2, w, depth, n, L, oracle.ACT_GELU, gamma, beta, 0.0, True)
    safe = margin > 1e-9
    assert np.array_equal(idx[safe], idx2[safe])
    assert np.allclose((out - x)[safe], (out2 - x2)[safe], rtol=1e-10, atol=1e-10)
    # and with eps > 0 the scale does matter: a tiny input is pulled towards beta
    out3, _, _ = _run(1e-6 * x, w, depth, n, L, oracle.ACT_GELU, gamma, beta, 1.0, False)
    ref3, _, _ = _run(np.tile(beta, (T, 1)), w, depth, n, L, oracle.ACT_GELU)
    assert np.allclose(out3, ref3, rtol=0, atol=1e-4)


def test_residual_adds_the_unnormalised_input():
    rng = np.random.default_rng(35)
    T, D, depth, n, L = 100, 10, 2, 3, 4
    x = rng.normal(size=(T, D))
    w = _fff(rng, depth, n, L, D, D)
    gamma, beta = rng.normal(size=D), rng.normal(size=D)
    a, ia, _ = _run(x, w, depth, n, L, oracle.ACT_RELU, gamma, beta, 1e-5, True)
    b, ib, _ = _run(x, w, depth, n, L, oracle.ACT_RELU, gamma, beta, 1e-5, False)
    assert np.array_equal(ia, ib)
    assert np.allclose(a - b, x, rtol=0, atol=1e-13)


def test_dead_hidden_neurons_leave_the_output_bias_to_decide():
    """ReLU neurons with a very negative bias are all zero, so the path is read off the signs
    of the output biases alone."""
    rng = np.random.default_rng(36)
    T, D, O, depth, n, L = 50, 8, 3, 5, 4, 1
    x = rng.normal(size=(T, D))
    w = _fff(rng, depth, n, L, D, O)
    w["node_b1"][:] = -1e6
    w["node_b2"][0] = 0.0                    # a logit of exactly 0 is an output of 1/2: right
    w["node_b2"][2] = -0.0
    _, idx, _ = _run(x, w, depth, n, L, oracle.ACT_RELU, want_out=False)
    i = 0
    for _ in range(depth):
        i = 2 * i + (2 if w["node_b2"][i] >= 0 else 1)
    assert np.all(idx == i - ((1 << depth) - 1))


def test_permuting_a_nodes_hidden_neurons_changes_nothing():
    rng = np.random.default_rng(37)
    T, D, O, depth, n, L = 300, 10, 4, 4, 5, 2
    x = rng.normal(size=(T, D))
    w = _fff(rng, depth, n, L, D, O)
    out, idx, margin = _run(x, w, depth, n, L, oracle.ACT_GELU)
    p = rng.permutation(n)
    w2 = dict(w, node_w1=w["node_w1"][:, p], node_b1=w["node_b1"][:, p], node_w2=w["node_w2"][:, p])
    out2, idx2, _ = _run(x, w2, depth, n, L, oracle.ACT_GELU)
    safe = margin > 1e-12
    assert np.array_equal(idx[safe], idx2[safe]) and np.array_equal(out[safe], out2[safe])
    assert len(set(idx.tolist())) > 8


def test_single_hidden_neuron_and_output_weight_by_scalar_arithmetic():
    """n = 1, one-hot input weights: the logit is v * relu(s * x[axis] + a) + c, scalar
    arithmetic per token; depth 1 so the leaf index is the decision itself."""
    rng = np.random.default_rng(38)
    T, D, O, L = 400, 6, 3, 2
    x = rng.normal(size=(T, D))
    w = _fff(rng, 1, 1, L, D, O)
    w["node_w1"][:] = 0.0
    w["node_w1"][0, 0, 4] = -1.5
    w["node_b1"][0, 0], w["node_w2"][0, 0], w["node_b2"][0] = 0.25, 2.0, -1.0
    _, idx, margin = _run(x, w, 1, 1, L, oracle.ACT_RELU, want_out=False)
    a, v, c = w["node_b1"][0, 0], w["node_w2"][0, 0], w["node_b2"][0]
    for t in range(T):
        pre = -1.5 * x[t, 4] + a
        logit = c + v * (pre if pre > 0 else 0.0)
        assert idx[t] == (1 if logit >= 0 else 0)
        # the margin relates the logit to the size of the terms it was summed from
        assert abs(margin[t] - abs(logit) / (abs(c) + abs(v) * (abs(1.5 * x[t, 4]) + abs(a)))) < 1e-14
    assert 0 < idx.sum() < T


def test_depth_zero_block_is_norm_ff_residual():
    rng = np.random.default_rng(39)
    T, D, L = 40, 8, 5
    x = rng.normal(size=(T, D))
    w = _fff(rng, 0, 2, L, D, D)
    gamma, beta, eps = rng.normal(size=D), rng.normal(size=D), 1e-2
    out, idx, margin = _run(x, w, 0, 2, L, oracle.ACT_RELU, gamma, beta, eps, True)
    z = torch.nn.functional.layer_norm(torch.from_numpy(x), (D,), torch.from_numpy(gamma), torch.from_numpy(beta), eps).numpy()
    ref = np.maximum(z @ w["leaf_w1"][0].T + w["leaf_b1"][0], 0) @ w["leaf_w2"][0] + w["leaf_b2"][0] + x
    assert np.all(idx == 0) and np.all(np.isinf(margin))
    assert np.allclose(out, ref, rtol=1e-12, atol=1e-12)


def test_block_rejects_a_residual_of_another_width():
    rng = np.random.default_rng(40)
    x = rng.normal(size=(4, 6))
    w = _fff(rng, 1, 2, 2, 6, 5)
    try:
        _run(x, w, 1, 2, 2, oracle.ACT_RELU, residual=True)
    except ValueError:
        return
    raise AssertionError("a residual with O != D was accepted")
