"""The seeded input generators: shapes, ranges, determinism, bf16 consistency."""
import numpy as np
import pytest

import fff_workloads as W


def test_c1_recipe():
    w = W.config("C1")
    assert (w.T, w.D, w.O, w.depth, w.leaf_width) == (256, 64, 10, 3, 8)
    assert w.f32["node_w"].shape == (7, 64) and w.f32["leaf_w1"].shape == (8, 8, 64)
    assert w.f32["leaf_w2"].shape == (8, 8, 10) and w.f32["leaf_b2"].shape == (8, 10)
    assert np.abs(w.f32["node_w"]).max() <= 1 / 8 and np.abs(w.f32["leaf_w2"]).max() <= 1 / np.sqrt(8)
    assert not w.f32["node_b"].any() and not w.f32["leaf_b1"].any() and not w.f32["leaf_b2"].any()
    assert abs(w.f32["x"].mean()) < 0.05 and abs(w.f32["x"].std() - 1) < 0.05
    w2 = W.config("C1")
    for k in W.TENSORS:
        assert np.array_equal(w.f32[k], w2.f32[k])
    w3 = W.config("C1", seed=1)
    assert not np.array_equal(w.f32["x"], w3.f32["x"])


def test_c2_recipe():
    w = W.config("C2", T=512)
    assert w.f32["x"].min() >= 0 and w.f32["x"].max() < 1
    assert abs(w.f32["node_b"].std() - 0.1) < 0.03
    assert np.abs(w.f32["leaf_w1"]).max() <= 1 / 28 + 1e-7


def test_bf16_workload_is_self_consistent():
    w = W.make_layer("t", 64, 32, 16, 4, 2, W.ACT_GELU, W.DTYPE_BF16, seed=3)
    for k in W.TENSORS:
        assert w.bits[k].dtype == np.uint16
        assert np.array_equal(W.bf16_widen(w.bits[k]).reshape(w.f32[k].shape), w.f32[k])
        assert np.array_equal(W.bf16_round(w.f32[k]).reshape(w.bits[k].shape), w.bits[k])   # already representable


def test_zipf_bias_targets():
    """The construction must give the root a right-branch probability equal to
    the right subtree's share of the Zipf mass (checked in closed form)."""
    from scipy.special import ndtr
    depth, D = 6, 256
    rng = np.random.default_rng(0)
    nw = rng.uniform(-1, 1, ((1 << depth) - 1, D)).astype(np.float32) / 16
    b = W.zipf_node_bias(nw, depth, seed=0, permute=False)
    p = np.arange(1, (1 << depth) + 1, dtype=np.float64) ** -1.1
    p /= p.sum()
    q_root = p[(1 << depth) // 2:].sum()
    assert abs(ndtr(b[0] / np.linalg.norm(nw[0].astype(np.float64))) - q_root) < 1e-6
    # last internal node splits the two rarest leaves
    q_last = p[-1] / (p[-1] + p[-2])
    assert abs(ndtr(b[-1] / np.linalg.norm(nw[-1].astype(np.float64))) - q_last) < 1e-6
