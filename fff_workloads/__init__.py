"""Seeded synthetic inputs for hard-routed FFF inference.

This module only draws numbers and lays them out; it holds none of the
method's arithmetic (no tree descent, no leaf evaluation).  Both the CPU
oracle and the HIP path are fed from the arrays built here, so neither side
ever sees a value produced by the other.

Every tensor comes from its own counter-based stream (Philox keyed by
``(seed, tensor tag)``), so a tensor does not depend on the order in which the
others were drawn.  Shapes follow the definition of an FFF of depth ``d`` and
leaf size ``l`` (Definition, Section "Algorithm"): ``2^d - 1`` node neurons in
heap order and ``2^d`` leaves, each a <D, l, O> feedforward block.

For bf16 workloads the values are drawn in fp32 and rounded once to bf16
(round to nearest, ties to even).  The rounded values are the inputs: the
uint16 bit patterns go to the GPU, the same values widened to fp32 go to the
oracle.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, Optional

import numpy as np

ACT_RELU = 0
ACT_GELU = 1

DTYPE_F32 = 0
DTYPE_BF16 = 1

_TAGS = {
    "x": 1, "node_w": 2, "node_b": 3, "leaf_w1": 4, "leaf_b1": 5,
    "leaf_w2": 6, "leaf_b2": 7, "perm": 8,
}


def _stream(seed: int, tag: str, sub: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[(seed << 8) | _TAGS[tag], sub]))


def bf16_round(a: np.ndarray) -> np.ndarray:
    """fp32 array -> uint16 bf16 bit patterns, round to nearest even."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_widen(bits: np.ndarray) -> np.ndarray:
    """uint16 bf16 bit patterns -> the same values as fp32 (exact)."""
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def _uniform(seed, tag, shape, bound, chunk_rows=4096):
    """U(-bound, bound) in fp32, drawn in row chunks to bound peak memory."""
    shape = tuple(int(s) for s in shape)
    out = np.empty(shape, dtype=np.float32)
    flat = out.reshape(shape[0], -1) if len(shape) > 1 else out.reshape(-1, 1)
    n0 = flat.shape[0]
    g = _stream(seed, tag)
    for r0 in range(0, n0, chunk_rows):
        r1 = min(n0, r0 + chunk_rows)
        blk = g.random((r1 - r0, flat.shape[1]), dtype=np.float32)
        flat[r0:r1] = (blk * np.float32(2.0) - np.float32(1.0)) * np.float32(bound)
    return out


def _normal(seed, tag, shape, sigma=1.0):
    g = _stream(seed, tag)
    return (g.standard_normal(shape, dtype=np.float32) * np.float32(sigma)).astype(np.float32)


@dataclass
class Workload:
    """One FFF layer plus a batch of tokens.

    ``f32`` holds every tensor as fp32 values (for bf16 workloads: the
    bf16-rounded values, widened).  ``bits`` holds the uint16 bf16 patterns
    of the same tensors for bf16 workloads and is empty for fp32 ones.
    """
    name: str
    T: int
    D: int
    O: int
    depth: int
    leaf_width: int
    act: int
    dtype: int
    f32: Dict[str, np.ndarray] = field(default_factory=dict)
    bits: Dict[str, np.ndarray] = field(default_factory=dict)
    note: str = ""

    @property
    def n_nodes(self) -> int:
        return (1 << self.depth) - 1

    @property
    def n_leaves(self) -> int:
        return 1 << self.depth

    def device_array(self, key: str) -> np.ndarray:
        """The array whose bytes are uploaded: uint16 bits (bf16) or fp32."""
        return self.bits[key] if self.dtype == DTYPE_BF16 else self.f32[key]


TENSORS = ("x", "node_w", "node_b", "leaf_w1", "leaf_b1", "leaf_w2", "leaf_b2")


def _finish(w: Workload, keep_f32: bool = True) -> Workload:
    if w.dtype == DTYPE_BF16:
        for k in TENSORS:
            b = bf16_round(w.f32[k])
            w.bits[k] = b
            if keep_f32:
                w.f32[k] = bf16_widen(b).reshape(w.f32[k].shape)
            else:
                del w.f32[k]
    return w


def make_layer(name, T, D, O, depth, leaf_width, act, dtype, seed=0,
               x_dist="normal", node_b="uniform", leaf_b="uniform",
               keep_f32=True, note="") -> Workload:
    """Draw one workload.

    Weights are U(-1/sqrt(fan_in), 1/sqrt(fan_in)): fan_in = D for node and
    leaf input weights, fan_in = leaf_width for leaf output weights.
    ``x_dist``: "normal" N(0,1) or "uniform01" U(0,1).
    ``node_b``: "zero", "uniform" (same bound as node_w), "normal0.1",
    "centred0.1" (N(0,0.1) minus half the row sum of node_w, which centres the
    logit of U(0,1) inputs), or "zipf" (see ``zipf_node_bias``).
    ``leaf_b``: "zero" or "uniform" (bound 1/sqrt(fan_in) of its layer).
    """
    NN, NL = (1 << depth) - 1, 1 << depth
    w = Workload(name, T, D, O, depth, leaf_width, act, dtype, note=note)
    f = w.f32
    if x_dist == "normal":
        f["x"] = _normal(seed, "x", (T, D))
    elif x_dist == "uniform01":
        f["x"] = _stream(seed, "x").random((T, D), dtype=np.float32)
    else:
        raise ValueError(x_dist)
    bD = 1.0 / np.sqrt(D)
    bL = 1.0 / np.sqrt(leaf_width)
    f["node_w"] = _uniform(seed, "node_w", (NN, D), bD)
    f["leaf_w1"] = _uniform(seed, "leaf_w1", (NL, leaf_width, D), bD)
    f["leaf_w2"] = _uniform(seed, "leaf_w2", (NL, leaf_width, O), bL)
    if leaf_b == "zero":
        f["leaf_b1"] = np.zeros((NL, leaf_width), np.float32)
        f["leaf_b2"] = np.zeros((NL, O), np.float32)
    else:
        f["leaf_b1"] = _uniform(seed, "leaf_b1", (NL, leaf_width), bD)
        f["leaf_b2"] = _uniform(seed, "leaf_b2", (NL, O), bL)
    if dtype == DTYPE_BF16:
        # biases that are built from node_w must see the rounded rows
        f["node_w"] = bf16_widen(bf16_round(f["node_w"])).reshape(NN, D)
    if node_b == "zero":
        f["node_b"] = np.zeros((NN,), np.float32)
    elif node_b == "uniform":
        f["node_b"] = _uniform(seed, "node_b", (NN,), bD)
    elif node_b == "normal0.1":
        f["node_b"] = _normal(seed, "node_b", (NN,), 0.1)
    elif node_b == "centred0.1":
        f["node_b"] = (_normal(seed, "node_b", (NN,), 0.1)
                       - 0.5 * f["node_w"].sum(axis=1, dtype=np.float64)).astype(np.float32)
    elif node_b == "zipf":
        f["node_b"] = zipf_node_bias(f["node_w"], depth, seed)
    else:
        raise ValueError(node_b)
    return _finish(w, keep_f32)


def zipf_node_bias(node_w: np.ndarray, depth: int, seed: int, s: float = 1.1,
                   permute: bool = True) -> np.ndarray:
    """Node biases that make leaf occupancy follow Zipf(s) for x ~ N(0, I).

    Leaf of rank r gets target probability proportional to r^-s; ranks are
    assigned to leaves by a seeded permutation.  Bottom-up, each node's mass
    is the sum of its children's, and the probability of branching right is
    q = mass(right) / mass(node), clamped to [1e-6, 1 - 1e-6].  Since
    w.x ~ N(0, |w|^2), the bias |w| * Phi^-1(q) makes P(w.x + b >= 0) = q.
    """
    from scipy.special import ndtri
    NL = 1 << depth
    p = np.arange(1, NL + 1, dtype=np.float64) ** (-s)
    p /= p.sum()
    if permute:
        p = p[_stream(seed, "perm").permutation(NL)]
    NN = NL - 1
    mass = np.empty(NN + NL, dtype=np.float64)      # heap order, leaves last
    mass[NN:] = p
    for i in range(NN - 1, -1, -1):
        mass[i] = mass[2 * i + 1] + mass[2 * i + 2]
    i = np.arange(NN)
    q = np.clip(mass[2 * i + 2] / mass[i], 1e-6, 1 - 1e-6)
    norm = np.sqrt((node_w.astype(np.float64) ** 2).sum(axis=1))
    return (norm * ndtri(q)).astype(np.float32)


# The five workloads (name -> recipe).  "C2c" is C2 with centred node biases.
def config(name: str, seed: int = 0, keep_f32: bool = True, T: Optional[int] = None) -> Workload:
    """Build a named workload; ``T`` overrides the token count (a prefix-free
    redraw of the same recipe with fewer tokens, used for bounded samples)."""
    if name == "C1":
        return make_layer("C1", T or 256, 64, 10, 3, 8, ACT_RELU, DTYPE_F32, seed,
                          node_b="zero", leaf_b="zero",
                          note="tiny fp32 FFF")
    if name == "C2":
        return make_layer("C2", T or 4096, 784, 10, 6, 4, ACT_RELU, DTYPE_F32, seed,
                          x_dist="uniform01", node_b="normal0.1",
                          note="MNIST-shaped, node biases N(0, sigma=0.1) as written")
    if name == "C2c":
        return make_layer("C2c", T or 4096, 784, 10, 6, 4, ACT_RELU, DTYPE_F32, seed,
                          x_dist="uniform01", node_b="centred0.1",
                          note="MNIST-shaped, node logits centred so occupancy is near-uniform")
    if name == "C3":
        return make_layer("C3", T or 256 * 197, 768, 768, 8, 8, ACT_GELU, DTYPE_BF16, seed,
                          keep_f32=keep_f32, note="ViT-block FFF")
    if name == "C4":
        return make_layer("C4", T or 128 * 512, 768, 768, 11, 1, ACT_GELU, DTYPE_BF16, seed,
                          keep_f32=keep_f32, note="BERT-base-sized FFF")
    if name == "C5":
        return make_layer("C5", T or 16384, 4096, 4096, 15, 4, ACT_GELU, DTYPE_BF16, seed,
                          node_b="zipf", keep_f32=keep_f32,
                          note="large skewed FFF, Zipf(1.1) leaf occupancy")
    raise KeyError(name)


CONFIG_NAMES = ("C1", "C2", "C2c", "C3", "C4", "C5")
