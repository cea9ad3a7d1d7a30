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
    "leaf_w2": 6, "leaf_b2": 7, "perm": 8, "gate_w": 9, "gate_b": 10,
    "node_w1": 11, "node_b1": 12, "node_w2": 13, "node_b2": 14, "ln_gamma": 15, "ln_beta": 16,
}


def _stream(seed: int, tag: str, sub: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[(seed << 8) | _TAGS[tag], sub]))


def _round_chunk(c32: np.ndarray, tmp: np.ndarray, out16: np.ndarray) -> None:
    """bf16 round-to-nearest-even of the uint32 view ``c32`` into ``out16``,
    using ``tmp`` (uint32, same length) as scratch; nothing is allocated."""
    np.right_shift(c32, np.uint32(16), out=tmp)
    np.bitwise_and(tmp, np.uint32(1), out=tmp)
    np.add(tmp, np.uint32(0x7FFF), out=tmp)
    np.add(tmp, c32, out=tmp)
    np.right_shift(tmp, np.uint32(16), out=tmp)
    np.copyto(out16, tmp, casting="unsafe")


def bf16_round(a: np.ndarray, chunk: int = 1 << 22) -> np.ndarray:
    """fp32 array -> uint16 bf16 bit patterns, round to nearest even."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.reshape(-1).view(np.uint32)
    out = np.empty(u.shape, dtype=np.uint16)
    tmp = np.empty((min(chunk, max(u.size, 1)),), dtype=np.uint32)
    for i in range(0, u.size, chunk):
        c = u[i:i + chunk]
        _round_chunk(c, tmp[:c.size], out[i:i + chunk])
    return out.reshape(a.shape)


def bf16_widen(bits: np.ndarray) -> np.ndarray:
    """uint16 bf16 bit patterns -> the same values as fp32 (exact)."""
    out = np.empty(bits.shape, dtype=np.uint32)
    np.copyto(out, bits, casting="unsafe")
    np.left_shift(out, np.uint32(16), out=out)
    return out.view(np.float32)


def _uniform(seed, tag, shape, bound, as_bf16_bits=False, chunk=1 << 22):
    """U(-bound, bound) drawn in fp32 in fixed-size chunks of one stream.
    Returns fp32 values, or (``as_bf16_bits``) their bf16 roundings as uint16
    without ever holding the fp32 tensor."""
    shape = tuple(int(s) for s in shape)
    n = int(np.prod(shape))
    g = _stream(seed, tag)
    two_b, b = np.float32(2.0 * bound), np.float32(bound)
    out = np.empty((n,), dtype=np.uint16 if as_bf16_bits else np.float32)
    buf = np.empty((min(chunk, max(n, 1)),), dtype=np.float32)
    tmp = np.empty(buf.shape, dtype=np.uint32) if as_bf16_bits else None
    for i in range(0, n, chunk):
        blk = buf[:min(chunk, n - i)]
        g.random(out=blk, dtype=np.float32)
        np.multiply(blk, two_b, out=blk)
        np.subtract(blk, b, out=blk)
        if as_bf16_bits:
            _round_chunk(blk.view(np.uint32), tmp[:blk.size], out[i:i + blk.size])
        else:
            out[i:i + blk.size] = blk
    return out.reshape(shape)


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
    ``keep_f32`` = False drops the fp32 copies of a bf16 workload (the oracle
    reads bf16 bit patterns directly), which matters for the largest one.
    """
    NN, NL = (1 << depth) - 1, 1 << depth
    w = Workload(name, T, D, O, depth, leaf_width, act, dtype, note=note)
    bf = dtype == DTYPE_BF16

    def put(key, arr, is_bits=False):
        """Store a tensor: fp32 workloads keep fp32; bf16 workloads keep the
        rounded bits and (optionally) the widened values."""
        if not bf:
            w.f32[key] = arr
            return
        bits = arr if is_bits else bf16_round(arr)
        w.bits[key] = bits
        if keep_f32 or key == "node_w":
            w.f32[key] = bf16_widen(bits)

    def uni(key, shape, bound):
        put(key, _uniform(seed, key, shape, bound, as_bf16_bits=bf), is_bits=bf)

    if x_dist == "normal":
        put("x", _normal(seed, "x", (T, D)))
    elif x_dist == "uniform01":
        put("x", _stream(seed, "x").random((T, D), dtype=np.float32))
    else:
        raise ValueError(x_dist)
    bD = 1.0 / np.sqrt(D)
    bL = 1.0 / np.sqrt(leaf_width)
    uni("node_w", (NN, D), bD)
    uni("leaf_w1", (NL, leaf_width, D), bD)
    uni("leaf_w2", (NL, leaf_width, O), bL)
    if leaf_b == "zero":
        put("leaf_b1", np.zeros((NL, leaf_width), np.float32))
        put("leaf_b2", np.zeros((NL, O), np.float32))
    else:
        uni("leaf_b1", (NL, leaf_width), bD)
        uni("leaf_b2", (NL, O), bL)
    nw = w.f32["node_w"]           # for bf16: the rounded rows, as the biases must see them
    if node_b == "zero":
        put("node_b", np.zeros((NN,), np.float32))
    elif node_b == "uniform":
        uni("node_b", (NN,), bD)
    elif node_b == "normal0.1":
        put("node_b", _normal(seed, "node_b", (NN,), 0.1))
    elif node_b == "centred0.1":
        put("node_b", (_normal(seed, "node_b", (NN,), 0.1)
                       - 0.5 * nw.sum(axis=1, dtype=np.float64)).astype(np.float32))
    elif node_b == "zipf":
        put("node_b", zipf_node_bias(nw, depth, seed))
    else:
        raise ValueError(node_b)
    if bf and not keep_f32:
        w.f32.pop("node_w", None)
    return w


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


def moe_gate(n_experts: int, D: int, dtype: int, seed: int = 0):
    """Gating weights of a mixture of experts standing beside a layer of `n_experts` leaves:
    gate_w [n_experts, D] and gate_b [n_experts], U(-1/sqrt(D), 1/sqrt(D)) like the node weights.
    Returns the arrays whose bytes are uploaded (uint16 bf16 bits or fp32)."""
    bD = 1.0 / np.sqrt(D)
    bf = dtype == DTYPE_BF16
    return (_uniform(seed, "gate_w", (n_experts, D), bD, as_bf16_bits=bf),
            _uniform(seed, "gate_b", (n_experts,), bD, as_bf16_bits=bf))


def wide_nodes(depth: int, node_size: int, D: int, dtype: int, seed: int = 0):
    """Node networks of `node_size` hidden neurons for a tree of the given depth (the <D, n, 1>
    networks of the Definition, heap order): node_w1 [NN, n, D] and node_b1 [NN, n] drawn
    U(-1/sqrt(D), 1/sqrt(D)), node_w2 [NN, n] U(-1/sqrt(n), 1/sqrt(n)), node_b2 [NN] a tenth of
    that (small, so that the tokens spread over the leaves).  Returns the arrays whose bytes are
    uploaded (uint16 bf16 bits or fp32)."""
    NN = (1 << depth) - 1
    bD, bn = 1.0 / np.sqrt(D), 1.0 / np.sqrt(node_size)
    bf = dtype == DTYPE_BF16
    return (_uniform(seed, "node_w1", (NN, node_size, D), bD, as_bf16_bits=bf),
            _uniform(seed, "node_b1", (NN, node_size), bD, as_bf16_bits=bf),
            _uniform(seed, "node_w2", (NN, node_size), bn, as_bf16_bits=bf),
            _uniform(seed, "node_b2", (NN,), 0.1 * bn, as_bf16_bits=bf))


def layer_norm_params(D: int, dtype: int, seed: int = 0):
    """Scale and shift of a layer normalisation over D features: gamma U(0.75, 1.25), beta
    U(-0.1, 0.1).  Returns the arrays whose bytes are uploaded."""
    g = _uniform(seed, "ln_gamma", (D,), 0.25) + np.float32(1.0)
    b = _uniform(seed, "ln_beta", (D,), 0.1)
    if dtype == DTYPE_BF16:
        return bf16_round(g), bf16_round(b)
    return g, b


CONFIG_NAMES = ("C1", "C2", "C2c", "C3", "C4", "C5")
