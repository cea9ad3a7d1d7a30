"""ctypes front end of the CPU oracle (oracle/fff_oracle.c).  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg import this
package.  It knows nothing of the HIP library and shares no code with it.
Arrays are numpy: float32, float64, or uint16 holding bf16 bit patterns.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "fff_oracle.c")
_LIB = os.path.join(_HERE, "libfff_oracle.so")

ACT_RELU = 0
ACT_GELU = 1


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (OpenMP over tokens)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared",
                               "-Wall", "-Wextra", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None
_lib_path = None


def use_library(path: Optional[str]) -> None:
    """Point the wrapper at another build of the oracle (tests that plant mistakes in a copy of
    the C source use this); None goes back to the regular build."""
    global _lib, _lib_path
    _lib = None
    _lib_path = path


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(_lib_path or build())
        vp, i32, i64, f64 = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_double
        _lib.fff_oracle_forward_hard.argtypes = [vp] * 7 + [i32, i32, i32, i64, i64, i64, i32, vp, vp, vp]
        _lib.fff_oracle_leaf_forward.argtypes = [vp] * 6 + [i32, i32, i32, i64, i64, i64, i32, vp]
        _lib.fff_oracle_forward_soft.argtypes = [vp] * 7 + [i32, i32, i32, i64, i64, i64, i32, f64, vp, vp]
        _lib.fff_oracle_bucket.argtypes = [vp, i64, i32, vp, vp, vp]
        _lib.fff_oracle_node_entropy.argtypes = [vp, vp, vp, i32, i64, i64, i32, vp]
        _lib.fff_oracle_moe_top1.argtypes = [vp] * 7 + [i64, i32, i32, i64, i64, i64, i32, vp, vp, vp]
        _lib.fff_oracle_forward_block.argtypes = ([vp] * 3 + [f64] + [vp] * 8 + [i32] * 6 + [i64] * 3 +
                                                  [i32, vp, vp, vp])
        _lib.fff_oracle_set_threads.argtypes = [i32]
        _lib.fff_oracle_set_threads.restype = None
        for n in ("training_size", "inference_size"):
            f = getattr(_lib, "fff_oracle_" + n)
            f.argtypes, f.restype = [i32, i32, i32], i64
        for n in ("training_width", "inference_width"):
            f = getattr(_lib, "fff_oracle_" + n)
            f.argtypes, f.restype = [i32, i32], i64
    return _lib


def _dtype_code(arrs) -> int:
    kinds = {a.dtype for a in arrs if a is not None}
    if kinds == {np.dtype(np.float32)}:
        return 0
    if kinds == {np.dtype(np.uint16)}:
        return 1
    if kinds == {np.dtype(np.float64)}:
        return 2
    raise TypeError("oracle inputs must all be float32, all float64, or all uint16 (bf16 bits): %s" % kinds)


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _c(a):
    return None if a is None else np.ascontiguousarray(a)


def _shapes(x, leaf_w1, leaf_w2, depth, leaf_width):
    T, D = x.shape
    NL = 1 << depth
    assert leaf_w1.shape == (NL, leaf_width, D), (leaf_w1.shape, (NL, leaf_width, D))
    assert leaf_w2.shape[:2] == (NL, leaf_width)
    return T, D, leaf_w2.shape[2]


def forward_hard(x, node_w, node_b, leaf_w1, leaf_b1, leaf_w2, leaf_b2, depth, leaf_width, act,
                 want_out: bool = True) -> Tuple[Optional[np.ndarray], np.ndarray, np.ndarray]:
    """Forward_I.  Returns (out [T,O] fp64 or None, leaf_idx [T] int32, margin [T] fp64)."""
    x, leaf_w1, leaf_b1, leaf_w2, leaf_b2 = map(_c, (x, leaf_w1, leaf_b1, leaf_w2, leaf_b2))
    T, D, O = _shapes(x, leaf_w1, leaf_w2, depth, leaf_width)
    if depth == 0:
        node_w = np.zeros((0, D), x.dtype)
        node_b = np.zeros((0,), x.dtype)
    node_w, node_b = _c(node_w), _c(node_b)
    assert node_w.shape == ((1 << depth) - 1, D) and node_b.shape == ((1 << depth) - 1,)
    assert leaf_b1.shape == (1 << depth, leaf_width) and leaf_b2.shape == (1 << depth, O)
    dt = _dtype_code((x, node_w, node_b, leaf_w1, leaf_b1, leaf_w2, leaf_b2))
    out = np.empty((T, O), np.float64) if want_out else None
    idx = np.empty((T,), np.int32)
    margin = np.empty((T,), np.float64)
    rc = _load().fff_oracle_forward_hard(_p(x), _p(node_w), _p(node_b), _p(leaf_w1), _p(leaf_b1),
                                         _p(leaf_w2), _p(leaf_b2), depth, leaf_width, act, T, D, O,
                                         dt, _p(out), _p(idx), _p(margin))
    if rc:
        raise ValueError("fff_oracle_forward_hard: bad arguments (%d)" % rc)
    return out, idx, margin


def leaf_forward(x, leaf_w1, leaf_b1, leaf_w2, leaf_b2, leaf_idx, depth, leaf_width, act) -> np.ndarray:
    """The leaf network of the given leaf, per token.  Returns out [T,O] fp64."""
    x, leaf_w1, leaf_b1, leaf_w2, leaf_b2 = map(_c, (x, leaf_w1, leaf_b1, leaf_w2, leaf_b2))
    T, D, O = _shapes(x, leaf_w1, leaf_w2, depth, leaf_width)
    leaf_idx = np.ascontiguousarray(leaf_idx, dtype=np.int32)
    assert leaf_idx.shape == (T,)
    dt = _dtype_code((x, leaf_w1, leaf_b1, leaf_w2, leaf_b2))
    out = np.empty((T, O), np.float64)
    rc = _load().fff_oracle_leaf_forward(_p(x), _p(leaf_w1), _p(leaf_b1), _p(leaf_w2), _p(leaf_b2),
                                         _p(leaf_idx), depth, leaf_width, act, T, D, O, dt, _p(out))
    if rc:
        raise ValueError("fff_oracle_leaf_forward: bad arguments (%d)" % rc)
    return out


def forward_soft(x, node_w, node_b, leaf_w1, leaf_b1, leaf_w2, leaf_b2, depth, leaf_width, act,
                 node_scale: float = 1.0) -> Tuple[np.ndarray, np.ndarray]:
    """Forward_T.  Returns (out [T,O] fp64, mixture weights [T, 2^d] fp64)."""
    x, leaf_w1, leaf_b1, leaf_w2, leaf_b2 = map(_c, (x, leaf_w1, leaf_b1, leaf_w2, leaf_b2))
    T, D, O = _shapes(x, leaf_w1, leaf_w2, depth, leaf_width)
    if depth == 0:
        node_w = np.zeros((0, D), x.dtype)
        node_b = np.zeros((0,), x.dtype)
    node_w, node_b = _c(node_w), _c(node_b)
    dt = _dtype_code((x, node_w, node_b, leaf_w1, leaf_b1, leaf_w2, leaf_b2))
    out = np.empty((T, O), np.float64)
    mix = np.empty((T, 1 << depth), np.float64)
    rc = _load().fff_oracle_forward_soft(_p(x), _p(node_w), _p(node_b), _p(leaf_w1), _p(leaf_b1),
                                         _p(leaf_w2), _p(leaf_b2), depth, leaf_width, act, T, D, O,
                                         dt, float(node_scale), _p(out), _p(mix))
    if rc:
        raise ValueError("fff_oracle_forward_soft: bad arguments (%d)" % rc)
    return out, mix


def node_entropy(x, node_w, node_b, depth) -> np.ndarray:
    """Batch mean Bernoulli entropy (nats) of every node's choice score, [2^depth - 1] fp64."""
    x, node_w, node_b = map(_c, (x, node_w, node_b))
    T, D = x.shape
    NN = (1 << depth) - 1
    assert node_w.shape == (NN, D) and node_b.shape == (NN,)
    dt = _dtype_code((x, node_w, node_b))
    ent = np.empty((NN,), np.float64)
    rc = _load().fff_oracle_node_entropy(_p(x), _p(node_w), _p(node_b), depth, T, D, dt, _p(ent))
    if rc:
        raise ValueError("fff_oracle_node_entropy: bad arguments (%d)" % rc)
    return ent


def moe_top1(x, gate_w, gate_b, leaf_w1, leaf_b1, leaf_w2, leaf_b2, leaf_width, act,
             want_out: bool = True) -> Tuple[Optional[np.ndarray], np.ndarray, np.ndarray]:
    """Mixture of experts, one engaged expert, noiseless gating.  gate_w [G, D], gate_b [G] or None;
    experts stored like leaves ([G, l, D] ...).  Returns (out [T,O] fp64 or None, expert_idx [T],
    margin [T]: relative gap between the two largest gating logits)."""
    x, gate_w, leaf_w1, leaf_b1, leaf_w2, leaf_b2 = map(_c, (x, gate_w, leaf_w1, leaf_b1, leaf_w2, leaf_b2))
    gate_b = _c(gate_b)
    T, D = x.shape
    G = gate_w.shape[0]
    assert gate_w.shape == (G, D) and leaf_w1.shape == (G, leaf_width, D) and leaf_w2.shape[:2] == (G, leaf_width)
    O = leaf_w2.shape[2]
    assert leaf_b1.shape == (G, leaf_width) and leaf_b2.shape == (G, O)
    assert gate_b is None or gate_b.shape == (G,)
    dt = _dtype_code((x, gate_w, gate_b, leaf_w1, leaf_b1, leaf_w2, leaf_b2))
    out = np.empty((T, O), np.float64) if want_out else None
    idx = np.empty((T,), np.int32)
    margin = np.empty((T,), np.float64)
    rc = _load().fff_oracle_moe_top1(_p(x), _p(gate_w), _p(gate_b), _p(leaf_w1), _p(leaf_b1), _p(leaf_w2),
                                     _p(leaf_b2), G, leaf_width, act, T, D, O, dt, _p(out), _p(idx), _p(margin))
    if rc:
        raise ValueError("fff_oracle_moe_top1: bad arguments (%d)" % rc)
    return out, idx, margin


def forward_block(x, ln_gamma, ln_beta, ln_eps, node_w1, node_b1, node_w2, node_b2, leaf_w1, leaf_b1,
                  leaf_w2, leaf_b2, depth, node_size, leaf_width, act, residual: bool,
                  want_out: bool = True) -> Tuple[Optional[np.ndarray], np.ndarray, np.ndarray]:
    """Forward_I with nodes of `node_size` hidden neurons, on the layer-normalised input when
    ln_gamma/ln_beta are given (None, None: no normalisation), plus x when `residual`.
    node_w1 [NN, n, D], node_b1 [NN, n], node_w2 [NN, n], node_b2 [NN].
    Returns (out [T,O] fp64 or None, leaf_idx [T] int32, margin [T] fp64)."""
    x, leaf_w1, leaf_b1, leaf_w2, leaf_b2 = map(_c, (x, leaf_w1, leaf_b1, leaf_w2, leaf_b2))
    T, D, O = _shapes(x, leaf_w1, leaf_w2, depth, leaf_width)
    NN = (1 << depth) - 1
    if depth == 0:
        node_w1 = np.zeros((0, node_size, D), x.dtype)
        node_b1 = np.zeros((0, node_size), x.dtype)
        node_w2 = np.zeros((0, node_size), x.dtype)
        node_b2 = np.zeros((0,), x.dtype)
    node_w1, node_b1, node_w2, node_b2 = map(_c, (node_w1, node_b1, node_w2, node_b2))
    assert node_w1.shape == (NN, node_size, D) and node_b1.shape == (NN, node_size)
    assert node_w2.shape == (NN, node_size) and node_b2.shape == (NN,)
    assert leaf_b1.shape == (1 << depth, leaf_width) and leaf_b2.shape == (1 << depth, O)
    norm = ln_gamma is not None
    assert norm == (ln_beta is not None)
    ln_gamma, ln_beta = _c(ln_gamma), _c(ln_beta)
    if norm:
        assert ln_gamma.shape == (D,) and ln_beta.shape == (D,)
    dt = _dtype_code((x, ln_gamma, ln_beta, node_w1, node_b1, node_w2, node_b2, leaf_w1, leaf_b1, leaf_w2, leaf_b2))
    out = np.empty((T, O), np.float64) if want_out else None
    idx = np.empty((T,), np.int32)
    margin = np.empty((T,), np.float64)
    rc = _load().fff_oracle_forward_block(_p(x), _p(ln_gamma), _p(ln_beta), float(ln_eps), _p(node_w1),
                                          _p(node_b1), _p(node_w2), _p(node_b2), _p(leaf_w1), _p(leaf_b1),
                                          _p(leaf_w2), _p(leaf_b2), depth, node_size, leaf_width, act,
                                          int(norm), int(bool(residual)), T, D, O, dt, _p(out), _p(idx), _p(margin))
    if rc:
        raise ValueError("fff_oracle_forward_block: bad arguments (%d)" % rc)
    return out, idx, margin


def bucket(leaf_idx, depth) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """(count [2^d], offset [2^d + 1], perm [T]) of the per-leaf token lists."""
    leaf_idx = np.ascontiguousarray(leaf_idx, dtype=np.int32)
    T, NL = leaf_idx.shape[0], 1 << depth
    count = np.empty((NL,), np.int32)
    offset = np.empty((NL + 1,), np.int32)
    perm = np.empty((T,), np.int32)
    rc = _load().fff_oracle_bucket(_p(leaf_idx), T, depth, _p(count), _p(offset), _p(perm))
    if rc:
        raise ValueError("fff_oracle_bucket: leaf index out of range (%d)" % rc)
    return count, offset, perm


def training_size(depth, node_size, leaf_size):
    return int(_load().fff_oracle_training_size(depth, node_size, leaf_size))


def inference_size(depth, node_size, leaf_size):
    return int(_load().fff_oracle_inference_size(depth, node_size, leaf_size))


def training_width(depth, leaf_size):
    return int(_load().fff_oracle_training_width(depth, leaf_size))


def inference_width(depth, leaf_size):
    return int(_load().fff_oracle_inference_width(depth, leaf_size))


def set_threads(n: int) -> None:
    """Use n OpenMP threads from now on (timing the oracle on one core beside all cores)."""
    _load().fff_oracle_set_threads(int(n))


def num_threads() -> int:
    return int(_load().fff_oracle_num_threads())
