"""ctypes binding of include/fff.h.  Argument marshalling only.

The C ABI takes plain pointers plus (T, D, O, dtype) and cannot see the extents of the arrays
behind them; this layer can, so it checks every tensor's shape and dtype against the
Definition's sizes (2^depth - 1 node rows, 2^depth leaves of leaf_width neurons, D inputs,
O outputs) on the host, before any pointer reaches the library."""
from __future__ import annotations

import ctypes
import os
from typing import Optional

from . import build as _build

ACT_RELU = 0
ACT_GELU = 1
DTYPE_F32 = 0
DTYPE_BF16 = 1
ERR_SHAPE = 2
ERR_DTYPE = 3
MAX_DEPTH = 24


class FffError(RuntimeError):
    def __init__(self, status: int, where: str, detail: Optional[str] = None):
        self.status = status
        if detail is None:
            detail = lib().fff_last_device_error().decode()
        msg = "%s: %s (status %d)" % (where, fff_status_string(status), status)
        super().__init__(msg + (" -- " + detail if detail else ""))


_lib = None


def library_path() -> str:
    return _build.LIB


def lib() -> ctypes.CDLL:
    """The loaded C-ABI library.  Built first if no library is there at all."""
    global _lib
    if _lib is None:
        if not os.path.exists(_build.LIB):
            _build.build_library(force=True)
        # PyTorch ships a HIP runtime of its own; the tensors and streams handed to this library
        # live in that one.  Loading torch first makes the library bind to the same runtime instance
        # (a process that loaded the library first ended up with two, and the second saw no device).
        import torch  # noqa: F401
        L = ctypes.CDLL(_build.LIB)
        vp, i32, i64 = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64
        L.fff_forward_hard.argtypes = [vp] * 7 + [i32, i32, i32, vp, vp, vp, i64, i64, i64, i32]
        L.fff_forward_hard_static.argtypes = L.fff_forward_hard.argtypes
        L.fff_static_scratch_bytes.argtypes = []
        L.fff_static_scratch_bytes.restype = ctypes.c_size_t
        L.fff_descend.argtypes = [vp, vp, vp, i32, vp, vp, i64, i64, i32]
        L.fff_bucket.argtypes = [vp, i64, i32, vp, vp, vp, vp]
        L.fff_leaf_forward.argtypes = [vp] * 6 + [i32, i32, i32, vp, vp, i64, i64, i64, i32]
        L.fff_moe_top1_forward.argtypes = [vp] * 7 + [i32, i32, i32, vp, vp, vp, i64, i64, i64, i32]
        L.fff_forward_soft.argtypes = [vp] * 7 + [i32, i32, i32, vp, vp, vp, vp, i64, i64, i64, i32]
        L.fff_forward_block.argtypes = ([vp] * 3 + [ctypes.c_float] + [vp] * 8 + [i32] * 5 + [vp, vp, vp] +
                                        [i64, i64, i64, i32])
        L.fff_workspace_bytes.argtypes = [i64, i32]
        L.fff_workspace_bytes.restype = ctypes.c_size_t
        L.fff_workspace_bytes_moe.argtypes = [i64, i32]
        L.fff_workspace_bytes_moe.restype = ctypes.c_size_t
        L.fff_workspace_bytes_soft.argtypes = [i64, i64, i32, i32]
        L.fff_workspace_bytes_soft.restype = ctypes.c_size_t
        L.fff_set_workspace.argtypes = [vp, ctypes.c_size_t, vp]
        L.fff_reserve_workspace.argtypes = [i64, i32]
        L.fff_reserve_workspace_bytes.argtypes = [ctypes.c_size_t]
        L.fff_release_workspace.argtypes = []
        L.fff_set_option.argtypes = [ctypes.c_char_p, i64]
        L.fff_get_option.argtypes = [ctypes.c_char_p, ctypes.POINTER(i64)]
        L.fff_debug_option.argtypes = [ctypes.c_char_p, i64, ctypes.POINTER(i64)]
        L.fff_status_string.argtypes = [i32]
        L.fff_status_string.restype = ctypes.c_char_p
        L.fff_last_device_error.argtypes = []
        L.fff_last_device_error.restype = ctypes.c_char_p
        L.fff_last_launch.argtypes = []
        L.fff_last_launch.restype = ctypes.c_char_p
        L.fff_version.argtypes = []
        L.fff_stage_times.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.POINTER(i64)]
        _lib = L
    return _lib


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _dtype_code(t) -> int:
    import torch
    if t.dtype == torch.float32:
        return DTYPE_F32
    if t.dtype == torch.bfloat16:
        return DTYPE_BF16
    raise TypeError("FFF tensors must be float32 or bfloat16, got %s" % t.dtype)


def _stream_handle(stream) -> Optional[int]:
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


def _check_dense(*tensors):
    for t in tensors:
        if t is None:
            continue
        if not t.is_cuda:
            raise ValueError("FFF tensors must live on the GPU")
        if not t.is_contiguous():
            raise ValueError("FFF tensors must be dense row-major")


def _check(rc: int, where: str) -> None:
    if rc != 0:
        raise FffError(rc, where)


def _expect(where: str, name: str, t, shape, dtype) -> None:
    """t must be a tensor of exactly `shape` and `dtype` (host-side check, no device access)."""
    if t is None:
        return      # a missing required tensor is the library's FFF_ERR_NULL
    if tuple(t.shape) != tuple(shape):
        raise FffError(ERR_SHAPE, where, "%s has shape %s, the other arguments imply %s"
                       % (name, tuple(t.shape), tuple(shape)))
    if t.dtype != dtype:
        raise FffError(ERR_DTYPE, where, "%s is %s, expected %s" % (name, t.dtype, dtype))


def _rows(where: str, name: str, t):
    if t is None or t.dim() != 2:
        raise FffError(ERR_SHAPE, where, "%s must be a matrix [tokens, features]" % name)
    return int(t.shape[0]), int(t.shape[1])


def _in_range(depth, *widths) -> bool:
    """Sizes the library itself rejects (FFF_ERR_RANGE) are left to it; shapes are only derived
    from values it accepts."""
    return isinstance(depth, int) and 0 <= depth <= MAX_DEPTH and all(isinstance(w, int) and w >= 1 for w in widths)


def _check_leaves(where, x, T, D, O, depth, leaf_width, leaf_w1, leaf_b1, leaf_w2, leaf_b2, out, idx, idx_name):
    import torch
    NL = 1 << depth
    _expect(where, "leaf_w1", leaf_w1, (NL, leaf_width, D), x.dtype)
    _expect(where, "leaf_b1", leaf_b1, (NL, leaf_width), x.dtype)
    _expect(where, "leaf_w2", leaf_w2, (NL, leaf_width, O), x.dtype)
    _expect(where, "leaf_b2", leaf_b2, (NL, O), x.dtype)
    _expect(where, "out", out, (T, O), x.dtype)
    _expect(where, idx_name, idx, (T,), torch.int32)


def fff_forward_hard(x, node_w, node_b, leaf_w1, leaf_b1, leaf_w2, leaf_b2, depth, leaf_width, act,
                     out, leaf_idx=None, stream=None, static_scratch=False) -> None:
    """Forward_I for x [T, D] -> out [T, O] (and leaf_idx [T] int32 if given).  static_scratch=True
    calls fff_forward_hard_static, the variant that allocates nothing."""
    where = "fff_forward_hard_static" if static_scratch else "fff_forward_hard"
    T, D = _rows(where, "x", x)
    _, O = _rows(where, "out", out)
    if _in_range(depth, leaf_width):
        if depth > 0:
            _expect(where, "node_w", node_w, ((1 << depth) - 1, D), x.dtype)
            _expect(where, "node_b", node_b, ((1 << depth) - 1,), x.dtype)
        _check_leaves(where, x, T, D, O, depth, leaf_width, leaf_w1, leaf_b1, leaf_w2, leaf_b2, out, leaf_idx, "leaf_idx")
    _check_dense(x, node_w, node_b, leaf_w1, leaf_b1, leaf_w2, leaf_b2, out, leaf_idx)
    entry = lib().fff_forward_hard_static if static_scratch else lib().fff_forward_hard
    _check(entry(_ptr(x), _ptr(node_w), _ptr(node_b), _ptr(leaf_w1), _ptr(leaf_b1), _ptr(leaf_w2), _ptr(leaf_b2),
                 depth, leaf_width, act, _ptr(out), _ptr(leaf_idx), _stream_handle(stream), T, D, O, _dtype_code(x)),
           where)


def fff_forward_hard_static(x, node_w, node_b, leaf_w1, leaf_b1, leaf_w2, leaf_b2, depth, leaf_width, act,
                            out, leaf_idx=None, stream=None) -> None:
    fff_forward_hard(x, node_w, node_b, leaf_w1, leaf_b1, leaf_w2, leaf_b2, depth, leaf_width, act, out, leaf_idx,
                     stream, static_scratch=True)


def fff_static_scratch_bytes() -> int:
    return int(lib().fff_static_scratch_bytes())


def fff_descend(x, node_w, node_b, depth, leaf_idx, stream=None) -> None:
    import torch
    where = "fff_descend"
    T, D = _rows(where, "x", x)
    if _in_range(depth):
        if depth > 0:
            _expect(where, "node_w", node_w, ((1 << depth) - 1, D), x.dtype)
            _expect(where, "node_b", node_b, ((1 << depth) - 1,), x.dtype)
        _expect(where, "leaf_idx", leaf_idx, (T,), torch.int32)
    _check_dense(x, node_w, node_b, leaf_idx)
    _check(lib().fff_descend(_ptr(x), _ptr(node_w), _ptr(node_b), depth, _ptr(leaf_idx),
                             _stream_handle(stream), T, D, _dtype_code(x)), where)


def fff_bucket(leaf_idx, depth, count=None, offset=None, perm=None, stream=None) -> None:
    import torch
    where = "fff_bucket"
    if leaf_idx is None or leaf_idx.dim() != 1:
        raise FffError(ERR_SHAPE, where, "leaf_idx must be a vector [tokens]")
    T = int(leaf_idx.shape[0])
    _expect(where, "leaf_idx", leaf_idx, (T,), torch.int32)
    if _in_range(depth):
        _expect(where, "count", count, (1 << depth,), torch.int32)
        _expect(where, "offset", offset, ((1 << depth) + 1,), torch.int32)
        _expect(where, "perm", perm, (T,), torch.int32)
    _check_dense(leaf_idx, count, offset, perm)
    _check(lib().fff_bucket(_ptr(leaf_idx), T, depth, _ptr(count), _ptr(offset),
                            _ptr(perm), _stream_handle(stream)), where)


def fff_leaf_forward(x, leaf_w1, leaf_b1, leaf_w2, leaf_b2, leaf_idx, depth, leaf_width, act, out,
                     stream=None) -> None:
    where = "fff_leaf_forward"
    T, D = _rows(where, "x", x)
    _, O = _rows(where, "out", out)
    if _in_range(depth, leaf_width):
        _check_leaves(where, x, T, D, O, depth, leaf_width, leaf_w1, leaf_b1, leaf_w2, leaf_b2, out, leaf_idx, "leaf_idx")
    _check_dense(x, leaf_w1, leaf_b1, leaf_w2, leaf_b2, leaf_idx, out)
    _check(lib().fff_leaf_forward(_ptr(x), _ptr(leaf_w1), _ptr(leaf_b1), _ptr(leaf_w2), _ptr(leaf_b2),
                                  _ptr(leaf_idx), depth, leaf_width, act, _ptr(out),
                                  _stream_handle(stream), T, D, O, _dtype_code(x)), where)


def fff_moe_top1_forward(x, gate_w, gate_b, leaf_w1, leaf_b1, leaf_w2, leaf_b2, log2_experts, leaf_width, act,
                         out, expert_idx=None, stream=None) -> None:
    where = "fff_moe_top1_forward"
    T, D = _rows(where, "x", x)
    _, O = _rows(where, "out", out)
    if _in_range(log2_experts, leaf_width):
        _expect(where, "gate_w", gate_w, (1 << log2_experts, D), x.dtype)
        _expect(where, "gate_b", gate_b, (1 << log2_experts,), x.dtype)
        _check_leaves(where, x, T, D, O, log2_experts, leaf_width, leaf_w1, leaf_b1, leaf_w2, leaf_b2, out,
                      expert_idx, "expert_idx")
    _check_dense(x, gate_w, gate_b, leaf_w1, leaf_b1, leaf_w2, leaf_b2, expert_idx, out)
    _check(lib().fff_moe_top1_forward(_ptr(x), _ptr(gate_w), _ptr(gate_b), _ptr(leaf_w1), _ptr(leaf_b1),
                                      _ptr(leaf_w2), _ptr(leaf_b2), log2_experts, leaf_width, act, _ptr(out),
                                      _ptr(expert_idx), _stream_handle(stream), T, D, O, _dtype_code(x)),
           where)


def fff_forward_soft(x, node_w, node_b, leaf_w1, leaf_b1, leaf_w2, leaf_b2, depth, leaf_width, act, out,
                     mix=None, entropy=None, stream=None) -> None:
    """Forward_T: the soft mixture over all leaves.  mix [T, 2^depth] and entropy [2^depth - 1] are
    optional float32 device outputs."""
    import torch
    where = "fff_forward_soft"
    T, D = _rows(where, "x", x)
    _, O = _rows(where, "out", out)
    if _in_range(depth, leaf_width):
        if depth > 0:
            _expect(where, "node_w", node_w, ((1 << depth) - 1, D), x.dtype)
            _expect(where, "node_b", node_b, ((1 << depth) - 1,), x.dtype)
        _check_leaves(where, x, T, D, O, depth, leaf_width, leaf_w1, leaf_b1, leaf_w2, leaf_b2, out, None, "")
        _expect(where, "mix", mix, (T, 1 << depth), torch.float32)
        if entropy is not None and entropy.dtype != torch.float32:
            raise FffError(ERR_DTYPE, where, "entropy is %s, expected torch.float32" % entropy.dtype)
        if entropy is not None and (entropy.dim() != 1 or entropy.shape[0] < (1 << depth) - 1):
            raise FffError(ERR_SHAPE, where, "entropy has shape %s, needs [%d]" % (tuple(entropy.shape), (1 << depth) - 1))
    _check_dense(x, node_w, node_b, leaf_w1, leaf_b1, leaf_w2, leaf_b2, out, mix, entropy)
    _check(lib().fff_forward_soft(_ptr(x), _ptr(node_w), _ptr(node_b), _ptr(leaf_w1), _ptr(leaf_b1),
                                  _ptr(leaf_w2), _ptr(leaf_b2), depth, leaf_width, act, _ptr(out),
                                  _ptr(mix), _ptr(entropy), _stream_handle(stream), T, D, O, _dtype_code(x)),
           where)


def fff_forward_block(x, ln_gamma, ln_beta, ln_eps, node_w1, node_b1, node_w2, node_b2, leaf_w1, leaf_b1,
                      leaf_w2, leaf_b2, depth, node_size, leaf_width, act, residual, out, leaf_idx=None,
                      stream=None) -> None:
    """Forward_I with nodes of `node_size` hidden neurons as a pre-norm residual layer:
    out = FFF(LayerNorm(x)) (+ x when `residual`); ln_gamma = ln_beta = None skips the
    normalisation.  out may be x itself."""
    where = "fff_forward_block"
    T, D = _rows(where, "x", x)
    _, O = _rows(where, "out", out)
    if _in_range(depth, leaf_width, node_size):
        NN = (1 << depth) - 1
        _expect(where, "ln_gamma", ln_gamma, (D,), x.dtype)
        _expect(where, "ln_beta", ln_beta, (D,), x.dtype)
        if depth > 0:
            _expect(where, "node_w1", node_w1, (NN, node_size, D), x.dtype)
            _expect(where, "node_b1", node_b1, (NN, node_size), x.dtype)
            _expect(where, "node_w2", node_w2, (NN, node_size), x.dtype)
            _expect(where, "node_b2", node_b2, (NN,), x.dtype)
        _check_leaves(where, x, T, D, O, depth, leaf_width, leaf_w1, leaf_b1, leaf_w2, leaf_b2, out, leaf_idx, "leaf_idx")
    _check_dense(x, ln_gamma, ln_beta, node_w1, node_b1, node_w2, node_b2, leaf_w1, leaf_b1, leaf_w2, leaf_b2,
                 out, leaf_idx)
    _check(lib().fff_forward_block(_ptr(x), _ptr(ln_gamma), _ptr(ln_beta), float(ln_eps), _ptr(node_w1),
                                   _ptr(node_b1), _ptr(node_w2), _ptr(node_b2), _ptr(leaf_w1), _ptr(leaf_b1),
                                   _ptr(leaf_w2), _ptr(leaf_b2), depth, node_size, leaf_width, act,
                                   int(bool(residual)), _ptr(out), _ptr(leaf_idx), _stream_handle(stream),
                                   T, D, O, _dtype_code(x)),
           where)


def fff_workspace_bytes(T: int, depth: int) -> int:
    return int(lib().fff_workspace_bytes(T, depth))


def fff_workspace_bytes_moe(T: int, log2_experts: int) -> int:
    return int(lib().fff_workspace_bytes_moe(T, log2_experts))


def fff_workspace_bytes_soft(T: int, O: int, depth: int, leaf_width: int) -> int:
    return int(lib().fff_workspace_bytes_soft(T, O, depth, leaf_width))


def fff_set_workspace(buf, stream=None) -> None:
    """Every later call on the current device works in `buf` (a dense device tensor the caller keeps
    alive), or in the library's own workspace again for buf = None."""
    if buf is None:
        _check(lib().fff_set_workspace(None, 0, _stream_handle(stream)), "fff_set_workspace")
        return
    _check_dense(buf)
    _check(lib().fff_set_workspace(_ptr(buf), buf.numel() * buf.element_size(), _stream_handle(stream)),
           "fff_set_workspace")


def fff_reserve_workspace(T: int, depth: int) -> None:
    _check(lib().fff_reserve_workspace(T, depth), "fff_reserve_workspace")


def fff_reserve_workspace_bytes(nbytes: int) -> None:
    _check(lib().fff_reserve_workspace_bytes(nbytes), "fff_reserve_workspace_bytes")


def fff_release_workspace() -> None:
    _check(lib().fff_release_workspace(), "fff_release_workspace")


def fff_set_option(name: str, value: int) -> None:
    _check(lib().fff_set_option(name.encode(), int(value)), "fff_set_option(%s)" % name)


def fff_get_option(name: str) -> int:
    v = ctypes.c_int64(0)
    _check(lib().fff_get_option(name.encode(), ctypes.byref(v)), "fff_get_option(%s)" % name)
    return int(v.value)


def fff_debug_option(name: str, value: int = -1) -> int:
    """Set (value >= 0) or read (value < 0) an experiment switch; returns its value afterwards."""
    v = ctypes.c_int64(0)
    _check(lib().fff_debug_option(name.encode(), int(value), ctypes.byref(v)), "fff_debug_option(%s)" % name)
    return int(v.value)


def fff_stage_times():
    """(ms_descent, ms_bucketing, ms_leaf_first_kernel, ms_leaf_second_kernel, calls) summed since
    the last read.  The leaf stage is two kernels (hidden activations, output rows) on the MFMA
    tile path and one otherwise (then the fourth figure is the gap between two marks)."""
    ms = (ctypes.c_double * 4)()
    calls = ctypes.c_int64(0)
    _check(lib().fff_stage_times(ms, ctypes.byref(calls)), "fff_stage_times")
    return ms[0], ms[1], ms[2], ms[3], int(calls.value)


def fff_status_string(status: int) -> str:
    return lib().fff_status_string(int(status)).decode()


def fff_last_launch() -> str:
    return lib().fff_last_launch().decode()


def fff_version() -> int:
    return int(lib().fff_version())
