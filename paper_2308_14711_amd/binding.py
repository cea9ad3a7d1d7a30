"""ctypes binding of include/fff.h.  Argument marshalling only."""
from __future__ import annotations

import ctypes
import os
from typing import Optional

from . import build as _build

ACT_RELU = 0
ACT_GELU = 1
DTYPE_F32 = 0
DTYPE_BF16 = 1


class FffError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
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
        L.fff_descend.argtypes = [vp, vp, vp, i32, vp, vp, i64, i64, i32]
        L.fff_bucket.argtypes = [vp, i64, i32, vp, vp, vp, vp]
        L.fff_leaf_forward.argtypes = [vp] * 6 + [i32, i32, i32, vp, vp, i64, i64, i64, i32]
        L.fff_moe_top1_forward.argtypes = [vp] * 7 + [i32, i32, i32, vp, vp, vp, i64, i64, i64, i32]
        L.fff_forward_soft.argtypes = [vp] * 7 + [i32, i32, i32, vp, vp, vp, vp, i64, i64, i64, i32]
        L.fff_forward_block.argtypes = ([vp] * 3 + [ctypes.c_float] + [vp] * 8 + [i32] * 5 + [vp, vp, vp] +
                                        [i64, i64, i64, i32])
        L.fff_probe_gather.argtypes = [vp, i64, i64, i32, i64, i32, i32, vp, vp]
        L.fff_workspace_bytes.argtypes = [i64, i32]
        L.fff_workspace_bytes.restype = ctypes.c_size_t
        L.fff_reserve_workspace.argtypes = [i64, i32]
        L.fff_release_workspace.argtypes = []
        L.fff_set_option.argtypes = [ctypes.c_char_p, i64]
        L.fff_get_option.argtypes = [ctypes.c_char_p, ctypes.POINTER(i64)]
        L.fff_status_string.argtypes = [i32]
        L.fff_status_string.restype = ctypes.c_char_p
        L.fff_last_device_error.argtypes = []
        L.fff_last_device_error.restype = ctypes.c_char_p
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


def fff_forward_hard(x, node_w, node_b, leaf_w1, leaf_b1, leaf_w2, leaf_b2, depth, leaf_width, act,
                     out, leaf_idx=None, stream=None) -> None:
    """Forward_I for x [T, D] -> out [T, O] (and leaf_idx [T] int32 if given)."""
    _check_dense(x, node_w, node_b, leaf_w1, leaf_b1, leaf_w2, leaf_b2, out, leaf_idx)
    T, D = x.shape
    O = out.shape[1]
    _check(lib().fff_forward_hard(_ptr(x), _ptr(node_w), _ptr(node_b), _ptr(leaf_w1), _ptr(leaf_b1),
                                  _ptr(leaf_w2), _ptr(leaf_b2), depth, leaf_width, act, _ptr(out),
                                  _ptr(leaf_idx), _stream_handle(stream), T, D, O, _dtype_code(x)),
           "fff_forward_hard")


def fff_descend(x, node_w, node_b, depth, leaf_idx, stream=None) -> None:
    _check_dense(x, node_w, node_b, leaf_idx)
    T, D = x.shape
    _check(lib().fff_descend(_ptr(x), _ptr(node_w), _ptr(node_b), depth, _ptr(leaf_idx),
                             _stream_handle(stream), T, D, _dtype_code(x)), "fff_descend")


def fff_bucket(leaf_idx, depth, count=None, offset=None, perm=None, stream=None) -> None:
    _check_dense(leaf_idx, count, offset, perm)
    _check(lib().fff_bucket(_ptr(leaf_idx), leaf_idx.shape[0], depth, _ptr(count), _ptr(offset),
                            _ptr(perm), _stream_handle(stream)), "fff_bucket")


def fff_leaf_forward(x, leaf_w1, leaf_b1, leaf_w2, leaf_b2, leaf_idx, depth, leaf_width, act, out,
                     stream=None) -> None:
    _check_dense(x, leaf_w1, leaf_b1, leaf_w2, leaf_b2, leaf_idx, out)
    T, D = x.shape
    O = out.shape[1]
    _check(lib().fff_leaf_forward(_ptr(x), _ptr(leaf_w1), _ptr(leaf_b1), _ptr(leaf_w2), _ptr(leaf_b2),
                                  _ptr(leaf_idx), depth, leaf_width, act, _ptr(out),
                                  _stream_handle(stream), T, D, O, _dtype_code(x)), "fff_leaf_forward")


def fff_moe_top1_forward(x, gate_w, gate_b, leaf_w1, leaf_b1, leaf_w2, leaf_b2, log2_experts, leaf_width, act,
                         out, expert_idx=None, stream=None) -> None:
    _check_dense(x, gate_w, gate_b, leaf_w1, leaf_b1, leaf_w2, leaf_b2, expert_idx, out)
    T, D = x.shape
    O = out.shape[1]
    _check(lib().fff_moe_top1_forward(_ptr(x), _ptr(gate_w), _ptr(gate_b), _ptr(leaf_w1), _ptr(leaf_b1),
                                      _ptr(leaf_w2), _ptr(leaf_b2), log2_experts, leaf_width, act, _ptr(out),
                                      _ptr(expert_idx), _stream_handle(stream), T, D, O, _dtype_code(x)),
           "fff_moe_top1_forward")


def fff_forward_soft(x, node_w, node_b, leaf_w1, leaf_b1, leaf_w2, leaf_b2, depth, leaf_width, act, out,
                     mix=None, entropy=None, stream=None) -> None:
    """Forward_T: the soft mixture over all leaves.  mix [T, 2^depth] and entropy [2^depth - 1] are
    optional float32 device outputs."""
    _check_dense(x, node_w, node_b, leaf_w1, leaf_b1, leaf_w2, leaf_b2, out, mix, entropy)
    T, D = x.shape
    O = out.shape[1]
    _check(lib().fff_forward_soft(_ptr(x), _ptr(node_w), _ptr(node_b), _ptr(leaf_w1), _ptr(leaf_b1),
                                  _ptr(leaf_w2), _ptr(leaf_b2), depth, leaf_width, act, _ptr(out),
                                  _ptr(mix), _ptr(entropy), _stream_handle(stream), T, D, O, _dtype_code(x)),
           "fff_forward_soft")


def fff_forward_block(x, ln_gamma, ln_beta, ln_eps, node_w1, node_b1, node_w2, node_b2, leaf_w1, leaf_b1,
                      leaf_w2, leaf_b2, depth, node_size, leaf_width, act, residual, out, leaf_idx=None,
                      stream=None) -> None:
    """Forward_I with nodes of `node_size` hidden neurons as a pre-norm residual layer:
    out = FFF(LayerNorm(x)) (+ x when `residual`); ln_gamma = ln_beta = None skips the
    normalisation.  out may be x itself."""
    _check_dense(x, ln_gamma, ln_beta, node_w1, node_b1, node_w2, node_b2, leaf_w1, leaf_b1, leaf_w2, leaf_b2,
                 out, leaf_idx)
    T, D = x.shape
    O = out.shape[1]
    _check(lib().fff_forward_block(_ptr(x), _ptr(ln_gamma), _ptr(ln_beta), float(ln_eps), _ptr(node_w1),
                                   _ptr(node_b1), _ptr(node_w2), _ptr(node_b2), _ptr(leaf_w1), _ptr(leaf_b1),
                                   _ptr(leaf_w2), _ptr(leaf_b2), depth, node_size, leaf_width, act,
                                   int(bool(residual)), _ptr(out), _ptr(leaf_idx), _stream_handle(stream),
                                   T, D, O, _dtype_code(x)),
           "fff_forward_block")


def fff_probe_gather(table, row_bytes: int, rows_in_flight: int, blocks: int, iters: int, dependent: bool,
                     sink, stream=None) -> int:
    """Row-gather microbenchmark over `table` (a zero-filled byte tensor whose size is a power of two
    rows of row_bytes).  Returns the bytes the launch reads."""
    _check_dense(table, sink)
    rows = table.numel() * table.element_size() // row_bytes
    _check(lib().fff_probe_gather(_ptr(table), rows, row_bytes, rows_in_flight, blocks, iters, int(bool(dependent)),
                                  _ptr(sink), _stream_handle(stream)), "fff_probe_gather")
    return blocks * 32 * iters * rows_in_flight * row_bytes


def fff_workspace_bytes(T: int, depth: int) -> int:
    return int(lib().fff_workspace_bytes(T, depth))


def fff_reserve_workspace(T: int, depth: int) -> None:
    _check(lib().fff_reserve_workspace(T, depth), "fff_reserve_workspace")


def fff_release_workspace() -> None:
    _check(lib().fff_release_workspace(), "fff_release_workspace")


def fff_set_option(name: str, value: int) -> None:
    _check(lib().fff_set_option(name.encode(), int(value)), "fff_set_option(%s)" % name)


def fff_get_option(name: str) -> int:
    v = ctypes.c_int64(0)
    _check(lib().fff_get_option(name.encode(), ctypes.byref(v)), "fff_get_option(%s)" % name)
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


def fff_version() -> int:
    return int(lib().fff_version())
