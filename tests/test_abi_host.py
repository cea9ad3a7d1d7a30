"""Host-side checks of the C-ABI library that need no GPU: it loads, exports
every symbol include/fff.h declares, and rejects bad arguments before touching
the device."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    import paper_2308_14711_amd as F
    return F.lib()


def test_every_declared_symbol_is_exported(L):
    header = open(os.path.join(ROOT, "include", "fff.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    names = set(re.findall(r"\b(fff_[a-z_]+)\s*\(", header))
    assert {"fff_forward_hard", "fff_descend", "fff_bucket", "fff_leaf_forward", "fff_workspace_bytes",
            "fff_status_string"} <= names
    for n in sorted(names):
        assert hasattr(L, n), "library does not export %s" % n


def test_status_strings(L):
    import paper_2308_14711_amd as F
    seen = {F.fff_status_string(i) for i in range(9)}
    assert len(seen) == 9 and "ok" in seen
    assert F.fff_status_string(99) == "unknown status"
    assert F.fff_version() >= 100


def test_workspace_size_is_monotone(L):
    import paper_2308_14711_amd as F
    a = F.fff_workspace_bytes(1000, 4)
    b = F.fff_workspace_bytes(100000, 4)
    c = F.fff_workspace_bytes(100000, 12)
    assert 0 < a < b < c
    assert F.fff_workspace_bytes(-1, 3) == 0 and F.fff_workspace_bytes(10, 25) == 0
    assert F.fff_workspace_bytes(1 << 20, 24) < (1 << 30)


def _call(lib_, **kw):
    P = ctypes.c_void_p
    a = dict(x=P(256), node_w=P(512), node_b=P(768), w1=P(1024), b1=P(1280), w2=P(1536), b2=P(1792),
             depth=3, L=4, act=0, out=P(1 << 40), idx=None, stream=None, T=8, D=64, O=16, dtype=0)
    a.update(kw)
    return lib_.fff_forward_hard(a["x"], a["node_w"], a["node_b"], a["w1"], a["b1"], a["w2"], a["b2"],
                              a["depth"], a["L"], a["act"], a["out"], a["idx"], a["stream"],
                              a["T"], a["D"], a["O"], a["dtype"])


def test_bad_arguments_are_rejected_on_the_host(L):
    """None of these reaches a HIP call (there is no GPU in this test)."""
    OK, NULL, SHAPE, DTYPE, RANGE, UNSUP, ALIAS = 0, 1, 2, 3, 4, 5, 8
    assert _call(L, T=0) == OK                       # empty batch: nothing to do
    assert _call(L, x=None) == NULL
    assert _call(L, out=None) == NULL
    assert _call(L, node_w=None) == NULL             # depth > 0 needs nodes
    assert _call(L, b2=None) == NULL
    assert _call(L, depth=-1) == RANGE
    assert _call(L, depth=25) == RANGE
    assert _call(L, L=0) == RANGE
    assert _call(L, L=5000) == RANGE
    assert _call(L, T=-3) == RANGE
    assert _call(L, D=0) == SHAPE
    assert _call(L, O=0) == SHAPE
    assert _call(L, T=1 << 30, D=1 << 20) == SHAPE
    assert _call(L, dtype=2) == DTYPE
    assert _call(L, act=7) == UNSUP
    assert _call(L, out=ctypes.c_void_p(256 + 64)) == ALIAS
    assert L.fff_descend(None, None, None, 2, None, None, 4, 8, 0) == NULL
    assert L.fff_descend(None, None, None, 2, None, None, 0, 8, 0) == OK
    assert L.fff_bucket(None, 5, 3, None, None, None, None) == NULL
    assert L.fff_bucket(None, 5, 30, None, None, None, None) == RANGE
    assert L.fff_leaf_forward(None, None, None, None, None, None, 2, 1, 0, None, None, 3, 8, 8, 1) == NULL
    moe = lambda **kw: L.fff_moe_top1_forward(
        kw.get("x", ctypes.c_void_p(256)), kw.get("gate_w", ctypes.c_void_p(1 << 20)), None, ctypes.c_void_p(2 << 20),
        ctypes.c_void_p(3 << 20), ctypes.c_void_p(4 << 20), ctypes.c_void_p(5 << 20), kw.get("g", 3), 2, kw.get("act", 0),
        ctypes.c_void_p(6 << 20), None, None, kw.get("T", 4), kw.get("D", 16), 8, kw.get("dtype", 1))
    assert moe(T=0) == OK
    assert moe(gate_w=None) == NULL
    assert moe(g=25) == RANGE
    assert moe(act=9) == UNSUP
    assert moe(dtype=0) == UNSUP                      # the gating runs on the bf16 matrix cores only
    assert moe(D=12) == UNSUP                         # rows must be whole 16-byte vectors
    assert L.fff_set_option(b"last_path", 1) == UNSUP  # read-only


def test_options(L):
    import paper_2308_14711_amd as F
    assert F.fff_get_option("bucketing") == 1
    F.fff_set_option("bucketing", 0)
    assert F.fff_get_option("bucketing") == 0
    F.fff_set_option("bucketing", 1)
    with pytest.raises(F.FffError):
        F.fff_set_option("no_such_option", 1)


def test_forward_soft_rejects_bad_arguments_on_the_host(L):
    OK, NULL, SHAPE, RANGE, UNSUP = 0, 1, 2, 4, 5
    soft = lambda **kw: L.fff_forward_soft(
        kw.get("x", ctypes.c_void_p(256)), kw.get("node_w", ctypes.c_void_p(1 << 20)), ctypes.c_void_p(2 << 20),
        ctypes.c_void_p(3 << 20), ctypes.c_void_p(4 << 20), ctypes.c_void_p(5 << 20), ctypes.c_void_p(6 << 20),
        kw.get("depth", 3), 2, kw.get("act", 0), kw.get("out", ctypes.c_void_p(7 << 20)), None, None, None,
        kw.get("T", 4), kw.get("D", 16), 8, kw.get("dtype", 1))
    assert soft(T=0) == OK
    assert soft(x=None) == NULL
    assert soft(node_w=None) == NULL
    assert soft(depth=25) == RANGE
    assert soft(act=9) == UNSUP
    assert soft(dtype=0) == UNSUP           # bf16 only
    assert soft(D=12) == UNSUP              # rows must be whole 16-byte vectors
    assert soft(T=1 << 20, depth=24, out=ctypes.c_void_p(1 << 44)) == SHAPE   # the dense intermediates would not fit any device


def test_forward_block_rejects_bad_arguments_on_the_host(L):
    OK, NULL, SHAPE, RANGE, UNSUP, ALIAS = 0, 1, 2, 4, 5, 8
    p = lambda mb: ctypes.c_void_p(mb << 20)
    blk = lambda **kw: L.fff_forward_block(
        kw.get("x", p(1)), kw.get("gamma", p(2)), kw.get("beta", p(3)), kw.get("eps", 1e-5),
        kw.get("node_w1", p(4)), p(5), p(6), p(7), p(8), p(9), p(10), p(11),
        kw.get("depth", 3), kw.get("n", 2), 2, kw.get("act", 0), kw.get("residual", 1),
        kw.get("out", p(12)), None, None, kw.get("T", 4), kw.get("D", 16), kw.get("O", 16), kw.get("dtype", 1))
    assert blk(T=0) == OK
    assert blk(x=None) == NULL
    assert blk(node_w1=None) == NULL
    assert blk(gamma=None) == NULL                    # scale without shift
    assert blk(beta=None) == NULL
    assert blk(eps=-1.0) == RANGE
    assert blk(eps=float("nan")) == RANGE
    assert blk(n=0) == RANGE
    assert blk(depth=25) == RANGE
    assert blk(O=8) == SHAPE                          # the residual sum needs rows of one width
    assert blk(act=9) == UNSUP
    assert blk(out=ctypes.c_void_p((1 << 20) + 32)) == ALIAS


def test_bench_probe_library_is_separate_and_checks_its_arguments():
    """The microbenchmarks of bench.py live in a library of their own: the product ABI exports none
    of them, and the probe library rejects bad arguments on the host."""
    import paper_2308_14711_amd as F
    from paper_2308_14711_amd import build
    assert not hasattr(F.lib(), "fff_probe_gather") and not hasattr(F.lib(), "fffb_gather")
    P = ctypes.CDLL(build.PROBE_LIB)
    vp, i32, i64 = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64
    P.fffb_gather.argtypes = [vp, i64, i64, i32, i64, i32, i32, vp, vp]
    P.fffb_copy.argtypes = [vp, vp, i64, i64, vp]
    p = lambda mb: ctypes.c_void_p(mb << 20)
    probe = lambda **kw: P.fffb_gather(kw.get("table", p(1)), kw.get("rows", 1024), kw.get("row_bytes", 1536),
                                       kw.get("k", 4), kw.get("blocks", 8), kw.get("iters", 2), 1,
                                       kw.get("sink", p(64)), None)
    for bad in (dict(table=None), dict(sink=None), dict(rows=1000), dict(row_bytes=100), dict(k=3), dict(blocks=0),
                dict(iters=0)):
        assert probe(**bad) == -1, bad
    assert P.fffb_copy(None, p(1), 1024, 8, None) == -1
    assert P.fffb_copy(p(2), p(1), 1000, 8, None) == -1      # whole 16-byte pieces only
    assert P.fffb_copy(p(2), p(1), 1024, 0, None) == -1


def test_workspace_entries_on_the_host(L):
    """Sizing functions and the argument checks of fff_set_workspace (no device is touched: a
    misaligned or too short buffer is rejected before the first HIP call)."""
    import paper_2308_14711_amd as F
    WORKSPACE = 6
    hard = F.fff_workspace_bytes(4096, 10)
    assert F.fff_workspace_bytes_moe(4096, 10) > hard            # plus the gating candidates
    assert F.fff_workspace_bytes_moe(4096, 30) == 0 and F.fff_workspace_bytes_moe(-1, 3) == 0
    soft = F.fff_workspace_bytes_soft(1000, 768, 8, 8)
    # the documented estimate: 4 T 2^(d+1) + 2 (T + O) 2^d (l + 1) bytes
    est = 4 * 1000 * 512 + 2 * (1000 + 768) * 256 * 9
    assert est <= soft <= est * 1.1 + 4096
    assert F.fff_workspace_bytes_soft(1000, 0, 8, 8) == 0 and F.fff_workspace_bytes_soft(1000, 768, 25, 8) == 0
    assert F.fff_workspace_bytes_soft(1 << 20, 768, 24, 8) == 0   # would not fit any device
    assert L.fff_set_workspace(ctypes.c_void_p(4096 + 64), 1 << 20, None) == WORKSPACE   # not 256-byte aligned
    assert L.fff_set_workspace(ctypes.c_void_p(4096), 100, None) == WORKSPACE           # shorter than the control words
    assert "workspace" in F.fff_status_string(WORKSPACE)


def test_debug_switches_are_not_public_options(L):
    import paper_2308_14711_amd as F
    UNSUP = 5
    for name in ("walk_tpg", "walk_block", "walk_top", "walk_bpc", "walk_prefetch", "block_top", "leaf_split",
                 "bucket_kernel", "token_max_T"):
        assert L.fff_set_option(name.encode(), 1) == UNSUP
        old = F.fff_debug_option(name)
        assert F.fff_debug_option(name, 3) == 3 and F.fff_debug_option(name) == 3
        F.fff_debug_option(name, old)
    assert L.fff_debug_option(b"path", 1, None) == UNSUP          # a public option is not a debug switch
    assert L.fff_debug_option(None, 1, None) == UNSUP


def _layer(T=6, D=8, O=4, depth=2, L=3, dtype=None):
    import torch
    dtype = dtype or torch.float32
    NN, NL = (1 << depth) - 1, 1 << depth
    z = lambda *s: torch.zeros(s, dtype=dtype)
    return dict(x=z(T, D), node_w=z(NN, D), node_b=z(NN), leaf_w1=z(NL, L, D), leaf_b1=z(NL, L), leaf_w2=z(NL, L, O),
                leaf_b2=z(NL, O), out=z(T, O), leaf_idx=torch.zeros(T, dtype=torch.int32))


def test_binding_checks_every_extent_before_the_library_sees_a_pointer():
    """The C ABI takes pointers and sizes and cannot see what is behind them; the binding checks each
    tensor against the sizes the Definition implies.  CPU tensors throughout: a call whose shapes are
    right gets as far as the 'must live on the GPU' check, every wrong one stops before it with
    FFF_ERR_SHAPE or FFF_ERR_DTYPE."""
    import torch
    import paper_2308_14711_amd as F
    SHAPE, DTYPE = 2, 3

    def hard(a, depth=2, L=3):
        F.fff_forward_hard(a["x"], a["node_w"], a["node_b"], a["leaf_w1"], a["leaf_b1"], a["leaf_w2"], a["leaf_b2"],
                           depth, L, 0, a["out"], a["leaf_idx"])

    with pytest.raises(ValueError, match="GPU"):
        hard(_layer())
    z = torch.zeros
    bad = {
        "node_w": z(2, 8), "node_b": z(4), "leaf_w1": z(4, 3, 7), "leaf_b1": z(4, 2), "leaf_w2": z(3, 3, 4),
        "leaf_b2": z(4, 5), "out": z(5, 4), "leaf_idx": z(5, dtype=torch.int32), "x": z(6, 8, 1),
    }
    for k, t in bad.items():
        a = _layer()
        a[k] = t
        with pytest.raises(F.FffError) as e:
            hard(a)
        assert e.value.status == SHAPE, k
    a = _layer()
    with pytest.raises(F.FffError) as e:       # a depth that does not match the tables
        hard(a, depth=3)
    assert e.value.status == SHAPE
    with pytest.raises(F.FffError) as e:       # a leaf width that does not match them
        hard(a, L=2)
    assert e.value.status == SHAPE
    for k in ("node_w", "leaf_w1", "leaf_b2", "out"):
        a = _layer()
        a[k] = a[k].to(torch.bfloat16)         # fp32 tokens with bf16 weights
        with pytest.raises(F.FffError) as e:
            hard(a)
        assert e.value.status == DTYPE, k
    a = _layer()
    a["leaf_idx"] = a["leaf_idx"].to(torch.int64)
    with pytest.raises(F.FffError) as e:
        hard(a)
    assert e.value.status == DTYPE

    # the stage entry points and the widened ones go through the same checks
    a = _layer()
    with pytest.raises(F.FffError) as e:
        F.fff_descend(a["x"], a["node_w"][:2], a["node_b"], 2, a["leaf_idx"])
    assert e.value.status == SHAPE
    with pytest.raises(F.FffError) as e:
        F.fff_bucket(a["leaf_idx"], 2, count=z(3, dtype=torch.int32))
    assert e.value.status == SHAPE
    with pytest.raises(F.FffError) as e:
        F.fff_bucket(a["leaf_idx"].to(torch.int64), 2)
    assert e.value.status == DTYPE
    with pytest.raises(F.FffError) as e:
        F.fff_leaf_forward(a["x"], a["leaf_w1"], a["leaf_b1"], a["leaf_w2"], a["leaf_b2"], a["leaf_idx"][:5], 2, 3, 0,
                           a["out"])
    assert e.value.status == SHAPE
    b = _layer(dtype=torch.bfloat16)
    with pytest.raises(F.FffError) as e:
        F.fff_moe_top1_forward(b["x"], z(3, 8, dtype=torch.bfloat16), None, b["leaf_w1"], b["leaf_b1"], b["leaf_w2"],
                               b["leaf_b2"], 2, 3, 0, b["out"])
    assert e.value.status == SHAPE
    with pytest.raises(F.FffError) as e:
        F.fff_forward_soft(b["x"], b["node_w"], b["node_b"], b["leaf_w1"], b["leaf_b1"], b["leaf_w2"], b["leaf_b2"], 2, 3,
                           0, b["out"], mix=z(6, 3))
    assert e.value.status == SHAPE
    with pytest.raises(F.FffError) as e:
        F.fff_forward_soft(b["x"], b["node_w"], b["node_b"], b["leaf_w1"], b["leaf_b1"], b["leaf_w2"], b["leaf_b2"], 2, 3,
                           0, b["out"], mix=z(6, 4, dtype=torch.bfloat16))
    assert e.value.status == DTYPE
    c = _layer(O=8)
    with pytest.raises(F.FffError) as e:       # node networks of 2 hidden neurons, a table built for 3
        F.fff_forward_block(c["x"], z(8), z(8), 1e-5, z(3, 3, 8), z(3, 2), z(3, 2), z(3), c["leaf_w1"], c["leaf_b1"],
                            c["leaf_w2"], c["leaf_b2"], 2, 2, 3, 0, True, c["out"])
    assert e.value.status == SHAPE
    with pytest.raises(F.FffError) as e:
        F.fff_forward_block(c["x"], z(7), z(8), 1e-5, z(3, 2, 8), z(3, 2), z(3, 2), z(3), c["leaf_w1"], c["leaf_b1"],
                            c["leaf_w2"], c["leaf_b2"], 2, 2, 3, 0, True, c["out"])
    assert e.value.status == SHAPE
    with pytest.raises(ValueError, match="GPU"):
        F.fff_forward_block(c["x"], z(8), z(8), 1e-5, z(3, 2, 8), z(3, 2), z(3, 2), z(3), c["leaf_w1"], c["leaf_b1"],
                            c["leaf_w2"], c["leaf_b2"], 2, 2, 3, 0, True, c["out"])


def test_packed_fp32_forms_are_really_switched_off():
    """The build passes a target feature that the host pass of hipcc does not know (and says so); what
    matters is the device pass: with the flag no packed fp32 VALU instruction may be left in the gfx950
    assembly of a kernel that otherwise gets them."""
    from paper_2308_14711_amd import build
    with_flag, without = build.packed_fp32_counts()
    assert with_flag == 0
    assert without > 0, "the probe kernel no longer invites packed instructions: the check shows nothing"


def test_header_is_plain_c99_and_links_from_c(tmp_path):
    """The boundary is a C ABI: a C99 translation unit includes include/fff.h with -pedantic, links
    against the library and calls it (host-side checks only: no GPU is touched)."""
    import subprocess
    import paper_2308_14711_amd as F
    src = tmp_path / "client.c"
    src.write_text(
        '#include "fff.h"\n#include <stdio.h>\n'
        'int main(void) {\n'
        '    printf("%d|%s|", fff_version(), fff_status_string(FFF_ERR_ALIAS));\n'
        '    printf("%d|", fff_forward_hard(0, 0, 0, 0, 0, 0, 0, 3, 2, 0, 0, 0, 0, 4, 16, 8, FFF_BF16));\n'
        '    printf("%d\\n", (int)(fff_workspace_bytes(1000, 4) > 0));\n'
        '    return 0;\n}\n')
    exe = tmp_path / "client"
    libdir = os.path.dirname(F.library_path())
    subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"),
                           str(src), "-o", str(exe), "-L", libdir, "-lfff_hip", "-Wl,-rpath," + libdir])
    out = subprocess.check_output([str(exe)], text=True).strip().split("|")
    assert int(out[0]) == F.fff_version() and out[1] == "out overlaps x" and out[2] == "1" and out[3] == "1"
