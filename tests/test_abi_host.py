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


def test_probe_gather_rejects_bad_arguments_on_the_host(L):
    OK, NULL, SHAPE, RANGE, UNSUP = 0, 1, 2, 4, 5
    p = lambda mb: ctypes.c_void_p(mb << 20)
    probe = lambda **kw: L.fff_probe_gather(kw.get("table", p(1)), kw.get("rows", 1024), kw.get("row_bytes", 1536),
                                            kw.get("k", 4), kw.get("blocks", 8), kw.get("iters", 2), 1,
                                            kw.get("sink", p(64)), None)
    assert probe(table=None) == NULL
    assert probe(sink=None) == NULL
    assert probe(rows=1000) == RANGE                  # a power of two
    assert probe(row_bytes=100) == SHAPE
    assert probe(k=3) == UNSUP
    assert probe(blocks=0) == RANGE
    assert probe(iters=0) == RANGE


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
