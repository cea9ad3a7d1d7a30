"""Builds libfff_hip.so (the C-ABI library) and the bench-only probe library for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import concurrent.futures
import os
import re
import subprocess
import sys
import tempfile

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libfff_hip.so")
PROBE_LIB = os.path.join(HERE, "libfff_bench_probes.so")   # measuring sticks of bench.py, not the product
OBJ_DIR = os.path.join(HERE, "_build")

SOURCES = ["fff_api.hip", "fff_walk.hip", "fff_bucket.hip", "fff_leaf.hip", "fff_leaf_tiles.hip", "fff_leaf_slices.hip",
           "fff_token_block.hip", "fff_moe_gate.hip", "fff_soft.hip", "fff_block.hip"]
PROBE_SOURCES = ["bench_probes.hip"]
HEADERS = ["fff_device.h", "fff_internal.h", "fff_mfma_tile.h", os.path.join("..", "..", "include", "fff.h")]

# packed fp32 VALU forms are switched off on purpose: some of them have given wrong results on
# the target machines; ordinary float code is compiled without them
PACKED_FP32_OFF = ["-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc"] + PACKED_FP32_OFF + \
              ["-Wall", "-Wno-unused-function"]

# The feature flag reaches both passes of hipcc.  The device pass (gfx950) knows the feature and
# obeys it; the host pass (x86-64) does not and says so, once per pass.  The message is dropped from
# the build output only after packed_fp32_is_off() has shown, on this compiler, that the device
# pass really stops emitting packed fp32 instructions.
HOST_PASS_NOTE = "'-packed-fp32-ops' is not a recognized feature for this target"

_PACKED_PROBE = """#include <hip/hip_runtime.h>
__global__ void k(float2* a, const float2* b) {
    const int i = threadIdx.x;
    float2 x = a[i];
    const float2 y = b[i];
    x.x = x.x * y.x + 1.f; x.y = x.y * y.y + 1.f;
    x.x += y.x; x.y += y.y;
    a[i] = x;
}
"""


def _hipcc() -> str:
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if c and (os.path.isabs(c) and os.path.exists(c) or not os.path.isabs(c)):
            return c
    return "hipcc"


def packed_fp32_counts() -> tuple:
    """(with the flag, without it): packed fp32 VALU instructions in the gfx950 assembly of a small
    kernel that invites them.  The flag works iff the first is 0 while the second is not."""
    counts = []
    with tempfile.TemporaryDirectory() as tmp:
        src = os.path.join(tmp, "probe.hip")
        with open(src, "w") as f:
            f.write(_PACKED_PROBE)
        for flags in (PACKED_FP32_OFF, []):
            out = os.path.join(tmp, "probe%d.s" % len(counts))
            r = subprocess.run([_hipcc(), "--offload-arch=gfx950", "-O3", "--cuda-device-only", "-S"] + flags +
                               [src, "-o", out], capture_output=True, text=True)
            if r.returncode != 0:
                raise RuntimeError("hipcc failed on the packed-fp32 probe:\n" + r.stderr)
            counts.append(len(re.findall(r"\bv_pk_(?:add|mul|fma)_f32\b", open(out).read())))
    return tuple(counts)


_flag_checked = False


def packed_fp32_is_off() -> None:
    global _flag_checked
    if _flag_checked:
        return
    with_flag, without = packed_fp32_counts()
    if with_flag != 0:
        raise RuntimeError("the device pass still emits packed fp32 instructions with %s" % " ".join(PACKED_FP32_OFF))
    if without == 0:
        sys.stderr.write("build: the probe kernel compiles without packed fp32 instructions even without the flag; "
                         "the flag's effect could not be observed on this compiler\n")
    _flag_checked = True


def _compile(src: str) -> str:
    obj = os.path.join(OBJ_DIR, src.replace(".hip", ".o"))
    cmd = [_hipcc()] + HIPCC_FLAGS + ["-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if HOST_PASS_NOTE not in l)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed on %s:\n%s" % (src, err))
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def stale() -> bool:
    if not os.path.exists(LIB) or not os.path.exists(PROBE_LIB):
        return True
    t = min(os.path.getmtime(LIB), os.path.getmtime(PROBE_LIB))
    deps = [os.path.join(CSRC, s) for s in SOURCES + PROBE_SOURCES] + \
           [os.path.normpath(os.path.join(CSRC, h)) for h in HEADERS]
    return any(os.path.getmtime(d) > t for d in deps)


def _link(objs, lib: str) -> None:
    tmp = lib + ".tmp%d" % os.getpid()
    r = subprocess.run([_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + objs,
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    os.replace(tmp, lib)


def _object_is_current(src: str) -> bool:
    obj = os.path.join(OBJ_DIR, src.replace(".hip", ".o"))
    if not os.path.exists(obj):
        return False
    t = os.path.getmtime(obj)
    deps = [os.path.join(CSRC, src)] + [os.path.normpath(os.path.join(CSRC, h)) for h in HEADERS]
    return all(os.path.getmtime(d) <= t for d in deps)


def build_library(force: bool = True, jobs: int = 4) -> str:
    """Compile every kernel source for gfx950 and link the shared libraries.  force=False compiles
    only the sources that changed since their object file was made (or nothing, if the libraries
    are newer than every source)."""
    if not force and not stale():
        return LIB
    packed_fp32_is_off()
    os.makedirs(OBJ_DIR, exist_ok=True)
    todo = [s for s in SOURCES + PROBE_SOURCES if force or not _object_is_current(s)]
    with concurrent.futures.ThreadPoolExecutor(max_workers=jobs) as ex:
        list(ex.map(_compile, todo))
    objs = [os.path.join(OBJ_DIR, s.replace(".hip", ".o")) for s in SOURCES + PROBE_SOURCES]
    _link(objs[:len(SOURCES)], LIB)
    _link(objs[len(SOURCES):], PROBE_LIB)
    return LIB


if __name__ == "__main__":
    print(build_library(force=True))
