"""The launch path chosen by shape and batch size against the forced ones, on shapes that none of the
rules in fff_api.hip was fitted on (row lengths other than 768 and 4096, inputs and outputs of different
width, fp32): the automatic choice must be within 30 % of the fastest path that takes the shape.  A
timing test, so with a wide margin: what it catches is a rule that sends a shape to a path that is half
as fast as another one, not a few percent."""
import numpy as np
import pytest

import fff_workloads as W

pytestmark = pytest.mark.gpu

SHAPES = [
    # T,      D,    O,    depth, L, dtype
    (20000,  1024, 1024, 9,  1,  W.DTYPE_BF16),
    (20000,  1024, 1024, 9,  6,  W.DTYPE_BF16),
    (100000, 512,  512,  10, 2,  W.DTYPE_BF16),
    (30000,  2048, 512,  12, 1,  W.DTYPE_BF16),
    (12000,  384,  1536, 8,  8,  W.DTYPE_BF16),
    (9000,   3072, 768,  9,  2,  W.DTYPE_BF16),
    (50000,  768,  3072, 5,  8,  W.DTYPE_BF16),
    (40000,  640,  640,  11, 2,  W.DTYPE_BF16),
    (1500,   768,  768,  8,  4,  W.DTYPE_BF16),
    (30000,  512,  512,  9,  2,  W.DTYPE_F32),
]


@pytest.mark.parametrize("shape", SHAPES, ids=["T%d_D%d_O%d_d%d_L%d_%s" % (s[0], s[1], s[2], s[3], s[4], "bf16" if s[5] else "f32")
                                               for s in SHAPES])
def test_automatic_choice_is_close_to_the_fastest_path(shape):
    import torch
    import paper_2308_14711_amd as F
    from fff_testlib import to_device
    T, D, O, depth, L, dtype = shape
    print("\n[case] auto choice T=%d D=%d O=%d depth=%d L=%d dtype=%d seed 71" % (T, D, O, depth, L, dtype), flush=True)
    w = W.make_layer("auto", T, D, O, depth, L, W.ACT_GELU, dtype, seed=71, keep_f32=False)
    dev = to_device(w)
    es = 2 if dtype == W.DTYPE_BF16 else 4
    n = max(2, min(6, int(6.0e8 / (T * (D + O) * es))))          # rotate buffers: no run finds its rows cached
    xs = [dev["x"]] + [dev["x"].clone() for _ in range(n - 1)]
    outs = [torch.empty((T, O), dtype=dev["x"].dtype, device="cuda") for _ in range(n)]
    idx = torch.empty((T,), dtype=torch.int32, device="cuda")
    times, took = {}, {}
    try:
        for path in (0, 1, 2, 4, 5):
            F.fff_set_option("path", path)

            def step(i):
                F.fff_forward_hard(xs[i % n], dev["node_w"], dev["node_b"], dev["leaf_w1"], dev["leaf_b1"], dev["leaf_w2"],
                                   dev["leaf_b2"], depth, L, w.act, outs[i % n], idx)

            for i in range(5):
                step(i)
            torch.cuda.synchronize()
            if path and F.fff_get_option("last_path") != path:
                continue                                   # the shape does not take this path
            best = float("inf")
            for rep in range(3):                           # best of three batches of 20 calls
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for i in range(20):
                    step(i)
                e1.record()
                torch.cuda.synchronize()
                best = min(best, e0.elapsed_time(e1) * 1000 / 20)
            times[path] = best
            took[path] = F.fff_get_option("last_path")
    finally:
        F.fff_set_option("path", 0)
    fastest = min(v for k, v in times.items() if k != 0)
    print("  auto -> path %d: %.1f us; forced: %s" % (took[0], times[0], {k: round(v, 1) for k, v in times.items() if k}), flush=True)
    assert times[0] <= 1.3 * fastest + 2.0, "auto took path %d at %.1f us, the fastest path needs %.1f us" % (took[0], times[0], fastest)
