"""fff_forward_hard_static -- the entry point for callers that cannot allocate -- through the C ABI,
against fff_forward_hard on the same inputs: same kernels, so the two must agree bit for bit (and
with the oracle, to the usual bar).  Two calls in a row share the static scratch array, the second
with a smaller input; then the bucketing kernels that rely on cleared control words, a single-launch
shape, and the size limit."""
import numpy as np
import pytest

import fff_workloads as W
from fff_testlib import check_against_oracle, to_device

pytestmark = pytest.mark.gpu
WORKSPACE = 6


def _both(F, w, want_idx=True):
    import torch
    dev = to_device(w)
    res = []
    for static in (False, True):
        out = torch.full((w.T, w.O), float("nan"), dtype=dev["x"].dtype, device="cuda")
        idx = torch.full((w.T,), -7, dtype=torch.int32, device="cuda") if want_idx else None
        nw = dev["node_w"] if w.depth > 0 else None
        nb = dev["node_b"] if w.depth > 0 else None
        F.fff_forward_hard(dev["x"], nw, nb, dev["leaf_w1"], dev["leaf_b1"], dev["leaf_w2"], dev["leaf_b2"],
                           w.depth, w.leaf_width, w.act, out, idx, static_scratch=static)
        torch.cuda.synchronize()
        res.append((out, idx, F.fff_get_option("last_path"), F.fff_last_launch()))
    (o0, i0, p0, k0), (o1, i1, p1, k1) = res
    assert p0 == p1 and k0 == k1, "the two entry points took different launches: %s / %s" % (k0, k1)
    bits = torch.int16 if o0.dtype == torch.bfloat16 else torch.int32
    assert torch.equal(o0.view(bits), o1.view(bits)), "outputs differ between the two entry points"
    if want_idx:
        assert torch.equal(i0, i1)
    return o1, i1, p1, k1


def test_static_scratch_entry_matches_the_allocating_one():
    import torch
    import paper_2308_14711_amd as F
    assert F.fff_static_scratch_bytes() == 16 << 20
    # 1. a batch the default rule sends down the staged path with the tile kernels (every scratch array in
    #    use: leaf ids, grouped order, slot leaves, hidden activations), then 2. a smaller one right after it
    for name, T, depth, seed in (("static_a", 12000, 6, 41), ("static_b", 9001, 5, 42)):
        print("\n[case] static scratch %s T=%d D=768 O=768 depth=%d L=8 bf16 seed %d" % (name, T, depth, seed), flush=True)
        w = W.make_layer(name, T, 768, 768, depth, 8, W.ACT_GELU, W.DTYPE_BF16, seed=seed)
        out, idx, path, kernels = _both(F, w)
        assert path == 2 and "leaf_hidden_kernel" in kernels, kernels
        check_against_oracle(w, out, idx)
    # 3. without a leaf_idx buffer from the caller (the scratch array holds it), fp32, gather kernel
    print("\n[case] static scratch fp32 T=9000 D=200 O=40 depth=7 L=12 seed 43, no leaf_idx", flush=True)
    w = W.make_layer("static_c", 9000, 200, 40, 7, 12, W.ACT_RELU, W.DTYPE_F32, seed=43)
    out, idx, path, kernels = _both(F, w, want_idx=False)
    assert path == 2
    check_against_oracle(w, out, None)
    # 4. the bucketing kernels that count on control words being zero when they start
    for bk in (2, 4, 1):
        print("\n[case] static scratch, bucket kernel %d: T=5000 D=256 O=128 depth=6 L=4 bf16 seed 44 path=2" % bk, flush=True)
        F.fff_set_option("path", 2)
        F.fff_debug_option("bucket_kernel", bk)
        try:
            w = W.make_layer("static_d", 5000, 256, 128, 6, 4, W.ACT_GELU, W.DTYPE_BF16, seed=44)
            out, idx, path, kernels = _both(F, w)
            check_against_oracle(w, out, idx)
        finally:
            F.fff_set_option("path", 0)
            F.fff_debug_option("bucket_kernel", 0)
    # 5. shapes that take one launch and no scratch at all go through the same entry point
    print("\n[case] static scratch, fused launch: T=3000 D=256 O=128 depth=6 L=4 bf16 seed 45", flush=True)
    w = W.make_layer("static_e", 3000, 256, 128, 6, 4, W.ACT_GELU, W.DTYPE_BF16, seed=45)
    out, idx, path, kernels = _both(F, w)
    assert path == 1
    check_against_oracle(w, out, idx)
    # 6. beyond the array: an error before anything is enqueued
    T, depth = 600000, 10
    assert F.fff_workspace_bytes(T, depth) > F.fff_static_scratch_bytes()
    x = torch.zeros((T, 16), dtype=torch.bfloat16, device="cuda")
    z = lambda *s: torch.zeros(s, dtype=torch.bfloat16, device="cuda")
    out = torch.full((T, 8), float("nan"), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(F.FffError) as e:
        F.fff_forward_hard_static(x, z(1023, 16), z(1023), z(1024, 2, 16), z(1024, 2), z(1024, 2, 8), z(1024, 8),
                                  depth, 2, 0, out)
    assert e.value.status == WORKSPACE and "static array holds" in str(e.value)
    torch.cuda.synchronize()
    assert bool(torch.isnan(out.float()).all())
    # the empty batch is fine
    assert F.lib().fff_forward_hard_static(None, None, None, None, None, None, None, 3, 2, 0, None, None, None, 0, 16, 8, 1) == 0
