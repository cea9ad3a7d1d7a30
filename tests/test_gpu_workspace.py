"""Caller-provided workspace (fff_set_workspace) through the C ABI: with one set, calls allocate
nothing and can be captured in a HIP graph with no preparation; a buffer that is too small is an
error before anything is enqueued; the sizing functions cover the mixture-of-experts and soft
entry points too."""
import numpy as np
import pytest

import fff_workloads as W
from fff_testlib import check_against_oracle, run_forward, to_device

pytestmark = pytest.mark.gpu
WORKSPACE = 6


def _forward(F, w, dev, out, idx):
    F.fff_forward_hard(dev["x"], dev["node_w"], dev["node_b"], dev["leaf_w1"], dev["leaf_b1"], dev["leaf_w2"],
                       dev["leaf_b2"], w.depth, w.leaf_width, w.act, out, idx)


def test_capture_on_a_caller_workspace_without_reserving():
    """The staged path (descent, bucketing, tile kernels: every workspace array in use) captured on a
    caller's buffer while the library owns no workspace at all; each replay, with eager work in
    between, reproduces the eager result bit for bit."""
    import torch
    import paper_2308_14711_amd as F
    print("\n[case] caller workspace, graph capture: T=12000 D=256 O=128 depth=6 L=4 bf16 seed 12 path=2", flush=True)
    w = W.make_layer("ws_graph", 12000, 256, 128, 6, 4, W.ACT_GELU, W.DTYPE_BF16, seed=12)
    dev = to_device(w)
    F.fff_set_option("path", 2)
    F.fff_set_option("leaf_path", 2)
    try:
        eager_out, eager_idx = run_forward(w, dev)           # on the library's own workspace
        check_against_oracle(w, eager_out, eager_idx)
        assert F.fff_get_option("last_path") == 2 and F.fff_get_option("last_leaf_path") == 2
        torch.cuda.synchronize()
        F.fff_release_workspace()                            # from here on the library owns nothing
        buf = torch.empty(F.fff_workspace_bytes(w.T, w.depth), dtype=torch.uint8, device="cuda")
        buf.fill_(0xA5)                                      # whatever the caller's memory holds
        F.fff_set_workspace(buf)
        out = torch.zeros_like(eager_out)
        idx = torch.zeros_like(eager_idx)
        g = torch.cuda.CUDAGraph()
        torch.cuda.synchronize()
        with torch.cuda.graph(g):
            _forward(F, w, dev, out, idx)
        for rep in range(4):
            out.fill_(float("nan"))
            idx.fill_(-1)
            scratch = torch.randn(1 << 16, device="cuda").sum().item()      # eager work between replays
            assert scratch == scratch
            g.replay()
            torch.cuda.synchronize()
            assert torch.equal(out.view(torch.int16), eager_out.view(torch.int16)), "replay %d differs" % rep
            assert torch.equal(idx, eager_idx)
        # a smaller call fits the same buffer; a larger one does not and says so before any launch
        w2 = W.make_layer("ws_small", 9000, 256, 128, 6, 4, W.ACT_GELU, W.DTYPE_BF16, seed=13)
        o2, i2 = run_forward(w2)
        check_against_oracle(w2, o2, i2)
        w3 = W.make_layer("ws_large", 20000, 256, 128, 6, 4, W.ACT_GELU, W.DTYPE_BF16, seed=14, keep_f32=False)
        dev3 = to_device(w3)
        out3 = torch.full((w3.T, w3.O), float("nan"), dtype=torch.bfloat16, device="cuda")
        with pytest.raises(F.FffError) as e:
            _forward(F, w3, dev3, out3, None)
        assert e.value.status == WORKSPACE and "needs" in str(e.value)
        torch.cuda.synchronize()
        assert bool(torch.isnan(out3.float()).all()), "a refused call must not have enqueued anything"
    finally:
        F.fff_set_workspace(None)
        F.fff_set_option("path", 0)
        F.fff_set_option("leaf_path", 0)
    # back on the library-owned workspace: it grows on demand again
    o3, i3 = run_forward(w3, dev3)
    check_against_oracle(w3, o3, i3)


def test_growth_is_refused_during_capture():
    """Library-owned workspace: a call that would have to grow it while its stream is being captured
    returns FFF_ERR_WORKSPACE instead of allocating; after reserving, the same capture succeeds."""
    import torch
    import paper_2308_14711_amd as F
    print("\n[case] growth during capture: T=10000 D=128 O=64 depth=5 L=4 bf16 seed 15 path=2", flush=True)
    w = W.make_layer("ws_capture", 10000, 128, 64, 5, 4, W.ACT_GELU, W.DTYPE_BF16, seed=15)
    dev = to_device(w)
    out = torch.full((w.T, w.O), float("nan"), dtype=torch.bfloat16, device="cuda")
    idx = torch.full((w.T,), -1, dtype=torch.int32, device="cuda")
    torch.cuda.synchronize()
    F.fff_release_workspace()
    F.fff_set_option("path", 2)
    try:
        status = []
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            try:
                _forward(F, w, dev, out, idx)
            except F.FffError as e:
                status.append(e.status)
        assert status == [WORKSPACE]
        F.fff_reserve_workspace(w.T, w.depth)
        g2 = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g2):
            _forward(F, w, dev, out, idx)
        g2.replay()
        torch.cuda.synchronize()
        check_against_oracle(w, out, idx)
    finally:
        F.fff_set_option("path", 0)


def test_moe_and_soft_on_a_caller_workspace():
    """fff_workspace_bytes_moe / _soft state what those entry points need: with exactly that much they
    run, with one aligned block less they return FFF_ERR_WORKSPACE."""
    import torch
    import oracle
    import paper_2308_14711_amd as F
    from fff_testlib import TOL, out_to_f64, oracle_inputs
    print("\n[case] moe + soft on a caller workspace: T=3000 D=128 O=64 depth=5 L=4 bf16 seed 16", flush=True)
    w = W.make_layer("ws_moe_soft", 3000, 128, 64, 5, 4, W.ACT_GELU, W.DTYPE_BF16, seed=16)
    gw, gb = W.moe_gate(32, 128, W.DTYPE_BF16, seed=16)
    dev = to_device(w)
    up = lambda a: torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    d_gw, d_gb = up(gw), up(gb)
    out = torch.full((w.T, w.O), float("nan"), dtype=torch.bfloat16, device="cuda")
    idx = torch.full((w.T,), -1, dtype=torch.int32, device="cuda")
    torch.cuda.synchronize()
    F.fff_release_workspace()
    F.fff_set_option("path", 2)        # the bucketed route of the experts, which uses the workspace
    try:
        need = F.fff_workspace_bytes_moe(w.T, 5)
        assert need > F.fff_workspace_bytes(w.T, 5)
        buf = torch.empty(need, dtype=torch.uint8, device="cuda")
        F.fff_set_workspace(buf[:need - 256])
        with pytest.raises(F.FffError) as e:
            F.fff_moe_top1_forward(dev["x"], d_gw, d_gb, dev["leaf_w1"], dev["leaf_b1"], dev["leaf_w2"], dev["leaf_b2"],
                                   5, 4, w.act, out, idx)
        assert e.value.status == WORKSPACE
        F.fff_set_workspace(buf)
        F.fff_moe_top1_forward(dev["x"], d_gw, d_gb, dev["leaf_w1"], dev["leaf_b1"], dev["leaf_w2"], dev["leaf_b2"],
                               5, 4, w.act, out, idx)
        torch.cuda.synchronize()
        ins = [w.bits[k] for k in ("leaf_w1", "leaf_b1", "leaf_w2", "leaf_b2")]
        ref_out, ref_idx, margin = oracle.moe_top1(w.bits["x"], gw, gb, *ins, 4, w.act)
        gi = idx.cpu().numpy()
        assert (margin[gi != ref_idx] < 1e-4).all()
        same = gi == ref_idx
        got = out_to_f64(out)
        err = np.abs(got[same] - ref_out[same]).max(axis=1) / np.maximum(np.abs(ref_out[same]).max(axis=1), 1e-30)
        assert err.max() <= TOL[W.DTYPE_BF16]

        need = F.fff_workspace_bytes_soft(w.T, w.O, w.depth, w.leaf_width)
        buf2 = torch.empty(need, dtype=torch.uint8, device="cuda")
        F.fff_set_workspace(buf2[:need - 256])
        out.fill_(float("nan"))
        with pytest.raises(F.FffError) as e:
            F.fff_forward_soft(dev["x"], dev["node_w"], dev["node_b"], dev["leaf_w1"], dev["leaf_b1"], dev["leaf_w2"],
                               dev["leaf_b2"], w.depth, w.leaf_width, w.act, out)
        assert e.value.status == WORKSPACE
        F.fff_set_workspace(buf2)
        F.fff_forward_soft(dev["x"], dev["node_w"], dev["node_b"], dev["leaf_w1"], dev["leaf_b1"], dev["leaf_w2"],
                           dev["leaf_b2"], w.depth, w.leaf_width, w.act, out)
        torch.cuda.synchronize()
        ref_soft, _ = oracle.forward_soft(*oracle_inputs(w), w.depth, w.leaf_width, w.act)
        got = out_to_f64(out)
        err = np.abs(got - ref_soft).max(axis=1) / np.maximum(np.abs(ref_soft).max(axis=1), 1e-30)
        assert err.max() <= TOL[W.DTYPE_BF16]
        with pytest.raises(F.FffError) as e:       # reserving is for the library's own workspace
            F.fff_reserve_workspace(w.T, w.depth)
        assert e.value.status == WORKSPACE
    finally:
        F.fff_set_workspace(None)
        F.fff_set_option("path", 0)


def test_a_failed_growth_is_an_error_and_the_next_call_recovers():
    """The library's own workspace cannot grow (forced through the test hook that makes the next growth
    fail the way an exhausted device does): the call returns FFF_ERR_WORKSPACE with nothing enqueued, the
    output is untouched, and the call after it allocates again and is right."""
    import torch
    import paper_2308_14711_amd as F
    print("\n[case] forced workspace growth failure: T=6000 D=128 O=64 depth=5 L=2 bf16 seed 31 path=2", flush=True)
    w = W.make_layer("ws_fail", 6000, 128, 64, 5, 2, W.ACT_RELU, W.DTYPE_BF16, seed=31)
    dev = to_device(w)
    torch.cuda.synchronize()
    F.fff_set_workspace(None)
    F.fff_release_workspace()                      # the next call has to allocate
    F.fff_set_option("path", 2)
    try:
        out = torch.full((w.T, w.O), float("nan"), dtype=torch.bfloat16, device="cuda")
        idx = torch.full((w.T,), -7, dtype=torch.int32, device="cuda")
        assert F.fff_debug_option("fail_workspace_growth", 1) == 1
        with pytest.raises(F.FffError) as e:
            _forward(F, w, dev, out, idx)
        assert e.value.status == WORKSPACE and "hipMalloc" in str(e.value)
        assert F.fff_debug_option("fail_workspace_growth") == 0      # the hook was used up
        torch.cuda.synchronize()
        assert bool(torch.isnan(out.float()).all()) and bool((idx == -7).all())
        _forward(F, w, dev, out, idx)
        torch.cuda.synchronize()
        check_against_oracle(w, out, idx)
    finally:
        F.fff_debug_option("fail_workspace_growth", 0)
        F.fff_set_option("path", 0)
