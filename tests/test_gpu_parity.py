"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle
on the same seeded inputs, element by element."""
import numpy as np
import pytest

import fff_workloads as W
import oracle
from fff_testlib import ROUTING_MARGIN, TOL, check_against_oracle, oracle_inputs, out_to_f64, run_forward, to_device

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def c5_workload():
    """Built once: drawing 1.3e9 weights takes a while."""
    import torch
    w = W.config("C5", keep_f32=False)
    dev = to_device(w)
    ref = oracle.forward_hard(*oracle_inputs(w), w.depth, w.leaf_width, w.act)
    # margin tokens are validated against the fp32 view of the node tensors only
    w.f32["x"] = W.bf16_widen(w.bits["x"])
    w.f32["node_w"] = W.bf16_widen(w.bits["node_w"])
    w.f32["node_b"] = W.bf16_widen(w.bits["node_b"])
    yield w, dev, ref
    del dev
    torch.cuda.empty_cache()


def _log(name, stats):
    print("\n[parity] %s: %s" % (name, stats), flush=True)


@pytest.mark.parametrize("name", ["C1", "C2", "C2c", "C3", "C4"])
def test_named_workloads(name):
    print("\n[case] workload %s seed 0" % name, flush=True)
    w = W.config(name)
    out, idx = run_forward(w)
    _log(name, check_against_oracle(w, out, idx))


def test_batch_beyond_the_token_chunk_bucketing():
    """A staged call whose batch is too large for the one-launch bucketing kernels' fast case:
    the chunk-matrix kernels run inside fff_forward_hard."""
    import paper_2308_14711_amd as F
    print("\n[case] large batch T=150001 D=256 O=128 depth=6 L=8 bf16 seed 4, staged", flush=True)
    w = W.make_layer("large_batch", 150001, 256, 128, 6, 8, W.ACT_GELU, W.DTYPE_BF16, seed=4)
    F.fff_set_option("path", 2)
    try:
        out, idx = run_forward(w)
    finally:
        F.fff_set_option("path", 0)
    assert F.fff_get_option("last_path") == 2
    _log("large_batch", check_against_oracle(w, out, idx))


@pytest.mark.parametrize("path", [0, 1, 2, 5], ids=["auto", "fused", "staged", "split"])
def test_large_skewed_workload(path, c5_workload):
    """C5 at full size (2.4 GB of leaf weights, Zipf leaf occupancy), both launch configurations."""
    import paper_2308_14711_amd as F
    print("\n[case] workload C5 seed 0 path=%d" % path, flush=True)
    w, dev, ref = c5_workload
    F.fff_set_option("path", path)
    try:
        out, idx = run_forward(w, dev)
    finally:
        F.fff_set_option("path", 0)
    _log("C5 path=%d" % path, check_against_oracle(w, out, idx, ref=ref))


SMALL = [
    # name,               T,   D,   O, depth, L, act,        dtype
    ("d0_f32",            70,  64,  12, 0, 3, W.ACT_RELU, W.DTYPE_F32),
    ("d1_bf16",           65,  64,  16, 1, 2, W.ACT_GELU, W.DTYPE_BF16),
    ("one_token",         1,   128, 8,  4, 4, W.ACT_GELU, W.DTYPE_F32),
    ("ragged_63",         63,  256, 24, 5, 8, W.ACT_GELU, W.DTYPE_BF16),
    ("ragged_257",        257, 96,  40, 3, 5, W.ACT_RELU, W.DTYPE_BF16),
    ("odd_dims_generic",  130, 50,  7,  4, 3, W.ACT_GELU, W.DTYPE_F32),
    ("odd_dims_bf16",     99,  77,  9,  3, 2, W.ACT_RELU, W.DTYPE_BF16),
    ("wide_leaf_64",      40,  64,  32, 2, 64, W.ACT_GELU, W.DTYPE_F32),
    ("wide_leaf_65",      40,  64,  32, 2, 65, W.ACT_GELU, W.DTYPE_F32),
    ("deep_sparse",       300, 128, 64, 12, 2, W.ACT_GELU, W.DTYPE_BF16),
    ("big_rows_f32",      50,  2048, 16, 3, 2, W.ACT_RELU, W.DTYPE_F32),
    ("big_rows_bf16",     50,  8192, 64, 2, 1, W.ACT_GELU, W.DTYPE_BF16),
    ("huge_rows_generic", 9,   8200, 8,  2, 1, W.ACT_RELU, W.DTYPE_BF16),
    ("vit_like_small",    777, 768, 768, 4, 8, W.ACT_GELU, W.DTYPE_BF16),
    ("bert_like_small",   1000, 768, 768, 6, 1, W.ACT_GELU, W.DTYPE_BF16),
    ("skew_like_small",   515, 4096, 4096, 7, 4, W.ACT_GELU, W.DTYPE_BF16),


    ("tiles_L1",          700, 96,  132, 5, 1, W.ACT_GELU, W.DTYPE_BF16),
    ("tiles_L2",          333, 40,  12,  6, 2, W.ACT_RELU, W.DTYPE_BF16),
    ("tiles_L3",          401, 72,  68,  4, 3, W.ACT_GELU, W.DTYPE_BF16),
    ("tiles_L5",          250, 64,  64,  3, 5, W.ACT_GELU, W.DTYPE_BF16),
    ("tiles_L16",         300, 128, 200, 2, 16, W.ACT_RELU, W.DTYPE_BF16),
    ("tiles_sparse",      200, 64,  64,  10, 4, W.ACT_GELU, W.DTYPE_BF16),
    ("tiles_L17",         150, 64,  64,  3, 17, W.ACT_GELU, W.DTYPE_BF16),
    ("tiles_L24",         500, 128, 264, 2, 24, W.ACT_RELU, W.DTYPE_BF16),
    ("tiles_L30_sparse",  260, 72,  40,  6, 30, W.ACT_GELU, W.DTYPE_BF16),
    ("tiles_L32",         900, 768, 768, 2, 32, W.ACT_GELU, W.DTYPE_BF16),
    ("gather_L33",        150, 64,  64,  3, 33, W.ACT_GELU, W.DTYPE_BF16),
    # small batches: the one-block-per-token launch (depths around multiples of its 3-level rounds,
    # rows of 1, 2, 4 and 8 vectors per lane, outputs wider than inputs, a batch above its grid cap)
    ("latency_L32_d7",    256, 768, 768, 7, 32, W.ACT_GELU, W.DTYPE_BF16),
    ("latency_L32_d9",    256, 768, 768, 9, 32, W.ACT_GELU, W.DTYPE_BF16),
    ("latency_f32_d5",    100, 768, 256, 5, 6,  W.ACT_RELU, W.DTYPE_F32),
    ("latency_wide_out",  64,  64,  1024, 4, 9, W.ACT_GELU, W.DTYPE_BF16),
    ("latency_4096_d5",   33,  4096, 512, 5, 3, W.ACT_GELU, W.DTYPE_BF16),
    ("latency_L70",       20,  128, 10, 2, 70, W.ACT_GELU, W.DTYPE_F32),
    ("latency_many",      9001, 32, 16, 8, 2, W.ACT_RELU, W.DTYPE_BF16),
]


# (path, leaf_path): the staged path picks its leaf kernels by bucket size, so the tile kernels get
# a run of their own on every shape they take
@pytest.mark.parametrize("path", [(0, 0), (1, 0), (2, 0), (2, 2), (4, 0), (5, 0)],
                         ids=["auto", "fused", "staged", "staged_tiles", "token", "split"])
@pytest.mark.parametrize("case", SMALL, ids=[c[0] for c in SMALL])
def test_small_and_edge_shapes(case, path):
    import paper_2308_14711_amd as F
    name, T, D, O, depth, L, act, dtype = case
    path, leaf_path = path
    print("\n[case] %s T=%d D=%d O=%d depth=%d L=%d dtype=%d seed 5 path=%d" % (name, T, D, O, depth, L, dtype, path),
          flush=True)
    w = W.make_layer(name, T, D, O, depth, L, act, dtype, seed=5,
                     node_b="zipf" if name.startswith("skew") else "uniform")
    F.fff_set_option("path", path)
    F.fff_set_option("leaf_path", leaf_path)
    try:
        out, idx = run_forward(w)
        took = F.fff_get_option("last_path")
    finally:
        F.fff_set_option("path", 0)
        F.fff_set_option("leaf_path", 0)
    per = 8 if dtype == W.DTYPE_BF16 else 4
    if D % per == 0 and D // per <= 512 and (path == 4 or (path == 0 and T <= 512)):
        assert took == 4, "the one-block-per-token launch takes this shape, but path %d ran" % took
    _log("%s path=%d took=%d" % (name, path, took), check_against_oracle(w, out, idx))


def test_empty_batch_is_a_noop():
    import torch
    import paper_2308_14711_amd as F
    w = W.make_layer("e", 4, 64, 8, 2, 2, W.ACT_RELU, W.DTYPE_F32, seed=1)
    dev = to_device(w)
    x0 = dev["x"][:0].contiguous()
    out = torch.empty((0, 8), device="cuda")
    F.fff_forward_hard(x0, dev["node_w"], dev["node_b"], dev["leaf_w1"], dev["leaf_b1"], dev["leaf_w2"],
                       dev["leaf_b2"], 2, 2, W.ACT_RELU, out, None)
    torch.cuda.synchronize()


def test_all_tokens_in_one_leaf():
    """Zero node weights: every logit is +0, ties go right, every token lands in the last leaf."""
    print("\n[case] one_leaf", flush=True)
    w = W.make_layer("one_leaf", 500, 128, 32, 5, 4, W.ACT_GELU, W.DTYPE_BF16, seed=2)
    for k in ("node_w", "node_b"):
        w.f32[k][...] = 0
        w.bits[k][...] = 0
    out, idx = run_forward(w)
    assert (idx.cpu().numpy() == 31).all()
    stats = check_against_oracle(w, out, idx)
    assert stats["idx_mismatch"] == 0


def test_every_leaf_gets_exactly_one_token():
    """Axis-aligned nodes (level m splits on axis m at 0) and tokens whose signs spell their index."""
    print("\n[case] one_token_per_leaf", flush=True)
    depth, D = 6, 64
    T = 1 << depth
    w = W.make_layer("perleaf", T, D, 16, depth, 2, W.ACT_RELU, W.DTYPE_F32, seed=3, node_b="zero")
    w.f32["node_w"][...] = 0
    for m in range(depth):
        w.f32["node_w"][(1 << m) - 1:(1 << (m + 1)) - 1, m] = 1.0
    bits = (np.arange(T)[:, None] >> (depth - 1 - np.arange(depth))[None, :]) & 1
    w.f32["x"][:, :depth] = np.where(bits == 1, 0.5, -0.5) * (1 + np.arange(depth))
    rng = np.random.default_rng(0)
    p = rng.permutation(T)
    w.f32["x"] = np.ascontiguousarray(w.f32["x"][p])
    out, idx = run_forward(w)
    assert np.array_equal(idx.cpu().numpy(), p.astype(np.int32))
    _log("perleaf", check_against_oracle(w, out, idx))


def test_leaf_idx_is_optional():
    w = W.make_layer("noidx", 300, 128, 48, 4, 4, W.ACT_GELU, W.DTYPE_BF16, seed=4)
    out, _ = run_forward(w, want_idx=False)
    _log("noidx", check_against_oracle(w, out, None))


def test_reruns_are_bit_identical_and_tokens_permute():
    import torch
    w = W.make_layer("det", 3000, 256, 128, 6, 4, W.ACT_GELU, W.DTYPE_BF16, seed=6)
    dev = to_device(w)
    o1, i1 = run_forward(w, dev)
    o2, i2 = run_forward(w, dev)
    assert torch.equal(o1.view(torch.int16), o2.view(torch.int16)) and torch.equal(i1, i2)
    p = torch.randperm(w.T, device="cuda", generator=torch.Generator(device="cuda").manual_seed(0))
    dev2 = dict(dev)
    dev2["x"] = dev["x"][p].contiguous()
    o3, i3 = run_forward(w, dev2)
    assert torch.equal(o3.view(torch.int16), o1[p].view(torch.int16)) and torch.equal(i3, i1[p])


def test_runs_on_a_side_stream():
    import torch
    w = W.make_layer("stream", 600, 128, 64, 5, 2, W.ACT_RELU, W.DTYPE_F32, seed=7)
    dev = to_device(w)
    s = torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        out, idx = run_forward(w, dev, stream=s)
    _log("stream", check_against_oracle(w, out, idx))


# ---- stages on their own ------------------------------------------------------

@pytest.mark.parametrize("depth,T,kind", [(0, 10, "u"), (3, 1, "u"), (3, 1000, "u"), (8, 5000, "zipf"),
                                          (11, 65536, "u"), (15, 16384, "zipf"), (20, 10000, "u"),
                                          (6, 4096, "one"), (19, 70001, "zipf"), (10, 300000, "u"),
                                          (8, 50432, "u"), (12, 131072, "zipf"), (12, 131071, "u"), (2, 63, "u"),
                                          (9, 16385, "zipf"), (3, 65535, "one"), (3, 65536, "one"),
                                          (8, 806912, "u"), (12, 131073, "zipf"), (10, 131072, "zipf"),
                                          (10, 100003, "u"), (7, 12001, "u"), (9, 262144, "one")])
@pytest.mark.parametrize("kernel", [0, 1, 2, 3, 4, 5])
def test_bucket_stage_is_bit_exact(depth, T, kind, kernel):
    import torch
    import paper_2308_14711_amd as F
    print("\n[case] bucket depth=%d T=%d %s kernel=%d" % (depth, T, kind, kernel), flush=True)
    F.fff_debug_option("bucket_kernel", kernel)
    rng = np.random.default_rng(depth * 1000 + T)
    NL = 1 << depth
    if kind == "u":
        li = rng.integers(0, NL, T).astype(np.int32)
    elif kind == "zipf":
        li = (rng.zipf(1.1, T) % NL).astype(np.int32)
    else:
        li = np.full(T, NL - 1, np.int32)
    count, offset, perm = oracle.bucket(li, depth)
    d_li = torch.from_numpy(li).cuda()
    if T % 2 == 1:           # odd sizes also come in through a pointer that is only 4-byte aligned
        d_li = torch.cat([torch.zeros(1, dtype=torch.int32, device="cuda"), d_li])[1:]
        assert d_li.data_ptr() % 16 != 0
    d_count = torch.full((NL,), -1, dtype=torch.int32, device="cuda")
    d_offset = torch.full((NL + 1,), -1, dtype=torch.int32, device="cuda")
    d_perm = torch.full((T,), -1, dtype=torch.int32, device="cuda")
    try:
        for _ in range(2):      # twice: the workspace must come back clean
            F.fff_bucket(d_li, depth, d_count, d_offset, d_perm)
            torch.cuda.synchronize()
            assert np.array_equal(d_count.cpu().numpy(), count)
            assert np.array_equal(d_offset.cpu().numpy(), offset)
            assert np.array_equal(d_perm.cpu().numpy(), perm)
            if kernel == 5 and depth <= 10 and T <= min(256, (128 * 1024) >> depth) * 1024:
                assert "bucket_fold_kernel" in F.fff_last_launch(), F.fff_last_launch()
    finally:
        F.fff_debug_option("bucket_kernel", 0)


def test_split_launch_equals_the_fused_one_bit_for_bit():
    """The fused launch cut in two (walk + hidden neurons, then output rows by column slices) does the
    same additions in the same order as the single launch: same bits, on rows of 12 lines (4 slices),
    of 8 lines (8 slices), of a line and a half (one short slice), fp32, no leaf_idx buffer."""
    import torch
    import paper_2308_14711_amd as F
    cases = [(20000, 768, 768, 9, 1, W.DTYPE_BF16), (9000, 512, 512, 7, 2, W.DTYPE_BF16), (5000, 256, 96, 6, 8, W.DTYPE_BF16),
             (7000, 768, 1032, 5, 3, W.DTYPE_BF16), (6000, 256, 200, 6, 2, W.DTYPE_F32), (3000, 64, 8, 4, 1, W.DTYPE_BF16)]
    for T, D, O, depth, L, dtype in cases:
        print("\n[case] split vs fused T=%d D=%d O=%d depth=%d L=%d dtype=%d seed 61" % (T, D, O, depth, L, dtype), flush=True)
        w = W.make_layer("split", T, D, O, depth, L, W.ACT_GELU, dtype, seed=61)
        dev = to_device(w)
        res = {}
        for path in (1, 5):
            F.fff_set_option("path", path)
            try:
                res[path] = run_forward(w, dev, want_idx=path == 1)
                assert F.fff_get_option("last_path") == path
            finally:
                F.fff_set_option("path", 0)
        bits = torch.int16 if dtype == W.DTYPE_BF16 else torch.int32
        assert torch.equal(res[1][0].view(bits), res[5][0].view(bits))
        _log("split T=%d" % T, check_against_oracle(w, res[1][0], res[1][1]))
    # the BERT-base-sized shape takes the split launch by itself
    w = W.config("C4", keep_f32=False)
    out, idx = run_forward(w)
    assert F.fff_get_option("last_path") == 5 and "leaf_slices_kernel" in F.fff_last_launch(), F.fff_last_launch()


def test_descent_hands_leaf_counts_to_the_bucketing_stage():
    """On the staged path the descent counts, per block, the tokens of every leaf, and one fold launch
    turns the counts into the grouped order: same rows, bit for bit, as with a bucketing kernel that
    histograms leaf_idx itself; routing and rows against the oracle."""
    import torch
    import paper_2308_14711_amd as F
    for T, depth, L, seed in ((12000, 6, 8, 51), (50432, 8, 8, 52), (9000, 9, 4, 53), (20000, 3, 16, 54)):
        print("\n[case] descent counts T=%d D=768 O=768 depth=%d L=%d bf16 seed %d path=2" % (T, depth, L, seed), flush=True)
        w = W.make_layer("fold", T, 768, 768, depth, L, W.ACT_GELU, W.DTYPE_BF16, seed=seed, keep_f32=T < 30000)
        dev = to_device(w)
        F.fff_set_option("path", 2)
        try:
            out, idx = run_forward(w, dev)
            launch = F.fff_last_launch()
            assert "descent+counts" in launch and "bucket_fold_kernel" in launch, launch
            F.fff_debug_option("bucket_kernel", 3)
            out3, idx3 = run_forward(w, dev)
            assert "bucket_hist_kernel" in F.fff_last_launch()
        finally:
            F.fff_set_option("path", 0)
            F.fff_debug_option("bucket_kernel", 0)
        assert torch.equal(out.view(torch.int16), out3.view(torch.int16)) and torch.equal(idx, idx3)
        if T < 30000:
            _log("descent counts T=%d" % T, check_against_oracle(w, out, idx))


def test_descend_and_leaf_stages():
    import torch
    import paper_2308_14711_amd as F
    w = W.make_layer("stages", 900, 256, 64, 7, 4, W.ACT_GELU, W.DTYPE_BF16, seed=8)
    dev = to_device(w)
    ins = oracle_inputs(w)
    _, ref_idx, margin = oracle.forward_hard(*ins, w.depth, w.leaf_width, w.act, want_out=False)
    idx = torch.empty((w.T,), dtype=torch.int32, device="cuda")
    F.fff_descend(dev["x"], dev["node_w"], dev["node_b"], w.depth, idx)
    torch.cuda.synchronize()
    gi = idx.cpu().numpy()
    assert np.array_equal(gi[margin >= 1e-4], ref_idx[margin >= 1e-4])
    # the leaf stage at leaves that have nothing to do with the tree
    forced = ((np.arange(w.T) * 37) % w.n_leaves).astype(np.int32)
    out = torch.empty((w.T, w.O), dtype=torch.bfloat16, device="cuda")
    F.fff_leaf_forward(dev["x"], dev["leaf_w1"], dev["leaf_b1"], dev["leaf_w2"], dev["leaf_b2"],
                       torch.from_numpy(forced).cuda(), w.depth, w.leaf_width, w.act, out)
    torch.cuda.synchronize()
    ref = oracle.leaf_forward(ins[0], ins[3], ins[4], ins[5], ins[6], forced, w.depth, w.leaf_width, w.act)
    got = out_to_f64(out)
    err = np.abs(got - ref).max(axis=1) / np.abs(ref).max(axis=1)
    assert err.max() <= 2e-2


@pytest.mark.parametrize("opt", [("bucketing", 0), ("path", 1), ("path", 2), ("path", 3), ("path", 4), ("path", 5),
                                 ("leaf_path", 1)])
def test_alternative_paths_agree_with_the_oracle(opt):
    import paper_2308_14711_amd as F
    w = W.make_layer("paths", 2000, 256, 128, 6, 4, W.ACT_GELU, W.DTYPE_BF16, seed=9)
    old = F.fff_get_option(opt[0])
    F.fff_set_option(*opt)
    try:
        out, idx = run_forward(w)
    finally:
        F.fff_set_option(opt[0], old)
    _log("paths %s" % (opt,), check_against_oracle(w, out, idx))


TILE_SIZES = [
    # the walk kernels cut a batch into tiles of 32, 64, 128 or 256 tokens by batch size and row width:
    # batches on both sides of the switches, for every row-width class
    # name,            T,     D,    O,   depth, L, dtype
    ("w64_small",      3000,  64,   64,  5,     2, W.DTYPE_BF16),
    ("w64_large",      20011, 64,   32,  6,     3, W.DTYPE_BF16),
    ("w128_large",     17000, 128,  128, 7,     1, W.DTYPE_BF16),
    ("w256_mid",       12000, 256,  64,  8,     4, W.DTYPE_BF16),
    ("w256_large",     16500, 256,  256, 5,     2, W.DTYPE_BF16),
    ("w512_large",     16500, 512,  128, 6,     2, W.DTYPE_BF16),
    ("w768_mid",       12001, 768,  768, 9,     1, W.DTYPE_BF16),
    ("w768_ragged",    9000,  760,  768, 7,     3, W.DTYPE_BF16),
    ("w768_tiles_96",  20000, 768,  768, 8,     2, W.DTYPE_BF16),
    ("w768_rounds",    40000, 768,  256, 7,     1, W.DTYPE_BF16),
    ("w1024_small",    5000,  1024, 256, 6,     2, W.DTYPE_BF16),
    ("w1024_large",    9000,  1024, 1024, 6,    2, W.DTYPE_BF16),
    ("f32_w64_large",  17000, 64,   16,  6,     2, W.DTYPE_F32),
    ("f32_w256_small", 4000,  256,  64,  7,     3, W.DTYPE_F32),
]


@pytest.mark.parametrize("path", [1, 2, 5], ids=["fused", "staged", "split"])
@pytest.mark.parametrize("case", TILE_SIZES, ids=[c[0] for c in TILE_SIZES])
def test_tile_sizes_of_the_walk_kernels(case, path):
    import paper_2308_14711_amd as F
    name, T, D, O, depth, L, dtype = case
    print("\n[case] tiles %s T=%d D=%d O=%d depth=%d L=%d dtype=%d seed 21 path=%d" % (name, T, D, O, depth, L, dtype, path),
          flush=True)
    w = W.make_layer(name, T, D, O, depth, L, W.ACT_GELU, dtype, seed=21)
    F.fff_set_option("path", path)
    try:
        out, idx = run_forward(w)
        assert F.fff_get_option("last_path") == path
    finally:
        F.fff_set_option("path", 0)
    _log("tiles %s path=%d" % (name, path), check_against_oracle(w, out, idx))


WALK_SWITCHES = [
    # the experiment switches of the walk kernels select other instantiations: (options, D)
    ({"walk_tpg": 1, "walk_block": 512}, 768), ({"walk_tpg": 1, "walk_block": 1024}, 768),
    ({"walk_tpg": 2, "walk_block": 512}, 768), ({"walk_tpg": 2, "walk_block": 1024}, 768),
    ({"walk_tpg": 3, "walk_block": 512}, 768), ({"walk_tpg": 4, "walk_block": 512}, 768),
    ({"walk_tpg": 4, "walk_block": 256}, 768), ({"walk_prefetch": 1}, 768),
    ({"walk_top": 1}, 768), ({"walk_top": 3}, 768), ({"walk_bpc": 2}, 768), ({"walk_bpc": 3, "walk_top": 4}, 768),
    ({"walk_tpg": 1, "walk_block": 1024}, 4096), ({"walk_tpg": 3, "walk_block": 512}, 4096),
    ({"walk_tpg": 4, "walk_block": 256}, 4096), ({"walk_tpg": 6, "walk_block": 256}, 4096),
]


@pytest.mark.parametrize("path", [1, 2, 5], ids=["fused", "staged", "split"])
@pytest.mark.parametrize("switches", WALK_SWITCHES, ids=["_".join("%s%d" % (k[5:], v) for k, v in o.items()) + "_w%d" % d
                                                         for o, d in WALK_SWITCHES])
def test_walk_kernel_switches(switches, path):
    """Every instantiation the switches reach, on a batch of several rounds with a ragged end."""
    import paper_2308_14711_amd as F
    opts, D = switches
    T = 40007 if D == 768 else 5003
    print("\n[case] walk switches %s T=%d D=%d depth=9 L=1 bf16 seed 31 path=%d" % (opts, T, D, path), flush=True)
    w = W.make_layer("switches", T, D, D, 9, 1, W.ACT_GELU, W.DTYPE_BF16, seed=31, keep_f32=False)
    F.fff_set_option("path", path)
    for k, v in opts.items():
        F.fff_debug_option(k, v)
    try:
        out, idx = run_forward(w)
        if "walk_top" in opts:
            assert F.fff_get_option("last_walk_top") <= opts["walk_top"] - 1
    finally:
        F.fff_set_option("path", 0)
        for k in opts:
            F.fff_debug_option(k, 0)
    _log("switches %s path=%d" % (opts, path), check_against_oracle(w, out, idx))


def test_token_block_threshold_option():
    """token_max_T moves the batch size up to which the one-block-per-token launch is taken."""
    import paper_2308_14711_amd as F
    print("\n[case] token_max_T T=700 D=256 depth=6 L=2 bf16 seed 8", flush=True)
    w = W.make_layer("threshold", 700, 256, 64, 6, 2, W.ACT_RELU, W.DTYPE_BF16, seed=8)
    old = F.fff_debug_option("token_max_T")
    try:
        for limit, expect in ((0, 1), (699, 1), (700, 4), (old, 1 if old < 700 else 4)):
            F.fff_debug_option("token_max_T", limit)
            out, idx = run_forward(w)
            assert F.fff_get_option("last_path") == expect, "token_max_T=%d took path %d" % (limit, F.fff_get_option("last_path"))
            _log("threshold %d" % limit, check_against_oracle(w, out, idx))
    finally:
        F.fff_debug_option("token_max_T", old)


SPLIT_CASES = [
    # name,          T,    D,    O,    depth, L,  node_b
    ("skewed",       6000, 256,  128,  10,    4,  "zipf"),      # popular leaves and a long tail of single tokens
    ("skewed_wide",  3000, 2048, 2048, 9,     8,  "zipf"),      # a wave per token in the gather kernel
    ("thin",         900,  128,  64,   8,     3,  "uniform"),   # 3.5 tokens a leaf, leaf width not a divisor of 16
    ("skewed_l20",   2500, 512,  256,  9,     20, "zipf"),      # leaves of 17..32 neurons
]


@pytest.mark.parametrize("case", SPLIT_CASES, ids=[c[0] for c in SPLIT_CASES])
def test_leaf_stage_split_between_tile_and_gather_kernels(case):
    """On request the staged leaf stage sends tiles (16 consecutive slots of the bucketed order) with
    many different leaves to the gather kernel and keeps the others on the tile kernels.  Every
    threshold, from "all tiles to the gather kernel" to "none", must give the oracle's rows, and
    every token's row is written by exactly one of the kernels (the output starts as NaN)."""
    import paper_2308_14711_amd as F
    name, T, D, O, depth, L, node_b = case
    print("\n[case] split %s T=%d D=%d O=%d depth=%d L=%d bf16 seed 12 node_b=%s" % case, flush=True)
    w = W.make_layer(name, T, D, O, depth, L, W.ACT_GELU, W.DTYPE_BF16, seed=12, node_b=node_b)
    F.fff_set_option("path", 2)
    try:
        out, idx = run_forward(w)
        # a small batch with few tokens a leaf: the gather kernel alone
        assert F.fff_get_option("last_leaf_path") == 1
        _log("split %s auto" % name, check_against_oracle(w, out, idx))
        F.fff_set_option("leaf_path", 2)
        for split in (1, 2, 5, 8, 13, 16, 17, 0):
            F.fff_debug_option("leaf_split", split)
            out, idx = run_forward(w)
            assert F.fff_get_option("last_leaf_path") == (3 if 1 <= split <= 16 else 2)
            _log("split %s %d" % (name, split), check_against_oracle(w, out, idx))
    finally:
        F.fff_set_option("path", 0)
        F.fff_set_option("leaf_path", 0)
        F.fff_debug_option("leaf_split", 0)


@pytest.mark.parametrize("path", [1, 2, 4, 5], ids=["fused", "staged", "token", "split"])
def test_capture_in_a_hip_graph_and_replay(path):
    """The call only enqueues kernels on the given stream (no allocation once the workspace is
    reserved, no memset nodes): it can be captured, and every replay, with eager work and
    synchronisations in between, must reproduce the eager result bit for bit."""
    import torch
    import paper_2308_14711_amd as F
    w = W.make_layer("graph", 3000, 256, 128, 6, 4, W.ACT_GELU, W.DTYPE_BF16, seed=11)
    dev = to_device(w)
    F.fff_set_option("path", path)
    try:
        eager_out, eager_idx = run_forward(w, dev)
        _log("graph eager path=%d" % path, check_against_oracle(w, eager_out, eager_idx))
        F.fff_reserve_workspace(w.T, w.depth)
        out = torch.zeros_like(eager_out)
        idx = torch.zeros_like(eager_idx)
        g = torch.cuda.CUDAGraph()
        torch.cuda.synchronize()
        with torch.cuda.graph(g):
            F.fff_forward_hard(dev["x"], dev["node_w"], dev["node_b"], dev["leaf_w1"], dev["leaf_b1"],
                               dev["leaf_w2"], dev["leaf_b2"], w.depth, w.leaf_width, w.act, out, idx)
        for rep in range(4):
            out.fill_(float("nan"))
            idx.fill_(-1)
            scratch = torch.randn(1 << 16, device="cuda").sum().item()      # eager work between replays
            assert scratch == scratch
            g.replay()
            torch.cuda.synchronize()
            assert torch.equal(out.view(torch.int16), eager_out.view(torch.int16)), "replay %d differs" % rep
            assert torch.equal(idx, eager_idx)
    finally:
        F.fff_set_option("path", 0)


def _random_cases(n, seed):
    """Seeded random layer shapes: every row length class of the vector kernels (multiples of 8
    and of 4, odd ones for the fallbacks), leaf widths across the gather / tile / wide-tile
    limits, depths 0..9, ragged batch sizes around the tile and chunk boundaries."""
    rng = np.random.default_rng(seed)
    cases = []
    for i in range(n):
        dtype = W.DTYPE_BF16 if rng.random() < 0.7 else W.DTYPE_F32
        per = 8 if dtype == W.DTYPE_BF16 else 4
        D = int(rng.choice([per * int(rng.integers(1, 40)), per * int(rng.integers(40, 140)), int(rng.integers(3, 300))],
                           p=[0.5, 0.35, 0.15]))
        O = int(rng.choice([per * int(rng.integers(1, 40)), 128 * int(rng.integers(1, 5)), int(rng.integers(1, 200))],
                           p=[0.5, 0.3, 0.2]))
        L = int(rng.choice([1, 2, 3, 4, 5, 7, 8, 9, 12, 16, 17, 24, 31, 32, 33, 40]))
        depth = int(rng.integers(0, 10))
        T = int(rng.choice([1, 15, 16, 17, 63, 64, 65, 255, 257, 511, 513, 1000, 2049, 4097]))
        act = W.ACT_GELU if rng.random() < 0.5 else W.ACT_RELU
        cases.append(("rand%02d" % i, T, D, O, depth, L, act, dtype))
    return cases


RANDOM_CASES = _random_cases(36, seed=2024)


@pytest.mark.parametrize("path", [(0, 0), (2, 0), (2, 2), (5, 0)], ids=["auto", "staged", "staged_tiles", "split"])
@pytest.mark.parametrize("case", RANDOM_CASES, ids=["%s_T%d_D%d_O%d_d%d_L%d_%s" % (c[0], c[1], c[2], c[3], c[4], c[5],
                                                                                    "bf16" if c[7] else "f32")
                                                    for c in RANDOM_CASES])
def test_random_shapes(case, path):
    import paper_2308_14711_amd as F
    name, T, D, O, depth, L, act, dtype = case
    path, leaf_path = path
    print("\n[case] %s T=%d D=%d O=%d depth=%d L=%d act=%d dtype=%d seed 77 path=%d" % (name, T, D, O, depth, L, act, dtype, path),
          flush=True)
    w = W.make_layer(name, T, D, O, depth, L, act, dtype, seed=77)
    F.fff_set_option("path", path)
    F.fff_set_option("leaf_path", leaf_path)
    try:
        out, idx = run_forward(w)
        took = F.fff_get_option("last_path")
    finally:
        F.fff_set_option("path", 0)
        F.fff_set_option("leaf_path", 0)
    _log("%s path=%d took=%d" % (name, path, took), check_against_oracle(w, out, idx))


@pytest.mark.parametrize("path", [1, 2, 4, 5], ids=["fused", "staged", "token", "split"])
def test_nan_tokens_go_left_and_do_not_disturb_their_neighbours(path):
    """A NaN logit compares false with 0: such a token takes the left child at every node (the
    oracle's `logit >= 0` does the same) and its output row is NaN; every other token is unaffected."""
    import torch
    import paper_2308_14711_amd as F
    w = W.make_layer("nan", 600, 128, 64, 5, 4, W.ACT_GELU, W.DTYPE_BF16, seed=13)
    bad = [3, 17, 599]
    for t in bad:
        w.bits["x"][t, 5] = 0x7FC0           # a bf16 quiet NaN
        w.f32["x"][t, 5] = np.nan
    F.fff_set_option("path", path)
    try:
        out, idx = run_forward(w)
    finally:
        F.fff_set_option("path", 0)
    ref_out, ref_idx, margin = oracle.forward_hard(*oracle_inputs(w), w.depth, w.leaf_width, w.act)
    gi = idx.cpu().numpy()
    got = out_to_f64(out)
    assert (ref_idx[bad] == 0).all() and (gi[bad] == 0).all()
    assert np.isnan(got[bad]).all() and np.isnan(ref_out[bad]).all()
    ok = np.ones(w.T, bool)
    ok[bad] = False
    safe = ok & (margin >= ROUTING_MARGIN)
    assert np.array_equal(gi[safe], ref_idx[safe])
    err = np.abs(got[safe] - ref_out[safe]).max(axis=1) / np.maximum(np.abs(ref_out[safe]).max(axis=1), 1e-30)
    assert np.isfinite(got[ok]).all() and err.max() <= TOL[W.DTYPE_BF16]


def test_loading_the_library_before_torch_in_a_fresh_process():
    """PyTorch brings a HIP runtime of its own; a process that loads this library first must still end
    up with one runtime (the binding imports torch before it opens the library)."""
    import os
    import subprocess
    import sys
    code = (
        "import sys; sys.path.insert(0, %r); sys.path.insert(0, %r)\n"
        "import paper_2308_14711_amd as F\n"
        "F.lib()\n"
        "import fff_workloads as W\n"
        "from fff_testlib import run_forward, check_against_oracle\n"
        "w = W.make_layer('order', 15, 153, 64, 6, 9, W.ACT_GELU, W.DTYPE_BF16, seed=1)\n"
        "out, idx = run_forward(w)\n"
        "print(check_against_oracle(w, out, idx))\n"
    ) % (os.path.dirname(os.path.dirname(os.path.abspath(__file__))), os.path.dirname(os.path.abspath(__file__)))
    print("\n[case] fresh process: library first, torch second", flush=True)
    r = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-2000:]
