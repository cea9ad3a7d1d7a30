"""GPU parity of Forward_I with nodes of size n >= 1 inside a pre-norm residual block against the
CPU oracle, through the C ABI: leaf indices bit-exact outside the routing margin (inside it the
path taken must still be legitimate), output rows within the tolerance of the dtype."""
import numpy as np
import pytest

import fff_workloads as W
import oracle
from fff_testlib import TOL, ROUTING_MARGIN, out_to_f64

pytestmark = pytest.mark.gpu

F32, BF16 = W.DTYPE_F32, W.DTYPE_BF16

CASES = [
    # name,             T,     D,    O,    depth, n, L,  act,         dtype, norm,  residual
    ("tiny_f32",        70,    64,   64,   3,     2, 2,  W.ACT_RELU,  F32,   True,  True),
    ("ragged_f32",      333,   200,  40,   4,     3, 5,  W.ACT_GELU,  F32,   True,  False),
    ("vit_block",       3000,  768,  768,  8,     4, 8,  W.ACT_GELU,  BF16,  True,  True),
    ("one_neuron",      1000,  768,  768,  5,     1, 1,  W.ACT_RELU,  BF16,  False, True),
    ("plain_wide_node", 500,   128,  32,   6,     2, 4,  W.ACT_GELU,  BF16,  False, False),
    ("ragged_bf16",     257,   1032, 520,  3,     5, 6,  W.ACT_GELU,  BF16,  True,  False),
    ("long_rows_bf16",  130,   4096, 4096, 2,     2, 3,  W.ACT_RELU,  BF16,  True,  True),
    ("long_rows_f32",   66,    2048, 2048, 2,     3, 2,  W.ACT_GELU,  F32,   True,  True),
    ("mid_rows_f32",    200,   520,  1000, 3,     2, 3,  W.ACT_RELU,  F32,   True,  False),
    ("depth_zero",      100,   256,  256,  0,     2, 5,  W.ACT_GELU,  BF16,  True,  True),
    ("one_token",       1,     768,  768,  4,     2, 2,  W.ACT_GELU,  BF16,  True,  True),
    ("more_than_waves", 16389, 64,   64,   4,     2, 2,  W.ACT_RELU,  BF16,  True,  True),
    ("many_neurons",    400,   256,  256,  3,     9, 11, W.ACT_GELU,  F32,   True,  True),
    ("deep",            2000,  256,  256,  12,    2, 1,  W.ACT_RELU,  BF16,  True,  True),
    ("group_max_bf16",  300,   1024, 1024, 4,     3, 5,  W.ACT_GELU,  BF16,  True,  True),
    ("group_ragged8",   257,   800,  1000, 3,     2, 3,  W.ACT_RELU,  BF16,  True,  False),
    ("group_max_f32",   200,   512,  384,  3,     6, 7,  W.ACT_GELU,  F32,   True,  False),
    ("group_f32_six",   150,   384,  384,  5,     1, 2,  W.ACT_RELU,  F32,   False, True),
    ("wide_leaf",       20,    40,   40,   1,     2, 300, W.ACT_RELU, F32,   True,  True),
]


def _upload(a):
    import torch
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(a).cuda()


def _widen(a):
    return (W.bf16_widen(a) if a.dtype == np.uint16 else a).astype(np.float64)


def _inputs(name, T, D, O, depth, n, L, act, dtype, norm, seed):
    w = W.make_layer(name, T, D, O, depth, L, act, dtype, seed=seed)
    nodes = W.wide_nodes(depth, n, D, dtype, seed=seed)
    ln = W.layer_norm_params(D, dtype, seed=seed) if norm else (None, None)
    leaves = [np.ascontiguousarray(w.device_array(k)) for k in ("leaf_w1", "leaf_b1", "leaf_w2", "leaf_b2")]
    return np.ascontiguousarray(w.device_array("x")), ln, nodes, leaves


def _normalised(x64, ln, eps):
    """z in fp64 from numpy's mean and var, for re-evaluating margin tokens."""
    if ln[0] is None:
        return x64
    return ((x64 - x64.mean(axis=1, keepdims=True)) / np.sqrt(x64.var(axis=1, keepdims=True) + eps)
            * _widen(ln[0]) + _widen(ln[1]))


def _path_is_legitimate(z, nodes, depth, n, act, leaf):
    """At every node on the way to `leaf` the decision agrees with the fp64 logit or that logit
    is inside the margin."""
    w1, b1, w2, b2 = (_widen(a) for a in nodes)
    from scipy.special import erf
    f = (lambda v: np.maximum(v, 0)) if act == W.ACT_RELU else (lambda v: 0.5 * v * (1 + erf(v / np.sqrt(2))))
    for m in range(depth):
        i = (1 << m) - 1 + (leaf >> (depth - m))
        terms = w1[i] * z
        logit = b2[i] + (w2[i] * f(terms.sum(axis=1) + b1[i])).sum()
        scale = abs(b2[i]) + (np.abs(w2[i]) * (np.abs(terms).sum(axis=1) + np.abs(b1[i]))).sum()
        bit = (leaf >> (depth - 1 - m)) & 1
        if (logit >= 0) != bool(bit) and abs(logit) >= ROUTING_MARGIN * scale:
            return False
    return True


def _check(case, seed=5, in_place=False, want_idx=True):
    import torch
    import paper_2308_14711_amd as F
    name, T, D, O, depth, n, L, act, dtype, norm, residual = case
    eps = 1e-5
    x, ln, nodes, leaves = _inputs(name, T, D, O, depth, n, L, act, dtype, norm, seed)
    d_x = _upload(x)
    d_ln = [None if a is None else _upload(a) for a in ln]
    d_nodes = [_upload(a) if depth > 0 else None for a in nodes]
    d_leaves = [_upload(a) for a in leaves]
    if in_place:
        out = d_x
    else:
        out = torch.full((T, O), float("nan"), dtype=d_x.dtype, device="cuda")
    idx = torch.full((T,), -9, dtype=torch.int32, device="cuda") if want_idx else None
    F.fff_forward_block(d_x, d_ln[0], d_ln[1], eps, *d_nodes, *d_leaves, depth, n, L, act, residual, out, idx)
    torch.cuda.synchronize()
    ref_out, ref_idx, margin = oracle.forward_block(x, ln[0], ln[1], eps, *nodes, *leaves, depth, n, L, act, residual)
    got = out_to_f64(out)
    assert got.shape == ref_out.shape and np.isfinite(got).all()
    keep = np.ones(T, bool)
    n_diff = 0
    if want_idx:
        gi = idx.cpu().numpy()
        assert gi.min() >= 0 and gi.max() < (1 << depth)
        diff = np.nonzero(gi != ref_idx)[0]
        n_diff = int(diff.size)
        assert (margin[diff] >= ROUTING_MARGIN).sum() == 0, "routing differs outside the margin at %s" % diff[:5]
        if diff.size:
            # the rest must be valid: a legitimate path, and the row of the leaf taken
            z = _normalised(_widen(x[diff]), ln, eps)
            for k, t in enumerate(diff):
                assert _path_is_legitimate(z[k], nodes, depth, n, act, int(gi[t])), "token %d took an illegitimate path" % t
            redo = oracle.leaf_forward(z, *[_widen(a) for a in leaves], gi[diff], depth, L, act)
            ref_out = ref_out.copy()
            ref_out[diff] = redo + (_widen(x[diff]) if residual else 0.0)
    else:
        keep = margin >= ROUTING_MARGIN
    scale = np.maximum(np.abs(ref_out).max(axis=1), 1e-30)
    err = (np.abs(got - ref_out).max(axis=1) / scale)[keep]
    assert err.max(initial=0.0) <= TOL[dtype], "row %d off by %.3e" % (int(np.argmax(err)), err.max())
    print("  block %s: %d margin tokens, %d routed differently, %d leaves used, max row error %.2e" % (
        name, int((margin < ROUTING_MARGIN).sum()), n_diff, len(set(ref_idx.tolist())), err.max(initial=0.0)), flush=True)
    return ref_idx


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_block_against_the_oracle(case):
    print("\n[case] block %s T=%d D=%d O=%d depth=%d n=%d L=%d act=%d dtype=%d norm=%s residual=%s seed 5" % case, flush=True)
    ref_idx = _check(case)
    if case[4] >= 3 and case[1] >= 200:
        assert len(set(ref_idx.tolist())) >= 4, "the workload does not spread over the leaves"


def test_block_in_place_and_without_an_index_buffer():
    print("\n[case] block in place (out = x), then without leaf_idx", flush=True)
    _check(("in_place", 900, 768, 768, 6, 3, 4, W.ACT_GELU, BF16, True, True), in_place=True)
    _check(("in_place_f32", 300, 128, 128, 4, 2, 2, W.ACT_RELU, F32, True, True), in_place=True)
    _check(("no_idx", 900, 768, 768, 6, 3, 4, W.ACT_GELU, BF16, True, True), want_idx=False)


STAGED = [
    # from 32768 tokens on the lane-group kernel keeps the top node levels' rows in LDS (last column:
    # how many levels)
    # name,              T,     D,    O,    depth, n, L, act,         dtype, norm,  residual, top
    ("staged_vit",       40000, 768,  768,  8,     4, 8, W.ACT_GELU,  BF16,  True,  True,  3),
    ("staged_one",       33000, 768,  768,  9,     1, 1, W.ACT_RELU,  BF16,  False, True,  5),
    ("staged_f32",       32768, 200,  40,   6,     3, 5, W.ACT_GELU,  F32,   True,  False, 4),
    ("staged_whole",     35003, 64,   64,   4,     2, 2, W.ACT_RELU,  BF16,  True,  True,  4),
    ("staged_widest",    32800, 1000, 1000, 5,     2, 3, W.ACT_GELU,  BF16,  True,  False, 4),
]


@pytest.mark.parametrize("case", STAGED, ids=[c[0] for c in STAGED])
def test_block_with_top_levels_in_lds(case):
    import torch
    import paper_2308_14711_amd as F
    print("\n[case] block %s T=%d D=%d O=%d depth=%d n=%d L=%d act=%d dtype=%d norm=%s residual=%s seed 5, %d levels in LDS" % case, flush=True)
    top = case[-1]
    _check(case[:-1])
    assert F.fff_get_option("last_block_kernel") == 1
    assert F.fff_get_option("last_block_top") == top
    # the same launch with fewer levels, and with every level read from memory, gives the same bits
    name, T, D, O, depth, n, L, act, dtype, norm, residual = case[:-1]
    x, ln, nodes, leaves = _inputs(name, T, D, O, depth, n, L, act, dtype, norm, 5)
    d = [_upload(x)] + [None if a is None else _upload(a) for a in ln]
    d_w = [_upload(a) for a in nodes] + [_upload(a) for a in leaves]
    bits = torch.int16 if dtype == BF16 else torch.int32
    outs = []
    try:
        for top_option, expect in ((0, top), (2, 1), (1, 0)):
            F.fff_debug_option("block_top", top_option)
            out = torch.empty((T, O), dtype=d[0].dtype, device="cuda")
            idx = torch.empty((T,), dtype=torch.int32, device="cuda")
            F.fff_forward_block(d[0], d[1], d[2], 1e-5, *d_w, depth, n, L, act, residual, out, idx)
            torch.cuda.synchronize()
            assert F.fff_get_option("last_block_top") == expect
            outs.append((out, idx))
    finally:
        F.fff_debug_option("block_top", 0)
    for out, idx in outs[1:]:
        assert torch.equal(outs[0][1], idx) and torch.equal(outs[0][0].view(bits), out.view(bits))


GENERIC = [
    # shapes the vector kernels do not take: the element-wise kernel
    ("odd_f32",        130,  50,   7,    4, 3, 3,  W.ACT_GELU, F32,  True,  False),
    ("odd_bf16",       99,   77,   77,   3, 2, 2,  W.ACT_RELU, BF16, True,  True),
    ("too_long_bf16",  40,   4104, 4104, 2, 2, 1,  W.ACT_GELU, BF16, True,  True),
    ("too_long_f32",   33,   2052, 16,   2, 1, 5,  W.ACT_RELU, F32,  False, False),
    ("odd_out_only",   200,  64,   30,   5, 4, 6,  W.ACT_GELU, BF16, True,  False),
    ("wide_leaf_odd",  20,   42,   42,   1, 2, 300, W.ACT_RELU, F32, True,  True),
]


@pytest.mark.parametrize("case", GENERIC, ids=[c[0] for c in GENERIC])
def test_block_shapes_for_the_element_wise_kernel(case):
    import paper_2308_14711_amd as F
    print("\n[case] block %s T=%d D=%d O=%d depth=%d n=%d L=%d act=%d dtype=%d norm=%s residual=%s seed 5" % case, flush=True)
    _check(case)
    assert F.fff_get_option("last_block_kernel") == 2
    _check(("vector_again", 70, 64, 64, 3, 2, 2, W.ACT_RELU, F32, True, True))
    assert F.fff_get_option("last_block_kernel") == 1


def test_block_two_relu_neurons_route_like_the_linear_node():
    """Hidden neurons (w, b), (-w, -b) with output weights (1, -1): the node is the linear neuron,
    so the block without normalisation and residual must agree with fff_forward_hard's routing
    wherever the oracle's margin is clear, and both with the oracle."""
    import torch
    import paper_2308_14711_amd as F
    print("\n[case] block with two-neuron linear nodes vs fff_forward_hard, T=2000 D=256 depth=7 seed 6", flush=True)
    T, D, O, depth, L = 2000, 256, 64, 7, 2
    w = W.make_layer("lin", T, D, O, depth, L, W.ACT_RELU, BF16, seed=6)
    nw, nb = w.bits["node_w"], w.bits["node_b"]
    neg = lambda a: a ^ np.uint16(0x8000)
    one, minus_one = np.uint16(0x3F80), np.uint16(0xBF80)
    NN = (1 << depth) - 1
    nodes = [np.ascontiguousarray(np.stack([nw, neg(nw)], axis=1)), np.ascontiguousarray(np.stack([nb, neg(nb)], axis=1)),
             np.tile(np.array([one, minus_one], np.uint16), (NN, 1)), np.zeros((NN,), np.uint16)]
    leaves = [w.bits[k] for k in ("leaf_w1", "leaf_b1", "leaf_w2", "leaf_b2")]
    d_x = _upload(w.bits["x"])
    out_a = torch.empty((T, O), dtype=torch.bfloat16, device="cuda")
    out_b = torch.empty((T, O), dtype=torch.bfloat16, device="cuda")
    idx_a = torch.empty((T,), dtype=torch.int32, device="cuda")
    idx_b = torch.empty((T,), dtype=torch.int32, device="cuda")
    d_leaves = [_upload(a) for a in leaves]
    F.fff_forward_block(d_x, None, None, 0.0, *[_upload(a) for a in nodes], *d_leaves, depth, 2, L, W.ACT_RELU,
                        False, out_a, idx_a)
    F.fff_forward_hard(d_x, _upload(nw), _upload(nb), *d_leaves, depth, L, W.ACT_RELU, out_b, idx_b)
    torch.cuda.synchronize()
    _, ref_idx, margin = oracle.forward_hard(w.bits["x"], nw, nb, *leaves, depth, L, W.ACT_RELU, want_out=False)
    clear = margin >= ROUTING_MARGIN
    ia, ib = idx_a.cpu().numpy(), idx_b.cpu().numpy()
    assert np.array_equal(ia[clear], ref_idx[clear]) and np.array_equal(ib[clear], ref_idx[clear])
    same = ia == ib
    a, b = out_to_f64(out_a)[same], out_to_f64(out_b)[same]
    assert np.abs(a - b).max() <= TOL[BF16] * np.abs(b).max()


def test_block_nan_token_is_routed_like_the_oracle_and_spoils_only_its_own_row():
    import torch
    import paper_2308_14711_amd as F
    print("\n[case] block with a NaN token, T=64 D=128 depth=4", flush=True)
    case = ("nan", 64, 128, 128, 4, 2, 2, W.ACT_RELU, F32, False, True)
    x, ln, nodes, leaves = _inputs(*case[:10], seed=8)
    x = x.copy()
    x[17, 5] = np.nan
    out = torch.zeros((64, 128), dtype=torch.float32, device="cuda")
    idx = torch.full((64,), -1, dtype=torch.int32, device="cuda")
    F.fff_forward_block(_upload(x), None, None, 0.0, *[_upload(a) for a in nodes], *[_upload(a) for a in leaves],
                        4, 2, 2, W.ACT_RELU, True, out, idx)
    torch.cuda.synchronize()
    ref_out, ref_idx, _ = oracle.forward_block(x, None, None, 0.0, *nodes, *leaves, 4, 2, 2, W.ACT_RELU, True)
    gi, got = idx.cpu().numpy(), out.cpu().numpy()
    assert gi[17] == ref_idx[17]
    rows = np.arange(64) != 17
    assert np.isfinite(got[rows]).all() and np.array_equal(gi[rows], ref_idx[rows])
    assert np.isnan(got[17]).any()


def test_block_captured_in_a_hip_graph_and_replayed():
    """The call enqueues one kernel and allocates nothing: it can be captured, and every replay, with
    eager work and synchronisations in between, must reproduce the eager result bit for bit."""
    import torch
    import paper_2308_14711_amd as F
    print("\n[case] block in a HIP graph, T=2500 D=768 depth=6 n=3 L=4 seed 12", flush=True)
    case = ("graph", 2500, 768, 768, 6, 3, 4, W.ACT_GELU, BF16, True, True)
    name, T, D, O, depth, n, L, act, dtype, norm, residual = case
    x, ln, nodes, leaves = _inputs(name, T, D, O, depth, n, L, act, dtype, norm, 12)
    d_x, d_ln = _upload(x), [_upload(a) for a in ln]
    d_nodes, d_leaves = [_upload(a) for a in nodes], [_upload(a) for a in leaves]
    eager = torch.empty((T, O), dtype=torch.bfloat16, device="cuda")
    eager_idx = torch.empty((T,), dtype=torch.int32, device="cuda")
    F.fff_forward_block(d_x, d_ln[0], d_ln[1], 1e-5, *d_nodes, *d_leaves, depth, n, L, act, residual, eager, eager_idx)
    torch.cuda.synchronize()
    out, idx = torch.zeros_like(eager), torch.zeros_like(eager_idx)
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        F.fff_forward_block(d_x, d_ln[0], d_ln[1], 1e-5, *d_nodes, *d_leaves, depth, n, L, act, residual, out, idx)
    for rep in range(4):
        out.fill_(float("nan"))
        idx.fill_(-1)
        scratch = torch.randn(1 << 16, device="cuda").sum().item()      # eager work between replays
        assert scratch == scratch
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(out.view(torch.int16), eager.view(torch.int16)), "replay %d differs" % rep
        assert torch.equal(idx, eager_idx)


def _random_block_cases(count, seed):
    """Seeded random shapes over both kernels: piece counts on either side of every template
    boundary, node sizes and leaf widths around the batch sizes, with and without the
    normalisation and the residual."""
    rng = np.random.default_rng(seed)
    cases = []
    for i in range(count):
        dtype = BF16 if rng.random() < 0.6 else F32
        per = 8 if dtype == BF16 else 4
        pieces = int(rng.choice([rng.integers(1, 33), rng.integers(33, 129), rng.integers(129, 300)], p=[0.4, 0.4, 0.2]))
        D = per * pieces
        residual = bool(rng.random() < 0.5)
        O = D if residual else per * int(rng.integers(1, 140))
        cases.append(("rnd%02d" % i, int(rng.integers(1, 700)), D, O, int(rng.integers(0, 8)), int(rng.integers(1, 8)),
                      int(rng.integers(1, 10)), int(rng.integers(0, 2)), dtype, bool(rng.random() < 0.7), residual))
    return cases


@pytest.mark.parametrize("case", _random_block_cases(24, 2024), ids=lambda c: c[0])
def test_block_random_shapes(case):
    print("\n[case] block %s T=%d D=%d O=%d depth=%d n=%d L=%d act=%d dtype=%d norm=%s residual=%s seed 9" % case, flush=True)
    _check(case, seed=9)
