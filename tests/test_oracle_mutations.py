"""The pins must have teeth: a copy of the oracle's C source with one planted mistake is
compiled (CPU only) and at least one pin has to fail for it.  Nothing here touches the GPU."""
import os
import subprocess
import tempfile

import pytest

import oracle
import test_oracle_pins as pins
import test_oracle_moe_pins as moe_pins
import test_oracle_block_pins as block_pins

SRC = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "oracle", "fff_oracle.c")

# (name, text to replace, replacement): each is a plausible slip in one place
MUTATIONS = [
    ("strict_tie", "if (logit >= 0.0) n = 2 * n + 1;", "if (logit > 0.0) n = 2 * n + 1;"),
    ("children_swapped", "if (logit >= 0.0) n = 2 * n + 1;   /* c >= 1/2 */\n            else n = 2 * n;",
     "if (logit >= 0.0) n = 2 * n;\n            else n = 2 * n + 1;"),
    ("heap_row_off_by_one", "int64_t row = (((int64_t)1 << m) - 1) + n;", "int64_t row = ((int64_t)1 << m) + n;"),
    ("node_bias_dropped", "return s + b;", "return s;"),
    ("w2_transposed", "s += h[r] * ld(w2, (k * L + r) * O + o, dtype);", "s += h[r] * ld(w2, (k * O + o) * L + r, dtype);"),
    ("w1_wrong_leaf_stride", "ld(w1, (k * L + r) * D + j, dtype)", "ld(w1, (k + r) * D + j, dtype)"),
    ("b1_dropped", "h[r] = activation(s + ld(b1, k * L + r, dtype), act);", "h[r] = activation(s, act);"),
    ("b2_dropped", "y[o] = s + ld(b2, k * O + o, dtype);", "y[o] = s;"),
    ("gelu_tanh", "return 0.5 * v * (1.0 + erf(v / sqrt(2.0)));",
     "return 0.5 * v * (1.0 + tanh(0.7978845608028654 * (v + 0.044715 * v * v * v)));"),
    ("relu_leaky", "return v > 0.0 ? v : 0.0;", "return v > 0.0 ? v : 0.01 * v;"),
    ("soft_children_swapped", "forward_t(c, m + 1, 2 * n + 1, weight * cmn, yr);\n    forward_t(c, m + 1, 2 * n, weight * (1.0 - cmn), yl);",
     "forward_t(c, m + 1, 2 * n, weight * cmn, yr);\n    forward_t(c, m + 1, 2 * n + 1, weight * (1.0 - cmn), yl);"),
    ("soft_no_complement", "y[o] = cmn * yr[o] + (1.0 - cmn) * yl[o];", "y[o] = cmn * yr[o] + cmn * yl[o];"),
    ("bucket_unstable", "for (int64_t t = 0; t < T; ++t) perm[cur[leaf_idx[t]]++] = (int32_t)t;",
     "for (int64_t t = T - 1; t >= 0; --t) perm[cur[leaf_idx[t]]++] = (int32_t)t;"),
    ("bucket_offset_inclusive", "offset[j + 1] = offset[j] + count[j];", "offset[j + 1] = offset[j] + count[j] + (j == 0);"),
    ("training_size_nodes", "return (((int64_t)1 << depth) - 1) * node_size + ((int64_t)1 << depth) * leaf_size;",
     "return ((int64_t)1 << depth) * node_size + ((int64_t)1 << depth) * leaf_size;"),
    ("inference_size", "return (int64_t)depth * node_size + leaf_size;", "return (int64_t)(depth + 1) * node_size + leaf_size;"),
    ("moe_tie_highest", "if (logit > best) {", "if (logit >= best) {"),
    ("moe_bias_dropped", "double logit = gate_b ? ld(gate_b, e, dtype) : 0.0;", "double logit = 0.0;"),
    ("moe_gate_row_stride", "ld(gate_w, e * D + j, dtype) * ld(x, t * D + j, dtype)", "ld(gate_w, e + j, dtype) * ld(x, t * D + j, dtype)"),
    ("moe_expert_not_used", "leaf_b2, arg, leaf_width, act", "leaf_b2, 0, leaf_width, act"),
    ("moe_margin_not_relative", "(sc > 0.0 ? (best - second) / sc : 0.0)", "(best - second)"),
    ("moe_second_not_tracked", "} else if (logit > second) {\n                second = logit; second_scale = scale;\n            }", "}"),
    ("entropy_one_sided", "sum += h0 + h1;\n            }\n            entropy[", "sum += h0;\n            }\n            entropy["),
    ("entropy_not_a_mean", "entropy[(((int64_t)1 << m) - 1) + n] = T > 0 ? sum / (double)T : 0.0;", "entropy[(((int64_t)1 << m) - 1) + n] = sum;"),
    ("entropy_level_order", "entropy[(((int64_t)1 << m) - 1) + n] =", "entropy[(((int64_t)1 << m) - 1) + (((int64_t)1 << m) - 1 - n)] ="),
    ("block_variance_unbiased", "var /= (double)D;", "var /= (double)(D - 1);"),
    ("block_mean_not_subtracted", "z[j] = (ld(x, xoff + j, dtype) - mean) / sqrt(var + eps)", "z[j] = ld(x, xoff + j, dtype) / sqrt(var + eps)"),
    ("block_eps_outside_root", "/ sqrt(var + eps) * ld(gamma, j, dtype)", "/ (sqrt(var) + eps) * ld(gamma, j, dtype)"),
    ("block_gamma_beta_swapped", "* ld(gamma, j, dtype) + ld(beta, j, dtype);", "* ld(beta, j, dtype) + ld(gamma, j, dtype);"),
    ("block_node_output_bias_dropped", "double logit = ld(b2, row, dtype);\n    double sc", "double logit = 0.0 * ld(b2, row, dtype);\n    double sc"),
    ("block_node_hidden_bias_dropped", "logit += v * activation(s + bias, act);", "logit += v * activation(s, act);"),
    ("block_node_not_activated", "logit += v * activation(s + bias, act);", "logit += v * (s + bias);"),
    ("block_node_output_weight_index", "const double v = ld(w2, neuron, dtype);", "const double v = ld(w2, row * n, dtype);"),
    ("block_node_neuron_stride", "const int64_t neuron = row * n + j;", "const int64_t neuron = row + j;"),
    ("block_children_swapped", "n = logit >= 0.0 ? 2 * n + 1 : 2 * n;", "n = logit >= 0.0 ? 2 * n : 2 * n + 1;"),
    ("block_strict_tie", "n = logit >= 0.0 ? 2 * n + 1 : 2 * n;", "n = logit > 0.0 ? 2 * n + 1 : 2 * n;"),
    ("block_residual_dropped", "out[t * O + o] += ld(x, t * D + o, dtype);", "out[t * O + o] += 0.0;"),
    ("block_residual_normalised", "out[t * O + o] += ld(x, t * D + o, dtype);", "out[t * O + o] += z[o];"),
    ("block_leaf_reads_raw_input", "leaf_eval_vec(z, leaf_w1,", "leaf_eval(x, t * D, leaf_w1,"),
    ("block_margin_scale_without_weight", "sc += fabs(v) * (a + fabs(bias));", "sc += (a + fabs(bias));"),
    ("bf16_widen_shift", "uint32_t u = (uint32_t)((const uint16_t *)p)[i] << 16;", "uint32_t u = (uint32_t)((const uint16_t *)p)[i] << 15;"),
]

PINS = [
    pins.test_sizes_match_the_papers_table,
    pins.test_hand_worked_depth2_example,
    pins.test_gelu_closed_form_points,
    lambda: pins.test_saturated_soft_equals_hard(3, 5, 3, 2, oracle.ACT_RELU),
    pins.test_mixture_is_a_stochastic_vector,
    pins.test_zero_node_weights_give_the_dense_ff,
    lambda: pins.test_depth_zero_is_a_plain_ff(oracle.ACT_GELU),
    lambda: pins.test_depth_zero_is_a_plain_ff(oracle.ACT_RELU),
    lambda: pins.test_bit_path_agrees_with_node_signs(3),
    pins.test_axis_aligned_nodes_route_like_a_kd_tree,
    pins.test_identical_leaves_make_routing_irrelevant,
    pins.test_leaf_forward_matches_forward_hard_and_library,
    pins.test_bf16_and_f32_inputs_are_widened_exactly,
    lambda: pins.test_bucket_against_library_sort(8, 5000),
    pins.test_node_entropy_closed_forms_and_library,
    moe_pins.test_moe_hand_worked_example,
    moe_pins.test_moe_one_hot_gates_pick_by_scalar_compares,
    moe_pins.test_moe_with_two_experts_is_a_depth_one_fff,
    moe_pins.test_moe_matches_library_argmax_and_dense_expert_on_tiny_inputs,
    moe_pins.test_moe_identical_experts_make_gating_irrelevant,
    moe_pins.test_moe_expert_permutation_permutes_the_indices_only,
    moe_pins.test_moe_ties_take_the_lowest_index_and_nan_never_wins,
    moe_pins.test_moe_bf16_bits_are_widened_exactly,
    block_pins.test_block_hand_worked_example,
    block_pins.test_two_relu_neurons_make_the_linear_node,
    block_pins.test_block_against_library_layer_norm_and_products,
    block_pins.test_layer_norm_is_numpy_standardisation_then_affine,
    block_pins.test_shift_and_scale_of_the_input_do_not_matter_under_layer_norm,
    block_pins.test_residual_adds_the_unnormalised_input,
    block_pins.test_dead_hidden_neurons_leave_the_output_bias_to_decide,
    block_pins.test_permuting_a_nodes_hidden_neurons_changes_nothing,
    block_pins.test_single_hidden_neuron_and_output_weight_by_scalar_arithmetic,
    block_pins.test_depth_zero_block_is_norm_ff_residual,
]


@pytest.fixture(scope="module")
def workdir():
    with tempfile.TemporaryDirectory() as d:
        yield d
    oracle.use_library(None)


@pytest.mark.parametrize("mutation", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_a_planted_mistake_is_caught(mutation, workdir):
    name, old, new = mutation
    src = open(SRC).read()
    assert src.count(old) >= 1, "mutation %s no longer matches the oracle source" % name
    mutated = os.path.join(workdir, name + ".c")
    lib = os.path.join(workdir, name + ".so")
    open(mutated, "w").write(src.replace(old, new))
    subprocess.check_call(["gcc", "-O1", "-std=c99", "-fPIC", "-shared", "-w", "-o", lib, mutated, "-lm"])
    oracle.use_library(lib)
    caught = []
    try:
        for pin in PINS:
            try:
                pin()
            except (AssertionError, ValueError):
                caught.append(pin)
    finally:
        oracle.use_library(None)
    assert caught, "no pin noticed the planted mistake '%s'" % name


def test_the_real_oracle_passes_the_same_pins():
    oracle.use_library(None)
    for pin in PINS:
        pin()
