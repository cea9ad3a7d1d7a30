/*
 * CPU oracle for Fast Feedforward (FFF) layers.  TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, one-token-at-a-time implementation of the FFF forward passes
 * as the paper defines them (Section "Algorithm": Definition and Algorithm 1),
 * in fp64.  It exists to check the HIP library; it shares no code with it and
 * the library never calls it.  Only tests, the smoke check and the benchmark's
 * cpu_baseline leg may use it.
 *
 * What is implemented, and the passage each part follows:
 *   fff_oracle_forward_hard  Forward_I of Algorithm 1: from the root, evaluate
 *                            one node per level, go to child 2n+1 if the node
 *                            output c >= 1/2, else to child 2n; at a leaf
 *                            return the leaf network's output.
 *   fff_oracle_forward_soft  Forward_T of Algorithm 1: the recursive mixture
 *                            c * F(right) + (1 - c) * F(left).
 *   fff_oracle_leaf_forward  the leaf <D, l, O> feedforward network of the
 *                            Definition, evaluated at a given leaf.
 *   fff_oracle_node_entropy  batch mean entropy of the node choice scores
 *                            (paragraph "Hardening").
 *   fff_oracle_moe_top1      mixture of experts with one engaged expert and
 *                            noiseless gating (section "Inference speed
 *                            comparison"): argmax of the gating logits, then
 *                            that expert's feedforward output.
 *   fff_oracle_forward_block Forward_I for nodes of size n >= 1 (the Definition's
 *                            <D, n, 1> node networks), with the layer normalised
 *                            input and the residual sum of a transformer block.
 *   fff_oracle_bucket        per-leaf token lists (count, exclusive offsets,
 *                            stable order).  Not in the paper; it is the plain
 *                            definition of what the bucketing stage produces.
 *   fff_oracle_*_size/width  the size and width formulas of the paragraph
 *                            "Size and width".
 *
 * Readings of the paper used here (the paper leaves these open):
 *   - node size n = 1 (the paper uses n = 1 in all its experiments): a node is
 *     one neuron, logit = w . x + b, output c = sigmoid(logit) (the multiply-
 *     accumulate and compare of paragraph "Inference complexity"); nodes with a
 *     hidden layer of n neurons are fff_oracle_forward_block's.  c >= 1/2 is
 *     decided as logit >= 0, which is the same predicate without the rounding
 *     of a floating-point sigmoid (the paper's implementation note also
 *     compares the logit to 0).
 *   - nodes are stored in heap order: N_{m,n} is row 2^m - 1 + n.
 *   - leaf_idx is the position n of the leaf N_{d,n}; since the children of
 *     position n are 2n and 2n+1, the root decision is the top bit.
 *   - a leaf computes h = act(W1 x + b1), y = W2^T h + b2 with W1 [l, D] and
 *     W2 [l, O] (per neuron: its input weights, then its output weights).
 *   - the activation is not named by the paper; ReLU and exact (erf) GELU are
 *     offered.
 *
 * Element types of the input arrays: 0 = float32, 1 = bfloat16 bit patterns
 * in uint16 (widened exactly), 2 = float64.  All arithmetic is fp64, in index
 * order, with no intermediate rounding.
 *
 * Parity pins (tests/test_oracle_*.py): saturated-soft brute force, one-hot
 * mixture, bit path vs node signs recomputed independently, stochastic
 * vector, zero-node identity vs a library matmul, depth 0 vs a library
 * matmul, axis-aligned (k-d) routing by scalar compares, identical leaves,
 * the sizes printed in the paper's vision-transformer table, permutation
 * invariance, a hand-worked two-token example; for the mixture of experts:
 * one-hot gating rows (argmax by scalar compares), a depth-1 FFF written as two
 * experts, identical experts, a library argmax on tiny inputs, expert
 * permutation, the tie and NaN rules; for the block: a two-neuron node that
 * reduces to the linear one, a library layer normalisation, shift and scale
 * invariance, dead hidden neurons routed by the output bias alone, neuron
 * permutation, the residual difference, a hand-worked example.  Numeric output values of a forward
 * pass are not printed anywhere in the paper.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_F32 0
#define ORACLE_BF16 1
#define ORACLE_F64 2

#define ORACLE_ACT_RELU 0
#define ORACLE_ACT_GELU 1

static double ld(const void *p, int64_t i, int dtype) {
    if (dtype == ORACLE_F32) return (double)((const float *)p)[i];
    if (dtype == ORACLE_F64) return ((const double *)p)[i];
    uint32_t u = (uint32_t)((const uint16_t *)p)[i] << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}

static double activation(double v, int act) {
    if (act == ORACLE_ACT_RELU) return v > 0.0 ? v : 0.0;
    return 0.5 * v * (1.0 + erf(v / sqrt(2.0)));   /* v * Phi(v) */
}

/* Several tokens may fail to get scratch memory at once: the shared status is written atomically. */
static void flag_out_of_memory(int *err) {
#ifdef _OPENMP
#pragma omp atomic write
#endif
    *err = 2;
}

static int args_ok(int depth, int leaf_width, int act, int64_t T, int64_t D, int64_t O, int dtype) {
    return depth >= 0 && depth <= 24 && leaf_width >= 1 && T >= 0 && D >= 1 && O >= 1 &&
           (act == ORACLE_ACT_RELU || act == ORACLE_ACT_GELU) && dtype >= 0 && dtype <= 2;
}

/* logit of node N_{m,n} for token row xt; also the sum of absolute terms */
static double node_logit(const void *x, int64_t xoff, const void *node_w, const void *node_b,
                         int m, int64_t n, int64_t D, int dtype, double *scale) {
    int64_t row = (((int64_t)1 << m) - 1) + n;
    double s = 0.0, a = 0.0;
    for (int64_t j = 0; j < D; ++j) {
        double t = ld(node_w, row * D + j, dtype) * ld(x, xoff + j, dtype);
        s += t;
        a += fabs(t);
    }
    double b = ld(node_b, row, dtype);
    if (scale) *scale = a + fabs(b);
    return s + b;
}

/* y[0..O) = leaf N_{d,k}(x_t) */
static void leaf_eval(const void *x, int64_t xoff, const void *w1, const void *b1, const void *w2,
                      const void *b2, int64_t k, int L, int act, int64_t D, int64_t O, int dtype,
                      double *h, double *y) {
    for (int r = 0; r < L; ++r) {
        double s = 0.0;
        for (int64_t j = 0; j < D; ++j) s += ld(w1, (k * L + r) * D + j, dtype) * ld(x, xoff + j, dtype);
        h[r] = activation(s + ld(b1, k * L + r, dtype), act);
    }
    for (int64_t o = 0; o < O; ++o) {
        double s = 0.0;
        for (int r = 0; r < L; ++r) s += h[r] * ld(w2, (k * L + r) * O + o, dtype);
        y[o] = s + ld(b2, k * O + o, dtype);
    }
}

/*
 * Forward_I.  out [T,O] fp64, leaf_idx [T], margin [T] (optional): the
 * smallest |logit| / (sum of |terms| + |bias|) over the nodes on the token's
 * path (+inf for depth 0) -- a token whose margin is tiny may legitimately be
 * routed differently by an fp32 implementation.
 */
int fff_oracle_forward_hard(const void *x, const void *node_w, const void *node_b,
                            const void *leaf_w1, const void *leaf_b1, const void *leaf_w2,
                            const void *leaf_b2, int depth, int leaf_width, int act, int64_t T,
                            int64_t D, int64_t O, int dtype, double *out, int32_t *leaf_idx,
                            double *margin) {
    if (!args_ok(depth, leaf_width, act, T, D, O, dtype)) return 1;
    int err = 0;
#ifdef _OPENMP
#pragma omp parallel for schedule(dynamic, 16)
#endif
    for (int64_t t = 0; t < T; ++t) {
        double *h = (double *)malloc(sizeof(double) * (size_t)leaf_width);
        if (!h) { flag_out_of_memory(&err); continue; }
        int64_t n = 0;                 /* position within the current level */
        double mg = INFINITY;
        for (int m = 0; m < depth; ++m) {
            double scale;
            double logit = node_logit(x, t * D, node_w, node_b, m, n, D, dtype, &scale);
            double rel = scale > 0.0 ? fabs(logit) / scale : 0.0;
            if (rel < mg) mg = rel;
            if (logit >= 0.0) n = 2 * n + 1;   /* c >= 1/2 */
            else n = 2 * n;
        }
        if (leaf_idx) leaf_idx[t] = (int32_t)n;
        if (margin) margin[t] = mg;
        if (out) leaf_eval(x, t * D, leaf_w1, leaf_b1, leaf_w2, leaf_b2, n, leaf_width, act, D, O, dtype, h, out + t * O);
        free(h);
    }
    return err;
}

/* The leaf network alone, at the leaf given per token. */
int fff_oracle_leaf_forward(const void *x, const void *leaf_w1, const void *leaf_b1,
                            const void *leaf_w2, const void *leaf_b2, const int32_t *leaf_idx,
                            int depth, int leaf_width, int act, int64_t T, int64_t D, int64_t O,
                            int dtype, double *out) {
    if (!args_ok(depth, leaf_width, act, T, D, O, dtype)) return 1;
    for (int64_t t = 0; t < T; ++t)
        if (leaf_idx[t] < 0 || (int64_t)leaf_idx[t] >= ((int64_t)1 << depth)) return 3;
    int err = 0;
#ifdef _OPENMP
#pragma omp parallel for schedule(dynamic, 16)
#endif
    for (int64_t t = 0; t < T; ++t) {
        double *h = (double *)malloc(sizeof(double) * (size_t)leaf_width);
        if (!h) { flag_out_of_memory(&err); continue; }
        leaf_eval(x, t * D, leaf_w1, leaf_b1, leaf_w2, leaf_b2, leaf_idx[t], leaf_width, act, D, O, dtype, h, out + t * O);
        free(h);
    }
    return err;
}

/* Forward_T by the recursion of Algorithm 1.  mixw (optional, [2^d]) collects
 * the product of choice factors on the way to each leaf (the vector c). */
typedef struct {
    const void *x, *node_w, *node_b, *w1, *b1, *w2, *b2;
    int depth, L, act, dtype;
    int64_t D, O, xoff;
    double node_scale;   /* multiplies every node logit (1 = as given) */
    double *mixw;
} soft_ctx;

static void forward_t(const soft_ctx *c, int m, int64_t n, double weight, double *y) {
    int64_t O = c->O;
    if (m == c->depth) {                      /* N_{m,n} is a leaf */
        double *h = (double *)malloc(sizeof(double) * (size_t)c->L);
        leaf_eval(c->x, c->xoff, c->w1, c->b1, c->w2, c->b2, n, c->L, c->act, c->D, O, c->dtype, h, y);
        free(h);
        if (c->mixw) c->mixw[n] = weight;
        return;
    }
    double logit = c->node_scale * node_logit(c->x, c->xoff, c->node_w, c->node_b, m, n, c->D, c->dtype, NULL);
    double cmn = 1.0 / (1.0 + exp(-logit));
    double *yr = (double *)malloc(sizeof(double) * (size_t)O);
    double *yl = (double *)malloc(sizeof(double) * (size_t)O);
    forward_t(c, m + 1, 2 * n + 1, weight * cmn, yr);
    forward_t(c, m + 1, 2 * n, weight * (1.0 - cmn), yl);
    for (int64_t o = 0; o < O; ++o) y[o] = cmn * yr[o] + (1.0 - cmn) * yl[o];
    free(yr);
    free(yl);
}

int fff_oracle_forward_soft(const void *x, const void *node_w, const void *node_b,
                            const void *leaf_w1, const void *leaf_b1, const void *leaf_w2,
                            const void *leaf_b2, int depth, int leaf_width, int act, int64_t T,
                            int64_t D, int64_t O, int dtype, double node_scale, double *out,
                            double *mix /* [T, 2^d] or NULL */) {
    if (!args_ok(depth, leaf_width, act, T, D, O, dtype) || depth > 12) return 1;
    for (int64_t t = 0; t < T; ++t) {
        soft_ctx c = {x, node_w, node_b, leaf_w1, leaf_b1, leaf_w2, leaf_b2, depth, leaf_width, act,
                      dtype, D, O, t * D, node_scale, mix ? mix + t * ((int64_t)1 << depth) : NULL};
        forward_t(&c, 0, 0, 1.0, out + t * O);
    }
    return 0;
}

/* Per-leaf token lists: count[j] = tokens routed to leaf j, offset = exclusive
 * prefix sum of count (offset[2^d] = T), perm = token ids grouped by leaf,
 * ascending within a leaf. */
int fff_oracle_bucket(const int32_t *leaf_idx, int64_t T, int depth, int32_t *count,
                      int32_t *offset, int32_t *perm) {
    int64_t NL = (int64_t)1 << depth;
    for (int64_t j = 0; j < NL; ++j) count[j] = 0;
    for (int64_t t = 0; t < T; ++t) {
        if (leaf_idx[t] < 0 || leaf_idx[t] >= NL) return 3;
        count[leaf_idx[t]] += 1;
    }
    offset[0] = 0;
    for (int64_t j = 0; j < NL; ++j) offset[j + 1] = offset[j] + count[j];
    int32_t *cur = (int32_t *)malloc(sizeof(int32_t) * (size_t)NL);
    if (!cur) return 2;
    for (int64_t j = 0; j < NL; ++j) cur[j] = offset[j];
    for (int64_t t = 0; t < T; ++t) perm[cur[leaf_idx[t]]++] = (int32_t)t;
    free(cur);
    return 0;
}

/* "Size and width": all neurons, and the neurons Forward_I engages. */
int64_t fff_oracle_training_size(int depth, int node_size, int leaf_size) {
    return (((int64_t)1 << depth) - 1) * node_size + ((int64_t)1 << depth) * leaf_size;
}
int64_t fff_oracle_inference_size(int depth, int node_size, int leaf_size) {
    return (int64_t)depth * node_size + leaf_size;
}
/*
 * Batch mean of the entropy of every node's choice score, read as a Bernoulli
 * probability (paragraph "Hardening": hardening is tracked by monitoring the
 * batch mean of entropies of the choice scores at each node).  Natural
 * logarithm; 0 log 0 = 0.  Every token visits every node here, as in Forward_T.
 * entropy [2^depth - 1], heap order.
 */
int fff_oracle_node_entropy(const void *x, const void *node_w, const void *node_b, int depth,
                            int64_t T, int64_t D, int dtype, double *entropy) {
    if (!args_ok(depth, 1, ORACLE_ACT_RELU, T, D, 1, dtype)) return 1;
    for (int m = 0; m < depth; ++m) {
        for (int64_t n = 0; n < ((int64_t)1 << m); ++n) {
            double sum = 0.0;
            for (int64_t t = 0; t < T; ++t) {
                double scale;
                const double logit = node_logit(x, t * D, node_w, node_b, m, n, D, dtype, &scale);
                const double c = 1.0 / (1.0 + exp(-logit));
                const double h0 = c > 0.0 ? -c * log(c) : 0.0;
                const double h1 = c < 1.0 ? -(1.0 - c) * log(1.0 - c) : 0.0;
                sum += h0 + h1;
            }
            entropy[(((int64_t)1 << m) - 1) + n] = T > 0 ? sum / (double)T : 0.0;
        }
    }
    return 0;
}

/*
 * Mixture of experts with k = 1 and noiseless gating, the configuration of the
 * paper's inference speed comparison (section "Inference speed comparison":
 * experts of the leaf's shape, one expert engaged): gating logits g_e = G_e . x
 * (+ bias, optional), the expert with the largest logit is evaluated (the
 * lowest index among equal ones; a NaN logit is never larger), and with a
 * single engaged expert its mixture weight is 1, so the output is that expert's
 * feedforward output.  Experts are stored like leaves.
 * expert_idx [T]; margin [T] (optional): (largest - second largest logit) over
 * the larger of the two rows' sum of |terms| + |bias| (+inf for one expert) --
 * a token whose margin is tiny may legitimately be gated differently by an
 * fp32 implementation.
 */
int fff_oracle_moe_top1(const void *x, const void *gate_w, const void *gate_b, const void *leaf_w1,
                        const void *leaf_b1, const void *leaf_w2, const void *leaf_b2,
                        int64_t n_experts, int leaf_width, int act, int64_t T, int64_t D, int64_t O,
                        int dtype, double *out, int32_t *expert_idx, double *margin) {
    if (!args_ok(0, leaf_width, act, T, D, O, dtype) || n_experts < 1 || n_experts > ((int64_t)1 << 24)) return 1;
    int err = 0;
#ifdef _OPENMP
#pragma omp parallel for schedule(dynamic, 16)
#endif
    for (int64_t t = 0; t < T; ++t) {
        double *h = (double *)malloc(sizeof(double) * (size_t)leaf_width);
        if (!h) { flag_out_of_memory(&err); continue; }
        double best = -INFINITY, second = -INFINITY, best_scale = 0.0, second_scale = 0.0;
        int64_t arg = 0;
        for (int64_t e = 0; e < n_experts; ++e) {
            double logit = gate_b ? ld(gate_b, e, dtype) : 0.0;
            double scale = fabs(logit);
            for (int64_t j = 0; j < D; ++j) {
                const double term = ld(gate_w, e * D + j, dtype) * ld(x, t * D + j, dtype);
                logit += term;
                scale += fabs(term);
            }
            if (logit > best) {
                second = best; second_scale = best_scale;
                best = logit; best_scale = scale; arg = e;
            } else if (logit > second) {
                second = logit; second_scale = scale;
            }
        }
        if (expert_idx) expert_idx[t] = (int32_t)arg;
        if (margin) {
            const double sc = best_scale > second_scale ? best_scale : second_scale;
            margin[t] = (n_experts < 2 || !(second > -INFINITY)) ? INFINITY : (sc > 0.0 ? (best - second) / sc : 0.0);
        }
        if (out) leaf_eval(x, t * D, leaf_w1, leaf_b1, leaf_w2, leaf_b2, arg, leaf_width, act, D, O, dtype, h, out + t * O);
        free(h);
    }
    return err;
}

/*
 * Forward_I for nodes of size n >= 1, inside a pre-norm residual block.
 *
 * The Definition makes a node a <D, n, 1> feedforward network with a sigmoid on
 * its output: n hidden neurons (input weights u_j, bias a_j, the activation),
 * one output weight v_j each and an output bias c,
 *     logit = c + sum_j v_j * act(u_j . z + a_j),   node output = sigmoid(logit),
 * and Forward_I goes to child 2i+1 when that output is >= 1/2 (logit >= 0).
 * node_w1 [NN, n, D], node_b1 [NN, n], node_w2 [NN, n], node_b2 [NN], heap order.
 *
 * In a transformer (section "Fast feedforward layers as building blocks") the
 * layer stands where the feedforward layer stands: z = LayerNorm(x) feeds both
 * the nodes and the leaf, and the block returns x + FFF(z).  The paper does not
 * spell the block out; this is the standard pre-norm arrangement:
 *     mean = sum_j x_j / D,  var = sum_j (x_j - mean)^2 / D   (divisor D),
 *     z_j = (x_j - mean) / sqrt(var + eps) * gamma_j + beta_j.
 * norm = 0 skips the normalisation (z = x); residual = 0 returns FFF(z) alone
 * (residual = 1 needs O == D).
 *
 * margin [T] (optional): smallest |logit| / (|c| + sum_j |v_j| (sum |terms of
 * u_j . z| + |a_j|)) over the path, as for fff_oracle_forward_hard.
 */
static void layer_norm(const void *x, int64_t xoff, const void *gamma, const void *beta, double eps,
                       int64_t D, int dtype, double *z) {
    double mean = 0.0, var = 0.0;
    for (int64_t j = 0; j < D; ++j) mean += ld(x, xoff + j, dtype);
    mean /= (double)D;
    for (int64_t j = 0; j < D; ++j) {
        const double c = ld(x, xoff + j, dtype) - mean;
        var += c * c;
    }
    var /= (double)D;
    for (int64_t j = 0; j < D; ++j)
        z[j] = (ld(x, xoff + j, dtype) - mean) / sqrt(var + eps) * ld(gamma, j, dtype) + ld(beta, j, dtype);
}

static double wide_node_logit(const double *z, const void *w1, const void *b1, const void *w2,
                              const void *b2, int64_t row, int n, int act, int64_t D, int dtype,
                              double *scale) {
    double logit = ld(b2, row, dtype);
    double sc = fabs(logit);
    for (int j = 0; j < n; ++j) {
        const int64_t neuron = row * n + j;
        double s = 0.0, a = 0.0;
        for (int64_t k = 0; k < D; ++k) {
            const double t = ld(w1, neuron * D + k, dtype) * z[k];
            s += t;
            a += fabs(t);
        }
        const double bias = ld(b1, neuron, dtype);
        const double v = ld(w2, neuron, dtype);
        logit += v * activation(s + bias, act);
        sc += fabs(v) * (a + fabs(bias));
    }
    *scale = sc;
    return logit;
}

/* y[0..O) = leaf N_{d,k}(z) for an input vector already in fp64 */
static void leaf_eval_vec(const double *z, const void *w1, const void *b1, const void *w2,
                          const void *b2, int64_t k, int L, int act, int64_t D, int64_t O, int dtype,
                          double *h, double *y) {
    for (int r = 0; r < L; ++r) {
        double s = 0.0;
        for (int64_t j = 0; j < D; ++j) s += ld(w1, (k * L + r) * D + j, dtype) * z[j];
        h[r] = activation(s + ld(b1, k * L + r, dtype), act);
    }
    for (int64_t o = 0; o < O; ++o) {
        double s = 0.0;
        for (int r = 0; r < L; ++r) s += h[r] * ld(w2, (k * L + r) * O + o, dtype);
        y[o] = s + ld(b2, k * O + o, dtype);
    }
}

int fff_oracle_forward_block(const void *x, const void *ln_gamma, const void *ln_beta, double ln_eps,
                             const void *node_w1, const void *node_b1, const void *node_w2,
                             const void *node_b2, const void *leaf_w1, const void *leaf_b1,
                             const void *leaf_w2, const void *leaf_b2, int depth, int node_size,
                             int leaf_width, int act, int norm, int residual, int64_t T, int64_t D,
                             int64_t O, int dtype, double *out, int32_t *leaf_idx, double *margin) {
    if (!args_ok(depth, leaf_width, act, T, D, O, dtype) || node_size < 1 || (residual && O != D) ||
        (norm && !(ln_eps >= 0.0)))
        return 1;
    int err = 0;
#ifdef _OPENMP
#pragma omp parallel for schedule(dynamic, 16)
#endif
    for (int64_t t = 0; t < T; ++t) {
        double *z = (double *)malloc(sizeof(double) * (size_t)D);
        double *h = (double *)malloc(sizeof(double) * (size_t)leaf_width);
        if (!z || !h) { flag_out_of_memory(&err); free(z); free(h); continue; }
        if (norm) layer_norm(x, t * D, ln_gamma, ln_beta, ln_eps, D, dtype, z);
        else for (int64_t j = 0; j < D; ++j) z[j] = ld(x, t * D + j, dtype);
        int64_t n = 0;
        double mg = INFINITY;
        for (int m = 0; m < depth; ++m) {
            double scale;
            const int64_t row = (((int64_t)1 << m) - 1) + n;
            const double logit = wide_node_logit(z, node_w1, node_b1, node_w2, node_b2, row, node_size,
                                                 act, D, dtype, &scale);
            const double rel = scale > 0.0 ? fabs(logit) / scale : 0.0;
            if (rel < mg) mg = rel;
            n = logit >= 0.0 ? 2 * n + 1 : 2 * n;
        }
        if (leaf_idx) leaf_idx[t] = (int32_t)n;
        if (margin) margin[t] = mg;
        if (out) {
            leaf_eval_vec(z, leaf_w1, leaf_b1, leaf_w2, leaf_b2, n, leaf_width, act, D, O, dtype, h, out + t * O);
            if (residual)
                for (int64_t o = 0; o < O; ++o) out[t * O + o] += ld(x, t * D + o, dtype);
        }
        free(z);
        free(h);
    }
    return err;
}

int64_t fff_oracle_training_width(int depth, int leaf_size) { return ((int64_t)1 << depth) * leaf_size; }
int64_t fff_oracle_inference_width(int depth, int leaf_size) { (void)depth; return leaf_size; }

/* Number of OpenMP threads the oracle's token loops use from now on (n >= 1); no-op without OpenMP. */
void fff_oracle_set_threads(int n) {
#ifdef _OPENMP
    extern void omp_set_num_threads(int);
    if (n >= 1) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

int fff_oracle_num_threads(void) {
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    return omp_get_max_threads();
#else
    return 1;
#endif
}
