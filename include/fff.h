/*
 * fff.h -- C ABI of the MI355X (gfx950) library for hard-routed inference of
 * Fast Feedforward (FFF) layers.
 *
 * An FFF of depth d and leaf size l (Definition, Section "Algorithm") is a
 * balanced binary tree of 2^d - 1 node neurons over 2^d leaf networks, each a
 * <D, l, O> feedforward block.  Inference (Forward_I of Algorithm 1) walks one
 * root-to-leaf path per token -- at each node the logit w.x + b is compared
 * with 0 (output c >= 1/2 goes to child 2n+1, else 2n; paragraph "Inference
 * complexity" describes exactly this multiply-accumulate / compare / advance
 * loop) -- and evaluates only the leaf it arrives at.
 *
 * Conventions shared by every entry point
 *   - All tensor pointers are DEVICE pointers to dense row-major arrays owned
 *     by the caller.  The library reads inputs, fully overwrites outputs, and
 *     keeps no reference to either after the enqueued work has run.
 *   - `dtype` selects the element type of every floating tensor of the call:
 *     FFF_F32 (float) or FFF_BF16 (bfloat16 bit patterns, 2 bytes).  All
 *     accumulation is fp32; bf16 outputs are rounded to nearest even.
 *   - Node rows are in heap order: node N_{m,n} is row 2^m - 1 + n, its
 *     children are rows 2i+1 (taken when logit < 0) and 2i+2 (logit >= 0, ties
 *     and -0.0 included; a NaN logit compares false and goes to 2i+1).
 *   - leaf_idx[t] is the position n of the leaf N_{d,n} that token t reaches:
 *     the d decisions read as a binary number, root decision first.
 *   - Leaf k computes h = act(W1[k] x + b1[k]), y = W2[k]^T h + b2[k], with
 *     W1 [l, D] and W2 [l, O]: per neuron its D input weights, then its O
 *     output weights (Definition, Section "Algorithm": a leaf is a <D, l, O>
 *     feedforward network, one set of l neurons).
 *   - `stream` is a hipStream_t (NULL = the default stream).  Calls only
 *     enqueue work on it and return; with one exception (next item) they
 *     never allocate, free or synchronise the device.
 *   - Every call returns an fff_status.  Arguments are checked on the host
 *     before any HIP call is made: a bad argument returns its error code and
 *     enqueues nothing.  Nothing throws or aborts.
 *   - Workspace (bucket tables, work lists, intermediates; the size for given
 *     arguments is what the fff_workspace_bytes* functions return).  Each
 *     device has one, used by every call on that device, so calls on one
 *     device must not overlap in time.  Either the caller provides it
 *     (fff_set_workspace): then no call allocates, frees, clears with a
 *     memset or synchronises, and a call that needs more than the caller gave
 *     returns FFF_ERR_WORKSPACE before it enqueues anything.  Or the library
 *     owns it: a call that needs more than is there frees the old block,
 *     allocates a larger one and clears its control words -- the exception to
 *     the rule above: hipFree waits for the device.  It cannot happen during
 *     stream capture (such a call returns FFF_ERR_WORKSPACE instead), and not
 *     at all after fff_reserve_workspace* with sizes at least as large.
 */
#ifndef FFF_H
#define FFF_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    FFF_OK = 0,
    FFF_ERR_NULL = 1,        /* a required pointer is NULL */
    FFF_ERR_SHAPE = 2,       /* sizes inconsistent or out of the supported range */
    FFF_ERR_DTYPE = 3,       /* unknown dtype */
    FFF_ERR_RANGE = 4,       /* depth / leaf_width / T out of range */
    FFF_ERR_UNSUPPORTED = 5, /* unknown activation or option */
    FFF_ERR_WORKSPACE = 6,   /* workspace too small (caller-provided, or growth needed during
                                stream capture), misaligned, or could not be allocated */
    FFF_ERR_DEVICE = 7,      /* a HIP call failed (see fff_last_device_error) */
    FFF_ERR_ALIAS = 8        /* out overlaps x */
} fff_status;

typedef enum { FFF_F32 = 0, FFF_BF16 = 1 } fff_dtype;

/* The paper does not name the leaf activation; ReLU and exact GELU
 * v * Phi(v) = 0.5 v (1 + erf(v / sqrt 2)) are offered. */
typedef enum { FFF_ACT_RELU = 0, FFF_ACT_GELU = 1 } fff_act;

#define FFF_MAX_DEPTH 24

/*
 * Forward_I of Algorithm 1 for T tokens: tree descent, per-leaf bucketing,
 * leaf networks, outputs written back in token order.
 *
 *   x        [T, D]                 tokens
 *   node_w   [2^depth - 1, D]       node neurons, heap order (ignored, may be NULL, when depth == 0)
 *   node_b   [2^depth - 1]
 *   leaf_w1  [2^depth, leaf_width, D]
 *   leaf_b1  [2^depth, leaf_width]
 *   leaf_w2  [2^depth, leaf_width, O]
 *   leaf_b2  [2^depth, O]
 *   depth    0..FFF_MAX_DEPTH; leaf_width >= 1; act: fff_act
 *   out      [T, O]  same dtype as x, every row written exactly once; must not overlap x
 *   leaf_idx [T] int32, or NULL if the caller does not want the regions
 *   stream   hipStream_t
 *   T >= 0 (T == 0 is FFF_OK and enqueues nothing), D >= 1, O >= 1, dtype: fff_dtype
 *
 * Errors: FFF_ERR_NULL, FFF_ERR_RANGE (depth, leaf_width, T), FFF_ERR_SHAPE
 * (D, O < 1, or T * max(D, O), 2^depth * leaf_width * max(D, O) beyond 2^40
 * elements), FFF_ERR_DTYPE, FFF_ERR_UNSUPPORTED (act), FFF_ERR_ALIAS,
 * FFF_ERR_WORKSPACE, FFF_ERR_DEVICE.
 */
int fff_forward_hard(const void* x, const void* node_w, const void* node_b,
                     const void* leaf_w1, const void* leaf_b1,
                     const void* leaf_w2, const void* leaf_b2,
                     int depth, int leaf_width, int act,
                     void* out, int32_t* leaf_idx, void* stream,
                     int64_t T, int64_t D, int64_t O, int dtype);

/*
 * fff_forward_hard_static: for callers that cannot allocate device memory -- code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc -- and do not want to manage a
 * workspace either.  Same arguments, same kernels, same results as fff_forward_hard, but the
 * intermediates of the staged path (bucket tables, the grouped token order, hidden activations)
 * live in a fixed block of fff_static_scratch_bytes() = 16 MiB inside the library's device image:
 * the call allocates nothing, frees nothing, creates no event ("stage_timing" is ignored) and
 * never touches the device's workspace.  Every GPU the library runs on holds that block until the
 * process ends.  Sizes whose intermediates do not fit (fff_workspace_bytes(T, depth) above
 * fff_static_scratch_bytes(); the five workloads of this library's benchmark all fit) return
 * FFF_ERR_WORKSPACE and enqueue nothing (the text of fff_last_device_error says how much was needed).
 * All calls on one GPU share the one block, which keeps the last call's contents: the call clears
 * the words that must start at zero itself, and two calls whose work overlaps in time on one GPU
 * (different streams, or a replaying graph beside an eager call) race.
 */
int fff_forward_hard_static(const void* x, const void* node_w, const void* node_b,
                            const void* leaf_w1, const void* leaf_b1,
                            const void* leaf_w2, const void* leaf_b2,
                            int depth, int leaf_width, int act,
                            void* out, int32_t* leaf_idx, void* stream,
                            int64_t T, int64_t D, int64_t O, int dtype);
size_t fff_static_scratch_bytes(void);

/*
 * The stages of fff_forward_hard on their own (same conventions, same
 * kernels); used by tests and profiles.
 *
 * fff_descend: the tree walk of Forward_I alone; writes leaf_idx [T].
 */
int fff_descend(const void* x, const void* node_w, const void* node_b, int depth,
                int32_t* leaf_idx, void* stream, int64_t T, int64_t D, int dtype);

/*
 * fff_bucket: per-leaf token lists from leaf_idx [T] (values in [0, 2^depth);
 * behaviour is undefined otherwise).  count [2^depth]; offset [2^depth + 1] =
 * exclusive prefix sum of count; perm [T] = token ids grouped by leaf, in
 * ascending token order inside a leaf (stable).  Any of the three outputs may
 * be NULL.  Not part of the paper's method: it only lets tokens of one leaf
 * share one read of that leaf's weights.
 */
int fff_bucket(const int32_t* leaf_idx, int64_t T, int depth,
               int32_t* count, int32_t* offset, int32_t* perm, void* stream);

/*
 * fff_leaf_forward: the leaf networks alone, token t evaluated at leaf
 * leaf_idx[t] (device array, values in [0, 2^depth)); small batches run one
 * block per token, larger ones are bucketed internally.  Writes out [T, O].
 */
int fff_leaf_forward(const void* x, const void* leaf_w1, const void* leaf_b1,
                     const void* leaf_w2, const void* leaf_b2, const int32_t* leaf_idx,
                     int depth, int leaf_width, int act, void* out, void* stream,
                     int64_t T, int64_t D, int64_t O, int dtype);

/*
 * fff_moe_top1_forward: the mixture-of-experts counterpart the paper times the tree
 * lookup against (section "Inference speed comparison": experts of the leaves'
 * shape, k = 1 engaged expert, no gating noise).  Gating logits
 * g[t][e] = gate_w[e] . x[t] (+ gate_b[e]); expert_idx[t] = the expert with the
 * largest logit (the lowest index among equal ones; a NaN logit never wins; fp32
 * accumulation on the matrix cores, so tokens whose two largest logits are
 * within rounding of each other may be gated to either); out[t] = that expert's
 * feedforward output, with mixture weight 1.  Only the lookup differs from
 * fff_forward_hard: bucketing and the leaf kernels are the same.
 *   gate_w [2^log2_experts, D], gate_b [2^log2_experts] or NULL, the experts in
 *   the leaves' layout (leaf_w1 [2^log2_experts, leaf_width, D], ...);
 *   expert_idx [T] int32 may be NULL; dtype must be FFF_BF16 with D % 8 == 0 and
 *   16-byte aligned rows (else FFF_ERR_UNSUPPORTED); other arguments, ownership,
 *   asynchrony and errors as for fff_forward_hard.  Workspace:
 *   fff_workspace_bytes_moe(T, log2_experts).
 */
int fff_moe_top1_forward(const void* x, const void* gate_w, const void* gate_b,
                         const void* leaf_w1, const void* leaf_b1, const void* leaf_w2,
                         const void* leaf_b2, int log2_experts, int leaf_width, int act,
                         void* out, int32_t* expert_idx, void* stream,
                         int64_t T, int64_t D, int64_t O, int dtype);

/*
 * fff_forward_soft: Forward_T of Algorithm 1, the soft pass used in training and
 * for the hardening diagnostics.  Every node gives a choice score
 * c = sigmoid(w . x + b); the weight of a leaf is the product over its path of
 * c (right turns) and 1 - c (left turns) -- a stochastic vector over the
 * leaves -- and out[t] = sum over leaves of weight * leaf output.  Dense: all
 * 2^depth leaves are evaluated for every token, as three contractions on the
 * matrix cores (fp32 accumulation; the weighted hidden activations are rounded
 * to bf16 before the last one).
 *   mix      optional, device, [T, 2^depth] fp32: the leaf weights
 *   entropy  optional, device, [2^depth - 1] fp32, heap order: batch mean of the
 *            Bernoulli entropy (natural logarithm) of each node's choice score
 *            (paragraph "Hardening")
 *   dtype must be FFF_BF16 with D % 8 == 0 and 16-byte aligned rows (else
 *   FFF_ERR_UNSUPPORTED); other arguments, ownership, asynchrony and errors as
 *   for fff_forward_hard.  Workspace:
 *   fff_workspace_bytes_soft(T, O, depth, leaf_width), about
 *   4 T (2^(depth+1)) + 2 (T + O) 2^depth (leaf_width + 1) bytes.
 */
int fff_forward_soft(const void* x, const void* node_w, const void* node_b,
                     const void* leaf_w1, const void* leaf_b1, const void* leaf_w2,
                     const void* leaf_b2, int depth, int leaf_width, int act,
                     void* out, float* mix, float* entropy, void* stream,
                     int64_t T, int64_t D, int64_t O, int dtype);

/*
 * fff_forward_block: Forward_I (Algorithm 1) for nodes of size n >= 1, as a
 * pre-norm residual transformer layer.  The Definition makes a node a
 * <D, n, 1> feedforward network with a sigmoid on its output:
 *     logit = node_b2[i] + sum_j node_w2[i][j] * act(node_w1[i][j] . z + node_b1[i][j]),
 * and the walk goes to child 2i+2 when logit >= 0 (node output >= 1/2), else
 * to 2i+1; the leaf reached is evaluated on z as in fff_forward_hard.  Standing
 * in a transformer (section "Fast feedforward layers as building blocks") the
 * network reads the layer-normalised token and the block adds the token back:
 *     z = (x - mean) / sqrt(var + ln_eps) * ln_gamma + ln_beta   (var with divisor D),
 *     out = FFF(z) + x.
 * z stays in registers (fp32, or for bf16 rows of up to 1024 features a pair of
 * bf16 rows hi + lo carrying 16 mantissa bits): it is never rounded to `dtype`
 * nor stored.
 *   ln_gamma, ln_beta  device, [D], or both NULL: no normalisation (z = x)
 *   ln_eps             >= 0
 *   node_w1 [2^depth - 1, node_size, D], node_b1 and node_w2 [2^depth - 1,
 *   node_size], node_b2 [2^depth - 1], heap order, `act` also on the node's
 *   hidden neurons; may be NULL when depth == 0
 *   residual           non-zero adds x (needs O == D, else FFF_ERR_SHAPE)
 *   out [T, O]; may be x itself (same pointer, O == D), any other overlap is
 *   FFF_ERR_ALIAS; leaf_idx [T] int32 may be NULL
 *   Rows that are 16-byte aligned with D and O multiples of 8 (bf16) or 4 (fp32)
 *   and at most 4096 (bf16) or 2048 (fp32) features take the vector kernels;
 *   any other shape an element-wise kernel (correct, slow; option
 *   "last_block_kernel" reads 1 or 2 after a call).  Needs no workspace.  Other arguments, ownership, asynchrony and errors as
 *   for fff_forward_hard.
 */
int fff_forward_block(const void* x, const void* ln_gamma, const void* ln_beta, float ln_eps,
                      const void* node_w1, const void* node_b1, const void* node_w2,
                      const void* node_b2, const void* leaf_w1, const void* leaf_b1,
                      const void* leaf_w2, const void* leaf_b2, int depth, int node_size,
                      int leaf_width, int act, int residual, void* out, int32_t* leaf_idx,
                      void* stream, int64_t T, int64_t D, int64_t O, int dtype);

/*
 * Workspace sizes, in bytes (0 for arguments out of range).  Sizes follow from
 * the Definition's counts alone: T tokens, 2^depth leaves (experts), leaves of
 * leaf_width neurons, O outputs.
 *   fff_workspace_bytes       fff_forward_hard, fff_descend, fff_bucket, fff_leaf_forward
 *   fff_workspace_bytes_moe   fff_moe_top1_forward (the above plus the gating candidates)
 *   fff_workspace_bytes_soft  fff_forward_soft (the dense intermediates)
 * fff_forward_block uses none.
 */
size_t fff_workspace_bytes(int64_t T, int depth);
size_t fff_workspace_bytes_moe(int64_t T, int log2_experts);
size_t fff_workspace_bytes_soft(int64_t T, int64_t O, int depth, int leaf_width);

/*
 * fff_set_workspace: from now on every call on the current device works in the
 * caller's memory: `dev_ptr` (device memory, 256-byte aligned, `bytes` long),
 * which stays the caller's and must outlive the work that uses it.  The first
 * 256 bytes are cleared by a small kernel enqueued on `stream`; later calls
 * must be ordered after it (same stream, or an event).  While set, no call
 * allocates, frees, memsets or synchronises: one that needs more than `bytes`
 * returns FFF_ERR_WORKSPACE and enqueues nothing, so calls can be captured in
 * a HIP graph with no preparation other than this one.  dev_ptr == NULL
 * returns the device to the library-owned workspace (what it held is kept).
 * Errors: FFF_ERR_WORKSPACE (misaligned, or shorter than 256 bytes),
 * FFF_ERR_DEVICE.
 */
int fff_set_workspace(void* dev_ptr, size_t bytes, void* stream);

/* Library-owned workspace: make sure the current device's holds at least
 * fff_workspace_bytes(T, depth), or `bytes` (allocates now, so that later calls with
 * sizes up to these do not).  FFF_ERR_WORKSPACE while a caller's workspace is set. */
int fff_reserve_workspace(int64_t T, int depth);
int fff_reserve_workspace_bytes(size_t bytes);

/* Free the library-owned workspaces of all devices (call with no work in flight). */
int fff_release_workspace(void);

/*
 * Options (process-wide; not thread-safe against running calls).
 *   "path"           0 = choose by shape and batch size (default), 1 = one fused launch
 *                    (walk, leaf network and output row per token; leaf_width <= 8),
 *                    2 = staged (descent, bucketing, leaf kernels), 3 = the element-wise
 *                    fallback kernel, 4 = one block per token (small batches), 5 = the fused
 *                    launch cut in two (walk and hidden neurons per token, then the output
 *                    rows by column slices, one slice of all rows per XCD; leaf_width <= 8,
 *                    16-byte aligned output rows); a path the shape does not allow falls back
 *                    to one it does
 *   "leaf_path"      staged path only: 0 = choose by shape and bucket size (default),
 *                    1 = always the gather kernel, 2 = the MFMA tile kernels whenever the
 *                    shape allows them (bf16, leaf_width <= 32, D % 8 == 0, O % 8 == 0,
 *                    16-byte aligned rows)
 *   "bucketing"      1 (default) = the leaf kernel visits tokens grouped by leaf,
 *                    0 = in token order (no bucketing stage)
 *   "stage_timing"   1 = fff_forward_hard records hipEvents around its stages
 *                    (read them with fff_stage_times); 0 (default) = off
 * Read-only, describing the last call: "last_path" (1..5 as above), "last_leaf_path"
 * (1 = gather kernel, 2 = the two tile kernels, 3 = both, each on its share of the tiles),
 * "last_walk_top" (tree levels the descent or fused launch kept in LDS),
 * "last_block_kernel" (fff_forward_block: 1 = a vector kernel, 2 = the element-wise one),
 * "last_block_top" (node levels fff_forward_block kept in LDS).
 * Unknown names or negative values return FFF_ERR_UNSUPPORTED.
 */
int fff_set_option(const char* name, int64_t value);
int fff_get_option(const char* name, int64_t* value);

/*
 * Experiment switches of the kernels, for tests and profiles: tile shapes, LDS
 * levels, kernel selection thresholds.  Results never depend on them beyond
 * rounding order; names and meanings are listed where they are read
 * (csrc/fff_api.hip, `debug_slot`) and are not a stable interface.  value < 0
 * reads: the current value is returned through *current (may be NULL when
 * setting).  FFF_ERR_UNSUPPORTED for an unknown name.
 */
int fff_debug_option(const char* name, int64_t value, int64_t* current);

/*
 * Waits for, sums and clears the stage events recorded since the last call:
 * ms[0..3] = total milliseconds of descent, bucketing, the leaf stage's first
 * kernel and its second (the MFMA tile path computes hidden activations, then
 * output rows; the gather kernel does both in one launch and ms[3] is then the
 * gap between two marks; a single-launch path reports its kernel in ms[0]),
 * *calls = number of fff_forward_hard calls summed.  Blocks until those calls
 * have finished.
 */
int fff_stage_times(double* ms, int64_t* calls);

/* Human-readable name of a status code (static string). */
const char* fff_status_string(int status);

/* Text of the last HIP error seen on this thread's calls ("" if none). */
const char* fff_last_device_error(void);

/* The kernels the last forward call of this process launched, in order, joined by " + ", each
 * with the tile parameters that select its instantiation, e.g.
 * "walk_kernel<bf16,16,6,4,512,fused,tight> top=6".  For logs and for matching a measurement
 * with the kernel it was taken on; valid until the next call. */
const char* fff_last_launch(void);

/* Library version as major * 10000 + minor * 100 + patch. */
int fff_version(void);

#ifdef __cplusplus
}
#endif
#endif /* FFF_H */
