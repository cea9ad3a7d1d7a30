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
 *     output weights (the paper's "one set of neurons that has both input and
 *     output weights").
 *   - `stream` is a hipStream_t (NULL = the default stream).  Calls only
 *     enqueue work on it and return; they never synchronise the device.
 *   - Every call returns an fff_status.  Arguments are checked on the host
 *     before any HIP call is made: a bad argument returns its error code and
 *     enqueues nothing.  Nothing throws or aborts.
 *   - The library keeps one workspace per device (bucket tables, work lists).
 *     It is grown with hipMalloc when a call needs more than is there (never
 *     shrunk), so calls on one device must not overlap in time, and a caller
 *     that cannot tolerate an allocation mid-stream calls
 *     fff_reserve_workspace first.
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
    FFF_ERR_WORKSPACE = 6,   /* workspace could not be allocated */
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
 *   asynchrony and errors as for fff_forward_hard.  The gating needs
 *   2 * T * ceil(2^log2_experts / 128) more words of workspace than
 *   fff_workspace_bytes reports; the first call with larger sizes allocates them.
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
 *   for fff_forward_hard.  Needs about
 *   4 T (2^(depth+1)) + 2 (T + O) 2^depth (leaf_width + 1) bytes of workspace,
 *   allocated by the first call with larger sizes (FFF_ERR_WORKSPACE if that fails).
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

/* Bytes of workspace a call with these sizes uses on the current device. */
size_t fff_workspace_bytes(int64_t T, int depth);

/* Make sure the current device's workspace holds at least fff_workspace_bytes(T, depth)
 * (allocates now, so that later calls with sizes up to these do not). */
int fff_reserve_workspace(int64_t T, int depth);

/* Free the workspaces of all devices (call with no work in flight). */
int fff_release_workspace(void);

/*
 * Tuning and test switches (process-wide; not thread-safe against running calls).
 *   "leaf_path"      staged path only: 0 = the MFMA tile kernels when the shape allows them
 *                    (bf16, 3 <= leaf_width <= 32, D % 8 == 0, O % 8 == 0, 16-byte aligned
 *                    rows) and a leaf sees at least 8 tokens on average or is wider than 8
 *                    neurons (32 tokens on average for batches of up to 8192 tokens), else
 *                    the gather kernel (default); 1 = always the gather kernel;
 *                    2 = the tile kernels whenever the shape allows them, also for
 *                    leaf_width 1 and 2
 *   "path"           0 = choose by shape and batch size (default), 1 = one fused launch
 *                    (walk, leaf network and output row per token, tokens streamed through
 *                    persistent blocks; leaf_width <= 8), 2 = staged (descent, bucketing,
 *                    leaf kernels), 3 = the element-wise fallback kernel, 4 = one block per
 *                    token (small batches: several tree levels per memory round trip, the
 *                    leaf's neurons split over the block's waves; rows of at most 512
 *                    16-byte vectors); a path the shape does not allow falls back to one it
 *                    does.  The default takes 4 for batches of up to "token_max_T" tokens
 *                    (6 times that where leaf_width > 8 rules out the fused launch), then
 *                    staged when there are more than 8192 tokens, the leaf rows a token meets
 *                    are many bytes (24 KB, or 12 KB with more than 8 MB of leaf weights in
 *                    total, or 8 KB with more than 16 MB) and a leaf sees >= 3 tokens on
 *                    average, else fused
 *   "token_max_T"    see "path" (default 512)
 *   "walk_tpg", "walk_block", "walk_top", "walk_bpc", "walk_prefetch"
 *                    experiment switches of the fused/descent kernel (tokens per lane
 *                    group, threads per block, k + 1 = at most k LDS-staged levels,
 *                    persistent blocks per compute unit, next-tile prefetch); 0 = built-in
 *                    choice, combinations the kernel is not built for are ignored
 *   "bucketing"      1 (default) = the leaf kernel visits tokens grouped by leaf,
 *                    0 = in token order (no bucketing stage)
 *   "last_path"      read it after a call: the path (1, 2, 3 or 4) fff_forward_hard took
 *   "last_walk_top"  read it after a call: the tree levels the last descent or fused launch kept
 *                    in LDS
 *   "last_block_kernel" read it after fff_forward_block: 1 = a vector kernel ran, 2 = the
 *                    element-wise one
 *   "block_top"      fff_forward_block, rows of up to 128 pieces, 32768 tokens and more: the
 *                    hidden-neuron rows of the top node levels are kept in LDS by persistent
 *                    blocks; k + 1 = at most k such levels, 0 = as many as fit (default).
 *                    The results do not depend on it, bit for bit.
 *   "last_block_top" read it after fff_forward_block: the levels its launch kept in LDS
 *   "last_leaf_path" read it after a staged call: 1 = its leaf stage ran the gather kernel,
 *                    2 = the two tile kernels, 3 = both, each on its share of the tiles
 *   "leaf_split"     staged leaf stage on the tile kernels: 1..16 = a tile (16 consecutive
 *                    slots of the bucketed order) with at least this many runs of equal leaf
 *                    goes to the gather kernel instead; 0 (default) or above 16 = no split
 *   "bucket_kernel"  0 = choose by size (default: the token-chunk kernel up to 131072 tokens
 *                    and 4096 leaves; beyond that the segment kernels for up to 4096
 *                    leaves, else the leaf-range kernel up to 2^21 tokens and 2^19 leaves,
 *                    else the chunk-matrix kernels), 4 = the segment kernels when the sizes
 *                    allow them, 1 = the leaf-range kernel when the
 *                    sizes allow it, 2 = always the chunk-matrix kernels, 3 = the token-chunk
 *                    kernel when the sizes allow it
 *   "stage_timing"   1 = fff_forward_hard records hipEvents around its stages
 *                    (read them with fff_stage_times); 0 (default) = off
 * Unknown names or negative values return FFF_ERR_UNSUPPORTED.
 */
int fff_set_option(const char* name, int64_t value);
int fff_get_option(const char* name, int64_t* value);

/*
 * fff_probe_gather: a measuring stick for the roofline discussion, not a step of
 * the method.  Launches `blocks` blocks of 512 threads; every 16 lanes read,
 * `iters` times, `rows_in_flight` (1 or 4) rows of `row_bytes` bytes picked at
 * random from `table` (device, table_rows rows, a power of two, 16-byte aligned,
 * row_bytes a multiple of 16; fill it with zeros) -- the access pattern of a
 * tree walk, one row per token and level.  `dependent` non-zero makes each row
 * index wait for the data of the previous one.  The caller times the launch;
 * bytes moved = blocks * 32 * iters * rows_in_flight * row_bytes.  `sink`: 4
 * bytes of device memory (never written for a table of zeros).
 */
int fff_probe_gather(const void* table, int64_t table_rows, int64_t row_bytes, int rows_in_flight,
                     int64_t blocks, int iters, int dependent, void* sink, void* stream);

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

/* Library version as major * 10000 + minor * 100 + patch. */
int fff_version(void);

#ifdef __cplusplus
}
#endif
#endif /* FFF_H */
