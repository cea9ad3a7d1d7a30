// Host-side declarations shared by the translation units of the library.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fff {

// One FFF call, as validated by the C ABI.
struct Problem {
    const void* x;
    const void* node_w;
    const void* node_b;
    const void* leaf_w1;
    const void* leaf_b1;
    const void* leaf_w2;
    const void* leaf_b2;
    void* out;
    int32_t* leaf_idx;
    int64_t T, D, O;
    int depth, L, act;
    bool bf16;
};

// Per-device scratch, carved out of one allocation (all int32 words).
struct Workspace {
    int32_t* leaf_idx;   // [T]      when the caller passes none
    int32_t* rank;       // [T]      rank of a token among same-leaf tokens of its chunk
    int32_t* slot_leaf;  // [T]      leaf of every slot of perm
    int32_t* perm;       // [T]      token ids grouped by leaf
    int32_t* count;      // [NL]
    int32_t* offset;     // [NL + 1]
    int32_t* tile_off;   // [NL + 1] exclusive prefix of per-leaf tile counts
    int32_t* chunk_cnt;  // [C, NL]  per-chunk histograms, then per-chunk bases
    int32_t* fold;       // [kFoldWords] per-block leaf counts of the descent (DescentCounts::M)
    int32_t* hidden;     // [16 T]   hidden activations of the tile path, T * L bf16 (L <= 32)
    int32_t* extra;      // caller-specific region (gating candidates of the mixture of experts)
    int32_t* ctrl;       // [16]     ticket counters and totals
    int64_t n_chunks;
};

constexpr int kChunkTokens = 256;   // tokens per bucketing chunk
constexpr int kTileRows = 16;       // rows of one MFMA tile
constexpr int kTilesMaxLeafWidth = 32;   // widest leaf the MFMA tile path takes

bool vec_ok(const void* p, int64_t row_elems, bool bf16);

// Every launch function names the kernel it starts, with the tile parameters that select the
// instantiation ("walk_kernel<bf16,16,6,4,512,fused,tight>"); a forward call's names, joined by
// " + ", are what fff_last_launch returns.
void note_launch(const char* fmt, ...) __attribute__((format(printf, 1, 2)));

// Per-block leaf counts, the hand-over from the descent to the bucketing stage: block b of the
// descent owns tokens [b * share, (b + 1) * share) and leaves M[b][leaf] = how many of them reach
// `leaf`, so that the bucketing stage needs no histogram pass of its own (launch_bucket_fold).
struct DescentCounts {
    int32_t* M = nullptr;    // in: room for `capacity` words
    int64_t capacity = 0;
    int blocks = 0;          // out: blocks that wrote a row of M; 0 = the launch left no counts
    int64_t share = 0;       // out: tokens per block
};
constexpr int kFoldMaxLeaves = 1024;
constexpr int kFoldMaxShare = 1024;
constexpr int64_t kFoldWords = 128 * 1024;   // [blocks, leaves] counters the fold kernel reads per block
bool bucket_fold_ok(int depth, int64_t blocks, int64_t share);

// K1: tree descent.  leaf_idx[t] for all t (any shape: falls back to element loads).
// dc (optional): the launch also leaves per-block leaf counts there when bucket_fold_ok.
hipError_t launch_descend(const Problem& p, int32_t* leaf_idx, hipStream_t s, DescentCounts* dc = nullptr);
// Descent + leaf network + output row in one launch; needs fused_shape_ok(p).
hipError_t launch_walk_fused(const Problem& p, int32_t* leaf_idx, hipStream_t s);
// The fused launch cut in two for leaf tables that outgrow an L2: walk + hidden neurons per token
// (launch_walk_hidden: leaf_idx [T] and hidden [T, L] fp32 out), then the output rows by column
// slices (launch_leaf_slices): every XCD writes one slice of all rows, so that its L2 only ever
// holds that slice of the output weights and biases.  Same arithmetic in the same order as the
// single launch.  Needs fused_shape_ok and slices_shape_ok.
hipError_t launch_walk_hidden(const Problem& p, int32_t* leaf_idx, float* hidden, hipStream_t s);
bool slices_shape_ok(const Problem& p);
hipError_t launch_leaf_slices(const Problem& p, const int32_t* leaf_idx, const float* hidden, hipStream_t s);
// Experiment switches of the walk kernel (0 = the built-in choice).
// Compute units, the dynamic LDS a block may ask for, the L2 of one XCD and the index of the current device (cached).
struct DeviceInfo {
    int cus = 0;
    size_t lds_per_block = 0;
    int dev = 0;
    int64_t l2_bytes = 0;   // one XCD's L2
};
DeviceInfo device_info();

struct WalkTuning {
    int64_t tpg = 0;     // tokens per lane group
    int64_t block = 0;   // threads per block
    int64_t top = 0;     // k + 1 forces at most k LDS-staged levels
    int64_t bpc = 0;     // persistent blocks per compute unit
    int64_t prefetch = 0; // 1: request the next tile's token rows one iteration ahead
    int64_t plain_x = 0;  // descent: 1 = read token rows without the streaming hint, 2 = with it, 0 = by batch size
    int64_t last_top = 0; // read-only: tree levels the last walk launch kept in LDS
};
extern WalkTuning g_walk_tuning;
bool walk_shape_ok(const Problem& p);
bool fused_shape_ok(const Problem& p);

// K2: bucketing.  Needs ws.chunk_cnt zeroed on entry; leaves it dirty.
//   slot_leaf (optional): the leaf of every slot of perm
hipError_t launch_bucket(const int32_t* leaf_idx, int64_t T, int depth, const Workspace& ws,
                         int32_t* count, int32_t* offset, int32_t* perm, int32_t* slot_leaf, hipStream_t s);
hipError_t launch_zero(int32_t* p, int64_t n, hipStream_t s);
// K2 in one launch (no workspace besides the outputs); any output may be null.
bool bucket_onepass_ok(int64_t T, int depth);
hipError_t launch_bucket_onepass(const int32_t* leaf_idx, int64_t T, int depth, int32_t* count,
                                 int32_t* offset, int32_t* perm, int32_t* slot_leaf, hipStream_t s);

// K2 in one launch with a block per chunk of tokens (every block histograms all tokens in LDS);
// for T up to 131072 and up to 4096 leaves; same outputs, any may be null.
bool bucket_hist_ok(int64_t T, int depth);
hipError_t launch_bucket_hist(const int32_t* leaf_idx, int64_t T, int depth, int32_t* count, int32_t* offset,
                              int32_t* perm, int32_t* slot_leaf, hipStream_t s);

// K2 from per-block leaf counts (the descent's, or launch_chunk_counts' for a leaf_idx array that
// came from elsewhere): one launch of dc.blocks blocks, each sums the columns of M, scans the leaves
// and places its own share of the tokens.  Needs dc.blocks > 0.
hipError_t launch_chunk_counts(const int32_t* leaf_idx, int64_t T, int depth, DescentCounts* dc, hipStream_t s);
hipError_t launch_bucket_fold(const int32_t* leaf_idx, int64_t T, int depth, const DescentCounts& dc,
                              int32_t* count, int32_t* offset, int32_t* perm, int32_t* slot_leaf, hipStream_t s);

// K2 for many tokens over few leaves (up to 4096): segments of 1024 tokens, three launches (count, scan,
// scatter); the matrix region of the workspace must hold a column per segment (bucket_segments_ok).
bool bucket_segments_ok(int64_t T, int depth, const Workspace& ws);
hipError_t launch_bucket_segments(const int32_t* leaf_idx, int64_t T, int depth, const Workspace& ws,
                                  int32_t* count, int32_t* offset, int32_t* perm, int32_t* slot_leaf,
                                  hipStream_t s);

// K3 + K4: leaf networks and output rows.
//   order == nullptr: slot i is token i.  Otherwise slot i is token order[i].
//   split > 0 (needs order, the leaf of every slot, and gather_takes_split(p)): only the tiles of 16
//   consecutive slots with at least `split` runs of equal leaf are handled, the rest is left to
//   launch_leaf_tiles with the same value.
bool gather_takes_split(const Problem& p);
hipError_t launch_leaf_gather(const Problem& p, const int32_t* leaf_idx, const int32_t* order,
                              hipStream_t s, const int32_t* slot_leaf = nullptr, int split = 0);
// MFMA tile path over tokens grouped by leaf (perm, and the leaf of every slot); needs tiles_shape_ok(p).
// Two launches (hidden activations, output rows); `between`, if given, is called between them.
bool tiles_shape_ok(const Problem& p);
//   split > 0: tiles with at least `split` runs of equal leaf are skipped (launch_leaf_gather's).
hipError_t launch_leaf_tiles(const Problem& p, const int32_t* slot_leaf, const int32_t* perm, void* hidden,
                             hipStream_t s, void (*between)(hipStream_t) = nullptr, int split = 0);

// Whole forward pass in one launch, one block per token: the small-batch path, built for the
// latency of the dependent loads rather than for throughput; needs token_shape_ok(p).
constexpr size_t kTokenMaxLds = 144 * 1024;
constexpr int64_t kTokenMaxBlocks = 8192;
// given_leaf (optional): the leaf of every token; then only the leaf networks run (the node
// weights are not read, token_shape_ok's condition on them does not apply).
bool token_shape_ok(const Problem& p);
hipError_t launch_token_block(const Problem& p, int32_t* leaf_idx, hipStream_t s,
                              const int32_t* given_leaf = nullptr);

// Gating of a mixture of experts with one engaged expert (fff_moe_gate.hip): expert_idx[t] =
// argmax_e gate_w[e] . x[t] (+ gate_b[e]).  cand: scratch of 2 * T * moe_gate_blocks(n_experts) words.
int64_t moe_gate_blocks(int64_t n_experts);
bool moe_gate_shape_ok(const void* x, const void* gate_w, int64_t D, bool bf16);
hipError_t launch_moe_gate(const void* x, const void* gate_w, const void* gate_b, int64_t T, int64_t D,
                           int64_t n_experts, int32_t* cand, int32_t* expert_idx, hipStream_t s);

// Forward_T (fff_soft.hip): the soft mixture over all leaves on the matrix cores.  scratch holds
// soft_scratch_words(p) 32-bit words; mix [T, 2^depth] and entropy [2^depth - 1] (fp32) are optional outputs.
extern int64_t g_soft_small_tiles;
bool soft_shape_ok(const Problem& p);
int64_t soft_scratch_words(const Problem& p);
hipError_t launch_forward_soft(const Problem& p, int32_t* scratch, float* mix_out, float* entropy_out,
                               hipStream_t s);

// Forward_I with nodes of `node_size` hidden neurons on the layer-normalised token (gamma null:
// no normalisation), plus the token itself when `residual` (fff_block.hip); one launch, a wave per
// token.  p.node_w / p.node_b are not used.  vector_rows needs block_shape_ok (and 16-byte aligned
// rows of every other tensor); without it an element-wise kernel takes any shape.
struct BlockTuning {
    int64_t top = 0;      // k + 1 forces at most k LDS-staged node levels
    int64_t last_top = 0; // read-only: node levels the last fff_forward_block launch kept in LDS
};
extern BlockTuning g_block_tuning;
bool block_shape_ok(const void* x, const void* out, const void* leaf_w1, const void* leaf_w2, int64_t D,
                    int64_t O, bool bf16);
hipError_t launch_forward_block(const Problem& p, const void* gamma, const void* beta, float eps,
                                const void* node_w1, const void* node_b1, const void* node_w2,
                                const void* node_b2, int node_size, bool residual, int32_t* leaf_idx,
                                hipStream_t s, bool vector_rows = true);

// Whole forward pass in one launch, one token per lane group (any shape).
hipError_t launch_fused_generic(const Problem& p, int32_t* leaf_idx, hipStream_t s);

}  // namespace fff
