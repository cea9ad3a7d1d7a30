// C ABI of the FFF library: argument checks (host only, before any HIP call),
// per-device workspace, and the sequence of kernel launches of Forward_I
// (Algorithm 1): descent -> bucketing -> leaf networks with fused output rows.
#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <string>
#include <vector>

#include "../../include/fff.h"
#include "fff_internal.h"

// Scratch of fff_forward_hard_static, the entry point for callers that cannot allocate: a fixed
// block in the device image of this library, so every GPU the library runs on holds one copy of it
// (at an address of its own) until the process ends.  The name is a host-side stand-in: host code
// never passes it anywhere, it asks each device for the array's address once (scratch_on_device)
// and uses that pointer.
#define FFF_STATIC_SCRATCH_BYTES (16u << 20)
static __device__ __align__(256) unsigned char scratch[FFF_STATIC_SCRATCH_BYTES];

namespace fff {
namespace {

thread_local std::string g_last_error;
std::string g_last_launch;   // kernels of the last forward call (process-wide, like the "last_*" options)

// One workspace per device: the library's own block (grown on demand), or the caller's
// (fff_set_workspace), which takes precedence while it is set.
struct DeviceWs {
    void* base = nullptr;        // library-owned
    size_t bytes = 0;
    void* user_base = nullptr;   // caller-provided
    size_t user_bytes = 0;
};
constexpr int kMaxDevices = 64;
DeviceWs g_ws[kMaxDevices];
std::mutex g_mu;

struct Options {
    int64_t path = 0;            // 0 auto, 1 fused walk, 2 staged, 3 generic one-wave-per-token
    int64_t leaf_path = 0;       // 0 auto, 1 gather kernel only, 2 MFMA tiles whenever the shape allows
    int64_t bucketing = 1;       // 0: leaf kernel visits tokens in token order
    int64_t stage_timing = 0;    // 1: bracket the stages of fff_forward_hard with events
    int64_t bucket_kernel = 0;   // 0 auto, 1 leaf-range kernel, 2 chunk-matrix kernels, 3 token-chunk kernel, 4 segment kernels
    int64_t last_path = 0;       // read-only: the path the last fff_forward_hard call took
    int64_t last_leaf_path = 0;  // read-only: leaf stage of the last staged call (1 gather kernel, 2 tile kernels, 3 both)
    int64_t leaf_split = 0;      // 1..16: tiles of 16 slots with that many runs of equal leaf go to the gather kernel
    int64_t last_block_kernel = 0; // read-only: 1 = fff_forward_block ran a vector kernel, 2 = the element-wise one
    int64_t token_max_T = 512;   // batches up to this many tokens (6x where no fused launch fits) go one block per token
} g_opt;

// the vector L1 of a compute unit (not reported by the runtime)
constexpr int64_t kVectorL1Bytes = 32 * 1024;

// Events recorded around the stages of fff_forward_hard while "stage_timing" is on:
// five per call (start, after descent, after bucketing, after the leaf stage's first kernel, after
// its second; a path with fewer kernels records the later marks back to back).
std::vector<hipEvent_t> g_stage_events;

void stage_mark(hipStream_t s) {
    if (!g_opt.stage_timing) return;
    hipEvent_t e;
    if (hipEventCreate(&e) != hipSuccess) return;
    if (hipEventRecord(e, s) != hipSuccess) {
        (void)hipEventDestroy(e);
        return;
    }
    std::lock_guard<std::mutex> lock(g_mu);
    g_stage_events.push_back(e);
}

constexpr int64_t kAlignWords = 64;            // 256-byte regions
constexpr int64_t kMaxMatrixWords = 8 << 20;   // per-chunk histogram budget (32 MiB)
constexpr int64_t kCtrlWords = 64;

int64_t round_up(int64_t v, int64_t a) { return (v + a - 1) / a * a; }

struct Layout {
    int64_t n_chunks;
    int64_t o_ctrl, o_leaf, o_rank, o_sleaf, o_perm, o_count, o_offset, o_tileoff, o_matrix, o_fold, o_hidden, o_extra, total;
};

// extra_words: room for a caller-specific scratch region (the gating candidates of the mixture of experts)
Layout layout_for(int64_t T, int depth, int64_t extra_words = 0) {
    Layout l;
    const int64_t NL = (int64_t)1 << depth;
    const int64_t per_round = (T + kChunkTokens - 1) / kChunkTokens;
    int64_t c = kMaxMatrixWords / NL;
    if (c < 1) c = 1;
    if (c > per_round) c = per_round;
    if (c < 1) c = 1;
    l.n_chunks = c;
    int64_t o = 0;
    auto take = [&](int64_t words) { int64_t at = o; o += round_up(words, kAlignWords); return at; };
    l.o_ctrl = take(kCtrlWords);
    l.o_leaf = take(T);
    l.o_rank = take(T);
    l.o_sleaf = take(T);
    l.o_perm = take(T);
    l.o_count = take(NL);
    l.o_offset = take(NL + 1);
    l.o_tileoff = take(NL + 1);
    l.o_matrix = take(c * NL);
    l.o_fold = take(T > 0 && depth <= 10 ? kFoldWords : 0);   // per-block leaf counts of the descent
    l.o_hidden = take((int64_t)(kTilesMaxLeafWidth / 2) * T);   // T * L bf16 values, L up to the tile path's limit
    l.o_extra = take(extra_words);
    l.total = o;
    return l;
}

// Called once the host-side checks have passed: forgets the message of an earlier failure and
// any error another user of the HIP runtime left in this thread's last-error slot, so that the
// launch checks below report this call's errors only.
void begin_device_call() {
    g_last_error.clear();
    g_last_launch.clear();
    (void)hipGetLastError();
}

int set_device_error(hipError_t e, const char* what) {
    g_last_error = std::string(what) + ": " + hipGetErrorString(e);
    return FFF_ERR_DEVICE;
}

int current_device(int* dev) {
    hipError_t e = hipGetDevice(dev);
    if (e != hipSuccess) return set_device_error(e, "hipGetDevice");
    if (*dev < 0 || *dev >= kMaxDevices) {
        g_last_error = "device ordinal out of range";
        return FFF_ERR_DEVICE;
    }
    return FFF_OK;
}

int64_t g_fail_growths = 0;   // debug option "fail_workspace_growth": how many of the next growths fail

// Makes the current device's library-owned block at least `need` bytes (g_mu held).  Growing frees
// the old block (which waits for the device) and cannot be done while `s` is being captured.
int grow_owned(DeviceWs& d, size_t need, hipStream_t s, bool check_capture) {
    if (d.bytes >= need) return FFF_OK;
    if (check_capture) {
        hipStreamCaptureStatus st = hipStreamCaptureStatusNone;
        if (hipStreamIsCapturing(s, &st) != hipSuccess) (void)hipGetLastError();
        if (st != hipStreamCaptureStatusNone) {
            g_last_error = "workspace must grow to " + std::to_string(need) +
                           " bytes, which cannot happen during stream capture: reserve or set it first";
            return FFF_ERR_WORKSPACE;
        }
    }
    hipError_t e;
    if (d.base) {
        e = hipFree(d.base);   // waits for work that may still use it
        d.base = nullptr;
        d.bytes = 0;
        if (e != hipSuccess) return set_device_error(e, "hipFree(workspace)");
    }
    void* p = nullptr;
    if (g_fail_growths > 0) {          // test hook: this growth fails the way an exhausted device would
        --g_fail_growths;
        e = hipErrorOutOfMemory;
    } else {
        e = hipMalloc(&p, need);
    }
    if (e != hipSuccess) {
        (void)hipGetLastError();
        g_last_error = std::string("hipMalloc(workspace): ") + hipGetErrorString(e);
        return FFF_ERR_WORKSPACE;
    }
    e = hipMemset(p, 0, kCtrlWords * sizeof(int32_t));   // ticket counters start at zero
    if (e != hipSuccess) {
        (void)hipFree(p);
        return set_device_error(e, "hipMemset(workspace)");
    }
    d.base = p;
    d.bytes = need;
    return FFF_OK;
}

void carve(void* base, const Layout& lay, Workspace* ws) {
    int32_t* b = (int32_t*)base;
    ws->ctrl = b + lay.o_ctrl;
    ws->leaf_idx = b + lay.o_leaf;
    ws->rank = b + lay.o_rank;
    ws->slot_leaf = b + lay.o_sleaf;
    ws->perm = b + lay.o_perm;
    ws->count = b + lay.o_count;
    ws->offset = b + lay.o_offset;
    ws->tile_off = b + lay.o_tileoff;
    ws->chunk_cnt = b + lay.o_matrix;
    ws->fold = b + lay.o_fold;
    ws->hidden = b + lay.o_hidden;
    ws->extra = b + lay.o_extra;
    ws->n_chunks = lay.n_chunks;
}

// The current device's workspace carved for (T, depth): the caller's if one is set (too small is
// an error, nothing is allocated), else the library's own, grown if needed.
int get_workspace(int64_t T, int depth, Workspace* ws, Layout* lay, hipStream_t s, int64_t extra_words = 0) {
    *lay = layout_for(T, depth, extra_words);
    const size_t need = (size_t)lay->total * sizeof(int32_t);
    int dev = 0;
    int rc = current_device(&dev);
    if (rc != FFF_OK) return rc;
    std::lock_guard<std::mutex> lock(g_mu);
    DeviceWs& d = g_ws[dev];
    if (d.user_base) {
        if (d.user_bytes < need) {
            g_last_error = "the caller's workspace holds " + std::to_string(d.user_bytes) + " bytes, this call needs " +
                           std::to_string(need);
            return FFF_ERR_WORKSPACE;
        }
        carve(d.user_base, *lay, ws);
        return FFF_OK;
    }
    if ((rc = grow_owned(d, need, s, true)) != FFF_OK) return rc;
    carve(d.base, *lay, ws);
    return FFF_OK;
}

constexpr int64_t kMaxElems = (int64_t)1 << 40;
constexpr int64_t kMaxTokens = ((int64_t)1 << 31) - 1024;
constexpr int kMaxLeafWidth = 4096;

int check_common(int depth, int64_t T, int64_t D, int dtype) {
    if (dtype != FFF_F32 && dtype != FFF_BF16) return FFF_ERR_DTYPE;
    if (depth < 0 || depth > FFF_MAX_DEPTH) return FFF_ERR_RANGE;
    if (T < 0 || T > kMaxTokens) return FFF_ERR_RANGE;
    if (D < 1 || D > kMaxElems) return FFF_ERR_SHAPE;
    if (T * D > kMaxElems || ((int64_t)1 << depth) * D > kMaxElems) return FFF_ERR_SHAPE;
    return FFF_OK;
}

int check_leaf(int depth, int leaf_width, int act, int64_t T, int64_t D, int64_t O) {
    if (leaf_width < 1 || leaf_width > kMaxLeafWidth) return FFF_ERR_RANGE;
    if (O < 1 || O > kMaxElems) return FFF_ERR_SHAPE;
    const int64_t m = D > O ? D : O;
    if (T * O > kMaxElems || ((int64_t)1 << depth) * leaf_width > kMaxElems / m) return FFF_ERR_SHAPE;
    if (act != FFF_ACT_RELU && act != FFF_ACT_GELU) return FFF_ERR_UNSUPPORTED;
    return FFF_OK;
}

bool overlaps(const void* a, int64_t abytes, const void* b, int64_t bbytes) {
    const uintptr_t a0 = (uintptr_t)a, b0 = (uintptr_t)b;
    return a0 < b0 + (uintptr_t)bbytes && b0 < a0 + (uintptr_t)abytes;
}

// Shapes the staged path's 16-byte vector kernels take.
bool staged_shape_ok(const Problem& p) {
    return walk_shape_ok(p) && vec_ok(p.leaf_w1, p.D, p.bf16) && p.L <= 64;
}

enum { kPathAuto = 0, kPathFused = 1, kPathStaged = 2, kPathGeneric = 3, kPathToken = 4, kPathSplit = 5 };

// One launch that keeps the token row in registers from the root to the output
// row wins while a leaf is narrow (its weights are a few rows per token, like a
// few more tree levels); wider leaves want tokens grouped so that a leaf's
// weights are read once per group.
int choose_path(const Problem& p) {
    const bool fused_ok = fused_shape_ok(p), staged_ok = staged_shape_ok(p), token_ok = token_shape_ok(p);
    const bool split_ok = fused_ok && slices_shape_ok(p);
    if (g_opt.path == kPathToken && token_ok) return kPathToken;
    if (g_opt.path == kPathSplit && split_ok) return kPathSplit;
    if (g_opt.path == kPathFused && fused_ok) return kPathFused;
    if (g_opt.path == kPathStaged && staged_ok) return kPathStaged;
    if (g_opt.path == kPathGeneric) return kPathGeneric;
    // a small batch cannot fill the chip with streaming work: one block per token, built for latency
    // (measured crossovers on 768-wide rows: the fused launch, with its smallest tiles, takes 9-12 us
    // from 256 to 2048 tokens, this one 9 us up to 512 tokens and 13-16 at 1024; leaves too wide for
    // the fused launch leave only the staged path, which overtakes between 2048 and 4096 tokens)
    if (g_opt.path == kPathAuto && token_ok &&
        p.T <= (fused_ok ? g_opt.token_max_T : 6 * g_opt.token_max_T))
        return kPathToken;
    if (!fused_ok && !staged_ok) return token_ok ? kPathToken : kPathGeneric;
    // The fused launch gathers, per token, the leaf's output-weight and bias rows from a table of
    // 2^depth (leaf_width + 1) rows.  Once that table outgrows the L2 of an XCD most of those rows
    // come back from memory; the launch cut in two (walk and hidden neurons per token, then the
    // output rows by column slices, one slice of all rows per XCD) keeps each slice in its L2.
    // Measured on 768-wide rows, 65536 tokens, one neuron a leaf: depth 11 (6 MB of output rows)
    // 80 -> 70 us, depth 12 93 -> 82, depth 13 106 -> 101; two neurons, depth 11: 99 -> 86;
    // 4096-wide rows, 16384 tokens, depth 10: 140 -> 108.  With one neuron a leaf and a full batch
    // (256 tokens per compute unit and more) it is ahead for smaller tables too (depth 8: 57 -> 53),
    // since the walk then runs in the descent's leaner tile shape.  Rows shorter than 1 KB and
    // batches of up to 32 tokens per compute unit stay on the single launch (two launches cost
    // more than they save: 16384 tokens, depth 10: 20.6 against 21.4 us).
    const auto fused_or_split = [&]() {
        if (!split_ok || g_opt.path == kPathFused) return (int)kPathFused;
        const DeviceInfo di = device_info();
        const int64_t es = p.bf16 ? 2 : 4;
        const int64_t out_table = ((int64_t)(p.L + 1) * p.O * es) << p.depth;
        const bool full_rows = p.O * es >= 1024 && p.D * es >= 1024;
        const bool big_batch = p.T > 32 * (int64_t)di.cus;
        // (from 128 tokens per compute unit on, three quarters of an L2 are enough: 100000 tokens, 512-wide
        // rows, two neurons, depth 10 -- 3.1 MB of output rows -- 94 us fused, 78 split)
        const int64_t table_min = p.T >= 128 * (int64_t)di.cus ? di.l2_bytes * 3 / 4 : di.l2_bytes;
        const bool split = full_rows && big_batch &&
                           out_table <= 64 * di.l2_bytes &&     // beyond that no slice of it stays in an L2 either
                           (out_table >= table_min || (p.L == 1 && p.T >= 256 * (int64_t)di.cus));
        return split ? (int)kPathSplit : (int)kPathFused;
    };
    if (!staged_ok) return fused_or_split();
    if (!fused_ok) return kPathStaged;
    // one or two neurons a leaf are "three more tree levels" whatever the row length: never worth
    // the passes of the staged path (9000 tokens, 3072 inputs, 768 outputs, two neurons, depth 9:
    // 71 us staged, 62 fused, 55 split; 768-wide rows, two neurons, depth 13: 133 / 132 / 128)
    if (p.L <= 2) return fused_or_split();
    // Grouping pays once the leaf rows a token meets are many bytes -- 24 KB (8 neurons on 768-wide
    // bf16 rows), or 12 KB (4 neurons) where the leaf weights together (8 MB) outgrow the 4 MB L2 of one XCD,
    // which the fused launch relies on for its per-token row fetches, or 8 KB (3 neurons) from 16 MB
    // on (measured on 768-wide rows: depth 8 ties at 6 neurons, depth 10 at 4, depth 4 only at 8;
    // 128-wide rows stay on the fused launch at 8 neurons, 256-wide ones leave it at depth 12) --
    // and a leaf is visited by a few tokens on average: in bucket order the tokens of a leaf find
    // its rows in cache, so the staged path stays ahead down to 3 tokens a leaf (50432 tokens,
    // 768-wide rows, 8 neurons, depth 13 and 14: 151 and 218 us against 224 and 260 fused; 16384
    // tokens, 4096-wide rows, 4 neurons, depth 12: 233 against 285); below that (the skewed workload:
    // half a token a leaf) the single launch wins again.  Up to 8192 tokens the fused launch, cut
    // into tiles of 32 tokens, is ahead for every leaf it takes (2048-8192 tokens, 8 neurons, depth
    // 9: 17-22 us against 25-31 staged; 16384 tokens: 42 against 34).
    // In the device's own units: a token's leaf rows against the vector L1 of a compute unit
    // (3/4, 3/8, 1/4 of its 32 KB), all leaf weights against the L2 of one XCD (2x, 4x its 4 MB),
    // the batch against 32 tokens per compute unit.
    const DeviceInfo di = device_info();
    const int64_t es = p.bf16 ? 2 : 4;
    const int64_t token_leaf_bytes = (p.L * (p.D + p.O) + p.O) * es;
    const int64_t leaf_bytes = token_leaf_bytes << p.depth;
    const bool wide = token_leaf_bytes * 4 >= 3 * kVectorL1Bytes ||
                      (token_leaf_bytes * 8 >= 3 * kVectorL1Bytes && leaf_bytes >= 2 * di.l2_bytes) ||
                      (token_leaf_bytes * 4 >= kVectorL1Bytes && leaf_bytes >= 4 * di.l2_bytes);
    const bool visited = p.T > 32 * (int64_t)di.cus && p.depth < 40 && p.T >= ((int64_t)3 << p.depth);
    return (wide && visited) ? (int)kPathStaged : fused_or_split();
}

// K2 with whichever kernel set takes the sizes; outputs may be null (then workspace arrays are used).
// dc (optional): per-block leaf counts the descent left behind; then one fold launch finishes the job.
int run_bucket(const int32_t* leaf_idx, int64_t T, int depth, const Workspace& ws, int32_t* count,
               int32_t* offset, int32_t* perm, int32_t* slot_leaf, hipStream_t s, const DescentCounts* dc = nullptr) {
    hipError_t e;
    if (dc && dc->blocks > 0 && (g_opt.bucket_kernel == 0 || g_opt.bucket_kernel == 5)) {
        e = launch_bucket_fold(leaf_idx, T, depth, *dc, count, offset, perm, slot_leaf, s);
        return e == hipSuccess ? FFF_OK : set_device_error(e, "bucket kernel launch");
    }
    if (g_opt.bucket_kernel == 5 && T > 0 && depth <= 10) {   // the same kernel fed by a counting launch of its own
        DescentCounts own;
        own.M = ws.fold;
        own.capacity = kFoldWords;
        if ((e = launch_chunk_counts(leaf_idx, T, depth, &own, s)) != hipSuccess)
            return set_device_error(e, "bucket kernel launch");
        if (own.blocks > 0) {
            e = launch_bucket_fold(leaf_idx, T, depth, own, count, offset, perm, slot_leaf, s);
            return e == hipSuccess ? FFF_OK : set_device_error(e, "bucket kernel launch");
        }
    }
    if ((g_opt.bucket_kernel == 0 || g_opt.bucket_kernel == 3) && bucket_hist_ok(T, depth)) {
        e = launch_bucket_hist(leaf_idx, T, depth, count, offset, perm, slot_leaf, s);
        return e == hipSuccess ? FFF_OK : set_device_error(e, "bucket kernel launch");
    }
    // beyond the token-chunk kernel's sizes: the leaf-range kernel reads leaf_idx once per block of
    // leaves, which pays for many leaves; for few leaves (up to 4096) and many tokens the segment
    // kernels (count / scan / scatter over segments of 1024 tokens) are faster, and so are the
    // chunk-matrix kernels (806912 tokens over 256 leaves: 102 against 224 us; 201728: 47 against 72 us)
    const bool few_leaves = g_opt.bucket_kernel == 0 && depth <= 12;
    if ((few_leaves || g_opt.bucket_kernel == 4) && bucket_segments_ok(T, depth, ws)) {
        e = launch_bucket_segments(leaf_idx, T, depth, ws, count, offset, perm, slot_leaf, s);
        return e == hipSuccess ? FFF_OK : set_device_error(e, "bucket kernel launch");
    }
    if (g_opt.bucket_kernel != 2 && !few_leaves && bucket_onepass_ok(T, depth)) {
        e = launch_bucket_onepass(leaf_idx, T, depth, count, offset, perm, slot_leaf, s);
        return e == hipSuccess ? FFF_OK : set_device_error(e, "bucket kernel launch");
    }
    const int64_t NL = (int64_t)1 << depth;
    if ((e = launch_zero(ws.chunk_cnt, round_up(ws.n_chunks * NL, 4), s)) != hipSuccess)
        return set_device_error(e, "zero kernel launch");
    if ((e = launch_bucket(leaf_idx, T, depth, ws, count, offset, perm, slot_leaf, s)) != hipSuccess)
        return set_device_error(e, "bucket kernel launch");
    return FFF_OK;
}

int run_leaf_stage(const Problem& p, const int32_t* leaf_idx, const Workspace& ws, hipStream_t s,
                   bool timed = false, const DescentCounts* dc = nullptr) {
    hipError_t e;
    if (!g_opt.bucketing) {
        if (timed) stage_mark(s);
        g_opt.last_leaf_path = 1;
        e = launch_leaf_gather(p, leaf_idx, nullptr, s);
        if (timed) stage_mark(s);
        if (timed) stage_mark(s);
        return e == hipSuccess ? FFF_OK : set_device_error(e, "leaf kernel launch");
    }
    const int rc = run_bucket(leaf_idx, p.T, p.depth, ws, nullptr, nullptr, ws.perm, ws.slot_leaf, s, dc);
    if (rc != FFF_OK) return rc;
    if (timed) stage_mark(s);
    // the MFMA tile path pays once a leaf has a few neurons (for 1-2 the VALU gather kernel is leaner)
    // and a tile of 16 slots holds few different leaves: from 8 tokens a leaf on average (measured
    // on 768-wide rows, 50432 tokens, 8 neurons: 12 tokens a leaf 118 us tiles against 128 gather,
    // 6 tokens a leaf 168 against 151; leaves of more than 8 neurons always, the gather kernel
    // needs twice the time there); up to 8192 tokens only from 32 tokens a leaf (4096 tokens, 8
    // neurons, 8 tokens a leaf: 40 us against 32)
    const int64_t per_leaf = p.depth < 40 ? p.T >> p.depth : 0;
    const bool filled = (p.T > 32 * (int64_t)device_info().cus && (p.L > 8 || per_leaf >= 8)) || per_leaf >= 32;
    const bool tiles = g_opt.leaf_path != 1 && tiles_shape_ok(p) &&
                       (g_opt.leaf_path == 2 || (p.L >= 3 && filled));
    // On request ("leaf_split"), tiles whose 16 slots hold that many different leaves or more are
    // left to the gather kernel, one lane group per token, and the tile kernels keep the tiles of
    // well-filled buckets.  Not the default: on every shape measured one of the two kernels alone
    // was at least as fast as the pair.
    const int split = tiles && gather_takes_split(p) && g_opt.leaf_split >= 1 && g_opt.leaf_split <= 16
                          ? (int)g_opt.leaf_split : 0;
    g_opt.last_leaf_path = tiles ? (split ? 3 : 2) : 1;
    if (tiles) {
        e = launch_leaf_tiles(p, ws.slot_leaf, ws.perm, ws.hidden, s, timed ? stage_mark : nullptr, split);
        if (e == hipSuccess && split) e = launch_leaf_gather(p, leaf_idx, ws.perm, s, ws.slot_leaf, split);
    } else {
        e = launch_leaf_gather(p, leaf_idx, ws.perm, s);
        if (timed) stage_mark(s);
    }
    if (e != hipSuccess) return set_device_error(e, "leaf kernel launch");
    if (timed) stage_mark(s);
    return FFF_OK;
}

// The leaf networks at given leaves: small batches go one block per token, larger ones are bucketed.
int run_leaf_any(const Problem& p, const int32_t* leaf_idx, hipStream_t s) {
    if (g_opt.path != kPathStaged && token_shape_ok(p) && p.T <= 6 * g_opt.token_max_T) {
        hipError_t e = launch_token_block(p, nullptr, s, leaf_idx);
        return e == hipSuccess ? FFF_OK : set_device_error(e, "token-block kernel launch");
    }
    Workspace ws;
    Layout lay;
    const int rc = get_workspace(p.T, p.depth, &ws, &lay, s);
    if (rc != FFF_OK) return rc;
    return run_leaf_stage(p, leaf_idx, ws, s);   // falls back per shape inside
}

// Host-side argument checks of fff_forward_hard (no HIP call).  FFF_OK with *empty set: nothing to do.
int check_forward_hard(const void* x, const void* node_w, const void* node_b, const void* leaf_w1,
                       const void* leaf_b1, const void* leaf_w2, const void* leaf_b2, int depth, int leaf_width,
                       int act, const void* out, int64_t T, int64_t D, int64_t O, int dtype, bool* empty) {
    *empty = false;
    int rc = check_common(depth, T, D, dtype);
    if (rc == FFF_OK) rc = check_leaf(depth, leaf_width, act, T, D, O);
    if (rc != FFF_OK) return rc;
    if (T == 0) {
        *empty = true;
        return FFF_OK;
    }
    if (!x || !leaf_w1 || !leaf_b1 || !leaf_w2 || !leaf_b2 || !out) return FFF_ERR_NULL;
    if (depth > 0 && (!node_w || !node_b)) return FFF_ERR_NULL;
    const int64_t es = dtype == FFF_BF16 ? 2 : 4;
    if (overlaps(x, T * D * es, out, T * O * es)) return FFF_ERR_ALIAS;
    return FFF_OK;
}

// The address of `scratch` on the current device, asked for once per device with that device
// current (each device has its own copy of the array).
void* g_scratch_ptr[kMaxDevices];

int scratch_on_device(void** ptr) {
    int dev = 0;
    const int rc = current_device(&dev);
    if (rc != FFF_OK) return rc;
    std::lock_guard<std::mutex> lock(g_mu);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) return set_device_error(e, "hipGetSymbolAddress(scratch)");
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    return FFF_OK;
}

// The launches of Forward_I.  fixed_scratch == nullptr: the staged path works in the device's
// workspace and the stages are bracketed by events when "stage_timing" is on.  Otherwise that block
// of device memory (large enough for layout_for(T, depth): the caller has checked) is carved
// instead, its control words are cleared by a kernel first, and no event is created.
int run_forward_hard(const Problem& p, int32_t* leaf_idx, hipStream_t s, void* fixed_scratch) {
    const bool marks = fixed_scratch == nullptr;
    const int path = choose_path(p);
    g_opt.last_path = path;
    if (path == kPathGeneric) {
        hipError_t e = launch_fused_generic(p, leaf_idx, s);
        return e == hipSuccess ? FFF_OK : set_device_error(e, "generic kernel launch");
    }
    if (path == kPathToken) {
        if (marks) stage_mark(s);
        hipError_t e = launch_token_block(p, leaf_idx, s);
        for (int k = 0; marks && k < 4; ++k) stage_mark(s);
        return e == hipSuccess ? FFF_OK : set_device_error(e, "token-block kernel launch");
    }
    if (path == kPathFused) {
        if (marks) stage_mark(s);
        hipError_t e = launch_walk_fused(p, leaf_idx, s);
        for (int k = 0; marks && k < 4; ++k) stage_mark(s);
        return e == hipSuccess ? FFF_OK : set_device_error(e, "fused walk kernel launch");
    }
    Workspace ws;
    Layout lay;
    hipError_t e;
    if (fixed_scratch) {
        lay = layout_for(p.T, p.depth);
        carve(fixed_scratch, lay, &ws);
        if (path == kPathStaged && (e = launch_zero(ws.ctrl, kCtrlWords, s)) != hipSuccess)
            return set_device_error(e, "zero kernel launch");
    } else {
        const int rc = get_workspace(p.T, p.depth, &ws, &lay, s);
        if (rc != FFF_OK) return rc;
    }
    int32_t* li = leaf_idx ? leaf_idx : ws.leaf_idx;
    if (path == kPathSplit) {
        // walk and hidden neurons per token, then the output rows by column slices; the hidden
        // activations (fp32, at most 8 a token) use the workspace's hidden-activation region
        float* hid = (float*)ws.hidden;
        if (marks) stage_mark(s);
        if ((e = launch_walk_hidden(p, li, hid, s)) != hipSuccess) return set_device_error(e, "walk kernel launch");
        for (int k = 0; marks && k < 2; ++k) stage_mark(s);
        if ((e = launch_leaf_slices(p, li, hid, s)) != hipSuccess) return set_device_error(e, "slice kernel launch");
        for (int k = 0; marks && k < 2; ++k) stage_mark(s);
        return FFF_OK;
    }
    // the descent leaves per-block leaf counts for the bucketing stage where the sizes allow it
    DescentCounts dc;
    const bool fold = g_opt.bucketing && p.depth <= 10 && (g_opt.bucket_kernel == 0 || g_opt.bucket_kernel == 5);
    dc.M = fold ? ws.fold : nullptr;
    dc.capacity = kFoldWords;
    if (marks) stage_mark(s);
    e = launch_descend(p, li, s, &dc);
    if (e != hipSuccess) return set_device_error(e, "descent kernel launch");
    if (marks) stage_mark(s);
    return run_leaf_stage(p, li, ws, s, marks, &dc);
}

}  // namespace

void note_launch(const char* fmt, ...) {
    char buf[256];
    va_list ap;
    va_start(ap, fmt);
    std::vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    if (!g_last_launch.empty()) g_last_launch += " + ";
    g_last_launch += buf;
}

}  // namespace fff

using namespace fff;

extern "C" {

int fff_forward_hard(const void* x, const void* node_w, const void* node_b, const void* leaf_w1,
                     const void* leaf_b1, const void* leaf_w2, const void* leaf_b2, int depth,
                     int leaf_width, int act, void* out, int32_t* leaf_idx, void* stream, int64_t T,
                     int64_t D, int64_t O, int dtype) {
    bool empty = false;
    const int rc = check_forward_hard(x, node_w, node_b, leaf_w1, leaf_b1, leaf_w2, leaf_b2, depth, leaf_width, act,
                                      out, T, D, O, dtype, &empty);
    if (rc != FFF_OK || empty) return rc;
    Problem p{x, node_w, node_b, leaf_w1, leaf_b1, leaf_w2, leaf_b2, out, leaf_idx,
              T, D, O, depth, leaf_width, act, dtype == FFF_BF16};
    begin_device_call();
    return run_forward_hard(p, leaf_idx, (hipStream_t)stream, nullptr);
}

int fff_forward_hard_static(const void* x, const void* node_w, const void* node_b, const void* leaf_w1,
                            const void* leaf_b1, const void* leaf_w2, const void* leaf_b2, int depth,
                            int leaf_width, int act, void* out, int32_t* leaf_idx, void* stream, int64_t T,
                            int64_t D, int64_t O, int dtype) {
    bool empty = false;
    const int rc = check_forward_hard(x, node_w, node_b, leaf_w1, leaf_b1, leaf_w2, leaf_b2, depth, leaf_width, act,
                                      out, T, D, O, dtype, &empty);
    if (rc != FFF_OK || empty) return rc;
    const size_t need = (size_t)layout_for(T, depth).total * sizeof(int32_t);
    if (need > FFF_STATIC_SCRATCH_BYTES) {
        g_last_error = "fff_forward_hard_static: T = " + std::to_string(T) + ", depth = " + std::to_string(depth) +
                       " need " + std::to_string(need) + " bytes of scratch, the static array holds " +
                       std::to_string((size_t)FFF_STATIC_SCRATCH_BYTES);
        return FFF_ERR_WORKSPACE;
    }
    Problem p{x, node_w, node_b, leaf_w1, leaf_b1, leaf_w2, leaf_b2, out, leaf_idx,
              T, D, O, depth, leaf_width, act, dtype == FFF_BF16};
    begin_device_call();
    void* ptr = nullptr;
    const int rs = scratch_on_device(&ptr);
    if (rs != FFF_OK) return rs;
    return run_forward_hard(p, leaf_idx, (hipStream_t)stream, ptr);
}

size_t fff_static_scratch_bytes(void) { return FFF_STATIC_SCRATCH_BYTES; }

int fff_descend(const void* x, const void* node_w, const void* node_b, int depth, int32_t* leaf_idx,
                void* stream, int64_t T, int64_t D, int dtype) {
    int rc = check_common(depth, T, D, dtype);
    if (rc != FFF_OK) return rc;
    if (T == 0) return FFF_OK;
    if (!x || !leaf_idx) return FFF_ERR_NULL;
    if (depth > 0 && (!node_w || !node_b)) return FFF_ERR_NULL;
    Problem p{x, node_w, node_b, nullptr, nullptr, nullptr, nullptr, nullptr, leaf_idx,
              T, D, 1, depth, 1, 0, dtype == FFF_BF16};
    begin_device_call();
    hipError_t e = launch_descend(p, leaf_idx, (hipStream_t)stream);
    return e == hipSuccess ? FFF_OK : set_device_error(e, "descent kernel launch");
}

int fff_bucket(const int32_t* leaf_idx, int64_t T, int depth, int32_t* count, int32_t* offset,
               int32_t* perm, void* stream) {
    if (depth < 0 || depth > FFF_MAX_DEPTH || T < 0 || T > kMaxTokens) return FFF_ERR_RANGE;
    if (T > 0 && !leaf_idx) return FFF_ERR_NULL;
    begin_device_call();
    Workspace ws;
    Layout lay;
    int rc = get_workspace(T, depth, &ws, &lay, (hipStream_t)stream);
    if (rc != FFF_OK) return rc;
    return run_bucket(leaf_idx, T, depth, ws, count, offset, perm, nullptr, (hipStream_t)stream);
}

int fff_leaf_forward(const void* x, const void* leaf_w1, const void* leaf_b1, const void* leaf_w2,
                     const void* leaf_b2, const int32_t* leaf_idx, int depth, int leaf_width, int act,
                     void* out, void* stream, int64_t T, int64_t D, int64_t O, int dtype) {
    int rc = check_common(depth, T, D, dtype);
    if (rc == FFF_OK) rc = check_leaf(depth, leaf_width, act, T, D, O);
    if (rc != FFF_OK) return rc;
    if (T == 0) return FFF_OK;
    if (!x || !leaf_w1 || !leaf_b1 || !leaf_w2 || !leaf_b2 || !out || !leaf_idx) return FFF_ERR_NULL;
    const int64_t es = dtype == FFF_BF16 ? 2 : 4;
    if (overlaps(x, T * D * es, out, T * O * es)) return FFF_ERR_ALIAS;
    Problem p{x, nullptr, nullptr, leaf_w1, leaf_b1, leaf_w2, leaf_b2, out, nullptr,
              T, D, O, depth, leaf_width, act, dtype == FFF_BF16};
    begin_device_call();
    return run_leaf_any(p, leaf_idx, (hipStream_t)stream);
}

int fff_moe_top1_forward(const void* x, const void* gate_w, const void* gate_b, const void* leaf_w1,
                         const void* leaf_b1, const void* leaf_w2, const void* leaf_b2, int log2_experts,
                         int leaf_width, int act, void* out, int32_t* expert_idx, void* stream, int64_t T,
                         int64_t D, int64_t O, int dtype) {
    int rc = check_common(log2_experts, T, D, dtype);
    if (rc == FFF_OK) rc = check_leaf(log2_experts, leaf_width, act, T, D, O);
    if (rc != FFF_OK) return rc;
    if (T == 0) return FFF_OK;
    if (!x || !gate_w || !leaf_w1 || !leaf_b1 || !leaf_w2 || !leaf_b2 || !out) return FFF_ERR_NULL;
    const int64_t es = dtype == FFF_BF16 ? 2 : 4;
    if (overlaps(x, T * D * es, out, T * O * es)) return FFF_ERR_ALIAS;
    if (!moe_gate_shape_ok(x, gate_w, D, dtype == FFF_BF16)) return FFF_ERR_UNSUPPORTED;
    const int64_t G = (int64_t)1 << log2_experts;
    Problem p{x, nullptr, nullptr, leaf_w1, leaf_b1, leaf_w2, leaf_b2, out, nullptr,
              T, D, O, log2_experts, leaf_width, act, dtype == FFF_BF16};
    begin_device_call();
    hipStream_t s = (hipStream_t)stream;
    Workspace ws;
    Layout lay;
    if ((rc = get_workspace(T, log2_experts, &ws, &lay, s, 2 * T * moe_gate_blocks(G))) != FFF_OK) return rc;
    int32_t* ei = expert_idx ? expert_idx : ws.leaf_idx;
    stage_mark(s);
    hipError_t e = launch_moe_gate(x, gate_w, gate_b, T, D, G, ws.extra, ei, s);
    if (e != hipSuccess) return set_device_error(e, "gating kernel launch");
    stage_mark(s);
    // the experts are leaves: small batches one block per token, larger ones bucketed
    if (g_opt.path != kPathStaged && token_shape_ok(p) && T <= 6 * g_opt.token_max_T) {
        g_opt.last_path = kPathToken;
        e = launch_token_block(p, nullptr, s, ei);
        for (int k = 0; k < 3; ++k) stage_mark(s);
        return e == hipSuccess ? FFF_OK : set_device_error(e, "token-block kernel launch");
    }
    g_opt.last_path = kPathStaged;
    return run_leaf_stage(p, ei, ws, s, true);
}

int fff_forward_soft(const void* x, const void* node_w, const void* node_b, const void* leaf_w1,
                     const void* leaf_b1, const void* leaf_w2, const void* leaf_b2, int depth, int leaf_width,
                     int act, void* out, float* mix, float* entropy, void* stream, int64_t T, int64_t D,
                     int64_t O, int dtype) {
    int rc = check_common(depth, T, D, dtype);
    if (rc == FFF_OK) rc = check_leaf(depth, leaf_width, act, T, D, O);
    if (rc != FFF_OK) return rc;
    if (T == 0) return FFF_OK;
    if (!x || !leaf_w1 || !leaf_b1 || !leaf_w2 || !leaf_b2 || !out) return FFF_ERR_NULL;
    if (depth > 0 && (!node_w || !node_b)) return FFF_ERR_NULL;
    const int64_t es = dtype == FFF_BF16 ? 2 : 4;
    if (overlaps(x, T * D * es, out, T * O * es)) return FFF_ERR_ALIAS;
    Problem p{x, node_w, node_b, leaf_w1, leaf_b1, leaf_w2, leaf_b2, out, nullptr,
              T, D, O, depth, leaf_width, act, dtype == FFF_BF16};
    if (!soft_shape_ok(p)) return FFF_ERR_UNSUPPORTED;
    // every token meets every leaf: the intermediate matrices are T x 2^depth x (leaf_width + 1) wide
    const int64_t words = soft_scratch_words(p);
    if (words > kMaxElems / 4) return FFF_ERR_SHAPE;
    begin_device_call();
    Workspace ws;
    Layout lay;
    if ((rc = get_workspace(0, 0, &ws, &lay, (hipStream_t)stream, words)) != FFF_OK) return rc;
    hipError_t e = launch_forward_soft(p, ws.extra, mix, entropy, (hipStream_t)stream);
    return e == hipSuccess ? FFF_OK : set_device_error(e, "soft forward kernel launch");
}

int fff_forward_block(const void* x, const void* ln_gamma, const void* ln_beta, float ln_eps,
                      const void* node_w1, const void* node_b1, const void* node_w2, const void* node_b2,
                      const void* leaf_w1, const void* leaf_b1, const void* leaf_w2, const void* leaf_b2,
                      int depth, int node_size, int leaf_width, int act, int residual, void* out,
                      int32_t* leaf_idx, void* stream, int64_t T, int64_t D, int64_t O, int dtype) {
    int rc = check_common(depth, T, D, dtype);
    if (rc == FFF_OK) rc = check_leaf(depth, leaf_width, act, T, D, O);
    if (rc != FFF_OK) return rc;
    if (node_size < 1 || node_size > kMaxLeafWidth) return FFF_ERR_RANGE;
    if ((((int64_t)1 << depth) - 1) * node_size > kMaxElems / D) return FFF_ERR_SHAPE;
    if (residual && O != D) return FFF_ERR_SHAPE;
    if ((ln_gamma != nullptr) != (ln_beta != nullptr)) return FFF_ERR_NULL;
    if (ln_gamma && !(ln_eps >= 0.0f)) return FFF_ERR_RANGE;
    if (T == 0) return FFF_OK;
    if (!x || !leaf_w1 || !leaf_b1 || !leaf_w2 || !leaf_b2 || !out) return FFF_ERR_NULL;
    if (depth > 0 && (!node_w1 || !node_b1 || !node_w2 || !node_b2)) return FFF_ERR_NULL;
    const int64_t es = dtype == FFF_BF16 ? 2 : 4;
    // in place (out == x with rows of one width) is fine: a wave reads its token before it writes it
    if (!(out == x && O == D) && overlaps(x, T * D * es, out, T * O * es)) return FFF_ERR_ALIAS;
    if (leaf_idx && overlaps(leaf_idx, T * 4, out, T * O * es)) return FFF_ERR_ALIAS;
    Problem p{x, nullptr, nullptr, leaf_w1, leaf_b1, leaf_w2, leaf_b2, out, leaf_idx,
              T, D, O, depth, leaf_width, act, dtype == FFF_BF16};
    // rows of whole 16-byte pieces, short enough for a lane group or a wave to hold, take the vector
    // kernels; everything else the element-wise one
    const bool vector_rows = block_shape_ok(x, out, leaf_w1, leaf_w2, D, O, p.bf16) &&
                             (depth == 0 || vec_ok(node_w1, D, p.bf16)) &&
                             (!ln_gamma || (vec_ok(ln_gamma, D, p.bf16) && vec_ok(ln_beta, D, p.bf16))) &&
                             vec_ok(leaf_b2, O, p.bf16);
    begin_device_call();
    g_opt.last_block_kernel = vector_rows ? 1 : 2;
    hipError_t e = launch_forward_block(p, ln_gamma, ln_beta, ln_eps, node_w1, node_b1, node_w2, node_b2,
                                        node_size, residual != 0, leaf_idx, (hipStream_t)stream, vector_rows);
    return e == hipSuccess ? FFF_OK : set_device_error(e, "block kernel launch");
}

size_t fff_workspace_bytes(int64_t T, int depth) {
    if (T < 0 || T > kMaxTokens || depth < 0 || depth > FFF_MAX_DEPTH) return 0;
    return (size_t)layout_for(T, depth).total * sizeof(int32_t);
}

size_t fff_workspace_bytes_moe(int64_t T, int log2_experts) {
    if (T < 0 || T > kMaxTokens || log2_experts < 0 || log2_experts > FFF_MAX_DEPTH) return 0;
    const int64_t G = (int64_t)1 << log2_experts;
    return (size_t)layout_for(T, log2_experts, 2 * T * moe_gate_blocks(G)).total * sizeof(int32_t);
}

size_t fff_workspace_bytes_soft(int64_t T, int64_t O, int depth, int leaf_width) {
    if (T < 0 || T > kMaxTokens || depth < 0 || depth > FFF_MAX_DEPTH || O < 1 || O > kMaxElems ||
        leaf_width < 1 || leaf_width > kMaxLeafWidth)
        return 0;
    Problem p{nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr,
              T, 8, O, depth, leaf_width, 0, true};
    const int64_t words = soft_scratch_words(p);
    if (words > kMaxElems / 4) return 0;
    return (size_t)layout_for(0, 0, words).total * sizeof(int32_t);
}

int fff_set_workspace(void* dev_ptr, size_t bytes, void* stream) {
    if (dev_ptr && ((reinterpret_cast<uintptr_t>(dev_ptr) & 255u) != 0 || bytes < kCtrlWords * sizeof(int32_t)))
        return FFF_ERR_WORKSPACE;
    begin_device_call();
    int dev = 0;
    int rc = current_device(&dev);
    if (rc != FFF_OK) return rc;
    if (dev_ptr) {   // ticket counters start at zero (a fill kernel: a memset node does not belong in a graph)
        hipError_t e = launch_zero((int32_t*)dev_ptr, kCtrlWords, (hipStream_t)stream);
        if (e != hipSuccess) return set_device_error(e, "zero kernel launch");
    }
    std::lock_guard<std::mutex> lock(g_mu);
    g_ws[dev].user_base = dev_ptr;
    g_ws[dev].user_bytes = dev_ptr ? bytes : 0;
    return FFF_OK;
}

int fff_reserve_workspace_bytes(size_t bytes) {
    begin_device_call();
    int dev = 0;
    int rc = current_device(&dev);
    if (rc != FFF_OK) return rc;
    std::lock_guard<std::mutex> lock(g_mu);
    if (g_ws[dev].user_base) {
        g_last_error = "a caller-provided workspace is set on this device";
        return FFF_ERR_WORKSPACE;
    }
    return grow_owned(g_ws[dev], bytes, nullptr, false);
}

int fff_reserve_workspace(int64_t T, int depth) {
    if (T < 0 || T > kMaxTokens || depth < 0 || depth > FFF_MAX_DEPTH) return FFF_ERR_RANGE;
    return fff_reserve_workspace_bytes(fff_workspace_bytes(T, depth));
}

int fff_release_workspace(void) {
    std::lock_guard<std::mutex> lock(g_mu);
    int cur = 0;
    if (hipGetDevice(&cur) != hipSuccess) return FFF_ERR_DEVICE;
    int rc = FFF_OK;
    for (int d = 0; d < kMaxDevices; ++d) {
        if (!g_ws[d].base) continue;
        if (hipSetDevice(d) != hipSuccess || hipFree(g_ws[d].base) != hipSuccess) rc = FFF_ERR_DEVICE;
        g_ws[d].base = nullptr;
        g_ws[d].bytes = 0;
    }
    (void)hipSetDevice(cur);
    return rc;
}

static int64_t* option_slot(const char* name) {
    if (!name) return nullptr;
    if (!std::strcmp(name, "path")) return &g_opt.path;
    if (!std::strcmp(name, "leaf_path")) return &g_opt.leaf_path;
    if (!std::strcmp(name, "bucketing")) return &g_opt.bucketing;
    if (!std::strcmp(name, "stage_timing")) return &g_opt.stage_timing;
    if (!std::strcmp(name, "last_path")) return &g_opt.last_path;
    if (!std::strcmp(name, "last_leaf_path")) return &g_opt.last_leaf_path;
    if (!std::strcmp(name, "last_walk_top")) return &g_walk_tuning.last_top;
    if (!std::strcmp(name, "last_block_kernel")) return &g_opt.last_block_kernel;
    if (!std::strcmp(name, "last_block_top")) return &g_block_tuning.last_top;
    return nullptr;
}

// Experiment switches (fff_debug_option); 0 = the built-in choice everywhere.
//   "token_max_T"    batches of up to this many tokens take the one-block-per-token launch (6 times
//                    that where leaf_width > 8 rules out the fused launch); default 512
//   "walk_tpg", "walk_block", "walk_top", "walk_bpc", "walk_prefetch"
//                    descent / fused kernel: tokens per lane group, threads per block, k + 1 = at most
//                    k LDS-staged levels, persistent blocks per compute unit, next-tile prefetch;
//                    combinations the kernel is not built for are ignored
//   "block_top"      fff_forward_block, persistent launch: k + 1 = at most k node levels in LDS
//   "leaf_split"     staged leaf stage on the tile kernels: 1..16 = a tile (16 consecutive slots of the
//                    bucketed order) with at least this many runs of equal leaf goes to the gather
//                    kernel instead; 0 or above 16 = no split
//   "bucket_kernel"  0 = choose by size (the token-chunk kernel up to 131072 tokens and 4096 leaves;
//                    beyond that the segment kernels for up to 4096 leaves, else the leaf-range kernel
//                    up to 2^21 tokens and 2^19 leaves, else the chunk-matrix kernels), 1 = the
//                    leaf-range kernel, 2 = the chunk-matrix kernels, 3 = the token-chunk kernel,
//                    4 = the segment kernels, 5 = the fold kernel on per-block leaf counts (the
//                    descent's inside fff_forward_hard, a counting launch's otherwise; up to 1024
//                    leaves and 1024 tokens a block), each when the sizes allow it; 0 also takes
//                    the fold kernel whenever the descent has left counts
//   "fail_workspace_growth" n = the next n growths of the library's own workspace fail as if the device
//                    were out of memory (FFF_ERR_WORKSPACE; the call after them allocates again)
//   "soft_small_tiles" 1 = fff_forward_soft uses the 64 x 128 MFMA tile for every contraction (default:
//                    the 128 x 256 tile where batch and width fill it)
//   "walk_plain_x"   the descent reads token rows 1 = without the streaming hint, 2 = with it,
//                    0 = without it while the batch fits half the last-level cache
static int64_t* debug_slot(const char* name) {
    if (!name) return nullptr;
    if (!std::strcmp(name, "token_max_T")) return &g_opt.token_max_T;
    if (!std::strcmp(name, "walk_tpg")) return &g_walk_tuning.tpg;
    if (!std::strcmp(name, "walk_block")) return &g_walk_tuning.block;
    if (!std::strcmp(name, "walk_top")) return &g_walk_tuning.top;
    if (!std::strcmp(name, "walk_bpc")) return &g_walk_tuning.bpc;
    if (!std::strcmp(name, "walk_prefetch")) return &g_walk_tuning.prefetch;
    if (!std::strcmp(name, "walk_plain_x")) return &g_walk_tuning.plain_x;
    if (!std::strcmp(name, "block_top")) return &g_block_tuning.top;
    if (!std::strcmp(name, "leaf_split")) return &g_opt.leaf_split;
    if (!std::strcmp(name, "bucket_kernel")) return &g_opt.bucket_kernel;
    if (!std::strcmp(name, "soft_small_tiles")) return &g_soft_small_tiles;
    if (!std::strcmp(name, "fail_workspace_growth")) return &g_fail_growths;
    return nullptr;
}

int fff_set_option(const char* name, int64_t value) {
    int64_t* s = option_slot(name);
    if (!s || value < 0) return FFF_ERR_UNSUPPORTED;
    if (s == &g_opt.last_path || s == &g_opt.last_leaf_path || s == &g_walk_tuning.last_top ||
        s == &g_opt.last_block_kernel || s == &g_block_tuning.last_top)
        return FFF_ERR_UNSUPPORTED;   // read-only
    *s = value;
    return FFF_OK;
}

int fff_get_option(const char* name, int64_t* value) {
    int64_t* s = option_slot(name);
    if (!s) return FFF_ERR_UNSUPPORTED;
    if (!value) return FFF_ERR_NULL;
    *value = *s;
    return FFF_OK;
}

int fff_debug_option(const char* name, int64_t value, int64_t* current) {
    int64_t* s = debug_slot(name);
    if (!s) return FFF_ERR_UNSUPPORTED;
    if (value >= 0) *s = value;
    if (current) *current = *s;
    return FFF_OK;
}

int fff_stage_times(double* ms, int64_t* calls) {
    if (!ms || !calls) return FFF_ERR_NULL;
    std::vector<hipEvent_t> ev;
    {
        std::lock_guard<std::mutex> lock(g_mu);
        ev.swap(g_stage_events);
    }
    for (int k = 0; k < 4; ++k) ms[k] = 0.0;
    *calls = 0;
    int rc = FFF_OK;
    for (size_t i = 0; i + 4 < ev.size(); i += 5) {
        if (hipEventSynchronize(ev[i + 4]) != hipSuccess) { rc = FFF_ERR_DEVICE; break; }
        float d[4];
        bool ok = true;
        for (int k = 0; k < 4; ++k) ok = ok && hipEventElapsedTime(&d[k], ev[i + k], ev[i + k + 1]) == hipSuccess;
        if (!ok) { rc = FFF_ERR_DEVICE; break; }
        for (int k = 0; k < 4; ++k) ms[k] += d[k];
        *calls += 1;
    }
    for (hipEvent_t e : ev) (void)hipEventDestroy(e);
    return rc;
}

const char* fff_status_string(int status) {
    switch (status) {
        case FFF_OK: return "ok";
        case FFF_ERR_NULL: return "a required pointer is NULL";
        case FFF_ERR_SHAPE: return "sizes are inconsistent or out of the supported range";
        case FFF_ERR_DTYPE: return "unknown dtype";
        case FFF_ERR_RANGE: return "depth, leaf_width or T out of range";
        case FFF_ERR_UNSUPPORTED: return "unknown activation or option";
        case FFF_ERR_WORKSPACE: return "workspace too small, misaligned or not allocatable";
        case FFF_ERR_DEVICE: return "a HIP call failed";
        case FFF_ERR_ALIAS: return "out overlaps x";
        default: return "unknown status";
    }
}

const char* fff_last_device_error(void) { return g_last_error.c_str(); }

const char* fff_last_launch(void) { return g_last_launch.c_str(); }

int fff_version(void) { return 300; }

}  // extern "C"
