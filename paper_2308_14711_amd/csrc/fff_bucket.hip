// K2 -- per-leaf token lists: histogram, prefix scan, stable scatter.
//
// Not in the paper (its implementation indexes weights per token); the lists
// only let the tokens of one leaf share a single read of that leaf's weights.
// Integer work throughout, and the result does not depend on scheduling:
//
//   rank    tokens are cut into chunks of 256 consecutive ids.  A block ranks
//           each token among the same-leaf tokens that precede it in its chunk
//           and stores the chunk's per-leaf totals in M[leaf][chunk].
//   scan    one wave per leaf turns M[leaf][*] into an exclusive prefix along
//           the chunks and emits count[leaf]; the block that finishes last
//           scans count[] into offset[] (and the per-leaf tile offsets).
//   scatter perm[offset[leaf] + M[leaf][chunk] + rank] = token -- ascending
//           token order inside a leaf by construction, no atomics on the
//           positions.
//
// M must be zero on entry (launch_zero) because a chunk touches only the
// leaves it contains.
//
// For trees of moderate size (2^depth <= 2^19 leaves, T <= 2^21 tokens) all
// three steps run as ONE launch with no global intermediate and no atomics on
// global memory (bucket_onepass_kernel): a block owns a contiguous range of
// leaves and reads the whole leaf_idx array twice.  Pass 1 counts, per wave
// (each wave owns a contiguous token range), the tokens of every owned leaf
// and the tokens of all lower-numbered leaves; an in-LDS scan turns that into
// the owned leaves' global offsets and each wave's starting position inside
// every leaf.  Pass 2 walks the same tokens in the same order and writes
// perm; same-leaf tokens of one 64-token batch are ranked with ballots.
#include "fff_device.h"
#include "fff_internal.h"

#include <type_traits>

namespace fff {

__device__ __forceinline__ int32_t load_l2(const int32_t* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__global__ __launch_bounds__(256) void zero_kernel(int4* __restrict__ p, int64_t n4) {
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += (int64_t)gridDim.x * 256)
        p[i] = make_int4(0, 0, 0, 0);
}

hipError_t launch_zero(int32_t* p, int64_t n, hipStream_t s) {
    // n is a multiple of 4 and p 16-byte aligned by construction of the workspace
    const int64_t n4 = n / 4;
    if (n4 == 0) return hipSuccess;
    int64_t blocks = (n4 + 255) / 256;
    if (blocks > 2048) blocks = 2048;
    zero_kernel<<<dim3((unsigned)blocks), dim3(256), 0, s>>>((int4*)p, n4);
    return hipGetLastError();
}

// One block per chunk of `rounds` * 256 tokens; M row stride = n_chunks.
__global__ __launch_bounds__(256) void bucket_rank_kernel(const int32_t* __restrict__ leaf_idx, int64_t T,
                                                          int rounds, int64_t n_chunks,
                                                          int32_t* __restrict__ rank,
                                                          int32_t* __restrict__ M) {
    __shared__ int32_t s_leaf[kChunkTokens];
    const int tid = threadIdx.x;
    const int64_t chunk = blockIdx.x;
    for (int r = 0; r < rounds; ++r) {
        const int64_t t = (chunk * rounds + r) * kChunkTokens + tid;
        const int32_t leaf = t < T ? leaf_idx[t] : -1;
        s_leaf[tid] = leaf;
        __syncthreads();
        int before = 0, after = 0;
        const int4* s4 = (const int4*)s_leaf;
#pragma unroll 4
        for (int j4 = 0; j4 < kChunkTokens / 4; ++j4) {
            const int4 v = s4[j4];     // same address in every lane: a broadcast read
            const int j = j4 * 4;
            before += (v.x == leaf && j + 0 < tid) + (v.y == leaf && j + 1 < tid) +
                      (v.z == leaf && j + 2 < tid) + (v.w == leaf && j + 3 < tid);
            after += (v.x == leaf && j + 0 > tid) + (v.y == leaf && j + 1 > tid) +
                     (v.z == leaf && j + 2 > tid) + (v.w == leaf && j + 3 > tid);
        }
        int32_t* cell = M + (int64_t)(leaf >= 0 ? leaf : 0) * n_chunks + chunk;
        int32_t base = 0;
        if (leaf >= 0) {
            // totals of earlier rounds of this chunk (written by this block, read back through L2)
            if (r > 0) base = load_l2(cell);
            rank[t] = base + before;
        }
        __syncthreads();               // every reader of the cell and of s_leaf is done
        if (leaf >= 0 && after == 0)
            __hip_atomic_store(cell, base + before + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (rounds > 1) {
            __threadfence();
            __syncthreads();
        }
    }
}

__device__ __forceinline__ int32_t wave_incl_scan(int32_t v, int lane) {
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        const int32_t o = __shfl_up(v, d, kWave);
        if (lane >= d) v += o;
    }
    return v;
}

// Exclusive scan of count[0..n) into offset[0..n], and of the per-leaf tile
// counts into tile_off[0..n]; run by one block of 1024 threads.
__device__ void block_scan_counts(const int32_t* __restrict__ count, int64_t n, int tile_rows,
                                  int32_t* __restrict__ offset, int32_t* __restrict__ tile_off,
                                  int32_t* __restrict__ ctrl) {
    __shared__ int32_t s_tot[2][16];
    __shared__ int32_t s_carry[2];
    const int tid = threadIdx.x, lane = tid % kWave, wv = tid / kWave;
    if (tid < 2) s_carry[tid] = 0;
    __syncthreads();
    for (int64_t base = 0; base < n; base += 1024) {
        const int64_t j = base + tid;
        const int32_t c = j < n ? load_l2(count + j) : 0;
        const int32_t nt = (c + tile_rows - 1) / tile_rows;
        const int32_t ic = wave_incl_scan(c, lane);
        const int32_t it = wave_incl_scan(nt, lane);
        if (lane == kWave - 1) { s_tot[0][wv] = ic; s_tot[1][wv] = it; }
        __syncthreads();
        int32_t pc = s_carry[0], pt = s_carry[1];
        for (int w = 0; w < wv; ++w) { pc += s_tot[0][w]; pt += s_tot[1][w]; }
        if (j < n) {
            if (offset) offset[j] = pc + ic - c;
            if (tile_off) tile_off[j] = pt + it - nt;
        }
        __syncthreads();
        if (tid == 1023) { s_carry[0] = pc + ic; s_carry[1] = pt + it; }
        __syncthreads();
    }
    if (tid == 0) {
        if (offset) offset[n] = s_carry[0];
        if (tile_off) tile_off[n] = s_carry[1];
        ctrl[1] = s_carry[1];          // number of tiles
    }
}

// 16 waves per block, one leaf per wave: M[leaf][*] -> exclusive prefix along chunks.
__global__ __launch_bounds__(1024) void bucket_scan_kernel(int32_t* __restrict__ M, int64_t n_leaves,
                                                           int64_t n_chunks, int tile_rows,
                                                           int32_t* __restrict__ count,
                                                           int32_t* __restrict__ offset,
                                                           int32_t* __restrict__ tile_off,
                                                           int32_t* __restrict__ ctrl) {
    __shared__ int s_last;
    const int lane = threadIdx.x % kWave;
    const int64_t leaf = (int64_t)blockIdx.x * 16 + threadIdx.x / kWave;
    if (leaf < n_leaves) {
        int32_t* row = M + leaf * n_chunks;
        int32_t carry = 0;
        // four steps of 64 chunks at a time: their loads are requested together
        for (int64_t c0 = 0; c0 < n_chunks; c0 += 4 * kWave) {
            int32_t v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int64_t c = c0 + u * kWave + lane;
                v[u] = c < n_chunks ? row[c] : 0;
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int64_t c = c0 + u * kWave + lane;
                const int32_t inc = wave_incl_scan(v[u], lane);
                if (c < n_chunks) row[c] = carry + inc - v[u];
                carry += __shfl(inc, kWave - 1, kWave);
            }
        }
        if (lane == 0) __hip_atomic_store(count + leaf, carry, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    // the block that arrives last sees every count and scans them
    __threadfence();
    __syncthreads();
    if (threadIdx.x == 0) {
        const int ticket = atomicAdd(ctrl, 1);
        s_last = ticket == (int)gridDim.x - 1;
    }
    __syncthreads();
    if (s_last) {
        __threadfence();
        block_scan_counts(count, n_leaves, tile_rows, offset, tile_off, ctrl);
        if (threadIdx.x == 0) ctrl[0] = 0;   // ready for the next call
    }
}

__global__ __launch_bounds__(256) void bucket_scatter_kernel(const int32_t* __restrict__ leaf_idx,
                                                             const int32_t* __restrict__ rank, int64_t T,
                                                             int rounds, int64_t n_chunks,
                                                             const int32_t* __restrict__ M,
                                                             const int32_t* __restrict__ offset,
                                                             int32_t* __restrict__ perm,
                                                             int32_t* __restrict__ slot_leaf) {
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= T) return;
    const int64_t leaf = leaf_idx[t];
    const int64_t chunk = t / ((int64_t)kChunkTokens * rounds);
    const int32_t pos = offset[leaf] + M[leaf * n_chunks + chunk] + rank[t];
    perm[pos] = (int32_t)t;
    if (slot_leaf) slot_leaf[pos] = (int32_t)leaf;
}


constexpr int kOnepassWaves = 16;
constexpr int kOnepassMaxLeavesPerBlock = 512;
constexpr int kAhead = 16;         // 16-byte loads in flight per lane (4096 tokens per wave)
constexpr int kBatch = 4 * kWave;  // tokens per wave step: lane l holds tokens 4 l .. 4 l + 3

__device__ __forceinline__ uint64_t lanes_below(int lane) { return lane == 0 ? 0ull : (~0ull >> (64 - lane)); }

// leaf ids of tokens t0 .. t0 + 3 (sentinel past the end); the fast form needs 16-byte alignment
__device__ __forceinline__ int4 load_leaf4(const int32_t* __restrict__ leaf_idx, int64_t t0, int64_t T, bool vec) {
    const int32_t none = 0x7fffffff;
    if (vec && t0 + 3 < T) return *(const int4*)(leaf_idx + t0);
    int4 v;
    v.x = t0 + 0 < T ? leaf_idx[t0 + 0] : none;
    v.y = t0 + 1 < T ? leaf_idx[t0 + 1] : none;
    v.z = t0 + 2 < T ? leaf_idx[t0 + 2] : none;
    v.w = t0 + 3 < T ? leaf_idx[t0 + 3] : none;
    return v;
}

// Pass 1 on one batch: tokens of lower leaves go to n_below, tokens of owned leaves to my_cnt.
__device__ __forceinline__ void onepass_count(const int4 v, int32_t lo, uint32_t n_own, int32_t& n_below,
                                              int32_t* my_cnt) {
    const int32_t e[4] = {v.x, v.y, v.z, v.w};
    bool own[4];
    bool any = false;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        n_below += e[k] < lo ? 1 : 0;
        own[k] = (uint32_t)(e[k] - lo) < n_own;
        any = any || own[k];
    }
    if (__ballot(any)) {             // rare: most batches hold no token of this block's leaves
#pragma unroll
        for (int k = 0; k < 4; ++k)
            if (own[k]) atomicAdd(&my_cnt[e[k] - lo], 1);
    }
}

// Pass 2 on one batch whose first token is t0 (lane l holds tokens t0 + 4 l .. + 3):
// position = start of the leaf + tokens of earlier waves + tokens this wave has already placed
// + rank inside the batch (lane-major, then element).
__device__ __forceinline__ void onepass_place(const int4 v, int64_t t0, int lane, int32_t lo, uint32_t n_own,
                                              const int32_t* lbase, int32_t* my_cnt,
                                              int32_t* __restrict__ perm, int32_t* __restrict__ slot_leaf) {
    const int32_t e[4] = {v.x, v.y, v.z, v.w};
    bool own[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) own[k] = (uint32_t)(e[k] - lo) < n_own;
    uint64_t pending = __ballot(own[0] || own[1] || own[2] || own[3]);
    while (pending) {
        // the smallest pending (lane, element) decides which leaf is placed next
        const int first = __ffsll((unsigned long long)pending) - 1;
        int32_t mine = 0x7fffffff;
#pragma unroll
        for (int k = 3; k >= 0; --k)
            if (own[k]) mine = e[k];
        const int32_t leaf = __shfl(mine, first, kWave);
        int c = 0, pre[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            pre[k] = c;
            c += (own[k] && e[k] == leaf) ? 1 : 0;
        }
        const uint64_t m0 = __ballot(c & 1), m1 = __ballot(c & 2), m2 = __ballot(c & 4);
        const uint64_t lt = lanes_below(lane);
        const int lanes_before = __popcll(m0 & lt) + 2 * __popcll(m1 & lt) + 4 * __popcll(m2 & lt);
        const int n_grp = __popcll(m0) + 2 * __popcll(m1) + 4 * __popcll(m2);
        const int local = leaf - lo;
        int32_t seen = 0;
        if (lane == first) seen = atomicAdd(&my_cnt[local], n_grp);
        seen = __shfl(seen, first, kWave);
        const int32_t at = lbase[local] + seen + lanes_before;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            if (own[k] && e[k] == leaf) {
                perm[at + pre[k]] = (int32_t)(t0 + 4 * lane + k);
                if (slot_leaf) slot_leaf[at + pre[k]] = leaf;
                own[k] = false;
            }
        }
        pending = __ballot(own[0] || own[1] || own[2] || own[3]);
    }
}

__global__ __launch_bounds__(1024) void bucket_onepass_kernel(const int32_t* __restrict__ leaf_idx, int64_t T,
                                                              int64_t n_leaves, int per_block, int vec,
                                                              int32_t* __restrict__ count,
                                                              int32_t* __restrict__ offset,
                                                              int32_t* __restrict__ perm,
                                                              int32_t* __restrict__ slot_leaf) {
    extern __shared__ int32_t sm[];
    int32_t* cnt = sm;                                       // [16][per_block] per-wave counts, then bases
    int32_t* lbase = sm + kOnepassWaves * per_block;         // [per_block] start of each owned leaf
    int32_t* below = lbase + per_block;                      // [16] tokens of lower leaves, per wave
    int32_t* wsum = below + kOnepassWaves;                   // [16] scratch of the block scan
    const int tid = threadIdx.x, lane = tid % kWave, w = tid / kWave;
    const int32_t lo = (int32_t)((int64_t)blockIdx.x * per_block);
    const int32_t hi = lo + per_block < n_leaves ? lo + per_block : (int32_t)n_leaves;
    const uint32_t n_own = (uint32_t)(hi - lo);

    for (int i = tid; i < kOnepassWaves * per_block; i += 1024) cnt[i] = 0;
    __syncthreads();

    // token range of this wave: whole batches of 256 tokens, in token order over the waves
    const int64_t batches = (T + kBatch - 1) / kBatch;
    const int64_t per_wave = (batches + kOnepassWaves - 1) / kOnepassWaves;
    const int64_t b_beg = per_wave * w < batches ? per_wave * w : batches;
    const int64_t b_end = b_beg + per_wave < batches ? b_beg + per_wave : batches;
    const int64_t full = vec ? T / kBatch : 0;      // batches read with one unguarded 16-byte load
    int32_t* my_cnt = cnt + w * per_block;
    const int4* src = (const int4*)leaf_idx + lane;
    const int4 none4 = make_int4(0x7fffffff, 0x7fffffff, 0x7fffffff, 0x7fffffff);
    auto load_batch = [&](int64_t b) {
        return b < b_end ? (b < full ? src[b * kWave] : load_leaf4(leaf_idx, b * kBatch + 4 * lane, T, vec)) : none4;
    };
    // kAhead batches are fetched before any is examined.  When the wave's whole range is one
    // such group (T <= 65536) it stays in registers for both passes.
    const bool single = per_wave <= kAhead;
    int4 keep[kAhead];

    int32_t n_below = 0;
    for (int64_t b = b_beg; b < b_end; b += kAhead) {
#pragma unroll
        for (int u = 0; u < kAhead; ++u) keep[u] = load_batch(b + u);
#pragma unroll
        for (int u = 0; u < kAhead; ++u) onepass_count(keep[u], lo, n_own, n_below, my_cnt);
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) n_below += __shfl_xor(n_below, d, kWave);
    if (lane == 0) below[w] = n_below;
    __syncthreads();

    // per owned leaf: exclusive prefix over the waves (token order), and the leaf's total
    int32_t total = 0;
    if ((uint32_t)tid < n_own) {
        for (int ww = 0; ww < kOnepassWaves; ++ww) {
            const int32_t v = cnt[ww * per_block + tid];
            cnt[ww * per_block + tid] = total;
            total += v;
        }
    }
    // exclusive scan of the totals over the owned leaves (per_block <= 512 <= 1024 threads)
    int32_t inc = total;
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        const int32_t o = __shfl_up(inc, d, kWave);
        if (lane >= d) inc += o;
    }
    if (lane == kWave - 1) wsum[w] = inc;
    __syncthreads();
    int32_t before = 0, n_below_all = 0;
    for (int ww = 0; ww < kOnepassWaves; ++ww) {
        if (ww < w) before += wsum[ww];
        n_below_all += below[ww];
    }
    if ((uint32_t)tid < n_own) {
        const int32_t start = n_below_all + before + inc - total;
        lbase[tid] = start;
        if (offset) offset[lo + tid] = start;
        if (count) count[lo + tid] = total;
    }
    if (offset && hi == n_leaves && tid == 0) offset[n_leaves] = (int32_t)T;
    __syncthreads();
    if (!perm) return;

    // pass 2: same tokens, same order
    for (int64_t b = b_beg; b < b_end; b += kAhead) {
        if (!single) {
#pragma unroll
            for (int u = 0; u < kAhead; ++u) keep[u] = load_batch(b + u);
        }
#pragma unroll
        for (int u = 0; u < kAhead; ++u)
            onepass_place(keep[u], (b + u) * kBatch, lane, lo, n_own, lbase, my_cnt, perm, slot_leaf);
    }
}

// true when the one-launch kernel takes (T, depth)
bool bucket_onepass_ok(int64_t T, int depth) { return depth <= 19 && T <= ((int64_t)1 << 21); }

hipError_t launch_bucket_onepass(const int32_t* leaf_idx, int64_t T, int depth, int32_t* count,
                                 int32_t* offset, int32_t* perm, int32_t* slot_leaf, hipStream_t s) {
    const int64_t NL = (int64_t)1 << depth;
    int64_t per_block = (NL + 255) / 256;
    if (per_block > kOnepassMaxLeavesPerBlock) per_block = kOnepassMaxLeavesPerBlock;
    const int64_t blocks = (NL + per_block - 1) / per_block;
    const size_t lds = sizeof(int32_t) * (size_t)(kOnepassWaves * per_block + per_block + 2 * kOnepassWaves);
    const int vec = (reinterpret_cast<uintptr_t>(leaf_idx) & 15u) == 0;
    note_launch("bucket_onepass_kernel");
    bucket_onepass_kernel<<<dim3((unsigned)blocks), dim3(1024), lds, s>>>(leaf_idx, T, NL, (int)per_block, vec,
                                                                          count, offset, perm, slot_leaf);
    return hipGetLastError();
}

// ---- one launch, a block per chunk of tokens (moderate T, up to 4096 leaves) ----
//
// Every block builds the histogram of ALL tokens in LDS by itself (one 64-bit LDS atomic per token:
// the low word counts the leaf's tokens, the high word those that come before the block's own
// chunk), scans it, and then places only its own chunk: position = start of the leaf + same-leaf
// tokens of earlier chunks + rank among the same-leaf tokens of the chunk (counted by comparing
// against the chunk's leaf ids in LDS, a broadcast read per step).  The histogram work is repeated
// by every block but reads 4 bytes per token from L2 and runs on all CUs at once; for the sizes
// taken here that is cheaper than two passes over the tokens with a block per leaf range.
constexpr int kHistMaxLeaves = 4096;     // 32 KB of 64-bit counters
constexpr int kHistMaxChunk = 512;       // tokens a block places
constexpr int kHistBlocks = 256;

// NARROW (T < 65536): both counts fit 16 bits and share one 32-bit counter, whose LDS atomics are
// cheaper than the 64-bit ones.
template <bool NARROW>
__global__ __launch_bounds__(1024) void bucket_hist_kernel(const int32_t* __restrict__ leaf_idx, int64_t T,
                                                           int n_leaves, int chunk, int vec,
                                                           int32_t* __restrict__ count,
                                                           int32_t* __restrict__ offset,
                                                           int32_t* __restrict__ perm,
                                                           int32_t* __restrict__ slot_leaf) {
    typedef typename std::conditional<NARROW, uint32_t, unsigned long long>::type Counter;
    constexpr int kHigh = NARROW ? 16 : 32;
    extern __shared__ unsigned long long hist_raw[];         // [n_leaves] counters: (before << kHigh) | total
    Counter* hist = (Counter*)hist_raw;
    __shared__ int32_t s_leaf[kHistMaxChunk];
    __shared__ int32_t s_wsum[kOnepassWaves];
    const int tid = threadIdx.x, lane = tid % kWave, w = tid / kWave;
    const int64_t lo = (int64_t)blockIdx.x * chunk;
    const int64_t hi = lo + chunk < T ? lo + chunk : T;
    const int n_own = (int)(hi - lo);

    for (int i = tid; i < n_leaves; i += 1024) hist[i] = 0;
    if (tid < n_own) s_leaf[tid] = leaf_idx[lo + tid];
    __syncthreads();

    // histogram of all tokens; a token before this block's chunk also counts in the high word
    const int64_t n4 = (T + 3) / 4;
    for (int64_t q0 = 0; q0 < n4; q0 += 4 * 1024) {
        int4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int64_t q = q0 + (int64_t)u * 1024 + tid;
            v[u] = q < n4 ? load_leaf4(leaf_idx, 4 * q, T, vec != 0) : make_int4(-1, -1, -1, -1);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int64_t t0 = 4 * (q0 + (int64_t)u * 1024 + tid);
            const int32_t e[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
            for (int k = 0; k < 4; ++k)
                if ((uint32_t)e[k] < (uint32_t)n_leaves)
                    atomicAdd(&hist[e[k]], (Counter)1 | (t0 + k < lo ? ((Counter)1 << kHigh) : (Counter)0));
        }
    }
    __syncthreads();

    // exclusive scan of the totals; afterwards hist[leaf] = (start of the leaf) + (tokens before the chunk)
    const int per = (n_leaves + 1023) / 1024;                // leaves per thread, at most 4
    Counter mine[kHistMaxLeaves / 1024];
    const Counter low = ((Counter)1 << kHigh) - 1;
    int32_t sum = 0;
#pragma unroll
    for (int i = 0; i < kHistMaxLeaves / 1024; ++i) {
        const int leaf = tid * per + i;
        mine[i] = (i < per && leaf < n_leaves) ? hist[leaf] : (Counter)0;
        sum += (int32_t)(mine[i] & low);
    }
    const int32_t inc = wave_incl_scan(sum, lane);
    if (lane == kWave - 1) s_wsum[w] = inc;
    __syncthreads();
    int32_t start = inc - sum;
    for (int ww = 0; ww < w; ++ww) start += s_wsum[ww];
#pragma unroll
    for (int i = 0; i < kHistMaxLeaves / 1024; ++i) {
        const int leaf = tid * per + i;
        if (i < per && leaf < n_leaves) {
            const int32_t total = (int32_t)(mine[i] & low);
            hist[leaf] = (Counter)(uint32_t)(start + (int32_t)(mine[i] >> kHigh));
            if (blockIdx.x == 0) {
                if (count) count[leaf] = total;
                if (offset) offset[leaf] = start;
            }
            start += total;
        }
    }
    if (blockIdx.x == 0 && offset && tid == 0) offset[n_leaves] = (int32_t)T;
    __syncthreads();
    if (!perm || tid >= n_own) return;

    // rank of token lo + tid among the chunk's earlier tokens of the same leaf
    const int32_t leaf = s_leaf[tid];
    if ((uint32_t)leaf >= (uint32_t)n_leaves) return;
    int rank = 0;
    const int4* s4 = (const int4*)s_leaf;
    for (int j4 = 0; 4 * j4 < tid; ++j4) {
        const int4 v = s4[j4];
        const int j = 4 * j4;
        rank += (v.x == leaf) + (v.y == leaf && j + 1 < tid) + (v.z == leaf && j + 2 < tid) + (v.w == leaf && j + 3 < tid);
    }
    const int32_t pos = (int32_t)(uint32_t)hist[leaf] + rank;
    perm[pos] = (int32_t)(lo + tid);
    if (slot_leaf) slot_leaf[pos] = leaf;
}

bool bucket_hist_ok(int64_t T, int depth) {
    return ((int64_t)1 << depth) <= kHistMaxLeaves && T <= (int64_t)kHistBlocks * kHistMaxChunk;
}

hipError_t launch_bucket_hist(const int32_t* leaf_idx, int64_t T, int depth, int32_t* count, int32_t* offset,
                              int32_t* perm, int32_t* slot_leaf, hipStream_t s) {
    const int NL = 1 << depth;
    int chunk = (int)((T + kHistBlocks - 1) / kHistBlocks);
    if (chunk < 64) chunk = 64;
    const int64_t blocks = (T + chunk - 1) / chunk;
    const int vec = (reinterpret_cast<uintptr_t>(leaf_idx) & 15u) == 0;
    note_launch("bucket_hist_kernel<%s>", T < 65536 ? "16+16" : "32+32");
    if (T < 65536)
        bucket_hist_kernel<true><<<dim3((unsigned)blocks), dim3(1024), sizeof(uint32_t) * (size_t)NL, s>>>(
            leaf_idx, T, NL, chunk, vec, count, offset, perm, slot_leaf);
    else
        bucket_hist_kernel<false><<<dim3((unsigned)blocks), dim3(1024), sizeof(unsigned long long) * (size_t)NL, s>>>(
            leaf_idx, T, NL, chunk, vec, count, offset, perm, slot_leaf);
    return hipGetLastError();
}

// ---- from per-block leaf counts: no histogram pass at all (up to 1024 leaves) ------------------
//
// The descent already knows, for every block, how many of its tokens reach each leaf: M[block][leaf]
// (launch_descend with a DescentCounts; launch_chunk_counts makes the same matrix from a leaf_idx
// array that came from elsewhere).  One launch with the same blocks and shares then finishes K2:
// every block sums the columns of M (all blocks: the leaf's total; the blocks before it: where its
// own tokens of that leaf start inside the leaf), scans the totals over the leaves, and places its
// own tokens at start(leaf) + before(leaf) + rank inside the share (counted by comparing against
// the share's leaf ids in LDS).  No atomics, ascending token order inside a leaf by construction.

bool bucket_fold_ok(int depth, int64_t blocks, int64_t share) {
    return depth <= 10 && share <= kFoldMaxShare && blocks >= 1 && (blocks << depth) <= kFoldWords;
}

__global__ __launch_bounds__(1024) void chunk_counts_kernel(const int32_t* __restrict__ leaf_idx, int64_t T,
                                                            int n_leaves, int64_t share, int32_t* __restrict__ M) {
    __shared__ int32_t s_hist[kFoldMaxLeaves];
    const int tid = threadIdx.x;
    for (int i = tid; i < n_leaves; i += 1024) s_hist[i] = 0;
    __syncthreads();
    const int64_t t = (int64_t)blockIdx.x * share + tid;
    if (tid < share && t < T) {
        const int32_t leaf = leaf_idx[t];
        if ((uint32_t)leaf < (uint32_t)n_leaves) atomicAdd(&s_hist[leaf], 1);
    }
    __syncthreads();
    for (int i = tid; i < n_leaves; i += 1024) M[(int64_t)blockIdx.x * n_leaves + i] = s_hist[i];
}

__global__ __launch_bounds__(1024) void bucket_fold_kernel(const int32_t* __restrict__ leaf_idx, int64_t T,
                                                           int n_leaves, int64_t share, int n_blocks,
                                                           const int32_t* __restrict__ M,
                                                           int32_t* __restrict__ count, int32_t* __restrict__ offset,
                                                           int32_t* __restrict__ perm, int32_t* __restrict__ slot_leaf) {
    __shared__ int32_t s_tot[4096], s_bef[4096];      // partial column sums: [range][leaf], at most 16 ranges
    __shared__ int32_t s_base[kFoldMaxLeaves];        // where this block's tokens of a leaf start
    __shared__ int32_t s_leaf[kFoldMaxShare];
    __shared__ int32_t s_wsum[16];
    const int tid = threadIdx.x, lane = tid % kWave, w = tid / kWave;
    const int b = blockIdx.x;
    const int64_t lo = (int64_t)b * share;
    const int64_t hi = lo + share < T ? lo + share : T;
    const int n_own = hi > lo ? (int)(hi - lo) : 0;
    if (tid < n_own) s_leaf[tid] = leaf_idx[lo + tid];

    // column sums of M (n_leaves is a power of two <= 1024): thread (r, g) takes the rows of range r
    // for the four leaves of column group g, 16 bytes a load, and all loads of a batch are issued
    // before the first is used -- a block is a chain of trips to L2 otherwise (256 blocks over 256
    // leaves: 16 ranges of 16 rows, two batches)
    int ranges;
    if (n_leaves >= 4) {
        const int groups = n_leaves / 4;
        ranges = 1024 / groups < 16 ? 1024 / groups : 16;
        const int g = tid % groups, r = tid / groups;
        const int per = (n_blocks + ranges - 1) / ranges;
        const int b0 = r * per, b1 = b0 + per < n_blocks ? b0 + per : n_blocks;
        int4 tot = make_int4(0, 0, 0, 0), bef = make_int4(0, 0, 0, 0);
        constexpr int kBatch = 8;
        if (r < ranges) {
            const int4* col = (const int4*)M + g;
            for (int bb = b0; bb < b1; bb += kBatch) {
                int4 v[kBatch];
#pragma unroll
                for (int u = 0; u < kBatch; ++u) {
                    const int row = bb + u < b1 ? bb + u : b1 - 1;      // clamped: the load is unconditional
                    v[u] = col[(int64_t)row * groups];
                }
#pragma unroll
                for (int u = 0; u < kBatch; ++u) {
                    const int in = bb + u < b1, early = bb + u < b;
                    tot.x += in ? v[u].x : 0; tot.y += in ? v[u].y : 0; tot.z += in ? v[u].z : 0; tot.w += in ? v[u].w : 0;
                    bef.x += early && in ? v[u].x : 0; bef.y += early && in ? v[u].y : 0;
                    bef.z += early && in ? v[u].z : 0; bef.w += early && in ? v[u].w : 0;
                }
            }
            ((int4*)s_tot)[r * groups + g] = tot;
            ((int4*)s_bef)[r * groups + g] = bef;
        }
    } else {                                          // one or two leaves: a row is shorter than a vector
        ranges = 16;
        const int l = tid % n_leaves, r = tid / n_leaves;
        const int per = (n_blocks + ranges - 1) / ranges;
        const int b0 = r * per, b1 = b0 + per < n_blocks ? b0 + per : n_blocks;
        if (r < ranges) {
            int32_t tot = 0, bef = 0;
            for (int bb = b0; bb < b1; ++bb) {
                const int32_t c = M[(int64_t)bb * n_leaves + l];
                tot += c;
                bef += bb < b ? c : 0;
            }
            s_tot[r * n_leaves + l] = tot;
            s_bef[r * n_leaves + l] = bef;
        }
    }
    __syncthreads();
    int32_t total = 0, before = 0;
    if (tid < n_leaves) {
        for (int q = 0; q < ranges; ++q) {
            total += s_tot[q * n_leaves + tid];
            before += s_bef[q * n_leaves + tid];
        }
    }
    // exclusive scan of the totals over the leaves
    const int32_t inc = wave_incl_scan(total, lane);
    if (lane == kWave - 1) s_wsum[w] = inc;
    __syncthreads();
    int32_t start = inc - total;
    for (int ww = 0; ww < w; ++ww) start += s_wsum[ww];
    if (tid < n_leaves) {
        s_base[tid] = start + before;
        if (b == 0) {
            if (count) count[tid] = total;
            if (offset) offset[tid] = start;
        }
    }
    if (b == 0 && offset && tid == 0) offset[n_leaves] = (int32_t)T;
    __syncthreads();
    if (!perm || tid >= n_own) return;

    // rank of token lo + tid among the share's earlier tokens of the same leaf
    const int32_t leaf = s_leaf[tid];
    if ((uint32_t)leaf >= (uint32_t)n_leaves) return;
    int rank = 0;
    const int4* s4 = (const int4*)s_leaf;
    for (int j4 = 0; 4 * j4 < tid; ++j4) {
        const int4 v = s4[j4];
        const int j = 4 * j4;
        rank += (v.x == leaf) + (v.y == leaf && j + 1 < tid) + (v.z == leaf && j + 2 < tid) + (v.w == leaf && j + 3 < tid);
    }
    const int32_t pos = s_base[leaf] + rank;
    perm[pos] = (int32_t)(lo + tid);
    if (slot_leaf) slot_leaf[pos] = leaf;
}

hipError_t launch_chunk_counts(const int32_t* leaf_idx, int64_t T, int depth, DescentCounts* dc, hipStream_t s) {
    dc->blocks = 0;
    if (T <= 0 || !dc->M) return hipSuccess;
    // as many blocks as the matrix has room for (at most 256), at least 64 tokens each
    int64_t blocks = dc->capacity >> depth;
    if (blocks > 256) blocks = 256;
    if (blocks < 1) return hipSuccess;
    int64_t share = (T + blocks - 1) / blocks;
    if (share < 64) share = 64;
    blocks = (T + share - 1) / share;
    if (!bucket_fold_ok(depth, blocks, share) || (blocks << depth) > dc->capacity) return hipSuccess;
    note_launch("chunk_counts_kernel");
    chunk_counts_kernel<<<dim3((unsigned)blocks), dim3(1024), 0, s>>>(leaf_idx, T, 1 << depth, share, dc->M);
    dc->blocks = (int)blocks;
    dc->share = share;
    return hipGetLastError();
}

hipError_t launch_bucket_fold(const int32_t* leaf_idx, int64_t T, int depth, const DescentCounts& dc,
                              int32_t* count, int32_t* offset, int32_t* perm, int32_t* slot_leaf, hipStream_t s) {
    if (dc.blocks <= 0 || !bucket_fold_ok(depth, dc.blocks, dc.share)) return hipErrorInvalidValue;
    note_launch("bucket_fold_kernel");
    bucket_fold_kernel<<<dim3((unsigned)dc.blocks), dim3(1024), 0, s>>>(leaf_idx, T, 1 << depth, dc.share, dc.blocks,
                                                                       dc.M, count, offset, perm, slot_leaf);
    return hipGetLastError();
}

// ---- many tokens over few leaves (up to 4096): segments of 1024 tokens, a wave each ----------
//
//   count    a wave histograms its segment in LDS and writes M[leaf][segment] for every leaf (so M
//            needs no clearing)
//   scan     bucket_scan_kernel, as for the chunk-matrix kernels
//   scatter  a wave walks its segment again in the same order, 64 tokens at a time: a token's
//            position is the running start of its leaf (LDS, initialised to offset[leaf] +
//            M[leaf][segment]) plus the number of lower lanes of the batch with the same leaf (from
//            one ballot per bit of the leaf index); the last lane of every leaf in the batch stores
//            the new running start.  One wave per
//            block, so a batch's reads of the running starts precede its writes by program order.
constexpr int kSegTokens = 1024;
constexpr int kSegMaxLeaves = 4096;

__global__ __launch_bounds__(kWave) void seg_count_kernel(const int32_t* __restrict__ leaf_idx, int64_t T,
                                                          int n_leaves, int64_t n_segs, int32_t* __restrict__ M) {
    __shared__ int32_t hist[kSegMaxLeaves];
    const int lane = threadIdx.x;
    const int64_t seg = blockIdx.x;
    for (int j = lane; j < n_leaves; j += kWave) hist[j] = 0;
    __syncthreads();
    const int64_t t0 = seg * kSegTokens;
    int32_t mine[kSegTokens / kWave];          // all requested before the first is used
#pragma unroll
    for (int k = 0; k < kSegTokens / kWave; ++k) {
        const int64_t t = t0 + (int64_t)k * kWave + lane;
        mine[k] = t < T ? leaf_idx[t] : -1;
    }
#pragma unroll
    for (int k = 0; k < kSegTokens / kWave; ++k)
        if ((uint32_t)mine[k] < (uint32_t)n_leaves) atomicAdd(&hist[mine[k]], 1);   // a caller's bad index is skipped, not followed
    __syncthreads();
    for (int j = lane; j < n_leaves; j += kWave) M[(int64_t)j * n_segs + seg] = hist[j];
}

__global__ __launch_bounds__(kWave) void seg_scatter_kernel(const int32_t* __restrict__ leaf_idx, int64_t T,
                                                            int n_leaves, int n_bits, int64_t n_segs,
                                                            const int32_t* __restrict__ M,
                                                            const int32_t* __restrict__ offset,
                                                            int32_t* __restrict__ perm,
                                                            int32_t* __restrict__ slot_leaf) {
    __shared__ int32_t start[kSegMaxLeaves];
    const int lane = threadIdx.x;
    const int64_t seg = blockIdx.x;
    for (int j = lane; j < n_leaves; j += kWave) start[j] = offset[j] + M[(int64_t)j * n_segs + seg];
    __syncthreads();
    const int64_t t0 = seg * kSegTokens;
    // the segment's leaf ids are requested at once: the batches below depend on each other through
    // the running starts, and a wave alone on its SIMD has nothing else to hide a load behind
    int32_t mine[kSegTokens / kWave];
#pragma unroll
    for (int k = 0; k < kSegTokens / kWave; ++k) {
        const int64_t t = t0 + (int64_t)k * kWave + lane;
        mine[k] = t < T ? leaf_idx[t] : -1;
    }
#pragma unroll
    for (int k = 0; k < kSegTokens / kWave; ++k) {
        const int64_t t = t0 + (int64_t)k * kWave + lane;
        const int32_t leaf = mine[k];
        const bool valid = (uint32_t)leaf < (uint32_t)n_leaves;
        // the lanes of the batch that hold my leaf: one ballot per bit of the index, each lane keeps
        // the lanes that agree with it on that bit
        uint64_t same = __ballot(valid);
#pragma unroll
        for (int b = 0; b < 12; ++b) {                          // kSegMaxLeaves = 2^12
            if (b < n_bits) {
                const bool bit = (leaf >> b) & 1;
                const uint64_t m = __ballot(bit);
                same &= bit ? m : ~m;
            }
        }
        if (valid) {
            const int below = __popcll(same & lanes_below(lane));
            const bool last = lane == kWave - 1 || (same >> (lane + 1)) == 0;
            const int32_t pos = start[leaf] + below;
            perm[pos] = (int32_t)t;
            if (slot_leaf) slot_leaf[pos] = leaf;
            if (last) start[leaf] = pos + 1;
        }
    }
}

bool bucket_segments_ok(int64_t T, int depth, const Workspace& ws) {
    const int64_t NL = (int64_t)1 << depth;
    const int64_t n_segs = (T + kSegTokens - 1) / kSegTokens;
    return T > 0 && NL <= kSegMaxLeaves && n_segs <= ws.n_chunks && n_segs < ((int64_t)1 << 31);
}

hipError_t launch_bucket_segments(const int32_t* leaf_idx, int64_t T, int depth, const Workspace& ws,
                                  int32_t* count, int32_t* offset, int32_t* perm, int32_t* slot_leaf,
                                  hipStream_t s) {
    const int64_t NL = (int64_t)1 << depth;
    const int64_t n_segs = (T + kSegTokens - 1) / kSegTokens;
    hipError_t e;
    note_launch("seg_count_kernel + bucket_scan_kernel%s", perm ? " + seg_scatter_kernel" : "");
    seg_count_kernel<<<dim3((unsigned)n_segs), dim3(kWave), 0, s>>>(leaf_idx, T, (int)NL, n_segs, ws.chunk_cnt);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    bucket_scan_kernel<<<dim3((unsigned)((NL + 15) / 16)), dim3(1024), 0, s>>>(
        ws.chunk_cnt, NL, n_segs, kTileRows, count ? count : ws.count, offset ? offset : ws.offset, ws.tile_off,
        ws.ctrl);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    if (perm) {
        seg_scatter_kernel<<<dim3((unsigned)n_segs), dim3(kWave), 0, s>>>(leaf_idx, T, (int)NL, depth, n_segs, ws.chunk_cnt,
                                                                         offset ? offset : ws.offset, perm, slot_leaf);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t launch_bucket(const int32_t* leaf_idx, int64_t T, int depth, const Workspace& ws,
                         int32_t* count, int32_t* offset, int32_t* perm, int32_t* slot_leaf, hipStream_t s) {
    const int64_t NL = (int64_t)1 << depth;
    const int64_t per_round = (T + kChunkTokens - 1) / kChunkTokens;
    const int rounds = (int)((per_round + ws.n_chunks - 1) / ws.n_chunks);
    hipError_t e;
    note_launch("bucket_rank_kernel + bucket_scan_kernel%s", perm ? " + bucket_scatter_kernel" : "");
    if (T > 0) {
        const int64_t blocks = (per_round + rounds - 1) / rounds;
        bucket_rank_kernel<<<dim3((unsigned)blocks), dim3(256), 0, s>>>(leaf_idx, T, rounds, ws.n_chunks,
                                                                       ws.rank, ws.chunk_cnt);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    bucket_scan_kernel<<<dim3((unsigned)((NL + 15) / 16)), dim3(1024), 0, s>>>(
        ws.chunk_cnt, NL, ws.n_chunks, kTileRows, count ? count : ws.count, offset ? offset : ws.offset,
        ws.tile_off, ws.ctrl);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    if (T > 0 && perm) {
        bucket_scatter_kernel<<<dim3((unsigned)((T + 255) / 256)), dim3(256), 0, s>>>(
            leaf_idx, ws.rank, T, rounds, ws.n_chunks, ws.chunk_cnt, offset ? offset : ws.offset, perm, slot_leaf);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace fff
