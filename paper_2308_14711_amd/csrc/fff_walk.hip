// K1 (and, fused, K3 + K4 for narrow leaves) -- the root-to-leaf walk of
// Forward_I (Algorithm 1): d node neurons per token, each a dot product plus
// bias followed by "logit >= 0 -> child 2n+1, else 2n", then optionally the
// leaf network of the leaf reached, written to the token's output row.
//
// Layout of the work
//   - A token is owned by a group of LPT consecutive lanes (one 16-lane DPP row,
//     or the whole wave for long rows); a group carries TPG tokens at once so
//     that TPG independent row fetches are in flight per lane.
//   - The token row is read once from HBM (16 bytes per lane, consecutive lanes
//     on consecutive addresses, streaming hint) and stays in registers for all
//     levels and for the leaf's hidden neurons.
//   - The rows of the top `top` levels of the tree (2^top - 1 rows, the ones
//     every token keeps hitting) are staged in LDS once per block; deeper rows,
//     which few tokens share, are fetched from L2/HBM.
//   - Partial dot products are reduced inside the group with DPP row rotations.
//   - Blocks are persistent: a block owns a contiguous share of the tokens and
//     takes it in equal rounds of at most one tile, so the LDS staging is paid
//     once per block and every block has the same number of tokens per round.
#include "fff_device.h"
#include "fff_internal.h"

namespace fff {

constexpr int kFusedMaxLeafWidth = 8;
constexpr int64_t kLastLevelCacheBytes = (int64_t)256 << 20;   // memory-side cache of the device (not reported by the runtime)

// xv . row, where row[v] is fetched by LOAD(v)
// TIGHT: the row is exactly LPT * NV vectors long, so no lane needs a bounds check.
template <bool BF16, int LPT, int NV, bool TIGHT, typename LoadRow>
__device__ __forceinline__ float row_dot(const uint4 (&xv)[NV], int sub, int nvec, LoadRow load) {
    uint4 wv[NV];
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int v = sub + i * LPT;
        wv[i] = (TIGHT || v < nvec) ? load(v) : make_uint4(0, 0, 0, 0);
    }
    float acc0 = 0.f, acc1 = 0.f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        if (i & 1) acc1 = Elem<BF16>::dot(xv[i], wv[i], acc1);
        else acc0 = Elem<BF16>::dot(xv[i], wv[i], acc0);
    }
    return acc0 + acc1;
}

template <bool BF16> __device__ __forceinline__ void unpack_vec(const uint4& v, float* f);
template <> __device__ __forceinline__ void unpack_vec<false>(const uint4& v, float* f) {
    f[0] = __uint_as_float(v.x); f[1] = __uint_as_float(v.y);
    f[2] = __uint_as_float(v.z); f[3] = __uint_as_float(v.w);
}
template <> __device__ __forceinline__ void unpack_vec<true>(const uint4& v, float* f) {
    f[0] = bf16_lo(v.x); f[1] = bf16_hi(v.x); f[2] = bf16_lo(v.y); f[3] = bf16_hi(v.y);
    f[4] = bf16_lo(v.z); f[5] = bf16_hi(v.z); f[6] = bf16_lo(v.w); f[7] = bf16_hi(v.w);
}
template <bool BF16> __device__ __forceinline__ uint4 pack_vec(const float* f);
template <> __device__ __forceinline__ uint4 pack_vec<false>(const float* f) {
    return make_uint4(__float_as_uint(f[0]), __float_as_uint(f[1]), __float_as_uint(f[2]), __float_as_uint(f[3]));
}
template <> __device__ __forceinline__ uint4 pack_vec<true>(const float* f) {
    return make_uint4(pack_bf16x2(f[0], f[1]), pack_bf16x2(f[2], f[3]), pack_bf16x2(f[4], f[5]),
                      pack_bf16x2(f[6], f[7]));
}

struct WalkArgs {
    const uint4* x;
    const uint4* node_w;
    const void* node_b;
    const uint4* w1;
    const void* b1;
    const void* w2;
    const void* b2;
    void* out;
    int32_t* leaf_idx;   // may be null when FUSED
    int64_t T, O;
    int64_t share;       // tokens per block (the last block may get fewer)
    int chunk;           // tokens per round, at most one tile
    int depth, top, nvec, L, act, out_vec;
    float* hidden_out;       // fused only, may be null: [T, L] hidden activations (fp32) instead of the output rows
    int32_t* block_counts;   // descent only, may be null: [blocks, 2^depth] tokens of every leaf in each block's share
    int plain_x;             // descent only: read the token rows without the streaming hint
};

// MODE: kWalkDescend writes leaf_idx only; kWalkFused also the leaf network (L <= 8) and the output
// row; kWalkHidden the leaf's hidden neurons, stored fp32 for a launch that writes the rows.
// TIGHT: D (and, when fused with vector output, O) is exactly LPT * NV vectors.
constexpr int kWalkDescend = 0, kWalkFused = 1, kWalkHidden = 2;
template <bool BF16, int LPT, int NV, int TPG, int kWalkBlock, int MODE, bool TIGHT, bool PREFETCH>
__global__ __launch_bounds__(kWalkBlock) void walk_kernel(const WalkArgs a) {
    constexpr bool HIDDEN = MODE == kWalkHidden, DESCEND = MODE == kWalkDescend;   // else the fused launch
    extern __shared__ uint4 lds[];                 // [(2^top - 1) * nvec] rows, then (2^top - 1) biases, then the leaf counts
    constexpr int VE = Elem<BF16>::kPerVec;
    const int nvec = a.nvec;
    const int n_top = (1 << a.top) - 1;
    float* lds_bias = (float*)(lds + (int64_t)n_top * nvec);
    // descent feeding the bucketing stage: how many of this block's tokens reach each leaf
    int* lds_hist = (int*)(lds_bias + n_top);
    const bool counting = DESCEND && a.block_counts != nullptr;
    const int n_leaves = 1 << a.depth;

    for (int i = threadIdx.x; i < n_top * nvec; i += kWalkBlock) lds[i] = a.node_w[i];
    for (int i = threadIdx.x; i < n_top; i += kWalkBlock) lds_bias[i] = Elem<BF16>::load(a.node_b, i);
    if (counting)
        for (int i = threadIdx.x; i < n_leaves; i += kWalkBlock) lds_hist[i] = 0;
    __syncthreads();

    const int sub = threadIdx.x % LPT;
    const int g = threadIdx.x / LPT;
    const int n_nodes = (1 << a.depth) - 1;

    // this block's tokens, taken a.chunk at a time: slot g TPG + k of a round holds token
    // base + g TPG + k while that is inside the round and the share (else the last token, unused)
    const int64_t lo = (int64_t)blockIdx.x * a.share;
    const int64_t hi = lo + a.share < a.T ? lo + a.share : a.T;
    auto fetch_rows = [&](int64_t base, uint4 (&xr)[TPG][NV]) {
#pragma unroll
        for (int k = 0; k < TPG; ++k) {
            const int64_t tt = base + (int64_t)g * TPG + k;
            const uint4* xrow = a.x + ((g * TPG + k < a.chunk && tt < hi) ? tt : a.T - 1) * nvec;
#pragma unroll
            for (int i = 0; i < NV; ++i) {
                const int v = sub + i * LPT;
                xr[k][i] = (TIGHT || v < nvec) ? ((DESCEND && a.plain_x) ? xrow[v] : load_stream(xrow + v))
                                               : make_uint4(0, 0, 0, 0);
            }
        }
    };
    const int64_t stride = a.chunk;
    uint4 xv[TPG][NV];
    if (PREFETCH) fetch_rows(lo, xv);

    for (int64_t base = lo; base < hi; base += stride) {
        int64_t t[TPG];
        bool live[TPG];
#pragma unroll
        for (int k = 0; k < TPG; ++k) {
            const int64_t tt = base + (int64_t)g * TPG + k;
            live[k] = g * TPG + k < a.chunk && tt < hi;
            t[k] = live[k] ? tt : a.T - 1;
        }
        // PREFETCH: the rows of this tile were requested one iteration ago; request the next
        // tile's now, so that they travel while this tile walks the tree
        uint4 xn[TPG][NV];
        if (PREFETCH) {
            if (base + stride < hi) fetch_rows(base + stride, xn);
        } else {
            fetch_rows(base, xv);
        }
        int node[TPG];
#pragma unroll
        for (int k = 0; k < TPG; ++k) node[k] = 0;

        // levels whose rows sit in LDS
        for (int m = 0; m < a.top; ++m) {
            float s[TPG];
#pragma unroll
            for (int k = 0; k < TPG; ++k) {
                const uint4* row = lds + (int64_t)node[k] * nvec;
                s[k] = row_dot<BF16, LPT, NV, TIGHT>(xv[k], sub, nvec, [&](int v) { return row[v]; });
            }
#pragma unroll
            for (int k = 0; k < TPG; ++k) {
                const float logit = group_sum<LPT>(s[k]) + lds_bias[node[k]];
                node[k] = 2 * node[k] + 1 + (logit >= 0.0f ? 1 : 0);
            }
        }
        // deeper levels: one row fetch per token per level, TPG of them in flight
        for (int m = a.top; m < a.depth; ++m) {
            float s[TPG], bias[TPG];
#pragma unroll
            for (int k = 0; k < TPG; ++k) {
                const uint4* row = a.node_w + (int64_t)node[k] * nvec;
                bias[k] = Elem<BF16>::load(a.node_b, node[k]);
                s[k] = row_dot<BF16, LPT, NV, TIGHT>(xv[k], sub, nvec, [&](int v) { return row[v]; });
            }
#pragma unroll
            for (int k = 0; k < TPG; ++k) {
                const float logit = group_sum<LPT>(s[k]) + bias[k];
                node[k] = 2 * node[k] + 1 + (logit >= 0.0f ? 1 : 0);
            }
        }
        int64_t leaf[TPG];
#pragma unroll
        for (int k = 0; k < TPG; ++k) {
            leaf[k] = node[k] - n_nodes;
            if (a.leaf_idx && live[k] && sub == 0) a.leaf_idx[t[k]] = (int32_t)leaf[k];
            if (counting && live[k] && sub == 0) atomicAdd(&lds_hist[leaf[k]], 1);
        }
        if (DESCEND) {
            if (PREFETCH) {
#pragma unroll
                for (int k = 0; k < TPG; ++k)
#pragma unroll
                    for (int i = 0; i < NV; ++i) xv[k][i] = xn[k][i];
            }
            continue;
        }

        // hidden neurons of the leaf reached: h[r] = act(W1[leaf][r] . x + b1[leaf][r])
        float h[TPG][kFusedMaxLeafWidth];
#pragma unroll
        for (int r = 0; r < kFusedMaxLeafWidth; ++r) {
            if (r < a.L) {
                float s[TPG], bias[TPG];
#pragma unroll
                for (int k = 0; k < TPG; ++k) {
                    const uint4* row = a.w1 + (leaf[k] * a.L + r) * nvec;
                    bias[k] = Elem<BF16>::load(a.b1, leaf[k] * a.L + r);
                    s[k] = row_dot<BF16, LPT, NV, TIGHT>(xv[k], sub, nvec, [&](int v) { return row[v]; });
                }
#pragma unroll
                for (int k = 0; k < TPG; ++k) h[k][r] = activate(group_sum<LPT>(s[k]) + bias[k], a.act);
            } else {
#pragma unroll
                for (int k = 0; k < TPG; ++k) h[k][r] = 0.f;
            }
        }
        if (HIDDEN) {
            // the output rows are left to a launch of their own (leaf_slices_kernel): lane r of the
            // group stores the r-th hidden activation, fp32 as it stands in the registers
#pragma unroll
            for (int k = 0; k < TPG; ++k) {
                float hv = h[k][0];
#pragma unroll
                for (int q = 1; q < kFusedMaxLeafWidth; ++q) hv = q == sub ? h[k][q] : hv;
                if (live[k] && sub < a.L) a.hidden_out[t[k] * a.L + sub] = hv;
            }
            if (PREFETCH) {
#pragma unroll
                for (int k = 0; k < TPG; ++k)
#pragma unroll
                    for (int i = 0; i < NV; ++i) xv[k][i] = xn[k][i];
            }
            continue;
        }
        // output row: y[o] = sum_r h[r] W2[leaf][r][o] + b2[leaf][o]
#pragma unroll
        for (int k = 0; k < TPG; ++k) {
            if (!live[k]) continue;
            if (a.out_vec) {
                // NV vectors per lane at a time, all of a row's fetches issued before they are used
                const int ovec = (int)(a.O / VE);
                const uint4* w2v = (const uint4*)a.w2 + leaf[k] * a.L * ovec;
                const uint4* b2v = (const uint4*)a.b2 + leaf[k] * ovec;
                uint4* orow = (uint4*)a.out + t[k] * ovec;
                for (int ov0 = sub; ov0 < ovec + sub; ov0 += LPT * NV) {
                    uint4 bv[NV], wv[NV];
#pragma unroll
                    for (int i = 0; i < NV; ++i) {
                        const int ov = ov0 + i * LPT;
                        const bool ok = TIGHT || ov < ovec;
                        bv[i] = ok ? b2v[ov] : make_uint4(0, 0, 0, 0);
                        wv[i] = ok ? w2v[ov] : make_uint4(0, 0, 0, 0);
                    }
                    float acc[NV][VE];
#pragma unroll
                    for (int i = 0; i < NV; ++i) {
                        float wf[VE];
                        unpack_vec<BF16>(bv[i], acc[i]);
                        unpack_vec<BF16>(wv[i], wf);
#pragma unroll
                        for (int e = 0; e < VE; ++e) acc[i][e] = fmaf(h[k][0], wf[e], acc[i][e]);
                    }
                    for (int r = 1; r < a.L; ++r) {
#pragma unroll
                        for (int i = 0; i < NV; ++i) {
                            const int ov = ov0 + i * LPT;
                            wv[i] = (TIGHT || ov < ovec) ? w2v[(int64_t)r * ovec + ov] : make_uint4(0, 0, 0, 0);
                        }
                        float hr = h[k][0];
#pragma unroll
                        for (int q = 1; q < kFusedMaxLeafWidth; ++q) hr = q == r ? h[k][q] : hr;
#pragma unroll
                        for (int i = 0; i < NV; ++i) {
                            float wf[VE];
                            unpack_vec<BF16>(wv[i], wf);
#pragma unroll
                            for (int e = 0; e < VE; ++e) acc[i][e] = fmaf(hr, wf[e], acc[i][e]);
                        }
                    }
#pragma unroll
                    for (int i = 0; i < NV; ++i) {
                        const int ov = ov0 + i * LPT;
                        if (TIGHT || ov < ovec) store_stream(orow + ov, pack_vec<BF16>(acc[i]));
                    }
                }
            } else {
                for (int64_t o = sub; o < a.O; o += LPT) {
                    float acc = Elem<BF16>::load(a.b2, leaf[k] * a.O + o);
#pragma unroll
                    for (int r = 0; r < kFusedMaxLeafWidth; ++r)
                        if (r < a.L) acc = fmaf(h[k][r], Elem<BF16>::load(a.w2, (leaf[k] * a.L + r) * a.O + o), acc);
                    Elem<BF16>::store(a.out, t[k] * a.O + o, acc);
                }
            }
        }
        if (PREFETCH) {
#pragma unroll
            for (int k = 0; k < TPG; ++k)
#pragma unroll
                for (int i = 0; i < NV; ++i) xv[k][i] = xn[k][i];
        }
    }
    if (counting) {
        __syncthreads();
        int32_t* row = a.block_counts + (int64_t)blockIdx.x * n_leaves;
        for (int i = threadIdx.x; i < n_leaves; i += kWalkBlock) row[i] = lds_hist[i];
    }
}

// Any D, any alignment: one wave per token, element-wise loads.
template <bool BF16>
__global__ __launch_bounds__(256) void descend_generic_kernel(const void* __restrict__ x,
                                                              const void* __restrict__ node_w,
                                                              const void* __restrict__ node_b,
                                                              int depth, int64_t T, int64_t D,
                                                              int32_t* __restrict__ leaf_idx) {
    const int lane = threadIdx.x % kWave;
    const int64_t t = (int64_t)blockIdx.x * (256 / kWave) + threadIdx.x / kWave;
    if (t >= T) return;
    int node = 0;
    for (int m = 0; m < depth; ++m) {
        float acc = 0.f;
        for (int64_t j = lane; j < D; j += kWave)
            acc = fmaf(Elem<BF16>::load(x, t * D + j), Elem<BF16>::load(node_w, (int64_t)node * D + j), acc);
        const float logit = group_sum<64>(acc) + Elem<BF16>::load(node_b, node);
        node = 2 * node + 1 + (logit >= 0.0f ? 1 : 0);
    }
    if (lane == 0) leaf_idx[t] = node - ((1 << depth) - 1);
}

// D % (16 bytes of elements) == 0 and all row starts 16-byte aligned.
bool vec_ok(const void* p, int64_t row_elems, bool bf16) {
    const int per = bf16 ? 8 : 4;
    return (reinterpret_cast<uintptr_t>(p) & 15u) == 0 && row_elems % per == 0;
}

DeviceInfo device_info() {
    static DeviceInfo info[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return DeviceInfo{256, 64 * 1024, 0, 4 << 20};
    if (info[dev].cus == 0) {
        hipDeviceProp_t p;
        if (hipGetDeviceProperties(&p, dev) == hipSuccess) {
            info[dev].cus = p.multiProcessorCount > 0 ? p.multiProcessorCount : 256;
            info[dev].lds_per_block = p.sharedMemPerBlockOptin > 0 ? p.sharedMemPerBlockOptin : p.sharedMemPerBlock;
            info[dev].l2_bytes = p.l2CacheSize > 0 ? p.l2CacheSize : 4 << 20;
        } else {
            (void)hipGetLastError();
            info[dev] = DeviceInfo{256, 64 * 1024, 0, 4 << 20};
        }
        info[dev].dev = dev;
    }
    return info[dev];
}

WalkTuning g_walk_tuning;
namespace {

// set by launch_descend for the duration of its dispatch: where the launch may leave per-block leaf counts
thread_local DescentCounts* t_counts = nullptr;
// set by launch_walk_hidden for the duration of its dispatch: where the fused launch leaves the hidden
// activations instead of writing output rows
thread_local float* t_hidden_out = nullptr;

template <bool BF16, int LPT, int NV, int TPG, int kWalkBlock, int MODE, bool TIGHT, bool PREFETCH = false>
hipError_t run_walk_t(const Problem& p, int32_t* leaf_idx, hipStream_t s) {
    constexpr bool FUSED = MODE == kWalkFused, HIDDEN = MODE == kWalkHidden;
    constexpr int kGroups = kWalkBlock / LPT;
    const DeviceInfo di = device_info();
    const int64_t tile = (int64_t)kGroups * TPG;
    // a block is worth starting for 32 tokens (or a tile, if that is smaller)
    const int64_t min_share = tile < 32 ? tile : 32;
    int64_t blocks = (p.T + min_share - 1) / min_share;
    const int64_t cap = (int64_t)di.cus * (g_walk_tuning.bpc > 0 ? g_walk_tuning.bpc : 1);
    if (blocks > cap) blocks = cap;
    // equal contiguous shares, each taken in equal rounds of at most one tile (a multiple of the
    // tokens a lane group carries)
    const int64_t tokens_per_block = (p.T + blocks - 1) / blocks;
    blocks = (p.T + tokens_per_block - 1) / tokens_per_block;
    const int64_t rounds = (tokens_per_block + tile - 1) / tile;
    int64_t chunk = ((tokens_per_block + rounds - 1) / rounds + TPG - 1) / TPG * TPG;
    if (chunk > tile) chunk = tile;
    // a descent that feeds the bucketing stage also counts, per block, the tokens of every leaf
    // (one LDS counter per leaf), when the tree and the shares are small enough for the fold kernel
    DescentCounts* dc = MODE == kWalkDescend ? t_counts : nullptr;
    size_t hist_bytes = 0;
    if (dc) {
        dc->blocks = 0;
        if (dc->M && bucket_fold_ok(p.depth, blocks, tokens_per_block) &&
            (blocks << p.depth) <= dc->capacity) {
            hist_bytes = sizeof(int32_t) << p.depth;
            dc->blocks = (int)blocks;
            dc->share = tokens_per_block;
        }
    }
    // stage the top levels while a block handles at least two tokens per staged row and they fit
    const int64_t row_bytes = p.D * (BF16 ? 2 : 4);
    size_t lds_cap = di.lds_per_block;
    if (lds_cap > 144 * 1024) lds_cap = 144 * 1024;
    lds_cap -= hist_bytes;
    int top = 0;
    while (top < p.depth) {
        const int64_t rows = ((int64_t)1 << (top + 1)) - 1;
        if (rows * 2 > tokens_per_block || (size_t)(rows * (row_bytes + 4)) > lds_cap) break;
        ++top;
    }
    if (g_walk_tuning.top > 0 && g_walk_tuning.top - 1 < top) top = (int)g_walk_tuning.top - 1;
    const size_t lds_bytes = (size_t)(((int64_t)1 << top) - 1) * (row_bytes + 4) + hist_bytes;
    auto kern = walk_kernel<BF16, LPT, NV, TPG, kWalkBlock, MODE, TIGHT, PREFETCH>;
    // raise this instantiation's dynamic LDS limit once per device (the limit only ever grows)
    static size_t lds_allowed_on[64];
    size_t& lds_allowed = lds_allowed_on[di.dev];
    if (lds_bytes > 48 * 1024 && lds_bytes > lds_allowed) {
        const size_t lds_max = lds_cap + hist_bytes;
        hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                           (int)lds_max);
        if (e != hipSuccess) return e;
        lds_allowed = lds_max;
    }
    WalkArgs a;
    a.x = (const uint4*)p.x;
    a.node_w = (const uint4*)p.node_w;
    a.node_b = p.node_b;
    a.w1 = (const uint4*)p.leaf_w1;
    a.b1 = p.leaf_b1;
    a.w2 = p.leaf_w2;
    a.b2 = p.leaf_b2;
    a.out = p.out;
    a.leaf_idx = leaf_idx;
    a.T = p.T;
    a.O = p.O;
    a.share = tokens_per_block;
    a.chunk = (int)chunk;
    a.depth = p.depth;
    a.top = top;
    g_walk_tuning.last_top = top;
    a.nvec = (int)(p.D / Elem<BF16>::kPerVec);
    a.L = p.L;
    a.act = p.act;
    a.out_vec = FUSED && vec_ok(p.out, p.O, BF16) && vec_ok(p.leaf_w2, p.O, BF16) && vec_ok(p.leaf_b2, p.O, BF16);
    a.block_counts = hist_bytes ? dc->M : nullptr;
    a.hidden_out = HIDDEN ? t_hidden_out : nullptr;
    // The descent of the staged path is followed by a leaf kernel that reads the same token rows
    // again: without the streaming hint they stay in the last-level cache for it (the ViT-block
    // workload: hidden kernel 19.9 -> 18.3 us, descent 25.0 -> 25.6).  Batches that cannot stay there
    // anyway (more than half of its 256 MB) keep the hint.
    const int64_t x_bytes = p.T * row_bytes;
    a.plain_x = g_walk_tuning.plain_x == 1 || (g_walk_tuning.plain_x == 0 && x_bytes <= kLastLevelCacheBytes / 2);
    note_launch("walk_kernel<%s,%d,%d,%d,%d,%s,%s%s> top=%d", BF16 ? "bf16" : "f32", LPT, NV, TPG, kWalkBlock,
                FUSED ? "fused" : HIDDEN ? "walk+hidden" : (hist_bytes ? "descent+counts" : "descent"),
                TIGHT ? "tight" : "checked",
                PREFETCH ? ",prefetch" : "", top);
    kern<<<dim3((unsigned)blocks), dim3(kWalkBlock), lds_bytes, s>>>(a);
    return hipGetLastError();
}

template <bool BF16, int LPT, int NV, int TPG, int kWalkBlock, int MODE>
hipError_t run_walk(const Problem& p, int32_t* leaf_idx, hipStream_t s) {
    constexpr bool FUSED = MODE == kWalkFused;
    const int64_t per = Elem<BF16>::kPerVec;
    const bool out_vec = FUSED && vec_ok(p.out, p.O, BF16) && vec_ok(p.leaf_w2, p.O, BF16) && vec_ok(p.leaf_b2, p.O, BF16);
    const bool tight = p.D == per * LPT * NV && (!FUSED || !out_vec || p.O == per * LPT * NV);
    return tight ? run_walk_t<BF16, LPT, NV, TPG, kWalkBlock, MODE, true>(p, leaf_idx, s)
                 : run_walk_t<BF16, LPT, NV, TPG, kWalkBlock, MODE, false>(p, leaf_idx, s);
}

template <bool BF16, int MODE>
hipError_t dispatch_walk(const Problem& p, int32_t* leaf_idx, hipStream_t s) {
    constexpr bool FUSED = MODE == kWalkFused;     // the walk + hidden launch takes the descent's tiles
    const int64_t nvec = p.D / Elem<BF16>::kPerVec;
    // (lanes per token, 16-byte vectors per lane, tokens per group, block size): blocks of 1024
    // threads leave 128 VGPRs per lane, blocks of 512 leave 256 for the long-row variants
    // A block's tile is (threads / lanes per token) x (tokens per group) tokens; a batch of up to
    // 32 tokens per compute unit is cut into tiles of 32, so that it still spreads over the chip.
    // (Rows of up to 64 vectors have no tile in between and keep the small one up to two tiles
    // per compute unit.)
    const bool untuned = g_walk_tuning.tpg == 0 && g_walk_tuning.block == 0;
    const int64_t cus = device_info().cus;
    const bool small_batch = untuned && p.T <= 32 * cus, smallish_batch = untuned && p.T <= 64 * cus;
    if (nvec <= 16) return smallish_batch ? run_walk<BF16, 16, 1, 1, 512, MODE>(p, leaf_idx, s)
                                          : run_walk<BF16, 16, 1, 4, 1024, MODE>(p, leaf_idx, s);
    if (nvec <= 32) return smallish_batch ? run_walk<BF16, 16, 2, 1, 512, MODE>(p, leaf_idx, s)
                                          : run_walk<BF16, 16, 2, 2, 1024, MODE>(p, leaf_idx, s);
    if (nvec <= 64) return smallish_batch ? run_walk<BF16, 16, 4, 1, 512, MODE>(p, leaf_idx, s)
                                          : run_walk<BF16, 16, 4, 2, 1024, MODE>(p, leaf_idx, s);
    if (nvec <= 96) {
        const int64_t tpg = g_walk_tuning.tpg, blk = g_walk_tuning.block;
        if (tpg == 1 && blk == 512) return run_walk<BF16, 16, 6, 1, 512, MODE>(p, leaf_idx, s);
        // measured best for the fused launch on 768-wide rows: blocks of 512 (256 VGPRs per lane) with
        // four tokens per lane group (82 us on the BERT-base-sized workload, against 83 with two and
        // 86 with two plus the next tile's rows requested one iteration ahead); the descent-only
        // launch is fastest with blocks of 1024 and two tokens per group
        const bool exact = nvec == 96 && FUSED && p.O == p.D && vec_ok(p.out, p.O, BF16) &&
                           vec_ok(p.leaf_w2, p.O, BF16) && vec_ok(p.leaf_b2, p.O, BF16);
        if (exact && g_walk_tuning.prefetch)
            return run_walk_t<BF16, 16, 6, 2, 512, MODE, true, true>(p, leaf_idx, s);
        if (tpg == 0 && blk == 0) {
            // at most one tile per compute unit before tiles get larger: 32 tokens a block up
            // to 8192 tokens, 64 up to 16384, then 128 (fused launch, depth 11, one neuron a leaf:
            // 2048 tokens 9.5 us against 23.4 with tiles of 128, 8192 tokens 14.8 against 30.3,
            // 16384 tokens 24.3 against 32.7, 24576 tokens 37.1 with tiles of 64 against 35.7).
            if (p.T <= 32 * cus) return run_walk<BF16, 16, 6, 1, 512, MODE>(p, leaf_idx, s);
            if (p.T <= 64 * cus) return run_walk<BF16, 16, 6, 1, 1024, MODE>(p, leaf_idx, s);
            if (FUSED) {
                // Beyond that a block takes its share in several rounds, and a round costs about
                // the same whether its tile is full or not: up to 512 tokens per compute unit a
                // smaller tile is taken where rounds x tile comes out 15 % shorter (18000-24576
                // tokens: tiles of 96, 27-35 us against 33-37; 40000 tokens: tiles of 32, 54 us
                // against 62-66; 80000 tokens: tiles of 64, 88-98 us against 99-102).
                const int64_t share = (p.T + cus - 1) / cus;
                const auto busy = [&](int64_t tile) { return (share + tile - 1) / tile * tile; };
                int64_t tile = 128;
                if (p.T <= 512 * cus)
                    for (const int64_t cand : {(int64_t)96, (int64_t)64, (int64_t)32})
                        if (busy(cand) * 115 <= busy(tile) * 100) tile = cand;
                if (tile == 96) return run_walk<BF16, 16, 6, 3, 512, MODE>(p, leaf_idx, s);
                if (tile == 64) return run_walk<BF16, 16, 6, 2, 512, MODE>(p, leaf_idx, s);
                if (tile == 32) return run_walk<BF16, 16, 6, 1, 512, MODE>(p, leaf_idx, s);
                return run_walk<BF16, 16, 6, 4, 512, MODE>(p, leaf_idx, s);
            }
        }
        if (tpg == 1) return run_walk<BF16, 16, 6, 1, 1024, MODE>(p, leaf_idx, s);
        if (tpg == 2 && blk == 512) return run_walk<BF16, 16, 6, 2, 512, MODE>(p, leaf_idx, s);
        if (tpg == 4 && blk == 512) return run_walk<BF16, 16, 6, 4, 512, MODE>(p, leaf_idx, s);
        if (tpg == 3 && blk == 512) return run_walk<BF16, 16, 6, 3, 512, MODE>(p, leaf_idx, s);
        if (tpg == 4 && blk == 256) return run_walk<BF16, 16, 6, 4, 256, MODE>(p, leaf_idx, s);
        return run_walk<BF16, 16, 6, 2, 1024, MODE>(p, leaf_idx, s);
    }
    if (nvec <= 128) return small_batch ? run_walk<BF16, 16, 8, 1, 512, MODE>(p, leaf_idx, s)
                                        : run_walk<BF16, 16, 8, 2, 512, MODE>(p, leaf_idx, s);
    if (nvec <= 256) return run_walk<BF16, 64, 4, 2, 1024, MODE>(p, leaf_idx, s);
    if (nvec <= 512) {
        const int64_t tpg = g_walk_tuning.tpg, blk = g_walk_tuning.block;
        if (tpg == 1 && blk == 1024) return run_walk<BF16, 64, 8, 1, 1024, MODE>(p, leaf_idx, s);
        if (tpg == 3 && blk == 512) return run_walk<BF16, 64, 8, 3, 512, MODE>(p, leaf_idx, s);
        if (tpg == 4 && blk == 256) return run_walk<BF16, 64, 8, 4, 256, MODE>(p, leaf_idx, s);
        if (tpg == 6 && blk == 256) return run_walk<BF16, 64, 8, 6, 256, MODE>(p, leaf_idx, s);
        return run_walk<BF16, 64, 8, 2, 512, MODE>(p, leaf_idx, s);
    }
    return run_walk<BF16, 64, 16, 1, 512, MODE>(p, leaf_idx, s);
}

}  // namespace

bool walk_shape_ok(const Problem& p) {
    const int64_t per = p.bf16 ? 8 : 4;
    return vec_ok(p.x, p.D, p.bf16) && (p.depth == 0 || vec_ok(p.node_w, p.D, p.bf16)) && p.D / per <= 1024;
}

bool fused_shape_ok(const Problem& p) {
    return walk_shape_ok(p) && vec_ok(p.leaf_w1, p.D, p.bf16) && p.L <= kFusedMaxLeafWidth;
}

hipError_t launch_descend(const Problem& p, int32_t* leaf_idx, hipStream_t s, DescentCounts* dc) {
    if (dc) dc->blocks = 0;
    if (p.T == 0) return hipSuccess;
    if (walk_shape_ok(p)) {
        t_counts = dc;
        const hipError_t e = p.bf16 ? dispatch_walk<true, kWalkDescend>(p, leaf_idx, s) : dispatch_walk<false, kWalkDescend>(p, leaf_idx, s);
        t_counts = nullptr;
        return e;
    }
    const int64_t blocks = (p.T + 3) / 4;
    note_launch("descend_generic_kernel<%s>", p.bf16 ? "bf16" : "f32");
    if (p.bf16)
        descend_generic_kernel<true><<<dim3((unsigned)blocks), dim3(256), 0, s>>>(p.x, p.node_w, p.node_b, p.depth,
                                                                                 p.T, p.D, leaf_idx);
    else
        descend_generic_kernel<false><<<dim3((unsigned)blocks), dim3(256), 0, s>>>(p.x, p.node_w, p.node_b, p.depth,
                                                                                  p.T, p.D, leaf_idx);
    return hipGetLastError();
}

// Descent, leaf network and output row in one launch (needs fused_shape_ok).
hipError_t launch_walk_fused(const Problem& p, int32_t* leaf_idx, hipStream_t s) {
    if (p.T == 0) return hipSuccess;
    return p.bf16 ? dispatch_walk<true, kWalkFused>(p, leaf_idx, s) : dispatch_walk<false, kWalkFused>(p, leaf_idx, s);
}

// The same launch stopping after the leaf's hidden neurons: leaf_idx [T] (required) and hidden [T, L]
// (fp32) are left for launch_leaf_slices.
hipError_t launch_walk_hidden(const Problem& p, int32_t* leaf_idx, float* hidden, hipStream_t s) {
    if (p.T == 0) return hipSuccess;
    if (!leaf_idx || !hidden) return hipErrorInvalidValue;
    t_hidden_out = hidden;
    const hipError_t e = p.bf16 ? dispatch_walk<true, kWalkHidden>(p, leaf_idx, s)
                                : dispatch_walk<false, kWalkHidden>(p, leaf_idx, s);
    t_hidden_out = nullptr;
    return e;
}

}  // namespace fff
