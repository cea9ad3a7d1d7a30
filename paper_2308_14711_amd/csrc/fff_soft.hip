// The soft forward pass of an FFF -- Forward_T of Algorithm 1: every node gives a choice score
// c = sigmoid(w . x + b), the leaves are mixed with the products of the scores along their paths
// (the stochastic vector over the leaves), out = sum_leaf mix[leaf] * Leaf_leaf(x).  This is the
// pass used in training and for the hardening diagnostics (batch mean entropy of the choice
// scores per node, paragraph "Hardening"); unlike Forward_I it is dense, so it runs on the matrix
// cores as three contractions over the shared 64 x 128 MFMA tile:
//
//   nodes   C[t][n]   = sigmoid(x[t] . node_w[n] + node_b[n])                       fp32, [T, 2^d - 1]
//   mix     M[t][l]   = prod over the path of leaf l of (bit ? c : 1 - c)           fp32, [T, 2^d]
//   hidden  H[t][k]   = act(x[t] . W1[k] + b1[k]) * M[t][k / l]   (k = leaf * l + neuron)   bf16
//           H[t][2^d l + leaf] = M[t][leaf]                          (carries the output bias)
//   out     out[t][o] = H[t] . W2x[o]   with W2x[o] = (W2[.][o], b2[.][o]): W2 and b2 transposed
//                                                                     once per call into [O, K2]
//
// so that the weighting by the mixture and the bias both ride inside the last contraction.
#include "fff_device.h"
#include "fff_internal.h"
#include "fff_mfma_tile.h"

namespace fff {
int64_t g_soft_small_tiles = 0;     // experiment switch: 1 = the 64 x 128 tile for every contraction
namespace {

struct SoftArgs {
    const uint16_t* x;
    const uint16_t* node_w;
    const uint16_t* node_b;
    const uint16_t* w1;
    const uint16_t* b1;
    const uint16_t* w2;
    const uint16_t* b2;
    float* choice;        // [T][NL]: NN scores per row, pitch NL so that rows start 16-byte aligned
    float* mix;           // [T][NL]
    uint16_t* hid;        // [T][K2]
    uint16_t* w2x;        // [O][K2]
    uint16_t* out;        // [T][O]
    int64_t T;
    int D, O, depth, L, act;
    int64_t NN, NL, K2;   // K2 = NL * (L + 1) rounded up to a multiple of 8
};

__device__ __forceinline__ int64_t tile_row0(int64_t n_col_blocks) { return (int64_t)(blockIdx.x / n_col_blocks) * kTileM; }
__device__ __forceinline__ int64_t tile_col0(int64_t n_col_blocks) { return (int64_t)(blockIdx.x % n_col_blocks) * kTileN; }

// nodes: choice scores
__global__ __launch_bounds__(256) void soft_nodes_kernel(const SoftArgs a) {
    __shared__ TileLds tile;
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6, j = lane & 15, kg = lane >> 4;
    const int64_t ncb = (a.NN + kTileN - 1) / kTileN;
    const int64_t t0 = tile_row0(ncb), n0 = tile_col0(ncb);
    f32x4_t acc[4][2];
    mfma_tile_64x128<2>(a.x, a.D, a.T, a.node_w, a.D, a.NN, a.D, t0, n0, tile, acc);
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) {
        const int64_t n = n0 + 32 * wv + 16 * nt + j;
        if (n >= a.NN) continue;
        const float b = bf16_to_f32(a.node_b[n]);
#pragma unroll
        for (int mt = 0; mt < 4; ++mt)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int64_t t = t0 + 16 * mt + 4 * kg + q;
                if (t < a.T) a.choice[t * a.NL + n] = 1.0f / (1.0f + __expf(-(acc[mt][nt][q] + b)));
            }
    }
}

// entropy of a Bernoulli variable of parameter c, natural logarithm
__device__ __forceinline__ float bernoulli_entropy(float c) {
    const float h0 = c > 0.0f ? -c * __logf(c) : 0.0f;
    const float h1 = c < 1.0f ? -(1.0f - c) * __logf(1.0f - c) : 0.0f;
    return h0 + h1;
}

// mixture weights: one thread per (token, leaf); also the bias columns of the hidden matrix
__global__ __launch_bounds__(256) void soft_mix_kernel(const SoftArgs a) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= a.T * a.NL) return;
    const int64_t t = i / a.NL, leaf = i % a.NL;
    const float* c = a.choice + t * a.NL;
    float m = 1.0f;
    for (int lvl = 0; lvl < a.depth; ++lvl) {
        const int64_t pos = leaf >> (a.depth - lvl);                  // the path's node at this level
        const int bit = (int)((leaf >> (a.depth - 1 - lvl)) & 1);
        const float cs = c[(((int64_t)1 << lvl) - 1) + pos];
        m *= bit ? cs : 1.0f - cs;
    }
    a.mix[i] = m;
    a.hid[t * a.K2 + a.NL * a.L + leaf] = f32_to_bf16(m);
    // the padding columns up to K2 (fewer than 8) are cleared by the thread of leaf 0
    if (leaf == 0)
        for (int64_t k = a.NL * (a.L + 1); k < a.K2; ++k) a.hid[t * a.K2 + k] = 0;
}

// The same for trees of up to 2048 leaves, a wave per token: the products grow level by level in a
// wave-private LDS row (entry n of level m = entry n / 2 of level m - 1 times c or 1 - c of that
// node), so a token's scores are read once instead of once per leaf and level; the factors are
// multiplied in the same order as above (root first): same bits.  The scores themselves come in
// through registers, all of a token's loads in flight at once and the next token's requested before
// this token's levels are walked (a load inside the level loop is a trip to memory per iteration),
// and are parked in a third LDS row for the levels to index.  LDS: 3 NL floats per wave; blocks of
// four waves, or of two for 2048 leaves (48 KB either way at most).
constexpr int kMixMaxLeaves = 2048;
constexpr int kMixRegs = kMixMaxLeaves / kWave;          // scores a lane holds for one token
__global__ __launch_bounds__(256) void soft_mix_rows_kernel(const SoftArgs a) {
    extern __shared__ float mix_lds[];                       // per wave: the scores, then two rows of NL products
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6, waves = blockDim.x >> 6;
    const int NL = (int)a.NL, NN = (int)a.NN;
    float* sc = mix_lds + (size_t)wv * 3 * NL;
    float* cur = sc + NL;
    float* nxt = cur + NL;
    const int per_lane = (NN + kWave - 1) / kWave;           // <= kMixRegs
    float creg[kMixRegs];
    const auto request = [&](int64_t t) {
        const float* c = a.choice + t * a.NL;
#pragma unroll
        for (int i = 0; i < kMixRegs; ++i)
            if (i < per_lane) creg[i] = lane + kWave * i < NN ? c[lane + kWave * i] : 0.0f;
    };
    const int64_t first = (int64_t)blockIdx.x * waves + wv, step = (int64_t)gridDim.x * waves;
    if (first < a.T) request(first);
    for (int64_t t = first; t < a.T; t += step) {
#pragma unroll
        for (int i = 0; i < kMixRegs; ++i)
            if (i < per_lane && lane + kWave * i < NN) sc[lane + kWave * i] = creg[i];
        if (t + step < a.T) request(t + step);               // travels while this token's levels are walked
        if (lane == 0) cur[0] = 1.0f;
        __builtin_amdgcn_wave_barrier();
        for (int lvl = 0; lvl < a.depth; ++lvl) {
            const int n_nodes = 1 << lvl;                    // nodes of this level; 2 n_nodes entries come out
            const float* cl = sc + (n_nodes - 1);
            for (int e = lane; e < 2 * n_nodes; e += kWave) {
                const float cs = cl[e >> 1];
                nxt[e] = cur[e >> 1] * ((e & 1) ? cs : 1.0f - cs);
            }
            __builtin_amdgcn_wave_barrier();                 // LDS executes a wave's accesses in order
            float* tmp = cur; cur = nxt; nxt = tmp;
        }
        for (int leaf = lane; leaf < NL; leaf += kWave) {
            const float m = cur[leaf];
            __builtin_nontemporal_store(m, a.mix + t * a.NL + leaf);
            __builtin_nontemporal_store(f32_to_bf16(m), a.hid + t * a.K2 + a.NL * a.L + leaf);
        }
        for (int64_t k = a.NL * (a.L + 1) + lane; k < a.K2; k += kWave) a.hid[t * a.K2 + k] = 0;
        __builtin_amdgcn_wave_barrier();
    }
}

// hidden: act(x . W1 + b1) scaled by the mixture weight of the neuron's leaf
__global__ __launch_bounds__(256) void soft_hidden_kernel(const SoftArgs a) {
    __shared__ TileLds tile;
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6, j = lane & 15;
    const int64_t NH = a.NL * a.L;
    const int64_t ncb = (NH + kTileN - 1) / kTileN;
    const int64_t t0 = tile_row0(ncb), n0 = tile_col0(ncb);
    f32x4_t acc[4][2];
    mfma_tile_64x128<2>(a.x, a.D, a.T, a.w1, a.D, NH, a.D, t0, n0, tile, acc);
    // the mixture weights this tile needs (64 tokens x the leaves of its 128 columns, at most 128)
    // go through the second tile buffer, read along a row of the weights
    float* mixt = (float*)tile.b;
    const int64_t last = n0 + kTileN - 1 < NH - 1 ? n0 + kTileN - 1 : NH - 1;
    const int64_t leaf_lo = n0 / a.L;
    const int n_leaf = (int)(last / a.L - leaf_lo + 1);
    for (int idx = threadIdx.x; idx < kTileM * n_leaf; idx += 256) {
        const int r = idx / n_leaf, c = idx % n_leaf;
        mixt[idx] = t0 + r < a.T ? a.mix[(t0 + r) * a.NL + leaf_lo + c] : 0.0f;
    }
    float bias[2];
    int lcol[2];
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) {
        const int64_t n = n0 + 32 * wv + 16 * nt + j;
        bias[nt] = n < NH ? bf16_to_f32(a.b1[n]) : 0.0f;
        lcol[nt] = n < NH ? (int)(n / a.L - leaf_lo) : 0;
    }
    __syncthreads();
    tile_store_bf16(tile, acc, a.hid, a.K2, a.T, NH, t0, n0, [&](int r, int c, float v) {
        const int nt = (c >> 4) & 1;
        return activate_bulk(v + bias[nt], a.act) * mixt[r * n_leaf + lcol[nt]];
    });
}

// The same two contractions over the 128 x 256 tile (batches and widths that fill it).
// Block -> tile so that the column tiles of one row tile run back to back on ONE XCD (blocks are
// dealt to the 8 XCDs round robin): the first of them brings the row tile's A rows into that
// XCD's L2, the others hit there instead of fetching them again from memory.  Row tile
// 8 (i / ncb) + xcd, column tile i % ncb for the i-th block of an XCD; the grid is rounded up to
// whole groups of 8 row tiles and blocks past the last row tile leave at once.
__device__ __forceinline__ bool big_tile_of_block(int64_t ncb, int64_t M, int64_t& m0, int64_t& n0) {
    const int64_t xcd = blockIdx.x & 7, i = blockIdx.x >> 3;
    m0 = (8 * (i / ncb) + xcd) * kBigM;
    n0 = (i % ncb) * kBigN;
    return m0 < M;
}
inline unsigned big_grid(int64_t M, int64_t ncb) {
    const int64_t row_tiles = (M + kBigM - 1) / kBigM;
    return (unsigned)(((row_tiles + 7) / 8) * 8 * ncb);
}

__global__ __launch_bounds__(256, 2) void soft_nodes_big_kernel(const SoftArgs a) {
    __shared__ BigTileLds tile;
    const int64_t ncb = (a.NN + kBigN - 1) / kBigN;
    int64_t t0, n0;
    if (!big_tile_of_block(ncb, a.T, t0, n0)) return;
    f32x4_t acc[4][8];
    mfma_tile_128x256(a.x, a.D, a.T, a.node_w, a.D, a.NN, a.D, t0, n0, tile, acc);
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6, j = lane & 15, kg = lane >> 4;
    const int wm = wv >> 1, wn = wv & 1;
#pragma unroll
    for (int nt = 0; nt < 8; ++nt) {
        const int64_t n = n0 + 128 * wn + 16 * nt + 4 * kg;          // this lane's nodes n .. n + 3
        if (n >= a.NL) continue;                                     // (the row's last float, past the NN scores, is padding)
        float b[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) b[q] = n + q < a.NN ? bf16_to_f32(a.node_b[n + q]) : 0.0f;
#pragma unroll
        for (int mt = 0; mt < 4; ++mt) {
            const int64_t t = t0 + 64 * wm + 16 * mt + j;
            if (t >= a.T) continue;
            float4 c;
            c.x = 1.0f / (1.0f + __expf(-(acc[mt][nt][0] + b[0])));
            c.y = 1.0f / (1.0f + __expf(-(acc[mt][nt][1] + b[1])));
            c.z = 1.0f / (1.0f + __expf(-(acc[mt][nt][2] + b[2])));
            c.w = 1.0f / (1.0f + __expf(-(acc[mt][nt][3] + b[3])));
            // NL >= 256 here: a multiple of 4, rows 16-byte aligned; read once by the mixture launch
            __builtin_nontemporal_store(f32x4_t{c.x, c.y, c.z, c.w}, (f32x4_t*)(a.choice + t * a.NL + n));
        }
    }
}

// Trees of up to 256 leaves (all nodes in one column tile): the node contraction, the mixture weights and
// the entropy sums in one launch -- the scores never go to memory.  After the contraction the tile's
// scores pass through LDS 64 rows at a time (column n of row r at 256 r + (n xor 4 (r mod 16)): a lane
// stores its four consecutive columns as 16 bytes, the 16 lanes of a group are 16 rows on equal
// columns, and the xor on the 16-byte piece index spreads them over the banks; the readers below run
// along a row).  Then a wave takes 16 of the rows and multiplies
// every leaf's path, root first (the factors and their order are those of soft_mix_kernel: same bits),
// writing the mixture weights and the bias columns of the hidden matrix; thread n adds the entropies
// of node n over the tile's rows in row order into part[row tile][n].
__device__ __forceinline__ int score_slot(int r, int n) { return 256 * r + (n ^ (4 * (r & 15))); }

__global__ __launch_bounds__(256, 2) void soft_nodes_mix_kernel(const SoftArgs a, float* __restrict__ ent_part) {
    __shared__ BigTileLds tile;
    int64_t t0, n0;
    if (!big_tile_of_block(1, a.T, t0, n0)) return;
    f32x4_t acc[4][8];
    mfma_tile_128x256(a.x, a.D, a.T, a.node_w, a.D, a.NN, a.D, t0, 0, tile, acc);
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, j = lane & 15, kg = lane >> 4;
    const int wm = wv >> 1, wn = wv & 1;
    const int NL = (int)a.NL, NN = (int)a.NN;
#pragma unroll
    for (int nt = 0; nt < 8; ++nt) {
        const int n = 128 * wn + 16 * nt + 4 * kg;                   // this lane's nodes n .. n + 3
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const float b = n + q < NN ? bf16_to_f32(a.node_b[n + q]) : 0.0f;
#pragma unroll
            for (int mt = 0; mt < 4; ++mt) acc[mt][nt][q] = 1.0f / (1.0f + __expf(-(acc[mt][nt][q] + b)));
        }
    }
    float* const S = (float*)&tile;                     // [64][256] scores of one half of the tile's rows
    const int per_log = NL >= 256 ? 2 : NL >= 128 ? 1 : 0;   // leaves per lane: 4, 2 or 1
    const bool mix_vec = (reinterpret_cast<uintptr_t>(a.mix) & 15u) == 0;
    float ent = 0.0f;
    for (int h = 0; h < 2; ++h) {
        if (wm == h) {
#pragma unroll
            for (int mt = 0; mt < 4; ++mt)
#pragma unroll
                for (int nt = 0; nt < 8; ++nt)
                    *(f32x4_t*)(S + score_slot(16 * mt + j, 128 * wn + 16 * nt + 4 * kg)) = acc[mt][nt];
        }
        __syncthreads();
        for (int rr = 0; rr < 16; ++rr) {
            const int r = 16 * wv + rr;
            const int64_t t = t0 + 64 * h + r;
            if (t >= a.T) break;
            const float* Sr = S + 256 * r;
            const int sw = 4 * (r & 15);
            // a lane takes `per` consecutive leaves (4 for 256 leaves): their paths share all but the last
            // log2(per) levels, so the shared factors are multiplied once, root first, and the product
            // then splits level by level -- every leaf still sees its factors in root-to-leaf order
            const int first = lane << per_log;
            if (first < NL) {
                float m[4];
                m[0] = 1.0f;
                const int shared = a.depth - per_log;
                for (int lvl = 0; lvl < shared; ++lvl) {
                    const int pos = first >> (a.depth - lvl);
                    const int bit = (first >> (a.depth - 1 - lvl)) & 1;
                    const float cs = Sr[(((1 << lvl) - 1) + pos) ^ sw];
                    m[0] *= bit ? cs : 1.0f - cs;
                }
                if (per_log == 2) {
                    const int n6 = ((1 << shared) - 1) + lane;                 // the lane's node on level depth - 2
                    const float c6 = Sr[n6 ^ sw];
                    const float c70 = Sr[(2 * n6 + 1) ^ sw], c71 = Sr[(2 * n6 + 2) ^ sw];
                    const float lo = m[0] * (1.0f - c6), hi = m[0] * c6;
                    m[0] = lo * (1.0f - c70); m[1] = lo * c70; m[2] = hi * (1.0f - c71); m[3] = hi * c71;
                    // one 16-byte store (a caller's mixture matrix may start anywhere: checked) and one 8-byte store
                    // (the hidden matrix is the library's, K2 a multiple of 8)
                    float* mp = a.mix + t * a.NL + first;
                    if (mix_vec) {
                        __builtin_nontemporal_store(f32x4_t{m[0], m[1], m[2], m[3]}, (f32x4_t*)mp);     // written once, read by a later launch
                    } else {
                        mp[0] = m[0]; mp[1] = m[1]; mp[2] = m[2]; mp[3] = m[3];
                    }
                    {
                        typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
                        const u32x2_t packed = {(uint32_t)f32_to_bf16(m[0]) | ((uint32_t)f32_to_bf16(m[1]) << 16),
                                                (uint32_t)f32_to_bf16(m[2]) | ((uint32_t)f32_to_bf16(m[3]) << 16)};
                        __builtin_nontemporal_store(packed, (u32x2_t*)(a.hid + t * a.K2 + a.NL * a.L + first));
                    }
                } else if (per_log == 1) {
                    const float c7 = Sr[(((1 << shared) - 1) + lane) ^ sw];
                    m[1] = m[0] * c7; m[0] = m[0] * (1.0f - c7);
                    float* mp = a.mix + t * a.NL + first;
                    mp[0] = m[0]; mp[1] = m[1];
                    uint16_t* hp = a.hid + t * a.K2 + a.NL * a.L + first;
                    hp[0] = f32_to_bf16(m[0]); hp[1] = f32_to_bf16(m[1]);
                } else {
                    a.mix[t * a.NL + first] = m[0];
                    a.hid[t * a.K2 + a.NL * a.L + first] = f32_to_bf16(m[0]);
                }
            }
            for (int64_t k = a.NL * (a.L + 1) + lane; k < a.K2; k += kWave) a.hid[t * a.K2 + k] = 0;
        }
        if (ent_part != nullptr && tid < NN) {
            for (int r = 0; r < 64 && t0 + 64 * h + r < a.T; ++r)
                ent += bernoulli_entropy(S[score_slot(r, tid)]);
        }
        __syncthreads();
    }
    if (ent_part != nullptr && tid < NN) ent_part[(t0 / kBigM) * a.NN + tid] = ent;
}

// GELU: the activation is a template parameter -- chosen per element at run time it puts a branch around
// every one of a lane's 128 evaluations, which then run one after the other
template <bool GELU>
__global__ __launch_bounds__(256, 2) void soft_hidden_big_kernel(const SoftArgs a) {
    __shared__ BigTileLds tile;
    const int64_t NH = a.NL * a.L;
    const int64_t ncb = (NH + kBigN - 1) / kBigN;
    int64_t t0, n0;
    if (!big_tile_of_block(ncb, a.T, t0, n0)) return;
    f32x4_t acc[4][8];
    mfma_tile_128x256(a.x, a.D, a.T, a.w1, a.D, NH, a.D, t0, n0, tile, acc);
    // bias, activation and the mixture weight of the neuron's leaf.  A lane holds four consecutive
    // neurons of a token per accumulator: one 8-byte load of biases and, where the four belong to one
    // leaf (leaf widths that are multiples of 4), one mixture weight serve all four.
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6, j = lane & 15, kg = lane >> 4;
    const int wm = wv >> 1, wn = wv & 1;
    const float* mrow[4];
#pragma unroll
    for (int mt = 0; mt < 4; ++mt) {
        const int64_t t = t0 + 64 * wm + 16 * mt + j;
        mrow[mt] = a.mix + (t < a.T ? t : a.T - 1) * a.NL;
    }
    const bool one_leaf = a.L % 4 == 0;
    const bool bias_vec = (reinterpret_cast<uintptr_t>(a.b1) & 7u) == 0;
    const uint32_t L32 = (uint32_t)a.L, last = (uint32_t)(NH - 1);       // the width fits 32 bits (soft_shape_ok)
#pragma unroll
    for (int nt = 0; nt < 8; ++nt) {
        const uint32_t n = (uint32_t)(n0 + 128 * wn + 16 * nt + 4 * kg);   // this lane's neurons n .. n + 3
        // columns past the last neuron are dropped by the store: their look-ups are clamped, not skipped
        const uint32_t nc = n < last ? n : last;
        float bias[4];
        if (bias_vec && n + 3 <= last) {
            const uint2 b = *(const uint2*)(a.b1 + n);
            bias[0] = bf16_to_f32((uint16_t)b.x); bias[1] = bf16_to_f32((uint16_t)(b.x >> 16));
            bias[2] = bf16_to_f32((uint16_t)b.y); bias[3] = bf16_to_f32((uint16_t)(b.y >> 16));
        } else {
#pragma unroll
            for (int q = 0; q < 4; ++q) bias[q] = bf16_to_f32(a.b1[nc + q < last ? nc + q : last]);
        }
        // one division per group of four: the leaf of neuron n + q is that of n plus the number of leaf
        // boundaries crossed, at most three (q <= 3)
        const uint32_t leaf0 = nc / L32, rem = nc - leaf0 * L32;
        uint32_t leaf[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const uint32_t o = rem + q;
            uint32_t lf = leaf0 + (o >= L32) + (o >= 2 * L32) + (o >= 3 * L32);
            leaf[q] = lf < (uint32_t)a.NL ? lf : (uint32_t)a.NL - 1;
        }
#pragma unroll
        for (int mt = 0; mt < 4; ++mt) {
            float m[4];
            m[0] = mrow[mt][leaf[0]];
#pragma unroll
            for (int q = 1; q < 4; ++q) m[q] = one_leaf ? m[0] : mrow[mt][leaf[q]];
            f32x4_t v;
#pragma unroll
            for (int q = 0; q < 4; ++q) v[q] = activate_bulk(acc[mt][nt][q] + bias[q], GELU ? 1 : 0) * m[q];
            big_tile_stage(tile, mt, nt, v);         // finished, packed and staged at once: nothing is held back
        }
    }
    big_tile_flush(tile, a.hid, a.K2, a.T, NH, t0, n0);
}

__global__ __launch_bounds__(256, 2) void soft_out_big_kernel(const SoftArgs a) {
    __shared__ BigTileLds tile;
    const int64_t ncb = ((int64_t)a.O + kBigN - 1) / kBigN;
    int64_t t0, n0;
    if (!big_tile_of_block(ncb, a.T, t0, n0)) return;
    f32x4_t acc[4][8];
    mfma_tile_128x256(a.hid, a.K2, a.T, a.w2x, a.K2, a.O, (int)a.K2, t0, n0, tile, acc);
    big_tile_store_bf16(tile, acc, a.out, a.O, a.T, a.O, t0, n0);
}

// W2x[o][k] = W2[k][o] for k < NL * L, b2[k - NL * L][o] for the next NL, zeros up to K2.
// A 32 x 32 tile through LDS: reads run along o, writes along k.
__global__ __launch_bounds__(256) void soft_w2x_kernel(const SoftArgs a) {
    __shared__ uint16_t t32[32][33];
    const int64_t kb = (a.K2 + 31) / 32;
    const int64_t k0 = (int64_t)(blockIdx.x % kb) * 32, o0 = (int64_t)(blockIdx.x / kb) * 32;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;     // 32 x 8
    const int64_t NH = a.NL * a.L;
    for (int r = ty; r < 32; r += 8) {
        const int64_t k = k0 + r, o = o0 + tx;
        uint16_t v = 0;
        if (o < a.O) {
            if (k < NH) v = a.w2[k * a.O + o];
            else if (k < NH + a.NL) v = a.b2[(k - NH) * a.O + o];
        }
        t32[r][tx] = v;
    }
    __syncthreads();
    for (int r = ty; r < 32; r += 8) {
        const int64_t o = o0 + r, k = k0 + tx;
        if (o < a.O && k < a.K2) a.w2x[o * a.K2 + k] = t32[tx][r];
    }
}

// out: the weighted leaf outputs and biases in one contraction over K2
__global__ __launch_bounds__(256) void soft_out_kernel(const SoftArgs a) {
    __shared__ TileLds tile;
    const int64_t ncb = ((int64_t)a.O + kTileN - 1) / kTileN;
    const int64_t t0 = tile_row0(ncb), n0 = tile_col0(ncb);
    f32x4_t acc[4][2];
    mfma_tile_64x128<2>(a.hid, a.K2, a.T, a.w2x, a.K2, a.O, (int)a.K2, t0, n0, tile, acc);
    tile_store_bf16(tile, acc, a.out, a.O, a.T, a.O, t0, n0, [](int, int, float v) { return v; });
}

// batch mean of the Bernoulli entropy of every node's choice score, in two passes with a fixed
// order of additions (so the result does not depend on scheduling): a block sums kEntTokens
// tokens for every node (thread = node, so the reads run along a row of scores), then one block
// per node adds the partial sums (strided over its threads, then a fixed tree).
constexpr int kEntTokens = 32;

__global__ __launch_bounds__(256) void soft_entropy_part_kernel(const float* __restrict__ choice, int64_t T, int64_t NN,
                                                                int64_t pitch, float* __restrict__ part) {
    const int64_t t0 = (int64_t)blockIdx.x * kEntTokens;
    const int64_t t1 = t0 + kEntTokens < T ? t0 + kEntTokens : T;
    for (int64_t n = threadIdx.x; n < NN; n += 256) {
        float s = 0.0f;
        for (int64_t t = t0; t < t1; ++t) {
            s += bernoulli_entropy(choice[t * pitch + n]);
        }
        part[(int64_t)blockIdx.x * NN + n] = s;
    }
}

__global__ __launch_bounds__(256) void soft_entropy_sum_kernel(const float* __restrict__ part, int64_t n_parts, int64_t T,
                                                               int64_t NN, float* __restrict__ entropy) {
    __shared__ float red[256];
    const int64_t n = blockIdx.x;       // one block per node: strided partial sums, then a fixed tree
    float s = 0.0f;
    for (int64_t b = threadIdx.x; b < n_parts; b += 256) s += part[b * NN + n];
    red[threadIdx.x] = s;
    __syncthreads();
    for (int d = 128; d > 0; d >>= 1) {
        if ((int)threadIdx.x < d) red[threadIdx.x] += red[threadIdx.x + d];
        __syncthreads();
    }
    if (threadIdx.x == 0) entropy[n] = red[0] / (float)T;
}

}  // namespace

// bf16, D a multiple of 8, 16-byte aligned rows of x, node_w, leaf_w1
bool soft_shape_ok(const Problem& p) {
    return p.bf16 && vec_ok(p.x, p.D, true) && (p.depth == 0 || vec_ok(p.node_w, p.D, true)) &&
           vec_ok(p.leaf_w1, p.D, true) && p.D < (1 << 30) && p.O < (1 << 30) &&
           (((int64_t)p.L + 1) << p.depth) < ((int64_t)1 << 30);        // the hidden matrix's width fits 32 bits
}

static int64_t soft_k2(const Problem& p) {
    const int64_t NL = (int64_t)1 << p.depth;
    return (NL * (p.L + 1) + 7) / 8 * 8;
}

// 32-bit words of scratch: choice scores, mixture weights, hidden matrix, transposed output weights
int64_t soft_scratch_words(const Problem& p) {
    const int64_t NL = (int64_t)1 << p.depth, NN = NL - 1, K2 = soft_k2(p);
    auto up = [](int64_t w) { return (w + 63) / 64 * 64; };
    return up(p.T * NL) + up(p.T * NL) + up((p.T * K2 + 1) / 2) + up((p.O * K2 + 1) / 2) +
           up((p.T + kEntTokens - 1) / kEntTokens * (NN > 0 ? NN : 1));
}

// mix (optional, [T, 2^d] fp32) and entropy (optional, [2^d - 1] fp32) are caller buffers
hipError_t launch_forward_soft(const Problem& p, int32_t* scratch, float* mix_out, float* entropy_out,
                               hipStream_t s) {
    if (p.T == 0) return hipSuccess;
    auto up = [](int64_t w) { return (w + 63) / 64 * 64; };
    SoftArgs a;
    a.NL = (int64_t)1 << p.depth;
    a.NN = a.NL - 1;
    a.K2 = soft_k2(p);
    a.x = (const uint16_t*)p.x;
    a.node_w = (const uint16_t*)p.node_w;
    a.node_b = (const uint16_t*)p.node_b;
    a.w1 = (const uint16_t*)p.leaf_w1;
    a.b1 = (const uint16_t*)p.leaf_b1;
    a.w2 = (const uint16_t*)p.leaf_w2;
    a.b2 = (const uint16_t*)p.leaf_b2;
    a.out = (uint16_t*)p.out;
    a.T = p.T;
    a.D = (int)p.D;
    a.O = (int)p.O;
    a.depth = p.depth;
    a.L = p.L;
    a.act = p.act;
    int32_t* w = scratch;
    a.choice = (float*)w;
    w += up(p.T * a.NL);
    a.mix = mix_out ? mix_out : (float*)w;
    w += up(p.T * a.NL);
    a.hid = (uint16_t*)w;
    w += up((p.T * a.K2 + 1) / 2);
    a.w2x = (uint16_t*)w;
    w += up((p.O * a.K2 + 1) / 2);
    float* ent_part = (float*)w;
    const int64_t mb = (p.T + kTileM - 1) / kTileM;
    hipError_t e;
    // the large tile where the batch and the width fill it (a batch of at least 16 row tiles, a full tile
    // of columns)
    const bool big = !g_soft_small_tiles && p.T >= 16 * kBigM;
    const bool big_nodes = big && a.NN >= kBigN - 1;
    const bool big_hidden = big && a.NL * a.L >= kBigN, big_out = big && p.O >= kBigN;
    // nodes, mixture weights and entropy sums in one launch where all nodes fit one column tile
    const bool fused_nodes = big && a.NN > 0 && a.NN < kBigN;
    const bool want_entropy = entropy_out && a.NN > 0;
    if (fused_nodes)
        note_launch("soft_nodes_mix_kernel + soft_hidden%s_kernel + soft_w2x_kernel + soft_out%s_kernel%s",
                    big_hidden ? "_big" : "", big_out ? "_big" : "", want_entropy ? " + soft_entropy_sum_kernel" : "");
    else
        note_launch("%s%ssoft_mix%s_kernel + soft_hidden%s_kernel + soft_w2x_kernel + soft_out%s_kernel%s",
                    a.NN > 0 ? (big_nodes ? "soft_nodes_big_kernel" : "soft_nodes_kernel") : "", a.NN > 0 ? " + " : "",
                    a.NL <= kMixMaxLeaves ? "_rows" : "", big_hidden ? "_big" : "", big_out ? "_big" : "",
                    want_entropy ? " + soft_entropy_part_kernel + soft_entropy_sum_kernel" : "");
    if (fused_nodes) {
        soft_nodes_mix_kernel<<<dim3(big_grid(p.T, 1)), dim3(256), 0, s>>>(a, want_entropy ? ent_part : nullptr);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    } else {
        if (a.NN > 0) {
            if (big_nodes)
                soft_nodes_big_kernel<<<dim3(big_grid(p.T, (a.NN + kBigN - 1) / kBigN)), dim3(256), 0, s>>>(a);
            else
                soft_nodes_kernel<<<dim3((unsigned)(mb * ((a.NN + kTileN - 1) / kTileN))), dim3(256), 0, s>>>(a);
            if ((e = hipGetLastError()) != hipSuccess) return e;
        }
        if (a.NL <= kMixMaxLeaves) {
            const int waves = a.NL > 1024 ? 2 : 4;
            int64_t blocks = (p.T + waves - 1) / waves;
            const int64_t cap = (int64_t)device_info().cus * 8;
            if (blocks > cap) blocks = cap;
            const size_t lds_bytes = sizeof(float) * 3 * waves * (size_t)a.NL;      // at most 48 KB
            soft_mix_rows_kernel<<<dim3((unsigned)blocks), dim3(64 * waves), lds_bytes, s>>>(a);
        } else {
            soft_mix_kernel<<<dim3((unsigned)((p.T * a.NL + 255) / 256)), dim3(256), 0, s>>>(a);
        }
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    if (big_hidden && a.act != 0)
        soft_hidden_big_kernel<true><<<dim3(big_grid(p.T, (a.NL * a.L + kBigN - 1) / kBigN)), dim3(256), 0, s>>>(a);
    else if (big_hidden)
        soft_hidden_big_kernel<false><<<dim3(big_grid(p.T, (a.NL * a.L + kBigN - 1) / kBigN)), dim3(256), 0, s>>>(a);
    else
        soft_hidden_kernel<<<dim3((unsigned)(mb * ((a.NL * a.L + kTileN - 1) / kTileN))), dim3(256), 0, s>>>(a);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    soft_w2x_kernel<<<dim3((unsigned)(((a.K2 + 31) / 32) * ((p.O + 31) / 32))), dim3(256), 0, s>>>(a);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    if (big_out)
        soft_out_big_kernel<<<dim3(big_grid(p.T, (p.O + kBigN - 1) / kBigN)), dim3(256), 0, s>>>(a);
    else
        soft_out_kernel<<<dim3((unsigned)(mb * ((p.O + kTileN - 1) / kTileN))), dim3(256), 0, s>>>(a);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    if (want_entropy) {
        int64_t n_parts = (p.T + kBigM - 1) / kBigM;        // the fused launch leaves one partial sum per row tile
        if (!fused_nodes) {
            n_parts = (p.T + kEntTokens - 1) / kEntTokens;
            soft_entropy_part_kernel<<<dim3((unsigned)n_parts), dim3(256), 0, s>>>(a.choice, p.T, a.NN, a.NL, ent_part);
            if ((e = hipGetLastError()) != hipSuccess) return e;
        }
        soft_entropy_sum_kernel<<<dim3((unsigned)a.NN), dim3(256), 0, s>>>(ent_part, n_parts, p.T, a.NN, entropy_out);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace fff
