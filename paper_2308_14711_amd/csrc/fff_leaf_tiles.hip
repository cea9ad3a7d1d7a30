// K3 + K4, MFMA tile path (bf16, leaf width <= 16) -- the leaf networks of the
// leaves the tokens arrived at (Definition: each leaf is a <D, l, O>
// feedforward block; Algorithm 1 returns its output), with every output row
// written straight to its token's position.
//
// Tokens arrive grouped by leaf (perm from the bucketing stage).  A block owns a
// tile of 16 consecutive slots of perm.  Inside a tile the slots form runs of
// equal leaf; because a leaf has few neurons, several runs share one MFMA:
//
//   first contraction  (v_mfma_f32_16x16x32_bf16, K = D)
//       rows  = (run r, neuron n) pairs, r * l + n < 16   -> W1[leaf_r][n][:]
//       cols  = the 16 tokens                              -> x[token][:]
//       C[(r, n)][token] is a hidden pre-activation wherever the token belongs
//       to run r; the other entries are discarded (set to zero).
//       The W waves of the block each take every W-th pair of K steps; the
//       partial C tiles are summed through LDS.
//   second contraction (v_mfma_f32_16x16x32_bf16, K = 32 slots)
//       A     = the activated, masked C of the first contraction -- it is
//               already in the lanes and registers the instruction wants --
//               plus, in the 16 spare K slots, a one-hot "token is in run r"
//       B     = W2[leaf_r][n][o] for the first 16 slots, b2[leaf_r][o] for the
//               spare ones, so the bias rides in the same instruction
//       D[token][o] = sum_n h[token][n] W2[leaf(token)][n][o] + b2[leaf(token)][o]
//       The waves each take every W-th 64-wide range of o.
//
// A tile with more than 16 / l runs takes several passes.  W2 is stored with o
// contiguous (per neuron, its O output weights), while the instruction wants K
// contiguous per lane: a lane loads 4 consecutive o of its 4 K rows and
// transposes the 4x4 block in registers; column j of the c-th MFMA of a
// 64-wide o range stands for o = 64 R + 4 j + c, which also makes every lane
// end up with 4 consecutive outputs of a token (8-byte stores, 128 contiguous
// bytes per token across 16 lanes).
#include "fff_device.h"
#include "fff_internal.h"

namespace fff {

struct TilesArgs {
    const uint16_t* x;
    const uint16_t* w1;
    const uint16_t* b1;
    const uint16_t* w2;
    const uint16_t* b2;
    uint16_t* out;
    const int32_t* perm;
    const int32_t* leaf_idx;
    int64_t T, n_tiles;
    int D, O, L, act;
};

constexpr int kChunk = 6;    // K steps of the first contraction fetched per lane per group (3 pairs)
constexpr int kPre = 1;      // 128-wide output ranges of the second contraction fetched ahead of the first

// the c-th bf16 of the 8 held by a 16-byte vector, for the 4x4 (here 4x8) register transposes
__device__ __forceinline__ uint32_t dword_of(const uint4& v, int c) {
    return (c >> 1) == 0 ? v.x : (c >> 1) == 1 ? v.y : (c >> 1) == 2 ? v.z : v.w;
}
__device__ __forceinline__ uint32_t pack_half(uint32_t a, uint32_t b, int hi) {
    return hi ? ((a >> 16) | (b & 0xffff0000u)) : ((a & 0xffffu) | (b << 16));
}

// Blocks are persistent and software-pipelined over work items (tile, pass): while the item at
// hand is reduced, activated, multiplied by W2 and stored, the token rows and W1 rows of the next
// item are already in flight, and so are the slot -> token -> leaf lookups of the tiles after it.
// Loads return in issue order, so within an item the W2 / b2 rows are requested first, then the
// next item's rows: waiting for the former never waits for the latter.
// W = waves per block (compile time, so that the strides between a wave's K pairs and output
// ranges are immediates).  DTAIL = D is not a multiple of 64 (lanes then check their K offset).
template <int W, bool DTAIL>
__global__ __launch_bounds__(64 * W) void leaf_tiles_kernel(const TilesArgs a) {
    __shared__ f32x4_t part[2 * W * 64];     // [2][W][64] partial tiles of the first contraction
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int j = lane & 15, kg = lane >> 4;
    const int D = a.D, O = a.O, L = a.L;
    const int P = 16 / L;                    // runs per pass
    const int n_pairs = (D + 63) / 64;       // pairs of K steps (64 elements of a row each)
    const int64_t G = gridDim.x;

    const int rr_i = j / L, n_i = j % L;     // A row j of the first contraction = (run rr_i of the pass, neuron n_i)
    int rr_q[4], n_q[4];                      // K slots 4 kg + q of the second contraction, same pairing
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        rr_q[q] = (4 * kg + q) / L;
        n_q[q] = (4 * kg + q) % L;
    }

    // slot -> token and token -> leaf of this lane's column (all four 16-lane rows hold the same
    // 16 columns); -1 marks a slot past the end
    auto load_tok = [&](int64_t tile) -> int32_t {
        const int64_t slot = tile * 16 + j;
        return (tile < a.n_tiles && slot < a.T) ? a.perm[slot] : -1;
    };
    auto load_leaf = [&](int32_t tok) -> int32_t { return tok >= 0 ? a.leaf_idx[tok] : -1; };
    // runs of equal leaf inside a tile: run index of this lane's column, and the number of runs
    auto derive = [&](int32_t leaf, int& run_j, int& n_runs) {
        const int32_t prev = __shfl_up(leaf, 1, 16);
        const uint32_t ch16 = (uint32_t)__ballot(leaf >= 0 && j > 0 && leaf != prev) & 0xffffu;
        run_j = __popc(ch16 & ((2u << j) - 1u));
        n_runs = __popc(ch16) + 1;
    };
    // leaf of every run of a pass, handed to the lanes that need it
    auto pass_leaves = [&](int32_t leaf, int run_j, int n_runs, int pass, int32_t& row_leaf,
                           int32_t (&w2_leaf)[4], int32_t (&b2_leaf)[4]) {
        row_leaf = -1;
#pragma unroll
        for (int q = 0; q < 4; ++q) w2_leaf[q] = b2_leaf[q] = -1;
        for (int rr = 0; rr < P && pass + rr < n_runs; ++rr) {
            const uint32_t m = (uint32_t)__ballot(leaf >= 0 && run_j == pass + rr) & 0xffffu;
            if (m == 0) break;                     // a tile past the end has no runs
            const int32_t lf = __shfl(leaf, __ffs(m) - 1, 64);
            if (rr_i == rr) row_leaf = lf;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                if (rr_q[q] == rr) w2_leaf[q] = lf;
                if (4 * kg + q == rr) b2_leaf[q] = lf;
            }
        }
    };
    // First contraction.  The K index is only a summation order, so step u of pair pp gives lane
    // group kg the 8 elements at 64 pp + 16 kg + 8 u: the two steps of a pair read 32 contiguous
    // bytes per lane and the four lane groups cover a whole 128-byte line.  This wave takes pairs
    // wave, wave + W, ...; group g of them is pairs wave + W (3 g + {0, 1, 2}).
    auto fetch_chunk = [&](int32_t tok, int32_t row_leaf, int g, uint4* av, uint4* bv) {
        const uint16_t* xrow = a.x + (int64_t)(tok >= 0 ? tok : 0) * D + 16 * kg;
        const uint16_t* arow = a.w1 + ((int64_t)(row_leaf >= 0 ? row_leaf : 0) * L + n_i) * D + 16 * kg;
        const int pp0 = wave + W * (kChunk / 2) * g;
#pragma unroll
        for (int u = 0; u < kChunk; ++u) {
            av[u] = make_uint4(0, 0, 0, 0);
            bv[u] = make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int u = 0; u < kChunk; ++u) {
            const int pp = pp0 + W * (u >> 1);                // wave-uniform
            const int k0 = 64 * pp + 8 * (u & 1);             // + 16 kg is in the row pointers
            const bool in = pp < n_pairs && (!DTAIL || k0 + 16 * kg < D);
            if (in && row_leaf >= 0) av[u] = *(const uint4*)(arow + k0);
            if (in && tok >= 0) bv[u] = *(const uint4*)(xrow + k0);
        }
    };
    const int n_groups = (n_pairs - wave + W * (kChunk / 2) - 1) / (W * (kChunk / 2));   // <= 0: nothing for this wave

    // metadata of the tile at hand (A), the next (B), and the token of the one after (C)
    int64_t tile = blockIdx.x;
    int32_t tokA = load_tok(tile), tokB = load_tok(tile + G), tokC = load_tok(tile + 2 * G);
    int32_t leafA = load_leaf(tokA), leafB = load_leaf(tokB);
    int run_j, n_runs, pass = 0;
    derive(leafA, run_j, n_runs);
    int32_t row_leaf, w2_leaf[4], b2_leaf[4];
    pass_leaves(leafA, run_j, n_runs, 0, row_leaf, w2_leaf, b2_leaf);
    uint4 av[kChunk], bv[kChunk];
    fetch_chunk(tokA, row_leaf, 0, av, bv);

    int buf = 0;
    while (tile < a.n_tiles) {
        // ---- rows of the second contraction for this item (requested before anything else).
        // A lane holds K rows 4 kg + q (W2 rows of (run, neuron) pairs, then b2 rows of runs) and
        // 8 consecutive outputs o0 .. o0 + 7 of a 128-wide range; rows that stand for nothing
        // are read from row 0 (always there) and zeroed.
        const uint16_t* wptr[4];
        const uint16_t* bptr[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            wptr[q] = a.w2 + ((int64_t)(w2_leaf[q] >= 0 ? w2_leaf[q] : 0) * L + n_q[q]) * O + 8 * j;
            bptr[q] = a.b2 + (int64_t)(b2_leaf[q] >= 0 ? b2_leaf[q] : 0) * O + 8 * j;
        }
        auto fetch_range = [&](int r, uint4* w, uint4* b) {      // r: index of a 128-wide range
            const int o0 = 128 * r;
            const bool ok = o0 + 8 * j < O;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                w[q] = make_uint4(0, 0, 0, 0);
                b[q] = make_uint4(0, 0, 0, 0);
                if (ok && w2_leaf[q] >= 0) w[q] = *(const uint4*)(wptr[q] + o0);
                if (ok && b2_leaf[q] >= 0) b[q] = *(const uint4*)(bptr[q] + o0);
            }
        };
        uint4 wpre[kPre][4], bpre[kPre][4];
#pragma unroll
        for (int g = 0; g < kPre; ++g) fetch_range(wave + W * g, wpre[g], bpre[g]);

        // ---- first contraction: the group in registers, then any further groups
        f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int u = 0; u < kChunk; ++u)
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, av[u]),
                                                          __builtin_bit_cast(bf16x8_t, bv[u]), acc, 0, 0, 0);
        for (int g = 1; g < n_groups; ++g) {
            fetch_chunk(tokA, row_leaf, g, av, bv);
#pragma unroll
            for (int u = 0; u < kChunk; ++u)
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, av[u]),
                                                              __builtin_bit_cast(bf16x8_t, bv[u]), acc, 0, 0, 0);
        }

        // ---- the next item: another pass over this tile, or the first pass of the next tile
        const bool same_tile = pass + P < n_runs;
        int32_t n_row_leaf, n_w2_leaf[4], n_b2_leaf[4];
        int n_run_j = run_j, n_n_runs = n_runs;
        if (same_tile) {
            pass_leaves(leafA, run_j, n_runs, pass + P, n_row_leaf, n_w2_leaf, n_b2_leaf);
            fetch_chunk(tokA, n_row_leaf, 0, av, bv);
        } else {
            derive(leafB, n_run_j, n_n_runs);
            pass_leaves(leafB, n_run_j, n_n_runs, 0, n_row_leaf, n_w2_leaf, n_b2_leaf);
            fetch_chunk(tokB, n_row_leaf, 0, av, bv);       // all-invalid past the last tile: no loads
        }
        int32_t leafC = -1, tokD = -1;
        if (!same_tile) {
            leafC = load_leaf(tokC);
            tokD = load_tok(tile + 3 * G);
        }

        // ---- sum the partial tiles of the W waves (two buffers, so one barrier per item is enough)
        f32x4_t* mine_part = part + (buf * W) * 64;
        mine_part[wave * 64 + lane] = acc;
        __syncthreads();
        acc = mine_part[lane];
#pragma unroll
        for (int w = 1; w < W; ++w) acc += mine_part[w * 64 + lane];

        // ---- activation, mask to the token's own run, append the run indicators
        float hq[4], iq[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const bool mine = leafA >= 0 && rr_q[q] < P && run_j == pass + rr_q[q];
            float v = 0.f;
            if (mine) v = activate(acc[q] + bf16_to_f32(a.b1[(int64_t)leafA * L + n_q[q]]), a.act);
            hq[q] = v;
            iq[q] = (leafA >= 0 && 4 * kg + q < P && run_j == pass + 4 * kg + q) ? 1.0f : 0.0f;
        }
        const uint4 a2u = make_uint4(pack_bf16x2(hq[0], hq[1]), pack_bf16x2(hq[2], hq[3]),
                                     pack_bf16x2(iq[0], iq[1]), pack_bf16x2(iq[2], iq[3]));
        const bf16x8_t a2 = __builtin_bit_cast(bf16x8_t, a2u);

        // ---- second contraction and the output rows of the tokens of this pass.  Column j of the
        // c-th MFMA of a range stands for output o0 + 8 j + c, so a lane ends with 8 consecutive
        // outputs of each of its 4 token rows: one 16-byte store per row.
        uint16_t* orow[4];
        bool st_ok[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int32_t tq = __shfl(tokA, 4 * kg + q, 64);
            const int rrow = __shfl(run_j, 4 * kg + q, 64);
            st_ok[q] = tq >= 0 && rrow >= pass && rrow < pass + P;
            orow[q] = a.out + (int64_t)(tq >= 0 ? tq : 0) * O + 8 * j;
        }
        auto mul_store = [&](const uint4* w, const uint4* b, int r) {
            const int o0 = 128 * r;
            const f32x4_t zero = {0.f, 0.f, 0.f, 0.f};
            f32x4_t d[8];
#pragma unroll
            for (int c = 0; c < 8; ++c) {
                const uint4 f = make_uint4(pack_half(dword_of(w[0], c), dword_of(w[1], c), c & 1),
                                           pack_half(dword_of(w[2], c), dword_of(w[3], c), c & 1),
                                           pack_half(dword_of(b[0], c), dword_of(b[1], c), c & 1),
                                           pack_half(dword_of(b[2], c), dword_of(b[3], c), c & 1));
                d[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a2, __builtin_bit_cast(bf16x8_t, f), zero, 0, 0, 0);
            }
            if (o0 + 8 * j < O) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    if (st_ok[q]) {
                        const uint4 o4 = make_uint4(pack_bf16x2(d[0][q], d[1][q]), pack_bf16x2(d[2][q], d[3][q]),
                                                    pack_bf16x2(d[4][q], d[5][q]), pack_bf16x2(d[6][q], d[7][q]));
                        store_stream((uint4*)(orow[q] + o0), o4);
                    }
                }
            }
        };
#pragma unroll
        for (int g = 0; g < kPre; ++g) mul_store(wpre[g], bpre[g], wave + W * g);
        for (int r = wave + W * kPre; 128 * r < O; r += W) {
            uint4 wv[4], bv2[4];
            fetch_range(r, wv, bv2);
            mul_store(wv, bv2, r);
        }

        // ---- move on
        row_leaf = n_row_leaf;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            w2_leaf[q] = n_w2_leaf[q];
            b2_leaf[q] = n_b2_leaf[q];
        }
        if (same_tile) {
            pass += P;
        } else {
            pass = 0;
            run_j = n_run_j;
            n_runs = n_n_runs;
            tile += G;
            tokA = tokB; leafA = leafB;
            tokB = tokC; leafB = leafC;
            tokC = tokD;
        }
        buf ^= 1;
    }
}

// bf16, leaf width <= 16, 16-byte aligned rows of x, W1, W2, b2 and out
bool tiles_shape_ok(const Problem& p) {
    auto al = [](const void* q, uintptr_t m) { return (reinterpret_cast<uintptr_t>(q) & (m - 1)) == 0; };
    return p.bf16 && p.L <= 16 && p.D % 8 == 0 && p.O % 8 == 0 && p.D < (1 << 30) && p.O < (1 << 30) &&
           al(p.x, 16) && al(p.leaf_w1, 16) && al(p.leaf_w2, 16) && al(p.leaf_b2, 16) && al(p.out, 16);
}

template <int W, bool DTAIL>
static hipError_t run_tiles(const TilesArgs& a, hipStream_t s) {
    // persistent blocks: as many as fit on the chip at once
    static int per_cu = 0, cus = 0;
    if (per_cu == 0) {
        int dev = 0, n = 0;
        hipDeviceProp_t prop;
        cus = 256;
        if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess &&
            prop.multiProcessorCount > 0)
            cus = prop.multiProcessorCount;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, leaf_tiles_kernel<W, DTAIL>, 64 * W, 0) != hipSuccess || n < 1) {
            (void)hipGetLastError();
            n = 1;
        }
        per_cu = n;
    }
    int64_t blocks = (int64_t)cus * per_cu;
    if (blocks > a.n_tiles) blocks = a.n_tiles;
    leaf_tiles_kernel<W, DTAIL><<<dim3((unsigned)blocks), dim3(64 * W), 0, s>>>(a);
    return hipGetLastError();
}

hipError_t launch_leaf_tiles(const Problem& p, const int32_t* leaf_idx, const int32_t* perm, hipStream_t s) {
    if (p.T == 0) return hipSuccess;
    TilesArgs a;
    a.x = (const uint16_t*)p.x;
    a.w1 = (const uint16_t*)p.leaf_w1;
    a.b1 = (const uint16_t*)p.leaf_b1;
    a.w2 = (const uint16_t*)p.leaf_w2;
    a.b2 = (const uint16_t*)p.leaf_b2;
    a.out = (uint16_t*)p.out;
    a.perm = perm;
    a.leaf_idx = leaf_idx;
    a.T = p.T;
    a.n_tiles = (p.T + 15) / 16;
    a.D = (int)p.D;
    a.O = (int)p.O;
    a.L = p.L;
    a.act = p.act;
    // waves per tile: enough that a wave's share is a few K-step pairs and output ranges
    const int64_t n_pairs = (p.D + 63) / 64, n_ranges = (p.O + 127) / 128;
    const bool wide = n_pairs > 24 || n_ranges > 16;
    const bool dtail = p.D % 64 != 0;
    if (wide) return dtail ? run_tiles<8, true>(a, s) : run_tiles<8, false>(a, s);
    return dtail ? run_tiles<4, true>(a, s) : run_tiles<4, false>(a, s);
}

}  // namespace fff
