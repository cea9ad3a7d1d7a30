// K3 + K4, MFMA tile path (bf16, leaf width <= 32) -- the leaf networks of the
// leaves the tokens arrived at (Definition: each leaf is a <D, l, O>
// feedforward block; Algorithm 1 returns its output), with every output row
// written straight to its token's position.
//
// Tokens arrive grouped by leaf (perm from the bucketing stage).  A tile is 16
// consecutive slots of perm.  Inside a tile the slots form runs of equal leaf;
// because a leaf has few neurons, several runs share one MFMA.  Two launches,
// each light on registers so that many waves overlap their memory phases:
//
//   hidden kernel (one wave per tile): v_mfma_f32_16x16x32_bf16 over K = D with
//       rows  = (run r, neuron n) pairs, r * l + n < 16   -> W1[leaf_r][n][:]
//       cols  = the 16 tokens                              -> x[token][:]
//       C[(r, n)][token] is a hidden pre-activation wherever the token belongs
//       to run r (the other entries are discarded); bias, activation, and the
//       l hidden values of each token go to a small buffer h[T][l] (bf16).
//   output kernel (one wave per tile and pair of 128-wide output ranges):
//       v_mfma_f32_16x16x32_bf16 with 32 K slots:
//       A     = h of the token in the (run, neuron) slots of its own run, zero
//               elsewhere, plus, in the 16 spare slots, a one-hot "token is in
//               run r"
//       B     = W2[leaf_r][n][o] for the first 16 slots, b2[leaf_r][o] for the
//               spare ones, so the bias rides in the same instruction
//       D[token][o] = sum_n h[token][n] W2[leaf(token)][n][o] + b2[leaf(token)][o]
//
// A tile with more than 16 / l runs takes several passes.  Leaves of 17..32 neurons take one run
// per pass, as two blocks of 16 rows in the hidden kernel (two accumulators over one token operand)
// and as a second, accumulating instruction in the output kernel.  W2 is stored with o
// contiguous (per neuron, its O output weights), while the instruction wants K
// contiguous per lane: a lane loads 8 consecutive o of its 4 K rows and
// transposes in registers; column j of the c-th MFMA of a 128-wide o range
// stands for o = 128 R + 8 j + c, which also makes every lane end up with 8
// consecutive outputs of a token (16-byte stores, 256 contiguous bytes per
// token across 16 lanes).  h is rounded to bf16 between the two contractions.
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
    uint16_t* hidden;        // [T][L] bf16
    const int32_t* perm;
    const int32_t* slot_leaf;   // leaf of every slot of perm
    int64_t T, n_tiles;
    int D, O, L, act;
    int units_per_tile;      // output kernel: waves per tile (each takes kRangesPerWave ranges)
    int split;               // > 0: tiles with at least this many runs belong to the gather kernel
};

constexpr int kChunk = 8;            // K steps of the first contraction fetched per lane per group (4 pairs)
constexpr int kChunkPipelined = 4;   // the same where two groups are in flight (narrow leaves)
constexpr int kRangesPerWave = 2;    // 128-wide output ranges per wave of the output kernel

// the c-th bf16 of the 8 held by a 16-byte vector, for the register transposes
__device__ __forceinline__ uint32_t dword_of(const uint4& v, int c) {
    return (c >> 1) == 0 ? v.x : (c >> 1) == 1 ? v.y : (c >> 1) == 2 ? v.z : v.w;
}
__device__ __forceinline__ uint32_t pack_half(uint32_t a, uint32_t b, int hi) {
    return hi ? ((a >> 16) | (b & 0xffff0000u)) : ((a & 0xffffu) | (b << 16));
}

// What both kernels derive for a tile: this lane's column (slot j of the tile; all four 16-lane
// rows of the wave hold the same 16 columns), its token and leaf (-1 past the end), the index of
// its run of equal leaves and the number of runs.
struct TileColumn {
    int32_t tok, leaf;
    int run, n_runs;
};
__device__ __forceinline__ TileColumn tile_column(const TilesArgs& a, int64_t tile, int j) {
    TileColumn c;
    const int64_t slot = tile * 16 + j;
    c.tok = slot < a.T ? a.perm[slot] : -1;
    c.leaf = slot < a.T ? a.slot_leaf[slot] : -1;
    const int32_t prev = __shfl_up(c.leaf, 1, 16);
    const uint32_t ch16 = (uint32_t)__ballot(c.leaf >= 0 && j > 0 && c.leaf != prev) & 0xffffu;
    c.run = __popc(ch16 & ((2u << j) - 1u));
    c.n_runs = __popc(ch16) + 1;
    return c;
}
// leaf of run `run` of the tile (the run exists)
__device__ __forceinline__ int32_t leaf_of_run(const TileColumn& c, int run) {
    const uint32_t m = (uint32_t)__ballot(c.leaf >= 0 && c.run == run) & 0xffffu;
    return __shfl(c.leaf, __ffs(m) - 1, 64);
}

// ---- hidden kernel: h[token][n] = act(W1[leaf][n] . x[token] + b1[leaf][n]) ----
//
// The K index is only a summation order: step u of pair pp gives lane group kg the 8 elements at
// 64 pp + 16 kg + 8 u of its row, so a pair of steps consumes one 128-byte line of every row.
// Token rows come from HBM with 8 consecutive lanes on one line (two loads cover the 16 rows of
// a pair) and are turned into the MFMA operand layout through a wave-private LDS buffer; piece c
// (16 bytes) of row r sits at slot tile_swz(r, c), which keeps both the writes and the operand
// reads free of bank conflicts.
//
// NB = 1: leaf width <= 16, several runs per pass.  NB = 2: leaf width 17..32, one run per pass,
// its neurons in two blocks of 16 rows that share the token operand (two accumulators).
template <bool DTAIL, int NB>
__global__ __launch_bounds__(256) void leaf_hidden_kernel(const TilesArgs a) {
    __shared__ uint4 stage[4][(kChunk / 2) * 128];   // per wave: kChunk / 2 pairs x 16 rows x 8 pieces
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t tile = xcd_contiguous_block() * 4 + wave;
    if (tile >= a.n_tiles) return;           // whole waves leave; nothing below synchronises the block
    const int j = lane & 15, kg = lane >> 4;
    constexpr int CH = NB == 1 ? kChunkPipelined : kChunk;   // K steps per group
    const int D = a.D, L = a.L;
    const int P = NB == 1 ? 16 / L : 1;      // runs per pass
    const int n_pairs = (D + 63) / 64;       // pairs of K steps (64 elements of a row each)
    const TileColumn c = tile_column(a, tile, j);
    if (a.split > 0 && c.n_runs >= a.split) return;
    // A row j of block b = (run rr_i of the pass, neuron n_i + 16 b)
    const int rr_i = NB == 1 ? j / L : 0, n_i = NB == 1 ? j % L : j;
    uint4* my_stage = stage[wave];

    // loader role of this lane: piece lane % 8 of rows lane / 8 and lane / 8 + 8
    const int lr = lane >> 3, lc = lane & 7;
    const int32_t tok_lo = __shfl(c.tok, lr, 64), tok_hi = __shfl(c.tok, lr + 8, 64);
    const uint16_t* src_lo = a.x + (int64_t)(tok_lo >= 0 ? tok_lo : 0) * D + 8 * lc;
    const uint16_t* src_hi = a.x + (int64_t)(tok_hi >= 0 ? tok_hi : 0) * D + 8 * lc;
    const int slot_lo = tile_swz(lr, lc), slot_hi = tile_swz(lr + 8, lc);
    // operand role: pieces 2 kg and 2 kg + 1 of row j
    const int rd0 = tile_swz(j, 2 * kg), rd1 = tile_swz(j, 2 * kg + 1);

    for (int pass = 0; pass < c.n_runs; pass += P) {
        int32_t row_leaf = -1;
        for (int rr = 0; rr < P && pass + rr < c.n_runs; ++rr) {
            const int32_t lf = leaf_of_run(c, pass + rr);
            if (rr_i == rr) row_leaf = lf;
        }
        const uint16_t* arow[NB];
        bool a_ok[NB];
        f32x4_t acc[NB];
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            a_ok[b] = row_leaf >= 0 && n_i + 16 * b < L;
            arow[b] = a.w1 + ((int64_t)(a_ok[b] ? row_leaf : 0) * L + (a_ok[b] ? n_i + 16 * b : 0)) * D + 16 * kg;
            acc[b] = f32x4_t{0.f, 0.f, 0.f, 0.f};
        }
        // one group = CH K steps: fetch (weights rows in operand layout, token rows coalesced) ...
        auto fetch = [&](int pp0, uint4 (&av)[NB][CH], uint4 (&xv)[CH]) {
#pragma unroll
            for (int u = 0; u < CH; ++u) {
#pragma unroll
                for (int b = 0; b < NB; ++b) av[b][u] = make_uint4(0, 0, 0, 0);
                xv[u] = make_uint4(0, 0, 0, 0);
            }
#pragma unroll
            for (int u = 0; u < CH; ++u) {
                const int pp = pp0 + (u >> 1);                  // wave-uniform
                const int k0 = 64 * pp + 8 * (u & 1);           // + 16 kg is in arow
#pragma unroll
                for (int b = 0; b < NB; ++b)
                    if (pp < n_pairs && a_ok[b] && (!DTAIL || k0 + 16 * kg < D)) av[b][u] = *(const uint4*)(arow[b] + k0);
                // u even: rows 0..7 of pair pp, u odd: rows 8..15
                const int32_t tk = (u & 1) ? tok_hi : tok_lo;
                if (pp < n_pairs && tk >= 0 && (!DTAIL || 64 * pp + 8 * lc < D))
                    xv[u] = load_stream((const uint4*)(((u & 1) ? src_hi : src_lo) + 64 * pp));
            }
        };
        // ... and consume: token rows through the wave's LDS buffer into operand layout, then the MFMAs
        auto consume = [&](const uint4 (&av)[NB][CH], const uint4 (&xv)[CH]) {
            __builtin_amdgcn_wave_barrier();     // the operand reads of the previous group are done
#pragma unroll
            for (int u = 0; u < CH; ++u) my_stage[128 * (u >> 1) + ((u & 1) ? slot_hi : slot_lo)] = xv[u];
            __builtin_amdgcn_wave_barrier();     // LDS executes a wave's accesses in order
#pragma unroll
            for (int u = 0; u < CH; ++u) {
                const uint4 bv = my_stage[128 * (u >> 1) + ((u & 1) ? rd1 : rd0)];
#pragma unroll
                for (int b = 0; b < NB; ++b)
                    acc[b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, av[b][u]),
                                                                     __builtin_bit_cast(bf16x8_t, bv), acc[b], 0, 0, 0);
            }
        };
        constexpr int kStep = CH / 2;        // pairs per group
        if (NB == 1) {
            // two groups in flight: the next one travels while this one is transposed and multiplied
            uint4 av0[NB][CH], xv0[CH], av1[NB][CH], xv1[CH];
            fetch(0, av0, xv0);
            for (int pp0 = 0; pp0 < n_pairs; pp0 += 2 * kStep) {
                const bool more = pp0 + kStep < n_pairs;
                if (more) fetch(pp0 + kStep, av1, xv1);
                consume(av0, xv0);
                if (more) {
                    if (pp0 + 2 * kStep < n_pairs) fetch(pp0 + 2 * kStep, av0, xv0);
                    consume(av1, xv1);
                }
            }
        } else {
            for (int pp0 = 0; pp0 < n_pairs; pp0 += kStep) {
                uint4 av[NB][CH], xv[CH];
                fetch(pp0, av, xv);
                consume(av, xv);
            }
        }
        // lane (j, kg) holds rows 4 kg + q of column j: the entries of the token's own run are its
        // hidden pre-activations
        if (NB > 1) {
            // one run per pass; rows 4 kg + q of block b are neurons 16 b + 4 kg + q
            if (c.tok >= 0 && c.run == pass) {
#pragma unroll
                for (int b = 0; b < NB; ++b) {
                    const int n0 = 16 * b + 4 * kg;
                    if (L % 4 == 0) {
                        if (n0 < L) {
                            float v[4];
#pragma unroll
                            for (int q = 0; q < 4; ++q)
                                v[q] = activate(acc[b][q] + bf16_to_f32(a.b1[(int64_t)c.leaf * L + n0 + q]), a.act);
                            *(uint2*)(a.hidden + (int64_t)c.tok * L + n0) =
                                make_uint2(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]));
                        }
                    } else {
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            if (n0 + q < L) {
                                const float v = activate(acc[b][q] + bf16_to_f32(a.b1[(int64_t)c.leaf * L + n0 + q]), a.act);
                                a.hidden[(int64_t)c.tok * L + n0 + q] = f32_to_bf16(v);
                            }
                        }
                    }
                }
            }
        } else if (L % 4 == 0) {
            const int rr = (4 * kg) / L, n0 = (4 * kg) % L;
            if (c.tok >= 0 && rr < P && c.run == pass + rr) {
                float v[4];
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    v[q] = activate(acc[0][q] + bf16_to_f32(a.b1[(int64_t)c.leaf * L + n0 + q]), a.act);
                *(uint2*)(a.hidden + (int64_t)c.tok * L + n0) = make_uint2(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]));
            }
        } else {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int rho = 4 * kg + q, rr = rho / L, n = rho % L;
                if (c.tok >= 0 && rr < P && c.run == pass + rr) {
                    const float v = activate(acc[0][q] + bf16_to_f32(a.b1[(int64_t)c.leaf * L + n]), a.act);
                    a.hidden[(int64_t)c.tok * L + n] = f32_to_bf16(v);
                }
            }
        }
    }
}

// ---- output kernel: out[token] = W2[leaf]^T h[token] + b2[leaf] ----
//
// WIDE (leaf width 17..32): one run per pass; the first instruction carries neurons 0..15 and the
// bias, a second one accumulates neurons 16..31 on top.
template <bool WIDE>
__global__ __launch_bounds__(256) void leaf_output_kernel(const TilesArgs a) {
    const int lane = threadIdx.x & 63;
    const int64_t unit = xcd_contiguous_block() * 4 + (threadIdx.x >> 6);
    const int64_t tile = unit / a.units_per_tile;
    if (tile >= a.n_tiles) return;
    const int r_first = (int)(unit % a.units_per_tile) * kRangesPerWave;   // first 128-wide range of this wave
    const int j = lane & 15, kg = lane >> 4;
    const int O = a.O, L = a.L;
    const int P = WIDE ? 1 : 16 / L;
    const TileColumn c = tile_column(a, tile, j);
    if (a.split > 0 && c.n_runs >= a.split) return;

    // token rows this lane stores: rows 4 kg + q of the tile
    uint16_t* orow[4];
    int run_row[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int32_t tq = __shfl(c.tok, 4 * kg + q, 64);
        run_row[q] = tq >= 0 ? __shfl(c.run, 4 * kg + q, 64) : -1;
        orow[q] = a.out + (int64_t)(tq >= 0 ? tq : 0) * O + 8 * j;
    }

    for (int pass = 0; pass < c.n_runs; pass += P) {
        // K slots 4 kg + q: W2 row of (run, neuron) pair rho = 4 kg + q, and b2 row of run 4 kg + q
        const uint16_t* wptr[4];
        const uint16_t* bptr[4];
        bool w_ok[4], b_ok[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) w_ok[q] = b_ok[q] = false;
        int32_t w_leaf[4] = {0, 0, 0, 0}, b_leaf[4] = {0, 0, 0, 0};
        for (int rr = 0; rr < P && pass + rr < c.n_runs; ++rr) {
            const int32_t lf = leaf_of_run(c, pass + rr);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                if (WIDE ? rr == 0 : (4 * kg + q) / L == rr) { w_leaf[q] = lf; w_ok[q] = true; }
                if (4 * kg + q == rr) { b_leaf[q] = lf; b_ok[q] = true; }
            }
        }
        uint32_t h01 = 0, h23 = 0;               // this lane's four K slots of h, as two bf16 pairs
        uint32_t g01 = 0, g23 = 0;               // WIDE: the same for neurons 16 + 4 kg + q
        float iq[4];
        if (L % 4 == 0) {
            // the four slots are four consecutive neurons of one run: one 8-byte load
            const int rr = WIDE ? 0 : (4 * kg) / L, n0 = WIDE ? 4 * kg : (4 * kg) % L;
            if (c.tok >= 0 && rr < P && c.run == pass + rr) {
                const uint2 hv = *(const uint2*)(a.hidden + (int64_t)c.tok * L + n0);
                h01 = hv.x;
                h23 = hv.y;
                if (WIDE && 16 + n0 < L) {
                    const uint2 gv = *(const uint2*)(a.hidden + (int64_t)c.tok * L + 16 + n0);
                    g01 = gv.x;
                    g23 = gv.y;
                }
            }
        }
        const uint16_t* wptr2[4];
        bool w2_ok[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int rho = 4 * kg + q, rr = WIDE ? 0 : rho / L, n = WIDE ? rho : rho % L;
            wptr[q] = a.w2 + ((int64_t)w_leaf[q] * L + n) * O + 8 * j;
            bptr[q] = a.b2 + (int64_t)b_leaf[q] * O + 8 * j;
            w2_ok[q] = WIDE && w_ok[q] && 16 + rho < L;
            wptr2[q] = a.w2 + ((int64_t)w_leaf[q] * L + (w2_ok[q] ? 16 + rho : 0)) * O + 8 * j;
            if (L % 4 != 0) {
                const bool mine = c.tok >= 0 && rr < P && c.run == pass + rr;
                const uint32_t hb = mine ? a.hidden[(int64_t)c.tok * L + n] : 0u;
                if (q < 2) h01 |= hb << (16 * q);
                else h23 |= hb << (16 * (q - 2));
                if (WIDE) {
                    const uint32_t gb = (mine && 16 + rho < L) ? a.hidden[(int64_t)c.tok * L + 16 + rho] : 0u;
                    if (q < 2) g01 |= gb << (16 * q);
                    else g23 |= gb << (16 * (q - 2));
                }
            }
            iq[q] = (c.tok >= 0 && rho < P && c.run == pass + rho) ? 1.0f : 0.0f;
        }
        const uint4 a2u = make_uint4(h01, h23, pack_bf16x2(iq[0], iq[1]), pack_bf16x2(iq[2], iq[3]));
        const bf16x8_t a2 = __builtin_bit_cast(bf16x8_t, a2u);
        const bf16x8_t a2w = __builtin_bit_cast(bf16x8_t, make_uint4(g01, g23, 0u, 0u));
        bool st_ok[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) st_ok[q] = run_row[q] >= pass && run_row[q] < pass + P;

        uint4 wv[kRangesPerWave][4], bv[kRangesPerWave][4], wv2[WIDE ? kRangesPerWave : 1][4];
#pragma unroll
        for (int g = 0; g < kRangesPerWave; ++g) {
            const int o0 = 128 * (r_first + g);
            const bool ok = o0 + 8 * j < O;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                wv[g][q] = make_uint4(0, 0, 0, 0);
                bv[g][q] = make_uint4(0, 0, 0, 0);
                if (ok && w_ok[q]) wv[g][q] = *(const uint4*)(wptr[q] + o0);
                if (ok && b_ok[q]) bv[g][q] = *(const uint4*)(bptr[q] + o0);
                if (WIDE) {
                    wv2[g][q] = make_uint4(0, 0, 0, 0);
                    if (ok && w2_ok[q]) wv2[g][q] = *(const uint4*)(wptr2[q] + o0);
                }
            }
        }
#pragma unroll
        for (int g = 0; g < kRangesPerWave; ++g) {
            const int o0 = 128 * (r_first + g);
            const uint4* w = wv[g];
            const uint4* b = bv[g];
            const f32x4_t zero = {0.f, 0.f, 0.f, 0.f};
            f32x4_t d[8];
#pragma unroll
            for (int cc = 0; cc < 8; ++cc) {
                const uint4 f = make_uint4(pack_half(dword_of(w[0], cc), dword_of(w[1], cc), cc & 1),
                                           pack_half(dword_of(w[2], cc), dword_of(w[3], cc), cc & 1),
                                           pack_half(dword_of(b[0], cc), dword_of(b[1], cc), cc & 1),
                                           pack_half(dword_of(b[2], cc), dword_of(b[3], cc), cc & 1));
                d[cc] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a2, __builtin_bit_cast(bf16x8_t, f), zero, 0, 0, 0);
                if (WIDE) {
                    const uint4* w2r = wv2[g];
                    const uint4 f2 = make_uint4(pack_half(dword_of(w2r[0], cc), dword_of(w2r[1], cc), cc & 1),
                                                pack_half(dword_of(w2r[2], cc), dword_of(w2r[3], cc), cc & 1), 0u, 0u);
                    d[cc] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a2w, __builtin_bit_cast(bf16x8_t, f2), d[cc], 0, 0, 0);
                }
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
        }
    }
}

// bf16, leaf width <= 32, 16-byte aligned rows of x, W1, W2, b2 and out
bool tiles_shape_ok(const Problem& p) {
    auto al = [](const void* q, uintptr_t m) { return (reinterpret_cast<uintptr_t>(q) & (m - 1)) == 0; };
    return p.bf16 && p.L <= kTilesMaxLeafWidth && p.D % 8 == 0 && p.O % 8 == 0 && p.D < (1 << 30) && p.O < (1 << 30) &&
           al(p.x, 16) && al(p.leaf_w1, 16) && al(p.leaf_w2, 16) && al(p.leaf_b2, 16) && al(p.out, 16);
}

// hidden: workspace of T * L bf16 values
hipError_t launch_leaf_tiles(const Problem& p, const int32_t* slot_leaf, const int32_t* perm, void* hidden,
                             hipStream_t s, void (*between)(hipStream_t), int split) {
    if (p.T == 0) return hipSuccess;
    TilesArgs a;
    a.split = split;
    a.x = (const uint16_t*)p.x;
    a.w1 = (const uint16_t*)p.leaf_w1;
    a.b1 = (const uint16_t*)p.leaf_b1;
    a.w2 = (const uint16_t*)p.leaf_w2;
    a.b2 = (const uint16_t*)p.leaf_b2;
    a.out = (uint16_t*)p.out;
    a.hidden = (uint16_t*)hidden;
    a.perm = perm;
    a.slot_leaf = slot_leaf;
    a.T = p.T;
    a.n_tiles = (p.T + 15) / 16;
    a.D = (int)p.D;
    a.O = (int)p.O;
    a.L = p.L;
    a.act = p.act;
    const int n_ranges = (int)((p.O + 127) / 128);
    a.units_per_tile = (n_ranges + kRangesPerWave - 1) / kRangesPerWave;
    const int64_t blocks_h = ((a.n_tiles + 3) / 4 + kXcds - 1) / kXcds * kXcds;
    const bool wide = p.L > 16;
    note_launch("leaf_hidden_kernel<%s,%d>", p.D % 64 != 0 ? "ktail" : "k64", wide ? 2 : 1);
    if (p.D % 64 != 0) {
        if (wide) leaf_hidden_kernel<true, 2><<<dim3((unsigned)blocks_h), dim3(256), 0, s>>>(a);
        else leaf_hidden_kernel<true, 1><<<dim3((unsigned)blocks_h), dim3(256), 0, s>>>(a);
    } else {
        if (wide) leaf_hidden_kernel<false, 2><<<dim3((unsigned)blocks_h), dim3(256), 0, s>>>(a);
        else leaf_hidden_kernel<false, 1><<<dim3((unsigned)blocks_h), dim3(256), 0, s>>>(a);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (between) between(s);
    const int64_t blocks_o = ((a.n_tiles * a.units_per_tile + 3) / 4 + kXcds - 1) / kXcds * kXcds;
    note_launch("leaf_output_kernel<%s>", wide ? "wide" : "narrow");
    if (wide) leaf_output_kernel<true><<<dim3((unsigned)blocks_o), dim3(256), 0, s>>>(a);
    else leaf_output_kernel<false><<<dim3((unsigned)blocks_o), dim3(256), 0, s>>>(a);
    return hipGetLastError();
}

}  // namespace fff
