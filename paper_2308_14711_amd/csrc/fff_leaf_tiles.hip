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

constexpr int kChunk = 8;    // K steps of the first contraction in flight per lane
constexpr int kRanges = 2;   // 64-wide output ranges of the second contraction in flight per lane

__device__ __forceinline__ uint32_t pack_lo(uint32_t a, uint32_t b) { return (a & 0xffffu) | (b << 16); }
__device__ __forceinline__ uint32_t pack_hi(uint32_t a, uint32_t b) { return (a >> 16) | (b & 0xffff0000u); }

__global__ __launch_bounds__(512) void leaf_tiles_kernel(const TilesArgs a) {
    extern __shared__ f32x4_t part[];        // [2][W][64] partial tiles of the first contraction
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, W = blockDim.x >> 6;
    const int64_t tile = blockIdx.x;
    const int j = lane & 15, kg = lane >> 4;
    const int D = a.D, O = a.O, L = a.L;
    const int P = 16 / L;                    // runs per pass

    // this lane's column: slot, token, leaf (all four 16-lane rows hold the same 16 columns)
    const int64_t slot = tile * 16 + j;
    const bool vj = slot < a.T;
    const int32_t tok = vj ? a.perm[slot] : 0;
    const int32_t leaf = vj ? a.leaf_idx[tok] : -1;
    const int32_t prev = __shfl_up(leaf, 1, 16);
    const uint32_t ch16 = (uint32_t)__ballot(vj && j > 0 && leaf != prev) & 0xffffu;
    const int run_j = __popc(ch16 & ((2u << j) - 1u));
    const int n_runs = __popc(ch16) + 1;

    // token rows this lane stores at the end: rows 4 kg + q
    int32_t tok_row[4], run_row[4];
    bool v_row[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        tok_row[q] = __shfl(tok, 4 * kg + q, 64);
        run_row[q] = __shfl(run_j, 4 * kg + q, 64);
        v_row[q] = tile * 16 + 4 * kg + q < a.T;
    }
    const int rr_i = j / L, n_i = j % L;     // A row j of the first contraction = (run rr_i of the pass, neuron n_i)
    int rr_q[4], n_q[4];                      // K slots 4 kg + q of the second contraction, same pairing
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        rr_q[q] = (4 * kg + q) / L;
        n_q[q] = (4 * kg + q) % L;
    }
    const uint16_t* xrow = a.x + (int64_t)tok * D;
    const int n_pairs = (D + 63) / 64;       // pairs of K steps (64 elements of a row each)

    int buf = 0;
    for (int pass = 0; pass < n_runs; pass += P, buf ^= 1) {
        // leaf of every run of this pass, handed to the lanes that need it
        int32_t row_leaf = -1, w2_leaf[4] = {-1, -1, -1, -1}, b2_leaf[4] = {-1, -1, -1, -1};
        for (int rr = 0; rr < P && pass + rr < n_runs; ++rr) {
            const uint32_t m = (uint32_t)__ballot(vj && run_j == pass + rr) & 0xffffu;
            const int32_t lf = __shfl(leaf, __ffs(m) - 1, 64);
            if (rr_i == rr) row_leaf = lf;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                if (rr_q[q] == rr) w2_leaf[q] = lf;
                if (4 * kg + q == rr) b2_leaf[q] = lf;
            }
        }

        // first contraction over D.  The K index is only a summation order, so step s gives
        // lane group kg the 8 elements at 64 (s / 2) + 16 kg + 8 (s % 2): the two steps of a pair
        // read 32 contiguous bytes per lane and the four lane groups cover a whole 128-byte line.
        // This wave takes pairs wave, wave + W, ...; kChunk steps are fetched before any is used.
        const uint16_t* arow = a.w1 + ((int64_t)(row_leaf >= 0 ? row_leaf : 0) * L + n_i) * D;
        const bool a_ok = row_leaf >= 0;
        f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
        for (int p0 = wave; p0 < n_pairs; p0 += W * (kChunk / 2)) {
            uint4 av[kChunk], bv[kChunk];
#pragma unroll
            for (int u = 0; u < kChunk; ++u) {
                const int k0 = 64 * (p0 + W * (u >> 1)) + 16 * kg + 8 * (u & 1);
                av[u] = make_uint4(0, 0, 0, 0);
                bv[u] = make_uint4(0, 0, 0, 0);
                if (a_ok && k0 < D) av[u] = *(const uint4*)(arow + k0);
                if (vj && k0 < D) bv[u] = *(const uint4*)(xrow + k0);
            }
#pragma unroll
            for (int u = 0; u < kChunk; ++u)
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, av[u]),
                                                              __builtin_bit_cast(bf16x8_t, bv[u]), acc, 0, 0, 0);
        }
        // sum the partial tiles of the W waves (two buffers, so one barrier per pass is enough)
        f32x4_t* mine_part = part + (buf * W) * 64;
        mine_part[wave * 64 + lane] = acc;
        __syncthreads();
        acc = mine_part[lane];
        for (int w = 1; w < W; ++w) acc += mine_part[w * 64 + lane];

        // activation, mask to the token's own run, append the run indicators
        float hq[4], iq[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const bool mine = vj && rr_q[q] < P && run_j == pass + rr_q[q];
            float v = 0.f;
            if (mine) v = activate(acc[q] + bf16_to_f32(a.b1[(int64_t)leaf * L + n_q[q]]), a.act);
            hq[q] = v;
            iq[q] = (vj && 4 * kg + q < P && run_j == pass + 4 * kg + q) ? 1.0f : 0.0f;
        }
        const uint4 a2u = make_uint4(pack_bf16x2(hq[0], hq[1]), pack_bf16x2(hq[2], hq[3]),
                                     pack_bf16x2(iq[0], iq[1]), pack_bf16x2(iq[2], iq[3]));
        const bf16x8_t a2 = __builtin_bit_cast(bf16x8_t, a2u);

        const uint16_t* wptr[4];
        const uint16_t* bptr[4];
        bool st_ok[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            wptr[q] = w2_leaf[q] >= 0 ? a.w2 + ((int64_t)w2_leaf[q] * L + n_q[q]) * O : nullptr;
            bptr[q] = b2_leaf[q] >= 0 ? a.b2 + (int64_t)b2_leaf[q] * O : nullptr;
            st_ok[q] = v_row[q] && run_row[q] >= pass && run_row[q] < pass + P;
        }

        // second contraction, 64 outputs per step; the rows of kRanges steps are fetched before
        // the first of them is multiplied, so their latencies overlap
        for (int og = 4 * j + 64 * wave; og < O + 4 * j; og += 64 * kRanges * W) {
            uint2 wv[kRanges][4], bv2[kRanges][4];
#pragma unroll
            for (int g = 0; g < kRanges; ++g) {
                const int o0 = og + 64 * W * g;
                const bool ok = o0 < O;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    wv[g][q] = (wptr[q] && ok) ? *(const uint2*)(wptr[q] + o0) : make_uint2(0, 0);
                    bv2[g][q] = (bptr[q] && ok) ? *(const uint2*)(bptr[q] + o0) : make_uint2(0, 0);
                }
            }
#pragma unroll
            for (int g = 0; g < kRanges; ++g) {
                const int o0 = og + 64 * W * g;
                const uint2* w = wv[g];
                const uint2* b = bv2[g];
                const f32x4_t zero = {0.f, 0.f, 0.f, 0.f};
                const uint4 f0 = make_uint4(pack_lo(w[0].x, w[1].x), pack_lo(w[2].x, w[3].x),
                                            pack_lo(b[0].x, b[1].x), pack_lo(b[2].x, b[3].x));
                const uint4 f1 = make_uint4(pack_hi(w[0].x, w[1].x), pack_hi(w[2].x, w[3].x),
                                            pack_hi(b[0].x, b[1].x), pack_hi(b[2].x, b[3].x));
                const uint4 f2 = make_uint4(pack_lo(w[0].y, w[1].y), pack_lo(w[2].y, w[3].y),
                                            pack_lo(b[0].y, b[1].y), pack_lo(b[2].y, b[3].y));
                const uint4 f3 = make_uint4(pack_hi(w[0].y, w[1].y), pack_hi(w[2].y, w[3].y),
                                            pack_hi(b[0].y, b[1].y), pack_hi(b[2].y, b[3].y));
                const f32x4_t d0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a2, __builtin_bit_cast(bf16x8_t, f0), zero, 0, 0, 0);
                const f32x4_t d1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a2, __builtin_bit_cast(bf16x8_t, f1), zero, 0, 0, 0);
                const f32x4_t d2 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a2, __builtin_bit_cast(bf16x8_t, f2), zero, 0, 0, 0);
                const f32x4_t d3 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a2, __builtin_bit_cast(bf16x8_t, f3), zero, 0, 0, 0);
                if (o0 < O) {
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        if (st_ok[q]) {
                            const uint2 o2 = make_uint2(pack_bf16x2(d0[q], d1[q]), pack_bf16x2(d2[q], d3[q]));
                            *(uint2*)(a.out + (int64_t)tok_row[q] * O + o0) = o2;
                        }
                    }
                }
            }
        }
    }
}

// bf16, leaf width <= 16, rows of x / W1 16-byte aligned, rows of W2 / b2 / out 8-byte aligned
bool tiles_shape_ok(const Problem& p) {
    auto al = [](const void* q, uintptr_t m) { return (reinterpret_cast<uintptr_t>(q) & (m - 1)) == 0; };
    return p.bf16 && p.L <= 16 && p.D % 8 == 0 && p.O % 4 == 0 && p.D < (1 << 30) && p.O < (1 << 30) &&
           al(p.x, 16) && al(p.leaf_w1, 16) && al(p.leaf_w2, 8) && al(p.leaf_b2, 8) && al(p.out, 8);
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
    const int64_t n_pairs = (p.D + 63) / 64, n_ranges = (p.O + 63) / 64;
    const int64_t big = n_pairs > n_ranges ? n_pairs : n_ranges;
    int W = 4;
    while (W < 8 && big > 4 * W) W *= 2;
    const size_t lds = sizeof(float) * 4 * 64 * 2 * (size_t)W;
    leaf_tiles_kernel<<<dim3((unsigned)a.n_tiles), dim3(64 * W), lds, s>>>(a);
    return hipGetLastError();
}

}  // namespace fff
