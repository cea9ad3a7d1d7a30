// Forward_I with nodes of size n >= 1 inside a pre-norm residual block, in one launch.
//
// The Definition (section "Algorithm") makes a node a <D, n, 1> feedforward network with a
// sigmoid on its output: logit = c + sum_j v_j act(u_j . z + a_j), and Forward_I (Algorithm 1)
// goes right when the node output is >= 1/2, i.e. logit >= 0.  Used as a transformer layer
// (section "Fast feedforward layers as building blocks") the network sees the layer-normalised
// token z = LayerNorm(x) and the block returns x + FFF(z).
//
// A token stays with the same lanes from the load of x to the store of its output row: the
// normalisation is two sums over those lanes and the normalised row is never written anywhere.
// Every weight row the token meets (n per node, l + l for the leaf) is one coalesced 16-byte load
// per lane and piece; the rows of a few neurons are requested together so that their latencies
// overlap.  All decisions come out of sums that give every lane of the token the same bits.
// Two kernels: rows of up to 128 pieces (1024 bf16 / 512 fp32 features) give a token the 16 lanes
// of a DPP row, four tokens to a wave (block_group_kernel); longer rows give it a whole wave and
// keep the row in fp32 (block_kernel).
#include "fff_device.h"
#include "fff_internal.h"

namespace fff {
BlockTuning g_block_tuning;
namespace {

struct BlockArgs {
    const void* x;
    const void* gamma;     // null: no normalisation
    const void* beta;
    const void* node_w1;   // [NN, n, D]
    const void* node_b1;   // [NN, n]
    const void* node_w2;   // [NN, n]
    const void* node_b2;   // [NN]
    const void* leaf_w1;
    const void* leaf_b1;
    const void* leaf_w2;
    const void* leaf_b2;
    void* out;
    int32_t* leaf_idx;     // may be null
    int64_t T;
    int D, O, depth, n, L, act, residual;
    int top;               // node levels whose rows the lane-group kernel keeps in LDS
    float eps;
};

// neurons whose rows are in flight together: up to 8 pieces per lane at a time
constexpr int batch_for(int nv) { return nv >= 8 ? 1 : nv >= 4 ? 2 : 4; }

// fp32 values of one 16-byte piece
template <bool BF16> struct Piece;
template <> struct Piece<true> {
    static constexpr int kElems = 8;
    static __device__ __forceinline__ void unpack(const uint4& p, float* f) {
        f[0] = bf16_lo(p.x); f[1] = bf16_hi(p.x); f[2] = bf16_lo(p.y); f[3] = bf16_hi(p.y);
        f[4] = bf16_lo(p.z); f[5] = bf16_hi(p.z); f[6] = bf16_lo(p.w); f[7] = bf16_hi(p.w);
    }
    static __device__ __forceinline__ uint4 pack(const float* f) {
        return make_uint4(pack_bf16x2(f[0], f[1]), pack_bf16x2(f[2], f[3]), pack_bf16x2(f[4], f[5]),
                          pack_bf16x2(f[6], f[7]));
    }
};
template <> struct Piece<false> {
    static constexpr int kElems = 4;
    static __device__ __forceinline__ void unpack(const uint4& p, float* f) {
        f[0] = __uint_as_float(p.x); f[1] = __uint_as_float(p.y); f[2] = __uint_as_float(p.z);
        f[3] = __uint_as_float(p.w);
    }
    static __device__ __forceinline__ uint4 pack(const float* f) {
        return make_uint4(__float_as_uint(f[0]), __float_as_uint(f[1]), __float_as_uint(f[2]),
                          __float_as_uint(f[3]));
    }
};

// NV: 16-byte pieces per lane, so rows of up to 64 NV pieces
template <bool BF16, int NV>
__global__ __launch_bounds__(256) void block_kernel(const BlockArgs a) {
    typedef Piece<BF16> P;
    constexpr int E = P::kElems;
    constexpr int kBatch = batch_for(NV);
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t wave = (int64_t)blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave;
    const int64_t n_waves = (int64_t)gridDim.x * (blockDim.x / kWave);
    const int pd = a.D / E, po = a.O / E;            // pieces per input row, per output row
    const int64_t first_leaf_row = ((int64_t)1 << a.depth) - 1;

    // piece index of slot i of this lane, clamped into the row (slots past the row hold zeros
    // in z, so whatever weight they fetch does not count), and whether the slot is real
    int vd[NV], vo[NV];
    bool okd[NV], oko[NV];
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int v = lane + kWave * i;
        okd[i] = v < pd;
        oko[i] = v < po;
        vd[i] = okd[i] ? v : pd - 1;
        vo[i] = oko[i] ? v : po - 1;
    }

    for (int64_t t = wave; t < a.T; t += n_waves) {
        float z[NV][E];
        const uint4* xrow = (const uint4*)a.x + t * pd;
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const uint4 p = xrow[vd[i]];
            P::unpack(p, z[i]);
#pragma unroll
            for (int e = 0; e < E; ++e) z[i][e] = okd[i] ? z[i][e] : 0.0f;
        }
        if (a.gamma) {
            // mean, then the mean of squared deviations (divisor D), both over the whole wave
            float s = 0.0f;
#pragma unroll
            for (int i = 0; i < NV; ++i)
#pragma unroll
                for (int e = 0; e < E; ++e) s += z[i][e];
            const float mean = group_sum<kWave>(s) / (float)a.D;
            float q = 0.0f;
#pragma unroll
            for (int i = 0; i < NV; ++i)
#pragma unroll
                for (int e = 0; e < E; ++e) {
                    const float c = okd[i] ? z[i][e] - mean : 0.0f;
                    q = fmaf(c, c, q);
                }
            const float var = group_sum<kWave>(q) / (float)a.D;
            const float rstd = 1.0f / sqrtf(var + a.eps);
#pragma unroll
            for (int i = 0; i < NV; ++i) {
                float g[E], b[E];
                P::unpack(((const uint4*)a.gamma)[vd[i]], g);
                P::unpack(((const uint4*)a.beta)[vd[i]], b);
#pragma unroll
                for (int e = 0; e < E; ++e) z[i][e] = okd[i] ? fmaf((z[i][e] - mean) * rstd, g[e], b[e]) : 0.0f;
            }
        }

        // dot products of z with `cnt` (1..kBatch) consecutive rows starting at row0 of w;
        // rows past cnt repeat the last one and are ignored by the caller
        auto dots = [&](const void* w, int64_t row0, int cnt, float* s) {
            uint4 p[kBatch][NV];
#pragma unroll
            for (int j = 0; j < kBatch; ++j) {
                const int64_t row = row0 + (j < cnt ? j : cnt - 1);
#pragma unroll
                for (int i = 0; i < NV; ++i) p[j][i] = ((const uint4*)w)[row * pd + vd[i]];
            }
#pragma unroll
            for (int j = 0; j < kBatch; ++j) {
                float acc = 0.0f;
#pragma unroll
                for (int i = 0; i < NV; ++i) {
                    float f[E];
                    P::unpack(p[j][i], f);
#pragma unroll
                    for (int e = 0; e < E; ++e) acc = fmaf(f[e], z[i][e], acc);
                }
                s[j] = acc;
            }
#pragma unroll
            for (int j = 0; j < kBatch; ++j) s[j] = group_sum<kWave>(s[j]);
        };

        // descent: node i (heap order) has hidden neurons i n .. i n + n - 1
        int64_t node = 0;
        for (int m = 0; m < a.depth; ++m) {
            float logit = Elem<BF16>::load(a.node_b2, node);
            for (int j0 = 0; j0 < a.n; j0 += kBatch) {
                const int cnt = a.n - j0 < kBatch ? a.n - j0 : kBatch;
                float s[kBatch];
                dots(a.node_w1, node * a.n + j0, cnt, s);
#pragma unroll
                for (int j = 0; j < kBatch; ++j) {
                    if (j < cnt) {
                        const int64_t neuron = node * a.n + j0 + j;
                        const float h = activate(s[j] + Elem<BF16>::load(a.node_b1, neuron), a.act);
                        logit = fmaf(Elem<BF16>::load(a.node_w2, neuron), h, logit);
                    }
                }
            }
            // the same bits in every lane: the branch is uniform
            node = 2 * node + (logit >= 0.0f ? 2 : 1);
            node = __builtin_amdgcn_readfirstlane((int)node);
        }
        const int64_t leaf = node - first_leaf_row;
        if (a.leaf_idx && lane == 0) a.leaf_idx[t] = (int32_t)leaf;

        // leaf: hidden neurons in batches, each batch added to the output row at once
        float y[NV][E];
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            P::unpack(((const uint4*)a.leaf_b2)[leaf * po + vo[i]], y[i]);
        }
        for (int r0 = 0; r0 < a.L; r0 += kBatch) {
            const int cnt = a.L - r0 < kBatch ? a.L - r0 : kBatch;
            float s[kBatch];
            dots(a.leaf_w1, leaf * a.L + r0, cnt, s);
            uint4 p[kBatch][NV];
#pragma unroll
            for (int j = 0; j < kBatch; ++j) {
                const int64_t row = leaf * a.L + r0 + (j < cnt ? j : cnt - 1);
#pragma unroll
                for (int i = 0; i < NV; ++i) p[j][i] = ((const uint4*)a.leaf_w2)[row * po + vo[i]];
            }
#pragma unroll
            for (int j = 0; j < kBatch; ++j) {
                const int64_t row = leaf * a.L + r0 + (j < cnt ? j : cnt - 1);
                float h = activate(s[j] + Elem<BF16>::load(a.leaf_b1, row), a.act);
                h = j < cnt ? h : 0.0f;
#pragma unroll
                for (int i = 0; i < NV; ++i) {
                    float f[E];
                    P::unpack(p[j][i], f);
#pragma unroll
                    for (int e = 0; e < E; ++e) y[i][e] = fmaf(h, f[e], y[i][e]);
                }
            }
        }

        // residual sum with the token as it came in (O == D then), and the store; a lane reads
        // exactly the pieces it then writes, so out may be x itself
        uint4* orow = (uint4*)a.out + t * po;
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            if (a.residual) {
                float f[E];
                P::unpack(xrow[vo[i]], f);
#pragma unroll
                for (int e = 0; e < E; ++e) y[i][e] += f[e];
            }
            if (oko[i]) orow[vo[i]] = P::pack(y[i]);
        }
    }
}

// Lanes 0..3 of every aligned group of four ("quad") hold a, b, c, d: every lane gets lane Q's value.
template <int Q> __device__ __forceinline__ float quad_pick(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), Q * 0x55, 0xf, 0xf, false));
}
// ... and their sum, the same bits in all four (each step adds the same two partial sums in both
// lanes of a pair)
__device__ __forceinline__ float quad_sum(float v) {
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0xB1, 0xf, 0xf, false));   // lanes 1 0 3 2
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x4E, 0xf, 0xf, false));   // lanes 2 3 0 1
    return v;
}

// Rows of up to 16 NV pieces: a token is owned by the 16 lanes of one DPP row, four tokens to a
// wave, so a weight-row instruction serves four tokens and a dot product is reduced with four row
// steps.  The normalised row is kept as two packed bf16 rows, z = hi + lo with hi = bf16(z) and
// lo = bf16(z - hi) (TWO; a relative 2^-17 of each element, below the fp32 accumulation noise of
// a 768-term dot product), so that the dot products run on the packed dot instruction against the
// weights as loaded: half the instructions of unpack-and-multiply, in the registers of one fp32
// row.  Without normalisation a bf16 token is its own hi row (TWO = false); fp32 rows stay fp32.
// The sums of a batch of neurons are spread over the lanes of a quad, so that one evaluation of
// the activation serves the batch.
template <bool BF16, int NV, bool TWO>
__global__ __launch_bounds__(256) void block_group_kernel(const BlockArgs a) {
    typedef Piece<BF16> P;
    constexpr int E = P::kElems;
    constexpr int kLpt = 16;                            // lanes per token
    constexpr int kRows = NV >= 6 ? 2 : 4;              // weight rows requested together per token
    static_assert(BF16 || !TWO, "fp32 rows are kept as they are");
    constexpr int kGroups = 256 / kLpt;                 // tokens a block holds at a time
    extern __shared__ uint4 top_rows[];                 // node_w1 rows of the levels above a.top
    const int sub = threadIdx.x & (kLpt - 1);
    const int quad = threadIdx.x & 3;
    const int grp_in_block = threadIdx.x / kLpt;
    const int pd = a.D / E, po = a.O / E;
    const int64_t first_leaf_row = ((int64_t)1 << a.depth) - 1;

    int vd[NV], vo[NV];
    bool okd[NV], oko[NV];
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int v = sub + kLpt * i;
        okd[i] = v < pd;
        oko[i] = v < po;
        vd[i] = okd[i] ? v : pd - 1;
        vo[i] = oko[i] ? v : po - 1;
    }

    // The hidden-neuron rows of the top levels are the first rows of node_w1 (heap order): one
    // copy per block, then every token of the block reads them at LDS latency.
    if (a.top > 0) {
        const int staged = a.n * ((1 << a.top) - 1) * pd;
        for (int i = threadIdx.x; i < staged; i += 256) top_rows[i] = ((const uint4*)a.node_w1)[i];
        __syncthreads();
    }
    const auto lds_row = [&](int64_t row, int i) { return top_rows[(int)row * pd + vd[i]]; };
    const auto mem_row = [&](int64_t row, int i) { return ((const uint4*)a.node_w1)[row * pd + vd[i]]; };

    for (int64_t t = (int64_t)blockIdx.x * kGroups + grp_in_block; t < a.T; t += (int64_t)gridDim.x * kGroups) {
        const uint4* xrow = (const uint4*)a.x + t * pd;
        uint4 zh[NV], zl[TWO ? NV : 1];
#pragma unroll
        for (int i = 0; i < NV; ++i) zh[i] = keep_if(okd[i], xrow[vd[i]]);
        if (a.gamma) {
            float f[NV][E];
            float s = 0.0f;
#pragma unroll
            for (int i = 0; i < NV; ++i) {
                P::unpack(zh[i], f[i]);
#pragma unroll
                for (int e = 0; e < E; ++e) s += f[i][e];
            }
            const float mean = group_sum<kLpt>(s) / (float)a.D;
            float q = 0.0f;
#pragma unroll
            for (int i = 0; i < NV; ++i)
#pragma unroll
                for (int e = 0; e < E; ++e) {
                    const float c = okd[i] ? f[i][e] - mean : 0.0f;
                    q = fmaf(c, c, q);
                }
            const float var = group_sum<kLpt>(q) / (float)a.D;
            const float rstd = 1.0f / sqrtf(var + a.eps);
#pragma unroll
            for (int i = 0; i < NV; ++i) {
                float g[E], b[E];
                P::unpack(((const uint4*)a.gamma)[vd[i]], g);
                P::unpack(((const uint4*)a.beta)[vd[i]], b);
#pragma unroll
                for (int e = 0; e < E; ++e) f[i][e] = okd[i] ? fmaf((f[i][e] - mean) * rstd, g[e], b[e]) : 0.0f;
                zh[i] = P::pack(f[i]);
                if (TWO) {
                    float hi[E];
                    P::unpack(zh[i], hi);
#pragma unroll
                    for (int e = 0; e < E; ++e) hi[e] = f[i][e] - hi[e];
                    zl[TWO ? i : 0] = P::pack(hi);
                }
            }
        } else if (TWO) {
#pragma unroll
            for (int i = 0; i < NV; ++i) zl[TWO ? i : 0] = make_uint4(0, 0, 0, 0);
        }

        // z . row for the pieces of one weight row, summed over the token's 16 lanes
        auto dotz = [&](const uint4 (&w)[NV]) {
            float a0 = 0.0f, a1 = 0.0f;
#pragma unroll
            for (int i = 0; i < NV; ++i) {
                a0 = Elem<BF16>::dot(zh[i], w[i], a0);
                if (TWO) a1 = Elem<BF16>::dot(zl[TWO ? i : 0], w[i], a1);
            }
            return a0 + a1;
        };

        int64_t node = 0;
        // nodes of one hidden neuron (the usual case) go a row at a time
        const auto narrow_level = [&](const auto& load_row) {
            uint4 w[NV];
#pragma unroll
            for (int i = 0; i < NV; ++i) w[i] = load_row(node, i);
            const float pre = group_sum<kLpt>(dotz(w)) + Elem<BF16>::load(a.node_b1, node);
            const float logit = fmaf(Elem<BF16>::load(a.node_w2, node), activate(pre, a.act), Elem<BF16>::load(a.node_b2, node));
            node = 2 * node + (logit >= 0.0f ? 2 : 1);
        };
        const auto wide_level = [&](const auto& load_row) {
            float logit = Elem<BF16>::load(a.node_b2, node);
            for (int j0 = 0; j0 < a.n; j0 += kRows) {
                // the rows of up to kRows hidden neurons are requested together; past the node's last
                // neuron the last row is asked for again (same addresses, no new traffic to L2) and
                // its result dropped -- a batch without conditionals keeps the register count down
                const int cnt = a.n - j0 < kRows ? a.n - j0 : kRows;
                uint4 w[kRows][NV];
#pragma unroll
                for (int j = 0; j < kRows; ++j) {
                    const int64_t row = node * a.n + j0 + (j < cnt ? j : cnt - 1);
#pragma unroll
                    for (int i = 0; i < NV; ++i) w[j][i] = load_row(row, i);
                }
                float sj[kRows];
#pragma unroll
                for (int j = 0; j < kRows; ++j) sj[j] = dotz(w[j]);
#pragma unroll
                for (int j = 0; j < kRows; ++j) sj[j] = group_sum<kLpt>(sj[j]);
                // every lane holds all the batch's sums; lane q of each quad takes neuron q through
                // the activation, so one evaluation serves the whole batch (kRows <= 4)
                float mine = sj[0];
#pragma unroll
                for (int j = 1; j < kRows; ++j) mine = quad == j ? sj[j] : mine;
                const bool live = quad < cnt;
                const int64_t neuron = node * a.n + j0 + (live ? quad : 0);
                const float h = activate(mine + Elem<BF16>::load(a.node_b1, neuron), a.act);
                logit += quad_sum(live ? Elem<BF16>::load(a.node_w2, neuron) * h : 0.0f);
            }
            // the 16 lanes of a token hold the same bits, so they take the same child
            node = 2 * node + (logit >= 0.0f ? 2 : 1);
        };
        if (a.n == 1) {
            for (int m = 0; m < a.top; ++m) narrow_level(lds_row);
            for (int m = a.top; m < a.depth; ++m) narrow_level(mem_row);
        } else {
            for (int m = 0; m < a.top; ++m) wide_level(lds_row);
            for (int m = a.top; m < a.depth; ++m) wide_level(mem_row);
        }
        const int64_t leaf = node - first_leaf_row;
        if (a.leaf_idx && sub == 0) a.leaf_idx[t] = (int32_t)leaf;

        float y[NV][E];
#pragma unroll
        for (int i = 0; i < NV; ++i) P::unpack(((const uint4*)a.leaf_b2)[leaf * po + vo[i]], y[i]);
        for (int r0 = 0; r0 < a.L; r0 += kRows) {
            const int cnt = a.L - r0 < kRows ? a.L - r0 : kRows;
            float h[kRows];
            {
                uint4 w[kRows][NV];
#pragma unroll
                for (int j = 0; j < kRows; ++j) {
                    const int64_t row = leaf * a.L + r0 + (j < cnt ? j : cnt - 1);
#pragma unroll
                    for (int i = 0; i < NV; ++i) w[j][i] = ((const uint4*)a.leaf_w1)[row * pd + vd[i]];
                }
#pragma unroll
                for (int j = 0; j < kRows; ++j) h[j] = dotz(w[j]);
            }
#pragma unroll
            for (int j = 0; j < kRows; ++j) h[j] = group_sum<kLpt>(h[j]);
            uint4 w2[kRows][NV];
#pragma unroll
            for (int j = 0; j < kRows; ++j) {
                const int64_t row = leaf * a.L + r0 + (j < cnt ? j : cnt - 1);
#pragma unroll
                for (int i = 0; i < NV; ++i) w2[j][i] = ((const uint4*)a.leaf_w2)[row * po + vo[i]];
            }
            // one activation for the batch, as in the nodes; then every lane picks up each neuron's
            float mine = h[0];
#pragma unroll
            for (int j = 1; j < kRows; ++j) mine = quad == j ? h[j] : mine;
            const bool live = quad < cnt;
            const float hq = live ? activate(mine + Elem<BF16>::load(a.leaf_b1, leaf * a.L + r0 + (live ? quad : 0)), a.act)
                                  : 0.0f;
            h[0] = quad_pick<0>(hq);
            if constexpr (kRows > 1) h[1] = quad_pick<1>(hq);
            if constexpr (kRows > 2) h[2] = quad_pick<2>(hq);
            if constexpr (kRows > 3) h[3] = quad_pick<3>(hq);
#pragma unroll
            for (int j = 0; j < kRows; ++j) {
#pragma unroll
                for (int i = 0; i < NV; ++i) {
                    float f[E];
                    P::unpack(w2[j][i], f);
#pragma unroll
                    for (int e = 0; e < E; ++e) y[i][e] = fmaf(h[j], f[e], y[i][e]);
                }
            }
        }
        uint4* orow = (uint4*)a.out + t * po;
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            if (a.residual) {
                float f[E];
                P::unpack(xrow[vo[i]], f);
#pragma unroll
                for (int e = 0; e < E; ++e) y[i][e] += f[e];
            }
            if (oko[i]) orow[vo[i]] = P::pack(y[i]);
        }
    }
}

// Launch shape of the lane-group kernel: blocks of 256 threads, 16 tokens at a time.  Small
// batches: a block per 16 tokens, no staging.  From 32768 tokens on: two persistent blocks per
// compute unit, each keeping the hidden-neuron rows of as many top levels as fit its half of the
// LDS (blocks of 512 threads with all of it were measured too: slower on every shape tried).
template <bool BF16, int NV, bool TWO> hipError_t run_group(BlockArgs a, hipStream_t s) {
    const DeviceInfo di = device_info();
    int64_t blocks = (a.T + 15) / 16;
    const int64_t cap = 256 * 16;
    const int64_t row_bytes = (int64_t)a.D * (BF16 ? 2 : 4);
    size_t lds_limit = di.lds_per_block;
    if (lds_limit > 144 * 1024) lds_limit = 144 * 1024;
    const size_t lds_cap = lds_limit / 2;
    int top = 0;
    if (a.T >= 32768) {
        while (top < a.depth && top < 12 &&
               (size_t)(a.n * (((int64_t)1 << (top + 1)) - 1) * row_bytes) <= lds_cap)
            ++top;
    }
    if (g_block_tuning.top > 0 && g_block_tuning.top - 1 < top) top = (int)g_block_tuning.top - 1;
    g_block_tuning.last_top = top;
    a.top = top;
    const size_t lds_bytes = (size_t)(a.n * (((int64_t)1 << top) - 1) * row_bytes);
    if (top > 0) {
        const int64_t resident = (int64_t)di.cus * 2;
        if (blocks > resident) blocks = resident;
    } else if (blocks > cap) {
        blocks = cap;
    }
    auto kern = block_group_kernel<BF16, NV, TWO>;
    // raise this instantiation's dynamic LDS limit once per device (the limit only ever grows)
    static size_t lds_allowed_on[64];
    size_t& lds_allowed = lds_allowed_on[di.dev];
    if (lds_bytes > 48 * 1024 && lds_bytes > lds_allowed) {
        hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                           (int)lds_limit);
        if (e != hipSuccess) return e;
        lds_allowed = lds_limit;
    }
    note_launch("block_group_kernel<%s,%d,%s> n=%d top=%d", BF16 ? "bf16" : "f32", NV, TWO ? "hi+lo" : "plain", a.n, top);
    kern<<<dim3((unsigned)blocks), dim3(256), lds_bytes, s>>>(a);
    return hipGetLastError();
}

template <bool BF16, bool TWO> hipError_t pick_group(const BlockArgs& a, int nv, hipStream_t s) {
    if (nv <= 2) return run_group<BF16, 2, TWO>(a, s);
    if (nv <= 4) return run_group<BF16, 4, TWO>(a, s);
    if (nv <= 6) return run_group<BF16, 6, TWO>(a, s);
    return run_group<BF16, 8, TWO>(a, s);
}

// Any row length and alignment: one wave (one block) per token, element loads, the normalised
// value of an element recomputed from x, gamma and beta wherever it is used, the leaf's hidden
// activations through LDS.  Correct for every shape the vector kernels do not take; not fast.
constexpr int kGenericMaxLeafWidth = 4096;

template <bool BF16>
__global__ __launch_bounds__(kWave) void block_generic_kernel(const BlockArgs a) {
    __shared__ float hid[kGenericMaxLeafWidth];
    const int lane = threadIdx.x;
    const int64_t D = a.D, O = a.O;
    const int64_t first_leaf_row = ((int64_t)1 << a.depth) - 1;
    for (int64_t t = blockIdx.x; t < a.T; t += gridDim.x) {
        float mean = 0.0f, rstd = 1.0f;
        if (a.gamma) {
            float s = 0.0f;
            for (int64_t k = lane; k < D; k += kWave) s += Elem<BF16>::load(a.x, t * D + k);
            mean = group_sum<kWave>(s) / (float)D;
            float q = 0.0f;
            for (int64_t k = lane; k < D; k += kWave) {
                const float c = Elem<BF16>::load(a.x, t * D + k) - mean;
                q = fmaf(c, c, q);
            }
            rstd = 1.0f / sqrtf(group_sum<kWave>(q) / (float)D + a.eps);
        }
        auto z = [&](int64_t k) {
            const float v = Elem<BF16>::load(a.x, t * D + k);
            return a.gamma ? fmaf((v - mean) * rstd, Elem<BF16>::load(a.gamma, k), Elem<BF16>::load(a.beta, k)) : v;
        };
        auto dot = [&](const void* w, int64_t row) {
            float acc = 0.0f;
            for (int64_t k = lane; k < D; k += kWave) acc = fmaf(z(k), Elem<BF16>::load(w, row * D + k), acc);
            return group_sum<kWave>(acc);
        };
        int64_t node = 0;
        for (int m = 0; m < a.depth; ++m) {
            float logit = Elem<BF16>::load(a.node_b2, node);
            for (int j = 0; j < a.n; ++j) {
                const int64_t neuron = node * a.n + j;
                const float h = activate(dot(a.node_w1, neuron) + Elem<BF16>::load(a.node_b1, neuron), a.act);
                logit = fmaf(Elem<BF16>::load(a.node_w2, neuron), h, logit);
            }
            node = 2 * node + (logit >= 0.0f ? 2 : 1);
        }
        const int64_t leaf = node - first_leaf_row;
        if (a.leaf_idx && lane == 0) a.leaf_idx[t] = (int32_t)leaf;
        __syncthreads();                       // the previous token's readers of hid are done
        for (int r = 0; r < a.L; ++r) {
            const float h = activate(dot(a.leaf_w1, leaf * a.L + r) + Elem<BF16>::load(a.leaf_b1, leaf * a.L + r), a.act);
            if (lane == 0) hid[r] = h;
        }
        __syncthreads();
        for (int64_t o = lane; o < O; o += kWave) {
            float y = Elem<BF16>::load(a.leaf_b2, leaf * O + o);
            for (int r = 0; r < a.L; ++r) y = fmaf(hid[r], Elem<BF16>::load(a.leaf_w2, (leaf * a.L + r) * O + o), y);
            if (a.residual) y += Elem<BF16>::load(a.x, t * D + o);
            Elem<BF16>::store(a.out, t * O + o, y);
        }
    }
}

template <bool BF16, int NV> hipError_t run(const BlockArgs& a, int64_t blocks, hipStream_t s) {
    note_launch("block_kernel<%s,%d> n=%d", BF16 ? "bf16" : "f32", NV, a.n);
    block_kernel<BF16, NV><<<dim3((unsigned)blocks), dim3(256), 0, s>>>(a);
    return hipGetLastError();
}

template <bool BF16> hipError_t pick(const BlockArgs& a, int nv, int64_t blocks, hipStream_t s) {
    if (nv <= 1) return run<BF16, 1>(a, blocks, s);
    if (nv <= 2) return run<BF16, 2>(a, blocks, s);
    if (nv <= 4) return run<BF16, 4>(a, blocks, s);
    return run<BF16, 8>(a, blocks, s);
}

}  // namespace

constexpr int kGroupMaxPieces = 8 * 16;      // longest row the 16-lanes-per-token kernel holds
constexpr int kBlockMaxPieces = 8 * kWave;   // 16-byte pieces of the longest row a wave holds

// rows of 16-byte pieces, at most 512 of them (4096 bf16 or 2048 fp32 features)
bool block_shape_ok(const void* x, const void* out, const void* leaf_w1, const void* leaf_w2, int64_t D,
                    int64_t O, bool bf16) {
    const int per = bf16 ? 8 : 4;
    return vec_ok(x, D, bf16) && vec_ok(out, O, bf16) && vec_ok(leaf_w1, D, bf16) && vec_ok(leaf_w2, O, bf16) &&
           D / per <= kBlockMaxPieces && O / per <= kBlockMaxPieces;
}

hipError_t launch_forward_block(const Problem& p, const void* gamma, const void* beta, float eps,
                                const void* node_w1, const void* node_b1, const void* node_w2,
                                const void* node_b2, int node_size, bool residual, int32_t* leaf_idx,
                                hipStream_t s, bool vector_rows) {
    if (p.T == 0) return hipSuccess;
    BlockArgs a;
    a.x = p.x;
    a.gamma = gamma;
    a.beta = beta;
    a.node_w1 = node_w1;
    a.node_b1 = node_b1;
    a.node_w2 = node_w2;
    a.node_b2 = node_b2;
    a.leaf_w1 = p.leaf_w1;
    a.leaf_b1 = p.leaf_b1;
    a.leaf_w2 = p.leaf_w2;
    a.leaf_b2 = p.leaf_b2;
    a.out = p.out;
    a.leaf_idx = leaf_idx;
    a.T = p.T;
    a.D = (int)p.D;
    a.O = (int)p.O;
    a.depth = p.depth;
    a.n = node_size;
    a.L = p.L;
    a.act = p.act;
    a.residual = residual ? 1 : 0;
    a.top = 0;
    a.eps = eps;
    g_block_tuning.last_top = 0;
    if (!vector_rows) {
        int64_t gblocks = p.T < 256 * 32 ? p.T : 256 * 32;
        note_launch("block_generic_kernel<%s> n=%d", p.bf16 ? "bf16" : "f32", node_size);
        if (p.bf16) block_generic_kernel<true><<<dim3((unsigned)gblocks), dim3(kWave), 0, s>>>(a);
        else block_generic_kernel<false><<<dim3((unsigned)gblocks), dim3(kWave), 0, s>>>(a);
        return hipGetLastError();
    }
    const int per = p.bf16 ? 8 : 4;
    const int64_t pieces = (p.D > p.O ? p.D : p.O) / per;
    const int nv = (int)((pieces + kWave - 1) / kWave);
    // four waves a block, a wave a token; enough blocks to fill the chip several times over,
    // then the waves stride through the remaining tokens
    int64_t blocks = (p.T + 3) / 4;
    const int64_t cap = 256 * 16;
    if (blocks > cap) blocks = cap;
    if (pieces <= kGroupMaxPieces) {
        // sixteen lanes a token
        const int gnv = (int)((pieces + 15) / 16);
        if (!p.bf16) return pick_group<false, false>(a, gnv, s);
        return gamma ? pick_group<true, true>(a, gnv, s) : pick_group<true, false>(a, gnv, s);
    }
    return p.bf16 ? pick<true>(a, nv, blocks, s) : pick<false>(a, nv, blocks, s);
}

}  // namespace fff
