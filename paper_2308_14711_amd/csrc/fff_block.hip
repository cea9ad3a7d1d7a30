// Forward_I with nodes of size n >= 1 inside a pre-norm residual block, in one launch.
//
// The Definition (section "Algorithm") makes a node a <D, n, 1> feedforward network with a
// sigmoid on its output: logit = c + sum_j v_j act(u_j . z + a_j), and Forward_I (Algorithm 1)
// goes right when the node output is >= 1/2, i.e. logit >= 0.  Used as a transformer layer
// (section "Fast feedforward layers as building blocks") the network sees the layer-normalised
// token z = LayerNorm(x) and the block returns x + FFF(z).
//
// One wave owns a token from the load of x to the store of the output row.  The row lives in
// fp32 registers (lane l holds the 16-byte pieces l, l + 64, ...), so the normalisation is two
// wave sums and the normalised row is never rounded or written anywhere.  Every weight row the
// token meets (n per node, l + l for the leaf) is one coalesced 16-byte load per lane; the rows
// of up to four neurons are requested together so that their latencies overlap, and their four
// dot products are reduced over the wave together.  All decisions come out of wave sums that
// give every lane the same bits, so the tree index is wave-uniform.
#include "fff_device.h"
#include "fff_internal.h"

namespace fff {
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

template <bool BF16, int NV> hipError_t run(const BlockArgs& a, int64_t blocks, hipStream_t s) {
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
                                hipStream_t s) {
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
    a.eps = eps;
    const int per = p.bf16 ? 8 : 4;
    const int64_t pieces = (p.D > p.O ? p.D : p.O) / per;
    const int nv = (int)((pieces + kWave - 1) / kWave);
    // four waves a block, a wave a token; enough blocks to fill the chip several times over,
    // then the waves stride through the remaining tokens
    int64_t blocks = (p.T + 3) / 4;
    const int64_t cap = 256 * 16;
    if (blocks > cap) blocks = cap;
    return p.bf16 ? pick<true>(a, nv, blocks, s) : pick<false>(a, nv, blocks, s);
}

}  // namespace fff
