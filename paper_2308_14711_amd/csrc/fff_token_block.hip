// Small-batch launch of hard-routed FFF inference (Algorithm 1, Forward_I): one block per token.
//
// With a few hundred tokens the call is a chain of dependent loads: a node's row
// cannot be requested before the decision above it is known, so the time is the
// depth of the tree times one memory round trip, plus the leaf.  This kernel
// shortens that chain instead of streaming: every wave of a block holds the token
// row in registers; wave 0 walks the tree S levels per round trip by requesting
// the whole S-level subtree below the current node at once (2^S - 1 rows,
// contiguous level by level in heap order) and taking the S decisions locally,
// with wave sums that end in scalar registers.  The leaf it reaches goes through
// LDS to the other waves, which split the hidden neurons among them (little
// arithmetic per wave, many loads in flight per block); a wave requests the input
// and the output weights of its neurons together, and the partial output rows of
// the waves meet in LDS.
#include "fff_device.h"
#include "fff_internal.h"

namespace fff {
namespace {

constexpr int kTokenBlock = 512;
constexpr int kTokenWaves = kTokenBlock / kWave;

struct TokenArgs {
    const uint4* x;
    const uint4* node_w;
    const void* node_b;
    const uint4* w1;
    const void* b1;
    const void* w2;
    const void* b2;
    void* out;
    int32_t* leaf_idx;
    const int32_t* given_leaf;   // non-null: the leaf of every token is given, nothing is descended
    int64_t T, O;
    int depth, nvec, ovec, L, act;
};

template <bool BF16> __device__ __forceinline__ void widen(const uint4& v, float* f);
template <> __device__ __forceinline__ void widen<false>(const uint4& v, float* f) {
    f[0] = __uint_as_float(v.x);
    f[1] = __uint_as_float(v.y);
    f[2] = __uint_as_float(v.z);
    f[3] = __uint_as_float(v.w);
}
template <> __device__ __forceinline__ void widen<true>(const uint4& v, float* f) {
    f[0] = bf16_lo(v.x);
    f[1] = bf16_hi(v.x);
    f[2] = bf16_lo(v.y);
    f[3] = bf16_hi(v.y);
    f[4] = bf16_lo(v.z);
    f[5] = bf16_hi(v.z);
    f[6] = bf16_lo(v.w);
    f[7] = bf16_hi(v.w);
}

// Sum over the wave, returned as a wave-uniform value: DPP rotations inside each 16-lane row,
// then the four row sums are read out as scalars.  Every wave that sums the same values gets
// the same bits (same order of additions).
__device__ __forceinline__ float wave_sum(float v) {
    v = group_sum<16>(v);
    const int b = __float_as_int(v);
    const float s0 = __int_as_float(__builtin_amdgcn_readlane(b, 0));
    const float s1 = __int_as_float(__builtin_amdgcn_readlane(b, 16));
    const float s2 = __int_as_float(__builtin_amdgcn_readlane(b, 32));
    const float s3 = __int_as_float(__builtin_amdgcn_readlane(b, 48));
    return (s0 + s1) + (s2 + s3);
}

// NV: 16-byte vectors of a row per lane (rows of up to 64 * NV vectors); S: tree levels per round
// trip; OUTVEC: output rows are whole aligned vectors (else element-wise output through LDS).
//
// Every load is unconditional (a predicated 16-byte load compiles to four guarded dword loads
// and a wait each): lanes past the end of a row re-read its last vector against zeros of the
// token row, subtree rows past the last level and neurons past the leaf width re-read a valid
// row and their results are dropped.
template <bool BF16, int NV, int S, bool OUTVEC>
__global__ __launch_bounds__(kTokenBlock) void token_block_kernel(TokenArgs a) {
    constexpr int kPer = Elem<BF16>::kPerVec;
    constexpr int kSub = (1 << S) - 1;
    constexpr int kBatch = NV >= 8 ? 2 : 4;   // leaf neurons in flight per wave
    // LDS: the leaf found by wave 0 (one 16-byte slot), then OUTVEC: [waves][O] partial output rows;
    // else [L] hidden activations
    extern __shared__ float lds_all[];
    int* const lds_leaf = (int*)lds_all;
    float* const lds = lds_all + 4;
    const int lane = threadIdx.x & (kWave - 1);
    const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const uint4 zero = make_uint4(0, 0, 0, 0);
    int col[NV], ocol[NV];   // this lane's vectors of an input row / an output row, clamped
#pragma unroll
    for (int v = 0; v < NV; ++v) {
        const int c = v * kWave + lane;
        col[v] = c < a.nvec ? c : a.nvec - 1;
        ocol[v] = OUTVEC ? (c < a.ovec ? c : a.ovec - 1) : 0;
    }
    const int64_t last_node = (((int64_t)1 << a.depth) - 1) - 1;

    for (int64_t t = blockIdx.x; t < a.T; t += gridDim.x) {
        uint4 xv[NV];
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            const uint4 q = a.x[t * a.nvec + col[v]];
            xv[v] = v * kWave + lane < a.nvec ? q : zero;
        }

        // ---- descent by wave 0: S levels per round trip (Algorithm 1: logit >= 0 takes the right child)
        int64_t n = 0;   // position within the current level
        for (int m = 0; wv == 0 && !a.given_leaf && m < a.depth; m += S) {
            const int s = a.depth - m < S ? a.depth - m : S;
            const int64_t root = (((int64_t)1 << m) - 1 + n) + 1;   // heap row of the subtree's root, plus one
            uint4 rows[kSub][NV];
            float bias[kSub], acc[kSub];
#pragma unroll
            for (int k = 0; k < S; ++k) {
#pragma unroll
                for (int j = 0; j < (1 << k); ++j) {
                    int64_t row = (root << k) - 1 + j;   // level k below the root, j-th node
                    row = row < last_node ? row : last_node;
                    const int q = (1 << k) - 1 + j;
#pragma unroll
                    for (int v = 0; v < NV; ++v) rows[q][v] = a.node_w[row * a.nvec + col[v]];
                    bias[q] = Elem<BF16>::load(a.node_b, row);
                }
            }
#pragma unroll
            for (int q = 0; q < kSub; ++q) {
                float p = 0.0f;
#pragma unroll
                for (int v = 0; v < NV; ++v) p = Elem<BF16>::dot(xv[v], rows[q][v], p);
                acc[q] = wave_sum(p) + bias[q];
            }
            int j = 0;
#pragma unroll
            for (int k = 0; k < S; ++k) {
                // acc[2^k - 1 + j] as a chain of selects (registers cannot be indexed at run time)
                float logit = acc[(1 << k) - 1];
#pragma unroll
                for (int q = 1; q < (1 << k); ++q) logit = j == q ? acc[(1 << k) - 1 + q] : logit;
                j = k < s ? 2 * j + (logit >= 0.0f ? 1 : 0) : j;
            }
            n = (n << s) + j;
        }
        if (threadIdx.x == 0) {
            if (a.given_leaf) n = a.given_leaf[t];
            lds_leaf[0] = (int)n;
            if (a.leaf_idx) a.leaf_idx[t] = (int32_t)n;
        }
        __syncthreads();
        const int64_t leaf = lds_leaf[0];

        // ---- leaf: wave wv takes neurons wv, wv + waves, ...
        const int64_t nrow0 = leaf * a.L;
        float oacc[OUTVEC ? NV : 1][kPer];
        if (OUTVEC) {
#pragma unroll
            for (int v = 0; v < NV; ++v)
#pragma unroll
                for (int e = 0; e < kPer; ++e) oacc[v][e] = 0.0f;
        }
        for (int r0 = wv; r0 < a.L; r0 += kTokenWaves * kBatch) {
            uint4 w1[kBatch][NV], w2[OUTVEC ? kBatch : 1][NV];
            float b1[kBatch];
#pragma unroll
            for (int i = 0; i < kBatch; ++i) {
                int r = r0 + i * kTokenWaves;
                r = r < a.L ? r : a.L - 1;
#pragma unroll
                for (int v = 0; v < NV; ++v) {
                    w1[i][v] = a.w1[(nrow0 + r) * a.nvec + col[v]];
                    if (OUTVEC) w2[i][v] = ((const uint4*)a.w2)[(nrow0 + r) * a.ovec + ocol[v]];
                }
                b1[i] = Elem<BF16>::load(a.b1, nrow0 + r);
            }
#pragma unroll
            for (int i = 0; i < kBatch; ++i) {
                const int r = r0 + i * kTokenWaves;
                float p = 0.0f;
#pragma unroll
                for (int v = 0; v < NV; ++v) p = Elem<BF16>::dot(xv[v], w1[i][v], p);
                float h = activate(wave_sum(p) + b1[i], a.act);
                h = r < a.L ? h : 0.0f;
                if (OUTVEC) {
#pragma unroll
                    for (int v = 0; v < NV; ++v) {
                        float w[kPer];
                        widen<BF16>(w2[i][v], w);
#pragma unroll
                        for (int e = 0; e < kPer; ++e) oacc[v][e] = fmaf(h, w[e], oacc[v][e]);
                    }
                } else if (lane == 0 && r < a.L) {
                    lds[r] = h;
                }
            }
        }

        if (OUTVEC) {
            // partial rows of the waves meet in LDS; then one thread per output vector
#pragma unroll
            for (int v = 0; v < NV; ++v) {
                const int c = v * kWave + lane;
                if (c < a.ovec) {
                    float* dst = lds + (int64_t)wv * a.O + (int64_t)c * kPer;
#pragma unroll
                    for (int e = 0; e < kPer; e += 4)
                        *(float4*)(dst + e) = make_float4(oacc[v][e], oacc[v][e + 1], oacc[v][e + 2], oacc[v][e + 3]);
                }
            }
            __syncthreads();
            for (int c = threadIdx.x; c < a.ovec; c += kTokenBlock) {
                float y[kPer];
                widen<BF16>(((const uint4*)a.b2)[leaf * a.ovec + c], y);
#pragma unroll
                for (int w = 0; w < kTokenWaves; ++w) {
                    const float4* src = (const float4*)(lds + (int64_t)w * a.O + (int64_t)c * kPer);
#pragma unroll
                    for (int e = 0; e < kPer; e += 4) {
                        const float4 f = src[e / 4];
                        y[e] += f.x;
                        y[e + 1] += f.y;
                        y[e + 2] += f.z;
                        y[e + 3] += f.w;
                    }
                }
                uint4 o;
                if (BF16) {
                    o = make_uint4(pack_bf16x2(y[0], y[1]), pack_bf16x2(y[2], y[3]),
                                   pack_bf16x2(y[4 % kPer], y[5 % kPer]), pack_bf16x2(y[6 % kPer], y[7 % kPer]));
                } else {
                    o = make_uint4(__float_as_uint(y[0]), __float_as_uint(y[1]), __float_as_uint(y[2]),
                                   __float_as_uint(y[3]));
                }
                ((uint4*)a.out)[t * a.ovec + c] = o;
            }
        } else {
            __syncthreads();
            for (int64_t o = threadIdx.x; o < a.O; o += kTokenBlock) {
                float y = Elem<BF16>::load(a.b2, leaf * a.O + o);
                for (int r = 0; r < a.L; ++r) y = fmaf(lds[r], Elem<BF16>::load(a.w2, (nrow0 + r) * a.O + o), y);
                Elem<BF16>::store(a.out, t * a.O + o, y);
            }
        }
        __syncthreads();   // LDS is reused by the block's next token
    }
}

template <bool BF16, int NV, int S, bool OUTVEC>
hipError_t run_token(const Problem& p, int32_t* leaf_idx, const int32_t* given_leaf, hipStream_t s) {
    constexpr int kPer = Elem<BF16>::kPerVec;
    TokenArgs a;
    a.x = (const uint4*)p.x;
    a.node_w = (const uint4*)p.node_w;
    a.node_b = p.node_b;
    a.w1 = (const uint4*)p.leaf_w1;
    a.b1 = p.leaf_b1;
    a.w2 = p.leaf_w2;
    a.b2 = p.leaf_b2;
    a.out = p.out;
    a.leaf_idx = leaf_idx;
    a.given_leaf = given_leaf;
    a.T = p.T;
    a.O = p.O;
    a.depth = p.depth;
    a.nvec = (int)(p.D / kPer);
    a.ovec = OUTVEC ? (int)(p.O / kPer) : 0;
    a.L = p.L;
    a.act = p.act;
    const size_t lds_bytes = 16 + (OUTVEC ? (size_t)kTokenWaves * p.O * sizeof(float) : (size_t)p.L * sizeof(float));
    auto kern = token_block_kernel<BF16, NV, S, OUTVEC>;
    static bool raised[64];
    if (lds_bytes > 48 * 1024) {
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) dev = 0;
        if (!raised[dev]) {
            hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                               (int)kTokenMaxLds);
            if (e != hipSuccess) return e;
            raised[dev] = true;
        }
    }
    const int64_t blocks = p.T < kTokenMaxBlocks ? p.T : kTokenMaxBlocks;
    note_launch("token_block_kernel<%s,%d,%d,%s>", BF16 ? "bf16" : "f32", NV, S, OUTVEC ? "vec" : "elem");
    kern<<<dim3((unsigned)blocks), dim3(kTokenBlock), lds_bytes, s>>>(a);
    return hipGetLastError();
}

template <bool BF16, bool OUTVEC>
hipError_t dispatch_token(const Problem& p, int32_t* leaf_idx, const int32_t* given_leaf, hipStream_t s) {
    constexpr int kPer = Elem<BF16>::kPerVec;
    int64_t vecs = p.D / kPer;
    if (OUTVEC && p.O / kPer > vecs) vecs = p.O / kPer;
    // (vectors per lane, levels per round trip): 2^S - 1 rows of NV vectors stay under 32 registers x 4
    if (vecs <= 64) return run_token<BF16, 1, 3, OUTVEC>(p, leaf_idx, given_leaf, s);
    if (vecs <= 128) return run_token<BF16, 2, 3, OUTVEC>(p, leaf_idx, given_leaf, s);
    if (vecs <= 256) return run_token<BF16, 4, 3, OUTVEC>(p, leaf_idx, given_leaf, s);
    return run_token<BF16, 8, 2, OUTVEC>(p, leaf_idx, given_leaf, s);
}

bool token_out_vec(const Problem& p) {
    const int64_t per = p.bf16 ? 8 : 4;
    return vec_ok(p.out, p.O, p.bf16) && vec_ok(p.leaf_w2, p.O, p.bf16) && vec_ok(p.leaf_b2, p.O, p.bf16) &&
           p.O / per <= 8 * kWave && 16 + (size_t)kTokenWaves * p.O * sizeof(float) <= kTokenMaxLds;
}

}  // namespace

bool token_shape_ok(const Problem& p) {
    const int64_t per = p.bf16 ? 8 : 4;
    if (!vec_ok(p.x, p.D, p.bf16) || !vec_ok(p.leaf_w1, p.D, p.bf16)) return false;
    if (p.depth > 0 && !vec_ok(p.node_w, p.D, p.bf16)) return false;
    if (p.D / per > 8 * kWave) return false;
    return token_out_vec(p) || 16 + (size_t)p.L * sizeof(float) <= kTokenMaxLds;
}

hipError_t launch_token_block(const Problem& p, int32_t* leaf_idx, hipStream_t s, const int32_t* given_leaf) {
    const bool ov = token_out_vec(p);
    if (p.bf16)
        return ov ? dispatch_token<true, true>(p, leaf_idx, given_leaf, s)
                  : dispatch_token<true, false>(p, leaf_idx, given_leaf, s);
    return ov ? dispatch_token<false, true>(p, leaf_idx, given_leaf, s)
              : dispatch_token<false, false>(p, leaf_idx, given_leaf, s);
}

}  // namespace fff
