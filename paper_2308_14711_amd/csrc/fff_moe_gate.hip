// Gating of a mixture of experts with one engaged expert and no noise -- the lookup the paper
// times against the tree descent (section "Inference speed comparison", k = 1): logits
// g[t][e] = gate_w[e] . x[t] (+ gate_b[e]), expert_idx[t] = argmax over e (lowest index among
// equal logits; a NaN logit never wins).  It replaces the descent; bucketing and the leaf
// kernels then run on expert_idx unchanged.
//
// The work is a dense [T, D] x [D, G] contraction, so it goes to the matrix cores: a block owns
// 64 tokens x 128 experts, walks K = D in chunks of 64 through double-buffered LDS tiles
// (16-byte pieces, coalesced loads, the rotation swizzle tile_swz that keeps the operand reads free
// of bank conflicts), and each of its 4 waves
// holds 4 x 2 accumulator tiles of v_mfma_f32_16x16x32_bf16.  The logits never reach memory: a
// wave reduces its 32 experts per token with DPP row steps, the waves meet in LDS, and the block
// writes one (value, index) candidate per token; a second small kernel picks the best candidate
// per token over the expert blocks.  The token tiles of one expert block run back to back on one
// XCD, so the gating matrix streams from HBM once while the (small) token rows stay cached.
#include "fff_device.h"
#include "fff_internal.h"
#include "fff_mfma_tile.h"

namespace fff {
namespace {

constexpr int kGateTokens = kTileM;     // tokens per block
constexpr int kGateExperts = kTileN;    // experts per block

struct GateArgs {
    const uint16_t* x;
    const uint16_t* gate_w;
    const uint16_t* gate_b;      // may be null
    float* cand_val;             // [T][n_eblocks]
    int32_t* cand_idx;           // [T][n_eblocks]
    int64_t T, G;
    int D, n_eblocks;
    int64_t n_ttiles;
};

// (v, i) <- the better of (v, i) and (v2, i2): larger value, then lower index
__device__ __forceinline__ void better(float& v, int32_t& i, float v2, int32_t i2) {
    const bool take = v2 > v || (v2 == v && i2 < i);
    v = take ? v2 : v;
    i = take ? i2 : i;
}

template <int N> __device__ __forceinline__ int32_t row_rotate_i(int32_t i) {
    return __builtin_amdgcn_update_dpp(0, i, 0x120 + N, 0xf, 0xf, false);
}

template <int N> __device__ __forceinline__ void row_step(float& v, int32_t& i) {
    const float v2 = row_rotate<N>(v);
    const int32_t i2 = __builtin_amdgcn_update_dpp(0, i, 0x120 + N, 0xf, 0xf, false);
    better(v, i, v2, i2);
}

__global__ __launch_bounds__(256) void moe_gate_kernel(const GateArgs a) {
    __shared__ TileLds tile;
    __shared__ float part_v[4][kGateTokens];
    __shared__ int32_t part_i[4][kGateTokens];
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int j = lane & 15, kg = lane >> 4;
    // the token tiles of one expert block run back to back on one XCD (whose L2 then serves the
    // expert block's rows to all of them): logical block = expert block * token tiles + token tile
    const int64_t lb = xcd_contiguous_block();
    if (lb >= (int64_t)a.n_eblocks * a.n_ttiles) return;      // padding of the grid to a multiple of 8
    const int eb = (int)(lb / a.n_ttiles);
    const int64_t t0 = (lb % a.n_ttiles) * kGateTokens;
    const int64_t e0 = (int64_t)eb * kGateExperts;
    const int D = a.D;

    f32x4_t acc[4][2];
    // the biases of this lane's two experts are requested now, long before they are needed
    const float ninf = -__builtin_inff();
    float bias[2];
    int32_t eidx[2];
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) {
        const int64_t e = e0 + 32 * wv + 16 * nt + j;
        const bool ok = e < a.G;
        eidx[nt] = ok ? (int32_t)e : 0x7fffffff;
        bias[nt] = !ok ? ninf : (a.gate_b ? bf16_to_f32(a.gate_b[e]) : 0.0f);
    }

    mfma_tile_64x128<4>(a.x, D, a.T, a.gate_w, D, a.G, D, t0, e0, tile, acc);

    // lane (j, kg) of tile (mt, nt) holds tokens 16 mt + 4 kg + q (q = 0..3) against expert
    // e0 + 32 wv + 16 nt + j: bias, then the best expert per token over the wave's 32
    // (the row maximum first, then the lowest index among the lanes that hold it: two chains of
    // single DPP instructions per token instead of a compare-and-select exchange of pairs)
#pragma unroll
    for (int mt = 0; mt < 4; ++mt) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            float v0 = acc[mt][0][q] + bias[0];
            float v1 = acc[mt][1][q] + bias[1];
            v0 = v0 != v0 ? ninf : v0;                     // a NaN logit never wins
            v1 = v1 != v1 ? ninf : v1;
            float m = fmaxf(v0, v1);
            m = fmaxf(m, row_rotate<8>(m));
            m = fmaxf(m, row_rotate<4>(m));
            m = fmaxf(m, row_rotate<2>(m));
            m = fmaxf(m, row_rotate<1>(m));
            int32_t c = v0 == m ? eidx[0] : (v1 == m ? eidx[1] : 0x7fffffff);
            c = min(c, row_rotate_i<8>(c));
            c = min(c, row_rotate_i<4>(c));
            c = min(c, row_rotate_i<2>(c));
            c = min(c, row_rotate_i<1>(c));
            if (j == 0) {
                part_v[wv][16 * mt + 4 * kg + q] = m;
                part_i[wv][16 * mt + 4 * kg + q] = c;
            }
        }
    }
    __syncthreads();
    if (tid < kGateTokens && t0 + tid < a.T) {
        float v = part_v[0][tid];
        int32_t i = part_i[0][tid];
#pragma unroll
        for (int w = 1; w < 4; ++w) better(v, i, part_v[w][tid], part_i[w][tid]);
        a.cand_val[(t0 + tid) * a.n_eblocks + eb] = v;
        a.cand_idx[(t0 + tid) * a.n_eblocks + eb] = i;
    }
}

// one wave per token: the best candidate over the expert blocks (lanes stride over the blocks)
__global__ __launch_bounds__(256) void moe_pick_kernel(const float* __restrict__ cand_val,
                                                       const int32_t* __restrict__ cand_idx, int64_t T,
                                                       int n_eblocks, int32_t* __restrict__ expert_idx) {
    const int lane = threadIdx.x & 63;
    const int64_t t = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (t >= T) return;
    float v = -__builtin_inff();
    int32_t i = 0x7fffffff;
    for (int b = lane; b < n_eblocks; b += kWave) better(v, i, cand_val[t * n_eblocks + b], cand_idx[t * n_eblocks + b]);
    row_step<8>(v, i);
    row_step<4>(v, i);
    row_step<2>(v, i);
    row_step<1>(v, i);
#pragma unroll
    for (int d = 16; d < kWave; d <<= 1) better(v, i, __shfl_xor(v, d, kWave), __shfl_xor(i, d, kWave));
    if (lane == 0) expert_idx[t] = i;
}

}  // namespace

int64_t moe_gate_blocks(int64_t n_experts) { return (n_experts + kGateExperts - 1) / kGateExperts; }

// bf16, D a multiple of 8, rows 16-byte aligned
bool moe_gate_shape_ok(const void* x, const void* gate_w, int64_t D, bool bf16) {
    return bf16 && vec_ok(x, D, true) && vec_ok(gate_w, D, true) && D < ((int64_t)1 << 30);
}

// cand: scratch of 2 * T * moe_gate_blocks(G) 32-bit words
hipError_t launch_moe_gate(const void* x, const void* gate_w, const void* gate_b, int64_t T, int64_t D,
                           int64_t n_experts, int32_t* cand, int32_t* expert_idx, hipStream_t s) {
    if (T == 0) return hipSuccess;
    GateArgs a;
    a.x = (const uint16_t*)x;
    a.gate_w = (const uint16_t*)gate_w;
    a.gate_b = (const uint16_t*)gate_b;
    a.n_eblocks = (int)moe_gate_blocks(n_experts);
    a.cand_val = (float*)cand;
    a.cand_idx = cand + T * a.n_eblocks;
    a.T = T;
    a.G = n_experts;
    a.D = (int)D;
    a.n_ttiles = (T + kGateTokens - 1) / kGateTokens;
    const int64_t blocks = (a.n_ttiles * a.n_eblocks + kXcds - 1) / kXcds * kXcds;
    note_launch("moe_gate_kernel + moe_pick_kernel");
    moe_gate_kernel<<<dim3((unsigned)blocks), dim3(256), 0, s>>>(a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    moe_pick_kernel<<<dim3((unsigned)((T + 3) / 4)), dim3(256), 0, s>>>(a.cand_val, a.cand_idx, T, a.n_eblocks,
                                                                           expert_idx);
    return hipGetLastError();
}

}  // namespace fff
