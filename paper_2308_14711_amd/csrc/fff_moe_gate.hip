// Gating of a mixture of experts with one engaged expert and no noise -- the lookup the paper
// times against the tree descent (section "Inference speed comparison", k = 1): logits
// g[t][e] = gate_w[e] . x[t] (+ gate_b[e]), expert_idx[t] = argmax over e (lowest index among
// equal logits; a NaN logit never wins).  It replaces the descent; bucketing and the leaf
// kernels then run on expert_idx unchanged.
//
// The work is a dense [T, D] x [D, G] contraction, so it goes to the matrix cores: a block owns
// 64 tokens x 128 experts, walks K = D in chunks of 64 through double-buffered LDS tiles
// (16-byte pieces, coalesced loads, the rotation swizzle that keeps the operand reads free of
// bank conflicts: piece c of row r at slot 8 r + ((c + r / 2) mod 8)), and each of its 4 waves
// holds 4 x 2 accumulator tiles of v_mfma_f32_16x16x32_bf16.  The logits never reach memory: a
// wave reduces its 32 experts per token with DPP row steps, the waves meet in LDS, and the block
// writes one (value, index) candidate per token; a second small kernel picks the best candidate
// per token over the expert blocks.  Blocks that share a token tile are adjacent in the grid, so
// the tile stays in L2 while the gating matrix streams from HBM once.
#include "fff_device.h"
#include "fff_internal.h"

namespace fff {
namespace {

constexpr int kGateTokens = 64;     // tokens per block
constexpr int kGateExperts = 128;   // experts per block
constexpr int kGateK = 64;          // K elements per chunk (8 pieces of 16 bytes per row)

struct GateArgs {
    const uint16_t* x;
    const uint16_t* gate_w;
    const uint16_t* gate_b;      // may be null
    float* cand_val;             // [T][n_eblocks]
    int32_t* cand_idx;           // [T][n_eblocks]
    int64_t T, G;
    int D, n_eblocks;
};

__device__ __forceinline__ int swz(int row, int piece) { return 8 * row + ((piece + (row >> 1)) & 7); }

// (v, i) <- the better of (v, i) and (v2, i2): larger value, then lower index
__device__ __forceinline__ void better(float& v, int32_t& i, float v2, int32_t i2) {
    const bool take = v2 > v || (v2 == v && i2 < i);
    v = take ? v2 : v;
    i = take ? i2 : i;
}

template <int N> __device__ __forceinline__ void row_step(float& v, int32_t& i) {
    const float v2 = row_rotate<N>(v);
    const int32_t i2 = __builtin_amdgcn_update_dpp(0, i, 0x120 + N, 0xf, 0xf, false);
    better(v, i, v2, i2);
}

__global__ __launch_bounds__(256) void moe_gate_kernel(const GateArgs a) {
    __shared__ uint4 lds_a[2][kGateTokens * 8];
    __shared__ uint4 lds_b[2][kGateExperts * 8];
    __shared__ float part_v[4][kGateTokens];
    __shared__ int32_t part_i[4][kGateTokens];
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int j = lane & 15, kg = lane >> 4;
    const int eb = (int)(blockIdx.x % a.n_eblocks);
    const int64_t t0 = (int64_t)(blockIdx.x / a.n_eblocks) * kGateTokens;
    const int64_t e0 = (int64_t)eb * kGateExperts;
    const int D = a.D;
    const int n_chunks = (D + kGateK - 1) / kGateK;
    const uint4 zero = make_uint4(0, 0, 0, 0);

    // loader roles: 2 pieces of the token tile, 4 of the expert tile (8 consecutive threads = one row's 128 bytes)
    uint4 ra[2], rb[4];
    auto fetch = [&](int kc) {
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int p = tid + 256 * u, row = p >> 3, c = p & 7;
            const int64_t t = t0 + row;
            const int k = kc * kGateK + 8 * c;
            ra[u] = (t < a.T && k < D) ? *(const uint4*)(a.x + t * D + k) : zero;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int p = tid + 256 * u, row = p >> 3, c = p & 7;
            const int64_t e = e0 + row;
            const int k = kc * kGateK + 8 * c;
            rb[u] = (e < a.G && k < D) ? *(const uint4*)(a.gate_w + e * D + k) : zero;
        }
    };
    auto stash = [&](int buf) {
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int p = tid + 256 * u;
            lds_a[buf][swz(p >> 3, p & 7)] = ra[u];
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int p = tid + 256 * u;
            lds_b[buf][swz(p >> 3, p & 7)] = rb[u];
        }
    };

    f32x4_t acc[4][2];
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) acc[mt][nt] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    fetch(0);
    stash(0);
    __syncthreads();
    for (int kc = 0; kc < n_chunks; ++kc) {
        const int buf = kc & 1;
        if (kc + 1 < n_chunks) fetch(kc + 1);
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            // K is only a summation order: step u gives lane group kg the piece 2 kg + u of every row
            bf16x8_t fa[4], fb[2];
#pragma unroll
            for (int mt = 0; mt < 4; ++mt)
                fa[mt] = __builtin_bit_cast(bf16x8_t, lds_a[buf][swz(16 * mt + j, 2 * kg + u)]);
#pragma unroll
            for (int nt = 0; nt < 2; ++nt)
                fb[nt] = __builtin_bit_cast(bf16x8_t, lds_b[buf][swz(32 * wv + 16 * nt + j, 2 * kg + u)]);
#pragma unroll
            for (int mt = 0; mt < 4; ++mt)
#pragma unroll
                for (int nt = 0; nt < 2; ++nt)
                    acc[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa[mt], fb[nt], acc[mt][nt], 0, 0, 0);
        }
        if (kc + 1 < n_chunks) stash(buf ^ 1);
        __syncthreads();
    }

    // lane (j, kg) of tile (mt, nt) holds tokens 16 mt + 4 kg + q (q = 0..3) against expert
    // e0 + 32 wv + 16 nt + j: bias, then the best expert per token over the wave's 32
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
#pragma unroll
    for (int mt = 0; mt < 4; ++mt) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            float v = acc[mt][0][q] + bias[0];
            v = v != v ? ninf : v;                       // a NaN logit never wins
            int32_t i = eidx[0];
            float v1 = acc[mt][1][q] + bias[1];
            v1 = v1 != v1 ? ninf : v1;
            better(v, i, v1, eidx[1]);
            row_step<8>(v, i);
            row_step<4>(v, i);
            row_step<2>(v, i);
            row_step<1>(v, i);
            if (j == 0) {
                part_v[wv][16 * mt + 4 * kg + q] = v;
                part_i[wv][16 * mt + 4 * kg + q] = i;
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

// one thread per token: the best candidate over the expert blocks
__global__ __launch_bounds__(256) void moe_pick_kernel(const float* __restrict__ cand_val,
                                                       const int32_t* __restrict__ cand_idx, int64_t T,
                                                       int n_eblocks, int32_t* __restrict__ expert_idx) {
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= T) return;
    float v = cand_val[t * n_eblocks];
    int32_t i = cand_idx[t * n_eblocks];
    for (int b = 1; b < n_eblocks; ++b) better(v, i, cand_val[t * n_eblocks + b], cand_idx[t * n_eblocks + b]);
    expert_idx[t] = i;
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
    const int64_t blocks = (T + kGateTokens - 1) / kGateTokens * a.n_eblocks;
    moe_gate_kernel<<<dim3((unsigned)blocks), dim3(256), 0, s>>>(a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    moe_pick_kernel<<<dim3((unsigned)((T + 255) / 256)), dim3(256), 0, s>>>(a.cand_val, a.cand_idx, T, a.n_eblocks,
                                                                           expert_idx);
    return hipGetLastError();
}

}  // namespace fff
