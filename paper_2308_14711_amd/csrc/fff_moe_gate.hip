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

// v or zeros, component by component (a conditional on the 16-byte struct itself is lowered
// through memory)
__device__ __forceinline__ uint4 keep_if(bool ok, const uint4& v) {
    return make_uint4(ok ? v.x : 0u, ok ? v.y : 0u, ok ? v.z : 0u, ok ? v.w : 0u);
}

__device__ __forceinline__ int swz(int row, int piece) { return 8 * row + ((piece + (row >> 1)) & 7); }

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

    // loader roles: 2 pieces of the token tile, 4 of the expert tile (8 consecutive threads = one
    // row's 128 bytes).  kDepth chunks are kept in flight in registers: with one chunk ahead the
    // loop is a chain of memory round trips (12 of them for D = 768), since a chunk's arithmetic
    // is only 16 MFMAs per wave.
    // Loads are unconditional with clamped addresses; rows past the end and K past D are zeroed
    // when the chunk goes to LDS.  (A predicated 16-byte load compiles to guarded dword loads with
    // a wait each, and a select right after the load makes the wave wait for it there.)
    constexpr int kDepth = 4;
    const int pc = tid & 7;                      // this thread's piece of every row it loads
    const int64_t ta0 = t0 + (tid >> 3), ta1 = ta0 + 32;
    const int64_t eb0 = e0 + (tid >> 3), eb1 = eb0 + 32, eb2 = eb0 + 64, eb3 = eb0 + 96;
    const uint16_t* const pa0 = a.x + (ta0 < a.T ? ta0 : a.T - 1) * D + 8 * pc;
    const uint16_t* const pa1 = a.x + (ta1 < a.T ? ta1 : a.T - 1) * D + 8 * pc;
    const uint16_t* const pb0 = a.gate_w + (eb0 < a.G ? eb0 : a.G - 1) * D + 8 * pc;
    const uint16_t* const pb1 = a.gate_w + (eb1 < a.G ? eb1 : a.G - 1) * D + 8 * pc;
    const uint16_t* const pb2 = a.gate_w + (eb2 < a.G ? eb2 : a.G - 1) * D + 8 * pc;
    const uint16_t* const pb3 = a.gate_w + (eb3 < a.G ? eb3 : a.G - 1) * D + 8 * pc;
    const bool va0 = ta0 < a.T, va1 = ta1 < a.T;
    const bool vb0 = eb0 < a.G, vb1 = eb1 < a.G, vb2 = eb2 < a.G, vb3 = eb3 < a.G;
    const int sa0 = swz(tid >> 3, pc), sa1 = swz((tid >> 3) + 32, pc);
    const int sb0 = sa0, sb1 = sa1, sb2 = swz((tid >> 3) + 64, pc), sb3 = swz((tid >> 3) + 96, pc);
    struct Chunk { uint4 a0, a1, b0, b1, b2, b3; };   // named members: they stay in registers
#define FFF_GATE_FETCH(KC, Q)                                                   \
    do {                                                                        \
        const int koff_ = (KC) * kGateK + 8 * pc < D ? (KC) * kGateK : 0;       \
        Q.a0 = *(const uint4*)(pa0 + koff_);                                    \
        Q.a1 = *(const uint4*)(pa1 + koff_);                                    \
        Q.b0 = *(const uint4*)(pb0 + koff_);                                    \
        Q.b1 = *(const uint4*)(pb1 + koff_);                                    \
        Q.b2 = *(const uint4*)(pb2 + koff_);                                    \
        Q.b3 = *(const uint4*)(pb3 + koff_);                                    \
    } while (0)
#define FFF_GATE_STASH(KC, BUF, Q)                                              \
    do {                                                                        \
        const bool kin_ = (KC) * kGateK + 8 * pc < D;                           \
        lds_a[BUF][sa0] = keep_if(kin_ && va0, Q.a0);                               \
        lds_a[BUF][sa1] = keep_if(kin_ && va1, Q.a1);                               \
        lds_b[BUF][sb0] = keep_if(kin_ && vb0, Q.b0);                               \
        lds_b[BUF][sb1] = keep_if(kin_ && vb1, Q.b1);                               \
        lds_b[BUF][sb2] = keep_if(kin_ && vb2, Q.b2);                               \
        lds_b[BUF][sb3] = keep_if(kin_ && vb3, Q.b3);                               \
    } while (0)

    f32x4_t acc[4][2];
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) acc[mt][nt] = f32x4_t{0.f, 0.f, 0.f, 0.f};

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

    // The loop body has no branches (the wait counters are only tracked along straight code):
    // chunks past the end are fetched from a clamped address and stored as zeros, and the trip
    // count is rounded up to a multiple of kDepth; the extra MFMAs add zeros.
    Chunk c0, c1, c2, c3;
    FFF_GATE_FETCH(0, c0);
    FFF_GATE_FETCH(1, c1);
    FFF_GATE_FETCH(2, c2);
    FFF_GATE_FETCH(3, c3);
    FFF_GATE_STASH(0, 0, c0);
    __syncthreads();
    // one chunk: refill the register slot the chunk came from, multiply out of LDS buffer BUF,
    // put the next chunk into the other buffer.  Step u of a chunk gives lane group kg the piece
    // 2 kg + u of every row (K is only a summation order).
#define FFF_GATE_STEP(KC, BUF, CUR, NEXT)                                                                          \
    do {                                                                                                           \
        FFF_GATE_FETCH((KC) + kDepth, CUR);                                                                        \
        _Pragma("unroll") for (int u = 0; u < 2; ++u) {                                                            \
            bf16x8_t fa[4], fb[2];                                                                                 \
            _Pragma("unroll") for (int mt = 0; mt < 4; ++mt)                                                       \
                fa[mt] = __builtin_bit_cast(bf16x8_t, lds_a[BUF][swz(16 * mt + j, 2 * kg + u)]);                   \
            _Pragma("unroll") for (int nt = 0; nt < 2; ++nt)                                                       \
                fb[nt] = __builtin_bit_cast(bf16x8_t, lds_b[BUF][swz(32 * wv + 16 * nt + j, 2 * kg + u)]);         \
            _Pragma("unroll") for (int mt = 0; mt < 4; ++mt)                                                       \
                _Pragma("unroll") for (int nt = 0; nt < 2; ++nt)                                                   \
                    acc[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa[mt], fb[nt], acc[mt][nt], 0, 0, 0);   \
        }                                                                                                          \
        FFF_GATE_STASH((KC) + 1, (BUF) ^ 1, NEXT);                                                                 \
        __syncthreads();                                                                                           \
    } while (0)
    for (int kc0 = 0; kc0 < n_chunks; kc0 += kDepth) {
        FFF_GATE_STEP(kc0 + 0, 0, c0, c1);
        FFF_GATE_STEP(kc0 + 1, 1, c1, c2);
        FFF_GATE_STEP(kc0 + 2, 0, c2, c3);
        FFF_GATE_STEP(kc0 + 3, 1, c3, c0);
    }
#undef FFF_GATE_STEP
#undef FFF_GATE_STASH
#undef FFF_GATE_FETCH

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
    const int64_t blocks = (T + kGateTokens - 1) / kGateTokens * a.n_eblocks;
    moe_gate_kernel<<<dim3((unsigned)blocks), dim3(256), 0, s>>>(a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    moe_pick_kernel<<<dim3((unsigned)((T + 3) / 4)), dim3(256), 0, s>>>(a.cand_val, a.cand_idx, T, a.n_eblocks,
                                                                           expert_idx);
    return hipGetLastError();
}

}  // namespace fff
