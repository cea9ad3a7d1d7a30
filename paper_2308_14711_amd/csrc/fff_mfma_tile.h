// The 64 x 128 MFMA tile shared by the dense contractions of this library (the gating of the
// mixture-of-experts comparator, the node and leaf contractions of the soft forward pass):
// C[m0 .. m0+63][n0 .. n0+127] = A[M, K] . B[N, K]^T for bf16 operands that are both K-contiguous,
// fp32 accumulation on v_mfma_f32_16x16x32_bf16.
//
// A block of 256 threads (4 waves) walks K in chunks of 64 through double-buffered LDS tiles
// (16-byte pieces, coalesced loads, piece c of row r at slot tile_swz(r, c): stores and operand
// reads are both free of bank conflicts).  Wave w owns columns 32 w .. 32 w + 31 of the
// tile and all 64 rows: acc[mt][nt], lane (j, kg) of which holds rows 16 mt + 4 kg + q (q = 0..3)
// against column 32 w + 16 nt + j.
#pragma once
#include "fff_device.h"

namespace fff {

constexpr int kTileM = 64;      // rows (tokens) per block
constexpr int kTileN = 128;     // columns per block
constexpr int kTileK = 64;      // K elements per chunk (8 pieces of 16 bytes per row)

struct TileLds {
    uint4 a[2][kTileM * 8];
    uint4 b[2][kTileN * 8];
};

// A: M rows of lda elements, B: N rows of ldb elements (row starts 16-byte aligned, K a multiple
// of 8); rows past M / N and K past the end count as zeros.  All 256 threads of the block call it.
// kDepth (2 or 4): chunks kept in flight in registers -- 4 for launches of few blocks, whose time is
// one block's chain of memory round trips; 2 where many blocks share a CU and registers are
// better spent on a third resident block.
template <int kDepth>
__device__ __forceinline__ void mfma_tile_64x128(const uint16_t* __restrict__ A, int64_t lda, int64_t M,
                                                 const uint16_t* __restrict__ B, int64_t ldb, int64_t N, int K,
                                                 int64_t m0, int64_t n0, TileLds& lds, f32x4_t (&acc)[4][2]) {
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int j = lane & 15, kg = lane >> 4;
    const int D = K;
    const int n_chunks = (K + kTileK - 1) / kTileK;
    uint4 (&lds_a)[2][kTileM * 8] = lds.a;
    uint4 (&lds_b)[2][kTileN * 8] = lds.b;
    // loader roles: 2 pieces of the token tile, 4 of the expert tile (8 consecutive threads = one
    // row's 128 bytes).  kDepth chunks are kept in flight in registers: with one chunk ahead the
    // loop is a chain of memory round trips (12 of them for D = 768), since a chunk's arithmetic
    // is only 16 MFMAs per wave.
    // Loads are unconditional with clamped addresses; rows past the end and K past D are zeroed
    // when the chunk goes to LDS.  (A predicated 16-byte load compiles to guarded dword loads with
    // a wait each, and a select right after the load makes the wave wait for it there.)
    static_assert(kDepth == 2 || kDepth == 4, "two or four chunks in flight");
    const int pc = tid & 7;                      // this thread's piece of every row it loads
    const int64_t ta0 = m0 + (tid >> 3), ta1 = ta0 + 32;
    const int64_t eb0 = n0 + (tid >> 3), eb1 = eb0 + 32, eb2 = eb0 + 64, eb3 = eb0 + 96;
    const uint16_t* const pa0 = A + (ta0 < M ? ta0 : M - 1) * lda + 8 * pc;
    const uint16_t* const pa1 = A + (ta1 < M ? ta1 : M - 1) * lda + 8 * pc;
    const uint16_t* const pb0 = B + (eb0 < N ? eb0 : N - 1) * ldb + 8 * pc;
    const uint16_t* const pb1 = B + (eb1 < N ? eb1 : N - 1) * ldb + 8 * pc;
    const uint16_t* const pb2 = B + (eb2 < N ? eb2 : N - 1) * ldb + 8 * pc;
    const uint16_t* const pb3 = B + (eb3 < N ? eb3 : N - 1) * ldb + 8 * pc;
    const bool va0 = ta0 < M, va1 = ta1 < M;
    const bool vb0 = eb0 < N, vb1 = eb1 < N, vb2 = eb2 < N, vb3 = eb3 < N;
    const int sa0 = tile_swz(tid >> 3, pc), sa1 = tile_swz((tid >> 3) + 32, pc);
    const int sb0 = sa0, sb1 = sa1, sb2 = tile_swz((tid >> 3) + 64, pc), sb3 = tile_swz((tid >> 3) + 96, pc);
    struct Chunk { uint4 a0, a1, b0, b1, b2, b3; };   // named members: they stay in registers
#define FFF_TILE_FETCH(KC, Q)                                                   \
    do {                                                                        \
        const int koff_ = (KC) * kTileK + 8 * pc < D ? (KC) * kTileK : 0;       \
        Q.a0 = *(const uint4*)(pa0 + koff_);                                    \
        Q.a1 = *(const uint4*)(pa1 + koff_);                                    \
        Q.b0 = *(const uint4*)(pb0 + koff_);                                    \
        Q.b1 = *(const uint4*)(pb1 + koff_);                                    \
        Q.b2 = *(const uint4*)(pb2 + koff_);                                    \
        Q.b3 = *(const uint4*)(pb3 + koff_);                                    \
    } while (0)
#define FFF_TILE_STASH(KC, BUF, Q)                                              \
    do {                                                                        \
        const bool kin_ = (KC) * kTileK + 8 * pc < D;                           \
        lds_a[BUF][sa0] = keep_if(kin_ && va0, Q.a0);                               \
        lds_a[BUF][sa1] = keep_if(kin_ && va1, Q.a1);                               \
        lds_b[BUF][sb0] = keep_if(kin_ && vb0, Q.b0);                               \
        lds_b[BUF][sb1] = keep_if(kin_ && vb1, Q.b1);                               \
        lds_b[BUF][sb2] = keep_if(kin_ && vb2, Q.b2);                               \
        lds_b[BUF][sb3] = keep_if(kin_ && vb3, Q.b3);                               \
    } while (0)

#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) acc[mt][nt] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    // The loop body has no branches (the wait counters are only tracked along straight code):
    // chunks past the end are fetched from a clamped address and stored as zeros, and the trip
    // count is rounded up to a multiple of kDepth; the extra MFMAs add zeros.
    Chunk c0, c1, c2, c3;
    FFF_TILE_FETCH(0, c0);
    FFF_TILE_FETCH(1, c1);
    if (kDepth == 4) {
        FFF_TILE_FETCH(2, c2);
        FFF_TILE_FETCH(3, c3);
    }
    FFF_TILE_STASH(0, 0, c0);
    __syncthreads();
    // one chunk: refill the register slot the chunk came from, multiply out of LDS buffer BUF,
    // put the next chunk into the other buffer.  Step u of a chunk gives lane group kg the piece
    // 2 kg + u of every row (K is only a summation order).
#define FFF_TILE_STEP(KC, BUF, CUR, NEXT)                                                                          \
    do {                                                                                                           \
        FFF_TILE_FETCH((KC) + kDepth, CUR);                                                                        \
        _Pragma("unroll") for (int u = 0; u < 2; ++u) {                                                            \
            bf16x8_t fa[4], fb[2];                                                                                 \
            _Pragma("unroll") for (int mt = 0; mt < 4; ++mt)                                                       \
                fa[mt] = __builtin_bit_cast(bf16x8_t, lds_a[BUF][tile_swz(16 * mt + j, 2 * kg + u)]);                   \
            _Pragma("unroll") for (int nt = 0; nt < 2; ++nt)                                                       \
                fb[nt] = __builtin_bit_cast(bf16x8_t, lds_b[BUF][tile_swz(32 * wv + 16 * nt + j, 2 * kg + u)]);         \
            _Pragma("unroll") for (int mt = 0; mt < 4; ++mt)                                                       \
                _Pragma("unroll") for (int nt = 0; nt < 2; ++nt)                                                   \
                    acc[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa[mt], fb[nt], acc[mt][nt], 0, 0, 0);   \
        }                                                                                                          \
        FFF_TILE_STASH((KC) + 1, (BUF) ^ 1, NEXT);                                                                 \
        __syncthreads();                                                                                           \
    } while (0)
    for (int kc0 = 0; kc0 < n_chunks; kc0 += kDepth) {
        if (kDepth == 2) {
            FFF_TILE_STEP(kc0 + 0, 0, c0, c1);
            FFF_TILE_STEP(kc0 + 1, 1, c1, c0);
            continue;
        }
        FFF_TILE_STEP(kc0 + 0, 0, c0, c1);
        FFF_TILE_STEP(kc0 + 1, 1, c1, c2);
        FFF_TILE_STEP(kc0 + 2, 0, c2, c3);
        FFF_TILE_STEP(kc0 + 3, 1, c3, c0);
    }
#undef FFF_TILE_STEP
#undef FFF_TILE_STASH
#undef FFF_TILE_FETCH

}

// Epilogue: the block's 64 x 128 results as bf16, staged through LDS (the first 16 KB of the tile
// buffers, free once mfma_tile_64x128 has returned) so that they leave as 16-byte pieces, 16
// consecutive threads on one row.  value(r, c, v) maps row r, column c of the tile and the
// accumulated v to the number stored; rows past M and columns past N are dropped.
template <typename Value>
__device__ __forceinline__ void tile_store_bf16(TileLds& lds, const f32x4_t (&acc)[4][2], uint16_t* __restrict__ C,
                                                int64_t ldc, int64_t M, int64_t N, int64_t m0, int64_t n0,
                                                Value value) {
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int j = lane & 15, kg = lane >> 4;
    uint16_t* st = (uint16_t*)lds.a;
#pragma unroll
    for (int nt = 0; nt < 2; ++nt)
#pragma unroll
        for (int mt = 0; mt < 4; ++mt)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int r = 16 * mt + 4 * kg + q, c = 32 * wv + 16 * nt + j;
                st[r * kTileN + c] = f32_to_bf16(value(r, c, acc[mt][nt][q]));
            }
    __syncthreads();
    const bool vec = (ldc & 7) == 0 && (reinterpret_cast<uintptr_t>(C) & 15u) == 0;
    for (int idx = tid; idx < kTileM * (kTileN / 8); idx += 256) {
        const int r = idx >> 4, pc = idx & 15;
        const int64_t t = m0 + r, n = n0 + 8 * pc;
        if (t >= M || n >= N) continue;
        if (vec && n + 8 <= N) {
            *(uint4*)(C + t * ldc + n) = *(const uint4*)(st + r * kTileN + 8 * pc);
        } else {
            for (int e = 0; e < 8 && n + e < N; ++e) C[t * ldc + n + e] = st[r * kTileN + 8 * pc + e];
        }
    }
}

// ---- the 128 x 256 tile of the large dense contractions (soft forward pass) -------------------
//
// Per clock a compute unit's LDS takes 128 bytes of stores and gives 256 bytes of 16-byte reads
// (conflict-free ones), its address unit moves 64 bytes of global loads, and its four matrix cores do
// 4096 bf16 flops: a chunk of K of a 64 x 128 tile costs the matrix cores 256 clocks, the LDS 384
// and the address unit 384 -- the small tile is bound by the traffic around the matrix cores.  For a
// block tile of M x N with four waves in a 2 x 2 arrangement every chunk is loaded and stored once
// ((M + N) K 2 bytes) and read once per wave ((M/2 + N/2) K 2 bytes, four waves) for 2 M N K flops:
// all three kinds of traffic per flop fall as M N / (M + N) grows.  128 x 256 (1024 matrix-core clocks
// per chunk against 768 of the LDS and 768 of the address unit) is the largest tile of which two
// blocks fit a compute unit with accumulators in ordinary registers.  So:
// 256 threads, wave (wm, wn) owns rows 64 wm .. + 63 and columns 128 wn .. + 127 as 4 x 8
// accumulators of v_mfma_f32_16x16x32_bf16 (128 registers).  The B rows go in as the instruction's
// first operand, so acc[mt][nt] of lane (j, kg) holds row 64 wm + 16 mt + j against the FOUR
// CONSECUTIVE columns 128 wn + 16 nt + 4 kg + q (q = 0..3): an epilogue handles 8 bytes of a bf16
// output row (or 16 of an fp32 one) per lane and tile, and whatever it looks up per column group
// (a bias, the leaf a neuron belongs to) once for four values; K walks in chunks of 64 through ONE
// LDS stage (16 KB of A rows, 32 KB of B rows, the same rotation swizzle), the next chunk
// travelling in registers meanwhile (12 pieces a thread); two blocks fit a compute unit, so one
// block's barriers and its wait for the chunk are covered by the other's arithmetic.
constexpr int kBigM = 128, kBigN = 256;

struct BigTileLds {
    uint4 a[kBigM * 8];      // 16 KB
    uint4 b[kBigN * 8];      // 32 KB
    uint4 pad[1024];         // the epilogue stages the tile's 128 x 256 bf16 results in all 64 KB
};

template <bool kInterior>
__device__ __forceinline__ void mfma_tile_128x256_body(const uint16_t* __restrict__ A, int64_t lda, int64_t M,
                                                  const uint16_t* __restrict__ B, int64_t ldb, int64_t N, int K,
                                                  int64_t m0, int64_t n0, BigTileLds& lds, f32x4_t (&acc)[4][8]) {
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int j = lane & 15, kg = lane >> 4;
    const int wm = wv >> 1, wn = wv & 1;
    const int n_chunks = (K + kTileK - 1) / kTileK;
    // loader roles: 8 consecutive threads fetch one row's 128 bytes of the chunk; a thread takes
    // piece pc of rows r0 + 32 i: 4 rows of the A tile, 8 of the B tile.  Loads are unconditional
    // with clamped addresses; rows past the end and K past the end are zeroed on the way to LDS.
    const int pc = tid & 7, r0 = tid >> 3;
    // addresses as a block-uniform base (tile origin + chunk) plus a 32-bit byte offset per row: half the
    // registers of twelve 64-bit pointers (a tile spans at most 256 rows, far below 4 GB)
    const char* const a_base = (const char*)(A + m0 * lda);
    const char* const b_base = (const char*)(B + n0 * ldb);
    uint32_t oa[4], ob[8];
    bool va[4], vb[8];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int64_t r = r0 + 32 * i;
        va[i] = m0 + r < M;
        oa[i] = (uint32_t)((va[i] ? r : M - 1 - m0) * lda * 2 + 16 * pc);
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int64_t r = r0 + 32 * i;
        vb[i] = n0 + r < N;
        ob[i] = (uint32_t)((vb[i] ? r : N - 1 - n0) * ldb * 2 + 16 * pc);
    }
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
        for (int nt = 0; nt < 8; ++nt) acc[mt][nt] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    uint4 qa[4], qb[8];
    // chunk kc of every row: the chunk's byte offset is uniform for interior tiles; at the ragged end of K a
    // thread whose piece lies past K re-reads chunk 0 (its value is zeroed on the way to LDS)
#define FFF_BIG_LOAD(BASE, OFF, KC) \
    (*(const uint4*)((BASE) + (kInterior ? (size_t)(KC) * (kTileK * 2) : (size_t)0) + \
                     ((OFF) + (kInterior ? 0u : ((KC) * kTileK + 8 * pc < K ? (uint32_t)(KC) * (kTileK * 2) : 0u)))))
#pragma unroll
    for (int i = 0; i < 4; ++i) qa[i] = FFF_BIG_LOAD(a_base, oa[i], 0);
#pragma unroll
    for (int i = 0; i < 8; ++i) qb[i] = FFF_BIG_LOAD(b_base, ob[i], 0);
    for (int kc = 0; kc < n_chunks; ++kc) {
        const bool kin = kInterior || kc * kTileK + 8 * pc < K;
        const int kn = kc + 1 < n_chunks ? kc + 1 : kc;
        __syncthreads();                                  // the previous chunk's operand reads are done
        // each piece goes to LDS and its register is refilled from the next chunk at once: the LDS
        // stores and the address unit's work on the loads overlap instead of queueing one behind the
        // other, and the loads travel while this chunk is multiplied
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            lds.a[tile_swz(r0 + 32 * i, pc)] = kInterior ? qa[i] : keep_if(kin && va[i], qa[i]);
            qa[i] = FFF_BIG_LOAD(a_base, oa[i], kn);
            __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            lds.b[tile_swz(r0 + 32 * i, pc)] = kInterior ? qb[i] : keep_if(kin && vb[i], qb[i]);
            qb[i] = FFF_BIG_LOAD(b_base, ob[i], kn);
            __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
        }
        __syncthreads();
        __builtin_amdgcn_sched_barrier(0);                // (left alone the scheduler sinks the loads to the next stash)
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            bf16x8_t fa[4], fb[8];
#pragma unroll
            for (int mt = 0; mt < 4; ++mt)
                fa[mt] = __builtin_bit_cast(bf16x8_t, lds.a[tile_swz(64 * wm + 16 * mt + j, 2 * kg + u)]);
#pragma unroll
            for (int nt = 0; nt < 8; ++nt)
                fb[nt] = __builtin_bit_cast(bf16x8_t, lds.b[tile_swz(128 * wn + 16 * nt + j, 2 * kg + u)]);
#pragma unroll
            for (int mt = 0; mt < 4; ++mt)
#pragma unroll
                for (int nt = 0; nt < 8; ++nt)
                    acc[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fb[nt], fa[mt], acc[mt][nt], 0, 0, 0);
        }
    }
    __syncthreads();
#undef FFF_BIG_LOAD
}

// Tiles with every row inside both matrices and K a whole number of chunks (all but the ragged
// edge) skip the zeroing selects on the way to LDS: a block-uniform choice.
__device__ __forceinline__ void mfma_tile_128x256(const uint16_t* __restrict__ A, int64_t lda, int64_t M,
                                                  const uint16_t* __restrict__ B, int64_t ldb, int64_t N, int K,
                                                  int64_t m0, int64_t n0, BigTileLds& lds, f32x4_t (&acc)[4][8]) {
    if (m0 + kBigM <= M && n0 + kBigN <= N && K % kTileK == 0)
        mfma_tile_128x256_body<true>(A, lda, M, B, ldb, N, K, m0, n0, lds, acc);
    else
        mfma_tile_128x256_body<false>(A, lda, M, B, ldb, N, K, m0, n0, lds, acc);
}

// Epilogue of the 128 x 256 tile: the accumulators (already finished by the caller: bias,
// activation, ...) leave as bf16 through all 64 KB of the tile's LDS so that the rows go out as
// 16-byte pieces (32 consecutive threads on one row); rows past M and columns past N are dropped.
// A lane's four values of a tile are 8 bytes of one row; piece p (16 bytes) of row r sits at piece
// p xor (r mod 32) of that row, which spreads the 16 rows that the lanes of a group write at once
// over the banks (the rows are 512 bytes apart).  The main loop ends with a barrier, so the staging may
// begin at once ...
// ... in two steps, so that an epilogue can finish, pack and stage one accumulator at a time (128
// finished values held until the end do not fit beside what the finishing needs):
// big_tile_stage puts the four values of acc[mt][nt] in place, big_tile_flush writes the tile out.
__device__ __forceinline__ void big_tile_stage(BigTileLds& lds, int mt, int nt, const f32x4_t& v) {
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int j = lane & 15, kg = lane >> 4;
    const int wm = wv >> 1, wn = wv & 1;
    uint2* st = (uint2*)&lds;                        // [128 rows][64 half pieces of 8 bytes]
    const int r = 64 * wm + 16 * mt + j;
    const int piece = (16 * wn + 2 * nt + (kg >> 1)) ^ (r & 31);
    st[r * 64 + 2 * piece + (kg & 1)] = make_uint2(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]));
}

__device__ __forceinline__ void big_tile_flush(BigTileLds& lds, uint16_t* __restrict__ C, int64_t ldc, int64_t M, int64_t N,
                                               int64_t m0, int64_t n0) {
    const int tid = threadIdx.x;
    __syncthreads();
    const uint4* sp = (const uint4*)&lds;            // [128 rows][32 pieces]
    const bool vec = (ldc & 7) == 0 && (reinterpret_cast<uintptr_t>(C) & 15u) == 0;
    for (int idx = tid; idx < kBigM * (kBigN / 8); idx += 256) {
        const int r = idx >> 5, pc = idx & 31;
        const int64_t t = m0 + r, n = n0 + 8 * pc;
        if (t >= M || n >= N) continue;
        const uint4 v = sp[r * 32 + (pc ^ (r & 31))];
        if (vec && n + 8 <= N) {
            store_stream((uint4*)(C + t * ldc + n), v);      // results are not read again by this launch: keep the L2 for operands
        } else {
            const uint32_t w[4] = {v.x, v.y, v.z, v.w};
            for (int e = 0; e < 8 && n + e < N; ++e) C[t * ldc + n + e] = (uint16_t)(w[e >> 1] >> (16 * (e & 1)));
        }
    }
}

__device__ __forceinline__ void big_tile_store_bf16(BigTileLds& lds, const f32x4_t (&acc)[4][8], uint16_t* __restrict__ C,
                                                    int64_t ldc, int64_t M, int64_t N, int64_t m0, int64_t n0) {
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
        for (int nt = 0; nt < 8; ++nt) big_tile_stage(lds, mt, nt, acc[mt][nt]);
    big_tile_flush(lds, C, ldc, M, N, m0, n0);
}

}  // namespace fff
