// Device-side helpers shared by the FFF kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fff {

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

constexpr int kWave = 64;

__device__ __forceinline__ float bf16_lo(uint32_t p) { return __uint_as_float(p << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t p) { return __uint_as_float(p & 0xffff0000u); }
__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

// Two fp32 -> packed bf16 pair, round to nearest even (v_cvt_pk_bf16_f32).
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    bf16x2_t v = {(__bf16)lo, (__bf16)hi};
    return __builtin_bit_cast(uint32_t, v);
}
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
    __bf16 b = (__bf16)f;
    return __builtin_bit_cast(uint16_t, b);
}

// acc + a.lo*b.lo + a.hi*b.hi on packed bf16 pairs, fp32 accumulate.
__device__ __forceinline__ float dot2_bf16(uint32_t a, uint32_t b, float acc) {
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a),
                                           __builtin_bit_cast(bf16x2_t, b), acc, false);
}

// 16 bytes of a row: 4 floats or 8 bf16.
template <bool BF16> struct Elem;
template <> struct Elem<false> {
    typedef float type;
    static constexpr int kPerVec = 4;
    static __device__ __forceinline__ float dot(const uint4& a, const uint4& b, float acc) {
        acc = fmaf(__uint_as_float(a.x), __uint_as_float(b.x), acc);
        acc = fmaf(__uint_as_float(a.y), __uint_as_float(b.y), acc);
        acc = fmaf(__uint_as_float(a.z), __uint_as_float(b.z), acc);
        acc = fmaf(__uint_as_float(a.w), __uint_as_float(b.w), acc);
        return acc;
    }
    static __device__ __forceinline__ float load(const void* p, int64_t i) { return ((const float*)p)[i]; }
    static __device__ __forceinline__ void store(void* p, int64_t i, float v) { ((float*)p)[i] = v; }
};
template <> struct Elem<true> {
    typedef uint16_t type;
    static constexpr int kPerVec = 8;
    static __device__ __forceinline__ float dot(const uint4& a, const uint4& b, float acc) {
        acc = dot2_bf16(a.x, b.x, acc);
        acc = dot2_bf16(a.y, b.y, acc);
        acc = dot2_bf16(a.z, b.z, acc);
        acc = dot2_bf16(a.w, b.w, acc);
        return acc;
    }
    static __device__ __forceinline__ float load(const void* p, int64_t i) { return bf16_to_f32(((const uint16_t*)p)[i]); }
    static __device__ __forceinline__ void store(void* p, int64_t i, float v) { ((uint16_t*)p)[i] = f32_to_bf16(v); }
};

// v from the lane `n` places further along this lane's 16-lane row (wrapping).
template <int N> __device__ __forceinline__ float row_rotate(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x120 + N, 0xf, 0xf, false));
}

// Sum over the LANES consecutive lanes this lane belongs to (LANES = 16 or 64);
// every lane of the group ends with the same bits: each step adds the same two
// partial sums in both lanes of a pair, and fp32 addition commutes.
template <int LANES> __device__ __forceinline__ float group_sum(float v) {
    v += row_rotate<8>(v);
    v += row_rotate<4>(v);
    v += row_rotate<2>(v);
    v += row_rotate<1>(v);
    if (LANES == 64) {
        v += __shfl_xor(v, 16, 64);
        v += __shfl_xor(v, 32, 64);
    }
    return v;
}

__device__ __forceinline__ float activate(float v, int act) {
    if (act == 0) return fmaxf(v, 0.0f);
    return 0.5f * v * (1.0f + erff(v * 0.70710678118654752440f));
}

// The same activation for epilogues that apply it to hundreds of millions of values (the dense
// contractions of the soft forward pass), where the library erf is what bounds the kernel:
// erfc(z) = t (a1 + t (a2 + t (a3 + t (a4 + t a5)))) exp(-z^2), t = 1 / (1 + p z) for z >= 0
// (Abramowitz & Stegun 7.1.26, absolute error <= 1.5e-7), 1 + erf(v / sqrt 2) = 2 - erfc(z) for v >= 0,
// erfc(z) for v < 0, z = |v| / sqrt 2.  The result differs from activate() by less than 5e-7 in absolute value (|v| <= 12, fp32 arithmetic),
// three orders below the bf16 rounding those epilogues end in.
__device__ __forceinline__ float activate_bulk(float v, int act) {
    if (act == 0) return fmaxf(v, 0.0f);
    const float z = fabsf(v) * 0.70710678118654752440f;
    const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, z, 1.0f));
    float p = fmaf(t, 1.061405429f, -1.453152027f);
    p = fmaf(p, t, 1.421413741f);
    p = fmaf(p, t, -0.284496736f);
    p = fmaf(p, t, 0.254829592f);
    const float erfc_z = p * t * __expf(-z * z);
    return 0.5f * v * (v >= 0.0f ? 2.0f - erfc_z : erfc_z);
}

// Streaming 16-byte load (tokens are read once; keep them out of the way of the weights).
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 load_stream(const uint4* p) {
    const u32x4_t v = __builtin_nontemporal_load((const u32x4_t*)p);
    return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void store_stream(uint4* p, const uint4& v) {
    const u32x4_t u = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(u, (u32x4_t*)p);
}

// v or zeros, component by component (a conditional on the 16-byte struct itself is lowered
// through memory)
__device__ __forceinline__ uint4 keep_if(bool ok, const uint4& v) {
    return make_uint4(ok ? v.x : 0u, ok ? v.y : 0u, ok ? v.z : 0u, ok ? v.w : 0u);
}

// Workgroups are dealt to the 8 XCDs round-robin (block b runs on XCD b mod 8) and every XCD
// has its own L2.  Work that is ordered by leaf wants consecutive items on one XCD, since they
// read the same weight rows: block b takes logical index (b mod 8) * (grid / 8) + b / 8, which
// gives each XCD one contiguous range of the work and lets a leaf's weights be fetched into one
// L2 instead of all eight.  The grid must be a multiple of 8; logical indices past the work are
// idle blocks.
constexpr int kXcds = 8;
__device__ __forceinline__ int64_t xcd_contiguous_block() {
    return (int64_t)(blockIdx.x % kXcds) * (gridDim.x / kXcds) + blockIdx.x / kXcds;
}

// Slot (16 bytes) of piece c of row r in an LDS tile of 128-byte rows that MFMA operands are read
// from: 8 r + ((c + rot(r)) mod 8), rot(r) = bit 1 of r + 4 * bit 2 of r.
//
// ds_read_b128 serves a wave in four passes of 16 lanes, and the passes are not runs of
// consecutive lanes: lanes {0-3, 12-15, 20-27}, {4-11, 16-19, 28-31}, and the same two sets + 32
// (measured with pairs of lanes aimed at one bank).  An operand read has lane (j, kg) on row j,
// piece 2 kg + u, so a pass holds every row j once: rows 0-3 and 12-15 with one kg, rows 4-11 with
// the neighbouring kg, two pieces apart.  The 16 slots of a pass must differ mod 16 (64 banks);
// rows of equal parity are told apart by rot(r), which takes {0, 1, 4, 5} on rows {0-3, 12-15} and
// the same values on rows {4-11}: adding the two-piece distance gives {2, 3, 6, 7} there.  With this
// rotation the operand reads run at the full 256 bytes a clock (the plain r / 2 rotation: half),
// and the 16-byte stores of whole rows (8 consecutive lanes per row) at the full store rate.
__device__ __forceinline__ int lds_rot(int row) { return ((row >> 1) & 1) + 4 * ((row >> 2) & 1); }
__device__ __forceinline__ int tile_swz(int row, int piece) { return 8 * row + ((piece + lds_rot(row)) & 7); }

}  // namespace fff
