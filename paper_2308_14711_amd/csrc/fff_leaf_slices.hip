// K3 (second half) + K4 by column slices -- the output rows of Forward_I (Algorithm 1) for narrow
// leaves whose output weights outgrow an L2:  y[t] = b2[leaf] + sum_r h[t][r] W2[leaf][r],  with the
// leaf and the hidden activations h (fp32) left by the walk launch.
//
// Taken per token, the rows W2[leaf][r] and b2[leaf] are gathered at random from a table that, for a
// few thousand leaves, is several times the 4 MB L2 of an XCD: most of them come back from memory, at
// the latency of a miss.  Here the work is cut the other way: a row of `out` is divided into slices
// of whole 128-byte lines, and an XCD writes ONE slice of ALL rows (two XCDs share a slice when there
// are fewer slices than XCDs, each taking every other tile of tokens).  Its L2 then only ever sees
// that slice of the table -- an eighth or a quarter of it -- and keeps it.  Workgroups are dealt to
// the XCDs round-robin, so block b works for XCD b mod 8.
//
// A thread owns one 16-byte piece of one token's slice; consecutive threads take consecutive pieces,
// then the next token.  Same additions in the same order as the fused launch (bias first, then the
// neurons in index order, fp32, one rounding at the end): the two produce the same bits.
#include "fff_device.h"
#include "fff_internal.h"

namespace fff {
namespace {

constexpr int kSliceBlock = 256;
constexpr int kSliceMaxLeafWidth = 8;

struct SliceArgs {
    const int32_t* leaf_idx;
    const float* hidden;     // [T, L]
    const uint4* w2;         // [leaves, L, ovec] pieces
    const uint4* b2;         // [leaves, ovec]
    uint4* out;              // [T, ovec]
    int64_t T;
    int ovec;                // 16-byte pieces per row
    int vps;                 // pieces per slice
    int slices;              // slices per row (a power of two, at most 8)
    int L;
};

template <bool BF16> __device__ __forceinline__ void unpack(const uint4& v, float* f);
template <> __device__ __forceinline__ void unpack<false>(const uint4& v, float* f) {
    f[0] = __uint_as_float(v.x); f[1] = __uint_as_float(v.y); f[2] = __uint_as_float(v.z); f[3] = __uint_as_float(v.w);
}
template <> __device__ __forceinline__ void unpack<true>(const uint4& v, float* f) {
    f[0] = bf16_lo(v.x); f[1] = bf16_hi(v.x); f[2] = bf16_lo(v.y); f[3] = bf16_hi(v.y);
    f[4] = bf16_lo(v.z); f[5] = bf16_hi(v.z); f[6] = bf16_lo(v.w); f[7] = bf16_hi(v.w);
}
template <bool BF16> __device__ __forceinline__ uint4 pack(const float* f);
template <> __device__ __forceinline__ uint4 pack<false>(const float* f) {
    return make_uint4(__float_as_uint(f[0]), __float_as_uint(f[1]), __float_as_uint(f[2]), __float_as_uint(f[3]));
}
template <> __device__ __forceinline__ uint4 pack<true>(const float* f) {
    return make_uint4(pack_bf16x2(f[0], f[1]), pack_bf16x2(f[2], f[3]), pack_bf16x2(f[4], f[5]), pack_bf16x2(f[6], f[7]));
}

}  // namespace

// kItems pieces a thread at a time (kItems tiles of a block's worth apart), all of a step's loads
// issued before any is used: the leaf index first, then the bias and weight pieces it points at.
// (Measured with 1 and 4 on 768-wide rows, one neuron a leaf: 24.6 us either way -- the launch is
// bound by its 100 MB of output rows -- and 4 costs wide leaves their registers; 1 it is.)
constexpr int kItems = 1;

template <bool BF16, int LW>    // LW: leaf widths up to this many neurons (1, 2 or 8)
__global__ __launch_bounds__(kSliceBlock) void leaf_slices_kernel(const SliceArgs a) {
    constexpr int VE = Elem<BF16>::kPerVec;
    const int xcd = blockIdx.x % kXcds;
    const int slice = xcd % a.slices;
    const int share = kXcds / a.slices;            // XCDs that share a slice
    const int part = xcd / a.slices;               // which of them this one is
    const int64_t blocks_per_xcd = gridDim.x / kXcds;
    // the slice's work: T * vps pieces, dealt to the sharing XCDs in tiles of a block's worth
    const int64_t n_items = a.T * a.vps;
    const int64_t n_tiles = (n_items + kSliceBlock - 1) / kSliceBlock;
    const int64_t step = blocks_per_xcd * share;
    for (int64_t tile0 = (int64_t)(blockIdx.x / kXcds) * share + part; tile0 < n_tiles; tile0 += kItems * step) {
        int64_t t[kItems], leaf[kItems];
        int v[kItems];
        bool live[kItems];
#pragma unroll
        for (int q = 0; q < kItems; ++q) {
            const int64_t i = (tile0 + q * step) * kSliceBlock + threadIdx.x;
            const int64_t tt = i / a.vps;
            v[q] = slice * a.vps + (int)(i - tt * a.vps);
            live[q] = tile0 + q * step < n_tiles && i < n_items && v[q] < a.ovec;
            t[q] = live[q] ? tt : 0;
            if (!live[q]) v[q] = 0;
            leaf[q] = a.leaf_idx[t[q]];
        }
        float h[kItems][LW];
        uint4 bv[kItems], wv[kItems][LW];
#pragma unroll
        for (int q = 0; q < kItems; ++q) {
#pragma unroll
            for (int r = 0; r < LW; ++r) h[q][r] = r < a.L ? a.hidden[t[q] * a.L + r] : 0.f;
            bv[q] = a.b2[leaf[q] * a.ovec + v[q]];
#pragma unroll
            for (int r = 0; r < LW; ++r) wv[q][r] = a.w2[(leaf[q] * a.L + (r < a.L ? r : 0)) * a.ovec + v[q]];
        }
#pragma unroll
        for (int q = 0; q < kItems; ++q) {
            float acc[VE];
            unpack<BF16>(bv[q], acc);
#pragma unroll
            for (int r = 0; r < LW; ++r) {
                if (r < a.L) {
                    float wf[VE];
                    unpack<BF16>(wv[q][r], wf);
#pragma unroll
                    for (int e = 0; e < VE; ++e) acc[e] = fmaf(h[q][r], wf[e], acc[e]);
                }
            }
            // streaming stores: the rows are not read again (23.2 us against 25.4 with plain ones)
            if (live[q]) store_stream(a.out + t[q] * a.ovec + v[q], pack<BF16>(acc));
        }
    }
}

// whole 16-byte pieces in rows that start on 16-byte boundaries, leaves of at most 8 neurons
bool slices_shape_ok(const Problem& p) {
    return p.L <= kSliceMaxLeafWidth && vec_ok(p.out, p.O, p.bf16) && vec_ok(p.leaf_w2, p.O, p.bf16) &&
           vec_ok(p.leaf_b2, p.O, p.bf16);
}

hipError_t launch_leaf_slices(const Problem& p, const int32_t* leaf_idx, const float* hidden, hipStream_t s) {
    if (p.T == 0) return hipSuccess;
    SliceArgs a;
    a.leaf_idx = leaf_idx;
    a.hidden = hidden;
    a.w2 = (const uint4*)p.leaf_w2;
    a.b2 = (const uint4*)p.leaf_b2;
    a.out = (uint4*)p.out;
    a.T = p.T;
    a.ovec = (int)(p.O / (p.bf16 ? 8 : 4));
    a.L = p.L;
    // slices of whole 128-byte lines (8 pieces), as many as there are XCDs if the row has that many lines
    // (a row of 12 lines: 4 slices of 3 lines, two XCDs a slice; the last slice of a row whose lines
    // do not divide evenly is shorter)
    const int lines = (a.ovec + 7) / 8;
    int slices = kXcds;
    while (slices > 1 && (lines % slices != 0 && lines < 4 * slices)) slices /= 2;
    const int lines_per_slice = (lines + slices - 1) / slices;
    a.slices = slices;
    a.vps = lines_per_slice * 8;
    const int64_t n_tiles = (p.T * a.vps + kSliceBlock - 1) / kSliceBlock;
    const int share = kXcds / slices;
    int64_t per_xcd = (n_tiles + share - 1) / share;
    const int64_t cap = (int64_t)device_info().cus * 16 / kXcds;    // a few waves of blocks per compute unit, then stride
    if (per_xcd > cap) per_xcd = cap;
    if (per_xcd < 1) per_xcd = 1;
    note_launch("leaf_slices_kernel<%s,%d> slices=%d", p.bf16 ? "bf16" : "f32", p.L <= 2 ? p.L : kSliceMaxLeafWidth, slices);
    const dim3 grid((unsigned)(per_xcd * kXcds)), block(kSliceBlock);
    if (p.L == 1) {
        if (p.bf16) leaf_slices_kernel<true, 1><<<grid, block, 0, s>>>(a);
        else leaf_slices_kernel<false, 1><<<grid, block, 0, s>>>(a);
    } else if (p.L == 2) {
        if (p.bf16) leaf_slices_kernel<true, 2><<<grid, block, 0, s>>>(a);
        else leaf_slices_kernel<false, 2><<<grid, block, 0, s>>>(a);
    } else {
        if (p.bf16) leaf_slices_kernel<true, kSliceMaxLeafWidth><<<grid, block, 0, s>>>(a);
        else leaf_slices_kernel<false, kSliceMaxLeafWidth><<<grid, block, 0, s>>>(a);
    }
    return hipGetLastError();
}

}  // namespace fff
