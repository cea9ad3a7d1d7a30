// K3 + K4 -- the leaf network of the leaf a token arrived at (Definition: a
// <D, l, O> feedforward block; Algorithm 1 returns its output), written
// straight to the token's own output row.
//
// Gather path (this file): a group of LPT lanes owns one token.  The token row
// sits in registers, the l hidden neurons are l dot products reduced across
// the group, and the O outputs are produced 16 bytes per lane from the leaf's
// output-weight rows.  Slots are visited in bucket order when an order array
// is given, so neighbouring groups read the same leaf's weights.
#include "fff_device.h"
#include "fff_internal.h"

namespace fff {

constexpr int kMaxLeafWidthGather = 64;

template <bool BF16, int LPT, int NV>
__global__ __launch_bounds__(256) void leaf_gather_kernel(
    const uint4* __restrict__ x, const uint4* __restrict__ w1, const void* __restrict__ b1,
    const void* __restrict__ w2, const void* __restrict__ b2, const int32_t* __restrict__ leaf_idx,
    const int32_t* __restrict__ order, int L, int act, int64_t T, int nvec, int64_t O, int out_vec,
    void* __restrict__ out, const int32_t* __restrict__ slot_leaf, int split) {
    constexpr int kGroups = 256 / LPT;
    constexpr int VE = Elem<BF16>::kPerVec;
    static_assert(16 % kGroups == 0, "the slots of a block lie in one tile of 16");
    __shared__ float hs[kGroups][kMaxLeafWidthGather];
    const int sub = threadIdx.x % LPT;
    const int g = threadIdx.x / LPT;
    // in bucket order consecutive slots share a leaf: keep them on one XCD
    const int64_t first_slot = (order ? xcd_contiguous_block() : (int64_t)blockIdx.x) * kGroups;
    if (split > 0) {
        // Shared with the tile kernels: only tiles (16 consecutive slots) with at least `split`
        // runs of equal leaf are this kernel's; the whole block leaves otherwise.  Every wave
        // counts the runs of the block's tile for itself.
        const int lane = threadIdx.x & 63;
        const int64_t ts = first_slot / 16 * 16 + (lane & 15);
        const int32_t lf = ts < T ? slot_leaf[ts] : -1;
        const int32_t prev = __shfl_up(lf, 1, 16);
        const uint32_t changes = (uint32_t)__ballot(lane > 0 && lane < 16 && lf >= 0 && lf != prev);
        if (__popc(changes) + 1 < split) return;
    }
    const int64_t slot = first_slot + g;
    const bool live = slot < T;
    const int64_t t = live ? (order ? (int64_t)order[slot] : slot) : 0;
    const int64_t leaf = leaf_idx[t];

    uint4 xv[NV];
    const uint4* xrow = x + t * nvec;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int v = sub + i * LPT;
        xv[i] = v < nvec ? load_stream(xrow + v) : make_uint4(0, 0, 0, 0);
    }

    // hidden neurons: h[r] = act(W1[leaf][r] . x + b1[leaf][r])
    const uint4* wl = w1 + leaf * L * nvec;
    for (int r = 0; r < L; ++r) {
        const uint4* wrow = wl + (int64_t)r * nvec;
        float acc0 = 0.f, acc1 = 0.f;
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const int v = sub + i * LPT;
            if (v < nvec) {
                const uint4 wv = wrow[v];
                if (i & 1) acc1 = Elem<BF16>::dot(xv[i], wv, acc1);
                else acc0 = Elem<BF16>::dot(xv[i], wv, acc0);
            }
        }
        const float pre = group_sum<LPT>(acc0 + acc1) + Elem<BF16>::load(b1, leaf * L + r);
        if (sub == 0) hs[g][r] = activate(pre, act);
    }
    __syncthreads();
    if (!live) return;

    // outputs: y[o] = sum_r h[r] W2[leaf][r][o] + b2[leaf][o]
    if (out_vec) {
        const int ovec = (int)(O / VE);
        const uint4* w2v = (const uint4*)w2 + leaf * L * ovec;
        const uint4* b2v = (const uint4*)b2 + leaf * ovec;
        uint4* orow = (uint4*)out + t * ovec;
        for (int ov = sub; ov < ovec; ov += LPT) {
            float acc[VE];
            const uint4 bv = b2v[ov];
            if (BF16) {
                acc[0] = bf16_lo(bv.x); acc[1] = bf16_hi(bv.x); acc[2] = bf16_lo(bv.y); acc[3] = bf16_hi(bv.y);
                acc[4 % VE] = bf16_lo(bv.z); acc[5 % VE] = bf16_hi(bv.z); acc[6 % VE] = bf16_lo(bv.w); acc[7 % VE] = bf16_hi(bv.w);
            } else {
                acc[0] = __uint_as_float(bv.x); acc[1] = __uint_as_float(bv.y);
                acc[2] = __uint_as_float(bv.z); acc[3] = __uint_as_float(bv.w);
            }
#pragma unroll 4
            for (int r = 0; r < L; ++r) {
                const float h = hs[g][r];
                const uint4 wv = w2v[(int64_t)r * ovec + ov];
                if (BF16) {
                    acc[0] = fmaf(h, bf16_lo(wv.x), acc[0]); acc[1] = fmaf(h, bf16_hi(wv.x), acc[1]);
                    acc[2] = fmaf(h, bf16_lo(wv.y), acc[2]); acc[3] = fmaf(h, bf16_hi(wv.y), acc[3]);
                    acc[4 % VE] = fmaf(h, bf16_lo(wv.z), acc[4 % VE]); acc[5 % VE] = fmaf(h, bf16_hi(wv.z), acc[5 % VE]);
                    acc[6 % VE] = fmaf(h, bf16_lo(wv.w), acc[6 % VE]); acc[7 % VE] = fmaf(h, bf16_hi(wv.w), acc[7 % VE]);
                } else {
                    acc[0] = fmaf(h, __uint_as_float(wv.x), acc[0]); acc[1] = fmaf(h, __uint_as_float(wv.y), acc[1]);
                    acc[2] = fmaf(h, __uint_as_float(wv.z), acc[2]); acc[3] = fmaf(h, __uint_as_float(wv.w), acc[3]);
                }
            }
            uint4 ov4;
            if (BF16) {
                ov4.x = pack_bf16x2(acc[0], acc[1]); ov4.y = pack_bf16x2(acc[2], acc[3]);
                ov4.z = pack_bf16x2(acc[4 % VE], acc[5 % VE]); ov4.w = pack_bf16x2(acc[6 % VE], acc[7 % VE]);
            } else {
                ov4.x = __float_as_uint(acc[0]); ov4.y = __float_as_uint(acc[1]);
                ov4.z = __float_as_uint(acc[2]); ov4.w = __float_as_uint(acc[3]);
            }
            store_stream(orow + ov, ov4);
        }
    } else {
        for (int64_t o = sub; o < O; o += LPT) {
            float acc = Elem<BF16>::load(b2, leaf * O + o);
            for (int r = 0; r < L; ++r)
                acc = fmaf(hs[g][r], Elem<BF16>::load(w2, (leaf * L + r) * O + o), acc);
            Elem<BF16>::store(out, t * O + o, acc);
        }
    }
}

// Whole forward pass, any shape, any alignment: one wave per token, element
// loads.  The fallback for shapes the vector kernels do not take, and the
// single launch used for small batches.
template <bool BF16>
__global__ __launch_bounds__(256) void fused_generic_kernel(
    const void* __restrict__ x, const void* __restrict__ node_w, const void* __restrict__ node_b,
    const void* __restrict__ w1, const void* __restrict__ b1, const void* __restrict__ w2,
    const void* __restrict__ b2, const int32_t* __restrict__ leaf_in, const int32_t* __restrict__ order,
    int depth, int L, int act, int64_t T, int64_t D, int64_t O, void* __restrict__ out,
    int32_t* __restrict__ leaf_out) {
    extern __shared__ float hbuf[];   // [4][L]
    const int lane = threadIdx.x % kWave;
    const int wv = threadIdx.x / kWave;
    const int64_t slot = (int64_t)blockIdx.x * 4 + wv;
    if (slot >= T) return;            // no block-wide barrier below
    const int64_t t = order ? (int64_t)order[slot] : slot;
    int64_t leaf;
    if (leaf_in) {
        leaf = leaf_in[t];
    } else {
        int node = 0;
        for (int m = 0; m < depth; ++m) {
            float acc = 0.f;
            for (int64_t j = lane; j < D; j += kWave)
                acc = fmaf(Elem<BF16>::load(x, t * D + j), Elem<BF16>::load(node_w, (int64_t)node * D + j), acc);
            const float logit = group_sum<64>(acc) + Elem<BF16>::load(node_b, node);
            node = 2 * node + 1 + (logit >= 0.0f ? 1 : 0);
        }
        leaf = node - ((1 << depth) - 1);
        if (leaf_out && lane == 0) leaf_out[t] = (int32_t)leaf;
    }
    if (!out) return;
    float* h = hbuf + (int64_t)wv * L;
    for (int r = 0; r < L; ++r) {
        float acc = 0.f;
        for (int64_t j = lane; j < D; j += kWave)
            acc = fmaf(Elem<BF16>::load(x, t * D + j), Elem<BF16>::load(w1, (leaf * L + r) * D + j), acc);
        const float pre = group_sum<64>(acc) + Elem<BF16>::load(b1, leaf * L + r);
        if (lane == 0) h[r] = activate(pre, act);
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    for (int64_t o = lane; o < O; o += kWave) {
        float acc = Elem<BF16>::load(b2, leaf * O + o);
        for (int r = 0; r < L; ++r) acc = fmaf(h[r], Elem<BF16>::load(w2, (leaf * L + r) * O + o), acc);
        Elem<BF16>::store(out, t * O + o, acc);
    }
}

template <bool BF16, int LPT, int NV>
static hipError_t run_gather(const Problem& p, const int32_t* leaf_idx, const int32_t* order, hipStream_t s,
                             const int32_t* slot_leaf, int split) {
    constexpr int kGroups = 256 / LPT;
    const int nvec = (int)(p.D / Elem<BF16>::kPerVec);
    const int out_vec = vec_ok(p.out, p.O, BF16) && vec_ok(p.leaf_w2, p.O, BF16) && vec_ok(p.leaf_b2, p.O, BF16);
    const int64_t blocks = ((p.T + kGroups - 1) / kGroups + kXcds - 1) / kXcds * kXcds;
    note_launch("leaf_gather_kernel<%s,%d,%d>%s", BF16 ? "bf16" : "f32", LPT, NV, split > 0 ? " split" : "");
    leaf_gather_kernel<BF16, LPT, NV><<<dim3((unsigned)blocks), dim3(256), 0, s>>>(
        (const uint4*)p.x, (const uint4*)p.leaf_w1, p.leaf_b1, p.leaf_w2, p.leaf_b2, leaf_idx, order,
        p.L, p.act, p.T, nvec, p.O, out_vec, p.out, slot_leaf, split);
    return hipGetLastError();
}

template <bool BF16>
static hipError_t run_generic(const Problem& p, const int32_t* leaf_in, const int32_t* order,
                              int32_t* leaf_out, hipStream_t s) {
    const int64_t blocks = (p.T + 3) / 4;
    const size_t lds = sizeof(float) * 4 * (size_t)p.L;
    note_launch("fused_generic_kernel<%s>", BF16 ? "bf16" : "f32");
    fused_generic_kernel<BF16><<<dim3((unsigned)blocks), dim3(256), lds, s>>>(
        p.x, p.node_w, p.node_b, p.leaf_w1, p.leaf_b1, p.leaf_w2, p.leaf_b2, leaf_in, order, p.depth,
        p.L, p.act, p.T, p.D, p.O, p.out, leaf_out);
    return hipGetLastError();
}

template <bool BF16>
static hipError_t dispatch_gather(const Problem& p, const int32_t* leaf_idx, const int32_t* order, hipStream_t s,
                                  const int32_t* slot_leaf, int split) {
    const int64_t nvec = p.D / Elem<BF16>::kPerVec;
    const bool fast = vec_ok(p.x, p.D, BF16) && vec_ok(p.leaf_w1, p.D, BF16) && p.L <= kMaxLeafWidthGather;
    if (fast && nvec <= 16) return run_gather<BF16, 16, 1>(p, leaf_idx, order, s, slot_leaf, split);
    if (fast && nvec <= 32) return run_gather<BF16, 16, 2>(p, leaf_idx, order, s, slot_leaf, split);
    if (fast && nvec <= 64) return run_gather<BF16, 16, 4>(p, leaf_idx, order, s, slot_leaf, split);
    if (fast && nvec <= 96) return run_gather<BF16, 16, 6>(p, leaf_idx, order, s, slot_leaf, split);
    if (fast && nvec <= 128) return run_gather<BF16, 16, 8>(p, leaf_idx, order, s, slot_leaf, split);
    if (fast && nvec <= 256) return run_gather<BF16, 64, 4>(p, leaf_idx, order, s, slot_leaf, split);
    if (fast && nvec <= 512) return run_gather<BF16, 64, 8>(p, leaf_idx, order, s, slot_leaf, split);
    if (fast && nvec <= 1024) return run_gather<BF16, 64, 16>(p, leaf_idx, order, s, slot_leaf, split);
    if (split > 0) return hipErrorInvalidValue;   // callers ask gather_takes_split() first
    return run_generic<BF16>(p, leaf_idx, order, nullptr, s);
}

// the shapes whose gather launch can leave tiles to the tile kernels (the lane-group kernels)
bool gather_takes_split(const Problem& p) {
    const int per = p.bf16 ? 8 : 4;
    return vec_ok(p.x, p.D, p.bf16) && vec_ok(p.leaf_w1, p.D, p.bf16) && p.L <= kMaxLeafWidthGather &&
           p.D / per <= 1024;
}

hipError_t launch_leaf_gather(const Problem& p, const int32_t* leaf_idx, const int32_t* order, hipStream_t s,
                              const int32_t* slot_leaf, int split) {
    if (p.T == 0) return hipSuccess;
    if (split > 0 && (!order || !slot_leaf)) return hipErrorInvalidValue;
    return p.bf16 ? dispatch_gather<true>(p, leaf_idx, order, s, slot_leaf, split)
                  : dispatch_gather<false>(p, leaf_idx, order, s, slot_leaf, split);
}

hipError_t launch_fused_generic(const Problem& p, int32_t* leaf_idx, hipStream_t s) {
    if (p.T == 0) return hipSuccess;
    return p.bf16 ? run_generic<true>(p, nullptr, nullptr, leaf_idx, s)
                  : run_generic<false>(p, nullptr, nullptr, leaf_idx, s);
}

}  // namespace fff
