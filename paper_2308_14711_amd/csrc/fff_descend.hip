// K1 -- tree descent of Forward_I (Algorithm 1): per token, d node neurons
// (dot product + bias), each followed by "logit >= 0 -> child 2n+1 else 2n".
//
// A token is owned by a group of LPT consecutive lanes (16 = one DPP row, or
// the whole wave).  The token row is read once from HBM, 16 bytes per lane
// with consecutive lanes on consecutive addresses, and stays in registers for
// all d levels; each level streams one node row through the same lanes and
// reduces the partial dot products across the group with DPP row rotations.
#include "fff_device.h"
#include "fff_internal.h"

namespace fff {

// D % (16 bytes of elements) == 0 and all row starts 16-byte aligned.
bool vec_ok(const void* p, int64_t row_elems, bool bf16) {
    const int per = bf16 ? 8 : 4;
    return (reinterpret_cast<uintptr_t>(p) & 15u) == 0 && row_elems % per == 0;
}

template <bool BF16, int LPT, int NV>
__global__ __launch_bounds__(256) void descend_kernel(const uint4* __restrict__ x,
                                                      const uint4* __restrict__ node_w,
                                                      const void* __restrict__ node_b, int depth,
                                                      int64_t T, int nvec,
                                                      int32_t* __restrict__ leaf_idx) {
    constexpr int kGroups = 256 / LPT;
    const int sub = threadIdx.x % LPT;
    const int64_t t = (int64_t)blockIdx.x * kGroups + threadIdx.x / LPT;
    if (t >= T) return;   // a group is whole DPP rows (and the whole wave when LPT == 64)

    uint4 xv[NV];
    const uint4* xrow = x + t * nvec;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int v = sub + i * LPT;
        xv[i] = v < nvec ? load_stream(xrow + v) : make_uint4(0, 0, 0, 0);
    }

    int node = 0;
    for (int m = 0; m < depth; ++m) {
        const uint4* wrow = node_w + (int64_t)node * nvec;
        const float bias = Elem<BF16>::load(node_b, node);
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
        const float logit = group_sum<LPT>(acc0 + acc1) + bias;
        node = 2 * node + 1 + (logit >= 0.0f ? 1 : 0);
    }
    if (sub == 0) leaf_idx[t] = node - ((1 << depth) - 1);
}

// Any D, any alignment: one wave per token, element-wise loads.
template <bool BF16>
__global__ __launch_bounds__(256) void descend_generic_kernel(const void* __restrict__ x,
                                                              const void* __restrict__ node_w,
                                                              const void* __restrict__ node_b,
                                                              int depth, int64_t T, int64_t D,
                                                              int32_t* __restrict__ leaf_idx) {
    const int lane = threadIdx.x % kWave;
    const int64_t t = (int64_t)blockIdx.x * (256 / kWave) + threadIdx.x / kWave;
    if (t >= T) return;
    int node = 0;
    for (int m = 0; m < depth; ++m) {
        float acc = 0.f;
        for (int64_t j = lane; j < D; j += kWave)
            acc = fmaf(Elem<BF16>::load(x, t * D + j), Elem<BF16>::load(node_w, (int64_t)node * D + j), acc);
        const float logit = group_sum<64>(acc) + Elem<BF16>::load(node_b, node);
        node = 2 * node + 1 + (logit >= 0.0f ? 1 : 0);
    }
    if (lane == 0) leaf_idx[t] = node - ((1 << depth) - 1);
}

template <bool BF16, int LPT, int NV>
static hipError_t run_descend(const Problem& p, int32_t* leaf_idx, hipStream_t s) {
    constexpr int kGroups = 256 / LPT;
    const int nvec = (int)(p.D / Elem<BF16>::kPerVec);
    const int64_t blocks = (p.T + kGroups - 1) / kGroups;
    descend_kernel<BF16, LPT, NV><<<dim3((unsigned)blocks), dim3(256), 0, s>>>(
        (const uint4*)p.x, (const uint4*)p.node_w, p.node_b, p.depth, p.T, nvec, leaf_idx);
    return hipGetLastError();
}

template <bool BF16>
static hipError_t dispatch_descend(const Problem& p, int32_t* leaf_idx, hipStream_t s) {
    const int64_t nvec = p.D / Elem<BF16>::kPerVec;
    const bool fast = p.depth == 0 || (vec_ok(p.x, p.D, BF16) && vec_ok(p.node_w, p.D, BF16));
    if (fast && nvec <= 16) return run_descend<BF16, 16, 1>(p, leaf_idx, s);
    if (fast && nvec <= 32) return run_descend<BF16, 16, 2>(p, leaf_idx, s);
    if (fast && nvec <= 64) return run_descend<BF16, 16, 4>(p, leaf_idx, s);
    if (fast && nvec <= 96) return run_descend<BF16, 16, 6>(p, leaf_idx, s);
    if (fast && nvec <= 128) return run_descend<BF16, 16, 8>(p, leaf_idx, s);
    if (fast && nvec <= 256) return run_descend<BF16, 64, 4>(p, leaf_idx, s);
    if (fast && nvec <= 512) return run_descend<BF16, 64, 8>(p, leaf_idx, s);
    if (fast && nvec <= 1024) return run_descend<BF16, 64, 16>(p, leaf_idx, s);
    const int64_t blocks = (p.T + 3) / 4;
    descend_generic_kernel<BF16><<<dim3((unsigned)blocks), dim3(256), 0, s>>>(
        p.x, p.node_w, p.node_b, p.depth, p.T, p.D, leaf_idx);
    return hipGetLastError();
}

hipError_t launch_descend(const Problem& p, int32_t* leaf_idx, hipStream_t s) {
    if (p.T == 0) return hipSuccess;
    return p.bf16 ? dispatch_descend<true>(p, leaf_idx, s) : dispatch_descend<false>(p, leaf_idx, s);
}

}  // namespace fff
