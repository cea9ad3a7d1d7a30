// A measuring stick, not a step of the method: how fast can the chip's compute units pull rows at
// random out of a table -- the access pattern of a tree walk, where every token fetches one row
// per level.  16 lanes read one row of `pieces` 16-byte pieces (the fused walk kernel's layout),
// the next row index comes from a per-group linear congruential sequence and, with `dependent`,
// also from the data just read (a chain like the walk's: the table holds zeros, so the sequence
// is the same, but the hardware cannot run ahead).  Rates for tables inside one XCD's L2, beyond
// it, and beyond the last-level cache bracket what a walk over a tree of that size can reach.
#include "fff_device.h"
#include "fff_internal.h"

namespace fff {
namespace {

template <int ROWS>
__global__ __launch_bounds__(512) void gather_probe_kernel(const uint4* __restrict__ table, uint32_t row_mask,
                                                           int pieces, int iters, int dependent,
                                                           uint32_t* __restrict__ sink) {
    const int sub = threadIdx.x & 15;
    uint32_t h = (((uint32_t)blockIdx.x * 512u + threadIdx.x) >> 4) * 2654435761u + 12345u;
    uint32_t acc = 0;
    for (int it = 0; it < iters; ++it) {
        uint32_t s = 0;
#pragma unroll
        for (int k = 0; k < ROWS; ++k) {
            h = h * 1664525u + 1013904223u;
            const uint4* row = table + (size_t)((h >> 8) & row_mask) * pieces;
            for (int v = sub; v < pieces; v += 16) {
                const uint4 p = row[v];
                s += p.x ^ p.y ^ p.z ^ p.w;
            }
        }
        acc += s;
        if (dependent) {
            uint32_t t = s;
            t ^= __shfl_xor(t, 1, 64);
            t ^= __shfl_xor(t, 2, 64);
            t ^= __shfl_xor(t, 4, 64);
            t ^= __shfl_xor(t, 8, 64);
            h += t;
        }
    }
    if (acc == 0x9e3779b9u) sink[0] = acc;   // keeps the loads alive; false for a table of zeros
}

}  // namespace

hipError_t launch_gather_probe(const void* table, int64_t table_rows, int pieces, int rows_in_flight,
                               int64_t blocks, int iters, bool dependent, uint32_t* sink, hipStream_t s) {
    const uint32_t mask = (uint32_t)(table_rows - 1);
    const dim3 g((unsigned)blocks), b(512);
    if (rows_in_flight >= 4)
        gather_probe_kernel<4><<<g, b, 0, s>>>((const uint4*)table, mask, pieces, iters, dependent, sink);
    else
        gather_probe_kernel<1><<<g, b, 0, s>>>((const uint4*)table, mask, pieces, iters, dependent, sink);
    return hipGetLastError();
}

}  // namespace fff
