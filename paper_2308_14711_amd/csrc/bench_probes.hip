// Measuring sticks for bench.py, built into a library of their own (libfff_bench_probes.so); no
// step of the method, and no part of the product ABI.
//
// fffb_gather: how fast can the chip's compute units pull rows at
// random out of a table -- the access pattern of a tree walk, where every token fetches one row
// per level.  16 lanes read one row of `pieces` 16-byte pieces (the fused walk kernel's layout),
// the next row index comes from a per-group linear congruential sequence and, with `dependent`,
// also from the data just read (a chain like the walk's: the table holds zeros, so the sequence
// is the same, but the hardware cannot run ahead).  Rates for tables inside one XCD's L2, beyond
// it, and beyond the last-level cache bracket what a walk over a tree of that size can reach.
//
// fffb_copy: a plain streaming copy, 16 bytes per lane, grid-stride, with the same streaming
// hints the walk kernels use on token and output rows: the ceiling a kernel that only moves rows
// can reach on this device.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(512) void copy_kernel(const u32x4_t* __restrict__ src, u32x4_t* __restrict__ dst,
                                                   int64_t n_vec) {
    const int64_t stride = (int64_t)gridDim.x * 512 * 4;
    for (int64_t i = (int64_t)blockIdx.x * 512 * 4 + threadIdx.x; i < n_vec; i += stride) {
        u32x4_t v[4];
#pragma unroll
        for (int k = 0; k < 4; ++k)
            if (i + k * 512 < n_vec) v[k] = __builtin_nontemporal_load(src + i + k * 512);
#pragma unroll
        for (int k = 0; k < 4; ++k)
            if (i + k * 512 < n_vec) __builtin_nontemporal_store(v[k], dst + i + k * 512);
    }
}

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

extern "C" {

// Launches `blocks` blocks of 512 threads; every 16 lanes read, `iters` times, `rows_in_flight` (1 or
// 4) rows of `row_bytes` bytes picked at random from `table` (device, table_rows rows, a power of
// two, 16-byte aligned, row_bytes a multiple of 16; fill it with zeros).  `dependent` non-zero makes
// each row index wait for the data of the previous one.  The caller times the launch; bytes moved =
// blocks * 32 * iters * rows_in_flight * row_bytes.  `sink`: 4 bytes of device memory (never written
// for a table of zeros).  Returns 0, or -1 for arguments out of range, or the hipError_t of the launch.
int fffb_gather(const void* table, int64_t table_rows, int64_t row_bytes, int rows_in_flight, int64_t blocks,
                int iters, int dependent, void* sink, void* stream) {
    if (!table || !sink || table_rows < 1 || (table_rows & (table_rows - 1)) != 0 || table_rows > ((int64_t)1 << 30) ||
        row_bytes < 16 || row_bytes % 16 != 0 || row_bytes > ((int64_t)1 << 20) || blocks < 1 ||
        blocks > ((int64_t)1 << 20) || iters < 1 || iters > (1 << 24) || (rows_in_flight != 1 && rows_in_flight != 4) ||
        (reinterpret_cast<uintptr_t>(table) & 15u) != 0)
        return -1;
    const uint32_t mask = (uint32_t)(table_rows - 1);
    const int pieces = (int)(row_bytes / 16);
    const dim3 g((unsigned)blocks), b(512);
    hipStream_t s = (hipStream_t)stream;
    if (rows_in_flight >= 4)
        gather_probe_kernel<4><<<g, b, 0, s>>>((const uint4*)table, mask, pieces, iters, dependent, (uint32_t*)sink);
    else
        gather_probe_kernel<1><<<g, b, 0, s>>>((const uint4*)table, mask, pieces, iters, dependent, (uint32_t*)sink);
    return (int)hipGetLastError();
}

// Copies `bytes` (a multiple of 16; both pointers 16-byte aligned, not overlapping) with `blocks`
// blocks of 512 threads.  Returns 0, -1 for bad arguments, or the hipError_t of the launch.
int fffb_copy(void* dst, const void* src, int64_t bytes, int64_t blocks, void* stream) {
    if (!dst || !src || bytes < 16 || bytes % 16 != 0 || blocks < 1 || blocks > ((int64_t)1 << 20) ||
        ((reinterpret_cast<uintptr_t>(dst) | reinterpret_cast<uintptr_t>(src)) & 15u) != 0)
        return -1;
    copy_kernel<<<dim3((unsigned)blocks), dim3(512), 0, (hipStream_t)stream>>>((const u32x4_t*)src, (u32x4_t*)dst,
                                                                             bytes / 16);
    return (int)hipGetLastError();
}

}  // extern "C"
