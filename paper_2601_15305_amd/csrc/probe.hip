// Measurement helper: whole-row gathers in the access shape of the sparse attention kernel, with no
// arithmetic behind them.  Timed by the benchmark on tables that fit the L2 of an XCD and on tables
// larger than every on-die cache, it gives the ceilings that the attention's gather rate is set against.
#include "common.hpp"

namespace gsa {

__global__ __launch_bounds__(256) void probe_gather_kernel(const u32x4* __restrict__ table, const int32_t* __restrict__ idx,
                                                           int64_t nchunks, int32_t waves, uint32_t* __restrict__ sink) {
    const int lane = threadIdx.x & 63;
    const int wave = blockIdx.x * 4 + (threadIdx.x >> 6);
    u32x4 acc = {0u, 0u, 0u, 0u};
    int64_t c = wave;
    int tok_next = c < nchunks ? idx[c * 64 + lane] : 0;
    for (; c < nchunks; c += waves) {
        const int tok = tok_next;
        if (c + waves < nchunks) tok_next = idx[(c + waves) * 64 + lane];  // one chunk ahead, like the kernel it mimics
        u32x4 v[16];
#pragma unroll
        for (int u = 0; u < 16; ++u) {  // four rows per instruction, 16 lanes x 16 bytes per row
            const int r = __shfl(tok, u * 4 + (lane >> 4), 64);
            v[u] = table[(int64_t)r * 16 + (lane & 15)];
        }
#pragma unroll
        for (int u = 0; u < 16; ++u) acc ^= v[u];
    }
    uint32_t x = acc[0] ^ acc[1] ^ acc[2] ^ acc[3];
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x ^= __shfl_xor(x, o, 64);
    if (lane == 0) sink[wave] = x;
}

// The same gather with every row passing through LDS on its way: rows -> registers -> a wave-private 16 KB tile ->
// registers (one 16-byte write and one 16-byte read per lane and row, as an MFMA operand staged through LDS
// needs at least).  Register-file return of the loads, LDS writes and LDS reads share the data path of a CU, so
// this rate, not the plain gather rate, is what a kernel that feeds gathered rows to the matrix cores can reach.
__global__ __launch_bounds__(256, 2) void probe_gather_staged_kernel(const u32x4* __restrict__ table, const int32_t* __restrict__ idx,
                                                                     int64_t nchunks, int32_t waves, uint32_t* __restrict__ sink) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int lane = threadIdx.x & 63;
    unsigned char* tile = smem + (threadIdx.x >> 6) * 16384;
    const int wave = blockIdx.x * 4 + (threadIdx.x >> 6);
    u32x4 acc = {0u, 0u, 0u, 0u};
    int64_t c = wave;
    int tok_next = c < nchunks ? idx[c * 64 + lane] : 0;
    for (; c < nchunks; c += waves) {
        const int tok = tok_next;
        if (c + waves < nchunks) tok_next = idx[(c + waves) * 64 + lane];
        u32x4 v[16];
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            const int r = __shfl(tok, u * 4 + (lane >> 4), 64);
            v[u] = table[(int64_t)r * 16 + (lane & 15)];
        }
#pragma unroll
        for (int u = 0; u < 16; ++u) *reinterpret_cast<u32x4*>(tile + u * 1024 + lane * 16) = v[u];
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
        for (int u = 0; u < 16; ++u) v[u] = *reinterpret_cast<const u32x4*>(tile + u * 1024 + ((lane * 16 + u * 16) & 1023));
#pragma unroll
        for (int u = 0; u < 16; ++u) acc ^= v[u];
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // reads done before the tile is overwritten
    }
    uint32_t x = acc[0] ^ acc[1] ^ acc[2] ^ acc[3];
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x ^= __shfl_xor(x, o, 64);
    if (lane == 0) sink[wave] = x;
}

hipError_t launch_probe_gather_staged(const void* table, const int32_t* idx, int64_t n_idx, int waves, uint32_t* sink, hipStream_t st) {
    static bool attr_set = false;  // (the attribute is per process; racing first calls set the same value)
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(probe_gather_staged_kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 65536);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL(probe_gather_staged_kernel, dim3((unsigned)(waves / 4)), dim3(256), 65536, st, static_cast<const u32x4*>(table),
                       idx, n_idx / 64, waves, sink);
    return hipGetLastError();
}

hipError_t launch_probe_gather(const void* table, const int32_t* idx, int64_t n_idx, int waves, uint32_t* sink, hipStream_t st) {
    hipLaunchKernelGGL(probe_gather_kernel, dim3((unsigned)(waves / 4)), dim3(256), 0, st, static_cast<const u32x4*>(table), idx,
                       n_idx / 64, waves, sink);
    return hipGetLastError();
}

}  // namespace gsa
