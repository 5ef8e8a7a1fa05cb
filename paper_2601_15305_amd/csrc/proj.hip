// Linear projections around the attention path: Q, K, V (Sec. 2.1 Eq. 1), the indexer's q^I, k^I and head
// weights sigma(h W^Iw) (Sec. 3.3), the gate logits h W^g_V and h W^g_O (Sec. 3.5), and the output projection
// W_O (App. B).  All of them are y = x W^T with W stored [out_features, in_features]; the input projections of
// one layer share x = h, so they run as ONE GEMM whose output features are the concatenation of up to eight
// segments, each with its own weight matrix, destination and epilogue (store as bf16, or sigmoid -> fp32 for
// the indexer head weights).  bf16 inputs, fp32 accumulation on v_mfma_f32_32x32x16_bf16.
//
// The product is computed transposed, C^T[feature, token] = W[feature, :] . x[token, :], so that in the 32x32
// accumulator layout a lane owns one token (column) and groups of four consecutive features (rows): token-major
// outputs are written with 8-byte stores.  A workgroup computes 256 features x 256 tokens with eight waves
// (128 x 128 with four on small calls).  Small shape: k advances in steps of 64 through double-buffered LDS tiles
// (144-byte padded rows, conflict-free 16-byte fragment reads), one barrier per step, the next step's global loads
// in flight (in registers) during the products.  Large shape: the tiles go straight from global memory into four
// LDS buffers, steps of 32, three steps in flight (see DIRECT below).
#include "common.hpp"

namespace gsa {

constexpr int kProjMaxSeg = 8;

#ifndef GSA_PROJ_DIRECT
#define GSA_PROJ_DIRECT 1
#endif

struct ProjArgs {
    const __bf16* x;                      // [tokens, K]
    const __bf16* w[kProjMaxSeg];         // segment s: [seg_begin[s+1] - seg_begin[s], K]
    void* out[kProjMaxSeg];               // segment s: [tokens, width_s]  (bf16, or fp32 for kind 1)
    int32_t seg_begin[kProjMaxSeg + 1];   // first feature of every segment; seg_begin[nseg] = N
    int32_t kind[kProjMaxSeg];            // 0 = store in bf16, 1 = sigmoid, stored in fp32
    int32_t nseg, tokens, N, K;
};

__device__ __forceinline__ int proj_segment_of(const ProjArgs& a, int f) {
    int s = 0;
#pragma unroll
    for (int i = 1; i < kProjMaxSeg; ++i) s += (i < a.nseg && f >= a.seg_begin[i]) ? 1 : 0;
    return s;
}

// WM x WN waves; a wave computes FI x FJ accumulators of 32 features x 32 tokens.  Two shapes are built:
//   2 x 2 waves of 2 x 2 accumulators: 128 features x 128 tokens, two workgroups per compute unit (small calls);
//   2 x 4 waves of 4 x 2 accumulators: 256 x 256, one workgroup of eight waves per compute unit -- per flop half
//   the LDS traffic and half the L2 traffic of the small shape.
// GROUP: feature blocks whose weight rows share an L2 residency (see the tile mapping below).
// DIRECT (the 256 x 256 shape): the tiles go from global memory straight into LDS (global_load_lds_dwordx4, lane l's
// 16 bytes land at M0 + 16 l), k advances in steps of 32 through FOUR buffers of unpadded 64-byte rows, three steps
// of loads in flight, no staging registers and no LDS writes by the waves.  The compiler would wait for every
// outstanding load before an LDS read that may see such data; the fragment reads are therefore instructions it does
// not look into, with hand-placed waits (vector-memory operations complete in order: "at most 8 outstanding" after
// the requests of three steps means the oldest step has landed).
typedef __attribute__((address_space(1))) const void proj_gmem_cv;
typedef __attribute__((address_space(3))) void proj_lds_v;
template <int OFF>
__device__ __forceinline__ u32x4 proj_lds_read128(uint32_t addr) {
    u32x4 v;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF));
    return v;
}
template <int N>
__device__ __forceinline__ void proj_wait_lds(u32x4 (&a)[4], u32x4 (&b)[2]) {
    asm volatile("s_waitcnt lgkmcnt(%6)" : "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3]), "+v"(b[0]), "+v"(b[1]) : "n"(N));
}
template <int N>
__device__ __forceinline__ void proj_wait_vmem() {
    __builtin_amdgcn_s_waitcnt(((N >> 4) << 14) | (0xF << 8) | (0x7 << 4) | (N & 15));  // vmcnt(N), other counters open
    asm volatile("" ::: "memory");
}

template <int WM, int WN, int FI, int FJ, int GROUP, bool DIRECT = false>
__global__ __launch_bounds__(64 * WM * WN, 2) void proj_gemm_bf16_kernel(ProjArgs a) {
    static_assert(!DIRECT || (WM * WN == 8 && FI == 4 && FJ == 2), "the direct-to-LDS loop is written for the 256 x 256 shape");
    constexpr int NT = 64 * WM * WN;               // threads
    constexpr int BM = WM * FI * 32, BN = WN * FJ * 32, BK = 64;   // features, tokens, k per step
    constexpr int LDSROW = BK * 2 + 16;            // padded row of a tile
    constexpr int WTILE = BM * LDSROW, XTILE = BN * LDSROW;   // bytes of the two tiles of a buffer
    constexpr int RPP = NT / 8;                    // rows staged per pass (8 threads x 16 bytes per row)
    constexpr int WCH = BM / RPP, XCH = BN / RPP;  // 16-byte chunks a thread stages per tile and k-step
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];  // [2 buffers][W tile, x tile]

    const int tid = threadIdx.x;
    const int lane = tid & 63, wv = tid >> 6;
    const int n = lane & 31, h = lane >> 5;
    const int wm = wv / WN, wn = wv % WN;          // wave position
    // Workgroup -> tile, for eight L2 caches that take workgroups in turn (id % 8): the feature blocks are taken
    // in groups of GROUP; inside a group every cache owns the token blocks tb = id % 8 (mod 8) and walks them
    // with the feature block varying fastest, so an x tile is fetched once per group and the group's weight rows
    // stay resident in that cache.
    const int ntb8 = (int)((cdiv(a.tokens, BN) + 7) & ~7), nfb = (int)cdiv(a.N, BM);
    const int grp = blockIdx.x / (ntb8 * GROUP);
    const int rem = blockIdx.x - grp * (ntb8 * GROUP);
    const int gw = min(GROUP, nfb - grp * GROUP);
    const int local = rem >> 3;
    const int fb = grp * GROUP + local % gw;
    const int tb = (local / gw) * 8 + (rem & 7);
    if (local / gw >= ntb8 / 8 || tb * BN >= a.tokens) return;  // padding of the grid (whole workgroups leave)
    const int f0 = fb * BM, t0 = tb * BN;

    f32x16 acc[FI][FJ];
#pragma unroll
    for (int i = 0; i < FI; ++i)
#pragma unroll
        for (int j = 0; j < FJ; ++j) acc[i][j] = f32x16{0};

    if constexpr (DIRECT) {
        constexpr int DK = 32;                         // k per step
        constexpr int DTILE = (BM + BN) * 64;          // bytes of one buffer: W tile [BM][64 B], then x tile [BN][64 B]
        const int wvu = __builtin_amdgcn_readfirstlane(wv);
        // Wave w requests transfers 4 w .. 4 w + 3 of the 32 of a step: transfer i covers rows 16 i .. 16 i + 15 of the
        // W tile (i < 16) or of the x tile; lane l fetches, for row r = l / 4 of the transfer, the 16-byte chunk
        // (l % 4) ^ ((row >> 2) & 3) of the row's 64 bytes: the chunk swizzle that makes the fragment reads (32 rows,
        // one chunk each) touch every bank twice, which 512 bytes need anyway.
        const unsigned char* src[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int i = wvu * 4 + u;
            const int row = (i & 15) * 16 + (lane >> 2);
            const int chunk = (lane & 3) ^ ((row >> 2) & 3);
            if (i < 16) {
                const int f = min(f0 + row, a.N - 1);  // rows beyond the last feature repeat it; never stored
                const int sg = proj_segment_of(a, f);
                src[u] = reinterpret_cast<const unsigned char*>(a.w[sg] + (int64_t)(f - a.seg_begin[sg]) * a.K) + chunk * 16;
            } else {
                const int t = min(t0 + row, a.tokens - 1);
                src[u] = reinterpret_cast<const unsigned char*>(a.x + (int64_t)t * a.K) + chunk * 16;
            }
        }
        auto request_step = [&](int step) {
            unsigned char* buf = smem + (step & 3) * DTILE;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int i = wvu * 4 + u;
                __builtin_amdgcn_global_load_lds((proj_gmem_cv*)(src[u] + (int64_t)step * (DK * 2)), (proj_lds_v*)(buf + i * 1024), 16, 0, 0);
            }
        };
        // fragment reads: W rows wm*FI*32 + i*32 + n, x rows wn*FJ*32 + j*32 + n, chunk 2 kk + h (swizzled by (n >> 2) & 3)
        const uint32_t lds0 = (uint32_t)(uintptr_t)(proj_lds_v*)smem;
        const uint32_t swz = (uint32_t)((n >> 2) & 3);
        const uint32_t wrow = lds0 + (uint32_t)(wm * FI * 32 + n) * 64u, xrow = lds0 + (uint32_t)(BM * 64) + (uint32_t)(wn * FJ * 32 + n) * 64u;
        const uint32_t koff[2] = {(((uint32_t)h) ^ swz) * 16u, ((2u + (uint32_t)h) ^ swz) * 16u};
        const int nstep = a.K / DK;
        request_step(0);
        if (nstep > 1) request_step(1);
        if (nstep > 2) request_step(2);
        if (nstep > 2)
            proj_wait_vmem<8>();
        else if (nstep > 1)
            proj_wait_vmem<4>();
        else
            proj_wait_vmem<0>();
        // (a bare barrier: the fence of __syncthreads would wait for EVERY outstanding transfer, also those of later steps;
        // what has to be ordered here is ordered by the waits above and below)
        __builtin_amdgcn_s_barrier();
        for (int it = 0; it < nstep; ++it) {
            if (it + 3 < nstep) request_step(it + 3);  // into the buffer that step it - 1 used: every wave is past it
            const uint32_t b = (uint32_t)(it & 3) * (uint32_t)DTILE;
            u32x4 a0[4], b0[2], a1[4], b1[2];
            {
                const uint32_t wa = wrow + b + koff[0], xa = xrow + b + koff[0];
                a0[0] = proj_lds_read128<0>(wa);
                a0[1] = proj_lds_read128<2048>(wa);
                a0[2] = proj_lds_read128<4096>(wa);
                a0[3] = proj_lds_read128<6144>(wa);
                b0[0] = proj_lds_read128<0>(xa);
                b0[1] = proj_lds_read128<2048>(xa);
            }
            {
                const uint32_t wa = wrow + b + koff[1], xa = xrow + b + koff[1];
                a1[0] = proj_lds_read128<0>(wa);
                a1[1] = proj_lds_read128<2048>(wa);
                a1[2] = proj_lds_read128<4096>(wa);
                a1[3] = proj_lds_read128<6144>(wa);
                b1[0] = proj_lds_read128<0>(xa);
                b1[1] = proj_lds_read128<2048>(xa);
            }
            proj_wait_lds<6>(a0, b0);
#pragma unroll
            for (int i = 0; i < FI; ++i)
#pragma unroll
                for (int j = 0; j < FJ; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a0[i]), __builtin_bit_cast(bf16x8, b0[j]),
                                                                        acc[i][j], 0, 0, 0);
            proj_wait_lds<0>(a1, b1);
#pragma unroll
            for (int i = 0; i < FI; ++i)
#pragma unroll
                for (int j = 0; j < FJ; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a1[i]), __builtin_bit_cast(bf16x8, b1[j]),
                                                                        acc[i][j], 0, 0, 0);
            // the next step's tiles have landed (this wave's share; the barrier covers the others')
            if (it + 3 < nstep)
                proj_wait_vmem<8>();
            else if (it + 2 < nstep)
                proj_wait_vmem<4>();
            else
                proj_wait_vmem<0>();
            __builtin_amdgcn_s_barrier();
        }
    } else {
        // ---- what each thread stages: rows tid/8 + RPP*c of both tiles, chunk tid%8 -------------------------------
        const unsigned char* wsrc[WCH];
        const unsigned char* xsrc[XCH];
    #pragma unroll
        for (int c = 0; c < WCH; ++c) {
            const int f = min(f0 + (tid >> 3) + RPP * c, a.N - 1);  // rows beyond the last feature repeat it; never stored
            const int s = proj_segment_of(a, f);
            wsrc[c] = reinterpret_cast<const unsigned char*>(a.w[s] + (int64_t)(f - a.seg_begin[s]) * a.K) + (tid & 7) * 16;
        }
    #pragma unroll
        for (int c = 0; c < XCH; ++c) {
            const int t = min(t0 + (tid >> 3) + RPP * c, a.tokens - 1);
            xsrc[c] = reinterpret_cast<const unsigned char*>(a.x + (int64_t)t * a.K) + (tid & 7) * 16;
        }
        u32x4 wreg[WCH], xreg[XCH];
        auto load_step = [&](int k0) {
    #pragma unroll
            for (int c = 0; c < WCH; ++c) wreg[c] = *reinterpret_cast<const u32x4*>(wsrc[c] + (int64_t)k0 * 2);
    #pragma unroll
            for (int c = 0; c < XCH; ++c) xreg[c] = *reinterpret_cast<const u32x4*>(xsrc[c] + (int64_t)k0 * 2);
        };
        auto store_step = [&](int buf) {
            unsigned char* wt = smem + buf * (WTILE + XTILE);
            unsigned char* xt = wt + WTILE;
    #pragma unroll
            for (int c = 0; c < WCH; ++c) *reinterpret_cast<u32x4*>(wt + ((tid >> 3) + RPP * c) * LDSROW + (tid & 7) * 16) = wreg[c];
    #pragma unroll
            for (int c = 0; c < XCH; ++c) *reinterpret_cast<u32x4*>(xt + ((tid >> 3) + RPP * c) * LDSROW + (tid & 7) * 16) = xreg[c];
        };

        const int nstep = a.K / BK;
        load_step(0);
        store_step(0);
        __syncthreads();
        for (int it = 0; it < nstep; ++it) {
            const bool more = it + 1 < nstep;
            if (more) load_step((it + 1) * BK);
            const unsigned char* wt = smem + (it & 1) * (WTILE + XTILE) + (wm * FI * 32 + n) * LDSROW + h * 16;
            const unsigned char* xt = smem + (it & 1) * (WTILE + XTILE) + WTILE + (wn * FJ * 32 + n) * LDSROW + h * 16;
    #pragma unroll
            for (int kk = 0; kk < BK / 16; ++kk) {
                bf16x8 af[FI], bf[FJ];
    #pragma unroll
                for (int i = 0; i < FI; ++i) af[i] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(wt + i * 32 * LDSROW + kk * 32));
    #pragma unroll
                for (int j = 0; j < FJ; ++j) bf[j] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(xt + j * 32 * LDSROW + kk * 32));
    #pragma unroll
                for (int i = 0; i < FI; ++i)
    #pragma unroll
                    for (int j = 0; j < FJ; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bf[j], acc[i][j], 0, 0, 0);
            }
            if (more) store_step((it + 1) & 1);
            __syncthreads();
        }

    }

    // ---- epilogue: lane (token n, half h) holds, per accumulator, features 8*g + 4*h + 0..3 for g = 0..3 --------
#pragma unroll
    for (int j = 0; j < FJ; ++j) {
        const int t = t0 + (wn * FJ + j) * 32 + n;
        if (t >= a.tokens) continue;
#pragma unroll
        for (int i = 0; i < FI; ++i) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int f = f0 + (wm * FI + i) * 32 + 8 * g + 4 * h;  // first of four consecutive features
                if (f >= a.N) continue;
                const int s = proj_segment_of(a, f);
                const int width = a.seg_begin[s + 1] - a.seg_begin[s];
                const int c0 = f - a.seg_begin[s];
                const float y[4] = {acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]};
                if (f + 3 < a.seg_begin[s + 1] && a.kind[s] == 0 && ((width | c0) & 3) == 0) {  // four features of one bf16 segment
                    const u32x2 v = {pack_bf16x2(y[0], y[1]), pack_bf16x2(y[2], y[3])};
                    *reinterpret_cast<u32x2*>(static_cast<__bf16*>(a.out[s]) + (int64_t)t * width + c0) = v;
                } else {  // segment boundary inside the group, a narrow segment, or the sigmoid segment
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int fe = f + e;
                        if (fe >= a.N) break;
                        const int se = proj_segment_of(a, fe);
                        const int we = a.seg_begin[se + 1] - a.seg_begin[se];
                        const int64_t o = (int64_t)t * we + (fe - a.seg_begin[se]);
                        if (a.kind[se] == 1)
                            static_cast<float*>(a.out[se])[o] = sigmoid_f32(y[e]);
                        else
                            static_cast<uint16_t*>(a.out[se])[o] = (uint16_t)f32_to_bf16_bits(y[e]);
                    }
                }
            }
        }
    }
}

template <int WM, int WN, int FI, int FJ, int GROUP, bool DIRECT = false>
static hipError_t launch_proj_shape(const ProjArgs& a, hipStream_t st) {
    constexpr int BM = WM * FI * 32, BN = WN * FJ * 32;
    const size_t smem = DIRECT ? (size_t)4 * (BM + BN) * 64 : (size_t)2 * (BM + BN) * (64 * 2 + 16);
    auto kern = proj_gemm_bf16_kernel<WM, WN, FI, FJ, GROUP, DIRECT>;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    const int64_t ntb8 = (cdiv(a.tokens, BN) + 7) & ~7, nfb = cdiv(a.N, BM);
    // every group of GROUP feature blocks takes ntb8 * GROUP ids (a smaller last group leaves some unused)
    const int64_t ngrp = cdiv(nfb, GROUP);
    hipLaunchKernelGGL(kern, dim3((unsigned)(ngrp * ntb8 * GROUP)), dim3(64 * WM * WN), smem, st, a);
    return hipGetLastError();
}

// One fused GEMM over nseg output segments; segment s has width[s] features, weights W[s] [width[s], K] and
// destination out[s] [tokens, width[s]] (bf16 for kind 0, fp32 holding the sigmoid for kind 1).
hipError_t launch_projection(const void* x, int64_t tokens, int K, int nseg, const void* const* W, void* const* out,
                             const int32_t* width, const int32_t* kind, hipStream_t st) {
    ProjArgs a{};
    a.x = static_cast<const __bf16*>(x);
    a.nseg = nseg;
    a.tokens = (int32_t)tokens;
    a.K = K;
    int32_t begin = 0;
    for (int s = 0; s < kProjMaxSeg; ++s) {
        const int u = s < nseg ? s : nseg - 1;   // unused slots repeat the last segment (never selected)
        a.w[s] = static_cast<const __bf16*>(W[u]);
        a.out[s] = out[u];
        a.kind[s] = kind[u];
        a.seg_begin[s] = begin;
        if (s < nseg) begin += width[s];
    }
    for (int s = nseg; s <= kProjMaxSeg; ++s) a.seg_begin[s] = begin;
    a.N = begin;
    // large calls: 256 x 256 tiles, one workgroup of eight waves per compute unit; small ones: 128 x 128
    if (a.tokens >= 2048 && a.N >= 512) return launch_proj_shape<2, 4, 4, 2, 4, GSA_PROJ_DIRECT != 0>(a, st);
    return launch_proj_shape<2, 2, 2, 2, 8>(a, st);
}

}  // namespace gsa
