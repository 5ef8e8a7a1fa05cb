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
// (128 x 128 with four on small calls); k advances in steps of 64 through double-buffered LDS tiles (144-byte
// padded rows, conflict-free 16-byte fragment reads), one barrier per step, the next step's global loads in
// flight during the products.
#include "common.hpp"

namespace gsa {

constexpr int kProjMaxSeg = 8;

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
template <int WM, int WN, int FI, int FJ, int GROUP>
__global__ __launch_bounds__(64 * WM * WN, 2) void proj_gemm_bf16_kernel(ProjArgs a) {
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

    f32x16 acc[FI][FJ];
#pragma unroll
    for (int i = 0; i < FI; ++i)
#pragma unroll
        for (int j = 0; j < FJ; ++j) acc[i][j] = f32x16{0};

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

template <int WM, int WN, int FI, int FJ, int GROUP>
static hipError_t launch_proj_shape(const ProjArgs& a, hipStream_t st) {
    constexpr int BM = WM * FI * 32, BN = WN * FJ * 32;
    const size_t smem = (size_t)2 * (BM + BN) * (64 * 2 + 16);
    auto kern = proj_gemm_bf16_kernel<WM, WN, FI, FJ, GROUP>;
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
    if (a.tokens >= 2048 && a.N >= 512) return launch_proj_shape<2, 4, 4, 2, 4>(a, st);
    return launch_proj_shape<2, 2, 2, 2, 8>(a, st);
}

}  // namespace gsa
