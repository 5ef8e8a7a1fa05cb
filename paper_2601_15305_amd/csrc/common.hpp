// Shared device helpers for the libgsa kernels (gfx950 only: wave64, MFMA, LDS transpose reads).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/gsa.h"

namespace gsa {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

constexpr float kLog2e = 1.4426950408889634f;

// One hardware exp2 / reciprocal (each about 1 ulp).
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float fast_rcp(float x) { return __builtin_amdgcn_rcpf(x); }

// sigmoid(z) = 1 / (1 + 2^(-z log2 e)).  Saturates cleanly: 2^x -> inf gives 0, 2^x -> 0 gives 1.
__device__ __forceinline__ float sigmoid_f32(float z) { return fast_rcp(1.0f + fast_exp2(-kLog2e * z)); }

// bf16 <-> fp32.  fp32 -> bf16 rounds to nearest even with the conversion instruction of gfx950 (one
// instruction per pair of values).
__device__ __forceinline__ float bf16_bits_to_f32(uint32_t hi16) { return __uint_as_float(hi16 << 16); }
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    typedef __attribute__((ext_vector_type(2))) float f32x2_;
    typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_;
    const f32x2_ v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_));
}
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) { return pack_bf16x2(f, 0.f) & 0xffffu; }

__device__ __forceinline__ int lane_id() { return threadIdx.x & 63; }

// Butterfly reductions over a 64-wide wavefront.
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// Position offset of batch element b: query row i has absolute position offset + i.  With per-sequence lengths
// (ragged decode batches) the Lq rows are the last Lq tokens of a sequence that holds seq_lens[b] tokens.
__device__ __forceinline__ int batch_q_offset(const int32_t* seq_lens, int b, int q_offset, int Lq, int Lk) {
    return seq_lens ? max(0, min(seq_lens[b] - Lq, Lk - Lq)) : q_offset;
}

// Where the cached rows of a sequence live.  Contiguous caches (table == nullptr): row s of sequence b is row
// b * Lk + s of a [B, Lk, ...] tensor.  Paged caches: a sequence's tokens sit in pages of 2^page_shift tokens
// scattered over a pool of pool_pages pages; table[b * max_pages + p] is the pool page that holds tokens
// p * 2^page_shift .. of sequence b (page numbers are clamped to the pool, so a bad table reads wrong rows,
// never memory outside the pool).
struct PageMap {
    const int32_t* table;
    int32_t page_shift;
    int32_t max_pages;
    int32_t pool_pages;
};
__device__ __forceinline__ int64_t cache_row(const PageMap& pm, int b, int s, int Lk) {
    if (!pm.table) return (int64_t)b * Lk + s;
    const int pg = max(0, min(pm.table[(int64_t)b * pm.max_pages + (s >> pm.page_shift)], pm.pool_pages - 1));
    return ((int64_t)pg << pm.page_shift) + (s & ((1 << pm.page_shift) - 1));
}

// Exact host/device ceil-div.
__host__ __device__ constexpr int64_t cdiv(int64_t a, int64_t b) { return (a + b - 1) / b; }

}  // namespace gsa
