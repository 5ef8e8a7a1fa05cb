// Decode-serving state: append-only per-sequence caches of indexer keys, keys and gated values.
// The value cache holds V' = V * sigmoid(g2) (Sec. 3.5), rounded to the storage type exactly as the value-gate
// pre-pass does, so a decode step gathers two rows per selected key and never reads gate logits of old tokens.
#include "common.hpp"

namespace gsa {

struct AppendArgs {
    const void* kI_new;
    const void* K_new;
    const void* V_new;
    const void* g2_new;
    void* kI_cache;
    void* K_cache;
    void* Vg_cache;
    const int32_t* seq_lens;
    int32_t* seq_lens_out;
    int32_t B, T, Lk;
    int32_t kv_chunks;  // 16-byte chunks of one token's K (or V) row: H_kv * d_h * element size / 16
    int32_t ki_chunks;  // 16-byte chunks of one token's indexer key
    PageMap pm;         // contiguous caches [B, Lk, ...] or pages of a pool
};

// One thread per 16-byte chunk of a new token's K row (and the matching V chunk), the first ki_chunks threads
// of a token also copy its indexer key.  Tokens that do not fit the capacity are dropped.
template <bool BF16>
__global__ void cache_append_kernel(AppendArgs a) {
    const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t per_tok = max(a.kv_chunks, a.ki_chunks);
    if (gid >= (int64_t)a.B * a.T * per_tok) return;
    const int c = (int)(gid % per_tok);
    const int64_t bt = gid / per_tok;
    const int j = (int)(bt % a.T);
    const int b = (int)(bt / a.T);
    const int len = max(0, min(a.seq_lens[b], a.Lk));
    if (c == 0 && j == 0 && a.seq_lens_out) a.seq_lens_out[b] = min(len + a.T, a.Lk);
    const int pos = len + j;
    if (pos >= a.Lk) return;
    const int64_t row = cache_row(a.pm, b, pos, a.Lk);
    if (c < a.ki_chunks)
        static_cast<u32x4*>(a.kI_cache)[row * a.ki_chunks + c] = static_cast<const u32x4*>(a.kI_new)[bt * a.ki_chunks + c];
    if (c >= a.kv_chunks) return;
    const int64_t src = bt * a.kv_chunks + c;
    const int64_t dst = row * a.kv_chunks + c;
    static_cast<u32x4*>(a.K_cache)[dst] = static_cast<const u32x4*>(a.K_new)[src];
    u32x4 v = static_cast<const u32x4*>(a.V_new)[src];
    const u32x4 g = static_cast<const u32x4*>(a.g2_new)[src];
    if constexpr (BF16) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float v0 = bf16_bits_to_f32(v[e] & 0xffffu) * sigmoid_f32(bf16_bits_to_f32(g[e] & 0xffffu));
            const float v1 = bf16_bits_to_f32(v[e] >> 16) * sigmoid_f32(bf16_bits_to_f32(g[e] >> 16));
            v[e] = pack_bf16x2(v0, v1);
        }
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = __float_as_uint(__uint_as_float(v[e]) * (1.0f / (1.0f + expf(-__uint_as_float(g[e])))));
    }
    static_cast<u32x4*>(a.Vg_cache)[dst] = v;
}

hipError_t launch_cache_append(const gsa_shape& sh, const void* kI_new, const void* K_new, const void* V_new, const void* g2_new,
                               const int32_t* seq_lens, void* kI_cache, void* K_cache, void* Vg_cache, int32_t* seq_lens_out,
                               const PageMap& pm, hipStream_t st) {
    const int eb = sh.dtype == GSA_BF16 ? 2 : 4;
    AppendArgs a;
    a.pm = pm;
    a.kI_new = kI_new;
    a.K_new = K_new;
    a.V_new = V_new;
    a.g2_new = g2_new;
    a.kI_cache = kI_cache;
    a.K_cache = K_cache;
    a.Vg_cache = Vg_cache;
    a.seq_lens = seq_lens;
    a.seq_lens_out = seq_lens_out;
    a.B = sh.B;
    a.T = sh.Lq;
    a.Lk = sh.Lk;
    a.kv_chunks = sh.H_kv * sh.d_h * eb / 16;
    a.ki_chunks = sh.dI * eb / 16;
    const int64_t n = (int64_t)sh.B * sh.Lq * (a.kv_chunks > a.ki_chunks ? a.kv_chunks : a.ki_chunks);
    if (sh.dtype == GSA_BF16)
        hipLaunchKernelGGL(cache_append_kernel<true>, dim3((unsigned)cdiv(n, 256)), dim3(256), 0, st, a);
    else
        hipLaunchKernelGGL(cache_append_kernel<false>, dim3((unsigned)cdiv(n, 256)), dim3(256), 0, st, a);
    return hipGetLastError();
}

// Paged caches: the selected token positions of every row, rewritten as rows of the pool (what the attention
// kernels gather in pool mode).  phys [B, row_end - row_begin, k_cap]; entries beyond n_sel are left alone.
__global__ void translate_indices_kernel(PageMap pm, const int32_t* idx, int idx_rows, int idx_row0, const int32_t* n_sel,
                                         int32_t* phys, int B, int Lq, int Lk, int row_begin, int row_end, int k_cap) {
    const int R = row_end - row_begin;
    const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= (int64_t)B * R * k_cap) return;
    const int j = (int)(gid % k_cap);
    const int64_t rid = gid / k_cap;
    const int b = (int)(rid / R);
    const int t = row_begin + (int)(rid % R);
    if (j >= n_sel[(int64_t)b * Lq + t]) return;
    const int tok = idx[((int64_t)b * idx_rows + (t - idx_row0)) * k_cap + j];
    phys[gid] = (int32_t)cache_row(pm, b, max(0, min(tok, Lk - 1)), Lk);
}

hipError_t launch_translate_indices(const gsa_shape& sh, const PageMap& pm, int row_begin, int row_end, const int32_t* idx,
                                    int idx_rows, int idx_row0, const int32_t* n_sel, int k_cap, int32_t* phys, hipStream_t st) {
    const int64_t n = (int64_t)sh.B * (row_end - row_begin) * k_cap;
    hipLaunchKernelGGL(translate_indices_kernel, dim3((unsigned)cdiv(n, 256)), dim3(256), 0, st, pm, idx, idx_rows, idx_row0, n_sel,
                       phys, sh.B, sh.Lq, sh.Lk, row_begin, row_end, k_cap);
    return hipGetLastError();
}

}  // namespace gsa
