// Training side (Sec. 6.1): gradients of the sparse gated attention of Sec. 3.5 / 3.6 with the selection S_t held
// fixed (top-k has no gradient), the sparse-phase loss of the indexer, KL(p_{t,S_t} || softmax(I_{t,S_t})), and
// the gradients of the indexer scores of Sec. 3.3 that this loss sends back.
//
// The attention backward has two forms.  Without a workspace: one kernel in plain fp32 vector arithmetic, one wave
// per query and up to four query heads of one kv group (a lane computes the logits of one selected token from the
// whole K row, then every lane owns d_h / 64 features for the sums over tokens); contributions to keys that several
// queries select are added with fp32 atomics.  With a workspace: a query-centred pass (on the matrix cores for bf16
// inputs) for dQ and dg1, the selection turned into per-key lists, and a key-centred pass that sums dK and dV' key
// by key without atomics.  The indexer loss kernel is vector arithmetic with atomics into dkI and dbI.  Wherever
// sums are formed by atomics, or over lists filled through atomic cursors, their last bits vary from run to run.
#include "common.hpp"

namespace gsa {

hipError_t launch_value_gate(const gsa_shape& sh, const void* V, const void* g2, void* Vg, hipStream_t st);

constexpr float kTrainNegBig = -1.0e30f;

template <typename T>
__device__ __forceinline__ float ldf(const T* p, int64_t i);
template <>
__device__ __forceinline__ float ldf<float>(const float* p, int64_t i) {
    return p[i];
}
template <>
__device__ __forceinline__ float ldf<__bf16>(const __bf16* p, int64_t i) {
    return bf16_bits_to_f32(reinterpret_cast<const uint16_t*>(p)[i]);
}
__device__ __forceinline__ float precise_sigmoid(float z) { return 1.0f / (1.0f + expf(-z)); }
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

struct AttnBwdArgs {
    const void* Q;
    const void* K;
    const void* V;
    const void* g2;
    const void* g1;
    const void* dout;
    const int32_t* idx;    // [B, Lq, k_cap]
    const int32_t* n_sel;  // [B, Lq]
    float* dQ;             // [B, Lq, H, d_h]
    float* dK;             // [B, Lk, H_kv, d_h], zeroed before the launch
    float* dVp;            // [B, Lk, H_kv, d_h], zeroed before the launch: gradient of the gated values V'
    float* dg1;            // [B, Lq, H, d_h] or null
    float* p_sum;          // [B, Lq, k_cap] or null, zeroed before the launch: attention weights averaged over the heads
    int32_t B, Lq, Lk, H, H_kv, k_cap;
    float scale;
    // Key-centred second pass (workspace given): the query-centred kernel leaves dK / dV' alone and stores what the
    // key-centred kernel needs instead.
    void* dO_ws;    // [B, Lq, H, d_h], element type of the inputs: gradient of the ungated outputs, dout * sigmoid(g1)
    float* lse_ws;  // [B, Lq, H]: log of the softmax denominator of the scaled logits (natural log)
    float* D_ws;    // [B, Lq, H]: dO . O
};

// Eight consecutive elements of a row as floats (one or two 16-byte loads).
__device__ __forceinline__ void load8(const float* p, float (&x)[8]) {
    const float4 a = *reinterpret_cast<const float4*>(p);
    const float4 b = *reinterpret_cast<const float4*>(p + 4);
    x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w;
    x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
}
__device__ __forceinline__ void load8(const __bf16* p, float (&x)[8]) {
    const u32x4 v = *reinterpret_cast<const u32x4*>(p);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        x[2 * e] = bf16_bits_to_f32(v[e] & 0xffffu);
        x[2 * e + 1] = bf16_bits_to_f32(v[e] >> 16);
    }
}

// N = 4 or 8 consecutive elements of a row as floats.
template <int N>
__device__ __forceinline__ void loadn(const float* p, float (&x)[N]) {
#pragma unroll
    for (int i = 0; i < N; i += 4) {
        const float4 a = *reinterpret_cast<const float4*>(p + i);
        x[i] = a.x; x[i + 1] = a.y; x[i + 2] = a.z; x[i + 3] = a.w;
    }
}
template <int N>
__device__ __forceinline__ void loadn(const __bf16* p, float (&x)[N]) {
    if constexpr (N == 8) {
        load8(p, x);
    } else {
        const u32x2 v = *reinterpret_cast<const u32x2*>(p);
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            x[2 * e] = bf16_bits_to_f32(v[e] & 0xffffu);
            x[2 * e + 1] = bf16_bits_to_f32(v[e] >> 16);
        }
    }
}

// One wave per (query, chunk of HC query heads of one kv group): dQ, dg1 of those heads and their contributions to
// dK and dV' of the selected keys.  The heads of a chunk share every K / V / g2 row the wave reads, and their
// contributions to a key are summed in registers before the one atomic add per feature.
// SCATTER: dK and dV' by fp32 atomic adds from here; otherwise they are left to attn_bwd_keys_kernel.
template <typename T, int DH, int HC, bool SCATTER>
__global__ __launch_bounds__(256) void attn_bwd_kernel(AttnBwdArgs a) {
    constexpr int DPL = DH / 64;  // features per lane
    __shared__ __attribute__((aligned(16))) float lds[4][2 * HC * DH];
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    float* qs = lds[wv];              // the queries of the chunk's heads [HC][DH]
    float* dos = lds[wv] + HC * DH;   // gradients of their ungated outputs [HC][DH]
    const int64_t qrow = blockIdx.x;  // (b, t)
    const int b = (int)(qrow / a.Lq);
    const int nsel = max(0, min(a.n_sel[qrow], a.k_cap));
    const int32_t* idxrow = a.idx + qrow * a.k_cap;
    const int G = a.H / a.H_kv;       // a multiple of HC (chosen by the host)
    const int nchunk = a.H / HC;
    const T* Q = static_cast<const T*>(a.Q);
    const T* K = static_cast<const T*>(a.K);
    const T* V = static_cast<const T*>(a.V);
    const T* G2 = static_cast<const T*>(a.g2);
    const T* G1 = static_cast<const T*>(a.g1);
    const T* DO = static_cast<const T*>(a.dout);
    const float inv_heads = 1.0f / (float)a.H;

    for (int ch = wv; ch < nchunk; ch += 4) {
        const int h0 = ch * HC;
        const int g = h0 / G;
        const int64_t qbase = (qrow * a.H + h0) * DH;  // head hh of the chunk: + hh * DH
        float q[HC][DPL];
#pragma unroll
        for (int hh = 0; hh < HC; ++hh)
#pragma unroll
            for (int e = 0; e < DPL; ++e) {
                q[hh][e] = ldf(Q, qbase + hh * DH + lane + 64 * e);
                qs[hh * DH + lane + 64 * e] = q[hh][e];
            }
        __builtin_amdgcn_s_waitcnt(0);  // (one wave per LDS region: its own writes, then its own reads)
        __builtin_amdgcn_wave_barrier();
        auto key_row = [&](int tok) { return (((int64_t)b * a.Lk + tok) * a.H_kv + g) * DH; };
        auto logits_of = [&](int64_t krow, float (&x)[HC]) {
#pragma unroll
            for (int hh = 0; hh < HC; ++hh) x[hh] = 0.f;
            for (int c = 0; c < DH; c += 8) {
                float kv[8];
                load8(K + krow + c, kv);
#pragma unroll
                for (int hh = 0; hh < HC; ++hh) {
                    const float4 q0 = *reinterpret_cast<const float4*>(qs + hh * DH + c);
                    const float4 q1 = *reinterpret_cast<const float4*>(qs + hh * DH + c + 4);
                    x[hh] = fmaf(q0.x, kv[0], x[hh]); x[hh] = fmaf(q0.y, kv[1], x[hh]);
                    x[hh] = fmaf(q0.z, kv[2], x[hh]); x[hh] = fmaf(q0.w, kv[3], x[hh]);
                    x[hh] = fmaf(q1.x, kv[4], x[hh]); x[hh] = fmaf(q1.y, kv[5], x[hh]);
                    x[hh] = fmaf(q1.z, kv[6], x[hh]); x[hh] = fmaf(q1.w, kv[7], x[hh]);
                }
            }
#pragma unroll
            for (int hh = 0; hh < HC; ++hh) x[hh] *= a.scale;
        };
        // ---- pass 1: running maximum m, sum l and the unnormalised output o of every head ------------------------
        float m[HC], l[HC], o[HC][DPL];
#pragma unroll
        for (int hh = 0; hh < HC; ++hh) {
            m[hh] = kTrainNegBig;
            l[hh] = 0.f;
#pragma unroll
            for (int e = 0; e < DPL; ++e) o[hh][e] = 0.f;
        }
        for (int j0 = 0; j0 < nsel; j0 += 64) {
            const int j = j0 + lane;
            const int tok = max(0, min(idxrow[min(j, nsel - 1)], a.Lk - 1));
            float x[HC], p[HC];
            logits_of(key_row(tok), x);
#pragma unroll
            for (int hh = 0; hh < HC; ++hh) {
                if (j >= nsel) x[hh] = kTrainNegBig;
                const float mnew = fmaxf(m[hh], wave_max(x[hh]));
                const float alpha = expf(m[hh] - mnew);
                p[hh] = j < nsel ? expf(x[hh] - mnew) : 0.f;
                l[hh] = l[hh] * alpha + wave_sum(p[hh]);
                m[hh] = mnew;
#pragma unroll
                for (int e = 0; e < DPL; ++e) o[hh][e] *= alpha;
            }
            const int cnt = min(64, nsel - j0);
            for (int u = 0; u < cnt; ++u) {
                const int64_t vrow = key_row(__shfl(tok, u, 64));
                float v[DPL];
#pragma unroll
                for (int e = 0; e < DPL; ++e) {
                    v[e] = ldf(V, vrow + lane + 64 * e);
                    if (G2) v[e] *= precise_sigmoid(ldf(G2, vrow + lane + 64 * e));
                }
#pragma unroll
                for (int hh = 0; hh < HC; ++hh) {
                    const float pu = __shfl(p[hh], u, 64);
#pragma unroll
                    for (int e = 0; e < DPL; ++e) o[hh][e] = fmaf(pu, v[e], o[hh][e]);
                }
            }
        }
        // ---- gradient of the ungated outputs, of the output gate; D = dO . O -----------------------------------
        float inv_l[HC], D[HC], dO[HC][DPL];
#pragma unroll
        for (int hh = 0; hh < HC; ++hh) {
            inv_l[hh] = l[hh] > 0.f ? 1.0f / l[hh] : 0.f;
            float dpart = 0.f;
#pragma unroll
            for (int e = 0; e < DPL; ++e) {
                const int64_t i = qbase + hh * DH + lane + 64 * e;
                const float Oe = o[hh][e] * inv_l[hh];
                const float dy = ldf(DO, i);
                float s1 = 1.0f;
                if (G1) {
                    s1 = precise_sigmoid(ldf(G1, i));
                    if (a.dg1) a.dg1[i] = dy * Oe * s1 * (1.0f - s1);
                }
                dO[hh][e] = dy * s1;
                dos[hh * DH + lane + 64 * e] = dO[hh][e];
                if constexpr (!SCATTER) static_cast<float*>(a.dO_ws)[i] = dO[hh][e];  // (this kernel: fp32 inputs only)
                dpart = fmaf(dO[hh][e], Oe, dpart);
            }
            D[hh] = wave_sum(dpart);
            if constexpr (!SCATTER) {
                if (lane == 0) {
                    a.lse_ws[qrow * a.H + h0 + hh] = l[hh] > 0.f ? m[hh] + logf(l[hh]) : 0.f;
                    a.D_ws[qrow * a.H + h0 + hh] = D[hh];
                }
            }
        }
        __builtin_amdgcn_s_waitcnt(0);
        __builtin_amdgcn_wave_barrier();
        // ---- pass 2: ds_j = P_j (dO . V'_j - D); dq, and the contributions to dK and dV' ------------------------
        float dq[HC][DPL];
#pragma unroll
        for (int hh = 0; hh < HC; ++hh)
#pragma unroll
            for (int e = 0; e < DPL; ++e) dq[hh][e] = 0.f;
        for (int j0 = 0; j0 < nsel; j0 += 64) {
            const int j = j0 + lane;
            const int tok = max(0, min(idxrow[min(j, nsel - 1)], a.Lk - 1));
            float P[HC], ds[HC];
#pragma unroll
            for (int hh = 0; hh < HC; ++hh) P[hh] = ds[hh] = 0.f;
            if (j < nsel) {
                const int64_t krow = key_row(tok);
                float x[HC], dP[HC];
                logits_of(krow, x);
#pragma unroll
                for (int hh = 0; hh < HC; ++hh) dP[hh] = 0.f;
                for (int c = 0; c < DH; c += 8) {
                    float v[8];
                    load8(V + krow + c, v);
                    if (G2) {
                        float gg[8];
                        load8(G2 + krow + c, gg);
#pragma unroll
                        for (int e = 0; e < 8; ++e) v[e] *= precise_sigmoid(gg[e]);
                    }
#pragma unroll
                    for (int hh = 0; hh < HC; ++hh)
#pragma unroll
                        for (int e = 0; e < 8; ++e) dP[hh] = fmaf(dos[hh * DH + c + e], v[e], dP[hh]);
                }
                float psum = 0.f;
#pragma unroll
                for (int hh = 0; hh < HC; ++hh) {
                    P[hh] = expf(x[hh] - m[hh]) * inv_l[hh];
                    ds[hh] = P[hh] * (dP[hh] - D[hh]) * a.scale;
                    psum += P[hh];
                }
                if (a.p_sum) atomicAdd(&a.p_sum[qrow * a.k_cap + j], psum * inv_heads);
            }
            const int cnt = min(64, nsel - j0);
            for (int u = 0; u < cnt; ++u) {
                const int64_t krow = key_row(__shfl(tok, u, 64));
                float kel[DPL], dk[DPL], dv[DPL];
#pragma unroll
                for (int e = 0; e < DPL; ++e) {
                    kel[e] = ldf(K, krow + lane + 64 * e);
                    dk[e] = dv[e] = 0.f;
                }
#pragma unroll
                for (int hh = 0; hh < HC; ++hh) {
                    const float dsu = __shfl(ds[hh], u, 64);
                    const float pu = __shfl(P[hh], u, 64);
#pragma unroll
                    for (int e = 0; e < DPL; ++e) {
                        dq[hh][e] = fmaf(dsu, kel[e], dq[hh][e]);
                        if constexpr (SCATTER) {
                            dk[e] = fmaf(dsu, q[hh][e], dk[e]);
                            dv[e] = fmaf(pu, dO[hh][e], dv[e]);
                        }
                    }
                }
                if constexpr (SCATTER) {
#pragma unroll
                    for (int e = 0; e < DPL; ++e) {
                        atomicAdd(&a.dK[krow + lane + 64 * e], dk[e]);
                        atomicAdd(&a.dVp[krow + lane + 64 * e], dv[e]);
                    }
                }
            }
        }
#pragma unroll
        for (int hh = 0; hh < HC; ++hh)
#pragma unroll
            for (int e = 0; e < DPL; ++e) a.dQ[qbase + hh * DH + lane + 64 * e] = dq[hh][e];
        __builtin_amdgcn_wave_barrier();  // the next chunk rewrites qs and dos
    }
}

// ---- query-centred pass on the matrix cores (bf16 inputs, workspace given) ------------------------------------------
// One wave per (query, kv head), the G = H / H_kv query heads of the kv head as the N dimension (padded to 16) of
// v_mfma_f32_16x16x32_bf16, the gathered tokens as M or K: the dataflow of the forward kernel (attention.hip: whole
// K and V' rows staged in wave-private LDS tiles of 32 tokens; V holds the gated values).  Two passes over the list:
//   1. the forward: S^T = K Q^T, online softmax, O^T += V'^T P^T  ->  O, the softmax maximum and denominator;
//      then dO = dout * sigmoid(g1), D = dO . O, dg1, and what the key-centred pass needs (dO, log-sum-exp, D);
//   2. S^T again and dP^T = V' dO^T (V' rows read as an A operand, like K), P = exp(S - lse),
//      dS = P (dP - D) scale, dQ^T += K^T dS^T (K read back transposed, like V' in the forward).
// P, dO and dS enter the products rounded to bf16, as P does in the forward.
struct QBwdArgs {
    const void* Q;
    const void* K;
    const void* V;
    const void* g1;
    const void* dout;
    const int32_t* idx;
    const int32_t* n_sel;
    float* dQ;
    float* dg1;
    float* p_sum;
    __bf16* dO_ws;
    float* lse_ws;
    float* D_ws;
    int32_t B, Lq, Lk, H, H_kv, k_cap;
    float scale;
};
typedef __attribute__((address_space(3))) s16x4 train_lds_s16x4;
__device__ __forceinline__ float train_quad_row_max(float x) {  // max over lanes {l, l^16, l^32, l^48}
    auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    x = fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
    r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float train_quad_row_sum(float x) {
    auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    x = __uint_as_float(r[0]) + __uint_as_float(r[1]);
    r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

template <int DH>
__global__ __launch_bounds__(256, 2) void attn_bwd_q_mfma_kernel(QBwdArgs a) {
    constexpr int KK = DH / 32, MB = DH / 16, ROWB = DH * 2, VROW = ROWB + 32, KROW = ROWB + 16;
    constexpr int VCH = ROWB / 16, TPI = 64 / VCH, NVL = 32 / TPI;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int n = lane & 15, q = lane >> 4;
    unsigned char* vlds = smem + wv * (32 * (VROW + KROW));
    unsigned char* klds = vlds + 32 * VROW;
    const int g = __builtin_amdgcn_readfirstlane(blockIdx.y * 4 + wv);
    if (g >= a.H_kv) return;  // (the waves of a workgroup never synchronise with each other)
    const int64_t qrow = blockIdx.x;
    const int b = (int)(qrow / a.Lq);
    const int G = a.H / a.H_kv;
    const int head = g * G + n;
    const bool head_ok = n < G;
    const float sl2 = a.scale * kLog2e;
    const uint32_t tokstride = (uint32_t)a.H_kv * ROWB;
    const int nsel = max(0, min(a.n_sel[qrow], a.k_cap));
    const int32_t* idxrow = a.idx + qrow * a.k_cap;
    const int64_t row0 = (int64_t)b * a.Lk;
    const unsigned char* Kb = static_cast<const unsigned char*>(a.K) + (row0 * a.H_kv + g) * ROWB;
    const unsigned char* Vb = static_cast<const unsigned char*>(a.V) + (row0 * a.H_kv + g) * ROWB;
    const int64_t hbase = (qrow * a.H + (head_ok ? head : 0)) * DH;  // this lane's head row in Q / dout / g1 / dQ

    // B operands: lane (head n, chunk q) holds features (4 kk + q) * 8 .. + 8
    bf16x8 qf[KK];
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
        const u32x4 v = head_ok ? reinterpret_cast<const u32x4*>(static_cast<const __bf16*>(a.Q) + hbase)[kk * 4 + q] : u32x4{0, 0, 0, 0};
        qf[kk] = __builtin_bit_cast(bf16x8, v);
    }
    u32x4 kr[NVL], vf[NVL];
    const int slot0 = (lane / VCH) * NVL;
    auto load_idx = [&](int j0, int (&tk)[NVL]) {
#pragma unroll
        for (int r = 0; r < NVL; ++r) tk[r] = idxrow[min(j0 + slot0 + r, nsel - 1)];
    };
    auto issue = [&](const int (&tokv)[NVL]) {
#pragma unroll
        for (int r = 0; r < NVL; ++r) {
            const int tk = max(0, min(tokv[r], a.Lk - 1));
            const uint32_t off = __umul24((uint32_t)tk, tokstride) + (uint32_t)(lane % VCH) * 16u;
            kr[r] = *reinterpret_cast<const u32x4*>(Kb + off);
            vf[r] = *reinterpret_cast<const u32x4*>(Vb + off);
        }
    };
    auto stage = [&]() {
#pragma unroll
        for (int r = 0; r < NVL; ++r) *reinterpret_cast<u32x4*>(klds + (slot0 + r) * KROW + (lane % VCH) * 16) = kr[r];
#pragma unroll
        for (int r = 0; r < NVL; ++r) *reinterpret_cast<u32x4*>(vlds + (slot0 + r) * VROW + (lane % VCH) * 16) = vf[r];
    };
    // S^T (or dP^T) of the tile in LDS: rows of `tile` (row stride ROWSTRIDE) against the B operand bf
    auto rows_times = [&](const unsigned char* tile, int rowstride, const bf16x8 (&bf)[KK], f32x4& r0, f32x4& r1) {
        r0 = f32x4{0.f, 0.f, 0.f, 0.f};
        r1 = f32x4{0.f, 0.f, 0.f, 0.f};
        const unsigned char* p0 = tile + n * rowstride + q * 16;
        const unsigned char* p1 = p0 + 16 * rowstride;
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
            const u32x4 a0 = *reinterpret_cast<const u32x4*>(p0 + kk * 64);
            const u32x4 a1 = *reinterpret_cast<const u32x4*>(p1 + kk * 64);
            r0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a0), bf[kk], r0, 0, 0, 0);
            r1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a1), bf[kk], r1, 0, 0, 0);
        }
    };
    // acc^T[d, head] += tile^T[d, token] . w^T[token, head], the tile read back transposed
    auto transposed_times = [&](const unsigned char* tile, int rowstride, const bf16x8 wfrag, f32x4 (&acc)[MB]) {
        const int r4 = (lane & 15) >> 2, c4 = lane & 3;
        const unsigned char* p0 = tile + (4 * q + r4) * rowstride + c4 * 8;
        const unsigned char* p1 = p0 + 16 * rowstride;
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            s16x4 a0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((train_lds_s16x4*)(p0 + mb * 32));
            s16x4 a1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((train_lds_s16x4*)(p1 + mb * 32));
            typedef __attribute__((ext_vector_type(8))) short s16x8;
            s16x8 av = {a0[0], a0[1], a0[2], a0[3], a1[0], a1[1], a1[2], a1[3]};
            acc[mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, av), wfrag, acc[mb], 0, 0, 0);
        }
    };
    const int ntile = (nsel + 31) >> 5;
    // walks the list tile by tile: the next tile's rows and the entries of the tile after it are in flight while
    // `body(j0)` works on the tile in LDS
    auto for_tiles = [&](auto&& body) {
        int tok[NVL];
        if (ntile > 0) {
            load_idx(0, tok);
            issue(tok);
            if (ntile > 1) load_idx(32, tok);
        }
        for (int it = 0; it < ntile; ++it) {
            stage();
            if (it + 1 < ntile) {
                issue(tok);
                if (it + 2 < ntile) load_idx((it + 2) * 32, tok);
            }
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // this wave's LDS writes have landed
            body(it * 32);
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // reads done before the tile is overwritten
        }
    };

    // ---- pass 1: the forward ---------------------------------------------------------------------------------------
    f32x4 o[MB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) o[mb] = f32x4{0.f, 0.f, 0.f, 0.f};
    float mrun = kTrainNegBig, lrun = 0.f;
    for_tiles([&](int j0) {
        f32x4 s0, s1;
        rows_times(klds, KROW, qf, s0, s1);
        float x[8];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            x[i] = j0 + 4 * q + i < nsel ? s0[i] * sl2 : kTrainNegBig;
            x[4 + i] = j0 + 16 + 4 * q + i < nsel ? s1[i] * sl2 : kTrainNegBig;
        }
        float tmax = fmaxf(fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3])), fmaxf(fmaxf(x[4], x[5]), fmaxf(x[6], x[7])));
        tmax = train_quad_row_max(tmax);
        const float mnew = fmaxf(mrun, tmax);
        const float alpha = fast_exp2(mrun - mnew);
        float psum = 0.f, p[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            p[i] = fast_exp2(x[i] - mnew);
            psum += p[i];
        }
        lrun = lrun * alpha + psum;
        mrun = mnew;
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) o[mb] *= alpha;
        const u32x4 pw = {pack_bf16x2(p[0], p[1]), pack_bf16x2(p[2], p[3]), pack_bf16x2(p[4], p[5]), pack_bf16x2(p[6], p[7])};
        transposed_times(vlds, VROW, __builtin_bit_cast(bf16x8, pw), o);
    });
    const float ltot = train_quad_row_sum(lrun);
    const float inv = ltot > 0.f ? 1.0f / ltot : 0.f;

    // ---- dO = dout * sigmoid(g1), D = dO . O, dg1; lane (head n, q) holds features mb * 16 + 4 q + i of O ---------------
    float dpart = 0.f;
    if (head_ok) {
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            const int d0 = mb * 16 + 4 * q;
            const u32x2 dw = *reinterpret_cast<const u32x2*>(static_cast<const __bf16*>(a.dout) + hbase + d0);
            const float dy[4] = {bf16_bits_to_f32(dw[0] & 0xffffu), bf16_bits_to_f32(dw[0] >> 16), bf16_bits_to_f32(dw[1] & 0xffffu),
                                 bf16_bits_to_f32(dw[1] >> 16)};
            float s1v[4] = {1.f, 1.f, 1.f, 1.f};
            if (a.g1) {
                const u32x2 gw = *reinterpret_cast<const u32x2*>(static_cast<const __bf16*>(a.g1) + hbase + d0);
                s1v[0] = precise_sigmoid(bf16_bits_to_f32(gw[0] & 0xffffu));
                s1v[1] = precise_sigmoid(bf16_bits_to_f32(gw[0] >> 16));
                s1v[2] = precise_sigmoid(bf16_bits_to_f32(gw[1] & 0xffffu));
                s1v[3] = precise_sigmoid(bf16_bits_to_f32(gw[1] >> 16));
            }
            f32x4 dOv, dgv;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float Oe = o[mb][i] * inv;
                dOv[i] = dy[i] * s1v[i];
                dgv[i] = dy[i] * Oe * s1v[i] * (1.0f - s1v[i]);
                dpart = fmaf(dOv[i], Oe, dpart);
            }
            *reinterpret_cast<u32x2*>(a.dO_ws + hbase + d0) = u32x2{pack_bf16x2(dOv[0], dOv[1]), pack_bf16x2(dOv[2], dOv[3])};
            if (a.dg1) *reinterpret_cast<f32x4*>(a.dg1 + hbase + d0) = dgv;
        }
    }
    const float D = train_quad_row_sum(dpart);
    if (head_ok && q == 0) {
        a.lse_ws[qrow * a.H + head] = ltot > 0.f ? (mrun + log2f(ltot)) * 0.6931471805599453f : 0.f;
        a.D_ws[qrow * a.H + head] = D;
    }
    // dO as a B operand: lane (head n, chunk q) holds features (4 kk + q) * 8 .. + 8
    bf16x8 dof[KK];
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
        u32x4 w = {0, 0, 0, 0};
        if (head_ok) {
            const u32x4 dv = reinterpret_cast<const u32x4*>(static_cast<const __bf16*>(a.dout) + hbase)[kk * 4 + q];
            u32x4 gv = {0, 0, 0, 0};
            if (a.g1) gv = reinterpret_cast<const u32x4*>(static_cast<const __bf16*>(a.g1) + hbase)[kk * 4 + q];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                float y0 = bf16_bits_to_f32(dv[e] & 0xffffu), y1 = bf16_bits_to_f32(dv[e] >> 16);
                if (a.g1) {
                    y0 *= precise_sigmoid(bf16_bits_to_f32(gv[e] & 0xffffu));
                    y1 *= precise_sigmoid(bf16_bits_to_f32(gv[e] >> 16));
                }
                w[e] = pack_bf16x2(y0, y1);
            }
        }
        dof[kk] = __builtin_bit_cast(bf16x8, w);
    }

    // ---- pass 2: P, dS, dQ ------------------------------------------------------------------------------------------
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) o[mb] = f32x4{0.f, 0.f, 0.f, 0.f};  // now dQ^T
    const float inv_heads = 1.0f / (float)a.H;
    for_tiles([&](int j0) {
        f32x4 s0, s1, d0, d1;
        rows_times(klds, KROW, qf, s0, s1);
        rows_times(vlds, VROW, dof, d0, d1);
        float p[8], ds[8];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            p[i] = j0 + 4 * q + i < nsel ? fast_exp2(s0[i] * sl2 - mrun) * inv : 0.f;
            p[4 + i] = j0 + 16 + 4 * q + i < nsel ? fast_exp2(s1[i] * sl2 - mrun) * inv : 0.f;
            ds[i] = p[i] * (d0[i] - D) * a.scale;
            ds[4 + i] = p[4 + i] * (d1[i] - D) * a.scale;
        }
        if (a.p_sum) {  // attention weights averaged over the heads: sum over the sixteen lanes of a token group
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                float v = head_ok ? p[i] : 0.f;
#pragma unroll
                for (int ofs = 8; ofs > 0; ofs >>= 1) v += __shfl_xor(v, ofs, 64);
                const int j = j0 + (i < 4 ? 4 * q + i : 16 + 4 * q + (i - 4));
                if (n == 0 && j < nsel) atomicAdd(&a.p_sum[qrow * a.k_cap + j], v * inv_heads);
            }
        }
        const u32x4 dw = {pack_bf16x2(ds[0], ds[1]), pack_bf16x2(ds[2], ds[3]), pack_bf16x2(ds[4], ds[5]), pack_bf16x2(ds[6], ds[7])};
        transposed_times(klds, KROW, __builtin_bit_cast(bf16x8, dw), o);
    });
    if (head_ok) {
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) *reinterpret_cast<f32x4*>(a.dQ + hbase + mb * 16 + 4 * q) = o[mb];
    }
}

// ---- key-centred second pass: dK and dV' without atomics ------------------------------------------------------------
// The selection is turned round first: for every key and every window of WQ consecutive queries, the list of the
// queries of that window that selected the key ("inverted lists": a two-level histogram, its exclusive prefix sum,
// and a fill through per-list cursors).  Then one wave per (key, kv head, query window) walks its list, recomputes
// p and ds of every (query, head) pair from the saved softmax denominators, and sums q ds and dO p in registers;
// the windows are separate launches in ascending order, so all waves of a launch gather query and dO rows of one
// window (a few MiB per kv head: they stay in the L2s) and a key's sums pass from window to window through dK / dV'
// themselves, read and written by the one wave that owns (key, kv head) in that launch.
struct InvArgs {
    const int32_t* idx;    // [B, Lq, k_cap]
    const int32_t* n_sel;  // [B, Lq]
    int32_t* off;          // [B * Lk * NW + 1]: counts, then (after the scan) list starts; list (key, window) = slot key * NW + window
    int32_t* cursor;       // [B * Lk * NW], zeroed: entries of the list already filled
    int32_t* inv;          // [B * Lq * k_cap]: the lists, query positions t
    int32_t B, Lq, Lk, k_cap, wq_shift, NW;
};

template <bool FILL>
__global__ __launch_bounds__(256) void inv_lists_kernel(InvArgs a) {  // one wave per query row
    const int lane = threadIdx.x & 63;
    const int64_t qrow = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (qrow >= (int64_t)a.B * a.Lq) return;
    const int b = (int)(qrow / a.Lq), t = (int)(qrow % a.Lq);
    const int nsel = max(0, min(a.n_sel[qrow], a.k_cap));
    const int w = t >> a.wq_shift;
    for (int j = lane; j < nsel; j += 64) {
        const int tok = max(0, min(a.idx[qrow * a.k_cap + j], a.Lk - 1));
        const int64_t slot = ((int64_t)b * a.Lk + tok) * a.NW + w;
        if constexpr (FILL)
            a.inv[a.off[slot] + atomicAdd(&a.cursor[slot], 1)] = t;
        else
            atomicAdd(&a.off[slot], 1);
    }
}

// Exclusive prefix sum over n int32 values in place, in three steps: sums of blocks of 2048 values, the exclusive
// sums of those (one workgroup, serial over chunks of 1024 block sums), then every block scans its values from
// its offset.  block_sums holds ceil(n / 2048) values.
constexpr int kScanBlock = 2048;
__global__ __launch_bounds__(256) void scan_block_sums_kernel(const int32_t* v, int64_t n, int32_t* block_sums) {
    __shared__ int32_t red[4];
    const int64_t base = (int64_t)blockIdx.x * kScanBlock;
    int32_t s = 0;
    for (int i = threadIdx.x; i < kScanBlock; i += 256)
        if (base + i < n) s += v[base + i];
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) block_sums[blockIdx.x] = red[0] + red[1] + red[2] + red[3];
}
__global__ __launch_bounds__(1024) void scan_of_sums_kernel(int32_t* block_sums, int64_t nb) {  // one workgroup
    __shared__ int32_t wsum[16];
    __shared__ int32_t carry_s;
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    if (threadIdx.x == 0) carry_s = 0;
    __syncthreads();
    for (int64_t c0 = 0; c0 < nb; c0 += 1024) {
        const int64_t i = c0 + threadIdx.x;
        const int32_t x = i < nb ? block_sums[i] : 0;
        int32_t incl = x;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int32_t y = __shfl_up(incl, o, 64);
            if (lane >= o) incl += y;
        }
        if (lane == 63) wsum[wv] = incl;
        __syncthreads();
        int32_t before = carry_s;
        for (int k = 0; k < wv; ++k) before += wsum[k];
        if (i < nb) block_sums[i] = before + incl - x;
        __syncthreads();
        if (threadIdx.x == 1023) carry_s = before + incl;
        __syncthreads();
    }
}
__global__ __launch_bounds__(256) void scan_blocks_kernel(int32_t* v, int64_t n, const int32_t* block_sums) {
    __shared__ int32_t wsum[4];
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int64_t base = (int64_t)blockIdx.x * kScanBlock + threadIdx.x * 8;  // eight consecutive values per thread
    int32_t x[8], tot = 0;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        x[e] = base + e < n ? v[base + e] : 0;
        tot += x[e];
    }
    int32_t incl = tot;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int32_t y = __shfl_up(incl, o, 64);
        if (lane >= o) incl += y;
    }
    if (lane == 63) wsum[wv] = incl;
    __syncthreads();
    int32_t run = block_sums[blockIdx.x] + incl - tot;
    for (int k = 0; k < wv; ++k) run += wsum[k];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        if (base + e < n) v[base + e] = run;
        run += x[e];
    }
}

// Sum over the sixteen lanes of a row (every lane gets it), without LDS: two quad permutes, then the mirrored halves.
template <int CTRL>
__device__ __forceinline__ float dpp_add(float x) {
    return x + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xF, 0xF, true));
}
__device__ __forceinline__ float row16_sum(float x) {
    x = dpp_add<0xB1>(x);   // quad_perm [1,0,3,2]
    x = dpp_add<0x4E>(x);   // quad_perm [2,3,0,1]
    x = dpp_add<0x141>(x);  // row_half_mirror
    return dpp_add<0x140>(x);  // row_mirror
}

struct KeyBwdArgs {
    const void* Q;
    const void* K;
    const void* V;
    const void* g2;
    const void* dO;    // [B, Lq, H, d_h], element type of the inputs
    const float* lse;  // [B, Lq, H]
    const float* D;    // [B, Lq, H]
    const int32_t* off;
    const int32_t* inv;
    float* dK;   // [B, Lk, H_kv, d_h]: sums of the windows before this one on entry
    float* dVp;
    int32_t B, Lq, Lk, H, H_kv, NW, win, keys;  // keys: the keys 0 .. keys-1 can have entries in this window
    float scale;
};

// One wave per (key, kv head) of one query window.  Lane = (head slot hh = lane / 16, feature chunk c = lane % 16): a
// lane holds DH / 16 consecutive features of the key's K and V' rows and, entry by entry, of one head's query and
// dO rows; the two dot products of a pair are reduced over the sixteen lanes of its head slot.  Groups of more than
// four query heads per kv head take several passes over the list.
template <typename T, int DH>
__global__ __launch_bounds__(256) void attn_bwd_keys_kernel(KeyBwdArgs a) {
    constexpr int FPL = DH / 16;
    const int lane = threadIdx.x & 63;
    const int hh = lane >> 4, c = lane & 15;
    const int key = blockIdx.x * 4 + (threadIdx.x >> 6);
    const int g = blockIdx.y, b = blockIdx.z;
    if (key >= a.keys) return;
    const int64_t slot = ((int64_t)b * a.Lk + key) * a.NW + a.win;
    const int e0 = a.off[slot], e1 = a.off[slot + 1];
    if (e0 >= e1) return;
    const int G = a.H / a.H_kv;
    const T* Q = static_cast<const T*>(a.Q);
    const int64_t krow = (((int64_t)b * a.Lk + key) * a.H_kv + g) * DH + c * FPL;
    float kf[FPL], vf[FPL], dk[FPL], dv[FPL];
    loadn<FPL>(static_cast<const T*>(a.K) + krow, kf);
    loadn<FPL>(static_cast<const T*>(a.V) + krow, vf);
    if (a.g2) {
        float gf[FPL];
        loadn<FPL>(static_cast<const T*>(a.g2) + krow, gf);
#pragma unroll
        for (int f = 0; f < FPL; ++f) vf[f] *= precise_sigmoid(gf[f]);
    }
#pragma unroll
    for (int f = 0; f < FPL; ++f) dk[f] = dv[f] = 0.f;
    for (int h0 = 0; h0 < G; h0 += 4) {
        const int hq = h0 + hh;
        const bool live = hq < G;
        const int head = g * G + (live ? hq : 0);
        int tq[4];  // the queries of the next step's entries, requested a step ahead
#pragma unroll
        for (int u = 0; u < 4; ++u) tq[u] = a.inv[min(e0 + u, e1 - 1)];
        for (int e = e0; e < e1; e += 4) {  // four entries per step: the loads of all go out before any is used
            int64_t r[4];
            float qv[4][FPL], ov[4][FPL], lse[4], Dv[4], sv[4], pv[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) r[u] = ((int64_t)b * a.Lq + tq[u]) * a.H + head;
#pragma unroll
            for (int u = 0; u < 4; ++u) tq[u] = a.inv[min(e + 4 + u, e1 - 1)];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                loadn<FPL>(Q + r[u] * DH + c * FPL, qv[u]);
                loadn<FPL>(static_cast<const T*>(a.dO) + r[u] * DH + c * FPL, ov[u]);
                lse[u] = a.lse[r[u]];
                Dv[u] = a.D[r[u]];
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                sv[u] = pv[u] = 0.f;
#pragma unroll
                for (int f = 0; f < FPL; ++f) {
                    sv[u] = fmaf(qv[u][f], kf[f], sv[u]);
                    pv[u] = fmaf(ov[u][f], vf[f], pv[u]);
                }
                sv[u] = row16_sum(sv[u]);
                pv[u] = row16_sum(pv[u]);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const float P = live && e + u < e1 ? expf(sv[u] * a.scale - lse[u]) : 0.f;
                const float ds = P * (pv[u] - Dv[u]) * a.scale;
#pragma unroll
                for (int f = 0; f < FPL; ++f) {
                    dk[f] = fmaf(ds, qv[u][f], dk[f]);
                    dv[f] = fmaf(P, ov[u][f], dv[f]);
                }
            }
        }
    }
    // sum over the four head slots; head slot 0 adds the result to what the earlier windows left
#pragma unroll
    for (int f = 0; f < FPL; ++f) {
        dk[f] += __shfl_xor(dk[f], 16, 64);
        dk[f] += __shfl_xor(dk[f], 32, 64);
        dv[f] += __shfl_xor(dv[f], 16, 64);
        dv[f] += __shfl_xor(dv[f], 32, 64);
    }
    if (hh == 0) {
#pragma unroll
        for (int f = 0; f < FPL; ++f) {
            a.dK[krow + f] += dk[f];
            a.dVp[krow + f] += dv[f];
        }
    }
}

// dV = dV' * sigmoid(g2) (in place), dg2 = dV' * V * sigmoid(g2) (1 - sigmoid(g2)); without g2, dV = dV' and dg2 = 0.
template <typename T>
__global__ void value_gate_bwd_kernel(const T* V, const T* g2, float* dV, float* dg2, int64_t n) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const float d = dV[i];
    if (g2) {
        const float s = precise_sigmoid(ldf(g2, i));
        dV[i] = d * s;
        if (dg2) dg2[i] = d * ldf(V, i) * s * (1.0f - s);
    } else if (dg2) {
        dg2[i] = 0.f;
    }
}

__global__ void fill_zero_kernel(float* p, int64_t n) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0.f;
}
static void zero_fill(float* p, int64_t n, hipStream_t st) {
    if (p && n > 0) hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)cdiv(n, 256)), dim3(256), 0, st, p, n);
}

// Workspace of the key-centred second pass.  Query windows of WQ = 2^wq_shift rows: the query and dO rows of one
// window and one kv head (G heads x d_h x (element + 4) bytes per row) stay near 3 MiB; at most 256 windows.
// (measured at C2-8k: 0.4 / 0.75 / 3 / 6 / 12 MiB per window and kv head: 9.8 / 9.0 / 8.4 / 8.2 / 8.5 ms)
constexpr int64_t kBwdWindowBytes = 3 << 20;
struct BwdPlan {
    int wq_shift, NW;
    int64_t n_slots;  // B * Lk * NW lists
    size_t o_dO, o_lse, o_D, o_off, o_cursor, o_sums, o_inv, o_vg, total;
};
static BwdPlan plan_bwd(const gsa_shape& sh, int k_cap) {
    BwdPlan p;
    const int elt = sh.dtype == GSA_BF16 ? 2 : 4;
    const int64_t row_bytes = (int64_t)(sh.H / sh.H_kv) * sh.d_h * (elt + 4);
    int shift = 6;
    while (shift < 20 && ((int64_t)2 << shift) * row_bytes <= kBwdWindowBytes) ++shift;
    while (cdiv(sh.Lq, (int64_t)1 << shift) > 256) ++shift;
    p.wq_shift = shift;
    p.NW = (int)cdiv(sh.Lq, (int64_t)1 << shift);
    p.n_slots = (int64_t)sh.B * sh.Lk * p.NW;
    auto up = [](size_t x) { return (x + 255) & ~(size_t)255; };
    size_t o = 0;
    p.o_dO = o;      o += up((size_t)sh.B * sh.Lq * sh.H * sh.d_h * elt);  // in the element type of the inputs
    p.o_lse = o;     o += up((size_t)sh.B * sh.Lq * sh.H * sizeof(float));
    p.o_D = o;       o += up((size_t)sh.B * sh.Lq * sh.H * sizeof(float));
    p.o_off = o;     o += up((size_t)(p.n_slots + 1) * sizeof(int32_t));
    p.o_cursor = o;  o += up((size_t)p.n_slots * sizeof(int32_t));
    p.o_sums = o;    o += up((size_t)cdiv(p.n_slots + 1, kScanBlock) * sizeof(int32_t));
    p.o_inv = o;     o += up((size_t)sh.B * sh.Lq * k_cap * sizeof(int32_t));
    p.o_vg = o;      o += sh.dtype == GSA_BF16 ? up((size_t)sh.B * sh.Lk * sh.H_kv * sh.d_h * elt) : 0;  // gated values (bf16 path)
    p.total = o;
    return p;
}
size_t attention_bwd_workspace_bytes(const gsa_shape& sh, int k_cap) { return plan_bwd(sh, k_cap).total; }

template <typename T, int DH, bool SCATTER>
static void (*pick_bwd_kernel(int hc))(AttnBwdArgs) {
    return hc == 4 ? attn_bwd_kernel<T, DH, 4, SCATTER> : (hc == 2 ? attn_bwd_kernel<T, DH, 2, SCATTER> : attn_bwd_kernel<T, DH, 1, SCATTER>);
}

hipError_t launch_attention_bwd(const gsa_shape& sh, const void* Q, const void* K, const void* V, const void* g2, const void* g1,
                                const int32_t* idx, const int32_t* n_sel, int k_cap, float scale, const void* dout, float* dQ,
                                float* dK, float* dV, float* dg1, float* dg2, float* p_sum, void* workspace, hipStream_t st) {
    AttnBwdArgs a;
    a.Q = Q;
    a.K = K;
    a.V = V;
    a.g2 = g2;
    a.g1 = g1;
    a.dout = dout;
    a.idx = idx;
    a.n_sel = n_sel;
    a.dQ = dQ;
    a.dK = dK;
    a.dVp = dV;
    a.dg1 = dg1;
    a.p_sum = p_sum;
    a.B = sh.B;
    a.Lq = sh.Lq;
    a.Lk = sh.Lk;
    a.H = sh.H;
    a.H_kv = sh.H_kv;
    a.k_cap = k_cap;
    a.scale = scale;
    const bool scatter = workspace == nullptr;
    unsigned char* ws = static_cast<unsigned char*>(workspace);
    const BwdPlan p = plan_bwd(sh, k_cap);
    a.dO_ws = scatter ? nullptr : static_cast<void*>(ws + p.o_dO);
    a.lse_ws = scatter ? nullptr : reinterpret_cast<float*>(ws + p.o_lse);
    a.D_ws = scatter ? nullptr : reinterpret_cast<float*>(ws + p.o_D);
    const int64_t kv_elems = (int64_t)sh.B * sh.Lk * sh.H_kv * sh.d_h;
    zero_fill(dK, kv_elems, st);
    zero_fill(dV, kv_elems, st);
    zero_fill(p_sum, (int64_t)sh.B * sh.Lq * k_cap, st);
    const dim3 grid((unsigned)((int64_t)sh.B * sh.Lq));
    const int G = sh.H / sh.H_kv;
    const int hc = G % 4 == 0 ? 4 : (G % 2 == 0 ? 2 : 1);  // query heads of one kv group a wave takes together
    void (*kern)(AttnBwdArgs) = nullptr;
    if (sh.dtype == GSA_BF16) {
        if (sh.d_h == 128)
            kern = scatter ? pick_bwd_kernel<__bf16, 128, true>(hc) : pick_bwd_kernel<__bf16, 128, false>(hc);
        else
            kern = scatter ? pick_bwd_kernel<__bf16, 64, true>(hc) : pick_bwd_kernel<__bf16, 64, false>(hc);
    } else {
        if (sh.d_h == 128)
            kern = scatter ? pick_bwd_kernel<float, 128, true>(hc) : pick_bwd_kernel<float, 128, false>(hc);
        else
            kern = scatter ? pick_bwd_kernel<float, 64, true>(hc) : pick_bwd_kernel<float, 64, false>(hc);
    }
    const bool mfma = !scatter && sh.dtype == GSA_BF16 && G <= 16;  // query-centred pass on the matrix cores
    // bf16 inputs with a workspace: the value gate runs once as a pre-pass (as in the forward of long prefills), both
    // passes then gather gated values
    const void* Vp = V;
    const void* g2p = g2;
    if (mfma && g2) {
        hipError_t e = launch_value_gate(sh, V, g2, ws + p.o_vg, st);
        if (e != hipSuccess) return e;
        Vp = ws + p.o_vg;
        g2p = nullptr;
    }
    if (mfma) {
        QBwdArgs qa;
        qa.Q = Q;
        qa.K = K;
        qa.V = Vp;  // gated values (the pre-pass above, or V itself when the layer has no value gate)
        qa.g1 = g1;
        qa.dout = dout;
        qa.idx = idx;
        qa.n_sel = n_sel;
        qa.dQ = dQ;
        qa.dg1 = dg1;
        qa.p_sum = p_sum;
        qa.dO_ws = static_cast<__bf16*>(a.dO_ws);
        qa.lse_ws = a.lse_ws;
        qa.D_ws = a.D_ws;
        qa.B = sh.B;
        qa.Lq = sh.Lq;
        qa.Lk = sh.Lk;
        qa.H = sh.H;
        qa.H_kv = sh.H_kv;
        qa.k_cap = k_cap;
        qa.scale = scale;
        void (*qk)(QBwdArgs) = sh.d_h == 128 ? attn_bwd_q_mfma_kernel<128> : attn_bwd_q_mfma_kernel<64>;
        const size_t smem = (size_t)4 * 32 * ((sh.d_h * 2 + 32) + (sh.d_h * 2 + 16));
        if (smem > 48 * 1024) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(qk), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
            if (e != hipSuccess) return e;
        }
        hipLaunchKernelGGL(qk, dim3((unsigned)((int64_t)sh.B * sh.Lq), (unsigned)cdiv(sh.H_kv, 4)), dim3(256), smem, st, qa);
    } else {
        hipLaunchKernelGGL(kern, grid, dim3(256), 0, st, a);
    }
    if (!scatter) {
        // inverted lists: counts -> exclusive prefix sum -> fill
        InvArgs ia;
        ia.idx = idx;
        ia.n_sel = n_sel;
        ia.off = reinterpret_cast<int32_t*>(ws + p.o_off);
        ia.cursor = reinterpret_cast<int32_t*>(ws + p.o_cursor);
        ia.inv = reinterpret_cast<int32_t*>(ws + p.o_inv);
        ia.B = sh.B;
        ia.Lq = sh.Lq;
        ia.Lk = sh.Lk;
        ia.k_cap = k_cap;
        ia.wq_shift = p.wq_shift;
        ia.NW = p.NW;
        int32_t* sums = reinterpret_cast<int32_t*>(ws + p.o_sums);
        const int64_t n = p.n_slots + 1;
        const unsigned nblk = (unsigned)cdiv(n, kScanBlock);
        // (int32 and fp32 zeros are the same bits; off and cursor are adjacent 256-byte multiples)
        zero_fill(reinterpret_cast<float*>(ia.off), (int64_t)((p.o_sums - p.o_off) / sizeof(int32_t)), st);
        const unsigned rgrid = (unsigned)cdiv((int64_t)sh.B * sh.Lq, 4);
        hipLaunchKernelGGL(inv_lists_kernel<false>, dim3(rgrid), dim3(256), 0, st, ia);
        hipLaunchKernelGGL(scan_block_sums_kernel, dim3(nblk), dim3(256), 0, st, ia.off, n, sums);
        hipLaunchKernelGGL(scan_of_sums_kernel, dim3(1), dim3(1024), 0, st, sums, (int64_t)nblk);
        hipLaunchKernelGGL(scan_blocks_kernel, dim3(nblk), dim3(256), 0, st, ia.off, n, sums);
        hipLaunchKernelGGL(inv_lists_kernel<true>, dim3(rgrid), dim3(256), 0, st, ia);
        KeyBwdArgs ka;
        ka.Q = Q;
        ka.K = K;
        ka.V = Vp;
        ka.g2 = g2p;
        ka.dO = a.dO_ws;
        ka.lse = a.lse_ws;
        ka.D = a.D_ws;
        ka.off = ia.off;
        ka.inv = ia.inv;
        ka.dK = dK;
        ka.dVp = dV;
        ka.B = sh.B;
        ka.Lq = sh.Lq;
        ka.Lk = sh.Lk;
        ka.H = sh.H;
        ka.H_kv = sh.H_kv;
        ka.NW = p.NW;
        ka.scale = scale;
        void (*kk)(KeyBwdArgs) = sh.dtype == GSA_BF16
                                     ? (sh.d_h == 128 ? attn_bwd_keys_kernel<__bf16, 128> : attn_bwd_keys_kernel<__bf16, 64>)
                                     : (sh.d_h == 128 ? attn_bwd_keys_kernel<float, 128> : attn_bwd_keys_kernel<float, 64>);
        ka.keys = sh.Lk;  // (lists are taken as they are: a list may name any key, visible to its query or not)
        for (int w = 0; w < p.NW; ++w) {
            ka.win = w;
            hipLaunchKernelGGL(kk, dim3((unsigned)cdiv(ka.keys, 4), (unsigned)sh.H_kv, (unsigned)sh.B), dim3(256), 0, st, ka);
        }
    }
    if (sh.dtype == GSA_BF16)
        hipLaunchKernelGGL(value_gate_bwd_kernel<__bf16>, dim3((unsigned)cdiv(kv_elems, 256)), dim3(256), 0, st,
                           static_cast<const __bf16*>(V), static_cast<const __bf16*>(g2), dV, dg2, kv_elems);
    else
        hipLaunchKernelGGL(value_gate_bwd_kernel<float>, dim3((unsigned)cdiv(kv_elems, 256)), dim3(256), 0, st,
                           static_cast<const float*>(V), static_cast<const float*>(g2), dV, dg2, kv_elems);
    return hipGetLastError();
}

// ---- sparse-phase indexer loss and the gradients it sends into the indexer (Sec. 6.1, Sec. 3.3) -----------------
struct IndexerKlArgs {
    const void* qI;        // [B, Lq, HI, dI]
    const void* kI;        // [B, Lk, dI]
    const float* w;        // [B, Lq, HI]
    const float* bI;       // [HI] or null
    const int32_t* idx;    // [B, Lq, k_cap]
    const int32_t* n_sel;  // [B, Lq]
    const float* p;        // [B, Lq, k_cap]: target distribution over the selected keys
    float* loss;           // [B, Lq]
    float* dqI;            // [B, Lq, HI, dI]
    float* dkI;            // [B, Lk, dI], zeroed before the launch
    float* dw;             // [B, Lq, HI]
    float* dbI;            // [HI] or null, zeroed before the launch
    int32_t B, Lq, Lk, HI, dI, k_cap;
};

// One wave per query.  A lane computes the logits z_{j,s} and the score I_s of one selected key (chunks of 64);
// the softmax over S_t takes two passes over the (recomputed) scores; then every lane owns dI / 64 features of
// dq (lanes beyond dI idle) for the sums over keys.  HI <= 8.
template <typename T>
__global__ __launch_bounds__(256) void indexer_kl_kernel(IndexerKlArgs a) {
    extern __shared__ float klds[];  // per wave: the query's heads [HI * dI]
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int64_t row = (int64_t)blockIdx.x * 4 + wv;
    if (row >= (int64_t)a.B * a.Lq) return;  // (the waves of a workgroup never synchronise with each other)
    const int b = (int)(row / a.Lq);
    const int HI = a.HI, DI = a.dI;
    float* qs = klds + wv * (8 * 128);
    const T* qI = static_cast<const T*>(a.qI) + row * HI * DI;
    const T* kI = static_cast<const T*>(a.kI) + (int64_t)b * a.Lk * DI;
    for (int c = lane; c < HI * DI; c += 64) qs[c] = ldf(qI, c);
    __builtin_amdgcn_s_waitcnt(0);
    __builtin_amdgcn_wave_barrier();
    const int nsel = max(0, min(a.n_sel[row], a.k_cap));
    const int32_t* idxrow = a.idx + row * a.k_cap;
    const float* prow = a.p + row * a.k_cap;
    float wj[8], bj[8];
#pragma unroll
    for (int h = 0; h < 8; ++h) {
        wj[h] = h < HI ? a.w[row * HI + h] : 0.f;
        bj[h] = (h < HI && a.bI) ? a.bI[h] : 0.f;
    }
    // sigma(z_{h,s}) of the lane's key for every head; returns the score
    auto score_of = [&](int tok, float (&sg)[8]) {
        const T* kr = kI + (int64_t)tok * DI;
        float z[8];
#pragma unroll
        for (int h = 0; h < 8; ++h) z[h] = 0.f;
        for (int c = 0; c < DI; c += 8) {  // (dI is a multiple of 32: whole 16-byte pieces of the key row)
            float kv[8];
            load8(kr + c, kv);
#pragma unroll
            for (int h = 0; h < 8; ++h)
                if (h < HI) {
                    const float4 q0 = *reinterpret_cast<const float4*>(qs + h * DI + c);
                    const float4 q1 = *reinterpret_cast<const float4*>(qs + h * DI + c + 4);
                    z[h] = fmaf(q0.x, kv[0], z[h]); z[h] = fmaf(q0.y, kv[1], z[h]);
                    z[h] = fmaf(q0.z, kv[2], z[h]); z[h] = fmaf(q0.w, kv[3], z[h]);
                    z[h] = fmaf(q1.x, kv[4], z[h]); z[h] = fmaf(q1.y, kv[5], z[h]);
                    z[h] = fmaf(q1.z, kv[6], z[h]); z[h] = fmaf(q1.w, kv[7], z[h]);
                }
        }
        float sc = 0.f;
#pragma unroll
        for (int h = 0; h < 8; ++h) {
            sg[h] = h < HI ? precise_sigmoid(z[h] + bj[h]) : 0.f;
            sc = fmaf(wj[h], sg[h], sc);
        }
        return sc;
    };
    // ---- softmax statistics of the scores over S_t ----------------------------------------------------------------
    float m = kTrainNegBig, l = 0.f;
    for (int j0 = 0; j0 < nsel; j0 += 64) {
        const int j = j0 + lane;
        const int tok = max(0, min(idxrow[min(j, nsel - 1)], a.Lk - 1));
        float sg[8];
        const float x = j < nsel ? score_of(tok, sg) : kTrainNegBig;
        const float mnew = fmaxf(m, wave_max(x));
        l = l * expf(m - mnew) + wave_sum(j < nsel ? expf(x - mnew) : 0.f);
        m = mnew;
    }
    const float logl = nsel > 0 ? logf(l) : 0.f;
    // ---- loss, dI = softmax(I) - p, and the gradients of Eq. "indexer" -------------------------------------------
    float loss = 0.f;
    float dwacc[8], dbacc[8];
#pragma unroll
    for (int h = 0; h < 8; ++h) dwacc[h] = dbacc[h] = 0.f;
    float dq[8][2];  // features lane and lane + 64 of every head
#pragma unroll
    for (int h = 0; h < 8; ++h) dq[h][0] = dq[h][1] = 0.f;
    for (int j0 = 0; j0 < nsel; j0 += 64) {
        const int j = j0 + lane;
        const int tok = max(0, min(idxrow[min(j, nsel - 1)], a.Lk - 1));
        float dz[8];
#pragma unroll
        for (int h = 0; h < 8; ++h) dz[h] = 0.f;
        if (j < nsel) {
            float sg[8];
            const float x = score_of(tok, sg);
            const float logq = x - m - logl;
            const float p = prow[j];
            if (p > 0.f) loss += p * (logf(p) - logq);
            const float dI = expf(logq) - p;
#pragma unroll
            for (int h = 0; h < 8; ++h) {
                dwacc[h] = fmaf(dI, sg[h], dwacc[h]);
                dz[h] = dI * wj[h] * sg[h] * (1.0f - sg[h]);
                dbacc[h] += dz[h];
            }
        }
        const int cnt = min(64, nsel - j0);
        for (int u = 0; u < cnt; ++u) {
            const int tu = __shfl(tok, u, 64);
            float dzu[8];
#pragma unroll
            for (int h = 0; h < 8; ++h) dzu[h] = h < HI ? __shfl(dz[h], u, 64) : 0.f;
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                const int c = lane + 64 * e;
                if (c < DI) {
                    const float kc = ldf(kI, (int64_t)tu * DI + c);
                    float dk = 0.f;
#pragma unroll
                    for (int h = 0; h < 8; ++h)
                        if (h < HI) {
                            dq[h][e] = fmaf(dzu[h], kc, dq[h][e]);
                            dk = fmaf(dzu[h], qs[h * DI + c], dk);
                        }
                    atomicAdd(&a.dkI[((int64_t)b * a.Lk + tu) * DI + c], dk);
                }
            }
        }
    }
    loss = wave_sum(loss);
    if (lane == 0) a.loss[row] = loss;
#pragma unroll
    for (int h = 0; h < 8; ++h) {
        if (h < HI) {
            const float dw = wave_sum(dwacc[h]);
            const float db = wave_sum(dbacc[h]);
            if (lane == 0) {
                a.dw[row * HI + h] = dw;
                if (a.dbI) atomicAdd(&a.dbI[h], db);
            }
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                const int c = lane + 64 * e;
                if (c < DI) a.dqI[(row * HI + h) * DI + c] = dq[h][e];
            }
        }
    }
}

hipError_t launch_indexer_kl(const gsa_shape& sh, const void* qI, const void* kI, const float* w, const float* bI, const int32_t* idx,
                             const int32_t* n_sel, int k_cap, const float* p, float* loss, float* dqI, float* dkI, float* dw,
                             float* dbI, hipStream_t st) {
    IndexerKlArgs a;
    a.qI = qI;
    a.kI = kI;
    a.w = w;
    a.bI = bI;
    a.idx = idx;
    a.n_sel = n_sel;
    a.p = p;
    a.loss = loss;
    a.dqI = dqI;
    a.dkI = dkI;
    a.dw = dw;
    a.dbI = dbI;
    a.B = sh.B;
    a.Lq = sh.Lq;
    a.Lk = sh.Lk;
    a.HI = sh.HI;
    a.dI = sh.dI;
    a.k_cap = k_cap;
    zero_fill(dkI, (int64_t)sh.B * sh.Lk * sh.dI, st);
    zero_fill(dbI, sh.HI, st);
    const size_t smem = 4 * 8 * 128 * sizeof(float);
    const dim3 grid((unsigned)cdiv((int64_t)sh.B * sh.Lq, 4));
    if (sh.dtype == GSA_BF16)
        hipLaunchKernelGGL(indexer_kl_kernel<__bf16>, grid, dim3(256), smem, st, a);
    else
        hipLaunchKernelGGL(indexer_kl_kernel<float>, grid, dim3(256), smem, st, a);
    return hipGetLastError();
}

}  // namespace gsa
