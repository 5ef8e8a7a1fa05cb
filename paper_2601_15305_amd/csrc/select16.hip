// Top-k_t selection for the fused forward, working on 16-bit keys instead of fp32 scores.
//
// Inside gsa_forward the indexer does not write fp32 scores but the monotone fixed-point key
// q = min(65535, floor(I * 65536 / HI)): half the bytes to write and to read back.  The selection of
// Eq. 4 (Sec. 2.2) on the scores themselves is recovered exactly up to fp32 rounding:
//   1. the n_sel-th largest key T_q and the number `need` of elements with key == T_q that belong to
//      the result are found in one pass over the row for long rows (a strided sample gives a
//      conservative threshold, the words holding a key at or above it are collected in LDS and the exact
//      threshold is found there; a failed estimate falls back to the exact multi-pass radix select, which
//      short rows use directly); every element with key > T_q is selected;
//   2. the elements with key == T_q (typically a handful) are the only ones whose order the keys do
//      not decide: their fp32 scores are recomputed from qI and the gathered kI rows (Eq. "indexer" of
//      Sec. 3.3, fp32 FMA chains, the same sigmoid as the indexer) and the `need` largest are taken,
//      equal scores lowest index first.  If more than kTieCap elements share T_q (saturated scores,
//      constant rows) the exact multi-pass radix select runs over the recomputed scores instead.
// Two recomputed scores can differ from the indexer's own by fp32 rounding only, i.e. only keys within
// about 1e-7 (relative) of a bin edge or of each other can be ordered differently.
#include "select_common.hpp"

namespace gsa {

struct Select16Args {
    const uint16_t* keys;
    int64_t ld;
    const int32_t* n_sel;
    int32_t* idx_out;
    const void* qI;
    const void* kI;
    const float* w;
    const float* bI;
    int32_t B, Lq, Lk, q_offset, row_begin, row_end, k_cap;
    int32_t nw;
    int32_t idx_rows, idx_row0;
    int32_t hi;  // indexer heads in memory; the kernel is built for the next power of two, the extra heads weigh zero
    const int32_t* seq_lens;  // per-sequence lengths (ragged decode) or null
};

constexpr int kKeysPerVec = 8;                                      // one 16-byte load
constexpr int kBatch16 = kSelThreads * kKeysPerVec * kVecPerBatch;  // keys per batch of a workgroup
// One-pass variant for long rows: a strided sample (32 consecutive keys out of every kSamplePeriod) gives a
// conservative threshold; one stream over the row then collects every 32-bit word that holds a key at or
// above it as a record {two keys, word index}, and the exact threshold is found on the records.
constexpr int kSamplePeriod = 256;
constexpr int kBitsS = 12;  // bits of the sample histogram
constexpr int kBinsS = 1 << kBitsS;
constexpr int kRecCap = 5632;            // records the one-pass variant can hold
constexpr int kRegion0_16 = 2 * kRecCap;  // words
static_assert(kRegion0_16 >= kBinsA && kRegion0_16 >= kBinsS && kRegion0_16 >= 2 * kTieCap, "LDS aliasing");

// Two 16-bit saturating differences in one instruction: each half of the result is max(x.half - y.half, 0).
// (Written as an instruction on purpose: with hipcc 7.2 the portable form, __builtin_elementwise_sub_sat on a
// 2 x u16 vector cast from one element of a 4 x u32 vector, used the first element's result for all four.)
__device__ __forceinline__ uint32_t pk_sub_sat_u16(uint32_t x, uint32_t y) {
    uint32_t d;
    asm("v_pk_sub_u16 %0, %1, %2 clamp" : "=v"(d) : "v"(x), "v"(y));
    return d;
}

// Stream the n visible keys of a row through f(index, key), two batches of 16-byte loads in flight.
template <class F>
__device__ __forceinline__ void stream_keys(const uint16_t* __restrict__ row, int n, F&& f) {
    const int tid = threadIdx.x;
    u32x4 cur[kVecPerBatch], nxt[kVecPerBatch];
    auto load = [&](int b0, u32x4* v) {
#pragma unroll
        for (int u = 0; u < kVecPerBatch; ++u) {
            const int base = b0 + (u * kSelThreads + tid) * kKeysPerVec;
            v[u] = base < n ? *reinterpret_cast<const u32x4*>(row + base) : u32x4{0, 0, 0, 0};
        }
    };
    load(0, cur);
    for (int b0 = 0; b0 < n; b0 += kBatch16) {
        const bool more = b0 + kBatch16 < n;
        if (more) load(b0 + kBatch16, nxt);
#pragma unroll
        for (int u = 0; u < kVecPerBatch; ++u) {
            const int base = b0 + (u * kSelThreads + tid) * kKeysPerVec;
#pragma unroll
            for (int e = 0; e < kKeysPerVec; ++e) {
                const uint32_t key = (cur[u][e >> 1] >> ((e & 1) * 16)) & 0xffffu;
                if (base + e < n) f(base + e, key);
            }
        }
        if (more) {
#pragma unroll
            for (int u = 0; u < kVecPerBatch; ++u) cur[u] = nxt[u];
        }
    }
}

// fp32 score of one (query, key) pair: Eq. "indexer" with the query's heads taken from LDS
// (q_lds[j*DI + c], w_lds[j], nb_lds[j] = -log2(e) * bias_j) and the key row read from global memory.
template <typename T, int DI, int HI>
__device__ __forceinline__ float recompute_score(const T* __restrict__ krow, const float* q_lds, const float* w_lds,
                                                 const float* nb_lds) {
    float z[HI];
#pragma unroll
    for (int j = 0; j < HI; ++j) z[j] = 0.f;
    for (int c = 0; c < DI; c += 8) {
        float kv[8];
        if constexpr (sizeof(T) == 2) {
            const u32x4 v = *reinterpret_cast<const u32x4*>(krow + c);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                kv[2 * e] = bf16_bits_to_f32(v[e] & 0xffffu);
                kv[2 * e + 1] = bf16_bits_to_f32(v[e] >> 16);
            }
        } else {
            const float4 v0 = *reinterpret_cast<const float4*>(krow + c);
            const float4 v1 = *reinterpret_cast<const float4*>(krow + c + 4);
            kv[0] = v0.x; kv[1] = v0.y; kv[2] = v0.z; kv[3] = v0.w;
            kv[4] = v1.x; kv[5] = v1.y; kv[6] = v1.z; kv[7] = v1.w;
        }
#pragma unroll
        for (int j = 0; j < HI; ++j)
#pragma unroll
            for (int e = 0; e < 8; ++e) z[j] = fmaf(q_lds[j * DI + c + e], kv[e], z[j]);
    }
    float sc = 0.f;
#pragma unroll
    for (int j = 0; j < HI; ++j) sc = fmaf(w_lds[j], fast_rcp(1.0f + fast_exp2(fmaf(z[j], -kLog2e, nb_lds[j]))), sc);
    return sc;
}

template <typename T, int DI, int HI>
__global__ __launch_bounds__(kSelThreads, 4) void topk_select16_kernel(Select16Args a) {
    extern __shared__ __attribute__((aligned(16))) uint32_t lds[];
    SelLds L;
    L.region0 = lds;
    L.bm_sel = lds + kRegion0_16;
    L.region2 = L.bm_sel + a.nw;
    const int r2 = max(a.nw, kBinsC + kTieCap);
    L.scratch = L.region2 + r2;
    unsigned long long* scan64 = reinterpret_cast<unsigned long long*>(L.scratch + 12);
    float* q_lds = reinterpret_cast<float*>(L.scratch + 32);  // HI*DI query values, then HI weights, HI biases
    float* w_lds = q_lds + HI * DI;
    float* nb_lds = w_lds + HI;
    uint32_t* scratch = L.scratch;

    const int tid = threadIdx.x;
    const int R = a.row_end - a.row_begin;
    const int64_t rid = (int64_t)gridDim.x - 1 - blockIdx.x;  // longest rows of the slab first
    const int b = (int)(rid / R);
    const int t = a.row_begin + (int)(rid % R);
    const int n = min(batch_q_offset(a.seq_lens, b, a.q_offset, a.Lq, a.Lk) + t, a.Lk - 1) + 1;
    int m = a.n_sel[(int64_t)b * a.Lq + t];
    m = max(0, min(m, min(n, a.k_cap)));
    int32_t* out = a.idx_out + ((int64_t)b * a.idx_rows + (t - a.idx_row0)) * a.k_cap;
    if (m == n || m == 0) {
        for (int j = tid; j < a.k_cap; j += kSelThreads) out[j] = j < m ? j : -1;
        return;
    }
    const uint16_t* krow = a.keys + ((int64_t)b * R + (t - a.row_begin)) * a.ld;
    const int nw_row = (n + 31) >> 5;
    uint32_t* bm_sel = L.bm_sel;

    // The query's indexer heads are needed when keys tie at the threshold (nearly every row): request them
    // now, park them in LDS once the first wait for memory is due anyway.
    constexpr int QPT = (HI * DI + kSelThreads - 1) / kSelThreads;
    float qreg[QPT];
    float wreg = 0.f, nbreg = 0.f;
#pragma unroll
    for (int i = 0; i < QPT; ++i) {
        const int c = tid + i * kSelThreads;
        qreg[i] = c < a.hi * DI ? (float)static_cast<const T*>(a.qI)[((int64_t)b * a.Lq + t) * a.hi * DI + c] : 0.f;
    }
    if (tid < a.hi) {
        wreg = a.w[((int64_t)b * a.Lq + t) * a.hi + tid];
        nbreg = a.bI ? -kLog2e * a.bI[tid] : 0.f;
    }
    auto park_query = [&]() {
#pragma unroll
        for (int i = 0; i < QPT; ++i) {
            const int c = tid + i * kSelThreads;
            if (c < HI * DI) q_lds[c] = qreg[i];
        }
        if (tid < HI) {
            w_lds[tid] = wreg;
            nb_lds[tid] = nbreg;
        }
    };

    // ---- 1. threshold key T_q, `need`, and the list (or bitmap) of elements with key == T_q ---------
    uint32_t Tq = 0, need = 0, ne = 0;
    uint32_t* tie_list = nullptr;  // indices of the elements with key == T_q when ne <= kTieCap
    float* tie_score = nullptr;
    bool have = false;
    if (n >= 8192 && n >= 4 * m) {
        uint32_t* hist = L.region0;                         // kBinsS words
        uint2* rec = reinterpret_cast<uint2*>(L.region0);   // kRecCap records {two keys, word index}, after hist
        uint32_t* hist_c = L.region2;
        // -- sample: 32 consecutive keys out of every kSamplePeriod (a quad of lanes per period)
        u32x4 sv[4];
        int sbase[4];
        auto sample_load = [&](int q0) {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int q = q0 + u * kSelThreads;
                sbase[u] = (q >> 2) * kSamplePeriod + (q & 3) * 8;
                sv[u] = sbase[u] < n ? *reinterpret_cast<const u32x4*>(krow + sbase[u]) : u32x4{0, 0, 0, 0};
            }
        };
        auto sample_count = [&]() {
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    if (sbase[u] + e < n)
                        atomicAdd(&hist[((sv[u][e >> 1] >> ((e & 1) * 16)) & 0xffffu) >> (16 - kBitsS)], 1u);
        };
        sample_load(tid);  // in flight while the histogram is cleared
        for (int i = tid; i < kBinsS; i += kSelThreads) hist[i] = 0;
        park_query();
        __syncthreads();
        sample_count();
        for (int q0 = tid + 4 * kSelThreads; (q0 >> 2) * kSamplePeriod < n; q0 += 4 * kSelThreads) {
            sample_load(q0);
            sample_count();
        }
        __syncthreads();
        const int ms = (n / kSamplePeriod) * 32 + min(32, n % kSamplePeriod);
        const float lam = (float)m * (float)ms / (float)n;
        const int r = (int)ceilf(lam + 3.5f * sqrtf(lam) + 2.0f);
        if (r <= ms) {
            // -- the stream: two batches of 16-byte loads in flight, the first one already during the search
            u32x4 cur[kVecPerBatch], nxt[kVecPerBatch];
            auto load = [&](int b0, u32x4* v) {
#pragma unroll
                for (int u = 0; u < kVecPerBatch; ++u) {
                    const int base = b0 + (u * kSelThreads + tid) * kKeysPerVec;
                    v[u] = base < n ? *reinterpret_cast<const u32x4*>(krow + base) : u32x4{0, 0, 0, 0};
                }
            };
            load(0, cur);
            int b_lo;
            uint32_t above;
            find_threshold_bin(hist, kBinsS, (uint32_t)r, scratch, &b_lo, &above);
            const uint32_t thr = (uint32_t)b_lo << (16 - kBitsS);  // every key >= thr is a candidate
            for (int i = tid; i < nw_row; i += kSelThreads) bm_sel[i] = 0;
            if (tid == 0) {
                scratch[kSelWaves + 2] = 0;
                scratch[kSelWaves + 3] = 0;
            }
            __syncthreads();
            uint32_t nrec = 0;
            if (thr > 0) {
                // key >= thr  <=>  the saturating 16-bit difference key - (thr - 1) is not zero
                const uint32_t thr2 = (thr - 1) * 0x00010001u;
                for (int b0 = 0; b0 < n; b0 += kBatch16) {
                    const bool more = b0 + kBatch16 < n;
                    if (more) {
                        load(b0 + kBatch16, nxt);
                    } else {  // last batch: keys beyond the visible range count as zero
#pragma unroll
                        for (int u = 0; u < kVecPerBatch; ++u)
#pragma unroll
                            for (int i = 0; i < 4; ++i) {
                                const int k0 = b0 + (u * kSelThreads + tid) * kKeysPerVec + 2 * i;
                                if (k0 + 1 >= n) cur[u][i] = k0 >= n ? 0u : (cur[u][i] & 0xffffu);
                            }
                    }
                    uint32_t d[kVecPerBatch][4];
                    uint32_t cnt = 0;
#pragma unroll
                    for (int u = 0; u < kVecPerBatch; ++u)
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            d[u][i] = pk_sub_sat_u16(cur[u][i], thr2);
                            cnt += d[u][i] != 0u ? 1u : 0u;
                        }
                    // one reservation per lane and batch; the words with a candidate follow it
                    uint32_t pos = cnt ? atomicAdd(&scratch[kSelWaves + 2], cnt) : 0u;
#pragma unroll
                    for (int u = 0; u < kVecPerBatch; ++u)
#pragma unroll
                        for (int i = 0; i < 4; ++i)
                            if (d[u][i] != 0u) {
                                if (pos < (uint32_t)kRecCap)
                                    rec[pos] = uint2{cur[u][i], (uint32_t)(((b0 + (u * kSelThreads + tid) * kKeysPerVec) >> 1) + i)};
                                ++pos;
                            }
                    if (more) {
#pragma unroll
                        for (int u = 0; u < kVecPerBatch; ++u) cur[u] = nxt[u];
                    }
                }
                __syncthreads();
                nrec = scratch[kSelWaves + 2];
            }
            if (nrec > 0 && nrec <= (uint32_t)kRecCap && 2 * nrec >= (uint32_t)m) {
                // -- exact threshold on the records.  A record may carry one key below thr; such keys are below
                // the m-th largest as long as that one turns out >= thr, which is checked afterwards.
                uint32_t prefix = 0;
                need = (uint32_t)m;
                int rb = 16;
                while (rb > 0) {  // 11 + 5 bits
                    const int nb = min(kBitsC, rb);
                    const uint32_t mask = (1u << nb) - 1u;
                    for (int i = tid; i < (1 << nb); i += kSelThreads) hist_c[i] = 0;
                    __syncthreads();
                    for (uint32_t c = tid; c < nrec; c += kSelThreads) {
                        const uint32_t kk = rec[c].x;
                        const uint32_t k0 = kk & 0xffffu, k1 = kk >> 16;
                        if ((k0 >> rb) == prefix) atomicAdd(&hist_c[(k0 >> (rb - nb)) & mask], 1u);
                        if ((k1 >> rb) == prefix) atomicAdd(&hist_c[(k1 >> (rb - nb)) & mask], 1u);
                    }
                    __syncthreads();
                    int bin;
                    find_threshold_bin(hist_c, 1 << nb, need, scratch, &bin, &above);
                    need -= above;
                    prefix = (prefix << nb) | (uint32_t)bin;
                    rb -= nb;
                }
                if (prefix >= thr) {
                    Tq = prefix;
                    tie_list = L.region2 + kBinsC;
                    tie_score = reinterpret_cast<float*>(L.region2);
                    for (uint32_t c = tid; c < nrec; c += kSelThreads) {
                        const uint2 rc = rec[c];
#pragma unroll
                        for (int hf = 0; hf < 2; ++hf) {
                            const uint32_t key = hf ? rc.x >> 16 : rc.x & 0xffffu;
                            const uint32_t si = 2 * rc.y + hf;
                            if (key > Tq) {
                                atomicOr(&bm_sel[si >> 5], 1u << (si & 31));
                            } else if (key == Tq) {
                                const uint32_t pos = atomicAdd(&scratch[kSelWaves + 3], 1u);
                                if (pos < (uint32_t)kTieCap) tie_list[pos] = si;
                            }
                        }
                    }
                    __syncthreads();
                    ne = scratch[kSelWaves + 3];
                    have = ne <= (uint32_t)kTieCap;  // otherwise the list is incomplete: take the exact path below
                }
            }
        }
        __syncthreads();
    } else {
        park_query();
    }
    if (!have) {
        // exact two-pass selection on the keys themselves (as floats: 0..65535 are exact and ordered)
        uint32_t thr_bits = 0;
        select_exact([&](auto&& f) { stream_keys(krow, n, [&](int si, uint32_t key) { f(si, (float)key); }); }, n, m, L,
                     &need, false, &thr_bits);
        Tq = (uint32_t)__uint_as_float(thr_bits);
        // elements with key == T_q are the bits of the tie bitmap; count them
        uint32_t* bm_tie = L.region2;
        if (tid == 0) scratch[kSelWaves + 3] = 0;
        __syncthreads();
        uint32_t cnt = 0;
        for (int i = tid; i < nw_row; i += kSelThreads) cnt += __popc(bm_tie[i]);
        if (cnt) atomicAdd(&scratch[kSelWaves + 3], cnt);
        __syncthreads();
        ne = scratch[kSelWaves + 3];
        tie_list = L.region0;
        tie_score = reinterpret_cast<float*>(L.region0 + kTieCap);
        if (need < ne && ne <= (uint32_t)kTieCap) {  // list them (order irrelevant)
            if (tid == 0) scratch[kSelWaves + 2] = 0;
            __syncthreads();
            for (int i = tid; i < nw_row; i += kSelThreads) {
                uint32_t wbits = bm_tie[i];
                while (wbits) {
                    const int bit = __ffs(wbits) - 1;
                    tie_list[atomicAdd(&scratch[kSelWaves + 2], 1u)] = (uint32_t)(i * 32 + bit);
                    wbits &= wbits - 1u;
                }
            }
            __syncthreads();
        } else if (need == ne) {  // every one of them is taken
            for (int i = tid; i < nw_row; i += kSelThreads) bm_sel[i] |= bm_tie[i];
            __syncthreads();
        }
    }

    // ---- 2. order the elements with key == T_q by their recomputed fp32 scores ------------------------
    uint32_t m_eq = 0;
    bool with_ties = false;
    if (need < ne) {
        const T* kbase = static_cast<const T*>(a.kI) + (int64_t)b * a.Lk * DI;
        if (ne <= (uint32_t)kTieCap) {
            // DI/8 lanes per element, eight channels each: one round trip to memory per pass
            constexpr int LPT = DI / 8;
            const int g = tid % LPT;
            for (uint32_t i0 = 0; i0 < ne; i0 += kSelThreads / LPT) {
                const uint32_t i = i0 + tid / LPT;
                float z[HI];
#pragma unroll
                for (int j = 0; j < HI; ++j) z[j] = 0.f;
                if (i < ne) {
                    const T* kr = kbase + (int64_t)tie_list[i] * DI + 8 * g;
                    float kv[8];
                    if constexpr (sizeof(T) == 2) {
                        const u32x4 v = *reinterpret_cast<const u32x4*>(kr);
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            kv[2 * e] = bf16_bits_to_f32(v[e] & 0xffffu);
                            kv[2 * e + 1] = bf16_bits_to_f32(v[e] >> 16);
                        }
                    } else {
                        const float4 v0 = *reinterpret_cast<const float4*>(kr);
                        const float4 v1 = *reinterpret_cast<const float4*>(kr + 4);
                        kv[0] = v0.x; kv[1] = v0.y; kv[2] = v0.z; kv[3] = v0.w;
                        kv[4] = v1.x; kv[5] = v1.y; kv[6] = v1.z; kv[7] = v1.w;
                    }
#pragma unroll
                    for (int j = 0; j < HI; ++j)
#pragma unroll
                        for (int e = 0; e < 8; ++e) z[j] = fmaf(q_lds[j * DI + 8 * g + e], kv[e], z[j]);
                }
#pragma unroll
                for (int j = 0; j < HI; ++j)
#pragma unroll
                    for (int o = 1; o < LPT; o <<= 1) z[j] += __shfl_xor(z[j], o, 64);
                if (i < ne && g == 0) {
                    float sc = 0.f;
#pragma unroll
                    for (int j = 0; j < HI; ++j)
                        sc = fmaf(w_lds[j], fast_rcp(1.0f + fast_exp2(fmaf(z[j], -kLog2e, nb_lds[j]))), sc);
                    tie_score[i] = sc;
                }
            }
            __syncthreads();
            for (uint32_t i = tid; i < ne; i += kSelThreads) {
                const float si = tie_score[i];
                const uint32_t xi = tie_list[i];
                uint32_t rank = 0;
                for (uint32_t j = 0; j < ne; ++j) {
                    const float sj = tie_score[j];
                    rank += (sj > si || (sj == si && tie_list[j] < xi)) ? 1u : 0u;
                }
                if (rank < need) atomicOr(&bm_sel[xi >> 5], 1u << (xi & 31));
            }
            __syncthreads();
        } else {
            // too many to list: exact radix select over the recomputed scores of exactly those elements
            select_exact(
                [&](auto&& f) {
                    stream_keys(krow, n, [&](int si, uint32_t key) {
                        if (key == Tq) f(si, recompute_score<T, DI, HI>(kbase + (int64_t)si * DI, q_lds, w_lds, nb_lds));
                    });
                },
                n, (int)need, L, &m_eq, true);
            with_ties = true;
        }
    } else if (have) {  // sampled path, all elements with key == T_q are taken
        for (uint32_t i = tid; i < ne; i += kSelThreads) {
            const uint32_t xi = tie_list[i];
            atomicOr(&bm_sel[xi >> 5], 1u << (xi & 31));
        }
        __syncthreads();
    }
    emit_selection(out, a.k_cap, m, n, bm_sel, with_ties ? L.region2 : nullptr, m_eq, scan64);
}

static int kernel_heads16(int hi) { return hi <= 1 ? 1 : (hi <= 2 ? 2 : (hi <= 4 ? 4 : 8)); }

size_t select16_lds_bytes(const gsa_shape& sh) {
    const int nw = ((sh.Lk + 31) / 32 + 3) & ~3;  // bitmap words, rounded so that what follows stays 16-byte aligned
    const int r2 = nw > kBinsC + kTieCap ? nw : kBinsC + kTieCap;
    const int HIK = kernel_heads16(sh.HI);
    return (size_t)(kRegion0_16 + nw + r2 + 32 + HIK * sh.dI + 2 * HIK) * sizeof(uint32_t);
}

template <typename T, int DI, int HI>
static hipError_t launch16_one(const Select16Args& a, size_t smem, int64_t rows, hipStream_t st) {
    auto kern = topk_select16_kernel<T, DI, HI>;
    if (smem > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)rows), dim3(kSelThreads), smem, st, a);
    return hipGetLastError();
}
template <typename T, int DI>
static hipError_t launch16_hi(const Select16Args& a, int HI, size_t smem, int64_t rows, hipStream_t st) {
    switch (HI) {
        case 1: return launch16_one<T, DI, 1>(a, smem, rows, st);
        case 2: return launch16_one<T, DI, 2>(a, smem, rows, st);
        case 4: return launch16_one<T, DI, 4>(a, smem, rows, st);
        case 8: return launch16_one<T, DI, 8>(a, smem, rows, st);
    }
    return hipErrorInvalidValue;
}
template <typename T>
static hipError_t launch16_di(const Select16Args& a, int DI, int HI, size_t smem, int64_t rows, hipStream_t st) {
    switch (DI) {
        case 32: return launch16_hi<T, 32>(a, HI, smem, rows, st);
        case 64: return launch16_hi<T, 64>(a, HI, smem, rows, st);
        case 128: return launch16_hi<T, 128>(a, HI, smem, rows, st);
    }
    return hipErrorInvalidValue;
}

hipError_t launch_select16(const gsa_shape& sh, int row_begin, int row_end, const uint16_t* keys, int64_t ld,
                           const int32_t* n_sel, int k_cap, int32_t* idx_out, int idx_rows, int idx_row0, const void* qI,
                           const void* kI, const float* w, const float* bI, const int32_t* seq_lens, hipStream_t st) {
    Select16Args a;
    a.seq_lens = seq_lens;
    a.keys = keys;
    a.ld = ld;
    a.n_sel = n_sel;
    a.idx_out = idx_out;
    a.qI = qI;
    a.kI = kI;
    a.w = w;
    a.bI = bI;
    a.B = sh.B;
    a.Lq = sh.Lq;
    a.Lk = sh.Lk;
    a.q_offset = sh.q_offset;
    a.row_begin = row_begin;
    a.row_end = row_end;
    a.k_cap = k_cap;
    a.nw = ((sh.Lk + 31) / 32 + 3) & ~3;
    a.idx_rows = idx_rows;
    a.idx_row0 = idx_row0;
    a.hi = sh.HI;
    const size_t smem = select16_lds_bytes(sh);
    const int64_t rows = (int64_t)sh.B * (row_end - row_begin);
    const int HIK = kernel_heads16(sh.HI);
    return sh.dtype == GSA_BF16 ? launch16_di<__bf16>(a, sh.dI, HIK, smem, rows, st)
                                : launch16_di<float>(a, sh.dI, HIK, smem, rows, st);
}

}  // namespace gsa
