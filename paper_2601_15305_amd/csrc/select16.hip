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
#include <algorithm>

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
    int32_t cap;         // wave-per-row kernel: records a row can hold in LDS
    int32_t m_lo, m_hi;  // wave-per-row kernel: this launch takes the rows with m_lo < budget <= m_hi
    int32_t group;       // workgroup-per-row kernel: rows a workgroup looks at; 0: one row, taken unconditionally
    PageMap pm;          // where the rows of kI live (contiguous tensor or pages of a pool)
};

// First entry of an output row that the wave-per-row kernel could not finish (never a valid index, and not the
// -1 of an unused entry): the workgroup-per-row code, launched afterwards, takes exactly these rows.
constexpr int32_t kRowDeferred = -2;

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

// One row by one workgroup of kSelThreads threads: exact for every input.
template <typename T, int DI, int HI>
__device__ __forceinline__ void select16_row(const Select16Args& a, int64_t rid, uint32_t* lds) {
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
        const T* kpool = static_cast<const T*>(a.kI);  // rows found through cache_row (contiguous or paged)
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
                    const T* kr = kpool + cache_row(a.pm, b, (int)tie_list[i], a.Lk) * DI + 8 * g;
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
                        if (key == Tq) f(si, recompute_score<T, DI, HI>(kpool + cache_row(a.pm, b, si, a.Lk) * DI, q_lds, w_lds, nb_lds));
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

// The rows the wave-per-row kernel left marked (kRowDeferred in the first entry of their output row): every
// workgroup looks at a.group (at most kDeferGroup) consecutive rows and takes the marked ones, one after the
// other.  With a.group = 0 a workgroup takes one row unconditionally (few rows: a workgroup per row from the start).
constexpr int kDeferGroup = 16;
template <typename T, int DI, int HI>
__global__ __launch_bounds__(kSelThreads, 4) void topk_select16_deferred_kernel(Select16Args a) {
    extern __shared__ __attribute__((aligned(16))) uint32_t lds[];
    const int R = a.row_end - a.row_begin;
    const int64_t rows = (int64_t)a.B * R;
    if (a.group == 0) {
        select16_row<T, DI, HI>(a, rows - 1 - (int64_t)blockIdx.x, lds);  // longest rows first
        return;
    }
    const int64_t r0 = (int64_t)blockIdx.x * a.group;
    uint32_t marked = 0;  // the same in every thread
#pragma unroll
    for (int i = 0; i < kDeferGroup; ++i) {
        const int64_t rid = r0 + i;
        if (i < a.group && rid < rows) {
            const int b = (int)(rid / R);
            const int t = a.row_begin + (int)(rid % R);
            marked |= a.idx_out[((int64_t)b * a.idx_rows + (t - a.idx_row0)) * a.k_cap] == kRowDeferred ? (1u << i) : 0u;
        }
    }
    while (marked) {
        const int i = __ffs(marked) - 1;
        marked &= marked - 1u;
        select16_row<T, DI, HI>(a, r0 + i, lds);
        __syncthreads();  // LDS is reused by the next row
    }
}

// ------------------------------------------------------------------------------------------------------------
// Wave-per-row form of the same selection: one 64-lane workgroup per query row and no barriers between waves,
// so that several rows per compute unit are in flight and the latency-bound steps of one row overlap the
// streaming of the others.  Steps (all wave-synchronous):
//   1. a strided sample of at most 8192 keys (quads of lanes read 32 consecutive keys out of every P; the whole
//      row when it has at most 8192 keys) is counted into a 4096-bin histogram of the top 12 key bits (16-bit
//      counters, two per LDS word); the bin holding the r-th largest sample key, r a 3-sigma upper estimate of
//      the rank the m-th largest key of the row has in the sample, gives a conservative threshold thr;
//   2. one stream over the row.  Stage A, per 16-byte vector: lanes whose vector holds a key >= thr push the
//      vector and its first index into a ring in LDS, behind those of the lower lanes (ballot prefix).  Stage B,
//      whenever 64 vectors wait: one lane per vector expands it into 32-bit records
//      {min(key - thr + 1, 8191) << 19 | index}, placed after the records of the lower lanes.  The wave walks
//      the row in order, so the record list is sorted by index;
//   3. the exact threshold among the records: a 2048-bin histogram of the top 11 bits of the 13-bit relative
//      key, then the last two bits; keys above it are taken, keys equal to it are ordered by their recomputed
//      fp32 scores (as in the workgroup-per-row kernel) when only some of them fit;
//   4. the taken records are written out in list order, which is ascending index order: no bitmap, no sort.
// A row the estimate fails on (too many or too few candidates, thr = 0, a threshold inside the saturated
// relative keys, more than kWaveTieCap keys at the threshold) is marked kRowDeferred and left to the
// workgroup-per-row kernel, which is exact for every input.
constexpr int kWaveSampleVec = 16;   // 16-byte vectors of the sample a lane holds: 8192 sampled keys at most
constexpr int kWaveSampleKeys = 64 * kWaveSampleVec * kKeysPerVec;
constexpr int kWaveStreamVec = 16;   // 16-byte vectors per lane in one batch of the stream (two batches in flight)
constexpr int kWaveBatch = 64 * kWaveStreamVec * kKeysPerVec;
constexpr int kWaveQueue = 128;      // ring of vectors waiting for stage B (a power of two, at least 2 * 64)
constexpr uint32_t kRelMax = 8191;   // relative keys saturate here (13 bits); index field: 19 bits
constexpr int kWaveTieCap = 256;
constexpr int kWaveHistWords = 1024; // the record histogram: 2048 bins of 16 bits; during the stream, the ring
static_assert(GSA_SELECT_MAX_LK <= (1 << 19), "record index field");
static_assert(kWaveQueue * 5 <= kWaveHistWords, "the ring lives where the record histogram will be");

__device__ __forceinline__ uint32_t pk_min_u16(uint32_t x, uint32_t y) {
    uint32_t d;
    asm("v_pk_min_u16 %0, %1, %2" : "=v"(d) : "v"(x), "v"(y));
    return d;
}
__device__ __forceinline__ uint32_t pk_max_u16(uint32_t x, uint32_t y) {
    uint32_t d;
    asm("v_pk_max_u16 %0, %1, %2" : "=v"(d) : "v"(x), "v"(y));
    return d;
}
// number of set bits of a wave mask in the lanes below this one
__device__ __forceinline__ uint32_t lanes_below(unsigned long long mask) {
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}
// inclusive sum over this lane and all higher lanes
__device__ __forceinline__ uint32_t wave_suffix_sum(uint32_t x, int lane) {
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t v = __shfl_down(x, o, 64);
        if (lane + o < 64) x += v;
    }
    return x;
}
// Exclusive prefix sum over the lanes of a small per-lane count (< 2^BITS), and the wave total, from ballots of
// the count's bit planes (planes nobody has set cost one branch).
template <int BITS>
__device__ __forceinline__ uint32_t wave_prefix_small(uint32_t cnt, uint32_t* total_out) {
    uint32_t below = 0, total = 0;
#pragma unroll
    for (int bit = 0; bit < BITS; ++bit) {
        const unsigned long long plane = __ballot((cnt >> bit) & 1u);
        if (plane != 0ull) {
            below += lanes_below(plane) << bit;
            total += (uint32_t)__popcll(plane) << bit;
        }
    }
    *total_out = total;
    return below;
}

// Wave-wide search in a histogram of NBINS 16-bit counters (two per word, bin b in half b & 1 of word b >> 1):
// the largest bin b with sum_{b' >= b} count[b'] >= need, and above = sum_{b' > b} count[b'].  Returns -1 when
// the histogram holds fewer than `need` elements.  The same result in every lane.
template <int NBINS>
__device__ __forceinline__ int wave_find_bin(const uint32_t* hist, uint32_t need, int lane, uint32_t* above_out) {
    constexpr int BPL = NBINS / 64;  // bins per lane
    constexpr int WPL = BPL / 2;     // words per lane
    uint32_t own = 0;
#pragma unroll
    for (int i = 0; i < WPL / 4; ++i) {
        const u32x4 v = *reinterpret_cast<const u32x4*>(hist + lane * WPL + 4 * i);
#pragma unroll
        for (int e = 0; e < 4; ++e) own = __builtin_amdgcn_sad_u16(v[e], 0u, own);
    }
    const uint32_t suf = wave_suffix_sum(own, lane);  // decreasing with the lane
    const unsigned long long ok = __ballot(suf >= need);
    if (ok == 0ull) return -1;
    const int owner = 63 - __clzll(ok);
    const uint32_t above_owner = __shfl(suf - own, owner, 64);
    uint32_t c = 0;
    if (lane < BPL) {
        const int bin = owner * BPL + lane;
        c = (hist[bin >> 1] >> ((bin & 1) * 16)) & 0xffffu;
    }
    const uint32_t suf2 = wave_suffix_sum(c, lane) + above_owner;
    const unsigned long long ok2 = __ballot(lane < BPL && suf2 >= need);
    const int j = 63 - __clzll(ok2);  // ok2 != 0: the owner's first bin reaches suf >= need
    *above_out = __shfl(suf2 - c, j, 64);
    return owner * BPL + j;
}

template <typename T, int DI, int HI>
__global__ __launch_bounds__(64) void topk_select16_wave_kernel(Select16Args a) {
    extern __shared__ __attribute__((aligned(16))) uint32_t lds[];
    uint32_t* rec = lds;            // a.cap records; before the stream, the sample histogram (2048 words)
    uint32_t* aux = lds + a.cap;    // the ring, then the record histogram, then the query, tie list and tie scores
    const int aux_words = max(kWaveHistWords, HI * DI + 2 * HI + 2 * kWaveTieCap);
    uint32_t* sub = aux + aux_words;  // 8 words: counters of the last two key bits

    const int lane = threadIdx.x;
    const int R = a.row_end - a.row_begin;
    const int64_t rid = (int64_t)gridDim.x - 1 - blockIdx.x;  // longest rows of the slab first
    const int b = (int)(rid / R);
    const int t = a.row_begin + (int)(rid % R);
    const int n = min(batch_q_offset(a.seq_lens, b, a.q_offset, a.Lq, a.Lk) + t, a.Lk - 1) + 1;
    const uint16_t* krow = a.keys + ((int64_t)b * R + (t - a.row_begin)) * a.ld;
    int m = a.n_sel[(int64_t)b * a.Lq + t];
    m = max(0, min(m, min(n, a.k_cap)));
    if (m <= a.m_lo || m > a.m_hi) return;  // a row of the other launch
    int32_t* out = a.idx_out + ((int64_t)b * a.idx_rows + (t - a.idx_row0)) * a.k_cap;
    if (m == n || m == 0) {
        for (int j = lane; j < a.k_cap; j += 64) out[j] = j < m ? j : -1;
        return;
    }
    // The sample (step 1) and the first batch of the stream (step 2) are requested right away: their addresses
    // depend on the row alone.
    const int P = 32 * ((n + kWaveSampleKeys - 1) / kWaveSampleKeys);  // keys from one sampled quad to the next
    const int ms = (n / P) * 32 + min(32, n % P);                      // sampled keys
    const int sb0 = (lane >> 2) * P + (lane & 3) * 8;                  // (rows are padded to a multiple of 8 keys)
    u32x4 sv[kWaveSampleVec];
#pragma unroll
    for (int u = 0; u < kWaveSampleVec; ++u) {
        const int sb = sb0 + u * 16 * P;
        sv[u] = sb < n ? *reinterpret_cast<const u32x4*>(krow + sb) : u32x4{0, 0, 0, 0};
    }
    // Loads of a batch of the stream; a vector beyond the row reads the row's last vector instead (and is never
    // looked at).  One batch is in flight while the other is worked on.
    const int last_vec = ((n - 1) / kKeysPerVec) * kKeysPerVec;
    auto load = [&](int b0, u32x4* v) {
#pragma unroll
        for (int u = 0; u < kWaveStreamVec; ++u) {
            const int base = min(b0 + (u * 64 + lane) * kKeysPerVec, last_vec);
            v[u] = *reinterpret_cast<const u32x4*>(krow + base);
        }
    };
    u32x4 bufA[kWaveStreamVec], bufB[kWaveStreamVec];
    load(0, bufA);  // on its way while the sample is counted
    const uint32_t cap = (uint32_t)a.cap;
    auto defer = [&]() {
        if (lane == 0) out[0] = kRowDeferred;
    };

    // The query's indexer heads, needed when keys tie at the threshold (most rows): requested now, parked in LDS
    // only if that happens.
    constexpr int QPL = (HI * DI + 63) / 64;
    float qreg[QPL];
    float wreg = 0.f, nbreg = 0.f;
#pragma unroll
    for (int i = 0; i < QPL; ++i) {
        const int c = lane + i * 64;
        qreg[i] = c < a.hi * DI ? (float)static_cast<const T*>(a.qI)[((int64_t)b * a.Lq + t) * a.hi * DI + c] : 0.f;
    }
    if (lane < a.hi) {
        wreg = a.w[((int64_t)b * a.Lq + t) * a.hi + lane];
        nbreg = a.bI ? -kLog2e * a.bI[lane] : 0.f;
    }

    // ---- 1 + 2. threshold from a sample, then the stream --------------------------------------------------------------
    for (int j = m + lane; j < a.k_cap; j += 64) out[j] = -1;          // the unused tail of the output row
    uint32_t thr2 = 0;                        // (thr - 1) in both halves
    u32x4* qv = reinterpret_cast<u32x4*>(aux);  // ring: the waiting vectors ...
    uint32_t* qk = aux + 4 * kWaveQueue;        // ... and the index of their first key
    uint32_t nrec = 0, qhead = 0, qtail = 0;    // wave-uniform

    // Stage B: the first `count` vectors of the ring, one lane each.
    auto expand = [&](uint32_t count) {
        __syncthreads();  // the ring entries written by other lanes
        u32x4 v = u32x4{0, 0, 0, 0};
        uint32_t kb = 0;
        if ((uint32_t)lane < count) {
            const uint32_t slot = (qhead + (uint32_t)lane) & (kWaveQueue - 1);
            v = qv[slot];
            kb = qk[slot];
        }
        uint32_t d[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) d[i] = pk_sub_sat_u16(v[i], thr2);
        // bit 2i of mm: the low key of word i is a candidate; bit 16 + 2i: its high key
        const uint32_t mm = pk_min_u16(d[0], 0x00010001u) | (pk_min_u16(d[1], 0x00010001u) << 2) |
                            (pk_min_u16(d[2], 0x00010001u) << 4) | (pk_min_u16(d[3], 0x00010001u) << 6);
        uint32_t mask8 = (mm | (mm >> 15)) & 0xffu;  // bit e: key kb + e is a candidate
        uint32_t total;
        uint32_t pos = nrec + wave_prefix_small<4>(__popc(mask8), &total);
        while (__ballot(mask8 != 0u) != 0ull) {
            if (mask8 != 0u) {
                const uint32_t e = (uint32_t)__ffs(mask8) - 1u;
                const uint32_t dw = (e & 4u) ? ((e & 2u) ? d[3] : d[2]) : ((e & 2u) ? d[1] : d[0]);
                const uint32_t rel = min((dw >> ((e & 1u) * 16)) & 0xffffu, kRelMax);
                if (pos < cap) rec[pos] = (rel << 19) | (kb + e);
                ++pos;
                mask8 &= mask8 - 1u;
            }
        }
        nrec += total;
        qhead += count;
    };
    // Stage A over one batch held in registers.
    auto consume = [&](const u32x4* buf, int b0) {
#pragma unroll
        for (int u = 0; u < kWaveStreamVec; ++u) {
            const int w0 = b0 + u * 64 * kKeysPerVec;  // first key of this wave-wide vector
            if (w0 >= n) break;
            const int kb = w0 + lane * kKeysPerVec;
            u32x4 v = buf[u];
            if (w0 + 64 * kKeysPerVec > n) {  // the vector holding the end of the row: keys beyond it count as zero
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int k0 = kb + 2 * i;
                    if (k0 + 1 >= n) v[i] = k0 >= n ? 0u : (v[i] & 0xffffu);
                }
            }
            const uint32_t mx = pk_max_u16(pk_max_u16(v[0], v[1]), pk_max_u16(v[2], v[3]));
            const bool hit = pk_sub_sat_u16(mx, thr2) != 0u;
            const unsigned long long H = __ballot(hit);
            if (H == 0ull) continue;
            if (hit) {
                const uint32_t slot = (qtail + lanes_below(H)) & (kWaveQueue - 1);
                qv[slot] = v;
                qk[slot] = (uint32_t)kb;
            }
            qtail += (uint32_t)__popcll(H);
            if (qtail - qhead >= 64u) expand(64u);  // at most 127 entries were waiting: the ring never overflows
        }
    };
    float rank = (float)m;  // rank in the sample whose key becomes the threshold
    if (P > 32) {
        const float lam = (float)m * (float)ms / (float)n;
        rank = ceilf(lam + 3.0f * sqrtf(lam) + 2.0f);
    }
    {
        // -- sample histogram
        {
#pragma unroll
            for (int i = 0; i < 8; ++i) reinterpret_cast<u32x4*>(rec)[i * 64 + lane] = u32x4{0, 0, 0, 0};  // 2048 words
            __syncthreads();
#pragma unroll
            for (int u = 0; u < kWaveSampleVec; ++u) {
                const int sb = sb0 + u * 16 * P;
                if (sb < n) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const uint32_t key = (sv[u][e >> 1] >> ((e & 1) * 16)) & 0xffffu;
                        const uint32_t one = (key & 16u) ? 0x10000u : 1u;
                        atomicAdd(&rec[key >> 5], sb + e < n ? one : 0u);
                    }
                }
            }
            __syncthreads();
        }
        if (kWaveBatch < n) load(kWaveBatch, bufB);  // the second batch, while the threshold is looked up
        // -- conservative threshold: the bin of the sample key with that rank
        uint32_t above;
        const uint32_t r = (uint32_t)fminf(fmaxf(rank, 1.0f), 1.0e9f);
        const int b_lo = r <= (uint32_t)ms ? wave_find_bin<4096>(rec, r, lane, &above) : -1;
        if (b_lo <= 0) {  // thr = 0 would make every key a candidate
            defer();
            return;
        }
        thr2 = (((uint32_t)b_lo << 4) - 1u) * 0x00010001u;
        __syncthreads();  // the histogram has been read; the records take its place

        // -- stream: the records of all keys >= thr, in index order
        // (key >= thr  <=>  the saturating 16-bit difference key - (thr - 1) is not zero; it is the relative key)
        nrec = qhead = qtail = 0;
        for (int b0 = 0; b0 < n; b0 += 2 * kWaveBatch) {
            consume(bufA, b0);
            if (b0 + kWaveBatch >= n) break;
            if (b0 + 2 * kWaveBatch < n) load(b0 + 2 * kWaveBatch, bufA);
            consume(bufB, b0 + kWaveBatch);
            if (b0 + 3 * kWaveBatch < n) load(b0 + 3 * kWaveBatch, bufB);
        }
        if (qtail != qhead) expand(qtail - qhead);
        if (nrec > cap || nrec < (uint32_t)m) {  // the estimate failed (either way)
            defer();
            return;
        }
    }
    __syncthreads();  // records complete; the ring is dead

    // ---- 3. exact threshold among the records ---------------------------------------------------------------------
#pragma unroll
    for (int i = 0; i < kWaveHistWords / 256; ++i) reinterpret_cast<u32x4*>(aux)[i * 64 + lane] = u32x4{0, 0, 0, 0};
    if (lane < 8) sub[lane] = 0;
    __syncthreads();
    for (uint32_t c0 = lane * 4; c0 < nrec; c0 += 256) {  // cap is a multiple of 4: the read stays inside rec
        const u32x4 rv = *reinterpret_cast<const u32x4*>(rec + c0);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const uint32_t bin = rv[e] >> 21;  // top 11 bits of the relative key
            if (c0 + e < nrec) atomicAdd(&aux[bin >> 1], (bin & 1u) ? 0x10000u : 1u);
        }
    }
    __syncthreads();
    uint32_t above;
    const int b1 = wave_find_bin<2048>(aux, (uint32_t)m, lane, &above);  // >= 0: nrec >= m
    uint32_t need = (uint32_t)m - above;  // to take among the records of bin b1
    for (uint32_t c0 = lane * 4; c0 < nrec; c0 += 256) {
        const u32x4 rv = *reinterpret_cast<const u32x4*>(rec + c0);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const uint32_t rel = rv[e] >> 19;
            if (c0 + e < nrec && (rel >> 2) == (uint32_t)b1) atomicAdd(&sub[rel & 3u], 1u);
        }
    }
    __syncthreads();
    uint32_t Tq = 0, ne = 0;  // relative key of the threshold, records that carry it
    for (int s = 3; s >= 0; --s) {
        ne = sub[s];
        if (need <= ne) {
            Tq = ((uint32_t)b1 << 2) | (uint32_t)s;
            break;
        }
        need -= ne;
    }
    if (Tq >= kRelMax || (need < ne && ne > (uint32_t)kWaveTieCap)) {  // saturated keys cannot be ordered here
        defer();
        return;
    }
    __syncthreads();  // aux is reused

    // ---- 3b. only some of the keys at the threshold fit: order them by their recomputed fp32 scores ------------------
    uint32_t take_from = Tq;  // records with a relative key >= take_from are taken
    if (need < ne) {
        float* q_lds = reinterpret_cast<float*>(aux);  // HI*DI query values, then HI weights, HI biases
        float* w_lds = q_lds + HI * DI;
        float* nb_lds = w_lds + HI;
        uint32_t* tie_pos = aux + HI * DI + 2 * HI;
        float* tie_score = reinterpret_cast<float*>(tie_pos + kWaveTieCap);
#pragma unroll
        for (int i = 0; i < QPL; ++i) {
            const int c = lane + i * 64;
            if (c < HI * DI) q_lds[c] = qreg[i];
        }
        if (lane < HI) {
            w_lds[lane] = wreg;
            nb_lds[lane] = nbreg;
        }
        uint32_t tn = 0;
        for (uint32_t c0 = 0; c0 < nrec; c0 += 256) {  // list order = index order (a lane holds 4 consecutive records)
            const uint32_t c = c0 + lane * 4;
            u32x4 rv = u32x4{0, 0, 0, 0};
            if (c < nrec) rv = *reinterpret_cast<const u32x4*>(rec + c);
            uint32_t tm = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) tm |= (c + e < nrec && (rv[e] >> 19) == Tq) ? (1u << e) : 0u;
            uint32_t total;
            uint32_t o = tn + wave_prefix_small<3>(__popc(tm), &total);
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (tm & (1u << e)) tie_pos[o++] = c + e;
            tn += total;
        }
        __syncthreads();
        const T* kpool = static_cast<const T*>(a.kI);
        for (uint32_t i = lane; i < ne; i += 64) {
            const uint32_t si = rec[tie_pos[i]] & 0x7ffffu;
            tie_score[i] = recompute_score<T, DI, HI>(kpool + cache_row(a.pm, b, (int)si, a.Lk) * DI, q_lds, w_lds, nb_lds);
        }
        __syncthreads();
        for (uint32_t i = lane; i < ne; i += 64) {
            const float si = tie_score[i];
            uint32_t rank = 0;
            for (uint32_t j = 0; j < ne; ++j) {
                const float sj = tie_score[j];
                rank += (sj > si || (sj == si && j < i)) ? 1u : 0u;  // equal scores: lowest index first
            }
            if (rank < need) rec[tie_pos[i]] |= kRelMax << 19;  // now above the threshold (Tq < kRelMax)
        }
        __syncthreads();
        take_from = Tq + 1;
    }

    // ---- 4. the taken records, in list order ----------------------------------------------------------------------
    uint32_t wpos = 0;
    for (uint32_t c0 = 0; c0 < nrec; c0 += 256) {
        const uint32_t c = c0 + lane * 4;
        u32x4 rv = u32x4{0, 0, 0, 0};
        if (c < nrec) rv = *reinterpret_cast<const u32x4*>(rec + c);
        uint32_t sm = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) sm |= (c + e < nrec && (rv[e] >> 19) >= take_from) ? (1u << e) : 0u;
        uint32_t total;
        uint32_t o = wpos + wave_prefix_small<3>(__popc(sm), &total);
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (sm & (1u << e)) {
                if (o < (uint32_t)a.k_cap) out[o] = (int32_t)(rv[e] & 0x7ffffu);
                ++o;
            }
        wpos += total;
    }
}

static int kernel_heads16(int hi) { return hi <= 1 ? 1 : (hi <= 2 ? 2 : (hi <= 4 ? 4 : 8)); }

size_t select16_lds_bytes(const gsa_shape& sh) {
    const int nw = ((sh.Lk + 31) / 32 + 3) & ~3;  // bitmap words, rounded so that what follows stays 16-byte aligned
    const int r2 = nw > kBinsC + kTieCap ? nw : kBinsC + kTieCap;
    const int HIK = kernel_heads16(sh.HI);
    return (size_t)(kRegion0_16 + nw + r2 + 32 + HIK * sh.dI + 2 * HIK) * sizeof(uint32_t);
}

// Records a row can hold in the wave-per-row kernel.  The candidates of a row with budget m number about
// 1.2 m +- 0.07 m (sampled one key in 16).  Budgets up to kWaveSplit get 4088 records (2.6 sigma at the split):
// eight workgroups of 20 KB per compute unit.  Rows with larger budgets run in a launch of their own with
// 11/8 of the largest budget (2.6 sigma again; six workgroups per compute unit at 4096).
constexpr int kWaveSplit = 2816;
static int wave_record_cap(int k_cap) { return k_cap <= kWaveSplit ? 4088 : std::min((k_cap * 11 / 8 + 3) & ~3, 14336); }
static size_t wave_lds_bytes(int k_cap, int HIK, int DI) {
    const int aux_words = std::max(kWaveHistWords, HIK * DI + 2 * HIK + 2 * kWaveTieCap);
    return (size_t)(wave_record_cap(k_cap) + aux_words + 8) * sizeof(uint32_t);
}

// Both kernels, one after the other on the stream: the wave-per-row kernel finishes nearly every row, the
// workgroup-per-row kernel then takes the rows left marked.  With few rows (decode) a wave per row would leave
// most of the chip idle and every row slow: the workgroup-per-row kernel takes them all.
constexpr int64_t kWaveMinRows = 2048;
template <typename T, int DI, int HI>
static hipError_t launch16_one(const Select16Args& a0, size_t smem, int64_t rows, int wave_min_rows, hipStream_t st) {
    Select16Args a = a0;
    hipError_t e;
    auto kern = topk_select16_deferred_kernel<T, DI, HI>;
    if (smem > 48 * 1024) {
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
    }
    if (wave_min_rows < 0 || rows < (wave_min_rows > 0 ? (int64_t)wave_min_rows : kWaveMinRows)) {
        a.group = 0;
        hipLaunchKernelGGL(kern, dim3((unsigned)rows), dim3(kSelThreads), smem, st, a);
        return hipGetLastError();
    }
    auto wave = topk_select16_wave_kernel<T, DI, HI>;
    const size_t wsmem = wave_lds_bytes(a.k_cap, HI, DI);
    if (wsmem > 48 * 1024) {
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(wave), hipFuncAttributeMaxDynamicSharedMemorySize, (int)wsmem);
        if (e != hipSuccess) return e;
    }
    if (a.k_cap > kWaveSplit) {  // the rows with large budgets first, with the larger record lists
        a.cap = wave_record_cap(a.k_cap);
        a.m_lo = kWaveSplit;
        a.m_hi = a.k_cap;
        hipLaunchKernelGGL(wave, dim3((unsigned)rows), dim3(64), wsmem, st, a);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    a.m_lo = -1;
    a.m_hi = std::min(a.k_cap, kWaveSplit);
    a.cap = wave_record_cap(a.m_hi);
    hipLaunchKernelGGL(wave, dim3((unsigned)rows), dim3(64), wave_lds_bytes(a.m_hi, HI, DI), st, a);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    a.group = kDeferGroup;
    hipLaunchKernelGGL(kern, dim3((unsigned)cdiv(rows, kDeferGroup)), dim3(kSelThreads), smem, st, a);
    return hipGetLastError();
}
template <typename T, int DI>
static hipError_t launch16_hi(const Select16Args& a, int HI, size_t smem, int64_t rows, int wmr, hipStream_t st) {
    switch (HI) {
        case 1: return launch16_one<T, DI, 1>(a, smem, rows, wmr, st);
        case 2: return launch16_one<T, DI, 2>(a, smem, rows, wmr, st);
        case 4: return launch16_one<T, DI, 4>(a, smem, rows, wmr, st);
        case 8: return launch16_one<T, DI, 8>(a, smem, rows, wmr, st);
    }
    return hipErrorInvalidValue;
}
template <typename T>
static hipError_t launch16_di(const Select16Args& a, int DI, int HI, size_t smem, int64_t rows, int wmr, hipStream_t st) {
    switch (DI) {
        case 32: return launch16_hi<T, 32>(a, HI, smem, rows, wmr, st);
        case 64: return launch16_hi<T, 64>(a, HI, smem, rows, wmr, st);
        case 128: return launch16_hi<T, 128>(a, HI, smem, rows, wmr, st);
    }
    return hipErrorInvalidValue;
}

hipError_t launch_select16(const gsa_shape& sh, int row_begin, int row_end, const uint16_t* keys, int64_t ld,
                           const int32_t* n_sel, int k_cap, int32_t* idx_out, int idx_rows, int idx_row0, const void* qI,
                           const void* kI, const float* w, const float* bI, const int32_t* seq_lens, int wave_min_rows,
                           const PageMap& pm, hipStream_t st) {
    Select16Args a;
    a.pm = pm;
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
    return sh.dtype == GSA_BF16 ? launch16_di<__bf16>(a, sh.dI, HIK, smem, rows, wave_min_rows, st)
                                : launch16_di<float>(a, sh.dI, HIK, smem, rows, wave_min_rows, st);
}

}  // namespace gsa
