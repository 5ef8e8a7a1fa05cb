// Pieces shared by the selection kernels: block-wide threshold search over an LDS histogram, streaming
// of a score row, the exact multi-pass radix select and the ordered emission from LDS bitmaps.
#pragma once
#include "common.hpp"

namespace gsa {

constexpr int kSelThreads = 512;
constexpr int kSelWaves = kSelThreads / 64;
constexpr int kVecPerBatch = 4;  // float4 loads a thread keeps in flight per batch (two batches are in flight)
constexpr int kBatch = kSelThreads * 4 * kVecPerBatch;
constexpr int kBinsA = 8192;  // 13 bits per global pass
constexpr int kBitsA = 13;
constexpr int kCandCap = 2048;
constexpr int kBinsC = 2048;  // 11 bits per LDS pass (size of hist_c)
constexpr int kBitsC = 11;
constexpr int kCandFast = 5632;  // candidate capacity of the sampled one-pass path
constexpr int kTieCap = 2048;    // ties at the threshold the sampled path resolves itself
constexpr int kRegion0 = 2 * kCandFast;
static_assert(2 * kCandCap + kBinsC <= kBinsA && (1 << kBitsC) == kBinsC && kBinsA <= kRegion0, "LDS aliasing");

__device__ __forceinline__ uint32_t score_key(float x) {
    const uint32_t u = __float_as_uint(x);
    return (u & 0x80000000u) ? 0u : u;  // negative values (and -0) rank as 0
}

// Block-wide: largest bin b with sum_{b' >= b} hist[b'] >= need; above = sum_{b' > b} hist[b'].
// Requires sum(hist) >= need >= 1.  scratch: kSelWaves + 2 words.  All threads return the same result.
__device__ void find_threshold_bin(const uint32_t* hist, int nbins, uint32_t need, uint32_t* scratch, int* bin_out,
                                   uint32_t* above_out) {
    const int tid = threadIdx.x;
    const int lane = tid & 63, wv = tid >> 6;
    const int per = nbins >= kSelThreads ? nbins / kSelThreads : 1;
    const int lo = tid * per;
    uint32_t local = 0;
    if (lo < nbins)
        for (int i = 0; i < per; ++i) local += hist[lo + i];
    // inclusive suffix sum inside the wave (towards higher lanes)
    uint32_t incl = local;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t v = __shfl_down(incl, o, 64);
        if (lane + o < 64) incl += v;
    }
    if (lane == 0) scratch[wv] = incl;  // wave total
    __syncthreads();
    uint32_t higher = 0;
    for (int x = wv + 1; x < kSelThreads / 64; ++x) higher += scratch[x];
    const uint32_t suf_incl = incl + higher;
    const uint32_t suf_excl = suf_incl - local;
    if (lo < nbins && suf_excl < need && need <= suf_incl) {
        uint32_t acc = suf_excl;
        for (int i = per - 1; i >= 0; --i) {
            const uint32_t c = hist[lo + i];
            if (acc + c >= need) {
                scratch[kSelWaves] = (uint32_t)(lo + i);
                scratch[kSelWaves + 1] = acc;
                break;
            }
            acc += c;
        }
    }
    __syncthreads();
    *bin_out = (int)scratch[kSelWaves];
    *above_out = scratch[kSelWaves + 1];
    __syncthreads();  // scratch may be reused right away
}

// Stream the n visible scores of a row through f(index, value).  Every thread keeps two batches of
// kVecPerBatch 16-byte loads in flight (the next batch is requested before the current one is
// consumed), which is what lets a workgroup cover the HBM latency.
template <class F>
__device__ __forceinline__ void stream_row(const float* __restrict__ row, int n, F&& f) {
    const int tid = threadIdx.x;
    float4 cur[kVecPerBatch], nxt[kVecPerBatch];
    auto load = [&](int b0, float4* v) {
#pragma unroll
        for (int u = 0; u < kVecPerBatch; ++u) {
            const int base = b0 + (u * kSelThreads + tid) * 4;
            v[u] = base < n ? *reinterpret_cast<const float4*>(row + base) : float4{0.f, 0.f, 0.f, 0.f};
        }
    };
    load(0, cur);
    for (int b0 = 0; b0 < n; b0 += kBatch) {
        const bool more = b0 + kBatch < n;
        if (more) load(b0 + kBatch, nxt);
#pragma unroll
        for (int u = 0; u < kVecPerBatch; ++u) {
            const int base = b0 + (u * kSelThreads + tid) * 4;
            const float x[4] = {cur[u].x, cur[u].y, cur[u].z, cur[u].w};
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (base + e < n) f(base + e, x[e]);
        }
        if (more) {
#pragma unroll
            for (int u = 0; u < kVecPerBatch; ++u) cur[u] = nxt[u];
        }
    }
}

struct SelLds {
    uint32_t* region0;  // kRegion0 words: histogram of a global pass, later the candidate lists
    uint32_t* bm_sel;   // nw words: one bit per key of the row, set for sure winners
    uint32_t* region2;  // max(nw, 4096) words: tie bitmap (exact path) or LDS histogram + tie list (sampled path)
    uint32_t* scratch;  // 32 words
};

// Exact two-pass path (any input).  On return bm_sel / bm_tie are final and *m_eq_out is the number of
// tie bits to take in index order.
// `stream(f)` must call f(index, score) once for every element of the (virtual) row, the same elements on
// every call.  keep_sel: bits already present in bm_sel are kept (they are winners decided elsewhere and are
// not part of the stream); the function then only adds to them.
template <class Stream>
__device__ void select_exact(Stream&& stream, int n, int m, const SelLds& L, uint32_t* m_eq_out, bool keep_sel = false,
                             uint32_t* thr_key_out = nullptr) {
    uint32_t* hist = L.region0;                 // kBinsA words
    uint32_t* cand_key = L.region0;             // kCandCap
    uint32_t* cand_idx = L.region0 + kCandCap;  // kCandCap
    uint32_t* hist_c = L.region0 + 2 * kCandCap;  // kBinsC
    uint32_t* bm_sel = L.bm_sel;
    uint32_t* bm_tie = L.region2;
    uint32_t* scratch = L.scratch;
    const int tid = threadIdx.x;

    // ---- A: radix descent over the row in global memory -------------------------------------
    uint32_t prefix = 0;
    int pbits = 0;  // resolved leading bits of the 31-bit key
    uint32_t need = (uint32_t)m;
    uint32_t cand = 0;
    while (true) {
        const int nb = min(kBitsA, 31 - pbits);
        const int shift = 31 - pbits - nb;
        const uint32_t mask = (1u << nb) - 1u;
        for (int i = tid; i < (1 << nb); i += kSelThreads) hist[i] = 0;
        __syncthreads();
        {
            const int pshift = 31 - pbits;
            const bool all = pbits == 0;
            stream([&](int, float xv) {
                const uint32_t key = score_key(xv);
                if (all || (key >> pshift) == prefix) atomicAdd(&hist[(key >> shift) & mask], 1u);
            });
        }
        __syncthreads();
        int bin;
        uint32_t above;
        find_threshold_bin(hist, 1 << nb, need, scratch, &bin, &above);
        cand = hist[bin];
        need -= above;
        prefix = (prefix << nb) | (uint32_t)bin;
        pbits += nb;
        __syncthreads();  // everyone has read hist[bin] before it is cleared or reused
        if (cand <= (uint32_t)kCandCap || pbits == 31) break;
    }
    const bool exact = (pbits == 31);  // the prefix is a whole key: candidates are exact ties
    const int rb0 = 31 - pbits;

    // ---- B: mark the sure winners, gather the candidates --------------------------------------
    const int nw_row = (n + 31) >> 5;
    for (int i = tid; i < nw_row; i += kSelThreads) {
        if (!keep_sel) bm_sel[i] = 0;
        bm_tie[i] = 0;
    }
    if (tid == 0) scratch[kSelWaves + 2] = 0;  // candidate counter
    __syncthreads();
    stream([&](int si, float xv) {
        const uint32_t key = score_key(xv);
        const uint32_t kp = key >> rb0;
        if (kp > prefix) {
            atomicOr(&bm_sel[si >> 5], 1u << (si & 31));
        } else if (kp == prefix) {
            if (exact) {
                atomicOr(&bm_tie[si >> 5], 1u << (si & 31));
            } else {
                const uint32_t pos = atomicAdd(&scratch[kSelWaves + 2], 1u);
                if (pos < (uint32_t)kCandCap) {
                    cand_key[pos] = key;
                    cand_idx[pos] = (uint32_t)si;
                }
            }
        }
    });
    __syncthreads();

    // ---- C: finish the descent on the candidate list -------------------------------------------
    if (!exact) {
        const int nc = (int)min(cand, (uint32_t)kCandCap);
        int rb = rb0;
        while (rb > 0) {
            const int nb = min(kBitsC, rb);
            const uint32_t mask = (1u << nb) - 1u;
            for (int i = tid; i < (1 << nb); i += kSelThreads) hist_c[i] = 0;
            __syncthreads();
            for (int c = tid; c < nc; c += kSelThreads) {
                const uint32_t key = cand_key[c];
                if ((key >> rb) == prefix) atomicAdd(&hist_c[(key >> (rb - nb)) & mask], 1u);
            }
            __syncthreads();
            int bin;
            uint32_t above;
            find_threshold_bin(hist_c, 1 << nb, need, scratch, &bin, &above);
            need -= above;
            prefix = (prefix << nb) | (uint32_t)bin;
            rb -= nb;
        }
        // prefix is now the threshold key T; `need` elements equal to T remain to be taken
        for (int c = tid; c < nc; c += kSelThreads) {
            const uint32_t key = cand_key[c];
            const uint32_t s = cand_idx[c];
            if (key > prefix)
                atomicOr(&bm_sel[s >> 5], 1u << (s & 31));
            else if (key == prefix)
                atomicOr(&bm_tie[s >> 5], 1u << (s & 31));
        }
        __syncthreads();
    }
    *m_eq_out = need;
    if (thr_key_out) *thr_key_out = prefix;  // bit pattern of the threshold score
}

// Walk the bitmaps in index order: every selection bit and the first m_eq tie bits are written to out
// (ascending), the rest of the k_cap entries is set to -1.  bm_tie may be null (no ties to take).
__device__ void emit_selection(int32_t* out, int k_cap, int m, int n, const uint32_t* bm_sel, const uint32_t* bm_tie,
                               uint32_t m_eq, unsigned long long* scan64) {
    const int tid = threadIdx.x;
    const bool with_ties = bm_tie != nullptr;
    const int nw_row = (n + 31) >> 5;
    const int wpt = (nw_row + kSelThreads - 1) / kSelThreads;
    const int w_lo = min(tid * wpt, nw_row), w_hi = min(w_lo + wpt, nw_row);
    uint32_t cs = 0, ct = 0;
    for (int wi = w_lo; wi < w_hi; ++wi) {
        cs += __popc(bm_sel[wi]);
        if (with_ties) ct += __popc(bm_tie[wi]);
    }
    unsigned long long packed = ((unsigned long long)ct << 32) | cs;
    unsigned long long incl = packed;
    const int lane = tid & 63, wv = tid >> 6;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const unsigned long long v = __shfl_up(incl, o, 64);
        if (lane >= o) incl += v;
    }
    if (lane == 63) scan64[wv] = incl;
    __syncthreads();
    unsigned long long lower = 0;
    for (int x = 0; x < wv; ++x) lower += scan64[x];
    const unsigned long long excl = incl - packed + lower;
    uint32_t ties_before = (uint32_t)(excl >> 32);
    uint32_t pos = (uint32_t)(excl & 0xffffffffu) + min(ties_before, m_eq);
    for (int wi = w_lo; wi < w_hi; ++wi) {
        uint32_t wt = with_ties ? bm_tie[wi] : 0u;
        const uint32_t ntie = __popc(wt);
        const uint32_t allow = m_eq - min(ties_before, m_eq);
        while ((uint32_t)__popc(wt) > allow) wt &= ~(0x80000000u >> __clz(wt));  // drop the highest tie bits
        uint32_t comb = bm_sel[wi] | wt;
        while (comb) {
            const int bit = __ffs(comb) - 1;
            if (pos < (uint32_t)k_cap) out[pos] = wi * 32 + bit;
            ++pos;
            comb &= comb - 1u;
        }
        ties_before += ntie;
    }
    for (int j = m + tid; j < k_cap; j += kSelThreads) out[j] = -1;
}

}  // namespace gsa
