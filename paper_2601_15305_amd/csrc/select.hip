// Top-k_t selection (Sec. 2.2 Eq. 4 with the per-query budget of Sec. 3.4) and the adaptive
// controller itself (Eq. "adaptive_k").
//
// Selection is an exact radix select on the fp32 bit pattern of the non-negative scores (which
// orders like the value), one workgroup of eight wavefronts per query row (steps A-C: select_exact in
// select_common.hpp, step D: emit_selection):
//   A. histogram the next 13 key bits of every element that still matches the resolved prefix
//      (LDS atomics), locate the bin holding the n_sel-th largest; repeat only while that bin
//      holds more candidates than fit in LDS (at most three passes: 13 + 13 + 5 bits);
//   B. stream the row once more: elements above the bin set a bit in an LDS bitmap of the row,
//      elements inside it go to an LDS candidate list (or, if the prefix is already a whole
//      key, to a second "tie" bitmap);
//   C. finish the radix descent on the candidate list in LDS, giving the exact threshold key T
//      and the number m_eq of elements equal to T that still have to be taken; candidates
//      above T set selection bits, candidates equal to T set tie bits;
//   D. walk the two bitmaps in index order: all selection bits and the first m_eq tie bits
//      are emitted, which yields ascending indices and the lowest-index tie-break for free.
// The result is deterministic and independent of the order in which atomics land.
// Long rows with a small budget first try a one-pass variant that gets its threshold bound from a
// strided sample of the row (select_sampled below); its result is verified and identical.
#include "select_common.hpp"

namespace gsa {

struct SelectArgs {
    const float* scores;
    int64_t ld;
    const int32_t* n_sel;
    int32_t* idx_out;
    int32_t B, Lq, Lk, q_offset, row_begin, row_end, k_cap;
    int32_t nw;  // bitmap words reserved per bitmap
    int32_t idx_rows, idx_row0;  // idx_out holds rows [idx_row0, idx_row0+idx_rows) of every batch element
    int32_t sampled;             // allow the sampled one-pass path
    const int32_t* seq_lens;     // per-sequence lengths (ragged decode) or null
};

// One-pass path for long rows with a small budget.  A strided sample of the row (16 consecutive scores
// out of every 256, i.e. one 64-byte piece per KiB) is histogrammed first; the sample's
// (expected rank + 4 sigma)-th largest value gives a lower bound tau such that, with overwhelming
// probability, at least m scores of the row lie above it and few enough to fit in LDS.  One pass over
// the row then gathers every score >= tau, and the exact radix select with lowest-index tie-break runs
// on that list.  The counts are verified: if fewer than m or more than the list capacity qualify (or
// too many tie at the threshold) the function returns false and the caller takes the exact path, so the
// sample only ever affects speed.  On success all m winners have their bit set in bm_sel.
__device__ bool select_sampled(const float* __restrict__ row, int n, int m, const SelLds& L) {
    uint32_t* hist = L.region0;                   // kBinsA words, dead before the lists are written
    uint32_t* cand_key = L.region0;               // kCandFast
    uint32_t* cand_idx = L.region0 + kCandFast;   // kCandFast
    uint32_t* hist_c = L.region2;                 // kBinsC
    uint32_t* tie_list = L.region2 + kBinsC;      // kTieCap
    uint32_t* bm_sel = L.bm_sel;
    uint32_t* scratch = L.scratch;
    const int tid = threadIdx.x;

    for (int i = tid; i < kBinsA; i += kSelThreads) hist[i] = 0;
    __syncthreads();
    for (int q0 = tid; (q0 >> 2) * 256 < n; q0 += 4 * kSelThreads) {  // four independent loads in flight
        float4 v[4];
        int base[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int q = q0 + u * kSelThreads;
            base[u] = (q >> 2) * 256 + (q & 3) * 4;
            v[u] = base[u] < n ? *reinterpret_cast<const float4*>(row + base[u]) : float4{0.f, 0.f, 0.f, 0.f};
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const float x[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (base[u] + e < n) atomicAdd(&hist[score_key(x[e]) >> (31 - kBitsA)], 1u);
        }
    }
    __syncthreads();
    const int ms = (n >> 8) * 16 + min(16, n & 255);  // sampled elements
    const float lam = (float)m * (float)ms / (float)n;
    const int r = (int)ceilf(lam + 4.0f * sqrtf(lam) + 2.0f);
    if (r > ms) return false;
    int b_lo;
    uint32_t above;
    find_threshold_bin(hist, kBinsA, (uint32_t)r, scratch, &b_lo, &above);

    const int nw_row = (n + 31) >> 5;
    for (int i = tid; i < nw_row; i += kSelThreads) bm_sel[i] = 0;
    if (tid == 0) {
        scratch[kSelWaves + 2] = 0;  // candidate counter
        scratch[kSelWaves + 3] = 0;  // tie counter
    }
    __syncthreads();
    stream_row(row, n, [&](int si, float xv) {
        const uint32_t key = score_key(xv);
        if ((int)(key >> (31 - kBitsA)) >= b_lo) {
            const uint32_t pos = atomicAdd(&scratch[kSelWaves + 2], 1u);
            if (pos < (uint32_t)kCandFast) {
                cand_key[pos] = key;
                cand_idx[pos] = (uint32_t)si;
            }
        }
    });
    __syncthreads();
    const uint32_t nc = scratch[kSelWaves + 2];
    if (nc < (uint32_t)m || nc > (uint32_t)kCandFast) return false;

    // exact radix select inside the list: 11 + 11 + 9 bits
    uint32_t prefix = 0, need = (uint32_t)m;
    int rb = 31;
    while (rb > 0) {
        const int nb = min(kBitsC, rb);
        const uint32_t mask = (1u << nb) - 1u;
        for (int i = tid; i < (1 << nb); i += kSelThreads) hist_c[i] = 0;
        __syncthreads();
        for (uint32_t c = tid; c < nc; c += kSelThreads) {
            const uint32_t key = cand_key[c];
            if ((key >> rb) == prefix) atomicAdd(&hist_c[(key >> (rb - nb)) & mask], 1u);
        }
        __syncthreads();
        int bin;
        find_threshold_bin(hist_c, 1 << nb, need, scratch, &bin, &above);
        need -= above;
        prefix = (prefix << nb) | (uint32_t)bin;
        rb -= nb;
    }
    // prefix = threshold key T; `need` of the elements equal to T are taken, lowest index first
    for (uint32_t c = tid; c < nc; c += kSelThreads) {
        const uint32_t key = cand_key[c];
        const uint32_t s = cand_idx[c];
        if (key > prefix) {
            atomicOr(&bm_sel[s >> 5], 1u << (s & 31));
        } else if (key == prefix) {
            const uint32_t pos = atomicAdd(&scratch[kSelWaves + 3], 1u);
            if (pos < (uint32_t)kTieCap) tie_list[pos] = s;
        }
    }
    __syncthreads();
    const uint32_t ne = scratch[kSelWaves + 3];
    if (ne > (uint32_t)kTieCap) return false;
    for (uint32_t i = tid; i < ne; i += kSelThreads) {
        const uint32_t s = tie_list[i];
        uint32_t rank = 0;
        if (need < ne)
            for (uint32_t j = 0; j < ne; ++j) rank += tie_list[j] < s ? 1u : 0u;
        if (rank < need) atomicOr(&bm_sel[s >> 5], 1u << (s & 31));
    }
    __syncthreads();
    return true;
}

__global__ __launch_bounds__(kSelThreads) void topk_select_kernel(SelectArgs a) {
    extern __shared__ __attribute__((aligned(16))) uint32_t lds[];
    SelLds L;
    L.region0 = lds;
    L.bm_sel = lds + kRegion0;
    L.region2 = L.bm_sel + a.nw;
    L.scratch = L.region2 + max(a.nw, kBinsC + kTieCap);
    unsigned long long* scan64 = reinterpret_cast<unsigned long long*>(L.scratch + 12);  // kSelWaves entries

    const int tid = threadIdx.x;
    const int R = a.row_end - a.row_begin;
    const int64_t rid = (int64_t)gridDim.x - 1 - blockIdx.x;  // longest rows of the slab first
    const int b = (int)(rid / R);
    const int t = a.row_begin + (int)(rid % R);
    const int n = min(batch_q_offset(a.seq_lens, b, a.q_offset, a.Lq, a.Lk) + t, a.Lk - 1) + 1;
    int m = a.n_sel[(int64_t)b * a.Lq + t];
    m = max(0, min(m, min(n, a.k_cap)));
    int32_t* out = a.idx_out + ((int64_t)b * a.idx_rows + (t - a.idx_row0)) * a.k_cap;

    if (m == n || m == 0) {  // everything visible is selected (or nothing is)
        for (int j = tid; j < a.k_cap; j += kSelThreads) out[j] = j < m ? j : -1;
        return;
    }
    const float* row = a.scores + ((int64_t)b * R + (t - a.row_begin)) * a.ld;

    uint32_t m_eq = 0;
    bool with_ties = false;
    bool done = false;
    if (a.sampled && n >= 16384 && n >= 8 * m) done = select_sampled(row, n, m, L);
    if (!done) {
        select_exact([&](auto&& f) { stream_row(row, n, f); }, n, m, L, &m_eq);
        with_ties = true;
    }
    emit_selection(out, a.k_cap, m, n, L.bm_sel, with_ties ? L.region2 : nullptr, m_eq, scan64);
}


size_t select_lds_bytes(int Lk) {
    const int nw = (Lk + 31) / 32;
    const int r2 = nw > kBinsC + kTieCap ? nw : kBinsC + kTieCap;
    return (size_t)(kRegion0 + nw + r2 + 32) * sizeof(uint32_t);
}

hipError_t launch_select(const gsa_shape& sh, int row_begin, int row_end, const float* scores, int64_t ld,
                         const int32_t* n_sel, int k_cap, int32_t* idx_out, int idx_rows, int idx_row0, bool exact_only,
                         const int32_t* seq_lens, hipStream_t st) {
    SelectArgs a;
    a.seq_lens = seq_lens;
    a.scores = scores;
    a.ld = ld;
    a.n_sel = n_sel;
    a.idx_out = idx_out;
    a.B = sh.B;
    a.Lq = sh.Lq;
    a.Lk = sh.Lk;
    a.q_offset = sh.q_offset;
    a.row_begin = row_begin;
    a.row_end = row_end;
    a.k_cap = k_cap;
    a.nw = (sh.Lk + 31) / 32;
    a.idx_rows = idx_rows;
    a.idx_row0 = idx_row0;
    a.sampled = exact_only ? 0 : 1;
    const size_t smem = select_lds_bytes(sh.Lk);
    if (smem > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(topk_select_kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
    }
    const int64_t rows = (int64_t)sh.B * (row_end - row_begin);
    hipLaunchKernelGGL(topk_select_kernel, dim3((unsigned)rows), dim3(kSelThreads), smem, st, a);
    return hipGetLastError();
}

// ---- adaptive controller ------------------------------------------------------------------------
// k_t = clamp(floor(k_base * Var / vbar), k_min, k_max)   (mode 1: k_base * vbar / Var), evaluated in
// double precision from the fp32 variance; floor before clamp, clamp before the integer conversion.
__global__ void adaptive_k_kernel(const float* row_var, int32_t* k_out, int32_t* n_sel_out, int B, int Lq, int Lk,
                                  int q_offset, int row_begin, int row_end, double vbar, int k_base, int k_min,
                                  int k_max, int k_fixed, int mode, const int32_t* seq_lens) {
    const int R = row_end - row_begin;
    const int64_t lid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (lid >= (int64_t)B * R) return;
    const int t = row_begin + (int)(lid % R);
    const int64_t gid = (lid / R) * Lq + t;
    int k;
    if (k_fixed > 0) {
        k = k_fixed;
    } else {
        const double var = (double)row_var[gid];
        double r;
        if (mode == 0)
            r = (double)k_base * var / vbar;
        else
            r = var > 0.0 ? (double)k_base * vbar / var : (double)k_max;
        r = floor(r);
        if (!(r >= (double)k_min)) r = (double)k_min;  // also catches NaN
        if (r > (double)k_max) r = (double)k_max;
        k = (int)r;
    }
    const int nvis = min(batch_q_offset(seq_lens, (int)(lid / R), q_offset, Lq, Lk) + t, Lk - 1) + 1;
    if (k_out) k_out[gid] = k;
    n_sel_out[gid] = min(k, nvis);
}

hipError_t launch_adaptive_k(const gsa_shape& sh, const gsa_adaptive& c, int row_begin, int row_end,
                             const float* row_var, int32_t* k_out, int32_t* n_sel_out, const int32_t* seq_lens, hipStream_t st) {
    const int64_t rows = (int64_t)sh.B * (row_end - row_begin);
    hipLaunchKernelGGL(adaptive_k_kernel, dim3((unsigned)cdiv(rows, 256)), dim3(256), 0, st, row_var, k_out, n_sel_out,
                       sh.B, sh.Lq, sh.Lk, sh.q_offset, row_begin, row_end, (double)c.vbar, c.k_base, c.k_min, c.k_max, c.k_fixed, c.mode, seq_lens);
    return hipGetLastError();
}

}  // namespace gsa
