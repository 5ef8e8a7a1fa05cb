// Sparse attention over the selected keys with the value gate G2 and the output gate G1
// (Sec. 3.5 and Sec. 3.6):
//   A[s] = softmax_{s in S_t}(scale * Q[t,h,:] . K[s,g,:]),  O = sum_s A[s] (V[s,g,:] * sigmoid(g2[s,g,:])),
//   out[t,h,:] = O * sigmoid(g1[t,h,:]),   g = h / (H / H_kv).
//
// bf16 kernel.  One wave per (query, kv head); a workgroup holds the waves of one query for one to four
// kv heads, grid.y walks over the kv-head slices and grid.z over pieces of the selected list (decode);
// long prefills are launched once per window of keys, each launch resuming the running softmax state
// (unnormalised O, running max, running sum) that the previous window left in the workspace
// (see launch_attention).  For one kv head the
// G = H/H_kv query heads that share it form the N dimension of the MFMAs (padded to 16), the
// gathered tokens form M for the score product and K for the value product:
//   S^T[token, head] = K[token, :] . Q[head, :]
//   O^T[d, head]    += V'^T[d, token] . P^T[token, head]
// The accumulator layout of S^T (a lane holds four tokens of one head) is exactly the B-operand
// layout the second product needs, so probabilities never move between lanes.  The gathered K and V'
// rows are loaded whole (16 lanes x 16 bytes per row, the access shape the memory pipeline serves
// fastest) into two wave-private LDS tiles.  K comes back as the A operand of the first product with
// plain 16-byte reads (a lane owns 16 consecutive bytes of a token's row), V' comes back transposed with
// the LDS transpose read of gfx950 (ds_read_b64_tr_b16), which turns 4 tokens x 16 features into the
// "feature row, token contraction" A operand of the second.  Softmax is the usual online form in base 2;
// G1 is applied to the accumulators before the store.
// Two ways of getting the rows into the tiles.  Staged: rows -> registers -> LDS (padded tiles), G2 applied to the
// V rows in registers on the way.  Direct (gated values given, 256-byte rows): global_load_lds_dwordx4 moves the
// rows straight into unpadded, XOR-swizzled tiles, with the K rows of the next tile and its V' rows requested as
// two separate streams and the waits for them placed by hand (see the DIRECT branch of the kernel).
#include "common.hpp"

namespace gsa {

struct AttnArgs {
    const void* Q;
    const void* K;
    const void* V;
    const void* g2;
    const void* g1;
    const int32_t* idx;
    const int32_t* n_sel;
    void* out;
    int32_t B, Lq, Lk, H, H_kv, row_begin, row_end, k_cap;
    int32_t idx_rows, idx_row0;  // idx holds rows [idx_row0, idx_row0+idx_rows) of every batch element
    float scale;  // softmax scale
    int32_t nsplit;  // > 1: a row's selected list is cut into nsplit pieces, partial results go to `part`
    float* part;     // [rows][H][nsplit][d_h + 4]: unnormalised O, running max (base 2), running sum, padding
    // Key-window mode (winoff != nullptr): piece z of a row is the part of its (ascending) list that falls
    // into keys [z*window, (z+1)*window); one launch handles one window for the rows that can see it and
    // carries the row's softmax state on in `part`, which then holds one record [rows][H][d_h + 4] per head.
    const int32_t* winoff;  // [rows][nsplit + 1] list positions of the window boundaries
    int32_t window, win;    // keys per window, window of this launch
    int32_t q_offset;
    int32_t part_row0, part_rows;  // rows of the slab that `part` and `winoff` are laid out for
    int32_t rpw;                   // query rows a wave of the bf16 kernel works through (1 .. 64)
    // Pool mode (paged caches): idx holds rows of one pool [pool_rows, H_kv, d_h] shared by all batch elements
    // (already translated through the block table); 0: idx holds token positions inside [B, Lk, H_kv, d_h].
    int64_t pool_rows;
};

constexpr float kNegBig = -1.0e30f;

#ifndef GSA_ATTN_DIRECT
#define GSA_ATTN_DIRECT 1
#endif

typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

// max over lanes {l, l^16, l^32, l^48} without a trip through LDS (row swaps of gfx950)
__device__ __forceinline__ float quad_row_max(float x) {
    auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    x = fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
    r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float quad_row_sum(float x) {
    auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    x = __uint_as_float(r[0]) + __uint_as_float(r[1]);
    r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// ---- pieces of the direct-to-LDS variant ------------------------------------------------------------------------
// Rows go from global memory straight into LDS (global_load_lds_dwordx4: lane l's 16 bytes land at the LDS address
// in M0 + 16 l), without passing through registers.  The compiler would wait for EVERY outstanding vector-memory
// operation before any LDS read that could see such data, which would serialise the two streams (K rows, V' rows)
// this variant keeps in flight; so the LDS reads of these tiles are written as instructions the compiler does not
// look into, each followed (in straight-line code) by a hand-placed wait that names the registers read.  The list
// entries take the same road (one 4-byte-per-lane transfer per tile into a small LDS buffer): a register whose
// load the compiler cannot see must not stay pending across a branch, where it may be copied before it has arrived.
typedef __attribute__((address_space(1))) const void gmem_cv;
typedef __attribute__((address_space(3))) void lds_v;
__device__ __forceinline__ void row_chunk_to_lds(const void* src, unsigned char* lds_dst) {
    __builtin_amdgcn_global_load_lds((gmem_cv*)src, (lds_v*)lds_dst, 16, 0, 0);
}
__device__ __forceinline__ uint32_t lds_addr(const unsigned char* p) { return (uint32_t)(uintptr_t)(lds_v*)p; }
template <int OFF>
__device__ __forceinline__ u32x4 lds_read128_raw(uint32_t addr) {
    u32x4 v;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF));
    return v;
}
template <int OFF>
__device__ __forceinline__ s16x4 lds_read_tr16_raw(uint32_t addr) {
    s16x4 v;
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF));
    return v;
}
template <int OFF>
__device__ __forceinline__ int lds_read32_raw(uint32_t addr) {
    int v;
    asm volatile("ds_read_b32 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF));
    return v;
}
// "at most N LDS operations outstanding"; the registers named are results of raw reads that are complete afterwards
template <int N>
__device__ __forceinline__ void wait_lds(u32x4& a, u32x4& b, u32x4& c, u32x4& d) {
    asm volatile("s_waitcnt lgkmcnt(%4)" : "+v"(a), "+v"(b), "+v"(c), "+v"(d) : "n"(N) : "memory");
}
template <int N>
__device__ __forceinline__ void wait_lds(s16x4& a, s16x4& b, s16x4& c, s16x4& d) {
    asm volatile("s_waitcnt lgkmcnt(%4)" : "+v"(a), "+v"(b), "+v"(c), "+v"(d) : "n"(N) : "memory");
}
__device__ __forceinline__ void wait_lds_all(int (&t)[8]) {
    asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(t[0]), "+v"(t[1]), "+v"(t[2]), "+v"(t[3]), "+v"(t[4]), "+v"(t[5]), "+v"(t[6]), "+v"(t[7]));
}
// "at most N vector-memory operations outstanding" (they complete in order).  This wait is one the compiler sees,
// so that it knows what has completed and adds no wait of its own for registers that older loads wrote.
template <int N>
__device__ __forceinline__ void wait_vmem() {
    __builtin_amdgcn_s_waitcnt(((N >> 4) << 14) | (0xF << 8) | (0x7 << 4) | (N & 15));  // vmcnt(N), other counters open
    asm volatile("" ::: "memory");
}

// A wave works through the pieces of `a.rpw` consecutive query rows (same batch element, same kv head) as ONE
// stream of 32-token tiles: while a tile is being multiplied, the K/V' rows of the next tile and the indices of
// the one after it are already on their way, also when those tiles belong to the next query row.  The list
// bounds of all rows of the wave are fetched once, up front (lane i keeps those of row i).  A row therefore
// costs no start-up chain of dependent loads (bounds -> indices -> rows), which is what a short piece -- a
// row's share of one key window -- would otherwise spend most of its time on.
// POOL: the lists hold rows of a pool that may exceed 4 GiB: row addresses are 64-bit per lane.
// DIRECT (d_h = 128, gated values given): K and V' rows go straight into LDS, see attn_direct_stream below.
template <int DH, bool HAS_G2, bool POOL = false, bool DIRECT = false>
__global__ __launch_bounds__(256, 2) void attn_bf16_kernel(AttnArgs a) {
    static_assert(!DIRECT || (DH == 128 && !HAS_G2), "the direct-to-LDS variant is written for 256-byte rows of gated values");
    constexpr int KK = DH / 32;        // MFMA k-steps of the score product
    constexpr int MB = DH / 16;        // 16-feature blocks of the value product
    constexpr int ROWB = DH * 2;       // bytes of one head row
    constexpr int VROW = ROWB + 32;    // padded LDS row of the V' tile
    constexpr int KROW = ROWB + 16;    // padded LDS row of the K tile
    constexpr int VCH = ROWB / 16;     // 16-byte chunks per row
    constexpr int TPI = 64 / VCH;      // tokens covered by one V load instruction
    constexpr int NVL = 32 / TPI;      // V load instructions per 32-token tile

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int tid = threadIdx.x;
    const int lane = tid & 63, wv = DIRECT ? __builtin_amdgcn_readfirstlane(tid >> 6) : tid >> 6;
    const int n = lane & 15;   // head within the group / token within a 16-token sub-tile
    const int q = lane >> 4;   // k-chunk selector
    // (DIRECT: two unpadded 32 x 256-byte tiles, chunks XOR-swizzled inside every row)
    unsigned char* vlds = smem + wv * (DIRECT ? 16640 + 1024 * ((a.H / a.H_kv + 3) >> 2) : 32 * (VROW + KROW));
    unsigned char* klds = vlds + (DIRECT ? 8192 : 32 * VROW);

    // blockDim.x / 64 kv heads per workgroup; blockIdx.y selects which ones.  Blocks are dispatched
    // x-fastest, so all queries work on one slice of kv heads before the next slice starts: the K/V'
    // columns in use at any time then fit the on-die memory-side cache even when the whole K/V' does not.
    const int g = __builtin_amdgcn_readfirstlane(blockIdx.y * (blockDim.x >> 6) + wv);  // uniform over the wave
    if (g >= a.H_kv) return;  // (the waves of a workgroup never synchronise with each other)
    const int R = a.row_end - a.row_begin;
    const int chunks = (R + a.rpw - 1) / a.rpw;
    const int b = blockIdx.x / chunks;
    const int t0 = a.row_begin + (blockIdx.x % chunks) * a.rpw;   // first row of this wave
    const int nrows = min(a.rpw, a.row_end - t0);
    const int G = a.H / a.H_kv;
    const int head = g * G + n;
    const bool head_ok = n < G;
    const float sl2 = a.scale * kLog2e;
    // Bytes between consecutive tokens.  The K, V' (and g2) rows of one batch element span less than 4 GiB
    // (checked on the host), so a row is addressed as a wave-uniform 64-bit base plus a 32-bit lane offset.
    const uint32_t tokstride = (uint32_t)a.H_kv * ROWB;
    // records per head in `part`: one per piece (split lists) or a single running one (key windows)
    const int rec_per_head = a.winoff ? 1 : a.nsplit;
    const int rec = a.winoff ? 0 : (int)blockIdx.z;

    // ---- the piece [jb, je) of every row's list that this wave handles; lane i holds row t0 + i -------------
    // Split lists (decode): piece z leaves a partial record that attn_merge_kernel combines.  Key windows: the
    // launch of window z adds what windows 0..z-1 left in the row's state record (resume) and passes the sum on
    // (carry) unless z is the last window the row sees.
    int m_jb = 0, m_je = 0, m_flags = 0;  // flags: bit 0 = resume, bit 1 = carry / partial
    if (lane < nrows) {
        const int t = t0 + lane;
        const int nsel = max(0, min(a.n_sel[(int64_t)b * a.Lq + t], a.k_cap));
        if (a.winoff) {
            const int64_t prow = (int64_t)b * a.part_rows + (t - a.part_row0);
            m_jb = min(a.winoff[prow * (a.nsplit + 1) + a.win], nsel);
            m_je = min(a.winoff[prow * (a.nsplit + 1) + a.win + 1], nsel);
            m_flags = (a.win > 0 ? 1 : 0) | (a.win < min(a.q_offset + t, a.Lk - 1) / a.window ? 2 : 0);
        } else {
            const int ntile_all = (nsel + 31) >> 5;
            const int tps = (ntile_all + a.nsplit - 1) / a.nsplit;  // tiles per split
            const int piece = blockIdx.z;
            m_jb = min(piece * tps, ntile_all) * 32;
            m_je = min(min(piece * tps + tps, ntile_all) * 32, nsel);
            m_flags = a.nsplit > 1 ? 2 : 0;
        }
    }
    // first row at or after ri that has a tile; j0/je are set to its bounds (ri == nrows: the stream has ended)
    auto seek = [&](int ri, int& j0, int& je) {
        while (ri < nrows) {
            j0 = __builtin_amdgcn_readlane(m_jb, ri);
            je = __builtin_amdgcn_readlane(m_je, ri);
            if (j0 < je) break;
            ++ri;
        }
        return ri;
    };
    auto advance = [&](int& ri, int& j0, int& je) {
        j0 += 32;
        if (j0 >= je) ri = seek(ri + 1, j0, je);
    };

    const int64_t row0 = POOL ? 0 : (int64_t)b * a.Lk;  // first row of this batch element's K / V'
    const unsigned char* Kb = static_cast<const unsigned char*>(a.K) + (row0 * a.H_kv + g) * ROWB;
    const unsigned char* Vb = static_cast<const unsigned char*>(a.V) + (row0 * a.H_kv + g) * ROWB;
    const unsigned char* Gb = HAS_G2 ? static_cast<const unsigned char*>(a.g2) + (row0 * a.H_kv + g) * ROWB : nullptr;
    const int32_t* idx0 = a.idx + ((int64_t)b * a.idx_rows + (t0 - a.idx_row0)) * a.k_cap;  // index list of row t0

    bf16x8 qf[KK], qf_next[KK];
    f32x4 o[MB];
    float mrun = kNegBig, lrun = 0.f;
    u32x4 kr[NVL];
    u32x4 vf[NVL];
    u32x4 gf[HAS_G2 ? NVL : 1];

    // The tokens of a tile are dealt to the lanes the way the row loads want them: load instruction r of a tile
    // fetches, in lane group lane / VCH, the row of tile slot (lane / VCH) * NVL + r.  A lane therefore reads the
    // NVL consecutive list entries of its group itself (clamped to the end of the piece, so always valid loads):
    // no cross-lane exchange sits between the index loads and the row loads.
    const int slot0 = (lane / VCH) * NVL;
    auto load_idx = [&](int ri, int j0, int je, int (&tk)[NVL]) {
        const int32_t* row = idx0 + (int64_t)ri * a.k_cap;
#pragma unroll
        for (int r = 0; r < NVL; ++r) tk[r] = row[min(j0 + slot0 + r, je - 1)];
    };
    // Q fragments of row ri (B operand): lane (head n, chunk q) holds features (4*kk+q)*8 .. +8
    auto load_q = [&](int ri) {
        const u32x4* src = reinterpret_cast<const u32x4*>(static_cast<const __bf16*>(a.Q) +
                                                          (((int64_t)b * a.Lq + t0 + ri) * a.H + (head_ok ? head : 0)) * DH);
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
            u32x4 v = head_ok ? src[kk * 4 + q] : u32x4{0, 0, 0, 0};
            qf_next[kk] = __builtin_bit_cast(bf16x8, v);
        }
    };
    auto issue = [&](const int (&tokv)[NVL]) {
#pragma unroll
        for (int r = 0; r < NVL; ++r) {  // whole rows, 16 bytes per lane: K and V' of a token at the same offset
            if constexpr (POOL) {
                const int64_t row = max((int64_t)0, min((int64_t)tokv[r], a.pool_rows - 1));
                const int64_t off = row * tokstride + (lane % VCH) * 16;
                kr[r] = *reinterpret_cast<const u32x4*>(Kb + off);
                vf[r] = *reinterpret_cast<const u32x4*>(Vb + off);
                if constexpr (HAS_G2) gf[r] = *reinterpret_cast<const u32x4*>(Gb + off);
            } else {
                const int tk = max(0, min(tokv[r], a.Lk - 1));
                const uint32_t off = __umul24((uint32_t)tk, tokstride) + (uint32_t)(lane % VCH) * 16u;  // token < 2^24, stride < 2^24
                kr[r] = *reinterpret_cast<const u32x4*>(Kb + off);
                vf[r] = *reinterpret_cast<const u32x4*>(Vb + off);
                if constexpr (HAS_G2) gf[r] = *reinterpret_cast<const u32x4*>(Gb + off);
            }
        }
    };
    // K and V' rows -> LDS (natural layout: row = token slot, 16 B per lane)
    auto stage = [&]() {
#pragma unroll
        for (int r = 0; r < NVL; ++r)
            *reinterpret_cast<u32x4*>(klds + (slot0 + r) * KROW + (lane % VCH) * 16) = kr[r];
#pragma unroll
        for (int r = 0; r < NVL; ++r) {
            u32x4 v = vf[r];
            if constexpr (HAS_G2) {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float v0 = bf16_bits_to_f32(v[e] & 0xffffu) * sigmoid_f32(bf16_bits_to_f32(gf[r][e] & 0xffffu));
                    const float v1 = bf16_bits_to_f32(v[e] >> 16) * sigmoid_f32(bf16_bits_to_f32(gf[r][e] >> 16));
                    v[e] = pack_bf16x2(v0, v1);
                }
            }
            *reinterpret_cast<u32x4*>(vlds + (slot0 + r) * VROW + (lane % VCH) * 16) = v;
        }
    };
    // the arithmetic of the tile that sits in LDS: list positions j0 .. j0+31 of a row whose piece ends at je
    auto compute = [&](int j0, int je) {
        // ---- S^T = K . Q^T for two 16-token sub-tiles; the A operand (token n, features (4*kk+q)*8 .. +8)
        // is read back from the K tile --------------------------------------------------------------
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // this wave's LDS writes have landed
        f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
        {
            const unsigned char* k0 = klds + n * KROW + q * 16;
            const unsigned char* k1 = k0 + 16 * KROW;
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) {
                const u32x4 a0 = *reinterpret_cast<const u32x4*>(k0 + kk * 64);
                const u32x4 a1 = *reinterpret_cast<const u32x4*>(k1 + kk * 64);
                s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a0), qf[kk], s0, 0, 0, 0);
                s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a1), qf[kk], s1, 0, 0, 0);
            }
        }
        // lane (head n, q): s0[i] is token j0 + 4q + i, s1[i] is token j0 + 16 + 4q + i
        float x[8];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            x[i] = s0[i] * sl2;
            x[4 + i] = s1[i] * sl2;
        }
        if (j0 + 32 > je) {  // last tile of a piece: slots beyond the list do not count
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                if (j0 + 4 * q + i >= je) x[i] = kNegBig;
                if (j0 + 16 + 4 * q + i >= je) x[4 + i] = kNegBig;
            }
        }
        float tmax = fmaxf(fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3])), fmaxf(fmaxf(x[4], x[5]), fmaxf(x[6], x[7])));
        tmax = quad_row_max(tmax);
        const float mnew = fmaxf(mrun, tmax);
        const float alpha = fast_exp2(mrun - mnew);
        float psum = 0.f;
        float p[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            p[i] = fast_exp2(x[i] - mnew);
            psum += p[i];
        }
        lrun = lrun * alpha + psum;
        mrun = mnew;
        if (__any(alpha != 1.0f)) {  // the running maximum of some head rose: rescale (rare after a row's first tiles)
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) o[mb] *= alpha;
        }
        u32x4 pw = {pack_bf16x2(p[0], p[1]), pack_bf16x2(p[2], p[3]), pack_bf16x2(p[4], p[5]), pack_bf16x2(p[6], p[7])};
        const bf16x8 pf = __builtin_bit_cast(bf16x8, pw);

        // ---- O^T += V'^T . P^T --------------------------------------------------------------------
        {
            const int r4 = (lane & 15) >> 2, c4 = lane & 3;
            const unsigned char* p0 = vlds + (4 * q + r4) * VROW + c4 * 8;
            const unsigned char* p1 = p0 + 16 * VROW;
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) {
                s16x4 a0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p0 + mb * 32));
                s16x4 a1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p1 + mb * 32));
                typedef __attribute__((ext_vector_type(8))) short s16x8;
                s16x8 av = {a0[0], a0[1], a0[2], a0[3], a1[0], a1[1], a1[2], a1[3]};
                o[mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, av), pf, o[mb], 0, 0, 0);
            }
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // transpose reads done before the tile is overwritten
    };
    auto reset_acc = [&]() {
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) o[mb] = f32x4{0.f, 0.f, 0.f, 0.f};
        mrun = kNegBig;
        lrun = 0.f;
    };
    // A row's piece is complete (accumulators o, mrun, lrun): add what earlier key windows left, then either
    // pass the state on / leave the partial record, or normalise, apply G1 and store the output row.
    auto finish_row = [&](int ri) {
        const int flags = __builtin_amdgcn_readlane(m_flags, ri);
        const int t = t0 + ri;
        const int64_t qrow = (int64_t)b * a.Lq + t;
        const int64_t prow = (int64_t)b * a.part_rows + (t - a.part_row0);
        float ltot = quad_row_sum(lrun);
        float* const state = a.part + (((prow * a.H) + (head_ok ? head : 0)) * rec_per_head + rec) * (DH + 4);
        if ((flags & 1) && head_ok) {  // merge with the state of the previous key windows
            f32x4 po[MB];
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) po[mb] = *reinterpret_cast<const f32x4*>(state + mb * 16 + 4 * q);
            const float pm = state[DH], pl = state[DH + 1];
            const float M = fmaxf(mrun, pm);
            const float wa = fast_exp2(mrun - M), wb = fast_exp2(pm - M);
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) o[mb] = o[mb] * wa + po[mb] * wb;
            ltot = ltot * wa + pl * wb;
            mrun = M;
        }
        if (flags & 2) {
            if (head_ok) {
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) *reinterpret_cast<f32x4*>(state + mb * 16 + 4 * q) = o[mb];
                if (q == 0) {
                    state[DH] = mrun;
                    state[DH + 1] = ltot;
                }
            }
            return;
        }
        if (head_ok) {
            const float inv = ltot > 0.f ? 1.0f / ltot : 0.f;
            const int64_t obase = (qrow * a.H + head) * DH;
            u32x2 gall[MB];  // all output-gate logits of this lane first, so that the loads overlap
            if (a.g1) {
#pragma unroll
                for (int mb = 0; mb < MB; ++mb)
                    gall[mb] = *reinterpret_cast<const u32x2*>(static_cast<const __bf16*>(a.g1) + obase + mb * 16 + 4 * q);
            }
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) {
                const int d0 = mb * 16 + 4 * q;
                float y[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) y[i] = o[mb][i] * inv;
                if (a.g1) {
                    const u32x2 gw = gall[mb];
                    y[0] *= sigmoid_f32(bf16_bits_to_f32(gw[0] & 0xffffu));
                    y[1] *= sigmoid_f32(bf16_bits_to_f32(gw[0] >> 16));
                    y[2] *= sigmoid_f32(bf16_bits_to_f32(gw[1] & 0xffffu));
                    y[3] *= sigmoid_f32(bf16_bits_to_f32(gw[1] >> 16));
                }
                u32x2 ow = {pack_bf16x2(y[0], y[1]), pack_bf16x2(y[2], y[3])};
                *reinterpret_cast<u32x2*>(static_cast<__bf16*>(a.out) + obase + d0) = ow;
            }
        }
    };

    if constexpr (DIRECT) {
        // ---- direct-to-LDS stream --------------------------------------------------------------------------------
        // One K tile and one V' tile per wave.  The K rows of the next tile are requested as soon as the score
        // product has read the current ones, its V' rows as soon as the value product has read the current ones:
        // each of the two streams is in flight while the other half of the arithmetic runs.  Tile slot s = 4 r + g
        // (load instruction r, lane group g = lane / 16) holds list entry j0 + s; lane p = lane % 16 of the group
        // fetches the 16-byte chunk p ^ (s & 15) of the K row and p ^ 2 (s & 7) of the V' row, which makes both the
        // 16-byte operand reads of K and the transposing reads of V' conflict-free on unpadded 256-byte rows.
        const int g4 = lane >> 4, p16 = lane & 15;
        uint32_t kcol[4], vcol[2];  // byte offset of this lane's chunk in the rows of load r: kcol[r & 3], vcol[r & 1]
#pragma unroll
        for (int r = 0; r < 4; ++r) kcol[r] = (uint32_t)(p16 ^ ((4 * r + g4) & 15)) * 16u;
#pragma unroll
        for (int r = 0; r < 2; ++r) vcol[r] = (uint32_t)(p16 ^ (2 * ((4 * r + g4) & 7))) * 16u;
        uint32_t kread[KK], vread[MB];  // LDS addresses of this lane's operand reads (sub-tile 1: + 4096)
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) kread[kk] = lds_addr(klds) + n * 256 + (((4 * kk + q) ^ n) << 4);
        {
            const int row = 4 * q + ((lane & 15) >> 2), c4 = lane & 3;
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
                vread[mb] = lds_addr(vlds) + row * 256 + ((2 * (mb ^ (row & 7)) + (c4 >> 1)) << 4) + (c4 & 1) * 8;
        }
        unsigned char* ilds = klds + 8192;  // list entries of the tile to request next: 64 x 4 bytes, the first 32 used
        // The query heads of a row take the same road: one transfer per four heads into a [heads][256 B] tile with the
        // K tile's chunk swizzle, read back as the B operand when the row starts.
        unsigned char* qlds = ilds + 256;
        const int qinstr = (G + 3) >> 2;
        uint32_t qread[KK];
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) qread[kk] = lds_addr(qlds) + n * 256 + (((4 * kk + q) ^ n) << 4);
        auto request_q = [&](int ri) {
            const unsigned char* qrow = static_cast<const unsigned char*>(a.Q) + (((int64_t)b * a.Lq + t0 + ri) * a.H + g * G) * ROWB;
            for (int i = 0; i < qinstr; ++i) {
                const int hh = min(4 * i + g4, G - 1);  // (heads past the group: a copy of the last one, never used)
                row_chunk_to_lds(qrow + hh * ROWB + ((p16 ^ ((4 * i + g4) & 15)) << 4), qlds + i * 1024);
            }
        };
        auto read_q = [&]() {
            u32x4 v[KK];
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) v[kk] = lds_read128_raw<0>(qread[kk]);
            wait_lds<0>(v[0], v[1], v[2], v[3]);
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) qf[kk] = __builtin_bit_cast(bf16x8, head_ok ? v[kk] : u32x4{0, 0, 0, 0});
        };
        const uint32_t iread = lds_addr(ilds) + g4 * 4;
        auto request_idx = [&](int ri, int j0, int je) {  // entries j0 .. of row ri (clamped to the piece) -> ilds[lane]
            const int32_t* row = idx0 + (int64_t)ri * a.k_cap;
            __builtin_amdgcn_global_load_lds((gmem_cv*)(row + min(j0 + lane, je - 1)), (lds_v*)ilds, 4, 0, 0);
        };
        auto read_idx = [&](int (&tk)[8]) {  // this lane's entries: slot 4 r + g4 for load instruction r
            tk[0] = lds_read32_raw<0>(iread);
            tk[1] = lds_read32_raw<16>(iread);
            tk[2] = lds_read32_raw<32>(iread);
            tk[3] = lds_read32_raw<48>(iread);
            tk[4] = lds_read32_raw<64>(iread);
            tk[5] = lds_read32_raw<80>(iread);
            tk[6] = lds_read32_raw<96>(iread);
            tk[7] = lds_read32_raw<112>(iread);
            wait_lds_all(tk);
            // clamped once for both tiles: a bad list reads wrong rows, never memory outside K / V'
#pragma unroll
            for (int r = 0; r < 8; ++r) {
                if constexpr (POOL)
                    tk[r] = (int)max((int64_t)0, min((int64_t)tk[r], a.pool_rows - 1));
                else
                    tk[r] = (int)__umul24((uint32_t)max(0, min(tk[r], a.Lk - 1)), tokstride);
            }
        };
        // (rows of one batch element span less than 4 GiB: 32-bit lane offsets on a wave-uniform base; pool: 64-bit)
        // (tk: what read_idx left: byte offsets of the rows, or clamped pool rows)
        auto request_rows = [&](const unsigned char* base, unsigned char* tile, const int (&tk)[8], const uint32_t* col, int colmask) {
#pragma unroll
            for (int r = 0; r < 8; ++r) {
                if constexpr (POOL)
                    row_chunk_to_lds(base + ((int64_t)tk[r] * tokstride + col[r & colmask]), tile + r * 1024);
                else
                    row_chunk_to_lds(base + ((uint32_t)tk[r] + col[r & colmask]), tile + r * 1024);
            }
        };
        auto request_k = [&](const int (&tk)[8]) { request_rows(Kb, klds, tk, kcol, 3); };
        auto request_v = [&](const int (&tk)[8]) { request_rows(Vb, vlds, tk, vcol, 1); };

        // The end of a row's piece (what finish_row does) in two steps,
        // so that what has to be read for it (the state the previous windows left, the output-gate logits) can be
        // requested while the row's last tile is still being multiplied.
        f32x4 st_o[MB];
        float st_m = 0.f, st_l = 0.f;
        u32x2 st_g1[MB];
        auto row_end_loads = [&](int ri) {
            const int flags = __builtin_amdgcn_readlane(m_flags, ri);
            const int t = t0 + ri;
            if (!head_ok) return;
            if (flags & 1) {
                const int64_t prow = (int64_t)b * a.part_rows + (t - a.part_row0);
                const float* const state = a.part + (((prow * a.H) + head) * rec_per_head + rec) * (DH + 4);
    #pragma unroll
                for (int mb = 0; mb < MB; ++mb) st_o[mb] = *reinterpret_cast<const f32x4*>(state + mb * 16 + 4 * q);
                st_m = state[DH];
                st_l = state[DH + 1];
            }
            if (!(flags & 2) && a.g1) {  // all output-gate logits of this lane together, so that the loads overlap
                const int64_t obase = (((int64_t)b * a.Lq + t) * a.H + head) * DH;
    #pragma unroll
                for (int mb = 0; mb < MB; ++mb)
                    st_g1[mb] = *reinterpret_cast<const u32x2*>(static_cast<const __bf16*>(a.g1) + obase + mb * 16 + 4 * q);
            }
        };
        auto row_end_finish = [&](int ri) {
            const int flags = __builtin_amdgcn_readlane(m_flags, ri);
            const int t = t0 + ri;
            const int64_t qrow = (int64_t)b * a.Lq + t;
            const int64_t prow = (int64_t)b * a.part_rows + (t - a.part_row0);
            float ltot = quad_row_sum(lrun);
            float* const state = a.part + (((prow * a.H) + (head_ok ? head : 0)) * rec_per_head + rec) * (DH + 4);
            if ((flags & 1) && head_ok) {  // merge with the state of the previous key windows
                const float M = fmaxf(mrun, st_m);
                const float wa = fast_exp2(mrun - M), wb = fast_exp2(st_m - M);
    #pragma unroll
                for (int mb = 0; mb < MB; ++mb) o[mb] = o[mb] * wa + st_o[mb] * wb;
                ltot = ltot * wa + st_l * wb;
                mrun = M;
            }
            if (flags & 2) {
                if (head_ok) {
    #pragma unroll
                    for (int mb = 0; mb < MB; ++mb) *reinterpret_cast<f32x4*>(state + mb * 16 + 4 * q) = o[mb];
                    if (q == 0) {
                        state[DH] = mrun;
                        state[DH + 1] = ltot;
                    }
                }
                return;
            }
            if (head_ok) {
                const float inv = ltot > 0.f ? 1.0f / ltot : 0.f;
                const int64_t obase = (qrow * a.H + head) * DH;
    #pragma unroll
                for (int mb = 0; mb < MB; ++mb) {
                    const int d0 = mb * 16 + 4 * q;
                    float y[4];
    #pragma unroll
                    for (int i = 0; i < 4; ++i) y[i] = o[mb][i] * inv;
                    if (a.g1) {
                        const u32x2 gw = st_g1[mb];
                        y[0] *= sigmoid_f32(bf16_bits_to_f32(gw[0] & 0xffffu));
                        y[1] *= sigmoid_f32(bf16_bits_to_f32(gw[0] >> 16));
                        y[2] *= sigmoid_f32(bf16_bits_to_f32(gw[1] & 0xffffu));
                        y[3] *= sigmoid_f32(bf16_bits_to_f32(gw[1] >> 16));
                    }
                    u32x2 ow = {pack_bf16x2(y[0], y[1]), pack_bf16x2(y[2], y[3])};
                    *reinterpret_cast<u32x2*>(static_cast<__bf16*>(a.out) + obase + d0) = ow;
                }
            }
        };
        auto finish_row_now = [&](int ri) {
            row_end_loads(ri);
            row_end_finish(ri);
        };

        int c_ri, c_j0 = 0, c_je = 0;
        c_ri = seek(0, c_j0, c_je);
        int n_ri = c_ri, n_j0 = c_j0, n_je = c_je;
        int p_ri = nrows, p_j0 = 0, p_je = 0;
        int tok_n[8];  // list entries (token numbers) of the tile whose rows are requested next
#pragma unroll
        for (int r = 0; r < 8; ++r) tok_n[r] = 0;
        if (c_ri < nrows) {
            // vector-memory order, here and in every pass of the loop: K rows, (query heads), list entries, V' rows
            request_idx(c_ri, c_j0, c_je);
            wait_vmem<0>();
            read_idx(tok_n);
            request_k(tok_n);
            request_q(c_ri);
            advance(n_ri, n_j0, n_je);
            p_ri = n_ri, p_j0 = n_j0, p_je = n_je;
            if (n_ri < nrows) {
                request_idx(n_ri, n_j0, n_je);
                advance(p_ri, p_j0, p_je);
            }
            request_v(tok_n);
        }
        int rows_done = 0, cur_row = -1;
        while (c_ri < nrows) {
            const bool has_n = n_ri < nrows, has_p = p_ri < nrows;
            const bool row_ends = c_j0 + 32 >= c_je;
            // K rows of this tile (and everything older: query heads, the next tile's list entries) have landed; its V'
            // rows may still fly
            wait_vmem<8>();
            if (c_ri != cur_row) {
                for (; rows_done < c_ri; ++rows_done) {
                    reset_acc();
                    finish_row_now(rows_done);
                }
                reset_acc();
                read_q();
                cur_row = c_ri;
            }
            u32x4 ka[KK], kb[KK];
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) ka[kk] = lds_read128_raw<0>(kread[kk]);
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) kb[kk] = lds_read128_raw<4096>(kread[kk]);
            f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
            wait_lds<4>(ka[0], ka[1], ka[2], ka[3]);
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, ka[kk]), qf[kk], s0, 0, 0, 0);
            wait_lds<0>(kb[0], kb[1], kb[2], kb[3]);
            if (has_n) {  // the K tile is free: next tile's K rows, then the list entries of the tile after it
                read_idx(tok_n);
                request_k(tok_n);
                if (n_ri != c_ri) request_q(n_ri);
                if (has_p) request_idx(p_ri, p_j0, p_je);
            }
            if (row_ends) row_end_loads(c_ri);  // (used after the value product)
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kb[kk]), qf[kk], s1, 0, 0, 0);
            // ---- online softmax of the 32 slots (as in the staged variant) ------------------------------------------
            const int j0 = c_j0, je = c_je;
            float x[8];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                x[i] = s0[i] * sl2;
                x[4 + i] = s1[i] * sl2;
            }
            if (j0 + 32 > je) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    if (j0 + 4 * q + i >= je) x[i] = kNegBig;
                    if (j0 + 16 + 4 * q + i >= je) x[4 + i] = kNegBig;
                }
            }
            float tmax = fmaxf(fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3])), fmaxf(fmaxf(x[4], x[5]), fmaxf(x[6], x[7])));
            tmax = quad_row_max(tmax);
            const float mnew = fmaxf(mrun, tmax);
            const float alpha = fast_exp2(mrun - mnew);
            float psum = 0.f;
            float pr[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                pr[i] = fast_exp2(x[i] - mnew);
                psum += pr[i];
            }
            lrun = lrun * alpha + psum;
            mrun = mnew;
            if (__any(alpha != 1.0f)) {
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) o[mb] *= alpha;
            }
            u32x4 pw = {pack_bf16x2(pr[0], pr[1]), pack_bf16x2(pr[2], pr[3]), pack_bf16x2(pr[4], pr[5]), pack_bf16x2(pr[6], pr[7])};
            const bf16x8 pf = __builtin_bit_cast(bf16x8, pw);
            // ---- the V' rows of this tile have landed (the requests made above may still fly) -----------------------
            if (has_n && has_p)
                wait_vmem<9>();
            else if (has_n)
                wait_vmem<8>();
            else
                wait_vmem<0>();
            s16x4 va[MB], vb[MB];
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) {
                va[mb] = lds_read_tr16_raw<0>(vread[mb]);
                vb[mb] = lds_read_tr16_raw<4096>(vread[mb]);
            }
            typedef __attribute__((ext_vector_type(8))) short s16x8;
#pragma unroll
            for (int h = 0; h < MB / 2; ++h) {
                if (h == 0) wait_lds<12>(va[0], vb[0], va[1], vb[1]);
                if (h == 1) wait_lds<8>(va[2], vb[2], va[3], vb[3]);
                if (h == 2) wait_lds<4>(va[4], vb[4], va[5], vb[5]);
                if (h == 3) wait_lds<0>(va[6], vb[6], va[7], vb[7]);
#pragma unroll
                for (int mb = 2 * h; mb < 2 * h + 2; ++mb) {
                    s16x8 av = {va[mb][0], va[mb][1], va[mb][2], va[mb][3], vb[mb][0], vb[mb][1], vb[mb][2], vb[mb][3]};
                    o[mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, av), pf, o[mb], 0, 0, 0);
                }
            }
            if (row_ends) {
                row_end_finish(c_ri);
                rows_done = c_ri + 1;
            }
            if (has_n) request_v(tok_n);  // the V' tile is free
            c_ri = n_ri, c_j0 = n_j0, c_je = n_je;
            n_ri = p_ri, n_j0 = p_j0, n_je = p_je;
            if (p_ri < nrows) advance(p_ri, p_j0, p_je);
        }
        for (; rows_done < nrows; ++rows_done) {
            reset_acc();
            finish_row_now(rows_done);
        }
    } else {
        // ---- the tile stream: c = tile being worked on, nx = tile whose rows are requested next, p = tile whose
        // indices are requested next ------------------------------------------------------------------------------
        int c_ri, c_j0 = 0, c_je = 0;
        c_ri = seek(0, c_j0, c_je);
        int n_ri = c_ri, n_j0 = c_j0, n_je = c_je;
        int p_ri = nrows, p_j0 = 0, p_je = 0;
        int tok_pref[NVL];
    #pragma unroll
        for (int r = 0; r < NVL; ++r) tok_pref[r] = 0;
        if (c_ri < nrows) {
            load_idx(c_ri, c_j0, c_je, tok_pref);
            issue(tok_pref);  // the one start-up chain of the wave: indices, then rows
            load_q(c_ri);
            advance(n_ri, n_j0, n_je);
            p_ri = n_ri, p_j0 = n_j0, p_je = n_je;
            if (n_ri < nrows) {
                load_idx(n_ri, n_j0, n_je, tok_pref);
                advance(p_ri, p_j0, p_je);
            }
        }
        int rows_done = 0;  // rows [0, rows_done) have been finished
        int cur_row = -1;   // row whose accumulators are live
        while (c_ri < nrows) {
            if (c_ri != cur_row) {  // first tile of a row
                for (; rows_done < c_ri; ++rows_done) {  // rows without a tile in this piece: only their state moves on
                    reset_acc();
                    finish_row(rows_done);
                }
                reset_acc();
    #pragma unroll
                for (int kk = 0; kk < KK; ++kk) qf[kk] = qf_next[kk];  // (before the next row's heads may be requested)
                cur_row = c_ri;
            }
            stage();
            if (n_ri < nrows) {  // the row registers are free again
                issue(tok_pref);
                if (n_ri != c_ri) load_q(n_ri);  // first tile of another row: its query heads come along
                if (p_ri < nrows) load_idx(p_ri, p_j0, p_je, tok_pref);
            }
            compute(c_j0, c_je);
            if (c_j0 + 32 >= c_je) {
                finish_row(c_ri);
                rows_done = c_ri + 1;
            }
            c_ri = n_ri, c_j0 = n_j0, c_je = n_je;
            n_ri = p_ri, n_j0 = p_j0, n_je = p_je;
            if (p_ri < nrows) advance(p_ri, p_j0, p_je);
        }
        for (; rows_done < nrows; ++rows_done) {
            reset_acc();
            finish_row(rows_done);
        }
    }
}

// Combine the partial results of a split row: out = (sum_s 2^(m_s - M) O_s) / (sum_s 2^(m_s - M) l_s) * sigmoid(g1).
// One wave per (row, head); lane s first takes the statistics of piece s (at most 64 pieces), then every
// lane sums DH/64 output features over the pieces.
template <int DH>
__global__ __launch_bounds__(256) void attn_merge_kernel(AttnArgs a) {
    constexpr int PS = DH + 4;  // floats per partial record (16-byte multiple)
    constexpr int DPL = DH / 64;
    const int lane = threadIdx.x & 63;
    const int R = a.row_end - a.row_begin;
    const int64_t rh = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);  // (row, head)
    if (rh >= (int64_t)a.B * R * a.H) return;
    const int64_t rid = rh / a.H;
    const int head = (int)(rh % a.H);
    const int b = (int)(rid / R);
    const int t = a.row_begin + (int)(rid % R);
    const int ns = a.nsplit;
    const float* pp = a.part + rh * a.nsplit * PS;
    const float m = lane < ns ? pp[lane * PS + DH] : kNegBig;
    const float l = lane < ns ? pp[lane * PS + DH + 1] : 0.f;
    float M = m;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) M = fmaxf(M, __shfl_xor(M, o, 64));
    const float wgt = lane < ns ? fast_exp2(m - M) : 0.f;
    const float L = wave_sum(wgt * l);
    float acc[DPL];
#pragma unroll
    for (int e = 0; e < DPL; ++e) acc[e] = 0.f;
    for (int sp = 0; sp < ns; ++sp) {
        const float w = __shfl(wgt, sp, 64);
#pragma unroll
        for (int e = 0; e < DPL; ++e) acc[e] = fmaf(w, pp[sp * PS + lane * DPL + e], acc[e]);
    }
    const int64_t oi = (((int64_t)b * a.Lq + t) * a.H + head) * DH + lane * DPL;
    uint32_t packed = 0;
#pragma unroll
    for (int e = 0; e < DPL; ++e) {
        float y = L > 0.f ? acc[e] / L : 0.f;
        if (a.g1) y *= sigmoid_f32(bf16_bits_to_f32(static_cast<const uint16_t*>(a.g1)[oi + e]));
        packed |= f32_to_bf16_bits(y) << (16 * e);
    }
    if (DPL == 2)
        *reinterpret_cast<uint32_t*>(static_cast<uint16_t*>(a.out) + oi) = packed;
    else
        static_cast<uint16_t*>(a.out)[oi] = (uint16_t)packed;
}

// Key-window mode: positions in a row's ascending index list where the key windows begin.
//   winoff[row][z] = number of selected keys below z * window   (z = 0 .. nwin; winoff[row][nwin] = n_sel)
// One wave per row: 64 evenly spaced probes of the list bracket every boundary, a second probe of the
// bracket pins it down.
__global__ __launch_bounds__(256) void attn_window_offsets_kernel(AttnArgs a, int32_t* winoff) {
    const int lane = threadIdx.x & 63;
    const int R = a.row_end - a.row_begin;
    const int64_t rid = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (rid >= (int64_t)a.B * R) return;
    const int b = (int)(rid / R);
    const int t = a.row_begin + (int)(rid % R);
    const int nsel = max(0, min(a.n_sel[(int64_t)b * a.Lq + t], a.k_cap));
    const int32_t* idxrow = a.idx + ((int64_t)b * a.idx_rows + (t - a.idx_row0)) * a.k_cap;
    int32_t* off = winoff + rid * (a.nsplit + 1);
    const int nwin = a.nsplit;
    if (lane == 0) {
        off[0] = 0;
        off[nwin] = nsel;
    }
    if (nsel == 0) {
        for (int z = 1 + lane; z < nwin; z += 64) off[z] = 0;
        return;
    }
    const int step = (nsel + 63) >> 6;
    const bool probe_ok = lane * step < nsel;
    const int probe = probe_ok ? idxrow[lane * step] : 0;
    for (int z = 1; z < nwin; ++z) {
        const int target = z * a.window;
        // c probes are below the target: the boundary lies in ((c-1)*step, c*step]
        const int c = __popcll(__ballot(probe_ok && probe < target));
        int pos = 0;
        if (c > 0) {
            const int s0 = (c - 1) * step + 1;
            const int s1 = min(c * step, nsel);  // exclusive end of the bracket
            pos = s0;
            for (int j0 = s0; j0 < s1; j0 += 64) {
                const int j = j0 + lane;
                const bool below = j < s1 && idxrow[j] < target;
                pos += __popcll(__ballot(below));
            }
        }
        if (lane == 0) off[z] = pos;
    }
}

// fp32 kernel: plain vector arithmetic, one wave per query head, online softmax over chunks of 64
// selected tokens (a lane computes one token's logit; then every lane owns DH/64 output features).
template <int DH>
__global__ __launch_bounds__(256) void attn_f32_kernel(AttnArgs a) {
    constexpr int DPL = DH / 64;  // features per lane (1 or 2)
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int R = a.row_end - a.row_begin;
    const int64_t rid = blockIdx.x;
    const int b = (int)(rid / R);
    const int t = a.row_begin + (int)(rid % R);
    const int64_t qrow = (int64_t)b * a.Lq + t;
    const int nsel = max(0, min(a.n_sel[qrow], a.k_cap));
    const int64_t row0 = a.pool_rows ? 0 : (int64_t)b * a.Lk;  // first row of this batch element's K / V
    const int32_t* idxrow = a.idx + ((int64_t)b * a.idx_rows + (t - a.idx_row0)) * a.k_cap;
    const int G = a.H / a.H_kv;
    const float* Q = static_cast<const float*>(a.Q);
    const float* K = static_cast<const float*>(a.K);
    const float* V = static_cast<const float*>(a.V);
    const float* G2 = static_cast<const float*>(a.g2);
    const float* G1 = static_cast<const float*>(a.g1);
    float* out = static_cast<float*>(a.out);

    for (int h = wv; h < a.H; h += 4) {
        const int g = h / G;
        const float* qp = Q + (qrow * a.H + h) * DH;
        float mrun = kNegBig, lrun = 0.f;
        float o[DPL];
#pragma unroll
        for (int e = 0; e < DPL; ++e) o[e] = 0.f;
        for (int j0 = 0; j0 < nsel; j0 += 64) {
            const int j = j0 + lane;
            int tok = idxrow[min(j, nsel - 1)];
            tok = (int)max((int64_t)0, min((int64_t)tok, (a.pool_rows ? a.pool_rows : (int64_t)a.Lk) - 1));
            const int64_t krow = ((row0 + tok) * a.H_kv + g) * DH;
            float acc = 0.f;
            for (int c = 0; c < DH; c += 4) {
                const float4 kv = *reinterpret_cast<const float4*>(K + krow + c);
                const float4 qv = *reinterpret_cast<const float4*>(qp + c);
                acc = fmaf(qv.x, kv.x, acc);
                acc = fmaf(qv.y, kv.y, acc);
                acc = fmaf(qv.z, kv.z, acc);
                acc = fmaf(qv.w, kv.w, acc);
            }
            const float x = j < nsel ? acc * a.scale : kNegBig;
            float cmax = x;
#pragma unroll
            for (int s = 32; s > 0; s >>= 1) cmax = fmaxf(cmax, __shfl_xor(cmax, s, 64));
            const float mnew = fmaxf(mrun, cmax);
            const float alpha = expf(mrun - mnew);
            const float p = j < nsel ? expf(x - mnew) : 0.f;
            lrun = lrun * alpha + wave_sum(p);
            mrun = mnew;
#pragma unroll
            for (int e = 0; e < DPL; ++e) o[e] *= alpha;
            const int cnt = min(64, nsel - j0);
            for (int u = 0; u < cnt; ++u) {
                const float pu = __shfl(p, u, 64);
                const int tu = __shfl(tok, u, 64);
                const int64_t vrow = ((row0 + tu) * a.H_kv + g) * DH;
#pragma unroll
                for (int e = 0; e < DPL; ++e) {
                    float v = V[vrow + lane + 64 * e];
                    if (G2) v *= 1.0f / (1.0f + expf(-G2[vrow + lane + 64 * e]));
                    o[e] = fmaf(pu, v, o[e]);
                }
            }
        }
        const float inv = lrun > 0.f ? 1.0f / lrun : 0.f;
#pragma unroll
        for (int e = 0; e < DPL; ++e) {
            const int64_t oi = (qrow * a.H + h) * DH + lane + 64 * e;
            float y = o[e] * inv;
            if (G1) y *= 1.0f / (1.0f + expf(-G1[oi]));
            out[oi] = y;
        }
    }
}

// Value gate as a dense pre-pass: Vg = V * sigmoid(g2), 8 elements (bf16) or 4 (f32) per thread.
__global__ void value_gate_bf16_kernel(const u32x4* V, const u32x4* g2, u32x4* Vg, int64_t nchunks) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= nchunks) return;
    u32x4 v = V[i];
    const u32x4 g = g2[i];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const float v0 = bf16_bits_to_f32(v[e] & 0xffffu) * sigmoid_f32(bf16_bits_to_f32(g[e] & 0xffffu));
        const float v1 = bf16_bits_to_f32(v[e] >> 16) * sigmoid_f32(bf16_bits_to_f32(g[e] >> 16));
        v[e] = pack_bf16x2(v0, v1);
    }
    Vg[i] = v;
}
__global__ void value_gate_f32_kernel(const float4* V, const float4* g2, float4* Vg, int64_t nchunks) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= nchunks) return;
    float4 v = V[i];
    const float4 g = g2[i];
    v.x *= 1.0f / (1.0f + expf(-g.x));
    v.y *= 1.0f / (1.0f + expf(-g.y));
    v.z *= 1.0f / (1.0f + expf(-g.z));
    v.w *= 1.0f / (1.0f + expf(-g.w));
    Vg[i] = v;
}

hipError_t launch_value_gate(const gsa_shape& sh, const void* V, const void* g2, void* Vg, hipStream_t st) {
    const int64_t elems = (int64_t)sh.B * sh.Lk * sh.H_kv * sh.d_h;
    if (sh.dtype == GSA_BF16) {
        const int64_t nch = elems / 8;
        hipLaunchKernelGGL(value_gate_bf16_kernel, dim3((unsigned)cdiv(nch, 256)), dim3(256), 0, st,
                           static_cast<const u32x4*>(V), static_cast<const u32x4*>(g2), static_cast<u32x4*>(Vg), nch);
    } else {
        const int64_t nch = elems / 4;
        hipLaunchKernelGGL(value_gate_f32_kernel, dim3((unsigned)cdiv(nch, 256)), dim3(256), 0, st,
                           static_cast<const float4*>(V), static_cast<const float4*>(g2), static_cast<float4*>(Vg), nch);
    }
    return hipGetLastError();
}

// kv heads handled by one workgroup (one wave each).  With many query rows the kv heads are cut
// into slices that are processed one after the other by the whole chip (see the kernel), sized so
// that a slice of K and V' stays near 64 MiB; with few rows (decode) one workgroup takes up to four.
static int attn_groups_per_block(const gsa_shape& sh, int64_t rows, const gsa_tuning& tn) {
    int gpb = sh.H_kv < 4 ? sh.H_kv : 4;
    while (sh.H_kv % gpb != 0) --gpb;
    if (tn.attn_kv_per_wg >= 1 && tn.attn_kv_per_wg <= 4 && sh.H_kv % tn.attn_kv_per_wg == 0) return tn.attn_kv_per_wg;
    if (rows < 4096) return gpb;
    const double slice_target = 64.0 * 1024 * 1024;
    while (gpb > 1 && (double)sh.B * sh.Lk * gpb * sh.d_h * 2 * 2 > slice_target && sh.H_kv % (gpb / 2) == 0) gpb /= 2;
    return gpb;
}

// Pieces a row's selected list is cut into (bf16 path): 1 when the launch has enough workgroups anyway,
// otherwise enough to reach about a thousand workgroups, at least two 32-token tiles per piece.
static int attn_splits(const gsa_shape& sh, int64_t rows, int k_cap, const gsa_tuning& tn) {
    if (sh.dtype != GSA_BF16) return 1;
    const int gpb = attn_groups_per_block(sh, rows, tn);
    const int64_t wgs = rows * (sh.H_kv / gpb);
    if (wgs >= 1024) return 1;
    int64_t by_len = cdiv(cdiv(k_cap, 32), 2);
    if (by_len < 1) by_len = 1;
    int64_t ns = cdiv(1024, wgs);
    if (ns > by_len) ns = by_len;
    if (ns > 64) ns = 64;
    return (int)(ns < 1 ? 1 : ns);
}

// Query rows a wave of the bf16 kernel streams through: as many as still leave about four thousand workgroups.
static int attn_rows_per_wave(int64_t lrows, int slices, bool direct, const gsa_tuning& tn) {
    if (tn.attn_rows_per_wave > 0) return tn.attn_rows_per_wave < 64 ? tn.attn_rows_per_wave : 64;
    const int64_t r = lrows * slices / 4096, cap = direct ? 4 : 8;  // (measured: C4, 30.6 ms with 4, 30.8 with 8)
    return (int)(r < 1 ? 1 : (r > cap ? cap : r));
}

// The direct-to-LDS variant of the bf16 kernel: gated values given, 256-byte rows.
static bool attn_direct(const gsa_shape& sh, const void* g2) { return GSA_ATTN_DIRECT && sh.dtype == GSA_BF16 && sh.d_h == 128 && !g2; }

// Key-window mode (bf16, many rows, long context): keys per window, 0 = off.  The K/V' rows of one window
// and kv-head slice (window * kv heads per workgroup * d_h * 4 bytes) then stay largely resident in the
// 4 MB L2 of every XCD while all rows gather from them, instead of every gather going out to the
// memory-side cache.  Two forces set the size.  A row needs enough selected keys per window to amortise
// the start of a row's piece: 256 * Lk / k_cap keys per window leave the longest rows about k_cap/16 keys
// (eight 32-key tiles) per window.  The footprint has to stay near the L2 size: it is kept between
// 2 MiB and 8 MiB whatever the head dimension.  (Measured at 128K context, k_cap 4096, direct-to-LDS kernel:
// 8192 keys 30.6 ms, 10240 30.9, 12288 32.2, 6144 33.0, 16384 38.3.)
static int attn_window(const gsa_shape& sh, int64_t rows, int k_cap, const gsa_tuning& tn) {
    if (tn.attn_window < 0 || sh.dtype != GSA_BF16) return 0;
    int w;
    const bool forced = tn.attn_window > 0;
    if (forced) {
        w = tn.attn_window;
    } else {
        const int gpb = attn_groups_per_block(sh, rows, tn);
        const int64_t key_bytes = (int64_t)gpb * sh.d_h * 4;  // K row + V' row of the kv heads a workgroup works on
        int64_t w64 = 256 * (int64_t)sh.Lk / (k_cap > 0 ? k_cap : 1);
        const int64_t w_lo = (2 << 20) / key_bytes, w_hi = (8 << 20) / key_bytes;
        w64 = w64 < w_lo ? w_lo : (w64 > w_hi ? w_hi : w64);
        w = (int)((w64 + 512) / 1024 * 1024);
    }
    if (w <= 0 || sh.Lk <= w) return 0;
    if (!forced && (rows < 8192 || sh.Lk < 2 * w)) return 0;
    if (!forced && (int64_t)w * k_cap < 128 * (int64_t)sh.Lk) return 0;  // too few keys per window to pay for a launch each
    if (cdiv(sh.Lk, w) > 64) w = (int)((cdiv(sh.Lk, 64) + 31) / 32 * 32);  // at most 64 windows
    return w;
}

size_t attn_workspace_bytes(const gsa_shape& sh, int row_begin, int row_end, int k_cap, const gsa_tuning& tn) {
    const int64_t rows = (int64_t)sh.B * (row_end - row_begin);
    if (const int w = attn_window(sh, rows, k_cap, tn)) {
        const int64_t nwin = cdiv(sh.Lk, w);
        const size_t offs = ((size_t)rows * (nwin + 1) * sizeof(int32_t) + 255) & ~(size_t)255;
        return offs + (size_t)rows * sh.H * (sh.d_h + 4) * sizeof(float);  // window offsets + one running state per head
    }
    const int ns = attn_splits(sh, rows, k_cap, tn);
    return ns > 1 ? (size_t)rows * sh.H * ns * (sh.d_h + 4) * sizeof(float) : 0;
}

hipError_t launch_attention(const gsa_shape& sh, int row_begin, int row_end, const void* Q, const void* K, const void* V,
                            const void* g2, const void* g1, const int32_t* idx, int idx_rows, int idx_row0,
                            const int32_t* n_sel, int k_cap, float scale, void* out, void* workspace, const gsa_tuning& tn,
                            int64_t pool_rows, hipStream_t st) {
    AttnArgs a;
    a.pool_rows = pool_rows;
    a.Q = Q;
    a.K = K;
    a.V = V;
    a.g2 = g2;
    a.g1 = g1;
    a.idx = idx;
    a.n_sel = n_sel;
    a.out = out;
    a.B = sh.B;
    a.Lq = sh.Lq;
    a.Lk = sh.Lk;
    a.H = sh.H;
    a.H_kv = sh.H_kv;
    a.row_begin = row_begin;
    a.row_end = row_end;
    a.k_cap = k_cap;
    a.idx_rows = idx_rows;
    a.idx_row0 = idx_row0;
    a.scale = scale;
    const int64_t rows = (int64_t)sh.B * (row_end - row_begin);
    a.winoff = nullptr;
    a.window = attn_window(sh, rows, k_cap, tn);
    a.win = 0;
    a.q_offset = sh.q_offset;
    a.part_row0 = row_begin;
    a.part_rows = row_end - row_begin;
    a.rpw = 1;
    if (a.window) {
        a.nsplit = (int)cdiv(sh.Lk, a.window);
        const size_t offs = ((size_t)rows * (a.nsplit + 1) * sizeof(int32_t) + 255) & ~(size_t)255;
        int32_t* winoff = static_cast<int32_t*>(workspace);
        a.part = reinterpret_cast<float*>(static_cast<unsigned char*>(workspace) + offs);
        hipLaunchKernelGGL(attn_window_offsets_kernel, dim3((unsigned)cdiv(rows, 4)), dim3(256), 0, st, a, winoff);
        a.winoff = winoff;
    } else {
        a.nsplit = attn_splits(sh, rows, k_cap, tn);
        a.part = static_cast<float*>(workspace);
    }
    if (sh.dtype == GSA_BF16) {
        const int gpb = attn_groups_per_block(sh, rows, tn);
        const dim3 block(64 * gpb);
        // gated values given, 256-byte rows: K and V' rows go straight into LDS (per wave two unpadded 8 KB tiles, 256 bytes of list entries, 1 KB per four query heads)
        const bool direct = attn_direct(sh, g2);
        const size_t smem = direct ? (size_t)gpb * (16640 + 1024 * ((sh.H / sh.H_kv + 3) / 4))
                                   : (size_t)gpb * 32 * ((sh.d_h * 2 + 32) + (sh.d_h * 2 + 16));  // V' tile + K tile per wave
        // one launch, or in key-window mode one launch per window over the rows that can see it
        const int nlaunch = a.window ? a.nsplit : 1;
        for (int z = 0; z < nlaunch; ++z) {
            if (a.window) {
                a.win = z;
                a.row_begin = row_begin > z * a.window - sh.q_offset ? row_begin : z * a.window - sh.q_offset;
                if (a.row_begin >= row_end) break;
            }
            const int lrows = row_end - a.row_begin;  // per batch element
            a.rpw = attn_rows_per_wave((int64_t)sh.B * lrows, sh.H_kv / gpb, direct, tn);
            const dim3 grid((unsigned)(sh.B * cdiv(lrows, a.rpw)), (unsigned)(sh.H_kv / gpb), (unsigned)(a.window ? 1 : a.nsplit));
            void (*kern)(AttnArgs) = sh.d_h == 128 ? (g2 ? attn_bf16_kernel<128, true> : attn_bf16_kernel<128, false>)
                                                   : (g2 ? attn_bf16_kernel<64, true> : attn_bf16_kernel<64, false>);
            if (pool_rows)  // (paged caches hold gated values: no g2 here, checked by the caller)
                kern = sh.d_h == 128 ? attn_bf16_kernel<128, false, true> : attn_bf16_kernel<64, false, true>;
            if (direct) kern = pool_rows ? attn_bf16_kernel<128, false, true, true> : attn_bf16_kernel<128, false, false, true>;
            if (z == 0 && smem > 48 * 1024) {
                hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
                if (e != hipSuccess) return e;
            }
            hipLaunchKernelGGL(kern, grid, block, smem, st, a);
        }
        a.row_begin = row_begin;
        if (a.nsplit > 1 && !a.window) {
            hipError_t e = hipGetLastError();
            if (e != hipSuccess) return e;
            const dim3 mgrid((unsigned)cdiv(rows * sh.H, 4));
            if (sh.d_h == 128)
                hipLaunchKernelGGL(attn_merge_kernel<128>, mgrid, dim3(256), 0, st, a);
            else
                hipLaunchKernelGGL(attn_merge_kernel<64>, mgrid, dim3(256), 0, st, a);
        }
    } else {
        if (sh.d_h == 128)
            hipLaunchKernelGGL(attn_f32_kernel<128>, dim3((unsigned)rows), dim3(256), 0, st, a);
        else
            hipLaunchKernelGGL(attn_f32_kernel<64>, dim3((unsigned)rows), dim3(256), 0, st, a);
    }
    return hipGetLastError();
}

}  // namespace gsa
