// Gated lightning indexer (Sec. 3.3, Eq. "indexer") with the row statistics that the adaptive
// controller of Sec. 3.4 consumes.
//
//   I[t,s] = sum_j w[t,j] * sigmoid(qI[t,j,:] . kI[s,:] + bI[j]),   s <= min(q_offset + t, Lk-1)
//
// Mapping to the matrix cores.  The logits of all heads of a block of queries form one GEMM
// C[(t,j), s] = A[(t,j), :] . B[s, :] with M = queries x heads (head fastest), N = keys, K = dI.
// A 32x32 MFMA accumulator leaves, in every lane, sixteen rows of one key column; with the head
// index fastest in M those sixteen rows are whole groups of heads of a few queries, so the
// sigmoid, the head weighting and the head sum all happen inside one lane, with no cross-lane
// traffic.  The keys of a 128-key tile are dealt to the four column blocks round-robin (column n of
// block nb is key 4n + nb), so after a tile a lane owns four consecutive keys per row and score rows
// are written with 16-byte stores, 512 contiguous bytes per wave and row.
//
// A workgroup is four waves; each wave owns 32 M-rows (32/HI queries) and keeps its A fragments
// in registers for the whole key loop.  Key tiles of 128 tokens are staged through LDS (double
// buffered, one barrier per tile) and shared by the four waves.  Tiles above the causal diagonal
// are skipped, tiles crossing it take a masked epilogue.
//
// Row statistics: every lane accumulates sum(d) and sum(d^2) of d = I - c_t, c_t = (1/2) sum_j w[t,j]
// (the row mean when logits are symmetric), which removes the cancellation of the one-pass
// variance formula.  The key range of a row may be split over several workgroups (grid.y); each
// writes its partial sums to the workspace and a second small kernel merges them in double
// precision into row_mean / row_var.
#include "common.hpp"

namespace gsa {

struct IndexerArgs {
    const void* qI;
    const void* kI;
    const float* w;
    const float* bI;
    float* scores;
    uint16_t* keys;  // alternative to scores: 16-bit keys, same indexing
    int64_t ld;
    float2* partial;  // [B][R][nsplit][4]
    int32_t B, Lq, Lk, q_offset, row_begin, row_end;
    int32_t kc;      // keys per split (multiple of 128)
    int32_t nsplit;
    int32_t ntiles;  // query tiles in the slab
    const int32_t* seq_lens;  // per-sequence lengths (ragged decode) or null
    int32_t hi;      // indexer heads in memory (the kernels work on the next power of two, the extra heads weigh zero)
    PageMap pm;      // where the rows of kI live (contiguous tensor or pages of a pool)
};

constexpr int kBN = 128;  // keys per LDS tile

template <typename T>
struct ElemTraits;
template <>
struct ElemTraits<__bf16> {
    static constexpr int kBytes = 2;
};
template <>
struct ElemTraits<float> {
    static constexpr int kBytes = 4;
};

// Row (t,j) index m of accumulator register i in lane half h (l/32) of a 32x32 MFMA result.
__device__ __forceinline__ constexpr int acc_row(int i, int h) { return 8 * (i / 4) + 4 * h + (i % 4); }

// STORE: 0 = statistics only, 1 = fp32 scores, 2 = 16-bit fixed-point keys floor(score * 65536 / HI)
// (saturated at 65535), a monotone compression of the score used inside the fused forward.
// ROW1: the launch covers one query row per batch element (decode); such launches get a kernel of their
// own so that the deeper prefetch of that case does not cost the prefill loops any registers.
// HI is the head count the kernel is built for (1, 2, 4 or 8); a.hi <= HI heads exist in memory, the others
// are given zero queries and zero weights, which adds exact zeros to every sum.
// RELU: the comparison variant of Sec. 2.2 Eq. 3 (ReLU instead of the sigmoid; statistics centred at zero).
template <typename T, int DI, int HI, int STORE, bool ROW1, bool RELU = false>
__global__ __launch_bounds__(256, STORE == 0 ? 3 : 2) void indexer_kernel(IndexerArgs a) {
    static_assert(!(RELU && STORE == 2), "16-bit keys need the bounded scores of the sigmoid indexer");
    constexpr int EB = ElemTraits<T>::kBytes;
    constexpr int ROWB = DI * EB;            // bytes of one key row
    constexpr int LDSROW = ROWB + 16;        // padded LDS row stride
    constexpr int NCH = kBN * ROWB / 16 / 256;  // 16-byte chunks staged per thread per tile
    constexpr int CHPR = ROWB / 16;          // chunks per key row
    constexpr int QW = 32 / HI;              // queries per wave
    constexpr int QT = 4 * QW;               // queries per workgroup
    constexpr int HL = HI < 4 ? HI : 4;      // heads of one query held by a lane
    constexpr int NSLOT = 16 / HL;           // (query) slots per lane
    constexpr bool kIsBf16 = (EB == 2);
    constexpr int KSTEPS = kIsBf16 ? DI / 16 : DI / 2;

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];  // 2 * kBN * LDSROW

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wv = tid >> 6;
    const int h = lane >> 5;   // lane half
    const int n = lane & 31;   // column (key) within an N-block / row within A
    const int b = blockIdx.z;
    const int split = blockIdx.y;
    const int tile = a.ntiles - 1 - (int)blockIdx.x;  // longest rows first
    const int R = a.row_end - a.row_begin;

    const int t_wg0 = a.row_begin + tile * QT;
    // A workgroup whose rows all fit in one wave's share (decode, or the ragged last tile) runs "narrow":
    // its four waves take the same rows and split the column blocks of every key tile between them.
    const bool narrow = (a.row_end - t_wg0) <= QW;
    const int t_w0 = narrow ? t_wg0 : t_wg0 + wv * QW;
    const int t_wg_last = min(t_wg0 + QT, a.row_end) - 1;
    const int qoff = batch_q_offset(a.seq_lens, b, a.q_offset, a.Lq, a.Lk);
    const int kmax_wg = min(qoff + t_wg_last, a.Lk - 1);  // last key any row of the workgroup sees
    const int key_lo = split * a.kc;
    const int key_hi = min(key_lo + a.kc, kmax_wg + 1);         // exclusive

    // ---- per-lane slot bookkeeping -------------------------------------------------------
    // Score rows of this wave start at a wave-uniform base; a lane adds a 32-bit element offset.
    float* const wave_scores = STORE == 1 ? a.scores + ((int64_t)b * R + (t_w0 - a.row_begin)) * a.ld : nullptr;
    uint16_t* const wave_keys = STORE == 2 ? a.keys + ((int64_t)b * R + (t_w0 - a.row_begin)) * a.ld : nullptr;
    // In key mode the head weights carry the key scale 65536/HI (a power of two, so every product and
    // sum is the scaled image of the unscaled one, bit for bit); the statistics are unscaled on the way out.
    constexpr float kKeyScale = STORE == 2 ? 65536.0f / HI : 1.0f;
    // Query of slot s relative to the wave: a wave-uniform part plus a multiple of the lane half.
    //   tl(s, h) = acc_row(s * HL, h) / HI = slot_row(s) + kHalfRows * h
    constexpr int kHalfRows = HI <= 4 ? 4 / HI : 0;
    auto slot_row = [](int s) { return acc_row(s * HL, 0) / HI; };
    // last visible key of the slot's query, -1 if the query is outside the row range (recomputed where
    // it is needed: the masked tiles at the diagonal and the final reduction)
    auto lim_of = [&](int s) {
        const int t = t_w0 + slot_row(s) + kHalfRows * h;
        return t < a.row_end ? min(qoff + t, a.Lk - 1) : -1;
    };
    // element offset of a slot's score row from the wave's base: lane part here, uniform part at the use
    const uint32_t half_off = (uint32_t)(kHalfRows * h) * (uint32_t)a.ld;
    auto row_off = [&](int s) { return (uint32_t)slot_row(s) * (uint32_t)a.ld; };  // wave-uniform
    float wreg[16];         // head weight of accumulator register i
    float nbias[HL];        // -log2(e) * bias of the lane's r-th head
    float center[NSLOT];
    float s1[NSLOT], s2[NSLOT];
    bool slot_live[NSLOT];  // wave-uniform: some lane of the wave has a valid row in this slot
#pragma unroll
    for (int r = 0; r < HL; ++r) {
        const int j = (HI == 8) ? 4 * h + r : r;  // head of accumulator register s*HL + r
        nbias[r] = (a.bI && j < a.hi) ? (RELU ? a.bI[j] : -kLog2e * a.bI[j]) : 0.f;  // ReLU: the bias itself
    }
#pragma unroll
    for (int s = 0; s < NSLOT; ++s) {
        const int tl = acc_row(s * HL, h) / HI;  // query of the slot, relative to the wave
        const int t = t_w0 + tl;
        const bool ok = t < a.row_end;
        slot_live[s] = __any(ok) != 0;
        float c = 0.f;
#pragma unroll
        for (int r = 0; r < HL; ++r) {
            const int j = (HI == 8) ? 4 * h + r : r;
            const float wv_ = (ok && j < a.hi) ? a.w[((int64_t)b * a.Lq + t) * a.hi + j] : 0.f;
            wreg[s * HL + r] = wv_ * kKeyScale;
            c += 0.5f * (wv_ * kKeyScale);
        }
        if (HI == 8) c += __shfl_xor(c, 32, 64);
        center[s] = RELU ? 0.f : c;
        s1[s] = 0.f;
        s2[s] = 0.f;
    }

    if (key_lo < key_hi) {
        // ---- A fragments: rows (t,j) of this wave, kept for the whole key loop ------------
        // bf16: register kk holds k = 16*kk + 8*h .. +8.   f32: register kk holds k = h*DI/2 + kk.
        bf16x8 afrag_b[kIsBf16 ? KSTEPS : 1];
        float afrag_f[kIsBf16 ? 1 : KSTEPS];
        {
            const int t = t_w0 + n / HI;
            const bool ok = t < a.row_end && (n % HI) < a.hi;
            const int64_t row = ((int64_t)b * a.Lq + (ok ? t : a.row_begin)) * a.hi + (ok ? n % HI : 0);
            if constexpr (kIsBf16) {
                const u32x4* src = reinterpret_cast<const u32x4*>(static_cast<const __bf16*>(a.qI) + row * DI);
#pragma unroll
                for (int kk = 0; kk < KSTEPS; ++kk) {
                    u32x4 v = ok ? src[kk * 2 + h] : u32x4{0, 0, 0, 0};
                    afrag_b[kk] = __builtin_bit_cast(bf16x8, v);
                }
            } else {
                const float4* src = reinterpret_cast<const float4*>(static_cast<const float*>(a.qI) + row * DI + h * (DI / 2));
#pragma unroll
                for (int c4 = 0; c4 < DI / 8; ++c4) {
                    float4 v = ok ? src[c4] : float4{0.f, 0.f, 0.f, 0.f};
                    afrag_f[c4 * 4 + 0] = v.x;
                    afrag_f[c4 * 4 + 1] = v.y;
                    afrag_f[c4 * 4 + 2] = v.z;
                    afrag_f[c4 * 4 + 3] = v.w;
                }
            }
        }

        // limits of this wave (uniform): first/last visible key over its valid rows
        const int t_w_last = min(t_w0 + QW, a.row_end) - 1;
        const bool wave_has_rows = t_w0 < a.row_end;
        const bool wave_rows_full = (t_w0 + QW) <= a.row_end;
        const int lim_first = min(qoff + t_w0, a.Lk - 1);
        const int lim_last = wave_has_rows ? min(qoff + t_w_last, a.Lk - 1) : -1;

        // First row of the key tile that starts at token s0 (a multiple of kBN; pages hold a multiple of kBN tokens,
        // so a tile never straddles two).  Tiles beyond the last one any row of the workgroup sees are only ever
        // requested by prefetches that run ahead: they read that last tile instead (with paged caches the pages
        // beyond a sequence's end need not exist).
        const int last_tile = kmax_wg & ~(kBN - 1);
        auto tile_ptr = [&](int s0) {
            return static_cast<const unsigned char*>(a.kI) + cache_row(a.pm, b, min(s0, last_tile), a.Lk) * ROWB;
        };
        u32x4 stage[NCH];
        auto load_tile = [&](int s0) {
            const unsigned char* tp = tile_ptr(s0);
#pragma unroll
            for (int c = 0; c < NCH; ++c) {
                const int ch = tid + c * 256;
                const int r = ch / CHPR;
                const int col = ch % CHPR;
                const int s = s0 + r;
                stage[c] = (s < a.Lk) ? *reinterpret_cast<const u32x4*>(tp + r * ROWB + col * 16) : u32x4{0, 0, 0, 0};
            }
        };
        auto store_tile = [&](int buf) {
            unsigned char* dst = smem + buf * (kBN * LDSROW);
#pragma unroll
            for (int c = 0; c < NCH; ++c) {
                const int ch = tid + c * 256;
                const int r = ch / CHPR;  // key within the tile; it is placed at LDS row (r % 4) * 32 + r / 4
                const int col = ch % CHPR;
                *reinterpret_cast<u32x4*>(dst + ((r & 3) * 32 + (r >> 2)) * LDSROW + col * 16) = stage[c];
            }
        };
        auto mfma_block = [&](const unsigned char* tileptr, int nb) -> f32x16 {
            f32x16 c = {0};
            const unsigned char* rowp = tileptr + (nb * 32 + n) * LDSROW;
            if constexpr (kIsBf16) {
#pragma unroll
                for (int kk = 0; kk < KSTEPS; ++kk) {
                    u32x4 v = *reinterpret_cast<const u32x4*>(rowp + kk * 32 + h * 16);
                    c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(afrag_b[kk], __builtin_bit_cast(bf16x8, v), c, 0, 0, 0);
                }
            } else {
#pragma unroll
                for (int c4 = 0; c4 < DI / 8; ++c4) {
                    float4 v = *reinterpret_cast<const float4*>(rowp + h * (DI * 2) + c4 * 16);
                    c = __builtin_amdgcn_mfma_f32_32x32x2f32(afrag_f[c4 * 4 + 0], v.x, c, 0, 0, 0);
                    c = __builtin_amdgcn_mfma_f32_32x32x2f32(afrag_f[c4 * 4 + 1], v.y, c, 0, 0, 0);
                    c = __builtin_amdgcn_mfma_f32_32x32x2f32(afrag_f[c4 * 4 + 2], v.z, c, 0, 0, 0);
                    c = __builtin_amdgcn_mfma_f32_32x32x2f32(afrag_f[c4 * 4 + 3], v.w, c, 0, 0, 0);
                }
            }
            return c;
        };
        // Sigmoid, head weights, head sum and statistics of one 32x32 accumulator.  Returns the score of
        // every slot in sc[]; in the masked form it also stores them one by one.
        auto epilogue = [&](const f32x16& c, int scol, bool masked, float (&sc_out)[NSLOT]) {
#pragma unroll
            for (int s = 0; s < NSLOT; ++s) {
                if (masked && !slot_live[s]) continue;
                float sc = 0.f;
#pragma unroll
                for (int r = 0; r < HL; ++r) {
                    const int i = s * HL + r;
                    if constexpr (RELU) {
                        sc = fmaf(wreg[i], fmaxf(c[i] + nbias[r], 0.f), sc);
                    } else {
                        const float e = fast_exp2(fmaf(c[i], -kLog2e, nbias[r]));
                        sc = fmaf(wreg[i], fast_rcp(1.0f + e), sc);
                    }
                }
                if (HI == 8) sc += __shfl_xor(sc, 32, 64);
                sc_out[s] = sc;
                bool valid = (HI == 8) ? (h == 0) : true;
                if (masked) valid = valid && (scol <= lim_of(s));
                if (valid) {
                    const float d = sc - center[s];
                    s1[s] += d;
                    s2[s] = fmaf(d, d, s2[s]);
                    if constexpr (STORE == 1) {
                        if (masked) (wave_scores + row_off(s))[half_off + (uint32_t)scol] = sc;
                    } else if constexpr (STORE == 2) {
                        if (masked) (wave_keys + row_off(s))[half_off + (uint32_t)scol] = (uint16_t)min((uint32_t)sc, 65535u);
                    }
                }
            }
        };
        // All four column blocks of a fully visible tile.  Column n of block nb is key s0 + 4n + nb, so
        // after the four blocks a lane owns four consecutive keys of each of its rows: one 16-byte store
        // per row and tile, and a wave writes 512 contiguous bytes of a score row at a time.
        auto full_tile = [&](const unsigned char* tileptr, int s0) {
            float sc4[4][NSLOT];
            uint32_t pk[2][NSLOT];  // key mode: pairs of keys, packed as soon as both exist
            f32x16 c = mfma_block(tileptr, 0);
#pragma unroll
            for (int nb = 0; nb < 4; ++nb) {
                f32x16 cn;
                if (nb < 3) cn = mfma_block(tileptr, nb + 1);
                epilogue(c, s0 + 4 * n + nb, false, sc4[nb]);
                if (nb < 3) c = cn;
                if constexpr (STORE == 2) {
                    if (nb & 1) {
                        typedef __attribute__((ext_vector_type(2))) unsigned short u16x2;
#pragma unroll
                        for (int s = 0; s < NSLOT; ++s)  // float -> uint truncates towards zero, the pack saturates at 65535
                            pk[nb >> 1][s] = __builtin_bit_cast(
                                uint32_t, (u16x2)__builtin_amdgcn_cvt_pk_u16((uint32_t)sc4[nb - 1][s], (uint32_t)sc4[nb][s]));
                    }
                }
            }
            if constexpr (STORE == 1) {
                if (HI != 8 || h == 0) {
#pragma unroll
                    for (int s = 0; s < NSLOT; ++s)
                        *reinterpret_cast<float4*>(wave_scores + row_off(s) + (half_off + (uint32_t)(s0 + 4 * n))) =
                            float4{sc4[0][s], sc4[1][s], sc4[2][s], sc4[3][s]};
                }
            } else if constexpr (STORE == 2) {
                if (HI != 8 || h == 0) {
#pragma unroll
                    for (int s = 0; s < NSLOT; ++s)
                        *reinterpret_cast<u32x2*>(wave_keys + row_off(s) + (half_off + (uint32_t)(s0 + 4 * n))) =
                            u32x2{pk[0][s], pk[1][s]};
                }
            }
        };

        // ---- key loop ---------------------------------------------------------------------
        const int ntile = (int)cdiv(key_hi - key_lo, kBN);
        // Leading tiles that are wholly visible to every row of the workgroup, and whose successor
        // tile lies wholly inside the key range, run a branch-free body: the compiler can then count
        // the score stores issued after the prefetch loads and wait for the loads alone
        // (vmcnt(#stores)) instead of draining every outstanding store at each tile boundary.
        int nlead = 0;
        if (!ROW1 && t_wg0 + QT <= a.row_end) {
            const int lim_wg_first = min(qoff + t_wg0, a.Lk - 1);
            nlead = (lim_wg_first + 1 - key_lo) / kBN;
            nlead = min(nlead, min(ntile - 1, (a.Lk - key_lo) / kBN - 1));
            nlead = max(nlead, 0);
        }
        load_tile(key_lo);
        store_tile(0);
        __syncthreads();
        int it = 0;
        // Single-row workgroups (decode: one query against a long cache) are bound by the latency of the
        // key stream, not by arithmetic: their leading tiles keep two tiles of loads in flight and do the
        // arithmetic of the one live slot only, again without branches.
        if constexpr (ROW1 && HI <= 4) {
            const int lim_row = min(qoff + t_wg0, a.Lk - 1);
            int nlead1 = (lim_row + 1 - key_lo) / kBN;  // wholly visible tiles
            nlead1 = max(min(nlead1, ntile - 1), 0);
            u32x4 stage2[NCH];
            auto load_clamped = [&](int s0, u32x4* st) {  // rows beyond the range repeat the last key: never used unmasked
                const unsigned char* tp = tile_ptr(s0);
                const int rmax = a.Lk - 1 - min(s0, last_tile);
#pragma unroll
                for (int c = 0; c < NCH; ++c) {
                    const int ch = tid + c * 256;
                    st[c] = *reinterpret_cast<const u32x4*>(tp + min(ch / CHPR, rmax) * ROWB + (ch % CHPR) * 16);
                }
            };
            if (nlead1 > 0) load_clamped(key_lo + kBN, stage);  // tile 1
            for (; it < nlead1; ++it) {
                const int s0 = key_lo + it * kBN;
                load_clamped(s0 + 2 * kBN, stage2);  // tile it+2
                const f32x16 c = mfma_block(smem + (it & 1) * (kBN * LDSROW), wv);
                float sc = 0.f;
#pragma unroll
                for (int r = 0; r < HL; ++r)
                    sc = fmaf(wreg[r], fast_rcp(1.0f + fast_exp2(fmaf(c[r], -kLog2e, nbias[r]))), sc);
                if (h == 0) {  // the row lives in slot 0 of the lower lane half
                    const float d = sc - center[0];
                    s1[0] += d;
                    s2[0] = fmaf(d, d, s2[0]);
                    const uint32_t col = (uint32_t)(s0 + 4 * n + wv);
                    if constexpr (STORE == 1) wave_scores[col] = sc;
                    if constexpr (STORE == 2) wave_keys[col] = (uint16_t)min((uint32_t)sc, 65535u);
                }
                store_tile((it + 1) & 1);  // tile it+1
                __syncthreads();
#pragma unroll
                for (int c2 = 0; c2 < NCH; ++c2) stage[c2] = stage2[c2];
            }
        }
        for (; !ROW1 && it < nlead; ++it) {
            const int s0 = key_lo + it * kBN;
            const unsigned char* tp = tile_ptr(s0 + kBN);
#pragma unroll
            for (int c = 0; c < NCH; ++c) {  // prefetch of the next tile, no bounds checks needed
                const int ch = tid + c * 256;
                stage[c] = *reinterpret_cast<const u32x4*>(tp + (ch / CHPR) * ROWB + (ch % CHPR) * 16);
            }
            full_tile(smem + (it & 1) * (kBN * LDSROW), s0);
            store_tile((it + 1) & 1);
            __syncthreads();
        }
        for (; it < ntile; ++it) {
            const int s0 = key_lo + it * kBN;
            const bool more = (it + 1) < ntile;
            if (more) load_tile(s0 + kBN);
            const unsigned char* tileptr = smem + (it & 1) * (kBN * LDSROW);
            if (wave_has_rows && s0 <= lim_last) {
                const bool full = !narrow && wave_rows_full && (s0 + kBN - 1 <= lim_first);
                if (full) {
                    full_tile(tileptr, s0);
                } else {
                    for (int nb = narrow ? wv : 0; nb < 4; nb += narrow ? 4 : 1) {
                        float sc[NSLOT];
                        f32x16 c = mfma_block(tileptr, nb);
                        epilogue(c, s0 + 4 * n + nb, true, sc);
                    }
                }
            }
            if (more) store_tile((it + 1) & 1);
            __syncthreads();
        }
    }

    // ---- reduce the statistics over the 32 lanes that share a lane half, write partials -------
#pragma unroll
    for (int s = 0; s < NSLOT; ++s) {
        float x1 = s1[s], x2 = s2[s];
#pragma unroll
        for (int o = 16; o > 0; o >>= 1) {
            x1 += __shfl_xor(x1, o, 64);
            x2 += __shfl_xor(x2, o, 64);
        }
        if (n == 0 && lim_of(s) >= 0 && !(HI == 8 && h == 1)) {
            // four partial slots per (row, split): one per wave in narrow mode, else the owner wave fills
            // slot 0 and clears the rest
            const int t = t_w0 + acc_row(s * HL, h) / HI;
            float2* dst = a.partial + (((int64_t)b * R + (t - a.row_begin)) * a.nsplit + split) * 4;
            x1 *= 1.0f / kKeyScale;  // exact: power of two
            x2 *= 1.0f / (kKeyScale * kKeyScale);
            if (narrow) {
                dst[wv] = float2{x1, x2};
            } else {
                dst[0] = float2{x1, x2};
                dst[1] = dst[2] = dst[3] = float2{0.f, 0.f};
            }
        }
    }
}

// Merge the per-split partial sums of a row in double precision:
//   mean = c + S1/n,  var = S2/n - (S1/n)^2   with d = I - c.
__global__ void indexer_finalize_kernel(const float2* partial, const float* w, float* row_mean, float* row_var,
                                        int B, int Lq, int Lk, int q_offset, int row_begin, int row_end, int nsplit,
                                        int HI, int hi, int relu, const int32_t* seq_lens) {
    const int R = row_end - row_begin;
    const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= (int64_t)B * R) return;
    const int b = (int)(gid / R);
    const int t = row_begin + (int)(gid % R);
    double S1 = 0.0, S2 = 0.0;
    for (int s = 0; s < nsplit * 4; ++s) {
        const float2 p = partial[gid * nsplit * 4 + s];
        S1 += (double)p.x;
        S2 += (double)p.y;
    }
    float c = 0.f;  // same association as in the kernel above so that the centre is bit-identical
    const float* wr = w + ((int64_t)b * Lq + t) * hi;  // hi heads in memory, HI in the kernel (the rest weigh zero)
    if (relu) {
        c = 0.f;  // the ReLU variant sums its scores uncentred
    } else if (HI == 8) {
        float c0 = 0.f, c1 = 0.f;
        for (int j = 0; j < 4; ++j) c0 += 0.5f * wr[j];
        for (int j = 4; j < hi; ++j) c1 += 0.5f * wr[j];
        c = c0 + c1;
    } else {
        for (int j = 0; j < hi; ++j) c += 0.5f * wr[j];
    }
    const double nvis = (double)(min(batch_q_offset(seq_lens, b, q_offset, Lq, Lk) + t, Lk - 1) + 1);
    const double m = S1 / nvis;
    double var = S2 / nvis - m * m;
    if (var < 0.0) var = 0.0;
    if (row_mean) row_mean[(int64_t)b * Lq + t] = (float)((double)c + m);
    row_var[(int64_t)b * Lq + t] = (float)var;
}

// ---- host side -----------------------------------------------------------------------------
static int kernel_heads(int hi) { return hi <= 1 ? 1 : (hi <= 2 ? 2 : (hi <= 4 ? 4 : 8)); }
static int queries_per_wg(int hi) { return 4 * (32 / kernel_heads(hi)); }

// Keys per split: enough splits that the launch fills the chip, never less than four key tiles.
// (With per-sequence lengths the visible range of a row is only known on the device; the plan is always made
// for the whole capacity, which bounds every sequence.)
void indexer_plan(const gsa_shape& sh, int row_begin, int row_end, int* kc_out, int* nsplit_out, int* ntiles_out, bool ragged) {
    const int QT = queries_per_wg(sh.HI);
    const int ntiles = (int)cdiv(row_end - row_begin, QT);
    const int maxvis = ragged ? sh.Lk : (sh.q_offset + row_end - 1 < sh.Lk - 1 ? sh.q_offset + row_end - 1 : sh.Lk - 1) + 1;
    const int64_t want_wgs = 2048;  // measured flat between 1500 and 2300 on 256 CUs
    int64_t nsplit = cdiv(want_wgs, (int64_t)ntiles * sh.B);
    if (nsplit < 1) nsplit = 1;
    int64_t kc = cdiv(cdiv(maxvis, nsplit), kBN) * kBN;
    if (kc < 4 * kBN) kc = 4 * kBN;
    nsplit = cdiv(maxvis, kc);
    *kc_out = (int)kc;
    *nsplit_out = (int)nsplit;
    *ntiles_out = ntiles;
}

size_t indexer_workspace_bytes(const gsa_shape& sh, int row_begin, int row_end, bool ragged) {
    int kc, nsplit, ntiles;
    indexer_plan(sh, row_begin, row_end, &kc, &nsplit, &ntiles, ragged);
    return (size_t)sh.B * (size_t)(row_end - row_begin) * (size_t)nsplit * 4 * sizeof(float2);
}

template <typename T, int DI, int HI>
static hipError_t launch_one(const IndexerArgs& a, bool relu, hipStream_t st) {
    constexpr int LDSROW = DI * ElemTraits<T>::kBytes + 16;
    const size_t smem = 2 * kBN * LDSROW;
    const bool row1 = (a.row_end - a.row_begin) == 1 && !relu;  // (the variant has no kernel of its own for single rows)
    auto kern = relu ? (a.scores ? indexer_kernel<T, DI, HI, 1, false, true> : indexer_kernel<T, DI, HI, 0, false, true>)
              : row1 ? (a.keys ? indexer_kernel<T, DI, HI, 2, true>
                               : (a.scores ? indexer_kernel<T, DI, HI, 1, true> : indexer_kernel<T, DI, HI, 0, true>))
                     : (a.keys ? indexer_kernel<T, DI, HI, 2, false>
                               : (a.scores ? indexer_kernel<T, DI, HI, 1, false> : indexer_kernel<T, DI, HI, 0, false>));
    if (smem > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
    }
    dim3 grid(a.ntiles, a.nsplit, a.B);
    hipLaunchKernelGGL(kern, grid, dim3(256), smem, st, a);
    return hipGetLastError();
}

template <typename T, int DI>
static hipError_t launch_hi(const IndexerArgs& a, int HI, bool relu, hipStream_t st) {
    switch (HI) {
        case 1: return launch_one<T, DI, 1>(a, relu, st);
        case 2: return launch_one<T, DI, 2>(a, relu, st);
        case 4: return launch_one<T, DI, 4>(a, relu, st);
        case 8: return launch_one<T, DI, 8>(a, relu, st);
    }
    return hipErrorInvalidValue;
}

template <typename T>
static hipError_t launch_di(const IndexerArgs& a, int DI, int HI, bool relu, hipStream_t st) {
    switch (DI) {
        case 32: return launch_hi<T, 32>(a, HI, relu, st);
        case 64: return launch_hi<T, 64>(a, HI, relu, st);
        case 128: return launch_hi<T, 128>(a, HI, relu, st);
    }
    return hipErrorInvalidValue;
}

hipError_t launch_indexer(const gsa_shape& sh, const void* qI, const void* kI, const float* w, const float* bI,
                          int row_begin, int row_end, float* scores, uint16_t* keys, int64_t ld, float* row_mean,
                          float* row_var, void* workspace, const int32_t* seq_lens, const PageMap& pm, hipStream_t st) {
    IndexerArgs a;
    a.pm = pm;
    a.seq_lens = seq_lens;
    a.keys = keys;
    a.qI = qI;
    a.kI = kI;
    a.w = w;
    a.bI = bI;
    a.scores = scores;
    a.ld = ld;
    a.partial = static_cast<float2*>(workspace);
    a.B = sh.B;
    a.Lq = sh.Lq;
    a.Lk = sh.Lk;
    a.q_offset = sh.q_offset;
    a.row_begin = row_begin;
    a.row_end = row_end;
    indexer_plan(sh, row_begin, row_end, &a.kc, &a.nsplit, &a.ntiles, seq_lens != nullptr);
    a.hi = sh.HI;
    const int HIK = kernel_heads(sh.HI);
    const bool relu = sh.indexer_act == GSA_ACT_RELU;
    if (relu && keys) return hipErrorInvalidValue;
    hipError_t e = (sh.dtype == GSA_BF16) ? launch_di<__bf16>(a, sh.dI, HIK, relu, st) : launch_di<float>(a, sh.dI, HIK, relu, st);
    if (e != hipSuccess) return e;
    const int64_t rows = (int64_t)sh.B * (row_end - row_begin);
    hipLaunchKernelGGL(indexer_finalize_kernel, dim3((unsigned)cdiv(rows, 256)), dim3(256), 0, st, a.partial, w, row_mean,
                       row_var, sh.B, sh.Lq, sh.Lk, sh.q_offset, row_begin, row_end, a.nsplit, HIK, sh.HI, relu ? 1 : 0, seq_lens);
    return hipGetLastError();
}

}  // namespace gsa
