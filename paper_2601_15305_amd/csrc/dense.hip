// Dense causal attention with the value gate G2 and the output gate G1: Eq. 2 (Sec. 2.1) over every visible
// key, with V replaced by V' = V * sigmoid(g2) (Sec. 3.5) and the result multiplied by sigmoid(g1).  This is the
// "gated only" comparison variant of Sec. 7.1 (with both gates absent: the "standard" one), and what the sparse
// path equals when the budget covers every visible key.  bf16 only.
//
// One workgroup of four waves takes a block of queries of one kv head and walks the visible keys in tiles of
// 32, staged through LDS once for all four waves (double buffered, one barrier per tile, dense coalesced row
// loads).  A wave owns 32 columns = (32 / Gp queries) x (Gp heads of the kv head's group, the group size G
// rounded up to a power of two), as two 16-column blocks of v_mfma_f32_16x16x32_bf16:
//   S^T[key, column] = K[key, :] . Q[column, :]        O^T[d, column] += V'^T[d, key] . P^T[key, column]
// so the K tile's A fragments and the transposed V' fragments are read from LDS once per tile and used for
// both column blocks.  The accumulator layout of S^T (a lane holds four keys of one column) is the B-operand
// layout of the second product; the online softmax (base 2) of a column needs one exchange across lane rows.
#include "common.hpp"

namespace gsa {

struct DenseArgs {
    const void* Q;
    const void* K;
    const void* V;   // already gated
    const void* g1;
    void* out;
    int32_t B, Lq, Lk, q_offset, H, H_kv, row_begin, row_end;
    int32_t Gp;      // heads of one group rounded up to a power of two (1, 2, 4, 8, 16)
    int32_t nblocks; // query blocks per batch element
    float scale;
};

typedef __attribute__((address_space(3))) s16x4 dense_lds_s16x4;

__device__ __forceinline__ float dense_quad_row_max(float x) {
    auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    x = fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
    r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float dense_quad_row_sum(float x) {
    auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    x = __uint_as_float(r[0]) + __uint_as_float(r[1]);
    r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

constexpr float kDenseNegBig = -1.0e30f;

template <int DH>
__global__ __launch_bounds__(256, 2) void dense_attn_bf16_kernel(DenseArgs a) {
    constexpr int KK = DH / 32;        // MFMA k-steps of the score product
    constexpr int MB = DH / 16;        // 16-feature blocks of the value product
    constexpr int ROWB = DH * 2;       // bytes of one head row
    constexpr int VROW = ROWB + 32;    // padded LDS row of the V' tile
    constexpr int KROW = ROWB + 16;    // padded LDS row of the K tile
    constexpr int VCH = ROWB / 16;     // 16-byte chunks per row
    constexpr int NCH = 32 * VCH / 256;  // chunks per thread, tile and tensor
    constexpr int TILEB = 32 * (KROW + VROW);

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];  // two tiles: K then V' each
    const int tid = threadIdx.x;
    const int lane = tid & 63, wv = tid >> 6;
    const int n = lane & 15, q = lane >> 4;
    const int g = blockIdx.y;
    const int b = blockIdx.z;
    const int Gp = a.Gp;
    const int G = a.H / a.H_kv;
    const int QW = 32 / Gp;  // queries per wave
    const int QB = 4 * QW;   // queries per workgroup
    const int blk = a.nblocks - 1 - (int)blockIdx.x;  // longest rows first
    const int t_wg0 = a.row_begin + blk * QB;
    const int t_w0 = t_wg0 + wv * QW;
    const float sl2 = a.scale * kLog2e;
    const uint32_t tokstride = (uint32_t)a.H_kv * ROWB;

    // last key any query of the workgroup / of this wave sees
    const int t_wg_last = min(t_wg0 + QB, a.row_end) - 1;
    const int kmax_wg = min(a.q_offset + t_wg_last, a.Lk - 1);
    const int t_w_last = min(t_w0 + QW, a.row_end) - 1;
    const bool wave_has_rows = t_w0 < a.row_end;
    const int kmax_w = wave_has_rows ? min(a.q_offset + t_w_last, a.Lk - 1) : -1;
    const int kfull_w = min(a.q_offset + t_w0, a.Lk - 1);  // keys up to here are visible to every query of the wave

    // ---- Q fragments of the two column blocks --------------------------------------------------------
    bf16x8 qf[2][KK];
    int col_t[2];      // query row of this lane's column in block cb (or -1)
    int col_head[2];
#pragma unroll
    for (int cb = 0; cb < 2; ++cb) {
        const int c = cb * 16 + n;
        const int t = t_w0 + c / Gp;
        const int hh = c % Gp;
        const bool ok = t < a.row_end && hh < G;
        col_t[cb] = ok ? t : -1;
        col_head[cb] = g * G + (ok ? hh : 0);
        const u32x4* src = reinterpret_cast<const u32x4*>(static_cast<const __bf16*>(a.Q) +
                                                          (((int64_t)b * a.Lq + (ok ? t : a.row_begin)) * a.H + col_head[cb]) * DH);
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
            u32x4 v = ok ? src[kk * 4 + q] : u32x4{0, 0, 0, 0};
            qf[cb][kk] = __builtin_bit_cast(bf16x8, v);
        }
    }
    // last visible key of this lane's two columns (-1: the column does not exist)
    int col_lim[2];
#pragma unroll
    for (int cb = 0; cb < 2; ++cb) col_lim[cb] = col_t[cb] >= 0 ? min(a.q_offset + col_t[cb], a.Lk - 1) : -1;

    f32x4 o[2][MB];
    float mrun[2], lrun[2];
#pragma unroll
    for (int cb = 0; cb < 2; ++cb) {
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) o[cb][mb] = f32x4{0.f, 0.f, 0.f, 0.f};
        mrun[cb] = kDenseNegBig;
        lrun[cb] = 0.f;
    }

    const unsigned char* Kb = static_cast<const unsigned char*>(a.K) + ((int64_t)b * a.Lk * a.H_kv + g) * ROWB;
    const unsigned char* Vb = static_cast<const unsigned char*>(a.V) + ((int64_t)b * a.Lk * a.H_kv + g) * ROWB;
    u32x4 ks[NCH], vs[NCH];
    auto load_tile = [&](int s0) {
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            const int ch = tid + c * 256;
            const int s = min(s0 + ch / VCH, a.Lk - 1);  // rows beyond the context repeat the last key; they are masked
            const uint32_t off = (uint32_t)s * tokstride + (uint32_t)(ch % VCH) * 16u;
            ks[c] = *reinterpret_cast<const u32x4*>(Kb + off);
            vs[c] = *reinterpret_cast<const u32x4*>(Vb + off);
        }
    };
    auto store_tile = [&](int buf) {
        unsigned char* kl = smem + buf * TILEB;
        unsigned char* vl = kl + 32 * KROW;
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            const int ch = tid + c * 256;
            *reinterpret_cast<u32x4*>(kl + (ch / VCH) * KROW + (ch % VCH) * 16) = ks[c];
            *reinterpret_cast<u32x4*>(vl + (ch / VCH) * VROW + (ch % VCH) * 16) = vs[c];
        }
    };
    auto compute = [&](const unsigned char* kl, int s0, bool masked) {
        const unsigned char* vl = kl + 32 * KROW;
        f32x4 s[2][2];  // [column block][16-key sub-tile]
#pragma unroll
        for (int cb = 0; cb < 2; ++cb) s[cb][0] = s[cb][1] = f32x4{0.f, 0.f, 0.f, 0.f};
        {
            const unsigned char* k0 = kl + n * KROW + q * 16;
            const unsigned char* k1 = k0 + 16 * KROW;
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) {
                const bf16x8 a0 = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(k0 + kk * 64));
                const bf16x8 a1 = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(k1 + kk * 64));
#pragma unroll
                for (int cb = 0; cb < 2; ++cb) {
                    s[cb][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0, qf[cb][kk], s[cb][0], 0, 0, 0);
                    s[cb][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, qf[cb][kk], s[cb][1], 0, 0, 0);
                }
            }
        }
        // lane (column n, q): s[cb][0][i] is key s0 + 4q + i, s[cb][1][i] is key s0 + 16 + 4q + i
        bf16x8 pf[2];
#pragma unroll
        for (int cb = 0; cb < 2; ++cb) {
            float x[8];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                x[i] = s[cb][0][i] * sl2;
                x[4 + i] = s[cb][1][i] * sl2;
            }
            if (masked) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    if (s0 + 4 * q + i > col_lim[cb]) x[i] = kDenseNegBig;
                    if (s0 + 16 + 4 * q + i > col_lim[cb]) x[4 + i] = kDenseNegBig;
                }
            }
            float tmax = fmaxf(fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3])), fmaxf(fmaxf(x[4], x[5]), fmaxf(x[6], x[7])));
            tmax = dense_quad_row_max(tmax);
            const float mnew = fmaxf(mrun[cb], tmax);
            const float alpha = fast_exp2(mrun[cb] - mnew);
            float psum = 0.f;
            float p[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                // a column none of whose keys is visible yet keeps mnew at the floor: its terms must stay zero
                p[i] = x[i] > 0.5f * kDenseNegBig ? fast_exp2(x[i] - mnew) : 0.f;
                psum += p[i];
            }
            lrun[cb] = lrun[cb] * alpha + psum;
            mrun[cb] = mnew;
            if (__any(alpha != 1.0f)) {
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) o[cb][mb] *= alpha;
            }
            u32x4 pw = {pack_bf16x2(p[0], p[1]), pack_bf16x2(p[2], p[3]), pack_bf16x2(p[4], p[5]), pack_bf16x2(p[6], p[7])};
            pf[cb] = __builtin_bit_cast(bf16x8, pw);
        }
        {
            const int r4 = (lane & 15) >> 2, c4 = lane & 3;
            const unsigned char* p0 = vl + (4 * q + r4) * VROW + c4 * 8;
            const unsigned char* p1 = p0 + 16 * VROW;
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) {
                s16x4 a0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((dense_lds_s16x4*)(p0 + mb * 32));
                s16x4 a1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((dense_lds_s16x4*)(p1 + mb * 32));
                typedef __attribute__((ext_vector_type(8))) short s16x8;
                const s16x8 av = {a0[0], a0[1], a0[2], a0[3], a1[0], a1[1], a1[2], a1[3]};
                const bf16x8 af = __builtin_bit_cast(bf16x8, av);
#pragma unroll
                for (int cb = 0; cb < 2; ++cb) o[cb][mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af, pf[cb], o[cb][mb], 0, 0, 0);
            }
        }
    };

    // ---- key loop ---------------------------------------------------------------------------------------
    const int ntile = kmax_wg / 32 + 1;
    load_tile(0);
    store_tile(0);
    __syncthreads();
    for (int it = 0; it < ntile; ++it) {
        const int s0 = it * 32;
        const bool more = it + 1 < ntile;
        if (more) load_tile(s0 + 32);
        if (wave_has_rows && s0 <= kmax_w) {
            // (columns that do not exist are never stored, so only keys beyond a real query's position need the mask)
            compute(smem + (it & 1) * TILEB, s0, s0 + 31 > kfull_w);
        }
        if (more) store_tile((it + 1) & 1);
        __syncthreads();
    }

    // ---- normalise, G1, store ---------------------------------------------------------------------------
#pragma unroll
    for (int cb = 0; cb < 2; ++cb) {
        const float ltot = dense_quad_row_sum(lrun[cb]);
        if (col_t[cb] < 0) continue;
        const float inv = ltot > 0.f ? 1.0f / ltot : 0.f;
        const int64_t obase = (((int64_t)b * a.Lq + col_t[cb]) * a.H + col_head[cb]) * DH;
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            const int d0 = mb * 16 + 4 * q;
            float y[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) y[i] = o[cb][mb][i] * inv;
            if (a.g1) {
                const u32x2 gw = *reinterpret_cast<const u32x2*>(static_cast<const __bf16*>(a.g1) + obase + d0);
                y[0] *= sigmoid_f32(bf16_bits_to_f32(gw[0] & 0xffffu));
                y[1] *= sigmoid_f32(bf16_bits_to_f32(gw[0] >> 16));
                y[2] *= sigmoid_f32(bf16_bits_to_f32(gw[1] & 0xffffu));
                y[3] *= sigmoid_f32(bf16_bits_to_f32(gw[1] >> 16));
            }
            const u32x2 ow = {pack_bf16x2(y[0], y[1]), pack_bf16x2(y[2], y[3])};
            *reinterpret_cast<u32x2*>(static_cast<__bf16*>(a.out) + obase + d0) = ow;
        }
    }
}

hipError_t launch_dense_attention(const gsa_shape& sh, int row_begin, int row_end, const void* Q, const void* K, const void* Vg,
                                  const void* g1, float scale, void* out, hipStream_t st) {
    DenseArgs a;
    a.Q = Q;
    a.K = K;
    a.V = Vg;
    a.g1 = g1;
    a.out = out;
    a.B = sh.B;
    a.Lq = sh.Lq;
    a.Lk = sh.Lk;
    a.q_offset = sh.q_offset;
    a.H = sh.H;
    a.H_kv = sh.H_kv;
    a.row_begin = row_begin;
    a.row_end = row_end;
    const int G = sh.H / sh.H_kv;
    int Gp = 1;
    while (Gp < G) Gp *= 2;
    a.Gp = Gp;
    const int QB = 4 * (32 / Gp);
    a.nblocks = (int)cdiv(row_end - row_begin, QB);
    a.scale = scale;
    const size_t smem = 2 * 32 * (size_t)((sh.d_h * 2 + 16) + (sh.d_h * 2 + 32));
    const dim3 grid((unsigned)a.nblocks, (unsigned)sh.H_kv, (unsigned)sh.B);
    if (sh.d_h == 128)
        hipLaunchKernelGGL(dense_attn_bf16_kernel<128>, grid, dim3(256), smem, st, a);
    else
        hipLaunchKernelGGL(dense_attn_bf16_kernel<64>, grid, dim3(256), smem, st, a);
    return hipGetLastError();
}

}  // namespace gsa
