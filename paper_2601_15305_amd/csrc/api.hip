// C ABI of libgsa: host-side argument validation, workspace carving and launch sequencing.
// Every error that can be decided from the arguments is returned before anything is launched.
#include <cmath>
#include <cstring>
#include <mutex>
#include <string>

#include "common.hpp"

namespace gsa {
// defined in indexer.hip / select.hip / attention.hip
size_t indexer_workspace_bytes(const gsa_shape& sh, int row_begin, int row_end, bool ragged);
hipError_t launch_indexer(const gsa_shape& sh, const void* qI, const void* kI, const float* w, const float* bI,
                          int row_begin, int row_end, float* scores, uint16_t* keys, int64_t ld, float* row_mean,
                          float* row_var, void* workspace, const int32_t* seq_lens, const PageMap& pm, hipStream_t st);
hipError_t launch_select(const gsa_shape& sh, int row_begin, int row_end, const float* scores, int64_t ld,
                         const int32_t* n_sel, int k_cap, int32_t* idx_out, int idx_rows, int idx_row0, bool exact_only,
                         const int32_t* seq_lens, hipStream_t st);
hipError_t launch_select16(const gsa_shape& sh, int row_begin, int row_end, const uint16_t* keys, int64_t ld,
                           const int32_t* n_sel, int k_cap, int32_t* idx_out, int idx_rows, int idx_row0, const void* qI,
                           const void* kI, const float* w, const float* bI, const int32_t* seq_lens, int wave_min_rows,
                           const PageMap& pm, hipStream_t st);
hipError_t launch_adaptive_k(const gsa_shape& sh, const gsa_adaptive& c, int row_begin, int row_end,
                             const float* row_var, int32_t* k_out, int32_t* n_sel_out, const int32_t* seq_lens, hipStream_t st);
hipError_t launch_value_gate(const gsa_shape& sh, const void* V, const void* g2, void* Vg, hipStream_t st);
hipError_t launch_attention(const gsa_shape& sh, int row_begin, int row_end, const void* Q, const void* K, const void* V,
                            const void* g2, const void* g1, const int32_t* idx, int idx_rows, int idx_row0,
                            const int32_t* n_sel, int k_cap, float scale, void* out, void* workspace, const gsa_tuning& tn,
                            int64_t pool_rows, hipStream_t st);
size_t attn_workspace_bytes(const gsa_shape& sh, int row_begin, int row_end, int k_cap, const gsa_tuning& tn);
hipError_t launch_dense_attention(const gsa_shape& sh, int row_begin, int row_end, const void* Q, const void* K, const void* Vg,
                                  const void* g1, float scale, void* out, hipStream_t st);
hipError_t launch_cache_append(const gsa_shape& sh, const void* kI_new, const void* K_new, const void* V_new, const void* g2_new,
                               const int32_t* seq_lens, void* kI_cache, void* K_cache, void* Vg_cache, int32_t* seq_lens_out,
                               const PageMap& pm, hipStream_t st);
hipError_t launch_translate_indices(const gsa_shape& sh, const PageMap& pm, int row_begin, int row_end, const int32_t* idx,
                                    int idx_rows, int idx_row0, const int32_t* n_sel, int k_cap, int32_t* phys, hipStream_t st);
hipError_t launch_projection(const void* x, int64_t tokens, int K, int nseg, const void* const* W, void* const* out,
                             const int32_t* width, const int32_t* kind, hipStream_t st);
hipError_t launch_attention_bwd(const gsa_shape& sh, const void* Q, const void* K, const void* V, const void* g2, const void* g1,
                                const int32_t* idx, const int32_t* n_sel, int k_cap, float scale, const void* dout, float* dQ,
                                float* dK, float* dV, float* dg1, float* dg2, float* p_sum, void* workspace, hipStream_t st);
size_t attention_bwd_workspace_bytes(const gsa_shape& sh, int k_cap);
hipError_t launch_indexer_kl(const gsa_shape& sh, const void* qI, const void* kI, const float* w, const float* bI, const int32_t* idx,
                             const int32_t* n_sel, int k_cap, const float* p, float* loss, float* dqI, float* dkI, float* dw,
                             float* dbI, hipStream_t st);
hipError_t launch_probe_gather(const void* table, const int32_t* idx, int64_t n_idx, int waves, uint32_t* sink, hipStream_t st);
hipError_t launch_probe_gather_staged(const void* table, const int32_t* idx, int64_t n_idx, int waves, uint32_t* sink, hipStream_t st);

static thread_local std::string g_last_error;

static int32_t hip_fail(hipError_t e, const char* where) {
    g_last_error = std::string(where) + ": " + hipGetErrorString(e);
    return GSA_ERR_HIP;
}

static int32_t check_shape(const gsa_shape* s) {
    if (!s) return GSA_ERR_NULL;
    if (s->B < 1 || s->Lq < 1 || s->Lk < 1 || s->q_offset < 0 || s->H < 1 || s->H_kv < 1 || s->d_h < 1 || s->HI < 1 ||
        s->dI < 1)
        return GSA_ERR_SHAPE;
    if (s->H % s->H_kv != 0) return GSA_ERR_SHAPE;
    if ((int64_t)s->q_offset + s->Lq > (int64_t)s->Lk) return GSA_ERR_SHAPE;
    if (s->dtype != GSA_F32 && s->dtype != GSA_BF16) return GSA_ERR_UNSUPPORTED;
    if (s->indexer_act != GSA_ACT_SIGMOID && s->indexer_act != GSA_ACT_RELU) return GSA_ERR_UNSUPPORTED;
    if (s->d_h != 64 && s->d_h != 128) return GSA_ERR_UNSUPPORTED;
    if (s->dI != 32 && s->dI != 64 && s->dI != 128) return GSA_ERR_UNSUPPORTED;
    if (s->HI > 8) return GSA_ERR_UNSUPPORTED;
    if (s->H / s->H_kv > 16) return GSA_ERR_UNSUPPORTED;
    if (s->Lk > (1 << 20)) return GSA_ERR_UNSUPPORTED;
    // the attention addresses a K / V row as a 64-bit base plus a 32-bit byte offset inside one batch element
    if ((int64_t)s->Lk * s->H_kv * s->d_h * (s->dtype == GSA_BF16 ? 2 : 4) > (1LL << 32)) return GSA_ERR_UNSUPPORTED;
    if ((int64_t)s->B * s->Lq > 0x7fffffffLL) return GSA_ERR_UNSUPPORTED;
    return GSA_OK;
}

static int32_t check_rows(const gsa_shape* s, int32_t row_begin, int32_t row_end) {
    if (row_begin < 0 || row_end > s->Lq || row_begin >= row_end) return GSA_ERR_SHAPE;
    return GSA_OK;
}

static int32_t check_ctl(const gsa_adaptive* c) {
    if (!c) return GSA_ERR_NULL;
    if (c->k_fixed < 0 || c->dense_below < 0) return GSA_ERR_SHAPE;
    if (c->k_fixed > 0) return GSA_OK;
    if (c->k_min < 1 || c->k_min > c->k_max || c->k_base < 1) return GSA_ERR_SHAPE;
    if (c->mode != 0 && c->mode != 1) return GSA_ERR_UNSUPPORTED;
    if (!(c->vbar > 0.0f) || !std::isfinite(c->vbar)) return GSA_ERR_VBAR;
    return GSA_OK;
}

// The selection kernels keep two bitmaps of a row in LDS: beyond this context length they do not fit.
static int32_t check_select_len(const gsa_shape* s) { return s->Lk > GSA_SELECT_MAX_LK ? GSA_ERR_UNSUPPORTED : GSA_OK; }

static const gsa_tuning kDefaultTuning = {0, 0, 0, 0, 0, 0};
static const gsa_tuning& tuning_or_default(const gsa_tuning* t) { return t ? *t : kDefaultTuning; }

static bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }
static size_t up256(size_t x) { return (x + 255) & ~(size_t)255; }
static size_t elt_bytes(const gsa_shape& s) { return s.dtype == GSA_BF16 ? 2 : 4; }

// ---- forward workspace plan ---------------------------------------------------------------------
// Fixed part: V' (when the value gate runs as a pre-pass) and the per-row outputs the caller did not ask
// for.  Per-slab part, reused by every slab: the slab's selected indices (when the caller did not ask for
// them), its scores (fp32) or keys (16 bit), the indexer's per-split partial sums and the attention's
// workspace.  A slab of rows [r0, r1) sees keys 0 .. q_offset + r1 - 1 only, which sets the leading
// dimension of its score rows: early slabs are narrow and hold more rows in the same bytes.
struct FixedPlan {
    size_t off_vg, off_var, off_k, off_nsel, total;
};
struct SlabPlan {
    int r0, r1;
    int64_t ld;
    size_t off_idx, off_phys, off_scores, off_partial, off_attn, total;  // offsets from the start of the per-slab part
};
// `ragged` arguments below: 0 = one position offset for the whole batch, 1 = per-sequence lengths (decode-serving
// caches), 2 = per-sequence lengths with paged caches (the slab also holds the selected rows as pool rows).
constexpr int kRagged = 1, kPaged = 2;
static const PageMap kNoPages = {nullptr, 0, 0, 0};

// The value gate runs as a dense pre-pass (once per key token) when the queries together gather
// clearly more rows than there are tokens; otherwise (decode: one query against a long cache) it
// is applied in registers to the gathered rows only.
static bool gate_as_prepass(const gsa_shape& s, int k_cap) {
    const int64_t k_eff = k_cap < s.Lk ? k_cap : s.Lk;
    return (int64_t)s.Lq * k_eff >= 4 * (int64_t)s.Lk;
}

static FixedPlan plan_fixed(const gsa_shape& s, int k_cap, bool has_g2) {
    FixedPlan p;
    size_t off = 0;
    p.off_vg = off;
    if (has_g2 && gate_as_prepass(s, k_cap)) off += up256((size_t)s.B * s.Lk * s.H_kv * s.d_h * elt_bytes(s));
    const size_t rows = (size_t)s.B * s.Lq;
    p.off_var = off;
    off += up256(rows * 4);
    p.off_k = off;
    off += up256(rows * 4);
    p.off_nsel = off;
    off += up256(rows * 4);
    p.total = off;
    return p;
}

static SlabPlan plan_slab(const gsa_shape& s, int k_cap, bool own_idx, bool use_keys, int ragged, int r0, int r1, const gsa_tuning& tn) {
    SlabPlan p;
    p.r0 = r0;
    p.r1 = r1;
    // (with per-sequence lengths a row may see up to the whole capacity)
    const int64_t last = ragged ? s.Lk - 1 : ((int64_t)s.q_offset + r1 - 1 < s.Lk - 1 ? (int64_t)s.q_offset + r1 - 1 : s.Lk - 1);
    p.ld = (last + 1 + 31) & ~(int64_t)31;
    const size_t rows = (size_t)s.B * (r1 - r0);
    size_t off = 0;
    p.off_idx = off;
    if (own_idx) off += up256(rows * (size_t)k_cap * 4);
    p.off_phys = off;
    if (ragged == kPaged) off += up256(rows * (size_t)k_cap * 4);
    p.off_scores = off;
    off += up256(rows * (size_t)p.ld * (use_keys ? 2 : 4));
    p.off_partial = off;
    off += up256(indexer_workspace_bytes(s, r0, r1, ragged != 0));
    p.off_attn = off;
    off += up256(attn_workspace_bytes(s, r0, r1, k_cap, tn));
    p.total = off;
    return p;
}

// Slab boundaries are multiples of 128 rows (the last slab ends at Lq).
static int slab_end(const gsa_shape& s, int r0, int64_t blocks) {
    const int64_t r1 = (int64_t)r0 + blocks * 128;
    return (int)(r1 < s.Lq ? r1 : s.Lq);
}

// 16-bit keys between indexer and selection need bounded scores: the sigmoid indexer only.
static bool forward_keys(const gsa_shape& s, const gsa_tuning& tn) {
    return tn.forward_fp32_scores == 0 && s.indexer_act == GSA_ACT_SIGMOID;
}

// The slab that starts at row r0: as many rows as fit into `avail` bytes of per-slab workspace.  Returns
// false if not even 128 rows (or the rest of the rows) fit.
static bool next_slab(const gsa_shape& s, int k_cap, bool own_idx, bool use_keys, int ragged, size_t avail, const gsa_tuning& tn, int r0,
                      SlabPlan* out) {
    const int64_t max_blocks = cdiv(s.Lq - r0, 128);
    SlabPlan best = plan_slab(s, k_cap, own_idx, use_keys, ragged, r0, slab_end(s, r0, max_blocks), tn);
    if (best.total > avail) {
        int64_t lo = 1, hi = max_blocks;  // invariant: `lo` blocks fit (checked first), `hi` blocks do not
        best = plan_slab(s, k_cap, own_idx, use_keys, ragged, r0, slab_end(s, r0, lo), tn);
        if (best.total > avail) return false;
        while (hi - lo > 1) {
            const int64_t mid = (lo + hi) / 2;
            const SlabPlan p = plan_slab(s, k_cap, own_idx, use_keys, ragged, r0, slab_end(s, r0, mid), tn);
            if (p.total <= avail) {
                lo = mid;
                best = p;
            } else {
                hi = mid;
            }
        }
    }
    *out = best;
    return true;
}

// Can [0, Lq) be cut into slabs that fit?  (The same walk the launches make, without launching.)
static bool slabs_fit(const gsa_shape& s, int k_cap, bool own_idx, bool use_keys, int ragged, size_t avail, const gsa_tuning& tn) {
    SlabPlan p;
    for (int r0 = 0; r0 < s.Lq; r0 = p.r1)
        if (!next_slab(s, k_cap, own_idx, use_keys, ragged, avail, tn, r0, &p)) return false;
    return true;
}

// The launches of gsa_forward for an already validated call whose slabs are known to fit.
static int32_t forward_launches(const gsa_shape& s, const gsa_adaptive& ctl, const void* Q, const void* K, const void* V,
                                const void* g1_logits, const void* g2_logits, const void* qI, const void* kI, const float* w,
                                const float* bI, float softmax_scale, void* out, int32_t* idx_out, int32_t* n_sel_out,
                                int32_t* k_out, float* row_var_out, int32_t k_cap, unsigned char* ws, size_t ws_bytes,
                                const int32_t* seq_lens, const PageMap& pm, const gsa_tuning& tn, hipStream_t st) {
    const FixedPlan fx = plan_fixed(s, k_cap, g2_logits != nullptr);
    const int ragged = pm.table ? kPaged : (seq_lens ? kRagged : 0);
    const int64_t pool_rows = pm.table ? ((int64_t)pm.pool_pages << pm.page_shift) : 0;
    const bool has_g2 = g2_logits != nullptr;
    const bool prepass = has_g2 && gate_as_prepass(s, k_cap);
    const bool own_idx = idx_out == nullptr;
    const bool use_keys = forward_keys(s, tn);
    const float scale = softmax_scale > 0.0f ? softmax_scale : 1.0f / std::sqrt((float)s.d_h);
    const void* Vuse = V;
    const void* g2use = has_g2 ? g2_logits : nullptr;
    hipError_t e;
    if (prepass) {  // stage (2) of Sec. 4: the value gate, once per token
        e = launch_value_gate(s, V, g2_logits, ws + fx.off_vg, st);
        if (e != hipSuccess) return hip_fail(e, "gsa_forward/value_gate");
        Vuse = ws + fx.off_vg;
        g2use = nullptr;
    }
    float* var = row_var_out ? row_var_out : reinterpret_cast<float*>(ws + fx.off_var);
    int32_t* kbuf = k_out ? k_out : reinterpret_cast<int32_t*>(ws + fx.off_k);
    int32_t* nsel = n_sel_out ? n_sel_out : reinterpret_cast<int32_t*>(ws + fx.off_nsel);
    unsigned char* sw = ws + fx.total;  // per-slab part
    SlabPlan p;
    for (int r0 = 0; r0 < s.Lq; r0 = p.r1) {
        if (!next_slab(s, k_cap, own_idx, use_keys, ragged, ws_bytes - fx.total, tn, r0, &p)) return GSA_ERR_WORKSPACE;
        const int r1 = p.r1;
        float* scores = reinterpret_cast<float*>(sw + p.off_scores);
        uint16_t* keys = reinterpret_cast<uint16_t*>(sw + p.off_scores);
        e = launch_indexer(s, qI, kI, w, bI, r0, r1, use_keys ? nullptr : scores, use_keys ? keys : nullptr, p.ld, nullptr,
                           var, sw + p.off_partial, seq_lens, pm, st);
        if (e != hipSuccess) return hip_fail(e, "gsa_forward/indexer");
        e = launch_adaptive_k(s, ctl, r0, r1, var, kbuf, nsel, seq_lens, st);
        if (e != hipSuccess) return hip_fail(e, "gsa_forward/adaptive_k");
        int32_t* idx = own_idx ? reinterpret_cast<int32_t*>(sw + p.off_idx) : idx_out;
        const int idx_rows = own_idx ? (r1 - r0) : s.Lq;
        const int idx_row0 = own_idx ? r0 : 0;
        e = use_keys ? launch_select16(s, r0, r1, keys, p.ld, nsel, k_cap, idx, idx_rows, idx_row0, qI, kI, w, bI, seq_lens,
                                       tn.select_wave_min_rows, pm, st)
                     : launch_select(s, r0, r1, scores, p.ld, nsel, k_cap, idx, idx_rows, idx_row0, tn.select_exact_only != 0,
                                     seq_lens, st);
        if (e != hipSuccess) return hip_fail(e, "gsa_forward/select");
        const int32_t* gather = idx;
        int gather_rows = idx_rows, gather_row0 = idx_row0;
        if (pm.table) {  // the attention gathers rows of the pool: translate the selected positions
            int32_t* phys = reinterpret_cast<int32_t*>(sw + p.off_phys);
            e = launch_translate_indices(s, pm, r0, r1, idx, idx_rows, idx_row0, nsel, k_cap, phys, st);
            if (e != hipSuccess) return hip_fail(e, "gsa_forward/translate");
            gather = phys;
            gather_rows = r1 - r0;
            gather_row0 = r0;
        }
        e = launch_attention(s, r0, r1, Q, K, Vuse, g2use, g1_logits, gather, gather_rows, gather_row0, nsel, k_cap, scale, out,
                             sw + p.off_attn, tn, pool_rows, st);
        if (e != hipSuccess) return hip_fail(e, "gsa_forward/attention");
    }
    return GSA_OK;
}

static int32_t check_forward_args(const gsa_shape* shape, const gsa_adaptive* ctl, const void* Q, const void* K, const void* V,
                                  const void* g1_logits, const void* g2_logits, const void* qI, const void* kI, const float* w,
                                  float softmax_scale, const void* out, int32_t k_cap) {
    int32_t rc = check_shape(shape);
    if (rc != GSA_OK) return rc;
    rc = check_select_len(shape);
    if (rc != GSA_OK) return rc;
    rc = check_ctl(ctl);
    if (rc != GSA_OK) return rc;
    if (!Q || !K || !V || !qI || !kI || !w || !out) return GSA_ERR_NULL;
    if (k_cap < 1 || k_cap > 8192) return GSA_ERR_SHAPE;
    if ((ctl->k_fixed > 0 ? ctl->k_fixed : ctl->k_max) > k_cap) return GSA_ERR_SHAPE;
    if (!(softmax_scale >= 0.0f) || !std::isfinite(softmax_scale)) return GSA_ERR_SHAPE;
    if (!aligned(Q, 16) || !aligned(K, 16) || !aligned(V, 16) || !aligned(out, 16) || !aligned(qI, 16) || !aligned(kI, 16) ||
        (g1_logits && !aligned(g1_logits, 16)) || (g2_logits && !aligned(g2_logits, 16)))
        return GSA_ERR_SHAPE;
    return GSA_OK;
}

// Bytes of the whole forward workspace when every slab holds `blocks` * 128 rows.
static size_t forward_bytes_uniform(const gsa_shape& s, int k_cap, bool has_g2, int64_t blocks, const gsa_tuning& tn, int ragged = 0) {
    const bool use_keys = forward_keys(s, tn);
    size_t slab = 0;
    for (int r0 = 0; r0 < s.Lq;) {
        const SlabPlan p = plan_slab(s, k_cap, true, use_keys, ragged, r0, slab_end(s, r0, blocks), tn);
        if (p.total > slab) slab = p.total;
        r0 = p.r1;
    }
    return plan_fixed(s, k_cap, has_g2).total + slab;
}

// ---- scratch of the allocation-free forward --------------------------------------------------------
// One array per GPU, part of the library's code object: it exists from the moment the library is loaded on
// a device until the process ends.  The array's name is only a host-side handle; its device address is
// looked up once per device (with that device current) and kept.
constexpr size_t kStaticScratchBytes = GSA_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) __attribute__((used)) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static unsigned char* g_scratch_ptr[kMaxDevices];

static int32_t static_scratch(unsigned char** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e, "gsa_forward_noalloc/hipGetDevice");
    if (dev < 0 || dev >= kMaxDevices) {
        g_last_error = "gsa_forward_noalloc: device ordinal beyond the per-device scratch table";
        return GSA_ERR_UNSUPPORTED;
    }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return hip_fail(e, "gsa_forward_noalloc/hipGetSymbolAddress");
        g_scratch_ptr[dev] = static_cast<unsigned char*>(p);
    }
    *out = g_scratch_ptr[dev];
    return GSA_OK;
}

}  // namespace gsa

using namespace gsa;

extern "C" {

const char* gsa_status_string(int32_t status) {
    switch (status) {
        case GSA_OK: return "ok";
        case GSA_ERR_NULL: return "a required pointer is NULL";
        case GSA_ERR_SHAPE: return "inconsistent or non-positive dimensions, row range or k bounds";
        case GSA_ERR_UNSUPPORTED: return "shape or dtype outside what the kernels are built for";
        case GSA_ERR_VBAR: return "vbar must be a positive finite number when the controller is on";
        case GSA_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case GSA_ERR_HIP: return "HIP launch failed (see gsa_last_error)";
    }
    return "unknown status";
}

const char* gsa_last_error(void) { return g_last_error.c_str(); }

int32_t gsa_version(void) { return 100; }

size_t gsa_indexer_workspace_bytes(const gsa_shape* shape, int32_t row_begin, int32_t row_end) {
    if (check_shape(shape) != GSA_OK || check_rows(shape, row_begin, row_end) != GSA_OK) return 0;
    return up256(indexer_workspace_bytes(*shape, row_begin, row_end, false));
}

int32_t gsa_indexer_scores(const gsa_shape* shape, const void* qI, const void* kI, const float* w, const float* bI,
                           int32_t row_begin, int32_t row_end, float* scores, int64_t ld_scores, float* row_mean,
                           float* row_var, void* workspace, size_t workspace_bytes, void* stream) {
    int32_t rc = check_shape(shape);
    if (rc != GSA_OK) return rc;
    if (!qI || !kI || !w || !row_var) return GSA_ERR_NULL;
    rc = check_rows(shape, row_begin, row_end);
    if (rc != GSA_OK) return rc;
    if (scores && (ld_scores < shape->Lk || (ld_scores & 3) != 0)) return GSA_ERR_SHAPE;
    if (!aligned(qI, 16) || !aligned(kI, 16) || (scores && !aligned(scores, 16))) return GSA_ERR_SHAPE;
    if (!workspace || !aligned(workspace, 256) || workspace_bytes < indexer_workspace_bytes(*shape, row_begin, row_end, false))
        return GSA_ERR_WORKSPACE;
    hipError_t e = launch_indexer(*shape, qI, kI, w, bI, row_begin, row_end, scores, nullptr, ld_scores, row_mean, row_var,
                                  workspace, nullptr, kNoPages, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? GSA_OK : hip_fail(e, "gsa_indexer_scores");
}

int32_t gsa_indexer_keys(const gsa_shape* shape, const void* qI, const void* kI, const float* w, const float* bI,
                         int32_t row_begin, int32_t row_end, uint16_t* keys, int64_t ld_keys, float* row_mean, float* row_var,
                         void* workspace, size_t workspace_bytes, void* stream) {
    int32_t rc = check_shape(shape);
    if (rc != GSA_OK) return rc;
    if (shape->indexer_act != GSA_ACT_SIGMOID) return GSA_ERR_UNSUPPORTED;  // keys need scores below HI
    if (!qI || !kI || !w || !row_var || !keys) return GSA_ERR_NULL;
    rc = check_rows(shape, row_begin, row_end);
    if (rc != GSA_OK) return rc;
    if (ld_keys < shape->Lk || (ld_keys & 7) != 0) return GSA_ERR_SHAPE;
    if (!aligned(qI, 16) || !aligned(kI, 16) || !aligned(keys, 16)) return GSA_ERR_SHAPE;
    if (!workspace || !aligned(workspace, 256) || workspace_bytes < indexer_workspace_bytes(*shape, row_begin, row_end, false))
        return GSA_ERR_WORKSPACE;
    hipError_t e = launch_indexer(*shape, qI, kI, w, bI, row_begin, row_end, nullptr, keys, ld_keys, row_mean, row_var,
                                  workspace, nullptr, kNoPages, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? GSA_OK : hip_fail(e, "gsa_indexer_keys");
}

int32_t gsa_adaptive_k(const gsa_shape* shape, const gsa_adaptive* ctl, const float* row_var, int32_t* k_out,
                       int32_t* n_sel_out, void* stream) {
    int32_t rc = check_shape(shape);
    if (rc != GSA_OK) return rc;
    rc = check_ctl(ctl);
    if (rc != GSA_OK) return rc;
    if (!n_sel_out || (ctl->k_fixed == 0 && !row_var)) return GSA_ERR_NULL;
    hipError_t e = launch_adaptive_k(*shape, *ctl, 0, shape->Lq, row_var, k_out, n_sel_out, nullptr, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? GSA_OK : hip_fail(e, "gsa_adaptive_k");
}

int32_t gsa_topk_select(const gsa_shape* shape, int32_t row_begin, int32_t row_end, const float* scores,
                        int64_t ld_scores, const int32_t* n_sel, int32_t k_cap, int32_t* idx_out, const gsa_tuning* tuning,
                        void* stream) {
    int32_t rc = check_shape(shape);
    if (rc != GSA_OK) return rc;
    rc = check_select_len(shape);
    if (rc != GSA_OK) return rc;
    if (!scores || !n_sel || !idx_out) return GSA_ERR_NULL;
    rc = check_rows(shape, row_begin, row_end);
    if (rc != GSA_OK) return rc;
    if (ld_scores < shape->Lk || (ld_scores & 3) != 0 || !aligned(scores, 16)) return GSA_ERR_SHAPE;
    if (k_cap < 1 || k_cap > 8192) return GSA_ERR_SHAPE;
    hipError_t e = launch_select(*shape, row_begin, row_end, scores, ld_scores, n_sel, k_cap, idx_out, shape->Lq, 0,
                                 tuning_or_default(tuning).select_exact_only != 0, nullptr, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? GSA_OK : hip_fail(e, "gsa_topk_select");
}

int32_t gsa_topk_select_keys(const gsa_shape* shape, int32_t row_begin, int32_t row_end, const uint16_t* keys,
                             int64_t ld_keys, const int32_t* n_sel, int32_t k_cap, int32_t* idx_out, const void* qI,
                             const void* kI, const float* w, const float* bI, const gsa_tuning* tuning, void* stream) {
    int32_t rc = check_shape(shape);
    if (rc != GSA_OK) return rc;
    rc = check_select_len(shape);
    if (rc != GSA_OK) return rc;
    if (shape->indexer_act != GSA_ACT_SIGMOID) return GSA_ERR_UNSUPPORTED;
    if (!keys || !n_sel || !idx_out || !qI || !kI || !w) return GSA_ERR_NULL;
    rc = check_rows(shape, row_begin, row_end);
    if (rc != GSA_OK) return rc;
    if (ld_keys < shape->Lk || (ld_keys & 7) != 0 || !aligned(keys, 16) || !aligned(qI, 16) || !aligned(kI, 16)) return GSA_ERR_SHAPE;
    if (k_cap < 1 || k_cap > 8192) return GSA_ERR_SHAPE;
    hipError_t e = launch_select16(*shape, row_begin, row_end, keys, ld_keys, n_sel, k_cap, idx_out, shape->Lq, 0, qI, kI, w,
                                   bI, nullptr, tuning_or_default(tuning).select_wave_min_rows, kNoPages,
                                   static_cast<hipStream_t>(stream));
    return e == hipSuccess ? GSA_OK : hip_fail(e, "gsa_topk_select_keys");
}

size_t gsa_attn_workspace_bytes(const gsa_shape* shape, int32_t row_begin, int32_t row_end, int32_t k_cap,
                                const gsa_tuning* tuning) {
    if (check_shape(shape) != GSA_OK || check_rows(shape, row_begin, row_end) != GSA_OK || k_cap < 1 || k_cap > 8192) return 0;
    return up256(attn_workspace_bytes(*shape, row_begin, row_end, k_cap, tuning_or_default(tuning)));
}

int32_t gsa_sparse_gated_attn(const gsa_shape* shape, int32_t row_begin, int32_t row_end, const void* Q, const void* K,
                              const void* V, const void* g2_logits, const void* g1_logits, const int32_t* idx,
                              const int32_t* n_sel, int32_t k_cap, float softmax_scale, void* out, void* workspace,
                              size_t workspace_bytes, const gsa_tuning* tuning, void* stream) {
    int32_t rc = check_shape(shape);
    if (rc != GSA_OK) return rc;
    if (!Q || !K || !V || !idx || !n_sel || !out) return GSA_ERR_NULL;
    rc = check_rows(shape, row_begin, row_end);
    if (rc != GSA_OK) return rc;
    if (k_cap < 1 || k_cap > 8192) return GSA_ERR_SHAPE;
    if (!(softmax_scale >= 0.0f) || !std::isfinite(softmax_scale)) return GSA_ERR_SHAPE;
    if (!aligned(Q, 16) || !aligned(K, 16) || !aligned(V, 16) || !aligned(out, 16) || (g1_logits && !aligned(g1_logits, 16)) ||
        (g2_logits && !aligned(g2_logits, 16)))
        return GSA_ERR_SHAPE;
    const gsa_tuning& tn = tuning_or_default(tuning);
    const size_t need = attn_workspace_bytes(*shape, row_begin, row_end, k_cap, tn);
    if (need > 0 && (!workspace || !aligned(workspace, 256) || workspace_bytes < need)) return GSA_ERR_WORKSPACE;
    const float scale = softmax_scale > 0.0f ? softmax_scale : 1.0f / std::sqrt((float)shape->d_h);
    hipError_t e = launch_attention(*shape, row_begin, row_end, Q, K, V, g2_logits, g1_logits, idx, shape->Lq, 0, n_sel,
                                    k_cap, scale, out, workspace, tn, 0, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? GSA_OK : hip_fail(e, "gsa_sparse_gated_attn");
}

size_t gsa_dense_attn_workspace_bytes(const gsa_shape* shape, int32_t has_g2) {
    if (check_shape(shape) != GSA_OK || !has_g2) return 0;
    return up256((size_t)shape->B * shape->Lk * shape->H_kv * shape->d_h * elt_bytes(*shape));
}

int32_t gsa_dense_gated_attn(const gsa_shape* shape, int32_t row_begin, int32_t row_end, const void* Q, const void* K,
                             const void* V, const void* g2_logits, const void* g1_logits, float softmax_scale, void* out,
                             void* workspace, size_t workspace_bytes, void* stream) {
    int32_t rc = check_shape(shape);
    if (rc != GSA_OK) return rc;
    if (shape->dtype != GSA_BF16) return GSA_ERR_UNSUPPORTED;
    if (!Q || !K || !V || !out) return GSA_ERR_NULL;
    rc = check_rows(shape, row_begin, row_end);
    if (rc != GSA_OK) return rc;
    if (!(softmax_scale >= 0.0f) || !std::isfinite(softmax_scale)) return GSA_ERR_SHAPE;
    if (!aligned(Q, 16) || !aligned(K, 16) || !aligned(V, 16) || !aligned(out, 16) || (g1_logits && !aligned(g1_logits, 16)) ||
        (g2_logits && !aligned(g2_logits, 16)))
        return GSA_ERR_SHAPE;
    const size_t need = gsa_dense_attn_workspace_bytes(shape, g2_logits != nullptr);
    if (need > 0 && (!workspace || !aligned(workspace, 256) || workspace_bytes < need)) return GSA_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const void* Vuse = V;
    if (g2_logits) {
        hipError_t e = launch_value_gate(*shape, V, g2_logits, workspace, st);
        if (e != hipSuccess) return hip_fail(e, "gsa_dense_gated_attn/value_gate");
        Vuse = workspace;
    }
    const float scale = softmax_scale > 0.0f ? softmax_scale : 1.0f / std::sqrt((float)shape->d_h);
    hipError_t e = launch_dense_attention(*shape, row_begin, row_end, Q, K, Vuse, g1_logits, scale, out, st);
    return e == hipSuccess ? GSA_OK : hip_fail(e, "gsa_dense_gated_attn");
}

int32_t gsa_value_gate(const gsa_shape* shape, const void* V, const void* g2_logits, void* Vg, void* stream) {
    int32_t rc = check_shape(shape);
    if (rc != GSA_OK) return rc;
    if (!V || !g2_logits || !Vg) return GSA_ERR_NULL;
    if (!aligned(V, 16) || !aligned(g2_logits, 16) || !aligned(Vg, 16)) return GSA_ERR_SHAPE;
    hipError_t e = launch_value_gate(*shape, V, g2_logits, Vg, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? GSA_OK : hip_fail(e, "gsa_value_gate");
}

int32_t gsa_probe_gather(const void* table, int64_t table_rows, const int32_t* idx, int64_t n_idx, int32_t waves,
                         uint32_t* sink, void* stream) {
    if (!table || !idx || !sink) return GSA_ERR_NULL;
    if (table_rows < 1 || table_rows > 0x7fffffffLL || n_idx < 64 || (n_idx & 63) != 0 || waves < 4 || (waves & 3) != 0)
        return GSA_ERR_SHAPE;
    if (!aligned(table, 16)) return GSA_ERR_SHAPE;
    hipError_t e = launch_probe_gather(table, idx, n_idx, waves, sink, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? GSA_OK : hip_fail(e, "gsa_probe_gather");
}

int32_t gsa_probe_gather_staged(const void* table, int64_t table_rows, const int32_t* idx, int64_t n_idx, int32_t waves,
                                uint32_t* sink, void* stream) {
    if (!table || !idx || !sink) return GSA_ERR_NULL;
    if (table_rows < 1 || table_rows > 0x7fffffffLL || n_idx < 64 || (n_idx & 63) != 0 || waves < 4 || (waves & 3) != 0)
        return GSA_ERR_SHAPE;
    if (!aligned(table, 16)) return GSA_ERR_SHAPE;
    hipError_t e = launch_probe_gather_staged(table, idx, n_idx, waves, sink, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? GSA_OK : hip_fail(e, "gsa_probe_gather_staged");
}

size_t gsa_forward_workspace_bytes(const gsa_shape* shape, int32_t k_cap, int32_t has_g2, int32_t slab_rows,
                                   const gsa_tuning* tuning) {
    if (check_shape(shape) != GSA_OK || check_select_len(shape) != GSA_OK || k_cap < 1 || k_cap > 8192) return 0;
    return forward_bytes_uniform(*shape, k_cap, has_g2 != 0, slab_rows <= 0 ? 1 : cdiv(slab_rows, 128), tuning_or_default(tuning));
}

int32_t gsa_forward(const gsa_shape* shape, const gsa_adaptive* ctl, const void* Q, const void* K, const void* V,
                    const void* g1_logits, const void* g2_logits, const void* qI, const void* kI, const float* w,
                    const float* bI, float softmax_scale, void* out, int32_t* idx_out, int32_t* n_sel_out,
                    int32_t* k_out, float* row_var_out, int32_t k_cap, void* workspace, size_t workspace_bytes,
                    const gsa_tuning* tuning, void* stream) {
    int32_t rc = check_forward_args(shape, ctl, Q, K, V, g1_logits, g2_logits, qI, kI, w, softmax_scale, out, k_cap);
    if (rc != GSA_OK) return rc;
    if (ctl->dense_below > shape->Lk) {  // short context: dense attention over every visible key (Sec. 8)
        if (idx_out || n_sel_out || k_out || row_var_out) return GSA_ERR_SHAPE;
        return gsa_dense_gated_attn(shape, 0, shape->Lq, Q, K, V, g2_logits, g1_logits, softmax_scale, out, workspace,
                                    workspace_bytes, stream);
    }
    if (!workspace || !aligned(workspace, 256)) return GSA_ERR_WORKSPACE;
    const gsa_shape& s = *shape;
    const gsa_tuning& tn = tuning_or_default(tuning);
    const size_t fixed = plan_fixed(s, k_cap, g2_logits != nullptr).total;
    if (fixed > workspace_bytes ||
        !slabs_fit(s, k_cap, idx_out == nullptr, forward_keys(s, tn), false, workspace_bytes - fixed, tn))
        return GSA_ERR_WORKSPACE;
    return forward_launches(s, *ctl, Q, K, V, g1_logits, g2_logits, qI, kI, w, bI, softmax_scale, out, idx_out, n_sel_out,
                            k_out, row_var_out, k_cap, static_cast<unsigned char*>(workspace), workspace_bytes, nullptr, kNoPages, tn,
                            static_cast<hipStream_t>(stream));
}

size_t gsa_decode_workspace_bytes(const gsa_shape* shape, int32_t k_cap, const gsa_tuning* tuning) {
    if (check_shape(shape) != GSA_OK || check_select_len(shape) != GSA_OK || k_cap < 1 || k_cap > 8192) return 0;
    gsa_tuning tn = tuning_or_default(tuning);
    tn.attn_window = -1;
    return forward_bytes_uniform(*shape, k_cap, false, cdiv(shape->Lq, 128), tn, kRagged);
}

int32_t gsa_decode_step(const gsa_shape* shape, const gsa_adaptive* ctl, const void* Q, const void* g1_logits, const void* qI,
                        const float* w, const float* bI, const void* kI_cache, const void* K_cache, const void* Vg_cache,
                        const int32_t* seq_lens, float softmax_scale, void* out, int32_t* idx_out, int32_t* n_sel_out,
                        int32_t* k_out, float* row_var_out, int32_t k_cap, void* workspace, size_t workspace_bytes,
                        const gsa_tuning* tuning, void* stream) {
    int32_t rc = check_forward_args(shape, ctl, Q, K_cache, Vg_cache, g1_logits, nullptr, qI, kI_cache, w, softmax_scale, out, k_cap);
    if (rc != GSA_OK) return rc;
    if (!seq_lens) return GSA_ERR_NULL;
    if (ctl->dense_below > 0) return GSA_ERR_UNSUPPORTED;  // the dense kernel takes one context length for the whole batch
    if (!workspace || !aligned(workspace, 256)) return GSA_ERR_WORKSPACE;
    const gsa_shape& s = *shape;
    gsa_tuning tn = tuning_or_default(tuning);
    tn.attn_window = -1;  // which rows see which key window is only known on the device: no windows
    const size_t fixed = plan_fixed(s, k_cap, false).total;
    if (fixed > workspace_bytes || !slabs_fit(s, k_cap, idx_out == nullptr, forward_keys(s, tn), kRagged, workspace_bytes - fixed, tn))
        return GSA_ERR_WORKSPACE;
    return forward_launches(s, *ctl, Q, K_cache, Vg_cache, g1_logits, nullptr, qI, kI_cache, w, bI, softmax_scale, out, idx_out,
                            n_sel_out, k_out, row_var_out, k_cap, static_cast<unsigned char*>(workspace), workspace_bytes,
                            seq_lens, kNoPages, tn, static_cast<hipStream_t>(stream));
}

// ---- paged caches ------------------------------------------------------------------------------------
// page_size: a power of two, at least 128 tokens (an indexer key tile must not straddle two pages); Lk (the capacity of
// a sequence) a multiple of it; the pool below 2^31 rows.
static int32_t make_page_map(const gsa_shape& s, int32_t page_size, const int32_t* block_table, int32_t pool_pages, PageMap* pm) {
    if (!block_table) return GSA_ERR_NULL;
    if (page_size < 128 || (page_size & (page_size - 1)) != 0 || s.Lk % page_size != 0 || pool_pages < 1) return GSA_ERR_SHAPE;
    if ((int64_t)pool_pages * page_size > 0x7fffffffLL) return GSA_ERR_UNSUPPORTED;
    int shift = 0;
    while ((1 << shift) < page_size) ++shift;
    *pm = PageMap{block_table, shift, s.Lk / page_size, pool_pages};
    return GSA_OK;
}

size_t gsa_paged_decode_workspace_bytes(const gsa_shape* shape, int32_t k_cap, const gsa_tuning* tuning) {
    if (check_shape(shape) != GSA_OK || k_cap < 1 || k_cap > 8192) return 0;
    gsa_tuning tn = tuning_or_default(tuning);
    tn.attn_window = -1;
    return forward_bytes_uniform(*shape, k_cap, false, cdiv(shape->Lq, 128), tn, kPaged);
}

int32_t gsa_paged_decode_step(const gsa_shape* shape, const gsa_adaptive* ctl, int32_t page_size, const int32_t* block_table,
                              int32_t pool_pages, const void* Q, const void* g1_logits, const void* qI, const float* w,
                              const float* bI, const void* kI_pool, const void* K_pool, const void* Vg_pool,
                              const int32_t* seq_lens, float softmax_scale, void* out, int32_t* idx_out, int32_t* n_sel_out,
                              int32_t* k_out, float* row_var_out, int32_t k_cap, void* workspace, size_t workspace_bytes,
                              const gsa_tuning* tuning, void* stream) {
    int32_t rc = check_forward_args(shape, ctl, Q, K_pool, Vg_pool, g1_logits, nullptr, qI, kI_pool, w, softmax_scale, out, k_cap);
    if (rc != GSA_OK) return rc;
    if (!seq_lens) return GSA_ERR_NULL;
    if (ctl->dense_below > 0) return GSA_ERR_UNSUPPORTED;
    PageMap pm;
    rc = make_page_map(*shape, page_size, block_table, pool_pages, &pm);
    if (rc != GSA_OK) return rc;
    if (!workspace || !aligned(workspace, 256)) return GSA_ERR_WORKSPACE;
    const gsa_shape& s = *shape;
    gsa_tuning tn = tuning_or_default(tuning);
    tn.attn_window = -1;
    const size_t fixed = plan_fixed(s, k_cap, false).total;
    if (fixed > workspace_bytes || !slabs_fit(s, k_cap, idx_out == nullptr, forward_keys(s, tn), kPaged, workspace_bytes - fixed, tn))
        return GSA_ERR_WORKSPACE;
    return forward_launches(s, *ctl, Q, K_pool, Vg_pool, g1_logits, nullptr, qI, kI_pool, w, bI, softmax_scale, out, idx_out,
                            n_sel_out, k_out, row_var_out, k_cap, static_cast<unsigned char*>(workspace), workspace_bytes,
                            seq_lens, pm, tn, static_cast<hipStream_t>(stream));
}

int32_t gsa_paged_cache_append(const gsa_shape* shape, int32_t page_size, const int32_t* block_table, int32_t pool_pages,
                               const void* kI_new, const void* K_new, const void* V_new, const void* g2_new,
                               const int32_t* seq_lens, void* kI_pool, void* K_pool, void* Vg_pool, int32_t* seq_lens_out,
                               void* stream) {
    int32_t rc = check_shape(shape);
    if (rc != GSA_OK) return rc;
    if (!kI_new || !K_new || !V_new || !g2_new || !seq_lens || !kI_pool || !K_pool || !Vg_pool) return GSA_ERR_NULL;
    if (seq_lens_out == seq_lens) return GSA_ERR_SHAPE;
    if (!aligned(kI_new, 16) || !aligned(K_new, 16) || !aligned(V_new, 16) || !aligned(g2_new, 16) || !aligned(kI_pool, 16) ||
        !aligned(K_pool, 16) || !aligned(Vg_pool, 16))
        return GSA_ERR_SHAPE;
    PageMap pm;
    rc = make_page_map(*shape, page_size, block_table, pool_pages, &pm);
    if (rc != GSA_OK) return rc;
    hipError_t e = launch_cache_append(*shape, kI_new, K_new, V_new, g2_new, seq_lens, kI_pool, K_pool, Vg_pool, seq_lens_out, pm,
                                       static_cast<hipStream_t>(stream));
    return e == hipSuccess ? GSA_OK : hip_fail(e, "gsa_paged_cache_append");
}

int32_t gsa_cache_append(const gsa_shape* shape, const void* kI_new, const void* K_new, const void* V_new, const void* g2_new,
                         const int32_t* seq_lens, void* kI_cache, void* K_cache, void* Vg_cache, int32_t* seq_lens_out,
                         void* stream) {
    int32_t rc = check_shape(shape);
    if (rc != GSA_OK) return rc;
    if (!kI_new || !K_new || !V_new || !g2_new || !seq_lens || !kI_cache || !K_cache || !Vg_cache) return GSA_ERR_NULL;
    if (seq_lens_out == seq_lens) return GSA_ERR_SHAPE;  // lengths are read by every thread while they would be rewritten
    if (!aligned(kI_new, 16) || !aligned(K_new, 16) || !aligned(V_new, 16) || !aligned(g2_new, 16) || !aligned(kI_cache, 16) ||
        !aligned(K_cache, 16) || !aligned(Vg_cache, 16))
        return GSA_ERR_SHAPE;
    hipError_t e = launch_cache_append(*shape, kI_new, K_new, V_new, g2_new, seq_lens, kI_cache, K_cache, Vg_cache, seq_lens_out,
                                       kNoPages, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? GSA_OK : hip_fail(e, "gsa_cache_append");
}

// Shared by both projection entry points: d_model is the contraction length of every weight matrix.
static int32_t check_projection(const gsa_shape* shape, int32_t d_model, const void* x) {
    int32_t rc = check_shape(shape);
    if (rc != GSA_OK) return rc;
    if (!x) return GSA_ERR_NULL;
    if (shape->dtype != GSA_BF16) return GSA_ERR_UNSUPPORTED;
    if (d_model < 64 || d_model % 64 != 0) return GSA_ERR_UNSUPPORTED;
    if (!aligned(x, 16)) return GSA_ERR_SHAPE;
    return GSA_OK;
}

int32_t gsa_input_projections(const gsa_shape* shape, int32_t d_model, const void* h, const void* W_Q, const void* W_K,
                              const void* W_V, const void* W_g1, const void* W_g2, const void* W_qI, const void* W_kI,
                              const void* W_Iw, void* Q, void* K, void* V, void* g1_logits, void* g2_logits, void* qI, void* kI,
                              float* w, void* stream) {
    int32_t rc = check_projection(shape, d_model, h);
    if (rc != GSA_OK) return rc;
    const gsa_shape& s = *shape;
    const void* Wm[8] = {W_Q, W_K, W_V, W_g1, W_g2, W_qI, W_kI, W_Iw};
    void* dst[8] = {Q, K, V, g1_logits, g2_logits, qI, kI, w};
    const int32_t feat[8] = {s.H * s.d_h, s.H_kv * s.d_h, s.H_kv * s.d_h, s.H * s.d_h, s.H_kv * s.d_h, s.HI * s.dI, s.dI, s.HI};
    const void* Wu[8];
    void* du[8];
    int32_t width[8], kind[8];
    int n = 0;
    for (int i = 0; i < 8; ++i) {
        if (!Wm[i] && !dst[i]) continue;              // a projection that is not asked for
        if (!Wm[i] || !dst[i]) return GSA_ERR_NULL;   // weights without a destination, or the reverse
        if (!aligned(Wm[i], 16) || !aligned(dst[i], 8)) return GSA_ERR_SHAPE;
        Wu[n] = Wm[i];
        du[n] = dst[i];
        width[n] = feat[i];
        kind[n] = i == 7 ? 1 : 0;
        ++n;
    }
    if (n == 0) return GSA_ERR_NULL;
    hipError_t e = launch_projection(h, (int64_t)s.B * s.Lq, d_model, n, Wu, du, width, kind, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? GSA_OK : hip_fail(e, "gsa_input_projections");
}

int32_t gsa_output_projection(const gsa_shape* shape, int32_t d_model, const void* attn_out, const void* W_O, void* y,
                              void* stream) {
    int32_t rc = check_shape(shape);
    if (rc != GSA_OK) return rc;
    if (!attn_out || !W_O || !y) return GSA_ERR_NULL;
    if (shape->dtype != GSA_BF16) return GSA_ERR_UNSUPPORTED;
    const int32_t Kc = shape->H * shape->d_h;         // contraction over the concatenated heads
    if (d_model < 1 || Kc % 64 != 0) return GSA_ERR_UNSUPPORTED;
    if (!aligned(attn_out, 16) || !aligned(W_O, 16) || !aligned(y, 8)) return GSA_ERR_SHAPE;
    const void* Wu[1] = {W_O};
    void* du[1] = {y};
    const int32_t width[1] = {d_model}, kind[1] = {0};
    hipError_t e = launch_projection(attn_out, (int64_t)shape->B * shape->Lq, Kc, 1, Wu, du, width, kind,
                                     static_cast<hipStream_t>(stream));
    return e == hipSuccess ? GSA_OK : hip_fail(e, "gsa_output_projection");
}

size_t gsa_attn_bwd_workspace_bytes(const gsa_shape* shape, int32_t k_cap) {
    if (check_shape(shape) != GSA_OK || k_cap < 1 || k_cap > 8192) return 0;
    return up256(attention_bwd_workspace_bytes(*shape, k_cap));
}

int32_t gsa_sparse_gated_attn_bwd(const gsa_shape* shape, const void* Q, const void* K, const void* V, const void* g2_logits,
                                  const void* g1_logits, const int32_t* idx, const int32_t* n_sel, int32_t k_cap,
                                  float softmax_scale, const void* dout, float* dQ, float* dK, float* dV, float* dg1, float* dg2,
                                  float* p_mean, void* workspace, size_t workspace_bytes, void* stream) {
    int32_t rc = check_shape(shape);
    if (rc != GSA_OK) return rc;
    if (!Q || !K || !V || !idx || !n_sel || !dout || !dQ || !dK || !dV) return GSA_ERR_NULL;
    if ((g1_logits == nullptr) != (dg1 == nullptr) || (g2_logits == nullptr) != (dg2 == nullptr)) return GSA_ERR_NULL;
    if (k_cap < 1 || k_cap > 8192) return GSA_ERR_SHAPE;
    if (!(softmax_scale >= 0.0f) || !std::isfinite(softmax_scale)) return GSA_ERR_SHAPE;
    if (workspace) {
        if (!aligned(workspace, 256)) return GSA_ERR_SHAPE;
        const size_t need = attention_bwd_workspace_bytes(*shape, k_cap);
        if (workspace_bytes < need) {
            g_last_error = "gsa_sparse_gated_attn_bwd: workspace of " + std::to_string(workspace_bytes) + " bytes, " + std::to_string(need) +
                           " needed (gsa_attn_bwd_workspace_bytes)";
            return GSA_ERR_WORKSPACE;
        }
        if ((int64_t)shape->B * shape->Lq * k_cap > 0x7fffffffLL) return GSA_ERR_UNSUPPORTED;  // list positions are 32-bit
    }
    const float scale = softmax_scale > 0.0f ? softmax_scale : 1.0f / std::sqrt((float)shape->d_h);
    hipError_t e = launch_attention_bwd(*shape, Q, K, V, g2_logits, g1_logits, idx, n_sel, k_cap, scale, dout, dQ, dK, dV, dg1, dg2,
                                        p_mean, workspace, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? GSA_OK : hip_fail(e, "gsa_sparse_gated_attn_bwd");
}

int32_t gsa_indexer_sparse_kl(const gsa_shape* shape, const void* qI, const void* kI, const float* w, const float* bI,
                              const int32_t* idx, const int32_t* n_sel, int32_t k_cap, const float* p, float* loss_rows,
                              float* dqI, float* dkI, float* dw, float* dbI, void* stream) {
    int32_t rc = check_shape(shape);
    if (rc != GSA_OK) return rc;
    if (shape->indexer_act != GSA_ACT_SIGMOID) return GSA_ERR_UNSUPPORTED;
    if (!qI || !kI || !w || !idx || !n_sel || !p || !loss_rows || !dqI || !dkI || !dw) return GSA_ERR_NULL;
    if ((bI == nullptr) != (dbI == nullptr)) return GSA_ERR_NULL;
    if (k_cap < 1 || k_cap > 8192) return GSA_ERR_SHAPE;
    hipError_t e = launch_indexer_kl(*shape, qI, kI, w, bI, idx, n_sel, k_cap, p, loss_rows, dqI, dkI, dw, dbI,
                                     static_cast<hipStream_t>(stream));
    return e == hipSuccess ? GSA_OK : hip_fail(e, "gsa_indexer_sparse_kl");
}

int32_t gsa_forward_noalloc(const gsa_shape* shape, const gsa_adaptive* ctl, const void* Q, const void* K, const void* V,
                            const void* g1_logits, const void* g2_logits, const void* qI, const void* kI, const float* w,
                            const float* bI, float softmax_scale, void* out, int32_t* idx_out, int32_t* n_sel_out,
                            int32_t* k_out, float* row_var_out, int32_t k_cap, const gsa_tuning* tuning, void* stream) {
    int32_t rc = check_forward_args(shape, ctl, Q, K, V, g1_logits, g2_logits, qI, kI, w, softmax_scale, out, k_cap);
    if (rc != GSA_OK) return rc;
    const gsa_shape& s = *shape;
    const gsa_tuning& tn = tuning_or_default(tuning);
    if (ctl->dense_below > s.Lk) {  // short context: dense attention over every visible key (Sec. 8)
        if (idx_out || n_sel_out || k_out || row_var_out) return GSA_ERR_SHAPE;
        if (gsa_dense_attn_workspace_bytes(shape, g2_logits != nullptr) > kStaticScratchBytes) {
            g_last_error = "gsa_forward_noalloc: the gated values of this problem exceed the library's static scratch";
            return GSA_ERR_WORKSPACE;
        }
        unsigned char* dws = nullptr;
        rc = static_scratch(&dws);
        if (rc != GSA_OK) return rc;
        return gsa_dense_gated_attn(shape, 0, s.Lq, Q, K, V, g2_logits, g1_logits, softmax_scale, out, dws, kStaticScratchBytes,
                                    stream);
    }
    const size_t fixed = plan_fixed(s, k_cap, g2_logits != nullptr).total;
    if (fixed > kStaticScratchBytes ||
        !slabs_fit(s, k_cap, idx_out == nullptr, forward_keys(s, tn), false, kStaticScratchBytes - fixed, tn)) {
        g_last_error = "gsa_forward_noalloc: this problem needs " +
                       std::to_string(forward_bytes_uniform(s, k_cap, g2_logits != nullptr, 1, tn)) +
                       " bytes of scratch, the library's static scratch holds " + std::to_string(kStaticScratchBytes) +
                       "; use gsa_forward with a workspace";
        return GSA_ERR_WORKSPACE;
    }
    unsigned char* ws = nullptr;
    rc = static_scratch(&ws);
    if (rc != GSA_OK) return rc;
    // nothing in the scratch has to start at zero: every kernel writes what it later reads
    return forward_launches(s, *ctl, Q, K, V, g1_logits, g2_logits, qI, kI, w, bI, softmax_scale, out, idx_out, n_sel_out,
                            k_out, row_var_out, k_cap, ws, kStaticScratchBytes, nullptr, kNoPages, tn,
                            static_cast<hipStream_t>(stream));
}

}  // extern "C"
