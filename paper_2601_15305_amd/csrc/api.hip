// C ABI of libgsa: host-side argument validation, workspace carving and launch sequencing.
// Every error that can be decided from the arguments is returned before anything is launched.
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <string>

#include "common.hpp"

namespace gsa {
// defined in indexer.hip / select.hip / attention.hip
void indexer_plan(const gsa_shape& sh, int row_begin, int row_end, int* kc_out, int* nsplit_out, int* ntiles_out);
size_t indexer_workspace_bytes(const gsa_shape& sh, int row_begin, int row_end);
hipError_t launch_indexer(const gsa_shape& sh, const void* qI, const void* kI, const float* w, const float* bI,
                          int row_begin, int row_end, float* scores, uint16_t* keys, int64_t ld, float* row_mean,
                          float* row_var, void* workspace, hipStream_t st);
hipError_t launch_select(const gsa_shape& sh, int row_begin, int row_end, const float* scores, int64_t ld,
                         const int32_t* n_sel, int k_cap, int32_t* idx_out, int idx_rows, int idx_row0, hipStream_t st);
hipError_t launch_select16(const gsa_shape& sh, int row_begin, int row_end, const uint16_t* keys, int64_t ld,
                           const int32_t* n_sel, int k_cap, int32_t* idx_out, int idx_rows, int idx_row0, const void* qI,
                           const void* kI, const float* w, const float* bI, hipStream_t st);
hipError_t launch_adaptive_k(const gsa_shape& sh, const gsa_adaptive& c, int row_begin, int row_end,
                             const float* row_var, int32_t* k_out, int32_t* n_sel_out, hipStream_t st);
hipError_t launch_value_gate(const gsa_shape& sh, const void* V, const void* g2, void* Vg, hipStream_t st);
hipError_t launch_attention(const gsa_shape& sh, int row_begin, int row_end, const void* Q, const void* K, const void* V,
                            const void* g2, const void* g1, const int32_t* idx, int idx_rows, int idx_row0,
                            const int32_t* n_sel, int k_cap, float scale, void* out, void* workspace, hipStream_t st);
size_t attn_workspace_bytes(const gsa_shape& sh, int row_begin, int row_end, int k_cap);

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
    if (s->d_h != 64 && s->d_h != 128) return GSA_ERR_UNSUPPORTED;
    if (s->dI != 32 && s->dI != 64 && s->dI != 128) return GSA_ERR_UNSUPPORTED;
    if (s->HI != 1 && s->HI != 2 && s->HI != 4 && s->HI != 8) return GSA_ERR_UNSUPPORTED;
    if (s->H / s->H_kv > 16) return GSA_ERR_UNSUPPORTED;
    if (s->Lk > (1 << 20)) return GSA_ERR_UNSUPPORTED;
    if ((int64_t)s->B * s->Lq > 0x7fffffffLL) return GSA_ERR_UNSUPPORTED;
    return GSA_OK;
}

static int32_t check_rows(const gsa_shape* s, int32_t row_begin, int32_t row_end) {
    if (row_begin < 0 || row_end > s->Lq || row_begin >= row_end) return GSA_ERR_SHAPE;
    return GSA_OK;
}

static int32_t check_ctl(const gsa_adaptive* c) {
    if (!c) return GSA_ERR_NULL;
    if (c->k_fixed < 0) return GSA_ERR_SHAPE;
    if (c->k_fixed > 0) return GSA_OK;
    if (c->k_min < 1 || c->k_min > c->k_max || c->k_base < 1) return GSA_ERR_SHAPE;
    if (c->mode != 0 && c->mode != 1) return GSA_ERR_UNSUPPORTED;
    if (!(c->vbar > 0.0f) || !std::isfinite(c->vbar)) return GSA_ERR_VBAR;
    return GSA_OK;
}

static bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }
static size_t up256(size_t x) { return (x + 255) & ~(size_t)255; }
static size_t elt_bytes(const gsa_shape& s) { return s.dtype == GSA_BF16 ? 2 : 4; }
static int64_t slab_ld(const gsa_shape& s) { return ((int64_t)s.Lk + 31) & ~(int64_t)31; }

// ---- forward workspace plan ---------------------------------------------------------------------
struct ForwardPlan {
    size_t off_vg, off_var, off_k, off_nsel, off_idx, off_scores, off_partial, off_attn, total;
    int slab_rows;
};

static int round_slab(const gsa_shape& s, int64_t rows) {
    if (rows >= s.Lq) return s.Lq;
    int64_t r = ((rows + 127) / 128) * 128;
    if (r < 128) r = 128;
    return (int)(r < s.Lq ? r : s.Lq);
}

// The value gate runs as a dense pre-pass (once per key token) when the queries together gather
// clearly more rows than there are tokens; otherwise (decode: one query against a long cache) it
// is applied in registers to the gathered rows only.
static bool gate_as_prepass(const gsa_shape& s, int k_cap) {
    const int64_t k_eff = k_cap < s.Lk ? k_cap : s.Lk;
    return (int64_t)s.Lq * k_eff >= 4 * (int64_t)s.Lk;
}

// Inside the fused forward the indexer hands 16-bit fixed-point keys to the selection instead of fp32
// scores (see select16.hip).  GSA_FORWARD_FP32_SCORES=1 in the environment keeps the fp32 slab, for
// comparison runs.
static bool forward_uses_keys() {
    const char* e = getenv("GSA_FORWARD_FP32_SCORES");
    return !(e && e[0] == '1');
}

static ForwardPlan plan_forward(const gsa_shape& s, int k_cap, bool has_g2, bool own_idx, int slab_rows) {
    ForwardPlan p;
    has_g2 = has_g2 && gate_as_prepass(s, k_cap);
    const int Rs = round_slab(s, slab_rows);
    p.slab_rows = Rs;
    size_t off = 0;
    p.off_vg = off;
    if (has_g2) off += up256((size_t)s.B * s.Lk * s.H_kv * s.d_h * elt_bytes(s));
    const size_t rows = (size_t)s.B * s.Lq;
    p.off_var = off;
    off += up256(rows * 4);
    p.off_k = off;
    off += up256(rows * 4);
    p.off_nsel = off;
    off += up256(rows * 4);
    p.off_idx = off;
    if (own_idx) off += up256((size_t)s.B * Rs * (size_t)k_cap * 4);
    p.off_scores = off;
    off += up256((size_t)s.B * Rs * (size_t)slab_ld(s) * 4);  // sized for fp32 scores; 16-bit keys use half of it
    p.off_partial = off;
    size_t part = 0, attn = 0;
    for (int r0 = 0; r0 < s.Lq; r0 += Rs) {
        const int r1 = r0 + Rs < s.Lq ? r0 + Rs : s.Lq;
        const size_t b = indexer_workspace_bytes(s, r0, r1);
        if (b > part) part = b;
        const size_t c = attn_workspace_bytes(s, r0, r1, k_cap);
        if (c > attn) attn = c;
    }
    off += up256(part);
    p.off_attn = off;
    off += up256(attn);
    p.total = off;
    return p;
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
    return up256(indexer_workspace_bytes(*shape, row_begin, row_end));
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
    if (!workspace || !aligned(workspace, 256) || workspace_bytes < indexer_workspace_bytes(*shape, row_begin, row_end))
        return GSA_ERR_WORKSPACE;
    hipError_t e = launch_indexer(*shape, qI, kI, w, bI, row_begin, row_end, scores, nullptr, ld_scores, row_mean, row_var,
                                  workspace, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? GSA_OK : hip_fail(e, "gsa_indexer_scores");
}

int32_t gsa_adaptive_k(const gsa_shape* shape, const gsa_adaptive* ctl, const float* row_var, int32_t* k_out,
                       int32_t* n_sel_out, void* stream) {
    int32_t rc = check_shape(shape);
    if (rc != GSA_OK) return rc;
    rc = check_ctl(ctl);
    if (rc != GSA_OK) return rc;
    if (!n_sel_out || (ctl->k_fixed == 0 && !row_var)) return GSA_ERR_NULL;
    hipError_t e = launch_adaptive_k(*shape, *ctl, 0, shape->Lq, row_var, k_out, n_sel_out, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? GSA_OK : hip_fail(e, "gsa_adaptive_k");
}

int32_t gsa_topk_select(const gsa_shape* shape, int32_t row_begin, int32_t row_end, const float* scores,
                        int64_t ld_scores, const int32_t* n_sel, int32_t k_cap, int32_t* idx_out, void* stream) {
    int32_t rc = check_shape(shape);
    if (rc != GSA_OK) return rc;
    if (!scores || !n_sel || !idx_out) return GSA_ERR_NULL;
    rc = check_rows(shape, row_begin, row_end);
    if (rc != GSA_OK) return rc;
    if (ld_scores < shape->Lk || (ld_scores & 3) != 0 || !aligned(scores, 16)) return GSA_ERR_SHAPE;
    if (k_cap < 1 || k_cap > 8192) return GSA_ERR_SHAPE;
    hipError_t e = launch_select(*shape, row_begin, row_end, scores, ld_scores, n_sel, k_cap, idx_out, shape->Lq, 0,
                                 static_cast<hipStream_t>(stream));
    return e == hipSuccess ? GSA_OK : hip_fail(e, "gsa_topk_select");
}

size_t gsa_attn_workspace_bytes(const gsa_shape* shape, int32_t row_begin, int32_t row_end, int32_t k_cap) {
    if (check_shape(shape) != GSA_OK || check_rows(shape, row_begin, row_end) != GSA_OK || k_cap < 1 || k_cap > 8192) return 0;
    return up256(attn_workspace_bytes(*shape, row_begin, row_end, k_cap));
}

int32_t gsa_sparse_gated_attn(const gsa_shape* shape, int32_t row_begin, int32_t row_end, const void* Q, const void* K,
                              const void* V, const void* g2_logits, const void* g1_logits, const int32_t* idx,
                              const int32_t* n_sel, int32_t k_cap, float softmax_scale, void* out, void* workspace,
                              size_t workspace_bytes, void* stream) {
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
    const size_t need = attn_workspace_bytes(*shape, row_begin, row_end, k_cap);
    if (need > 0 && (!workspace || !aligned(workspace, 256) || workspace_bytes < need)) return GSA_ERR_WORKSPACE;
    const float scale = softmax_scale > 0.0f ? softmax_scale : 1.0f / std::sqrt((float)shape->d_h);
    hipError_t e = launch_attention(*shape, row_begin, row_end, Q, K, V, g2_logits, g1_logits, idx, shape->Lq, 0, n_sel,
                                    k_cap, scale, out, workspace, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? GSA_OK : hip_fail(e, "gsa_sparse_gated_attn");
}

int32_t gsa_value_gate(const gsa_shape* shape, const void* V, const void* g2_logits, void* Vg, void* stream) {
    int32_t rc = check_shape(shape);
    if (rc != GSA_OK) return rc;
    if (!V || !g2_logits || !Vg) return GSA_ERR_NULL;
    if (!aligned(V, 16) || !aligned(g2_logits, 16) || !aligned(Vg, 16)) return GSA_ERR_SHAPE;
    hipError_t e = launch_value_gate(*shape, V, g2_logits, Vg, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? GSA_OK : hip_fail(e, "gsa_value_gate");
}

size_t gsa_forward_workspace_bytes(const gsa_shape* shape, int32_t k_cap, int32_t has_g2, int32_t slab_rows) {
    if (check_shape(shape) != GSA_OK || k_cap < 1 || k_cap > 8192) return 0;
    return plan_forward(*shape, k_cap, has_g2 != 0, true, slab_rows <= 0 ? 1 : slab_rows).total;
}

int32_t gsa_forward(const gsa_shape* shape, const gsa_adaptive* ctl, const void* Q, const void* K, const void* V,
                    const void* g1_logits, const void* g2_logits, const void* qI, const void* kI, const float* w,
                    const float* bI, float softmax_scale, void* out, int32_t* idx_out, int32_t* n_sel_out,
                    int32_t* k_out, float* row_var_out, int32_t k_cap, void* workspace, size_t workspace_bytes,
                    void* stream) {
    int32_t rc = check_shape(shape);
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
    if (!workspace || !aligned(workspace, 256)) return GSA_ERR_WORKSPACE;
    const gsa_shape& s = *shape;
    const bool has_g2 = g2_logits != nullptr;
    const bool prepass = has_g2 && gate_as_prepass(*shape, k_cap);
    const bool own_idx = idx_out == nullptr;
    // largest slab that fits the workspace: whole problem first, then halve
    ForwardPlan plan;
    int64_t rows = s.Lq;
    while (true) {
        plan = plan_forward(s, k_cap, has_g2, own_idx, (int)rows);
        if (plan.total <= workspace_bytes) break;
        if (plan.slab_rows <= 128 || plan.slab_rows <= 1) return GSA_ERR_WORKSPACE;
        rows = (plan.slab_rows + 1) / 2;
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    unsigned char* ws = static_cast<unsigned char*>(workspace);
    const float scale = softmax_scale > 0.0f ? softmax_scale : 1.0f / std::sqrt((float)s.d_h);
    const void* Vuse = V;
    const void* g2use = has_g2 ? g2_logits : nullptr;
    hipError_t e;
    if (prepass) {  // stage (2) of Sec. 4: the value gate, once per token
        e = launch_value_gate(s, V, g2_logits, ws + plan.off_vg, st);
        if (e != hipSuccess) return hip_fail(e, "gsa_forward/value_gate");
        Vuse = ws + plan.off_vg;
        g2use = nullptr;
    }
    float* var = row_var_out ? row_var_out : reinterpret_cast<float*>(ws + plan.off_var);
    int32_t* kbuf = k_out ? k_out : reinterpret_cast<int32_t*>(ws + plan.off_k);
    int32_t* nsel = n_sel_out ? n_sel_out : reinterpret_cast<int32_t*>(ws + plan.off_nsel);
    float* scores = reinterpret_cast<float*>(ws + plan.off_scores);
    uint16_t* keys = reinterpret_cast<uint16_t*>(ws + plan.off_scores);
    const bool use_keys = forward_uses_keys();
    const int64_t ld = slab_ld(s);
    const int Rs = plan.slab_rows;
    for (int r0 = 0; r0 < s.Lq; r0 += Rs) {
        const int r1 = r0 + Rs < s.Lq ? r0 + Rs : s.Lq;
        e = launch_indexer(s, qI, kI, w, bI, r0, r1, use_keys ? nullptr : scores, use_keys ? keys : nullptr, ld, nullptr, var,
                           ws + plan.off_partial, st);
        if (e != hipSuccess) return hip_fail(e, "gsa_forward/indexer");
        e = launch_adaptive_k(s, *ctl, r0, r1, var, kbuf, nsel, st);
        if (e != hipSuccess) return hip_fail(e, "gsa_forward/adaptive_k");
        int32_t* idx = own_idx ? reinterpret_cast<int32_t*>(ws + plan.off_idx) : idx_out;
        const int idx_rows = own_idx ? (r1 - r0) : s.Lq;
        const int idx_row0 = own_idx ? r0 : 0;
        e = use_keys ? launch_select16(s, r0, r1, keys, ld, nsel, k_cap, idx, idx_rows, idx_row0, qI, kI, w, bI, st)
                     : launch_select(s, r0, r1, scores, ld, nsel, k_cap, idx, idx_rows, idx_row0, st);
        if (e != hipSuccess) return hip_fail(e, "gsa_forward/select");
        e = launch_attention(s, r0, r1, Q, K, Vuse, g2use, g1_logits, idx, idx_rows, idx_row0, nsel, k_cap, scale, out,
                             ws + plan.off_attn, st);
        if (e != hipSuccess) return hip_fail(e, "gsa_forward/attention");
    }
    return GSA_OK;
}

}  // extern "C"
