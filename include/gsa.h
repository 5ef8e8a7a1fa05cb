/*
 * libgsa -- forward path of Gated Sparse Attention (GSA) on AMD MI355X (gfx950).
 *
 * C ABI.  Every pointer named "device" is GPU memory owned by the caller; the
 * library never allocates, never frees and never synchronises: each call
 * validates its arguments on the host, enqueues kernels on the caller's HIP
 * stream (`stream` is a hipStream_t passed as void*, NULL = default stream)
 * and returns.  Scratch memory is a caller-supplied workspace whose size is
 * queried with the *_workspace_bytes helpers.  The library keeps no state
 * between calls apart from the text of the last HIP error of the calling
 * thread, and reads no environment variables: every switch is an argument
 * (gsa_tuning).
 *
 * Notation follows the paper: L (Lq query rows, Lk keys), H = n_h query
 * heads, H_kv = n_kv key-value heads, d_h = d_k head dimension, HI = H^I
 * indexer heads, dI = d^I indexer dimension, k_min/k_max/k_base the budget
 * bounds of the adaptive controller.
 *
 * Layouts (row-major, token-major, innermost index last):
 *   qI [B, Lq, HI, dI]   kI [B, Lk, dI]          w [B, Lq, HI] fp32   bI [HI] fp32
 *   Q, g1, out [B, Lq, H, d_h]                   K, V, g2 [B, Lk, H_kv, d_h]
 *   idx [B, Lq, k_cap] int32                     n_sel, k [B, Lq] int32
 *   row_mean, row_var [B, Lq] fp32
 * qI, kI, Q, K, V, g1, g2, out have the element type named by gsa_shape.dtype;
 * all base pointers must be 16-byte aligned.
 *
 * Causality: query row i has absolute position p = q_offset + i and sees keys
 * s = 0 .. min(p, Lk-1), itself included.  Prefill: Lq = Lk, q_offset = 0.
 * Decode: Lq = 1, q_offset = Lk - 1.
 *
 * Return value of every call: GSA_OK or a negative gsa_status.  All argument
 * errors are detected before anything is launched.
 */
#ifndef GSA_H
#define GSA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum gsa_dtype { GSA_F32 = 0, GSA_BF16 = 1 };

/* Activation of the indexer.  GSA_ACT_SIGMOID is the gated lightning indexer of Sec. 3.3 (the method).
 * GSA_ACT_RELU is the comparison variant of Sec. 2.2 Eq. 3, I[t,s] = sum_j w[t,j] * ReLU(qI[t,j,:] . kI[s,:] (+ bI[j])):
 * with k_fixed and no gates it gives the "sparse only" baseline of Sec. 7.1.  Its scores are unbounded, so the
 * fused forward keeps fp32 scores for it (no 16-bit keys); w must be >= 0 (the selection ranks negative
 * scores as zero). */
enum gsa_indexer_act { GSA_ACT_SIGMOID = 0, GSA_ACT_RELU = 1 };

enum gsa_status {
    GSA_OK = 0,
    GSA_ERR_NULL = -1,        /* a required pointer is NULL */
    GSA_ERR_SHAPE = -2,       /* non-positive or inconsistent dimensions / row range / k bounds */
    GSA_ERR_UNSUPPORTED = -3, /* d_h, dI, HI, H/H_kv or dtype outside what the kernels are built for */
    GSA_ERR_VBAR = -4,        /* controller on and vbar not a positive finite number */
    GSA_ERR_WORKSPACE = -5,   /* workspace NULL, misaligned (256 B) or too small */
    GSA_ERR_HIP = -6          /* a launch failed; see gsa_last_error() */
};

/* Problem shape.  Supported: d_h in {64,128}; dI in {32,64,128}; 1 <= HI <= 8;
 * H % H_kv == 0 and H/H_kv <= 16; Lk * H_kv * d_h * sizeof(element) <= 2^32 (the keys of one batch element
 * span at most 4 GiB); Lk <= 2^20 (the selection calls, gsa_topk_select and gsa_forward, keep
 * bitmaps of a row on chip and take Lk <= GSA_SELECT_MAX_LK); q_offset + Lq <= Lk. */
#define GSA_SELECT_MAX_LK 393216
typedef struct gsa_shape {
    int32_t B, Lq, Lk, q_offset;
    int32_t H, H_kv, d_h;
    int32_t HI, dI;
    int32_t dtype;       /* gsa_dtype */
    int32_t indexer_act; /* gsa_indexer_act */
} gsa_shape;

/* Adaptive sparsity controller, Sec. 3.4, Eq. "adaptive_k":
 *   k_t = clamp(floor(k_base * Var(I_t,:) / vbar), k_min, k_max).
 * mode 0 is that equation as printed; mode 1 uses the inverse ratio
 * k_base * vbar / Var (Var = 0 gives k_max), which is what the prose of the
 * same section describes.  k_fixed > 0 turns the controller off: k_t = k_fixed.
 * vbar is the moving average of the score variance, a frozen input here. */
typedef struct gsa_adaptive {
    float vbar;
    int32_t k_base, k_min, k_max;
    int32_t k_fixed;
    int32_t mode;
    int32_t dense_below; /* gsa_forward only: a context shorter than this many keys (Lk < dense_below) is attended
                            densely -- no indexer, no selection, every visible key (Sec. 8: below about 4K tokens the
                            indexer costs more than it saves).  0 = never.  See gsa_forward. */
} gsa_adaptive;

/* Launch-shape switches.  Every call that takes one accepts NULL (all fields 0 = the library decides).
 * They change how the work is cut up, never what is computed (results agree up to fp32 summation
 * order); a *_workspace_bytes helper and the call it sizes must be given the same values. */
typedef struct gsa_tuning {
    int32_t attn_window;         /* keys per key window of the sparse attention (see gsa_sparse_gated_attn):
                                    0 = chosen by the library, -1 = no windows, > 0 = this size, also on small calls */
    int32_t attn_kv_per_wg;      /* kv heads per attention workgroup: 0 = chosen by the library, else 1, 2 or 4 */
    int32_t select_exact_only;   /* 1 = gsa_topk_select never takes its sampled one-pass variant */
    int32_t forward_fp32_scores; /* 1 = gsa_forward keeps fp32 scores between indexer and selection, not 16-bit keys */
    int32_t attn_rows_per_wave;  /* query rows one wave of the bf16 attention streams through: 0 = chosen by the library, else 1..64 */
    int32_t select_wave_min_rows; /* selection on 16-bit keys: calls with at least this many rows (B * rows in range) run
                                    one wave per row (rows the estimate fails on fall back), smaller calls one workgroup
                                    per row: 0 = chosen by the library (2048), 1 = always a wave per row, -1 = never */
} gsa_tuning;

/* ---- stage 1: gated lightning indexer, Sec. 3.3, Eq. "indexer" ----------------------
 *   I[t,s] = sum_j w[t,j] * sigmoid(qI[t,j,:] . kI[s,:] + bI[j])   for every visible s,
 * with no 1/sqrt(dI) factor, plus the mean and the population variance of each
 * row's visible scores (the Var(I_t,:) that Sec. 3.4 consumes).
 * Rows [row_begin, row_end) of every batch element are computed.
 *   qI, kI   device, in   dtype elements
 *   w        device, in   fp32, the head weights sigma(h_t W^Iw_j), already in (0,1)
 *   bI       device, in   fp32 [HI], or NULL for zero bias
 *   scores   device, out  fp32, or NULL to compute only the statistics.  Element
 *            (b, t, s) is written at scores[(b*(row_end-row_begin) + (t-row_begin))*ld_scores + s];
 *            positions of invisible keys are left untouched.  ld_scores >= Lk, multiple of 4.
 *   row_mean device, out  fp32 [B, Lq] (only rows in range written), may be NULL
 *   row_var  device, out  fp32 [B, Lq] (only rows in range written)
 *   workspace device scratch of gsa_indexer_workspace_bytes(shape, row_begin, row_end) bytes.
 */
int32_t gsa_indexer_scores(const gsa_shape* shape, const void* qI, const void* kI, const float* w,
                           const float* bI, int32_t row_begin, int32_t row_end, float* scores,
                           int64_t ld_scores, float* row_mean, float* row_var, void* workspace,
                           size_t workspace_bytes, void* stream);
size_t gsa_indexer_workspace_bytes(const gsa_shape* shape, int32_t row_begin, int32_t row_end);

/* The same stage in the form the fused forward uses: instead of fp32 scores it writes the monotone
 * 16-bit fixed-point key  min(65535, floor(I[t,s] * 65536 / HIK))  of every visible score, HIK = HI rounded
 * up to a power of two (half the bytes to write and to read back); the statistics are those of the fp32
 * scores, bit for bit.  keys: device, out, uint16, indexed like `scores` above with ld_keys >= Lk, a
 * multiple of 8.  w must lie in [0,1] for the keys to resolve the scores (larger weights saturate keys). */
int32_t gsa_indexer_keys(const gsa_shape* shape, const void* qI, const void* kI, const float* w,
                         const float* bI, int32_t row_begin, int32_t row_end, uint16_t* keys,
                         int64_t ld_keys, float* row_mean, float* row_var, void* workspace,
                         size_t workspace_bytes, void* stream);

/* ---- stage 2: adaptive sparsity controller, Sec. 3.4 --------------------------------
 *   k[b,t]     = the budget of Eq. "adaptive_k" (always within [k_min, k_max], or k_fixed)
 *   n_sel[b,t] = min(k[b,t], number of visible keys of row t)
 *   row_var device, in, fp32 [B, Lq];  k_out (may be NULL), n_sel_out device, out, int32 [B, Lq].
 * The ratio is evaluated in double precision from the fp32 variance; floor comes
 * before the clamp.  Errors: GSA_ERR_VBAR, GSA_ERR_SHAPE (k_min < 1, k_min > k_max, k_base < 1). */
int32_t gsa_adaptive_k(const gsa_shape* shape, const gsa_adaptive* ctl, const float* row_var,
                       int32_t* k_out, int32_t* n_sel_out, void* stream);

/* ---- stage 3: top-k_t selection, Sec. 2.2 Eq. 4 (used with k_t in Sec. 3.2) ---------
 * For each row in [row_begin,row_end): the n_sel[b,t] visible keys with the largest score;
 * equal scores are taken lowest index first.  idx_out[b,t,0:n_sel] holds them in ascending
 * order, the rest of the k_cap entries is -1.  One set per query, shared by all heads.
 *   scores  device, in, fp32, laid out as written by gsa_indexer_scores for the same row range;
 *           must be >= 0 and finite (the paper's scores lie in (0, HI)); negative values
 *           are ranked as 0.
 *   n_sel   device, in, int32 [B, Lq]; values above min(k_cap, visible) are clamped.
 *   idx_out device, out, int32 [B, Lq, k_cap] (only rows in range written); 1 <= k_cap <= 8192.
 * No workspace.  Lk above GSA_SELECT_MAX_LK: GSA_ERR_UNSUPPORTED. */
int32_t gsa_topk_select(const gsa_shape* shape, int32_t row_begin, int32_t row_end, const float* scores,
                        int64_t ld_scores, const int32_t* n_sel, int32_t k_cap, int32_t* idx_out,
                        const gsa_tuning* tuning, void* stream);

/* The same stage on the 16-bit keys of gsa_indexer_keys (the form the fused forward uses).  Every element
 * whose key lies above the n_sel-th largest key is selected; the elements that share that key are the
 * only ones the keys do not order: their fp32 scores are recomputed from qI, kI, w, bI (Sec. 3.3,
 * Eq. "indexer") and ranked, equal scores lowest index first.  The result equals gsa_topk_select on the
 * fp32 scores except between scores that agree to within fp32 rounding (about 1e-7 relative). */
int32_t gsa_topk_select_keys(const gsa_shape* shape, int32_t row_begin, int32_t row_end, const uint16_t* keys,
                             int64_t ld_keys, const int32_t* n_sel, int32_t k_cap, int32_t* idx_out,
                             const void* qI, const void* kI, const float* w, const float* bI,
                             const gsa_tuning* tuning, void* stream);

/* ---- stage 4: sparse attention with value gate G2 and output gate G1, Sec. 3.5-3.6 --
 * For query head h (kv head g = h / (H/H_kv)) over S_t = idx[b,t,0:n_sel[b,t]]:
 *   A[s]  = softmax_{s in S_t}(softmax_scale * Q[t,h,:] . K[s,g,:])
 *   O     = sum_s A[s] * (V[s,g,:] * sigmoid(g2[s,g,:]))          (G2, before aggregation)
 *   out[t,h,:] = O * sigmoid(g1[t,h,:])                            (G1, after SDPA)
 * Rows [row_begin,row_end) are computed.  g2 == NULL: V is taken as already gated.
 * g1 == NULL: no output gate.  softmax_scale == 0 selects 1/sqrt(d_h).  A row with
 * n_sel == 0 produces zeros.  Indices are clamped into [0, Lk-1] before use.
 * bf16: products on the matrix cores with fp32 accumulation, probabilities and gated
 * values rounded to bf16 before the PV product, result rounded to bf16.  f32: fp32 throughout.
 * The rows of one call may be worked through in pieces: pieces of each selected list whose partial
 * softmax states are merged at the end when B*(row_end-row_begin) is small (decode), or, for bf16
 * calls with at least 8192 rows and a context of at least two windows, one launch per window of keys
 * that continues each row's running softmax state, so that the rows being gathered stay in the
 * on-die caches.  Same result up to fp32 summation order.
 *   workspace: gsa_attn_workspace_bytes(...) bytes (0 when neither applies). */
int32_t gsa_sparse_gated_attn(const gsa_shape* shape, int32_t row_begin, int32_t row_end, const void* Q,
                              const void* K, const void* V, const void* g2_logits, const void* g1_logits,
                              const int32_t* idx, const int32_t* n_sel, int32_t k_cap, float softmax_scale,
                              void* out, void* workspace, size_t workspace_bytes, const gsa_tuning* tuning,
                              void* stream);
size_t gsa_attn_workspace_bytes(const gsa_shape* shape, int32_t row_begin, int32_t row_end, int32_t k_cap,
                                const gsa_tuning* tuning);

/* ---- the value gate as a dense pre-pass, Sec. 3.5 / stage (2) of Sec. 4 -------------
 * Vg = V * sigmoid(g2), element-wise over [B, Lk, H_kv, d_h], rounded to dtype.  Vg may alias V. */
int32_t gsa_value_gate(const gsa_shape* shape, const void* V, const void* g2_logits, void* Vg, void* stream);

/* ---- fused forward: stages 1-4 in the order of Sec. 3.2 / Sec. 4 --------------------
 * G2 -> indexer -> controller -> top-k_t -> sparse SDPA -> G1, processed in slabs of query
 * rows so that the score matrix need not exist as a whole.  When g2 != NULL the value gate
 * runs as a dense pre-pass into the workspace if the queries together gather at least four
 * times more rows than there are key tokens (Lq * min(k_cap, Lk) >= 4 * Lk, prefill);
 * otherwise (decode) it is applied in registers to the gathered rows.  Both give the same
 * bits: V * sigmoid(g2) rounded to dtype.
 * Between the indexer and the selection the fused call keeps 16-bit fixed-point keys
 * min(65535, floor(I * 65536 / HI)) instead of fp32 scores (w must lie in [0,1] for the keys to
 * resolve the scores; larger weights only cost speed).  Elements that share the threshold key are
 * re-scored in fp32, so the selected sets equal those of gsa_indexer_scores + gsa_topk_select
 * except between scores that agree to within fp32 rounding (about 1e-7 relative).
 * The query rows are worked through in slabs; the call fits as many rows into each slab as the
 * workspace allows (early rows see few keys, so early slabs hold more rows).
 *   out          device, out [B, Lq, H, d_h]
 *   idx_out      device, out [B, Lq, k_cap] or NULL (then kept per slab in the workspace)
 *   n_sel_out, k_out   device, out [B, Lq] or NULL
 *   row_var_out  device, out [B, Lq] or NULL
 *   k_cap        >= k_max (or >= k_fixed), <= 8192
 *   workspace    at least gsa_forward_workspace_bytes(shape, k_cap, g2 != NULL, 0, tuning) bytes;
 *                a larger workspace lets the call use larger slabs (fewer launches).
 * gsa_forward_workspace_bytes(.., slab_rows, ..): bytes that let every slab hold at least that many
 * query rows (rounded up to a multiple of 128); slab_rows = 0 gives the minimum.
 * Lk above GSA_SELECT_MAX_LK: GSA_ERR_UNSUPPORTED.
 * Dense fallback (ctl->dense_below > Lk, bf16 only): the call is gsa_dense_gated_attn over all rows; it
 * produces `out` alone, so idx_out, n_sel_out, k_out and row_var_out must be NULL (GSA_ERR_SHAPE otherwise),
 * and the workspace must hold gsa_dense_attn_workspace_bytes(shape, g2 != NULL) bytes. */
int32_t gsa_forward(const gsa_shape* shape, const gsa_adaptive* ctl, const void* Q, const void* K,
                    const void* V, const void* g1_logits, const void* g2_logits, const void* qI,
                    const void* kI, const float* w, const float* bI, float softmax_scale, void* out,
                    int32_t* idx_out, int32_t* n_sel_out, int32_t* k_out, float* row_var_out,
                    int32_t k_cap, void* workspace, size_t workspace_bytes, const gsa_tuning* tuning,
                    void* stream);
size_t gsa_forward_workspace_bytes(const gsa_shape* shape, int32_t k_cap, int32_t has_g2, int32_t slab_rows,
                                   const gsa_tuning* tuning);

/* ---- decode-serving state (the "Decode" column of Table 9) -----------------------------------------
 * Per-sequence append-only caches with a capacity of Lk tokens each:
 *   kI_cache [B, Lk, dI]   K_cache, Vg_cache [B, Lk, H_kv, d_h]   seq_lens [B] int32 (device)
 * Vg_cache holds the gated values V * sigmoid(g2) (Sec. 3.5), rounded to dtype exactly as gsa_value_gate
 * does, so a decode step gathers two rows per selected key and never reads the gate logits of old tokens.
 * The sequences of a batch may have different lengths (ragged): seq_lens[b] tokens of sequence b are valid.
 *
 * gsa_cache_append: shape->Lq = T new tokens per sequence.  Token j of sequence b is written at position
 * seq_lens[b] + j (dropped if that is beyond the capacity); seq_lens_out[b] = min(seq_lens[b] + T, Lk)
 * (may be NULL; must not alias seq_lens).  kI_new [B,T,dI]; K_new, V_new, g2_new [B,T,H_kv,d_h].
 *
 * gsa_decode_step: gsa_forward for the last Lq tokens of every sequence against its own context: query row
 * i of sequence b has position seq_lens[b] - Lq + i (seq_lens counts the new tokens, which must already be in
 * the caches) and sees keys 0 .. that position; keys at or beyond seq_lens[b] are never read.  Values outside
 * [Lq, Lk] are clamped.  Everything else (controller, selection, outputs, k_cap, tuning) as in gsa_forward;
 * key windows and the dense fallback do not apply.  workspace: gsa_decode_workspace_bytes(shape, k_cap, tuning). */
int32_t gsa_cache_append(const gsa_shape* shape, const void* kI_new, const void* K_new, const void* V_new,
                         const void* g2_new, const int32_t* seq_lens, void* kI_cache, void* K_cache,
                         void* Vg_cache, int32_t* seq_lens_out, void* stream);
int32_t gsa_decode_step(const gsa_shape* shape, const gsa_adaptive* ctl, const void* Q, const void* g1_logits,
                        const void* qI, const float* w, const float* bI, const void* kI_cache,
                        const void* K_cache, const void* Vg_cache, const int32_t* seq_lens, float softmax_scale,
                        void* out, int32_t* idx_out, int32_t* n_sel_out, int32_t* k_out, float* row_var_out,
                        int32_t k_cap, void* workspace, size_t workspace_bytes, const gsa_tuning* tuning,
                        void* stream);
size_t gsa_decode_workspace_bytes(const gsa_shape* shape, int32_t k_cap, const gsa_tuning* tuning);

/* The same two calls on paged (block-table) caches, as serving engines keep them: the tokens of a sequence sit in
 * pages of page_size tokens scattered over pools shared by all sequences,
 *   kI_pool [pool_pages, page_size, dI]   K_pool, Vg_pool [pool_pages, page_size, H_kv, d_h]
 *   block_table [B, Lk / page_size] int32 (device): block_table[b][p] = pool page holding tokens p*page_size .. of
 *   sequence b.  Only the entries up to a sequence's last token are read; page numbers are clamped to the pool.
 * shape->Lk is the capacity of one sequence (a multiple of page_size); page_size is a power of two >= 128 (an
 * indexer key tile never straddles two pages); pool_pages * page_size < 2^31; one pool may exceed 4 GiB.
 * Everything else as in gsa_cache_append / gsa_decode_step (same results bit for bit for the same cached rows);
 * idx_out holds token positions inside the sequence, not pool rows.
 * Errors: GSA_ERR_SHAPE for a bad page_size / capacity / pool size, GSA_ERR_NULL for a missing table. */
int32_t gsa_paged_cache_append(const gsa_shape* shape, int32_t page_size, const int32_t* block_table, int32_t pool_pages,
                               const void* kI_new, const void* K_new, const void* V_new, const void* g2_new,
                               const int32_t* seq_lens, void* kI_pool, void* K_pool, void* Vg_pool,
                               int32_t* seq_lens_out, void* stream);
int32_t gsa_paged_decode_step(const gsa_shape* shape, const gsa_adaptive* ctl, int32_t page_size,
                              const int32_t* block_table, int32_t pool_pages, const void* Q, const void* g1_logits,
                              const void* qI, const float* w, const float* bI, const void* kI_pool,
                              const void* K_pool, const void* Vg_pool, const int32_t* seq_lens, float softmax_scale,
                              void* out, int32_t* idx_out, int32_t* n_sel_out, int32_t* k_out, float* row_var_out,
                              int32_t k_cap, void* workspace, size_t workspace_bytes, const gsa_tuning* tuning,
                              void* stream);
size_t gsa_paged_decode_workspace_bytes(const gsa_shape* shape, int32_t k_cap, const gsa_tuning* tuning);

/* ---- the linear projections around the path (Sec. 2.1 Eq. 1, Sec. 3.3, Sec. 3.5, App. B) ------------
 * Every projection is y = x W^T with W stored row-major [out_features, in_features], bf16 in, fp32
 * accumulation, bf16 out (GSA_BF16 shapes only; GSA_ERR_UNSUPPORTED otherwise).  All pointers are device
 * pointers owned by the caller; weights and inputs 16-byte aligned.
 *
 * gsa_input_projections: one fused GEMM over the hidden states h [B, Lq, d_model] (d_model a multiple of
 * 64) that writes, for the B*Lq tokens of h, every input of the path in the layouts gsa_forward reads:
 *   Q = h W_Q^T          [B, Lq, H, d_h]        W_Q  [H*d_h, d_model]       (Sec. 2.1 Eq. 1)
 *   K, V                 [B, Lq, H_kv, d_h]     W_K, W_V [H_kv*d_h, d_model]
 *   g1_logits = h W_g1^T [B, Lq, H, d_h]        W_g1 [H*d_h, d_model]       (output gate G1, Sec. 3.5)
 *   g2_logits = h W_g2^T [B, Lq, H_kv, d_h]     W_g2 [H_kv*d_h, d_model]    (value gate G2, Sec. 3.5)
 *   qI = h W_qI^T        [B, Lq, HI, dI]        W_qI [HI*dI, d_model]       (Sec. 3.3)
 *   kI = h W_kI^T        [B, Lq, dI]            W_kI [dI, d_model]
 *   w  = sigmoid(h W_Iw^T) [B, Lq, HI] fp32     W_Iw [HI, d_model]          (indexer head weights, Sec. 3.3)
 * A projection is skipped when both its weight and its destination are NULL (one of the two alone:
 * GSA_ERR_NULL).  In a prefill Lq = Lk and K, V, g2_logits, kI are the whole context; in a decode step they
 * are the rows gsa_cache_append takes.
 *
 * gsa_output_projection: y = attn_out W_O^T with attn_out [B, Lq, H*d_h] (the gated heads, concatenated;
 * H*d_h a multiple of 64), W_O [d_model, H*d_h], y [B, Lq, d_model] (App. B). */
int32_t gsa_input_projections(const gsa_shape* shape, int32_t d_model, const void* h, const void* W_Q,
                              const void* W_K, const void* W_V, const void* W_g1, const void* W_g2,
                              const void* W_qI, const void* W_kI, const void* W_Iw, void* Q, void* K, void* V,
                              void* g1_logits, void* g2_logits, void* qI, void* kI, float* w, void* stream);
int32_t gsa_output_projection(const gsa_shape* shape, int32_t d_model, const void* attn_out, const void* W_O,
                              void* y, void* stream);

/* ---- training side, Sec. 6.1 ------------------------------------------------------------------------
 * gsa_sparse_gated_attn_bwd: gradients of stage 4 (Sec. 3.5, 3.6) for the upstream gradient dout
 * [B, Lq, H, d_h] (dtype elements) of its output, with the selection idx / n_sel held fixed (top-k has no
 * gradient) and Lq = the rows idx covers (row range = all rows).  With s_j = scale * q.k_j, P = softmax(s),
 * V'_j = V_j * sigmoid(g2_j), O = sum_j P_j V'_j, out = O * sigmoid(g1):
 *   dO = dout * sigmoid(g1)         dg1 = dout * O * sigmoid(g1) (1 - sigmoid(g1))
 *   ds_j = P_j (dO.V'_j - dO.O)     dq = scale * sum_j ds_j k_j     dk_j += scale * ds_j q     dV'_j += P_j dO
 *   dV = dV' * sigmoid(g2)          dg2 = dV' * V * sigmoid(g2) (1 - sigmoid(g2))
 * All gradients are fp32: dQ, dg1 [B, Lq, H, d_h]; dK, dV, dg2 [B, Lk, H_kv, d_h] (written entirely: rows no
 * query selected are zero).  g1_logits and dg1 are given together or both NULL, likewise g2_logits and dg2.
 *   workspace  device, scratch, 256-byte aligned, gsa_attn_bwd_workspace_bytes(shape, k_cap) bytes, or NULL.
 *           Given: dK and dV' are summed key by key in a second pass over inverted lists (for every key, the
 *           queries that selected it, grouped by windows of queries), without atomics on the gradients; only
 *           the order of a key's list, and with it the last bits of its sums, varies between runs.  For
 *           GSA_BF16 shapes the first pass runs on the matrix cores and, like the forward, rounds the
 *           operands of its products (P, dO, dS) to bf16: gradients within about 1e-2 of their largest
 *           entry; GSA_F32 shapes stay in fp32 arithmetic.  Needs B * Lq * k_cap < 2^31
 *           (GSA_ERR_UNSUPPORTED otherwise); too small: GSA_ERR_WORKSPACE.
 *           NULL: one pass, every (query, key) contribution added with fp32 atomics (several times slower).
 *   p_mean  device, out, fp32 [B, Lq, k_cap] or NULL: the attention weights of every row over its selected keys,
 *           averaged over the H heads -- the target p_{t,S_t} of the sparse-phase indexer loss.
 *
 * gsa_indexer_sparse_kl: the sparse-phase indexer loss of Sec. 6.1, per query row,
 *   loss_rows[b,t] = KL(p_{t,S_t} || softmax_{s in S_t} I_{t,s}),   p taken as a constant (the frozen target),
 * and the gradients it sends into the indexer of Sec. 3.3 (dI_s = softmax(I)_s - p_s):
 *   dqI [B, Lq, HI, dI]   dkI [B, Lk, dI] (atomics)   dw [B, Lq, HI] (w.r.t. the post-sigmoid head weights)
 *   dbI [HI] (atomics; given together with bI or both NULL), all fp32.  Sigmoid indexer only. */
int32_t gsa_sparse_gated_attn_bwd(const gsa_shape* shape, const void* Q, const void* K, const void* V,
                                  const void* g2_logits, const void* g1_logits, const int32_t* idx,
                                  const int32_t* n_sel, int32_t k_cap, float softmax_scale, const void* dout,
                                  float* dQ, float* dK, float* dV, float* dg1, float* dg2, float* p_mean,
                                  void* workspace, size_t workspace_bytes, void* stream);
size_t gsa_attn_bwd_workspace_bytes(const gsa_shape* shape, int32_t k_cap); /* 0 for a bad shape */
int32_t gsa_indexer_sparse_kl(const gsa_shape* shape, const void* qI, const void* kI, const float* w,
                              const float* bI, const int32_t* idx, const int32_t* n_sel, int32_t k_cap,
                              const float* p, float* loss_rows, float* dqI, float* dkI, float* dw, float* dbI,
                              void* stream);

/* ---- comparison variants: dense causal attention, Sec. 2.1 Eq. 2 ------------------------------------
 * Every visible key, no indexer and no selection: with g2 and g1 given this is the "gated only" variant of
 * Sec. 7.1 (Eq. 2 with V' = V * sigmoid(g2) and the result multiplied by sigmoid(g1)), with both NULL the
 * "standard" attention the paper's ratios are quoted against, and in either case what the sparse path
 * equals when the budget covers every visible key.  bf16 only (GSA_ERR_UNSUPPORTED otherwise).
 * Rows [row_begin,row_end).  workspace: gsa_dense_attn_workspace_bytes(shape, g2 != NULL) bytes (the gated
 * values; 0 when g2 == NULL). */
int32_t gsa_dense_gated_attn(const gsa_shape* shape, int32_t row_begin, int32_t row_end, const void* Q,
                             const void* K, const void* V, const void* g2_logits, const void* g1_logits,
                             float softmax_scale, void* out, void* workspace, size_t workspace_bytes, void* stream);
size_t gsa_dense_attn_workspace_bytes(const gsa_shape* shape, int32_t has_g2);

/* ---- gsa_forward for callers that cannot allocate ---------------------------------------------------
 * For code under HIP graph capture, tight serving loops and harnesses that forbid hipMalloc: the same
 * computation as gsa_forward with the workspace taken from an array of GSA_STATIC_SCRATCH_BYTES bytes that
 * is part of the library's device code (every GPU the library is loaded on holds its own copy until the
 * process ends).  The call allocates and frees nothing, on the device or through any library.  Problems
 * whose minimum workspace, gsa_forward_workspace_bytes(shape, k_cap, g2 != NULL, 0, tuning), exceeds the
 * array are refused with GSA_ERR_WORKSPACE before anything is launched (gsa_last_error() names both
 * sizes): decode steps and short prefills fit, a 128K-token prefill does not.  All calls on one GPU share
 * that GPU's array: calls that overlap in time on one GPU (different streams or threads) race; calls on
 * one stream are ordered and safe.  Nothing in the array has to be cleared between calls. */
#define GSA_STATIC_SCRATCH_BYTES (64u << 20)
int32_t gsa_forward_noalloc(const gsa_shape* shape, const gsa_adaptive* ctl, const void* Q, const void* K,
                            const void* V, const void* g1_logits, const void* g2_logits, const void* qI,
                            const void* kI, const float* w, const float* bI, float softmax_scale, void* out,
                            int32_t* idx_out, int32_t* n_sel_out, int32_t* k_out, float* row_var_out,
                            int32_t k_cap, const gsa_tuning* tuning, void* stream);

/* ---- measurement helper (no part of the method) ---------------------------------------
 * Gathers whole rows of a table in the access shape of the sparse attention (16 lanes x 16 bytes per
 * 256-byte row, four rows per load instruction, sixteen loads in flight per wave): wave v of `waves`
 * reads the rows idx[c*64 .. c*64+64) of every chunk c = v, v + waves, ..., XORs what it reads and
 * stores one word per wave in sink[v].  The benchmark times it on cache-resident and on HBM-resident
 * tables to measure the gather ceilings that the attention's achieved rate is compared with.
 *   table device, in, table_rows rows of 256 bytes;  idx device, in, int32 [n_idx], values in
 *   [0, table_rows), n_idx a multiple of 64;  sink device, out, uint32 [waves];  waves a multiple of 4. */
int32_t gsa_probe_gather(const void* table, int64_t table_rows, const int32_t* idx, int64_t n_idx, int32_t waves,
                         uint32_t* sink, void* stream);
/* The same gather with every row staged through LDS (registers -> a wave-private 16 KB tile -> registers, the
 * least an MFMA operand built from gathered rows needs; 64 KB of LDS per 256-thread workgroup, so eight waves
 * per CU).  Same arguments and sink values as gsa_probe_gather.  The register return of the loads and the LDS
 * writes and reads share a CU's data path: this rate is the ceiling for the attention kernel's dataflow. */
int32_t gsa_probe_gather_staged(const void* table, int64_t table_rows, const int32_t* idx, int64_t n_idx, int32_t waves,
                                uint32_t* sink, void* stream);

/* ---- misc ---------------------------------------------------------------------------- */
const char* gsa_status_string(int32_t status); /* static string */
const char* gsa_last_error(void);              /* text of the calling thread's last HIP error, "" if none */
int32_t gsa_version(void);                     /* major*10000 + minor*100 + patch */

#ifdef __cplusplus
}
#endif
#endif /* GSA_H */
