"""libgsa: forward path of Gated Sparse Attention on MI355X.

Thin ctypes binding over the C ABI declared in include/gsa.h.  The functions
have the same names as the C entry points and only marshal arguments: torch
tensors supply device memory and the current stream, every step of the path
runs in the HIP kernels of libgsa.so.  There is no fallback: if the library
has not been built, loading it raises.
"""
import ctypes
import os

import torch

from . import synthetic  # noqa: F401  (input generators, no arithmetic of the method)

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libgsa.so")

GSA_F32, GSA_BF16 = 0, 1
GSA_ACT_SIGMOID, GSA_ACT_RELU = 0, 1
GSA_OK = 0
GSA_ERR_NULL, GSA_ERR_SHAPE, GSA_ERR_UNSUPPORTED, GSA_ERR_VBAR, GSA_ERR_WORKSPACE, GSA_ERR_HIP = -1, -2, -3, -4, -5, -6

ENTRY_POINTS = (
    "gsa_indexer_scores", "gsa_indexer_keys", "gsa_indexer_workspace_bytes", "gsa_adaptive_k", "gsa_topk_select",
    "gsa_topk_select_keys", "gsa_sparse_gated_attn", "gsa_attn_workspace_bytes", "gsa_value_gate", "gsa_forward",
    "gsa_forward_workspace_bytes", "gsa_forward_noalloc", "gsa_dense_gated_attn", "gsa_dense_attn_workspace_bytes",
    "gsa_cache_append", "gsa_decode_step", "gsa_decode_workspace_bytes", "gsa_paged_cache_append", "gsa_paged_decode_step",
    "gsa_paged_decode_workspace_bytes", "gsa_input_projections", "gsa_output_projection", "gsa_sparse_gated_attn_bwd",
    "gsa_attn_bwd_workspace_bytes",
    "gsa_indexer_sparse_kl",
    "gsa_probe_gather", "gsa_probe_gather_staged", "gsa_status_string", "gsa_last_error", "gsa_version",
)


class GsaShape(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("B", "Lq", "Lk", "q_offset", "H", "H_kv", "d_h", "HI", "dI", "dtype", "indexer_act")]


class GsaAdaptive(ctypes.Structure):
    _fields_ = [("vbar", ctypes.c_float)] + [(n, ctypes.c_int32) for n in ("k_base", "k_min", "k_max", "k_fixed", "mode", "dense_below")]


class GsaTuning(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("attn_window", "attn_kv_per_wg", "select_exact_only", "forward_fp32_scores",
                                                  "attn_rows_per_wave", "select_wave_min_rows")]


class GsaError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        lib = load()
        msg = lib.gsa_status_string(status).decode()
        extra = lib.gsa_last_error().decode() if status == GSA_ERR_HIP else ""
        super().__init__("%s: %s (%d) %s" % (where, msg, status, extra))


_lib = None


def load():
    """Load libgsa.so (built in-tree by paper_2601_15305_amd.build).  Raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("libgsa.so is not built: run `python -m paper_2601_15305_amd.build` (no fallback path exists)")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, i64, sz, f32 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t, ctypes.c_float
    shp, ctl, tun = ctypes.POINTER(GsaShape), ctypes.POINTER(GsaAdaptive), ctypes.POINTER(GsaTuning)
    lib.gsa_indexer_scores.argtypes = [shp, vp, vp, vp, vp, i32, i32, vp, i64, vp, vp, vp, sz, vp]
    lib.gsa_indexer_scores.restype = i32
    lib.gsa_indexer_keys.argtypes = [shp, vp, vp, vp, vp, i32, i32, vp, i64, vp, vp, vp, sz, vp]
    lib.gsa_indexer_keys.restype = i32
    lib.gsa_topk_select_keys.argtypes = [shp, i32, i32, vp, i64, vp, i32, vp, vp, vp, vp, vp, tun, vp]
    lib.gsa_topk_select_keys.restype = i32
    lib.gsa_probe_gather.argtypes = [vp, i64, vp, i64, i32, vp, vp]
    lib.gsa_probe_gather.restype = i32
    lib.gsa_probe_gather_staged.argtypes = [vp, i64, vp, i64, i32, vp, vp]
    lib.gsa_probe_gather_staged.restype = i32
    lib.gsa_indexer_workspace_bytes.argtypes = [shp, i32, i32]
    lib.gsa_indexer_workspace_bytes.restype = sz
    lib.gsa_adaptive_k.argtypes = [shp, ctl, vp, vp, vp, vp]
    lib.gsa_adaptive_k.restype = i32
    lib.gsa_topk_select.argtypes = [shp, i32, i32, vp, i64, vp, i32, vp, tun, vp]
    lib.gsa_topk_select.restype = i32
    lib.gsa_sparse_gated_attn.argtypes = [shp, i32, i32, vp, vp, vp, vp, vp, vp, vp, i32, f32, vp, vp, sz, tun, vp]
    lib.gsa_sparse_gated_attn.restype = i32
    lib.gsa_attn_workspace_bytes.argtypes = [shp, i32, i32, i32, tun]
    lib.gsa_attn_workspace_bytes.restype = sz
    lib.gsa_value_gate.argtypes = [shp, vp, vp, vp, vp]
    lib.gsa_value_gate.restype = i32
    lib.gsa_forward.argtypes = [shp, ctl, vp, vp, vp, vp, vp, vp, vp, vp, vp, f32, vp, vp, vp, vp, vp, i32, vp, sz, tun, vp]
    lib.gsa_forward.restype = i32
    lib.gsa_forward_noalloc.argtypes = [shp, ctl, vp, vp, vp, vp, vp, vp, vp, vp, vp, f32, vp, vp, vp, vp, vp, i32, tun, vp]
    lib.gsa_forward_noalloc.restype = i32
    lib.gsa_cache_append.argtypes = [shp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.gsa_cache_append.restype = i32
    lib.gsa_input_projections.argtypes = [shp, i32] + [vp] * 18
    lib.gsa_input_projections.restype = i32
    lib.gsa_output_projection.argtypes = [shp, i32, vp, vp, vp, vp]
    lib.gsa_output_projection.restype = i32
    lib.gsa_decode_step.argtypes = [shp, ctl, vp, vp, vp, vp, vp, vp, vp, vp, vp, f32, vp, vp, vp, vp, vp, i32, vp, sz, tun, vp]
    lib.gsa_decode_step.restype = i32
    lib.gsa_decode_workspace_bytes.argtypes = [shp, i32, tun]
    lib.gsa_decode_workspace_bytes.restype = sz
    lib.gsa_sparse_gated_attn_bwd.argtypes = [shp, vp, vp, vp, vp, vp, vp, vp, i32, f32] + [vp] * 8 + [sz, vp]
    lib.gsa_sparse_gated_attn_bwd.restype = i32
    lib.gsa_attn_bwd_workspace_bytes.argtypes = [shp, i32]
    lib.gsa_attn_bwd_workspace_bytes.restype = sz
    lib.gsa_indexer_sparse_kl.argtypes = [shp, vp, vp, vp, vp, vp, vp, i32] + [vp] * 7
    lib.gsa_indexer_sparse_kl.restype = i32
    lib.gsa_paged_cache_append.argtypes = [shp, i32, vp, i32] + [vp] * 10
    lib.gsa_paged_cache_append.restype = i32
    lib.gsa_paged_decode_step.argtypes = [shp, ctl, i32, vp, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, f32, vp, vp, vp, vp, vp, i32, vp, sz,
                                          tun, vp]
    lib.gsa_paged_decode_step.restype = i32
    lib.gsa_paged_decode_workspace_bytes.argtypes = [shp, i32, tun]
    lib.gsa_paged_decode_workspace_bytes.restype = sz
    lib.gsa_dense_gated_attn.argtypes = [shp, i32, i32, vp, vp, vp, vp, vp, f32, vp, vp, sz, vp]
    lib.gsa_dense_gated_attn.restype = i32
    lib.gsa_dense_attn_workspace_bytes.argtypes = [shp, i32]
    lib.gsa_dense_attn_workspace_bytes.restype = sz
    lib.gsa_forward_workspace_bytes.argtypes = [shp, i32, i32, i32, tun]
    lib.gsa_forward_workspace_bytes.restype = sz
    lib.gsa_status_string.argtypes = [i32]
    lib.gsa_status_string.restype = ctypes.c_char_p
    lib.gsa_last_error.argtypes = []
    lib.gsa_last_error.restype = ctypes.c_char_p
    lib.gsa_version.argtypes = []
    lib.gsa_version.restype = i32
    _lib = lib
    return lib


# ------------------------------------------------------------------------------- marshalling
def _ptr(t):
    if t is None:
        return None
    if isinstance(t, int):
        return t
    assert t.is_contiguous(), "libgsa takes dense row-major tensors"
    return t.data_ptr()


def _stream(stream):
    if stream is not None:
        return stream
    if torch.cuda.is_available():
        return torch.cuda.current_stream().cuda_stream
    return None


def make_shape(B, Lq, Lk, q_offset, H, H_kv, d_h, HI, dI, dtype, indexer_act="sigmoid"):
    code = {"f32": GSA_F32, "bf16": GSA_BF16, torch.float32: GSA_F32, torch.bfloat16: GSA_BF16}.get(dtype, dtype)
    act = {"sigmoid": GSA_ACT_SIGMOID, "relu": GSA_ACT_RELU}.get(indexer_act, indexer_act)
    return GsaShape(B, Lq, Lk, q_offset, H, H_kv, d_h, HI, dI, code, act)


def shape_of(wl):
    """gsa_shape of a synthetic.Workload."""
    return make_shape(wl.B, wl.Lq, wl.Lk, wl.q_offset, wl.H, wl.H_kv, wl.d_h, wl.HI, wl.dI, wl.dtype, wl.indexer_act)


def make_adaptive(vbar, k_base, k_min, k_max, k_fixed=0, mode=0, dense_below=0):
    return GsaAdaptive(float(vbar), k_base, k_min, k_max, k_fixed, mode, dense_below)


def make_tuning(attn_window=0, attn_kv_per_wg=0, select_exact_only=0, forward_fp32_scores=0, attn_rows_per_wave=0,
                select_wave_min_rows=0):
    """gsa_tuning: launch-shape switches (0 = the library decides).  Pass None for all defaults."""
    return GsaTuning(attn_window, attn_kv_per_wg, select_exact_only, forward_fp32_scores, attn_rows_per_wave,
                     select_wave_min_rows)


def _tun(tuning):
    return ctypes.byref(tuning) if tuning is not None else None


def _check(rc, where):
    if rc != GSA_OK:
        raise GsaError(rc, where)


# ------------------------------------------------------------------------------- entry points
def gsa_version():
    return load().gsa_version()


def gsa_indexer_workspace_bytes(shape, row_begin, row_end):
    return load().gsa_indexer_workspace_bytes(ctypes.byref(shape), row_begin, row_end)


def gsa_indexer_scores(shape, qI, kI, w, bI, row_begin, row_end, scores, ld_scores, row_mean, row_var, workspace,
                       workspace_bytes=None, stream=None):
    if workspace_bytes is None:
        workspace_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    rc = load().gsa_indexer_scores(ctypes.byref(shape), _ptr(qI), _ptr(kI), _ptr(w), _ptr(bI), row_begin, row_end,
                                   _ptr(scores), ld_scores, _ptr(row_mean), _ptr(row_var), _ptr(workspace),
                                   workspace_bytes, _stream(stream))
    _check(rc, "gsa_indexer_scores")


def gsa_indexer_keys(shape, qI, kI, w, bI, row_begin, row_end, keys, ld_keys, row_mean, row_var, workspace,
                     workspace_bytes=None, stream=None):
    if workspace_bytes is None:
        workspace_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    rc = load().gsa_indexer_keys(ctypes.byref(shape), _ptr(qI), _ptr(kI), _ptr(w), _ptr(bI), row_begin, row_end, _ptr(keys),
                                 ld_keys, _ptr(row_mean), _ptr(row_var), _ptr(workspace), workspace_bytes, _stream(stream))
    _check(rc, "gsa_indexer_keys")


def gsa_topk_select_keys(shape, row_begin, row_end, keys, ld_keys, n_sel, k_cap, idx_out, qI, kI, w, bI, tuning=None, stream=None):
    rc = load().gsa_topk_select_keys(ctypes.byref(shape), row_begin, row_end, _ptr(keys), ld_keys, _ptr(n_sel), k_cap,
                                     _ptr(idx_out), _ptr(qI), _ptr(kI), _ptr(w), _ptr(bI), _tun(tuning), _stream(stream))
    _check(rc, "gsa_topk_select_keys")


def gsa_probe_gather(table, table_rows, idx, n_idx, waves, sink, stream=None):
    rc = load().gsa_probe_gather(_ptr(table), table_rows, _ptr(idx), n_idx, waves, _ptr(sink), _stream(stream))
    _check(rc, "gsa_probe_gather")


def gsa_probe_gather_staged(table, table_rows, idx, n_idx, waves, sink, stream=None):
    rc = load().gsa_probe_gather_staged(_ptr(table), table_rows, _ptr(idx), n_idx, waves, _ptr(sink), _stream(stream))
    _check(rc, "gsa_probe_gather_staged")


def gsa_adaptive_k(shape, ctl, row_var, k_out, n_sel_out, stream=None):
    rc = load().gsa_adaptive_k(ctypes.byref(shape), ctypes.byref(ctl) if ctl is not None else None, _ptr(row_var),
                               _ptr(k_out), _ptr(n_sel_out), _stream(stream))
    _check(rc, "gsa_adaptive_k")


def gsa_topk_select(shape, row_begin, row_end, scores, ld_scores, n_sel, k_cap, idx_out, tuning=None, stream=None):
    rc = load().gsa_topk_select(ctypes.byref(shape), row_begin, row_end, _ptr(scores), ld_scores, _ptr(n_sel), k_cap,
                                _ptr(idx_out), _tun(tuning), _stream(stream))
    _check(rc, "gsa_topk_select")


def gsa_attn_workspace_bytes(shape, row_begin, row_end, k_cap, tuning=None):
    return load().gsa_attn_workspace_bytes(ctypes.byref(shape), row_begin, row_end, k_cap, _tun(tuning))


def gsa_sparse_gated_attn(shape, row_begin, row_end, Q, K, V, g2_logits, g1_logits, idx, n_sel, k_cap, softmax_scale,
                          out, workspace=None, workspace_bytes=None, tuning=None, stream=None):
    if workspace_bytes is None:
        workspace_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    rc = load().gsa_sparse_gated_attn(ctypes.byref(shape), row_begin, row_end, _ptr(Q), _ptr(K), _ptr(V),
                                      _ptr(g2_logits), _ptr(g1_logits), _ptr(idx), _ptr(n_sel), k_cap,
                                      float(softmax_scale), _ptr(out), _ptr(workspace), workspace_bytes, _tun(tuning),
                                      _stream(stream))
    _check(rc, "gsa_sparse_gated_attn")


def gsa_value_gate(shape, V, g2_logits, Vg, stream=None):
    rc = load().gsa_value_gate(ctypes.byref(shape), _ptr(V), _ptr(g2_logits), _ptr(Vg), _stream(stream))
    _check(rc, "gsa_value_gate")


def gsa_forward_workspace_bytes(shape, k_cap, has_g2, slab_rows=0, tuning=None):
    return load().gsa_forward_workspace_bytes(ctypes.byref(shape), k_cap, int(bool(has_g2)), slab_rows, _tun(tuning))


def gsa_forward(shape, ctl, Q, K, V, g1_logits, g2_logits, qI, kI, w, bI, softmax_scale, out, idx_out, n_sel_out, k_out,
                row_var_out, k_cap, workspace, workspace_bytes=None, tuning=None, stream=None):
    if workspace_bytes is None:
        workspace_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    rc = load().gsa_forward(ctypes.byref(shape) if shape is not None else None,
                            ctypes.byref(ctl) if ctl is not None else None, _ptr(Q), _ptr(K), _ptr(V),
                            _ptr(g1_logits), _ptr(g2_logits), _ptr(qI), _ptr(kI), _ptr(w), _ptr(bI), float(softmax_scale),
                            _ptr(out), _ptr(idx_out), _ptr(n_sel_out), _ptr(k_out), _ptr(row_var_out), k_cap,
                            _ptr(workspace), workspace_bytes, _tun(tuning), _stream(stream))
    _check(rc, "gsa_forward")


STATIC_SCRATCH_BYTES = 64 << 20


def gsa_forward_noalloc(shape, ctl, Q, K, V, g1_logits, g2_logits, qI, kI, w, bI, softmax_scale, out, idx_out, n_sel_out,
                        k_out, row_var_out, k_cap, tuning=None, stream=None):
    rc = load().gsa_forward_noalloc(ctypes.byref(shape) if shape is not None else None,
                                    ctypes.byref(ctl) if ctl is not None else None, _ptr(Q), _ptr(K), _ptr(V),
                                    _ptr(g1_logits), _ptr(g2_logits), _ptr(qI), _ptr(kI), _ptr(w), _ptr(bI),
                                    float(softmax_scale), _ptr(out), _ptr(idx_out), _ptr(n_sel_out), _ptr(k_out),
                                    _ptr(row_var_out), k_cap, _tun(tuning), _stream(stream))
    if rc == GSA_ERR_WORKSPACE:
        raise GsaError(rc, "gsa_forward_noalloc: " + load().gsa_last_error().decode())
    _check(rc, "gsa_forward_noalloc")


def gsa_cache_append(shape, kI_new, K_new, V_new, g2_new, seq_lens, kI_cache, K_cache, Vg_cache, seq_lens_out=None, stream=None):
    rc = load().gsa_cache_append(ctypes.byref(shape), _ptr(kI_new), _ptr(K_new), _ptr(V_new), _ptr(g2_new), _ptr(seq_lens),
                                 _ptr(kI_cache), _ptr(K_cache), _ptr(Vg_cache), _ptr(seq_lens_out), _stream(stream))
    _check(rc, "gsa_cache_append")


def gsa_input_projections(shape, d_model, h, W_Q, W_K, W_V, W_g1, W_g2, W_qI, W_kI, W_Iw, Q, K, V, g1_logits, g2_logits, qI, kI, w,
                          stream=None):
    rc = load().gsa_input_projections(ctypes.byref(shape), int(d_model), _ptr(h), _ptr(W_Q), _ptr(W_K), _ptr(W_V), _ptr(W_g1),
                                      _ptr(W_g2), _ptr(W_qI), _ptr(W_kI), _ptr(W_Iw), _ptr(Q), _ptr(K), _ptr(V), _ptr(g1_logits),
                                      _ptr(g2_logits), _ptr(qI), _ptr(kI), _ptr(w), _stream(stream))
    _check(rc, "gsa_input_projections")


def gsa_output_projection(shape, d_model, attn_out, W_O, y, stream=None):
    rc = load().gsa_output_projection(ctypes.byref(shape), int(d_model), _ptr(attn_out), _ptr(W_O), _ptr(y), _stream(stream))
    _check(rc, "gsa_output_projection")


def gsa_decode_workspace_bytes(shape, k_cap, tuning=None):
    return load().gsa_decode_workspace_bytes(ctypes.byref(shape), k_cap, _tun(tuning))


def gsa_decode_step(shape, ctl, Q, g1_logits, qI, w, bI, kI_cache, K_cache, Vg_cache, seq_lens, softmax_scale, out, idx_out,
                    n_sel_out, k_out, row_var_out, k_cap, workspace, workspace_bytes=None, tuning=None, stream=None):
    if workspace_bytes is None:
        workspace_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    rc = load().gsa_decode_step(ctypes.byref(shape), ctypes.byref(ctl) if ctl is not None else None, _ptr(Q), _ptr(g1_logits),
                                _ptr(qI), _ptr(w), _ptr(bI), _ptr(kI_cache), _ptr(K_cache), _ptr(Vg_cache), _ptr(seq_lens),
                                float(softmax_scale), _ptr(out), _ptr(idx_out), _ptr(n_sel_out), _ptr(k_out), _ptr(row_var_out),
                                k_cap, _ptr(workspace), workspace_bytes, _tun(tuning), _stream(stream))
    _check(rc, "gsa_decode_step")


def gsa_paged_cache_append(shape, page_size, block_table, pool_pages, kI_new, K_new, V_new, g2_new, seq_lens, kI_pool, K_pool, Vg_pool,
                           seq_lens_out=None, stream=None):
    rc = load().gsa_paged_cache_append(ctypes.byref(shape), page_size, _ptr(block_table), pool_pages, _ptr(kI_new), _ptr(K_new),
                                       _ptr(V_new), _ptr(g2_new), _ptr(seq_lens), _ptr(kI_pool), _ptr(K_pool), _ptr(Vg_pool),
                                       _ptr(seq_lens_out), _stream(stream))
    _check(rc, "gsa_paged_cache_append")


def gsa_paged_decode_workspace_bytes(shape, k_cap, tuning=None):
    return load().gsa_paged_decode_workspace_bytes(ctypes.byref(shape), k_cap, _tun(tuning))


def gsa_paged_decode_step(shape, ctl, page_size, block_table, pool_pages, Q, g1_logits, qI, w, bI, kI_pool, K_pool, Vg_pool, seq_lens,
                          softmax_scale, out, idx_out, n_sel_out, k_out, row_var_out, k_cap, workspace, workspace_bytes=None,
                          tuning=None, stream=None):
    if workspace_bytes is None:
        workspace_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    rc = load().gsa_paged_decode_step(ctypes.byref(shape), ctypes.byref(ctl) if ctl is not None else None, page_size,
                                      _ptr(block_table), pool_pages, _ptr(Q), _ptr(g1_logits), _ptr(qI), _ptr(w), _ptr(bI),
                                      _ptr(kI_pool), _ptr(K_pool), _ptr(Vg_pool), _ptr(seq_lens), float(softmax_scale), _ptr(out),
                                      _ptr(idx_out), _ptr(n_sel_out), _ptr(k_out), _ptr(row_var_out), k_cap, _ptr(workspace),
                                      workspace_bytes, _tun(tuning), _stream(stream))
    _check(rc, "gsa_paged_decode_step")


def gsa_sparse_gated_attn_bwd(shape, Q, K, V, g2_logits, g1_logits, idx, n_sel, k_cap, softmax_scale, dout, dQ, dK, dV, dg1, dg2,
                              p_mean=None, workspace=None, stream=None):
    rc = load().gsa_sparse_gated_attn_bwd(ctypes.byref(shape), _ptr(Q), _ptr(K), _ptr(V), _ptr(g2_logits), _ptr(g1_logits), _ptr(idx),
                                          _ptr(n_sel), k_cap, float(softmax_scale), _ptr(dout), _ptr(dQ), _ptr(dK), _ptr(dV), _ptr(dg1),
                                          _ptr(dg2), _ptr(p_mean), _ptr(workspace),
                                          0 if workspace is None else workspace.numel() * workspace.element_size(), _stream(stream))
    _check(rc, "gsa_sparse_gated_attn_bwd")


def gsa_attn_bwd_workspace_bytes(shape, k_cap):
    return int(load().gsa_attn_bwd_workspace_bytes(ctypes.byref(shape), k_cap))


def gsa_indexer_sparse_kl(shape, qI, kI, w, bI, idx, n_sel, k_cap, p, loss_rows, dqI, dkI, dw, dbI=None, stream=None):
    rc = load().gsa_indexer_sparse_kl(ctypes.byref(shape), _ptr(qI), _ptr(kI), _ptr(w), _ptr(bI), _ptr(idx), _ptr(n_sel), k_cap, _ptr(p),
                                      _ptr(loss_rows), _ptr(dqI), _ptr(dkI), _ptr(dw), _ptr(dbI), _stream(stream))
    _check(rc, "gsa_indexer_sparse_kl")


def gsa_dense_attn_workspace_bytes(shape, has_g2):
    return load().gsa_dense_attn_workspace_bytes(ctypes.byref(shape), int(bool(has_g2)))


def gsa_dense_gated_attn(shape, row_begin, row_end, Q, K, V, g2_logits, g1_logits, softmax_scale, out, workspace=None,
                         workspace_bytes=None, stream=None):
    if workspace_bytes is None:
        workspace_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    rc = load().gsa_dense_gated_attn(ctypes.byref(shape), row_begin, row_end, _ptr(Q), _ptr(K), _ptr(V), _ptr(g2_logits),
                                     _ptr(g1_logits), float(softmax_scale), _ptr(out), _ptr(workspace), workspace_bytes,
                                     _stream(stream))
    _check(rc, "gsa_dense_gated_attn")


def workspace(nbytes, device="cuda"):
    """Device scratch of at least nbytes, 256-byte aligned (torch's allocator aligns to 512)."""
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)
