"""The C ABI loads, exports what include/gsa.h declares, and rejects bad arguments on the host
before anything is launched (so none of this needs a GPU)."""
import ctypes
import os
import re

import pytest

import paper_2601_15305_amd as G

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "gsa.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(gsa_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    lib = G.load()
    names = _declared()
    assert set(names) == set(G.ENTRY_POINTS)
    for n in names:
        assert getattr(lib, n) is not None
    assert G.gsa_version() >= 100


def _shape(**kw):
    d = dict(B=1, Lq=64, Lk=64, q_offset=0, H=4, H_kv=2, d_h=64, HI=4, dI=32, dtype="bf16")
    d.update(kw)
    return G.make_shape(**d)


FAKE = 0x1000  # a 256-aligned non-null "pointer"; never dereferenced because validation fails first


def test_status_strings():
    lib = G.load()
    for s in (0, -1, -2, -3, -4, -5, -6):
        assert len(lib.gsa_status_string(s)) > 0
    assert lib.gsa_last_error() == b""


@pytest.mark.parametrize("kw,status", [
    (dict(B=0), G.GSA_ERR_SHAPE), (dict(Lq=0), G.GSA_ERR_SHAPE), (dict(H=3), G.GSA_ERR_SHAPE),
    (dict(q_offset=1), G.GSA_ERR_SHAPE), (dict(d_h=96), G.GSA_ERR_UNSUPPORTED), (dict(dI=48), G.GSA_ERR_UNSUPPORTED),
    (dict(HI=9), G.GSA_ERR_UNSUPPORTED), (dict(dtype=7), G.GSA_ERR_UNSUPPORTED), (dict(H=32, H_kv=1), G.GSA_ERR_UNSUPPORTED),
    (dict(Lk=(1 << 20) + 64, Lq=64), G.GSA_ERR_UNSUPPORTED),
])
def test_bad_shapes_rejected(kw, status):
    lib = G.load()
    sh = _shape(**kw)
    rc = lib.gsa_indexer_scores(ctypes.byref(sh), FAKE, FAKE, FAKE, None, 0, 1, None, 64, None, FAKE, FAKE, 1 << 20, None)
    assert rc == status
    ctl = G.make_adaptive(1.0, 8, 4, 16)
    assert lib.gsa_adaptive_k(ctypes.byref(sh), ctypes.byref(ctl), FAKE, None, FAKE, None) == status
    assert lib.gsa_topk_select(ctypes.byref(sh), 0, 1, FAKE, 64, FAKE, 16, FAKE, None, None) == status
    assert lib.gsa_sparse_gated_attn(ctypes.byref(sh), 0, 1, FAKE, FAKE, FAKE, None, None, FAKE, FAKE, 16, 0.0, FAKE, None, 0, None, None) == status
    assert lib.gsa_forward_workspace_bytes(ctypes.byref(sh), 16, 1, 0, None) == 0


def test_null_and_range_errors():
    lib = G.load()
    sh = _shape()
    assert lib.gsa_indexer_scores(None, FAKE, FAKE, FAKE, None, 0, 1, None, 64, None, FAKE, FAKE, 1 << 20, None) == G.GSA_ERR_NULL
    assert lib.gsa_indexer_scores(ctypes.byref(sh), None, FAKE, FAKE, None, 0, 1, None, 64, None, FAKE, FAKE, 1 << 20, None) == G.GSA_ERR_NULL
    assert lib.gsa_indexer_scores(ctypes.byref(sh), FAKE, FAKE, FAKE, None, 0, 1, None, 64, None, None, FAKE, 1 << 20, None) == G.GSA_ERR_NULL
    # row range
    for (r0, r1) in [(-1, 4), (4, 4), (0, 65), (9, 3)]:
        assert lib.gsa_indexer_scores(ctypes.byref(sh), FAKE, FAKE, FAKE, None, r0, r1, None, 64, None, FAKE, FAKE, 1 << 20, None) == G.GSA_ERR_SHAPE
        assert lib.gsa_topk_select(ctypes.byref(sh), r0, r1, FAKE, 64, FAKE, 16, FAKE, None, None) == G.GSA_ERR_SHAPE
    # leading dimension too small / not a multiple of 4, misaligned pointers
    assert lib.gsa_indexer_scores(ctypes.byref(sh), FAKE, FAKE, FAKE, None, 0, 1, FAKE, 60, None, FAKE, FAKE, 1 << 20, None) == G.GSA_ERR_SHAPE
    assert lib.gsa_indexer_scores(ctypes.byref(sh), FAKE, FAKE, FAKE, None, 0, 1, FAKE, 66, None, FAKE, FAKE, 1 << 20, None) == G.GSA_ERR_SHAPE
    assert lib.gsa_indexer_scores(ctypes.byref(sh), FAKE + 2, FAKE, FAKE, None, 0, 1, None, 64, None, FAKE, FAKE, 1 << 20, None) == G.GSA_ERR_SHAPE
    # workspace missing / too small / misaligned
    need = G.gsa_indexer_workspace_bytes(sh, 0, 64)
    assert need >= 64 * 8 and need % 256 == 0
    assert lib.gsa_indexer_scores(ctypes.byref(sh), FAKE, FAKE, FAKE, None, 0, 64, None, 64, None, FAKE, None, need, None) == G.GSA_ERR_WORKSPACE
    assert lib.gsa_indexer_scores(ctypes.byref(sh), FAKE, FAKE, FAKE, None, 0, 64, None, 64, None, FAKE, FAKE, 8, None) == G.GSA_ERR_WORKSPACE
    assert lib.gsa_indexer_scores(ctypes.byref(sh), FAKE, FAKE, FAKE, None, 0, 64, None, 64, None, FAKE, FAKE + 16, need, None) == G.GSA_ERR_WORKSPACE
    # k_cap bounds
    assert lib.gsa_topk_select(ctypes.byref(sh), 0, 1, FAKE, 64, FAKE, 0, FAKE, None, None) == G.GSA_ERR_SHAPE
    assert lib.gsa_topk_select(ctypes.byref(sh), 0, 1, FAKE, 64, FAKE, 8193, FAKE, None, None) == G.GSA_ERR_SHAPE
    assert lib.gsa_topk_select(ctypes.byref(sh), 0, 1, None, 64, FAKE, 16, FAKE, None, None) == G.GSA_ERR_NULL
    assert lib.gsa_sparse_gated_attn(ctypes.byref(sh), 0, 1, FAKE, FAKE, None, None, None, FAKE, FAKE, 16, 0.0, FAKE, None, 0, None, None) == G.GSA_ERR_NULL
    assert lib.gsa_sparse_gated_attn(ctypes.byref(sh), 0, 1, FAKE, FAKE, FAKE, None, None, FAKE, FAKE, 16, -1.0, FAKE, None, 0, None, None) == G.GSA_ERR_SHAPE
    assert lib.gsa_value_gate(ctypes.byref(sh), FAKE, None, FAKE, None) == G.GSA_ERR_NULL


def test_controller_argument_errors():
    lib = G.load()
    sh = _shape()

    def call(ctl):
        return lib.gsa_adaptive_k(ctypes.byref(sh), ctypes.byref(ctl), FAKE, None, FAKE, None)

    assert call(G.make_adaptive(0.0, 8, 4, 16)) == G.GSA_ERR_VBAR
    assert call(G.make_adaptive(-1.0, 8, 4, 16)) == G.GSA_ERR_VBAR
    assert call(G.make_adaptive(float("inf"), 8, 4, 16)) == G.GSA_ERR_VBAR
    assert call(G.make_adaptive(float("nan"), 8, 4, 16)) == G.GSA_ERR_VBAR
    assert call(G.make_adaptive(1.0, 8, 0, 16)) == G.GSA_ERR_SHAPE
    assert call(G.make_adaptive(1.0, 8, 17, 16)) == G.GSA_ERR_SHAPE
    assert call(G.make_adaptive(1.0, 0, 4, 16)) == G.GSA_ERR_SHAPE
    assert call(G.make_adaptive(1.0, 8, 4, 16, mode=2)) == G.GSA_ERR_UNSUPPORTED
    assert call(G.make_adaptive(1.0, 8, 4, 16, k_fixed=-3)) == G.GSA_ERR_SHAPE
    assert lib.gsa_adaptive_k(ctypes.byref(sh), None, FAKE, None, FAKE, None) == G.GSA_ERR_NULL
    # forward: k_max above k_cap, workspace too small
    ctl = G.make_adaptive(1.0, 8, 4, 16)
    args = [FAKE] * 9  # Q K V g1 g2 qI kI w bI
    assert lib.gsa_forward(ctypes.byref(sh), ctypes.byref(ctl), *args, 0.0, FAKE, None, None, None, None, 8, FAKE, 1 << 30, None, None) == G.GSA_ERR_SHAPE
    assert lib.gsa_forward(ctypes.byref(sh), ctypes.byref(ctl), *args, 0.0, FAKE, None, None, None, None, 16, FAKE, 1024, None, None) == G.GSA_ERR_WORKSPACE
    assert lib.gsa_forward(ctypes.byref(sh), ctypes.byref(ctl), *args, 0.0, FAKE, None, None, None, None, 16, None, 1 << 30, None, None) == G.GSA_ERR_WORKSPACE


def test_forward_workspace_grows_with_slab():
    sh = G.make_shape(1, 8192, 8192, 0, 16, 4, 128, 4, 64, "bf16")
    small = G.gsa_forward_workspace_bytes(sh, 2048, True, 0)
    big = G.gsa_forward_workspace_bytes(sh, 2048, True, 8192)
    assert 0 < small < big
    # the key slab dominates: rows * Lk * 2 bytes (fp32 scores on request: 4 bytes)
    assert big >= 8192 * 8192 * 2 and small >= 128 * 8192 * 2
    assert G.gsa_forward_workspace_bytes(sh, 2048, True, 8192, G.make_tuning(forward_fp32_scores=1)) >= 8192 * 8192 * 4
    assert G.gsa_forward_workspace_bytes(sh, 2048, False, 0) < small
    # the 128K prefill runs in well under 8 GiB with 8192-row slabs
    c4 = G.make_shape(1, 131072, 131072, 0, 16, 4, 128, 4, 64, "bf16")
    assert G.gsa_forward_workspace_bytes(c4, 4096, True, 8192) < 4 * (1 << 30)


def test_backward_workspace_size_and_host_side_checks():
    """The workspace of the two-pass attention backward: what it has to hold (the inverted lists, B * Lq * k_cap entries;
    dO in the element type; the gated values for bf16), and the argument checks that are decided before any launch."""
    import ctypes
    sh = G.make_shape(1, 8192, 8192, 0, 16, 4, 128, 4, 64, "bf16")
    w1, w2 = G.gsa_attn_bwd_workspace_bytes(sh, 1024), G.gsa_attn_bwd_workspace_bytes(sh, 4096)
    assert w1 % 256 == 0 and w2 % 256 == 0 and 0 < w1 < w2
    assert w2 - w1 == 8192 * (4096 - 1024) * 4                        # the lists: one int32 per (query, list slot)
    assert w1 >= 8192 * 1024 * 4 + 8192 * 16 * 128 * 2 + 8192 * 4 * 128 * 2
    f32 = G.make_shape(1, 8192, 8192, 0, 16, 4, 128, 4, 64, "f32")
    assert G.gsa_attn_bwd_workspace_bytes(f32, 1024) >= 8192 * 1024 * 4 + 8192 * 16 * 128 * 4
    assert G.gsa_attn_bwd_workspace_bytes(_shape(d_h=96), 64) == 0     # a shape the library does not take
    assert G.gsa_attn_bwd_workspace_bytes(sh, 0) == 0 and G.gsa_attn_bwd_workspace_bytes(sh, 9000) == 0
    lib = G.load()
    p = ctypes.c_void_p(FAKE)

    def call(workspace, nbytes, k_cap=1024, dg1=None, g1=None, shape=sh):
        return lib.gsa_sparse_gated_attn_bwd(ctypes.byref(shape), p, p, p, None, g1, p, p, k_cap, 0.0, p, p, p, p, dg1, None, None,
                                             workspace, nbytes, None)

    assert call(p, w1 - 256) == G.GSA_ERR_WORKSPACE and b"gsa_attn_bwd_workspace_bytes" in lib.gsa_last_error()
    assert call(ctypes.c_void_p(FAKE + 8), w1) == G.GSA_ERR_SHAPE      # workspace not 256-byte aligned
    assert call(p, w1, g1=p) == G.GSA_ERR_NULL                         # g1 without dg1
    assert call(p, w1, k_cap=0) == G.GSA_ERR_SHAPE
    huge = G.make_shape(64, 131072, 131072, 0, 16, 4, 128, 4, 64, "bf16")   # B * Lq * k_cap beyond 32-bit list positions
    assert call(p, 1 << 62, k_cap=4096, shape=huge) == G.GSA_ERR_UNSUPPORTED


def test_selection_rejects_contexts_beyond_the_on_chip_bitmaps():
    """The selection kernels keep bitmaps of a row in LDS; a context they cannot hold is refused on the host."""
    lib = G.load()
    text = open(os.path.join(ROOT, "include", "gsa.h")).read()
    max_lk = int(re.search(r"#define\s+GSA_SELECT_MAX_LK\s+(\d+)", text).group(1))
    ok = _shape(Lk=max_lk, Lq=64, q_offset=0)
    big = _shape(Lk=max_lk + 32, Lq=64, q_offset=0)
    assert lib.gsa_topk_select(ctypes.byref(big), 0, 1, FAKE, max_lk + 32, FAKE, 16, FAKE, None, None) == G.GSA_ERR_UNSUPPORTED
    assert lib.gsa_topk_select(ctypes.byref(ok), 0, 1, None, max_lk, FAKE, 16, FAKE, None, None) == G.GSA_ERR_NULL
    assert G.gsa_forward_workspace_bytes(big, 16, True, 0) == 0 and G.gsa_forward_workspace_bytes(ok, 16, True, 0) > 0
    ctl = G.make_adaptive(1.0, 8, 4, 16)
    args = [FAKE] * 9
    assert lib.gsa_forward(ctypes.byref(big), ctypes.byref(ctl), *args, 0.0, FAKE, None, None, None, None, 16, FAKE, 1 << 40, None, None) == G.GSA_ERR_UNSUPPORTED
    # the indexer and the attention alone still take it
    assert G.gsa_indexer_workspace_bytes(big, 0, 64) > 0


def test_missing_library_is_loud(monkeypatch, tmp_path):
    monkeypatch.setattr(G, "_lib", None)
    monkeypatch.setattr(G, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(RuntimeError):
        G.load()
