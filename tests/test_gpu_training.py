"""Training side (Sec. 6.1): gradients of the sparse gated attention (Sec. 3.5, 3.6) with the selection held fixed,
the sparse-phase indexer loss and the gradients it sends into the indexer (Sec. 3.3), against the fp64 oracle on
the same inputs and the same selection.

Tolerances: everything is fp32 arithmetic on bf16 or fp32 inputs, sums of up to k_cap * H products per entry,
added in an order that varies (atomics, or lists filled through atomic cursors): |got - ref| <= 2e-4 *
scale_of_that_tensor + 1e-6, where the scale is the largest |ref| entry (gradient entries of one tensor are sums of
the same kind).  Both forms of the attention backward run: with a workspace (dK, dV' summed key by key over inverted
lists) and without (fp32 atomics).  With a workspace and bf16 inputs the query-centred pass is the matrix-core
kernel, whose products take P, dO and dS rounded to bf16 like the forward's: 1e-2 of the scale there."""
import numpy as np
import pytest
import torch

import paper_2601_15305_amd as G
from paper_2601_15305_amd import synthetic as S
from oracle import gsa_oracle as O

import gsa_testlib as T

pytestmark = pytest.mark.gpu


def _close(got, ref, what, rel=2e-4):
    got = got.double().cpu().numpy() if isinstance(got, torch.Tensor) else np.asarray(got)
    scale = max(float(np.abs(ref).max()), 1e-30)
    err = float(np.abs(got - ref).max())
    assert np.isfinite(got).all(), what
    assert err <= rel * scale + 1e-6, "%s: max error %.3g against scale %.3g" % (what, err, scale)


def _selection(wl, t, k_fixed):
    """A fixed-budget selection from the library's own forward stages (any valid ascending index lists would do)."""
    ctl = G.make_adaptive(1.0, 1, 1, 1, k_fixed=k_fixed)
    res = T.gpu_forward(wl, t, ctl, k_cap=k_fixed)
    return res["idx"], res["n_sel"]


CASES = [
    # dtype, B, L, H, Hkv, dh, HI, dI, k, gates, bias
    ("bf16", 2, 150, 4, 2, 64, 2, 32, 48, True, True),
    ("bf16", 1, 200, 16, 4, 128, 4, 64, 70, True, False),
    ("f32", 1, 130, 4, 4, 64, 3, 64, 33, False, True),
    ("f32", 2, 90, 8, 2, 128, 8, 128, 90, True, False),     # budget covers every visible key of every row
    ("bf16", 1, 140, 16, 1, 64, 5, 32, 130, True, True),    # sixteen query heads on one kv head: four chunks of four heads
    ("bf16", 1, 150, 12, 4, 64, 2, 32, 40, True, False),    # groups of three heads: a head slot of the key-centred pass stays idle
    ("bf16", 1, 300, 16, 1, 128, 2, 32, 64, True, False),   # wide rows: the key-centred pass runs over three windows of 128 queries
    ("f32", 2, 200, 16, 1, 128, 2, 32, 50, False, True),    # ... four windows of 64 queries, two batch elements, fp32 throughout
]


@pytest.mark.parametrize("two_pass", [True, False], ids=["key-centred second pass", "atomics"])
@pytest.mark.parametrize("dtype,B,L,H,Hkv,dh,HI,dI,k,gates,bias", CASES)
def test_attention_backward_and_sparse_kl(dtype, B, L, H, Hkv, dh, HI, dI, k, gates, bias, two_pass):
    wl = S.Workload("train", B, L, L, 0, H, Hkv, dh, HI, dI, dtype, k, k, k, k_fixed=k, seed=400 + L)
    t_cpu = S.make_inputs(wl, "cpu", with_bias=bias)
    t = T.to_device(t_cpu)
    sh = G.shape_of(wl)
    idx, n_sel = _selection(wl, t, k)
    gen = torch.Generator().manual_seed(L)
    dout = torch.randn(t_cpu["Q"].shape, generator=gen).to(t_cpu["Q"].dtype).cuda()
    f32 = dict(dtype=torch.float32, device="cuda")
    dQ = torch.full(t["Q"].shape, float("nan"), **f32)
    dK = torch.full(t["K"].shape, float("nan"), **f32)
    dV = torch.full(t["K"].shape, float("nan"), **f32)
    dg1 = torch.full(t["Q"].shape, float("nan"), **f32) if gates else None
    dg2 = torch.full(t["K"].shape, float("nan"), **f32) if gates else None
    p_mean = torch.full((B, L, k), float("nan"), **f32)
    ws = None
    if two_pass:
        ws = G.workspace(G.gsa_attn_bwd_workspace_bytes(sh, k))
        ws.fill_(0x7F)      # nothing in the workspace has to be cleared by the caller
    G.gsa_sparse_gated_attn_bwd(sh, t["Q"], t["K"], t["V"], t["g2"] if gates else None, t["g1"] if gates else None, idx, n_sel, k, 0.0,
                                dout, dQ, dK, dV, dg1, dg2, p_mean, workspace=ws)
    loss = torch.full((B, L), float("nan"), **f32)
    dqI = torch.full(t["qI"].shape, float("nan"), **f32)
    dkI = torch.full(t["kI"].shape, float("nan"), **f32)
    dw = torch.full(t["w"].shape, float("nan"), **f32)
    dbI = torch.full((HI,), float("nan"), **f32) if bias else None
    G.gsa_indexer_sparse_kl(sh, t["qI"], t["kI"], t["w"], t["bI"] if bias else None, idx, n_sel, k, p_mean, loss, dqI, dkI, dw, dbI)
    torch.cuda.synchronize()

    o = T.oracle_inputs(t_cpu)
    idx_h, n_h = idx.cpu().numpy(), n_sel.cpu().numpy()
    d64 = dout.double().cpu().numpy()
    r_dQ = np.zeros(o["Q"].shape); r_dg1 = np.zeros(o["Q"].shape)
    r_dK = np.zeros(o["K"].shape); r_dV = np.zeros(o["K"].shape); r_dg2 = np.zeros(o["K"].shape)
    r_p = np.zeros((B, L, k)); r_loss = np.zeros((B, L))
    r_dqI = np.zeros(o["qI"].shape); r_dkI = np.zeros(o["kI"].shape); r_dw = np.zeros(o["w"].shape); r_dbI = np.zeros(HI)
    for b in range(B):
        for i in range(L):
            m = int(n_h[b, i])
            sel = idx_h[b, i, :m]
            g2b = o["g2"][b] if gates else None
            g1r = o["g1"][b, i] if gates else None
            a, c, dk_, dv_, dg2_ = O.sparse_gated_attn_bwd_row(o["Q"][b, i], o["K"][b], o["V"][b], g2b, g1r, sel, d64[b, i])
            r_dQ[b, i] = a; r_dg1[b, i] = c
            np.add.at(r_dK[b], sel, dk_); np.add.at(r_dV[b], sel, dv_); np.add.at(r_dg2[b], sel, dg2_)
            _, A = O.sparse_gated_attn_row(o["Q"][b, i], o["K"][b], o["V"][b], g2b, g1r, sel)
            r_p[b, i, :m] = A.mean(0)
            I_sel = O.indexer_scores_row(o["qI"][b, i], o["kI"][b][sel], o["w"][b, i], o["bI"] if bias else None)
            r_loss[b, i], dI = O.indexer_sparse_kl_row(A, I_sel)
            q_, k_, w_, b_ = O.indexer_scores_bwd_row(o["qI"][b, i], o["kI"][b][sel], o["w"][b, i], o["bI"] if bias else None, dI)
            r_dqI[b, i] = q_; r_dw[b, i] = w_; r_dbI += b_
            np.add.at(r_dkI[b], sel, k_)
    # bf16 inputs with a workspace: the query-centred pass runs on the matrix cores with P, dO and dS rounded to bf16
    # (unit roundoff u = 2^-9 per operand).  An entry of dQ is a sum of signed products dS_j K_jd whose absolute values
    # add up to a few times the largest entry, so the rounding of dS alone can move it by a few u of the scale: 5 u = 1e-2
    rel = 1e-2 if (two_pass and dtype == "bf16") else 2e-4
    _close(dQ, r_dQ, "dQ", rel); _close(dK, r_dK, "dK", rel); _close(dV, r_dV, "dV", rel)
    if gates:
        _close(dg1, r_dg1, "dg1", rel); _close(dg2, r_dg2, "dg2", rel)
    valid = (np.arange(k)[None, None, :] < n_h[..., None])
    _close(torch.where(torch.from_numpy(valid).cuda(), p_mean, torch.zeros_like(p_mean)), r_p, "p_mean", rel=2e-5)
    assert np.allclose(np.where(valid, p_mean.cpu().numpy(), 0).sum(-1)[n_h > 0], 1.0, atol=1e-5)
    got_loss = loss.double().cpu().numpy()
    assert np.all(np.abs(got_loss - r_loss) <= 2e-4 * np.abs(r_loss) + 2e-5), float(np.abs(got_loss - r_loss).max())
    _close(dqI, r_dqI, "dqI"); _close(dkI, r_dkI, "dkI"); _close(dw, r_dw, "dw")
    if bias:
        _close(dbI, r_dbI, "dbI")
    # keys that no query selected receive exactly zero
    touched = np.zeros((B, L), bool)
    for b in range(B):
        for i in range(L):
            touched[b, idx_h[b, i, :n_h[b, i]]] = True
    assert not dK.cpu().numpy()[~touched].any() and not dkI.cpu().numpy()[~touched].any()


def test_training_entry_points_reject_half_given_pairs():
    wl = S.Workload("trainerr", 1, 64, 64, 0, 4, 2, 64, 2, 32, "bf16", 8, 8, 8, k_fixed=8, seed=1)
    t = S.make_inputs(wl, "cuda")
    sh = G.shape_of(wl)
    idx, n_sel = _selection(wl, t, 8)
    f = lambda like: torch.empty(like.shape, dtype=torch.float32, device="cuda")
    with pytest.raises(G.GsaError) as e:      # g1 without dg1
        G.gsa_sparse_gated_attn_bwd(sh, t["Q"], t["K"], t["V"], None, t["g1"], idx, n_sel, 8, 0.0, t["Q"], f(t["Q"]), f(t["K"]), f(t["K"]),
                                    None, None)
    assert e.value.status == G.GSA_ERR_NULL
    with pytest.raises(G.GsaError) as e:      # a workspace that is too small
        G.gsa_sparse_gated_attn_bwd(sh, t["Q"], t["K"], t["V"], None, None, idx, n_sel, 8, 0.0, t["Q"], f(t["Q"]), f(t["K"]), f(t["K"]),
                                    None, None, workspace=G.workspace(256))
    assert e.value.status == G.GSA_ERR_WORKSPACE
    with pytest.raises(G.GsaError) as e:      # dbI without bI
        G.gsa_indexer_sparse_kl(sh, t["qI"], t["kI"], t["w"], None, idx, n_sel, 8, torch.zeros((1, 64, 8), device="cuda"),
                                torch.empty((1, 64), device="cuda"), f(t["qI"]), f(t["kI"]), f(t["w"]), torch.empty(2, device="cuda"))
    assert e.value.status == G.GSA_ERR_NULL
