"""GPU parity: every stage of the HIP path, called through the C ABI, against the fp64 oracle on the
same seeded inputs.  Sizes span several tiles and ragged tails; index work is compared bit-exactly,
floating point within the stated tolerances (see gsa_testlib)."""
import math

import numpy as np
import pytest
import torch

import paper_2601_15305_amd as G
from paper_2601_15305_amd import synthetic as S
from oracle import gsa_oracle as O

import gsa_testlib as T

pytestmark = pytest.mark.gpu


def wl_(name, B, Lq, Lk, off, H, Hkv, dh, HI, dI, dtype, kmin=8, kmax=64, kbase=None, **kw):
    return S.Workload(name, B, Lq, Lk, off, H, Hkv, dh, HI, dI, dtype, kbase or int(math.sqrt(kmin * kmax)), kmin, kmax, **kw)


# ------------------------------------------------------------------------------------ stage 1
INDEXER_CASES = [
    # dtype, HI, dI, B, Lq, Lk, q_offset, bias
    ("f32", 4, 32, 1, 512, 512, 0, False),
    ("bf16", 4, 64, 2, 700, 700, 0, True),
    ("bf16", 4, 64, 1, 100, 1000, 900, False),
    ("bf16", 1, 32, 1, 300, 300, 0, True),
    ("bf16", 2, 128, 1, 260, 260, 0, False),
    ("bf16", 8, 64, 2, 150, 333, 183, True),
    ("f32", 8, 64, 1, 130, 130, 0, True),
    ("f32", 2, 128, 1, 200, 200, 0, False),
    ("f32", 1, 64, 1, 257, 257, 0, False),
    # head counts that are not a power of two: the kernels pad them with zero-weight heads
    ("bf16", 3, 64, 1, 300, 300, 0, True),
    ("bf16", 6, 32, 2, 200, 260, 60, False),
    ("f32", 5, 64, 1, 150, 150, 0, True),
    ("bf16", 7, 128, 1, 140, 140, 0, True),
]


@pytest.mark.parametrize("dtype,HI,dI,B,Lq,Lk,off,bias", INDEXER_CASES)
def test_indexer_scores_and_stats(dtype, HI, dI, B, Lq, Lk, off, bias):
    wl = wl_("idx", B, Lq, Lk, off, 4, 2, 64, HI, dI, dtype, seed=11 + HI + dI)
    t = S.make_inputs(wl, "cpu", with_bias=bias)
    ref, rmean, rvar = O.indexer_scores(*(T.to64(t[k]) for k in ("qI", "kI", "w")), T.to64(t["bI"]), off)
    d = T.to_device(t)
    scores, mean, var = T.gpu_indexer(wl, d)
    got = T.to64(scores)[:, :, :Lk]
    vis = ~np.isnan(ref)
    assert np.all(np.isnan(got[~vis])), "invisible positions must be left untouched"
    err = np.abs(got[vis] - ref[vis]).max()
    atol = 3e-6 if dtype == "bf16" else 1e-5
    assert err <= atol, "score error %.3g" % err
    wsum = T.to64(t["w"]).sum(-1)[..., None]
    assert np.all(got[vis] >= 0) and np.all((got <= wsum * (1 + 1e-6))[vis])      # Sec. 3.3: I in (0, sum w) up to rounding
    assert np.abs(T.to64(mean) - rmean).max() <= 3e-6
    assert np.all(np.abs(T.to64(var) - rvar) <= 2e-5 * rvar + 5e-8)
    # statistics-only mode gives the same statistics; a slab of rows gives the same scores
    _, mean2, var2 = T.gpu_indexer(wl, d, want_scores=False)
    assert torch.equal(mean2, mean) and torch.equal(var2, var)
    r0, r1 = Lq // 5, Lq - Lq // 7
    s3, _, var3 = T.gpu_indexer(wl, d, r0, r1)
    g3 = T.to64(s3)[:, :, :Lk]
    assert np.array_equal(np.nan_to_num(g3, nan=-1.0), np.nan_to_num(got[:, r0:r1], nan=-1.0))
    assert np.all(np.abs(T.to64(var3)[:, r0:r1] - rvar[:, r0:r1]) <= 2e-5 * rvar[:, r0:r1] + 5e-8)


KEY_CASES = [
    # dtype, HI, dI, B, Lq, Lk, q_offset, bias, k_cap
    ("bf16", 4, 64, 2, 700, 700, 0, True, 96),
    ("bf16", 3, 64, 1, 300, 1000, 700, False, 128),
    ("f32", 5, 32, 1, 400, 400, 0, True, 64),
    ("bf16", 8, 32, 1, 260, 260, 0, False, 200),
    ("bf16", 4, 32, 1, 9000, 9000, 0, False, 512),      # rows long enough for the one-pass sampled selection
]


@pytest.mark.parametrize("wave", [1, -1])
@pytest.mark.parametrize("dtype,HI,dI,B,Lq,Lk,off,bias,k_cap", KEY_CASES)
def test_indexer_keys_and_selection_on_keys(dtype, HI, dI, B, Lq, Lk, off, bias, k_cap, wave):
    """The two stage calls in the form the fused forward uses: 16-bit fixed-point keys of the scores
    (Sec. 3.3) and the top-k_t selection on them (Eq. 4), against the fp64 oracle.  Both selection kernels:
    one wave per row (wave = 1; rows its estimate fails on fall back) and one workgroup per row (wave = -1)."""
    wl = wl_("keys", B, Lq, Lk, off, 4, 2, 64, HI, dI, dtype, seed=300 + HI + dI)
    t = S.make_inputs(wl, "cpu", with_bias=bias)
    d = T.to_device(t)
    sh = G.shape_of(wl)
    ld = (Lk + 31) // 32 * 32
    keys = torch.full((B, Lq, ld), 0x7777, dtype=torch.int16, device="cuda")
    mean = torch.empty((B, Lq), dtype=torch.float32, device="cuda")
    var = torch.empty_like(mean)
    ws = G.workspace(G.gsa_indexer_workspace_bytes(sh, 0, Lq), "cuda")
    G.gsa_indexer_keys(sh, d["qI"], d["kI"], d["w"], d["bI"], 0, Lq, keys, ld, mean, var, ws)
    _, mean2, var2 = T.gpu_indexer(wl, d, want_scores=False)
    assert torch.equal(mean, mean2) and torch.equal(var, var2), "the statistics do not depend on the output mode"
    r = np.random.default_rng(HI)
    n_sel = torch.from_numpy(r.integers(1, k_cap + 1, (B, Lq)).astype(np.int32)).cuda()
    idx = torch.full((B, Lq, k_cap), -7, dtype=torch.int32, device="cuda")
    G.gsa_topk_select_keys(sh, 0, Lq, keys, ld, n_sel, k_cap, idx, d["qI"], d["kI"], d["w"], d["bI"],
                           tuning=G.make_tuning(select_wave_min_rows=wave))
    torch.cuda.synchronize()
    HIK = 1 << (HI - 1).bit_length()
    kh = keys.cpu().numpy().view(np.uint16).astype(np.int64)
    o = T.oracle_inputs(t)
    idx_h, n_h = idx.cpu().numpy(), n_sel.cpu().numpy()
    rows = [(int(b), int(i)) for b, i in zip(r.integers(0, B, 50), r.integers(0, Lq, 50))] + [(0, 0), (B - 1, Lq - 1)]
    exact = total = excused = 0
    for (b, i) in rows:
        n = O.n_visible(i, off, Lk)
        I = O.indexer_scores_row(o["qI"][b, i], o["kI"][b, :n], o["w"][b, i], o["bI"])
        want = np.minimum(65535, np.floor(I * (65536.0 / HIK))).astype(np.int64)
        assert np.abs(kh[b, i, :n] - want).max() <= 1, "a key is the floor of the scaled score up to fp32 rounding"
        assert np.all(kh[b, i, n:Lk] == 0x7777), "positions of invisible keys are left untouched"
        exact += int((kh[b, i, :n] == want).sum())
        total += n
        m = int(min(n_h[b, i], n))
        T.check_index_row_wellformed(idx_h[b, i], m, n, k_cap)
        excused += T.check_selection_vs_fp64(idx_h[b, i], m, I)
    assert exact >= 0.9 * total
    assert excused <= len(rows) // 4


RELU_CASES = [
    # dtype, HI, dI, B, Lq, Lk, q_offset, bias
    ("bf16", 4, 64, 2, 700, 700, 0, False),
    ("bf16", 3, 32, 1, 260, 900, 640, True),
    ("f32", 8, 64, 1, 300, 300, 0, False),
    ("bf16", 1, 128, 1, 1, 2000, 1999, False),
]


@pytest.mark.parametrize("dtype,HI,dI,B,Lq,Lk,off,bias", RELU_CASES)
def test_relu_indexer_scores_and_stats(dtype, HI, dI, B, Lq, Lk, off, bias):
    """The ungated indexer of Sec. 2.2 Eq. 3 (comparison variant): scores and row statistics against the oracle."""
    wl = wl_("relu", B, Lq, Lk, off, 4, 2, 64, HI, dI, dtype, seed=500 + HI + dI, indexer_act="relu")
    t = S.make_inputs(wl, "cpu", with_bias=bias)
    ref, rmean, rvar = O.indexer_scores(*(T.to64(t[k]) for k in ("qI", "kI", "w")), T.to64(t["bI"]), off, act="relu")
    d = T.to_device(t)
    scores, mean, var = T.gpu_indexer(wl, d)
    got = T.to64(scores)[:, :, :Lk]
    vis = ~np.isnan(ref)
    assert np.all(np.isnan(got[~vis])), "invisible positions must be left untouched"
    assert np.abs(got[vis] - ref[vis]).max() <= 1e-4, "64-term fp32 sums of logits of magnitude up to ~40, times w"
    assert np.all(got[vis] >= 0) and ((got[vis] == 0) == (ref[vis] == 0)).mean() > 0.9999
    assert np.abs(T.to64(mean) - rmean).max() <= 1e-4
    assert np.all(np.abs(T.to64(var) - rvar) <= 2e-4 * rvar + 1e-6)
    _, mean2, var2 = T.gpu_indexer(wl, d, want_scores=False)
    assert torch.equal(mean2, mean) and torch.equal(var2, var)
    # the key form needs bounded scores: refused for this variant
    sh = G.shape_of(wl)
    with pytest.raises(G.GsaError) as ei:
        G.gsa_indexer_keys(sh, d["qI"], d["kI"], d["w"], None, 0, Lq, scores, scores.shape[-1], None, var, scores)
    assert ei.value.status == G.GSA_ERR_UNSUPPORTED


@pytest.mark.parametrize("gated", [False, True])
def test_forward_relu_indexer_fixed_k(gated):
    """The "sparse only" comparison variant of Sec. 7.1 (ReLU indexer, fixed k, no gates), and the same indexer
    with the gates on: selection and outputs against the oracle."""
    wl = wl_("sparse-only", 2, 1300, 1300, 0, 16, 4, 128, 4, 64, "bf16", kmin=96, kmax=96, kbase=96, seed=88, indexer_act="relu",
             k_fixed=96)
    t = S.make_inputs(wl, "cpu")
    d = T.to_device(t)
    ctl = G.make_adaptive(1.0, 1, 1, 1, k_fixed=96)
    kw = dict(vbar=1.0, k_base=1, k_min=1, k_max=1, k_fixed=96, mode=0)
    res = T.gpu_forward(wl, d, ctl, use_g1=gated, use_g2=gated, slab_rows=512)
    o = T.oracle_inputs(t)
    idx, n_sel, out = res["idx"].cpu().numpy(), res["n_sel"].cpu().numpy(), T.to64(res["out"])
    r = np.random.default_rng(4)
    rows = sorted({(int(b), int(i)) for b, i in zip(r.integers(0, 2, 40), r.integers(0, 1300, 40))} | {(0, 0), (1, 1299), (0, 95), (1, 96)})
    excused = 0
    for (b, i) in rows:
        n = i + 1
        I = O.indexer_scores_row(o["qI"][b, i], o["kI"][b, :n], o["w"][b, i], None, "relu")
        assert n_sel[b, i] == min(96, n)
        T.check_index_row_wellformed(idx[b, i], n_sel[b, i], n, 96)
        excused += T.check_selection_vs_fp64(idx[b, i], int(n_sel[b, i]), I)
        ref, _ = O.sparse_gated_attn_row(o["Q"][b, i], o["K"][b], o["V"][b], o["g2"][b] if gated else None,
                                         o["g1"][b, i] if gated else None, idx[b, i, :n_sel[b, i]])
        T.check_out(out[b, i], ref, "bf16")
    assert excused <= 4


def test_indexer_closed_forms_on_gpu():
    """q^I = 0: every score is (1/2) sum_j w_j and the variance is 0; saturated logits give exact ties."""
    wl = wl_("idx0", 1, 200, 200, 0, 4, 2, 64, 4, 64, "bf16", seed=5)
    t = S.make_inputs(wl, "cpu")
    t["qI"].zero_()
    d = T.to_device(t)
    scores, mean, var = T.gpu_indexer(wl, d)
    want = 0.5 * T.to64(t["w"]).sum(-1)
    got = T.to64(scores)
    for i in (0, 57, 199):
        assert np.abs(got[0, i, :i + 1] - want[0, i]).max() <= 3e-7
    assert T.to64(var).max() <= 1e-12 and np.abs(T.to64(mean) - want).max() <= 3e-7


# ------------------------------------------------------------------------------------ stage 2
@pytest.mark.parametrize("mode", [0, 1])
def test_adaptive_k_bit_exact(mode):
    wl = wl_("ctl", 3, 1000, 1000, 0, 4, 2, 64, 4, 64, "bf16")
    g = torch.Generator().manual_seed(3)
    var = (torch.rand((3, 1000), generator=g) ** 2 * 2.0).float()
    var[0, :5] = torch.tensor([0.0, 1e-30, 0.35, 0.35 * (1 + 2 ** -20), 1e30])
    vbar = float(np.float32(0.35))
    ctl = G.make_adaptive(vbar, 300, 40, 700, 0, mode)
    k, n_sel = T.gpu_adaptive_k(wl, ctl, var.cuda())
    ref = O.adaptive_k(var.double().numpy(), vbar, 300, 40, 700, 0, mode)
    assert np.array_equal(k.cpu().numpy().astype(np.int64), ref)
    nvis = np.arange(1, 1001)[None, :]
    assert np.array_equal(n_sel.cpu().numpy().astype(np.int64), np.minimum(ref, nvis))
    assert ref.min() == 40 and ref.max() == 700 and len(np.unique(ref)) > 100
    k2, n2 = T.gpu_adaptive_k(wl, G.make_adaptive(0.0, 1, 1, 1, k_fixed=77), var.cuda())
    assert torch.all(k2 == 77) and np.array_equal(n2.cpu().numpy(), np.minimum(77, nvis).repeat(3, 0))


# ------------------------------------------------------------------------------------ stage 3
def _select_case(scores_np, n_sel_np, k_cap, q_offset):
    """scores_np [B, Lq, Lk] float32 (full rows; only the visible prefix matters)."""
    B, Lq, Lk = scores_np.shape
    wl = wl_("sel", B, Lq, Lk, q_offset, 4, 2, 64, 4, 64, "bf16")
    ld = (Lk + 31) // 32 * 32
    sc = torch.full((B, Lq, ld), float("nan"))
    sc[:, :, :Lk] = torch.from_numpy(scores_np)
    for i in range(Lq):                       # poison what is not visible: it must never be read as data
        sc[:, i, O.n_visible(i, q_offset, Lk):] = float("inf")
    idx = T.gpu_select(wl, sc.cuda(), torch.from_numpy(n_sel_np.astype(np.int32)).cuda(), k_cap).cpu().numpy()
    for b in range(B):
        for i in range(Lq):
            n = O.n_visible(i, q_offset, Lk)
            m = int(min(n_sel_np[b, i], n, k_cap))
            T.check_index_row_wellformed(idx[b, i], m, n, k_cap)
            want = O.topk_select_row(scores_np[b, i, :n].astype(np.float64), m)
            assert np.array_equal(idx[b, i, :m], want), "row (%d,%d) n=%d m=%d" % (b, i, n, m)


def test_select_small_rows_all_distributions():
    r = np.random.default_rng(21)
    B, L, k_cap = 2, 600, 128
    base = r.uniform(0, 4, (B, L, L)).astype(np.float32)
    n_sel = r.integers(1, k_cap + 1, (B, L))
    n_sel[0, :8] = [1, 1, 2, 3, 128, 128, 5, 8]
    _select_case(base, n_sel, k_cap, 0)
    ties = np.round(base * 4) / 4            # 17 distinct values: exact ties everywhere
    _select_case(ties, n_sel, k_cap, 0)
    const = np.full_like(base, 1.25)
    _select_case(const, n_sel, k_cap, 0)
    inc = np.broadcast_to(np.linspace(0.01, 3.9, L, dtype=np.float32), (B, L, L)).copy()
    _select_case(inc, n_sel, k_cap, 0)
    _select_case(inc[:, :, ::-1].copy(), n_sel, k_cap, 0)
    tiny = (base * 1e-30).astype(np.float32)  # denormal-adjacent magnitudes and zeros
    tiny[:, :, ::7] = 0.0
    _select_case(tiny, n_sel, k_cap, 0)


@pytest.mark.parametrize("kind", ["uniform", "saturated", "constant", "narrow"])
def test_select_long_rows(kind):
    """Rows of 131072 scores (the 128K configuration): several histogram passes, candidate overflow, ties."""
    r = np.random.default_rng(33)
    B, Lq, Lk, k_cap = 1, 6, 131072, 4096
    if kind == "uniform":
        sc = r.uniform(0, 4, (B, Lq, Lk)).astype(np.float32)
    elif kind == "saturated":             # sums of a few fixed weights: at most 16 distinct values
        wts = np.array([0.31, 0.77, 0.52, 0.93], np.float32)
        bits = r.integers(0, 16, (B, Lq, Lk))
        sc = sum(((bits >> j) & 1).astype(np.float32) * wts[j] for j in range(4)).astype(np.float32)
    elif kind == "constant":
        sc = np.full((B, Lq, Lk), 2.5, np.float32)
    else:                                  # everything inside one 13-bit bin, distinct low bits
        sc = (2.0 + r.uniform(0, 1e-3, (B, Lq, Lk))).astype(np.float32)
    n_sel = np.array([[1, 1000, 2048, 4096, 4095, 3]])
    _select_case(sc, n_sel, k_cap, Lk - Lq)


# ------------------------------------------------------------------------------------ stage 4
def _random_sets(r, wl, k_cap):
    idx = np.full((wl.B, wl.Lq, k_cap), -1, np.int32)
    n_sel = np.zeros((wl.B, wl.Lq), np.int32)
    for b in range(wl.B):
        for i in range(wl.Lq):
            n = O.n_visible(i, wl.q_offset, wl.Lk)
            m = int(r.integers(1, min(k_cap, n) + 1))
            n_sel[b, i] = m
            idx[b, i, :m] = np.sort(r.choice(n, m, replace=False))
    return idx, n_sel


ATTN_CASES = [
    # dtype, H, Hkv, dh, B, Lq, Lk, off, k_cap
    ("bf16", 16, 4, 128, 2, 150, 150, 0, 100),
    ("bf16", 16, 16, 128, 1, 90, 90, 0, 70),
    ("bf16", 16, 1, 128, 1, 70, 70, 0, 70),
    ("bf16", 8, 2, 64, 1, 130, 130, 0, 96),
    ("bf16", 16, 4, 128, 3, 1, 400, 399, 333),
    ("bf16", 12, 4, 128, 1, 80, 80, 0, 60),      # groups of three heads (the fourth head slot of a transfer is a copy)
    ("bf16", 12, 2, 128, 1, 80, 80, 0, 60),      # groups of six heads: two query-head transfers per row
    ("f32", 4, 4, 64, 1, 200, 200, 0, 64),
    ("f32", 4, 1, 128, 2, 100, 100, 0, 100),
]


@pytest.mark.parametrize("dtype,H,Hkv,dh,B,Lq,Lk,off,k_cap", ATTN_CASES)
def test_sparse_gated_attention(dtype, H, Hkv, dh, B, Lq, Lk, off, k_cap):
    _attention_case(dtype, H, Hkv, dh, B, Lq, Lk, off, k_cap)


@pytest.mark.parametrize("rpw", [2, 7, 64])
@pytest.mark.parametrize("dtype,H,Hkv,dh,B,Lq,Lk,off,k_cap", [c for c in ATTN_CASES if c[0] == "bf16"])
def test_sparse_gated_attention_rows_per_wave(rpw, dtype, H, Hkv, dh, B, Lq, Lk, off, k_cap):
    """Several query rows streamed through one wave (what long prefills do), forced onto small shapes: rows whose
    list is empty, rows that end inside a tile, a last wave with fewer rows than the others."""
    _attention_case(dtype, H, Hkv, dh, B, Lq, Lk, off, k_cap, G.make_tuning(attn_rows_per_wave=rpw))


@pytest.mark.parametrize("window", [16, 50, 64])
@pytest.mark.parametrize("dtype,H,Hkv,dh,B,Lq,Lk,off,k_cap", [c for c in ATTN_CASES if c[0] == "bf16"])
def test_sparse_gated_attention_key_windows(window, dtype, H, Hkv, dh, B, Lq, Lk, off, k_cap):
    """The key-window launch scheme of long prefills (one launch per window of keys, partial results merged
    afterwards), forced onto small shapes so that the oracle covers every row: windows that a row does not
    reach, windows without a selected key, lists that end inside a window."""
    _attention_case(dtype, H, Hkv, dh, B, Lq, Lk, off, k_cap, G.make_tuning(attn_window=window, attn_rows_per_wave=1 + window % 5))


def _attention_case(dtype, H, Hkv, dh, B, Lq, Lk, off, k_cap, tuning=None):
    wl = wl_("att", B, Lq, Lk, off, H, Hkv, dh, 4, 32, dtype, seed=40 + H + Hkv, gate_std=1.5)
    t = S.make_inputs(wl, "cpu")
    r = np.random.default_rng(7)
    idx, n_sel = _random_sets(r, wl, k_cap)
    if Lq > 3:
        n_sel[0, -1] = min(k_cap, O.n_visible(Lq - 1, off, Lk))       # a full row
        idx[0, -1, :n_sel[0, -1]] = np.sort(r.choice(O.n_visible(Lq - 1, off, Lk), n_sel[0, -1], replace=False))
        n_sel[0, 2] = 0                                                # an empty row -> zeros
        idx[0, 2] = -1
    d = T.to_device(t)
    di, dn = torch.from_numpy(idx).cuda(), torch.from_numpy(n_sel).cuda()
    o = T.oracle_inputs(t)

    def ref(use_g2, use_g1, scale=None):
        out = np.zeros((B, Lq, H, dh))
        for b in range(B):
            for i in range(Lq):
                out[b, i], _ = O.sparse_gated_attn_row(o["Q"][b, i], o["K"][b], o["V"][b], o["g2"][b] if use_g2 else None,
                                                       o["g1"][b, i] if use_g1 else None, idx[b, i, :n_sel[b, i]], scale)
        return out

    full = ref(True, True)
    T.check_out(T.gpu_attention(wl, d, di, dn, k_cap, tuning=tuning), full, dtype)
    T.check_out(T.gpu_attention(wl, d, di, dn, k_cap, use_g1=False, tuning=tuning), ref(True, False), dtype)
    T.check_out(T.gpu_attention(wl, d, di, dn, k_cap, use_g2=False, use_g1=False, scale=0.2, tuning=tuning), ref(False, False, 0.2), dtype)
    # G2 as a dense pre-pass followed by the ungated-V kernel is the same computation
    Vg = torch.empty_like(d["V"])
    G.gsa_value_gate(G.shape_of(wl), d["V"], d["g2"], Vg)
    T.check_out(T.gpu_attention(wl, d, di, dn, k_cap, use_g2=False, V=Vg, tuning=tuning), full, dtype)
    # a row range leaves the other rows alone
    if Lq > 8:
        part = T.gpu_attention(wl, d, di, dn, k_cap, row_begin=3, row_end=Lq - 2, tuning=tuning)
        assert torch.isnan(part[:, :3]).all() and torch.isnan(part[:, Lq - 2:]).all()
        T.check_out(part[:, 3:Lq - 2], full[:, 3:Lq - 2], dtype)


DENSE_CASES = [
    # H, Hkv, dh, B, Lq, Lk, off
    (16, 4, 128, 2, 300, 300, 0),
    (16, 16, 128, 1, 200, 200, 0),      # one head per kv head
    (16, 1, 128, 1, 130, 130, 0),       # sixteen heads share one kv head
    (12, 4, 64, 1, 150, 150, 0),        # a group of three heads (padded to four columns)
    (8, 2, 64, 2, 100, 500, 400),       # a chunk of queries after a context
    (16, 4, 128, 3, 1, 700, 699),       # decode shape
]


@pytest.mark.parametrize("H,Hkv,dh,B,Lq,Lk,off", DENSE_CASES)
def test_dense_causal_gated_attention(H, Hkv, dh, B, Lq, Lk, off):
    """The comparison variants (Sec. 2.1 Eq. 2; Sec. 7.1 "gated only" and "standard"): every visible key."""
    wl = wl_("dense", B, Lq, Lk, off, H, Hkv, dh, 4, 32, "bf16", seed=60 + H + Hkv, gate_std=1.5)
    t = S.make_inputs(wl, "cpu")
    d = T.to_device(t)
    o = T.oracle_inputs(t)
    sh = G.shape_of(wl)

    def gpu(use_g2, use_g1, scale=0.0, rows=(0, Lq)):
        out = torch.full_like(d["Q"], float("nan"))
        ws = G.workspace(G.gsa_dense_attn_workspace_bytes(sh, use_g2))
        ws.fill_(0xFF)
        G.gsa_dense_gated_attn(sh, rows[0], rows[1], d["Q"], d["K"], d["V"], d["g2"] if use_g2 else None,
                               d["g1"] if use_g1 else None, scale, out, ws)
        torch.cuda.synchronize()
        return out

    def ref(use_g2, use_g1, scale=None):
        out = np.zeros((B, Lq, H, dh))
        for b in range(B):
            for i in range(Lq):
                n = O.n_visible(i, off, Lk)
                out[b, i], _ = O.sparse_gated_attn_row(o["Q"][b, i], o["K"][b], o["V"][b], o["g2"][b] if use_g2 else None,
                                                       o["g1"][b, i] if use_g1 else None, np.arange(n), scale)
        return out

    full = ref(True, True)
    T.check_out(gpu(True, True), full, "bf16")
    T.check_out(gpu(False, False, 0.15), ref(False, False, 0.15), "bf16")
    T.check_out(gpu(True, False), ref(True, False), "bf16")
    if Lq > 8:
        part = gpu(True, True, rows=(3, Lq - 2))
        assert torch.isnan(part[:, :3]).all() and torch.isnan(part[:, Lq - 2:]).all()
        T.check_out(part[:, 3:Lq - 2], full[:, 3:Lq - 2], "bf16")
    if Lq * Lk <= 45000:     # the brute-force statement of Eq. 2 itself, where it is affordable
        brute = O.dense_causal_gated_attn(o["Q"], o["K"], o["V"], o["g1"], o["g2"], off)
        T.check_out(gpu(True, True), brute, "bf16")


def test_sparse_path_with_full_budget_equals_dense_kernel():
    """k_t >= number of visible keys: the sparse forward and the dense kernel compute the same thing."""
    wl = wl_("full", 2, 400, 400, 0, 16, 4, 128, 4, 64, "bf16", kmin=400, kmax=400, kbase=400, seed=8)
    t = S.make_inputs(wl, "cpu")
    d = T.to_device(t)
    res = T.gpu_forward(wl, d, G.make_adaptive(1.0, 1, 1, 1, k_fixed=400), k_cap=400)
    sh = G.shape_of(wl)
    out = torch.empty_like(d["Q"])
    ws = G.workspace(G.gsa_dense_attn_workspace_bytes(sh, True))
    G.gsa_dense_gated_attn(sh, 0, 400, d["Q"], d["K"], d["V"], d["g2"], d["g1"], 0.0, out, ws)
    torch.cuda.synchronize()
    assert (out.float() - res["out"].float()).abs().max().item() <= 1e-2


def test_forward_dense_fallback_below_a_context_length():
    """Sec. 8: below a few thousand tokens the indexer costs more than it saves; gsa_adaptive.dense_below makes
    gsa_forward attend every visible key for such contexts (the dense kernel), and changes nothing above it."""
    wl = wl_("fallback", 2, 900, 900, 0, 16, 4, 128, 4, 64, "bf16", kmin=32, kmax=128, seed=17)
    t = S.make_inputs(wl, "cpu")
    d = T.to_device(t)
    sh = G.shape_of(wl)
    ws = G.workspace(G.gsa_forward_workspace_bytes(sh, 128, True, 900))

    def fwd(ctl, want_aux):
        out = torch.full_like(d["Q"], float("nan"))
        aux = [torch.empty((2, 900), dtype=torch.int32, device="cuda") for _ in range(2)] if want_aux else [None, None]
        G.gsa_forward(sh, ctl, d["Q"], d["K"], d["V"], d["g1"], d["g2"], d["qI"], d["kI"], d["w"], None, 0.0, out, None, aux[0],
                      aux[1], None, 128, ws)
        torch.cuda.synchronize()
        return out

    sparse = fwd(G.make_adaptive(0.3, 64, 32, 128), True)
    assert torch.equal(fwd(G.make_adaptive(0.3, 64, 32, 128, dense_below=900), True), sparse), "Lk == dense_below: still sparse"
    dense = fwd(G.make_adaptive(0.3, 64, 32, 128, dense_below=901), False)
    ref = torch.empty_like(d["Q"])
    G.gsa_dense_gated_attn(sh, 0, 900, d["Q"], d["K"], d["V"], d["g2"], d["g1"], 0.0, ref, ws)
    torch.cuda.synchronize()
    assert torch.equal(dense, ref)
    assert (dense.float() - sparse.float()).abs().max().item() > 1e-2, "the two paths really differ at this budget"
    o = T.oracle_inputs(t)
    for (b, i) in [(0, 0), (1, 899), (0, 450)]:
        want, _ = O.sparse_gated_attn_row(o["Q"][b, i], o["K"][b], o["V"][b], o["g2"][b], o["g1"][b, i], np.arange(i + 1))
        T.check_out(dense[b, i], want, "bf16")
    with pytest.raises(G.GsaError) as ei:      # the fallback produces no index sets
        fwd(G.make_adaptive(0.3, 64, 32, 128, dense_below=901), True)
    assert ei.value.status == G.GSA_ERR_SHAPE


def test_attention_gate_limits_on_gpu():
    """Saturated gate logits: +40 makes both sigmoids 1 in fp32 (plain SDPA on the set), -40 kills the output."""
    wl = wl_("attlim", 1, 64, 64, 0, 8, 2, 128, 4, 32, "bf16", seed=9)
    t = S.make_inputs(wl, "cpu")
    r = np.random.default_rng(1)
    idx, n_sel = _random_sets(r, wl, 48)
    d = T.to_device(t)
    di, dn = torch.from_numpy(idx).cuda(), torch.from_numpy(n_sel).cuda()
    plain = T.gpu_attention(wl, d, di, dn, 48, use_g2=False, use_g1=False)
    d["g1"].fill_(40.0)
    d["g2"].fill_(40.0)
    assert torch.equal(T.gpu_attention(wl, d, di, dn, 48), plain)
    d["g1"].fill_(-40.0)
    assert T.gpu_attention(wl, d, di, dn, 48).abs().max().item() <= 1e-15
    d["g1"].fill_(0.0)
    d["g2"].fill_(0.0)
    quarter = T.gpu_attention(wl, d, di, dn, 48).float()
    assert (quarter - 0.25 * plain.float()).abs().max().item() <= 2e-2


# ------------------------------------------------------------------------------------ whole path
def _check_forward(wl, t, res, ctl_kw, rows=None, k_cap=None):
    """Stage-wise validation of a forward result against the fp64 oracle on rows (b, i)."""
    o = T.oracle_inputs(t)
    k_cap = wl.k_cap if k_cap is None else k_cap
    idx = res["idx"].cpu().numpy()
    n_sel = res["n_sel"].cpu().numpy()
    kk = res["k"].cpu().numpy()
    var = res["var"].cpu().numpy()
    out = T.to64(res["out"])
    rows = [(b, i) for b in range(wl.B) for i in range(wl.Lq)] if rows is None else rows
    excused = kband = 0
    worst = 0.0
    for (b, i) in rows:
        n = O.n_visible(i, wl.q_offset, wl.Lk)
        I = O.indexer_scores_row(o["qI"][b, i], o["kI"][b, :n], o["w"][b, i], o["bI"], wl.indexer_act)
        _, v64 = O.row_stats(I)
        assert abs(var[b, i] - v64) <= (2e-5 if wl.indexer_act == "sigmoid" else 2e-4) * v64 + 5e-8
        kband += T.k_band_ok(kk[b, i:i + 1], np.array([v64]), ctl_kw)
        assert n_sel[b, i] == min(kk[b, i], n)
        T.check_index_row_wellformed(idx[b, i], n_sel[b, i], n, k_cap)
        excused += T.check_selection_vs_fp64(idx[b, i], int(n_sel[b, i]), I)
        ref, _ = O.sparse_gated_attn_row(o["Q"][b, i], o["K"][b], o["V"][b], o["g2"][b], o["g1"][b, i], idx[b, i, :n_sel[b, i]])
        worst = max(worst, T.check_out(out[b, i], ref, wl.dtype))
    return excused, kband, worst


def _ctl_for(wl, vbar):
    kw = dict(vbar=float(np.float32(vbar)), k_base=wl.k_base, k_min=wl.k_min, k_max=wl.k_max, k_fixed=wl.k_fixed, mode=0)
    return G.make_adaptive(kw["vbar"], wl.k_base, wl.k_min, wl.k_max, wl.k_fixed, 0), kw


def _vbar_from_gpu(wl, d):
    _, _, var = T.gpu_indexer(wl, d, want_scores=False, want_mean=False)
    return float(var.double().mean().item())


@pytest.mark.parametrize("wl", [S.C1_FIXED, S.C1], ids=lambda w: w.name)
def test_forward_tiny_fp32_configs(wl):
    t = S.make_inputs(wl, "cpu")
    d = T.to_device(t)
    ctl, kw = _ctl_for(wl, _vbar_from_gpu(wl, d))
    res = T.gpu_forward(wl, d, ctl)
    excused, kband, worst = _check_forward(wl, t, res, kw)
    assert excused <= 4 and kband <= 8
    if wl.k_fixed == 0:
        kk = res["k"].cpu().numpy()
        assert kk.min() >= wl.k_min and kk.max() <= wl.k_max and len(np.unique(kk)) > 10
    # end to end against the oracle's own selection wherever the sets agree (they do except inside the band)
    o = T.oracle_inputs(t)
    full = O.gsa_forward(o["Q"], o["K"], o["V"], o["g1"], o["g2"], o["qI"], o["kI"], o["w"], None, 0, kw, k_cap=wl.k_cap)
    same = np.all(full["idx"] == res["idx"].cpu().numpy(), axis=-1)
    assert same.mean() > 0.97
    T.check_out(T.to64(res["out"])[same], full["out"][same], wl.dtype)


@pytest.mark.parametrize("heavy", [False, True])
def test_forward_bf16_mid_size(heavy):
    wl = wl_("mid", 2, 1536, 1536, 0, 16, 4, 128, 4, 64, "bf16", kmin=64, kmax=256, seed=77, gate_std=2.0,
             heavy_frac=0.05 if heavy else 0.0, heavy_scale=4.0 if heavy else 1.0)
    t = S.make_inputs(wl, "cpu")
    d = T.to_device(t)
    ctl, kw = _ctl_for(wl, _vbar_from_gpu(wl, d))
    res = T.gpu_forward(wl, d, ctl)
    r = np.random.default_rng(2)
    rows = [(int(b), int(i)) for b, i in zip(r.integers(0, 2, 60), r.integers(0, 1536, 60))] + [(0, 0), (1, 1535), (0, 63), (1, 64)]
    excused, kband, worst = _check_forward(wl, t, res, kw, rows)
    assert excused <= 6 and kband <= 3
    kk = res["k"].cpu().numpy()
    assert len(np.unique(kk)) > 20
    # slabbed execution (several slabs, split key ranges) selects the same sets wherever k_t agrees
    res2 = T.gpu_forward(wl, d, ctl, slab_rows=128)
    same_k = (res2["k"] == res["k"])
    assert same_k.float().mean().item() > 0.995
    assert torch.equal(res2["idx"][same_k], res["idx"][same_k])
    # (small slabs cut each selected list into pieces: probabilities are rounded to bf16 against another running maximum)
    assert (res2["out"][same_k].float() - res["out"][same_k].float()).abs().max().item() <= 1e-2
    # no index output requested: same result
    res3 = T.gpu_forward(wl, d, ctl, want_idx=False)
    assert torch.equal(res3["out"], res["out"]) and torch.equal(res3["n_sel"], res["n_sel"])
    # determinism
    res4 = T.gpu_forward(wl, d, ctl)
    assert torch.equal(res4["out"], res["out"]) and torch.equal(res4["idx"], res["idx"]) and torch.equal(res4["var"], res["var"])


@pytest.mark.parametrize("Lq,Lk,off", [(1100, 1100, 0), (300, 1000, 700)], ids=["prefill", "chunk-after-context"])
def test_forward_key_windows_match_single_launch(Lq, Lk, off):
    """Attention by key windows (forced here; chosen automatically for long prefills) against the single-launch
    attention of the same forward, and against the oracle on sampled rows."""
    wl = wl_("win", 2, Lq, Lk, off, 16, 4, 128, 4, 64, "bf16", kmin=48, kmax=200, seed=78, gate_std=2.0)
    t = S.make_inputs(wl, "cpu")
    d = T.to_device(t)
    ctl, kw = _ctl_for(wl, _vbar_from_gpu(wl, d))
    one = T.gpu_forward(wl, d, ctl, tuning=G.make_tuning(attn_window=-1))
    for window in (96, 256, 1024):
        tn = G.make_tuning(attn_window=window, attn_rows_per_wave=window // 90)
        res = T.gpu_forward(wl, d, ctl, tuning=tn)
        assert torch.equal(res["idx"], one["idx"]) and torch.equal(res["n_sel"], one["n_sel"])
        assert (res["out"].float() - one["out"].float()).abs().max().item() <= 1e-2
        r = np.random.default_rng(window)
        rows = [(int(b), int(i)) for b, i in zip(r.integers(0, 2, 24), r.integers(0, Lq, 24))]
        rows += [(0, 0), (1, Lq - 1), (0, min(Lq - 1, max(0, window - 1 - off))), (1, min(Lq - 1, max(0, window - off)))]
        _check_forward(wl, t, res, kw, rows)
        # slabs whose first row lies beyond the first windows
        res2 = T.gpu_forward(wl, d, ctl, slab_rows=128 if Lq < 512 else 384, tuning=tn)
        same_k = (res2["k"] == res["k"])
        assert same_k.float().mean().item() > 0.995
        assert (res2["out"][same_k].float() - res["out"][same_k].float()).abs().max().item() <= 1e-2


def test_forward_decode_shape_equals_prefill_last_row():
    """Lq = 1 with q_offset = Lk-1 is the last row of the prefill (same kernels, different launch shape)."""
    wl = wl_("pre", 3, 640, 640, 0, 16, 4, 128, 4, 64, "bf16", kmin=32, kmax=128, seed=5)
    t = S.make_inputs(wl, "cpu")
    d = T.to_device(t)
    ctl, kw = _ctl_for(wl, 0.3)
    pre = T.gpu_forward(wl, d, ctl)
    wd = wl.with_(Lq=1, q_offset=639)
    dd = dict(d)
    for name in ("Q", "g1", "qI", "w"):
        dd[name] = d[name][:, 639:].contiguous()
    dec = T.gpu_forward(wd, dd, ctl)
    same_k = dec["k"][:, 0] == pre["k"][:, 639]          # the two launches sum the variance in different orders
    assert same_k.sum().item() >= 2
    assert torch.equal(dec["idx"][:, 0][same_k], pre["idx"][:, 639][same_k])
    # the decode launch cuts each selected list into pieces and merges them: same values up to rounding
    assert (dec["out"][:, 0][same_k].float() - pre["out"][:, 639][same_k].float()).abs().max().item() <= 1e-2
    td = {k: (v[:, 639:] if k in ("Q", "g1", "qI", "w") else v) for k, v in t.items()}
    _check_forward(wd, td, dec, kw)


def test_forward_constant_and_saturated_rows_take_lowest_indices():
    """Degenerate score rows inside the fused forward: q^I = 0 makes every score of a row equal (one 16-bit
    key, thousands of exact fp32 ties), huge logits saturate every sigmoid (a handful of distinct values).
    The selection must still be the oracle's: ties resolved towards the lowest index."""
    wl = wl_("ties", 1, 20000, 20000, 0, 16, 4, 128, 4, 64, "bf16", kmin=40, kmax=2100, kbase=300, seed=21)
    t = S.make_inputs(wl, "cpu")
    t["qI"][:, ::2] = 0                      # even rows: constant scores
    t["qI"][:, 1::2] *= 16                   # odd rows: saturated sigmoids
    d = T.to_device(t)
    ctl = G.make_adaptive(1.0, 1, 1, 1, k_fixed=2100)
    res = T.gpu_forward(wl, d, ctl, k_cap=2100)
    idx = res["idx"].cpu().numpy()
    n_sel = res["n_sel"].cpu().numpy()
    o = T.oracle_inputs(t)
    for i in (0, 5, 2098, 2099, 2100, 2101, 4444, 17001, 19998, 19999):
        n = i + 1
        m = min(2100, n)
        assert n_sel[0, i] == m
        T.check_index_row_wellformed(idx[0, i], m, n, 2100)
        I = O.indexer_scores_row(o["qI"][0, i], o["kI"][0, :n], o["w"][0, i], None)
        if i % 2 == 0:
            assert np.array_equal(idx[0, i, :m], np.arange(m)), "constant row %d" % i
        T.check_selection_vs_fp64(idx[0, i], m, I)
    assert torch.isfinite(res["out"].float()).all()


def test_forward_matches_staged_calls():
    """gsa_forward (16-bit keys between indexer and selection) against the four stage calls chained by hand
    (fp32 scores): identical sets except where two fp32 scores are within rounding of each other."""
    wl = wl_("staged", 1, 3000, 3000, 0, 16, 4, 128, 4, 64, "bf16", kmin=64, kmax=512, seed=31)
    t = S.make_inputs(wl, "cpu")
    d = T.to_device(t)
    ctl, kw = _ctl_for(wl, _vbar_from_gpu(wl, d))
    res = T.gpu_forward(wl, d, ctl)
    scores, _, var = T.gpu_indexer(wl, d, want_mean=False)
    k, n_sel = T.gpu_adaptive_k(wl, ctl, var)
    idx = T.gpu_select(wl, scores, n_sel, wl.k_cap)
    out = T.gpu_attention(wl, d, idx, n_sel, wl.k_cap)
    assert torch.equal(res["var"], var) and torch.equal(res["k"], k) and torch.equal(res["n_sel"], n_sel)
    same = (res["idx"] == idx).all(-1)
    assert same.float().mean().item() >= 0.995
    assert torch.equal(res["out"][same], out[same])
    sc = T.to64(scores)
    for (b, i) in (~same).nonzero().tolist():          # differing rows: only elements tied within fp32 rounding
        m = int(n_sel[b, i])
        a_, b_ = set(res["idx"][b, i, :m].tolist()), set(idx[b, i, :m].tolist())
        diff = np.array(sorted(a_ ^ b_))
        thr = np.sort(sc[b, i, :i + 1])[i + 1 - m]
        assert np.all(np.abs(sc[b, i, diff] - thr) <= 4e-7 * thr)


FORWARD_VARIANTS = [
    # dtype, HI, dI, H, Hkv, dh, B, Lq, Lk, off, bias, slab_rows, largest number of in-band substitutions over the 42 rows
    ("f32", 2, 128, 8, 8, 64, 2, 700, 700, 0, False, 256, 4),
    ("bf16", 8, 32, 16, 2, 64, 1, 900, 900, 0, True, None, 4),
    ("bf16", 1, 128, 4, 1, 128, 3, 500, 500, 0, True, 128, 300),    # 192 observed
    ("bf16", 4, 64, 16, 4, 128, 2, 300, 1000, 700, False, None, 4),   # a chunk of queries against a longer cache
    ("f32", 4, 32, 4, 2, 128, 1, 1, 600, 599, False, None, 4),        # single-query decode in fp32
    ("bf16", 3, 64, 16, 4, 128, 1, 700, 700, 0, True, None, 4),       # head counts that need padding
    ("bf16", 7, 32, 8, 2, 64, 2, 400, 400, 0, False, 128, 4),
    ("f32", 5, 64, 4, 4, 64, 1, 300, 300, 0, True, None, 4),
    ("bf16", 6, 64, 4, 1, 128, 1, 1, 800, 799, True, None, 4),
]


@pytest.mark.parametrize("dtype,HI,dI,H,Hkv,dh,B,Lq,Lk,off,bias,slab,max_excused", FORWARD_VARIANTS)
def test_forward_shape_variants(dtype, HI, dI, H, Hkv, dh, B, Lq, Lk, off, bias, slab, max_excused):
    wl = wl_("var", B, Lq, Lk, off, H, Hkv, dh, HI, dI, dtype, kmin=16, kmax=96, seed=100 + HI + dI + H)
    t = S.make_inputs(wl, "cpu", with_bias=bias)
    d = T.to_device(t)
    ctl, kw = _ctl_for(wl, _vbar_from_gpu(wl, d))
    res = T.gpu_forward(wl, d, ctl, slab_rows=slab)
    r = np.random.default_rng(9)
    rows = sorted({(int(b), int(i)) for b, i in zip(r.integers(0, B, 40), r.integers(0, Lq, 40))} | {(0, 0), (B - 1, Lq - 1)})
    # (with one or two indexer heads and d^I = 128 most sigmoids saturate: many fp64 scores differ only beyond
    # fp32 resolution, so those cases are allowed more in-band substitutions than the others)
    excused, kband, worst = _check_forward(wl, t, res, kw, rows)
    print("in-band substitutions: %d (bound %d), k_t band: %d" % (excused, max_excused, kband))
    assert kband <= 3 and excused <= max_excused


@pytest.mark.parametrize("L", [1, 2, 5, 33, 129])
def test_forward_tiny_lengths(L):
    """Lengths below one tile of every kernel, budgets smaller and larger than the row."""
    wl = wl_("tiny", 2, L, L, 0, 8, 2, 64, 4, 32, "bf16", kmin=2, kmax=7, kbase=4, seed=L)
    t = S.make_inputs(wl, "cpu")
    d = T.to_device(t)
    ctl, kw = _ctl_for(wl, 0.05)
    res = T.gpu_forward(wl, d, ctl)
    _check_forward(wl, t, res, kw)


def test_select_budget_up_to_8192():
    """The largest supported k_cap on 128K-long rows: the one-pass list overflows and the exact path takes over."""
    r = np.random.default_rng(5)
    B, Lq, Lk, k_cap = 1, 4, 131072, 8192
    sc = r.uniform(0, 4, (B, Lq, Lk)).astype(np.float32)
    _select_case(sc, np.array([[8192, 8191, 5000, 4097]]), k_cap, Lk - Lq)


def test_forward_head_weights_above_one():
    """Head weights above 1 (outside what Sec. 3.3 produces, allowed by the interface): scores above the range
    of the 16-bit keys saturate them, and the saturated elements are ordered by their recomputed fp32 scores."""
    wl = wl_("bigw", 1, 2500, 2500, 0, 16, 4, 128, 4, 64, "bf16", kmin=32, kmax=300, seed=41)
    t = S.make_inputs(wl, "cpu")
    t["w"] = (t["w"] * 3.0).contiguous()
    d = T.to_device(t)
    ctl, kw = _ctl_for(wl, _vbar_from_gpu(wl, d))
    res = T.gpu_forward(wl, d, ctl)
    r = np.random.default_rng(3)
    rows = [(0, int(i)) for i in r.integers(0, 2500, 40)] + [(0, 0), (0, 2499)]
    excused, kband, worst = _check_forward(wl, t, res, kw, rows)
    assert excused <= 6 and kband <= 3
    assert len(np.unique(res["k"].cpu().numpy())) > 20


def _random_case(r):
    dtype = ["bf16", "f32"][int(r.integers(0, 2))]
    HI = int(r.choice([1, 2, 3, 4, 5, 6, 7, 8]))
    dI = int(r.choice([32, 64, 128]))
    dh = int(r.choice([64, 128]))
    Hkv = int(r.choice([1, 2, 4, 8]))
    G_ = int(r.choice([1, 2, 4, 16]))
    B = int(r.integers(1, 4))
    Lk = int(r.integers(3, 900))
    Lq = int(r.integers(1, Lk + 1))
    off = int(r.integers(0, Lk - Lq + 1))
    kmin = int(r.integers(1, 40))
    kmax = kmin + int(r.integers(0, 120))
    slab = [None, 128, 256][int(r.integers(0, 3))]
    return dtype, HI, dI, Hkv * G_, Hkv, dh, B, Lq, Lk, off, bool(r.integers(0, 2)), slab, kmin, kmax


@pytest.mark.parametrize("case", range(48))
def test_forward_random_shapes(case):
    """Seeded random shapes (all supported head counts and dimensions, ragged lengths, offsets, slabs)."""
    r = np.random.default_rng(1000 + case)
    dtype, HI, dI, H, Hkv, dh, B, Lq, Lk, off, bias, slab, kmin, kmax = _random_case(r)
    wl = wl_("rnd", B, Lq, Lk, off, H, Hkv, dh, HI, dI, dtype, kmin=kmin, kmax=kmax, seed=2000 + case)
    t = S.make_inputs(wl, "cpu", with_bias=bias)
    d = T.to_device(t)
    ctl, kw = _ctl_for(wl, _vbar_from_gpu(wl, d) + 1e-6)
    # odd cases: the selection on keys runs one wave per row however few rows there are
    res = T.gpu_forward(wl, d, ctl, slab_rows=slab, tuning=G.make_tuning(select_wave_min_rows=case % 2))
    rows = {(int(b), int(i)) for b, i in zip(r.integers(0, B, 12), r.integers(0, Lq, 12))} | {(0, 0), (B - 1, Lq - 1)}
    _check_forward(wl, t, res, kw, sorted(rows))


@pytest.mark.parametrize("case", range(24))
def test_forward_random_shapes_key_windows(case):
    """The same kind of random shapes (bf16 only) with the attention forced into key windows of a random size."""
    r = np.random.default_rng(5000 + case)
    _, HI, dI, H, Hkv, dh, B, Lq, Lk, off, bias, slab, kmin, kmax = _random_case(r)
    window = int(r.integers(8, 300))
    tn = G.make_tuning(attn_window=window, attn_rows_per_wave=int(r.integers(1, 10)), select_wave_min_rows=(case + 1) % 2)
    wl = wl_("rndw", B, Lq, Lk, off, H, Hkv, dh, HI, dI, "bf16", kmin=kmin, kmax=kmax, seed=6000 + case)
    t = S.make_inputs(wl, "cpu", with_bias=bias)
    d = T.to_device(t)
    ctl, kw = _ctl_for(wl, _vbar_from_gpu(wl, d) + 1e-6)
    res = T.gpu_forward(wl, d, ctl, slab_rows=slab, tuning=tn)
    rows = {(int(b), int(i)) for b, i in zip(r.integers(0, B, 12), r.integers(0, Lq, 12))} | {(0, 0), (B - 1, Lq - 1)}
    _check_forward(wl, t, res, kw, sorted(rows))


def test_gather_probes_return_the_xor_of_the_rows_they_read():
    """The two measurement helpers (plain whole-row gather, and the same rows staged through LDS) against the plain
    definition of what they leave in `sink`: wave v XORs every 32-bit word of the rows idx[c*64 .. c*64+64), c = v, v + waves, ..."""
    rows, n_idx, waves = 4096, 64 * 300, 64
    g = torch.Generator().manual_seed(5)
    table = torch.randint(-2**31, 2**31 - 1, (rows, 64), dtype=torch.int32, generator=g)
    idx = torch.randint(0, rows, (n_idx,), dtype=torch.int32, generator=g)
    row_x = np.bitwise_xor.reduce(table.numpy().view(np.uint32), axis=1)
    per_chunk = np.bitwise_xor.reduce(row_x[idx.numpy().reshape(-1, 64)], axis=1)
    want = np.zeros(waves, np.uint32)
    for c, x in enumerate(per_chunk):
        want[c % waves] ^= x
    for fn in (G.gsa_probe_gather, G.gsa_probe_gather_staged):
        sink = torch.zeros(waves, dtype=torch.int32, device="cuda")
        fn(table.cuda(), rows, idx.cuda(), n_idx, waves, sink)
        torch.cuda.synchronize()
        assert np.array_equal(sink.cpu().numpy().view(np.uint32), want), fn.__name__
