"""Decode-serving state: append-only caches with gated values, and decode steps over a batch of sequences of
different lengths (the "Decode" column of Table 9 is the only place the paper touches it), against the fp64 oracle."""
import numpy as np
import pytest
import torch

import paper_2601_15305_amd as G
from paper_2601_15305_amd import synthetic as S
from oracle import gsa_oracle as O

import gsa_testlib as T

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype,Hkv,dh,dI", [("bf16", 4, 128, 64), ("f32", 2, 64, 32), ("bf16", 1, 64, 128)])
def test_cache_append_writes_gated_values_at_each_sequences_end(dtype, Hkv, dh, dI):
    B, T_, cap = 4, 3, 50
    wl = S.Workload("append", B, T_, cap, 0, 4 * Hkv, Hkv, dh, 4, dI, dtype, 8, 4, 16, seed=5)
    t = S.make_inputs(wl.with_(Lk=T_), "cuda")           # K, V, g2, kI of the T new tokens
    sh = G.shape_of(wl)
    dt = S.torch_dtype(dtype)
    lens = torch.tensor([0, 17, cap - 1, cap - 3], dtype=torch.int32, device="cuda")
    caches = [torch.full((B, cap, dI), 7.0, dtype=dt, device="cuda"), torch.full((B, cap, Hkv, dh), 7.0, dtype=dt, device="cuda"),
              torch.full((B, cap, Hkv, dh), 7.0, dtype=dt, device="cuda")]
    lens_out = torch.full((B,), -1, dtype=torch.int32, device="cuda")
    G.gsa_cache_append(sh, t["kI"], t["K"], t["V"], t["g2"], lens, caches[0], caches[1], caches[2], lens_out)
    torch.cuda.synchronize()
    assert lens_out.tolist() == [3, 20, cap, cap]
    Vg = torch.empty_like(t["V"])
    G.gsa_value_gate(G.shape_of(wl.with_(Lk=T_)), t["V"], t["g2"], Vg)      # the same rounding as the pre-pass
    ref = T.to64(t["V"]) * O.sigmoid(T.to64(t["g2"]))
    assert np.abs(T.to64(Vg) - ref).max() <= (2e-2 if dtype == "bf16" else 1e-6)
    for b, l0 in enumerate(lens.tolist()):
        fit = min(T_, cap - l0)
        assert torch.equal(caches[0][b, l0:l0 + fit], t["kI"][b, :fit])
        assert torch.equal(caches[1][b, l0:l0 + fit], t["K"][b, :fit])
        assert torch.equal(caches[2][b, l0:l0 + fit], Vg[b, :fit])
        for c in caches:      # everything else is untouched
            assert (c[b, :l0] == 7.0).all() and (c[b, l0 + fit:] == 7.0).all()
    with pytest.raises(G.GsaError):
        G.gsa_cache_append(sh, t["kI"], t["K"], t["V"], t["g2"], lens, caches[0], caches[1], caches[2], lens)


@pytest.mark.parametrize("wave", [0, 1])
@pytest.mark.parametrize("Lq", [1, 3])
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_decode_step_over_ragged_batch(dtype, Lq, wave):
    """Sequences of different lengths in one batch; the cache beyond a sequence's length holds NaN and must never
    reach a result.  wave = 1: the selection runs its wave-per-row kernel even on this small batch."""
    tn = G.make_tuning(select_wave_min_rows=wave)
    B, cap = 6, 2600
    lens = [Lq, 37, 300, 2600, 1024, 2599]
    wl = S.Workload("ragged", B, Lq, cap, 0, 16 if dtype == "bf16" else 4, 4 if dtype == "bf16" else 2, 128 if dtype == "bf16" else 64,
                    4, 64, dtype, 45, 16, 128, seed=23)
    t = S.make_inputs(wl, "cuda")
    sh = G.shape_of(wl)
    Vg = torch.empty_like(t["V"])
    G.gsa_value_gate(sh, t["V"], t["g2"], Vg)
    kI_c, K_c, Vg_c = t["kI"].clone(), t["K"].clone(), Vg
    for b, l in enumerate(lens):
        kI_c[b, l:] = float("nan")
        K_c[b, l:] = float("nan")
        Vg_c[b, l:] = float("nan")
    seq_lens = torch.tensor(lens, dtype=torch.int32, device="cuda")
    ctl_kw = dict(vbar=0.3, k_base=45, k_min=16, k_max=128, k_fixed=0, mode=0)
    ctl = G.make_adaptive(0.3, 45, 16, 128)
    out = torch.full_like(t["Q"], float("nan"))
    idx = torch.full((B, Lq, 128), -7, dtype=torch.int32, device="cuda")
    n_sel = torch.empty((B, Lq), dtype=torch.int32, device="cuda")
    k = torch.empty_like(n_sel)
    var = torch.empty((B, Lq), dtype=torch.float32, device="cuda")
    ws = G.workspace(G.gsa_decode_workspace_bytes(sh, 128))
    ws.fill_(0xFF)
    G.gsa_decode_step(sh, ctl, t["Q"], t["g1"], t["qI"], t["w"], None, kI_c, K_c, Vg_c, seq_lens, 0.0, out, idx, n_sel, k, var, 128, ws,
                      tuning=tn)
    torch.cuda.synchronize()
    assert torch.isfinite(out.float()).all(), "nothing beyond a sequence's length may be read"
    o = {name: T.to64(v) for name, v in t.items()}
    idx_h, n_h, k_h, var_h, out_h = idx.cpu().numpy(), n_sel.cpu().numpy(), k.cpu().numpy(), var.cpu().numpy(), T.to64(out)
    excused = 0
    for b, l in enumerate(lens):
        for i in range(Lq):
            n = l - Lq + i + 1
            I = O.indexer_scores_row(o["qI"][b, i], o["kI"][b, :n], o["w"][b, i], None)
            _, v64 = O.row_stats(I)
            assert abs(var_h[b, i] - v64) <= 2e-5 * v64 + 5e-8
            T.k_band_ok(k_h[b, i:i + 1], np.array([v64]), ctl_kw)
            assert n_h[b, i] == min(k_h[b, i], n)
            T.check_index_row_wellformed(idx_h[b, i], n_h[b, i], n, 128)
            excused += T.check_selection_vs_fp64(idx_h[b, i], int(n_h[b, i]), I)
            ref, _ = O.sparse_gated_attn_row(o["Q"][b, i], o["K"][b], o["V"][b], o["g2"][b], o["g1"][b, i], idx_h[b, i, :n_h[b, i]])
            T.check_out(out_h[b, i], ref, dtype)
    assert excused <= 3
    # a batch whose sequences all have the same length is the plain forward with that offset
    same = torch.full((B,), 1500, dtype=torch.int32, device="cuda")
    out2 = torch.empty_like(out)
    Vg_full = torch.empty_like(t["V"])
    G.gsa_value_gate(sh, t["V"], t["g2"], Vg_full)
    G.gsa_decode_step(sh, ctl, t["Q"], t["g1"], t["qI"], t["w"], None, t["kI"], t["K"], Vg_full, same, 0.0, out2, None, None, None,
                      None, 128, ws, tuning=tn)
    wl2 = wl.with_(Lk=1500, q_offset=1500 - Lq)
    t2 = dict(t)
    for name in ("K", "V", "g2", "kI"):
        t2[name] = t[name][:, :1500].contiguous()
    res = T.gpu_forward(wl2, t2, ctl, k_cap=128, tuning=tn)
    torch.cuda.synchronize()
    assert torch.equal(out2, res["out"])



def test_decode_step_replays_from_a_hip_graph():
    """gsa_decode_step launches kernels only (no allocation, no memset, no synchronisation), so a serving loop can
    capture it once and replay it.  Every replay, with fresh inputs written by eager work in between, must give the
    bits of the eager call on the same inputs."""
    B, cap, Lq, k_cap = 8, 3000, 1, 128
    wl = S.Workload("graph", B, Lq, cap, 0, 16, 4, 128, 4, 64, "bf16", 45, 16, 128, seed=29)
    t = S.make_inputs(wl, "cuda")
    sh = G.shape_of(wl)
    Vg = torch.empty_like(t["V"])
    G.gsa_value_gate(sh, t["V"], t["g2"], Vg)
    seq_lens = torch.tensor([3000, 17, 2999, 1500, 64, 2048, 1, 777], dtype=torch.int32, device="cuda")
    ctl = G.make_adaptive(0.3, 45, 16, 128)
    Q, qI, w = t["Q"].clone(), t["qI"].clone(), t["w"].clone()
    bufs = [dict(out=torch.empty_like(Q), idx=torch.empty((B, Lq, k_cap), dtype=torch.int32, device="cuda"),
                 n=torch.empty((B, Lq), dtype=torch.int32, device="cuda"), k=torch.empty((B, Lq), dtype=torch.int32, device="cuda"),
                 var=torch.empty((B, Lq), dtype=torch.float32, device="cuda")) for _ in range(2)]
    ws = G.workspace(G.gsa_decode_workspace_bytes(sh, k_cap))

    def step(o):
        G.gsa_decode_step(sh, ctl, Q, t["g1"], qI, w, None, t["kI"], t["K"], Vg, seq_lens, 0.0, o["out"], o["idx"], o["n"], o["k"],
                          o["var"], k_cap, ws)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step(bufs[0])                       # warm-up outside the capture (kernel attributes, lazy module load)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step(bufs[0])
    gen = torch.Generator(device="cuda").manual_seed(5)
    for rep in range(4):
        # eager work between the replays: new queries, new indexer queries, new lengths
        Q.copy_(torch.randn(Q.shape, generator=gen, device="cuda").to(Q.dtype))
        qI.copy_(torch.randn(qI.shape, generator=gen, device="cuda").to(qI.dtype))
        seq_lens.copy_(torch.randint(1, cap + 1, (B,), generator=gen, device="cuda").to(torch.int32))
        ws.fill_(0xFF)
        graph.replay()
        torch.cuda.synchronize()
        step(bufs[1])
        torch.cuda.synchronize()
        for name in ("out", "idx", "n", "k", "var"):
            assert torch.equal(bufs[0][name], bufs[1][name]), "replay %d differs from the eager call in %s" % (rep, name)


def _paged_copy(lens, cap, page, tensors, seed):
    """Scatter contiguous caches [B, cap, ...] into pools of shuffled pages.  Only the pages a sequence needs exist;
    the other table entries point far outside the pool (they must never be used), unused pool pages hold NaN."""
    B = len(lens)
    max_pages = cap // page
    need = [(l + page - 1) // page for l in lens]
    pool_pages = sum(need) + 5
    g = torch.Generator().manual_seed(seed)
    perm = torch.randperm(pool_pages, generator=g).tolist()
    table = torch.full((B, max_pages), 2 ** 30, dtype=torch.int32)
    pools = [torch.full((pool_pages, page) + tuple(t.shape[2:]), float("nan"), dtype=t.dtype, device=t.device) for t in tensors]
    nxt = 0
    for b in range(B):
        for p in range(need[b]):
            pg = perm[nxt]
            nxt += 1
            table[b, p] = pg
            n = min(page, lens[b] - p * page)
            for pool, t in zip(pools, tensors):
                pool[pg, :n] = t[b, p * page:p * page + n]
    return table.cuda(), pool_pages, pools


@pytest.mark.parametrize("wave", [0, 1])
@pytest.mark.parametrize("dtype,Lq,page", [("bf16", 1, 256), ("bf16", 3, 128), ("f32", 2, 512)])
def test_paged_decode_step_equals_the_contiguous_one(dtype, Lq, page, wave):
    """The same cached rows behind a shuffled block table: every output of the paged call equals the contiguous
    call's bit for bit; pages a sequence does not own hold NaN and the table entries beyond its length point
    outside the pool."""
    B, cap, k_cap = 6, 2560, 128
    lens = [Lq, 37, 300, 2560, 1024, 2559]
    wl = S.Workload("paged", B, Lq, cap, 0, 16 if dtype == "bf16" else 4, 4 if dtype == "bf16" else 2, 128 if dtype == "bf16" else 64,
                    4, 64, dtype, 45, 16, 128, seed=31)
    t = S.make_inputs(wl, "cuda")
    sh = G.shape_of(wl)
    Vg = torch.empty_like(t["V"])
    G.gsa_value_gate(sh, t["V"], t["g2"], Vg)
    seq_lens = torch.tensor(lens, dtype=torch.int32, device="cuda")
    ctl = G.make_adaptive(0.3, 45, 16, 128)
    tn = G.make_tuning(select_wave_min_rows=wave)

    def outputs():
        return dict(out=torch.full_like(t["Q"], float("nan")), idx=torch.full((B, Lq, k_cap), -7, dtype=torch.int32, device="cuda"),
                    n=torch.empty((B, Lq), dtype=torch.int32, device="cuda"), k=torch.empty((B, Lq), dtype=torch.int32, device="cuda"),
                    var=torch.empty((B, Lq), dtype=torch.float32, device="cuda"))
    ref = outputs()
    ws = G.workspace(G.gsa_decode_workspace_bytes(sh, k_cap))
    G.gsa_decode_step(sh, ctl, t["Q"], t["g1"], t["qI"], t["w"], None, t["kI"], t["K"], Vg, seq_lens, 0.0, ref["out"], ref["idx"], ref["n"],
                      ref["k"], ref["var"], k_cap, ws, tuning=tn)
    table, pool_pages, (kI_p, K_p, Vg_p) = _paged_copy(lens, cap, page, [t["kI"], t["K"], Vg], seed=page + Lq)
    got = outputs()
    ws2 = G.workspace(G.gsa_paged_decode_workspace_bytes(sh, k_cap))
    ws2.fill_(0xFF)
    G.gsa_paged_decode_step(sh, ctl, page, table, pool_pages, t["Q"], t["g1"], t["qI"], t["w"], None, kI_p, K_p, Vg_p, seq_lens, 0.0,
                            got["out"], got["idx"], got["n"], got["k"], got["var"], k_cap, ws2, tuning=tn)
    torch.cuda.synchronize()
    assert torch.isfinite(got["out"].float()).all(), "a page outside a sequence was read"
    for name in ("n", "k", "var", "out"):
        assert torch.equal(got[name], ref[name]), name
    valid = torch.arange(k_cap, device="cuda")[None, None, :] < ref["n"][..., None]
    assert torch.equal(got["idx"][valid], ref["idx"][valid])
    # argument errors are decided on the host
    for bad_page in (100, 64, 384):
        with pytest.raises(G.GsaError) as e:
            G.gsa_paged_decode_step(sh, ctl, bad_page, table, pool_pages, t["Q"], t["g1"], t["qI"], t["w"], None, kI_p, K_p, Vg_p, seq_lens,
                                    0.0, got["out"], None, None, None, None, k_cap, ws2)
        assert e.value.status == G.GSA_ERR_SHAPE
    with pytest.raises(G.GsaError) as e:
        G.gsa_paged_decode_step(sh, ctl, page, None, pool_pages, t["Q"], t["g1"], t["qI"], t["w"], None, kI_p, K_p, Vg_p, seq_lens, 0.0,
                                got["out"], None, None, None, None, k_cap, ws2)
    assert e.value.status == G.GSA_ERR_NULL


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_paged_cache_append_fills_the_pages_of_each_sequence(dtype):
    """T new tokens per sequence land at each sequence's own end, in the page the block table names; the pools hold
    exactly what the contiguous caches hold at the same positions."""
    B, cap, page, T_new = 4, 1024, 128, 5
    Hkv, dh, dI = 2, 64, 32
    lens = [0, 126, 500, 1021]        # crossing a page boundary; running into the capacity
    wl = S.Workload("pappend", B, T_new, cap, 0, 4, Hkv, dh, 2, dI, dtype, 8, 4, 16, seed=37)
    t = S.make_inputs(wl, "cuda")
    sh = G.shape_of(wl)
    new = {n: t[n][:, :T_new].contiguous() for n in ("kI", "K", "V", "g2")}
    seq_lens = torch.tensor(lens, dtype=torch.int32, device="cuda")
    dt = t["K"].dtype
    kI_c = torch.zeros((B, cap, dI), dtype=dt, device="cuda")
    K_c = torch.zeros((B, cap, Hkv, dh), dtype=dt, device="cuda")
    Vg_c = torch.zeros_like(K_c)
    out_c = torch.empty_like(seq_lens)
    G.gsa_cache_append(sh, new["kI"], new["K"], new["V"], new["g2"], seq_lens, kI_c, K_c, Vg_c, out_c)
    max_pages = cap // page
    pool_pages = B * max_pages + 3
    perm = torch.randperm(pool_pages, generator=torch.Generator().manual_seed(3))[:B * max_pages].reshape(B, max_pages).to(torch.int32).cuda()
    kI_p = torch.zeros((pool_pages, page, dI), dtype=dt, device="cuda")
    K_p = torch.zeros((pool_pages, page, Hkv, dh), dtype=dt, device="cuda")
    Vg_p = torch.zeros_like(K_p)
    out_p = torch.empty_like(seq_lens)
    G.gsa_paged_cache_append(sh, page, perm, pool_pages, new["kI"], new["K"], new["V"], new["g2"], seq_lens, kI_p, K_p, Vg_p, out_p)
    torch.cuda.synchronize()
    assert torch.equal(out_p, out_c) and out_c.tolist() == [5, 131, 505, 1024]
    for b in range(B):
        for p in range(max_pages):
            pg = int(perm[b, p])
            assert torch.equal(kI_p[pg], kI_c[b, p * page:(p + 1) * page])
            assert torch.equal(K_p[pg], K_c[b, p * page:(p + 1) * page])
            assert torch.equal(Vg_p[pg], Vg_c[b, p * page:(p + 1) * page])
    used = set(perm.flatten().tolist())
    for pg in range(pool_pages):
        if pg not in used:
            assert not K_p[pg].any() and not kI_p[pg].any(), "a page outside the table was written"
