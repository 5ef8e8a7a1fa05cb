"""The linear projections around the path (Sec. 2.1 Eq. 1, Sec. 3.3, Sec. 3.5, App. B): the fused input
projections and the output projection against the fp64 oracle on the same bf16 inputs.

Tolerance: a bf16 output carries one rounding (relative 2^-9) of a sum accumulated in fp32 over d_model
bf16 products (each exact in fp32); the accumulation error is below d_model * 2^-24 * sum|x_c W_oc|.  The test
bounds |y - ref| <= 2^-8 |ref| + 1e-5 * sum|x W|; the fp32 head weights sigma(.) are within 1e-5."""
import numpy as np
import pytest
import torch

import paper_2601_15305_amd as G
from oracle import gsa_oracle as O

pytestmark = pytest.mark.gpu

NAMES = ("Q", "K", "V", "g1", "g2", "qI", "kI", "Iw")


def _widths(sh):
    return dict(Q=sh.H * sh.d_h, K=sh.H_kv * sh.d_h, V=sh.H_kv * sh.d_h, g1=sh.H * sh.d_h, g2=sh.H_kv * sh.d_h,
                qI=sh.HI * sh.dI, kI=sh.dI, Iw=sh.HI)


def _make(sh, d_model, seed, skip=()):
    g = torch.Generator().manual_seed(seed)
    h = torch.randn((sh.B, sh.Lq, d_model), generator=g).to(torch.bfloat16).cuda()
    W = {n: (torch.randn((wd, d_model), generator=g) * d_model ** -0.5).to(torch.bfloat16).cuda()
         for n, wd in _widths(sh).items() if n not in skip}
    return h, W


def _run(sh, d_model, h, W):
    out = {}
    for n, wd in _widths(sh).items():
        if n in W:
            # NaN-filled destinations: a feature the kernel never writes fails the comparison
            out[n] = torch.full((sh.B, sh.Lq, wd), float("nan"), dtype=torch.float32 if n == "Iw" else torch.bfloat16, device="cuda")
    G.gsa_input_projections(sh, d_model, h, *[W.get(n) for n in NAMES], *[out.get(n) for n in NAMES])
    torch.cuda.synchronize()
    return out


def _check(h, W, out, tokens):
    """Compare the given tokens (flat indices into B*Lq) of every produced projection with the oracle."""
    hf = h.reshape(-1, h.shape[-1])[tokens].double().cpu().numpy()
    worst = 0.0
    for n, Wn in W.items():
        W64 = Wn.double().cpu().numpy()
        got = out[n].reshape(-1, out[n].shape[-1])[tokens].double().cpu().numpy()
        assert not np.isnan(got).any(), "unwritten outputs in %s" % n
        if n == "Iw":
            ref = O.indexer_head_weights(hf, W64)
            err = np.abs(got - ref)
            assert err.max() <= 1e-5, (n, err.max())
        else:
            ref = O.linear(hf, W64)
            mag = O.linear(np.abs(hf), np.abs(W64))
            err = np.abs(got - ref)
            bad = err > 2.0 ** -8 * np.abs(ref) + 1e-5 * mag
            assert not bad.any(), (n, float(err.max()), int(bad.sum()))
        worst = max(worst, float(err.max()))
    return worst


@pytest.mark.parametrize("B,Lq,d_model,H,H_kv,d_h,HI,dI", [
    (2, 77, 192, 4, 2, 64, 3, 32),     # 154 tokens (ragged token tile), 1027 features: 9 feature blocks, narrow last segment
    (1, 1, 64, 2, 1, 64, 1, 32),       # one token, one k-step
    (3, 128, 320, 16, 4, 128, 4, 64),  # the layer shape of Table 9 at a small width; 5636 features, 3 token blocks
    (1, 1000, 128, 2, 2, 64, 7, 128),  # seven indexer heads: the sigmoid segment straddles a group of four features
    (1, 2100, 128, 4, 2, 64, 3, 32),   # large-call shape (256 x 256 tiles): 9 ragged token blocks, 1027 features = 4 blocks + 3
    (2, 1300, 192, 16, 4, 128, 4, 64), # large-call shape, 5636 features: 23 feature blocks in groups of four (last group: 3)
])
def test_input_projections_match_oracle(B, Lq, d_model, H, H_kv, d_h, HI, dI):
    sh = G.make_shape(B, Lq, Lq, 0, H, H_kv, d_h, HI, dI, "bf16")
    h, W = _make(sh, d_model, seed=B * 1000 + Lq)
    out = _run(sh, d_model, h, W)
    n_tok = B * Lq
    tokens = np.arange(n_tok) if n_tok <= 160 else np.unique(np.concatenate(
        [np.arange(0, 8), np.arange(n_tok - 8, n_tok), np.arange(120, 136), np.arange(250, 262), np.random.default_rng(5).integers(0, n_tok, 64)]))
    _check(h, W, out, torch.from_numpy(tokens).cuda())


def test_skipped_projections_and_pairing():
    """A projection with neither weights nor destination is left out; the others are unchanged by its absence."""
    sh = G.make_shape(2, 40, 40, 0, 4, 2, 64, 2, 32, "bf16")
    h, W = _make(sh, 128, seed=9)
    full = _run(sh, 128, h, W)
    part = {n: W[n] for n in ("Q", "kI", "Iw")}
    got = _run(sh, 128, h, part)
    assert set(got) == {"Q", "kI", "Iw"}
    for n in got:
        assert torch.equal(got[n], full[n]), n
    with pytest.raises(G.GsaError) as e:
        G.gsa_input_projections(sh, 128, h, W["Q"], *([None] * 7), *([None] * 8))      # weights without a destination
    assert e.value.status == G.GSA_ERR_NULL
    with pytest.raises(G.GsaError) as e:
        G.gsa_input_projections(sh, 100, h, W["Q"], *([None] * 7), full["Q"], *([None] * 7))   # d_model not a multiple of 64
    assert e.value.status == G.GSA_ERR_UNSUPPORTED
    sh32 = G.make_shape(2, 40, 40, 0, 4, 2, 64, 2, 32, "f32")
    with pytest.raises(G.GsaError) as e:
        G.gsa_input_projections(sh32, 128, h, W["Q"], *([None] * 7), full["Q"], *([None] * 7))
    assert e.value.status == G.GSA_ERR_UNSUPPORTED


@pytest.mark.parametrize("B,Lq,H,d_h,d_model", [(2, 77, 4, 64, 192), (1, 300, 16, 128, 130), (4, 1, 2, 64, 2048), (1, 2500, 8, 64, 770)])
def test_output_projection_matches_oracle(B, Lq, H, d_h, d_model):
    sh = G.make_shape(B, Lq, Lq, 0, H, H, d_h, 1, 32, "bf16")
    g = torch.Generator().manual_seed(Lq)
    u = torch.randn((B, Lq, H * d_h), generator=g).to(torch.bfloat16).cuda()
    W_O = (torch.randn((d_model, H * d_h), generator=g) * (H * d_h) ** -0.5).to(torch.bfloat16).cuda()
    y = torch.full((B, Lq, d_model), float("nan"), dtype=torch.bfloat16, device="cuda")
    G.gsa_output_projection(sh, d_model, u, W_O, y)
    torch.cuda.synchronize()
    n_tok = B * Lq
    tokens = torch.arange(n_tok, device="cuda") if n_tok <= 400 else torch.cat(
        [torch.arange(0, 8, device="cuda"), torch.arange(n_tok - 8, n_tok, device="cuda"), torch.arange(250, 262, device="cuda"),
         torch.randint(0, n_tok, (48,), generator=torch.Generator().manual_seed(1)).cuda()])
    _check(u, {"O": W_O}, {"O": y}, tokens)


def test_projections_feed_the_forward_path():
    """h -> projections -> gsa_forward -> output projection, against the oracle chained the same way on the bf16
    values the kernels hand to one another (each stage is compared on the inputs it actually received)."""
    import gsa_testlib as T
    from paper_2601_15305_amd import synthetic as S
    wl = S.Workload("proj-chain", B=1, Lq=320, Lk=320, q_offset=0, H=4, H_kv=2, d_h=64, HI=2, dI=32, k_base=32, k_min=8,
                    k_max=64, k_fixed=48, dtype="bf16")
    sh = G.shape_of(wl)
    d_model = 256
    h, W = _make(sh, d_model, seed=21)
    p = _run(sh, d_model, h, W)
    _check(h, W, p, torch.arange(wl.Lq, device="cuda"))
    t = dict(Q=p["Q"].view(1, wl.Lq, wl.H, wl.d_h), K=p["K"].view(1, wl.Lq, wl.H_kv, wl.d_h), V=p["V"].view(1, wl.Lq, wl.H_kv, wl.d_h),
             g1=p["g1"].view(1, wl.Lq, wl.H, wl.d_h), g2=p["g2"].view(1, wl.Lq, wl.H_kv, wl.d_h),
             qI=p["qI"].view(1, wl.Lq, wl.HI, wl.dI), kI=p["kI"], w=p["Iw"], bI=None)
    ctl = G.make_adaptive(0.0, wl.k_base, wl.k_min, wl.k_max, k_fixed=48)
    res = T.gpu_forward(wl, t, ctl)
    out = res["out"]
    n_sel, idx = res["n_sel"].cpu().numpy(), res["idx"].cpu().numpy()
    for i in (0, 47, 48, 200, 319):
        m = int(n_sel[0, i])
        sel = idx[0, i, :m]
        ref, _ = O.sparse_gated_attn_row(T.to64(t["Q"][0, i]), T.to64(t["K"][0])[sel], T.to64(t["V"][0])[sel], T.to64(t["g2"][0])[sel],
                                         T.to64(t["g1"][0, i]), np.arange(m))
        T.check_out(out[0, i], ref, "bf16")
    W_O = (torch.randn((d_model, wl.H * wl.d_h), generator=torch.Generator().manual_seed(4)) * 0.06).to(torch.bfloat16).cuda()
    y = torch.empty((1, wl.Lq, d_model), dtype=torch.bfloat16, device="cuda")
    G.gsa_output_projection(sh, d_model, out, W_O, y)
    torch.cuda.synchronize()
    _check(out.reshape(1, wl.Lq, -1), {"O": W_O}, {"O": y}, torch.arange(wl.Lq, device="cuda"))
