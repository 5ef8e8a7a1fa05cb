"""gsa_forward_noalloc (the workspace is an array inside the library's device code) against gsa_forward on the
same inputs: two calls in a row, the second on a smaller problem, plus the size limit.  Collected last on
purpose: it is the only test that touches the library's static scratch."""
import ctypes

import numpy as np
import pytest
import torch

import paper_2601_15305_amd as G
from paper_2601_15305_amd import synthetic as S

import gsa_testlib as T

pytestmark = pytest.mark.gpu


def _both(wl, vbar, seed_shift=0):
    t = S.make_inputs(wl.with_(seed=wl.seed + seed_shift), "cuda")
    sh = G.shape_of(wl)
    ctl = G.make_adaptive(vbar, wl.k_base, wl.k_min, wl.k_max)
    assert G.gsa_forward_workspace_bytes(sh, wl.k_cap, True, 0) <= G.STATIC_SCRATCH_BYTES
    ref = T.gpu_forward(wl, t, ctl)                     # caller-supplied workspace
    out = torch.full_like(t["Q"], float("nan"))
    idx = torch.full((wl.B, wl.Lq, wl.k_cap), -7, dtype=torch.int32, device="cuda")
    n_sel = torch.full((wl.B, wl.Lq), -7, dtype=torch.int32, device="cuda")
    k = torch.full_like(n_sel, -7)
    var = torch.full((wl.B, wl.Lq), float("nan"), dtype=torch.float32, device="cuda")
    G.gsa_forward_noalloc(sh, ctl, t["Q"], t["K"], t["V"], t["g1"], t["g2"], t["qI"], t["kI"], t["w"], t["bI"], 0.0, out, idx,
                          n_sel, k, var, wl.k_cap)
    torch.cuda.synchronize()
    assert torch.equal(var, ref["var"]) and torch.equal(k, ref["k"]) and torch.equal(n_sel, ref["n_sel"])
    assert torch.equal(idx, ref["idx"]), "same kernels, same inputs: identical index sets"
    # the slabs (hence the split of the indexer's key ranges) may differ with the workspace size; k_t then agrees
    # and so do the sets, and the attention is the same launch: bit-identical outputs
    assert torch.equal(out, ref["out"])
    assert torch.isfinite(out.float()).all()
    return ref


def test_noalloc_forward_matches_forward_twice():
    big = S.Workload("noalloc-decode", 8, 1, 40000, 39999, 16, 4, 128, 4, 64, "bf16", 181, 128, 256, seed=71)
    small = S.Workload("noalloc-prefill", 2, 700, 700, 0, 16, 4, 128, 4, 64, "bf16", 45, 32, 64, seed=72)
    _both(big, 0.3)
    _both(small, 0.3)          # a smaller problem after a larger one: stale scratch contents must not matter
    _both(big, 0.3, seed_shift=5)


def test_noalloc_forward_refuses_what_does_not_fit():
    lib = G.load()
    wl = S.C4
    sh = G.shape_of(wl)
    assert G.gsa_forward_workspace_bytes(sh, wl.k_cap, True, 0) > G.STATIC_SCRATCH_BYTES
    ctl = G.make_adaptive(1.0, wl.k_base, wl.k_min, wl.k_max)
    fake = 0x1000
    rc = lib.gsa_forward_noalloc(ctypes.byref(sh), ctypes.byref(ctl), *([fake] * 9), 0.0, fake, None, None, None, None,
                                 wl.k_cap, None, None)
    assert rc == G.GSA_ERR_WORKSPACE
    assert b"static scratch" in lib.gsa_last_error()
