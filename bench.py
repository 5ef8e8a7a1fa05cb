#!/usr/bin/env python3
"""Benchmark of the GSA forward hot path on one MI355X.

One step = one gsa_forward call (value gate -> indexer -> adaptive k_t -> top-k_t -> sparse gated
attention) over one batch of synthetic input shaped like the paper's 1.7B model at 128K context
(Sec. 7.1; indexer defaults of Sec. 4.1), with a bounded workspace (--workspace-gib, default 8).
Inputs are resident in HBM before the timed region.  Prints one JSON line:

  value / ms_per_step   whole-path queries/s of the bounded-workspace call
  roofline              the dominant kernel (gathered sparse attention): achieved gather rate against the
                        gather ceiling of cache-resident rows measured in this same run (a fraction that
                        can fail), the compulsory-byte HBM fraction, and the bytes that left the L2
                        (rocprofv3 counters collected by two child runs of this script)
  stages                per-stage times and rates (both forms of indexer and selection)
  one_slab              the same call with the whole problem in one slab (large workspace), for comparison
  decode_c5, c4_h_kv16  the decode configuration (eager calls, and one call captured in a HIP graph and replayed)
                        and the 16-kv-head reading of the 128K prefill
  projections           the layer's input and output projections at the same token count (d_model 2048)
  training_c2           backward of the sparse gated attention and the sparse-phase indexer loss at the 8K configuration
  cpu_baseline          the CPU oracle timed on a bounded sample of the same workload on this machine's host cores
"""
import argparse
import csv
import glob
import json
import os
import shutil
import subprocess
import sys
import tempfile
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0        # MI355X HBM3E
PEAK_MFMA_BF16_TFLOPS = 2500.0
# sigmoids per second the vector ALUs can retire: mul, exp2, add, rcp, fma = 3 full-rate + 2 half-rate
# (transcendental) instructions = 7 lane-cycles each, on 256 CUs x 64 lanes at 2.4 GHz
PEAK_SIGMOID_PER_S = 256 * 64 * 2.4e9 / 7.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="C4-128k-prefill")
    ap.add_argument("--h-kv", type=int, default=0, help="override the number of key-value heads")
    ap.add_argument("--workspace-gib", type=float, default=8.0, help="workspace handed to gsa_forward (0 = whole problem in one slab)")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="budget for the CPU oracle leg (0 = skip)")
    ap.add_argument("--stage-steps", type=int, default=0, help="steps of the per-stage timing loop (0 = same as --steps)")
    ap.add_argument("--no-traffic", action="store_true", help="do not collect the HBM-side byte counters (two child runs under rocprofv3)")
    ap.add_argument("--no-extras", action="store_true", help="skip the one-slab, decode and 16-kv-head legs")
    ap.add_argument("--training-only", action="store_true", help="run only the training leg (C2-8k) and print its figures as one JSON line")
    ap.add_argument("--traffic-child", action="store_true", help=argparse.SUPPRESS)
    return ap.parse_args()


# ------------------------------------------------------------------------------------------------ counters
def collect_traffic(args):
    """HBM-side bytes of the attention launches of ONE gsa_forward call, from rocprofv3 --pmc FETCH_SIZE and
    WRITE_SIZE (one run each, the same workload and workspace as the timed call).  The raw counters are scaled
    by what they read for a kernel of known traffic in the same run: the value gate reads V and g2 once and
    writes V' once.  Runs before this process touches the GPU.  Returns a dict, or a reason string."""
    exe = shutil.which("rocprofv3")
    if exe is None:
        return "rocprofv3 not found"
    out = {}
    for counter in ("FETCH_SIZE", "WRITE_SIZE"):
        d = tempfile.mkdtemp(prefix="gsa_pmc_", dir="/tmp")
        cmd = ["timeout", "-s", "KILL", "170", exe, "--pmc", counter, "--output-format", "csv", "-d", d, "-o", "p", "--",
               sys.executable, os.path.join(ROOT, "bench.py"), "--traffic-child", "--workload", args.workload,
               "--workspace-gib", str(args.workspace_gib)] + (["--h-kv", str(args.h_kv)] if args.h_kv else [])
        print("[bench] collecting %s under rocprofv3 ..." % counter, file=sys.stderr, flush=True)
        env = dict(os.environ, TMPDIR="/tmp")
        try:
            r = subprocess.run(cmd, cwd="/tmp", env=env, capture_output=True, text=True, timeout=200)
        except subprocess.TimeoutExpired:
            shutil.rmtree(d, ignore_errors=True)
            return "rocprofv3 %s run timed out" % counter
        rows = []
        for f in glob.glob(os.path.join(d, "**", "*counter_collection.csv"), recursive=True):
            rows += list(csv.DictReader(open(f)))
        shutil.rmtree(d, ignore_errors=True)
        if r.returncode != 0 or not rows:
            return "rocprofv3 %s run failed (rc %d): %s" % (counter, r.returncode, (r.stderr or "")[-200:])
        agg = {}
        for row in rows:
            if row.get("Counter_Name") != counter:
                continue
            name = row["Kernel_Name"]
            key = "gate" if "value_gate" in name else ("attn" if "attn_" in name else None)
            if key:
                agg[key] = agg.get(key, 0.0) + float(row["Counter_Value"])
                agg[key + "_n"] = agg.get(key + "_n", 0) + 1
        if "gate" not in agg or "attn" not in agg:
            return "no attention / value-gate dispatches in the %s trace" % counter
        out[counter] = agg
    return out


def traffic_child(args):
    """What the rocprofv3 child runs: one bounded-workspace gsa_forward call, nothing else."""
    import torch
    import paper_2601_15305_amd as G
    from paper_2601_15305_amd import synthetic as S
    wl = S.CONFIGS[args.workload]
    if args.h_kv:
        wl = wl.with_(H_kv=args.h_kv)
    dev = torch.device("cuda:0")
    t = S.make_inputs(wl, dev)
    run = ForwardRun(G, wl, t, args.workspace_gib)
    run.step()
    torch.cuda.synchronize()


# ------------------------------------------------------------------------------------------------ the timed call
class ForwardRun:
    """Buffers and controller of one workload; step() is one gsa_forward call."""

    def __init__(self, G, wl, t, workspace_gib):
        import numpy as np
        import torch
        self.G, self.wl, self.t = G, wl, t
        dev = t["Q"].device
        self.sh = sh = G.shape_of(wl)
        self.k_cap = wl.k_cap
        # moving-average variance: the batch mean of the row variances of this same data (a frozen input)
        self.var = torch.empty((wl.B, wl.Lq), dtype=torch.float32, device=dev)
        ws_i = G.workspace(G.gsa_indexer_workspace_bytes(sh, 0, wl.Lq), dev)
        G.gsa_indexer_scores(sh, t["qI"], t["kI"], t["w"], None, 0, wl.Lq, None, 0, None, self.var, ws_i)
        torch.cuda.synchronize()
        self.vbar = float(np.float32(self.var.double().mean().item()))
        self.ctl_kw = dict(vbar=self.vbar, k_base=wl.k_base, k_min=wl.k_min, k_max=wl.k_max, k_fixed=wl.k_fixed, mode=0)
        self.ctl = G.make_adaptive(self.vbar, wl.k_base, wl.k_min, wl.k_max, wl.k_fixed, 0)
        lo = G.gsa_forward_workspace_bytes(sh, self.k_cap, True, 0)
        hi = G.gsa_forward_workspace_bytes(sh, self.k_cap, True, wl.Lq)
        want = hi if workspace_gib <= 0 else int(workspace_gib * (1 << 30))
        self.ws_bytes = max(lo, min(hi, want))
        self.ws = G.workspace(self.ws_bytes, dev)
        self.out = torch.empty_like(t["Q"])
        self.idx = torch.empty((wl.B, wl.Lq, self.k_cap), dtype=torch.int32, device=dev)
        self.n_sel = torch.empty((wl.B, wl.Lq), dtype=torch.int32, device=dev)
        self.kbuf = torch.empty_like(self.n_sel)

    def step(self):
        t = self.t
        self.G.gsa_forward(self.sh, self.ctl, t["Q"], t["K"], t["V"], t["g1"], t["g2"], t["qI"], t["kI"], t["w"], None, 0.0,
                           self.out, self.idx, self.n_sel, self.kbuf, self.var, self.k_cap, self.ws)

    def time(self, steps, warmup):
        import torch
        for _ in range(warmup):
            self.step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        e0, e1 = ev(), ev()
        e0.record()
        for _ in range(steps):
            self.step()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / steps, (time.perf_counter() - t0) * 1e3 / steps


def ev():
    import torch
    return torch.cuda.Event(enable_timing=True)


def timed(fn, steps):
    """Average milliseconds of fn() over `steps` calls after one warm-up call, by events on the launch stream."""
    import torch
    fn()
    e0, e1 = ev(), ev()
    e0.record()
    for _ in range(steps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / steps


def gather_ceilings(G, dev):
    """Whole-row (256-byte) gather rates of this chip with no arithmetic behind them, in the access shape of the
    attention kernel: rows drawn uniformly from a table that fits the 4 MB L2 of every XCD, and from a table
    larger than every on-die cache.  GB/s."""
    import torch
    res = {}
    n_idx = 1 << 25
    waves = 256 * 32
    sink = torch.empty(waves, dtype=torch.int32, device=dev)
    g = torch.Generator(device=dev)
    g.manual_seed(99)
    for name, table_bytes in (("l2_resident_2MiB_table", 2 << 20), ("hbm_resident_4GiB_table", 4 << 30)):
        rows = table_bytes // 256
        table = torch.ones(table_bytes // 4, dtype=torch.int32, device=dev)
        idx = torch.randint(0, rows, (n_idx,), dtype=torch.int32, device=dev, generator=g)
        ms = timed(lambda: G.gsa_probe_gather(table, rows, idx, n_idx, waves, sink), 5)
        res[name] = round(n_idx * 256 / (ms * 1e-3) / 1e9, 1)
        if table_bytes == 2 << 20:
            # the same rows, each staged through LDS (write + read back) as an MFMA operand has to be: eight waves per CU
            ms = timed(lambda: G.gsa_probe_gather_staged(table, rows, idx, n_idx, 256 * 8, sink), 5)
            res[name + "_staged_through_lds"] = round(n_idx * 256 / (ms * 1e-3) / 1e9, 1)
        del table, idx
    return res


def stage_breakdown(G, CM, wl, t, run, ssteps):
    """The launches gsa_forward makes, as the stage calls of the C ABI chained by hand over the whole problem, events
    between them.  Both forms of stages 1 and 3: fp32 scores (gsa_indexer_scores / gsa_topk_select) and the
    16-bit keys the fused call uses (gsa_indexer_keys / gsa_topk_select_keys)."""
    import torch
    sh, k_cap, ctl = run.sh, run.k_cap, run.ctl
    dev = t["Q"].device
    R = wl.Lq
    ld = (wl.Lk + 31) // 32 * 32
    prepass = wl.Lq * min(k_cap, wl.Lk) >= 4 * wl.Lk     # the same rule gsa_forward applies to the value gate
    var = torch.empty((wl.B, wl.Lq), dtype=torch.float32, device=dev)
    n_sel = torch.empty((wl.B, wl.Lq), dtype=torch.int32, device=dev)
    kbuf = torch.empty_like(n_sel)
    idx = torch.empty((wl.B, wl.Lq, k_cap), dtype=torch.int32, device=dev)
    out = torch.empty_like(t["Q"])
    Vg = torch.empty_like(t["V"])
    ws_i = G.workspace(G.gsa_indexer_workspace_bytes(sh, 0, R), dev)
    ws_a = G.workspace(G.gsa_attn_workspace_bytes(sh, 0, R, k_cap), dev)
    ms = {}
    # fp32 form
    scores = torch.empty((wl.B, R, ld), dtype=torch.float32, device=dev)
    ms["indexer_fp32_scores"] = timed(lambda: G.gsa_indexer_scores(sh, t["qI"], t["kI"], t["w"], None, 0, R, scores, ld, None, var, ws_i), ssteps)
    G.gsa_adaptive_k(sh, ctl, var, kbuf, n_sel)
    ms["select_fp32_scores"] = timed(lambda: G.gsa_topk_select(sh, 0, R, scores, ld, n_sel, k_cap, idx), ssteps)
    del scores
    torch.cuda.empty_cache()
    # 16-bit key form (the fused path)
    keys = torch.empty((wl.B, R, ld), dtype=torch.int16, device=dev)
    ms["indexer_keys"] = timed(lambda: G.gsa_indexer_keys(sh, t["qI"], t["kI"], t["w"], None, 0, R, keys, ld, None, var, ws_i), ssteps)
    ms["adaptive_k"] = timed(lambda: G.gsa_adaptive_k(sh, ctl, var, kbuf, n_sel), ssteps)
    ms["select_keys"] = timed(lambda: G.gsa_topk_select_keys(sh, 0, R, keys, ld, n_sel, k_cap, idx, t["qI"], t["kI"], t["w"], None), ssteps)
    del keys
    torch.cuda.empty_cache()
    ms["indexer_stats_only"] = timed(lambda: G.gsa_indexer_scores(sh, t["qI"], t["kI"], t["w"], None, 0, R, None, 0, None, var, ws_i), ssteps)
    ms["value_gate"] = timed(lambda: G.gsa_value_gate(sh, t["V"], t["g2"], Vg), ssteps) if prepass else 0.0
    ms["attention"] = timed(lambda: G.gsa_sparse_gated_attn(sh, 0, R, t["Q"], t["K"], Vg if prepass else t["V"], None if prepass else t["g2"],
                                                            t["g1"], idx, n_sel, k_cap, 0.0, out, ws_a), ssteps)
    sum_nsel = int(n_sel.sum().item())
    return ms, sum_nsel, prepass


def comparison_variants(G, S, CM, wl, t, run, gsa_ms):
    """The paper's comparison systems (Sec. 7.1) on the same tensors and the same GPU: dense causal attention with both
    gates ("gated only") and without ("standard"), and the ReLU-indexer / fixed-k / ungated forward ("sparse only")."""
    import torch
    dev = t["Q"].device
    sh = run.sh
    out = torch.empty_like(t["Q"])
    ws_d = G.workspace(G.gsa_dense_attn_workspace_bytes(sh, True), dev)
    gated = timed(lambda: G.gsa_dense_gated_attn(sh, 0, wl.Lq, t["Q"], t["K"], t["V"], t["g2"], t["g1"], 0.0, out, ws_d), 2)
    plain = timed(lambda: G.gsa_dense_gated_attn(sh, 0, wl.Lq, t["Q"], t["K"], t["V"], None, None, 0.0, out, None), 2)
    pairs = CM.causal_pairs(wl.B, wl.Lq, wl.Lk, wl.q_offset)
    dense_flops = 4 * wl.d_h * wl.H * pairs
    res = {"dense_gated_ms": round(gated, 3), "dense_standard_ms": round(plain, 3),
           "dense_standard_tflops": round(dense_flops / (plain * 1e-3) / 1e12, 1),
           "dense_standard_frac_mfma_bf16_peak": round(dense_flops / (plain * 1e-3) / 1e12 / PEAK_MFMA_BF16_TFLOPS, 4),
           "gsa_ms": round(gsa_ms, 3)}
    del ws_d
    if wl.k_fixed == 0:
        wr = wl.with_(indexer_act="relu", k_fixed=wl.k_base)
        shr = G.shape_of(wr)
        ctl = G.make_adaptive(1.0, 1, 1, 1, k_fixed=wl.k_base)
        ws = G.workspace(run.ws_bytes, dev)
        idx = torch.empty((wl.B, wl.Lq, wl.k_base), dtype=torch.int32, device=dev)
        so = timed(lambda: G.gsa_forward(shr, ctl, t["Q"], t["K"], t["V"], None, None, t["qI"], t["kI"], t["w"], None, 0.0, out, idx,
                                         run.n_sel, None, None, wl.k_base, ws), 2)
        res["sparse_only_ms"] = round(so, 3)
        res["sparse_only_k"] = wl.k_base
        del ws, idx
    res["speedup_gsa_vs_standard"] = round(plain / gsa_ms, 2)
    res["speedup_gated_only_vs_standard"] = round(plain / gated, 3)
    if "sparse_only_ms" in res:
        res["speedup_sparse_only_vs_standard"] = round(plain / res["sparse_only_ms"], 2)
    res["paper_ratios_context"] = ("Table 9 (128K, 1.7B model, 8x H100, precision not stated): prefill latency relative to standard "
                                   "0.09 (GSA), 0.08 (sparse only), 1.02 (gated only); abstract: 12-16x")
    torch.cuda.empty_cache()
    return res


def projections_leg(G, wl, d_model, dev):
    """The layer's linear projections at the workload's token count (Sec. 2.1 Eq. 1, Sec. 3.3, Sec. 3.5, App. B):
    the fused input GEMM (all eight segments) and the output projection, against the dense bf16 MFMA peak."""
    import torch
    sh = G.shape_of(wl.with_(Lk=wl.Lq, q_offset=0))
    tokens = wl.B * wl.Lq
    g = torch.Generator(device=dev).manual_seed(7)
    h = torch.randn((wl.B, wl.Lq, d_model), generator=g, device=dev).to(torch.bfloat16)
    widths = [wl.H * wl.d_h, wl.H_kv * wl.d_h, wl.H_kv * wl.d_h, wl.H * wl.d_h, wl.H_kv * wl.d_h, wl.HI * wl.dI, wl.dI, wl.HI]
    W = [(torch.randn((n, d_model), generator=g, device=dev) * d_model ** -0.5).to(torch.bfloat16) for n in widths]
    outs = [torch.empty((wl.B, wl.Lq, n), dtype=torch.float32 if i == 7 else torch.bfloat16, device=dev) for i, n in enumerate(widths)]
    ims = timed(lambda: G.gsa_input_projections(sh, d_model, h, *W, *outs), 5)
    W_O = (torch.randn((d_model, wl.H * wl.d_h), generator=g, device=dev) * (wl.H * wl.d_h) ** -0.5).to(torch.bfloat16)
    y = torch.empty((wl.B, wl.Lq, d_model), dtype=torch.bfloat16, device=dev)
    oms = timed(lambda: G.gsa_output_projection(sh, d_model, outs[0], W_O, y), 5)
    fi = 2.0 * tokens * d_model * sum(widths)
    fo = 2.0 * tokens * d_model * wl.H * wl.d_h
    return {"d_model": d_model, "tokens": tokens, "input_features": sum(widths),
            "input_ms": round(ims, 3), "input_tflops": round(fi / (ims * 1e-3) / 1e12, 1),
            "input_frac_mfma_peak": round(fi / (ims * 1e-3) / 1e12 / PEAK_MFMA_BF16_TFLOPS, 4),
            "output_ms": round(oms, 3), "output_tflops": round(fo / (oms * 1e-3) / 1e12, 1),
            "output_frac_mfma_peak": round(fo / (oms * 1e-3) / 1e12 / PEAK_MFMA_BF16_TFLOPS, 4)}


def training_leg(G, S, wl, dev):
    """Training side (Sec. 6.1) at a training-length context: the backward of the sparse gated attention (selection
    held fixed) and the sparse-phase indexer loss with its gradients, after one forward call that fixes the selection."""
    import torch
    t = S.make_inputs(wl, dev)
    run = ForwardRun(G, wl, t, 8)
    run.step()
    torch.cuda.synchronize()
    sh, k_cap = run.sh, run.k_cap
    f32 = dict(dtype=torch.float32, device=dev)
    dout = torch.randn(t["Q"].shape, generator=torch.Generator(device=dev).manual_seed(3), device=dev).to(t["Q"].dtype)
    dQ, dg1 = torch.empty(t["Q"].shape, **f32), torch.empty(t["Q"].shape, **f32)
    dK, dV, dg2 = (torch.empty(t["K"].shape, **f32) for _ in range(3))
    p_mean = torch.empty((wl.B, wl.Lq, k_cap), **f32)
    bwd = lambda ws: G.gsa_sparse_gated_attn_bwd(sh, t["Q"], t["K"], t["V"], t["g2"], t["g1"], run.idx, run.n_sel, k_cap, 0.0, dout,
                                                 dQ, dK, dV, dg1, dg2, p_mean, workspace=ws)
    ams = timed(lambda: bwd(None), 2)                      # one pass, dK / dV' by fp32 atomics
    dK_atomic = dK.clone()
    bws_bytes = G.gsa_attn_bwd_workspace_bytes(sh, k_cap)
    bws = G.workspace(bws_bytes)
    bms = timed(lambda: bwd(bws), 3)                       # with a workspace: key-centred second pass over inverted lists
    dk_diff = float((dK - dK_atomic).abs().max().item() / max(float(dK_atomic.abs().max().item()), 1e-30))
    loss = torch.empty((wl.B, wl.Lq), **f32)
    dqI, dkI, dw = torch.empty(t["qI"].shape, **f32), torch.empty(t["kI"].shape, **f32), torch.empty(t["w"].shape, **f32)
    kms = timed(lambda: G.gsa_indexer_sparse_kl(sh, t["qI"], t["kI"], t["w"], None, run.idx, run.n_sel, k_cap, p_mean, loss, dqI, dkI, dw),
                2)
    fms, _ = run.time(3, 1)
    pairs = int(run.n_sel.sum().item())
    # rows gathered by the backward per (query, selected key, kv head): K and gated-value rows in the query-centred pass
    # (twice), the query and dO rows of the group's heads in the key-centred pass (bf16 inputs: all bf16)
    elt = 2 if wl.dtype == "bf16" else 4
    G_ = wl.H // wl.H_kv
    gathered = pairs * wl.H_kv * wl.d_h * ((2 * 2 * elt + G_ * 2 * elt) if wl.dtype == "bf16" else (2 * 3 * elt + G_ * 2 * elt))
    return {"workload": wl.name, "forward_ms": round(fms, 3), "attn_backward_ms": round(bms, 3),
            "attn_backward_workspace_bytes": bws_bytes, "attn_backward_gathered_gbs": round(gathered / (bms * 1e-3) / 1e9, 1),
            "attn_backward_atomics_ms": round(ams, 3), "dK_max_rel_diff_between_the_two": dk_diff,
            "indexer_kl_ms": round(kms, 3), "selected_pairs": pairs,
            "mean_kl_per_row": round(float(loss.double().mean().item()), 5)}


def small_leg(G, S, CM, wl, steps, warmup, workspace_gib):
    """queries/s of another configuration (fresh inputs), with the indexer's key-scan rate for decode shapes."""
    import torch
    dev = torch.device("cuda:0")
    t = S.make_inputs(wl, dev)
    run = ForwardRun(G, wl, t, workspace_gib)
    ms, _ = run.time(steps, warmup)
    sum_nsel = int(run.n_sel.sum().item())
    res = {"workload": wl.name, "H_kv": wl.H_kv, "ms_per_step": round(ms, 4), "queries_per_s": round(wl.B * wl.Lq / (ms * 1e-3), 1),
           "workspace_bytes": run.ws_bytes, "mean_k": round(sum_nsel / (wl.B * wl.Lq), 1)}
    if wl.Lq == 1:   # decode: the scan of the cached indexer keys dominates and is HBM-bound
        var = torch.empty((wl.B, wl.Lq), dtype=torch.float32, device=dev)
        ws_i = G.workspace(G.gsa_indexer_workspace_bytes(run.sh, 0, 1), dev)
        ld = (wl.Lk + 31) // 32 * 32
        keys = torch.empty((wl.B, 1, ld), dtype=torch.int16, device=dev)
        ims = timed(lambda: G.gsa_indexer_keys(run.sh, t["qI"], t["kI"], t["w"], None, 0, 1, keys, ld, None, var, ws_i), max(steps, 10))
        scan = wl.B * wl.Lk * wl.dI * 2
        res["indexer_ms"] = round(ims, 4)
        res["indexer_key_scan_gbs"] = round(scan / (ims * 1e-3) / 1e9, 1)
        res["indexer_frac_hbm_peak"] = round(scan / (ims * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)
        # the same step captured once in a HIP graph and replayed (the call launches kernels only)
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            run.step()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            run.step()
        gms = timed(graph.replay, max(steps, 20))
        res["graph_replay_ms_per_step"] = round(gms, 4)
        res["graph_replay_queries_per_s"] = round(wl.B * wl.Lq / (gms * 1e-3), 1)
        # the same step on paged caches: the rows of every sequence behind a shuffled block table (pages of 256 tokens)
        page = 256
        max_pages = wl.Lk // page
        pool_pages = wl.B * max_pages
        gen = torch.Generator(device=dev).manual_seed(11)
        table = torch.randperm(pool_pages, generator=gen, device=dev).to(torch.int32).reshape(wl.B, max_pages)
        Vg = torch.empty_like(t["V"])
        G.gsa_value_gate(run.sh, t["V"], t["g2"], Vg)

        def to_pool(x):   # [B, Lk, ...] -> [pool_pages, page, ...] with page table[b, p] holding tokens p*page.. of sequence b
            pool = torch.empty((pool_pages, page) + tuple(x.shape[2:]), dtype=x.dtype, device=dev)
            pool[table.reshape(-1).long()] = x.reshape((pool_pages, page) + tuple(x.shape[2:]))
            return pool
        kI_p, K_p = to_pool(t["kI"]), to_pool(t["K"])
        Vg_p = to_pool(Vg)
        del Vg
        seq_lens = torch.full((wl.B,), wl.Lk, dtype=torch.int32, device=dev)
        out_p = torch.empty_like(run.out)
        ws_p = G.workspace(G.gsa_paged_decode_workspace_bytes(run.sh, run.k_cap), dev)
        pms = timed(lambda: G.gsa_paged_decode_step(run.sh, run.ctl, page, table, pool_pages, t["Q"], t["g1"], t["qI"], t["w"], None, kI_p,
                                                    K_p, Vg_p, seq_lens, 0.0, out_p, None, None, None, None, run.k_cap, ws_p), max(steps, 20))
        run.step()
        torch.cuda.synchronize()
        res["paged_ms_per_step"] = round(pms, 4)
        res["paged_queries_per_s"] = round(wl.B * wl.Lq / (pms * 1e-3), 1)
        res["paged_equals_contiguous"] = bool(torch.equal(out_p, run.out))
        del kI_p, K_p, Vg_p
    else:
        sh, k_cap = run.sh, run.k_cap
        ws_a = G.workspace(G.gsa_attn_workspace_bytes(sh, 0, wl.Lq, k_cap), dev)
        Vg = torch.empty_like(t["V"])
        G.gsa_value_gate(sh, t["V"], t["g2"], Vg)
        out = torch.empty_like(t["Q"])
        ams = timed(lambda: G.gsa_sparse_gated_attn(sh, 0, wl.Lq, t["Q"], t["K"], Vg, None, t["g1"], run.idx, run.n_sel, k_cap, 0.0, out, ws_a), 2)
        gb = CM.gathered_bytes(sum_nsel, wl.H_kv, wl.d_h, 2 if wl.dtype == "bf16" else 4)
        res["attention_ms"] = round(ams, 3)
        res["attention_gathered_gbs"] = round(gb / (ams * 1e-3) / 1e9, 1)
    del run, t
    torch.cuda.empty_cache()
    return res


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    if args.traffic_child:
        traffic_child(args)
        return
    if args.training_only:
        import torch
        import paper_2601_15305_amd as G
        from paper_2601_15305_amd import synthetic as S
        assert torch.cuda.is_available(), "bench.py needs the GPU"
        G.load()
        torch.cuda.set_device(0)
        print(json.dumps({"training_c2": training_leg(G, S, S.C2, torch.device("cuda:0"))}))
        return
    traffic = "not collected (--no-traffic)" if args.no_traffic else collect_traffic(args)

    import numpy as np
    import torch
    import paper_2601_15305_amd as G
    from paper_2601_15305_amd import cost_model as CM
    from paper_2601_15305_amd import synthetic as S

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    G.load()
    wl = S.CONFIGS[args.workload]
    if args.h_kv:
        wl = wl.with_(H_kv=args.h_kv)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    t = S.make_inputs(wl, dev)
    elt = 2 if wl.dtype == "bf16" else 4
    queries = wl.B * wl.Lq

    # ---- the timed call -----------------------------------------------------------------------------
    print("[bench] timing gsa_forward on %s ..." % wl.name, file=sys.stderr, flush=True)
    run = ForwardRun(G, wl, t, args.workspace_gib)
    ms_per_step, wall_ms = run.time(args.steps, args.warmup)
    sum_nsel = int(run.n_sel.sum().item())
    fused = {k: getattr(run, k).clone() for k in ("out", "n_sel")}     # the timed path's own result, for the CPU leg
    fused["idx"] = run.idx
    ws_bytes, vbar, ctl_kw = run.ws_bytes, run.vbar, run.ctl_kw
    run.ws = None
    torch.cuda.empty_cache()

    one_slab = None
    if not args.no_extras and args.workspace_gib > 0:
        hi = G.gsa_forward_workspace_bytes(run.sh, run.k_cap, True, wl.Lq)
        if hi > ws_bytes and hi < 150 * (1 << 30):
            run.ws = G.workspace(hi, dev)
            run.ws_bytes = hi
            keep = run.idx
            run.idx = torch.empty_like(keep)
            ms1, _ = run.time(max(2, args.steps // 2), 1)
            one_slab = {"ms_per_step": round(ms1, 3), "queries_per_s": round(queries / (ms1 * 1e-3), 1), "workspace_bytes": hi}
            run.idx = keep
            run.ws = None
            torch.cuda.empty_cache()

    # ---- per-stage timing and the gather ceilings -------------------------------------------------------
    print("[bench] per-stage timing ...", file=sys.stderr, flush=True)
    ssteps = args.stage_steps or args.steps
    stage_ms, sum_nsel_st, prepass = stage_breakdown(G, CM, wl, t, run, ssteps)
    ceil = gather_ceilings(G, dev)

    pairs = CM.causal_pairs(wl.B, wl.Lq, wl.Lk, wl.q_offset)
    fl_idx = CM.indexer_flops(pairs, wl.HI, wl.dI)
    fl_att = CM.attention_flops(sum_nsel, wl.H, wl.d_h)
    gbytes = CM.gathered_bytes(sum_nsel_st, wl.H_kv, wl.d_h, elt, gate_in_kernel=not prepass)
    # compulsory bytes of the attention: every K and V' row, Q, g1 and the output once, the index lists once
    compulsory = (2 * wl.B * wl.Lk * wl.H_kv * wl.d_h + 3 * wl.B * wl.Lq * wl.H * wl.d_h) * elt + sum_nsel_st * 4
    att_s = stage_ms["attention"] * 1e-3
    att_gbs = gbytes / att_s / 1e9

    def idx_fig(ms):
        s = ms * 1e-3
        return {"ms": round(ms, 4), "tflops": round(fl_idx / s / 1e12, 2), "frac_mfma_bf16_peak": round(fl_idx / s / 1e12 / PEAK_MFMA_BF16_TFLOPS, 4),
                "frac_valu_sigmoid_ceiling": round(pairs * wl.HI / s / PEAK_SIGMOID_PER_S, 4)}

    stages = {
        "ms": {n: round(v, 4) for n, v in stage_ms.items()},
        "indexer_keys": dict(idx_fig(stage_ms["indexer_keys"]), key_write_gbs=round(pairs * 2 / (stage_ms["indexer_keys"] * 1e-3) / 1e9, 1)),
        "indexer_fp32_scores": dict(idx_fig(stage_ms["indexer_fp32_scores"]), score_write_gbs=round(pairs * 4 / (stage_ms["indexer_fp32_scores"] * 1e-3) / 1e9, 1)),
        "indexer_stats_only": idx_fig(stage_ms["indexer_stats_only"]),
        "select_keys": {"algorithmic_gbs": round((pairs * 2 + sum_nsel_st * 4) / (stage_ms["select_keys"] * 1e-3) / 1e9, 1),
                        "frac_hbm_peak": round((pairs * 2 + sum_nsel_st * 4) / (stage_ms["select_keys"] * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)},
        "select_fp32_scores": {"algorithmic_gbs": round((pairs * 4 + sum_nsel_st * 4) / (stage_ms["select_fp32_scores"] * 1e-3) / 1e9, 1),
                               "frac_hbm_peak": round((pairs * 4 + sum_nsel_st * 4) / (stage_ms["select_fp32_scores"] * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)},
        "attention": {"gathered_gbs": round(att_gbs, 1), "tflops": round(fl_att / att_s / 1e12, 2)},
        "sum_n_sel": sum_nsel, "mean_k": round(sum_nsel / queries, 1), "pairs": pairs,
        "sigmoid_ceiling_per_s": PEAK_SIGMOID_PER_S,
    }

    peak_l2 = ceil["l2_resident_2MiB_table"]
    roofline = {
        "kernel": "attn_bf16_kernel (gathered sparse gated attention; one gsa_sparse_gated_attn call over all rows = "
                  "one launch per key window + the window-offset kernel)",
        "bound": "l2-gather",
        "achieved": round(att_gbs, 1), "peak": peak_l2, "unit": "GB/s", "frac": round(att_gbs / peak_l2, 4),
        "peak_source": "whole 256-byte-row gather rate of an L2-resident table, measured in this run with gsa_probe_gather",
        "algorithmic_bytes_per_call": gbytes, "avg_call_ms": round(stage_ms["attention"], 4),
        "hbm": {"compulsory_bytes": compulsory, "achieved": round(compulsory / att_s / 1e9, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                "frac": round(compulsory / att_s / 1e9 / PEAK_HBM_GBS, 4)},
        "hbm_gather_ceiling_gbs": ceil["hbm_resident_4GiB_table"],
        "staged_gather_probe_gbs": ceil["l2_resident_2MiB_table_staged_through_lds"],
        "ratio_to_staged_gather_probe": round(att_gbs / ceil["l2_resident_2MiB_table_staged_through_lds"], 4),
        "staged_gather_probe_note": "the same gather with every row written to LDS and read back once, no arithmetic "
                                    "(gsa_probe_gather_staged, eight waves per CU): what a plain kernel reaches when gathered rows have to "
                                    "pass through LDS, as MFMA operands do; a reference point, not a bound (frac above is against the bound)",
        "traffic": None,
    }
    if isinstance(traffic, dict):
        v_bytes = wl.B * wl.Lk * wl.H_kv * wl.d_h * elt
        f, w_ = traffic["FETCH_SIZE"], traffic["WRITE_SIZE"]
        fscale = 2.0 * v_bytes / f["gate"]          # bytes per counter unit, from the value gate's known reads (V and g2)
        wscale = 1.0 * v_bytes / w_["gate"]         # ... and writes (V')
        fetched, written = f["attn"] * fscale, w_["attn"] * wscale
        roofline["traffic"] = int(fetched + written)
        roofline["traffic_detail"] = {"fetch_bytes": int(fetched), "write_bytes": int(written), "attention_dispatches": f["attn_n"],
                                      "fetch_bytes_per_counter_unit": round(fscale, 1), "write_bytes_per_counter_unit": round(wscale, 1),
                                      "scope": "all attention dispatches of one gsa_forward call at this workspace",
                                      "fabric_bytes_per_compulsory_byte": round((fetched + written) / compulsory, 2),
                                      "fabric_bytes_per_gathered_byte": round((fetched + written) / gbytes, 4)}
    else:
        roofline["traffic_note"] = "%s; see profiles/ for the committed counter summary" % traffic

    result = {
        "metric": "GSA fwd queries/s at 128K ctx" if wl.Lk == 131072 else "GSA fwd queries/s",
        "value": round(queries / (ms_per_step * 1e-3), 1),
        "unit": "queries/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 3), "wall_ms_per_step": round(wall_ms, 3),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": wl.name, "B": wl.B, "Lq": wl.Lq, "Lk": wl.Lk, "H": wl.H, "H_kv": wl.H_kv, "d_h": wl.d_h,
                   "HI": wl.HI, "dI": wl.dI, "k_min": wl.k_min, "k_max": wl.k_max, "k_base": wl.k_base, "vbar": vbar,
                   "workspace_bytes": ws_bytes},
        "tflops": round((fl_idx + fl_att) / (ms_per_step * 1e-3) / 1e12, 2),
        "roofline": roofline,
        "stages": stages,
        "gather_ceilings_gbs": ceil,
        "paper_context": "the paper reports only ratios: 12-16x over dense attention at 128K context, 1.7B model, "
                         "8x H100, precision not stated (abstract, Table 11); no absolute throughput to compare with",
    }
    if one_slab:
        result["one_slab"] = one_slab
    if not args.no_extras and wl.dtype == "bf16":
        print("[bench] comparison variants (dense gated / standard, sparse only) ...", file=sys.stderr, flush=True)
        n_keep = run.n_sel.clone()
        result["comparison"] = comparison_variants(G, S, CM, wl, t, run, ms_per_step)
        run.n_sel = n_keep

    if args.cpu_seconds > 0:
        print("[bench] CPU oracle leg ...", file=sys.stderr, flush=True)
        result["cpu_baseline"] = cpu_baseline(wl, t, ctl_kw, fused["idx"], fused["n_sel"], fused["out"], args.cpu_seconds)
    if not args.no_extras and wl.name == "C4-128k-prefill" and not args.h_kv:
        del t, run, fused
        torch.cuda.empty_cache()
        print("[bench] projections, decode and 16-kv-head legs ...", file=sys.stderr, flush=True)
        result["projections"] = projections_leg(G, S.C4, 2048, dev)
        torch.cuda.empty_cache()
        result["training_c2"] = training_leg(G, S, S.C2, dev)
        torch.cuda.empty_cache()
        result["decode_c5"] = small_leg(G, S, CM, S.C5, 20, 3, args.workspace_gib)
        result["c4_h_kv16"] = small_leg(G, S, CM, S.C4.with_(H_kv=16), 3, 1, args.workspace_gib)
    print(json.dumps(result))


def cpu_baseline(wl, t, ctl_kw, idx_gpu, n_sel_gpu, out_gpu, budget_s):
    """The fp64 oracle, as it stands, on a seeded uniform sample of query rows of the same tensors.
    Rows are independent given vbar, so rows/second over a uniform sample is the oracle's throughput
    on the whole job.  The sampled rows are compared with the timed GPU path's result on the way."""
    import numpy as np
    import torch
    from oracle import gsa_oracle as O
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        threads = os.cpu_count() or 1
    o = {k: (None if v is None else v.to("cpu", torch.float64).numpy()) for k, v in t.items()}
    n_h = n_sel_gpu.cpu().numpy()
    r = np.random.default_rng(12345)
    order = [(int(b), int(i)) for b, i in zip(r.integers(0, wl.B, 4096), r.integers(0, wl.Lq, 4096))]
    done = 0
    same = 0
    worst = 0.0
    spent = 0.0
    for (b, i) in order:
        t0 = time.perf_counter()
        res = O.gsa_forward_row(b, i, o["Q"], o["K"], o["V"], o["g1"], o["g2"], o["qI"], o["kI"], o["w"], None, wl.q_offset, ctl_kw)
        spent += time.perf_counter() - t0          # only the oracle is timed, not the comparison
        done += 1
        m = int(n_h[b, i])
        if res["n_sel"] == m and np.array_equal(res["idx"], idx_gpu[b, i, :m].cpu().numpy()):
            same += 1
            worst = max(worst, float(np.abs(out_gpu[b, i].double().cpu().numpy() - res["out"]).max()))
        if spent > budget_s and done >= 8:
            break
    return {"value": round(done / spent, 3), "unit": "queries/s", "cores": threads, "kind": "oracle",
            "sample": "%d uniformly drawn query rows (seed 12345) of the same tensors, %.1f s" % (done, spent),
            "rows_with_identical_selection": same, "max_abs_err_on_those": worst}


if __name__ == "__main__":
    main()
