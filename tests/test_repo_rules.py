"""Structural rules of the repository that can be checked without a GPU: the product never touches
the CPU oracle, bench.py refuses more than one GPU, the pins really catch planted mistakes."""
import importlib
import importlib.util
import os
import re
import subprocess
import sys

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_product_does_not_use_the_oracle():
    pkg = os.path.join(ROOT, "paper_2601_15305_amd")
    for dirpath, _, files in os.walk(pkg):
        if "_build" in dirpath:
            continue
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f), errors="replace").read()
                assert not re.search(r"^\s*(from|import)\s+oracle\b", text, re.M), f
                assert "oracle/" not in text and "gsa_oracle" not in text, f
    # and the oracle never imports the product
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith(".py"):
            text = open(os.path.join(ROOT, "oracle", f)).read()
            assert "paper_2601_15305_amd" not in text and "ctypes" not in text, f


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "one GPU" in r.stderr


# ---- planted mistakes: each plausible slip in the oracle must trip at least one pin ---------------------
def _run_pins(monkeypatch_fn):
    """Run a few pin tests in-process with the oracle patched; return the names of the pins that fail."""
    spec = importlib.util.spec_from_file_location("pins_under_mutation", os.path.join(ROOT, "tests", "test_oracle_pins.py"))
    P = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(P)
    failed = []
    pins = [n for n in dir(P) if n.startswith("test_") and "cost_model" not in n]
    for n in pins:
        try:
            getattr(P, n)()
        except AssertionError:
            failed.append(n)
        except Exception:
            failed.append(n)
    return failed


MUTANTS = {
    "sigmoid sign": ("sigmoid", lambda O: (lambda z: 1.0 - O._orig_sigmoid(z))),
    "variance with n-1": ("row_stats", lambda O: (lambda I: (float(np.mean(I)), float(np.var(I, ddof=1)) if len(I) > 1 else 0.0))),
    "ties to the highest index": ("topk_select_row", lambda O: (
        lambda I, m: np.sort(np.lexsort((-np.arange(len(I)), -np.asarray(I, float)))[:min(int(m), len(I))]).astype(np.int64))),
    "smallest instead of largest": ("topk_select_row", lambda O: (
        lambda I, m: np.sort(np.lexsort((np.arange(len(I)), np.asarray(I, float)))[:min(int(m), len(I))]).astype(np.int64))),
    "ceil instead of floor": ("adaptive_k", lambda O: (
        lambda var, vbar, kb, kmin, kmax, k_fixed=0, mode=0: (
            np.full(np.shape(var), int(k_fixed), np.int64) if k_fixed > 0 else
            (_ for _ in ()).throw(ValueError()) if not vbar > 0 else
            np.clip(np.ceil(kb * np.asarray(var, float) / vbar), kmin, kmax).astype(np.int64)))),
    "no self in the visible set": ("n_visible", lambda O: (lambda i, off, Lk: max(1, min(off + i, Lk - 1)))),
}


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_pins_catch_planted_mistake(name, monkeypatch):
    sys.path.insert(0, ROOT)
    from oracle import gsa_oracle as O
    attr, make = MUTANTS[name]
    if not hasattr(O, "_orig_sigmoid"):
        O._orig_sigmoid = O.sigmoid
    monkeypatch.setattr(O, attr, make(O))
    failed = _run_pins(None)
    assert failed, "no pin noticed: " + name
