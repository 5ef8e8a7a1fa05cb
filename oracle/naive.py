"""Pure-Python restatement of the GSA forward path for tiny cases.  TEST INFRASTRUCTURE.

Written with explicit loops over every index and ``math`` scalars only, so it
shares no vectorised expression with ``gsa_oracle``.  Inputs are nested lists
or arrays indexed ``x[b][t][...]``; outputs are nested lists.
"""
import math


def _sig(z):
    if z >= 0.0:
        return 1.0 / (1.0 + math.exp(-z))
    e = math.exp(z)
    return e / (1.0 + e)


def indexer_scores(qI, kI, w, bI, q_offset, B, Lq, Lk, HI, dI, relu=False):
    """Sec. 3.3: I[b][t][s] for visible s (list of length n per row); relu=True: Sec. 2.2 Eq. 3 instead."""
    out = []
    for b in range(B):
        rows = []
        for t in range(Lq):
            n = min(q_offset + t, Lk - 1) + 1
            row = []
            for s in range(n):
                acc = 0.0
                for j in range(HI):
                    z = 0.0
                    for c in range(dI):
                        z += float(qI[b][t][j][c]) * float(kI[b][s][c])
                    if bI is not None:
                        z += float(bI[j])
                    acc += float(w[b][t][j]) * ((z if z > 0.0 else 0.0) if relu else _sig(z))
                row.append(acc)
            rows.append(row)
        out.append(rows)
    return out


def variance(row):
    """Population variance of a list (Sec. 3.4)."""
    n = len(row)
    m = 0.0
    for x in row:
        m += x
    m /= n
    v = 0.0
    for x in row:
        v += (x - m) * (x - m)
    return v / n


def adaptive_k(var, vbar, k_base, k_min, k_max, mode=0):
    """Sec. 3.4, one scalar."""
    if mode == 0:
        r = k_base * var / vbar
    else:
        r = math.inf if var <= 0.0 else k_base * vbar / var
    r = math.floor(r) if math.isfinite(r) else r
    if r < k_min:
        r = k_min
    if r > k_max:
        r = k_max
    return int(r)


def topk(row, n_sel):
    """Eq. 4 by repeated arg-max: strictly-greater comparison keeps the lowest index on ties."""
    n = len(row)
    n_sel = min(n_sel, n)
    taken = [False] * n
    chosen = []
    for _ in range(n_sel):
        best = -1
        for s in range(n):
            if taken[s]:
                continue
            if best < 0 or row[s] > row[best]:
                best = s
        taken[best] = True
        chosen.append(best)
    chosen.sort()
    return chosen


def sparse_gated_attn(Q_t, K, V, g2, g1_t, idx, H, Hkv, dh, scale=None):
    """Sec. 3.5-3.6 for one query; returns out[h][c]."""
    if scale is None:
        scale = 1.0 / math.sqrt(dh)
    group = H // Hkv
    out = []
    for h in range(H):
        g = h // group
        logits = []
        for s in idx:
            acc = 0.0
            for c in range(dh):
                acc += float(Q_t[h][c]) * float(K[s][g][c])
            logits.append(acc * scale)
        m = max(logits)
        es = [math.exp(x - m) for x in logits]
        den = 0.0
        for e in es:
            den += e
        o = [0.0] * dh
        for a, s in zip(es, idx):
            p = a / den
            for c in range(dh):
                v = float(V[s][g][c])
                if g2 is not None:
                    v *= _sig(float(g2[s][g][c]))
                o[c] += p * v
        if g1_t is not None:
            for c in range(dh):
                o[c] *= _sig(float(g1_t[h][c]))
        out.append(o)
    return out
