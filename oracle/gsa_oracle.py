"""fp64 numpy oracle of the GSA forward path.  TEST INFRASTRUCTURE, not product code.

Each function restates one passage of the paper, in the paper's order and
notation, with no blocking, fusion or reordering.  All arithmetic is float64.
Inputs are the values the GPU sees (already rounded to bf16 / fp32 by the
caller and then widened), so input quantisation is not counted as error.

Shapes (paper symbol -> axis):
  qI [B, Lq, HI, dI]   indexer queries q^I_{t,j}
  kI [B, Lk, dI]       one indexer key k^I_s per token
  w  [B, Lq, HI]       head weights sigma(h_t W^{Iw}_j), i.e. already in (0,1)
  bI [HI] or None      per-head bias b^I_j
  Q  [B, Lq, H, dh]; K, V [B, Lk, Hkv, dh]
  g2 [B, Lk, Hkv, dh]  value-gate logits h_s W^g_V      (None: V is already gated)
  g1 [B, Lq, H, dh]    output-gate logits h_t W^g_{O,h} (None: no output gate)
Query row i has absolute position p = q_offset + i and sees keys s <= min(p, Lk-1)
(self included).

Readings taken where the paper is silent are listed in the design notes of the
repository; the ones that show up here: no 1/sqrt(d^I) factor on the indexer
logit (Eq. "indexer" prints none); population variance over the visible
prefix; floor before clamp; n_sel = min(k_t, #visible); ties go to the lowest
index; one index set per query shared by all heads; kv head of query head h is
h // (H // Hkv).

The moving average Vbar of Sec. 3.4 is an input here (a frozen scalar): the
paper names the average but gives no decay, initial value or update order, so
no update rule is implemented.  Every function of this file is pinned by
tests/test_oracle_pins.py.
"""
import math

import numpy as np


# --------------------------------------------------------------------------- helpers
def sigmoid(z):
    """Logistic function, evaluated without overflow on either side."""
    z = np.asarray(z, dtype=np.float64)
    out = np.empty_like(z)
    pos = z >= 0
    out[pos] = 1.0 / (1.0 + np.exp(-z[pos]))
    ez = np.exp(z[~pos])
    out[~pos] = ez / (1.0 + ez)
    return out


def n_visible(i, q_offset, Lk):
    """Number of keys query row i may look at: s = 0 .. min(q_offset+i, Lk-1)."""
    return min(q_offset + i, Lk - 1) + 1


# --------------------------------------------------------------------------- projections around the path
def linear(x, W):
    """y = x W^T for W stored [out_features, in_features]: the form of every projection of the layer --
    Q, K, V (Sec. 2.1 Eq. 1), q^I and k^I (Sec. 3.3), the gate logits h W^g_V and h W^g_O (Sec. 3.5), and the
    output projection W_O applied to the gated heads (App. B).  x [..., in] -> [..., out]."""
    x = np.asarray(x, np.float64)
    W = np.asarray(W, np.float64)
    out = np.zeros(x.shape[:-1] + (W.shape[0],), np.float64)
    for o in range(W.shape[0]):
        out[..., o] = np.sum(x * W[o], axis=-1)
    return out


def indexer_head_weights(h, W_Iw):
    """w_{t,j} = sigma(h_t W^{Iw}_j) (Sec. 3.3): the per-head weights of the indexer, in (0, 1)."""
    return sigmoid(linear(h, W_Iw))


# --------------------------------------------------------------------------- Sec. 3.3
def indexer_scores_row(qI_t, kI_vis, w_t, bI=None, act="sigmoid"):
    """Eq. "indexer" (Sec. 3.3) for one query: I_{t,s} = sum_j w_{t,j} sigma(q^I_{t,j}.k^I_s + b^I_j).

    act="relu" is the comparison variant of Sec. 2.2 Eq. 3 (the ungated lightning indexer):
    I_{t,s} = sum_j w_{t,j} ReLU(q^I_{t,j}.k^I_s); a bias, if given, is added before the activation there too.

    qI_t [HI, dI], kI_vis [n, dI] (the visible keys only), w_t [HI] -> I [n].
    """
    qI_t = np.asarray(qI_t, np.float64)
    kI_vis = np.asarray(kI_vis, np.float64)
    w_t = np.asarray(w_t, np.float64)
    HI = qI_t.shape[0]
    I = np.zeros(kI_vis.shape[0], np.float64)
    for j in range(HI):
        z = kI_vis @ qI_t[j]
        if bI is not None:
            z = z + float(bI[j])
        if act == "sigmoid":
            I += w_t[j] * sigmoid(z)
        elif act == "relu":
            I += w_t[j] * np.maximum(z, 0.0)
        else:
            raise ValueError("unknown indexer activation: %r" % (act,))
    return I


def row_stats(I_vis):
    """Mean and population variance of the visible scores (Var(I_{t,:}) of Eq. "adaptive_k"), two-pass."""
    I_vis = np.asarray(I_vis, np.float64)
    n = I_vis.shape[0]
    mean = float(np.sum(I_vis) / n)
    var = float(np.sum((I_vis - mean) ** 2) / n)
    return mean, var


def indexer_scores(qI, kI, w, bI=None, q_offset=0, act="sigmoid"):
    """All rows of Sec. 3.3.  Returns scores [B, Lq, Lk] (NaN where the key is not
    visible), row_mean [B, Lq], row_var [B, Lq]."""
    B, Lq, HI, dI = qI.shape
    Lk = kI.shape[1]
    scores = np.full((B, Lq, Lk), np.nan, np.float64)
    mean = np.zeros((B, Lq), np.float64)
    var = np.zeros((B, Lq), np.float64)
    for b in range(B):
        for i in range(Lq):
            n = n_visible(i, q_offset, Lk)
            I = indexer_scores_row(qI[b, i], kI[b, :n], w[b, i], bI, act)
            scores[b, i, :n] = I
            mean[b, i], var[b, i] = row_stats(I)
    return scores, mean, var


# --------------------------------------------------------------------------- Sec. 3.4
def adaptive_k(var, vbar, k_base, k_min, k_max, k_fixed=0, mode=0):
    """Eq. "adaptive_k" (Sec. 3.4): k_t = clamp(floor(k_base * Var / Vbar), k_min, k_max).

    mode 0 is the equation as printed (k_t grows with the variance).  mode 1 is
    the inverse ratio k_base * Vbar / Var, which follows the prose of Sec. 3.4
    (a confident, high-variance query gets a smaller budget); Var = 0 then maps
    to k_max.  k_fixed > 0 switches the controller off.  Returns int64 array.
    """
    var = np.asarray(var, np.float64)
    if k_fixed > 0:
        return np.full(var.shape, int(k_fixed), np.int64)
    if not (vbar > 0 and math.isfinite(vbar)):
        raise ValueError("vbar must be positive and finite")
    if mode == 0:
        r = float(k_base) * var / float(vbar)
    else:
        with np.errstate(divide="ignore"):
            r = np.where(var > 0, float(k_base) * float(vbar) / np.where(var > 0, var, 1.0), np.inf)
    r = np.floor(r)
    r = np.minimum(np.maximum(r, float(k_min)), float(k_max))  # clamp while still floating
    return r.astype(np.int64)


# --------------------------------------------------------------------------- Eq. 4 (Sec. 2.2)
def topk_select_row(I_vis, n_sel):
    """S_t of Eq. 4: indices of the n_sel largest visible scores; equal scores are
    taken lowest index first.  Returned ascending."""
    I_vis = np.asarray(I_vis, np.float64)
    n = I_vis.shape[0]
    n_sel = int(min(n_sel, n))
    # lexsort: last key is primary.  Primary = score descending, secondary = index ascending.
    order = np.lexsort((np.arange(n), -I_vis))
    return np.sort(order[:n_sel]).astype(np.int64)


# --------------------------------------------------------------------------- Sec. 3.5 / 3.6
def sparse_gated_attn_row(Q_t, K, V, g2, g1_t, idx, scale=None):
    """Sec. 3.6 over S_t = idx with the value gate G2 applied to V before aggregation and
    the output gate G1 after it (Sec. 3.5).

    Q_t [H, dh], K/V [Lk, Hkv, dh], g2 [Lk, Hkv, dh] or None, g1_t [H, dh] or None,
    idx ascending int array.  Returns out [H, dh] and A [H, |S|] (the attention weights).
    """
    Q_t = np.asarray(Q_t, np.float64)
    H, dh = Q_t.shape
    Hkv = K.shape[1]
    group = H // Hkv
    if scale is None:
        scale = 1.0 / math.sqrt(dh)
    idx = np.asarray(idx, np.int64)
    out = np.zeros((H, dh), np.float64)
    A_all = np.zeros((H, idx.shape[0]), np.float64)
    if idx.shape[0] == 0:
        return out, A_all
    for h in range(H):
        g = h // group
        Ks = np.asarray(K[idx, g], np.float64)             # [|S|, dh]
        Vs = np.asarray(V[idx, g], np.float64)
        if g2 is not None:
            Vs = Vs * sigmoid(np.asarray(g2[idx, g], np.float64))   # V'_s = V_s * sigma(h_s W^g_V)
        logit = (Ks @ Q_t[h]) * scale
        logit = logit - np.max(logit)
        e = np.exp(logit)
        A = e / np.sum(e)                                   # softmax over S_t only
        O = A @ Vs
        if g1_t is not None:
            O = O * sigmoid(np.asarray(g1_t[h], np.float64))    # O_gated = O_sparse * sigma(h_t W^g_{O,h})
        out[h] = O
        A_all[h] = A
    return out, A_all


# --------------------------------------------------------------------------- training side (Sec. 6.1)
def sparse_gated_attn_bwd_row(Q_t, K, V, g2, g1_t, idx, dout_t, scale=None):
    """Gradients of one query row of Sec. 3.5 / 3.6 (the selection S_t = idx is held fixed: top-k has no
    gradient), for the upstream gradient dout_t [H, dh] of the gated output.  With s_j = scale * q.k_j,
    P = softmax(s), V'_j = V_j * sigma(g2_j), O = sum_j P_j V'_j, out = O * sigma(g1):
        dO   = dout * sigma(g1)                 dg1  = dout * O * sigma(g1) (1 - sigma(g1))
        dP_j = dO . V'_j                        ds_j = P_j (dP_j - sum_i P_i dP_i)
        dq   = scale * sum_j ds_j k_j           dk_j = scale * ds_j q          dV'_j = P_j dO
        dV_j = dV'_j * sigma(g2_j)              dg2_j = dV'_j * V_j * sigma(g2_j) (1 - sigma(g2_j))
    Returns dQ_t [H, dh], dg1_t [H, dh], and dK, dV, dg2 [|S|, Hkv, dh]: the contributions of this row to
    the selected keys (heads of one kv group summed), in the order of idx."""
    Q_t = np.asarray(Q_t, np.float64)
    dout_t = np.asarray(dout_t, np.float64)
    H, dh = Q_t.shape
    Hkv = K.shape[1]
    group = H // Hkv
    if scale is None:
        scale = 1.0 / math.sqrt(dh)
    idx = np.asarray(idx, np.int64)
    n = idx.shape[0]
    dQ = np.zeros((H, dh), np.float64)
    dg1 = np.zeros((H, dh), np.float64)
    dK = np.zeros((n, Hkv, dh), np.float64)
    dV = np.zeros((n, Hkv, dh), np.float64)
    dg2 = np.zeros((n, Hkv, dh), np.float64)
    if n == 0:
        return dQ, dg1, dK, dV, dg2
    for h in range(H):
        g = h // group
        Ks = np.asarray(K[idx, g], np.float64)
        Vs = np.asarray(V[idx, g], np.float64)
        s2 = sigmoid(np.asarray(g2[idx, g], np.float64)) if g2 is not None else np.ones_like(Vs)
        Vp = Vs * s2
        logit = (Ks @ Q_t[h]) * scale
        e = np.exp(logit - np.max(logit))
        P = e / np.sum(e)
        O = P @ Vp
        s1 = sigmoid(np.asarray(g1_t[h], np.float64)) if g1_t is not None else np.ones(dh)
        dO = dout_t[h] * s1
        if g1_t is not None:
            dg1[h] = dout_t[h] * O * s1 * (1.0 - s1)
        dP = Vp @ dO
        ds = P * (dP - np.sum(P * dP))
        dQ[h] = scale * (ds @ Ks)
        dK[:, g] += scale * ds[:, None] * Q_t[h][None, :]
        dVp = P[:, None] * dO[None, :]
        dV[:, g] += dVp * s2
        if g2 is not None:
            dg2[:, g] += dVp * Vs * s2 * (1.0 - s2)
    return dQ, dg1, dK, dV, dg2


def indexer_sparse_kl_row(A, I_sel):
    """Sparse-phase indexer loss of one query (Sec. 6.1, second equation):
        L_t = KL(p_{t,S_t} || softmax(I_{t,S_t})),
    with the target p the attention distribution over S_t, averaged over the query heads (the score has no head
    index) and treated as a constant, and the softmax of the indexer scores taken over S_t.  A [H, |S|] attention
    weights (rows sum to 1), I_sel [|S|] the scores of the selected keys.  Returns the loss and its gradient with
    respect to I_sel, softmax(I_sel) - p.  Terms with p = 0 contribute nothing."""
    A = np.asarray(A, np.float64)
    I_sel = np.asarray(I_sel, np.float64)
    if I_sel.shape[0] == 0:
        return 0.0, np.zeros(0)
    p = A.mean(axis=0)
    z = I_sel - np.max(I_sel)
    logq = z - math.log(np.sum(np.exp(z)))
    pos = p > 0
    loss = float(np.sum(p[pos] * (np.log(p[pos]) - logq[pos])))
    return loss, np.exp(logq) - p


def indexer_scores_bwd_row(qI_t, kI_sel, w_t, bI, dI_sel):
    """Gradients of Eq. "indexer" (Sec. 3.3) for one query, given dL/dI_{t,s} for the keys in kI_sel [|S|, dI]:
        z_{j,s} = q_j . k_s + b_j,   I_s = sum_j w_j sigma(z_{j,s})
        dw_j = sum_s dI_s sigma(z_{j,s})                    dz_{j,s} = dI_s w_j sigma (1 - sigma)
        dq_j = sum_s dz_{j,s} k_s      dk_s = sum_j dz_{j,s} q_j      db_j = sum_s dz_{j,s}
    Returns dqI [HI, dI], dkI [|S|, dI] (this row's contribution), dw [HI], dbI [HI]."""
    q = np.asarray(qI_t, np.float64)
    k = np.asarray(kI_sel, np.float64)
    w = np.asarray(w_t, np.float64)
    d = np.asarray(dI_sel, np.float64)
    z = k @ q.T                                   # [|S|, HI]
    if bI is not None:
        z = z + np.asarray(bI, np.float64)[None, :]
    sg = sigmoid(z)
    dw = d @ sg
    dz = d[:, None] * w[None, :] * sg * (1.0 - sg)
    return dz.T @ k, dz @ q, dw, dz.sum(axis=0)


# --------------------------------------------------------------------------- whole path
def gsa_forward_row(b, i, Q, K, V, g1, g2, qI, kI, w, bI, q_offset, ctl, scale=None, act="sigmoid"):
    """The four stages for one query row (b, i).  ctl: dict(vbar, k_base, k_min, k_max,
    k_fixed, mode).  Returns dict with I, mean, var, k, n_sel, idx, out."""
    Lk = kI.shape[1]
    n = n_visible(i, q_offset, Lk)
    I = indexer_scores_row(qI[b, i], kI[b, :n], w[b, i], bI, act)
    mean, var = row_stats(I)
    k = int(adaptive_k(np.array(var), ctl["vbar"], ctl["k_base"], ctl["k_min"], ctl["k_max"],
                       ctl.get("k_fixed", 0), ctl.get("mode", 0)))
    n_sel = min(k, n)
    idx = topk_select_row(I, n_sel)
    out, _ = sparse_gated_attn_row(Q[b, i], K[b], V[b], None if g2 is None else g2[b],
                                   None if g1 is None else g1[b, i], idx, scale)
    return dict(I=I, mean=mean, var=var, k=k, n_sel=n_sel, idx=idx, out=out)


def gsa_forward(Q, K, V, g1, g2, qI, kI, w, bI, q_offset, ctl, scale=None, k_cap=None):
    """All rows.  Returns out [B,Lq,H,dh], idx [B,Lq,k_cap] (ascending, padded -1),
    n_sel, k, var, mean."""
    B, Lq, H, dh = Q.shape
    if k_cap is None:
        k_cap = int(ctl["k_fixed"]) if ctl.get("k_fixed", 0) > 0 else int(ctl["k_max"])
    out = np.zeros((B, Lq, H, dh), np.float64)
    idx = np.full((B, Lq, k_cap), -1, np.int64)
    n_sel = np.zeros((B, Lq), np.int64)
    k = np.zeros((B, Lq), np.int64)
    var = np.zeros((B, Lq), np.float64)
    mean = np.zeros((B, Lq), np.float64)
    for b in range(B):
        for i in range(Lq):
            r = gsa_forward_row(b, i, Q, K, V, g1, g2, qI, kI, w, bI, q_offset, ctl, scale)
            out[b, i] = r["out"]
            idx[b, i, :r["n_sel"]] = r["idx"]
            n_sel[b, i], k[b, i], var[b, i], mean[b, i] = r["n_sel"], r["k"], r["var"], r["mean"]
    return dict(out=out, idx=idx, n_sel=n_sel, k=k, var=var, mean=mean)


# --------------------------------------------------------------------------- Eq. 2 brute force
def dense_causal_gated_attn(Q, K, V, g1, g2, q_offset=0, scale=None):
    """Eq. 2 (Sec. 2.1) over every visible key, with V replaced by V' (G2) and the G1
    factor on the result: what the sparse path must equal when k_t >= #visible."""
    B, Lq, H, dh = Q.shape
    Lk, Hkv = K.shape[1], K.shape[2]
    group = H // Hkv
    if scale is None:
        scale = 1.0 / math.sqrt(dh)
    out = np.zeros((B, Lq, H, dh), np.float64)
    for b in range(B):
        Vp = np.asarray(V[b], np.float64)
        if g2 is not None:
            Vp = Vp * sigmoid(np.asarray(g2[b], np.float64))
        for i in range(Lq):
            n = n_visible(i, q_offset, Lk)
            for h in range(H):
                g = h // group
                num = np.zeros(dh, np.float64)
                den = 0.0
                logits = [float(np.dot(np.asarray(Q[b, i, h], np.float64), np.asarray(K[b, s, g], np.float64))) * scale
                          for s in range(n)]
                m = max(logits)
                for s in range(n):
                    e = math.exp(logits[s] - m)
                    den += e
                    num += e * Vp[s, g]
                o = num / den
                if g1 is not None:
                    o = o * sigmoid(np.asarray(g1[b, i, h], np.float64))
                out[b, i, h] = o
    return out
