"""Operation and byte counts of the GSA forward path (host-side bookkeeping for reports).

The closed forms are those of the complexity theorem (Sec. 5.1, Thm. 1), its
corollary (Cor. 2) and the breakdown in App. A; the exact counts use the
causal pair count and the realised selection sizes instead of L^2 and L*k.
"""


def speedup_vs_dense(d, dI, HI, k, L):
    """App. A, "Speedup Factor": (d / (d^I H^I)) / (1 + k d / (L d^I H^I))."""
    return (d / (dI * HI)) / (1.0 + (k * d) / (L * dI * HI))


def indexer_cost_ratio(dI, HI, d, n_h):
    """App. A item 2: d^I H^I / (d n_h), the indexer's cost relative to full attention as printed there."""
    return (dI * HI) / (d * n_h)


def causal_pairs(B, Lq, Lk, q_offset):
    """Number of (query, visible key) pairs: query i sees min(q_offset+i, Lk-1)+1 keys."""
    total = 0
    full_from = max(0, Lk - 1 - q_offset)        # rows i >= full_from see all Lk keys
    m = min(Lq, full_from)
    # rows 0..m-1 see q_offset+i+1 keys
    total += m * (q_offset + 1) + m * (m - 1) // 2
    total += (Lq - m) * Lk
    return B * total


def indexer_flops(pairs, HI, dI):
    """Multiply-adds of the indexer contraction, 2 flops each (Thm. 1 term L^2 d^I H^I)."""
    return 2 * dI * HI * pairs


def attention_flops(sum_n_sel, H, d_h):
    """QK^T and PV over the selected keys, 2 flops per multiply-add (Thm. 1 term L k d)."""
    return 4 * d_h * H * sum_n_sel


def gathered_bytes(sum_n_sel, H_kv, d_h, elt_bytes, gate_in_kernel=False):
    """Bytes of K and V' rows the sparse attention must fetch: one K row and one V row of
    H_kv*d_h elements per (query, selected key); a third row when G2 logits are gathered too."""
    rows = 3 if gate_in_kernel else 2
    return rows * H_kv * d_h * elt_bytes * sum_n_sel
