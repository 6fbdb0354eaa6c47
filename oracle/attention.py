"""fp64 dense masked softmax attention, its gradients, and the partial-merge reference.
Test infrastructure (numpy only, no torch, nothing shared with the HIP path).

Definitions followed:
  * Sec. 2.1, masked self-attention: O = RowSoftmax((Q K^T [masked by M]) / sqrt(D)) V.  The
    boolean mask removes unwanted interactions; masked pairs are excluded from the softmax
    (score -inf, probability 0) -- the paper states the attention algorithm is unchanged.
  * Listing 1, line 6 "RescaleAndSum" (online-softmax merge of per-KV-block partials):
    LSE = ln sum_p exp(LSE_p);  O = sum_p exp(LSE_p - LSE) O_p.
  * Backward: the analytic gradient of L = sum(O * dO) through the definition above
    (the paper gives no backward algorithm; this is the textbook softmax-attention gradient).

Layouts: q, o, do, dq [T, Hq, D]; k, v, dk, dv [T, Hkv, D]; lse, delta [Hq, T]; query head h
reads KV head h // (Hq / Hkv).  Sequences are packed along T by cu_seqlens.
`vis.rows(s, r0, r1)` supplies the dense bool visibility of query rows [r0, r1) of sequence s.
"""
import numpy as np


def _scores(qh, kg, scale, M):
    S = scale * (qh @ kg.T)
    return np.where(M, S, -np.inf)


def _softmax_rows(S):
    """Row-wise log-sum-exp and probabilities; a row with no finite entry gives lse=-inf, P=0."""
    m = S.max(axis=1, initial=-np.inf)
    m_safe = np.where(np.isfinite(m), m, 0.0)
    E = np.exp(S - m_safe[:, None])            # exp(-inf) = 0 for masked entries
    l = E.sum(axis=1)
    with np.errstate(divide="ignore"):
        lse = np.where(l > 0, m_safe + np.log(l), -np.inf)
    P = np.where(l[:, None] > 0, E / np.where(l > 0, l, 1.0)[:, None], 0.0)
    return lse, P


def _row_span(rows, s, L):
    """Query-row window [r0, r1) of sequence s: the whole sequence unless `rows` (a dict
    sequence -> (r0, r1)) narrows it."""
    if rows is None or s not in rows:
        return 0, L
    r0, r1 = rows[s]
    return max(0, int(r0)), min(L, int(r1))


def attention_fwd(q, k, v, cu_seqlens, vis, scale, seqs=None, row_chunk=2048, rows=None):
    """Returns (O [T,Hq,D], LSE [Hq,T]).  Sequences not in `seqs`, and query rows outside the
    window `rows[s]`, are left NaN."""
    q, k, v = (np.asarray(a, dtype=np.float64) for a in (q, k, v))
    T, Hq, D = q.shape
    G = Hq // k.shape[1]
    cu = np.asarray(cu_seqlens, dtype=np.int64)
    O = np.full((T, Hq, D), np.nan)
    LSE = np.full((Hq, T), np.nan)
    for s in (range(len(cu) - 1) if seqs is None else seqs):
        b, e = int(cu[s]), int(cu[s + 1])
        w0, w1 = _row_span(rows, s, e - b)
        for r0 in range(w0, w1, row_chunk):
            r1 = min(w1, r0 + row_chunk)
            M = vis.rows(s, r0, r1)
            for h in range(Hq):
                S = _scores(q[b + r0:b + r1, h], k[b:e, h // G], scale, M)
                lse, P = _softmax_rows(S)
                O[b + r0:b + r1, h] = P @ v[b:e, h // G]
                LSE[h, b + r0:b + r1] = lse
    return O, LSE


def delta_rows(o, do):
    """Delta[h, t] = sum_d dO[t,h,d] * O[t,h,d]  (uses the final, merged O)."""
    return np.einsum("thd,thd->ht", np.asarray(o, np.float64), np.asarray(do, np.float64))


def attention_bwd(q, k, v, do, cu_seqlens, vis, scale, lse=None, delta=None, seqs=None,
                  row_chunk=2048, rows=None):
    """Gradients (dQ, dK, dV) of sum(O * dO).

    With lse/delta None they are derived from `vis` itself (plain full attention).  For one
    device's share of the computation blocks, pass the *global* LSE and Delta (of the merged
    output) and a `vis` restricted to the share: P = exp(S - LSE) on the share's visible pairs,
    dV = P^T dO, dP = dO V^T, dS = P * (dP - Delta), dQ = scale dS K, dK = scale dS^T Q; the
    KV-head gradients sum over the query heads of the group.  Sequences not in `seqs` stay NaN.
    With a query-row window `rows[s]`, dQ is filled for those rows only and dK / dV hold the
    contributions of those query rows only (complete for a key all of whose viewers lie inside)."""
    q, k, v, do = (np.asarray(a, dtype=np.float64) for a in (q, k, v, do))
    T, Hq, D = q.shape
    Hkv = k.shape[1]
    G = Hq // Hkv
    cu = np.asarray(cu_seqlens, dtype=np.int64)
    dq = np.full((T, Hq, D), np.nan)
    dk = np.full((T, Hkv, D), np.nan)
    dv = np.full((T, Hkv, D), np.nan)
    for s in (range(len(cu) - 1) if seqs is None else seqs):
        b, e = int(cu[s]), int(cu[s + 1])
        dk[b:e] = 0.0
        dv[b:e] = 0.0
        w0, w1 = _row_span(rows, s, e - b)
        for r0 in range(w0, w1, row_chunk):
            r1 = min(w1, r0 + row_chunk)
            M = vis.rows(s, r0, r1)
            sl = slice(b + r0, b + r1)
            for h in range(Hq):
                g = h // G
                S = _scores(q[sl, h], k[b:e, g], scale, M)
                if lse is None:
                    row_lse, P = _softmax_rows(S)
                else:
                    row_lse = np.asarray(lse, np.float64)[h, sl]
                    fin = np.isfinite(row_lse)
                    P = np.where(fin[:, None], np.exp(S - np.where(fin, row_lse, 0.0)[:, None]), 0.0)
                dP = do[sl, h] @ v[b:e, g].T
                if delta is None:
                    dl = (P * dP).sum(axis=1)          # equals sum_d dO*O for the full softmax
                else:
                    dl = np.asarray(delta, np.float64)[h, sl]
                dS = P * (dP - dl[:, None])
                dq[sl, h] = scale * (dS @ k[b:e, g])
                dk[b:e, g] += scale * (dS.T @ q[sl, h])
                dv[b:e, g] += P.T @ do[sl, h]
    return dq, dk, dv


def merge_partials(o_parts, lse_parts):
    """RescaleAndSum (Listing 1, line 6).  o_parts [P, n, H, D], lse_parts [P, H, n] ->
    (O [n,H,D], LSE [H,n]).  A partial with LSE=-inf has weight 0; all -inf gives O=0, LSE=-inf."""
    o_parts = np.asarray(o_parts, dtype=np.float64)
    lse_parts = np.asarray(lse_parts, dtype=np.float64)
    m = lse_parts.max(axis=0)
    m_safe = np.where(np.isfinite(m), m, 0.0)
    w = np.exp(lse_parts - m_safe[None])                 # [P,H,n], 0 where lse_p = -inf
    tot = w.sum(axis=0)
    with np.errstate(divide="ignore"):
        lse = np.where(tot > 0, m_safe + np.log(tot), -np.inf)
    wn = np.where(tot[None] > 0, w / np.where(tot > 0, tot, 1.0)[None], 0.0)
    o = np.einsum("phn,pnhd->nhd", wn, np.nan_to_num(o_parts, nan=0.0))
    return o, lse


def sum_partials(parts):
    """Gradient reduction across blocks: plain sum of partials that target the same block."""
    return np.asarray(parts, dtype=np.float64).sum(axis=0)
