"""Linear-time closed forms that hold for special inputs, driven by a block table; they pin the HIP path on EVERY
element at sizes where the dense fp64 oracle is too slow.  Test infrastructure: numpy only, nothing from the product
but the seeded workload description.  tests/test_oracle_pins.py checks each of them against the oracle on small cases.

Q = 0, or all keys of a sequence identical: every visible score of a row is the same number s_i, so the softmax is
uniform over the row's visible set (n_i keys): LSE_i = s_i + ln n_i, O_i = mean of the visible V,
dV_j = sum over the viewers i of j of dO_i / n_i; with Q = 0 dK = 0; with identical keys dQ = 0 and
dK_j = scale * sum_i [i sees j] (1 / n_i) (dO_i . (v_j - O_i)) q_i.
For one device's share of a table (the backward takes the GLOBAL LSE and O): n_i in the weights becomes the global
count N_i, O_i the global mean, and dQ_i = scale * k * (n_i / N_i) dO_i . (O_i^share - O_i^global)."""
import numpy as np

from oracle import blocks as OB
from paper_2510_10620_amd import workloads as W


def _vis_tile(kind, q0, q1, c0, c1, ranges):
    i = np.arange(q0, q1, dtype=np.int64)[:, None]
    j = np.arange(c0, c1, dtype=np.int64)[None, :]
    if kind == W.MASK_NONE:
        return np.ones((q1 - q0, c1 - c0), dtype=bool)
    if kind == W.MASK_CAUSAL:
        return j <= i
    r = ranges[q0:q1].astype(np.int64)
    return ((j >= r[:, 0:1]) & (j < r[:, 1:2])) | ((j >= r[:, 2:3]) & (j < r[:, 3:4]))


def q0_closed_form(w, table, v64, do64, n_global=None):
    """Uniform-softmax closed form driven by the table: returns n [T], O [T,Hkv,D], dV [T,Hkv,D].
    Counts are exact integers; the tile products run in fp32 (sums of at most a few thousand
    O(1) terms: error ~1e-6, far below the 2e-2 being checked) to keep the full-size check fast."""
    part = OB.block_partition(w.cu_seqlens, w.block_size)
    T, Hkv, D = v64.shape
    G = w.hq // Hkv
    n = np.zeros(T)
    num = np.zeros((T, Hkv * D))
    vflat = v64.reshape(T, Hkv * D).astype(np.float32)
    tiles, vsum, q_add, k_add, dsum = [], {}, {}, {}, {}
    for qb, kb, kind in np.asarray(table, dtype=np.int64):
        if kind == W.MASK_SKIP:
            continue
        q0, q1, c0, c1 = (int(part[k][b]) for k, b in (("blk_start", qb), ("blk_end", qb), ("blk_start", kb), ("blk_end", kb)))
        if kind == W.MASK_NONE:                       # all ones: the tile product is a column sum
            n[q0:q1] += c1 - c0
            if kb not in vsum:
                vsum[kb] = vflat[c0:c1].sum(axis=0, dtype=np.float64)
            q_add[qb] = q_add.get(qb, 0.0) + vsum[kb]
            tiles.append((qb, kb, None))
            continue
        vis = _vis_tile(kind, q0, q1, c0, c1, w.ranges).astype(np.float32)
        n[q0:q1] += vis.sum(axis=1, dtype=np.float64)
        num[q0:q1] += vis @ vflat[c0:c1]
        tiles.append((qb, kb, vis))
    bs, be = part["blk_start"], part["blk_end"]
    for qb, add in q_add.items():
        num[int(bs[qb]):int(be[qb])] += add[None, :]
    O = np.where(n[:, None] > 0, num / np.maximum(n, 1)[:, None], 0.0).reshape(T, Hkv, D)
    ng = n if n_global is None else n_global
    don = (do64 / np.maximum(ng, 1)[:, None, None]).reshape(T, Hkv, G, D).sum(axis=2).reshape(T, Hkv * D)
    don[ng == 0] = 0.0
    don = don.astype(np.float32)
    dV = np.zeros((T, Hkv * D))
    for qb, kb, vis in tiles:
        q0, q1, c0, c1 = int(bs[qb]), int(be[qb]), int(bs[kb]), int(be[kb])
        if vis is None:
            if qb not in dsum:
                dsum[qb] = don[q0:q1].sum(axis=0, dtype=np.float64)
            k_add[kb] = k_add.get(kb, 0.0) + dsum[qb]
        else:
            dV[c0:c1] += vis.T @ don[q0:q1]
    for kb, add in k_add.items():
        dV[int(bs[kb]):int(be[kb])] += add[None, :]
    return n, O, dV.reshape(T, Hkv, D)




def identical_k_dk(w, table, q, v, do, kvh, n_global, o_global):
    """dK [T, D] of KV head `kvh` when all keys of a sequence are identical, for the table rows given (a full table,
    or a share's rows with the global counts n_global [T] and the global output o_global [T, Hkv, D]).
    q, do [T, Hq, D], v [T, Hkv, D].  fp32 tile products (relative error ~1e-6)."""
    part = OB.block_partition(w.cu_seqlens, w.block_size)
    bs, be = part["blk_start"], part["blk_end"]
    T, Hq, D = q.shape
    G = Hq // v.shape[1]
    heads = range(kvh * G, kvh * G + G)
    inv_n = np.where(n_global > 0, 1.0 / np.maximum(n_global, 1), 0.0)
    vk = v[:, kvh].astype(np.float32)
    qn = {h: (q[:, h] * inv_n[:, None]).astype(np.float32) for h in heads}                 # q_i / N_i
    cq = {h: (q[:, h] * ((do[:, h] * o_global[:, kvh]).sum(-1) * inv_n)[:, None]).astype(np.float32) for h in heads}
    dof = {h: do[:, h].astype(np.float32) for h in heads}
    dk = np.zeros((T, D))
    xq, cs = {}, {}   # per (q block, head): sum_i dO_i (x) q_i / N_i  [D, D], and sum_i c_i q_i [D]
    for qb, kb, kind in np.asarray(table, dtype=np.int64):
        if kind == W.MASK_SKIP:
            continue
        q0, q1, c0, c1 = int(bs[qb]), int(be[qb]), int(bs[kb]), int(be[kb])
        vis = None if kind == W.MASK_NONE else _vis_tile(kind, q0, q1, c0, c1, w.ranges).astype(np.float32)
        for h in heads:
            if vis is None:
                if (qb, h) not in xq:
                    xq[(qb, h)] = dof[h][q0:q1].T @ qn[h][q0:q1]
                    cs[(qb, h)] = cq[h][q0:q1].sum(axis=0, dtype=np.float64)
                dk[c0:c1] += vk[c0:c1] @ xq[(qb, h)] - cs[(qb, h)][None, :]
            else:
                a = (dof[h][q0:q1] @ vk[c0:c1].T) * vis
                dk[c0:c1] += a.T @ qn[h][q0:q1] - vis.T @ cq[h][q0:q1]
    return w.softmax_scale * dk
