"""Pins for the CPU oracle: brute force, finite differences, closed forms, invariants, a
library second opinion, and the counts the paper fixes.  No GPU, no HIP code."""
import math
import os

import numpy as np
import pytest

from oracle import attention as A
from oracle import blocks as Bk
from oracle import masks as Mk
from paper_2510_10620_amd import workloads as W

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def mask_rows_fn(spec):
    return lambda s, L, r0, r1: Mk.dense_rows(spec, L, r0, r1)


SPECS = [W.MaskSpec("causal"), W.MaskSpec("window", window=5), W.MaskSpec("lambda", window=4, sink=2),
         W.MaskSpec("causal_blockwise", window=2, sink=1, mblock=3), W.MaskSpec("shared_question")]


def small_case(spec, lens, B, Hq, Hkv, D, seed):
    cu = W.cu_from_lengths(lens)
    rng = np.random.default_rng(seed)
    T = int(cu[-1])
    q = rng.standard_normal((T, Hq, D))
    k = rng.standard_normal((T, Hkv, D))
    v = rng.standard_normal((T, Hkv, D))
    do = rng.standard_normal((T, Hq, D))
    table = Bk.table_from_mask(mask_rows_fn(spec), cu, B)
    ranges = W.attn_ranges(spec, cu)
    return cu, q, k, v, do, table, ranges


# ---------------------------------------------------------------- brute force
def brute_forward(q, k, v, cu, spec, scale):
    """Scalar loops straight from the definition, with the mask taken from the formula."""
    T, Hq, D = q.shape
    G = Hq // k.shape[1]
    O = np.zeros((T, Hq, D))
    LSE = np.full((Hq, T), -math.inf)
    for s in range(len(cu) - 1):
        b, e = int(cu[s]), int(cu[s + 1])
        M = Mk.dense_rows(spec, e - b)
        for h in range(Hq):
            for i in range(b, e):
                sc = {}
                for j in range(b, e):
                    if M[i - b, j - b]:
                        sc[j] = scale * sum(q[i, h, d] * k[j, h // G, d] for d in range(D))
                if not sc:
                    continue
                z = sum(math.exp(x) for x in sc.values())
                LSE[h, i] = math.log(z)
                for j, x in sc.items():
                    p = math.exp(x) / z
                    for d in range(D):
                        O[i, h, d] += p * v[j, h // G, d]
    return O, LSE


@pytest.mark.parametrize("spec", SPECS, ids=lambda s: s.kind)
def test_forward_matches_brute_force(spec):
    cu, q, k, v, do, table, ranges = small_case(spec, [7, 9], 3, 2, 1, 4, seed=11)
    vis = Bk.Visibility(cu, 3, table, ranges)
    O, LSE = A.attention_fwd(q, k, v, cu, vis, 0.5, row_chunk=4)
    Ob, Lb = brute_forward(q, k, v, cu, spec, 0.5)
    np.testing.assert_allclose(O, Ob, atol=1e-12)
    np.testing.assert_allclose(LSE, Lb, atol=1e-12)


@pytest.mark.parametrize("spec", SPECS, ids=lambda s: s.kind)
def test_backward_matches_finite_differences(spec):
    cu, q, k, v, do, table, ranges = small_case(spec, [6, 5], 2, 2, 1, 3, seed=5)
    vis = Bk.Visibility(cu, 2, table, ranges)
    scale = 0.7
    dq, dk, dv = A.attention_bwd(q, k, v, do, cu, vis, scale, row_chunk=3)

    def loss(qq, kk, vv):
        O, _ = brute_forward(qq, kk, vv, cu, spec, scale)
        return float((O * do).sum())

    eps = 1e-6
    for name, x, g in (("q", q, dq), ("k", k, dk), ("v", v, dv)):
        fd = np.zeros_like(x)
        it = np.nditer(x, flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            xp, xm = x.copy(), x.copy()
            xp[idx] += eps
            xm[idx] -= eps
            args_p = [q, k, v]
            args_m = [q, k, v]
            pos = "qkv".index(name)
            args_p[pos], args_m[pos] = xp, xm
            fd[idx] = (loss(*args_p) - loss(*args_m)) / (2 * eps)
        np.testing.assert_allclose(g, fd, atol=2e-8, err_msg=name)


# ---------------------------------------------------------------- invariants
def test_softmax_rows_sum_to_one_and_empty_rows():
    S = np.random.default_rng(0).standard_normal((9, 13)) * 5
    S[3] = -np.inf
    S[5, 4:] = -np.inf
    lse, P = A._softmax_rows(S)
    rows = np.delete(np.arange(9), 3)
    np.testing.assert_allclose(P[rows].sum(axis=1), 1.0, atol=1e-12)
    assert lse[3] == -np.inf and not P[3].any() and not np.isnan(P).any()
    np.testing.assert_allclose(lse[rows], np.log(np.exp(S[rows]).sum(axis=1)), atol=1e-12)


def test_merge_of_per_kv_block_partials_is_unsplit_attention():
    spec = W.MaskSpec("causal")
    cu, q, k, v, do, table, ranges = small_case(spec, [37, 50], 8, 4, 2, 8, seed=3)
    vis = Bk.Visibility(cu, 8, table, ranges)
    O, LSE = A.attention_fwd(q, k, v, cu, vis, 0.3)
    part = Bk.block_partition(cu, 8)
    n_blk = len(part["blk_seq"])
    T = int(cu[-1])
    Om, Lm = np.zeros_like(O), np.full_like(LSE, -np.inf)
    for qb in range(n_blk):
        ents = [e for e in range(len(table)) if table[e, 0] == qb]
        r0, r1 = int(part["blk_start"][qb]), int(part["blk_end"][qb])
        ops, lps = [], []
        for e in ents:
            vs = Bk.Visibility(cu, 8, table, ranges, select=[e])
            s = int(part["blk_seq"][qb])
            Oe, Le = A.attention_fwd(q, k, v, cu, vs, 0.3, seqs=[s])
            ops.append(Oe[r0:r1])
            lps.append(Le[:, r0:r1])
        rng = np.random.default_rng(qb)
        order = rng.permutation(len(ents))
        o1, l1 = A.merge_partials(np.stack([ops[i] for i in order]), np.stack([lps[i] for i in order]))
        Om[r0:r1], Lm[:, r0:r1] = o1, l1
        if len(ents) >= 3:  # merge tree: ((a,b),c...) == flat
            oa, la = A.merge_partials(np.stack(ops[:2]), np.stack(lps[:2]))
            ob, lb = A.merge_partials(np.stack([oa] + ops[2:]), np.stack([la] + lps[2:]))
            np.testing.assert_allclose(ob, o1, atol=1e-12)
            np.testing.assert_allclose(lb, l1, atol=1e-12)
        # a partial with LSE = -inf changes nothing
        o2, l2 = A.merge_partials(np.stack(ops + [np.full_like(ops[0], 7.0)]),
                                  np.stack(lps + [np.full_like(lps[0], -np.inf)]))
        np.testing.assert_allclose(o2, o1, atol=1e-12)
        np.testing.assert_allclose(l2, l1, atol=1e-12)
    np.testing.assert_allclose(Om, O, atol=1e-12)
    np.testing.assert_allclose(Lm, LSE, atol=1e-12)
    assert T == 87


def test_merge_all_empty():
    o, l = A.merge_partials(np.ones((3, 4, 2, 5)), np.full((3, 2, 4), -np.inf))
    assert not o.any() and np.all(l == -np.inf)


def test_fully_masked_blocks_contribute_nothing():
    """SKIP entries and CAUSAL entries above the diagonal leave the result bit-identical."""
    cu = W.cu_from_lengths([20, 13])
    spec = W.MaskSpec("causal")
    _, q, k, v, do, table, ranges = small_case(spec, [20, 13], 4, 2, 2, 4, seed=8)
    dense = Bk.dense_causal_table(cu, 4)                 # includes kv_blk > q_blk, tagged CAUSAL
    skip = table.copy()
    extra = np.array([[0, 4, W.MASK_SKIP], [5, 6, W.MASK_SKIP]], dtype=np.int32)
    with_skip = np.concatenate([skip, extra])
    res = []
    for t in (table, dense, with_skip):
        vis = Bk.Visibility(cu, 4, t, ranges)
        O, L = A.attention_fwd(q, k, v, cu, vis, 0.5)
        g = A.attention_bwd(q, k, v, do, cu, vis, 0.5)
        res.append((O, L) + g)
    for r in res[1:]:
        for a, b in zip(res[0], r):
            assert np.array_equal(a, b)


def test_library_second_opinion_sdpa_and_autograd():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(21)
    L, H, D = 33, 2, 8
    cu = W.cu_from_lengths([L])
    q, k, v, do = (rng.standard_normal((L, H, D)) for _ in range(4))
    table = Bk.table_from_mask(lambda s, L_, r0, r1: np.ones((r1 - r0, L_), bool), cu, 8)
    assert (table[:, 2] == W.MASK_NONE).all()
    vis = Bk.Visibility(cu, 8, table)
    scale = 1 / math.sqrt(D)
    O, LSE = A.attention_fwd(q, k, v, cu, vis, scale)
    dq, dk, dv = A.attention_bwd(q, k, v, do, cu, vis, scale)
    tq, tk, tv = (torch.tensor(x.transpose(1, 0, 2), dtype=torch.float64, requires_grad=True) for x in (q, k, v))
    to = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv)
    to.backward(torch.tensor(do.transpose(1, 0, 2)))
    np.testing.assert_allclose(O, to.detach().numpy().transpose(1, 0, 2), atol=1e-12)
    for g, t in ((dq, tq), (dk, tk), (dv, tv)):
        np.testing.assert_allclose(g, t.grad.numpy().transpose(1, 0, 2), atol=1e-12)
    ref_lse = torch.logsumexp(scale * tq @ tk.transpose(1, 2), dim=-1).detach().numpy()
    np.testing.assert_allclose(LSE, ref_lse, atol=1e-12)
    # causal, GQA, autograd on an explicit masked softmax
    cu2 = W.cu_from_lengths([L])
    ctab = Bk.table_from_mask(mask_rows_fn(W.MaskSpec("causal")), cu2, 8)
    vis2 = Bk.Visibility(cu2, 8, ctab)
    k1, v1 = k[:, :1], v[:, :1]
    O2, _ = A.attention_fwd(q, k1, v1, cu2, vis2, scale)
    g2 = A.attention_bwd(q, k1, v1, do, cu2, vis2, scale)
    tk1, tv1 = (torch.tensor(x.transpose(1, 0, 2), dtype=torch.float64, requires_grad=True) for x in (k1, v1))
    tq2 = torch.tensor(q.transpose(1, 0, 2), dtype=torch.float64, requires_grad=True)
    to2 = torch.nn.functional.scaled_dot_product_attention(tq2, tk1.expand(2, -1, -1), tv1.expand(2, -1, -1), is_causal=True)
    to2.backward(torch.tensor(do.transpose(1, 0, 2)))
    np.testing.assert_allclose(O2, to2.detach().numpy().transpose(1, 0, 2), atol=1e-12)
    for g, t in zip(g2, (tq2, tk1, tv1)):
        np.testing.assert_allclose(g, t.grad.numpy().transpose(1, 0, 2), atol=1e-12)


# ---------------------------------------------------------------- closed forms
def visible_counts(spec, L):
    i = np.arange(L)
    if spec.kind == "causal":
        return i + 1
    if spec.kind == "window":
        return np.minimum(i + 1, spec.window)
    if spec.kind == "lambda":
        return np.minimum(i + 1, spec.window) + np.minimum(spec.sink, np.maximum(i - spec.window + 1, 0))
    raise ValueError


@pytest.mark.parametrize("spec", [W.MaskSpec("causal"), W.MaskSpec("window", window=37),
                                  W.MaskSpec("lambda", window=29, sink=6)], ids=lambda s: s.kind)
def test_closed_form_q_zero_uniform_softmax(spec):
    """Q = 0 makes P uniform on the visible set: LSE = ln n_i, O = mean of visible V,
    dV_j = sum_{i sees j} dO_i / n_i, dK = 0."""
    lens, B, Hq, Hkv, D = [101, 64, 77], 16, 4, 2, 8
    cu, q, k, v, do, table, ranges = small_case(spec, lens, B, Hq, Hkv, D, seed=2)
    q[:] = 0
    vis = Bk.Visibility(cu, B, table, ranges)
    O, LSE = A.attention_fwd(q, k, v, cu, vis, 0.2)
    dq, dk, dv = A.attention_bwd(q, k, v, do, cu, vis, 0.2)
    for s in range(len(lens)):
        b, e = int(cu[s]), int(cu[s + 1])
        n = visible_counts(spec, e - b)
        np.testing.assert_allclose(LSE[:, b:e], np.broadcast_to(np.log(n), (Hq, e - b)), atol=1e-12)
        M = Mk.dense_rows(spec, e - b)
        for h in range(Hq):
            mean_v = (M / n[:, None]) @ v[b:e, h // 2]
            np.testing.assert_allclose(O[b:e, h], mean_v, atol=1e-12)
        for g in range(Hkv):
            ref = sum((M / n[:, None]).T @ do[b:e, h] for h in (2 * g, 2 * g + 1))
            np.testing.assert_allclose(dv[b:e, g], ref, atol=1e-12)
    np.testing.assert_allclose(dk, 0, atol=1e-12)


def test_closed_form_identical_keys():
    """All K rows of a sequence equal: every visible score is s_i = scale q_i.k, so
    LSE_i = s_i + ln n_i and P is uniform again (nonzero scores exercised)."""
    spec = W.MaskSpec("causal")
    cu, q, k, v, do, table, ranges = small_case(spec, [45, 30], 8, 2, 1, 4, seed=4)
    for s in range(2):
        k[cu[s]:cu[s + 1]] = k[cu[s]]
    vis = Bk.Visibility(cu, 8, table, ranges)
    O, LSE = A.attention_fwd(q, k, v, cu, vis, 0.9)
    for s in range(2):
        b, e = int(cu[s]), int(cu[s + 1])
        n = np.arange(1, e - b + 1)
        for h in range(2):
            si = 0.9 * q[b:e, h] @ k[b, 0]
            np.testing.assert_allclose(LSE[h, b:e], si + np.log(n), atol=1e-12)
            np.testing.assert_allclose(O[b:e, h], np.cumsum(v[b:e, 0], axis=0) / n[:, None], atol=1e-12)


def test_backward_invariants():
    spec = W.MaskSpec("lambda", window=9, sink=3)
    cu, q, k, v, do, table, ranges = small_case(spec, [40, 23], 8, 4, 2, 8, seed=9)
    vis = Bk.Visibility(cu, 8, table, ranges)
    dq, dk, dv = A.attention_bwd(q, k, v, do, cu, vis, 0.4)
    # rows of P sum to one => column sums of dV equal the group's summed dO
    for s in range(2):
        b, e = int(cu[s]), int(cu[s + 1])
        for g in range(2):
            np.testing.assert_allclose(dv[b:e, g].sum(axis=0), do[b:e, 2 * g:2 * g + 2].sum(axis=(0, 1)), atol=1e-10)
    # softmax is shift invariant: adding c * k-independent vector to all keys of a sequence leaves O
    # unchanged, hence sum_j dK_j = 0 per (sequence, kv head)
    for s in range(2):
        b, e = int(cu[s]), int(cu[s + 1])
        np.testing.assert_allclose(dk[b:e].sum(axis=0), 0, atol=1e-10)
    # Delta from the final O equals rowsum(P * dP)
    O, _ = A.attention_fwd(q, k, v, cu, vis, 0.4)
    dl = A.delta_rows(O, do)
    dq2, dk2, dv2 = A.attention_bwd(q, k, v, do, cu, vis, 0.4, delta=dl)
    np.testing.assert_allclose(dq2, dq, atol=1e-12)
    np.testing.assert_allclose(dk2, dk, atol=1e-12)


# ---------------------------------------------------------------- block generation
def _golden_rows():
    rows = []
    with open(os.path.join(GOLDEN, "block_counts.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            rows.append([c.strip() for c in line.split("|")])
    return rows


@pytest.mark.parametrize("row", _golden_rows(), ids=lambda r: r[0])
def test_block_counts_fixed_by_the_paper(row):
    name, lens, B, mask, expected = row[0], [int(x) for x in row[1].split(",")], int(row[2]), row[3], int(row[4])
    cu = W.cu_from_lengths(lens)
    part = Bk.block_partition(cu, B)
    n_data = len(part["blk_seq"])
    if name.startswith("data_blocks"):
        assert n_data == expected
    elif name.startswith("hyperedges"):
        assert 3 * n_data == expected
    else:
        spec = W.MaskSpec(mask)
        table = Bk.table_from_mask(mask_rows_fn(spec), cu, B)
        assert len(table) == expected


@pytest.mark.parametrize("spec", [W.MaskSpec("causal"), W.MaskSpec("window", window=50),
                                  W.MaskSpec("lambda", window=40, sink=7),
                                  W.MaskSpec("causal_blockwise", window=2, sink=1, mblock=16),
                                  W.MaskSpec("shared_question")], ids=lambda s: s.kind)
def test_table_defined_mask_equals_formula_mask(spec):
    """Two independent routes to M: the mask formula, and table + per-token ranges."""
    rng = np.random.default_rng(17)
    lens = [int(x) for x in rng.integers(20, 200, size=4)]
    B = 16
    cu = W.cu_from_lengths(lens)
    table = Bk.table_from_mask(mask_rows_fn(spec), cu, B)
    ranges = W.attn_ranges(spec, cu)
    vis = Bk.Visibility(cu, B, table, ranges)
    total = 0
    for s, L in enumerate(lens):
        M = Mk.dense_rows(spec, L)
        assert np.array_equal(vis.rows(s, 0, L), M)
        total += int(M.sum())
        # ranges lie inside the query's own sequence
        r = ranges[cu[s]:cu[s + 1]].astype(np.int64)
        nonempty = r[:, [1, 3]] > r[:, [0, 2]]
        assert (r[:, [0, 2]][nonempty] >= cu[s]).all() and (r[:, [1, 3]][nonempty] <= cu[s + 1]).all()
    assert int(vis.pair_counts().sum()) == total
    # all-zero tiles are never constructed; every listed tile has a visible pair
    assert (vis.pair_counts() > 0).all()


@pytest.mark.parametrize("W_,sink", [(50, 0), (40, 7), (16, 16), (1, 0), (300, 3), (5, 400)])
def test_window_kind_table_equals_formula_mask(W_, sink):
    """A table whose edge tiles carry the WINDOW kind, with (window, sink) as its only parameters, defines the
    sliding-window / lambda mask of Sec. 2.4: checked against the formula-side masks, which know nothing of
    tables, and against the RANGES route on the same specification."""
    rng = np.random.default_rng(23)
    lens = [int(x) for x in rng.integers(20, 200, size=4)] + [1, 16]
    B = 16
    cu = W.cu_from_lengths(lens)
    spec = W.MaskSpec("lambda", window=W_, sink=sink) if sink else W.MaskSpec("window", window=W_)
    table = Bk.table_from_mask(mask_rows_fn(spec), cu, B, other_kind=Bk.MASK_WINDOW)
    assert not (table[:, 2] == Bk.MASK_RANGES).any()
    vis = Bk.Visibility(cu, B, table, window=(W_, sink))
    total = 0
    for s, L in enumerate(lens):
        M = Mk.lambda_mask(L, W_, sink) if sink else Mk.window(L, W_)
        assert np.array_equal(vis.rows(s, 0, L), M)
        total += int(M.sum())
    counts = vis.pair_counts()
    assert int(counts.sum()) == total and (counts > 0).all()
    # same rows, same counts as the RANGES route
    t2 = Bk.table_from_mask(mask_rows_fn(spec), cu, B)
    assert np.array_equal(table[:, :2], t2[:, :2])
    assert np.array_equal(np.where(table[:, 2] == Bk.MASK_WINDOW, Bk.MASK_RANGES, table[:, 2]), t2[:, 2])
    assert np.array_equal(Bk.Visibility(cu, B, t2, W.attn_ranges(spec, cu)).pair_counts(), counts)
    # hand case: 6 tokens, window 3, sink 1 -> row 5 sees keys {0, 3, 4, 5}
    v = Bk.Visibility([0, 6], 2, Bk.table_from_mask(mask_rows_fn(W.MaskSpec("lambda", window=3, sink=1)), [0, 6], 2,
                                                    other_kind=Bk.MASK_WINDOW), window=(3, 1))
    assert v.rows(0, 5, 6)[0].tolist() == [True, False, False, True, True, True]


def test_block_partition_ragged():
    cu = W.cu_from_lengths([5, 8, 1])
    p = Bk.block_partition(cu, 4)
    assert p["seq_first_blk"].tolist() == [0, 2, 4, 5]
    assert p["blk_start"].tolist() == [0, 4, 5, 9, 13]
    assert p["blk_end"].tolist() == [4, 5, 9, 13, 14]
    assert p["blk_seq"].tolist() == [0, 0, 1, 1, 2]


def test_group_entries_csr():
    table = np.array([[2, 0, 0], [0, 0, 1], [2, 2, 1], [1, 0, 3], [2, 1, 0], [1, 1, 1]], dtype=np.int32)
    ptr, idx = Bk.group_entries(table, 0, 3)
    assert ptr.tolist() == [0, 1, 2, 5] and idx.tolist() == [1, 5, 0, 4, 2]
    ptr, idx = Bk.group_entries(table, 1, 3)
    assert ptr.tolist() == [0, 2, 4, 5] and idx.tolist() == [1, 0, 5, 4, 2]


# ---------------------------------------------------------------- shares (one device of a plan)
def test_shares_partition_the_pairs_and_recombine():
    spec = W.MaskSpec("causal")
    lens, B, Hq, Hkv, D = [70, 45, 90], 16, 2, 1, 4
    cu, q, k, v, do, table, ranges = small_case(spec, lens, B, Hq, Hkv, D, seed=13)
    n = len(table)
    vis_full = Bk.Visibility(cu, B, table, ranges)
    O, LSE = A.attention_fwd(q, k, v, cu, vis_full, 0.5)
    dq, dk, dv = A.attention_bwd(q, k, v, do, cu, vis_full, 0.5)
    delta = A.delta_rows(O, do)
    shares = [W.deal_share(n, 8, 205, s) for s in range(8)]
    assert sorted(np.concatenate(shares).tolist()) == list(range(n))
    ops, lps, gq, gk, gv = [], [], 0, 0, 0
    for sel in shares:
        vs = Bk.Visibility(cu, B, table, ranges, select=sel)
        o_s, l_s = A.attention_fwd(q, k, v, cu, vs, 0.5)
        ops.append(o_s)
        lps.append(l_s)
        a, b, c = A.attention_bwd(q, k, v, do, cu, vs, 0.5, lse=LSE, delta=delta)
        gq, gk, gv = gq + a, gk + b, gv + c
    om, lm = A.merge_partials(np.stack(ops), np.stack(lps))
    np.testing.assert_allclose(om, O, atol=1e-12)
    np.testing.assert_allclose(lm, LSE, atol=1e-12)
    np.testing.assert_allclose(gq, dq, atol=1e-12)
    np.testing.assert_allclose(gk, dk, atol=1e-12)
    np.testing.assert_allclose(gv, dv, atol=1e-12)
    # divisions of one share: slots are (division, q_blk) pairs
    sel = shares[0]
    slot, n_slots, slot_q = W.deal_divisions(table[sel, 0], 4, 305)
    assert n_slots == len(set(zip(slot.tolist(), table[sel, 0].tolist())))
    assert all(slot_q[slot[i]] == table[sel[i], 0] for i in range(len(sel)))


def test_bf16_rounding_helper_is_nearest_even_and_exact_on_widening():
    torch = pytest.importorskip("torch")
    x = np.random.default_rng(0).standard_normal(4096).astype(np.float32) * 3
    x[:4] = [1.0, 1.00390625, 1.01171875, -0.0]     # ties
    bits = W.f32_to_bf16_bits(x)
    ref = torch.from_numpy(x).to(torch.bfloat16)
    assert np.array_equal(bits.view(np.int16), ref.view(torch.int16).numpy())
    assert np.array_equal(W.bf16_bits_to_f64(bits), ref.to(torch.float64).numpy())


def test_row_window_matches_full_computation():
    """The query-row window of the oracle (used to sample full-size batches) agrees with the
    full computation on its rows, and its dK/dV are complete for keys only the window sees."""
    spec = W.MaskSpec("lambda", window=30, sink=4)
    cu, q, k, v, do, table, ranges = small_case(spec, [90, 41], 16, 4, 2, 8, seed=23)
    vis = Bk.Visibility(cu, 16, table, ranges)
    O, LSE = A.attention_fwd(q, k, v, cu, vis, 0.3)
    dq, dk, dv = A.attention_bwd(q, k, v, do, cu, vis, 0.3)
    rows = {0: (60, 90)}
    Ow, Lw = A.attention_fwd(q, k, v, cu, vis, 0.3, seqs=[0], rows=rows, row_chunk=7)
    dqw, dkw, dvw = A.attention_bwd(q, k, v, do, cu, vis, 0.3, seqs=[0], rows=rows, row_chunk=7)
    np.testing.assert_allclose(Ow[60:90], O[60:90], atol=1e-12)
    np.testing.assert_allclose(Lw[:, 60:90], LSE[:, 60:90], atol=1e-12)
    np.testing.assert_allclose(dqw[60:90], dq[60:90], atol=1e-12)
    assert np.isnan(Ow[:60]).all() and np.isnan(Ow[90:]).all() and np.isnan(dqw[:60]).all()
    # keys >= 60 are seen only by queries >= 60 (every mask here is causal-bounded)
    np.testing.assert_allclose(dkw[60:90], dk[60:90], atol=1e-12)
    np.testing.assert_allclose(dvw[60:90], dv[60:90], atol=1e-12)


# ------------------------------------------------------------------ block buffers, Blockwise Copy
def _blocks_and_slots(rng, lens, B):
    from oracle import blocks as OB_
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    part = OB_.block_partition(cu, B)
    bs, bl = part["blk_start"], part["blk_end"] - part["blk_start"]
    n_slots = len(bs) + 3
    slots = rng.permutation(n_slots)[:len(bs)].astype(np.int32)
    return cu, np.asarray(bs), np.asarray(bl), slots, n_slots


def test_blockwise_copy_is_row_assignment():
    """Sec. 5 "Blockwise Copy": against numpy's own fancy-index row assignment, and an identity round trip."""
    from oracle import blockbuf as BB
    rng = np.random.default_rng(7)
    src = rng.standard_normal((40, 3, 4))
    entries = np.array([[0, 10, 5], [30, 0, 10], [12, 25, 1], [7, 30, 0]], dtype=np.int32)
    dst = np.full((35, 3, 4), -1.0)
    BB.blockwise_copy(src, dst, entries)
    want = np.full((35, 3, 4), -1.0)
    idx_s = np.concatenate([np.arange(s, s + n) for s, _, n in entries])
    idx_d = np.concatenate([np.arange(d, d + n) for _, d, n in entries])
    want[idx_d] = src[idx_s]
    assert np.array_equal(dst, want)
    assert (dst[15:25] == -1).all() and (dst[26:30] == -1).all()      # rows no entry names stay untouched


def test_block_buffer_gather_scatter_and_copy_lists_agree():
    """Sec. 5 "Block buffers": packed -> buffer -> packed is the identity on the rows blocks use; the copy
    list route (copy_entries_for_blocks + blockwise_copy) equals the direct gather (two code paths)."""
    from oracle import blockbuf as BB
    rng = np.random.default_rng(8)
    B = 6
    cu, bs, bl, slots, n_slots = _blocks_and_slots(rng, [13, 6, 20, 1], B)
    T = int(cu[-1])
    x = rng.standard_normal((T, 2, 3))
    buf = BB.gather_blocks(x, bs, bl, slots, n_slots, B, fill=np.nan)
    assert np.array_equal(BB.scatter_blocks(buf, bs, bl, slots, B, T), x)
    # every buffer row is either a block row or still the fill value, and the counts match
    assert np.isnan(buf).all(axis=(1, 2)).sum() == n_slots * B - T
    to_buf = BB.copy_entries_for_blocks(bs, bl, slots, B, to_buffer=True)
    buf2 = BB.blockwise_copy(x, np.full_like(buf, np.nan), to_buf)
    assert np.array_equal(np.nan_to_num(buf2, nan=-7.0), np.nan_to_num(buf, nan=-7.0))
    back = BB.copy_entries_for_blocks(bs, bl, slots, B, to_buffer=False)
    assert np.array_equal(BB.blockwise_copy(buf2, np.zeros_like(x), back), x)
    # block b, row r sits at slot * B + r
    b = 3
    assert np.array_equal(buf[slots[b] * B + 2], x[bs[b] + 2])
    # [H, T] scalars take the same route
    l = rng.standard_normal((2, T))
    lb = BB.gather_rows_hT(l, bs, bl, slots, n_slots, B, fill=np.inf)
    assert np.array_equal(BB.scatter_rows_hT(lb, bs, bl, slots, B, T), l)
    assert lb[1, slots[b] * B + 2] == l[1, bs[b] + 2]


# ------------------------------------------------------------------ communication volume of a placement
def _sq_example():
    """Sec. 4.1's example: one sequence of 6 tokens, block size 2, shared-question mask (a question and two answers)."""
    from oracle import blocks as OB_, masks as OM_
    cu = np.array([0, 6], dtype=np.int32)
    spec = W.MaskSpec("shared_question", n_answers=2, frac=1.0 / 3.0)
    table = OB_.table_from_mask(lambda s, L, r0, r1: OM_.dense_rows(spec, L, r0, r1), cu, 2)
    return cu, table


def test_comm_volume_paper_example_and_hand_cases():
    from oracle import placement as OP
    cu, table = _sq_example()
    pairs = sorted((int(q), int(k)) for q, k, _ in table)
    assert pairs == [(0, 0), (1, 0), (1, 1), (2, 0), (2, 2)]          # the second answer does not see the first
    blk_len = [2, 2, 2]
    # Sec. 4.2: "Nine hyperedges are built in total" (3 Q + 3 KV + 3 O data blocks)
    r = OP.comm_volume(blk_len, table, [0, 0, 0], [0] * 5, 2, 10, 6, 10)
    assert r["hyperedges"] == 9 and r["pairwise"] == 0 and r["connectivity"] == 0
    # block 2 and its computation on device 1: it fetches KV block 0 once (its own K/V is local)
    r = OP.comm_volume(blk_len, table, [0, 0, 1], [0, 0, 0, 1, 1], 2, 10, 6, 10)
    assert r["pairwise"] == 2 * 6 and r["connectivity"] == 2 * 6 and r["send"] == [12, 0] and r["recv"] == [0, 12]
    # the same tokens, but both computation blocks of Q block 2 run on device 0: Q_2 and KV_2 go to device 0
    # (Q once per hyperedge, twice per computation block) and two partial outputs come back (once per hyperedge)
    r = OP.comm_volume(blk_len, table, [0, 0, 1], [0] * 5, 2, 10, 6, 10)
    assert r["pairwise"] == 2 * (2 * 10 + 2 * 10) + 2 * 6
    assert r["connectivity"] == 2 * 10 + 2 * 6 + 2 * 10
    assert r["send"] == [20, 32] and r["recv"] == [32, 20]


def test_comm_volume_invariants_on_random_placements():
    """connectivity <= pairwise (a device that needs a block for several computation blocks moves it once), equality
    when no (block, remote device) pair repeats; sends and receives balance; one device or data-parallel placement
    (each sequence and its computation on one device) moves nothing."""
    from oracle import placement as OP, blocks as OB_
    rng = np.random.default_rng(12)
    cu = np.array([0, 70, 100, 230], dtype=np.int32)
    table = OB_.dense_causal_table(cu, 16)
    table = table[table[:, 0] >= table[:, 1]]
    part = OB_.block_partition(cu, 16)
    blk_len = part["blk_end"] - part["blk_start"]
    nb = len(blk_len)
    for R in (1, 2, 5):
        blk_dev = rng.integers(0, R, nb)
        comp_dev = rng.integers(0, R, len(table))
        r = OP.comm_volume(blk_len, table, blk_dev, comp_dev, R, 8, 4, 8)
        assert r["connectivity"] <= r["pairwise"]
        assert sum(r["send"]) == sum(r["recv"]) == r["connectivity"]
        assert r["hyperedges"] == 3 * nb
        if R == 1:
            assert r["pairwise"] == 0
        # second opinion on the connectivity: distinct (block, remote device) pairs counted with numpy
        tot = 0
        for col, per_tok in ((0, 8), (1, 4), (0, 8)):
            prs = np.unique(np.stack([table[:, col], comp_dev], axis=1), axis=0)
            tot += sum(int(blk_len[b]) * per_tok for b, d in prs if blk_dev[b] != d)
        assert tot == r["connectivity"]
    dp = part["blk_seq"] % 2                                   # sequence s lives on device s % 2
    r = OP.comm_volume(blk_len, table, dp, dp[table[:, 0]], 2, 8, 4, 8)
    assert r["pairwise"] == 0 and r["connectivity"] == 0
    # computation on the Q owner: only KV moves, each remote (kv, device) pair once per row -> pairwise == rows counted
    owner = rng.integers(0, 3, nb)
    r = OP.comm_volume(blk_len, table, owner, owner[table[:, 0]], 3, 8, 4, 8)
    rows = sum(int(blk_len[k]) * 4 for q, k, _ in table if owner[q] != owner[k])
    assert r["pairwise"] == rows


# ---------------------------------------------------------------- masks.causal_blockwise: hand case at the paper's parameters
def test_causal_blockwise_hand_case_at_the_papers_parameters():
    """Sec. 7.1 "Attention Masks": mask blocks of 256 tokens, a sliding window of 2 blocks, one sink block, and the
    final block (the test sample) attends to everything before it.  Six mask blocks, L = 1536; counts worked out by
    hand from that description: a token of block 0, 1 or 2 sees every earlier token (block 2's window is blocks 1-2
    and block 0 is the sink), a token i of block 3 sees the sink block (256) and blocks 2-3 up to itself (i - 511), a
    token of block 4 the sink and blocks 3-4 up to itself (i - 767), a token of the last block everything (i + 1)."""
    L = 1536
    M = Mk.causal_blockwise(L, 256, 2, 1)
    n = M.sum(axis=1)
    hand = {0: 1, 255: 256, 256: 257, 600: 601, 767: 768, 768: 256 + 257, 1023: 256 + 512, 1024: 256 + 257,
            1279: 256 + 512, 1280: 1281, 1535: 1536}
    for i, c in hand.items():
        assert n[i] == c, (i, n[i], c)
    # rows 0..767: 768 * 769 / 2 = 295 296; blocks 3 and 4: 256 * 256 + (257 + ... + 512) = 163 968 each;
    # last block: 1281 + ... + 1536 = 360 576
    assert int(n.sum()) == 295296 + 2 * 163968 + 360576 == 983808
    # single pairs: a token of block 3 sees the sink and block 2 but not block 1; the test sample sees block 1
    assert M[800, 100] and M[800, 520] and not M[800, 300] and not M[800, 801]
    assert M[1300, 300] and M[1279, 255] and not M[1279, 256] and not M[1279, 767] and M[1279, 768]
    # a ragged sequence: the last, short block (tokens 1280..1399) is the test sample
    M2 = Mk.causal_blockwise(1400, 256, 2, 1)
    assert M2[1399].sum() == 1400 and M2[1280].sum() == 1281 and M2[1279].sum() == 768
    # rows [r0, r1) of the same mask
    assert np.array_equal(Mk.causal_blockwise(L, 256, 2, 1, 700, 1300), M[700:1300])


def test_sum_partials_hand_values():
    parts = np.array([[[1.0, 2.0], [3.0, -4.0]], [[10.0, 20.0], [30.0, 40.0]], [[100.0, 200.0], [300.0, 0.5]]])
    np.testing.assert_array_equal(A.sum_partials(parts), np.array([[111.0, 222.0], [333.0, 36.5]]))
    np.testing.assert_array_equal(A.sum_partials(parts[:1]), parts[0])
    # fp64 accumulation of values an fp32 sum would lose
    np.testing.assert_array_equal(A.sum_partials(np.array([[1e8], [1.0], [-1e8]])), np.array([1.0]))


# ---------------------------------------------------------------- the linear-time closed forms of tests/closed_forms.py
@pytest.mark.parametrize("spec", [W.MaskSpec("causal"), W.MaskSpec("lambda", window=40, sink=9),
                                  W.MaskSpec("causal_blockwise", window=2, sink=1, mblock=16), W.MaskSpec("shared_question")],
                         ids=lambda s: s.kind)
@pytest.mark.parametrize("share", [False, True], ids=["full", "share"])
def test_closed_forms_agree_with_the_oracle(spec, share):
    """The table-driven closed forms that the full-size GPU tests compare every element with (uniform softmax for
    Q = 0 and for identical keys) against the dense oracle on a small ragged batch, for a full table and for one
    device's share of it (global LSE and O)."""
    from tests.closed_forms import identical_k_dk, q0_closed_form
    w = W.custom_workload("cf", [150, 77, 260], 64, 4, 2, 16, "f32", spec, seed=5)
    cu, B, scale = w.cu_seqlens, w.block_size, w.softmax_scale
    rng = np.random.default_rng(77)
    T = w.total_tokens
    q = rng.standard_normal((T, 4, 16))
    v = rng.standard_normal((T, 2, 16))
    do = rng.standard_normal((T, 4, 16))
    k = np.zeros((T, 2, 16))
    for s in range(len(cu) - 1):
        k[cu[s]:cu[s + 1]] = rng.standard_normal((1, 2, 16))           # all keys of a sequence identical
    table = Bk.table_from_mask(mask_rows_fn(spec), cu, B)
    sub = table[W.deal_share(len(table), 3, 11, 0)] if share else table
    vis_full, vis = Bk.Visibility(cu, B, table, w.ranges), Bk.Visibility(cu, B, sub, w.ranges)
    Og, Lg = A.attention_fwd(q, k, v, cu, vis_full, scale)
    O, LSE = A.attention_fwd(q, k, v, cu, vis, scale)
    dq, dk, dv = A.attention_bwd(q, k, v, do, cu, vis, scale, lse=Lg, delta=A.delta_rows(Og, do))
    n_glob, O_glob, _ = q0_closed_form(w, table, v, do)
    n, O_cf, dV_cf = q0_closed_form(w, sub, v, do, n_glob)
    s_i = scale * np.einsum("thd,thd->ht", q, np.repeat(k, 2, axis=1))
    with np.errstate(divide="ignore"):
        np.testing.assert_allclose(LSE, np.where(n > 0, s_i + np.log(n), -np.inf), atol=1e-12)
    np.testing.assert_allclose(O, np.repeat(O_cf, 2, axis=1), atol=1e-5)
    np.testing.assert_allclose(dv, dV_cf, atol=1e-4)
    for kvh in range(2):
        np.testing.assert_allclose(dk[:, kvh], identical_k_dk(w, sub, q, v, do, kvh, n_glob, O_glob), atol=1e-4)
    # dQ: zero for a full table; for a share scale * k * (n / N) dO . (O_share - O_global)
    coef = (n / np.maximum(n_glob, 1))[None, :] * np.einsum("thd,thd->ht", do, np.repeat(O_cf - O_glob, 2, axis=1))
    np.testing.assert_allclose(dq, scale * coef.T[:, :, None] * np.repeat(k, 2, axis=1), atol=1e-5)
    if not share:
        assert np.abs(dq).max() < 1e-5
    # Q = 0 on the same batch: LSE = ln n, same O and dV, dK = 0
    z = np.zeros_like(q)
    O0, L0 = A.attention_fwd(z, k, v, cu, vis, scale)
    _, dk0, dv0 = A.attention_bwd(z, k, v, do, cu, vis, scale, lse=np.where(n_glob > 0, np.log(np.maximum(n_glob, 1)), -np.inf)[None, :].repeat(4, 0),
                                  delta=A.delta_rows(np.repeat(O_glob, 2, axis=1), do))
    np.testing.assert_allclose(O0, np.repeat(O_cf, 2, axis=1), atol=1e-5)
    np.testing.assert_allclose(dv0, dV_cf, atol=1e-4)
    assert np.abs(dk0).max() < 1e-12
