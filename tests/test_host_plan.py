"""Host-side logic of the C-ABI library (no GPU needed): symbols, block generation, pair counts,
plan groupings bit-exact against the oracle's integer reference, and every error path."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2510_10620_amd as P
from oracle import blocks as OB
from oracle import masks as OM
from paper_2510_10620_amd import _lib
from paper_2510_10620_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    with open(os.path.join(ROOT, "include", "dcp.h")) as f:
        src = f.read()
    declared = set(re.findall(r"\b(dcp_[a-z_]+)\s*\(", src))
    lib = ctypes.CDLL(_lib.LIB_PATH)
    assert declared, "no declarations found"
    for name in declared:
        assert hasattr(lib, name), f"{name} declared in dcp.h but not exported"
    assert declared == set(_lib.exported_names())
    assert P.dcp_version().startswith("dcp_attn")


@pytest.mark.parametrize("seed", range(8))
def test_block_table_from_arbitrary_ranges_bit_exact_vs_oracle(seed):
    """Range arrays no mask family produces: per token two random ranges inside its sequence, either of them possibly
    empty, overlapping, the second before the first, and blocks of rows that all see a whole KV block through one range
    or through none (the cases the generator settles from the bounds of a block's rows without looking at the rows)."""
    rng = np.random.default_rng(500 + seed)
    lens = [int(x) for x in rng.integers(1, 260, size=4)]
    B = int(rng.choice([8, 16, 32]))
    cu = W.cu_from_lengths(lens)
    T = int(cu[-1])
    ranges = np.zeros((T, 4), dtype=np.int32)
    dense = {}
    for s, L in enumerate(lens):
        s0 = int(cu[s])
        m = np.zeros((L, L), dtype=bool)
        base = rng.integers(0, L + 1, size=4)              # a block-wide pattern, so that whole blocks are covered or missed
        for i in range(L):
            r = np.sort(rng.integers(0, L + 1, size=2)), np.sort(rng.integers(0, L + 1, size=2))
            mode = int(rng.integers(0, 4))
            if mode == 0:                                  # the shared pattern
                r = np.sort(base[:2]), np.sort(base[2:])
            elif mode == 1:                                # first range empty
                r = (np.array([0, 0]), r[1])
            elif mode == 2:                                # everything through one range
                r = (np.array([0, L]), np.array([0, 0]))
            for k in range(2):
                ranges[s0 + i, 2 * k], ranges[s0 + i, 2 * k + 1] = s0 + r[k][0], s0 + r[k][1]
                m[i, r[k][0]:r[k][1]] = True
        dense[s] = m
    want = OB.table_from_mask(lambda s, L, r0, r1: dense[s][r0:r1], cu, B)
    got = P.dcp_build_block_table(cu, B, ranges)
    assert np.array_equal(got, want)


def test_bench_refuses_more_than_one_gpu():
    """bench.py measures one GPU: asked for more it must say so and exit, before it touches a device."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0 and "one GPU" in r.stderr and r.stdout.strip() == ""


def _oracle_table(spec, cu, B):
    return OB.table_from_mask(lambda s, L, r0, r1: OM.dense_rows(spec, L, r0, r1), cu, B)


SPECS = [W.MaskSpec("causal"), W.MaskSpec("window", window=90), W.MaskSpec("lambda", window=70, sink=9),
         W.MaskSpec("causal_blockwise", window=2, sink=1, mblock=24), W.MaskSpec("shared_question")]


@pytest.mark.parametrize("spec", SPECS, ids=lambda s: s.kind)
@pytest.mark.parametrize("B", [1, 16, 37])
def test_block_table_bit_exact_vs_oracle(spec, B):
    rng = np.random.default_rng(B)
    lens = [int(x) for x in rng.integers(1, 40 if B == 1 else 300, size=5)]
    cu = W.cu_from_lengths(lens)
    ranges = W.attn_ranges(spec, cu)
    got = P.dcp_build_block_table(cu, B, ranges)
    ref = _oracle_table(spec, cu, B)
    assert got.dtype == np.int32 and np.array_equal(got, ref)
    pc = P.dcp_count_pairs(cu, B, got, ranges)
    assert np.array_equal(pc, OB.Visibility(cu, B, ref, ranges).pair_counts())


@pytest.mark.parametrize("cfg", [2, 3, 4, 5, 6, 7, 8])
def test_block_table_full_size_configs(cfg):
    w = W.make_workload(cfg)
    got = P.dcp_build_block_table(w.cu_seqlens, w.block_size, w.ranges)
    ref = _oracle_table(w.mask, w.cu_seqlens, w.block_size)
    assert np.array_equal(got, ref)
    part = OB.block_partition(w.cu_seqlens, w.block_size)
    plan = P.dcp_plan_create(w.cu_seqlens, w.block_size, got)
    assert np.array_equal(plan.export("BLK_START"), part["blk_start"])
    assert np.array_equal(plan.export("BLK_LEN"), part["blk_end"] - part["blk_start"])
    # visible-pair totals from closed forms of the mask families
    total = 0
    for s in range(len(w.cu_seqlens) - 1):
        L = int(w.cu_seqlens[s + 1] - w.cu_seqlens[s])
        i = np.arange(L, dtype=np.int64)
        if w.mask.kind == "causal":
            total += int((i + 1).sum())
        elif w.mask.kind == "window":
            total += int(np.minimum(i + 1, w.mask.window).sum())
        elif w.mask.kind in ("causal_blockwise", "shared_question"):
            # no one-line closed form: count the formula-side dense mask (pinned by hand cases) in row chunks
            for r0 in range(0, L, 2048):
                total += int(OM.dense_rows(w.mask, L, r0, min(L, r0 + 2048)).sum())
        else:
            total += int((np.minimum(i + 1, w.mask.window) + np.minimum(w.mask.sink, np.maximum(i - w.mask.window + 1, 0))).sum())
    assert int(P.dcp_count_pairs(w.cu_seqlens, w.block_size, got, w.ranges).sum()) == total


def test_plan_groupings_bit_exact_vs_oracle():
    rng = np.random.default_rng(7)
    lens = [150, 64, 33, 200]
    B = 32
    cu = W.cu_from_lengths(lens)
    spec = W.MaskSpec("lambda", window=60, sink=10)
    table = _oracle_table(spec, cu, B)
    table = table[rng.permutation(len(table))]            # arbitrary row order
    table[::7, 2] = W.MASK_SKIP                            # some rows dropped
    part = OB.block_partition(cu, B)
    nb = len(part["blk_seq"])
    plan = P.dcp_plan_create(cu, B, table)
    assert np.array_equal(plan.export("BLK_SEQ"), part["blk_seq"])
    for col, ptr_name, idx_name in ((0, "FWD_PTR", "FWD_IDX"), (0, "BWDQ_PTR", "BWDQ_IDX"), (1, "BWDKV_PTR", "BWDKV_IDX")):
        ptr, idx = OB.group_entries(table, col, nb)
        assert np.array_equal(plan.export(ptr_name), ptr), ptr_name
        assert np.array_equal(plan.export(idx_name), idx), idx_name
    # with output slots: forward units are the slots
    keep = np.arange(len(table))
    slot, n_slots, slot_q = W.deal_divisions(table[:, 0], 3, 99)
    plan2 = P.dcp_plan_create(cu, B, table, slot, n_slots + 2)   # two slots nobody uses
    ptr, idx = OB.group_entries(table, 0, n_slots + 2, group_of=slot)
    assert np.array_equal(plan2.export("FWD_PTR"), ptr)
    assert np.array_equal(plan2.export("FWD_IDX"), idx)
    sq = np.full(n_slots + 2, -1, dtype=np.int64)
    for e in keep:
        if table[e, 2] != W.MASK_SKIP:
            sq[slot[e]] = table[e, 0]
    assert np.array_equal(plan2.export("SLOT_QBLK"), sq)
    mptr, midx = plan2.export("MERGE_PTR"), plan2.export("MERGE_IDX")
    for b in range(nb):
        assert midx[mptr[b]:mptr[b + 1]].tolist() == [s for s in range(n_slots + 2) if sq[s] == b]
    # bwd groupings ignore slots
    ptr, idx = OB.group_entries(table, 1, nb)
    assert np.array_equal(plan2.export("BWDKV_IDX"), idx)


@pytest.mark.parametrize("spec,lens,B,hkv", [
    (W.MaskSpec("causal"), [5000, 300, 1200], 256, 2),                       # a long sequence: early key tiles see far more
    (W.MaskSpec("causal_blockwise", window=2, sink=1, mblock=64), [4096, 700], 128, 4),   # sink keys seen by every query
    (W.MaskSpec("causal"), [100], 128, 1),                                     # one block, one table row: nothing to cut
])
def test_dkv_work_list_is_an_exact_partition(spec, lens, B, hkv):
    """Every (kv_blk, 128-key tile) appears either once, whole, with pslot -1, or as parts whose table-row ranges
    tile the block's CSR range in order without gap or overlap, with consecutive slots nobody else uses."""
    cu = W.cu_from_lengths(lens)
    table = _oracle_table(spec, cu, B)
    plan = P.dcp_plan_create(cu, B, table)
    items = P.dcp_plan_export_dkv_items(plan, hkv)
    ptr = plan.export("BWDKV_PTR")
    blk_len = plan.export("BLK_LEN")
    by_tile = {}
    for u, t, e0, e1, ps in items.tolist():
        by_tile.setdefault((u, t), []).append((e0, e1, ps))
    want = {(u, t) for u in range(len(blk_len)) if ptr[u + 1] > ptr[u] for t in range((blk_len[u] + 127) // 128)}
    assert set(by_tile) == want
    slots = []
    n_split = 0
    for (u, t), parts in by_tile.items():
        parts.sort()
        assert parts[0][0] == ptr[u] and parts[-1][1] == ptr[u + 1]
        for (a0, a1, _), (b0, b1, _) in zip(parts, parts[1:]):
            assert a1 == b0
        assert all(e1 > e0 for e0, e1, _ in parts)
        if len(parts) == 1:
            assert parts[0][2] == -1
        else:
            n_split += 1
            ps = [p for _, _, p in parts]
            assert ps == list(range(ps[0], ps[0] + len(ps)))     # table-row order = slot order = summation order
            slots += ps
    assert sorted(slots) == list(range(len(slots)))
    if len(lens) > 1:
        assert n_split > 0            # the long items of these workloads are cut
    else:
        assert n_split == 0
    # the workspace grows by the partial sums: 2 x 128 x 128 fp32 per slot and KV head
    base = P.dcp_bwd_workspace_bytes(plan, 4 * hkv, hkv, 64, P.DCP_BF16)       # D = 64: scalar kernels, no partial sums
    full = P.dcp_bwd_workspace_bytes(plan, 4 * hkv, hkv, 128, P.DCP_BF16)
    assert full - base == len(slots) * hkv * 2 * 128 * 128 * 4


@pytest.mark.parametrize("hkv", [1, 2, 3, 4, 6, 8, 12, 16])
def test_dkv_work_list_segments_balance_the_xcds(hkv):
    """With KV heads that are no multiple of 8 an XCD takes (KV head, segment) pairs: the segments must cover the work
    list in order, keep every sequence that is small against a segment in one of them, and hold about equal numbers
    of visible (query, key) pairs (counted here from the sequence lengths: a causal key tile is seen by the queries
    from its first key on)."""
    w = W.make_workload(2)                      # 65 536 causal tokens in 23 sequences of 512 .. 12 K
    cu, B = w.cu_seqlens, w.block_size
    table = P.dcp_build_block_table(cu, B, w.ranges)
    plan = P.dcp_plan_create(cu, B, table)
    items = P.dcp_plan_export_dkv_items(plan, hkv)
    n_seg, seg = P.dcp_plan_export_dkv_segments(plan, hkv)
    assert n_seg == 8 // np.gcd(8, hkv)
    assert seg[0] == 0 and seg[n_seg] == len(items) and np.all(np.diff(seg) >= 0) and np.all(seg[n_seg:] == len(items))
    if n_seg == 1:
        return
    blk_start, blk_len, blk_seq = plan.export("BLK_START"), plan.export("BLK_LEN"), plan.export("BLK_SEQ")
    ptr, idx = plan.export("BWDKV_PTR"), plan.export("BWDKV_IDX")
    kv_of_unit = [u for u in range(len(blk_len))]            # BWDKV CSR: unit = kv_blk
    cost = np.zeros(len(items))
    seq_of = np.zeros(len(items), dtype=np.int64)
    for i, (u, t, e0, e1, ps) in enumerate(items.tolist()):
        kb = kv_of_unit[u]
        k0 = blk_start[kb] + 128 * t
        k1 = min(k0 + 128, blk_start[kb] + blk_len[kb])
        seq_of[i] = blk_seq[kb]
        for e in range(e0, e1):
            qb = table[idx[e], 0]
            q0, q1 = blk_start[qb], blk_start[qb] + blk_len[qb]
            ks = np.arange(k0, k1)
            cost[i] += np.sum(q1 - np.maximum(q0, ks)) if table[idx[e], 2] == P.DCP_MASK_CAUSAL else (q1 - q0) * (k1 - k0)
    per_seg = np.array([cost[seg[s]:seg[s + 1]].sum() for s in range(n_seg)])
    assert per_seg.max() <= 1.10 * per_seg.mean(), per_seg / per_seg.mean()
    # sequences that are at most half a segment stay whole
    seq_cost = np.bincount(seq_of, weights=cost)
    seg_of_item = np.searchsorted(seg[1:n_seg + 1], np.arange(len(items)), side="right")
    for q in np.unique(seq_of):
        if seq_cost[q] <= 0.45 * per_seg.mean():
            assert len(set(seg_of_item[seq_of == q])) == 1, f"sequence {q} is spread over several segments"


@pytest.mark.parametrize("window,sink", [(50, 0), (40, 7), (16, 16), (1, 0), (300, 3), (5, 400)])
def test_window_table_and_pair_counts_bit_exact_vs_oracle(window, sink):
    rng = np.random.default_rng(29)
    lens = [int(x) for x in rng.integers(20, 200, size=4)] + [1, 16]
    B = 16
    cu = W.cu_from_lengths(lens)
    spec = W.MaskSpec("lambda", window=window, sink=sink) if sink else W.MaskSpec("window", window=window)
    want = OB.table_from_mask(lambda s, L, r0, r1: OM.dense_rows(spec, L, r0, r1), cu, B, other_kind=OB.MASK_WINDOW)
    got = P.dcp_build_block_table_window(cu, B, window, sink)
    assert np.array_equal(got, want)
    counts = OB.Visibility(cu, B, want, window=(window, sink)).pair_counts()
    assert np.array_equal(P.dcp_count_pairs_window(cu, B, got, window, sink), counts)


def test_window_kind_error_paths():
    cu = W.cu_from_lengths([64, 64])
    t_win = np.array([[0, 0, P.DCP_MASK_WINDOW], [1, 1, P.DCP_MASK_CAUSAL]], dtype=np.int32)
    plan = P.dcp_plan_create(cu, 64, t_win)
    assert _status(P.dcp_plan_set_window, plan, 0, 0) == P.DCP_ERR_INVALID_ARG
    assert _status(P.dcp_plan_set_window, plan, 5, -1) == P.DCP_ERR_INVALID_ARG
    P.dcp_plan_set_window(plan, 5, 2)
    mixed = np.array([[0, 0, P.DCP_MASK_WINDOW], [1, 1, P.DCP_MASK_RANGES]], dtype=np.int32)
    assert _status(P.dcp_plan_create, cu, 64, mixed) == P.DCP_ERR_BAD_TABLE
    assert _status(P.dcp_plan_create, cu, 64, np.array([[0, 0, 5]], dtype=np.int32)) == P.DCP_ERR_BAD_TABLE
    assert _status(P.dcp_build_block_table_window, cu, 64, 0, 0) == P.DCP_ERR_INVALID_ARG
    assert _status(P.dcp_count_pairs_window, cu, 64, mixed, 5, 0) == P.DCP_ERR_BAD_TABLE
    assert _status(P.dcp_count_pairs, cu, 64, t_win) == P.DCP_ERR_BAD_TABLE      # WINDOW rows need the window counter


@pytest.mark.parametrize("seed", range(12))
def test_random_plans_groupings_and_work_lists(seed):
    """Random lengths, block sizes, mask families, row orders, SKIP rows and head counts: the CSR groupings equal the
    oracle's, and the dK/dV work list is an exact partition of every (kv_blk, tile)'s table rows whatever gets cut."""
    rng = np.random.default_rng(1000 + seed)
    lens = [int(x) for x in rng.integers(1, 900, size=int(rng.integers(1, 7)))]
    B = int(rng.choice([16, 48, 128, 256]))
    spec = [W.MaskSpec("causal"), W.MaskSpec("window", window=int(rng.integers(1, 300))),
            W.MaskSpec("lambda", window=int(rng.integers(1, 200)), sink=int(rng.integers(1, 40))),
            W.MaskSpec("causal_blockwise", window=2, sink=1, mblock=int(rng.choice([8, 32, 96]))),
            W.MaskSpec("shared_question")][seed % 5]
    cu = W.cu_from_lengths(lens)
    table = _oracle_table(spec, cu, B)
    table = table[rng.permutation(len(table))]
    if len(table) > 3:
        table[rng.choice(len(table), size=len(table) // 5, replace=False), 2] = W.MASK_SKIP
    nb = len(OB.block_partition(cu, B)["blk_seq"])
    plan = P.dcp_plan_create(cu, B, table)
    for col, ptr_name, idx_name in ((0, "FWD_PTR", "FWD_IDX"), (0, "BWDQ_PTR", "BWDQ_IDX"), (1, "BWDKV_PTR", "BWDKV_IDX")):
        ptr, idx = OB.group_entries(table, col, nb)
        assert np.array_equal(plan.export(ptr_name), ptr), ptr_name
        assert np.array_equal(plan.export(idx_name), idx), idx_name
    hkv = int(rng.choice([1, 2, 8]))
    items = P.dcp_plan_export_dkv_items(plan, hkv)
    ptr, blk_len = plan.export("BWDKV_PTR"), plan.export("BLK_LEN")
    by_tile = {}
    for u, t, e0, e1, ps in items.tolist():
        by_tile.setdefault((u, t), []).append((e0, e1, ps))
    # every tile of every block is there, also of blocks no kept row lists as kv_blk: their dK / dV rows get zeros
    assert set(by_tile) == {(u, t) for u in range(nb) for t in range((blk_len[u] + 127) // 128)}
    slots = []
    for (u, t), parts in by_tile.items():
        parts.sort()
        assert parts[0][0] == ptr[u] and parts[-1][1] == ptr[u + 1]
        assert all(a[1] == b[0] for a, b in zip(parts, parts[1:]))
        assert all(e1 > e0 for e0, e1, _ in parts) or (len(parts) == 1 and ptr[u] == ptr[u + 1])
        if len(parts) == 1:
            assert parts[0][2] == -1
        else:
            ps = [p for _, _, p in parts]
            assert ps == list(range(ps[0], ps[0] + len(ps)))
            slots += ps
    assert sorted(slots) == list(range(len(slots)))
    assert P.dcp_bwd_workspace_bytes(plan, 4 * hkv, hkv, 128, P.DCP_BF16) - P.dcp_bwd_workspace_bytes(plan, 4 * hkv, hkv, 64, P.DCP_BF16) \
        == len(slots) * hkv * 2 * 128 * 128 * 4


def _status(fn, *a, **k):
    with pytest.raises(P.DcpError) as ei:
        fn(*a, **k)
    assert str(ei.value) and P.dcp_last_error()
    return ei.value.status


def test_error_paths():
    cu = W.cu_from_lengths([10, 6])
    ok = np.array([[0, 0, 1], [2, 2, 1]], dtype=np.int32)       # B=8: blocks 0,1 | 2
    P.dcp_plan_create(cu, 8, ok)
    P.dcp_plan_create(cu, 8, np.zeros((0, 3), np.int32))          # empty table is legal
    assert _status(P.dcp_plan_create, np.array([1, 5], np.int32), 8, ok) == P.DCP_ERR_BAD_CU_SEQLENS
    assert _status(P.dcp_plan_create, np.array([0, 5, 5], np.int32), 8, ok) == P.DCP_ERR_BAD_CU_SEQLENS
    assert _status(P.dcp_plan_create, cu, 0, ok) == P.DCP_ERR_INVALID_ARG
    assert _status(P.dcp_plan_create, cu, 8, np.array([[0, 3, 0]], np.int32)) == P.DCP_ERR_BAD_TABLE     # id out of range
    assert _status(P.dcp_plan_create, cu, 8, np.array([[-1, 0, 0]], np.int32)) == P.DCP_ERR_BAD_TABLE
    assert _status(P.dcp_plan_create, cu, 8, np.array([[0, 2, 0]], np.int32)) == P.DCP_ERR_BAD_TABLE     # two sequences
    assert _status(P.dcp_plan_create, cu, 8, np.array([[0, 0, 5]], np.int32)) == P.DCP_ERR_BAD_TABLE     # bad kind
    assert _status(P.dcp_plan_create, cu, 8, np.array([[1, 0, 0], [1, 0, 1]], np.int32)) == P.DCP_ERR_BAD_TABLE  # duplicate
    P.dcp_plan_create(cu, 8, np.array([[1, 0, 0], [1, 0, 3]], np.int32))                                  # SKIP duplicate is ignored
    two = np.array([[0, 0, 1], [1, 0, 0]], np.int32)
    assert _status(P.dcp_plan_create, cu, 8, two, np.array([0, 0], np.int32), 1) == P.DCP_ERR_BAD_TABLE  # slot with two q_blks
    assert _status(P.dcp_plan_create, cu, 8, two, np.array([0, 2], np.int32), 2) == P.DCP_ERR_BAD_TABLE  # slot out of range
    assert _status(P.dcp_count_pairs, cu, 8, np.array([[0, 0, 2]], np.int32), None) == P.DCP_ERR_INVALID_ARG
    lib = _lib.load()
    n = ctypes.c_int64()
    rg = W.attn_ranges(W.MaskSpec("causal"), cu)
    small = np.zeros((1, 3), np.int32)
    st = lib.dcp_build_block_table(cu.ctypes.data_as(_lib.i32p), 2, 8, rg.ctypes.data_as(_lib.i32p),
                                   small.ctypes.data_as(_lib.i32p), 1, ctypes.byref(n))
    assert st == P.DCP_ERR_INVALID_ARG and n.value == 4
    assert lib.dcp_plan_destroy(None) == 0


def test_share_dealing_is_a_partition_with_valid_slots():
    w = W.make_workload(5)
    table = P.dcp_build_block_table(w.cu_seqlens, w.block_size, w.ranges)
    n_shares, share_seed, n_div, div_seed = w.share
    sels = [W.deal_share(len(table), n_shares, share_seed, s) for s in range(n_shares)]
    assert sorted(np.concatenate(sels).tolist()) == list(range(len(table)))
    sub = table[sels[0]]
    slot, n_slots, slot_q = W.deal_divisions(sub[:, 0], n_div, div_seed)
    plan = P.dcp_plan_create(w.cu_seqlens, w.block_size, sub, slot, n_slots)
    assert np.array_equal(plan.export("SLOT_QBLK"), slot_q)
    mptr = plan.export("MERGE_PTR")
    assert (np.diff(mptr) <= n_div).all() and mptr[-1] == n_slots


# ------------------------------------------------------------------ Blockwise Copy list (host side)
def _copy_err(entries, src_rows, dst_rows):
    with pytest.raises(P.DcpError) as e:
        P.CopyList(entries, src_rows, dst_rows)
    return e.value


def test_copy_list_validation():
    P.CopyList(np.zeros((0, 3), np.int32), 0, 0).close()
    P.CopyList([[0, 5, 5], [5, 0, 5], [3, 10, 0]], 10, 10).close()
    assert _copy_err([[0, 0, -1]], 4, 4).status == P.DCP_ERR_BAD_TABLE
    assert _copy_err([[-1, 0, 1]], 4, 4).status == P.DCP_ERR_BAD_TABLE
    assert _copy_err([[2, 0, 3]], 4, 4).status == P.DCP_ERR_BAD_TABLE          # reads past the source
    assert _copy_err([[0, 2, 3]], 4, 4).status == P.DCP_ERR_BAD_TABLE          # writes past the destination
    assert _copy_err([[0, 0, 3], [4, 2, 2]], 8, 8).status == P.DCP_ERR_BAD_TABLE  # destinations overlap
    assert _copy_err([[0, 0, 1]], -1, 4).status == P.DCP_ERR_INVALID_ARG


def test_block_buffer_slot_validation():
    cu = np.array([0, 100, 150], dtype=np.int32)
    table = OB.dense_causal_table(cu, 32)                 # 4 + 2 blocks
    table = table[table[:, 0] >= table[:, 1]]
    def plan():
        return P.dcp_plan_create(cu, 32, table)
    ok = np.arange(6, dtype=np.int32)
    P.dcp_plan_set_block_buffers(plan(), ok[::-1].copy(), 6, ok, 9)
    for q_slot, nq, kv_slot, nk in ((np.array([0, 1, 2, 3, 4, 6]), 6, ok, 6),      # out of range
                                    (np.array([0, 1, 2, 3, 4, 4]), 6, ok, 6),      # two blocks in one slot
                                    (ok, 6, np.array([0, 1, 2, 3, 4, -1]), 6),     # a used block is absent
                                    (np.array([0, 1, 2, 3, 4, -2]), 6, ok, 6)):
        with pytest.raises(P.DcpError) as e:
            P.dcp_plan_set_block_buffers(plan(), np.asarray(q_slot, np.int32), nq, np.asarray(kv_slot, np.int32), nk)
        assert e.value.status == P.DCP_ERR_BAD_TABLE
    with pytest.raises(P.DcpError) as e:
        P.dcp_plan_set_block_buffers(plan(), ok, -1, ok, 6)
    assert e.value.status == P.DCP_ERR_INVALID_ARG
    # a block no row uses may be absent
    sub = table[(table[:, 0] != 5) & (table[:, 1] != 5)]
    pl = P.dcp_plan_create(cu, 32, sub)
    s5 = ok.copy(); s5[5] = -1
    P.dcp_plan_set_block_buffers(pl, s5, 6, s5, 6)


# ------------------------------------------------------------------ communication volume (host side)
@pytest.mark.parametrize("spec", SPECS, ids=lambda s: s.kind)
def test_comm_volume_matches_oracle(spec):
    from oracle import placement as OP
    rng = np.random.default_rng(13)
    cu = W.cu_from_lengths([150, 37, 260])
    B = 24
    table = _oracle_table(spec, cu, B)
    skip = np.array([[0, 0, 3]], dtype=np.int32)            # a SKIP row is no computation block
    table = np.concatenate([table, skip])
    part = OB.block_partition(cu, B)
    blk_len = part["blk_end"] - part["blk_start"]
    for R in (1, 3, 8):
        blk_dev = rng.integers(0, R, len(blk_len)).astype(np.int32)
        comp_dev = rng.integers(0, R, len(table)).astype(np.int32)
        got = P.dcp_comm_volume(cu, B, table, blk_dev, comp_dev, R, 8192, 4096, 8320)
        ref = OP.comm_volume(blk_len, table, blk_dev, comp_dev, R, 8192, 4096, 8320)
        assert got == ref


def test_comm_volume_errors():
    cu = np.array([0, 64], dtype=np.int32)
    table = np.array([[0, 0, 1], [1, 0, 0], [1, 1, 1]], dtype=np.int32)
    ok = dict(blk_dev=np.array([0, 1], np.int32), comp_dev=np.array([0, 1, 1], np.int32))
    P.dcp_comm_volume(cu, 32, table, ok["blk_dev"], ok["comp_dev"], 2, 1, 1, 1)
    for kw, code in ((dict(blk_dev=np.array([0, 2], np.int32)), P.DCP_ERR_BAD_TABLE),
                     (dict(comp_dev=np.array([0, 1, -1], np.int32)), P.DCP_ERR_BAD_TABLE)):
        a = dict(ok); a.update(kw)
        with pytest.raises(P.DcpError) as e:
            P.dcp_comm_volume(cu, 32, table, a["blk_dev"], a["comp_dev"], 2, 1, 1, 1)
        assert e.value.status == code
    with pytest.raises(P.DcpError) as e:
        P.dcp_comm_volume(cu, 32, np.array([[2, 0, 0]], np.int32), ok["blk_dev"], np.array([0], np.int32), 2, 1, 1, 1)
    assert e.value.status == P.DCP_ERR_BAD_TABLE
    with pytest.raises(P.DcpError) as e:
        P.dcp_comm_volume(cu, 32, table, ok["blk_dev"], ok["comp_dev"], 0, 1, 1, 1)
    assert e.value.status == P.DCP_ERR_INVALID_ARG


# ------------------------------------------------------------------ execution plans (host-side validation)
def test_program_validation():
    from paper_2510_10620_amd import _lib as L
    P.Program([]).close()
    w1, w2 = P.instr_comm_wait(0), P.instr_comm_wait(3)
    for bad in ([w1],):                                   # wait before any launch
        with pytest.raises(P.DcpError) as e:
            P.Program(bad)
        assert e.value.status == P.DCP_ERR_INVALID_ARG
    ins = L.Instr()
    ins.op = 99
    with pytest.raises(P.DcpError):
        P.Program([ins])
    ins = L.Instr()
    ins.op = P.OP_ATTN_FWD                                # no plan
    with pytest.raises(P.DcpError):
        P.Program([ins])
    ins = L.Instr()
    ins.op, ins.comm_id = P.OP_COMM_LAUNCH, 0             # no copy list
    with pytest.raises(P.DcpError):
        P.Program([ins])
    assert w2.comm_id == 3
