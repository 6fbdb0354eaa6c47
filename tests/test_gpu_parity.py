"""Parity of the HIP path (through the C ABI) against the fp64 oracle, element by element, on
seeded inputs small enough for the oracle yet spanning several kernel tiles and ragged tails."""
import numpy as np
import pytest

from oracle import attention as OA
from oracle import blocks as OB
from paper_2510_10620_amd import workloads as W
from tests import helpers as H

pytestmark = pytest.mark.gpu

ALL = ("out", "lse", "dq", "dk", "dv")
IMPLS = {"scalar": 1, "auto": 0}


def run_case(w, table, impl, out_slot=None, n_slots=0, label=""):
    import paper_2510_10620_amd as P
    tensors = W.make_tensors(w)
    # the library's own block generation must agree with the oracle's table bit for bit
    if not w.dense_causal_table and out_slot is None:
        assert np.array_equal(P.dcp_build_block_table(w.cu_seqlens, w.block_size, w.ranges), table)
    g = H.GpuRun(w, tensors, table, out_slot, n_slots, impl)
    out, lse = g.forward()
    dq, dk, dv = g.backward()
    got = dict(out=out, lse=lse, dq=dq, dk=dk, dv=dv)
    ref = H.oracle_full(w, tensors, table)
    H.check(w, got, ref, ALL, label)
    return g, got, ref


def test_config1_tiny_causal_fp32():
    """Config 1: 1 head, D 64, fp32, lengths 128 + 384, block 64, all 40 same-sequence pairs CAUSAL."""
    w = W.make_workload(1)
    table = H.oracle_table(w)
    assert len(table) == 40 and (table[:, 2] == W.MASK_CAUSAL).all()
    run_case(w, table, 0, label="config1")


SPECS = [W.MaskSpec("causal"), W.MaskSpec("window", window=200), W.MaskSpec("lambda", window=150, sink=20),
         W.MaskSpec("causal_blockwise", window=2, sink=1, mblock=96), W.MaskSpec("shared_question")]


@pytest.mark.parametrize("impl", list(IMPLS), ids=list(IMPLS))
@pytest.mark.parametrize("spec", SPECS, ids=lambda s: s.kind)
def test_small_bf16_all_masks(spec, impl):
    w = W.custom_workload("small", [300, 77, 1000, 1, 130], 128, 4, 2, 128, "bf16", spec, seed=31, input_scale=0.5)
    table = H.oracle_table(w)
    g, _, _ = run_case(w, table, IMPLS[impl], label=f"{spec.kind}/{impl}")
    if impl == "auto":
        # the 1000-token sequence's key tiles are long items for so small a launch: the run above went through split
        # dK/dV items, their fp32 partial sums and the reduce kernel
        import paper_2510_10620_amd as P
        assert (P.dcp_plan_export_dkv_items(g.plan, w.hkv)[:, 4] >= 0).any()


@pytest.mark.parametrize("impl", list(IMPLS), ids=list(IMPLS))
@pytest.mark.parametrize("window,sink", [(200, 0), (150, 20), (40, 300), (1, 1)])
def test_window_kind_rows_need_no_range_array(window, sink, impl):
    """Sliding window / lambda masks through WINDOW rows: the library gets two numbers, no range array, and must
    produce what the oracle computes for the mask that table defines (and the same table as the oracle's)."""
    import paper_2510_10620_amd as P
    spec = W.MaskSpec("lambda", window=window, sink=sink) if sink else W.MaskSpec("window", window=window)
    w = W.custom_workload("small_window", [300, 77, 1000, 1, 130], 128, 4, 2, 128, "bf16", spec, seed=33, input_scale=0.5)
    table = OB.table_from_mask(lambda s, L, r0, r1: H.OM.dense_rows(w.mask, L, r0, r1), w.cu_seqlens, w.block_size,
                               other_kind=OB.MASK_WINDOW)
    assert (table[:, 2] == OB.MASK_WINDOW).any()
    assert np.array_equal(P.dcp_build_block_table_window(w.cu_seqlens, w.block_size, window, sink), table)
    tensors = W.make_tensors(w)
    g = H.GpuRun(w, tensors, table, impl=IMPLS[impl], window=(window, sink))
    out, lse = g.forward()
    dq, dk, dv = g.backward()
    ref = H.oracle_full(w, tensors, table, window=(window, sink))
    # window 1 + sink 1: every query gives the sink key a weight near 1/2, so that key's dK / dV rows are sums of a
    # thousand large terms that cancel (|dV| up to 70 beside elements near 0); the rounding of P and dS to bf16
    # before the second GEMM costs about 2^-9 * sqrt(2000) * |term| in every element of the row: dK and dV of this one
    # case are bounded by row (the raw errors are printed)
    H.check(w, dict(out=out, lse=lse, dq=dq, dk=dk, dv=dv), ref, ALL, f"window-kind {window}/{sink}/{impl}",
            by_row=("dk", "dv") if window == 1 else ())


@pytest.mark.parametrize("seed", range(6))
def test_random_small_cases(seed):
    """Random lengths (ragged, some below a tile), block size, head counts, mask family and table row order."""
    rng = np.random.default_rng(2000 + seed)
    lens = [int(x) for x in rng.integers(1, 700, size=int(rng.integers(1, 6)))]
    B = int(rng.choice([32, 64, 128, 256]))
    hq, hkv = [(4, 2), (8, 2), (4, 4)][seed % 3]
    spec = [W.MaskSpec("causal"), W.MaskSpec("window", window=int(rng.integers(1, 300))),
            W.MaskSpec("lambda", window=int(rng.integers(1, 200)), sink=int(rng.integers(1, 40))),
            W.MaskSpec("causal_blockwise", window=2, sink=1, mblock=int(rng.choice([8, 32, 96]))),
            W.MaskSpec("shared_question")][int(rng.integers(0, 5))]
    w = W.custom_workload("random", lens, B, hq, hkv, 128, "bf16", spec, seed=40 + seed, input_scale=0.5)
    table = H.oracle_table(w)
    table = table[rng.permutation(len(table))]
    tensors = W.make_tensors(w)
    g = H.GpuRun(w, tensors, table, impl=IMPLS["auto"])
    out, lse = g.forward()
    dq, dk, dv = g.backward()
    H.check(w, dict(out=out, lse=lse, dq=dq, dk=dk, dv=dv), H.oracle_full(w, tensors, table), ALL,
            f"random {seed}: lens {lens} B {B} {hq}/{hkv} {spec.kind}")


@pytest.mark.parametrize("dtype,d", [("bf16", 64), ("bf16", 32), ("f32", 128), ("f32", 32)])
def test_shapes_only_the_scalar_family_covers(dtype, d):
    """dtype / head-dim pairs outside the MFMA family (bf16, D 128): AUTO must pick the scalar kernels and be right."""
    w = W.custom_workload("scalar_shapes", [210, 75], 64, 4, 2, d, dtype, W.MaskSpec("lambda", window=60, sink=5), seed=37,
                          input_scale=0.5)
    run_case(w, H.oracle_table(w), IMPLS["auto"], label=f"{dtype}/D{d}")


@pytest.mark.parametrize("hq,hkv", [(2, 2), (8, 1), (6, 2), (6, 3), (12, 12), (16, 16)])
def test_head_group_sizes(hq, hkv):
    """Query heads per KV head other than the benchmark's 4: 1 (no sharing), 8 and 3 (not a power of two); and KV head
    counts that divide the work among the XCDs in every way there is: 1, 2 and 3 (lists in 8, 4 and 8 segments,
    one, one and three (head, segment) pairs per XCD), 12 (two segments, three pairs) and 16 (two whole heads)."""
    w = W.custom_workload("groups", [333, 200], 128, hq, hkv, 128, "bf16", W.MaskSpec("lambda", window=90, sink=9), seed=35,
                          input_scale=0.5)
    run_case(w, H.oracle_table(w), IMPLS["auto"], label=f"hq{hq}/hkv{hkv}")


def test_library_loaded_before_torch_touches_the_gpu():
    """A fresh process that calls a host function of the binding (which loads the library) before anything has
    imported torch must still find the GPU afterwards: the loader imports torch first so that the process holds one
    HIP runtime.  One child process, one small forward."""
    import os
    import subprocess
    import sys
    code = (
        "import sys; sys.path.insert(0, %r)\n"
        "import paper_2510_10620_amd as P\n"
        "from paper_2510_10620_amd import workloads as W\n"
        "w = W.custom_workload('x', [300], 128, 4, 2, 128, 'bf16', W.MaskSpec('causal'), seed=1, input_scale=0.5)\n"
        "table = P.dcp_build_block_table(w.cu_seqlens, w.block_size, w.ranges)\n"
        "import torch\n"
        "q = torch.randn((300, 4, 128), device='cuda').to(torch.bfloat16); k = torch.randn((300, 2, 128), device='cuda').to(torch.bfloat16)\n"
        "out = torch.empty_like(q); lse = torch.empty((4, 300), dtype=torch.float32, device='cuda')\n"
        "plan = P.dcp_plan_create(w.cu_seqlens, w.block_size, table)\n"
        "P.dcp_block_attn_fwd(plan, q, k, k, out, lse, w.softmax_scale, None)\n"
        "torch.cuda.synchronize(); assert bool(torch.isfinite(out.float()).all()); print('ok')\n"
    ) % os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, timeout=110)
    assert r.returncode == 0 and "ok" in r.stdout, r.stdout + r.stderr


def test_window_rows_without_parameters_are_refused():
    import paper_2510_10620_amd as P
    spec = W.MaskSpec("window", window=40)
    w = W.custom_workload("small_window", [300], 128, 4, 2, 128, "bf16", spec, seed=34, input_scale=0.5)
    table = P.dcp_build_block_table_window(w.cu_seqlens, w.block_size, 40, 0)
    g = H.GpuRun(w, W.make_tensors(w), table)          # no dcp_plan_set_window
    with pytest.raises(P.DcpError) as ei:
        P.dcp_block_attn_fwd(g.plan, g.q, g.k, g.v, g.out, g.lse, w.softmax_scale, None)
    assert ei.value.status == P.DCP_ERR_INVALID_ARG and "dcp_plan_set_window" in str(ei.value)


@pytest.mark.parametrize("impl", list(IMPLS), ids=list(IMPLS))
def test_large_scores_bf16(impl):
    """N(0,1) inputs: scores of magnitude ~ sqrt(D) * scale ~ 1..4 exercise the softmax range."""
    w = W.custom_workload("sharp", [520, 260], 256, 8, 2, 128, "bf16", W.MaskSpec("causal"), seed=32, input_scale=1.0)
    run_case(w, H.oracle_table(w), IMPLS[impl], label=f"sharp/{impl}")


@pytest.mark.parametrize("impl", list(IMPLS), ids=list(IMPLS))
def test_row_order_and_skip_rows_do_not_matter(impl):
    w = W.custom_workload("perm", [400, 150], 64, 4, 4, 128, "bf16", W.MaskSpec("lambda", window=100, sink=10), seed=33, input_scale=0.5)
    table = H.oracle_table(w)
    rng = np.random.default_rng(1)
    shuffled = table[rng.permutation(len(table))]
    extra = np.array([[0, 3, W.MASK_SKIP], [2, 1, W.MASK_SKIP]], dtype=np.int32)
    t2 = np.concatenate([shuffled, extra])
    tensors = W.make_tensors(w)
    ref = H.oracle_full(w, tensors, table)
    g = H.GpuRun(w, tensors, t2, impl=IMPLS[impl])
    out, lse = g.forward()
    dq, dk, dv = g.backward()
    H.check(w, dict(out=out, lse=lse, dq=dq, dk=dk, dv=dv), ref, ALL, "perm")


@pytest.mark.parametrize("impl", list(IMPLS), ids=list(IMPLS))
def test_share_with_divisions_and_merge(impl):
    """One device's share of a causal plan, executed as 4 divisions with partial slots merged by
    LSE; backward of the share uses the global O / LSE."""
    import torch
    w = W.custom_workload("share", [700, 90, 333, 1200], 128, 4, 2, 128, "bf16", W.MaskSpec("causal"), seed=34, input_scale=0.5)
    table = H.oracle_table(w)
    tensors = W.make_tensors(w)
    full = H.oracle_full(w, tensors, table)
    delta = OA.delta_rows(full["out"], W.to_f64(w, tensors["dout"]))
    # global O / LSE on the device come from the HIP path's own full-table forward
    gfull = H.GpuRun(w, tensors, table, impl=IMPLS[impl])
    out_full, lse_full = gfull.forward()
    H.check(w, dict(out=out_full, lse=lse_full), full, ("out", "lse"), "full")
    sel = W.deal_share(len(table), 3, 205, 0)
    sub = table[sel]
    slot, n_slots, slot_q = W.deal_divisions(sub[:, 0], 4, 305)
    g = H.GpuRun(w, tensors, sub, slot, n_slots, impl=IMPLS[impl])
    out, lse = g.forward()
    ref = H.oracle_full(w, tensors, table, select=sel, lse=full["lse"], delta=delta)
    H.check(w, dict(out=out, lse=lse), ref, ("out", "lse"), "share fwd")
    # each partial slot against the oracle's partial for that slot
    o_part, lse_part = H.from_torch(g.o_part), H.from_torch(g.lse_part)
    part = OB.block_partition(w.cu_seqlens, w.block_size)
    for s in range(0, n_slots, 5):
        rows = sel[slot == s]
        qb = int(slot_q[s])
        r0, n = int(part["blk_start"][qb]), int(part["blk_end"][qb] - part["blk_start"][qb])
        ps = H.oracle_full(w, tensors, table, select=rows, bwd=False, seqs=[int(part["blk_seq"][qb])])
        assert H.max_abs(o_part[s, :n], ps["out"][r0:r0 + n]) <= 2e-2
        assert H.max_abs(lse_part[s, :, :n], ps["lse"][:, r0:r0 + n]) <= 1e-5
    dq, dk, dv = g.backward(out=gfull.out, lse=gfull.lse)
    H.check(w, dict(dq=dq, dk=dk, dv=dv), ref, ("dq", "dk", "dv"), "share bwd")
    # q blocks the share never touches: O = 0, LSE = -inf, dQ = 0
    untouched = sorted(set(range(len(part["blk_seq"]))) - set(sub[:, 0].tolist()))
    for qb in untouched:
        r0, r1 = int(part["blk_start"][qb]), int(part["blk_end"][qb])
        assert not out[r0:r1].any() and np.all(lse[:, r0:r1] == -np.inf) and not dq[r0:r1].any()


@pytest.mark.parametrize("impl", list(IMPLS), ids=list(IMPLS))
def test_edge_cases(impl):
    import paper_2510_10620_amd as P
    # empty table: O = 0, LSE = -inf, gradients 0
    w = W.custom_workload("empty", [70, 5], 32, 4, 2, 128, "bf16", W.MaskSpec("causal"), seed=35)
    tensors = W.make_tensors(w)
    g = H.GpuRun(w, tensors, np.zeros((0, 3), np.int32), impl=IMPLS[impl])
    out, lse = g.forward()
    assert not out.any() and np.all(lse == -np.inf)
    dq, dk, dv = g.backward()
    assert not dq.any() and not dk.any() and not dv.any()
    # a single token, and a table whose only entries are fully masked (CAUSAL above the diagonal)
    w1 = W.custom_workload("one", [1], 16, 4, 4, 128, "bf16", W.MaskSpec("causal"), seed=36)
    run_case(w1, H.oracle_table(w1), IMPLS[impl], label="single token")
    w2 = W.custom_workload("masked", [64], 32, 4, 2, 128, "bf16", W.MaskSpec("causal"), seed=37)
    t2 = np.array([[0, 1, W.MASK_CAUSAL]], dtype=np.int32)
    ten2 = W.make_tensors(w2)
    g2 = H.GpuRun(w2, ten2, t2, impl=IMPLS[impl])
    out, lse = g2.forward()
    assert not out.any() and np.all(lse == -np.inf)
    # RANGES rows without the range array are refused before any launch
    w3 = W.custom_workload("rng", [100], 32, 4, 2, 128, "bf16", W.MaskSpec("window", window=20), seed=38)
    g3 = H.GpuRun(w3, W.make_tensors(w3), H.oracle_table(w3), impl=IMPLS[impl])
    with pytest.raises(P.DcpError) as ei:
        P.dcp_block_attn_fwd(g3.plan, g3.q, g3.k, g3.v, g3.out, g3.lse, w3.softmax_scale, None, IMPLS[impl])
    assert ei.value.status == P.DCP_ERR_INVALID_ARG
    with pytest.raises(P.DcpError) as ei:   # unsupported head_dim
        P.dcp_block_attn_fwd(g3.plan, g3.q[:, :, :48], g3.k[:, :, :48], g3.v[:, :, :48], g3.out, g3.lse, 1.0, g3.ranges, 0)
    assert ei.value.status in (P.DCP_ERR_UNSUPPORTED, P.DCP_ERR_INVALID_ARG)


@pytest.mark.parametrize("kind,B", [("causal", 64), ("causal", 192), ("causal", 1024), ("shared_question", 256), ("lambda", 320)])
def test_lengths_around_the_tile_grid(kind, B):
    """Sequence lengths one below, at and one above multiples of the 64-key tile and the 128-row query tile: the steps
    where a wave passes from the short step (this tile and the next whole and fully visible, copies of the next tile
    issued between its MFMAs) to the general one, at every offset of the block size against the tiles; causal tables
    run the kernels without per-token ranges, the other two the kernels with them (NONE, CAUSAL and RANGES rows)."""
    spec = {"causal": W.MaskSpec("causal"), "shared_question": W.MaskSpec("shared_question"),
            "lambda": W.MaskSpec("lambda", window=150, sink=70)}[kind]
    lens = [63, 64, 65, 127, 128, 129, 191, 193, 256, 257, 321, 640, 705]
    w = W.custom_workload("grid", lens, B, 4, 2, 128, "bf16", spec, seed=77, input_scale=0.5)
    run_case(w, H.oracle_table(w), IMPLS["auto"], label=f"{kind} B{B}")


@pytest.mark.parametrize("B", [32, 96, 4096])
def test_block_sizes_off_the_tile_grid(B):
    """Block sizes below the kernels' 128-row / 64-key tiles, not a multiple of them, and larger than every
    sequence, with the lambda mask and with the WINDOW kind on top of block buffers and partial slots."""
    import paper_2510_10620_amd as P
    spec = W.MaskSpec("lambda", window=70, sink=11)
    w = W.custom_workload("blocks", [333, 97, 500], B, 4, 2, 128, "bf16", spec, seed=36, input_scale=0.5)
    run_case(w, H.oracle_table(w), IMPLS["auto"], label=f"B{B}")
    # the same mask as WINDOW rows, through block buffers with permuted slots and divisions into partial slots
    table = P.dcp_build_block_table_window(w.cu_seqlens, w.block_size, 70, 11)
    rng = np.random.default_rng(B)
    slot, n_slots, _ = W.deal_divisions(table[:, 0], 2, 5)
    _buffer_case(w, table, IMPLS["auto"], rng, out_slot=slot, n_slots=n_slots, window=(70, 11))


def test_strided_inputs_fused_qkv_layout():
    """q, k, v as views of one [T, (Hq + 2 Hkv) * D] projection output."""
    import torch
    w = W.custom_workload("strided", [200, 120], 64, 4, 2, 128, "bf16", W.MaskSpec("causal"), seed=39, input_scale=0.5)
    tensors = W.make_tensors(w)
    table = H.oracle_table(w)
    g = H.GpuRun(w, tensors, table)
    fused = torch.cat([g.q, g.k, g.v], dim=1).contiguous()
    g.q, g.k, g.v = fused[:, :4], fused[:, 4:6], fused[:, 6:8]
    out, lse = g.forward()
    dq, dk, dv = g.backward()
    H.check(w, dict(out=out, lse=lse, dq=dq, dk=dk, dv=dv), H.oracle_full(w, tensors, table), ALL, "strided")


def test_delta_and_sum_partials_streaming_kernels():
    import torch
    import paper_2510_10620_amd as P
    rng = np.random.default_rng(40)
    T, Hq, D = 1000, 8, 128
    o = W.f32_to_bf16_bits(rng.standard_normal((T, Hq, D)).astype(np.float32))
    do = W.f32_to_bf16_bits(rng.standard_normal((T, Hq, D)).astype(np.float32))
    w = W.custom_workload("x", [T], 64, Hq, Hq, D, "bf16", W.MaskSpec("causal"), seed=0)
    to, tdo = H.to_torch(w, o), H.to_torch(w, do)
    delta = torch.full((Hq, T), float("nan"), dtype=torch.float32, device="cuda")
    P.dcp_bwd_delta(to, tdo, delta)
    ref = OA.delta_rows(W.bf16_bits_to_f64(o), W.bf16_bits_to_f64(do))
    err = H.max_abs(H.from_torch(delta), ref)
    assert err <= 1e-4, err
    parts = [torch.from_numpy((0.2 * rng.standard_normal((T, Hq, D))).astype(np.float32)).cuda() for _ in range(5)]  # |sum| < 4: bf16 half-ulp < 2e-2
    dst = torch.empty((T, Hq, D), dtype=torch.bfloat16, device="cuda")
    P.dcp_sum_partials(parts, dst)
    ref = OA.sum_partials([H.from_torch(p) for p in parts])
    err = H.max_abs(H.from_torch(dst), ref)
    assert err <= 2e-2, err
    dst32 = torch.empty((T, Hq, D), dtype=torch.float32, device="cuda")
    P.dcp_sum_partials(parts, dst32)
    err = H.max_abs(H.from_torch(dst32), ref)
    assert err <= 1e-5, err


def test_blockwise_copy_bit_exact():
    """Blockwise Copy between a packed tensor and a block buffer (and inside one buffer), bit for bit against
    the oracle's row loops: ragged last blocks, rows narrower than a lane group, padded row strides, and a
    second, smaller list on the same buffers."""
    import torch
    import paper_2510_10620_amd as P
    from oracle import blockbuf as BB
    rng = np.random.default_rng(41)
    B = 48
    cu = np.concatenate([[0], np.cumsum([200, 37, 48, 301])]).astype(np.int32)
    part = OB.block_partition(cu, B)
    bs, bl = part["blk_start"], part["blk_end"] - part["blk_start"]
    n_slots = len(bs) + 2
    slots = rng.permutation(n_slots)[:len(bs)].astype(np.int32)
    T = int(cu[-1])
    for shape, dtype in (((4, 128), np.uint16), ((1, 8), np.uint16), ((2, 36), np.float32)):
        x = rng.integers(0, 60000, size=(T,) + shape).astype(dtype)
        to_buf = BB.copy_entries_for_blocks(bs, bl, slots, B, to_buffer=True)
        ref_buf = BB.blockwise_copy(x, np.full((n_slots * B,) + shape, 7, dtype=dtype), to_buf)
        tx = torch.from_numpy(x.view(np.int16) if dtype == np.uint16 else x).cuda()
        tbuf = torch.full((n_slots * B,) + shape, 7, dtype=tx.dtype, device="cuda")
        cl = P.CopyList(to_buf, T, n_slots * B)
        P.dcp_blockwise_copy(cl, tx, tbuf)
        got = tbuf.cpu().numpy()
        assert np.array_equal(got.view(dtype), ref_buf), (shape, "packed -> buffer")
        # back through a padded destination (row stride > row bytes)
        back = BB.copy_entries_for_blocks(bs, bl, slots, B, to_buffer=False)
        wide = torch.zeros((T, shape[0] * 2, shape[1]), dtype=tx.dtype, device="cuda")
        P.dcp_blockwise_copy(P.CopyList(back, n_slots * B, T), tbuf, wide[:, :shape[0]])
        assert np.array_equal(wide[:, :shape[0]].cpu().numpy().view(dtype), x), (shape, "buffer -> packed, strided")
        assert int(wide[:, shape[0]:].abs().sum()) == 0, "padding was written"
        # a smaller list on the same buffers: one block moved inside the buffer to a free slot
        free = sorted(set(range(n_slots)) - set(slots.tolist()))[0]
        b = 2
        inside = np.array([[slots[b] * B, free * B, bl[b]]], dtype=np.int32)
        ref2 = BB.blockwise_copy(ref_buf.copy(), ref_buf.copy(), inside)
        P.dcp_blockwise_copy(P.CopyList(inside, n_slots * B, n_slots * B), tbuf, tbuf)
        assert np.array_equal(tbuf.cpu().numpy().view(dtype), ref2), (shape, "inside one buffer")
    # same buffer with a destination that overlaps a source range is refused
    bad = P.CopyList(np.array([[0, 10, 20]], dtype=np.int32), n_slots * B, n_slots * B)
    with pytest.raises(P.DcpError):
        P.dcp_blockwise_copy(bad, tbuf, tbuf)
    # an empty list does nothing
    P.dcp_blockwise_copy(P.CopyList(np.zeros((0, 3), np.int32), T, n_slots * B), tx, tbuf)


def _buffer_case(w, table, impl, rng, absent_ok=False, out_slot=None, n_slots=0, window=None):
    """Runs forward + backward with every tensor held in block buffers (permuted slots, free slots in
    between, unused rows poisoned) and compares what comes back, block by block, with the oracle on the
    packed tensors.  Returns nothing; asserts."""
    import torch
    import paper_2510_10620_amd as P
    from oracle import blockbuf as BB
    tensors = W.make_tensors(w)
    table = np.asarray(table, dtype=np.int32).reshape(-1, 3)
    part = OB.block_partition(w.cu_seqlens, w.block_size)
    bs, bl = part["blk_start"], part["blk_end"] - part["blk_start"]
    nb, B, T = len(bs), w.block_size, w.total_tokens
    live = table[table[:, 2] != 3]
    used_q, used_kv = np.zeros(nb, bool), np.zeros(nb, bool)
    used_q[live[:, 0]] = True
    used_kv[live[:, 1]] = True
    n_qs, n_ks = nb + 2, nb + 3
    q_slot = rng.permutation(n_qs)[:nb].astype(np.int32)
    kv_slot = rng.permutation(n_ks)[:nb].astype(np.int32)
    if absent_ok:
        q_slot[~used_q] = -1
        kv_slot[~used_kv] = -1
    plan = P.dcp_plan_create(w.cu_seqlens, B, table, out_slot, n_slots)
    P.dcp_plan_set_block_buffers(plan, q_slot, n_qs, kv_slot, n_ks)
    if window is not None:            # WINDOW rows: two numbers, no range array
        P.dcp_plan_set_window(plan, *window)
    nan16 = np.uint16(0x7FC0)
    fill = nan16 if w.dtype == "bf16" else np.float32("nan")
    buf = {n: BB.gather_blocks(tensors[n], bs, bl, q_slot if n in ("q", "dout") else kv_slot,
                               n_qs if n in ("q", "dout") else n_ks, B, fill=fill) for n in ("q", "k", "v", "dout")}
    tq, tk, tv, tdo = (H.to_torch(w, buf[n]) for n in ("q", "k", "v", "dout"))
    rg = None if window is not None else torch.from_numpy(np.ascontiguousarray(w.ranges)).cuda()
    out = torch.full((n_qs * B, w.hq, w.d), 768.0, dtype=tq.dtype, device="cuda")
    lse = torch.full((w.hq, n_qs * B), 768.0, dtype=torch.float32, device="cuda")
    if out_slot is not None:
        o_part = torch.full((n_slots, B, w.hq, w.d), float("nan"), dtype=tq.dtype, device="cuda")
        lse_part = torch.full((n_slots, w.hq, B), float("nan"), dtype=torch.float32, device="cuda")
        P.dcp_block_attn_fwd(plan, tq, tk, tv, o_part, lse_part, w.softmax_scale, rg, impl)
        P.dcp_merge_partials(plan, o_part, lse_part, out, lse)
    else:
        P.dcp_block_attn_fwd(plan, tq, tk, tv, out, lse, w.softmax_scale, rg, impl)
    dq = torch.full_like(out, 768.0)
    dk = torch.full((n_ks * B, w.hkv, w.d), 768.0, dtype=tq.dtype, device="cuda")
    dv = torch.full_like(dk, 768.0)
    ws = torch.empty(max(256, P.dcp_bwd_workspace_bytes(plan, w.hq, w.hkv, w.d, P.DCP_BF16 if w.dtype == "bf16" else P.DCP_F32)),
                     dtype=torch.uint8, device="cuda")
    ref = H.oracle_full(w, tensors, table, window=window)
    # the backward takes the forward's out / lse when the table is complete; for a share, the oracle's global ones
    P.dcp_block_attn_bwd(plan, tq, tk, tv, out, lse, tdo, dq, dk, dv, w.softmax_scale, ws, rg, impl)
    torch.cuda.synchronize()
    got_buf = dict(out=H.from_torch(out), dq=H.from_torch(dq), dk=H.from_torch(dk), dv=H.from_torch(dv))
    got = {n: BB.scatter_blocks(got_buf[n], bs, bl, q_slot if n in ("out", "dq") else kv_slot, B, T) for n in got_buf}
    got["lse"] = BB.scatter_rows_hT(H.from_torch(lse), bs, bl, q_slot, B, T)
    # blocks that are absent from a buffer have no result: compare the oracle's zeros / -inf there with what
    # scatter leaves (zeros), except lse, which scatter also leaves at 0
    for n, slot in (("out", q_slot), ("dq", q_slot), ("dk", kv_slot), ("dv", kv_slot), ("lse", q_slot)):
        for b in np.nonzero(slot < 0)[0]:
            sl = slice(bs[b], bs[b] + bl[b])
            if n == "lse":
                ref[n][:, sl] = 0.0
            else:
                assert not np.abs(ref[n][sl]).max() > 0, "a block the table uses was declared absent"
    H.check(w, got, ref, ALL, "block buffers")
    # rows no block owns keep the sentinel
    for n, slot, rows in (("out", q_slot, n_qs * B), ("dq", q_slot, n_qs * B), ("dk", kv_slot, n_ks * B), ("dv", kv_slot, n_ks * B)):
        owned = np.zeros(rows, bool)
        for b in range(nb):
            if slot[b] >= 0:
                owned[slot[b] * B: slot[b] * B + bl[b]] = True
        assert (got_buf[n][~owned] == 768.0).all(), n + ": a row outside every block was written"


@pytest.mark.parametrize("impl", list(IMPLS), ids=list(IMPLS))
def test_block_buffer_addressing(impl):
    """Sec. 5: Q / KV / O blocks addressed through block buffers (slot * block_size + row) give what the packed
    tensors give.  Causal and lambda masks (NONE, CAUSAL and RANGES rows), ragged last blocks, blocks spanning
    several kernel tiles."""
    rng = np.random.default_rng(42)
    w = W.custom_workload("buf_causal", [300, 77, 520], 160, 4, 2, 128, "bf16", W.MaskSpec("causal"), seed=43, input_scale=0.5)
    _buffer_case(w, H.oracle_table(w), IMPLS[impl], rng)
    w = W.custom_workload("buf_lambda", [413, 90], 96, 4, 2, 128, "bf16", W.MaskSpec("lambda", window=130, sink=20), seed=44, input_scale=0.5)
    _buffer_case(w, H.oracle_table(w), IMPLS[impl], rng)


def test_block_buffer_with_absent_blocks_and_partial_slots():
    """A window mask whose table leaves some blocks unused on one side is run with those blocks absent from the
    buffer (slot -1), and with partial output slots merged into the Q-type buffer."""
    rng = np.random.default_rng(45)
    w = W.custom_workload("buf_slots", [400, 200], 64, 4, 4, 128, "bf16", W.MaskSpec("causal"), seed=46, input_scale=0.5)
    table = H.oracle_table(w)
    slot, n_slots, _ = W.deal_divisions(table[:, 0], 3, 5)
    _buffer_case(w, table, 0, rng, out_slot=slot, n_slots=n_slots)
    # drop every row that has q_blk 2 or kv_blk 5: block 2 produces no output, block 5 receives no gradient
    sub = table[(table[:, 0] != 2) & (table[:, 1] != 5)]
    _buffer_case(w, sub, 0, rng, absent_ok=True)


def test_execution_plan_with_divisions_and_transfers():
    """Sec. 5 / Sec. 4.3: an execution plan of three divisions.  Division 0 attends with the KV blocks that are already
    in the KV block buffer; the blocks divisions 1 and 2 need first are moved in by Comm.Launch (a Blockwise Copy on
    the second stream) and awaited by Comm.Wait right before their attention.  Every division writes partial slots,
    a Blockwise Reduction merges them, a backward instruction follows.  Buffer rows start poisoned, so an attention
    that ran before its transfer had landed would produce NaN."""
    import torch
    import paper_2510_10620_amd as P
    from oracle import blockbuf as BB
    rng = np.random.default_rng(47)
    w = W.custom_workload("exec", [330, 200, 90], 64, 4, 2, 128, "bf16", W.MaskSpec("causal"), seed=48, input_scale=0.5)
    tensors = W.make_tensors(w)
    table = H.oracle_table(w)
    part = OB.block_partition(w.cu_seqlens, w.block_size)
    bs, bl = part["blk_start"], part["blk_end"] - part["blk_start"]
    nb, B, T = len(bs), w.block_size, w.total_tokens
    n_div = 3
    slot, n_slots, _ = W.deal_divisions(table[:, 0], n_div, 9)
    div = np.zeros(len(table), dtype=np.int64)
    # recover each row's division from its slot: deal_divisions numbers slots per (division, q_blk)
    perm = np.random.default_rng(9).permutation(len(table))
    div[perm] = np.arange(len(table)) % n_div
    assert len(set(zip(div.tolist(), table[:, 0].tolist()))) == n_slots
    # KV buffer: permuted slots; a block is "remote" for the first division that uses it unless division 0 does
    kv_slot = rng.permutation(nb + 1)[:nb].astype(np.int32)
    q_slot = np.arange(nb, dtype=np.int32)                      # Q side stays in packed order (slot b = block b)
    first_div = np.full(nb, n_div)
    for d, kb in zip(div, table[:, 1]):
        first_div[kb] = min(first_div[kb], d)
    nan16 = np.uint16(0x7FC0)
    kbuf = BB.gather_blocks(tensors["k"], bs, bl, np.where(first_div == 0, kv_slot, -1), nb + 1, B, fill=nan16)
    vbuf = BB.gather_blocks(tensors["v"], bs, bl, np.where(first_div == 0, kv_slot, -1), nb + 1, B, fill=nan16)
    qbuf = BB.gather_blocks(tensors["q"], bs, bl, q_slot, nb, B, fill=nan16)
    dobuf = BB.gather_blocks(tensors["dout"], bs, bl, q_slot, nb, B, fill=nan16)
    tq, tk, tv, tdo = (H.to_torch(w, a) for a in (qbuf, kbuf, vbuf, dobuf))
    k_far, v_far = H.to_torch(w, tensors["k"]), H.to_torch(w, tensors["v"])     # where remote blocks come from
    rg = torch.from_numpy(np.ascontiguousarray(w.ranges)).cuda()
    o_part = torch.full((n_slots, B, w.hq, w.d), float("nan"), dtype=tq.dtype, device="cuda")
    lse_part = torch.full((n_slots, w.hq, B), float("nan"), dtype=torch.float32, device="cuda")
    out = torch.full((nb * B, w.hq, w.d), float("nan"), dtype=tq.dtype, device="cuda")
    lse = torch.full((w.hq, nb * B), float("nan"), dtype=torch.float32, device="cuda")
    dq = torch.zeros_like(out)
    dk = torch.zeros(((nb + 1) * B, w.hkv, w.d), dtype=tq.dtype, device="cuda")
    dv = torch.zeros_like(dk)

    def make_plan(rows):
        pl = P.dcp_plan_create(w.cu_seqlens, B, table[rows], slot[rows], n_slots)
        P.dcp_plan_set_block_buffers(pl, q_slot, nb, kv_slot, nb + 1)
        return pl
    full = make_plan(np.arange(len(table)))
    plain = P.dcp_plan_create(w.cu_seqlens, B, table)               # backward of the whole table, no slots
    P.dcp_plan_set_block_buffers(plain, q_slot, nb, kv_slot, nb + 1)
    ws = torch.empty(max(256, P.dcp_bwd_workspace_bytes(plain, w.hq, w.hkv, w.d, P.DCP_BF16)), dtype=torch.uint8, device="cuda")
    instrs = []
    for d in range(1, n_div):                                         # launch every transfer up front
        need = np.nonzero(first_div == d)[0]
        entries = np.stack([bs[need], kv_slot[need].astype(np.int64) * B, bl[need]], axis=1).astype(np.int32)
        cl = P.CopyList(entries, T, (nb + 1) * B)
        instrs.append(P.instr_comm_launch(2 * d, cl, k_far, tk))
        instrs.append(P.instr_comm_launch(2 * d + 1, cl, v_far, tv))
    for d in range(n_div):
        if d > 0:
            instrs += [P.instr_comm_wait(2 * d), P.instr_comm_wait(2 * d + 1)]
        instrs.append(P.instr_attn_fwd(make_plan(np.nonzero(div == d)[0]), tq, tk, tv, o_part, lse_part, w.softmax_scale, rg))
    instrs.append(P.instr_merge(full, o_part, lse_part, out, lse))
    instrs.append(P.instr_attn_bwd(plain, tq, tk, tv, out, lse, tdo, dq, dk, dv, w.softmax_scale, ws, rg))
    prog = P.Program(instrs)
    side = torch.cuda.Stream()
    for rep in range(2):                                              # a plan is replayed for every layer
        if rep == 1:                                                  # poison the remote blocks again
            tk.copy_(H.to_torch(w, kbuf)); tv.copy_(H.to_torch(w, vbuf))
            torch.cuda.synchronize()
        prog.run(side)
        torch.cuda.synchronize()
        got = dict(out=BB.scatter_blocks(H.from_torch(out), bs, bl, q_slot, B, T),
                   lse=BB.scatter_rows_hT(H.from_torch(lse), bs, bl, q_slot, B, T),
                   dq=BB.scatter_blocks(H.from_torch(dq), bs, bl, q_slot, B, T),
                   dk=BB.scatter_blocks(H.from_torch(dk), bs, bl, kv_slot, B, T),
                   dv=BB.scatter_blocks(H.from_torch(dv), bs, bl, kv_slot, B, T))
        H.check(w, got, H.oracle_full(w, tensors, table), ALL, f"execution plan, replay {rep}")
    # a program with transfers refuses to run on one stream
    with pytest.raises(P.DcpError):
        prog.run(None)


def test_two_runs_are_bit_identical():
    """No atomics, fixed reduction orders: forward, merge and backward run twice on the same inputs give the same
    bits, with cut dK/dV items (fp32 partial sums added up by the reduce kernel) and with partial output slots."""
    import torch
    import paper_2510_10620_amd as P
    lens = W.draw_lengths(8192, "lognormal", 512, 4096, seed=2, median=1024)
    w = W.custom_workload("twice", lens, 256, 8, 2, 128, "bf16", W.MaskSpec("causal"), seed=51, input_scale=1.0 / np.sqrt(128))
    tensors = W.make_tensors(w)
    table = H.oracle_table(w)
    slot, n_slots, _ = W.deal_divisions(table[:, 0], 3, 52)
    for label, args in (("plain", ()), ("slots", (slot, n_slots))):
        g = H.GpuRun(w, tensors, table, *args)
        if label == "plain":
            assert (P.dcp_plan_export_dkv_items(g.plan, w.hkv)[:, 4] >= 0).any(), "the case is meant to have cut dK/dV items"
        runs = []
        for rep in range(2):
            g.out.fill_(float("nan")); g.lse.fill_(float("nan"))
            g.forward_only()
            g.backward_only(g.out, g.lse)
            runs.append({n: getattr(g, n).clone() for n in ALL})
        for n in ALL:
            assert torch.equal(runs[0][n].view(torch.int16 if n != "lse" else torch.int32),
                               runs[1][n].view(torch.int16 if n != "lse" else torch.int32)), f"{label}: {n} differs between two runs"


def test_two_streams_share_a_plan():
    """A plan holds nothing a launch writes (work lists and table are read-only on the device; partial sums, delta and
    LSE copies live in the caller's workspace), so two streams may run the same plan at the same time on tensors of
    their own.  Two forward + backward passes on different inputs, enqueued on two streams without a wait between
    them, must give the bits of the same passes run one after the other."""
    import torch
    import paper_2510_10620_amd as P
    lens = W.draw_lengths(8192, "lognormal", 512, 4096, seed=2, median=1024)
    w = W.custom_workload("streams", lens, 256, 8, 2, 128, "bf16", W.MaskSpec("causal"), seed=59, input_scale=1.0 / np.sqrt(128))
    table = H.oracle_table(w)
    plan = P.dcp_plan_create(w.cu_seqlens, w.block_size, table)
    P.dcp_plan_prepare(plan, w.hq, w.hkv, w.d, P.DCP_BF16)
    need = max(256, P.dcp_bwd_workspace_bytes(plan, w.hq, w.hkv, w.d, P.DCP_BF16))
    T = w.total_tokens
    sets = []
    for i in range(2):
        gen = torch.Generator(device="cuda")
        gen.manual_seed(100 + i)
        mk = lambda h, sc: (torch.randn((T, h, w.d), device="cuda", generator=gen) * sc).to(torch.bfloat16)
        q, k, v, do = mk(w.hq, w.input_scale), mk(w.hkv, w.input_scale), mk(w.hkv, w.input_scale), mk(w.hq, 1.0)
        bufs = dict(out=torch.empty_like(q), lse=torch.empty((w.hq, T), dtype=torch.float32, device="cuda"),
                    dq=torch.empty_like(q), dk=torch.empty_like(k), dv=torch.empty_like(v))
        sets.append(dict(q=q, k=k, v=v, do=do, bufs=bufs, ws=torch.empty(need, dtype=torch.uint8, device="cuda")))

    def run(s):
        b = s["bufs"]
        P.dcp_block_attn_fwd(plan, s["q"], s["k"], s["v"], b["out"], b["lse"], w.softmax_scale, None)
        P.dcp_block_attn_bwd(plan, s["q"], s["k"], s["v"], b["out"], b["lse"], s["do"], b["dq"], b["dk"], b["dv"],
                             w.softmax_scale, s["ws"], None)

    for s in sets:                                   # one after the other, on the current stream
        run(s)
    torch.cuda.synchronize()
    ref = [{n: t.clone() for n, t in s["bufs"].items()} for s in sets]
    for s in sets:
        for t in s["bufs"].values():
            t.fill_(float("nan"))
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    for rep in range(3):                             # interleaved so that the launches of the two streams overlap
        for s, st in zip(sets, streams):
            with torch.cuda.stream(st):
                run(s)
    torch.cuda.synchronize()
    for i, s in enumerate(sets):
        for n in ALL:
            view = torch.int32 if n == "lse" else torch.int16
            assert torch.equal(s["bufs"][n].view(view), ref[i][n].view(view)), f"stream {i}: {n} differs from the sequential run"


def test_dv_of_a_sink_key_is_the_sum_with_p_rounded_to_bf16():
    """Where the plain bound on dV is tight: a sink key under a small window is seen by every later query of every head
    of its group (here 447 x 4), each with a weight near 1 / 8, and P goes into the dV product as bf16.  The rounding
    of P, 2^-9 relative per term, then adds up over a sum whose root sum of squares is larger than the sum itself.  The
    kernel's value must be that sum exactly: P from the oracle's scores and LSE, rounded to bf16 (nearest even), times
    dO, summed in fp64, then rounded to bf16 once -- to one bf16 step (scores in fp32 against fp64 can turn a rounding
    of P the other way)."""
    w = W.custom_workload("sink", [447, 26], 256, 8, 2, 128, "bf16", W.MaskSpec("lambda", window=7, sink=1), seed=433, input_scale=0.5)
    table = H.oracle_table(w)
    tensors = W.make_tensors(w)
    g = H.GpuRun(w, tensors, table, impl=IMPLS["auto"])
    out, lse = g.forward()
    dq, dk, dv = g.backward()
    got = dict(out=out, lse=lse, dq=dq, dk=dk, dv=dv)
    ref = H.oracle_full(w, tensors, table)
    # everything but the sink key's dV row at the usual bound (that row is put aside for the comparison below)
    rest = dict(got, dv=got["dv"].copy())
    rest["dv"][0] = ref["dv"][0]
    H.check(w, rest, ref, ALL, "sink key, all but the sink's dV")
    q, k, do = (W.to_f64(w, tensors[n]) for n in ("q", "k", "dout"))
    vis = OB.Visibility(w.cu_seqlens, w.block_size, table, w.ranges)
    G = w.hq // w.hkv
    L = 447
    M = np.asarray(vis.rows(0, 0, L)).astype(bool)
    assert M[:, 0].all()                                     # every query of the sequence sees its first token
    worst_plain = worst_emul = 0.0
    for kvh in range(w.hkv):
        emul = np.zeros(w.d)
        for h in range(G * kvh, G * kvh + G):
            s_col = (q[:L, h] @ k[0, kvh]) * w.softmax_scale
            p = np.exp(s_col - ref["lse"][h, :L])
            p16 = W.bf16_bits_to_f64(W.f32_to_bf16_bits(p.astype(np.float32)))
            emul += p16 @ do[:L, h]
        step = 2.0 ** -7 * np.maximum(1.0, 2.0 ** np.floor(np.log2(np.maximum(np.abs(emul), 1e-30))))   # one bf16 step at |emul|
        d_emul = np.abs(got["dv"][0, kvh] - emul)
        assert (d_emul <= step).all(), f"kv head {kvh}: {d_emul.max():.4f} from the sum with bf16 P"
        worst_emul = max(worst_emul, d_emul.max())
        worst_plain = max(worst_plain, np.abs(got["dv"][0, kvh] - ref["dv"][0, kvh]).max())
    print(f"sink key dV: max |kernel - exact| {worst_plain:.4f}, max |kernel - sum with bf16 P| {worst_emul:.4f}")


def test_step_replays_from_a_hip_graph():
    """With a prepared plan the forward, the merge and the backward only launch kernels (no allocation, no
    synchronisation, no memset node), so a caller can record the step in a HIP graph.  Recorded once here, on a case
    with partial output slots and cut dK/dV items, then replayed three times with eager work and a synchronisation
    between the replays; every replay must give the bits of the eager run."""
    import torch
    import paper_2510_10620_amd as P
    lens = W.draw_lengths(8192, "lognormal", 512, 4096, seed=2, median=1024)
    w = W.custom_workload("graph", lens, 256, 8, 2, 128, "bf16", W.MaskSpec("causal"), seed=57, input_scale=1.0 / np.sqrt(128))
    tensors = W.make_tensors(w)
    table = H.oracle_table(w)
    slot, n_slots, _ = W.deal_divisions(table[:, 0], 3, 58)
    g = H.GpuRun(w, tensors, table, slot, n_slots)
    P.dcp_plan_prepare(g.plan, w.hq, w.hkv, w.d, P.DCP_BF16)
    g.forward_only()
    g.backward_only(g.out, g.lse)
    ref = {n: getattr(g, n).clone() for n in ALL}
    bufs = {n: torch.full_like(ref[n], float("nan")) for n in ALL}
    o_part, lse_part = torch.full_like(g.o_part, float("nan")), torch.full_like(g.lse_part, float("nan"))
    ws = torch.empty(max(256, P.dcp_bwd_workspace_bytes(g.plan, w.hq, w.hkv, w.d, P.DCP_BF16)), dtype=torch.uint8, device="cuda")
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        P.dcp_block_attn_fwd(g.plan, g.q, g.k, g.v, o_part, lse_part, w.softmax_scale, g.ranges)
        P.dcp_merge_partials(g.plan, o_part, lse_part, bufs["out"], bufs["lse"])
        P.dcp_block_attn_bwd(g.plan, g.q, g.k, g.v, bufs["out"], bufs["lse"], g.dout, bufs["dq"], bufs["dk"], bufs["dv"],
                             w.softmax_scale, ws, g.ranges)
    for rep in range(3):
        for t in list(bufs.values()) + [o_part, lse_part]:
            t.fill_(float("nan"))                      # eager work between the replays
        ws.random_(0, 255)                             # the partial sums of the last replay are no input of the next
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for n in ALL:
            assert torch.equal(bufs[n].view(torch.int16 if n != "lse" else torch.int32),
                               ref[n].view(torch.int16 if n != "lse" else torch.int32)), f"replay {rep}: {n} differs from the eager run"


def test_execution_plan_inline_copy_and_gradient_sum():
    """The two instruction types the division test does not use: an in-line Blockwise Copy (it runs on the compute
    stream, in order) that fills the K / V tensors the attention then reads, and Blockwise Reduction used on gradients
    (the plain sum): the table is dealt to two shares, each share's backward leaves its partial dQ / dK / dV in
    buffers of its own, and three sums add them up.  Checked against the oracle's full gradients, on two replays."""
    import torch
    import paper_2510_10620_amd as P
    w = W.custom_workload("exec_sum", [420, 130, 77], 64, 4, 2, 128, "bf16", W.MaskSpec("lambda", window=150, sink=12), seed=53,
                          input_scale=0.5)
    tensors = W.make_tensors(w)
    table = H.oracle_table(w)
    T = w.total_tokens
    part = OB.block_partition(w.cu_seqlens, w.block_size)
    bs, bl = part["blk_start"], part["blk_end"] - part["blk_start"]
    tq, tdo = H.to_torch(w, tensors["q"]), H.to_torch(w, tensors["dout"])
    k_src, v_src = H.to_torch(w, tensors["k"]), H.to_torch(w, tensors["v"])
    tk = torch.full_like(k_src, float("nan"))
    tv = torch.full_like(v_src, float("nan"))
    rg = torch.from_numpy(np.ascontiguousarray(w.ranges)).cuda()
    out = torch.full((T, w.hq, w.d), float("nan"), dtype=tq.dtype, device="cuda")
    lse = torch.full((w.hq, T), float("nan"), dtype=torch.float32, device="cuda")
    full = P.dcp_plan_create(w.cu_seqlens, w.block_size, table)
    cl = P.CopyList(np.stack([bs, bs, bl], axis=1).astype(np.int32), T, T)     # every block, block by block
    instrs = [P.instr_copy(cl, k_src, tk), P.instr_copy(cl, v_src, tv),
              P.instr_attn_fwd(full, tq, tk, tv, out, lse, w.softmax_scale, rg)]
    parts = {n: [] for n in ("dq", "dk", "dv")}
    for share in range(2):
        rows = W.deal_share(len(table), 2, 54, share)
        pl = P.dcp_plan_create(w.cu_seqlens, w.block_size, table[rows])
        ws = torch.empty(max(256, P.dcp_bwd_workspace_bytes(pl, w.hq, w.hkv, w.d, P.DCP_BF16)), dtype=torch.uint8, device="cuda")
        g = [torch.full((T, h, w.d), float("nan"), dtype=tq.dtype, device="cuda") for h in (w.hq, w.hkv, w.hkv)]
        for n, t in zip(("dq", "dk", "dv"), g):
            parts[n].append(t)
        instrs.append(P.instr_attn_bwd(pl, tq, tk, tv, out, lse, tdo, g[0], g[1], g[2], w.softmax_scale, ws, rg))
    total = {n: torch.full_like(parts[n][0], float("nan")) for n in parts}
    for n in ("dq", "dk", "dv"):
        instrs.append(P.instr_sum(parts[n], total[n]))
    prog = P.Program(instrs)
    ref = H.oracle_full(w, tensors, table)
    for rep in range(2):
        if rep == 1:
            for t in (tk, tv, out, lse, *total.values()):
                t.fill_(float("nan"))
        prog.run()                                   # no transfers: one stream is enough
        torch.cuda.synchronize()
        assert torch.equal(tk.view(torch.int16), k_src.view(torch.int16)) and torch.equal(tv.view(torch.int16), v_src.view(torch.int16))
        got = dict(out=H.from_torch(out), lse=H.from_torch(lse), **{n: H.from_torch(total[n]) for n in total})
        H.check(w, got, ref, ALL, f"in-line copy + gradient sum, replay {rep}")
