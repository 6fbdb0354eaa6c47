#!/usr/bin/env python3
"""Benchmark of the block-attention hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

A step is one pass of the hot path over one synthetic packed batch of the causal varlen bf16
configuration (32/8 heads, D 128, 65 536 tokens, log-normal lengths, block 1024): forward, then
backward (delta, dQ, dK/dV kernels).  Inputs are resident in HBM and the plan is created before
the timed region.  Prints ONE JSON line: effective TFLOP/s counting 14*D flops per visible
(query, key) pair per query head, the roofline of the dominant kernel from HIP events recorded
around every kernel launch, and the CPU oracle timed on a bounded sample of the same batch.
A second, shorter section times one device's share of a plan (partial slots + LSE merge) so that
the merge and the streaming kernels are measured too; it is reported under "extra".
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2516.6   # 256 CU x 2.4 GHz x 4096 flop/clk/CU, dense bf16 MFMA
PEAK_HBM_GBPS = 8000.0


def gen_tensors(torch, w, seed):
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    T = w.total_tokens
    mk = lambda h, sc: (torch.randn((T, h, w.d), device="cuda", generator=g, dtype=torch.float32) * sc).to(torch.bfloat16)
    return mk(w.hq, w.input_scale), mk(w.hkv, w.input_scale), mk(w.hkv, w.input_scale), mk(w.hq, 1.0)


def time_steps(torch, fn, steps, warmup):
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / steps


def cpu_baseline(w, table, q, k, v, do, budget_pairs=3.0e8):
    """The oracle as it stands, timed on the first sequences of the batch (until their dense
    L^2 reaches the budget) for the 4 query heads of KV group 0, forward + backward."""
    import numpy as np
    from oracle import attention as OA
    from oracle import blocks as OB
    cu = w.cu_seqlens
    seqs, dense = [], 0.0
    for s in range(len(cu) - 1):
        L = int(cu[s + 1] - cu[s])
        if seqs and dense + float(L) * L > budget_pairs:
            continue
        seqs.append(s)
        dense += float(L) * L
        if dense >= 0.8 * budget_pairs:
            break
    G = w.hq // w.hkv
    hi = int(cu[max(seqs) + 1])
    qh = q[:hi, :G].double().cpu().numpy()
    kh = k[:hi, :1].double().cpu().numpy()
    vh = v[:hi, :1].double().cpu().numpy()
    doh = do[:hi, :G].double().cpu().numpy()
    vis = OB.Visibility(cu, w.block_size, table, w.ranges)
    pairs = 0
    for s in seqs:
        L = int(cu[s + 1] - cu[s])
        pairs += L * (L + 1) // 2 if w.mask.kind == "causal" else int(vis.rows(s, 0, L).sum())
    t0 = time.perf_counter()
    OA.attention_fwd(qh, kh, vh, cu, vis, w.softmax_scale, seqs=seqs)
    OA.attention_bwd(qh, kh, vh, doh, cu, vis, w.softmax_scale, seqs=seqs)
    dt = time.perf_counter() - t0
    flops = pairs * G * w.d * 14
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count()
    return dict(value=flops / dt / 1e12, unit="TFLOP/s", cores=int(threads), kind="oracle", seconds=round(dt, 2),
                sample=f"sequences {seqs} of the batch ({sum(int(cu[s+1]-cu[s]) for s in seqs)} tokens), "
                       f"the {G} query heads of KV head 0, fp64 dense forward + backward; "
                       f"{pairs} visible pairs x {G} heads x 14*D flops")


def measured_traffic(kernel):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 --pmc summary (FETCH_SIZE and
    WRITE_SIZE, scaled by a copy of known size), or None if the summary does not list it.  The
    summary is a measurement of an earlier run of this same command, not of this run."""
    path = os.path.join(ROOT, "profiles", "bench_config2_hbm_traffic.md")
    try:
        with open(path) as f:
            for line in f:
                parts = line.split()
                if len(parts) == 4 and parts[0] == "traffic" and parts[1] == kernel:
                    return sum(int(float(p.split("=")[1])) for p in parts[2:])
    except OSError:
        pass
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=2)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extra", action="store_true")
    ap.add_argument("--only-stream", action="store_true", help="print only the share (merge) and Blockwise Copy sections")
    ap.add_argument("--only-executor", action="store_true", help="print only the execution-plan section")
    ap.add_argument("--only-short", type=int, default=0, help="print only the short-sequence section for this sequence length")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2510_10620_amd as P
    from paper_2510_10620_amd import workloads as W

    torch.cuda.set_device(0)
    if args.only_short:
        print(json.dumps(short_section(torch, P, W, np, steps=30, seq_len=args.only_short)))
        return
    if args.only_executor:
        print(json.dumps(executor_section(torch, P, W, np, steps=5)))
        return
    w = W.make_workload(args.config)
    if args.only_stream:
        table = P.dcp_build_block_table(w.cu_seqlens, w.block_size, w.ranges)
        q = gen_tensors(torch, w, w.tensor_seed)[0]
        plan = P.dcp_plan_create(w.cu_seqlens, w.block_size, table)
        out_, do_ = torch.randn_like(q), torch.randn_like(q)
        dbuf = torch.empty((w.hq, w.total_tokens), dtype=torch.float32, device="cuda")
        P.dcp_bwd_delta(out_, do_, dbuf)
        torch.cuda.synchronize()
        P.dcp_profile_enable(True)
        for _ in range(10):
            P.dcp_bwd_delta(out_, do_, dbuf)
        torch.cuda.synchronize()
        tot, n = P.dcp_profile_read("delta")
        P.dcp_profile_enable(False)
        dgb = w.total_tokens * w.hq * (4 * w.d + 4) / (tot / n * 1e-3) / 1e9
        print(json.dumps(dict(share=share_section(torch, P, W, np, steps=5, warmup=2),
                              blockwise_copy=copy_section(torch, P, np, plan, q, steps=10),
                              gradient_sum=sum_section(torch, P, q, steps=10),
                              delta=dict(ms=round(tot / n, 4), GBps=round(dgb, 1), frac_hbm=round(dgb / PEAK_HBM_GBPS, 3)))))
        return
    table = P.dcp_build_block_table(w.cu_seqlens, w.block_size, w.ranges)
    pairs = int(P.dcp_count_pairs(w.cu_seqlens, w.block_size, table, w.ranges).sum())
    q, k, v, do = gen_tensors(torch, w, w.tensor_seed)
    T = w.total_tokens
    out = torch.empty_like(q)
    lse = torch.empty((w.hq, T), dtype=torch.float32, device="cuda")
    dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
    rg = torch.from_numpy(np.ascontiguousarray(w.ranges)).cuda()
    t0 = time.perf_counter()
    plan = P.dcp_plan_create(w.cu_seqlens, w.block_size, table)
    plan_ms = (time.perf_counter() - t0) * 1e3
    ws = torch.empty(max(256, P.dcp_bwd_workspace_bytes(plan, w.hq, w.hkv, w.d, P.DCP_BF16)), dtype=torch.uint8, device="cuda")

    def step():
        P.dcp_block_attn_fwd(plan, q, k, v, out, lse, w.softmax_scale, rg)
        P.dcp_block_attn_bwd(plan, q, k, v, out, lse, do, dq, dk, dv, w.softmax_scale, ws, rg)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    P.dcp_profile_enable(True)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(args.steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / args.steps
    P.dcp_profile_enable(False)

    unit = pairs * w.hq * w.d            # one "D flops per pair per head" unit
    flops = 14 * unit
    # algorithmic flops per launch: forward 4D; the backward's 10D split over its two kernels as
    # dK/dV: dV + dK + half of the shared (S, dP) recompute = 6D;  dQ: dQ + the other half = 4D
    alg = dict(fwd=4 * unit, dq=4 * unit, dkv=6 * unit)
    executed = dict(fwd=4 * unit, dq=6 * unit, dkv=8 * unit)
    kern = {}
    for name in ("fwd", "delta", "dq", "dkv"):
        tot, n = P.dcp_profile_read(name)
        kern[name] = dict(ms=tot / max(n, 1), launches=n)
    delta_note = None
    if kern["delta"]["launches"] == 0:
        # the bf16 MFMA backward computes delta inside its dQ kernel: the standalone preprocess entry point (the
        # streaming kernel other shapes use) is timed on the same tensors, outside the step
        dbuf = torch.empty((w.hq, T), dtype=torch.float32, device="cuda")
        P.dcp_bwd_delta(out, do, dbuf)
        torch.cuda.synchronize()
        P.dcp_profile_enable(True)
        for _ in range(5):
            P.dcp_bwd_delta(out, do, dbuf)
        torch.cuda.synchronize()
        tot, n = P.dcp_profile_read("delta")
        P.dcp_profile_enable(False)
        kern["delta"] = dict(ms=tot / max(n, 1), launches=n)
        delta_note = "fused into the dQ kernel in the step; this is dcp_bwd_delta alone"
    dom = max(("fwd", "dq", "dkv"), key=lambda n: kern[n]["ms"])
    ach = alg[dom] / (kern[dom]["ms"] * 1e-3) / 1e12
    kname = {"fwd": "mfma_fwd_kernel", "dq": "mfma_dq_kernel", "dkv": "mfma_dkv_kernel"}[dom]
    roofline = dict(kernel=kname,
                    bound="mfma", achieved=round(ach, 1), peak=PEAK_BF16_TFLOPS, unit="TFLOP/s",
                    frac=round(ach / PEAK_BF16_TFLOPS, 4),
                    traffic=measured_traffic(kname) if args.config == 2 else None,
                    executed_tflops=round(executed[dom] / (kern[dom]["ms"] * 1e-3) / 1e12, 1))
    delta_bytes = T * w.hq * (4 * w.d + 4)
    per_kernel = {n: dict(ms=round(kern[n]["ms"], 4),
                          tflops=round(alg[n] / (kern[n]["ms"] * 1e-3) / 1e12, 1) if n in alg else None)
                  for n in kern}
    per_kernel["delta"]["GBps"] = round(delta_bytes / (kern["delta"]["ms"] * 1e-3) / 1e9, 1)
    per_kernel["delta"]["frac_hbm"] = round(per_kernel["delta"]["GBps"] / PEAK_HBM_GBPS, 3)
    if delta_note:
        per_kernel["delta"]["note"] = delta_note

    extra = dict(per_kernel=per_kernel, plan_create_ms=round(plan_ms, 3), visible_pairs=pairs,
                 table_rows=int(len(table)), n_seq=int(len(w.cu_seqlens) - 1))
    if not args.no_extra:
        extra["share"] = share_section(torch, P, W, np, steps=max(3, args.steps // 4), warmup=2)
        extra["blockwise_copy"] = copy_section(torch, P, np, plan, q, steps=max(3, args.steps // 2))
        extra["gradient_sum"] = sum_section(torch, P, q, steps=max(3, args.steps // 2))
        extra["short_sequences"] = short_section(torch, P, W, np, steps=30)
        # config 2's batch with the heads of an 8-way tensor-parallel shard: the KV heads no longer divide among the 8
        # XCDs as whole heads, the work lists are dealt into balanced segments instead
        extra["fewer_heads"] = short_section(torch, P, W, np, steps=50, heads=(4, 1), lens=np.diff(w.cu_seqlens))
        extra["other_masks"] = masks_section(torch, P, W, np, steps=3)
        extra["execution_plan"] = executor_section(torch, P, W, np, steps=3)

    # one plain copy of known size (256 MiB read + 256 MiB written) through the library's sum
    # kernel with a single part: the reference dispatch that scales hardware byte counters
    cal_src = torch.empty(128 << 20, dtype=torch.bfloat16, device="cuda").fill_(1.0)
    cal_dst = torch.empty_like(cal_src)
    P.dcp_sum_partials([cal_src], cal_dst)
    torch.cuda.synchronize()
    extra["calibration_copy"] = "sum_kernel<bf16,bf16> with 1 part: 268435456 bytes read, 268435456 bytes written"

    value = flops / (ms * 1e-3) / 1e12
    line = dict(metric="effective attention TFLOP/s fwd+bwd (unmasked FLOPs) and % of bf16 MFMA peak",
                value=round(value, 1), unit="TFLOP/s", pct_of_bf16_mfma_peak=round(100 * value / PEAK_BF16_TFLOPS, 2),
                n_gpus=1, steps=args.steps, warmup=args.warmup, ms_per_step=round(ms, 4), higher_is_better=True,
                scaling="weak", vs_baseline=None, dtype="bf16", data="synthetic",
                config=dict(workload=f"config {args.config}: {w.name}, {T} packed tokens in {len(w.cu_seqlens) - 1} "
                                     f"sequences, {w.hq}/{w.hkv} heads, D {w.d}, block {w.block_size}, mask {w.mask.kind}",
                            global_batch_tokens=T, block_size=w.block_size, parallelism="single GPU"),
                roofline=roofline, extra=extra)
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(w, table, q, k, v, do)
    print(json.dumps(line))


def share_section(torch, P, W, np, steps, warmup):
    """One device's share (1/8 of the computation blocks, 4 divisions) of the 262 144-token causal
    plan: forward into partial slots, LSE merge, backward of the share.  Times the merge kernel
    against HBM bandwidth."""
    w = W.make_workload(5)
    table = P.dcp_build_block_table(w.cu_seqlens, w.block_size, w.ranges)
    n_shares, share_seed, n_div, div_seed = w.share
    sel = W.deal_share(len(table), n_shares, share_seed, 0)
    sub = table[sel]
    slot, n_slots, slot_q = W.deal_divisions(sub[:, 0], n_div, div_seed)
    pairs = int(P.dcp_count_pairs(w.cu_seqlens, w.block_size, sub, w.ranges).sum())
    q, k, v, do = gen_tensors(torch, w, w.tensor_seed)
    T = w.total_tokens
    plan = P.dcp_plan_create(w.cu_seqlens, w.block_size, sub, slot, n_slots)
    o_part = torch.empty((n_slots, w.block_size, w.hq, w.d), dtype=torch.bfloat16, device="cuda")
    lse_part = torch.empty((n_slots, w.hq, w.block_size), dtype=torch.float32, device="cuda")
    out = torch.empty_like(q)
    lse = torch.empty((w.hq, T), dtype=torch.float32, device="cuda")
    dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
    rg = torch.from_numpy(np.ascontiguousarray(w.ranges)).cuda()
    ws = torch.empty(max(256, P.dcp_bwd_workspace_bytes(plan, w.hq, w.hkv, w.d, P.DCP_BF16)), dtype=torch.uint8, device="cuda")
    # global O / LSE for the share's backward: an untimed full-table forward
    full = P.dcp_plan_create(w.cu_seqlens, w.block_size, table)
    out_g, lse_g = torch.empty_like(q), torch.empty_like(lse)
    P.dcp_block_attn_fwd(full, q, k, v, out_g, lse_g, w.softmax_scale, rg)
    torch.cuda.synchronize()

    def step():
        P.dcp_block_attn_fwd(plan, q, k, v, o_part, lse_part, w.softmax_scale, rg)
        P.dcp_merge_partials(plan, o_part, lse_part, out, lse)
        P.dcp_block_attn_bwd(plan, q, k, v, out_g, lse_g, do, dq, dk, dv, w.softmax_scale, ws, rg)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    P.dcp_profile_enable(True)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / steps
    P.dcp_profile_enable(False)
    res = dict(workload=f"config 5: share 0 of {n_shares} of a {T}-token causal plan, {len(sub)} of {len(table)} "
                        f"computation blocks, {n_div} divisions -> {n_slots} partial slots, block {w.block_size}",
               ms_per_step=round(ms, 4), tflops=round(14 * pairs * w.hq * w.d / (ms * 1e-3) / 1e12, 1), steps=steps)
    blk_len = plan.export("BLK_LEN").astype(np.int64)
    mptr = plan.export("MERGE_PTR").astype(np.int64)
    rowhead = w.hq * (2 * w.d + 4)
    merge_bytes = int((blk_len * (np.diff(mptr) + 1)).sum()) * rowhead
    for name in ("fwd", "merge", "delta", "dq", "dkv"):
        tot, n = P.dcp_profile_read(name)
        res[name + "_ms"] = round(tot / max(n, 1), 4)
    res["merge_GBps"] = round(merge_bytes / (res["merge_ms"] * 1e-3) / 1e9, 1)
    res["merge_frac_hbm"] = round(res["merge_GBps"] / PEAK_HBM_GBPS, 3)
    n_parts = np.diff(mptr)
    res["merge_rows_by_partials"] = {int(k): int(blk_len[n_parts == k].sum()) for k in np.unique(n_parts)}
    del o_part, lse_part, plan
    # the merge where every q block really has partials to merge: the WHOLE causal table of the same batch executed as
    # 4 divisions (each q block's rows dealt to 4 slots), forward into the slots, then the merge alone
    slot4, n_slots4, _ = W.deal_divisions(table[:, 0], n_div, div_seed)
    plan4 = P.dcp_plan_create(w.cu_seqlens, w.block_size, table, slot4, n_slots4)
    o4 = torch.empty((n_slots4, w.block_size, w.hq, w.d), dtype=torch.bfloat16, device="cuda")
    l4 = torch.empty((n_slots4, w.hq, w.block_size), dtype=torch.float32, device="cuda")
    P.dcp_block_attn_fwd(plan4, q, k, v, o4, l4, w.softmax_scale, rg)
    P.dcp_merge_partials(plan4, o4, l4, out, lse)
    torch.cuda.synchronize()
    P.dcp_profile_enable(True)
    for _ in range(steps):
        P.dcp_merge_partials(plan4, o4, l4, out, lse)
    torch.cuda.synchronize()
    tot, n = P.dcp_profile_read("merge")
    P.dcp_profile_enable(False)
    mptr4 = plan4.export("MERGE_PTR").astype(np.int64)
    bytes4 = int((blk_len * (np.diff(mptr4) + 1)).sum()) * rowhead
    ms4 = tot / max(n, 1)
    res["merge_whole_table"] = dict(workload=f"the whole {len(table)}-row table as {n_div} divisions -> {n_slots4} partial slots",
                                    rows_by_partials={int(kk): int(blk_len[np.diff(mptr4) == kk].sum()) for kk in np.unique(np.diff(mptr4))},
                                    ms=round(ms4, 4), GBps=round(bytes4 / (ms4 * 1e-3) / 1e9, 1),
                                    frac_hbm=round(bytes4 / (ms4 * 1e-3) / 1e9 / PEAK_HBM_GBPS, 3))
    return res


def executor_section(torch, P, W, np, steps):
    """Config 5's share as an execution plan of 4 divisions (Sec. 4.3): the forward of each division into partial slots,
    the merge, the backward.  Every Q, K and V block a division uses arrives by a transfer (as if all of them were
    remote): Comm.Launch hands a Blockwise Copy per tensor to a second stream, Comm.Wait precedes the division's
    attention, and the transfers of division d + 1 are launched before the attention of division d, into the other of
    two sets of buffers, so that they run beside it.  Timed against the same instructions with the copies in line on
    the compute stream, and against the transfers alone."""
    w = W.make_workload(5)
    table = P.dcp_build_block_table(w.cu_seqlens, w.block_size, w.ranges)
    n_shares, share_seed, n_div, div_seed = w.share
    sub = table[W.deal_share(len(table), n_shares, share_seed, 0)]
    slot, n_slots, _ = W.deal_divisions(sub[:, 0], n_div, div_seed)
    perm = np.random.default_rng(div_seed).permutation(len(sub))
    div = np.empty(len(sub), dtype=np.int64)
    div[perm] = np.arange(len(sub)) % n_div
    q_far, k_far, v_far, do = gen_tensors(torch, w, w.tensor_seed)        # where the blocks come from
    T, B = w.total_tokens, w.block_size
    bufs = [tuple(torch.zeros_like(x) for x in (q_far, k_far, v_far)) for _ in range(2)]
    full = P.dcp_plan_create(w.cu_seqlens, B, sub, slot, n_slots)
    plain = P.dcp_plan_create(w.cu_seqlens, B, sub)
    blk_start, blk_len = full.export("BLK_START").astype(np.int64), full.export("BLK_LEN").astype(np.int64)
    o_part = torch.empty((n_slots, B, w.hq, w.d), dtype=torch.bfloat16, device="cuda")
    lse_part = torch.empty((n_slots, w.hq, B), dtype=torch.float32, device="cuda")
    out, lse = torch.empty_like(q_far), torch.empty((w.hq, T), dtype=torch.float32, device="cuda")
    dq, dk, dv = torch.empty_like(q_far), torch.empty_like(k_far), torch.empty_like(v_far)
    rg = torch.from_numpy(np.ascontiguousarray(w.ranges)).cuda()
    ws = torch.empty(max(256, P.dcp_bwd_workspace_bytes(plain, w.hq, w.hkv, w.d, P.DCP_BF16)), dtype=torch.uint8, device="cuda")
    lists_q, lists_kv, moved = {}, {}, 0
    for d in range(n_div):
        qb, kb = np.unique(sub[div == d, 0]), np.unique(sub[div == d, 1])
        lists_q[d] = P.CopyList(np.stack([blk_start[qb], blk_start[qb], blk_len[qb]], axis=1).astype(np.int32), T, T)
        lists_kv[d] = P.CopyList(np.stack([blk_start[kb], blk_start[kb], blk_len[kb]], axis=1).astype(np.int32), T, T)
        moved += int(blk_len[qb].sum()) * q_far[0].numel() * 2 + 2 * int(blk_len[kb].sum()) * k_far[0].numel() * 2
    fwd = [P.instr_attn_fwd(P.dcp_plan_create(w.cu_seqlens, B, sub[div == d], slot[div == d], n_slots), *bufs[d % 2], o_part, lse_part,
                            w.softmax_scale, rg) for d in range(n_div)]
    tail = [P.instr_merge(full, o_part, lse_part, out, lse),
            P.instr_attn_bwd(plain, q_far, k_far, v_far, out, lse, do, dq, dk, dv, w.softmax_scale, ws, rg)]

    def transfers(d, launch):
        srcs, dsts, lsts = (q_far, k_far, v_far), bufs[d % 2], (lists_q[d], lists_kv[d], lists_kv[d])
        if launch:
            return [P.instr_comm_launch(3 * d + i, lsts[i], srcs[i], dsts[i]) for i in range(3)]
        return [P.instr_copy(lsts[i], srcs[i], dsts[i]) for i in range(3)]
    overlapped = transfers(0, True)
    in_line, only_transfers = [], []
    for d in range(n_div):
        overlapped += [P.instr_comm_wait(3 * d + i) for i in range(3)]
        if d + 1 < n_div:
            overlapped += transfers(d + 1, True)       # runs beside the attention of division d
        overlapped.append(fwd[d])
        in_line += transfers(d, False) + [fwd[d]]
        only_transfers += transfers(d, False)
    side = torch.cuda.Stream()
    res = dict(workload=f"config 5 share as {n_div} divisions; every Q / K / V block a division uses arrives by a transfer: "
                        f"{moved} bytes moved per run", instructions=len(overlapped) + len(tail))
    for name, prog in (("transfers_on_second_stream_ms", P.Program(overlapped + tail)), ("copies_in_line_ms", P.Program(in_line + tail)),
                       ("transfers_alone_ms", P.Program(only_transfers))):
        prog.run(side)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(steps):
            prog.run(side)
        e1.record()
        torch.cuda.synchronize()
        res[name] = round(e0.elapsed_time(e1) / steps, 3)
    res["hidden_ms"] = round(res["copies_in_line_ms"] - res["transfers_on_second_stream_ms"], 3)
    return res


def masks_section(torch, P, W, np, steps):
    """The same step (forward + backward) on the other mask families of the paper at their full shapes: sliding
    window (config 3), lambda (4), causal blockwise (6), shared question (7), and on one causal sequence of the
    paper's maximum length (8).  Not the headline metric."""
    res = {}
    # (config, through WINDOW rows): the window / lambda masks are also timed with the WINDOW mask kind, which
    # takes the window and sink sizes instead of the [T, 4] range array
    for cfg, window_kind in ((3, False), (3, True), (4, False), (4, True), (6, False), (7, False), (8, False)):
        w = W.make_workload(cfg)
        if window_kind:
            table = P.dcp_build_block_table_window(w.cu_seqlens, w.block_size, w.mask.window, w.mask.sink)
            pairs = int(P.dcp_count_pairs_window(w.cu_seqlens, w.block_size, table, w.mask.window, w.mask.sink).sum())
        else:
            table = P.dcp_build_block_table(w.cu_seqlens, w.block_size, w.ranges)
            pairs = int(P.dcp_count_pairs(w.cu_seqlens, w.block_size, table, w.ranges).sum())
        q, k, v, do = gen_tensors(torch, w, w.tensor_seed)
        plan = P.dcp_plan_create(w.cu_seqlens, w.block_size, table)
        out = torch.empty_like(q)
        lse = torch.empty((w.hq, w.total_tokens), dtype=torch.float32, device="cuda")
        dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
        rg = None
        if window_kind:
            P.dcp_plan_set_window(plan, w.mask.window, w.mask.sink)
        else:
            rg = torch.from_numpy(np.ascontiguousarray(w.ranges)).cuda()
        ws = torch.empty(max(256, P.dcp_bwd_workspace_bytes(plan, w.hq, w.hkv, w.d, P.DCP_BF16)), dtype=torch.uint8, device="cuda")

        def step():
            P.dcp_block_attn_fwd(plan, q, k, v, out, lse, w.softmax_scale, rg)
            P.dcp_block_attn_bwd(plan, q, k, v, out, lse, do, dq, dk, dv, w.softmax_scale, ws, rg)

        step()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(steps):
            step()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / steps
        kinds = np.bincount(np.where(table[:, 2] == P.DCP_MASK_WINDOW, P.DCP_MASK_RANGES, table[:, 2]), minlength=3)
        res[w.name + ("_window_kind" if window_kind else "")] = dict(
                           tokens=int(w.total_tokens), table_rows=int(len(table)), rows_none_causal_ranges=[int(x) for x in kinds[:3]],
                           visible_pairs=pairs, ms_per_step=round(ms, 3),
                           tflops=round(14 * pairs * w.hq * w.d / (ms * 1e-3) / 1e12, 1))
        del q, k, v, do, out, lse, dq, dk, dv, ws, plan
    return res


def short_section(torch, P, W, np, steps, seq_len=1024, tokens=65536, heads=(32, 8), lens=None):
    """The headline step on a batch of short sequences: the same 65 536 tokens, heads and block size as config 2, cut
    into equal causal sequences of 1 024 tokens (the short end of the paper's length-scale 0.5 batches, Sec. 7.1):
    every work item is a handful of key tiles long, so the fixed cost of a work item shows.
    lens: other sequence lengths; heads: other (query, KV) head counts (what a tensor-parallel shard would hold)."""
    lens = [seq_len] * (tokens // seq_len) if lens is None else [int(x) for x in lens]
    w = W.custom_workload("causal_short", lens, 1024, heads[0], heads[1], 128, "bf16", W.MaskSpec("causal"), seed=109,
                          input_scale=1.0 / np.sqrt(128))
    table = P.dcp_build_block_table(w.cu_seqlens, w.block_size, w.ranges)
    pairs = int(P.dcp_count_pairs(w.cu_seqlens, w.block_size, table, w.ranges).sum())
    q, k, v, do = gen_tensors(torch, w, 109)
    plan = P.dcp_plan_create(w.cu_seqlens, w.block_size, table)
    out = torch.empty_like(q)
    lse = torch.empty((w.hq, w.total_tokens), dtype=torch.float32, device="cuda")
    dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
    ws = torch.empty(max(256, P.dcp_bwd_workspace_bytes(plan, w.hq, w.hkv, w.d, P.DCP_BF16)), dtype=torch.uint8, device="cuda")

    def step():
        P.dcp_block_attn_fwd(plan, q, k, v, out, lse, w.softmax_scale, None)
        P.dcp_block_attn_bwd(plan, q, k, v, out, lse, do, dq, dk, dv, w.softmax_scale, ws, None)

    # a step takes a few ms here: the chip raises its clocks only after some tens of ms of load, so the warm-up is as
    # long as the timed part (timed cold, five steps read 10 % low)
    for _ in range(max(1, steps)):
        step()
    torch.cuda.synchronize()
    P.dcp_profile_enable(True)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / steps
    unit = pairs * w.hq * w.d
    shape = f"{len(lens)} causal sequences of {seq_len}" if len(set(lens)) == 1 else f"{len(lens)} causal sequences of {min(lens)} .. {max(lens)}"
    res = dict(workload=f"{sum(lens)} tokens in {shape}, {w.hq}/{w.hkv} heads, D {w.d}",
               visible_pairs=pairs, ms_per_step=round(ms, 4), tflops=round(14 * unit / (ms * 1e-3) / 1e12, 1))
    for name, f in (("fwd", 4), ("dq", 4), ("dkv", 6)):
        tot, n = P.dcp_profile_read(name)
        res[name + "_ms"] = round(tot / max(n, 1), 4)
        res[name + "_tflops"] = round(f * unit / (tot / max(n, 1) * 1e-3) / 1e12, 1)
    P.dcp_profile_enable(False)
    return res


def sum_section(torch, P, q, steps):
    """Blockwise Reduction used on gradients: two bf16 partials of the size of dQ summed into a third tensor
    (fp32 accumulation): algorithmic bytes = two reads + one write of every element."""
    a, b, dst = torch.ones_like(q), torch.ones_like(q), torch.empty_like(q)
    P.dcp_sum_partials([a, b], dst)
    torch.cuda.synchronize()
    P.dcp_profile_enable(True)
    for _ in range(steps):
        P.dcp_sum_partials([a, b], dst)
    torch.cuda.synchronize()
    tot, n = P.dcp_profile_read("sum")
    P.dcp_profile_enable(False)
    ms = tot / max(n, 1)
    gbps = 3 * q.numel() * q.element_size() / (ms * 1e-3) / 1e9
    return dict(workload=f"2 bf16 partials of {q.numel()} elements -> bf16", ms=round(ms, 4), GBps=round(gbps, 1),
                frac_hbm=round(gbps / PEAK_HBM_GBPS, 3))


def copy_section(torch, P, np, plan, q, steps):
    """Blockwise Copy of every Q block of the workload from the packed tensor into a block buffer with
    permuted slots (the executor's buffer fill): algorithmic bytes = read + write of every row."""
    blk_start = plan.export("BLK_START").astype(np.int64)
    blk_len = plan.export("BLK_LEN").astype(np.int64)
    B = int(blk_len.max())
    slots = np.random.default_rng(11).permutation(len(blk_start))
    entries = np.stack([blk_start, slots * B, blk_len], axis=1).astype(np.int32)
    buf = torch.empty((len(blk_start) * B,) + tuple(q.shape[1:]), dtype=q.dtype, device="cuda")
    cl = P.CopyList(entries, q.shape[0], buf.shape[0])
    P.dcp_blockwise_copy(cl, q, buf)
    torch.cuda.synchronize()
    P.dcp_profile_enable(True)
    for _ in range(steps):
        P.dcp_blockwise_copy(cl, q, buf)
    torch.cuda.synchronize()
    tot, n = P.dcp_profile_read("copy")
    P.dcp_profile_enable(False)
    ms = tot / max(n, 1)
    nbytes = 2 * int(blk_len.sum()) * q[0].numel() * q.element_size()
    gbps = nbytes / (ms * 1e-3) / 1e9
    return dict(workload=f"{len(entries)} Q blocks ({int(blk_len.sum())} rows of {q[0].numel() * q.element_size()} B) packed -> permuted slots",
                ms=round(ms, 4), GBps=round(gbps, 1), frac_hbm=round(gbps / PEAK_HBM_GBPS, 3))


if __name__ == "__main__":
    main()
