"""dcp_block_attn_bwd_static (the backward with a fixed workspace inside the library, for callers that cannot
allocate) against dcp_block_attn_bwd on the same inputs: the same kernels run, so the results must agree bit for bit.
Two calls in a row on the one shared array, the second on a smaller input; then the refusals."""
import numpy as np
import pytest

from paper_2510_10620_amd import workloads as W
from tests import helpers as H

pytestmark = pytest.mark.gpu


def _both_ways(lens, block, seed):
    import torch
    import paper_2510_10620_amd as P
    w = W.custom_workload("static_ws", lens, block, 8, 2, 128, "bf16", W.MaskSpec("lambda", window=700, sink=40), seed=seed,
                          input_scale=1.0 / np.sqrt(128))
    tensors = W.make_tensors(w)
    table = P.dcp_build_block_table(w.cu_seqlens, w.block_size, w.ranges)
    g = H.GpuRun(w, tensors, table)
    P.dcp_plan_prepare(g.plan, w.hq, w.hkv, w.d, P.DCP_BF16)
    need = P.dcp_bwd_workspace_bytes(g.plan, w.hq, w.hkv, w.d, P.DCP_BF16)
    assert 0 < need <= P.DCP_STATIC_SCRATCH_BYTES
    g.forward_only()
    g.backward_only(g.out, g.lse)                                   # the existing entry point, caller's workspace
    ref = {n: getattr(g, n).clone() for n in ("dq", "dk", "dv")}
    outs = {n: torch.full_like(ref[n], float("nan")) for n in ref}
    P.dcp_block_attn_bwd_static(g.plan, g.q, g.k, g.v, g.out, g.lse, g.dout, outs["dq"], outs["dk"], outs["dv"],
                                w.softmax_scale, g.ranges)
    torch.cuda.synchronize()
    for n in ref:
        assert torch.equal(outs[n].view(torch.int16), ref[n].view(torch.int16)), f"{n} differs from dcp_block_attn_bwd (lens {list(lens)})"
    return (P.dcp_plan_export_dkv_items(g.plan, w.hkv)[:, 4] >= 0).any(), need


def test_static_workspace_backward_matches_and_survives_a_smaller_second_call():
    lens = W.draw_lengths(8192, "lognormal", 512, 4096, seed=2, median=1024)
    cut, need_big = _both_ways(lens, 256, 61)
    assert cut, "the first case is meant to leave partial sums of cut dK/dV items in the shared array"
    _, need_small = _both_ways([700, 333, 90], 128, 62)             # smaller: reuses the array over the first call's contents
    assert need_small < need_big


def test_static_workspace_backward_refuses_what_it_cannot_serve():
    import torch
    import paper_2510_10620_amd as P
    # not prepared: the call must not create the plan's device copies itself
    w = W.custom_workload("static_unprepared", [300, 100], 128, 4, 2, 128, "bf16", W.MaskSpec("causal"), seed=63, input_scale=0.5)
    g = H.GpuRun(w, W.make_tensors(w), H.oracle_table(w))
    dq, dk, dv = torch.zeros_like(g.q), torch.zeros_like(g.k), torch.zeros_like(g.v)
    out, lse = torch.zeros_like(g.q), torch.zeros((w.hq, w.total_tokens), dtype=torch.float32, device="cuda")
    with pytest.raises(P.DcpError) as ei:
        P.dcp_block_attn_bwd_static(g.plan, g.q, g.k, g.v, out, lse, g.dout, dq, dk, dv, w.softmax_scale, g.ranges)
    assert ei.value.status == P.DCP_ERR_INVALID_ARG and "dcp_plan_prepare" in str(ei.value)
    # too large for the fixed array: refused on the host before anything is launched (the tensors are never touched)
    big = W.custom_workload("static_too_big", [300000], 4096, 32, 8, 128, "bf16", W.MaskSpec("causal"), seed=64)
    table = np.array([[i, j, 1 if i == j else 0] for i in range(74) for j in range(i + 1)], dtype=np.int32)
    plan = P.dcp_plan_create(big.cu_seqlens, big.block_size, table)
    assert P.dcp_bwd_workspace_bytes(plan, 32, 8, 128, P.DCP_BF16) > P.DCP_STATIC_SCRATCH_BYTES
    q = torch.zeros((8, 32, 128), dtype=torch.bfloat16, device="cuda")
    k = torch.zeros((8, 8, 128), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(P.DcpError) as ei:
        P.dcp_block_attn_bwd_static(plan, q, k, k, q, lse, q, q, k, k, 0.1, None)
    assert ei.value.status == P.DCP_ERR_WORKSPACE and "static scratch" in str(ei.value)
    assert bool((q == 0).all()) and bool((k == 0).all())
