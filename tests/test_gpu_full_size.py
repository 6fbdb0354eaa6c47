"""Parity at the benchmark's full sizes and launch configuration (configs 2-5, the two remaining mask
families of the paper at the same scale, 6-7, and one causal sequence of the paper's maximum length, 8): the HIP path on the
whole batch, checked (a) against the fp64 oracle on sampled query-row windows (complete O, LSE and
dQ for the window's rows; complete dK / dV for the keys only the window sees) and, for config 2, on
every sequence for one whole KV group (all rows of O, LSE, dQ, dK, dV: the keys at the start of a long
sequence, which thousands of query tiles and the cut work items accumulate into, included);
(b) on EVERY element against linear-time closed forms (tests/closed_forms.py): with Q = 0 the softmax is
uniform over the visible set, so LSE = ln n, O = mean of the visible V, dV = sum over viewers of
dO / n, dK = 0; with all keys of a sequence identical (scores of order 1) the softmax is uniform again,
LSE = s + ln n, dQ = 0 and dK has a closed form, checked on every element of two KV heads; and
(c) on the invariants of the backward at full size with the real inputs: sum_j dV_j = sum of dO over the
query heads of the group and the rows of the sequence, sum_j dK_j = 0."""
import numpy as np
import pytest

from oracle import attention as OA
from oracle import blocks as OB
from paper_2510_10620_amd import workloads as W
from tests import helpers as H
from tests.closed_forms import identical_k_dk, q0_closed_form

pytestmark = pytest.mark.gpu


def _knee_errors(got, exp, knee=4.0):
    """(largest |got - exp|, the largest where |exp| < knee, the largest |got - exp| / |exp| where |exp| >= knee) of two
    device tensors: the bf16 tolerance of tests/helpers.py evaluated on the device."""
    import torch
    d = (got.float() - exp).abs()
    mag = exp.abs()
    lo, hi = mag < knee, mag >= knee
    low = d[lo].max().item() if bool(lo.any()) else 0.0
    rel = (d[hi] / mag[hi]).max().item() if bool(hi.any()) else 0.0
    return d.max().item(), low, rel


def _windows(w):
    """Query-row windows {sequence: (r0, r1)} per probe: the tail of the longest and the shortest
    sequence, and a window across the first block boundary of the longest."""
    lens = np.diff(w.cu_seqlens.astype(np.int64))
    long_s, short_s = int(np.argmax(lens)), int(np.argmin(lens))
    B = w.block_size
    probes = [("tail_long", long_s, max(0, lens[long_s] - 384), lens[long_s]),
              ("tail_short", short_s, max(0, lens[short_s] - 256), lens[short_s])]
    if lens[long_s] > B + 64:
        probes.append(("block_edge", long_s, B - 64, B + 64))
    if w.share:   # a share touches only some blocks: also take one whole mid-length sequence
        mid = int(np.argmin(np.abs(lens - 14000)))
        probes.append(("tail_whole_seq", mid, 0, lens[mid]))
    return [(n, s, int(a), int(b)) for n, s, a, b in probes]


@pytest.mark.parametrize("cfg", [2, 3, 4, 5, 6, 7, 8])
def test_full_size_config(cfg):
    import torch
    import paper_2510_10620_amd as P
    w = W.make_workload(cfg)
    tensors = W.make_tensors(w)
    table = P.dcp_build_block_table(w.cu_seqlens, w.block_size, w.ranges)
    sel, slot, n_slots = None, None, 0
    sub = table
    if w.share:
        n_shares, share_seed, n_div, div_seed = w.share
        sel = W.deal_share(len(table), n_shares, share_seed, 0)
        sub = table[sel]
        slot, n_slots, _ = W.deal_divisions(sub[:, 0], n_div, div_seed)
    g = H.GpuRun(w, tensors, sub, slot, n_slots)          # AUTO -> MFMA kernels, as bench.py
    g.forward_only()
    out_g, lse_g = g.out, g.lse
    gfull = None
    if w.share:                                            # global O / LSE of the whole plan
        gfull = H.GpuRun(w, tensors, table)
        gfull.forward_only()
        out_g, lse_g = gfull.out, gfull.lse
    g.backward_only(out_g, lse_g)
    G = w.hq // w.hkv
    T = w.total_tokens

    # ---- (a) sampled oracle windows, query heads of KV group 0 and of the last KV group
    for kvh in (0, w.hkv - 1):
        qh = list(range(kvh * G, kvh * G + G))
        for name, s, r0, r1 in _windows(w):
            if name == "tail_whole_seq" and kvh != 0:
                continue
            b = int(w.cu_seqlens[s])
            rows = {s: (r0, r1)}
            q, k, v, do = (W.to_f64(w, tensors[nm][:, hs]) for nm, hs in (("q", qh), ("k", [kvh]), ("v", [kvh]), ("dout", qh)))
            vis_full = OB.Visibility(w.cu_seqlens, w.block_size, table, w.ranges)
            vis = OB.Visibility(w.cu_seqlens, w.block_size, table, w.ranges, select=sel)
            O, LSE = OA.attention_fwd(q, k, v, w.cu_seqlens, vis, w.softmax_scale, seqs=[s], rows=rows)
            lse_ref, delta_ref = None, None
            if w.share:
                Of, Lf = OA.attention_fwd(q, k, v, w.cu_seqlens, vis_full, w.softmax_scale, seqs=[s], rows=rows)
                lse_ref = Lf
                delta_ref = np.einsum("thd,thd->ht", np.nan_to_num(Of), do)
                # the library's full-table forward is itself checked on these rows
                sl = slice(b + r0, b + r1)
                H.check(w, dict(out=H.from_torch(gfull.out[sl][:, qh]), lse=H.from_torch(gfull.lse[qh][:, sl])),
                        dict(out=Of[sl], lse=Lf[:, sl]), ("out", "lse"), f"cfg{cfg} {name} kv{kvh} full-table")
            dq, dk, dv = OA.attention_bwd(q, k, v, do, w.cu_seqlens, vis, w.softmax_scale, lse=lse_ref, delta=delta_ref,
                                          seqs=[s], rows=rows)
            sl = slice(b + r0, b + r1)
            got = dict(out=H.from_torch(g.out[sl][:, qh]), lse=H.from_torch(g.lse[qh][:, sl]), dq=H.from_torch(g.dq[sl][:, qh]))
            ref = dict(out=O[sl], lse=LSE[:, sl], dq=dq[sl])
            names = ["out", "lse", "dq"]
            if name.startswith("tail"):                    # keys of a tail window are seen by the window only
                got.update(dk=H.from_torch(g.dk[sl][:, [kvh]]), dv=H.from_torch(g.dv[sl][:, [kvh]]))
                ref.update(dk=dk[sl], dv=dv[sl])
                names += ["dk", "dv"]
            H.check(w, got, ref, names, f"cfg{cfg} {name} kv{kvh}")

    # ---- (a2) config 2: the oracle on every sequence for one whole KV group -- every row of O, LSE, dQ, dK, dV
    if cfg == 2:
        kvh = 3
        qh = list(range(kvh * G, kvh * G + G))
        ref = H.oracle_full(w, tensors, table, heads=(qh, kvh))
        got = dict(out=H.from_torch(g.out[:, qh]), lse=H.from_torch(g.lse[qh]), dq=H.from_torch(g.dq[:, qh]),
                   dk=H.from_torch(g.dk[:, [kvh]]), dv=H.from_torch(g.dv[:, [kvh]]))
        H.check(w, got, ref, ("out", "lse", "dq", "dk", "dv"), f"cfg{cfg} whole KV group {kvh}")
        # the first 128 keys of the longest sequence: the rows most query tiles accumulate into
        b0 = int(w.cu_seqlens[int(np.argmax(np.diff(w.cu_seqlens)))])
        H.check(w, {n: got[n][b0:b0 + 128] for n in ("dk", "dv")}, {n: ref[n][b0:b0 + 128] for n in ("dk", "dv")},
                ("dk", "dv"), f"cfg{cfg} first keys of the longest sequence, KV head {kvh}")

    # ---- (c) invariants of the backward on the real inputs (full tables): rows of P sum to 1, rows of dS to 0
    if not w.share:
        cu = w.cu_seqlens.astype(np.int64)
        seg = torch.from_numpy(np.repeat(np.arange(len(cu) - 1), np.diff(cu))).cuda()
        n_seq = len(cu) - 1
        def seq_sum(x):   # [T, H, D] -> [n_seq, H, D] in fp64
            return torch.zeros((n_seq,) + tuple(x.shape[1:]), dtype=torch.float64, device="cuda").index_add_(0, seg, x.double())
        do_sum = seq_sum(g.dout).reshape(n_seq, w.hkv, G, w.d).sum(dim=2)
        dv_sum, dk_sum = seq_sum(g.dv), seq_sum(g.dk)
        # what the bf16 rounding of the outputs and of the P / dS operands allows: each term carries an independent
        # relative error of about 2^-9, so the sum's error has a standard deviation near 2^-9 sqrt(sum_j x_j^2);
        # the bound is 6 * 2^-8 of that root (about 15 standard deviations) plus a small floor
        dv_rss = torch.sqrt(seq_sum(g.dv.double() ** 2))
        dk_rss = torch.sqrt(seq_sum(g.dk.double() ** 2))
        dv_ratio = ((dv_sum - do_sum).abs() / (6 * 2.0 ** -8 * dv_rss + 1e-3)).max().item()
        dk_ratio = (dk_sum.abs() / (6 * 2.0 ** -8 * dk_rss + 1e-3)).max().item()
        print(f"cfg{cfg} invariants: |sum dV - sum dO| max {(dv_sum - do_sum).abs().max().item():.2e} (|sum dO| max "
              f"{do_sum.abs().max().item():.1f}), |sum dK| max {dk_sum.abs().max().item():.2e} (rss max {dk_rss.max().item():.2e}); "
              f"error / bound: dV {dv_ratio:.2f}, dK {dk_ratio:.2f}", flush=True)
        assert dv_ratio <= 1.0 and dk_ratio <= 1.0

    # ---- (b) Q = 0: closed form on every element
    v64, do64 = W.to_f64(w, tensors["v"]), W.to_f64(w, tensors["dout"])
    n_glob = None
    if w.share:
        n_glob, O_glob, _ = q0_closed_form(w, table, v64, do64)
    n, O_ref, dV_ref = q0_closed_form(w, sub, v64, do64, n_glob)
    g.q.zero_()
    g.forward_only()
    if w.share:                                            # global O / LSE from the closed form itself
        og = torch.from_numpy(O_glob).to("cuda", torch.bfloat16).repeat_interleave(G, dim=1).contiguous()
        lg = torch.from_numpy(np.log(np.maximum(n_glob, 1))).to("cuda", torch.float32).expand(w.hq, T).contiguous()
        g.backward_only(og, lg)
    else:
        g.backward_only(g.out, g.lse)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    o_exp = dev(O_ref.astype(np.float32)).repeat_interleave(G, dim=1)
    with np.errstate(divide="ignore"):
        lse_exp = dev(np.log(n).astype(np.float32))
    o_err = (g.out.float() - o_exp).abs().max().item()
    fin = torch.isfinite(lse_exp)
    lse_err = (g.lse[:, fin] - lse_exp[fin]).abs().max().item()
    assert bool((g.lse[:, ~fin] == float("-inf")).all())
    dv_exp = dev(dV_ref.astype(np.float32))
    dv_raw, dv_low, dv_rel = _knee_errors(g.dv, dv_exp)
    dk_max = g.dk.float().abs().max().item()
    print(f"cfg{cfg} Q=0 closed form: out {o_err:.2e} lse {lse_err:.2e} dv raw {dv_raw:.2e} (|ref|<4: {dv_low:.2e}; above: rel "
          f"{dv_rel:.2e}; max|ref| {dv_exp.abs().max().item():.2f}) |dk| {dk_max:.2e}", flush=True)
    assert o_err <= 2e-2 and lse_err <= 1e-5 and dv_low <= 2e-2 and dv_rel <= 2.0 ** -7 and dk_max <= 2e-2

    # ---- (b2) all keys of a sequence identical, scores of order 1 (q x 8, k row x 16: exact in bf16): uniform softmax
    # again, LSE = s_i + ln n_i with s_i = scale q_i . k, same O and dV as above, dQ = 0 (a share: its closed form),
    # dK from its closed form for the first and the last KV head
    cu = w.cu_seqlens.astype(np.int64)
    first = torch.from_numpy(np.repeat(cu[:-1], np.diff(cu))).cuda()
    g.q.copy_(H.to_torch(w, tensors["q"]) * 8)
    g.k.copy_((H.to_torch(w, tensors["k"]) * 16)[first])
    q64 = W.to_f64(w, tensors["q"]) * 8
    k64 = (W.to_f64(w, tensors["k"]) * 16)[np.repeat(cu[:-1], np.diff(cu))]
    s_i = w.softmax_scale * np.einsum("tgxd,tgd->gxt", q64.reshape(T, w.hkv, G, w.d), k64).reshape(w.hq, T)
    g.forward_only()
    N = n if n_glob is None else n_glob
    if w.share:
        lg = torch.from_numpy(s_i + np.log(np.maximum(N, 1))[None, :]).to("cuda", torch.float32).contiguous()
        g.backward_only(og, lg)
    else:
        g.backward_only(g.out, g.lse)
    o_err = (g.out.float() - o_exp).abs().max().item()
    with np.errstate(divide="ignore"):
        lse_exp = dev((s_i + np.log(n)[None, :]).astype(np.float32))
    fin = torch.isfinite(lse_exp)
    lse_err = (g.lse[fin] - lse_exp[fin]).abs().max().item()
    assert bool((g.lse[~fin] == float("-inf")).all())
    dv_raw, dv_low, dv_rel = _knee_errors(g.dv, dv_exp)
    if w.share:
        coef = (n / np.maximum(N, 1))[:, None, None] * np.einsum("tgxd,tgd->tgx", do64.reshape(T, w.hkv, G, w.d), O_ref - O_glob)
        dq_exp = dev((w.softmax_scale * coef[..., None] * k64[:, :, None, :]).astype(np.float32).reshape(T, w.hq, w.d))
        dq_err = (g.dq.float() - dq_exp).abs().max().item()
    else:
        dq_err = g.dq.float().abs().max().item()
    dk_err, dk_mag = 0.0, 0.0
    for kvh in (0, w.hkv - 1):
        dk_ref = identical_k_dk(w, sub, q64, v64, do64, kvh, N, O_glob if w.share else O_ref)
        dk_exp = dev(dk_ref.astype(np.float32))
        dk_err = max(dk_err, (g.dk[:, kvh].float() - dk_exp).abs().max().item())
        dk_mag = max(dk_mag, float(np.abs(dk_ref).max()))
    print(f"cfg{cfg} identical keys closed form: out {o_err:.2e} lse {lse_err:.2e} dv raw {dv_raw:.2e} (|ref|<4: {dv_low:.2e}; "
          f"above: rel {dv_rel:.2e}) dq {dq_err:.2e} dk {dk_err:.2e} (max|dk ref| {dk_mag:.2f})", flush=True)
    assert o_err <= 2e-2 and lse_err <= 1e-5 and dv_low <= 2e-2 and dv_rel <= 2.0 ** -7 and dq_err <= 2e-2 and dk_err <= 2e-2


@pytest.mark.parametrize("cfg", [3, 4])
def test_full_size_window_kind_is_the_ranges_route_bit_for_bit(cfg):
    """Configs 3 (window 4096) and 4 (window 8192, 64 sink tokens) through WINDOW rows, which take two numbers instead
    of the [T, 4] range array: the kernels work out the same per-token ranges, so every output must equal, bit for
    bit, what the RANGES route gives on the same batch (that route is checked against the oracle above)."""
    import torch
    import paper_2510_10620_amd as P
    w = W.make_workload(cfg)
    tensors = W.make_tensors(w)
    t_rng = P.dcp_build_block_table(w.cu_seqlens, w.block_size, w.ranges)
    t_win = P.dcp_build_block_table_window(w.cu_seqlens, w.block_size, w.mask.window, w.mask.sink)
    assert np.array_equal(t_win[:, :2], t_rng[:, :2])
    assert np.array_equal(np.where(t_win[:, 2] == W.MASK_WINDOW, W.MASK_RANGES, t_win[:, 2]), t_rng[:, 2])
    assert int(P.dcp_count_pairs_window(w.cu_seqlens, w.block_size, t_win, w.mask.window, w.mask.sink).sum()) == \
        int(P.dcp_count_pairs(w.cu_seqlens, w.block_size, t_rng, w.ranges).sum())
    a = H.GpuRun(w, tensors, t_rng)
    b = H.GpuRun(w, tensors, t_win, window=(w.mask.window, w.mask.sink))
    for g in (a, b):
        g.forward_only()
        g.backward_only(g.out, g.lse)
    for name in ("out", "lse", "dq", "dk", "dv"):
        assert torch.equal(getattr(a, name), getattr(b, name)), name
