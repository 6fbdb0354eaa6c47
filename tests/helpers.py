"""Shared helpers for the parity tests: run the HIP path through the Python binding of the C ABI
and the oracle on the same seeded inputs."""
import numpy as np

from oracle import attention as OA
from oracle import blocks as OB
from oracle import masks as OM
from paper_2510_10620_amd import workloads as W


def oracle_table(w):
    """Block table from the oracle's own block generation (dense mask formula)."""
    if w.dense_causal_table:
        return OB.dense_causal_table(w.cu_seqlens, w.block_size)
    return OB.table_from_mask(lambda s, L, r0, r1: OM.dense_rows(w.mask, L, r0, r1), w.cu_seqlens, w.block_size)


def to_torch(w, a, device="cuda"):
    import torch
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).view(torch.bfloat16).to(device)
    return torch.from_numpy(a).to(device)


def from_torch(x):
    import torch
    return x.detach().to(torch.float64).cpu().numpy()


class GpuRun:
    """Holds device tensors of one workload and runs forward / merge / backward via the C ABI."""

    def __init__(self, w, tensors, table, out_slot=None, n_slots=0, impl=0, window=None):
        """window = (window, sink): the table has WINDOW rows; no range array is passed to the library."""
        import torch
        import paper_2510_10620_amd as P
        self.P, self.torch, self.w, self.impl = P, torch, w, impl
        self.table = np.asarray(table, dtype=np.int32).reshape(-1, 3)
        self.plan = P.dcp_plan_create(w.cu_seqlens, w.block_size, self.table, out_slot, n_slots)
        if window is not None:
            P.dcp_plan_set_window(self.plan, *window)
        self.use_slots = out_slot is not None
        self.n_slots = n_slots
        self.q, self.k, self.v = (to_torch(w, tensors[n]) for n in ("q", "k", "v"))
        self.dout = to_torch(w, tensors["dout"]) if "dout" in tensors else None
        self.ranges = None if window is not None else torch.from_numpy(np.ascontiguousarray(w.ranges)).cuda()
        T = w.total_tokens
        self.out = torch.full((T, w.hq, w.d), float("nan"), dtype=self.q.dtype, device="cuda")
        self.lse = torch.full((w.hq, T), float("nan"), dtype=torch.float32, device="cuda")

    def forward(self):
        P, torch, w = self.P, self.torch, self.w
        if self.use_slots:
            self.o_part = torch.full((self.n_slots, w.block_size, w.hq, w.d), float("nan"), dtype=self.q.dtype, device="cuda")
            self.lse_part = torch.full((self.n_slots, w.hq, w.block_size), float("nan"), dtype=torch.float32, device="cuda")
            P.dcp_block_attn_fwd(self.plan, self.q, self.k, self.v, self.o_part, self.lse_part, w.softmax_scale, self.ranges, self.impl)
            P.dcp_merge_partials(self.plan, self.o_part, self.lse_part, self.out, self.lse)
        else:
            P.dcp_block_attn_fwd(self.plan, self.q, self.k, self.v, self.out, self.lse, w.softmax_scale, self.ranges, self.impl)
        torch.cuda.synchronize()
        return from_torch(self.out), from_torch(self.lse)

    def forward_only(self):
        """forward() without copying the results to the host."""
        P, torch, w = self.P, self.torch, self.w
        if self.use_slots:
            if not hasattr(self, "o_part"):
                self.o_part = torch.full((self.n_slots, w.block_size, w.hq, w.d), float("nan"), dtype=self.q.dtype, device="cuda")
                self.lse_part = torch.full((self.n_slots, w.hq, w.block_size), float("nan"), dtype=torch.float32, device="cuda")
            P.dcp_block_attn_fwd(self.plan, self.q, self.k, self.v, self.o_part, self.lse_part, w.softmax_scale, self.ranges, self.impl)
            P.dcp_merge_partials(self.plan, self.o_part, self.lse_part, self.out, self.lse)
        else:
            P.dcp_block_attn_fwd(self.plan, self.q, self.k, self.v, self.out, self.lse, w.softmax_scale, self.ranges, self.impl)
        torch.cuda.synchronize()

    def backward_only(self, out, lse):
        """backward() on device tensors, results left on the device (dq, dk, dv)."""
        P, torch, w = self.P, self.torch, self.w
        T = w.total_tokens
        self.dq = torch.full((T, w.hq, w.d), float("nan"), dtype=self.q.dtype, device="cuda")
        self.dk = torch.full((T, w.hkv, w.d), float("nan"), dtype=self.q.dtype, device="cuda")
        self.dv = torch.full((T, w.hkv, w.d), float("nan"), dtype=self.q.dtype, device="cuda")
        nbytes = P.dcp_bwd_workspace_bytes(self.plan, w.hq, w.hkv, w.d, P.DCP_BF16 if w.dtype == "bf16" else P.DCP_F32)
        ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device="cuda")
        P.dcp_block_attn_bwd(self.plan, self.q, self.k, self.v, out, lse, self.dout, self.dq, self.dk, self.dv,
                             w.softmax_scale, ws, self.ranges, self.impl)
        torch.cuda.synchronize()

    def backward(self, out=None, lse=None):
        """Uses the forward's out/lse unless the global ones are passed (device tensors)."""
        P, torch, w = self.P, self.torch, self.w
        out = self.out if out is None else out
        lse = self.lse if lse is None else lse
        T = w.total_tokens
        self.dq = torch.full((T, w.hq, w.d), float("nan"), dtype=self.q.dtype, device="cuda")
        self.dk = torch.full((T, w.hkv, w.d), float("nan"), dtype=self.q.dtype, device="cuda")
        self.dv = torch.full((T, w.hkv, w.d), float("nan"), dtype=self.q.dtype, device="cuda")
        nbytes = P.dcp_bwd_workspace_bytes(self.plan, w.hq, w.hkv, w.d, P.DCP_BF16 if w.dtype == "bf16" else P.DCP_F32)
        ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device="cuda")
        P.dcp_block_attn_bwd(self.plan, self.q, self.k, self.v, out, lse, self.dout, self.dq, self.dk, self.dv,
                             w.softmax_scale, ws, self.ranges, self.impl)
        torch.cuda.synchronize()
        return from_torch(self.dq), from_torch(self.dk), from_torch(self.dv)


def oracle_full(w, tensors, table, select=None, lse=None, delta=None, bwd=True, seqs=None, heads=None, window=None):
    """Oracle forward (+ backward) on the full tensors, or on q heads `heads` (a list that must
    cover whole KV groups' worth of the heads it names: heads are given as (q_heads, kv_head))."""
    q, k, v = (W.to_f64(w, tensors[n]) for n in ("q", "k", "v"))
    do = W.to_f64(w, tensors["dout"]) if "dout" in tensors else None
    if heads is not None:
        qh, kvh = heads
        q, k, v = q[:, qh], k[:, [kvh]], v[:, [kvh]]
        do = do[:, qh] if do is not None else None
        lse = lse[qh] if lse is not None else None
        delta = delta[qh] if delta is not None else None
    vis = OB.Visibility(w.cu_seqlens, w.block_size, table, None if window is not None else w.ranges, select=select, window=window)
    O, LSE = OA.attention_fwd(q, k, v, w.cu_seqlens, vis, w.softmax_scale, seqs=seqs)
    res = dict(out=O, lse=LSE)
    if bwd:
        dq, dk, dv = OA.attention_bwd(q, k, v, do, w.cu_seqlens, vis, w.softmax_scale, lse=lse, delta=delta, seqs=seqs)
        res.update(dq=dq, dk=dk, dv=dv)
    return res


def _cmp_mask(a, b):
    same_inf = np.isinf(b) & (a == b)
    return ~np.isnan(b) & ~same_inf


def max_abs(a, b):
    """Max abs difference where the reference b is finite or both are equal infinities; positions
    where b is NaN (not computed by the oracle) are ignored."""
    a, b = np.asarray(a, np.float64), np.asarray(b, np.float64)
    cmp = _cmp_mask(a, b)
    if not cmp.any():
        return 0.0
    d = np.abs(a[cmp] - b[cmp])
    return float(np.nan_to_num(d, nan=np.inf, posinf=np.inf).max())


def err_stats(a, b, knee, by_row=False):
    """Errors of a against the reference b, split at |b| = knee: `raw` the largest |a - b| anywhere, `rms` its root mean
    square, `low` the largest
    |a - b| where |b| < knee, `high_rel` the largest |a - b| / |b| where |b| >= knee, `max_ref` the largest |b|.
    by_row: the magnitude that decides the side and divides the error is the largest |b| of the element's row
    (last axis) instead of the element's own."""
    a, b = np.asarray(a, np.float64), np.asarray(b, np.float64)
    cmp = _cmp_mask(a, b)
    if not cmp.any():
        return dict(raw=0.0, low=0.0, high_rel=0.0, max_ref=0.0, rms=0.0)
    mag = np.abs(b)
    if by_row:
        mag = np.broadcast_to(np.where(np.isfinite(mag), mag, 0.0).max(axis=-1, keepdims=True), b.shape)
    d = np.nan_to_num(np.abs(a[cmp] - b[cmp]), nan=np.inf, posinf=np.inf)
    m = mag[cmp]
    lo, hi = m < knee, m >= knee
    fin = np.isfinite(d)
    return dict(raw=float(d.max()), low=float(d[lo].max()) if lo.any() else 0.0,
                rms=float(np.sqrt(np.mean(d[fin] ** 2))) if fin.any() else 0.0,
                high_rel=float((d[hi] / m[hi]).max()) if hi.any() else 0.0,
                max_ref=float(np.where(np.isfinite(np.abs(b[cmp])), np.abs(b[cmp]), 0.0).max()))


# Tolerances.  LSE (fp32): max abs 1e-5.  fp32 I/O: max abs 1e-4.  bf16 I/O: plain max abs 2e-2 wherever
# |reference| < 4.  From 4 on the bf16 output grid alone uses up most of that bound (half an ulp is 0.0156 on [4, 8),
# 0.031 on [8, 16)), so there the bound is relative: |error| <= 2^-7 |reference|, one bf16 ulp at the lower end of a
# binade -- half an ulp for rounding the output, as much again for the rounding of the P / dS operands of the second
# GEMM.  Only dV reaches such values (the first keys of a sequence, seen by every later query, with dO ~ N(0, 1));
# the largest relative error measured there at full size is 5.2e-3.
# Because the benchmark inputs are scaled by 1/sqrt(D), most outputs are far smaller than 2e-2 and the absolute bound
# alone would say little; every comparison therefore also requires the largest error to stay below 2^-6 (1.6 %) of the
# largest reference magnitude of the compared tensor (measured: 0.2-0.5 %).
# by_row (only where a test says why): a gradient row that sums very many large terms which cancel.  All D elements
# of the row share the coefficients (P or dS) whose rounding to bf16 makes the error, so the error of every element
# is about 2^-9 of the row's root-mean-square, whatever the element's own value; the row's largest |ref| then takes
# the place of |ref| in the bound above.
TOL = {"bf16": dict(o=2e-2, lse=1e-5, knee=4.0, rel=2.0 ** -7, rel_max=2.0 ** -6),
       "f32": dict(o=1e-4, lse=1e-5, knee=None, rel=None, rel_max=None)}


def check(w, got, ref, names, label="", verbose=True, by_row=()):
    """Asserts the tolerances above for every named tensor; returns {name: raw max abs error}.  by_row: names of the
    tensors judged by row.  The raw error, the error below the knee and the relative error above it are printed
    (pytest shows them with -rA or -s)."""
    tol = TOL[w.dtype]
    errs, lines = {}, []
    for n in names:
        if n == "lse" or tol["knee"] is None:
            err, lim = max_abs(got[n], ref[n]), (tol["lse"] if n == "lse" else tol["o"])
            errs[n] = err
            lines.append(f"{n} {err:.2e}")
            assert err <= lim, f"{label} {n}: max abs err {err:.3e} > {lim:.1e}"
            continue
        st = err_stats(got[n], ref[n], tol["knee"], n in by_row)
        errs[n] = st["raw"]
        lines.append(f"{n}{' [by row]' if n in by_row else ''} raw {st['raw']:.2e} rms {st['rms']:.1e} (|ref|<{tol['knee']:g}: {st['low']:.2e}; above: rel {st['high_rel']:.2e}; max|ref| {st['max_ref']:.3g})")
        assert st["low"] <= tol["o"], f"{label} {n}: max abs err {st['low']:.3e} > {tol['o']:.1e} where |ref| < {tol['knee']:g}"
        assert st["high_rel"] <= tol["rel"], f"{label} {n}: relative err {st['high_rel']:.3e} > {tol['rel']:.1e} where |ref| >= {tol['knee']:g}"
        if n not in by_row and st["max_ref"] > 0:
            lines[-1] += f" [{100 * st['raw'] / st['max_ref']:.2f} % of max|ref|]"
            assert st["raw"] <= tol["rel_max"] * st["max_ref"], \
                f"{label} {n}: max abs err {st['raw']:.3e} is more than {tol['rel_max']:.3g} of max |ref| {st['max_ref']:.3e}"
    if verbose or by_row:
        print(label, "; ".join(lines), flush=True)
    return errs
