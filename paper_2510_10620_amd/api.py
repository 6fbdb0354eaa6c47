"""Thin Python binding of the C ABI in include/dcp.h: same names, argument marshalling only.
Host-side calls take numpy int32 arrays; launching calls take torch tensors (device memory and
the current HIP stream come from PyTorch) and run entirely in the library's kernels."""
import ctypes

import numpy as np

from . import _lib
from ._lib import Tensors

DCP_OK = 0
DCP_ERR_INVALID_ARG, DCP_ERR_BAD_CU_SEQLENS, DCP_ERR_BAD_TABLE = -1, -2, -3
DCP_ERR_UNSUPPORTED, DCP_ERR_WORKSPACE, DCP_ERR_HIP = -4, -5, -6
DCP_MASK_NONE, DCP_MASK_CAUSAL, DCP_MASK_RANGES, DCP_MASK_SKIP, DCP_MASK_WINDOW = 0, 1, 2, 3, 4
DCP_BF16, DCP_F32 = 0, 1
DCP_IMPL_AUTO, DCP_IMPL_SCALAR, DCP_IMPL_MFMA = 0, 1, 2
EXPORTS = dict(BLK_START=0, BLK_LEN=1, BLK_SEQ=2, FWD_PTR=3, FWD_IDX=4, BWDQ_PTR=5, BWDQ_IDX=6,
               BWDKV_PTR=7, BWDKV_IDX=8, SLOT_QBLK=9, MERGE_PTR=10, MERGE_IDX=11)


class DcpError(RuntimeError):
    def __init__(self, status, msg):
        super().__init__(f"dcp status {status}: {msg}")
        self.status = status


def _check(st):
    if st != DCP_OK:
        raise DcpError(st, _lib.load().dcp_last_error().decode())


def _i32(a):
    if a is None:
        return None, None
    arr = np.ascontiguousarray(a, dtype=np.int32)
    return arr, arr.ctypes.data_as(_lib.i32p)


def dcp_last_error():
    return _lib.load().dcp_last_error().decode()


def dcp_version():
    return _lib.load().dcp_version().decode()


def dcp_build_block_table(cu_seqlens, block_size, attn_ranges):
    """-> int32[n, 3] table of (q_blk, kv_blk, mask_kind)."""
    lib = _lib.load()
    cu, cu_p = _i32(cu_seqlens)
    rg, rg_p = _i32(attn_ranges)
    n = ctypes.c_int64(0)
    _check(lib.dcp_build_block_table(cu_p, len(cu) - 1, block_size, rg_p, None, 0, ctypes.byref(n)))
    table = np.zeros((n.value, 3), dtype=np.int32)
    _check(lib.dcp_build_block_table(cu_p, len(cu) - 1, block_size, rg_p, table.ctypes.data_as(_lib.i32p), n.value, ctypes.byref(n)))
    return table


def dcp_build_block_table_window(cu_seqlens, block_size, window, sink=0):
    """-> int32[n, 3] table for a sliding window of `window` keys with `sink` sink tokens; edge tiles are WINDOW rows."""
    lib = _lib.load()
    cu, cu_p = _i32(cu_seqlens)
    n = ctypes.c_int64(0)
    _check(lib.dcp_build_block_table_window(cu_p, len(cu) - 1, block_size, window, sink, None, 0, ctypes.byref(n)))
    table = np.zeros((n.value, 3), dtype=np.int32)
    _check(lib.dcp_build_block_table_window(cu_p, len(cu) - 1, block_size, window, sink, table.ctypes.data_as(_lib.i32p),
                                            n.value, ctypes.byref(n)))
    return table


def dcp_count_pairs_window(cu_seqlens, block_size, table, window, sink=0):
    lib = _lib.load()
    cu, cu_p = _i32(cu_seqlens)
    tb, tb_p = _i32(np.asarray(table).reshape(-1, 3))
    out = np.zeros(len(tb), dtype=np.int64)
    _check(lib.dcp_count_pairs_window(cu_p, len(cu) - 1, block_size, tb_p, len(tb), window, sink, out.ctypes.data_as(_lib.i64p)))
    return out


def dcp_plan_set_window(plan, window, sink=0):
    _check(_lib.load().dcp_plan_set_window(plan.handle, int(window), int(sink)))


def dcp_count_pairs(cu_seqlens, block_size, table, attn_ranges=None):
    lib = _lib.load()
    cu, cu_p = _i32(cu_seqlens)
    tb, tb_p = _i32(np.asarray(table).reshape(-1, 3))
    rg, rg_p = _i32(attn_ranges)
    out = np.zeros(len(tb), dtype=np.int64)
    _check(lib.dcp_count_pairs(cu_p, len(cu) - 1, block_size, tb_p, len(tb), rg_p, out.ctypes.data_as(_lib.i64p)))
    return out


def dcp_comm_volume(cu_seqlens, block_size, table, blk_dev, comp_dev, n_devices, q_bytes, kv_bytes, o_bytes):
    """-> dict(pairwise, connectivity, hyperedges, send[n_devices], recv[n_devices]); host only."""
    lib = _lib.load()
    cu, cu_p = _i32(cu_seqlens)
    tb = np.ascontiguousarray(np.asarray(table, dtype=np.int32).reshape(-1, 3))
    bd, bd_p = _i32(blk_dev)
    cd, cd_p = _i32(comp_dev)
    pw, cn, ne = ctypes.c_int64(0), ctypes.c_int64(0), ctypes.c_int64(0)
    send = np.zeros(n_devices, dtype=np.int64)
    recv = np.zeros(n_devices, dtype=np.int64)
    _check(lib.dcp_comm_volume(cu_p, len(cu) - 1, block_size, tb.ctypes.data_as(_lib.i32p), len(tb), bd_p, cd_p, n_devices,
                               q_bytes, kv_bytes, o_bytes, ctypes.byref(pw), ctypes.byref(cn), ctypes.byref(ne),
                               send.ctypes.data_as(_lib.i64p), recv.ctypes.data_as(_lib.i64p)))
    return dict(pairwise=pw.value, connectivity=cn.value, hyperedges=ne.value, send=send.tolist(), recv=recv.tolist())


class Plan:
    """Owner of a dcp_plan_t*."""

    def __init__(self, handle, n_slots, block_size, total_tokens):
        self.handle, self.n_slots, self.block_size, self.total_tokens = handle, n_slots, block_size, total_tokens

    def export(self, which):
        return dcp_plan_export(self, which)

    def destroy(self):
        if self.handle:
            dcp_plan_destroy(self)

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def dcp_plan_create(cu_seqlens, block_size, table, out_slot=None, n_slots=0):
    lib = _lib.load()
    cu, cu_p = _i32(cu_seqlens)
    tb = np.ascontiguousarray(np.asarray(table, dtype=np.int32).reshape(-1, 3))
    sl, sl_p = _i32(out_slot)
    h = ctypes.c_void_p()
    _check(lib.dcp_plan_create(ctypes.byref(h), cu_p, len(cu) - 1, block_size, tb.ctypes.data_as(_lib.i32p), len(tb), sl_p, n_slots))
    return Plan(h, n_slots if out_slot is not None else 0, block_size, int(cu[-1]) if len(cu) else 0)


def dcp_plan_set_block_buffers(plan, q_slot, n_q_slots, kv_slot, n_kv_slots):
    """Q-type tensors become [n_q_slots * block_size, ...] buffers, KV-type [n_kv_slots * block_size, ...]."""
    qs, qs_p = _i32(q_slot)
    ks, ks_p = _i32(kv_slot)
    _check(_lib.load().dcp_plan_set_block_buffers(plan.handle, qs_p, n_q_slots, ks_p, n_kv_slots))
    plan.q_rows, plan.kv_rows = n_q_slots * plan.block_size, n_kv_slots * plan.block_size


def dcp_plan_prepare(plan, hq, hkv, d, dtype_code, impl=DCP_IMPL_AUTO):
    """Uploads the plan's arrays and work lists for this shape now (the only call that allocates and synchronises)."""
    _check(_lib.load().dcp_plan_prepare(plan.handle, hq, hkv, d, dtype_code, impl, _stream()))


def dcp_plan_destroy(plan):
    _check(_lib.load().dcp_plan_destroy(plan.handle))
    plan.handle = None


def dcp_plan_export(plan, which):
    lib = _lib.load()
    wid = EXPORTS[which] if isinstance(which, str) else int(which)
    n = ctypes.c_int64(0)
    _check(lib.dcp_plan_export(plan.handle, wid, None, 0, ctypes.byref(n)))
    out = np.zeros(n.value, dtype=np.int32)
    _check(lib.dcp_plan_export(plan.handle, wid, out.ctypes.data_as(_lib.i32p), n.value, ctypes.byref(n)))
    return out


def dcp_plan_export_dkv_items(plan, hkv):
    """[n_items, 5] int32 rows (unit, tile, e0, e1, pslot) of the MFMA dK/dV work list for `hkv` KV heads."""
    lib = _lib.load()
    n = ctypes.c_int64(0)
    _check(lib.dcp_plan_export_dkv_items(plan.handle, int(hkv), None, 0, ctypes.byref(n)))
    out = np.zeros((n.value, 5), dtype=np.int32)
    _check(lib.dcp_plan_export_dkv_items(plan.handle, int(hkv), out.ctypes.data_as(_lib.i32p), n.value, ctypes.byref(n)))
    return out


def dcp_plan_export_dkv_segments(plan, hkv):
    """(n_seg, seg[9]): how the dK/dV work list for `hkv` KV heads is divided among the XCDs."""
    lib = _lib.load()
    n = ctypes.c_int32(0)
    seg = np.zeros(9, dtype=np.int32)
    _check(lib.dcp_plan_export_dkv_segments(plan.handle, int(hkv), ctypes.byref(n), seg.ctypes.data_as(_lib.i32p)))
    return int(n.value), seg


# ------------------------------------------------------------------ launching calls (torch)
def _dtype_code(t):
    import torch
    if t.dtype == torch.bfloat16:
        return DCP_BF16
    if t.dtype == torch.float32:
        return DCP_F32
    raise TypeError(f"unsupported dtype {t.dtype}")


def _stream():
    import torch
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _set(ts, name, tensor):
    if tensor is None:
        return
    assert tensor.is_cuda and tensor.stride(-1) == 1, f"{name}: device tensor with contiguous last dim required"
    setattr(ts, name, tensor.data_ptr())
    prefix = {"q": "q", "k": "k", "v": "v", "out": "o", "dout": "do", "dq": "dq", "dk": "dk", "dv": "dv"}[name]
    setattr(ts, prefix + "_stride_t", tensor.stride(0))
    setattr(ts, prefix + "_stride_h", tensor.stride(1))


def _descr(q, k, v, softmax_scale, attn_ranges, impl):
    ts = Tensors()
    ts.hq, ts.hkv, ts.d = q.shape[1], k.shape[1], q.shape[2]
    ts.dtype, ts.impl, ts.softmax_scale = _dtype_code(q), impl, softmax_scale
    _set(ts, "q", q)
    _set(ts, "k", k)
    _set(ts, "v", v)
    if attn_ranges is not None:
        assert attn_ranges.is_cuda and attn_ranges.is_contiguous()
        ts.attn_ranges = attn_ranges.data_ptr()
    return ts


def dcp_block_attn_fwd(plan, q, k, v, out, lse, softmax_scale, attn_ranges=None, impl=DCP_IMPL_AUTO):
    """out/lse: packed [T,Hq,D] / [Hq,T], or the partial-slot buffers when the plan has slots."""
    ts = _descr(q, k, v, softmax_scale, attn_ranges, impl)
    if plan.n_slots or out.dim() == 4:
        assert out.is_contiguous() and lse.is_contiguous()
        ts.out = out.data_ptr()
    else:
        _set(ts, "out", out)
    ts.lse = lse.data_ptr()
    _check(_lib.load().dcp_block_attn_fwd(plan.handle, ctypes.byref(ts), _stream()))


def dcp_merge_partials(plan, o_part, lse_part, out, lse):
    _check(_lib.load().dcp_merge_partials(plan.handle, o_part.data_ptr(), lse_part.data_ptr(), out.data_ptr(),
                                          out.stride(0), out.stride(1), lse.data_ptr(), out.shape[1], out.shape[2],
                                          _dtype_code(out), _stream()))


def dcp_bwd_delta(out, dout, delta):
    ts = Tensors()
    ts.hq, ts.hkv, ts.d, ts.dtype = out.shape[1], out.shape[1], out.shape[2], _dtype_code(out)
    _set(ts, "out", out)
    _set(ts, "dout", dout)
    _check(_lib.load().dcp_bwd_delta(ctypes.byref(ts), out.shape[0], delta.data_ptr(), _stream()))


def dcp_bwd_workspace_bytes(plan, hq, hkv, d, dtype_code):
    return int(_lib.load().dcp_bwd_workspace_bytes(plan.handle, hq, hkv, d, dtype_code))


def dcp_block_attn_bwd(plan, q, k, v, out, lse, dout, dq, dk, dv, softmax_scale, workspace, attn_ranges=None,
                       impl=DCP_IMPL_AUTO):
    ts = _descr(q, k, v, softmax_scale, attn_ranges, impl)
    for name, t in (("out", out), ("dout", dout), ("dq", dq), ("dk", dk), ("dv", dv)):
        _set(ts, name, t)
    ts.lse = lse.data_ptr()
    _check(_lib.load().dcp_block_attn_bwd(plan.handle, ctypes.byref(ts), workspace.data_ptr(),
                                          workspace.numel() * workspace.element_size(), _stream()))


DCP_STATIC_SCRATCH_BYTES = 64 << 20


def dcp_block_attn_bwd_static(plan, q, k, v, out, lse, dout, dq, dk, dv, softmax_scale, attn_ranges=None, impl=DCP_IMPL_AUTO):
    """dcp_block_attn_bwd without a workspace argument and without any allocation (the plan must have been prepared)."""
    ts = _descr(q, k, v, softmax_scale, attn_ranges, impl)
    for name, t in (("out", out), ("dout", dout), ("dq", dq), ("dk", dk), ("dv", dv)):
        _set(ts, name, t)
    ts.lse = lse.data_ptr()
    _check(_lib.load().dcp_block_attn_bwd_static(plan.handle, ctypes.byref(ts), _stream()))


def dcp_sum_partials(parts, dst):
    arr = (ctypes.c_void_p * len(parts))(*[p.data_ptr() for p in parts])
    _check(_lib.load().dcp_sum_partials(arr, len(parts), _dtype_code(parts[0]), dst.data_ptr(), _dtype_code(dst),
                                        dst.numel(), _stream()))


class CopyList:
    """Blockwise Copy list: entries int32 [n,3] (src_row, dst_row, n_rows) over 2-D row views of two buffers."""

    def __init__(self, entries, src_rows, dst_rows):
        e = np.ascontiguousarray(np.asarray(entries, dtype=np.int32).reshape(-1, 3))
        self.n = e.shape[0]
        self.src_rows, self.dst_rows = int(src_rows), int(dst_rows)
        h = ctypes.c_void_p()
        _check(_lib.load().dcp_copy_list_create(ctypes.byref(h), e.ctypes.data_as(_lib.i32p), self.n, self.src_rows, self.dst_rows))
        self.handle = h

    def close(self):
        if getattr(self, "handle", None):
            _lib.load().dcp_copy_list_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def dcp_blockwise_copy(copy_list, src, dst):
    """src, dst: tensors whose first axis is the row and whose rows are contiguous (e.g. [rows, H, D])."""
    def row_view(t):
        assert t.dim() >= 1 and (t.dim() == 1 or t[0].is_contiguous()), "rows must be contiguous"
        row_bytes = (t[0].numel() if t.dim() > 1 else 1) * t.element_size()
        stride = (t.stride(0) if t.shape[0] > 1 else (t[0].numel() if t.dim() > 1 else 1)) * t.element_size()
        return row_bytes, stride
    rb_s, st_s = row_view(src)
    rb_d, st_d = row_view(dst)
    assert rb_s == rb_d, "source and destination rows differ in size"
    assert src.shape[0] == copy_list.src_rows and dst.shape[0] == copy_list.dst_rows
    _check(_lib.load().dcp_blockwise_copy(copy_list.handle, src.data_ptr(), st_s, dst.data_ptr(), st_d, rb_s, _stream()))


# ---------------------------------------------------------------------------------------------
# execution plans: instruction constructors (they fill a dcp_instr_t and keep the tensors alive) and Program
OP_ATTN_FWD, OP_ATTN_BWD, OP_MERGE, OP_COPY, OP_SUM, OP_COMM_LAUNCH, OP_COMM_WAIT = range(7)


def _row_view(t):
    assert t.dim() >= 1 and (t.dim() == 1 or t[0].is_contiguous()), "rows must be contiguous"
    row_bytes = (t[0].numel() if t.dim() > 1 else 1) * t.element_size()
    stride = (t.stride(0) if t.shape[0] > 1 else (t[0].numel() if t.dim() > 1 else 1)) * t.element_size()
    return row_bytes, stride


def instr_attn_fwd(plan, q, k, v, out, lse, softmax_scale, attn_ranges=None, impl=DCP_IMPL_AUTO):
    ins = _lib.Instr()
    ins.op, ins.plan = OP_ATTN_FWD, plan.handle
    ts = _descr(q, k, v, softmax_scale, attn_ranges, impl)
    if plan.n_slots or out.dim() == 4:
        ts.out = out.data_ptr()
    else:
        _set(ts, "out", out)
    ts.lse = lse.data_ptr()
    ins.tensors = ts
    ins._keep = (plan, q, k, v, out, lse, attn_ranges)
    return ins


def instr_attn_bwd(plan, q, k, v, out, lse, dout, dq, dk, dv, softmax_scale, workspace, attn_ranges=None, impl=DCP_IMPL_AUTO):
    ins = _lib.Instr()
    ins.op, ins.plan = OP_ATTN_BWD, plan.handle
    ts = _descr(q, k, v, softmax_scale, attn_ranges, impl)
    for name, t in (("out", out), ("dout", dout), ("dq", dq), ("dk", dk), ("dv", dv)):
        _set(ts, name, t)
    ts.lse = lse.data_ptr()
    ins.tensors = ts
    ins.workspace, ins.workspace_bytes = workspace.data_ptr(), workspace.numel() * workspace.element_size()
    ins._keep = (plan, q, k, v, out, lse, dout, dq, dk, dv, workspace, attn_ranges)
    return ins


def instr_merge(plan, o_part, lse_part, out, lse):
    ins = _lib.Instr()
    ins.op, ins.plan = OP_MERGE, plan.handle
    ins.o_part, ins.lse_part = o_part.data_ptr(), lse_part.data_ptr()
    ts = Tensors()
    ts.hq, ts.d, ts.dtype = out.shape[1], out.shape[2], _dtype_code(out)
    _set(ts, "out", out)
    ts.lse = lse.data_ptr()
    ins.tensors = ts
    ins._keep = (plan, o_part, lse_part, out, lse)
    return ins


def _fill_copy(ins, copy_list, src, dst):
    rb_s, st_s = _row_view(src)
    rb_d, st_d = _row_view(dst)
    assert rb_s == rb_d and src.shape[0] == copy_list.src_rows and dst.shape[0] == copy_list.dst_rows
    ins.copy_list, ins.src, ins.dst = copy_list.handle, src.data_ptr(), dst.data_ptr()
    ins.src_row_stride, ins.dst_row_stride, ins.row_bytes = st_s, st_d, rb_s
    ins._keep = (copy_list, src, dst)


def instr_copy(copy_list, src, dst):
    ins = _lib.Instr()
    ins.op = OP_COPY
    _fill_copy(ins, copy_list, src, dst)
    return ins


def instr_sum(parts, dst):
    ins = _lib.Instr()
    ins.op, ins.n_parts, ins.parts_dtype = OP_SUM, len(parts), _dtype_code(parts[0])
    for i, p in enumerate(parts):
        ins.parts[i] = p.data_ptr()
    ins.dst, ins.dst_dtype, ins.n_elems = dst.data_ptr(), _dtype_code(dst), dst.numel()
    ins._keep = (list(parts), dst)
    return ins


def instr_comm_launch(comm_id, copy_list, src, dst):
    """On one device the transfer is a Blockwise Copy on the second stream."""
    ins = _lib.Instr()
    ins.op, ins.comm_id = OP_COMM_LAUNCH, comm_id
    _fill_copy(ins, copy_list, src, dst)
    return ins


def instr_comm_wait(comm_id):
    ins = _lib.Instr()
    ins.op, ins.comm_id = OP_COMM_WAIT, comm_id
    return ins


class Program:
    """An execution plan: instructions run in order by dcp_program_run."""

    def __init__(self, instrs):
        self._instrs = list(instrs)                      # keeps tensors, plans and copy lists alive
        arr = (_lib.Instr * max(1, len(self._instrs)))()
        for i, ins in enumerate(self._instrs):
            ctypes.memmove(ctypes.byref(arr[i]), ctypes.byref(ins), ctypes.sizeof(_lib.Instr))
        h = ctypes.c_void_p()
        _check(_lib.load().dcp_program_create(ctypes.byref(h), arr, len(self._instrs)))
        self.handle = h

    def run(self, comm_stream=None):
        """Compute stream = torch's current stream; comm_stream: a torch.cuda.Stream (needed if the plan has transfers)."""
        cs = comm_stream.cuda_stream if comm_stream is not None else _stream()
        _check(_lib.load().dcp_program_run(self.handle, _stream(), cs))

    def close(self):
        if getattr(self, "handle", None):
            _lib.load().dcp_program_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


KERNEL_IDS = dict(fwd=0, merge=1, delta=2, dq=3, dkv=4, sum=5, copy=6)


def dcp_profile_enable(enable):
    _check(_lib.load().dcp_profile_enable(1 if enable else 0))


def dcp_profile_read(kernel):
    """-> (total_ms, launches) of one kernel since dcp_profile_enable(True)."""
    kid = KERNEL_IDS[kernel] if isinstance(kernel, str) else int(kernel)
    ms, n = ctypes.c_double(0), ctypes.c_int64(0)
    _check(_lib.load().dcp_profile_read(kid, ctypes.byref(ms), ctypes.byref(n)))
    return ms.value, n.value
