// Executor of an execution plan (Sec. 5): a list of instructions run in order on one stream, with
// Comm.Launch handing its transfer to a second stream and Comm.Wait making the first stream wait
// for it, so that the transfer of one division overlaps the attention of another (Sec. 4.3).  On a
// single device a transfer is a Blockwise Copy on the second stream.
#include <memory>
#include <string>
#include <vector>

#include "dcp_internal.h"

struct dcp_program {
  std::vector<dcp_instr_t> instrs;
  int32_t n_comm = 0;                 // transfers are numbered 0 .. n_comm - 1
  std::vector<hipEvent_t> done;       // per transfer: recorded on the transfer stream when it has finished
  hipEvent_t fork = nullptr;          // recorded on the compute stream before each launch
  int device = -1;
};

using dcp::fail;

extern "C" dcp_status_t dcp_program_create(dcp_program_t** out, const dcp_instr_t* instrs, int64_t n) {
  if (!out) return fail(DCP_ERR_INVALID_ARG, "program output pointer is NULL");
  *out = nullptr;
  if (n < 0 || (n > 0 && !instrs)) return fail(DCP_ERR_INVALID_ARG, "instrs is NULL or n < 0");
  std::unique_ptr<dcp_program> p(new dcp_program);
  p->instrs.assign(instrs, instrs + n);
  std::vector<int> state;   // per transfer: 0 unseen, 1 launched, 2 waited
  for (int64_t i = 0; i < n; i++) {
    const dcp_instr_t& in = instrs[i];
    const std::string at = "instruction " + std::to_string(i) + ": ";
    switch (in.op) {
      case DCP_OP_ATTN_FWD:
      case DCP_OP_ATTN_BWD:
      case DCP_OP_MERGE:
        if (!in.plan) return fail(DCP_ERR_INVALID_ARG, at + "plan is NULL");
        break;
      case DCP_OP_COPY:
        if (!in.copy_list) return fail(DCP_ERR_INVALID_ARG, at + "copy list is NULL");
        break;
      case DCP_OP_SUM:
        if (in.n_parts < 1 || in.n_parts > 8) return fail(DCP_ERR_INVALID_ARG, at + "n_parts must be 1..8");
        break;
      case DCP_OP_COMM_LAUNCH:
      case DCP_OP_COMM_WAIT: {
        if (in.comm_id < 0 || in.comm_id > (1 << 20)) return fail(DCP_ERR_INVALID_ARG, at + "bad transfer id");
        if ((size_t)in.comm_id >= state.size()) state.resize(in.comm_id + 1, 0);
        if (in.op == DCP_OP_COMM_LAUNCH) {
          if (!in.copy_list) return fail(DCP_ERR_INVALID_ARG, at + "Comm.Launch carries no copy list");
          if (state[in.comm_id] != 0) return fail(DCP_ERR_INVALID_ARG, at + "transfer id launched twice");
          state[in.comm_id] = 1;
        } else {
          if (state[in.comm_id] != 1) return fail(DCP_ERR_INVALID_ARG, at + "Comm.Wait for a transfer that is not in flight");
          state[in.comm_id] = 2;
        }
        break;
      }
      default:
        return fail(DCP_ERR_INVALID_ARG, at + "unknown op");
    }
  }
  p->n_comm = (int32_t)state.size();
  *out = p.release();
  return DCP_OK;
}

extern "C" dcp_status_t dcp_program_destroy(dcp_program_t* p) {
  if (!p) return DCP_OK;
  for (hipEvent_t e : p->done)
    if (e) (void)hipEventDestroy(e);
  if (p->fork) (void)hipEventDestroy(p->fork);
  delete p;
  return DCP_OK;
}

extern "C" dcp_status_t dcp_program_run(dcp_program_t* p, void* compute_stream, void* comm_stream) {
  if (!p) return fail(DCP_ERR_INVALID_ARG, "program is NULL");
  hipStream_t cs = (hipStream_t)compute_stream, ts = (hipStream_t)comm_stream;
  if (p->n_comm > 0 && cs == ts) return fail(DCP_ERR_INVALID_ARG, "a program with transfers needs two different streams");
  int dev = -1;
  DCP_HIP_TRY(hipGetDevice(&dev));
  if (p->device >= 0 && p->device != dev) return fail(DCP_ERR_INVALID_ARG, "program was first run on another device");
  if (p->device < 0) {
    p->done.assign(p->n_comm, nullptr);
    for (auto& e : p->done) DCP_HIP_TRY(hipEventCreateWithFlags(&e, hipEventDisableTiming));
    DCP_HIP_TRY(hipEventCreateWithFlags(&p->fork, hipEventDisableTiming));
    p->device = dev;
  }
  std::vector<char> waited(p->n_comm, 0), launched(p->n_comm, 0);
  dcp_status_t st = DCP_OK;
  for (const dcp_instr_t& in : p->instrs) {
    switch (in.op) {
      case DCP_OP_ATTN_FWD:
        st = dcp_block_attn_fwd(in.plan, &in.tensors, cs);
        break;
      case DCP_OP_ATTN_BWD:
        st = dcp_block_attn_bwd(in.plan, &in.tensors, in.workspace, in.workspace_bytes, cs);
        break;
      case DCP_OP_MERGE:
        st = dcp_merge_partials(in.plan, in.o_part, in.lse_part, in.tensors.out, in.tensors.o_stride_t, in.tensors.o_stride_h,
                                in.tensors.lse, in.tensors.hq, in.tensors.d, in.tensors.dtype, cs);
        break;
      case DCP_OP_COPY:
        st = dcp_blockwise_copy(in.copy_list, in.src, in.src_row_stride, in.dst, in.dst_row_stride, in.row_bytes, cs);
        break;
      case DCP_OP_SUM:
        st = dcp_sum_partials(in.parts, in.n_parts, in.parts_dtype, in.dst, in.dst_dtype, in.n_elems, cs);
        break;
      case DCP_OP_COMM_LAUNCH:
        // the transfer starts after everything issued so far and runs beside what follows
        DCP_HIP_TRY(hipEventRecord(p->fork, cs));
        DCP_HIP_TRY(hipStreamWaitEvent(ts, p->fork, 0));
        st = dcp_blockwise_copy(in.copy_list, in.src, in.src_row_stride, in.dst, in.dst_row_stride, in.row_bytes, ts);
        if (st == DCP_OK) {
          DCP_HIP_TRY(hipEventRecord(p->done[in.comm_id], ts));
          launched[in.comm_id] = 1;
        }
        break;
      case DCP_OP_COMM_WAIT:
        DCP_HIP_TRY(hipStreamWaitEvent(cs, p->done[in.comm_id], 0));
        waited[in.comm_id] = 1;
        break;
    }
    if (st != DCP_OK) break;
  }
  // join: whoever synchronises the compute stream has waited for every transfer (also after an error)
  for (int32_t i = 0; i < p->n_comm; i++)
    if (launched[i] && !waited[i]) (void)hipStreamWaitEvent(cs, p->done[i], 0);
  return st;
}
