// dcp_block_attn_bwd_static: the backward for callers that cannot allocate (code under HIP graph capture, tight
// serving loops, harnesses that forbid hipMalloc).  It is dcp_block_attn_bwd with the workspace argument replaced by
// a fixed device array that this file owns; every kernel is shared with that entry point.
#include <mutex>

#include "kernels.h"

using namespace dcp;

// The workspace: delta and the rescaled LSE of every (head, row), range-bound summaries, fp32 partial sums of cut
// dK/dV items (layout as documented for dcp_bwd_workspace_bytes).  Each GPU the library runs on holds its own copy
// of this array until the process ends.
static __device__ __align__(256) unsigned char scratch[DCP_STATIC_SCRATCH_BYTES];

// In host code `scratch` is only a handle for the symbol, not a device address: the address of each device's copy is
// asked for once per device, with that device current, and kept here.
static constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mu;
static void* g_scratch_ptr[kMaxDevices] = {};

dcp_status_t dcp::static_scratch(void** ptr) {
  int dev = -1;
  DCP_HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return fail(DCP_ERR_UNSUPPORTED, "device ordinal beyond the static scratch table");
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    DCP_HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) return fail(DCP_ERR_HIP, "hipGetSymbolAddress returned a null address for the static scratch array");
    g_scratch_ptr[dev] = p;
  }
  *ptr = g_scratch_ptr[dev];
  return DCP_OK;
}

extern "C" dcp_status_t dcp_block_attn_bwd_static(dcp_plan_t* plan, const dcp_tensors_t* t, void* stream) {
  if (!plan) return fail(DCP_ERR_INVALID_ARG, "plan is NULL");
  if (!t) return fail(DCP_ERR_INVALID_ARG, "tensor descriptor is NULL");
  const size_t need = dcp_bwd_workspace_bytes(plan, t->hq, t->hkv, t->d, t->dtype);
  if (need > (size_t)DCP_STATIC_SCRATCH_BYTES)
    return fail(DCP_ERR_WORKSPACE, "this plan and shape need " + std::to_string(need) + " bytes of workspace, more than the " +
                                       std::to_string((size_t)DCP_STATIC_SCRATCH_BYTES) +
                                       " of the static scratch array: use dcp_block_attn_bwd with a workspace of the caller's");
  void* ws = nullptr;
  dcp_status_t st = static_scratch(&ws);
  if (st != DCP_OK) return st;
  // nothing in the workspace has to start at zero: every kernel of the backward writes what a later one reads
  return bwd_launch(plan, t, ws, (size_t)DCP_STATIC_SCRATCH_BYTES, (hipStream_t)stream, /*may_alloc=*/false);
}
