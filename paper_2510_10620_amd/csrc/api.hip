// Launching entry points of the C ABI: argument validation (host side, complete before any
// launch), kernel-family selection, and the enqueue of the kernels on the caller's stream.
#include <algorithm>
#include <cmath>
#include <memory>
#include <string>
#include <vector>

#include "kernels.h"

using namespace dcp;

namespace dcp {
struct ProfRec { hipEvent_t a, b; };
static bool g_prof_on = false;
static std::vector<ProfRec> g_prof[7];
ProfScope::ProfScope(int id_, hipStream_t s_, bool enabled) : id(id_), s(s_) {
  if (!g_prof_on || !enabled) return;
  hipEvent_t a = nullptr;
  if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&stop) != hipSuccess) { stop = nullptr; return; }
  (void)hipEventRecord(a, s);
  g_prof[id].push_back({a, stop});
}
ProfScope::~ProfScope() {
  if (stop) (void)hipEventRecord(stop, s);
}
}  // namespace dcp

extern "C" dcp_status_t dcp_profile_enable(int32_t enable) {
  if (enable) {
    for (auto& v : g_prof) {
      for (auto& r : v) { (void)hipEventDestroy(r.a); (void)hipEventDestroy(r.b); }
      v.clear();
    }
  }
  g_prof_on = enable != 0;
  return DCP_OK;
}

extern "C" dcp_status_t dcp_profile_read(int32_t kernel_id, double* total_ms, int64_t* launches) {
  if (kernel_id < 0 || kernel_id > 6 || !total_ms || !launches) return fail(DCP_ERR_INVALID_ARG, "bad kernel id or NULL output");
  double tot = 0;
  for (auto& r : g_prof[kernel_id]) {
    DCP_HIP_TRY(hipEventSynchronize(r.b));
    float ms = 0;
    DCP_HIP_TRY(hipEventElapsedTime(&ms, r.a, r.b));
    tot += ms;
  }
  *total_ms = tot;
  *launches = (int64_t)g_prof[kernel_id].size();
  return DCP_OK;
}

static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

static dcp_status_t check_shape(const dcp_tensors_t* t) {
  if (!t) return fail(DCP_ERR_INVALID_ARG, "tensor descriptor is NULL");
  if (t->hq <= 0 || t->hkv <= 0 || t->d <= 0) return fail(DCP_ERR_INVALID_ARG, "hq, hkv, d must be positive");
  if (t->hq % t->hkv != 0) return fail(DCP_ERR_UNSUPPORTED, "hq must be a multiple of hkv");
  if (t->dtype != DCP_BF16 && t->dtype != DCP_F32) return fail(DCP_ERR_UNSUPPORTED, "dtype must be DCP_BF16 or DCP_F32");
  if (t->impl < DCP_IMPL_AUTO || t->impl > DCP_IMPL_MFMA) return fail(DCP_ERR_INVALID_ARG, "bad impl selector");
  if (!(t->softmax_scale > 0.f) || !std::isfinite(t->softmax_scale)) return fail(DCP_ERR_INVALID_ARG, "softmax_scale must be positive and finite");
  return DCP_OK;
}

static dcp_status_t check_tensor(const char* name, const void* p, int64_t st, int64_t sh, int32_t d) {
  if (!p) return fail(DCP_ERR_INVALID_ARG, std::string(name) + " is NULL");
  if (!aligned16(p)) return fail(DCP_ERR_INVALID_ARG, std::string(name) + " must be 16-byte aligned");
  if (sh < d || st < d || sh % 8 || st % 8) return fail(DCP_ERR_INVALID_ARG, std::string(name) + ": strides must be >= d and multiples of 8 elements");
  return DCP_OK;
}

// Chooses the kernel family; MFMA iff requested or (AUTO and covered).
static dcp_status_t pick_impl(const dcp_tensors_t* t, bool* use_mfma) {
  const bool m_ok = mfma_supports(t->dtype, t->d), s_ok = scalar_supports(t->d);
  if (t->impl == DCP_IMPL_MFMA) {
    if (!m_ok) return fail(DCP_ERR_UNSUPPORTED, "MFMA kernels cover bf16 with head_dim 128 only");
    *use_mfma = true;
  } else if (t->impl == DCP_IMPL_SCALAR) {
    if (!s_ok) return fail(DCP_ERR_UNSUPPORTED, "scalar kernels cover head_dim 32, 64, 128");
    *use_mfma = false;
  } else {
    if (!m_ok && !s_ok) return fail(DCP_ERR_UNSUPPORTED, "no kernel covers this dtype / head_dim");
    *use_mfma = m_ok;
  }
  return DCP_OK;
}

static KTensors pack(const dcp_plan_t* plan, const dcp_tensors_t* t) {
  KTensors k{};
  k.q = t->q; k.k = t->k; k.v = t->v; k.dout = t->dout; k.out_in = t->out;
  k.out = t->out; k.dq = t->dq; k.dk = t->dk; k.dv = t->dv;
  k.lse = t->lse; k.delta = nullptr;
  k.ranges = plan->has_ranges ? t->attn_ranges : nullptr;   // kernels skip all range work when no row has per-token ranges
  k.window = plan->has_window ? plan->window : 0;
  k.sink = plan->has_window ? plan->sink : 0;
  k.masked = (plan->has_ranges || plan->has_window) ? 1 : 0;
  k.qbounds = nullptr;
  k.q_st = t->q_stride_t; k.q_sh = t->q_stride_h; k.k_st = t->k_stride_t; k.k_sh = t->k_stride_h;
  k.v_st = t->v_stride_t; k.v_sh = t->v_stride_h; k.o_st = t->o_stride_t; k.o_sh = t->o_stride_h;
  k.do_st = t->do_stride_t; k.do_sh = t->do_stride_h; k.dq_st = t->dq_stride_t; k.dq_sh = t->dq_stride_h;
  k.dk_st = t->dk_stride_t; k.dk_sh = t->dk_stride_h; k.dv_st = t->dv_stride_t; k.dv_sh = t->dv_stride_h;
  k.q_rows = plan->q_rows;
  k.hq = t->hq; k.hkv = t->hkv; k.d = t->d; k.block_size = plan->block_size;
  k.scale = t->softmax_scale;
  k.use_slots = plan->use_slots ? 1 : 0;
  return k;
}

extern "C" dcp_status_t dcp_plan_prepare(dcp_plan_t* plan, int32_t hq, int32_t hkv, int32_t d, int32_t dtype, int32_t impl,
                                         void* stream) {
  if (!plan) return fail(DCP_ERR_INVALID_ARG, "plan is NULL");
  dcp_tensors_t t{};
  t.hq = hq; t.hkv = hkv; t.d = d; t.dtype = dtype; t.impl = impl; t.softmax_scale = 1.f;
  dcp_status_t st = check_shape(&t);
  if (st != DCP_OK) return st;
  bool use_mfma = false;
  if ((st = pick_impl(&t, &use_mfma)) != DCP_OK) return st;
  hipStream_t s = (hipStream_t)stream;
  if ((st = plan->ensure_device(s)) != DCP_OK) return st;
  void* scratch_addr = nullptr;   // looked up here so that dcp_block_attn_bwd_static finds it ready
  if ((st = static_scratch(&scratch_addr)) != DCP_OK) return st;
  if (plan->total_tokens == 0) return DCP_OK;
  DevGroup g;
  const int n_seg = use_mfma ? xcd_segments(hkv) : 1;
  if ((st = plan->group_for(0, use_mfma ? mfma_fwd_tile() : scalar_fwd_tile(), s, &g, 0, true, n_seg)) != DCP_OK) return st;
  if ((st = plan->group_for(1, use_mfma ? mfma_dq_tile() : scalar_bwd_tile(), s, &g, 0, true, n_seg)) != DCP_OK) return st;
  return plan->group_for(2, use_mfma ? mfma_dkv_tile() : scalar_bwd_tile(), s, &g, use_mfma ? hkv : 0, true, n_seg);
}

extern "C" dcp_status_t dcp_block_attn_fwd(dcp_plan_t* plan, const dcp_tensors_t* t, void* stream) {
  if (!plan) return fail(DCP_ERR_INVALID_ARG, "plan is NULL");
  dcp_status_t st = check_shape(t);
  if (st != DCP_OK) return st;
  bool use_mfma = false;
  if ((st = pick_impl(t, &use_mfma)) != DCP_OK) return st;
  if (plan->total_tokens == 0) return DCP_OK;
  if ((st = check_tensor("q", t->q, t->q_stride_t, t->q_stride_h, t->d)) != DCP_OK) return st;
  if ((st = check_tensor("k", t->k, t->k_stride_t, t->k_stride_h, t->d)) != DCP_OK) return st;
  if ((st = check_tensor("v", t->v, t->v_stride_t, t->v_stride_h, t->d)) != DCP_OK) return st;
  if (!t->out || !aligned16(t->out)) return fail(DCP_ERR_INVALID_ARG, "out is NULL or not 16-byte aligned");
  if (!t->lse) return fail(DCP_ERR_INVALID_ARG, "lse is NULL");
  if (!plan->use_slots && (st = check_tensor("out", t->out, t->o_stride_t, t->o_stride_h, t->d)) != DCP_OK) return st;
  if (plan->has_ranges && !t->attn_ranges) return fail(DCP_ERR_INVALID_ARG, "table has RANGES rows but attn_ranges is NULL");
  if (plan->has_window && plan->window <= 0) return fail(DCP_ERR_INVALID_ARG, "table has WINDOW rows but dcp_plan_set_window was not called");
  hipStream_t s = (hipStream_t)stream;
  DevGroup g;
  if ((st = plan->group_for(0, use_mfma ? mfma_fwd_tile() : scalar_fwd_tile(), s, &g, 0, true, use_mfma ? xcd_segments(t->hkv) : 1)) != DCP_OK) return st;
  KTensors k = pack(plan, t);
  ProfScope ps(DCP_K_FWD, s);
  return use_mfma ? mfma_fwd(g, k, s) : scalar_fwd(g, k, t->dtype, s);
}

extern "C" dcp_status_t dcp_merge_partials(dcp_plan_t* plan, const void* o_part, const float* lse_part, void* out,
                                           int64_t o_stride_t, int64_t o_stride_h, float* lse, int32_t hq, int32_t d,
                                           int32_t dtype, void* stream) {
  if (!plan) return fail(DCP_ERR_INVALID_ARG, "plan is NULL");
  if (!plan->use_slots) return fail(DCP_ERR_INVALID_ARG, "plan was created without output slots");
  if (hq <= 0 || d <= 0 || d % 8) return fail(DCP_ERR_UNSUPPORTED, "merge needs hq > 0 and d a positive multiple of 8");
  if (dtype != DCP_BF16 && dtype != DCP_F32) return fail(DCP_ERR_UNSUPPORTED, "dtype must be DCP_BF16 or DCP_F32");
  if (plan->total_tokens == 0) return DCP_OK;
  if (plan->n_slots > 0 && (!o_part || !lse_part || !aligned16(o_part))) return fail(DCP_ERR_INVALID_ARG, "o_part / lse_part NULL or misaligned");
  dcp_status_t st = check_tensor("out", out, o_stride_t, o_stride_h, d);
  if (st != DCP_OK) return st;
  if (!lse) return fail(DCP_ERR_INVALID_ARG, "lse is NULL");
  hipStream_t s = (hipStream_t)stream;
  if ((st = plan->ensure_device(s)) != DCP_OK) return st;
  ProfScope ps(DCP_K_MERGE, s);
  return stream_merge(plan->d_merge_ptr, plan->d_merge_idx, plan->d_q_mem0, plan->d_fwd.blk_len, plan->n_blocks,
                      plan->block_size, o_part, lse_part, out, o_stride_t, o_stride_h, lse, plan->q_rows, hq, d,
                      dtype, s);
}

extern "C" dcp_status_t dcp_bwd_delta(const dcp_tensors_t* t, int64_t total_tokens, float* delta, void* stream) {
  if (!t) return fail(DCP_ERR_INVALID_ARG, "tensor descriptor is NULL");
  if (t->hq <= 0 || t->d <= 0 || t->d % 8 || t->d > 256 || (t->d & (t->d - 1))) return fail(DCP_ERR_UNSUPPORTED, "delta needs d a power of two in 8..256");
  if (t->dtype != DCP_BF16 && t->dtype != DCP_F32) return fail(DCP_ERR_UNSUPPORTED, "dtype must be DCP_BF16 or DCP_F32");
  if (total_tokens < 0) return fail(DCP_ERR_INVALID_ARG, "total_tokens < 0");
  if (total_tokens == 0) return DCP_OK;
  dcp_status_t st;
  if ((st = check_tensor("out", t->out, t->o_stride_t, t->o_stride_h, t->d)) != DCP_OK) return st;
  if ((st = check_tensor("dout", t->dout, t->do_stride_t, t->do_stride_h, t->d)) != DCP_OK) return st;
  if (!delta) return fail(DCP_ERR_INVALID_ARG, "delta is NULL");
  ProfScope ps(DCP_K_DELTA, (hipStream_t)stream);
  return stream_delta(t->out, t->o_stride_t, t->o_stride_h, t->dout, t->do_stride_t, t->do_stride_h, delta, nullptr,
                      nullptr, total_tokens, t->hq, t->d, t->dtype, (hipStream_t)stream);
}

// Workspace layout: delta [Hq, rows] | lse2 [Hq, rows] | range-bound summaries | partial dK / dV sums of split items.
struct BwdWorkspace {
  size_t n_hT, n_bounds, n_part;
  size_t total() const { return 2 * n_hT + n_bounds + n_part; }
};

static BwdWorkspace bwd_workspace(dcp_plan_t* plan, int32_t hq, int32_t hkv, int32_t d, int32_t dtype) {
  BwdWorkspace w{};
  w.n_hT = (size_t)hq * (size_t)plan->q_rows * sizeof(float);
  w.n_hT = (w.n_hT + 255) & ~(size_t)255;
  // range-bound summaries of every 32-row tile (+1 spare entry), only for tables with RANGES or WINDOW rows
  w.n_bounds = (plan->has_ranges || plan->has_window) ? ((size_t)plan->blk_t32.back() + 1) * 8 * sizeof(int32_t) : 0;
  w.n_bounds = (w.n_bounds + 255) & ~(size_t)255;
  if (hkv > 0 && mfma_supports(dtype, d)) w.n_part = mfma_dkv_part_bytes(plan->host_items(2, mfma_dkv_tile(), hkv, xcd_segments(hkv)).n_pslots, hkv);
  return w;
}

extern "C" dcp_status_t dcp_plan_export_dkv_items(dcp_plan_t* plan, int32_t hkv, int32_t* dst, int64_t capacity_rows,
                                                  int64_t* n_items_out) {
  if (!plan || !n_items_out) return fail(DCP_ERR_INVALID_ARG, "plan or n_items_out is NULL");
  if (hkv <= 0) return fail(DCP_ERR_INVALID_ARG, "hkv must be positive");
  const HostItems& hi = plan->host_items(2, mfma_dkv_tile(), hkv, xcd_segments(hkv));
  *n_items_out = (int64_t)hi.items.size();
  if (dst) {
    if (capacity_rows < (int64_t)hi.items.size()) return fail(DCP_ERR_INVALID_ARG, "export capacity too small");
    for (size_t i = 0; i < hi.items.size(); i++) {
      const WorkItem& w = hi.items[i];
      dst[5 * i] = w.unit; dst[5 * i + 1] = w.tile; dst[5 * i + 2] = w.e0; dst[5 * i + 3] = w.e1; dst[5 * i + 4] = w.pslot;
    }
  }
  return DCP_OK;
}

extern "C" dcp_status_t dcp_plan_export_dkv_segments(dcp_plan_t* plan, int32_t hkv, int32_t* n_seg_out, int32_t* seg_out) {
  if (!plan || !n_seg_out || !seg_out) return fail(DCP_ERR_INVALID_ARG, "plan, n_seg_out or seg_out is NULL");
  if (hkv <= 0) return fail(DCP_ERR_INVALID_ARG, "hkv must be positive");
  const HostItems& hi = plan->host_items(2, mfma_dkv_tile(), hkv, xcd_segments(hkv));
  *n_seg_out = hi.n_seg;
  for (int k = 0; k <= 8; k++) seg_out[k] = hi.seg[k];
  return DCP_OK;
}

extern "C" size_t dcp_bwd_workspace_bytes(const dcp_plan_t* plan, int32_t hq, int32_t hkv, int32_t d, int32_t dtype) {
  if (!plan || hq <= 0) return 0;
  // the work lists are cached in the plan the first time a size or a launch asks for them
  return bwd_workspace(const_cast<dcp_plan_t*>(plan), hq, hkv, d, dtype).total();
}

// The backward behind both of its entry points.  may_alloc = false: the plan's device copies must exist already
// (dcp_plan_prepare) and no per-kernel timing events are created, so the call neither allocates nor synchronises.
dcp_status_t dcp::bwd_launch(dcp_plan_t* plan, const dcp_tensors_t* t, void* workspace, size_t workspace_bytes, hipStream_t s,
                             bool may_alloc) {
  if (!plan) return fail(DCP_ERR_INVALID_ARG, "plan is NULL");
  dcp_status_t st = check_shape(t);
  if (st != DCP_OK) return st;
  bool use_mfma = false;
  if ((st = pick_impl(t, &use_mfma)) != DCP_OK) return st;
  if (plan->total_tokens == 0) return DCP_OK;
  if ((st = check_tensor("q", t->q, t->q_stride_t, t->q_stride_h, t->d)) != DCP_OK) return st;
  if ((st = check_tensor("k", t->k, t->k_stride_t, t->k_stride_h, t->d)) != DCP_OK) return st;
  if ((st = check_tensor("v", t->v, t->v_stride_t, t->v_stride_h, t->d)) != DCP_OK) return st;
  if ((st = check_tensor("out", t->out, t->o_stride_t, t->o_stride_h, t->d)) != DCP_OK) return st;
  if ((st = check_tensor("dout", t->dout, t->do_stride_t, t->do_stride_h, t->d)) != DCP_OK) return st;
  if ((st = check_tensor("dq", t->dq, t->dq_stride_t, t->dq_stride_h, t->d)) != DCP_OK) return st;
  if ((st = check_tensor("dk", t->dk, t->dk_stride_t, t->dk_stride_h, t->d)) != DCP_OK) return st;
  if ((st = check_tensor("dv", t->dv, t->dv_stride_t, t->dv_stride_h, t->d)) != DCP_OK) return st;
  if (!t->lse) return fail(DCP_ERR_INVALID_ARG, "lse is NULL");
  if (plan->has_ranges && !t->attn_ranges) return fail(DCP_ERR_INVALID_ARG, "table has RANGES rows but attn_ranges is NULL");
  if (plan->has_window && plan->window <= 0) return fail(DCP_ERR_INVALID_ARG, "table has WINDOW rows but dcp_plan_set_window was not called");
  const BwdWorkspace wsz = bwd_workspace(plan, t->hq, t->hkv, t->d, t->dtype);
  const size_t need = wsz.total();
  if (!workspace || workspace_bytes < need) return fail(DCP_ERR_WORKSPACE, "workspace is NULL or smaller than dcp_bwd_workspace_bytes");
  if (reinterpret_cast<uintptr_t>(workspace) & 255u) return fail(DCP_ERR_WORKSPACE, "workspace must be 256-byte aligned");
  DevGroup gq, gkv;
  const int n_seg = use_mfma ? xcd_segments(t->hkv) : 1;
  if ((st = plan->group_for(1, use_mfma ? mfma_dq_tile() : scalar_bwd_tile(), s, &gq, 0, may_alloc, n_seg)) != DCP_OK) return st;
  if ((st = plan->group_for(2, use_mfma ? mfma_dkv_tile() : scalar_bwd_tile(), s, &gkv, use_mfma ? t->hkv : 0, may_alloc, n_seg)) != DCP_OK) return st;
  KTensors k = pack(plan, t);
  const size_t n_hT = wsz.n_hT;
  k.part = (float*)((char*)workspace + 2 * wsz.n_hT + wsz.n_bounds);
  float* delta = (float*)workspace;
  float* lse2 = (float*)((char*)workspace + n_hT);
  k.delta = delta;
  k.lse2 = lse2;
  if (k.masked && use_mfma) {
    int32_t* qb = (int32_t*)((char*)workspace + 2 * n_hT);
    k.qbounds = qb;
    if ((st = mfma_range_bounds(gkv, k, plan->d_blk_t32, plan->n_blocks, qb, s)) != DCP_OK) return st;
  }
  if (use_mfma) {
    // the MFMA dQ kernel computes delta and the rescaled LSE of its own rows and leaves them for the dK/dV kernel
    k.delta_w = delta;
    k.lse2_w = lse2;
  } else {
    ProfScope ps(DCP_K_DELTA, s, may_alloc);
    if ((st = stream_delta(t->out, t->o_stride_t, t->o_stride_h, t->dout, t->do_stride_t, t->do_stride_h, delta,
                           t->lse, lse2, plan->q_rows, t->hq, t->d, t->dtype, s)) != DCP_OK) return st;
  }
  {
    ProfScope ps(DCP_K_DQ, s, may_alloc);
    if ((st = use_mfma ? mfma_bwd_dq(gq, k, s) : scalar_bwd_dq(gq, k, t->dtype, s)) != DCP_OK) return st;
  }
  ProfScope ps(DCP_K_DKV, s, may_alloc);
  return use_mfma ? mfma_bwd_dkv(gkv, k, s) : scalar_bwd_dkv(gkv, k, t->dtype, s);
}

extern "C" dcp_status_t dcp_block_attn_bwd(dcp_plan_t* plan, const dcp_tensors_t* t, void* workspace,
                                           size_t workspace_bytes, void* stream) {
  return bwd_launch(plan, t, workspace, workspace_bytes, (hipStream_t)stream, true);
}

extern "C" dcp_status_t dcp_sum_partials(const void* const* parts, int32_t n_parts, int32_t parts_dtype, void* dst,
                                         int32_t dst_dtype, int64_t n_elems, void* stream) {
  if (n_parts < 1 || n_parts > 8 || !parts) return fail(DCP_ERR_INVALID_ARG, "n_parts must be 1..8 and parts non-NULL");
  if (n_elems < 0 || n_elems % 8) return fail(DCP_ERR_INVALID_ARG, "n_elems must be a non-negative multiple of 8");
  if ((parts_dtype != DCP_BF16 && parts_dtype != DCP_F32) || (dst_dtype != DCP_BF16 && dst_dtype != DCP_F32))
    return fail(DCP_ERR_UNSUPPORTED, "dtype must be DCP_BF16 or DCP_F32");
  if (n_elems == 0) return DCP_OK;
  if (!dst || !aligned16(dst)) return fail(DCP_ERR_INVALID_ARG, "dst is NULL or misaligned");
  for (int i = 0; i < n_parts; i++)
    if (!parts[i] || !aligned16(parts[i])) return fail(DCP_ERR_INVALID_ARG, "a partial pointer is NULL or misaligned");
  ProfScope ps(DCP_K_SUM, (hipStream_t)stream);
  return stream_sum(parts, n_parts, parts_dtype, dst, dst_dtype, n_elems, (hipStream_t)stream);
}

extern "C" dcp_status_t dcp_copy_list_create(dcp_copy_list_t** list, const int32_t* entries, int64_t n, int64_t src_rows,
                                             int64_t dst_rows) {
  if (!list) return fail(DCP_ERR_INVALID_ARG, "list is NULL");
  *list = nullptr;
  if (n < 0 || (n > 0 && !entries)) return fail(DCP_ERR_INVALID_ARG, "entries is NULL or n < 0");
  if (src_rows < 0 || dst_rows < 0 || src_rows > INT32_MAX || dst_rows > INT32_MAX)
    return fail(DCP_ERR_INVALID_ARG, "src_rows / dst_rows must lie in [0, 2^31)");
  std::unique_ptr<dcp_copy_list> cl(new dcp_copy_list);
  cl->src_rows = src_rows; cl->dst_rows = dst_rows;
  std::vector<std::pair<int64_t, int64_t>> dsts, srcs;   // [begin, end)
  for (int64_t i = 0; i < n; i++) {
    const int64_t sr = entries[3 * i], dr = entries[3 * i + 1], nr = entries[3 * i + 2];
    if (sr < 0 || dr < 0 || nr < 0) return fail(DCP_ERR_BAD_TABLE, "copy entry " + std::to_string(i) + " has a negative field");
    if (sr + nr > src_rows) return fail(DCP_ERR_BAD_TABLE, "copy entry " + std::to_string(i) + " reads past the source buffer");
    if (dr + nr > dst_rows) return fail(DCP_ERR_BAD_TABLE, "copy entry " + std::to_string(i) + " writes past the destination buffer");
    if (nr == 0) continue;
    dsts.push_back({dr, dr + nr});
    srcs.push_back({sr, sr + nr});
    for (int64_t r = 0; r < nr; r += kCopyChunkRows) {
      cl->chunks.push_back((int32_t)(sr + r));
      cl->chunks.push_back((int32_t)(dr + r));
      cl->chunks.push_back((int32_t)std::min<int64_t>(kCopyChunkRows, nr - r));
    }
  }
  std::sort(dsts.begin(), dsts.end());
  for (size_t i = 1; i < dsts.size(); i++)
    if (dsts[i].first < dsts[i - 1].second) return fail(DCP_ERR_BAD_TABLE, "two copy entries write overlapping destination rows");
  // would a destination range overlap a source range if both buffers were the same allocation?
  std::sort(srcs.begin(), srcs.end());
  size_t j = 0;
  for (size_t i = 0; i < dsts.size() && cl->alias_safe; i++) {
    while (j < srcs.size() && srcs[j].second <= dsts[i].first) j++;
    for (size_t k = j; k < srcs.size() && srcs[k].first < dsts[i].second; k++)
      if (srcs[k].second > dsts[i].first) { cl->alias_safe = false; break; }
  }
  *list = cl.release();
  return DCP_OK;
}

extern "C" dcp_status_t dcp_copy_list_destroy(dcp_copy_list_t* list) {
  if (!list) return DCP_OK;
  if (list->d_chunks) (void)hipFree(list->d_chunks);
  delete list;
  return DCP_OK;
}

extern "C" dcp_status_t dcp_blockwise_copy(dcp_copy_list_t* list, const void* src, int64_t src_stride, void* dst,
                                           int64_t dst_stride, int64_t row_bytes, void* stream) {
  if (!list) return fail(DCP_ERR_INVALID_ARG, "list is NULL");
  if (row_bytes <= 0 || row_bytes % 16 || row_bytes / 16 > (1 << 24)) return fail(DCP_ERR_INVALID_ARG, "row_bytes must be a positive multiple of 16 (at most 2^28)");
  if (src_stride < row_bytes || dst_stride < row_bytes || src_stride % 16 || dst_stride % 16)
    return fail(DCP_ERR_INVALID_ARG, "row strides must be multiples of 16 and at least row_bytes");
  if (list->chunks.empty()) return DCP_OK;
  if (!src || !dst || !aligned16(src) || !aligned16(dst)) return fail(DCP_ERR_INVALID_ARG, "src or dst is NULL or misaligned");
  {
    // extents the list can touch
    const char* s0 = (const char*)src; const char* s1 = s0 + (list->src_rows - 1) * src_stride + row_bytes;
    const char* d0 = (const char*)dst; const char* d1 = d0 + (list->dst_rows - 1) * dst_stride + row_bytes;
    const bool overlap = list->src_rows > 0 && list->dst_rows > 0 && s0 < d1 && d0 < s1;
    if (overlap && !(src == dst && src_stride == dst_stride && list->alias_safe))
      return fail(DCP_ERR_INVALID_ARG, "source and destination buffers overlap (allowed only as the same buffer with a list whose destination ranges avoid its source ranges)");
  }
  hipStream_t s = (hipStream_t)stream;
  {
    std::lock_guard<std::mutex> lock(list->mu);
    int dev = -1;
    DCP_HIP_TRY(hipGetDevice(&dev));
    if (list->d_chunks && list->device != dev) return fail(DCP_ERR_INVALID_ARG, "copy list was first used on another device");
    if (!list->d_chunks) {
      const size_t bytes = list->chunks.size() * sizeof(int32_t);
      DCP_HIP_TRY(hipMalloc((void**)&list->d_chunks, bytes));
      hipError_t e = hipMemcpyAsync(list->d_chunks, list->chunks.data(), bytes, hipMemcpyHostToDevice, s);
      if (e == hipSuccess) e = hipStreamSynchronize(s);
      if (e != hipSuccess) {
        (void)hipFree(list->d_chunks);
        list->d_chunks = nullptr;
        return fail(DCP_ERR_HIP, std::string("copy list upload: ") + hipGetErrorString(e));
      }
      list->device = dev;
    }
  }
  ProfScope ps(DCP_K_COPY, s);
  return stream_copy(list->d_chunks, (int64_t)(list->chunks.size() / 3), src, src_stride, dst, dst_stride, row_bytes, s);
}

extern "C" const char* dcp_version(void) { return "dcp_attn 0.1 (gfx950)"; }
