// Launcher declarations: one function per kernel family, defined in the .hip files.
#pragma once
#include "dcp_internal.h"

namespace dcp {

// Plain-old-data copy of the caller's tensor descriptor plus derived fields, passed by value.
struct KTensors {
  const void *q, *k, *v, *dout, *out_in;
  void *out, *dq, *dk, *dv;
  float* lse;              // forward: output; backward: input
  float* delta_w;          // backward, MFMA family: where the dQ kernel leaves -delta and lse2 (the same arrays as below) for
  float* lse2_w;           //   the dK/dV kernel; null in the scalar family, where a preprocess kernel has filled them
  const float* delta;      // backward input [Hq,T]: delta (scalar family), -delta (MFMA family dK/dV, from the dQ kernel)
  const float* lse2;       // backward input [Hq,T]: max(lse * log2(e), -FLT_MAX)
  const int32_t* ranges;   // [T,4] or null (tables without RANGES rows)
  int32_t window, sink;    // window > 0: the table has WINDOW rows; their per-token ranges are worked out, not read
  int32_t masked;          // the table has RANGES or WINDOW rows (rows with per-token ranges)
  float* part;             // backward, or null: fp32 partial sums of split dK/dV items, [slot][KV head][dK, dV][128 keys][D]
  const int32_t* qbounds;  // backward, or null: [32-row tiles of all blocks + 1][8] bounds of the rows' ranges (RangeBounds order)
  int64_t q_st, q_sh, k_st, k_sh, v_st, v_sh, o_st, o_sh, do_st, do_sh, dq_st, dq_sh, dk_st, dk_sh, dv_st, dv_sh;
  int64_t q_rows;   // rows of the Q-type buffers (= packed tokens without block buffers): row pitch of lse / delta / lse2
  int32_t hq, hkv, d, block_size;
  float scale;
  int32_t use_slots;
};

#ifdef __HIPCC__
// The range-array entry of packed token i (s0 = first token of its sequence): read from the array, or, for a
// sliding window with sink, the window [lo, i + 1) with lo = max(i - window + 1, s0) and the sink tokens before it,
// [s0, min(s0 + sink, lo)) (two ranges that do not overlap).
__device__ __forceinline__ int4 range_row(const KTensors& t, int i, int s0) {
  if (t.window > 0) {
    const int lo = max(i - t.window + 1, s0);
    return make_int4(s0, min(s0 + t.sink, lo), lo, i + 1);
  }
  return ((const int4*)t.ranges)[i];
}
#endif

// Grid of a launch whose workgroups find their work with decode_wg: 8 times the largest number of workgroups any XCD
// needs for its (KV head, segment) units.
inline int xcd_grid(const DevGroup& g, int heads_outer, int heads_inner) {
  const int upx = (heads_outer * g.n_seg) / 8;
  int most = 0;
  for (int x = 0; x < 8; x++) {
    int n = 0;
    for (int u = x * upx; u < (x + 1) * upx; u++) n += (g.seg[u % g.n_seg + 1] - g.seg[u % g.n_seg]) * heads_inner;
    most = n > most ? n : most;
  }
  return 8 * most;
}

// Optional per-kernel event timing (see dcp_profile_enable).
struct ProfScope {
  int id;
  hipStream_t s;
  hipEvent_t stop = nullptr;
  ProfScope(int id, hipStream_t s, bool enabled = true);
  ~ProfScope();
};

// the backward behind dcp_block_attn_bwd (api.hip); may_alloc = false: fail rather than create device copies or events
dcp_status_t bwd_launch(dcp_plan_t* plan, const dcp_tensors_t* t, void* workspace, size_t workspace_bytes, hipStream_t s,
                        bool may_alloc);

// device address, on the current device, of the fixed workspace of dcp_block_attn_bwd_static (bwd_static.hip); the first
// call on a device looks it up
dcp_status_t static_scratch(void** ptr);

// scalar fp32-ALU family (any dtype; D in {32, 64, 128})
bool scalar_supports(int32_t d);
int scalar_fwd_tile();
int scalar_bwd_tile();
dcp_status_t scalar_fwd(const DevGroup& g, const KTensors& t, int32_t dtype, hipStream_t s);
dcp_status_t scalar_bwd_dq(const DevGroup& g, const KTensors& t, int32_t dtype, hipStream_t s);
dcp_status_t scalar_bwd_dkv(const DevGroup& g, const KTensors& t, int32_t dtype, hipStream_t s);

// bf16 MFMA family (D = 128)
bool mfma_supports(int32_t dtype, int32_t d);
int mfma_fwd_tile();
int mfma_dq_tile();
int mfma_dkv_tile();
size_t mfma_dkv_part_bytes(int32_t n_pslots, int32_t hkv);   // size of KTensors::part for that many slots
dcp_status_t mfma_fwd(const DevGroup& g, const KTensors& t, hipStream_t s);
dcp_status_t mfma_bwd_dq(const DevGroup& g, const KTensors& t, hipStream_t s);
dcp_status_t mfma_bwd_dkv(const DevGroup& g, const KTensors& t, hipStream_t s);
void mfma_dkv_launch_ranges(const DevGroup& g, const KTensors& t, int grid, hipStream_t s);   // kernels_mfma_dkv_ranges.hip
// per 32-row tile of every block: bounds of its rows' range arrays -> qbounds [n_t32 + 1][8]
dcp_status_t mfma_range_bounds(const DevGroup& g, const KTensors& t, const int32_t* blk_t32, int32_t n_blocks, int32_t* qbounds,
                               hipStream_t s);

// streaming (HBM-bound) kernels
dcp_status_t stream_merge(const int32_t* merge_ptr, const int32_t* merge_idx, const int32_t* blk_mem0,
                          const int32_t* blk_len, int32_t n_blocks, int32_t block_size, const void* o_part,
                          const float* lse_part, void* out, int64_t o_st, int64_t o_sh, float* lse,
                          int64_t total_tokens, int32_t hq, int32_t d, int32_t dtype, hipStream_t s);
dcp_status_t stream_delta(const void* o, int64_t o_st, int64_t o_sh, const void* dout, int64_t do_st, int64_t do_sh,
                          float* delta, const float* lse, float* lse2, int64_t total_tokens, int32_t hq, int32_t d,
                          int32_t dtype, hipStream_t s);
dcp_status_t stream_sum(const void* const* parts, int32_t n_parts, int32_t parts_dtype, void* dst, int32_t dst_dtype,
                        int64_t n, hipStream_t s);

// chunks: device int32 [n_chunks, 3] (src_row, dst_row, n_rows)
dcp_status_t stream_copy(const int32_t* chunks, int64_t n_chunks, const void* src, int64_t src_stride, void* dst,
                         int64_t dst_stride, int64_t row_bytes, hipStream_t s);

}  // namespace dcp
