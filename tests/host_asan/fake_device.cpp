// A stand-in for the GPU side of libdcp_attn.so, for a CPU build of the library's host code under
// AddressSanitizer and UndefinedBehaviorSanitizer (test infrastructure; never part of the product).
//
//  * the HIP runtime calls the host code makes are served from host memory (hipMalloc = malloc, a
//    copy is a memcpy, a stream is always idle), so "device" arrays are exactly as large as the host
//    code asked for and the sanitizer sees every access to them;
//  * each kernel launcher is replaced by a host walk over the same plan arrays, in the order and with
//    the index arithmetic of the kernel it stands for (work item -> unit -> table rows -> block
//    records -> tensor rows), so an index that would leave an array on the GPU leaves it here and
//    is reported.  Rows and slots are checked against the extents the plan states for the tensors.
#include <hip/hip_runtime.h>

#include <cstdlib>
#include <cstring>
#include <string>

#include "kernels.h"

// ---------------------------------------------------------------- HIP runtime, host memory only
extern "C" {
hipError_t hipMalloc(void** p, size_t n) { *p = std::malloc(n ? n : 1); return *p ? hipSuccess : hipErrorOutOfMemory; }
hipError_t hipFree(void* p) { std::free(p); return hipSuccess; }
hipError_t hipMemcpyAsync(void* d, const void* s, size_t n, hipMemcpyKind, hipStream_t) { std::memcpy(d, s, n); return hipSuccess; }
hipError_t hipStreamSynchronize(hipStream_t) { return hipSuccess; }
hipError_t hipGetDevice(int* d) { *d = 0; return hipSuccess; }
hipError_t hipSetDevice(int) { return hipSuccess; }
const char* hipGetErrorString(hipError_t) { return "fake runtime error"; }
hipError_t hipEventCreate(hipEvent_t* e) { *e = (hipEvent_t)std::malloc(8); return hipSuccess; }
hipError_t hipEventCreateWithFlags(hipEvent_t* e, unsigned) { *e = (hipEvent_t)std::malloc(8); return hipSuccess; }
hipError_t hipEventDestroy(hipEvent_t e) { std::free((void*)e); return hipSuccess; }
hipError_t hipEventRecord(hipEvent_t, hipStream_t) { return hipSuccess; }
hipError_t hipEventSynchronize(hipEvent_t) { return hipSuccess; }
hipError_t hipEventElapsedTime(float* ms, hipEvent_t, hipEvent_t) { *ms = 0.f; return hipSuccess; }
hipError_t hipStreamWaitEvent(hipStream_t, hipEvent_t, unsigned) { return hipSuccess; }
}

namespace dcp {

static long g_rows_walked = 0;
long fake_rows_walked() { return g_rows_walked; }

#define WALK_CHECK(cond, what) \
  do { if (!(cond)) return fail(DCP_ERR_HIP, std::string("fake launch: ") + (what)); } while (0)

// What every attention kernel reads before its tile loop, and per table row inside it.
// own_rows / other_rows: extents of the tensors on the unit's side and on the other side.
static dcp_status_t walk_group(const DevGroup& g, int tile_rows, int64_t own_rows, int64_t other_rows, int32_t n_slots,
                               int32_t block_size, bool reduce_list) {
  // the segments of the work list cover it in order
  WALK_CHECK(g.n_seg >= 1 && g.n_seg <= 8 && g.seg[0] == 0 && g.seg[g.n_seg] == g.n_items, "work-list segments do not cover the list");
  for (int s = 0; s < 8; s++) WALK_CHECK(g.seg[s] <= g.seg[s + 1], "work-list segments not in order");
  for (int32_t i = 0; i < g.n_items; i++) {
    const WorkItem w = g.items[i];
    WALK_CHECK(w.unit >= 0 && w.unit < g.n_units, "work item names a unit out of range");
    const int32_t b = g.unit_blk[w.unit];
    WALK_CHECK(b >= 0, "work item for a unit without a block");
    WALK_CHECK(g.blk_start[b] == w.blk_start && g.blk_len[b] == w.blk_len, "work item's block record disagrees with the block arrays");
    WALK_CHECK(g.unit_moff[w.unit] == w.moff, "work item's memory offset disagrees with the unit's");
    WALK_CHECK(g.blk_s0[b] <= w.blk_start, "sequence start after the block");
    WALK_CHECK(w.tile >= 0 && (int64_t)w.tile * tile_rows < w.blk_len, "tile past the block");
    WALK_CHECK(g.ptr[w.unit] <= w.e0 && w.e0 <= w.e1 && w.e1 <= g.ptr[w.unit + 1], "table rows outside the unit's CSR range");
    const int64_t r0 = (int64_t)w.blk_start + (int64_t)w.tile * tile_rows + w.moff;
    const int64_t r1 = (int64_t)w.blk_start + std::min<int64_t>(w.blk_len, (int64_t)(w.tile + 1) * tile_rows) + w.moff;
    const int32_t slot = g.unit_out[w.unit];
    if (slot >= 0) WALK_CHECK(slot < n_slots && w.blk_len <= block_size, "output slot out of range");
    else WALK_CHECK(r0 >= 0 && r1 <= own_rows, "own rows outside the tensor");
    for (int32_t e = w.e0; e < w.e1; e++) {
      const int32_t* rec = g.ent_rec + 8 * (int64_t)e;
      WALK_CHECK(rec[0] == g.ent_start[e] && rec[1] == g.ent_len[e] && rec[2] == g.ent_kind[e] && rec[3] == g.ent_moff[e] &&
                 rec[4] == g.ent_t32[e], "table-row record disagrees with the per-field arrays");
      WALK_CHECK(rec[2] >= 0 && rec[2] <= 2, "device mask kind out of range");
      WALK_CHECK(rec[1] > 0 && (int64_t)rec[0] + rec[3] >= 0 && (int64_t)rec[0] + rec[1] + rec[3] <= other_rows, "other block's rows outside the tensor");
      g_rows_walked++;
    }
  }
  if (reduce_list)
    for (int32_t i = 0; i < g.n_reduce; i++) {
      const ReduceItem r = g.reduce[i];
      WALK_CHECK(r.unit >= 0 && r.unit < g.n_units && g.unit_blk[r.unit] >= 0, "reduce item names a bad unit");
      WALK_CHECK(r.n_parts >= 2 && r.first_pslot >= 0, "reduce item with fewer than two parts");
    }
  return DCP_OK;
}

// the fixed workspace of dcp_block_attn_bwd_static lives in a file with device code that this build leaves out
dcp_status_t static_scratch(void** ptr) { static char buf[256]; *ptr = buf; return DCP_OK; }

bool scalar_supports(int32_t d) { return d == 32 || d == 64 || d == 128; }
int scalar_fwd_tile() { return 64; }
int scalar_bwd_tile() { return 64; }
bool mfma_supports(int32_t dtype, int32_t d) { return dtype == DCP_BF16 && d == 128; }
int mfma_fwd_tile() { return 128; }
int mfma_dq_tile() { return 128; }
int mfma_dkv_tile() { return 128; }
size_t mfma_dkv_part_bytes(int32_t n_pslots, int32_t hkv) { return (size_t)n_pslots * (size_t)hkv * 2 * 128 * 128 * sizeof(float); }

// the fake tensors' extents travel in KTensors::q_rows (Q side) and, for the KV side, in a global the driver sets
int64_t g_fake_kv_rows = 0;
int32_t g_fake_n_slots = 0;

dcp_status_t scalar_fwd(const DevGroup& g, const KTensors& t, int32_t, hipStream_t) { return walk_group(g, 64, t.q_rows, g_fake_kv_rows, g_fake_n_slots, t.block_size, false); }
dcp_status_t scalar_bwd_dq(const DevGroup& g, const KTensors& t, int32_t, hipStream_t) { return walk_group(g, 64, t.q_rows, g_fake_kv_rows, 0, t.block_size, false); }
dcp_status_t scalar_bwd_dkv(const DevGroup& g, const KTensors& t, int32_t, hipStream_t) { return walk_group(g, 64, g_fake_kv_rows, t.q_rows, 0, t.block_size, false); }
dcp_status_t mfma_fwd(const DevGroup& g, const KTensors& t, hipStream_t) { return walk_group(g, 128, t.q_rows, g_fake_kv_rows, g_fake_n_slots, t.block_size, false); }
dcp_status_t mfma_bwd_dq(const DevGroup& g, const KTensors& t, hipStream_t) {
  // the preprocess fused into this kernel writes one float per (head, row) into each of the two workspace arrays
  if (g.n_items > 0) { t.delta_w[(int64_t)t.hq * t.q_rows - 1] = 0.f; t.lse2_w[(int64_t)t.hq * t.q_rows - 1] = 0.f; }
  return walk_group(g, 128, t.q_rows, g_fake_kv_rows, 0, t.block_size, false);
}
dcp_status_t mfma_bwd_dkv(const DevGroup& g, const KTensors& t, hipStream_t) {
  dcp_status_t st = walk_group(g, 128, g_fake_kv_rows, t.q_rows, 0, t.block_size, true);
  if (st != DCP_OK) return st;
  // every part slot of a cut item lies inside the partial-sum area of the workspace: touch its last float
  for (int32_t i = 0; i < g.n_items; i++)
    if (g.items[i].pslot >= 0) t.part[((int64_t)(g.items[i].pslot + 1) * t.hkv) * 2 * 128 * 128 - 1] = 0.f;
  return DCP_OK;
}
dcp_status_t mfma_range_bounds(const DevGroup& g, const KTensors& t, const int32_t* blk_t32, int32_t n_blocks, int32_t* qbounds,
                               hipStream_t) {
  for (int32_t b = 0; b < n_blocks; b++) {
    const int32_t n32 = (g.blk_len[b] + 31) / 32;
    WALK_CHECK(blk_t32[b + 1] - blk_t32[b] == n32, "32-row tile prefix sums disagree with the block lengths");
    for (int32_t x = 0; x < n32; x++)
      for (int k = 0; k < 8; k++) qbounds[(int64_t)(blk_t32[b] + x) * 8 + k] = 0;   // inside the workspace area
    (void)t;
  }
  return DCP_OK;
}

dcp_status_t stream_merge(const int32_t* merge_ptr, const int32_t* merge_idx, const int32_t* blk_mem0, const int32_t* blk_len,
                          int32_t n_blocks, int32_t block_size, const void*, const float*, void*, int64_t, int64_t, float*,
                          int64_t q_rows, int32_t, int32_t, int32_t, hipStream_t) {
  for (int32_t b = 0; b < n_blocks; b++) {
    WALK_CHECK(merge_ptr[b] <= merge_ptr[b + 1], "merge CSR not monotone");
    for (int32_t p = merge_ptr[b]; p < merge_ptr[b + 1]; p++) WALK_CHECK(merge_idx[p] >= 0 && merge_idx[p] < g_fake_n_slots, "merge slot out of range");
    if (blk_mem0[b] >= 0) WALK_CHECK((int64_t)blk_mem0[b] + blk_len[b] <= q_rows && blk_len[b] <= block_size, "merged block outside the output");
  }
  return DCP_OK;
}
dcp_status_t stream_delta(const void*, int64_t, int64_t, const void*, int64_t, int64_t, float* delta, const float*, float* lse2,
                          int64_t rows, int32_t hq, int32_t, int32_t, hipStream_t) {
  if (rows > 0) { delta[(int64_t)hq * rows - 1] = 0.f; if (lse2) lse2[(int64_t)hq * rows - 1] = 0.f; }
  return DCP_OK;
}
dcp_status_t stream_sum(const void* const*, int32_t, int32_t, void*, int32_t, int64_t, hipStream_t) { return DCP_OK; }
dcp_status_t stream_copy(const int32_t* chunks, int64_t n_chunks, const void* src, int64_t src_stride, void* dst, int64_t dst_stride,
                         int64_t row_bytes, hipStream_t) {
  // the copy itself, on host memory: the sanitizer checks every row against the buffers the driver allocated
  for (int64_t c = 0; c < n_chunks; c++)
    for (int32_t r = 0; r < chunks[3 * c + 2]; r++)
      std::memmove((char*)dst + (int64_t)(chunks[3 * c + 1] + r) * dst_stride, (const char*)src + (int64_t)(chunks[3 * c] + r) * src_stride, row_bytes);
  return DCP_OK;
}

}  // namespace dcp
