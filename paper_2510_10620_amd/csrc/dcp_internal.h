// Internal declarations shared by the host-side plan code and the kernel launchers.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>
#include <map>
#include <mutex>
#include <string>
#include <tuple>
#include <vector>

#include "dcp.h"

namespace dcp {

void set_error(const std::string& msg);
dcp_status_t fail(dcp_status_t code, const std::string& msg);

#define DCP_HIP_TRY(expr)                                                                     \
  do {                                                                                        \
    hipError_t e__ = (expr);                                                                  \
    if (e__ != hipSuccess)                                                                    \
      return ::dcp::fail(DCP_ERR_HIP, std::string(#expr) + ": " + hipGetErrorString(e__));    \
  } while (0)

// One piece of work: `unit` indexes a Group's units, `tile` is the tile number inside the unit's own block
// (tile * tile_rows is the first row), [e0, e1) the table rows of the unit this piece covers (all of them, unless
// the work list was built with splitting).  `pslot` >= 0: the piece is one part of a split (unit, tile) and leaves
// its fp32 result in that slot of the partial-sum workspace; -1: it writes the output itself.  32 bytes.
struct WorkItem {
  int32_t unit;
  int32_t tile;
  int32_t e0, e1;
  int32_t pslot;
  // the unit's own block, so that a workgroup needs one load, not a chain of them, before it can address its rows:
  int32_t blk_start, blk_len;   // first packed token and length
  int32_t moff;                 // memory row = packed index + moff (block buffers; 0 for packed tensors)
};

// A split (unit, tile): the parts' slots are first_pslot .. first_pslot + n_parts - 1, summed in that order.
struct ReduceItem {
  int32_t unit, tile, first_pslot, n_parts;
};

// Device view of a grouping of table rows by a unit (an output block / slot, or a KV block).
// Entry arrays describe the OTHER block of each row (the KV block for query-side groups, the
// Q block for the KV-side group): first packed token, length, mask kind.
struct DevGroup {
  const int32_t* unit_blk;   // [n_units] block that owns the unit's rows
  const int32_t* unit_out;   // [n_units] output slot (or -1: write to the packed tensor)
  const int32_t* ptr;        // [n_units + 1]
  const int32_t* ent_start;  // [nnz]
  const int32_t* ent_len;    // [nnz]
  const int32_t* ent_kind;   // [nnz]     0 NONE, 1 CAUSAL, 2 per-row ranges (RANGES, and WINDOW rows: their ranges are worked out)
  const int32_t* blk_start;  // [n_blocks]
  const int32_t* blk_len;    // [n_blocks]
  const int32_t* blk_s0;     // [n_blocks] first packed token of the block's sequence
  // Block buffers (Sec. 5): a token's row in memory is its packed index plus the offset of its block,
  // slot * block_size - blk_start (0 for packed tensors).
  const int32_t* unit_moff;  // [n_units] offset of the unit's own block (Q side for fwd / dQ, KV side for dK/dV)
  const int32_t* ent_moff;   // [nnz]     offset of each row's other block
  const int32_t* ent_t32;    // [nnz]     index of the other block's first 32-row tile (range-bound summaries)
  const int32_t* ent_rec;    // [nnz][8]  the same per row in one record: start, len, kind, moff, t32, 0, 0, 0 (32-byte aligned)
  const WorkItem* items;     // [n_items] longest first inside each segment
  const ReduceItem* reduce;  // [n_reduce] split (unit, tile)s, or null
  int32_t n_items;
  int32_t n_reduce;
  int32_t n_units;
  // The work list in n_seg segments of about equal cost (n_seg = xcd_segments(KV heads): 1, 2, 4 or 8):
  // segment s = items [seg[s], seg[s + 1]); entries past n_seg repeat n_items.
  int32_t n_seg;
  int32_t seg[9];
};

// Segments the work list is cut into so that (KV head, segment) pairs divide evenly among the 8 XCDs: one when the
// KV heads are a multiple of 8 (an XCD takes whole heads), 8 when there is one KV head.
inline int xcd_segments(int kv_heads) {
  int g = 8;
  while (kv_heads % g) g >>= 1;   // gcd(8, kv_heads)
  return 8 / g;
}

struct HostGroup {
  std::vector<int32_t> unit_blk, unit_out, ptr, idx, ent_blk, ent_start, ent_len, ent_kind;
};

struct HostItems {
  std::vector<WorkItem> items;
  std::vector<ReduceItem> reduce;
  int32_t n_pslots = 0;
  int32_t n_seg = 1;
  int32_t seg[9] = {0, 0, 0, 0, 0, 0, 0, 0, 0};
};

struct DevItems {
  WorkItem* items = nullptr;
  ReduceItem* reduce = nullptr;
  int32_t n_items = 0, n_reduce = 0;
};

}  // namespace dcp

struct dcp_plan {
  int32_t n_seq = 0, block_size = 0, n_blocks = 0, n_slots = 0;
  int64_t total_tokens = 0, n_kept = 0;
  bool use_slots = false, has_ranges = false, has_window = false;
  int32_t window = 0, sink = 0;   // parameters of the WINDOW rows (window 0: not set)
  // block buffers: slot of every block in the Q-type and the KV-type buffer (-1: absent), rows per buffer
  bool buffers = false;
  std::vector<int32_t> q_slot, kv_slot, q_moff, kv_moff;
  int64_t q_rows = 0, kv_rows = 0;
  std::vector<int32_t> blk_t32;   // [n_blocks + 1] prefix sums of ceil(blk_len / 32)
  std::vector<int32_t> cu, blk_start, blk_len, blk_seq;
  std::vector<int32_t> table;  // original rows [n,3]
  std::vector<int32_t> slot_qblk, merge_ptr, merge_idx;
  dcp::HostGroup fwd, bwdq, bwdkv;

  // device mirrors (created lazily on the device that is current at first launch)
  std::mutex mu;
  int device = -1;
  int32_t* dev_arena = nullptr;
  dcp::DevGroup d_fwd{}, d_bwdq{}, d_bwdkv{};
  const int32_t *d_merge_ptr = nullptr, *d_merge_idx = nullptr, *d_slot_qblk = nullptr, *d_q_mem0 = nullptr, *d_blk_t32 = nullptr;
  // (group id, tile rows, split heads, segments) -> work list; split heads = 0: no splitting, else the number of
  // workgroups launched per item (the long items are cut so that no workgroup outlasts the rest of the grid by much);
  // segments: see DevGroup
  typedef std::tuple<int, int, int, int> ItemKey;
  std::map<ItemKey, dcp::HostItems> h_items;
  std::map<ItemKey, dcp::DevItems> items;

  // may_alloc = false: fail (DCP_ERR_INVALID_ARG) instead of creating a device copy that does not exist yet
  dcp_status_t ensure_device(hipStream_t stream, bool may_alloc = true);
  // group id: 0 fwd, 1 bwdq, 2 bwdkv.  Host only; takes the plan's lock.
  const dcp::HostItems& host_items(int group_id, int tile_rows, int split_heads, int n_seg = 1);
  dcp_status_t group_for(int group_id, int tile_rows, hipStream_t stream, dcp::DevGroup* out, int split_heads = 0,
                         bool may_alloc = true, int n_seg = 1);
};

// Blockwise Copy list: validated entries cut into chunks of at most kCopyChunkRows rows.
static constexpr int kCopyChunkRows = 8;
struct dcp_copy_list {
  int64_t src_rows = 0, dst_rows = 0;
  bool alias_safe = true;            // no destination range overlaps a source range (as row intervals)
  std::vector<int32_t> chunks;       // [n_chunks, 3]
  std::mutex mu;
  int device = -1;
  int32_t* d_chunks = nullptr;
};

