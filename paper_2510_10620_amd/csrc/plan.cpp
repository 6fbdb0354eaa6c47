// Host side of the library: block generation from range arrays, pair counting, plan creation
// (validation, block token ranges, CSR groupings, longest-first work lists) and the lazy device
// mirror of the plan's integer arrays.  Follows Sec. 4.1 (block generation) and Sec. 5 (block
// tables, block buffers) of the DCP paper; integer-only, compared bit-exactly with the tests'
// independent reference.
#include <algorithm>
#include <cstring>
#include <memory>
#include <numeric>
#include <queue>
#include <set>

#include "dcp_internal.h"

namespace dcp {

static thread_local std::string g_err;
void set_error(const std::string& msg) { g_err = msg; }
dcp_status_t fail(dcp_status_t code, const std::string& msg) {
  g_err = msg;
  return code;
}

struct Partition {
  std::vector<int32_t> first, start, len, seq;
};

static dcp_status_t make_partition(const int32_t* cu, int32_t n_seq, int32_t B, Partition* p) {
  if (n_seq < 0 || (n_seq > 0 && !cu)) return fail(DCP_ERR_INVALID_ARG, "cu_seqlens is NULL or n_seq < 0");
  if (B <= 0) return fail(DCP_ERR_INVALID_ARG, "block_size must be positive");
  if (n_seq > 0 && cu[0] != 0) return fail(DCP_ERR_BAD_CU_SEQLENS, "cu_seqlens[0] must be 0");
  p->first.assign(1, 0);
  for (int32_t s = 0; s < n_seq; s++) {
    if (cu[s + 1] <= cu[s]) return fail(DCP_ERR_BAD_CU_SEQLENS, "cu_seqlens must be strictly increasing");
    int32_t L = cu[s + 1] - cu[s];
    int32_t nb = (L + B - 1) / B;
    for (int32_t i = 0; i < nb; i++) {
      p->start.push_back(cu[s] + i * B);
      p->len.push_back(std::min(B, L - i * B));
      p->seq.push_back(s);
    }
    p->first.push_back(p->first.back() + nb);
  }
  return DCP_OK;
}

// number of keys of [c0, c1) inside the union of a row's two ranges
static inline int64_t row_visible(const int32_t* r, int64_t c0, int64_t c1) {
  auto clip = [&](int64_t lo, int64_t hi) { return std::max<int64_t>(0, std::min(hi, c1) - std::max(lo, c0)); };
  int64_t a = clip(r[0], r[1]), b = clip(r[2], r[3]);
  int64_t olo = std::max<int64_t>(r[0], r[2]), ohi = std::min<int64_t>(r[1], r[3]);
  return a + b - clip(olo, ohi);
}

}  // namespace dcp

using namespace dcp;

extern "C" const char* dcp_last_error(void) { return g_err.c_str(); }

// Per-token ranges of a sliding window with sink: the window [lo, i + 1), lo = max(i - window + 1, s0), and the
// sink tokens before it, [s0, min(s0 + sink, lo)).
static std::vector<int32_t> window_ranges(const int32_t* cu, int32_t n_seq, int64_t window, int64_t sink) {
  std::vector<int32_t> r((size_t)(n_seq > 0 ? cu[n_seq] : 0) * 4);
  for (int32_t s = 0; s < n_seq; s++)
    for (int64_t i = cu[s]; i < cu[s + 1]; i++) {
      const int64_t lo = std::max<int64_t>(i - window + 1, cu[s]);
      r[4 * i] = cu[s];
      r[4 * i + 1] = (int32_t)std::min<int64_t>(cu[s] + sink, lo);
      r[4 * i + 2] = (int32_t)lo;
      r[4 * i + 3] = (int32_t)(i + 1);
    }
  return r;
}

static dcp_status_t check_window(int32_t window, int32_t sink) {
  if (window < 1 || window > (1 << 30)) return fail(DCP_ERR_INVALID_ARG, "window must lie in [1, 2^30]");
  if (sink < 0 || sink > (1 << 30)) return fail(DCP_ERR_INVALID_ARG, "sink must lie in [0, 2^30]");
  return DCP_OK;
}

static dcp_status_t build_table(const Partition& p, int32_t n_seq, const int32_t* ranges, int32_t other_kind,
                                int32_t* table_out, int64_t capacity, int64_t* n_out) {
  int64_t n = 0;
  for (int32_t s = 0; s < n_seq; s++) {
    for (int32_t qb = p.first[s]; qb < p.first[s + 1]; qb++) {
      int64_t q0 = p.start[qb], q1 = q0 + p.len[qb];
      // Bounds of the block's rows, per range: most KV blocks are settled by them (no row's range reaches the block:
      // no entry; one range of every row covers it: NONE) and only the blocks on a mask edge need the rows themselves.
      int64_t smin[2] = {INT64_MAX, INT64_MAX}, smax[2] = {INT64_MIN, INT64_MIN};
      int64_t emin[2] = {INT64_MAX, INT64_MAX}, emax[2] = {INT64_MIN, INT64_MIN};
      bool every[2] = {true, true};   // every row has this range non-empty
      for (int64_t i = q0; i < q1; i++)
        for (int k = 0; k < 2; k++) {
          const int64_t lo = ranges[4 * i + 2 * k], hi = ranges[4 * i + 2 * k + 1];
          if (hi > lo) {
            smin[k] = std::min(smin[k], lo); smax[k] = std::max(smax[k], lo);
            emin[k] = std::min(emin[k], hi); emax[k] = std::max(emax[k], hi);
          } else {
            every[k] = false;
          }
        }
      for (int32_t kb = p.first[s]; kb < p.first[s + 1]; kb++) {
        int64_t c0 = p.start[kb], c1 = c0 + p.len[kb];
        const bool out0 = emax[0] == INT64_MIN || c0 >= emax[0] || c1 <= smin[0];   // no row's first range reaches the block
        const bool out1 = emax[1] == INT64_MIN || c0 >= emax[1] || c1 <= smin[1];
        if (out0 && out1) continue;
        bool covered = false;
        for (int k = 0; k < 2; k++) covered |= every[k] && smax[k] <= c0 && emin[k] >= c1;
        if (covered) {
          if (table_out && n < capacity) {
            table_out[3 * n + 0] = qb;
            table_out[3 * n + 1] = kb;
            table_out[3 * n + 2] = DCP_MASK_NONE;
          }
          n++;
          continue;
        }
        bool any = false, all = true, causal = true;
        for (int64_t i = q0; i < q1; i++) {
          const int32_t* r = ranges + 4 * i;
          int64_t nvis = row_visible(r, c0, c1);
          any |= nvis > 0;
          all &= nvis == c1 - c0;
          // the causal predicate on this tile shows keys [c0, min(i + 1, c1)); the row matches it
          // iff it sees exactly that many keys, all of them inside that prefix
          int64_t want = std::max<int64_t>(0, std::min(i + 1, c1) - c0);
          causal &= (nvis == want) && (row_visible(r, c0, c0 + want) == want);
        }
        if (!any) continue;
        int32_t kind = all ? DCP_MASK_NONE : (causal ? DCP_MASK_CAUSAL : other_kind);
        if (table_out && n < capacity) {
          table_out[3 * n + 0] = qb;
          table_out[3 * n + 1] = kb;
          table_out[3 * n + 2] = kind;
        }
        n++;
      }
    }
  }
  *n_out = n;
  if (table_out && n > capacity) return fail(DCP_ERR_INVALID_ARG, "block table capacity too small");
  return DCP_OK;
}

extern "C" dcp_status_t dcp_build_block_table(const int32_t* cu, int32_t n_seq, int32_t B, const int32_t* ranges,
                                              int32_t* table_out, int64_t capacity, int64_t* n_out) {
  if (!n_out) return fail(DCP_ERR_INVALID_ARG, "n_entries_out is NULL");
  Partition p;
  dcp_status_t st = make_partition(cu, n_seq, B, &p);
  if (st != DCP_OK) return st;
  if (!ranges && n_seq > 0) return fail(DCP_ERR_INVALID_ARG, "attn_ranges is NULL");
  return build_table(p, n_seq, ranges, DCP_MASK_RANGES, table_out, capacity, n_out);
}

extern "C" dcp_status_t dcp_build_block_table_window(const int32_t* cu, int32_t n_seq, int32_t B, int32_t window, int32_t sink,
                                                     int32_t* table_out, int64_t capacity, int64_t* n_out) {
  if (!n_out) return fail(DCP_ERR_INVALID_ARG, "n_entries_out is NULL");
  Partition p;
  dcp_status_t st = make_partition(cu, n_seq, B, &p);
  if (st != DCP_OK) return st;
  if ((st = check_window(window, sink)) != DCP_OK) return st;
  const std::vector<int32_t> r = window_ranges(cu, n_seq, window, sink);
  return build_table(p, n_seq, r.data(), DCP_MASK_WINDOW, table_out, capacity, n_out);
}

extern "C" dcp_status_t dcp_count_pairs_window(const int32_t* cu, int32_t n_seq, int32_t B, const int32_t* table,
                                               int64_t n_entries, int32_t window, int32_t sink, int64_t* pairs_out) {
  Partition p;
  dcp_status_t st = make_partition(cu, n_seq, B, &p);
  if (st != DCP_OK) return st;
  if ((st = check_window(window, sink)) != DCP_OK) return st;
  if (n_entries < 0 || (n_entries > 0 && (!table || !pairs_out))) return fail(DCP_ERR_INVALID_ARG, "bad table / output pointer");
  std::vector<int32_t> t2(table, table + 3 * n_entries);
  for (int64_t e = 0; e < n_entries; e++) {
    if (t2[3 * e + 2] == DCP_MASK_RANGES) return fail(DCP_ERR_BAD_TABLE, "RANGES row in a WINDOW table");
    if (t2[3 * e + 2] == DCP_MASK_WINDOW) t2[3 * e + 2] = DCP_MASK_RANGES;
  }
  const std::vector<int32_t> r = window_ranges(cu, n_seq, window, sink);
  return dcp_count_pairs(cu, n_seq, B, t2.data(), n_entries, r.data(), pairs_out);
}

extern "C" dcp_status_t dcp_count_pairs(const int32_t* cu, int32_t n_seq, int32_t B, const int32_t* table,
                                        int64_t n_entries, const int32_t* ranges, int64_t* pairs_out) {
  Partition p;
  dcp_status_t st = make_partition(cu, n_seq, B, &p);
  if (st != DCP_OK) return st;
  if (n_entries < 0 || (n_entries > 0 && (!table || !pairs_out))) return fail(DCP_ERR_INVALID_ARG, "bad table / output pointer");
  const int32_t nb = (int32_t)p.start.size();
  for (int64_t e = 0; e < n_entries; e++) {
    int32_t qb = table[3 * e], kb = table[3 * e + 1], kind = table[3 * e + 2];
    if (qb < 0 || qb >= nb || kb < 0 || kb >= nb) return fail(DCP_ERR_BAD_TABLE, "block id out of range");
    int64_t q0 = p.start[qb], q1 = q0 + p.len[qb], c0 = p.start[kb], c1 = c0 + p.len[kb];
    int64_t n = 0;
    if (kind == DCP_MASK_NONE) {
      n = (q1 - q0) * (c1 - c0);
    } else if (kind == DCP_MASK_CAUSAL) {
      for (int64_t i = q0; i < q1; i++) n += std::max<int64_t>(0, std::min(i + 1, c1) - c0);
    } else if (kind == DCP_MASK_RANGES) {
      if (!ranges) return fail(DCP_ERR_INVALID_ARG, "RANGES row without attn_ranges");
      for (int64_t i = q0; i < q1; i++) n += row_visible(ranges + 4 * i, c0, c1);
    } else if (kind != DCP_MASK_SKIP) {
      return fail(DCP_ERR_BAD_TABLE, "bad mask_kind");
    }
    pairs_out[e] = n;
  }
  return DCP_OK;
}

extern "C" dcp_status_t dcp_comm_volume(const int32_t* cu, int32_t n_seq, int32_t B, const int32_t* table, int64_t n_entries,
                                        const int32_t* blk_dev, const int32_t* comp_dev, int32_t n_devices, int64_t q_bytes,
                                        int64_t kv_bytes, int64_t o_bytes, int64_t* pairwise, int64_t* connectivity,
                                        int64_t* n_hyperedges, int64_t* send, int64_t* recv) {
  Partition p;
  dcp_status_t st = make_partition(cu, n_seq, B, &p);
  if (st != DCP_OK) return st;
  const int32_t nb = (int32_t)p.start.size();
  if (n_entries < 0 || (n_entries > 0 && (!table || !comp_dev))) return fail(DCP_ERR_INVALID_ARG, "table / comp_dev is NULL or n_entries < 0");
  if (nb > 0 && !blk_dev) return fail(DCP_ERR_INVALID_ARG, "blk_dev is NULL");
  if (n_devices <= 0) return fail(DCP_ERR_INVALID_ARG, "n_devices must be positive");
  if (q_bytes < 0 || kv_bytes < 0 || o_bytes < 0) return fail(DCP_ERR_INVALID_ARG, "negative bytes per token");
  for (int32_t b = 0; b < nb; b++)
    if (blk_dev[b] < 0 || blk_dev[b] >= n_devices) return fail(DCP_ERR_BAD_TABLE, "blk_dev[" + std::to_string(b) + "] out of range");
  // per data block: the set of devices that compute with it (one bit set per device, kept as sorted vectors)
  std::vector<std::vector<int32_t>> q_users(nb), kv_users(nb);
  int64_t pw = 0;
  for (int64_t e = 0; e < n_entries; e++) {
    const int32_t qb = table[3 * e], kb = table[3 * e + 1], kind = table[3 * e + 2], d = comp_dev[e];
    if (kind < 0 || kind > 4) return fail(DCP_ERR_BAD_TABLE, "row " + std::to_string(e) + ": bad mask_kind");
    if (qb < 0 || qb >= nb || kb < 0 || kb >= nb) return fail(DCP_ERR_BAD_TABLE, "row " + std::to_string(e) + ": block id out of range");
    if (kind == DCP_MASK_SKIP) continue;
    if (d < 0 || d >= n_devices) return fail(DCP_ERR_BAD_TABLE, "comp_dev[" + std::to_string(e) + "] out of range");
    if (blk_dev[qb] != d) pw += (int64_t)p.len[qb] * (q_bytes + o_bytes);
    if (blk_dev[kb] != d) pw += (int64_t)p.len[kb] * kv_bytes;
    q_users[qb].push_back(d);
    kv_users[kb].push_back(d);
  }
  int64_t conn = 0, edges = 0;
  if (send) std::fill(send, send + n_devices, 0);
  if (recv) std::fill(recv, recv + n_devices, 0);
  for (int32_t b = 0; b < nb; b++) {
    const int32_t owner = blk_dev[b];
    for (int side = 0; side < 3; side++) {          // 0: Q block, 1: KV block, 2: O block (made by the users of the Q block)
      std::vector<int32_t>& u = side == 1 ? kv_users[b] : q_users[b];
      if (u.empty()) continue;
      if (side != 2) { std::sort(u.begin(), u.end()); u.erase(std::unique(u.begin(), u.end()), u.end()); }
      edges++;
      const int64_t size = (int64_t)p.len[b] * (side == 0 ? q_bytes : (side == 1 ? kv_bytes : o_bytes));
      for (int32_t d : u) {
        if (d == owner) continue;
        conn += size;
        if (side != 2) { if (send) send[owner] += size; if (recv) recv[d] += size; }
        else { if (send) send[d] += size; if (recv) recv[owner] += size; }
      }
    }
  }
  if (pairwise) *pairwise = pw;
  if (connectivity) *connectivity = conn;
  if (n_hyperedges) *n_hyperedges = edges;
  return DCP_OK;
}

// Groups kept rows by unit_of(row); inside a unit ascending by other(row), stable.
template <class UnitOf, class OtherOf>
static void build_group(const dcp_plan& pl, const std::vector<int64_t>& kept, int32_t n_units, UnitOf unit_of,
                        OtherOf other_of, HostGroup* g) {
  std::vector<int64_t> order(kept);
  std::stable_sort(order.begin(), order.end(), [&](int64_t a, int64_t b) {
    int32_t ua = unit_of(a), ub = unit_of(b);
    if (ua != ub) return ua < ub;
    return other_of(a) < other_of(b);
  });
  g->ptr.assign(n_units + 1, 0);
  for (int64_t e : order) g->ptr[unit_of(e) + 1]++;
  for (int32_t u = 0; u < n_units; u++) g->ptr[u + 1] += g->ptr[u];
  g->idx.clear();
  g->ent_blk.clear();
  g->ent_start.clear();
  g->ent_len.clear();
  g->ent_kind.clear();
  for (int64_t e : order) {
    int32_t ob = other_of(e);
    g->idx.push_back((int32_t)e);
    g->ent_blk.push_back(ob);
    g->ent_start.push_back(pl.blk_start[ob]);
    g->ent_len.push_back(pl.blk_len[ob]);
    g->ent_kind.push_back(pl.table[3 * e + 2]);
  }
}

extern "C" dcp_status_t dcp_plan_create(dcp_plan_t** out, const int32_t* cu, int32_t n_seq, int32_t B,
                                        const int32_t* table, int64_t n_entries, const int32_t* out_slot,
                                        int32_t n_slots) {
  if (!out) return fail(DCP_ERR_INVALID_ARG, "plan output pointer is NULL");
  *out = nullptr;
  Partition p;
  dcp_status_t st = make_partition(cu, n_seq, B, &p);
  if (st != DCP_OK) return st;
  if (n_entries < 0 || (n_entries > 0 && !table)) return fail(DCP_ERR_INVALID_ARG, "block table is NULL or n_entries < 0");
  if (out_slot && n_slots < 0) return fail(DCP_ERR_INVALID_ARG, "n_slots < 0");
  if (n_entries > INT32_MAX) return fail(DCP_ERR_INVALID_ARG, "too many table rows");

  std::unique_ptr<dcp_plan> pl(new dcp_plan);
  pl->n_seq = n_seq;
  pl->block_size = B;
  pl->n_blocks = (int32_t)p.start.size();
  pl->total_tokens = n_seq > 0 ? cu[n_seq] : 0;
  pl->q_rows = pl->kv_rows = pl->total_tokens;
  pl->q_moff.assign(pl->n_blocks, 0);
  pl->blk_t32.assign(pl->n_blocks + 1, 0);
  for (int32_t b = 0; b < pl->n_blocks; b++) pl->blk_t32[b + 1] = pl->blk_t32[b] + (p.len[b] + 31) / 32;
  pl->kv_moff.assign(pl->n_blocks, 0);
  pl->cu.assign(cu, cu + (n_seq > 0 ? n_seq + 1 : 0));
  pl->blk_start = p.start;
  pl->blk_len = p.len;
  pl->blk_seq = p.seq;
  pl->table.assign(table, table + 3 * n_entries);
  pl->use_slots = out_slot != nullptr;
  pl->n_slots = out_slot ? n_slots : 0;
  pl->slot_qblk.assign(pl->n_slots, -1);

  std::vector<int64_t> kept;
  std::set<std::pair<int32_t, int32_t>> seen;
  for (int64_t e = 0; e < n_entries; e++) {
    int32_t qb = table[3 * e], kb = table[3 * e + 1], kind = table[3 * e + 2];
    if (kind < 0 || kind > 4) return fail(DCP_ERR_BAD_TABLE, "row " + std::to_string(e) + ": bad mask_kind");
    if (qb < 0 || qb >= pl->n_blocks || kb < 0 || kb >= pl->n_blocks)
      return fail(DCP_ERR_BAD_TABLE, "row " + std::to_string(e) + ": block id out of range");
    if (p.seq[qb] != p.seq[kb])
      return fail(DCP_ERR_BAD_TABLE, "row " + std::to_string(e) + ": q_blk and kv_blk belong to different sequences");
    if (out_slot && (out_slot[e] < 0 || out_slot[e] >= n_slots))
      return fail(DCP_ERR_BAD_TABLE, "row " + std::to_string(e) + ": output slot out of range");
    if (kind == DCP_MASK_SKIP) continue;
    if (!seen.insert({qb, kb}).second)
      return fail(DCP_ERR_BAD_TABLE, "row " + std::to_string(e) + ": duplicate (q_blk, kv_blk)");
    if (out_slot) {
      int32_t& sq = pl->slot_qblk[out_slot[e]];
      if (sq >= 0 && sq != qb)
        return fail(DCP_ERR_BAD_TABLE, "row " + std::to_string(e) + ": output slot shared by two q_blks");
      sq = qb;
    }
    if (kind == DCP_MASK_RANGES) pl->has_ranges = true;
    if (kind == DCP_MASK_WINDOW) pl->has_window = true;
    if (pl->has_ranges && pl->has_window) return fail(DCP_ERR_BAD_TABLE, "a table holds RANGES rows or WINDOW rows, not both");
    kept.push_back(e);
  }
  pl->n_kept = (int64_t)kept.size();

  auto qb_of = [&](int64_t e) { return table[3 * e]; };
  auto kb_of = [&](int64_t e) { return table[3 * e + 1]; };
  if (out_slot) {
    build_group(*pl, kept, n_slots, [&](int64_t e) { return out_slot[e]; }, kb_of, &pl->fwd);
    pl->fwd.unit_blk = pl->slot_qblk;
    pl->fwd.unit_out.resize(n_slots);
    std::iota(pl->fwd.unit_out.begin(), pl->fwd.unit_out.end(), 0);
  } else {
    build_group(*pl, kept, pl->n_blocks, qb_of, kb_of, &pl->fwd);
    pl->fwd.unit_blk.resize(pl->n_blocks);
    std::iota(pl->fwd.unit_blk.begin(), pl->fwd.unit_blk.end(), 0);
    pl->fwd.unit_out.assign(pl->n_blocks, -1);
  }
  build_group(*pl, kept, pl->n_blocks, qb_of, kb_of, &pl->bwdq);
  build_group(*pl, kept, pl->n_blocks, kb_of, qb_of, &pl->bwdkv);
  for (HostGroup* g : {&pl->bwdq, &pl->bwdkv}) {
    g->unit_blk.resize(pl->n_blocks);
    std::iota(g->unit_blk.begin(), g->unit_blk.end(), 0);
    g->unit_out.assign(pl->n_blocks, -1);
  }
  // merge lists: the used slots of every q_blk, ascending
  pl->merge_ptr.assign(pl->n_blocks + 1, 0);
  for (int32_t s = 0; s < pl->n_slots; s++)
    if (pl->slot_qblk[s] >= 0) pl->merge_ptr[pl->slot_qblk[s] + 1]++;
  for (int32_t b = 0; b < pl->n_blocks; b++) pl->merge_ptr[b + 1] += pl->merge_ptr[b];
  pl->merge_idx.assign(pl->merge_ptr.back(), 0);
  {
    std::vector<int32_t> fill(pl->merge_ptr.begin(), pl->merge_ptr.end() - 1);
    for (int32_t s = 0; s < pl->n_slots; s++)
      if (pl->slot_qblk[s] >= 0) pl->merge_idx[fill[pl->slot_qblk[s]]++] = s;
  }
  *out = pl.release();
  return DCP_OK;
}

extern "C" dcp_status_t dcp_plan_set_block_buffers(dcp_plan_t* plan, const int32_t* q_slot, int32_t n_q_slots,
                                                   const int32_t* kv_slot, int32_t n_kv_slots) {
  if (!plan) return fail(DCP_ERR_INVALID_ARG, "plan is NULL");
  std::lock_guard<std::mutex> lock(plan->mu);
  if (plan->dev_arena) return fail(DCP_ERR_INVALID_ARG, "block buffers must be set before the plan is first used on a device");
  if (plan->n_blocks > 0 && (!q_slot || !kv_slot)) return fail(DCP_ERR_INVALID_ARG, "slot array is NULL");
  if (n_q_slots < 0 || n_kv_slots < 0) return fail(DCP_ERR_INVALID_ARG, "negative slot count");
  const int64_t B = plan->block_size;
  if ((int64_t)n_q_slots * B > INT32_MAX || (int64_t)n_kv_slots * B > INT32_MAX)
    return fail(DCP_ERR_INVALID_ARG, "a block buffer would hold 2^31 rows or more");
  std::vector<char> used_q(plan->n_blocks, 0), used_kv(plan->n_blocks, 0);
  for (size_t e = 0; e + 2 < plan->table.size(); e += 3) {
    if (plan->table[e + 2] == DCP_MASK_SKIP) continue;
    used_q[plan->table[e]] = 1;
    used_kv[plan->table[e + 1]] = 1;
  }
  for (int side = 0; side < 2; side++) {
    const int32_t* slot = side ? kv_slot : q_slot;
    const int32_t n = side ? n_kv_slots : n_q_slots;
    const std::vector<char>& used = side ? used_kv : used_q;
    std::vector<char> taken(n, 0);
    for (int32_t b = 0; b < plan->n_blocks; b++) {
      const int32_t s = slot[b];
      const std::string what = std::string(side ? "kv" : "q") + " slot of block " + std::to_string(b);
      if (s < -1 || s >= n) return fail(DCP_ERR_BAD_TABLE, what + " is out of range");
      if (s < 0) {
        if (used[b]) return fail(DCP_ERR_BAD_TABLE, what + " is absent but the table uses the block");
        continue;
      }
      if (taken[s]) return fail(DCP_ERR_BAD_TABLE, what + " is taken by another block");
      taken[s] = 1;
    }
  }
  plan->buffers = true;
  plan->h_items.clear();   // work lists leave out absent blocks
  plan->q_slot.assign(q_slot, q_slot + plan->n_blocks);
  plan->kv_slot.assign(kv_slot, kv_slot + plan->n_blocks);
  for (int32_t b = 0; b < plan->n_blocks; b++) {
    plan->q_moff[b] = q_slot[b] < 0 ? 0 : (int32_t)((int64_t)q_slot[b] * B - plan->blk_start[b]);
    plan->kv_moff[b] = kv_slot[b] < 0 ? 0 : (int32_t)((int64_t)kv_slot[b] * B - plan->blk_start[b]);
  }
  plan->q_rows = (int64_t)n_q_slots * B;
  plan->kv_rows = (int64_t)n_kv_slots * B;
  return DCP_OK;
}

extern "C" dcp_status_t dcp_plan_set_window(dcp_plan_t* plan, int32_t window, int32_t sink) {
  if (!plan) return fail(DCP_ERR_INVALID_ARG, "plan is NULL");
  dcp_status_t st = check_window(window, sink);
  if (st != DCP_OK) return st;
  std::lock_guard<std::mutex> lock(plan->mu);
  plan->window = window;
  plan->sink = sink;
  return DCP_OK;
}

extern "C" dcp_status_t dcp_plan_destroy(dcp_plan_t* plan) {
  if (!plan) return DCP_OK;
  if (plan->dev_arena || !plan->items.empty()) {
    int cur = -1;
    (void)hipGetDevice(&cur);
    if (plan->device >= 0 && cur != plan->device) (void)hipSetDevice(plan->device);
    if (plan->dev_arena) (void)hipFree(plan->dev_arena);
    for (auto& kv : plan->items) {
      if (kv.second.items) (void)hipFree(kv.second.items);
      if (kv.second.reduce) (void)hipFree(kv.second.reduce);
    }
    if (plan->device >= 0 && cur >= 0 && cur != plan->device) (void)hipSetDevice(cur);
  }
  delete plan;
  return DCP_OK;
}

extern "C" dcp_status_t dcp_plan_export(const dcp_plan_t* plan, dcp_export_t which, int32_t* dst, int64_t capacity,
                                        int64_t* n_out) {
  if (!plan || !n_out) return fail(DCP_ERR_INVALID_ARG, "plan or n_out is NULL");
  const std::vector<int32_t>* v = nullptr;
  switch (which) {
    case DCP_EXPORT_BLK_START: v = &plan->blk_start; break;
    case DCP_EXPORT_BLK_LEN: v = &plan->blk_len; break;
    case DCP_EXPORT_BLK_SEQ: v = &plan->blk_seq; break;
    case DCP_EXPORT_FWD_PTR: v = &plan->fwd.ptr; break;
    case DCP_EXPORT_FWD_IDX: v = &plan->fwd.idx; break;
    case DCP_EXPORT_BWDQ_PTR: v = &plan->bwdq.ptr; break;
    case DCP_EXPORT_BWDQ_IDX: v = &plan->bwdq.idx; break;
    case DCP_EXPORT_BWDKV_PTR: v = &plan->bwdkv.ptr; break;
    case DCP_EXPORT_BWDKV_IDX: v = &plan->bwdkv.idx; break;
    case DCP_EXPORT_SLOT_QBLK: v = &plan->slot_qblk; break;
    case DCP_EXPORT_MERGE_PTR: v = &plan->merge_ptr; break;
    case DCP_EXPORT_MERGE_IDX: v = &plan->merge_idx; break;
    default: return fail(DCP_ERR_INVALID_ARG, "unknown export id");
  }
  *n_out = (int64_t)v->size();
  if (dst) {
    if (capacity < (int64_t)v->size()) return fail(DCP_ERR_INVALID_ARG, "export capacity too small");
    if (!v->empty()) std::memcpy(dst, v->data(), v->size() * sizeof(int32_t));
  }
  return DCP_OK;
}

// ------------------------------------------------------------------------------------------------
// device mirror
dcp_status_t dcp_plan::ensure_device(hipStream_t stream, bool may_alloc) {
  std::lock_guard<std::mutex> lock(mu);
  int cur = 0;
  DCP_HIP_TRY(hipGetDevice(&cur));
  if (dev_arena) {
    if (cur != device) return fail(DCP_ERR_INVALID_ARG, "plan was first used on another device");
    return DCP_OK;
  }
  if (!may_alloc) return fail(DCP_ERR_INVALID_ARG, "the plan has no device copy yet: call dcp_plan_prepare first");
  std::vector<int32_t> host;
  auto put = [&](const std::vector<int32_t>& v) {
    size_t off = host.size();
    host.insert(host.end(), v.begin(), v.end());
    while (host.size() % 4) host.push_back(0);
    return off;
  };
  std::vector<int32_t> blk_s0(n_blocks);
  for (int32_t b = 0; b < n_blocks; b++) blk_s0[b] = cu[blk_seq[b]];
  size_t o_bs = put(blk_start), o_bl = put(blk_len), o_s0 = put(blk_s0);
  struct Off { size_t ub, uo, ptr, es, el, ek, um, em, et, er; } go[3];
  HostGroup* gs[3] = {&fwd, &bwdq, &bwdkv};
  for (int i = 0; i < 3; i++) {
    // memory offsets: own side = Q for the query-side groups, KV for the dK/dV group
    const std::vector<int32_t>& own = i == 2 ? kv_moff : q_moff;
    const std::vector<int32_t>& other = i == 2 ? q_moff : kv_moff;
    std::vector<int32_t> um(gs[i]->unit_blk.size(), 0), em(gs[i]->ent_blk.size(), 0);
    for (size_t u = 0; u < um.size(); u++)
      if (gs[i]->unit_blk[u] >= 0) um[u] = own[gs[i]->unit_blk[u]];
    std::vector<int32_t> et(gs[i]->ent_blk.size(), 0);
    for (size_t e = 0; e < em.size(); e++) { em[e] = other[gs[i]->ent_blk[e]]; et[e] = blk_t32[gs[i]->ent_blk[e]]; }
    // on the device a WINDOW row is a row with per-token ranges like a RANGES row; only where the ranges come from differs
    std::vector<int32_t> dk(gs[i]->ent_kind);
    for (int32_t& k : dk)
      if (k == DCP_MASK_WINDOW) k = DCP_MASK_RANGES;
    go[i] = {put(gs[i]->unit_blk), put(gs[i]->unit_out), put(gs[i]->ptr), put(gs[i]->ent_start), put(gs[i]->ent_len), put(dk),
             put(um), put(em), put(et), 0};
    {
      std::vector<int32_t> rec(gs[i]->ent_blk.size() * 8, 0);
      for (size_t e = 0; e < em.size(); e++) {
        rec[8 * e] = gs[i]->ent_start[e]; rec[8 * e + 1] = gs[i]->ent_len[e]; rec[8 * e + 2] = dk[e];
        rec[8 * e + 3] = em[e]; rec[8 * e + 4] = et[e];
      }
      while (host.size() % 8) host.push_back(0);   // records are read as 16-byte vectors
      go[i].er = put(rec);
    }
  }
  size_t o_mp = put(merge_ptr), o_mi = put(merge_idx), o_sq = put(slot_qblk);
  // first row of every block in the Q-type buffers (-1: absent), for the merge
  std::vector<int32_t> q_mem0(n_blocks);
  for (int32_t b = 0; b < n_blocks; b++) q_mem0[b] = (buffers && q_slot[b] < 0) ? -1 : blk_start[b] + q_moff[b];
  size_t o_qm = put(q_mem0), o_t32 = put(blk_t32);
  host.push_back(0);
  DCP_HIP_TRY(hipMalloc((void**)&dev_arena, host.size() * sizeof(int32_t)));
  hipError_t e = hipMemcpyAsync(dev_arena, host.data(), host.size() * sizeof(int32_t), hipMemcpyHostToDevice, stream);
  if (e == hipSuccess) e = hipStreamSynchronize(stream);  // `host` dies at scope exit
  if (e != hipSuccess) {
    (void)hipFree(dev_arena);
    dev_arena = nullptr;
    return fail(DCP_ERR_HIP, std::string("plan upload: ") + hipGetErrorString(e));
  }
  device = cur;
  DevGroup* ds[3] = {&d_fwd, &d_bwdq, &d_bwdkv};
  for (int i = 0; i < 3; i++) {
    ds[i]->unit_blk = dev_arena + go[i].ub;
    ds[i]->unit_out = dev_arena + go[i].uo;
    ds[i]->ptr = dev_arena + go[i].ptr;
    ds[i]->ent_start = dev_arena + go[i].es;
    ds[i]->ent_len = dev_arena + go[i].el;
    ds[i]->ent_kind = dev_arena + go[i].ek;
    ds[i]->unit_moff = dev_arena + go[i].um;
    ds[i]->ent_moff = dev_arena + go[i].em;
    ds[i]->ent_t32 = dev_arena + go[i].et;
    ds[i]->ent_rec = dev_arena + go[i].er;
    ds[i]->blk_start = dev_arena + o_bs;
    ds[i]->blk_len = dev_arena + o_bl;
    ds[i]->blk_s0 = dev_arena + o_s0;
    ds[i]->items = nullptr;
    ds[i]->reduce = nullptr;
    ds[i]->n_items = 0;
    ds[i]->n_reduce = 0;
    ds[i]->n_units = (int32_t)gs[i]->unit_blk.size();
  }
  d_merge_ptr = dev_arena + o_mp;
  d_merge_idx = dev_arena + o_mi;
  d_slot_qblk = dev_arena + o_sq;
  d_q_mem0 = dev_arena + o_qm;
  d_blk_t32 = dev_arena + o_t32;
  return DCP_OK;
}

// Estimated visible pairs between packed rows [r0, r1) and the block [c0, c1) under `kind`;
// `rows_are_keys` flips the causal predicate (rows are keys j, columns are queries i).
static int64_t tile_cost(int32_t kind, int64_t r0, int64_t r1, int64_t c0, int64_t c1, bool rows_are_keys) {
  int64_t n = 0;
  if (kind == DCP_MASK_NONE) return (r1 - r0) * (c1 - c0);
  if (kind == DCP_MASK_CAUSAL) {
    if (!rows_are_keys)
      for (int64_t i = r0; i < r1; i++) n += std::max<int64_t>(0, std::min(i + 1, c1) - c0);
    else
      for (int64_t j = r0; j < r1; j++) n += std::max<int64_t>(0, c1 - std::max(j, c0));
    return n;
  }
  return (r1 - r0) * (c1 - c0) / 2;  // RANGES: unknown without the arrays; half is the estimate
}

// Workgroups the chip holds at once in the kernels that split their items (2 per CU, 256 CUs).
static constexpr int64_t kResidentWorkgroups = 512;
static constexpr int32_t kMaxParts = 64;

const HostItems& dcp_plan::host_items(int gid, int tile_rows, int split_heads, int n_seg) {
  std::lock_guard<std::mutex> lock(mu);
  const ItemKey key(gid, tile_rows, split_heads, n_seg);
  auto hit = h_items.find(key);
  if (hit != h_items.end()) return hit->second;
  HostGroup* hg = gid == 0 ? &fwd : (gid == 1 ? &bwdq : &bwdkv);
  struct Scored { WorkItem w; int64_t cost; };
  std::vector<Scored> sc;
  std::vector<int64_t> ecost;   // per-entry costs of the item being built
  // first pass: whole items and the total cost
  int64_t total = 0;
  for (int32_t u = 0; u < (int32_t)hg->unit_blk.size(); u++) {
    int32_t b = hg->unit_blk[u];
    if (b < 0) continue;  // unused slot
    if (buffers && (gid == 2 ? kv_slot[b] : q_slot[b]) < 0) continue;  // block absent from its buffer: nothing to write
    int32_t nt = (blk_len[b] + tile_rows - 1) / tile_rows;
    for (int32_t t = 0; t < nt; t++) {
      int64_t r0 = blk_start[b] + (int64_t)t * tile_rows;
      int64_t r1 = std::min<int64_t>(r0 + tile_rows, blk_start[b] + blk_len[b]);
      int64_t cost = 0;
      for (int32_t e = hg->ptr[u]; e < hg->ptr[u + 1]; e++)
        cost += tile_cost(hg->ent_kind[e], r0, r1, hg->ent_start[e], hg->ent_start[e] + hg->ent_len[e], gid == 2);
      sc.push_back({{u, t, hg->ptr[u], hg->ptr[u + 1], -1, blk_start[b], blk_len[b], (gid == 2 ? kv_moff : q_moff)[b]}, cost});
      total += cost;
    }
  }
  HostItems hi;
  if (split_heads > 0) {
    // Long items are cut, along their table rows, into parts (each with a slot of fp32 partial sums that a reduce
    // kernel adds up): one key tile under a sink, or the first keys of the one long sequence of a small batch, can
    // otherwise outlast the rest of the grid.  Cutting costs partial-sum traffic and a second start-up per part
    // (measured on the 65 536-token causal batch: every doubling of the number of parts beyond need costs 2-5 % of
    // the kernel), so the least cutting that balances the launch is chosen: the launch is played through as list
    // scheduling (items in the order they are issued, longest first, each on the workgroup slot that frees up
    // first) and items longer than 1/d of a slot's share are cut for d = 0 (none), 1, 2, 4 until the estimated
    // finish is within 5 % of the share, or d = 4 is reached.  Parts hold whole table rows, at most kMaxParts.
    const double share = (double)total * split_heads / kResidentWorkgroups;
    auto finish_time = [&](std::vector<Scored> v) {
      std::stable_sort(v.begin(), v.end(), [](const Scored& a, const Scored& b) { return a.cost > b.cost; });
      std::priority_queue<int64_t, std::vector<int64_t>, std::greater<int64_t>> slots;
      for (int64_t i = 0; i < kResidentWorkgroups; i++) slots.push(0);
      int64_t end = 0;
      for (int h = 0; h < split_heads; h++)          // the grid runs the list once per head, head-major
        for (const Scored& it : v) {
          int64_t t0 = slots.top();
          slots.pop();
          slots.push(t0 + it.cost);
          end = std::max(end, t0 + it.cost);
        }
      return (double)end;
    };
    auto cut_at = [&](int64_t limit, HostItems* out) {
      std::vector<Scored> cut;
      out->reduce.clear();
      out->n_pslots = 0;
      for (const Scored& it : sc) {
        const int32_t n_ent = it.w.e1 - it.w.e0;
        int64_t want = (it.cost + limit - 1) / limit;
        const int32_t n_parts = (int32_t)std::min<int64_t>(std::min<int64_t>(want, n_ent), kMaxParts);
        if (n_parts <= 1) { cut.push_back(it); continue; }
        const WorkItem& w = it.w;
        int64_t r0 = blk_start[hg->unit_blk[w.unit]] + (int64_t)w.tile * tile_rows;
        int64_t r1 = std::min<int64_t>(r0 + tile_rows, blk_start[hg->unit_blk[w.unit]] + blk_len[hg->unit_blk[w.unit]]);
        ecost.assign(n_ent, 0);
        for (int32_t e = w.e0; e < w.e1; e++)
          ecost[e - w.e0] = tile_cost(hg->ent_kind[e], r0, r1, hg->ent_start[e], hg->ent_start[e] + hg->ent_len[e], gid == 2);
        // contiguous chunks of table rows of about cost / n_parts each, every chunk non-empty
        out->reduce.push_back({w.unit, w.tile, out->n_pslots, n_parts});
        int32_t e = w.e0;
        int64_t done = 0;
        for (int32_t p = 0; p < n_parts; p++) {
          const int32_t left_parts = n_parts - p - 1;
          const int64_t goal = it.cost * (p + 1) / n_parts;
          int32_t e_hi = e + 1;
          int64_t c = ecost[e - w.e0];
          while (e_hi < w.e1 - left_parts && done + c < goal) { c += ecost[e_hi - w.e0]; e_hi++; }
          if (p == n_parts - 1) { while (e_hi < w.e1) { c += ecost[e_hi - w.e0]; e_hi++; } }
          cut.push_back({{w.unit, w.tile, e, e_hi, out->n_pslots + p, w.blk_start, w.blk_len, w.moff}, c});
          done += c;
          e = e_hi;
        }
        out->n_pslots += n_parts;
      }
      return cut;
    };
    if (total > 0 && finish_time(sc) > 1.05 * share) {
      std::vector<Scored> best;
      for (int d = 1; d <= 4; d *= 2) {
        best = cut_at(std::max<int64_t>(1, (int64_t)(share / d)), &hi);
        if (finish_time(best) <= 1.05 * std::max(share, 1.0)) break;
      }
      sc.swap(best);
    }
  }
  std::stable_sort(sc.begin(), sc.end(), [](const Scored& a, const Scored& b) { return a.cost > b.cost; });
  if (gid == 2 && split_heads > 0 && !sc.empty()) {
    // dK/dV: sequence by sequence (the costliest sequence first, longest item first inside it) when that balances as
    // well as strict longest-first does.  The key tiles of one sequence that run at the same time stream the same
    // Q / dO rows (each walks its query tiles from the last one down), so their XCD's L2 serves those rows once:
    // 13.9 -> 7.5 GB fetched per launch on the 65 536-token causal batch, and the step gains 1 % -- not in this kernel's
    // own time but in the clock the chip grants its neighbours, its power being what is limited.  A batch of equal
    // sequences balances badly in this order (every round of workgroups mixes long and short items), which the
    // launch played through as list scheduling shows; it keeps strict longest-first.  (Longest-first by four or eight
    // classes of length with sequences grouped inside a class was in between on traffic and 0.8 % slower; the same
    // order for the forward and dQ lists changed nothing measurable.)
    auto play = [&](const std::vector<Scored>& v) {
      std::priority_queue<int64_t, std::vector<int64_t>, std::greater<int64_t>> slots;
      for (int64_t i = 0; i < kResidentWorkgroups; i++) slots.push(0);
      int64_t end = 0;
      for (int h = 0; h < split_heads; h++)          // the grid runs the list once per head, head-major
        for (const Scored& it : v) {
          const int64_t t0 = slots.top();
          slots.pop();
          slots.push(t0 + it.cost);
          end = std::max(end, t0 + it.cost);
        }
      return end;
    };
    std::vector<int64_t> seq_cost(n_seq, 0);
    for (const Scored& x : sc) seq_cost[blk_seq[hg->unit_blk[x.w.unit]]] += x.cost;
    std::vector<Scored> by_seq(sc);
    std::stable_sort(by_seq.begin(), by_seq.end(), [&](const Scored& a, const Scored& b) {
      const int32_t sa = blk_seq[hg->unit_blk[a.w.unit]], sb = blk_seq[hg->unit_blk[b.w.unit]];
      if (sa == sb) return false;
      return seq_cost[sa] != seq_cost[sb] ? seq_cost[sa] > seq_cost[sb] : sa < sb;
    });
    if ((double)play(by_seq) <= 1.01 * (double)play(sc)) sc.swap(by_seq);
  }
  hi.n_seg = n_seg;
  for (int s = 0; s <= 8; s++) hi.seg[s] = (int32_t)sc.size();
  hi.seg[0] = 0;
  if (n_seg > 1 && !sc.empty()) {
    // With fewer KV heads than a multiple of 8 an XCD takes a part of a head's list, and contiguous parts of a list
    // that runs from the longest item to the shortest are anything but equal.  The list is dealt into n_seg segments
    // of about equal cost, the order inside a segment kept: first the sequences that are at most half a segment, whole
    // (their tiles read the same K / V or Q / dO rows and are better off in one XCD's L2), costliest first, then the
    // items of the larger sequences one by one, which level the segments out; each goes to the segment that holds
    // least so far.
    std::vector<int64_t> seq_cost(n_seq, 0);
    int64_t sum = 0;
    for (const Scored& x : sc) { seq_cost[blk_seq[hg->unit_blk[x.w.unit]]] += x.cost; sum += x.cost; }
    const int64_t half = std::max<int64_t>(1, sum / n_seg / 2);
    std::vector<int64_t> load(n_seg, 0);
    std::vector<int32_t> bin(sc.size(), 0), seq_bin(n_seq, -1);
    auto lightest = [&]() { return (int32_t)(std::min_element(load.begin(), load.end()) - load.begin()); };
    std::vector<int32_t> small;
    for (int32_t q = 0; q < n_seq; q++)
      if (seq_cost[q] > 0 && seq_cost[q] <= half) small.push_back(q);
    std::stable_sort(small.begin(), small.end(), [&](int32_t a, int32_t b) { return seq_cost[a] > seq_cost[b]; });
    for (int32_t q : small) { seq_bin[q] = lightest(); load[seq_bin[q]] += seq_cost[q]; }
    std::vector<size_t> big;
    for (size_t i = 0; i < sc.size(); i++)
      if (seq_cost[blk_seq[hg->unit_blk[sc[i].w.unit]]] > half) big.push_back(i);
    std::stable_sort(big.begin(), big.end(), [&](size_t a, size_t b) { return sc[a].cost > sc[b].cost; });
    for (size_t i : big) { bin[i] = lightest(); load[bin[i]] += sc[i].cost; }
    for (size_t i = 0; i < sc.size(); i++) {
      const int32_t q = blk_seq[hg->unit_blk[sc[i].w.unit]];
      if (seq_bin[q] >= 0) bin[i] = seq_bin[q];
    }
    std::vector<Scored> dealt;
    dealt.reserve(sc.size());
    for (int s = 0; s < n_seg; s++) {
      for (size_t i = 0; i < sc.size(); i++)
        if (bin[i] == s) dealt.push_back(sc[i]);
      hi.seg[s + 1] = (int32_t)dealt.size();
    }
    sc.swap(dealt);
  }
  hi.items.resize(sc.size());
  for (size_t i = 0; i < sc.size(); i++) hi.items[i] = sc[i].w;
  return h_items.emplace(key, std::move(hi)).first->second;
}

template <class T>
static dcp_status_t upload(const std::vector<T>& v, T** dev, hipStream_t stream) {
  *dev = nullptr;
  if (v.empty()) return DCP_OK;
  DCP_HIP_TRY(hipMalloc((void**)dev, v.size() * sizeof(T)));
  hipError_t e = hipMemcpyAsync(*dev, v.data(), v.size() * sizeof(T), hipMemcpyHostToDevice, stream);
  if (e == hipSuccess) e = hipStreamSynchronize(stream);
  if (e != hipSuccess) {
    (void)hipFree(*dev);
    *dev = nullptr;
    return fail(DCP_ERR_HIP, std::string("work list upload: ") + hipGetErrorString(e));
  }
  return DCP_OK;
}

dcp_status_t dcp_plan::group_for(int gid, int tile_rows, hipStream_t stream, DevGroup* out, int split_heads, bool may_alloc,
                                 int n_seg) {
  dcp_status_t st = ensure_device(stream, may_alloc);
  if (st != DCP_OK) return st;
  const HostItems& hi = host_items(gid, tile_rows, split_heads, n_seg);
  std::lock_guard<std::mutex> lock(mu);
  DevGroup dg = gid == 0 ? d_fwd : (gid == 1 ? d_bwdq : d_bwdkv);
  const ItemKey key(gid, tile_rows, split_heads, n_seg);
  auto it = items.find(key);
  if (it == items.end()) {
    if (!may_alloc) return fail(DCP_ERR_INVALID_ARG, "the plan has no work list for this shape yet: call dcp_plan_prepare first");
    DevItems di;
    di.n_items = (int32_t)hi.items.size();
    di.n_reduce = (int32_t)hi.reduce.size();
    if ((st = upload(hi.items, &di.items, stream)) != DCP_OK) return st;
    if ((st = upload(hi.reduce, &di.reduce, stream)) != DCP_OK) {
      if (di.items) (void)hipFree(di.items);
      return st;
    }
    it = items.emplace(key, di).first;
  }
  dg.items = it->second.items;
  dg.n_items = it->second.n_items;
  dg.reduce = it->second.reduce;
  dg.n_reduce = it->second.n_reduce;
  dg.n_seg = hi.n_seg;
  for (int k = 0; k <= 8; k++) dg.seg[k] = hi.seg[k];
  *out = dg;
  return DCP_OK;
}
