// Drives the host code of libdcp_attn.so (plan.cpp, api.hip, executor.hip) through its C ABI on the CPU, in a build
// with AddressSanitizer and UndefinedBehaviorSanitizer, against the stand-in device of fake_device.cpp.  Test
// infrastructure: seeded random batches, tables (valid ones, and ones damaged in every way dcp_plan_create must refuse),
// block buffers, partial slots, copy lists and instruction lists; every entry point is called as the GPU tests call
// it, with host buffers of exactly the documented sizes.  Prints "host-asan ok" and exits 0 when nothing is reported.
#include <algorithm>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <random>
#include <vector>

#include "dcp.h"

namespace dcp {
extern int64_t g_fake_kv_rows;
extern int32_t g_fake_n_slots;
long fake_rows_walked();
}

static int g_fail = 0;
#define EXPECT(cond)                                                                         \
  do {                                                                                       \
    if (!(cond)) { std::printf("EXPECT failed, line %d: %s (%s)\n", __LINE__, #cond, dcp_last_error()); g_fail++; } \
  } while (0)

typedef std::mt19937_64 Rng;
static int rnd(Rng& r, int lo, int hi) { return lo + (int)(r() % (uint64_t)(hi - lo + 1)); }

// per-token ranges of a random mask family: causal, sliding window, sink + window, or two arbitrary ranges
static std::vector<int32_t> make_ranges(Rng& r, const std::vector<int32_t>& cu, int family) {
  const int T = cu.back();
  std::vector<int32_t> g((size_t)T * 4, 0);
  const int window = rnd(r, 1, 200), sink = rnd(r, 0, 40);
  for (size_t s = 0; s + 1 < cu.size(); s++)
    for (int i = cu[s]; i < cu[s + 1]; i++) {
      int32_t* x = &g[4 * (size_t)i];
      if (family == 0) { x[0] = cu[s]; x[1] = i + 1; }
      else if (family == 1) { x[0] = std::max(cu[s], i - window + 1); x[1] = i + 1; }
      else if (family == 2) { const int lo = std::max(cu[s], i - window + 1); x[0] = cu[s]; x[1] = std::min(cu[s] + sink, lo); x[2] = lo; x[3] = i + 1; }
      else { x[0] = rnd(r, cu[s], cu[s + 1]); x[1] = rnd(r, cu[s], cu[s + 1]); x[2] = rnd(r, cu[s], cu[s + 1]); x[3] = rnd(r, cu[s], cu[s + 1]); }
    }
  return g;
}

static void one_case(Rng& r, int iter) {
  const int n_seq = rnd(r, 1, 5), B = (iter % 7 == 0) ? 1 : rnd(r, 1, 300);
  std::vector<int32_t> cu(1, 0);
  for (int s = 0; s < n_seq; s++) cu.push_back(cu.back() + rnd(r, 1, B == 1 ? 30 : 700));
  const int T = cu.back(), family = rnd(r, 0, 3);
  const std::vector<int32_t> ranges = make_ranges(r, cu, family);
  int64_t n = 0;
  EXPECT(dcp_build_block_table(cu.data(), n_seq, B, ranges.data(), nullptr, 0, &n) == DCP_OK);
  std::vector<int32_t> table((size_t)n * 3 + 3);
  EXPECT(dcp_build_block_table(cu.data(), n_seq, B, ranges.data(), table.data(), n, &n) == DCP_OK);
  if (n > 1) { int64_t m = 0; EXPECT(dcp_build_block_table(cu.data(), n_seq, B, ranges.data(), table.data(), n - 1, &m) == DCP_ERR_INVALID_ARG && m == n); }
  table.resize((size_t)n * 3);
  std::vector<int64_t> pairs((size_t)n + 1);
  EXPECT(dcp_count_pairs(cu.data(), n_seq, B, table.data(), n, ranges.data(), pairs.data()) == DCP_OK);
  { // the WINDOW route of the same generator
    int64_t nw = 0;
    const int win = rnd(r, 1, 300), sink = rnd(r, 0, 50);
    EXPECT(dcp_build_block_table_window(cu.data(), n_seq, B, win, sink, nullptr, 0, &nw) == DCP_OK);
    std::vector<int32_t> tw((size_t)nw * 3 + 3);
    EXPECT(dcp_build_block_table_window(cu.data(), n_seq, B, win, sink, tw.data(), nw, &nw) == DCP_OK);
    std::vector<int64_t> pw((size_t)nw + 1);
    EXPECT(dcp_count_pairs_window(cu.data(), n_seq, B, tw.data(), nw, win, sink, pw.data()) == DCP_OK);
    EXPECT(dcp_build_block_table_window(cu.data(), n_seq, B, 0, sink, nullptr, 0, &nw) == DCP_ERR_INVALID_ARG);
  }
  int n_blocks = 0;
  for (int s = 0; s < n_seq; s++) n_blocks += (cu[s + 1] - cu[s] + B - 1) / B;

  // damaged tables must be refused, not read out of bounds
  if (n > 0) {
    dcp_plan_t* bad = nullptr;
    std::vector<int32_t> t2 = table;
    t2[3 * rnd(r, 0, (int)n - 1) + rnd(r, 0, 1)] = (iter & 1) ? n_blocks + rnd(r, 0, 5) : -1 - rnd(r, 0, 5);
    EXPECT(dcp_plan_create(&bad, cu.data(), n_seq, B, t2.data(), n, nullptr, 0) == DCP_ERR_BAD_TABLE && !bad);
    t2 = table; t2[3 * rnd(r, 0, (int)n - 1) + 2] = 5 + rnd(r, 0, 100);
    EXPECT(dcp_plan_create(&bad, cu.data(), n_seq, B, t2.data(), n, nullptr, 0) == DCP_ERR_BAD_TABLE && !bad);
    t2 = table; t2.insert(t2.end(), table.begin(), table.begin() + 3);   // a duplicate row
    if (table[2] != DCP_MASK_SKIP) EXPECT(dcp_plan_create(&bad, cu.data(), n_seq, B, t2.data(), n + 1, nullptr, 0) == DCP_ERR_BAD_TABLE && !bad);
    if (n_seq > 1) {   // a row that joins blocks of two sequences
      t2 = table; t2[0] = 0; t2[1] = n_blocks - 1;
      EXPECT(dcp_plan_create(&bad, cu.data(), n_seq, B, t2.data(), n, nullptr, 0) == DCP_ERR_BAD_TABLE && !bad);
    }
    std::vector<int32_t> cu2 = cu; cu2[rnd(r, 1, n_seq)] = cu2[0];
    EXPECT(dcp_plan_create(&bad, cu2.data(), n_seq, B, table.data(), n, nullptr, 0) == DCP_ERR_BAD_CU_SEQLENS && !bad);
  }

  // a random subset of the rows (a device's share), optionally with partial slots, optionally in block buffers
  std::vector<int32_t> sub;
  for (int64_t e = 0; e < n; e++)
    if (rnd(r, 0, 3) != 0) sub.insert(sub.end(), table.begin() + 3 * e, table.begin() + 3 * e + 3);
  const int64_t ns = (int64_t)sub.size() / 3;
  const bool slots = rnd(r, 0, 1) == 1 && ns > 0;   // (an empty share has no row to give a slot to)
  std::vector<int32_t> out_slot;
  int32_t n_slots = 0;
  if (slots) {   // (division, q_blk) -> slot
    const int n_div = rnd(r, 1, 4);
    std::vector<int32_t> id((size_t)n_div * n_blocks, -1);
    for (int64_t e = 0; e < ns; e++) {
      int32_t& s = id[(size_t)rnd(r, 0, n_div - 1) * n_blocks + sub[3 * e]];
      if (s < 0) s = n_slots++;
      out_slot.push_back(s);
    }
    n_slots += rnd(r, 0, 2);   // unused slots are legal
  }
  dcp_plan_t* plan = nullptr;
  EXPECT(dcp_plan_create(&plan, cu.data(), n_seq, B, sub.data(), ns, slots ? out_slot.data() : nullptr, n_slots) == DCP_OK && plan);
  if (!plan) return;
  if (slots && ns > 1 && sub[0] != sub[3 * (ns - 1)]) {   // one slot for two q blocks
    std::vector<int32_t> os2 = out_slot; os2[ns - 1] = os2[0];
    dcp_plan_t* bad = nullptr;
    EXPECT(dcp_plan_create(&bad, cu.data(), n_seq, B, sub.data(), ns, os2.data(), n_slots) == DCP_ERR_BAD_TABLE && !bad);
  }
  int64_t q_rows = T, kv_rows = T;
  if (rnd(r, 0, 2) == 0) {   // block buffers: a permutation of slots, a few spare ones
    const int nq = n_blocks + rnd(r, 0, 2), nk = n_blocks + rnd(r, 0, 2);
    std::vector<int32_t> qs(nq), ks(nk);
    for (int i = 0; i < nq; i++) qs[i] = i;
    for (int i = 0; i < nk; i++) ks[i] = i;
    std::shuffle(qs.begin(), qs.end(), r);
    std::shuffle(ks.begin(), ks.end(), r);
    std::vector<int32_t> bad_q(qs.begin(), qs.begin() + n_blocks);
    if (n_blocks > 1) { bad_q[1] = bad_q[0]; EXPECT(dcp_plan_set_block_buffers(plan, bad_q.data(), nq, ks.data(), nk) == DCP_ERR_BAD_TABLE); }
    EXPECT(dcp_plan_set_block_buffers(plan, qs.data(), nq, ks.data(), nk) == DCP_OK);
    q_rows = (int64_t)nq * B; kv_rows = (int64_t)nk * B;
  }
  for (int which = 0; which <= 11; which++) {
    int64_t len = 0;
    EXPECT(dcp_plan_export(plan, (dcp_export_t)which, nullptr, 0, &len) == DCP_OK);
    std::vector<int32_t> buf((size_t)len + 1);
    EXPECT(dcp_plan_export(plan, (dcp_export_t)which, buf.data(), len, &len) == DCP_OK);
  }
  const bool mfma = rnd(r, 0, 1) == 1;
  const int hkv = rnd(r, 1, 3), hq = hkv * rnd(r, 1, 4), d = mfma ? 128 : 64, dtype = mfma ? DCP_BF16 : DCP_F32;
  { int64_t ni = 0; EXPECT(dcp_plan_export_dkv_items(plan, hkv, nullptr, 0, &ni) == DCP_OK);
    std::vector<int32_t> it((size_t)ni * 5 + 1); EXPECT(dcp_plan_export_dkv_items(plan, hkv, it.data(), ni, &ni) == DCP_OK); }

  // launches against the stand-in device: buffers of exactly the documented sizes
  dcp::g_fake_kv_rows = kv_rows; dcp::g_fake_n_slots = n_slots;
  const size_t es = dtype == DCP_BF16 ? 2 : 4;
  std::vector<char> q((size_t)q_rows * hq * d * es + 16), kv((size_t)kv_rows * hkv * d * es + 16);
  std::vector<float> lse((size_t)hq * q_rows + 1);
  std::vector<char> o_part((size_t)n_slots * B * hq * d * es + 16);
  std::vector<float> lse_part((size_t)n_slots * hq * B + 1);
  dcp_tensors_t t{};
  t.hq = hq; t.hkv = hkv; t.d = d; t.dtype = dtype; t.impl = DCP_IMPL_AUTO; t.softmax_scale = 0.1f;
  t.q = q.data(); t.k = kv.data(); t.v = kv.data(); t.dout = q.data(); t.dq = q.data(); t.dk = kv.data(); t.dv = kv.data();
  t.q_stride_t = t.do_stride_t = t.dq_stride_t = t.o_stride_t = (int64_t)hq * d; t.q_stride_h = t.do_stride_h = t.dq_stride_h = t.o_stride_h = d;
  t.k_stride_t = t.v_stride_t = t.dk_stride_t = t.dv_stride_t = (int64_t)hkv * d; t.k_stride_h = t.v_stride_h = t.dk_stride_h = t.dv_stride_h = d;
  t.attn_ranges = ranges.data();
  t.out = slots ? (void*)o_part.data() : (void*)q.data();
  t.lse = slots ? lse_part.data() : lse.data();
  if (rnd(r, 0, 1)) EXPECT(dcp_plan_prepare(plan, hq, hkv, d, dtype, DCP_IMPL_AUTO, nullptr) == DCP_OK);
  EXPECT(dcp_block_attn_fwd(plan, &t, nullptr) == DCP_OK);
  if (slots) EXPECT(dcp_merge_partials(plan, o_part.data(), lse_part.data(), q.data(), (int64_t)hq * d, d, lse.data(), hq, d, dtype, nullptr) == DCP_OK);
  t.out = q.data(); t.lse = lse.data();
  const size_t wsb = dcp_bwd_workspace_bytes(plan, hq, hkv, d, dtype);
  void* ws = nullptr;
  EXPECT(posix_memalign(&ws, 256, wsb ? wsb : 256) == 0);
  EXPECT(dcp_block_attn_bwd(plan, &t, ws, wsb, nullptr) == DCP_OK);
  if (wsb > 256) EXPECT(dcp_block_attn_bwd(plan, &t, ws, wsb - 1, nullptr) == DCP_ERR_WORKSPACE);
  EXPECT(dcp_bwd_delta(&t, q_rows, (float*)ws, nullptr) == DCP_OK || wsb < (size_t)hq * q_rows * 4);

  // Blockwise Copy: block-wise moves into the Q-type buffer; lists that leave their buffers or collide are refused
  {
    std::vector<int32_t> ent;
    int64_t row = 0;
    for (int b = 0; b < n_blocks && row + B <= q_rows; b++) { const int len = rnd(r, 0, B); ent.insert(ent.end(), {rnd(r, 0, (int)(q_rows - len)), (int32_t)row, len}); row += len; }
    dcp_copy_list_t* cl = nullptr;
    EXPECT(dcp_copy_list_create(&cl, ent.data(), (int64_t)ent.size() / 3, q_rows, q_rows) == DCP_OK && cl);
    std::vector<char> dst(q.size());
    EXPECT(dcp_blockwise_copy(cl, q.data(), (int64_t)hq * d * es, dst.data(), (int64_t)hq * d * es, (int64_t)hq * d * es, nullptr) == DCP_OK);
    dcp_copy_list_t* bad = nullptr;
    std::vector<int32_t> e2 = {0, (int32_t)q_rows - 1, 2};
    EXPECT(dcp_copy_list_create(&bad, e2.data(), 1, q_rows, q_rows) == DCP_ERR_BAD_TABLE && !bad);
    e2 = {0, 0, 2, 1, 1, 1};
    if (q_rows >= 2) EXPECT(dcp_copy_list_create(&bad, e2.data(), 2, q_rows, q_rows) == DCP_ERR_BAD_TABLE && !bad);
    // an execution plan over what this case has: copy, forward, (merge), backward, a gradient sum, one transfer
    std::vector<dcp_instr_t> prog(7);
    std::memset(prog.data(), 0, prog.size() * sizeof(dcp_instr_t));
    prog[0].op = DCP_OP_COMM_LAUNCH; prog[0].comm_id = 0; prog[0].copy_list = cl; prog[0].src = q.data(); prog[0].dst = dst.data();
    prog[0].src_row_stride = prog[0].dst_row_stride = prog[0].row_bytes = (int64_t)hq * d * es;
    prog[1] = prog[0]; prog[1].op = DCP_OP_COPY;
    prog[2].op = DCP_OP_ATTN_FWD; prog[2].plan = plan; prog[2].tensors = t;
    prog[2].tensors.out = slots ? (void*)o_part.data() : (void*)q.data(); prog[2].tensors.lse = slots ? lse_part.data() : lse.data();
    prog[3].op = DCP_OP_COMM_WAIT; prog[3].comm_id = 0;
    prog[4].op = slots ? DCP_OP_MERGE : DCP_OP_COMM_WAIT; prog[4].plan = plan; prog[4].o_part = o_part.data(); prog[4].lse_part = lse_part.data(); prog[4].tensors = t;
    prog[5].op = DCP_OP_ATTN_BWD; prog[5].plan = plan; prog[5].tensors = t; prog[5].workspace = ws; prog[5].workspace_bytes = wsb;
    prog[6].op = DCP_OP_SUM; prog[6].n_parts = 2; prog[6].parts[0] = q.data(); prog[6].parts[1] = dst.data(); prog[6].dst = dst.data();
    prog[6].parts_dtype = prog[6].dst_dtype = dtype; prog[6].n_elems = (int64_t)q_rows * hq * d;
    dcp_program_t* pg = nullptr;
    if (!slots) {   // Comm.Wait twice for one transfer is refused
      EXPECT(dcp_program_create(&pg, prog.data(), 7) == DCP_ERR_INVALID_ARG && !pg);
      prog[4] = prog[1];
    }
    EXPECT(dcp_program_create(&pg, prog.data(), 7) == DCP_OK && pg);
    int s1 = 0, s2 = 0;   // any two distinct handles serve as streams here
    EXPECT(dcp_program_run(pg, &s1, &s1) == DCP_ERR_INVALID_ARG);
    EXPECT(dcp_program_run(pg, &s1, &s2) == DCP_OK);
    EXPECT(dcp_program_run(pg, &s1, &s2) == DCP_OK);
    EXPECT(dcp_program_destroy(pg) == DCP_OK);
    EXPECT(dcp_copy_list_destroy(cl) == DCP_OK);
  }
  std::free(ws);

  // communication volume of a random placement
  {
    const int n_dev = rnd(r, 1, 5);
    std::vector<int32_t> bd(n_blocks), cd((size_t)ns + 1);
    for (auto& x : bd) x = rnd(r, 0, n_dev - 1);
    for (auto& x : cd) x = rnd(r, 0, n_dev - 1);
    int64_t pw = 0, cn = 0, ne = 0;
    std::vector<int64_t> send(n_dev), recv(n_dev);
    EXPECT(dcp_comm_volume(cu.data(), n_seq, B, sub.data(), ns, bd.data(), cd.data(), n_dev, 8, 4, 8, &pw, &cn, &ne, send.data(), recv.data()) == DCP_OK);
    EXPECT(cn <= pw);
    if (ns > 0) { cd[0] = n_dev; EXPECT(dcp_comm_volume(cu.data(), n_seq, B, sub.data(), ns, bd.data(), cd.data(), n_dev, 8, 4, 8, &pw, &cn, &ne, nullptr, nullptr) == DCP_ERR_BAD_TABLE); }
  }
  EXPECT(dcp_plan_destroy(plan) == DCP_OK);
}

int main(int argc, char** argv) {
  const int iters = argc > 1 ? std::atoi(argv[1]) : 150;
  Rng r(20251028);
  for (int i = 0; i < iters && g_fail == 0; i++) one_case(r, i);
  // the empty plan and NULL arguments
  dcp_plan_t* plan = nullptr;
  int32_t cu0 = 0;
  EXPECT(dcp_plan_create(&plan, &cu0, 0, 16, nullptr, 0, nullptr, 0) == DCP_OK && plan);
  EXPECT(dcp_plan_destroy(plan) == DCP_OK);
  EXPECT(dcp_plan_create(nullptr, &cu0, 0, 16, nullptr, 0, nullptr, 0) == DCP_ERR_INVALID_ARG);
  EXPECT(dcp_block_attn_fwd(nullptr, nullptr, nullptr) == DCP_ERR_INVALID_ARG);
  std::printf("table rows walked by the stand-in kernels: %ld\n", dcp::fake_rows_walked());
  if (g_fail == 0) std::printf("host-asan ok\n");
  return g_fail ? 1 : 0;
}
