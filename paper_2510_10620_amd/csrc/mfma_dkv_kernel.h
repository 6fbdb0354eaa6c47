// Device code of the dK/dV kernel (see kernels_mfma_dkv.hip), in a header because its two variants are built in two
// translation units: the backend's instruction-scheduling strategy is a per-file flag and each variant has its own best.
#pragma once
#include "mfma_common.h"

namespace dcp {


static constexpr float kLog2e = 1.44269504088896340736f;

// ------------------------------------------------------------------------------------ dK / dV
// LDS stage of the dK/dV kernel: a 64-query tile of Q and dO plus the rows' LSE, delta and ranges.
static constexpr int kStageLse = 2 * kTileBytes;
static constexpr int kStageDelta = kStageLse + 256;
static constexpr int kStageRanges = kStageDelta + 256;
static constexpr int kStageBounds = kStageRanges + 1024;   // range bounds of the tile's two 32-row halves (2 x 8 ints; 1 KB reserved)
static constexpr int kStageBytes = kStageBounds + 1024;

// Walks (table row, query head of the group, 64-query tile) for one KV tile.
template <bool RANGES>
struct QIter {
  const int4* rec;       // per table row: {first query, length, mask kind, memory offset of the Q block}, {first 32-row tile, ..}
  const int4* qbounds;   // range-bound summaries per 32-row tile, or null
  int e, e_end, hh, G, jt, n_t, jt0;
  int q0, q1, kind;
  int moff;  // the Q block's rows sit at (packed index + moff) in the Q-type buffers
  int t32;   // index of the Q block's first 32-row tile in qbounds
  int qs;    // first query of the current tile
  // [e0, e1): the table rows of the unit this workgroup covers.  They, and the query tiles of each, are walked from
  // the last to the first: the key tiles of one sequence that start together then stream the same Q / dO rows at
  // the same time (each is a prefix of one common order) and share them in the L2; walked forwards, each tile would
  // start at its own diagonal, two steps behind its neighbour, which is as far apart as the L2 is large.
  __device__ QIter(const DevGroup& g, int e0, int e1, int G_, const int32_t* qb)
      : rec((const int4*)g.ent_rec), qbounds((const int4*)qb) {
    e = e1; e_end = e0; hh = G_ - 1; G = G_; jt = 0; n_t = 0; jt0 = 0; q0 = q1 = kind = 0; moff = 0; t32 = 0; qs = 0;
  }
  // Which of the (at most 64) 64-query tiles of the current RANGES row may see a key of [k_lo, k_end): lane l merges
  // the bounds of the two 32-row halves of tile l.  Returns the ballot (wave-uniform).
  __device__ unsigned long long tiles_that_see(int k_lo, int k_end) const {
    const int tile = threadIdx.x & 63;
    bool see = false;
    if (tile < n_t) {
      const int n32 = (q1 - q0 + 31) >> 5;
      const int4* p = qbounds + (int64_t)(t32 + 2 * tile) * 2;
      int4 a = p[0], b = p[1];
      if (2 * tile + 1 < n32) {
        const int4 c = p[2], d = p[3];
        a.x = min(a.x, c.x); a.w = max(a.w, c.w); b.x = min(b.x, d.x); b.w = max(b.w, d.w);
      }
      see = (k_lo < a.w && k_end > a.x) || (k_lo < b.w && k_end > b.x);   // x = smallest start, w = largest end
    }
    return __ballot(see);
  }
  // [k_lo, k_end): the keys of the workgroup's tile.  Under CAUSAL, query tiles that end before k_lo see nothing;
  // under RANGES, the walk is narrowed to the span between the first and the last tile whose rows' ranges reach the
  // keys (tiles inside the span that see nothing are left to the per-sub-tile test).
  __device__ bool next(int k_lo, int k_end) {
    for (;;) {
      jt--;
      if (jt < jt0) {
        hh++;
        if (hh >= G) {
          e--;
          if (e < e_end) return false;
          hh = 0;
          const int4 r = rec[2 * e];
          q0 = uni(r.x); q1 = q0 + uni(r.y); kind = uni(r.z); moff = uni(r.w); t32 = uni(rec[2 * e + 1].x);
          n_t = (q1 - q0 + kTN - 1) / kTN;
          jt0 = kind == 1 ? max(0, (k_lo - q0) / kTN) : 0;
          if (RANGES && kind == 2 && qbounds && n_t <= 64) {
            const unsigned long long m = tiles_that_see(k_lo, k_end);
            if (m == 0) { n_t = 0; }
            else { jt0 = __builtin_ctzll(m); n_t = 64 - __builtin_clzll(m); }
          }
        }
        jt = n_t;   // one past the last tile of the row
        continue;
      }
      qs = q0 + jt * kTN;
      return true;
    }
  }
};

// Fragment addresses from two registers: the swizzle makes every other address an XOR of these with a constant.
struct FragAddr2 {
  int rm0, tr00;
  __device__ __forceinline__ void init(int lane) {
    const int li = lane & 31, lh = lane >> 5;
    rm0 = tile_off(li, lh);
    const int j = lane & 15, blk = lane >> 4, h = blk >> 1;
    const int col = 16 * (blk & 1) + 4 * (j & 3);
    tr00 = tile_off(4 * h + (j >> 2), col >> 3) + (col & 7) * 2;
  }
};
__device__ __forceinline__ bf16x8 frag_rm2(const char* tile, const FragAddr2& fa, int row0, int ks) {
  return as_frag(*(const uint4*)(tile + row0 * kRowBytes + (fa.rm0 ^ (ks << 5))));
}
__device__ __forceinline__ bf16x8 frag_tr2(const char* tile, const FragAddr2& fa, int row0, int dt) {
  typedef __attribute__((address_space(3))) s16x4* lds_p;
  const int a0 = fa.tr00 ^ (dt << 6);
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_p)(tile + row0 * kRowBytes + a0));
  const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_p)(tile + row0 * kRowBytes + (a0 ^ 0x820)));
  s16x8 v;
  v[0] = lo[0]; v[1] = lo[1]; v[2] = lo[2]; v[3] = lo[3]; v[4] = hi[0]; v[5] = hi[1]; v[6] = hi[2]; v[7] = hi[3];
  return __builtin_bit_cast(bf16x8, v);
}

// Bits [0, x - base) of a 32-key window that starts at key `base`: the keys of the window below key x.
__device__ __forceinline__ uint32_t keys_below(int x, int base) {
  const int n = min(max(x, base), base + 32) - base;   // 0..32, no overflow for any x
  return n >= 32 ? 0xffffffffu : (1u << n) - 1u;
}

// What a wave keeps for the whole kernel: its 32 keys' K and V fragments and the dK^T / dV^T accumulators (192
// registers).  Two workgroups share a CU (two waves per SIMD), so everything else has to fit in 64.
struct DkvState {
  bf16x8 kf[8], vf[8];
  f32x16 dk[4], dv[4];
};

// One 32-query sub-tile against the wave's 32 keys.  Operands are read where they are used: the SIMD's other wave
// hides the latency.  Everything that depends on the lane alone (fragment addresses, the key index, the rows'
// LSE / delta addresses) is recomputed in every call from an opaque copy of the lane number, or the compiler
// hoists two dozen loop-invariant registers out of the query loop and spills.
template <bool RANGES>
__device__ __forceinline__ void dkv_subtile(DkvState& st, const char* stage, int qt, int qs32, int q1, int kind,
                                            int wk_lo, int k_end, float c_log2, bool MASK) {
  int lane = threadIdx.x & 63;
  asm volatile("" : "+v"(lane));
  const int lh = lane >> 5;
  const int kj = wk_lo + (lane & 31);   // may lie past k_end: masked, never stored
  const char* q_lds = stage;
  const char* do_lds = stage + kTileBytes;
  FragAddr2 fa;
  fa.init(lane);
  // dP starts from -delta of its query rows (element 4a + b of the tile is query row 8a + 4 lh + b), so that the
  // accumulator ends as dP - delta and dS is one multiplication
  const float* lse_lds = (const float*)(stage + kStageLse) + 32 * qt + 4 * lh;
  const float* dl_lds = (const float*)(stage + kStageDelta) + 32 * qt + 4 * lh;
  f32x16 s, dp;
#pragma unroll
  for (int a = 0; a < 4; a++) {
    const float4 d4 = *(const float4*)(dl_lds + 8 * a);
    dp[4 * a] = d4.x; dp[4 * a + 1] = d4.y; dp[4 * a + 2] = d4.z; dp[4 * a + 3] = d4.w;
  }
#pragma unroll
  for (int r = 0; r < 16; r++) s[r] = 0.f;
  if constexpr (!RANGES) {
    // operands one k-step ahead of the MFMAs that use them (8 more registers in flight; the kernel for tables with
    // per-token ranges has no registers left for it here, where s and dp are live: it spills and gets slower); the
    // fences keep the requests in front of the MFMAs of the step before
    bf16x8 qa = frag_rm2(q_lds, fa, 32 * qt, 0), da = frag_rm2(do_lds, fa, 32 * qt, 0);
#pragma unroll
    for (int ksd = 0; ksd < 8; ksd++) {
      bf16x8 qn = qa, dn = da;
      if (ksd < 7) { qn = frag_rm2(q_lds, fa, 32 * qt, ksd + 1); dn = frag_rm2(do_lds, fa, 32 * qt, ksd + 1); }
      __builtin_amdgcn_sched_barrier(0);
      s = mfma(qa, st.kf[ksd], s);
      dp = mfma(da, st.vf[ksd], dp);
      qa = qn; da = dn;
      __builtin_amdgcn_sched_barrier(0);
    }
  } else {
#pragma unroll
    for (int ksd = 0; ksd < 8; ksd++) {
      s = mfma(frag_rm2(q_lds, fa, 32 * qt, ksd), st.kf[ksd], s);
      dp = mfma(frag_rm2(do_lds, fa, 32 * qt, ksd), st.vf[ksd], dp);
    }
  }
  if (MASK) {
    // Lane l works out, once, which of the wave's 32 keys query row (l & 31) of the sub-tile sees, as a bit mask
    // (bit j = key wk_lo + j).  Element r = 4a + b of the score tile is (query row 8a + 4 lh + b, key lane & 31), so
    // its 64-lane condition is the pair {mask of row 8a + b, mask of row 8a + 4 + b}: two lane reads and one select
    // per element instead of the range comparisons.  Rows past the block end (clamped duplicates of its last
    // row) and keys past the tile end see nothing.
    const int row = lane & 31;
    const int q = qs32 + row;
    int lo1 = 0, hi1 = kind == 1 ? q + 1 : INT32_MAX, lo2 = 0, hi2 = 0;   // NONE: every key; CAUSAL: keys up to the query
    if (RANGES && kind == 2) {
      asm volatile("" ::: "memory");   // keeps the read inside the branch
      const int4 rg = ((const int4*)(stage + kStageRanges))[32 * qt + row];
      lo1 = rg.x; hi1 = rg.y; lo2 = rg.z; hi2 = rg.w;
    }
    uint32_t m = (keys_below(hi1, wk_lo) & ~keys_below(lo1, wk_lo)) | (keys_below(hi2, wk_lo) & ~keys_below(lo2, wk_lo));
    m &= keys_below(k_end, wk_lo);
    m = q < q1 ? m : 0u;
#pragma unroll
    for (int r = 0; r < 16; r++) {
      const int r0 = 8 * (r / 4) + (r % 4);
      const uint64_t cond = (uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)m, r0) |
                            ((uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)m, r0 + 4) << 32);
      s[r] = __builtin_amdgcn_inverse_ballot_w64(cond) ? s[r] : -INFINITY;
    }
  }
#pragma unroll
  for (int a = 0; a < 4; a++) {
    const float4 l4 = *(const float4*)(lse_lds + 8 * a);
    const float lv[4] = {l4.x, l4.y, l4.z, l4.w};
#pragma unroll
    for (int b = 0; b < 4; b++) {
      const int r = 4 * a + b;
      const float p = __builtin_amdgcn_exp2f(fmaf(s[r], c_log2, -lv[b]));
      s[r] = p;
      dp[r] *= p;
    }
  }
  {
    // P and dS packed first (s and dp are dead after that), then the transposed operands one step ahead
    bf16x8 pb[2], dsb[2];
#pragma unroll
    for (int c = 0; c < 2; c++) { pb[c] = pack_frag(s, c); dsb[c] = pack_frag(dp, c); }
    bf16x8 ta = frag_tr2(do_lds, fa, 32 * qt, 0), tb = frag_tr2(q_lds, fa, 32 * qt, 0);
#pragma unroll
    for (int i = 0; i < 8; i++) {
      const int c = i >> 2, dt = i & 3;
      bf16x8 tan = ta, tbn = tb;
      if (i < 7) {
        tan = frag_tr2(do_lds, fa, 32 * qt + 16 * ((i + 1) >> 2), (i + 1) & 3);
        tbn = frag_tr2(q_lds, fa, 32 * qt + 16 * ((i + 1) >> 2), (i + 1) & 3);
      }
      __builtin_amdgcn_sched_barrier(0);
      st.dv[dt] = mfma(ta, pb[c], st.dv[dt]);
      st.dk[dt] = mfma(tb, dsb[c], st.dk[dt]);
      ta = tan; tb = tbn;
      __builtin_amdgcn_sched_barrier(0);
    }
  }
}

// RANGES = false: the table has no row with per-token ranges (RANGES or WINDOW); everything that serves them is
// compiled out.  Two workgroups per CU: at most 256 registers.
template <bool RANGES>
__global__ __launch_bounds__(256, 2) void mfma_dkv_kernel(DevGroup g, KTensors t) {
  constexpr int TK = 128;
  __shared__ __attribute__((aligned(1024))) char stages[2 * kStageBytes];   // double buffer

  int item, hk;
  if (!decode_wg(g, t.hkv, 1, &item, &hk)) return;
  const int G = t.hq / t.hkv;
  WorkItem w = g.items[item];
  w.unit = uni(w.unit); w.tile = uni(w.tile); w.e0 = uni(w.e0); w.e1 = uni(w.e1); w.pslot = uni(w.pslot);

  const int tid = threadIdx.x, lane = tid & 63, wave = uni(tid >> 6);
  const int li = lane & 31, lh = lane >> 5;
  const int blk_start = uni(w.blk_start), blk_len = uni(w.blk_len);
  const int koff = uni(w.moff);   // rows of the KV-type buffers: packed index + koff
  const int seq0 = RANGES ? uni(g.blk_s0[uni(g.unit_blk[w.unit])]) : 0;   // first token of the sequence (keys and queries share it)
  const int row0 = w.tile * TK;
  const int n_rows = min(TK, blk_len - row0);
  const int k_lo = blk_start + row0, k_end = k_lo + n_rows;
  const int wrow0 = wave * 32;
  const int w_rows = max(0, min(32, n_rows - wrow0));
  const int wk_lo = k_lo + wrow0, wk_hi = wk_lo + w_rows - 1;

  DkvState st;
  const bool kvalid = wrow0 + li < n_rows;
  {
    const int kl = min(wk_lo + li, k_end - 1);
    const bf16_t* kp = (const bf16_t*)t.k + (int64_t)(kl + koff) * t.k_st + (int64_t)hk * t.k_sh + 8 * lh;
    const bf16_t* vp = (const bf16_t*)t.v + (int64_t)(kl + koff) * t.v_st + (int64_t)hk * t.v_sh + 8 * lh;
#pragma unroll
    for (int ks = 0; ks < 8; ks++) {
      st.kf[ks] = as_frag(*(const uint4*)(kp + 16 * ks));
      st.vf[ks] = as_frag(*(const uint4*)(vp + 16 * ks));
    }
#pragma unroll
    for (int dt = 0; dt < 4; dt++)
#pragma unroll
      for (int x = 0; x < 16; x++) { st.dk[dt][x] = 0.f; st.dv[dt][x] = 0.f; }
  }
  const float c_log2 = t.scale * kLog2e;

  QIter<RANGES> it(g, w.e0, w.e1, G, t.qbounds);
  auto issue = [&](char* stage) {
    const int head = hk * G + it.hh;
    const int last = it.q1 - 1;
    tile_dma_lean<4>(stage, (const bf16_t*)t.q + (int64_t)head * t.q_sh, (int)t.q_st * 2, it.qs + it.moff, last + it.moff, wave);
    tile_dma_lean<4>(stage + kTileBytes, (const bf16_t*)t.dout + (int64_t)head * t.do_sh, (int)t.do_st * 2, it.qs + it.moff, last + it.moff, wave);
    const int qrow = min(it.qs + lane, last);   // packed index: the range array is not a data block
    const int qmem = qrow + it.moff;
    if (wave == 0) dma4((unsigned)qmem * 4u, uni_ptr(t.lse2 + (int64_t)head * t.q_rows), lds_addr(stage + kStageLse));
    if (wave == 1) dma4((unsigned)qmem * 4u, uni_ptr(t.delta + (int64_t)head * t.q_rows), lds_addr(stage + kStageDelta));
    if (RANGES && wave == 2 && it.kind == 2) {
      // the rows' ranges: copied from the array, or (WINDOW rows) worked out and stored; the barrier that ends the
      // step orders the store before the reads
      if (t.window > 0) *((int4*)(stage + kStageRanges) + lane) = range_row(t, qrow, seq0);
      else dma16((unsigned)qrow * 16u, uni_ptr(t.ranges), lds_addr(stage + kStageRanges));
    }
    // the bounds of the tile's two halves (4 x 16 B; the other lanes repeat them into the reserved space)
    if (RANGES && wave == 3 && it.kind == 2 && t.qbounds)
      dma16((unsigned)(lane & 3) * 16u, uni_ptr(t.qbounds + (int64_t)(it.t32 + 2 * it.jt) * 8), lds_addr(stage + kStageBounds));
  };
  bool have = it.next(k_lo, k_end);
  if (have) issue(stages);
  DCP_WAIT_VMCNT(0);
  __syncthreads();
  // one copy of the sub-tile code for both buffers and both halves of a tile: the accumulators keep their registers
  int buf = 0;
  while (have) {
    const char* cur = stages + buf;
    const int qs = it.qs, q1 = it.q1, kind = it.kind;
    have = it.next(k_lo, k_end);
    if (have) issue(stages + (buf ^ kStageBytes));
    if (w_rows > 0) {
#pragma unroll 1
      for (int qt = 0; qt < 2; qt++) {
        const int qs32 = qs + 32 * qt;
        if (qs32 >= q1) break;
        const bool whole = qs32 + 32 <= q1 && w_rows == 32;
        int cls = kPartial;
        if (kind == 0) cls = whole ? kFull : kPartial;
        if (kind == 1) cls = min(qs32 + 31, q1 - 1) < wk_lo ? kSkip : ((whole && qs32 >= wk_hi) ? kFull : kPartial);
        if (RANGES && kind == 2 && t.qbounds) {
          // the 32 queries' range bounds against the wave's keys (the empty asm keeps the compiler from hoisting
          // these LDS reads, and their wait, out of the branch into every step)
          asm volatile("" ::: "memory");
          const int4* bp = (const int4*)(cur + kStageBounds) + 2 * qt;
          const int4 a = bp[0], b = bp[1];
          RangeBounds qb;
          qb.lo_min[0] = uni(a.x); qb.lo_max[0] = uni(a.y); qb.hi_min[0] = uni(a.z); qb.hi_max[0] = uni(a.w);
          qb.lo_min[1] = uni(b.x); qb.lo_max[1] = uni(b.y); qb.hi_min[1] = uni(b.z); qb.hi_max[1] = uni(b.w);
          if (!qb.may_see(wk_lo, wk_hi + 1)) cls = kSkip;
          else if (whole && qb.all_see(wk_lo, wk_hi + 1)) cls = kFull;
        }
        if (cls != kSkip) dkv_subtile<RANGES>(st, cur, qt, qs32, q1, kind, wk_lo, k_end, c_log2, cls == kPartial);
      }
    }
    DCP_WAIT_VMCNT(0);
    __syncthreads();
    buf ^= kStageBytes;
  }
  if (w.pslot >= 0) {
    if (!kvalid) return;
    // one part of a split item: the fp32 sums go to the part's slot, the reduce kernel adds the parts up
    float* pk = t.part + (((int64_t)w.pslot * t.hkv + hk) * 2 * TK + wrow0 + li) * 128 + 4 * lh;
    float* pv = pk + TK * 128;
#pragma unroll
    for (int dt = 0; dt < 4; dt++)
#pragma unroll
      for (int a = 0; a < 4; a++) {
        *(float4*)(pk + 32 * dt + 8 * a) = make_float4(st.dk[dt][4 * a] * t.scale, st.dk[dt][4 * a + 1] * t.scale,
                                                       st.dk[dt][4 * a + 2] * t.scale, st.dk[dt][4 * a + 3] * t.scale);
        *(float4*)(pv + 32 * dt + 8 * a) = make_float4(st.dv[dt][4 * a], st.dv[dt][4 * a + 1], st.dv[dt][4 * a + 2], st.dv[dt][4 * a + 3]);
      }
    return;
  }
  // dK and dV go out in whole rows, turned round through the stages (free after the last step's barrier), one
  // region per wave, dK first and dV after it through the same region
  static_assert(4 * 32 * kORow <= 2 * kStageBytes, "the four waves' output tiles fit in the stages");
  char* ot = stages + wave * (32 * kORow);
  store_tile32(ot, st.dk, t.scale, lane, w_rows, (bf16_t*)t.dk + (int64_t)(wk_lo + koff) * t.dk_st + (int64_t)hk * t.dk_sh, t.dk_st);
  store_tile32(ot, st.dv, 1.f, lane, w_rows, (bf16_t*)t.dv + (int64_t)(wk_lo + koff) * t.dv_st + (int64_t)hk * t.dv_sh, t.dv_st);
}

}  // namespace dcp
