// Blockwise attention backward on bf16 MFMA, dK/dV kernel (the other half of the two-kernel backward): grouped by
// kv_blk; S = Q K^T, dP = dO V^T with keys as MFMA columns, then dV^T += dO^T P, dK^T += Q^T dS, looping over the
// query heads of the KV group and the queries of every listed q_blk (Q^T / dO^T fragments by transposing reads).
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

// Bounds of the range arrays of every 32-row tile of every block (rows of a tile = lanes 0..31), so that the
// dK/dV kernel, which streams query tiles past fixed keys, can tell without reading the rows whether a tile
// sees any of its keys (skip) or all of them (no per-element test).  Entry layout = RangeBounds member order.
__global__ __launch_bounds__(256) void range_bounds_kernel(const int32_t* __restrict__ blk_start, const int32_t* __restrict__ blk_len,
                                                           const int32_t* __restrict__ blk_t32, const int4* __restrict__ ranges,
                                                           int32_t* __restrict__ qbounds) {
  const int b = blockIdx.y;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int t = blockIdx.x * 4 + wave;
  const int len = blk_len[b];
  if (32 * t >= len) return;
  const int row = 32 * t + (lane & 31);
  RangeBounds rb;
  rb.init();
  if (row < len) rb.add(ranges[blk_start[b] + row]);
  rb.wave_reduce();
  if (lane == 0) {
    int32_t* o = qbounds + (int64_t)(blk_t32[b] + t) * 8;
    o[0] = rb.lo_min[0]; o[1] = rb.lo_max[0]; o[2] = rb.hi_min[0]; o[3] = rb.hi_max[0];
    o[4] = rb.lo_min[1]; o[5] = rb.lo_max[1]; o[6] = rb.hi_min[1]; o[7] = rb.hi_max[1];
  }
}

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
  __device__ QIter(const DevGroup& g, int unit, int G_, const int32_t* qb)
      : rec((const int4*)g.ent_rec), qbounds((const int4*)qb) {
    e = uni(g.ptr[unit]) - 1; e_end = uni(g.ptr[unit + 1]); hh = G_ - 1; G = G_; jt = 0; n_t = 0; jt0 = 0; q0 = q1 = kind = 0; moff = 0; t32 = 0; qs = 0;
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
      jt++;
      if (jt >= n_t) {
        hh++;
        if (hh >= G) {
          e++;
          if (e >= e_end) return false;
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
        jt = jt0 - 1;
        continue;
      }
      qs = q0 + jt * kTN;
      return true;
    }
  }
};

struct DkvState {
  bf16x8 kf[8], vf[8];
  f32x16 dk[4], dv[4];
  int kj;
  FragAddr fa;
  TileDma dmaq, dmao;
};

template <bool RANGES>
__device__ __forceinline__ void dkv_subtile(DkvState& st, const char* stage, int qt, int qs32, int q1, int kind,
                                            int k_end, float c_log2, int lane, bool MASK) {
  const int lh = lane >> 5;
  const char* q_lds = stage;
  const char* do_lds = stage + kTileBytes;
  f32x16 s, dp;
#pragma unroll
  for (int r = 0; r < 16; r++) { s[r] = 0.f; dp[r] = 0.f; }
  // operand fragments are requested four k-steps ahead of the MFMAs that use them: one exposed LDS round
  // trip per sub-tile, not one per k-step (left alone, the compiler reuses two registers and waits for every pair)
  bf16x8 qa[8], da[8];
  // rows of the C tile are queries 8a + 4 lh + b: their LSE / delta come from LDS (broadcast reads), requested
  // first so that nothing queued later stands between them and the exponentials
  const float* lse_lds = (const float*)(stage + kStageLse) + 32 * qt + 4 * lh;
  const float* dl_lds = (const float*)(stage + kStageDelta) + 32 * qt + 4 * lh;
  float4 l4[4], d4[4];
#pragma unroll
  for (int a = 0; a < 4; a++) {
    l4[a] = *(const float4*)(lse_lds + 8 * a);
    d4[a] = *(const float4*)(dl_lds + 8 * a);
  }
#pragma unroll
  for (int ksd = 0; ksd < 4; ksd++) {
    qa[ksd] = frag_rm(q_lds, st.fa, 32 * qt, ksd);
    da[ksd] = frag_rm(do_lds, st.fa, 32 * qt, ksd);
  }
  // transposed operands of the second half (dO^T, Q^T; two groups of 16 queries): the first group is requested
  // under the score MFMAs, the second under the exponentials
  bf16x8 dot[2][4], qt_[2][4];
#pragma unroll
  for (int ksd = 0; ksd < 8; ksd++) {
    __builtin_amdgcn_sched_barrier(0);
    if (ksd + 4 < 8) {
      qa[ksd + 4] = frag_rm(q_lds, st.fa, 32 * qt, ksd + 4);
      da[ksd + 4] = frag_rm(do_lds, st.fa, 32 * qt, ksd + 4);
    } else {
      dot[0][ksd - 4] = frag_tr(do_lds, st.fa, 32 * qt, ksd - 4);
      qt_[0][ksd - 4] = frag_tr(q_lds, st.fa, 32 * qt, ksd - 4);
    }
    s = mfma(qa[ksd], st.kf[ksd], s);
    dp = mfma(da[ksd], st.vf[ksd], dp);
  }
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int dt = 0; dt < 4; dt++) {
    dot[1][dt] = frag_tr(do_lds, st.fa, 32 * qt + 16, dt);
    qt_[1][dt] = frag_tr(q_lds, st.fa, 32 * qt + 16, dt);
  }
  __builtin_amdgcn_sched_barrier(0);
  if (MASK) {
    // element r = 4a + b is (query qs32 + 8a + 4 lh + b, key kj); queries past the block end are
    // clamped duplicates of its last row and must not count
    const int qb0 = qs32 + 4 * lh;
    const bool kok = st.kj < k_end;
    if (RANGES && kind == 2) {
      const int4* rg_lds = (const int4*)(stage + kStageRanges) + 32 * qt + 4 * lh;
#pragma unroll
      for (int r = 0; r < 16; r++) {
        const int4 rg = rg_lds[8 * (r / 4) + (r % 4)];
        const int q = qb0 + 8 * (r / 4) + (r % 4);
        const bool vis = kok & (q < q1) & (((st.kj >= rg.x) & (st.kj < rg.y)) | ((st.kj >= rg.z) & (st.kj < rg.w)));
        s[r] = vis ? s[r] : -INFINITY;
      }
    } else {
      const int kcmp = kind == 1 ? st.kj : INT32_MIN;   // causal: key <= query
#pragma unroll
      for (int r = 0; r < 16; r++) {
        const int q = qb0 + 8 * (r / 4) + (r % 4);
        const bool vis = kok & (q < q1) & (kcmp <= q);
        s[r] = vis ? s[r] : -INFINITY;
      }
    }
  }
#pragma unroll
  for (int a = 0; a < 4; a++) {
    const float lv[4] = {l4[a].x, l4[a].y, l4[a].z, l4[a].w}, dv4[4] = {d4[a].x, d4[a].y, d4[a].z, d4[a].w};
#pragma unroll
    for (int b = 0; b < 4; b++) {
      const int r = 4 * a + b;
      const float p = __builtin_amdgcn_exp2f(fmaf(s[r], c_log2, -lv[b]));
      s[r] = p;
      dp[r] = p * (dp[r] - dv4[b]);
    }
  }
#pragma unroll
  for (int c = 0; c < 2; c++) {
    const bf16x8 pb = pack_frag(s, c), dsb = pack_frag(dp, c);
#pragma unroll
    for (int dt = 0; dt < 4; dt++) {
      st.dv[dt] = mfma(dot[c][dt], pb, st.dv[dt]);
      st.dk[dt] = mfma(qt_[c][dt], dsb, st.dk[dt]);
    }
  }
}

// RANGES = false: the table has no RANGES row; everything that serves them is compiled out.
template <bool RANGES>
__global__ __launch_bounds__(256, 1) void mfma_dkv_kernel(DevGroup g, KTensors t) {
  constexpr int TK = 128;
  __shared__ __attribute__((aligned(1024))) char stage0[kStageBytes];
  __shared__ __attribute__((aligned(1024))) char stage1[kStageBytes];

  int item, hk;
  if (!decode_wg(g.n_items, t.hkv, 1, &item, &hk)) return;
  const int G = t.hq / t.hkv;
  WorkItem w = g.items[item];
  w.unit = uni(w.unit); w.tile = uni(w.tile);
  const int kb = uni(g.unit_blk[w.unit]);
  const int tid = threadIdx.x, lane = tid & 63, wave = uni(tid >> 6);
  const int li = lane & 31, lh = lane >> 5;
  const int blk_start = uni(g.blk_start[kb]), blk_len = uni(g.blk_len[kb]);
  const int koff = uni(g.unit_moff[w.unit]);   // rows of the KV-type buffers: packed index + koff
  const int row0 = w.tile * TK;
  const int n_rows = min(TK, blk_len - row0);
  const int k_lo = blk_start + row0, k_end = k_lo + n_rows;
  const int wrow0 = wave * 32;
  const int w_rows = max(0, min(32, n_rows - wrow0));
  const int wk_lo = k_lo + wrow0, wk_hi = wk_lo + w_rows - 1;

  DkvState st;
  st.fa.init(lane);
  st.dmaq.init(wave, lane, t.q_st);
  st.dmao.init(wave, lane, t.do_st);
  const bool kvalid = wrow0 + li < n_rows;
  st.kj = k_lo + wrow0 + li;                       // may lie past k_end: masked, never stored
  {
    const int kl = min(st.kj, k_end - 1);
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

  QIter<RANGES> it(g, w.unit, G, t.qbounds);
  auto issue = [&](char* stage) {
    const int head = hk * G + it.hh;
    const int last = it.q1 - 1;
    st.dmaq.load(stage, (const bf16_t*)t.q + (int64_t)head * t.q_sh, it.qs + it.moff, last + it.moff, wave);
    st.dmao.load(stage + kTileBytes, (const bf16_t*)t.dout + (int64_t)head * t.do_sh, it.qs + it.moff, last + it.moff, wave);
    const int qrow = min(it.qs + lane, last);   // packed index: the range array is not a data block
    const int qmem = qrow + it.moff;
    if (wave == 0) dma4((unsigned)qmem * 4u, uni_ptr(t.lse2 + (int64_t)head * t.q_rows), lds_addr(stage + kStageLse));
    if (wave == 1) dma4((unsigned)qmem * 4u, uni_ptr(t.delta + (int64_t)head * t.q_rows), lds_addr(stage + kStageDelta));
    if (RANGES && wave == 2 && it.kind == 2) dma16((unsigned)qrow * 16u, uni_ptr(t.ranges), lds_addr(stage + kStageRanges));
    // the bounds of the tile's two halves (4 x 16 B; the other lanes repeat them into the reserved space)
    if (RANGES && wave == 3 && it.kind == 2 && t.qbounds)
      dma16((unsigned)(lane & 3) * 16u, uni_ptr(t.qbounds + (int64_t)(it.t32 + 2 * it.jt) * 8), lds_addr(stage + kStageBounds));
  };
  bool have = it.next(k_lo, k_end);
  if (have) issue(stage0);
  DCP_WAIT_VMCNT(0);
  __syncthreads();
  auto step = [&](const char* cur, char* nxt) {
    const int qs = it.qs, q1 = it.q1, kind = it.kind;
    have = it.next(k_lo, k_end);
    if (have) issue(nxt);
    if (w_rows > 0) {
#pragma unroll
      for (int qt = 0; qt < 2; qt++) {
        const int qs32 = qs + 32 * qt;
        if (qs32 >= q1) continue;
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
        if (cls != kSkip) dkv_subtile<RANGES>(st, cur, qt, qs32, q1, kind, k_end, c_log2, lane, cls == kPartial);
      }
    }
    DCP_WAIT_VMCNT(0);
    __syncthreads();
  };
  while (have) {
    step(stage0, stage1);
    if (!have) break;
    step(stage1, stage0);
  }
  if (!kvalid) return;
  bf16_t* dkp = (bf16_t*)t.dk + (int64_t)(st.kj + koff) * t.dk_st + (int64_t)hk * t.dk_sh;
  bf16_t* dvp = (bf16_t*)t.dv + (int64_t)(st.kj + koff) * t.dv_st + (int64_t)hk * t.dv_sh;
#pragma unroll
  for (int dt = 0; dt < 4; dt++)
#pragma unroll
    for (int a = 0; a < 4; a++) {
      uint2 pk, pv;
      pk.x = (uint32_t)f32_to_bf16(st.dk[dt][4 * a] * t.scale) | ((uint32_t)f32_to_bf16(st.dk[dt][4 * a + 1] * t.scale) << 16);
      pk.y = (uint32_t)f32_to_bf16(st.dk[dt][4 * a + 2] * t.scale) | ((uint32_t)f32_to_bf16(st.dk[dt][4 * a + 3] * t.scale) << 16);
      pv.x = (uint32_t)f32_to_bf16(st.dv[dt][4 * a]) | ((uint32_t)f32_to_bf16(st.dv[dt][4 * a + 1]) << 16);
      pv.y = (uint32_t)f32_to_bf16(st.dv[dt][4 * a + 2]) | ((uint32_t)f32_to_bf16(st.dv[dt][4 * a + 3]) << 16);
      *(uint2*)(dkp + 32 * dt + 8 * a + 4 * lh) = pk;
      *(uint2*)(dvp + 32 * dt + 8 * a + 4 * lh) = pv;
    }
}

dcp_status_t mfma_range_bounds(const int32_t* blk_start, const int32_t* blk_len, const int32_t* blk_t32, int32_t n_blocks,
                               int32_t block_size, const int32_t* ranges, int32_t* qbounds, hipStream_t s) {
  if (n_blocks == 0) return DCP_OK;
  hipLaunchKernelGGL(range_bounds_kernel, dim3((block_size + 127) / 128, n_blocks), dim3(256), 0, s, blk_start, blk_len, blk_t32,
                     (const int4*)ranges, qbounds);
  DCP_HIP_TRY(hipGetLastError());
  return DCP_OK;
}

int mfma_dkv_tile() { return 128; }

dcp_status_t mfma_bwd_dkv(const DevGroup& g, const KTensors& t, hipStream_t s) {
  if (g.n_items == 0) return DCP_OK;
  const int per_xcd = (g.n_items * t.hkv + 7) / 8;
  if (t.ranges) hipLaunchKernelGGL(mfma_dkv_kernel<true>, dim3(per_xcd * 8), dim3(256), 0, s, g, t);
  else hipLaunchKernelGGL(mfma_dkv_kernel<false>, dim3(per_xcd * 8), dim3(256), 0, s, g, t);
  DCP_HIP_TRY(hipGetLastError());
  return DCP_OK;
}

}  // namespace dcp
