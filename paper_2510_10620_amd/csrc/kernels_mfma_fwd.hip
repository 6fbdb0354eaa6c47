// Blockwise attention forward on bf16 MFMA (Listing 1 line 5 + the in-kernel part of line 6).
//
// One workgroup (4 waves) owns a query tile of 4 * 32 * NQ rows of one head and walks the KV tiles
// (64 keys) of every table row of its output unit.  Scores are computed transposed,
// S^T = K Q^T, so that a lane owns one query column: the running max / sum are per-lane scalars,
// the only cross-lane step is one exchange between the two wave halves per 32 keys, and P^T in the
// MFMA accumulator layout is directly the B operand of O^T += V^T P^T.  K and V tiles are copied
// global -> LDS asynchronously one tile ahead into the other of two buffers; V^T fragments come
// from transposing LDS reads.  A 64-key tile that is fully visible to the wave takes a path with two
// independent score chains; tiles on a mask edge are handled per 32 keys with the per-element test.
#include "mfma_common.h"

namespace dcp {

static constexpr float kLazy = 8.f;  // rescale threshold, log2 units

#ifndef DCP_FWD_NW
#define DCP_FWD_NW 4
#endif
static constexpr int kFwdWaves = DCP_FWD_NW;   // waves per workgroup
static_assert(kFwdWaves == 4, "the step's inline tile copies are written for four waves (four copy instructions per wave and tile)");

template <int NQ>
struct FwdCfg {
  static constexpr int kWaveRows = 32 * NQ;
  static constexpr int kTileM = kFwdWaves * kWaveRows;
};

template <int NQ>
struct FwdState {
  bf16x8 qf[NQ][8];
  f32x16 o[NQ][4];
  float m[NQ], l[NQ];
  int qi[NQ];
  int4 qr[NQ];
  FragAddr fa;
  TileDmaT<16 / kFwdWaves> dmak, dmav;
};

// Scores of one 32-key sub-tile, S^T = K Q^T (one chain of 8 MFMAs), with the per-element mask test if MASK.
template <int NQ>
__device__ __forceinline__ void fwd_scores32(const FwdState<NQ>& st, const char* k_lds, int kt, int ks32, int kind, int c0,
                                             int c1, int lane, bool MASK, f32x16 (&s)[NQ]) {
  const int lh = lane >> 5;
#pragma unroll
  for (int nq = 0; nq < NQ; nq++)
#pragma unroll
    for (int r = 0; r < 16; r++) s[nq][r] = 0.f;
#pragma unroll
  for (int ksd = 0; ksd < 8; ksd++) {
    const bf16x8 a = frag_rm(k_lds, st.fa, 32 * kt, ksd);
#pragma unroll
    for (int nq = 0; nq < NQ; nq++) s[nq] = mfma(a, st.qf[nq][ksd], s[nq]);
  }
  if (MASK) {
#pragma unroll
    for (int nq = 0; nq < NQ; nq++) {
      const RowRanges rr = row_ranges(kind, st.qi[nq], c0, c1, st.qr[nq]);
      const int kb = ks32 + 4 * lh;
#pragma unroll
      for (int r = 0; r < 16; r++) {
        const int key = kb + 8 * (r / 4) + (r % 4);
        if (!rr.sees(key)) s[nq][r] = -INFINITY;
      }
    }
  }
}

// Scores of a whole 64-key tile every pair of which is visible to the wave: the two 32-key score tiles are two
// independent MFMA chains, K fragments requested four k-steps ahead of the MFMAs that use them.
// DMA: the eight copy instructions of the next K and V tiles are issued here, one per k-step between the MFMAs
// (kb / vb: the tiles' first rows, lk / lv: the wave's part of the LDS stage they go to).
template <int NQ, bool DMA>
__device__ __forceinline__ void fwd_scores64(const FwdState<NQ>& st, const char* k_lds, f32x16 (&s)[2][NQ],
                                             const void* kb = nullptr, const void* vb = nullptr, unsigned lk = 0, unsigned lv = 0) {
#pragma unroll
  for (int kt = 0; kt < 2; kt++)
#pragma unroll
    for (int nq = 0; nq < NQ; nq++)
#pragma unroll
      for (int r = 0; r < 16; r++) s[kt][nq][r] = 0.f;
  constexpr int PF = 4;
  bf16x8 ka[8][2];
#pragma unroll
  for (int ksd = 0; ksd < PF; ksd++)
#pragma unroll
    for (int kt = 0; kt < 2; kt++) ka[ksd][kt] = frag_rm(k_lds, st.fa, 32 * kt, ksd);
#pragma unroll
  for (int ksd = 0; ksd < 8; ksd++) {
    __builtin_amdgcn_sched_barrier(0);
    if (DMA) {
      if (ksd < 4) st.dmak.issue(ksd, kb, lk);
      else st.dmav.issue(ksd - 4, vb, lv);
      __builtin_amdgcn_sched_barrier(0);
    }
    if (ksd + PF < 8) {
#pragma unroll
      for (int kt = 0; kt < 2; kt++) ka[ksd + PF][kt] = frag_rm(k_lds, st.fa, 32 * kt, ksd + PF);
    }
#pragma unroll
    for (int kt = 0; kt < 2; kt++)
#pragma unroll
      for (int nq = 0; nq < NQ; nq++) s[kt][nq] = mfma(ka[ksd][kt], st.qf[nq][ksd], s[kt][nq]);
  }
  __builtin_amdgcn_sched_barrier(0);
}

// Online softmax over the 64 keys of a tile and O^T += V^T P^T.  This is the only code that touches the output
// accumulators: every kind of tile (fully visible, mask edge, half skipped) computes its scores on its own path and
// joins here, so the accumulators never meet at a control-flow merge with different register assignments (which
// costs a copy of all 64 of them, there and back, per tile).  There is no branch on which sub-tiles are active
// either (a skipped one has scores -inf, so P = 0 and its MFMAs add nothing): one straight block, in which the P.V
// MFMAs of the first 32 keys are issued between the exponentials of the second 32 (the scheduling groups below say
// so; exponentials are their own instruction class there).  NQ = 1.
template <int NQ>
__device__ __forceinline__ void fwd_softmax_pv(FwdState<NQ>& st, f32x16 (&s)[2][NQ], const char* v_lds, float c_log2) {
  static_assert(NQ == 1, "one query per lane");
  bf16x8 va[4];
#pragma unroll
  for (int dt = 0; dt < 4; dt++) va[dt] = frag_tr(v_lds, st.fa, 0, dt);
  __builtin_amdgcn_sched_barrier(0);
  float mx = fmaxf(fmaxf(s[0][0][0], s[0][0][1]), s[1][0][0]);
  mx = fmaxf(mx, s[1][0][1]);
#pragma unroll
  for (int r = 2; r < 16; r += 2) {
    mx = fmaxf(fmaxf(mx, s[0][0][r]), s[0][0][r + 1]);
    mx = fmaxf(fmaxf(mx, s[1][0][r]), s[1][0][r + 1]);
  }
  mx = xhalf_max(mx);
  // the reference max is raised lazily (see fwd_subtile); a row that has seen no key yet keeps m = -inf and uses 0
  const bool raise = (mx - st.m[0]) * c_log2 > kLazy;
  const float m_new = raise ? mx : st.m[0];
  const float m_use = m_new == -INFINITY ? 0.f : m_new;
  const float mc = m_use * c_log2;
  if (__any(raise)) {
    const float alpha = raise ? __builtin_amdgcn_exp2f((st.m[0] - m_use) * c_log2) : 1.f;
    st.l[0] *= alpha;
#pragma unroll
    for (int dt = 0; dt < 4; dt++)
#pragma unroll
      for (int r = 0; r < 16; r++) st.o[0][dt][r] *= alpha;
  }
  st.m[0] = m_new;
  // first 32 keys
  float sum0 = 0.f;
#pragma unroll
  for (int r = 0; r < 16; r++) {
    const float e = __builtin_amdgcn_exp2f(fmaf(s[0][0][r], c_log2, -mc));
    s[0][0][r] = e;
    sum0 += e;
  }
  const bf16x8 p00 = pack_frag(s[0][0], 0), p01 = pack_frag(s[0][0], 1);
  __builtin_amdgcn_sched_barrier(0);
  // region: 8 MFMAs of the first 32 keys + the exponentials of the second 32, interleaved by the group barriers below
  bf16x8 vb[4], vc[4];
#pragma unroll
  for (int dt = 0; dt < 4; dt++) vb[dt] = frag_tr(v_lds, st.fa, 16, dt);
#pragma unroll
  for (int dt = 0; dt < 4; dt++) st.o[0][dt] = mfma(va[dt], p00, st.o[0][dt]);
#pragma unroll
  for (int dt = 0; dt < 4; dt++) vc[dt] = frag_tr(v_lds, st.fa, 32, dt);
#pragma unroll
  for (int dt = 0; dt < 4; dt++) st.o[0][dt] = mfma(vb[dt], p01, st.o[0][dt]);
  float sum1 = 0.f;
#pragma unroll
  for (int r = 0; r < 16; r++) {
    const float e = __builtin_amdgcn_exp2f(fmaf(s[1][0][r], c_log2, -mc));
    s[1][0][r] = e;
    sum1 += e;
  }
#pragma unroll
  for (int i = 0; i < 8; i++) {
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // one MFMA
    __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);   // two LDS reads for the MFMAs to come
    __builtin_amdgcn_sched_group_barrier(0x400, 2, 0);   // two exponentials
    __builtin_amdgcn_sched_group_barrier(0x002, 4, 0);   // their multiply-adds and the running sum
  }
  __builtin_amdgcn_sched_barrier(0);
  st.l[0] += sum0 + sum1;
  const bf16x8 p10 = pack_frag(s[1][0], 0), p11 = pack_frag(s[1][0], 1);
#pragma unroll
  for (int dt = 0; dt < 4; dt++) vb[dt] = frag_tr(v_lds, st.fa, 48, dt);
#pragma unroll
  for (int dt = 0; dt < 4; dt++) st.o[0][dt] = mfma(vc[dt], p10, st.o[0][dt]);
#pragma unroll
  for (int dt = 0; dt < 4; dt++) st.o[0][dt] = mfma(vb[dt], p11, st.o[0][dt]);
}

// One 32-key sub-tile: S^T = K Q^T, mask, online softmax, O^T += V^T P^T.
template <int NQ>
__device__ __forceinline__ void fwd_subtile(FwdState<NQ>& st, const char* k_lds, const char* v_lds, int kt, int ks32,
                                            int kind, int c0, int c1, float c_log2, int lane, bool MASK) {
  const int lh = lane >> 5;
  f32x16 s[NQ];
#pragma unroll
  for (int nq = 0; nq < NQ; nq++)
#pragma unroll
    for (int r = 0; r < 16; r++) s[nq][r] = 0.f;
#pragma unroll
  for (int ksd = 0; ksd < 8; ksd++) {
    const bf16x8 a = frag_rm(k_lds, st.fa, 32 * kt, ksd);
#pragma unroll
    for (int nq = 0; nq < NQ; nq++) s[nq] = mfma(a, st.qf[nq][ksd], s[nq]);
  }
  if (MASK) {
#pragma unroll
    for (int nq = 0; nq < NQ; nq++) {
      const RowRanges rr = row_ranges(kind, st.qi[nq], c0, c1, st.qr[nq]);
      const int kb = ks32 + 4 * lh;
#pragma unroll
      for (int r = 0; r < 16; r++) {
        const int key = kb + 8 * (r / 4) + (r % 4);
        if (!rr.sees(key)) s[nq][r] = -INFINITY;
      }
    }
  }
  bf16x8 p[NQ][2];
#pragma unroll
  for (int nq = 0; nq < NQ; nq++) {
    float mx = fmaxf(fmaxf(s[nq][0], s[nq][1]), s[nq][2]);
#pragma unroll
    for (int r = 3; r < 15; r += 2) mx = fmaxf(fmaxf(mx, s[nq][r]), s[nq][r + 1]);
    mx = fmaxf(mx, s[nq][15]);
    mx = xhalf_max(mx);
    // The reference max m is raised only when the tile's max exceeds it by more than 2^kLazy
    // (in the exp2 domain): until then P = exp2(c (s - m)) stays below 2^kLazy, exact in fp32 and
    // bf16 range, and the accumulators need no rescaling.  O and l are divided by the same sum at
    // the end, so the result does not depend on which m was used.
    const bool raise = (mx - st.m[nq]) * c_log2 > kLazy;   // also true for the first visible key (m = -inf)
    const float m_new = raise ? mx : st.m[nq];
    const float m_use = m_new == -INFINITY ? 0.f : m_new;
    const float mc = m_use * c_log2;
    if (__any(raise)) {
      const float alpha = raise ? __builtin_amdgcn_exp2f((st.m[nq] - m_use) * c_log2) : 1.f;
      st.l[nq] *= alpha;
#pragma unroll
      for (int dt = 0; dt < 4; dt++)
#pragma unroll
        for (int r = 0; r < 16; r++) st.o[nq][dt][r] *= alpha;
    }
    st.m[nq] = m_new;
    float sum = 0.f;
#pragma unroll
    for (int r = 0; r < 16; r++) {
      const float e = __builtin_amdgcn_exp2f(fmaf(s[nq][r], c_log2, -mc));
      s[nq][r] = e;
      sum += e;
    }
    st.l[nq] += sum;
#pragma unroll
    for (int c = 0; c < 2; c++) p[nq][c] = pack_frag(s[nq], c);
  }
#pragma unroll
  for (int c = 0; c < 2; c++)
#pragma unroll
    for (int dt = 0; dt < 4; dt++) {
      const bf16x8 a = frag_tr(v_lds, st.fa, 32 * kt + 16 * c, dt);
#pragma unroll
      for (int nq = 0; nq < NQ; nq++) st.o[nq][dt] = mfma(a, p[nq][c], st.o[nq][dt]);
    }
}

// A whole 64-key tile every pair of which is visible to the wave (kernel variant for tables with per-token ranges).
template <int NQ>
__device__ __forceinline__ void fwd_tile64(FwdState<NQ>& st, const char* k_lds, const char* v_lds, float c_log2) {
  f32x16 s[2][NQ];
  fwd_scores64<NQ, false>(st, k_lds, s);
  fwd_softmax_pv<NQ>(st, s, v_lds, c_log2);
}

// RANGES = false: the table has no row with per-token ranges (RANGES or WINDOW) and every use of them folds away.
template <int NQ, bool RANGES>
__global__ __launch_bounds__(64 * kFwdWaves, (NQ == 1 ? 2 : 1)) void mfma_fwd_kernel(DevGroup g, KTensors t) {
  if (!RANGES) t.masked = 0;
  constexpr int WR = FwdCfg<NQ>::kWaveRows, TM = FwdCfg<NQ>::kTileM;
  // two stages, each [K tile | V tile]
  __shared__ __attribute__((aligned(1024))) char stage0[2 * kTileBytes];
  __shared__ __attribute__((aligned(1024))) char stage1[2 * kTileBytes];
  __shared__ int wg_bounds[kFwdWaves][8];

  int item, head;
  const int G = t.hq / t.hkv;
  if (!decode_wg(g, t.hkv, G, &item, &head)) return;
  const int hk = head / G;
  WorkItem w = g.items[item];
  w.unit = uni(w.unit); w.tile = uni(w.tile); w.e0 = uni(w.e0); w.e1 = uni(w.e1);
  const int tid = threadIdx.x, lane = tid & 63, wave = uni(tid >> 6);
  const int li = lane & 31, lh = lane >> 5;
  const int blk_start = uni(w.blk_start), blk_len = uni(w.blk_len);
  const int qoff = uni(w.moff);                       // rows of the Q-type buffers: packed index + qoff
  const int row0 = w.tile * TM;                       // first row of the tile inside the block
  const int n_rows = min(TM, blk_len - row0);         // valid rows of the tile (>= 1)
  const int q_lo = blk_start + row0, q_hi = q_lo + n_rows - 1;
  const int wrow0 = wave * WR;                        // wave's first row inside the tile
  const int w_rows = max(0, min(WR, n_rows - wrow0)); // wave's valid rows
  const int wq_lo = q_lo + wrow0, wq_hi = wq_lo + w_rows - 1;

  FwdState<NQ> st;
  st.fa.init(lane);
  st.dmak.init(wave, lane, t.k_st);
  st.dmav.init(wave, lane, t.v_st);
  bool qv[NQ];
  RangeBounds wrb;
  wrb.init();
#pragma unroll
  for (int nq = 0; nq < NQ; nq++) {
    const int r = wrow0 + nq * 32 + li;
    qv[nq] = r < n_rows;
    st.qi[nq] = q_lo + min(r, n_rows - 1);
    st.qr[nq] = make_int4(0, 0, 0, 0);
    if (t.masked) {
      st.qr[nq] = range_row(t, st.qi[nq], uni(g.blk_s0[uni(g.unit_blk[w.unit])]));
      if (qv[nq]) wrb.add(st.qr[nq]);
    }
  }
  RangeBounds rb = wrb;  // workgroup bounds
  if (t.masked) {
    wrb.wave_reduce();
    if (lane == 0) {
      wg_bounds[wave][0] = wrb.lo_min[0]; wg_bounds[wave][1] = wrb.lo_max[0]; wg_bounds[wave][2] = wrb.hi_min[0]; wg_bounds[wave][3] = wrb.hi_max[0];
      wg_bounds[wave][4] = wrb.lo_min[1]; wg_bounds[wave][5] = wrb.lo_max[1]; wg_bounds[wave][6] = wrb.hi_min[1]; wg_bounds[wave][7] = wrb.hi_max[1];
    }
    __syncthreads();
    rb.init();
    for (int x = 0; x < kFwdWaves; x++) {
      rb.lo_min[0] = min(rb.lo_min[0], wg_bounds[x][0]); rb.lo_max[0] = max(rb.lo_max[0], wg_bounds[x][1]);
      rb.hi_min[0] = min(rb.hi_min[0], wg_bounds[x][2]); rb.hi_max[0] = max(rb.hi_max[0], wg_bounds[x][3]);
      rb.lo_min[1] = min(rb.lo_min[1], wg_bounds[x][4]); rb.lo_max[1] = max(rb.lo_max[1], wg_bounds[x][5]);
      rb.hi_min[1] = min(rb.hi_min[1], wg_bounds[x][6]); rb.hi_max[1] = max(rb.hi_max[1], wg_bounds[x][7]);
    }
#pragma unroll
    for (int k = 0; k < 2; k++) {
      rb.lo_min[k] = uni(rb.lo_min[k]); rb.lo_max[k] = uni(rb.lo_max[k]); rb.hi_min[k] = uni(rb.hi_min[k]); rb.hi_max[k] = uni(rb.hi_max[k]);
      wrb.lo_min[k] = uni(wrb.lo_min[k]); wrb.lo_max[k] = uni(wrb.lo_max[k]); wrb.hi_min[k] = uni(wrb.hi_min[k]); wrb.hi_max[k] = uni(wrb.hi_max[k]);
    }
  }

  // Q fragments (B operand: lane = query column li, d = 16 ks + 8 lh ..)
#pragma unroll
  for (int nq = 0; nq < NQ; nq++) {
    const bf16_t* qp = (const bf16_t*)t.q + (int64_t)(st.qi[nq] + qoff) * t.q_st + (int64_t)head * t.q_sh + 8 * lh;
#pragma unroll
    for (int ks = 0; ks < 8; ks++) st.qf[nq][ks] = as_frag(*(const uint4*)(qp + 16 * ks));
    st.m[nq] = -INFINITY; st.l[nq] = 0.f;
#pragma unroll
    for (int dt = 0; dt < 4; dt++)
#pragma unroll
      for (int r = 0; r < 16; r++) st.o[nq][dt][r] = 0.f;
  }
  const float c_log2 = t.scale * 1.44269504088896340736f;
  const bf16_t* kbase = (const bf16_t*)t.k + (int64_t)hk * t.k_sh;
  const bf16_t* vbase = (const bf16_t*)t.v + (int64_t)hk * t.v_sh;

  KvIter it(g, w.e0, w.e1);
  bool have = it.next<RANGES>(q_hi, rb);
  if (have) {
    st.dmak.load(stage0, kbase, it.ks + it.moff, it.c1 - 1 + it.moff, wave);
    st.dmav.load(stage0 + kTileBytes, vbase, it.ks + it.moff, it.c1 - 1 + it.moff, wave);
  }
  DCP_WAIT_VMCNT(0);
  __syncthreads();

  // one pipeline step: prefetch the next tile into `nxt`, compute the current one from `cur`
  auto step = [&](const char* cur, char* nxt) {
    const int ks = it.ks, c0 = it.c0, c1 = it.c1, kind = RANGES ? it.kind : (it.kind & 1);
    if constexpr (RANGES) {
      // the same short test as below spares the iterator and the classification: NONE and CAUSAL rows as there, rows
      // with per-token ranges when one of the two ranges of every row of the wave covers this tile and the next
      int cls0 = kFull, cls1 = kFull;
      if (w_rows > 0 && (kind < 2 ? ks + 2 * kTN <= (kind ? min(c1, wq_lo + 1) : c1)
                                  : ks + 2 * kTN <= c1 && wrb.all_see(ks, ks + 2 * kTN))) {
        it.jt++;
        it.ks += kTN;
      } else {
        have = it.next<RANGES>(q_hi, rb);
        if (w_rows > 0) { cls0 = classify32(kind, ks, c1, wq_lo, wq_hi, wrb); cls1 = classify32(kind, ks + 32, c1, wq_lo, wq_hi, wrb); }
      }
      if (have) {
        st.dmak.load(nxt, kbase, it.ks + it.moff, it.c1 - 1 + it.moff, wave);
        st.dmav.load(nxt + kTileBytes, vbase, it.ks + it.moff, it.c1 - 1 + it.moff, wave);
      }
      if (w_rows > 0) {
        // tables with per-token ranges: three self-contained paths (measured 4-5 % faster there than the joined form)
        if (cls0 == kFull && cls1 == kFull) {
          fwd_tile64<NQ>(st, cur, cur + kTileBytes, c_log2);
        } else {
          if (cls0 != kSkip) fwd_subtile<NQ>(st, cur, cur + kTileBytes, 0, ks, kind, c0, c1, c_log2, lane, cls0 == kPartial);
          if (cls1 != kSkip) fwd_subtile<NQ>(st, cur, cur + kTileBytes, 1, ks + 32, kind, c0, c1, c_log2, lane, cls1 == kPartial);
        }
      }
    } else {
      // NONE / CAUSAL tables: the score paths join in one softmax + PV section (4 % faster there: no copies of the
      // accumulators at the merge)
      f32x16 s[2][NQ];
      bool pv;
      if (w_rows > 0 && ks + 2 * kTN <= (kind ? min(c1, wq_lo + 1) : c1)) {
        // The common step, found with a handful of scalar instructions: this tile and the next one of the same table
        // row are whole and visible to every row of the wave.  The iterator moves by one tile, nothing is classified,
        // and the copies of the next tile are issued between the score MFMAs: issued back to back at the top of the
        // step, the copy instructions of the four waves queue behind one another at the address unit and the waves
        // issue nothing else meanwhile; the general path's scalar bookkeeping costs some hundred issue slots more.
        it.jt++;
        it.ks += kTN;
        fwd_scores64<NQ, true>(st, cur, s, uni_ptr((const char*)kbase + (int64_t)(it.ks + it.moff) * st.dmak.sb),
                               uni_ptr((const char*)vbase + (int64_t)(it.ks + it.moff) * st.dmav.sb),
                               st.dmak.lds_of(nxt, wave), st.dmav.lds_of(nxt + kTileBytes, wave));
        pv = true;
      } else {
        have = it.next<RANGES>(q_hi, rb);
        if (have) {
          st.dmak.load(nxt, kbase, it.ks + it.moff, it.c1 - 1 + it.moff, wave);
          st.dmav.load(nxt + kTileBytes, vbase, it.ks + it.moff, it.c1 - 1 + it.moff, wave);
        }
        const int cls0 = w_rows > 0 ? classify32(kind, ks, c1, wq_lo, wq_hi, wrb) : kSkip;
        const int cls1 = w_rows > 0 ? classify32(kind, ks + 32, c1, wq_lo, wq_hi, wrb) : kSkip;
        pv = cls0 != kSkip || cls1 != kSkip;
        if (cls0 == kFull && cls1 == kFull) {
          fwd_scores64<NQ, false>(st, cur, s);
        } else if (pv) {
#pragma unroll
          for (int kt = 0; kt < 2; kt++) {
            const int cls = kt ? cls1 : cls0;
            if (cls != kSkip) {
              fwd_scores32<NQ>(st, cur, kt, ks + 32 * kt, kind, c0, c1, lane, cls == kPartial, s[kt]);
            } else {
#pragma unroll
              for (int nq = 0; nq < NQ; nq++)
#pragma unroll
                for (int r = 0; r < 16; r++) s[kt][nq][r] = -INFINITY;
            }
          }
        }
      }
      if (pv) fwd_softmax_pv<NQ>(st, s, cur + kTileBytes, c_log2);
    }
    DCP_WAIT_VMCNT(0);
    __syncthreads();  // the copy into `nxt` has landed and `cur` may be overwritten
  };
  while (have) {
    step(stage0, stage1);
    if (!have) break;
    step(stage1, stage0);
  }

  // ---- epilogue: O = acc / l, LSE = ln2 * (m c + log2 l); the output tile goes out in whole rows (the tile stages
  // are free after the last step's barrier, two waves stage in each)
  static_assert(2 * 32 * kORow <= 2 * kTileBytes, "two waves stage their output tiles in one tile stage");
  char* ot = (wave < 2 ? stage0 : stage1) + (wave & 1) * (32 * kORow);
  const int slot = g.unit_out[w.unit];
#pragma unroll
  for (int nq = 0; nq < NQ; nq++) {
    const float lt = xhalf_sum(st.l[nq]);
    const float inv = lt > 0.f ? 1.f / lt : 0.f;
    const float lse = lt > 0.f ? (st.m[nq] * c_log2 + __builtin_amdgcn_logf(lt)) * 0.69314718055994530942f : -INFINITY;
    const int brow0 = row0 + wrow0 + nq * 32;   // the wave's first row inside the block
    if (qv[nq] && lh == 0) {
      if (slot < 0) t.lse[(int64_t)head * t.q_rows + blk_start + brow0 + li + qoff] = lse;
      else t.lse[((int64_t)slot * t.hq + head) * t.block_size + brow0 + li] = lse;
    }
    bf16_t* op = slot < 0 ? (bf16_t*)t.out + (int64_t)(blk_start + brow0 + qoff) * t.o_st + (int64_t)head * t.o_sh
                          : (bf16_t*)t.out + (((int64_t)slot * t.block_size + brow0) * t.hq + head) * kD;
    store_tile32(ot, st.o[nq], inv, lane, n_rows - wrow0 - nq * 32, op, slot < 0 ? t.o_st : (int64_t)t.hq * kD);
  }
}

bool mfma_supports(int32_t dtype, int32_t d) { return dtype == DCP_BF16 && d == kD; }

#ifndef DCP_FWD_NQ
#define DCP_FWD_NQ 1
#endif
int mfma_fwd_tile() { return FwdCfg<DCP_FWD_NQ>::kTileM; }

dcp_status_t mfma_fwd(const DevGroup& g, const KTensors& t, hipStream_t s) {
  if (g.n_items == 0) return DCP_OK;
  const int grid = xcd_grid(g, t.hkv, t.hq / t.hkv);
  if (t.masked) hipLaunchKernelGGL((mfma_fwd_kernel<DCP_FWD_NQ, true>), dim3(grid), dim3(64 * kFwdWaves), 0, s, g, t);
  else hipLaunchKernelGGL((mfma_fwd_kernel<DCP_FWD_NQ, false>), dim3(grid), dim3(64 * kFwdWaves), 0, s, g, t);
  DCP_HIP_TRY(hipGetLastError());
  return DCP_OK;
}

}  // namespace dcp
