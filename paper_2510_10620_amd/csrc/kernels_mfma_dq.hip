// Blockwise attention backward on bf16 MFMA, dQ kernel.  The backward is two kernels that each recompute P from
// the saved LSE (no atomics, deterministic); this one is grouped by q_blk and has the shape of the forward:
// S^T = K Q^T, dP^T = V dO^T, dS^T = P^T * (dP^T - delta), dQ^T += K^T dS^T (K^T fragments by transposing reads).
#include "mfma_common.h"

namespace dcp {

static constexpr float kLog2e = 1.44269504088896340736f;

// ------------------------------------------------------------------------------------ dQ
struct DqState {
  bf16x8 qf[8], dof[8];
  f32x16 dq[4];
  f32x16 neg_delta;   // -delta of the lane's query in every element
  float lse2, delta;  // lse * log2(e) clamped to a finite value (a row that saw nothing has every score masked), delta
  int qi;
  int4 qr;
  FragAddr fa;
  TileDma dmak, dmav;
};

__device__ __forceinline__ void dq_subtile(DqState& st, const char* k_lds, const char* v_lds, int kt, int ks32,
                                           int kind, int c0, int c1, float c_log2, int lane, bool MASK) {
  const int lh = lane >> 5;
  // dP starts from -delta of the lane's query (a block of 16 registers kept for the whole kernel: the first MFMA
  // reads its accumulator input from there and writes elsewhere), so dS is one multiplication per element
  f32x16 s, dp = st.neg_delta;
#pragma unroll
  for (int r = 0; r < 16; r++) s[r] = 0.f;
#pragma unroll
  for (int ksd = 0; ksd < 8; ksd++) {
    s = mfma(frag_rm(k_lds, st.fa, 32 * kt, ksd), st.qf[ksd], s);
    dp = mfma(frag_rm(v_lds, st.fa, 32 * kt, ksd), st.dof[ksd], dp);
  }
  if (MASK) {
    const RowRanges rr = row_ranges(kind, st.qi, c0, c1, st.qr);
    const int kb = ks32 + 4 * lh;
#pragma unroll
    for (int r = 0; r < 16; r++) {
      const int key = kb + 8 * (r / 4) + (r % 4);
      if (!rr.sees(key)) s[r] = -INFINITY;
    }
  }
#pragma unroll
  for (int r = 0; r < 16; r++) {
    const float p = __builtin_amdgcn_exp2f(fmaf(s[r], c_log2, -st.lse2));
    s[r] = p * dp[r];
  }
#pragma unroll
  for (int c = 0; c < 2; c++) {
    const bf16x8 b = pack_frag(s, c);
#pragma unroll
    for (int dt = 0; dt < 4; dt++) st.dq[dt] = mfma(frag_tr(k_lds, st.fa, 32 * kt + 16 * c, dt), b, st.dq[dt]);
  }
}

template <bool RANGES>
__global__ __launch_bounds__(256, 2) void mfma_dq_kernel(DevGroup g, KTensors t) {
  if (!RANGES) t.masked = 0;
  constexpr int TM = 128;
  __shared__ __attribute__((aligned(1024))) char stage0[2 * kTileBytes];
  __shared__ __attribute__((aligned(1024))) char stage1[2 * kTileBytes];
  __shared__ int wg_bounds[4][8];

  int item, head;
  const int G = t.hq / t.hkv;
  if (!decode_wg(g, t.hkv, G, &item, &head)) return;
  const int hk = head / G;
  WorkItem w = g.items[item];
  w.unit = uni(w.unit); w.tile = uni(w.tile); w.e0 = uni(w.e0); w.e1 = uni(w.e1);
  const int tid = threadIdx.x, lane = tid & 63, wave = uni(tid >> 6);
  const int li = lane & 31, lh = lane >> 5;
  const int blk_start = uni(w.blk_start), blk_len = uni(w.blk_len);
  const int qoff = uni(w.moff);                // rows of the Q-type buffers: packed index + qoff
  const int row0 = w.tile * TM;
  const int n_rows = min(TM, blk_len - row0);
  const int q_lo = blk_start + row0, q_hi = q_lo + n_rows - 1;
  const int wrow0 = wave * 32;
  const int w_rows = max(0, min(32, n_rows - wrow0));
  const int wq_lo = q_lo + wrow0, wq_hi = wq_lo + w_rows - 1;

  DqState st;
  st.fa.init(lane);
  st.dmak.init(wave, lane, t.k_st);
  st.dmav.init(wave, lane, t.v_st);
  const int r = wrow0 + li;
  const bool qv = r < n_rows;
  st.qi = q_lo + min(r, n_rows - 1);
  st.qr = make_int4(0, 0, 0, 0);
  RangeBounds wrb;
  wrb.init();
  if (t.masked) {
    st.qr = range_row(t, st.qi, uni(g.blk_s0[uni(g.unit_blk[w.unit])]));
    if (qv) wrb.add(st.qr);
  }
  RangeBounds rb = wrb;
  if (t.masked) {
    wrb.wave_reduce();
    if (lane == 0) {
      wg_bounds[wave][0] = wrb.lo_min[0]; wg_bounds[wave][1] = wrb.lo_max[0]; wg_bounds[wave][2] = wrb.hi_min[0]; wg_bounds[wave][3] = wrb.hi_max[0];
      wg_bounds[wave][4] = wrb.lo_min[1]; wg_bounds[wave][5] = wrb.lo_max[1]; wg_bounds[wave][6] = wrb.hi_min[1]; wg_bounds[wave][7] = wrb.hi_max[1];
    }
    __syncthreads();
    rb.init();
    for (int x = 0; x < 4; x++) {
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
  {
    const bf16_t* qp = (const bf16_t*)t.q + (int64_t)(st.qi + qoff) * t.q_st + (int64_t)head * t.q_sh + 8 * lh;
    const bf16_t* dop = (const bf16_t*)t.dout + (int64_t)(st.qi + qoff) * t.do_st + (int64_t)head * t.do_sh + 8 * lh;
#pragma unroll
    for (int ks = 0; ks < 8; ks++) {
      st.qf[ks] = as_frag(*(const uint4*)(qp + 16 * ks));
      st.dof[ks] = as_frag(*(const uint4*)(dop + 16 * ks));
    }
    {
      // the backward preprocess, fused: delta = sum_d dO * O of the lane's row from the final O, and the saved LSE in
      // the exp2 domain (clamped to a finite value: a row that saw nothing has every score masked); -delta and the
      // LSE are left in the workspace for the dK/dV kernel, which runs after this one and starts its dP accumulators
      // from -delta
      const bf16_t* outp = (const bf16_t*)t.out_in + (int64_t)(st.qi + qoff) * t.o_st + (int64_t)head * t.o_sh + 8 * lh;
      float dl = 0.f;
#pragma unroll
      for (int ks = 0; ks < 8; ks++) {
        const uint4 u = *(const uint4*)(outp + 16 * ks);
        const uint32_t ow[4] = {u.x, u.y, u.z, u.w};
        const uint4 dd = __builtin_bit_cast(uint4, st.dof[ks]);
        const uint32_t dw[4] = {dd.x, dd.y, dd.z, dd.w};
#pragma unroll
        for (int i = 0; i < 4; i++) {
          dl = fmaf(__uint_as_float(ow[i] << 16), __uint_as_float(dw[i] << 16), dl);
          dl = fmaf(__uint_as_float(ow[i] & 0xffff0000u), __uint_as_float(dw[i] & 0xffff0000u), dl);
        }
      }
      st.delta = xhalf_sum(dl);
#pragma unroll
      for (int r = 0; r < 16; r++) st.neg_delta[r] = -st.delta;
      st.lse2 = fmaxf(t.lse[(int64_t)head * t.q_rows + st.qi + qoff] * kLog2e, -3.402823466e38f);
      if (qv && lh == 0) {
        t.delta_w[(int64_t)head * t.q_rows + st.qi + qoff] = -st.delta;
        t.lse2_w[(int64_t)head * t.q_rows + st.qi + qoff] = st.lse2;
      }
    }
#pragma unroll
    for (int dt = 0; dt < 4; dt++)
#pragma unroll
      for (int x = 0; x < 16; x++) st.dq[dt][x] = 0.f;
  }
  const float c_log2 = t.scale * kLog2e;
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
  auto step = [&](const char* cur, char* nxt) {
    const int ks = it.ks, c0 = it.c0, c1 = it.c1, kind = RANGES ? it.kind : (it.kind & 1);
    int cls0 = kFull, cls1 = kFull;
    bool fast;
    // (rows with per-token ranges take the general path: the test on the range bounds that would spare it costs as
    // much as it saves here)
    fast = (!RANGES || kind < 2) && w_rows > 0 && ks + 2 * kTN <= (kind ? min(c1, wq_lo + 1) : c1);
    if (fast) {
      // the common step, found with a handful of scalar instructions: this tile and the next one of the same table
      // row are whole and visible to every row of the wave; the iterator moves by one tile and nothing is classified
      it.jt++;
      it.ks += kTN;
    } else {
      have = it.next<RANGES>(q_hi, rb);
      cls0 = w_rows > 0 ? classify32(kind, ks, c1, wq_lo, wq_hi, wrb) : kSkip;
      cls1 = w_rows > 0 ? classify32(kind, ks + 32, c1, wq_lo, wq_hi, wrb) : kSkip;
    }
    if (cls0 != kSkip) dq_subtile(st, cur, cur + kTileBytes, 0, ks, kind, c0, c1, c_log2, lane, cls0 == kPartial);
    // the copies of the next tiles are issued between the two sub-tiles: at the top of the step, right after the
    // barrier, the copy instructions of the four waves queue behind one another at the address unit (2 % slower)
    if (have) {
      st.dmak.load(nxt, kbase, it.ks + it.moff, it.c1 - 1 + it.moff, wave);
      st.dmav.load(nxt + kTileBytes, vbase, it.ks + it.moff, it.c1 - 1 + it.moff, wave);
    }
    if (cls1 != kSkip) dq_subtile(st, cur, cur + kTileBytes, 1, ks + 32, kind, c0, c1, c_log2, lane, cls1 == kPartial);
    DCP_WAIT_VMCNT(0);
    __syncthreads();
  };
  while (have) {
    step(stage0, stage1);
    if (!have) break;
    step(stage1, stage0);
  }
  // dQ goes out in whole rows, turned round through the tile stages (free after the last step's barrier)
  static_assert(2 * 32 * kORow <= 2 * kTileBytes, "two waves stage their output tiles in one tile stage");
  bf16_t* op = (bf16_t*)t.dq + (int64_t)(wq_lo + qoff) * t.dq_st + (int64_t)head * t.dq_sh;
  store_tile32((wave < 2 ? stage0 : stage1) + (wave & 1) * (32 * kORow), st.dq, t.scale, lane, w_rows, op, t.dq_st);
}

int mfma_dq_tile() { return 128; }

dcp_status_t mfma_bwd_dq(const DevGroup& g, const KTensors& t, hipStream_t s) {
  if (g.n_items == 0) return DCP_OK;
  const int grid = xcd_grid(g, t.hkv, t.hq / t.hkv);
  if (t.masked) hipLaunchKernelGGL(mfma_dq_kernel<true>, dim3(grid), dim3(256), 0, s, g, t);
  else hipLaunchKernelGGL(mfma_dq_kernel<false>, dim3(grid), dim3(256), 0, s, g, t);
  DCP_HIP_TRY(hipGetLastError());
  return DCP_OK;
}

}  // namespace dcp
