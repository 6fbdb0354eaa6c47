// Blockwise attention backward on bf16 MFMA, dK/dV kernel (the other half of the two-kernel backward): grouped by
// kv_blk; S = Q K^T, dP = dO V^T with keys as MFMA columns, then dV^T += dO^T P, dK^T += Q^T dS, looping over the
// query heads of the KV group and the queries of every listed q_blk (Q^T / dO^T fragments by transposing reads).
#include "mfma_dkv_kernel.h"

namespace dcp {

// Bounds of the range arrays of every 32-row tile of every block (rows of a tile = lanes 0..31), so that the
// dK/dV kernel, which streams query tiles past fixed keys, can tell without reading the rows whether a tile
// sees any of its keys (skip) or all of them (no per-element test).  Entry layout = RangeBounds member order.
__global__ __launch_bounds__(256) void range_bounds_kernel(DevGroup g, KTensors t, const int32_t* __restrict__ blk_t32,
                                                           int32_t* __restrict__ qbounds) {
  const int b = blockIdx.y;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int tile = blockIdx.x * 4 + wave;
  const int len = g.blk_len[b];
  if (32 * tile >= len) return;
  const int row = 32 * tile + (lane & 31);
  RangeBounds rb;
  rb.init();
  if (row < len) rb.add(range_row(t, g.blk_start[b] + row, g.blk_s0[b]));
  rb.wave_reduce();
  if (lane == 0) {
    int32_t* o = qbounds + (int64_t)(blk_t32[b] + tile) * 8;
    o[0] = rb.lo_min[0]; o[1] = rb.lo_max[0]; o[2] = rb.hi_min[0]; o[3] = rb.hi_max[0];
    o[4] = rb.lo_min[1]; o[5] = rb.lo_max[1]; o[6] = rb.hi_min[1]; o[7] = rb.hi_max[1];
  }
}

// Adds up the parts of every split (KV tile, KV head) in slot order (the same sum whatever ran first) and writes
// the bf16 dK / dV rows.  One workgroup per (split item, KV head); thread x owns 8 floats of a 128-float row.
__global__ __launch_bounds__(256) void dkv_reduce_kernel(DevGroup g, KTensors t) {
  constexpr int TK = 128;
  const ReduceItem r = g.reduce[blockIdx.x];
  const int hk = blockIdx.y;
  const int kb = g.unit_blk[r.unit];
  const int n_rows = min(TK, g.blk_len[kb] - r.tile * TK);
  const int64_t mem0 = (int64_t)g.blk_start[kb] + r.tile * TK + g.unit_moff[r.unit];
  const int col = 8 * (threadIdx.x & 15);
  for (int which = 0; which < 2; which++) {
    bf16_t* dst = which ? (bf16_t*)t.dv : (bf16_t*)t.dk;
    const int64_t st_t = which ? t.dv_st : t.dk_st, st_h = which ? t.dv_sh : t.dk_sh;
    for (int row = threadIdx.x >> 4; row < n_rows; row += 16) {
      float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
      for (int p = 0; p < r.n_parts; p++) {
        const float* src = t.part + ((((int64_t)(r.first_pslot + p) * t.hkv + hk) * 2 + which) * TK + row) * 128 + col;
        const float4 a = *(const float4*)src, b = *(const float4*)(src + 4);
        acc[0] += a.x; acc[1] += a.y; acc[2] += a.z; acc[3] += a.w;
        acc[4] += b.x; acc[5] += b.y; acc[6] += b.z; acc[7] += b.w;
      }
      uint4 o;
      o.x = pack_bf16x2(acc[0], acc[1]);
      o.y = pack_bf16x2(acc[2], acc[3]);
      o.z = pack_bf16x2(acc[4], acc[5]);
      o.w = pack_bf16x2(acc[6], acc[7]);
      *(uint4*)(dst + (mem0 + row) * st_t + (int64_t)hk * st_h + col) = o;
    }
  }
}

dcp_status_t mfma_range_bounds(const DevGroup& g, const KTensors& t, const int32_t* blk_t32, int32_t n_blocks, int32_t* qbounds,
                               hipStream_t s) {
  if (n_blocks == 0) return DCP_OK;
  hipLaunchKernelGGL(range_bounds_kernel, dim3((t.block_size + 127) / 128, n_blocks), dim3(256), 0, s, g, t, blk_t32, qbounds);
  DCP_HIP_TRY(hipGetLastError());
  return DCP_OK;
}

int mfma_dkv_tile() { return 128; }

dcp_status_t mfma_bwd_dkv(const DevGroup& g, const KTensors& t, hipStream_t s) {
  if (g.n_items == 0) return DCP_OK;
  const int grid = xcd_grid(g, t.hkv, 1);
  if (t.masked) mfma_dkv_launch_ranges(g, t, grid, s);   // the variant for per-token ranges lives in its own file
  else hipLaunchKernelGGL(mfma_dkv_kernel<false>, dim3(grid), dim3(256), 0, s, g, t);
  DCP_HIP_TRY(hipGetLastError());
  if (g.n_reduce > 0) {
    hipLaunchKernelGGL(dkv_reduce_kernel, dim3(g.n_reduce, t.hkv), dim3(256), 0, s, g, t);
    DCP_HIP_TRY(hipGetLastError());
  }
  return DCP_OK;
}

size_t mfma_dkv_part_bytes(int32_t n_pslots, int32_t hkv) { return (size_t)n_pslots * (size_t)hkv * 2 * 128 * 128 * sizeof(float); }

}  // namespace dcp
