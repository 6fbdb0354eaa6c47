// Scalar (fp32 vector-ALU) kernels for blockwise attention: one thread owns one query row (forward,
// dQ) or one key row (dK/dV) of one head and walks the listed blocks key by key.  They cover the
// fp32 I/O configuration and any (dtype, D) the MFMA family does not, and compute exactly the
// steps of the block-parallel attention listing (Listing 1, line 5) with the online-softmax
// accumulation across the rows of one output unit.
#include "device_utils.h"
#include "kernels.h"

namespace dcp {

static constexpr int kTile = 64;  // rows per workgroup = one wavefront

template <typename T, int D>
__global__ __launch_bounds__(kTile) void scalar_fwd_kernel(DevGroup g, KTensors t) {
  const WorkItem w = g.items[blockIdx.x];
  const int h = blockIdx.y, hk = h / (t.hq / t.hkv);
  const int qb = g.unit_blk[w.unit];
  const int row = w.tile * kTile + threadIdx.x;
  const bool valid = row < g.blk_len[qb];
  const int i = g.blk_start[qb] + (valid ? row : 0);
  const int im = i + g.unit_moff[w.unit];   // the row's place in the Q-type buffers
  const T* qp = (const T*)t.q + (int64_t)im * t.q_st + (int64_t)h * t.q_sh;
  float q[D], acc[D];
#pragma unroll
  for (int d = 0; d < D; d++) { q[d] = Elem<T>::load(qp + d) * t.scale; acc[d] = 0.f; }
  float m = -INFINITY, l = 0.f;
  int4 r = make_int4(0, 0, 0, 0);
  if (t.masked) r = range_row(t, i, g.blk_s0[qb]);
  for (int e = g.ptr[w.unit]; e < g.ptr[w.unit + 1]; e++) {
    const int c0 = g.ent_start[e], c1 = c0 + g.ent_len[e], kind = g.ent_kind[e], km = g.ent_moff[e];
    for (int j = c0; j < c1; j++) {
      const bool vis = valid && key_visible(kind, i, j, r);
      if (!__any(vis)) continue;
      const T* kp = (const T*)t.k + (int64_t)(j + km) * t.k_st + (int64_t)hk * t.k_sh;
      const T* vp = (const T*)t.v + (int64_t)(j + km) * t.v_st + (int64_t)hk * t.v_sh;
      float s = 0.f;
#pragma unroll
      for (int d = 0; d < D; d++) s = fmaf(q[d], Elem<T>::load(kp + d), s);
      if (vis) {
        if (s > m) {
          const float c = expf(m - s);  // exp(-inf) = 0 on the first visible key
          l *= c;
#pragma unroll
          for (int d = 0; d < D; d++) acc[d] *= c;
          m = s;
        }
        const float p = expf(s - m);
        l += p;
#pragma unroll
        for (int d = 0; d < D; d++) acc[d] = fmaf(p, Elem<T>::load(vp + d), acc[d]);
      }
    }
  }
  if (!valid) return;
  const float inv = l > 0.f ? 1.f / l : 0.f;
  const float lse = l > 0.f ? m + logf(l) : -INFINITY;
  const int slot = g.unit_out[w.unit];
  T* op;
  if (slot < 0) {
    op = (T*)t.out + (int64_t)im * t.o_st + (int64_t)h * t.o_sh;
    t.lse[(int64_t)h * t.q_rows + im] = lse;
  } else {
    op = (T*)t.out + (((int64_t)slot * t.block_size + row) * t.hq + h) * D;
    t.lse[((int64_t)slot * t.hq + h) * t.block_size + row] = lse;
  }
#pragma unroll
  for (int d = 0; d < D; d++) Elem<T>::store(op + d, acc[d] * inv);
}

template <typename T, int D>
__global__ __launch_bounds__(kTile) void scalar_dq_kernel(DevGroup g, KTensors t) {
  const WorkItem w = g.items[blockIdx.x];
  const int h = blockIdx.y, hk = h / (t.hq / t.hkv);
  const int qb = g.unit_blk[w.unit];
  const int row = w.tile * kTile + threadIdx.x;
  const bool valid = row < g.blk_len[qb];
  const int i = g.blk_start[qb] + (valid ? row : 0);
  const int im = i + g.unit_moff[w.unit];
  const T* qp = (const T*)t.q + (int64_t)im * t.q_st + (int64_t)h * t.q_sh;
  const T* dop = (const T*)t.dout + (int64_t)im * t.do_st + (int64_t)h * t.do_sh;
  float q[D], dO[D], dq[D];
#pragma unroll
  for (int d = 0; d < D; d++) { q[d] = Elem<T>::load(qp + d) * t.scale; dO[d] = Elem<T>::load(dop + d); dq[d] = 0.f; }
  const float lse = t.lse[(int64_t)h * t.q_rows + im];
  const float delta = t.delta[(int64_t)h * t.q_rows + im];
  const bool row_on = valid && lse > -INFINITY;
  int4 r = make_int4(0, 0, 0, 0);
  if (t.masked) r = range_row(t, i, g.blk_s0[qb]);
  for (int e = g.ptr[w.unit]; e < g.ptr[w.unit + 1]; e++) {
    const int c0 = g.ent_start[e], c1 = c0 + g.ent_len[e], kind = g.ent_kind[e], km = g.ent_moff[e];
    for (int j = c0; j < c1; j++) {
      const bool vis = row_on && key_visible(kind, i, j, r);
      if (!__any(vis)) continue;
      const T* kp = (const T*)t.k + (int64_t)(j + km) * t.k_st + (int64_t)hk * t.k_sh;
      const T* vp = (const T*)t.v + (int64_t)(j + km) * t.v_st + (int64_t)hk * t.v_sh;
      float s = 0.f, dp = 0.f;
#pragma unroll
      for (int d = 0; d < D; d++) {
        s = fmaf(q[d], Elem<T>::load(kp + d), s);
        dp = fmaf(dO[d], Elem<T>::load(vp + d), dp);
      }
      if (vis) {
        const float ds = expf(s - lse) * (dp - delta);
#pragma unroll
        for (int d = 0; d < D; d++) dq[d] = fmaf(ds, Elem<T>::load(kp + d), dq[d]);
      }
    }
  }
  if (!valid) return;
  T* dqp = (T*)t.dq + (int64_t)im * t.dq_st + (int64_t)h * t.dq_sh;
#pragma unroll
  for (int d = 0; d < D; d++) Elem<T>::store(dqp + d, dq[d] * t.scale);
}

// One thread per key row of one KV head; sums over the query heads of the group.
template <typename T, int D>
__global__ __launch_bounds__(kTile) void scalar_dkv_kernel(DevGroup g, KTensors t) {
  const WorkItem w = g.items[blockIdx.x];
  const int hk = blockIdx.y, G = t.hq / t.hkv;
  const int kb = g.unit_blk[w.unit];
  const int row = w.tile * kTile + threadIdx.x;
  const bool valid = row < g.blk_len[kb];
  const int j = g.blk_start[kb] + (valid ? row : 0);
  const int jm = j + g.unit_moff[w.unit];   // the row's place in the KV-type buffers
  const T* kp = (const T*)t.k + (int64_t)jm * t.k_st + (int64_t)hk * t.k_sh;
  const T* vp = (const T*)t.v + (int64_t)jm * t.v_st + (int64_t)hk * t.v_sh;
  float k[D], v[D], dk[D], dv[D];
#pragma unroll
  for (int d = 0; d < D; d++) { k[d] = Elem<T>::load(kp + d); v[d] = Elem<T>::load(vp + d); dk[d] = 0.f; dv[d] = 0.f; }
  for (int hh = 0; hh < G; hh++) {
    const int h = hk * G + hh;
    for (int e = g.ptr[w.unit]; e < g.ptr[w.unit + 1]; e++) {
      const int q0 = g.ent_start[e], q1 = q0 + g.ent_len[e], kind = g.ent_kind[e], qm = g.ent_moff[e];
      for (int i = q0; i < q1; i++) {
        int4 r = make_int4(0, 0, 0, 0);
        if (kind == 2) r = range_row(t, i, g.blk_s0[kb]);   // same sequence as the key block
        const float lse = t.lse[(int64_t)h * t.q_rows + i + qm];
        const bool vis = valid && lse > -INFINITY && key_visible(kind, i, j, r);
        if (!__any(vis)) continue;
        const T* qp = (const T*)t.q + (int64_t)(i + qm) * t.q_st + (int64_t)h * t.q_sh;
        const T* dop = (const T*)t.dout + (int64_t)(i + qm) * t.do_st + (int64_t)h * t.do_sh;
        float s = 0.f, dp = 0.f;
#pragma unroll
        for (int d = 0; d < D; d++) {
          s = fmaf(Elem<T>::load(qp + d), k[d], s);
          dp = fmaf(Elem<T>::load(dop + d), v[d], dp);
        }
        if (vis) {
          const float p = expf(s * t.scale - lse);
          const float ds = p * (dp - t.delta[(int64_t)h * t.q_rows + i + qm]) * t.scale;
#pragma unroll
          for (int d = 0; d < D; d++) {
            dv[d] = fmaf(p, Elem<T>::load(dop + d), dv[d]);
            dk[d] = fmaf(ds, Elem<T>::load(qp + d), dk[d]);
          }
        }
      }
    }
  }
  if (!valid) return;
  T* dkp = (T*)t.dk + (int64_t)jm * t.dk_st + (int64_t)hk * t.dk_sh;
  T* dvp = (T*)t.dv + (int64_t)jm * t.dv_st + (int64_t)hk * t.dv_sh;
#pragma unroll
  for (int d = 0; d < D; d++) { Elem<T>::store(dkp + d, dk[d]); Elem<T>::store(dvp + d, dv[d]); }
}

bool scalar_supports(int32_t d) { return d == 32 || d == 64 || d == 128; }
int scalar_fwd_tile() { return kTile; }
int scalar_bwd_tile() { return kTile; }

#define DCP_SCALAR_DISPATCH(KERNEL, HEADS)                                                              \
  if (g.n_items == 0) return DCP_OK;                                                                    \
  dim3 grid(g.n_items, HEADS), block(kTile);                                                            \
  if (dtype == DCP_F32) {                                                                               \
    if (t.d == 32) hipLaunchKernelGGL((KERNEL<float, 32>), grid, block, 0, s, g, t);                    \
    else if (t.d == 64) hipLaunchKernelGGL((KERNEL<float, 64>), grid, block, 0, s, g, t);               \
    else hipLaunchKernelGGL((KERNEL<float, 128>), grid, block, 0, s, g, t);                             \
  } else {                                                                                              \
    if (t.d == 32) hipLaunchKernelGGL((KERNEL<bf16_t, 32>), grid, block, 0, s, g, t);                   \
    else if (t.d == 64) hipLaunchKernelGGL((KERNEL<bf16_t, 64>), grid, block, 0, s, g, t);              \
    else hipLaunchKernelGGL((KERNEL<bf16_t, 128>), grid, block, 0, s, g, t);                            \
  }                                                                                                     \
  DCP_HIP_TRY(hipGetLastError());                                                                       \
  return DCP_OK;

dcp_status_t scalar_fwd(const DevGroup& g, const KTensors& t, int32_t dtype, hipStream_t s) {
  DCP_SCALAR_DISPATCH(scalar_fwd_kernel, t.hq)
}
dcp_status_t scalar_bwd_dq(const DevGroup& g, const KTensors& t, int32_t dtype, hipStream_t s) {
  DCP_SCALAR_DISPATCH(scalar_dq_kernel, t.hq)
}
dcp_status_t scalar_bwd_dkv(const DevGroup& g, const KTensors& t, int32_t dtype, hipStream_t s) {
  DCP_SCALAR_DISPATCH(scalar_dkv_kernel, t.hkv)
}

}  // namespace dcp
