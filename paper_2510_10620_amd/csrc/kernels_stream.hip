// HBM-bound streaming kernels: the LSE-carrying merge of partial outputs ("RescaleAndSum",
// Listing 1 line 6; the paper's Blockwise Reduction instruction), the backward preprocess
// delta = rowsum(dO * O), and the plain gradient sum across blocks.  Each thread moves 16-byte
// vectors; all arithmetic is fp32.
#include "device_utils.h"
#include "kernels.h"

namespace dcp {

template <typename T> struct Vec8;  // 8 elements of D per thread
template <> struct Vec8<bf16_t> {
  typedef __bf16 hb8 __attribute__((ext_vector_type(8)));
  typedef float f8 __attribute__((ext_vector_type(8)));
  typedef uint32_t u4 __attribute__((ext_vector_type(4)));
  static __device__ __forceinline__ void load(const bf16_t* p, float* f) {
    const uint4 u = *(const uint4*)p;
    const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
    for (int i = 0; i < 4; i++) { f[2 * i] = __uint_as_float(w[i] << 16); f[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u); }
  }
  // round to nearest even with the hardware conversion (two values per instruction)
  static __device__ __forceinline__ u4 pack(const float* f) {
    const f8 v = {f[0], f[1], f[2], f[3], f[4], f[5], f[6], f[7]};
    return __builtin_bit_cast(u4, __builtin_convertvector(v, hb8));
  }
  static __device__ __forceinline__ void store(bf16_t* p, const float* f) { *(u4*)p = pack(f); }
  // nontemporal: the line is not kept in the caches on its way out
  static __device__ __forceinline__ void store_nt(bf16_t* p, const float* f) { __builtin_nontemporal_store(pack(f), (u4*)p); }
};
template <> struct Vec8<float> {
  static __device__ __forceinline__ void load(const float* p, float* f) {
    const float4 a = *(const float4*)p, b = *(const float4*)(p + 4);
    f[0] = a.x; f[1] = a.y; f[2] = a.z; f[3] = a.w; f[4] = b.x; f[5] = b.y; f[6] = b.z; f[7] = b.w;
  }
  static __device__ __forceinline__ void store(float* p, const float* f) {
    *(float4*)p = make_float4(f[0], f[1], f[2], f[3]);
    *(float4*)(p + 4) = make_float4(f[4], f[5], f[6], f[7]);
  }
  static __device__ __forceinline__ void store_nt(float* p, const float* f) {
    typedef float f32x4 __attribute__((ext_vector_type(4)));
    const f32x4 a = {f[0], f[1], f[2], f[3]}, b = {f[4], f[5], f[6], f[7]};
    __builtin_nontemporal_store(a, (f32x4*)p);
    __builtin_nontemporal_store(b, (f32x4*)(p + 4));
  }
};

// grid (8 * ceil(row groups / 8), n_blocks); a workgroup merges one group of ROWS rows of one q block for all heads.
// A thread item = (row, head, 8-wide chunk of D).
// Which row group a workgroup takes is chosen by XCD: the partial LSEs (and the merged LSE) of one head are
// contiguous along the rows, so 128 / (4 ROWS) neighbouring row groups share each of their cache lines; workgroup
// ids are dealt round-robin to the 8 XCDs, each with an L2 of its own, so with row group = blockIdx.x those
// neighbours sit on 8 different XCDs, every XCD fetches the whole line for 4 ROWS of its bytes, and the merged LSE
// goes out as partial lines (measured on the share benchmark: 48 % more bytes fetched than the partials hold).  With
// XCD x taking the x-th eighth of the row groups, the groups that share a line run on one XCD, close in time.
template <typename T, int ROWS>
__global__ __launch_bounds__(256) void merge_kernel(const int32_t* __restrict__ merge_ptr, const int32_t* __restrict__ merge_idx,
                                                    const int32_t* __restrict__ blk_mem0, const int32_t* __restrict__ blk_len,
                                                    int32_t block_size, const T* __restrict__ o_part,
                                                    const float* __restrict__ lse_part, T* __restrict__ out, int64_t o_st,
                                                    int64_t o_sh, float* __restrict__ lse, int64_t q_rows, int32_t hq,
                                                    int32_t d) {
  const int b = blockIdx.y;
  const int len = blk_len[b];
  const int mem0 = blk_mem0[b];   // the block's first row in out / lse; negative: the block is not in the buffer
  if (mem0 < 0) return;
  const int per_xcd = gridDim.x >> 3;
  const int row0 = ((blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3)) * ROWS;
  if (row0 >= len) return;
  const int p0 = merge_ptr[b], p1 = merge_ptr[b + 1];
  const int chunks = d / 8;
  const int n_items = min(ROWS, len - row0) * hq * chunks;
  for (int it = threadIdx.x; it < n_items; it += blockDim.x) {
    const int c = it % chunks, h = (it / chunks) % hq, row = row0 + it / (chunks * hq);
    float m = -INFINITY;
    float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    float tot = 0.f;
    for (int p = p0; p < p1; p++) m = fmaxf(m, lse_part[((int64_t)merge_idx[p] * hq + h) * block_size + row]);
    if (m > -INFINITY) {
      for (int p = p0; p < p1; p++) {
        const int slot = merge_idx[p];
        const float lp = lse_part[((int64_t)slot * hq + h) * block_size + row];
        if (lp == -INFINITY) continue;  // weight 0: never touch the partial's values
        const float wgt = expf(lp - m);
        tot += wgt;
        float f[8];
        Vec8<T>::load(o_part + (((int64_t)slot * block_size + row) * hq + h) * d + c * 8, f);
#pragma unroll
        for (int i = 0; i < 8; i++) acc[i] = fmaf(wgt, f[i], acc[i]);
      }
      const float inv = 1.f / tot;
#pragma unroll
      for (int i = 0; i < 8; i++) acc[i] *= inv;
    }
    const int64_t tok = (int64_t)mem0 + row;
    Vec8<T>::store_nt(out + tok * o_st + (int64_t)h * o_sh + c * 8, acc);
    if (c == 0) lse[(int64_t)h * q_rows + tok] = m > -INFINITY ? m + logf(tot) : -INFINITY;
  }
}

// The merge for bf16 with D = 128 and hq a multiple of 16, the shape of the benchmark configurations.  The kernel above
// is bound by its own instructions, not by memory (index arithmetic with run-time divisors, software bf16 rounding, and
// arithmetic it does not need when a q block has no partial or only one): this one gives lane t chunk t % 16 of head
// t / 16 (+ 16 per pass) of every row, so an item's address is a sum, rounds with the hardware conversion, and has
// three paths chosen per q block: no partial (the rows are zero-filled), one partial (weight 1: the row is copied,
// or zero-filled where its LSE is -inf), several (up to kMergePreload with every load issued before the arithmetic).
static constexpr int kMergePreload = 4;   // partial slots per q block up to which all of an item's loads are issued at once
typedef __bf16 hbf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

template <int ROWS>
__global__ __launch_bounds__(256) void merge128_kernel(const int32_t* __restrict__ merge_ptr, const int32_t* __restrict__ merge_idx,
                                                       const int32_t* __restrict__ blk_mem0, const int32_t* __restrict__ blk_len,
                                                       int32_t block_size, const bf16_t* __restrict__ o_part,
                                                       const float* __restrict__ lse_part, bf16_t* __restrict__ out, int64_t o_st,
                                                       int64_t o_sh, float* __restrict__ lse, int64_t q_rows, int32_t hq) {
  const int b = blockIdx.y;
  const int len = blk_len[b];
  const int mem0 = blk_mem0[b];
  if (mem0 < 0) return;
  const int per_xcd = gridDim.x >> 3;
  const int row0 = ((blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3)) * ROWS;   // row groups by XCD, see merge_kernel
  if (row0 >= len) return;
  const int n_rows = min(ROWS, len - row0);
  const int p0 = merge_ptr[b], n_p = merge_ptr[b + 1] - p0;
  const int c = threadIdx.x & 15, hs = threadIdx.x >> 4;
  const u32x4 zero = {0u, 0u, 0u, 0u};
  if (n_p == 0) {
    for (int r = 0; r < n_rows; r++)
      for (int h = hs; h < hq; h += 16) {
        const int64_t tok = (int64_t)mem0 + row0 + r;
        __builtin_nontemporal_store(zero, (u32x4*)(out + tok * o_st + (int64_t)h * o_sh + c * 8));
        if (c == 0) lse[(int64_t)h * q_rows + tok] = -INFINITY;
      }
    return;
  }
  if (n_p == 1) {
    const int slot = merge_idx[p0];
    for (int r = 0; r < n_rows; r++)
      for (int h = hs; h < hq; h += 16) {
        const int row = row0 + r;
        const float lp = lse_part[((int64_t)slot * hq + h) * block_size + row];
        const u32x4 v = __builtin_nontemporal_load((const u32x4*)(o_part + (((int64_t)slot * block_size + row) * hq + h) * 128 + c * 8));
        const int64_t tok = (int64_t)mem0 + row;
        __builtin_nontemporal_store(lp > -INFINITY ? v : zero, (u32x4*)(out + tok * o_st + (int64_t)h * o_sh + c * 8));
        if (c == 0) lse[(int64_t)h * q_rows + tok] = lp;
      }
    return;
  }
  for (int r = 0; r < n_rows; r++)
    for (int h = hs; h < hq; h += 16) {
      const int row = row0 + r;
      float m = -INFINITY, tot = 0.f;
      f32x8 acc = {0, 0, 0, 0, 0, 0, 0, 0};
      if (n_p <= kMergePreload) {
        float lp[kMergePreload];
        u32x4 raw[kMergePreload];
#pragma unroll
        for (int k = 0; k < kMergePreload; k++)
          if (k < n_p) {
            const int slot = merge_idx[p0 + k];
            lp[k] = lse_part[((int64_t)slot * hq + h) * block_size + row];
            raw[k] = __builtin_nontemporal_load((const u32x4*)(o_part + (((int64_t)slot * block_size + row) * hq + h) * 128 + c * 8));
            m = fmaxf(m, lp[k]);
          }
#pragma unroll
        for (int k = 0; k < kMergePreload; k++)
          if (k < n_p) {
            const bool live = lp[k] > -INFINITY;
            const float wgt = live ? expf(lp[k] - m) : 0.f;   // m = -inf only if every partial is dead
            tot += wgt;
#pragma unroll
            for (int i = 0; i < 4; i++) {
              acc[2 * i] = fmaf(wgt, live ? __uint_as_float(raw[k][i] << 16) : 0.f, acc[2 * i]);
              acc[2 * i + 1] = fmaf(wgt, live ? __uint_as_float(raw[k][i] & 0xffff0000u) : 0.f, acc[2 * i + 1]);
            }
          }
      } else {
        for (int k = 0; k < n_p; k++) m = fmaxf(m, lse_part[((int64_t)merge_idx[p0 + k] * hq + h) * block_size + row]);
        for (int k = 0; k < n_p; k++) {
          const int slot = merge_idx[p0 + k];
          const float lpk = lse_part[((int64_t)slot * hq + h) * block_size + row];
          if (lpk == -INFINITY) continue;
          const float wgt = expf(lpk - m);
          tot += wgt;
          const u32x4 rw = *(const u32x4*)(o_part + (((int64_t)slot * block_size + row) * hq + h) * 128 + c * 8);
#pragma unroll
          for (int i = 0; i < 4; i++) {
            acc[2 * i] = fmaf(wgt, __uint_as_float(rw[i] << 16), acc[2 * i]);
            acc[2 * i + 1] = fmaf(wgt, __uint_as_float(rw[i] & 0xffff0000u), acc[2 * i + 1]);
          }
        }
      }
      const float inv = tot > 0.f ? 1.f / tot : 0.f;
      acc *= inv;
      const hbf16x8 ob = __builtin_convertvector(acc, hbf16x8);   // round to nearest even in hardware
      const int64_t tok = (int64_t)mem0 + row;
      __builtin_nontemporal_store(__builtin_bit_cast(u32x4, ob), (u32x4*)(out + tok * o_st + (int64_t)h * o_sh + c * 8));
      if (c == 0) lse[(int64_t)h * q_rows + tok] = tot > 0.f ? m + logf(tot) : -INFINITY;
    }
}

dcp_status_t stream_merge(const int32_t* merge_ptr, const int32_t* merge_idx, const int32_t* blk_mem0,
                          const int32_t* blk_len, int32_t n_blocks, int32_t block_size, const void* o_part,
                          const float* lse_part, void* out, int64_t o_st, int64_t o_sh, float* lse,
                          int64_t total_tokens, int32_t hq, int32_t d, int32_t dtype, hipStream_t s) {
  if (n_blocks == 0) return DCP_OK;
  if (dtype == DCP_BF16 && d == 128 && hq % 16 == 0) {
    // one row per workgroup: the most workgroups in flight measured fastest (5.4 / 5.6 / 5.9 TB/s with 4 / 2 / 1 rows)
    hipLaunchKernelGGL((merge128_kernel<1>), dim3(8 * ((block_size + 7) / 8), n_blocks), dim3(256), 0, s, merge_ptr, merge_idx,
                       blk_mem0, blk_len, block_size, (const bf16_t*)o_part, lse_part, (bf16_t*)out, o_st, o_sh, lse, total_tokens, hq);
  } else {
#define DCP_MERGE(T)                                                                                                      \
  hipLaunchKernelGGL((merge_kernel<T, 4>), dim3(8 * (((block_size + 3) / 4 + 7) / 8), n_blocks), dim3(256), 0, s, merge_ptr,     \
                     merge_idx, blk_mem0, blk_len, block_size, (const T*)o_part, lse_part, (T*)out, o_st, o_sh, lse, total_tokens, \
                     hq, d)
    if (dtype == DCP_BF16) DCP_MERGE(bf16_t);
    else DCP_MERGE(float);
  }
  DCP_HIP_TRY(hipGetLastError());
  return DCP_OK;
}

// delta[h, t] = sum_d dO[t,h,d] * O[t,h,d].  A workgroup covers kDeltaTok tokens x all heads; the
// d/8 lanes of one (token, head) reduce with shuffles; results pass through LDS so that each head
// row of delta is written in contiguous runs of kDeltaTok floats.
static constexpr int kDeltaTok = 32;

template <typename T>
__global__ __launch_bounds__(256) void delta_kernel(const T* __restrict__ o, int64_t o_st, int64_t o_sh,
                                                    const T* __restrict__ dout, int64_t do_st, int64_t do_sh,
                                                    float* __restrict__ delta, const float* __restrict__ lse,
                                                    float* __restrict__ lse2, int64_t total_tokens, int32_t hq,
                                                    int32_t d) {
  extern __shared__ float sm[];  // [hq][kDeltaTok + 1]
  const int64_t t0 = (int64_t)blockIdx.x * kDeltaTok;
  const int ntok = (int)min((int64_t)kDeltaTok, total_tokens - t0);
  const int chunks = d / 8;  // power of two <= 32 (d in 32..256)
  const int n_items = ntok * hq * chunks;
  const int n_iter = (n_items + blockDim.x - 1) / blockDim.x;
  for (int k = 0; k < n_iter; k++) {
    const int it = k * blockDim.x + threadIdx.x;
    float sum = 0.f;
    const int c = it % chunks, h = (it / chunks) % hq, tl = it / (chunks * hq);
    if (it < n_items) {
      float a[8], b[8];
      Vec8<T>::load(o + (t0 + tl) * o_st + (int64_t)h * o_sh + c * 8, a);
      Vec8<T>::load(dout + (t0 + tl) * do_st + (int64_t)h * do_sh + c * 8, b);
#pragma unroll
      for (int i = 0; i < 8; i++) sum = fmaf(a[i], b[i], sum);
    }
    for (int off = chunks / 2; off > 0; off >>= 1) sum += __shfl_xor(sum, off);
    if (it < n_items && c == 0) sm[h * (kDeltaTok + 1) + tl] = sum;
  }
  __syncthreads();
  for (int it = threadIdx.x; it < hq * ntok; it += blockDim.x) {
    const int h = it / ntok, tl = it % ntok;
    delta[(int64_t)h * total_tokens + t0 + tl] = sm[h * (kDeltaTok + 1) + tl];
    // log-sum-exp in the exp2 domain for the backward kernels; -inf (a row that saw nothing) becomes
    // the lowest finite float so that (masked score = -inf) - lse2 stays -inf and P = 0
    if (lse2) lse2[(int64_t)h * total_tokens + t0 + tl] = fmaxf(lse[(int64_t)h * total_tokens + t0 + tl] * 1.44269504088896340736f, -3.402823466e38f);
  }
}

dcp_status_t stream_delta(const void* o, int64_t o_st, int64_t o_sh, const void* dout, int64_t do_st, int64_t do_sh,
                          float* delta, const float* lse, float* lse2, int64_t total_tokens, int32_t hq, int32_t d,
                          int32_t dtype, hipStream_t s) {
  if (total_tokens == 0) return DCP_OK;
  dim3 grid((unsigned)((total_tokens + kDeltaTok - 1) / kDeltaTok)), block(256);
  const size_t sm = (size_t)hq * (kDeltaTok + 1) * sizeof(float);
  if (dtype == DCP_BF16)
    hipLaunchKernelGGL(delta_kernel<bf16_t>, grid, block, sm, s, (const bf16_t*)o, o_st, o_sh, (const bf16_t*)dout,
                       do_st, do_sh, delta, lse, lse2, total_tokens, hq, d);
  else
    hipLaunchKernelGGL(delta_kernel<float>, grid, block, sm, s, (const float*)o, o_st, o_sh, (const float*)dout, do_st,
                       do_sh, delta, lse, lse2, total_tokens, hq, d);
  DCP_HIP_TRY(hipGetLastError());
  return DCP_OK;
}

struct PartPtrs {
  const void* p[8];
};

template <typename TI, typename TO>
__global__ __launch_bounds__(256) void sum_kernel(PartPtrs parts, int32_t n_parts, TO* __restrict__ dst, int64_t n8) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n8; i += (int64_t)gridDim.x * blockDim.x) {
    float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    for (int p = 0; p < n_parts; p++) {
      float f[8];
      Vec8<TI>::load((const TI*)parts.p[p] + i * 8, f);
#pragma unroll
      for (int k = 0; k < 8; k++) acc[k] += f[k];
    }
    Vec8<TO>::store(dst + i * 8, acc);
  }
}

dcp_status_t stream_sum(const void* const* parts, int32_t n_parts, int32_t parts_dtype, void* dst, int32_t dst_dtype,
                        int64_t n, hipStream_t s) {
  if (n == 0) return DCP_OK;
  PartPtrs pp{};
  for (int i = 0; i < n_parts; i++) pp.p[i] = parts[i];
  const int64_t n8 = n / 8;
  dim3 grid((unsigned)std::min<int64_t>((n8 + 255) / 256, 256 * 16)), block(256);
  if (parts_dtype == DCP_F32 && dst_dtype == DCP_BF16)
    hipLaunchKernelGGL((sum_kernel<float, bf16_t>), grid, block, 0, s, pp, n_parts, (bf16_t*)dst, n8);
  else if (parts_dtype == DCP_F32 && dst_dtype == DCP_F32)
    hipLaunchKernelGGL((sum_kernel<float, float>), grid, block, 0, s, pp, n_parts, (float*)dst, n8);
  else if (parts_dtype == DCP_BF16 && dst_dtype == DCP_BF16)
    hipLaunchKernelGGL((sum_kernel<bf16_t, bf16_t>), grid, block, 0, s, pp, n_parts, (bf16_t*)dst, n8);
  else
    hipLaunchKernelGGL((sum_kernel<bf16_t, float>), grid, block, 0, s, pp, n_parts, (float*)dst, n8);
  DCP_HIP_TRY(hipGetLastError());
  return DCP_OK;
}

// ------------------------------------------------------------------------------------ copy
// Blockwise Copy: one workgroup per chunk of at most kCopyChunkRows rows, 16 bytes per lane and
// load, four loads in flight per lane.  HBM-bound: 2 * row_bytes algorithmic bytes per row.
__global__ __launch_bounds__(256) void copy_kernel(const int32_t* __restrict__ chunks, int64_t n_chunks,
                                                   const char* __restrict__ src, int64_t src_stride,
                                                   char* __restrict__ dst, int64_t dst_stride, int32_t vec_per_row) {
  // every byte is touched once: nontemporal loads and stores keep the copy from displacing what the attention kernels
  // that run beside it hold in the caches (5.33 -> 5.77 TB/s on the 512 MiB Q-block copy)
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  auto ld = [](const char* p, int32_t i) -> u32x4 { return __builtin_nontemporal_load((const u32x4*)p + i); };
  auto st = [](char* p, int32_t i, u32x4 v) { __builtin_nontemporal_store(v, (u32x4*)p + i); };
  for (int64_t c = blockIdx.x; c < n_chunks; c += gridDim.x) {
    const int32_t sr = chunks[3 * c], dr = chunks[3 * c + 1], nr = chunks[3 * c + 2];
    const char* sp = src + (int64_t)sr * src_stride;
    char* dp = dst + (int64_t)dr * dst_stride;
    const int32_t total = nr * vec_per_row;
    if (src_stride == (int64_t)vec_per_row * 16 && dst_stride == src_stride) {
      // rows are back to back in both buffers: one linear span
      int32_t i = threadIdx.x;
      for (; i + 768 < total; i += 1024) {
        const u32x4 a = ld(sp, i), b = ld(sp, i + 256), e = ld(sp, i + 512), f = ld(sp, i + 768);
        st(dp, i, a); st(dp, i + 256, b); st(dp, i + 512, e); st(dp, i + 768, f);
      }
      for (; i < total; i += 256) st(dp, i, ld(sp, i));
    } else {
      for (int32_t i = threadIdx.x; i < total; i += 256) {
        const int32_t r = i / vec_per_row, v = i - r * vec_per_row;
        st(dp + (int64_t)r * dst_stride, v, ld(sp + (int64_t)r * src_stride, v));
      }
    }
  }
}

dcp_status_t stream_copy(const int32_t* chunks, int64_t n_chunks, const void* src, int64_t src_stride, void* dst,
                         int64_t dst_stride, int64_t row_bytes, hipStream_t s) {
  if (n_chunks == 0) return DCP_OK;
  dim3 grid((unsigned)std::min<int64_t>(n_chunks, 256 * 64)), block(256);
  hipLaunchKernelGGL(copy_kernel, grid, block, 0, s, chunks, n_chunks, (const char*)src, src_stride, (char*)dst, dst_stride,
                     (int32_t)(row_bytes / 16));
  DCP_HIP_TRY(hipGetLastError());
  return DCP_OK;
}

}  // namespace dcp
