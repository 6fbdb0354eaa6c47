// Microbenchmark: which ingredients of the attention inner loop cost MFMA throughput (2 waves/SIMD, 256-thread WGs, 2 WG/CU)
#include <hip/hip_runtime.h>
#include <cstdio>
typedef __bf16 bf8 __attribute__((ext_vector_type(8)));
typedef float f16v __attribute__((ext_vector_type(16)));
typedef short s4 __attribute__((ext_vector_type(4)));
typedef short s8 __attribute__((ext_vector_type(8)));
__device__ __forceinline__ f16v mf(bf8 a, bf8 b, f16v c) { return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0); }
__device__ __forceinline__ int swz(int row) { return ((row & 3) << 2) | ((row >> 2) & 3); }

template <int MODE>
__global__ __launch_bounds__(256, 2) void k(float* out, int iters, float cl) {
  __shared__ __attribute__((aligned(1024))) char smem[32768];
  int t = threadIdx.x, lane = t & 63, li = lane & 31, lh = lane >> 5;
  for (int i = t; i < 8192; i += 256) ((float*)smem)[i] = (i % 7) * 0.01f;
  __syncthreads();
  bf8 qf[8];
  for (int k = 0; k < 8; k++) for (int e = 0; e < 8; e++) qf[k][e] = (__bf16)(0.01f * (k + e + lane % 3));
  f16v o[4]; for (int d = 0; d < 4; d++) o[d] = 0;
  int rm[8], tr[4][2];
  for (int ks = 0; ks < 8; ks++) rm[ks] = li * 256 + (((2 * ks + lh) ^ swz(li)) << 4);
  { int j = lane & 15, blk = lane >> 4, h = blk >> 1;
    for (int dt = 0; dt < 4; dt++) { int col = 32 * dt + 16 * (blk & 1) + 4 * (j & 3); int r0 = 4 * h + (j >> 2);
      tr[dt][0] = r0 * 256 + (((col >> 3) ^ swz(r0)) << 4) + (col & 7) * 2; tr[dt][1] = (r0 + 8) * 256 + (((col >> 3) ^ swz(r0 + 8)) << 4) + (col & 7) * 2; } }
  float m = 0.f, l = 0.f;
  typedef __attribute__((address_space(3))) s4* lp;
  for (int it = 0; it < iters; it++) {
    const char* kt = smem + (it & 1) * 8192;         // a 32-key K tile
    const char* vt = smem + 16384 + (it & 1) * 8192; // a 32-key V tile
    f16v s = 0;
    // S^T chain: 8 dependent MFMAs
#pragma unroll
    for (int ks = 0; ks < 8; ks++) {
      bf8 a;
      if (MODE & 1) a = __builtin_bit_cast(bf8, *(const uint4*)(kt + rm[ks]));   // operand from LDS
      else a = qf[(ks + 1) & 7];
      s = mf(a, qf[ks], s);
    }
    bf8 p[2];
    if (MODE & 2) {  // softmax VALU
      float mx = s[0];
#pragma unroll
      for (int r = 1; r < 16; r++) mx = fmaxf(mx, s[r]);
      mx = fmaxf(mx, __shfl_xor(mx, 32));
      m = fmaxf(m, mx * 1e-9f);
      float sum = 0;
#pragma unroll
      for (int r = 0; r < 16; r++) { float e = __builtin_amdgcn_exp2f(fmaf(s[r], cl, -m)); s[r] = e; sum += e; }
      l += sum;
    }
#pragma unroll
    for (int c = 0; c < 2; c++)
#pragma unroll
      for (int e = 0; e < 8; e++) p[c][e] = (__bf16)s[8 * c + e];
    // PV: 8 MFMAs on 4 accumulators
#pragma unroll
    for (int c = 0; c < 2; c++)
#pragma unroll
      for (int dt = 0; dt < 4; dt++) {
        bf8 a;
        if (MODE & 4) {  // transposed operand from LDS
          s4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lp)(vt + tr[dt][0] + c * 4096));
          s4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lp)(vt + tr[dt][1] + c * 4096));
          s8 v; for (int e = 0; e < 4; e++) { v[e] = lo[e]; v[4 + e] = hi[e]; }
          a = __builtin_bit_cast(bf8, v);
        } else a = qf[(dt + c) & 7];
        o[dt] = mf(a, p[c], o[dt]);
      }
    if (MODE & 8) __syncthreads();
  }
  float acc = l + m;
  for (int d = 0; d < 4; d++) for (int r = 0; r < 16; r++) acc += o[d][r];
  out[blockIdx.x * 256 + t] = acc;
}
template <int MODE> void run(float* d, const char* name) {
  hipEvent_t a, b; hipEventCreate(&a); hipEventCreate(&b);
  int iters = 20000, blocks = 512;
  for (int rep = 0; rep < 2; rep++) {
    hipEventRecord(a); hipLaunchKernelGGL(k<MODE>, dim3(blocks), dim3(256), 0, 0, d, iters, 0.01f); hipEventRecord(b); hipEventSynchronize(b);
    float ms; hipEventElapsedTime(&ms, a, b);
    double fl = (double)blocks * 4 * iters * 16 * 32768.0;
    if (rep) printf("%-44s %.3f ms  %.0f TFLOP/s (%.1f%% of 2516)\n", name, ms, fl / ms / 1e9, fl / ms / 1e9 / 25.166);
  }
}
int main() {
  float* d; hipMalloc(&d, 1024 * 256 * 4);
  run<0>(d, "mfma only (regs)");
  run<1>(d, "+ K from LDS (b128)");
  run<4>(d, "+ V^T from LDS (tr)");
  run<5>(d, "+ K and V^T from LDS");
  run<2>(d, "+ softmax VALU (regs operands)");
  run<7>(d, "+ LDS operands + softmax");
  run<15>(d, "+ LDS + softmax + barrier");
  return 0;
}
