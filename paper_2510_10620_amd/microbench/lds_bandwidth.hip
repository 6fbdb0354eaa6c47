#include <hip/hip_runtime.h>
#include <cstdio>
typedef short s4 __attribute__((ext_vector_type(4)));
__global__ __launch_bounds__(256) void k_b128(float* out, int iters) {
  __shared__ __attribute__((aligned(16))) char smem[32768];
  int t = threadIdx.x;
  for (int i = t; i < 8192; i += 256) ((float*)smem)[i] = i;
  __syncthreads();
  const char* p = smem + (t & 63) * 16 + (t >> 6) * 4096;
  typedef float f4 __attribute__((ext_vector_type(4)));
  f4 acc[8];
  for (int u = 0; u < 8; u++) acc[u] = 0;
  for (int it = 0; it < iters; it++) {
    f4 v[8];
#pragma unroll
    for (int u = 0; u < 8; u++) v[u] = *(const volatile __attribute__((address_space(3))) f4*)((__attribute__((address_space(3))) char*)p + ((u * 1024 + it * 64) & 3071));
#pragma unroll
    for (int u = 0; u < 8; u++) acc[u] += v[u];
  }
  f4 a = acc[0] + acc[1] + acc[2] + acc[3] + acc[4] + acc[5] + acc[6] + acc[7];
  out[blockIdx.x * 256 + t] = a.x + a.y + a.z + a.w;
}
__global__ __launch_bounds__(256) void k_tr(float* out, int iters) {
  __shared__ __attribute__((aligned(16))) char smem[32768];
  int t = threadIdx.x;
  for (int i = t; i < 8192; i += 256) ((float*)smem)[i] = i;
  __syncthreads();
  typedef __attribute__((address_space(3))) s4* lp;
  const char* p = smem + (t & 63) * 8 + (t >> 6) * 4096;
  int acc = 0;
  for (int it = 0; it < iters; it++) {
#pragma unroll
    for (int u = 0; u < 8; u++) {
      s4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lp)(p + ((u * 512 + it * 64) & 3071)));
      acc += v[0] + v[1] + v[2] + v[3];
    }
  }
  out[blockIdx.x * 256 + t] = acc;
}
__global__ __launch_bounds__(256) void k_b64(float* out, int iters) {
  __shared__ __attribute__((aligned(16))) char smem[32768];
  int t = threadIdx.x;
  for (int i = t; i < 8192; i += 256) ((float*)smem)[i] = i;
  __syncthreads();
  typedef float f2 __attribute__((ext_vector_type(2)));
  const char* p = smem + (t & 63) * 8 + (t >> 6) * 4096;
  f2 acc[8];
  for (int u = 0; u < 8; u++) acc[u] = 0;
  for (int it = 0; it < iters; it++) {
    f2 v[8];
#pragma unroll
    for (int u = 0; u < 8; u++) v[u] = *(const volatile __attribute__((address_space(3))) f2*)((__attribute__((address_space(3))) char*)p + ((u * 512 + it * 64) & 3071));
#pragma unroll
    for (int u = 0; u < 8; u++) acc[u] += v[u];
  }
  f2 a = acc[0] + acc[1] + acc[2] + acc[3] + acc[4] + acc[5] + acc[6] + acc[7];
  out[blockIdx.x * 256 + t] = a.x + a.y;
}
int main() {
  float* d; hipMalloc(&d, 1024 * 256 * 4);
  hipEvent_t a, b; hipEventCreate(&a); hipEventCreate(&b);
  for (int waves = 1; waves <= 4; waves *= 2) {
    int blocks = 256 * waves;  // waves = workgroups per CU
    int iters = 20000;
    for (int rep = 0; rep < 2; rep++) {
      hipEventRecord(a); hipLaunchKernelGGL(k_b128, dim3(blocks), dim3(256), 0, 0, d, iters); hipEventRecord(b); hipEventSynchronize(b);
      float ms; hipEventElapsedTime(&ms, a, b);
      double bytes = (double)blocks * 256 * 16 * 8 * iters;
      if (rep) printf("b128: %d WG/CU: %.3f ms, %.1f B/clk/CU (at 2.4 GHz, 256 CUs)\n", waves, ms, bytes / (ms * 1e-3) / 2.4e9 / 256);
      hipEventRecord(a); hipLaunchKernelGGL(k_b64, dim3(blocks), dim3(256), 0, 0, d, iters); hipEventRecord(b); hipEventSynchronize(b);
      hipEventElapsedTime(&ms, a, b);
      bytes = (double)blocks * 256 * 8 * 8 * iters;
      if (rep) printf("b64: %d WG/CU: %.3f ms, %.1f B/clk/CU\n", waves, ms, bytes / (ms * 1e-3) / 2.4e9 / 256);
      hipEventRecord(a); hipLaunchKernelGGL(k_tr, dim3(blocks), dim3(256), 0, 0, d, iters); hipEventRecord(b); hipEventSynchronize(b);
      hipEventElapsedTime(&ms, a, b);
      bytes = (double)blocks * 256 * 8 * 8 * iters;
      if (rep) printf("tr_b64: %d WG/CU: %.3f ms, %.1f B/clk/CU\n", waves, ms, bytes / (ms * 1e-3) / 2.4e9 / 256);
    }
  }
  return 0;
}
