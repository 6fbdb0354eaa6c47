#include <hip/hip_runtime.h>
#include <cstdio>
typedef __bf16 bf8 __attribute__((ext_vector_type(8)));
typedef float f16v __attribute__((ext_vector_type(16)));
__global__ void k(long long* out, int iters) {
  long long c0 = clock64(), w0 = wall_clock64();
  float x = threadIdx.x;
  for (int i = 0; i < iters; i++) x = x * 1.0001f + 0.5f;
  long long c1 = clock64(), w1 = wall_clock64();
  if (threadIdx.x == 0 && blockIdx.x == 0) { out[0] = c1 - c0; out[1] = w1 - w0; out[2] = (long long)x; }
}
// MFMA throughput: 4 independent accumulators per wave, 4 waves per CU
__global__ __launch_bounds__(256) void mf(float* out, int iters) {
  bf8 a, b; for (int e = 0; e < 8; e++) { a[e] = (__bf16)1.0f; b[e] = (__bf16)0.5f; }
  f16v c[4]; for (int j = 0; j < 4; j++) c[j] = 0;
  for (int i = 0; i < iters; i++) {
#pragma unroll
    for (int j = 0; j < 4; j++) c[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c[j], 0, 0, 0);
  }
  float s = 0; for (int j = 0; j < 4; j++) for (int r = 0; r < 16; r++) s += c[j][r];
  out[blockIdx.x * 256 + threadIdx.x] = s;
}
// The same loop on operands that look like data (hashed per lane and per step, roughly uniform in
// [-2, 2)): the rate under the power a real kernel draws, with the shader clock read inside the kernel.
__global__ __launch_bounds__(256) void mf_data(float* out, long long* clk, int iters) {
  unsigned h = (blockIdx.x * 256u + threadIdx.x) * 2654435761u + 12345u;
  bf8 a[4], b[4];
  for (int j = 0; j < 4; j++)
    for (int e = 0; e < 8; e++) {
      h = h * 1664525u + 1013904223u; a[j][e] = (__bf16)(((int)(h >> 8) - (1 << 23)) * (1.0f / (1 << 22)));
      h = h * 1664525u + 1013904223u; b[j][e] = (__bf16)(((int)(h >> 8) - (1 << 23)) * (1.0f / (1 << 22)));
    }
  f16v c[4]; for (int j = 0; j < 4; j++) c[j] = 0;
  long long c0 = clock64(), w0 = wall_clock64();
  for (int i = 0; i < iters; i += 4) {
#pragma unroll
    for (int u = 0; u < 4; u++)
#pragma unroll
      for (int j = 0; j < 4; j++) c[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[j], b[(j + u) & 3], c[j], 0, 0, 0);
  }
  long long c1 = clock64(), w1 = wall_clock64();
  float s = 0; for (int j = 0; j < 4; j++) for (int r = 0; r < 16; r++) s += c[j][r];
  out[blockIdx.x * 256 + threadIdx.x] = s;
  if (threadIdx.x == 0 && blockIdx.x == 0) { clk[0] = c1 - c0; clk[1] = w1 - w0; }
}
int main() {
  long long* d; hipMalloc(&d, 64); float* f; hipMalloc(&f, 2048 * 256 * 4);
  hipLaunchKernelGGL(k, 1, 64, 0, 0, d, 10000000); hipDeviceSynchronize();
  long long h[3]; hipMemcpy(h, d, 24, hipMemcpyDeviceToHost);
  int wrate = 0; hipDeviceGetAttribute(&wrate, hipDeviceAttributeWallClockRate, 0);
  printf("clock64 ticks %lld, wall ticks %lld, wall rate %d kHz -> clock64 rate %.1f MHz\n", h[0], h[1], wrate, (double)h[0] / h[1] * wrate / 1e3);
  hipEvent_t a, b; hipEventCreate(&a); hipEventCreate(&b);
  for (int wg = 1; wg <= 2; wg++) {
    int iters = 100000;
    for (int rep = 0; rep < 2; rep++) {
      hipEventRecord(a); hipLaunchKernelGGL(mf, dim3(256 * wg), dim3(256), 0, 0, f, iters); hipEventRecord(b); hipEventSynchronize(b);
      float ms; hipEventElapsedTime(&ms, a, b);
      double fl = (double)256 * wg * 4 * iters * 4 * 32768.0;
      if (rep) printf("mfma 32x32x16 bf16: %d WG/CU: %.3f ms, %.1f TFLOP/s => %.0f MHz equivalent at 4096 flop/clk/CU\n", wg, ms, fl / ms / 1e9, fl / (ms * 1e-3) / 256 / 4096 / 1e6);
    }
  }
  for (int rep = 0; rep < 3; rep++) {
    int iters = 200000;
    hipEventRecord(a); hipLaunchKernelGGL(mf_data, dim3(256), dim3(256), 0, 0, f, d, iters); hipEventRecord(b); hipEventSynchronize(b);
    float ms; hipEventElapsedTime(&ms, a, b);
    hipMemcpy(h, d, 16, hipMemcpyDeviceToHost);
    double fl = (double)256 * 4 * iters * 4 * 32768.0;
    printf("mfma on data-like operands: %.3f ms, %.1f TFLOP/s, shader clock inside the kernel %.0f MHz\n", ms, fl / ms / 1e9, (double)h[0] / h[1] * wrate / 1e3);
  }
  return 0;
}
