// Cycles per v_mfma_f32_32x32x16_bf16 when N accumulators are updated round-robin by one wave per
// SIMD (N = 1: every MFMA waits for the previous one's result as its C operand).  Counted with the
// shader clock inside the kernel, so the figure does not depend on the clock the chip settles at.
#include <hip/hip_runtime.h>
#include <cstdio>
typedef __bf16 bf8 __attribute__((ext_vector_type(8)));
typedef float f16v __attribute__((ext_vector_type(16)));

template <int N>
__global__ __launch_bounds__(256) void chains(float* out, long long* clk, int iters) {
  bf8 a, b;
  for (int e = 0; e < 8; e++) { a[e] = (__bf16)(0.001f * (threadIdx.x + e)); b[e] = (__bf16)0.5f; }
  f16v c[N];
  for (int j = 0; j < N; j++) c[j] = 0;
  const long long c0 = clock64();
  for (int i = 0; i < iters; i++) {
#pragma unroll
    for (int u = 0; u < 8; u++)
#pragma unroll
      for (int j = 0; j < N; j++) c[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c[j], 0, 0, 0);
  }
  const long long c1 = clock64();
  float s = 0;
  for (int j = 0; j < N; j++) for (int r = 0; r < 16; r++) s += c[j][r];
  out[blockIdx.x * 256 + threadIdx.x] = s;
  if (threadIdx.x == 0 && blockIdx.x == 0) clk[0] = c1 - c0;
}

template <int N>
void run(float* f, long long* d) {
  const int iters = 2000;
  long long h = 0;
  for (int rep = 0; rep < 2; rep++) {
    hipLaunchKernelGGL(chains<N>, dim3(256), dim3(256), 0, 0, f, d, iters);
    hipDeviceSynchronize();
    hipMemcpy(&h, d, 8, hipMemcpyDeviceToHost);
  }
  printf("%d accumulator(s) round-robin: %.1f cycles per MFMA (32 = pipe rate)\n", N, (double)h / ((double)iters * 8 * N));
}

int main() {
  long long* d; hipMalloc(&d, 64);
  float* f; hipMalloc(&f, 256 * 256 * 4);
  run<1>(f, d); run<2>(f, d); run<3>(f, d); run<4>(f, d); run<8>(f, d);
  return 0;
}
