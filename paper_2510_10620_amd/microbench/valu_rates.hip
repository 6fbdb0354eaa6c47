// Shader-clock cycles per wave instruction of the vector-ALU instructions the softmax is made of, with one wave per
// SIMD and with two: what a single wave can issue, and whether a second wave adds to it.
#include <hip/hip_runtime.h>
#include <cstdio>
template <int MODE>
__global__ __launch_bounds__(512) void k(float* out, long long* clk, int iters) {
  float x[8];
  for (int j = 0; j < 8; j++) x[j] = 0.001f * (threadIdx.x + j);
  const float m = 1.0001f, d = 0.0001f;
  const long long t0 = clock64();
  for (int i = 0; i < iters; i++) {
#pragma unroll
    for (int u = 0; u < 32; u++) {
      float& r = x[u & 7];
      if (MODE == 0) asm volatile("v_fma_f32 %0, %0, %1, %2" : "+v"(r) : "v"(m), "v"(d));
      if (MODE == 1) asm volatile("v_exp_f32 %0, %0" : "+v"(r));
      if (MODE == 2) { if (u & 1) asm volatile("v_exp_f32 %0, %0" : "+v"(r)); else asm volatile("v_fma_f32 %0, %0, %1, %2" : "+v"(r) : "v"(m), "v"(d)); }
      if (MODE == 3) { if ((u & 3) == 3) asm volatile("v_exp_f32 %0, %0" : "+v"(r)); else asm volatile("v_fma_f32 %0, %0, %1, %2" : "+v"(r) : "v"(m), "v"(d)); }
      if (MODE == 4) asm volatile("v_max3_f32 %0, %0, %1, %2" : "+v"(r) : "v"(m), "v"(d));
      if (MODE == 5) asm volatile("v_cvt_pk_bf16_f32 %0, %0, %1" : "+v"(r) : "v"(m));
      if (MODE == 6) asm volatile("v_add_f32 %0, %0, %1" : "+v"(r) : "v"(d));
      if (MODE == 7) asm volatile("v_mul_f32 %0, %0, %1" : "+v"(r) : "v"(m));
    }
  }
  const long long t1 = clock64();
  float s = 0;
  for (int j = 0; j < 8; j++) s += x[j];
  out[blockIdx.x * blockDim.x + threadIdx.x] = s;
  if (threadIdx.x == 0 && blockIdx.x == 0) clk[0] = t1 - t0;
}
template <int MODE>
void run(const char* name, float* f, long long* d) {
  for (int threads : {256, 512}) {
    long long h = 0;
    for (int rep = 0; rep < 2; rep++) {
      hipLaunchKernelGGL(k<MODE>, dim3(256), dim3(threads), 0, 0, f, d, 2000);
      hipDeviceSynchronize();
      hipMemcpy(&h, d, 8, hipMemcpyDeviceToHost);
    }
    printf("%s, %d wave(s) per SIMD: %.2f cycles per instruction per wave\n", name, threads / 256, (double)h / 2000 / 32);
  }
}
int main() {
  long long* d; hipMalloc(&d, 64);
  float* f; hipMalloc(&f, 256 * 512 * 4);
  run<0>("v_fma_f32", f, d); run<1>("v_exp_f32", f, d); run<2>("exp:fma 1:1", f, d); run<3>("exp:fma 1:3", f, d);
  run<4>("v_max3_f32", f, d); run<5>("v_cvt_pk_bf16_f32", f, d); run<6>("v_add_f32", f, d); run<7>("v_mul_f32", f, d);
  return 0;
}
