// Do vector-ALU instructions run in the shadow of v_mfma_f32_32x32x16_bf16 (32 cycles each)?  Three answers, all in
// shader-clock cycles per loop iteration of 8 MFMAs and / or 8 x V independent v_fma_f32 (V = 2, 4, 6):
//   one wave per SIMD, the VALU instructions placed between the MFMAs of the same wave;
//   two waves per SIMD, one issuing only MFMAs, the other only VALU instructions;
//   each kind alone, for reference.
// If they overlap a mixed iteration costs max(MFMA, VALU) cycles; if they do not, the sum.
#include <hip/hip_runtime.h>
#include <cstdio>
typedef __bf16 bf8 __attribute__((ext_vector_type(8)));
typedef float f16v __attribute__((ext_vector_type(16)));

// MODE 0: MFMA only; 1: VALU only; 2: interleaved in one wave; 3: even waves MFMA only, odd waves VALU only
template <int MODE, int V>
__global__ __launch_bounds__(512) void overlap(float* out, long long* clk, int iters) {
  bf8 a, b;
  for (int e = 0; e < 8; e++) { a[e] = (__bf16)(0.001f * (threadIdx.x + e)); b[e] = (__bf16)0.5f; }
  f16v c0 = 0, c1 = 0;
  float x[8];
  for (int j = 0; j < 8; j++) x[j] = 0.001f * (threadIdx.x + j);
  const float m = 1.0001f, d = 0.0001f;
  const int wave = threadIdx.x >> 6;
  const bool do_mfma = MODE == 0 || MODE == 2 || (MODE == 3 && (wave >> 2) == 0);   // waves 0..3: one per SIMD
  const bool do_valu = MODE == 1 || MODE == 2 || (MODE == 3 && (wave >> 2) == 1);
  const long long t0 = clock64();
  if (do_mfma && do_valu) {
    for (int i = 0; i < iters; i++) {
#pragma unroll
      for (int u = 0; u < 8; u++) {
        if (u & 1) c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c1, 0, 0, 0);
        else c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c0, 0, 0, 0);
#pragma unroll
        for (int v = 0; v < V; v++) {
          // volatile asm: the compiler may neither drop nor move these across the MFMAs
          asm volatile("v_fma_f32 %0, %0, %1, %2" : "+v"(x[(u * V + v) & 7]) : "v"(m), "v"(d));
        }
      }
    }
  } else if (do_mfma) {   // a loop of its own: no branch inside
    for (int i = 0; i < iters; i++) {
#pragma unroll
      for (int u = 0; u < 8; u++) {
        if (u & 1) c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c1, 0, 0, 0);
        else c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c0, 0, 0, 0);
      }
    }
  } else {
    for (int i = 0; i < iters; i++) {
#pragma unroll
      for (int u = 0; u < 8 * V; u++) asm volatile("v_fma_f32 %0, %0, %1, %2" : "+v"(x[u & 7]) : "v"(m), "v"(d));
    }
  }
  const long long t1 = clock64();
  float s = 0;
  for (int r = 0; r < 16; r++) s += c0[r] + c1[r];
  for (int j = 0; j < 8; j++) s += x[j];
  out[blockIdx.x * blockDim.x + threadIdx.x] = s;
  if (threadIdx.x == 0 && blockIdx.x == 0) clk[0] = t1 - t0;
  if (threadIdx.x == 256 && blockIdx.x == 0) clk[1] = t1 - t0;
}

template <int MODE, int V>
double run(float* f, long long* dclk, int threads, int which = 0) {
  const int iters = 2000;
  long long h[2] = {0, 0};
  for (int rep = 0; rep < 2; rep++) {
    hipLaunchKernelGGL((overlap<MODE, V>), dim3(256), dim3(threads), 0, 0, f, dclk, iters);
    hipDeviceSynchronize();
    hipMemcpy(h, dclk, 16, hipMemcpyDeviceToHost);
  }
  return (double)h[which] / iters;
}

template <int V>
void report(float* f, long long* d) {
  printf("V = %d VALU per MFMA: MFMA alone %.0f, VALU alone %.0f, same wave %.0f, two waves: the MFMA wave %.0f and the VALU wave %.0f "
         "cycles per 8 MFMAs / 8 x V VALU\n", V,
         run<0, V>(f, d, 256), run<1, V>(f, d, 256), run<2, V>(f, d, 256), run<3, V>(f, d, 512, 0), run<3, V>(f, d, 512, 1));
}

int main() {
  long long* d; hipMalloc(&d, 64);
  float* f; hipMalloc(&f, 256 * 512 * 4);
  report<2>(f, d); report<4>(f, d); report<6>(f, d); report<8>(f, d);
  return 0;
}
