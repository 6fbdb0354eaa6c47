#include <hip/hip_runtime.h>
#include <cstdio>
typedef float f4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) char* lc;
__device__ int swz(int row) { return ((row & 3) << 2) | ((row >> 2) & 3); }
template <int PAT>
__global__ __launch_bounds__(256) void k(float* out, int iters) {
  __shared__ __attribute__((aligned(1024))) char smem[65536];
  int t = threadIdx.x, lane = t & 63;
  for (int i = t; i < 16384; i += 256) ((float*)smem)[i] = i;
  __syncthreads();
  int li = lane & 31, lh = lane >> 5;
  int off[8];
  for (int ks = 0; ks < 8; ks++) {
    if (PAT == 0) off[ks] = lane * 16 + ks * 1024;                                   // contiguous
    if (PAT == 1) off[ks] = li * 256 + (((2 * ks + lh) ^ swz(li)) << 4);            // kernel's row-major fragment
    if (PAT == 2) off[ks] = li * 256 + ((2 * ks + lh) << 4);                        // no swizzle
    if (PAT == 3) off[ks] = li * 272 + ((2 * ks + lh) << 4);                        // padded rows
    if (PAT == 4) off[ks] = li * 256 + (((2 * ks + lh) ^ (li & 15)) << 4);          // plain xor swizzle
  }
  lc p = (lc)smem;
  f4 acc[8];
  for (int u = 0; u < 8; u++) acc[u] = 0;
  for (int it = 0; it < iters; it++) {
    f4 v[8];
    int o = (it & 3) * 8704;
#pragma unroll
    for (int u = 0; u < 8; u++) v[u] = *(const volatile __attribute__((address_space(3))) f4*)(p + off[u] + o);
#pragma unroll
    for (int u = 0; u < 8; u++) acc[u] += v[u];
  }
  f4 a = acc[0] + acc[1] + acc[2] + acc[3] + acc[4] + acc[5] + acc[6] + acc[7];
  out[blockIdx.x * 256 + t] = a.x + a.y + a.z + a.w;
}
template <int PAT> void run(float* d, const char* name) {
  hipEvent_t a, b; hipEventCreate(&a); hipEventCreate(&b);
  int iters = 20000, blocks = 256;
  for (int rep = 0; rep < 2; rep++) {
    hipEventRecord(a); hipLaunchKernelGGL(k<PAT>, dim3(blocks), dim3(256), 0, 0, d, iters); hipEventRecord(b); hipEventSynchronize(b);
    float ms; hipEventElapsedTime(&ms, a, b);
    double bytes = (double)blocks * 256 * 16 * 8 * iters;
    if (rep) printf("%s: %.3f ms, %.1f B/clk/CU\n", name, ms, bytes / (ms * 1e-3) / 2.4e9 / 256);
  }
}
int main() {
  float* d; hipMalloc(&d, 1024 * 256 * 4);
  run<0>(d, "contiguous"); run<1>(d, "kernel swizzle"); run<2>(d, "no swizzle"); run<3>(d, "padded 272"); run<4>(d, "xor row&15");
  return 0;
}
