// What it costs a wave to issue global_load_lds_dwordx4 (the tile copies of the attention kernels): N instructions
// back to back from one wave or from the four waves of a workgroup at once, cycles until the last is issued and
// cycles until the data has landed.  The source rows are re-read every iteration, so they come from the L2.
#include <hip/hip_runtime.h>
#include <cstdio>
__device__ __forceinline__ void dma16(unsigned voffset, const void* sbase, unsigned lds) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(voffset), "s"(sbase), "s"(lds) : "memory");
}
template <int N>
__global__ __launch_bounds__(256) void k(const char* src, long long* clk, int iters, int stride) {
  __shared__ __attribute__((aligned(1024))) char buf[65536];
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const unsigned off = (unsigned)((lane >> 4) * stride + (lane & 15) * 16);
  const unsigned l0 = (unsigned)(size_t)(__attribute__((address_space(3))) char*)buf + wave * 16384;
  const char* base = src + (size_t)blockIdx.x * 64 * stride + (size_t)wave * 16 * stride;
  long long t_issue = 0, t_wait = 0;
  for (int i = 0; i < iters; i++) {
    __syncthreads();
    const long long t0 = clock64();
#pragma unroll
    for (int u = 0; u < N; u++) dma16(off, base + (size_t)(4 * u) * stride, l0 + u * 1024);
    const long long t1 = clock64();
    __builtin_amdgcn_s_waitcnt(0 | (7 << 4) | (15 << 8));
    const long long t2 = clock64();
    t_issue += t1 - t0; t_wait += t2 - t1;
  }
  if (lane == 0 && blockIdx.x == 0) { clk[2 * wave] = t_issue; clk[2 * wave + 1] = t_wait; }
}
template <int N>
void run(const char* src, long long* d, int threads, int grid) {
  long long h[8];
  const int iters = 200;
  for (int rep = 0; rep < 2; rep++) {
    hipLaunchKernelGGL(k<N>, dim3(grid), dim3(threads), 0, 0, src, d, iters, 8192);
    hipDeviceSynchronize();
    hipMemcpy(h, d, 64, hipMemcpyDeviceToHost);
  }
  printf("%d copies per wave, %d wave(s) per workgroup, %d workgroups: issue %.0f cycles (%.1f per instruction), then wait %.0f\n", N, threads / 64, grid,
         (double)h[0] / iters, (double)h[0] / iters / N, (double)h[1] / iters);
}
int main() {
  char* src; hipMalloc(&src, 1ll << 30);
  hipMemset(src, 1, 1ll << 30);
  long long* d; hipMalloc(&d, 64);
  for (int grid : {256, 512}) {
    run<4>(src, d, 64, grid); run<8>(src, d, 64, grid); run<4>(src, d, 256, grid); run<8>(src, d, 256, grid);
  }
  return 0;
}
