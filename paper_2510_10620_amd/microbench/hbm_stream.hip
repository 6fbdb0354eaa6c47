// What plain streaming kernels reach on this device, to read the HBM-bound kernels' GB/s against: read-only (sum of
// 1 GiB), write-only (fill of 1 GiB) and copy (512 MiB -> 512 MiB), 16 bytes per lane and access, U accesses in flight
// per lane, grid-stride over 2048 or 8192 workgroups of 256 threads.
#include <hip/hip_runtime.h>
#include <cstdio>

template <int U>
__global__ __launch_bounds__(256) void k_read(const uint4* __restrict__ src, long long n, unsigned* out) {
  unsigned acc = 0;
  const long long stride = (long long)gridDim.x * 256;
  long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  for (; i + (U - 1) * stride < n; i += U * stride) {
    uint4 v[U];
#pragma unroll
    for (int u = 0; u < U; u++) v[u] = src[i + u * stride];
#pragma unroll
    for (int u = 0; u < U; u++) acc += v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
  }
  for (; i < n; i += stride) { const uint4 v = src[i]; acc += v.x ^ v.y ^ v.z ^ v.w; }
  if (acc == 0x12345678u) out[0] = acc;   // never true for the test pattern; keeps the loads alive
}

template <int U>
__global__ __launch_bounds__(256) void k_write(uint4* __restrict__ dst, long long n) {
  const long long stride = (long long)gridDim.x * 256;
  const uint4 v = make_uint4(threadIdx.x, blockIdx.x, 3, 4);
  long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  for (; i + (U - 1) * stride < n; i += U * stride) {
#pragma unroll
    for (int u = 0; u < U; u++) dst[i + u * stride] = v;
  }
  for (; i < n; i += stride) dst[i] = v;
}

template <int U>
__global__ __launch_bounds__(256) void k_copy(const uint4* __restrict__ src, uint4* __restrict__ dst, long long n) {
  const long long stride = (long long)gridDim.x * 256;
  long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  for (; i + (U - 1) * stride < n; i += U * stride) {
    uint4 v[U];
#pragma unroll
    for (int u = 0; u < U; u++) v[u] = src[i + u * stride];
#pragma unroll
    for (int u = 0; u < U; u++) dst[i + u * stride] = v[u];
  }
  for (; i < n; i += stride) dst[i] = src[i];
}

template <class F>
double time_ms(F launch) {
  hipEvent_t e0, e1;
  hipEventCreate(&e0); hipEventCreate(&e1);
  launch();
  hipDeviceSynchronize();
  hipEventRecord(e0);
  for (int r = 0; r < 10; r++) launch();
  hipEventRecord(e1);
  hipEventSynchronize(e1);
  float ms = 0;
  hipEventElapsedTime(&ms, e0, e1);
  return ms / 10;
}

template <int U>
void run(uint4* a, uint4* b, unsigned* out, int grid) {
  const long long n1g = (1ll << 30) / 16, n512 = (512ll << 20) / 16;
  const double r = time_ms([&] { hipLaunchKernelGGL(k_read<U>, dim3(grid), dim3(256), 0, 0, a, n1g, out); });
  const double w = time_ms([&] { hipLaunchKernelGGL(k_write<U>, dim3(grid), dim3(256), 0, 0, a, n1g); });
  const double c = time_ms([&] { hipLaunchKernelGGL(k_copy<U>, dim3(grid), dim3(256), 0, 0, a, b, n512); });
  printf("U = %d, %d workgroups: read %.0f GB/s, write %.0f GB/s, copy %.0f GB/s (read + written)\n", U, grid,
         (1 << 30) / r / 1e6, (1 << 30) / w / 1e6, (1 << 30) / c / 1e6);
}

int main() {
  uint4 *a, *b;
  unsigned* out;
  hipMalloc(&a, 1ll << 30);
  hipMalloc(&b, 512ll << 20);
  hipMalloc(&out, 64);
  hipMemset(a, 1, 1ll << 30);
  for (int grid : {2048, 8192}) { run<1>(a, b, out, grid); run<4>(a, b, out, grid); run<8>(a, b, out, grid); }
  return 0;
}
