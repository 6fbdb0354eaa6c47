// Probe: documented gfx950 instruction semantics (ds_read_b64_tr_b16, MFMA operand layouts), device props.
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdint>
#include <vector>
#include <cmath>

typedef short s4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf8 __attribute__((ext_vector_type(8)));
typedef float f16v __attribute__((ext_vector_type(16)));
typedef float f4v __attribute__((ext_vector_type(4)));

#define CK(x) do{hipError_t e=(x); if(e!=hipSuccess){printf("HIP error %s at %d\n", hipGetErrorString(e), __LINE__); return 1;}}while(0)

__global__ void probe_tr(uint16_t* out) {
  __shared__ uint16_t lds[1024];
  int l = threadIdx.x;
  for (int i = l; i < 1024; i += 64) lds[i] = (uint16_t)i;
  __syncthreads();
  // lane l points at elements 4l..4l+3
  s4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s4 __attribute__((address_space(3)))*)(lds + 4 * l));
  for (int e = 0; e < 4; e++) out[l * 4 + e] = (uint16_t)v[e];
}

// A[32][16], B[16][32] row-major bf16 in global; C[32][32]
__global__ void probe_mfma32(const __bf16* A, const __bf16* B, float* C) {
  int l = threadIdx.x; int i = l % 32, h = l / 32;
  bf8 a, b;
  for (int e = 0; e < 8; e++) { a[e] = A[i * 16 + 8 * h + e]; b[e] = B[(8 * h + e) * 32 + i]; }
  f16v c = {0};
  c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
  for (int r = 0; r < 16; r++) { int row = 8 * (r / 4) + 4 * h + (r % 4); C[row * 32 + i] = c[r]; }
}
// A[16][32], B[32][16]; C[16][16]
__global__ void probe_mfma16(const __bf16* A, const __bf16* B, float* C) {
  int l = threadIdx.x; int i = l % 16, g = l / 16;
  bf8 a, b;
  for (int e = 0; e < 8; e++) { a[e] = A[i * 32 + 8 * g + e]; b[e] = B[(8 * g + e) * 16 + i]; }
  f4v c = {0};
  c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
  for (int r = 0; r < 4; r++) { int row = 4 * g + r; C[row * 16 + i] = c[r]; }
}

int main() {
  hipDeviceProp_t p; CK(hipGetDeviceProperties(&p, 0));
  printf("name=%s arch=%s CUs=%d clock_khz=%d lds_per_block=%zu lds_per_cu=%zu regs_per_block=%d l2=%d mem=%zu wave=%d memclk=%d buswidth=%d\n",
    p.name, p.gcnArchName, p.multiProcessorCount, p.clockRate, p.sharedMemPerBlock, p.maxSharedMemoryPerMultiProcessor, p.regsPerBlock, p.l2CacheSize, p.totalGlobalMem, p.warpSize, p.memoryClockRate, p.memoryBusWidth);
  uint16_t* d; CK(hipMalloc(&d, 256 * 2));
  hipLaunchKernelGGL(probe_tr, 1, 64, 0, 0, d);
  CK(hipDeviceSynchronize());
  uint16_t h[256]; CK(hipMemcpy(h, d, 512, hipMemcpyDeviceToHost));
  printf("ds_read_tr16_b64: lane: e0 e1 e2 e3 (value = source element index; source lane = v/4, elem = v%%4)\n");
  for (int l = 0; l < 64; l++) printf("lane %2d: %4d %4d %4d %4d\n", l, h[4*l], h[4*l+1], h[4*l+2], h[4*l+3]);
  // mfma checks
  {
    std::vector<__bf16> A(32*16), B(16*32); std::vector<float> Af(32*16), Bf(16*32);
    for (int i = 0; i < 32*16; i++) { Af[i] = (float)((i * 7) % 13 - 6); A[i] = (__bf16)Af[i]; }
    for (int i = 0; i < 16*32; i++) { Bf[i] = (float)((i * 5) % 11 - 5); B[i] = (__bf16)Bf[i]; }
    __bf16 *dA, *dB; float* dC; CK(hipMalloc(&dA, A.size()*2)); CK(hipMalloc(&dB, B.size()*2)); CK(hipMalloc(&dC, 32*32*4));
    CK(hipMemcpy(dA, A.data(), A.size()*2, hipMemcpyHostToDevice)); CK(hipMemcpy(dB, B.data(), B.size()*2, hipMemcpyHostToDevice));
    hipLaunchKernelGGL(probe_mfma32, 1, 64, 0, 0, dA, dB, dC); CK(hipDeviceSynchronize());
    std::vector<float> C(32*32); CK(hipMemcpy(C.data(), dC, 32*32*4, hipMemcpyDeviceToHost));
    int bad = 0; for (int i = 0; i < 32; i++) for (int j = 0; j < 32; j++) { float r = 0; for (int k = 0; k < 16; k++) r += Af[i*16+k]*Bf[k*32+j]; if (fabsf(r - C[i*32+j]) > 1e-3) bad++; }
    printf("mfma32x32x16 layout mismatches: %d\n", bad);
  }
  {
    std::vector<__bf16> A(16*32), B(32*16); std::vector<float> Af(16*32), Bf(32*16);
    for (int i = 0; i < 16*32; i++) { Af[i] = (float)((i * 7) % 13 - 6); A[i] = (__bf16)Af[i]; }
    for (int i = 0; i < 32*16; i++) { Bf[i] = (float)((i * 5) % 11 - 5); B[i] = (__bf16)Bf[i]; }
    __bf16 *dA, *dB; float* dC; CK(hipMalloc(&dA, A.size()*2)); CK(hipMalloc(&dB, B.size()*2)); CK(hipMalloc(&dC, 16*16*4));
    CK(hipMemcpy(dA, A.data(), A.size()*2, hipMemcpyHostToDevice)); CK(hipMemcpy(dB, B.data(), B.size()*2, hipMemcpyHostToDevice));
    hipLaunchKernelGGL(probe_mfma16, 1, 64, 0, 0, dA, dB, dC); CK(hipDeviceSynchronize());
    std::vector<float> C(16*16); CK(hipMemcpy(C.data(), dC, 16*16*4, hipMemcpyDeviceToHost));
    int bad = 0; for (int i = 0; i < 16; i++) for (int j = 0; j < 16; j++) { float r = 0; for (int k = 0; k < 32; k++) r += Af[i*32+k]*Bf[k*16+j]; if (fabsf(r - C[i*16+j]) > 1e-3) bad++; }
    printf("mfma16x16x32 layout mismatches: %d\n", bad);
  }
  return 0;
}
