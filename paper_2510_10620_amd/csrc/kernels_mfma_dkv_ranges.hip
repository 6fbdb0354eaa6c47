// The dK/dV kernel for tables with per-token ranges (RANGES or WINDOW rows), in a file of its own so that it can be
// built with another instruction-scheduling strategy than the variant for NONE / CAUSAL tables.
#include "mfma_dkv_kernel.h"

namespace dcp {

void mfma_dkv_launch_ranges(const DevGroup& g, const KTensors& t, int grid, hipStream_t s) {
  hipLaunchKernelGGL(mfma_dkv_kernel<true>, dim3(grid), dim3(256), 0, s, g, t);
}

}  // namespace dcp
