#include "kernels.h"
namespace dcp {
int mfma_dq_tile() { return 128; }
int mfma_dkv_tile() { return 128; }
dcp_status_t mfma_bwd_dq(const DevGroup&, const KTensors&, hipStream_t) { return fail(DCP_ERR_UNSUPPORTED, "stub"); }
dcp_status_t mfma_bwd_dkv(const DevGroup&, const KTensors&, hipStream_t) { return fail(DCP_ERR_UNSUPPORTED, "stub"); }
}
