// placeholder until the MFMA attention kernels land
#include "device_utils.h"
#include "kernels.h"
namespace zpp {
bool attn_mfma_supported(int64_t, int64_t) { return false; }
hipError_t launch_attn_fwd(int, const void *, void *, float *, int64_t, int64_t, int64_t, int64_t, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_attn_bwd(int, const void *, const void *, const void *, const float *, float *, void *, int64_t, int64_t, int64_t, int64_t, hipStream_t) { return hipErrorNotSupported; }
}
