// An entry point for callers that may not allocate device memory (code under HIP graph capture, tight
// serving loops, harnesses that forbid hipMalloc): the attention backward of zpp_op_attention_bwd with
// its per-query scratch (delta = rowsum(dO o O) and a scaled log-sum-exp, 2 * b * nh * seq floats) in a file-scope
// device array
// instead of a caller-supplied buffer.  Same kernels as zpp_op_attention_bwd.
#include "../../include/zpp_ops.h"
#include "kernels.h"
#include "stage_internal.h"

#include <mutex>

namespace zpp {
hipError_t launch_attn_simple_bwd(int dt, const void *qkv, const void *attn, const void *dattn,
                                  const float *lse, float *delta, void *dqkv, int64_t b, int64_t seq,
                                  int64_t nh, int64_t d, hipStream_t s);
}

namespace {

// 8 MiB per device that runs this library, held until the process ends.
constexpr uint64_t kScratchRows = 1ull << 20;        // queries (b * nh * seq) a call may have
constexpr uint64_t kScratchFloats = 2 * kScratchRows;  // two floats of scratch per query
static __device__ __align__(256) float scratch[kScratchFloats];

// In host code `scratch` is only a handle of the symbol, not a device address: each device has its own copy
// of the array at its own address, looked up once per device and kept here.
constexpr int kMaxDevices = 64;
std::mutex g_mu;
float *g_scratch_ptr[kMaxDevices] = {};

zpp_status scratch_of_current_device(float **out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return zpp::set_error(ZPP_ERR_DEVICE, "hipGetDevice: %s", hipGetErrorString(e));
    if (dev < 0 || dev >= kMaxDevices) return zpp::set_error(ZPP_ERR_UNSUPPORTED, "device ordinal %d out of range", dev);
    std::lock_guard<std::mutex> lock(g_mu);
    if (!g_scratch_ptr[dev]) {
        float *p = nullptr;
        e = hipGetSymbolAddress((void **)&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p)
            return zpp::set_error(ZPP_ERR_DEVICE, "hipGetSymbolAddress(scratch): %s", hipGetErrorString(e));
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return ZPP_OK;
}

}  // namespace

extern "C" {

uint64_t zpp_op_attention_bwd_noalloc_max_rows(void) { return kScratchRows; }

zpp_status zpp_op_attention_bwd_noalloc(int32_t dtype, int32_t impl, const void *qkv, const void *attn,
                                        const void *dattn, const float *lse, void *dqkv, int64_t b, int64_t seq,
                                        int64_t nh, int64_t d, void *hip_stream)
{
    using namespace zpp;
    if (!qkv || !attn || !dattn || !lse || !dqkv) return set_error(ZPP_ERR_ARG, "NULL pointer");
    if (b <= 0 || seq <= 0 || nh <= 0 || d <= 0 || b > 65535 || nh > 65535) return set_error(ZPP_ERR_ARG, "bad sizes");
    if ((uint64_t)b * (uint64_t)nh > kScratchRows || (uint64_t)b * (uint64_t)nh * (uint64_t)seq > kScratchRows)
        return set_error(ZPP_ERR_WORKSPACE, "b * nh * seq = %llu exceeds the static scratch of %llu rows: use "
                                            "zpp_op_attention_bwd with a buffer of your own",
                         (unsigned long long)((uint64_t)b * nh * seq), (unsigned long long)kScratchRows);
    float *delta = nullptr;
    if (zpp_status st = scratch_of_current_device(&delta)) return st;
    hipStream_t s = (hipStream_t)hip_stream;
    hipError_t e;
    if (impl == 1) {
        if (dtype != ZPP_DTYPE_BF16 || !attn_mfma_supported(seq, d))
            return set_error(ZPP_ERR_UNSUPPORTED, "MFMA attention needs bf16, d = 128 and seq %% 128 == 0");
        e = launch_attn_bwd(DT_BF16, qkv, attn, dattn, lse, delta, dqkv, b, seq, nh, d, s);
    } else {
        if ((2 * d + 2 * seq) * 4 > 64 * 1024) return set_error(ZPP_ERR_UNSUPPORTED, "sequence too long");
        e = launch_attn_simple_bwd(dtype == ZPP_DTYPE_BF16 ? DT_BF16 : DT_F32, qkv, attn, dattn, lse, delta, dqkv, b,
                                   seq, nh, d, s);
    }
    if (e != hipSuccess) return set_error(ZPP_ERR_DEVICE, "attention backward launch: %s", hipGetErrorString(e));
    return ZPP_OK;
}

}  // extern "C"
