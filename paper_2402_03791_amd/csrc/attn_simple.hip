// Causal attention forward and backward, one wavefront per query (or key) row, fp32 arithmetic,
// any sequence length and head dimension.  Used by the all-fp32 configuration (tiny, launch bound);
// the bf16 configurations use the MFMA kernels.  Operates on packed qkv[T, 3h] (Q | K | V,
// head-major inside each); samples of a micro-batch do not attend to each other.
#include "device_utils.h"
#include "kernels.h"

namespace zpp {

template <class T>
__global__ __launch_bounds__(64) void attn_simple_fwd_kernel(const T *__restrict__ qkv, T *__restrict__ attn,
                                                             float *__restrict__ lse, int64_t seq, int64_t nh,
                                                             int64_t d, float scale)
{
    extern __shared__ float smem[];
    float *qs = smem;       // [d]
    float *sc = smem + d;   // [seq]
    const int lane = threadIdx.x;
    const int64_t i = blockIdx.x, n = blockIdx.y, bi = blockIdx.z;
    const int64_t h = nh * d, ld = 3 * h;
    const int64_t row_i = bi * seq + i;
    for (int64_t e = lane; e < d; e += 64) qs[e] = to_f32(qkv[row_i * ld + n * d + e]);
    __syncthreads();
    float mx = -INFINITY;
    for (int64_t j = lane; j <= i; j += 64) {
        const T *kr = qkv + (bi * seq + j) * ld + h + n * d;
        float acc = 0.0f;
        for (int64_t e = 0; e < d; ++e) acc += qs[e] * to_f32(kr[e]);
        acc *= scale;
        sc[j] = acc;
        mx = fmaxf(mx, acc);
    }
    mx = wave_max(mx);
    float sum = 0.0f;
    for (int64_t j = lane; j <= i; j += 64) {
        const float p = expf(sc[j] - mx);
        sc[j] = p;
        sum += p;
    }
    sum = wave_sum(sum);
    __syncthreads();
    for (int64_t e = lane; e < d; e += 64) {
        float acc = 0.0f;
        for (int64_t j = 0; j <= i; ++j) acc += sc[j] * to_f32(qkv[(bi * seq + j) * ld + 2 * h + n * d + e]);
        attn[row_i * h + n * d + e] = from_f32<T>(acc / sum);
    }
    if (lane == 0) lse[(bi * nh + n) * seq + i] = mx + logf(sum);
}

// delta[b, nh, s] = sum_e dattn * attn  (= rowsum(dPr o Pr))
template <class T>
__global__ __launch_bounds__(64) void attn_delta_kernel(const T *__restrict__ attn, const T *__restrict__ dattn,
                                                        float *__restrict__ delta, int64_t seq, int64_t nh,
                                                        int64_t d)
{
    const int lane = threadIdx.x;
    const int64_t i = blockIdx.x, n = blockIdx.y, bi = blockIdx.z;
    const int64_t h = nh * d;
    const int64_t base = (bi * seq + i) * h + n * d;
    float acc = 0.0f;
    for (int64_t e = lane; e < d; e += 64) acc += to_f32(attn[base + e]) * to_f32(dattn[base + e]);
    acc = wave_sum(acc);
    if (lane == 0) delta[(bi * nh + n) * seq + i] = acc;
}

template <class T>
__global__ __launch_bounds__(64) void attn_simple_dq_kernel(const T *__restrict__ qkv,
                                                            const T *__restrict__ dattn,
                                                            const float *__restrict__ lse,
                                                            const float *__restrict__ delta,
                                                            T *__restrict__ dqkv, int64_t seq, int64_t nh,
                                                            int64_t d, float scale)
{
    extern __shared__ float smem[];
    float *qs = smem, *das = smem + d, *ds = smem + 2 * d;  // [d], [d], [seq]
    const int lane = threadIdx.x;
    const int64_t i = blockIdx.x, n = blockIdx.y, bi = blockIdx.z;
    const int64_t h = nh * d, ld = 3 * h;
    const int64_t row_i = bi * seq + i;
    for (int64_t e = lane; e < d; e += 64) {
        qs[e] = to_f32(qkv[row_i * ld + n * d + e]);
        das[e] = to_f32(dattn[row_i * h + n * d + e]);
    }
    __syncthreads();
    const float l = lse[(bi * nh + n) * seq + i], dl = delta[(bi * nh + n) * seq + i];
    for (int64_t j = lane; j <= i; j += 64) {
        const T *kr = qkv + (bi * seq + j) * ld + h + n * d;
        const T *vr = qkv + (bi * seq + j) * ld + 2 * h + n * d;
        float sij = 0.0f, dp = 0.0f;
        for (int64_t e = 0; e < d; ++e) {
            sij += qs[e] * to_f32(kr[e]);
            dp += das[e] * to_f32(vr[e]);
        }
        const float p = expf(sij * scale - l);
        ds[j] = p * (dp - dl);
    }
    __syncthreads();
    for (int64_t e = lane; e < d; e += 64) {
        float acc = 0.0f;
        for (int64_t j = 0; j <= i; ++j) acc += ds[j] * to_f32(qkv[(bi * seq + j) * ld + h + n * d + e]);
        dqkv[row_i * ld + n * d + e] = from_f32<T>(acc * scale);
    }
}

template <class T>
__global__ __launch_bounds__(64) void attn_simple_dkv_kernel(const T *__restrict__ qkv,
                                                             const T *__restrict__ dattn,
                                                             const float *__restrict__ lse,
                                                             const float *__restrict__ delta,
                                                             T *__restrict__ dqkv, int64_t seq, int64_t nh,
                                                             int64_t d, float scale)
{
    extern __shared__ float smem[];
    float *ks = smem, *vs = smem + d, *ps = smem + 2 * d, *dss = smem + 2 * d + seq;  // [d],[d],[seq],[seq]
    const int lane = threadIdx.x;
    const int64_t j = blockIdx.x, n = blockIdx.y, bi = blockIdx.z;
    const int64_t h = nh * d, ld = 3 * h;
    const int64_t row_j = bi * seq + j;
    for (int64_t e = lane; e < d; e += 64) {
        ks[e] = to_f32(qkv[row_j * ld + h + n * d + e]);
        vs[e] = to_f32(qkv[row_j * ld + 2 * h + n * d + e]);
    }
    __syncthreads();
    for (int64_t i = j + lane; i < seq; i += 64) {
        const T *qr = qkv + (bi * seq + i) * ld + n * d;
        const T *dar = dattn + (bi * seq + i) * h + n * d;
        float sij = 0.0f, dp = 0.0f;
        for (int64_t e = 0; e < d; ++e) {
            sij += to_f32(qr[e]) * ks[e];
            dp += to_f32(dar[e]) * vs[e];
        }
        const float p = expf(sij * scale - lse[(bi * nh + n) * seq + i]);
        ps[i] = p;
        dss[i] = p * (dp - delta[(bi * nh + n) * seq + i]);
    }
    __syncthreads();
    for (int64_t e = lane; e < d; e += 64) {
        float dk = 0.0f, dv = 0.0f;
        for (int64_t i = j; i < seq; ++i) {
            dv += ps[i] * to_f32(dattn[(bi * seq + i) * h + n * d + e]);
            dk += dss[i] * to_f32(qkv[(bi * seq + i) * ld + n * d + e]);
        }
        dqkv[row_j * ld + h + n * d + e] = from_f32<T>(dk * scale);
        dqkv[row_j * ld + 2 * h + n * d + e] = from_f32<T>(dv);
    }
}

template <class T>
static hipError_t attn_simple_fwd(const void *qkv, void *attn, float *lse, int64_t b, int64_t seq, int64_t nh,
                                  int64_t d, hipStream_t s)
{
    const dim3 grid((unsigned)seq, (unsigned)nh, (unsigned)b);
    const float scale = 1.0f / sqrtf((float)d);
    attn_simple_fwd_kernel<T><<<grid, 64, (size_t)(d + seq) * 4, s>>>((const T *)qkv, (T *)attn, lse, seq, nh, d,
                                                                      scale);
    return hipGetLastError();
}

template <class T>
static hipError_t attn_simple_bwd(const void *qkv, const void *attn, const void *dattn, const float *lse,
                                  float *delta, void *dqkv, int64_t b, int64_t seq, int64_t nh, int64_t d,
                                  hipStream_t s)
{
    const dim3 grid((unsigned)seq, (unsigned)nh, (unsigned)b);
    const float scale = 1.0f / sqrtf((float)d);
    attn_delta_kernel<T><<<grid, 64, 0, s>>>((const T *)attn, (const T *)dattn, delta, seq, nh, d);
    attn_simple_dq_kernel<T><<<grid, 64, (size_t)(2 * d + seq) * 4, s>>>((const T *)qkv, (const T *)dattn, lse,
                                                                         delta, (T *)dqkv, seq, nh, d, scale);
    attn_simple_dkv_kernel<T><<<grid, 64, (size_t)(2 * d + 2 * seq) * 4, s>>>(
        (const T *)qkv, (const T *)dattn, lse, delta, (T *)dqkv, seq, nh, d, scale);
    return hipGetLastError();
}

hipError_t launch_attn_simple_fwd(int dt, const void *qkv, void *attn, float *lse, int64_t b, int64_t seq,
                                  int64_t nh, int64_t d, hipStream_t s)
{
    if (b * seq == 0) return hipSuccess;
    return dt == DT_BF16 ? attn_simple_fwd<bf16>(qkv, attn, lse, b, seq, nh, d, s)
                         : attn_simple_fwd<float>(qkv, attn, lse, b, seq, nh, d, s);
}

hipError_t launch_attn_simple_bwd(int dt, const void *qkv, const void *attn, const void *dattn,
                                  const float *lse, float *delta, void *dqkv, int64_t b, int64_t seq,
                                  int64_t nh, int64_t d, hipStream_t s)
{
    if (b * seq == 0) return hipSuccess;
    return dt == DT_BF16 ? attn_simple_bwd<bf16>(qkv, attn, dattn, lse, delta, dqkv, b, seq, nh, d, s)
                         : attn_simple_bwd<float>(qkv, attn, dattn, lse, delta, dqkv, b, seq, nh, d, s);
}

}  // namespace zpp
