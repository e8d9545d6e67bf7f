// Generic strided fp32 GEMM for the all-fp32 configuration (a correctness configuration whose
// GEMMs are tiny and launch bound).  64x64x16 LDS tiles, 4x4 outputs per thread, plain FMAs,
// arbitrary sizes and operand strides, same epilogues as the bf16 MFMA kernel.
#include "device_utils.h"
#include "kernels.h"

namespace zpp {

struct EpiF32 {
    const float *bias, *resid, *aux;
    float *out2;
    int act, gelu_mode, accumulate;
    float accum_scale;
};

__global__ __launch_bounds__(256) void gemm_f32_kernel(int64_t M, int64_t N, int64_t K,
                                                       const float *__restrict__ A, int64_t sam, int64_t sak,
                                                       const float *__restrict__ B, int64_t sbn, int64_t sbk,
                                                       float *__restrict__ C, int64_t ldc, EpiF32 epi)
{
    __shared__ float As[16][64 + 4];
    __shared__ float Bs[16][64 + 4];
    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;
    const int64_t m0 = (int64_t)blockIdx.y * 64, n0 = (int64_t)blockIdx.x * 64;
    float acc[4][4] = {};
    for (int64_t k0 = 0; k0 < K; k0 += 16) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int e = tid + i * 256;
            int mm, kk;
            if (sak == 1) { kk = e & 15; mm = e >> 4; } else { mm = e & 63; kk = e >> 6; }
            const int64_t gm = m0 + mm, gk = k0 + kk;
            As[kk][mm] = (gm < M && gk < K) ? A[gm * sam + gk * sak] : 0.0f;
            int nn;
            if (sbk == 1) { kk = e & 15; nn = e >> 4; } else { nn = e & 63; kk = e >> 6; }
            const int64_t gn = n0 + nn;
            const int64_t gk2 = k0 + kk;
            Bs[kk][nn] = (gn < N && gk2 < K) ? B[gn * sbn + gk2 * sbk] : 0.0f;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < 16; ++kk) {
            float a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) b[j] = Bs[kk][tx * 4 + j];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] += a[i] * b[j];
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int64_t m = m0 + ty * 4 + i;
        if (m >= M) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int64_t n = n0 + tx * 4 + j;
            if (n >= N) continue;
            float v = acc[i][j];
            if (epi.bias) v += epi.bias[n];
            if (epi.resid) v += epi.resid[m * ldc + n];
            if (epi.act == ACT_DGELU_MUL) v *= gelu_bwd(epi.aux[m * ldc + n], epi.gelu_mode);
            C[m * ldc + n] = epi.accumulate ? grad_accum(C[m * ldc + n], epi.accum_scale, v) : v;
            if (epi.act == ACT_GELU_DUAL) epi.out2[m * ldc + n] = gelu_fwd(v, epi.gelu_mode);
        }
    }
}

hipError_t launch_gemm_f32(int64_t M, int64_t N, int64_t K, const float *A, int64_t sam, int64_t sak,
                           const float *B, int64_t sbn, int64_t sbk, float *C, int64_t ldc,
                           const GemmEpi &epi, hipStream_t s)
{
    if (M == 0 || N == 0) return hipSuccess;
    EpiF32 e{(const float *)epi.bias, (const float *)epi.resid, (const float *)epi.aux, (float *)epi.out2,
             epi.act, epi.gelu_mode, epi.out_f32 == 2, epi.accum_scale};
    const dim3 grid((unsigned)((N + 63) / 64), (unsigned)((M + 63) / 64));
    gemm_f32_kernel<<<grid, 256, 0, s>>>(M, N, K, A, sam, sak, B, sbn, sbk, C, ldc, e);
    return hipGetLastError();
}

}  // namespace zpp
