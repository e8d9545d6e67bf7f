// Flat-buffer passes over the ZeRO-3-style shard: materialise (stand-in for the per-unit parameter
// all-gather), gradient accumulation (stand-in for the per-unit reduce-scatter) and the fused Adam
// step (the optimizer-step task).  All three are HBM-bandwidth bound: 16-byte accesses, 64-bit
// indexing (the flat buffers exceed 4 GiB at the wide configuration), grid-stride loops.
#include "device_utils.h"
#include "kernels.h"

namespace zpp {

static inline int flat_grid(uint64_t work_items, int per_block)
{
    uint64_t blocks = (work_items + per_block - 1) / per_block;
    const uint64_t cap = 256ull * 16;  // 16 resident blocks per CU is plenty for a streaming pass
    if (blocks > cap) blocks = cap;
    if (blocks == 0) blocks = 1;
    return (int)blocks;
}

// ---------------------------------------------------------------- materialise
__global__ __launch_bounds__(256) void materialize_bf16_kernel(const float *__restrict__ P,
                                                               bf16 *__restrict__ W, uint64_t n)
{
    const uint64_t nvec = n / 8;
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < nvec; i += stride) {
        const f32x4 a = *reinterpret_cast<const f32x4 *>(P + i * 8);
        const f32x4 b = *reinterpret_cast<const f32x4 *>(P + i * 8 + 4);
        bf16x8 o;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            o[k] = (bf16)a[k];
            o[k + 4] = (bf16)b[k];
        }
        *reinterpret_cast<bf16x8 *>(W + i * 8) = o;
    }
    // ragged tail
    for (uint64_t i = nvec * 8 + (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride)
        W[i] = (bf16)P[i];
}

__global__ __launch_bounds__(256) void materialize_f32_kernel(const float *__restrict__ P,
                                                              float *__restrict__ W, uint64_t n)
{
    const uint64_t nvec = n / 4;
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < nvec; i += stride)
        *reinterpret_cast<f32x4 *>(W + i * 4) = *reinterpret_cast<const f32x4 *>(P + i * 4);
    for (uint64_t i = nvec * 4 + (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride)
        W[i] = P[i];
}

hipError_t launch_materialize(const float *P, void *W, uint64_t n, int dt, hipStream_t s)
{
    if (n == 0) return hipSuccess;
    if (dt == DT_BF16)
        materialize_bf16_kernel<<<flat_grid(n / 8 + 1, 256), 256, 0, s>>>(P, (bf16 *)W, n);
    else
        materialize_f32_kernel<<<flat_grid(n / 4 + 1, 256), 256, 0, s>>>(P, (float *)W, n);
    return hipGetLastError();
}

// Wt[c, r] = bf16(P[r, c]).  64x64 tiles through LDS; reads and writes are both row-contiguous.
__global__ __launch_bounds__(256) void transpose_cast_kernel(const float *__restrict__ P,
                                                             bf16 *__restrict__ Wt, uint64_t rows,
                                                             uint64_t cols)
{
    __shared__ float tile[64][65];
    const uint64_t r0 = (uint64_t)blockIdx.y * 64, c0 = (uint64_t)blockIdx.x * 64;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    for (int i = ty; i < 64; i += 4) {
        const uint64_t r = r0 + i, c = c0 + tx;
        tile[i][tx] = (r < rows && c < cols) ? P[r * cols + c] : 0.0f;
    }
    __syncthreads();
    for (int i = ty; i < 64; i += 4) {
        const uint64_t c = c0 + i, r = r0 + tx;
        if (c < cols && r < rows) Wt[c * rows + r] = (bf16)tile[tx][i];
    }
}

hipError_t launch_transpose_cast(const float *P, void *Wt, uint64_t rows, uint64_t cols, hipStream_t s)
{
    if (rows == 0 || cols == 0) return hipSuccess;
    dim3 grid((unsigned)((cols + 63) / 64), (unsigned)((rows + 63) / 64));
    transpose_cast_kernel<<<grid, 256, 0, s>>>(P, (bf16 *)Wt, rows, cols);
    return hipGetLastError();
}

// ---------------------------------------------------------------- accumulate
__global__ __launch_bounds__(256) void accumulate_kernel(float *__restrict__ G, const float *__restrict__ S,
                                                         uint64_t n, float scale)
{
    const uint64_t nvec = n / 4;
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < nvec; i += stride) {
        f32x4 g = *reinterpret_cast<const f32x4 *>(G + i * 4);
        const f32x4 v = *reinterpret_cast<const f32x4 *>(S + i * 4);
#pragma unroll
        for (int k = 0; k < 4; ++k) g[k] = g[k] + scale * v[k];
        *reinterpret_cast<f32x4 *>(G + i * 4) = g;
    }
    for (uint64_t i = nvec * 4 + (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride)
        G[i] = G[i] + scale * S[i];
}

hipError_t launch_accumulate(float *G, const float *S, uint64_t n, float scale, hipStream_t s)
{
    if (n == 0) return hipSuccess;
    accumulate_kernel<<<flat_grid(n / 4 + 1, 256), 256, 0, s>>>(G, S, n, scale);
    return hipGetLastError();
}

// ---------------------------------------------------------------- Adam
// Every operation is rounded on its own (no fused multiply-add) and division and square root are
// correctly rounded, so the update is the plain left-to-right evaluation of the Adam formulas in
// fp32; the pass is HBM bound, the extra roundings are free.
__device__ __forceinline__ void adam_one(float &p, float &m, float &v, float &g, const AdamArgs &a)
{
#pragma clang fp contract(off)
    float gh = a.grad_scale * g;
    if (!a.decoupled) gh = gh + a.wd * p;
    m = a.beta1 * m + a.omb1 * gh;
    v = a.beta2 * v + (a.omb2 * gh) * gh;
    const float mhat = m / a.c1;
    const float vhat = v / a.c2;
    float upd = mhat / (sqrtf(vhat) + a.eps);
    if (a.decoupled) upd = upd + a.wd * p;
    p = p - a.lr * upd;
    if (a.zero_grad) g = 0.0f;
}

__global__ __launch_bounds__(256) void adam_kernel(float *__restrict__ P, float *__restrict__ M,
                                                   float *__restrict__ V, float *__restrict__ G, uint64_t n,
                                                   AdamArgs a)
{
    const uint64_t nvec = n / 4;
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < nvec; i += stride) {
        f32x4 p = *reinterpret_cast<const f32x4 *>(P + i * 4);
        f32x4 m = *reinterpret_cast<const f32x4 *>(M + i * 4);
        f32x4 v = *reinterpret_cast<const f32x4 *>(V + i * 4);
        f32x4 g = *reinterpret_cast<const f32x4 *>(G + i * 4);
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            float pp = p[k], mm = m[k], vv = v[k], gg = g[k];
            adam_one(pp, mm, vv, gg, a);
            p[k] = pp;
            m[k] = mm;
            v[k] = vv;
            g[k] = gg;
        }
        *reinterpret_cast<f32x4 *>(P + i * 4) = p;
        *reinterpret_cast<f32x4 *>(M + i * 4) = m;
        *reinterpret_cast<f32x4 *>(V + i * 4) = v;
        if (a.zero_grad) *reinterpret_cast<f32x4 *>(G + i * 4) = g;
    }
    for (uint64_t i = nvec * 4 + (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        float pp = P[i], mm = M[i], vv = V[i], gg = G[i];
        adam_one(pp, mm, vv, gg, a);
        P[i] = pp;
        M[i] = mm;
        V[i] = vv;
        if (a.zero_grad) G[i] = gg;
    }
}

hipError_t launch_adam(float *P, float *M, float *V, float *G, uint64_t n, const AdamArgs &a, hipStream_t s)
{
    if (n == 0) return hipSuccess;
    adam_kernel<<<flat_grid(n / 4 + 1, 256), 256, 0, s>>>(P, M, V, G, n, a);
    return hipGetLastError();
}

}  // namespace zpp
