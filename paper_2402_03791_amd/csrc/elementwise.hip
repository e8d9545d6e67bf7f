// Small HBM-bound kernels: matrix transpose, rotary embedding, SwiGLU forward and backward.
#include "device_utils.h"
#include "kernels.h"

namespace zpp {

// ------------------------------------------------------------------ transpose
// out[c, r] = in[r, c], 64x64 tiles staged in LDS; both sides touch memory row-contiguously.
template <class T>
__global__ __launch_bounds__(256) void transpose_kernel(const T *__restrict__ in, int64_t R, int64_t C,
                                                        int64_t ld_in, T *__restrict__ out, int64_t ld_out)
{
    __shared__ T tile[64][64 + 2];
    const int64_t r0 = (int64_t)blockIdx.y * 64, c0 = (int64_t)blockIdx.x * 64;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    for (int i = ty; i < 64; i += 4) {
        const int64_t r = r0 + i, c = c0 + tx;
        tile[i][tx] = (r < R && c < C) ? in[r * ld_in + c] : from_f32<T>(0.0f);
    }
    __syncthreads();
    for (int i = ty; i < 64; i += 4) {
        const int64_t c = c0 + i, r = r0 + tx;
        if (c < C && r < R) out[c * ld_out + r] = tile[tx][i];
    }
}

hipError_t launch_transpose(int dt, const void *in, int64_t R, int64_t C, int64_t ld_in, void *out,
                            int64_t ld_out, hipStream_t s)
{
    if (R == 0 || C == 0) return hipSuccess;
    const dim3 grid((unsigned)((C + 63) / 64), (unsigned)((R + 63) / 64));
    if (dt == DT_BF16)
        transpose_kernel<bf16><<<grid, 256, 0, s>>>((const bf16 *)in, R, C, ld_in, (bf16 *)out, ld_out);
    else
        transpose_kernel<float><<<grid, 256, 0, s>>>((const float *)in, R, C, ld_in, (float *)out, ld_out);
    return hipGetLastError();
}

// ------------------------------------------------------------------ rotary embedding
// table[p][i] = (cos, sin)(p * base^(-2i/d)); evaluated in double so that large angles keep their phase.
__global__ void rope_table_kernel(float *__restrict__ table, int64_t seq, int64_t half, double base, double d)
{
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= seq * half) return;
    const int64_t p = idx / half, i = idx % half;
    const double theta = (double)p * pow(base, -2.0 * (double)i / d);
    table[idx * 2] = (float)cos(theta);
    table[idx * 2 + 1] = (float)sin(theta);
}

hipError_t launch_rope_table(float *table, int64_t seq, int64_t d, double base, hipStream_t s)
{
    const int64_t n = seq * (d / 2);
    if (n == 0) return hipSuccess;
    rope_table_kernel<<<(unsigned)((n + 255) / 256), 256, 0, s>>>(table, seq, d / 2, base, (double)d);
    return hipGetLastError();
}

// Rotates adjacent pairs (2i, 2i+1) of every head of the Q and K parts of qkv[T, 3h] in place.
template <class T>
__global__ __launch_bounds__(256) void rope_kernel(T *__restrict__ qkv, const float *__restrict__ table,
                                                   int64_t rows, int64_t seq, int64_t h, int64_t d, float sign)
{
    const int64_t half_row = h;  // pairs in the Q and K parts of one row: 2h/2
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= rows * half_row) return;
    const int64_t t = idx / half_row, pr = idx % half_row;  // pr indexes pairs over [Q | K]
    const int64_t col = pr * 2;                             // column inside the first 2h columns
    const int64_t i = (col % d) / 2;
    const int64_t p = t % seq;
    const float c = table[(p * (d / 2) + i) * 2], sn = sign * table[(p * (d / 2) + i) * 2 + 1];
    T *e = qkv + t * 3 * h + col;
    const float a = to_f32(e[0]), b = to_f32(e[1]);
    e[0] = from_f32<T>(a * c - b * sn);
    e[1] = from_f32<T>(a * sn + b * c);
}

hipError_t launch_rope(int dt, void *qkv, const float *table, int64_t T, int64_t seq, int64_t nh, int64_t d,
                       int sign, hipStream_t s)
{
    const int64_t h = nh * d;
    const int64_t n = T * h;
    if (n == 0) return hipSuccess;
    const unsigned grid = (unsigned)((n + 255) / 256);
    if (dt == DT_BF16)
        rope_kernel<bf16><<<grid, 256, 0, s>>>((bf16 *)qkv, table, T, seq, h, d, (float)sign);
    else
        rope_kernel<float><<<grid, 256, 0, s>>>((float *)qkv, table, T, seq, h, d, (float)sign);
    return hipGetLastError();
}

// ------------------------------------------------------------------ SwiGLU
__device__ __forceinline__ float sigmoidf_(float z) { return 1.0f / (1.0f + expf(-z)); }

template <class T>
__global__ __launch_bounds__(256) void swiglu_fwd_kernel(const T *__restrict__ gu, T *__restrict__ act,
                                                         int64_t rows, int64_t f)
{
    constexpr int VN = Vec16<T>::N;
    const int64_t nv = f / VN;
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= rows * nv) return;
    const int64_t t = idx / nv, c = (idx % nv) * VN;
    const Vec16<T> g = load16(gu + t * 2 * f + c);
    const Vec16<T> u = load16(gu + t * 2 * f + f + c);
    Vec16<T> o;
#pragma unroll
    for (int k = 0; k < VN; ++k) {
        const float gv = g.get(k);
        o.set(k, gv * sigmoidf_(gv) * u.get(k));
    }
    store16(act + t * f + c, o);
}

template <class T>
__global__ __launch_bounds__(256) void swiglu_bwd_kernel(const T *__restrict__ gu, const T *__restrict__ dact,
                                                         T *__restrict__ dgu, int64_t rows, int64_t f)
{
    constexpr int VN = Vec16<T>::N;
    const int64_t nv = f / VN;
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= rows * nv) return;
    const int64_t t = idx / nv, c = (idx % nv) * VN;
    const Vec16<T> g = load16(gu + t * 2 * f + c);
    const Vec16<T> u = load16(gu + t * 2 * f + f + c);
    const Vec16<T> da = load16(dact + t * f + c);
    Vec16<T> dg, du;
#pragma unroll
    for (int k = 0; k < VN; ++k) {
        const float gv = g.get(k), sg = sigmoidf_(gv), d = da.get(k);
        du.set(k, d * gv * sg);
        dg.set(k, d * u.get(k) * (sg + gv * sg * (1.0f - sg)));
    }
    store16(dgu + t * 2 * f + c, dg);
    store16(dgu + t * 2 * f + f + c, du);
}

hipError_t launch_swiglu_fwd(int dt, const void *gu, void *act, int64_t T, int64_t f, hipStream_t s)
{
    const int64_t n = T * (f / (dt == DT_BF16 ? 8 : 4));
    if (n == 0) return hipSuccess;
    const unsigned grid = (unsigned)((n + 255) / 256);
    if (dt == DT_BF16)
        swiglu_fwd_kernel<bf16><<<grid, 256, 0, s>>>((const bf16 *)gu, (bf16 *)act, T, f);
    else
        swiglu_fwd_kernel<float><<<grid, 256, 0, s>>>((const float *)gu, (float *)act, T, f);
    return hipGetLastError();
}

hipError_t launch_swiglu_bwd(int dt, const void *gu, const void *dact, void *dgu, int64_t T, int64_t f,
                             hipStream_t s)
{
    const int64_t n = T * (f / (dt == DT_BF16 ? 8 : 4));
    if (n == 0) return hipSuccess;
    const unsigned grid = (unsigned)((n + 255) / 256);
    if (dt == DT_BF16)
        swiglu_bwd_kernel<bf16><<<grid, 256, 0, s>>>((const bf16 *)gu, (const bf16 *)dact, (bf16 *)dgu, T, f);
    else
        swiglu_bwd_kernel<float><<<grid, 256, 0, s>>>((const float *)gu, (const float *)dact, (float *)dgu, T, f);
    return hipGetLastError();
}

}  // namespace zpp
