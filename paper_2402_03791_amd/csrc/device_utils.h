// Device-side helpers shared by the gfx950 kernels: element types, vector loads, wave reductions.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace zpp {

typedef __bf16 bf16;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

constexpr int kWave = 64;

__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(bf16 v) { return (float)v; }

template <class T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
// float -> bf16, round to nearest even (hardware conversion on gfx950)
template <> __device__ __forceinline__ bf16 from_f32<bf16>(float v) { return (bf16)v; }

// 16-byte vector of elements: 4 floats or 8 bf16
template <class T> struct Vec16;
template <> struct Vec16<float> {
    static constexpr int N = 4;
    f32x4 v;
    __device__ __forceinline__ float get(int i) const { return v[i]; }
    __device__ __forceinline__ void set(int i, float x) { v[i] = x; }
};
template <> struct Vec16<bf16> {
    static constexpr int N = 8;
    bf16x8 v;
    __device__ __forceinline__ float get(int i) const { return (float)v[i]; }
    __device__ __forceinline__ void set(int i, float x) { v[i] = (bf16)x; }
};

template <class T> __device__ __forceinline__ Vec16<T> load16(const T *p)
{
    Vec16<T> r;
    r.v = *reinterpret_cast<const decltype(r.v) *>(p);
    return r;
}
template <class T> __device__ __forceinline__ void store16(T *p, const Vec16<T> &r)
{
    *reinterpret_cast<decltype(r.v) *>(p) = r.v;
}

// One gradient-accumulation step g + scale * v (Section 3.1), a single fused multiply-add.  Every kernel
// that adds into the flat gradient buffer uses this form, so the separate accumulate pass and the
// weight-gradient epilogues that accumulate in place give bit-identical sums.
__device__ __forceinline__ float grad_accum(float g, float scale, float v) { return __builtin_fmaf(scale, v, g); }

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

// GeLU, tanh form, written with the logistic function: tanh(y) = 2 s(2y) - 1, so
//   gelu(u)  = 0.5 u (1 + tanh(y)) = u s(z),            z = 2y = 2c (u + a u^3),
//   gelu'(u) = s + u s (1 - s) z',                      z' = 2c (1 + 3a u^2),
// with s(z) = 1 / (1 + e^-z) on the hardware exp2 and reciprocal and 1 - s = e^-z / (1 + e^-z) (no
// cancellation): 8 and 13 instruction slots per element against about 30 for the library tanh - the GEMM
// epilogues evaluate these for every output element while the matrix cores wait.  Saturates correctly
// (e^-z = 0 or inf); absolute error of s ~1e-7.
struct GeluLogistic {
    float s, one_minus_s;
    __device__ __forceinline__ explicit GeluLogistic(float u)
    {
        const float k1 = -2.0f * 0.79788456080286535588f * 1.44269504088896340736f;  // -2c log2(e)
        const float k2 = k1 * 0.044715f;
        const float u2 = u * u;
        // e^-z, the exponent capped so that e stays finite and e * s = 1 - s holds for very negative u
        const float e = __builtin_amdgcn_exp2f(fminf(u * __builtin_fmaf(k2, u2, k1), 64.0f));
        s = __builtin_amdgcn_rcpf(1.0f + e);
        one_minus_s = e * s;
    }
};
__device__ __forceinline__ float gelu_fwd(float u, int mode)
{
    if (mode == 1) return 0.5f * u * (1.0f + erff(u * 0.70710678118654752440f));
    return u * GeluLogistic(u).s;
}
__device__ __forceinline__ float gelu_bwd(float u, int mode)
{
    if (mode == 1) {
        const float phi = expf(-0.5f * u * u) * 0.39894228040143267794f;
        return 0.5f * (1.0f + erff(u * 0.70710678118654752440f)) + u * phi;
    }
    const float c2 = 2.0f * 0.79788456080286535588f;
    const GeluLogistic g(u);
    const float zp = __builtin_fmaf(c2 * 3.0f * 0.044715f, u * u, c2);
    return g.s * __builtin_fmaf(u * g.one_minus_s, zp, 1.0f);
}
// Both at once, from one logistic function: the same operations as gelu_fwd and gelu_bwd, so the same bits.
__device__ __forceinline__ void gelu_both(float u, int mode, float &val, float &der)
{
    if (mode == 1) {
        val = gelu_fwd(u, 1);
        der = gelu_bwd(u, 1);
        return;
    }
    const float c2 = 2.0f * 0.79788456080286535588f;
    const GeluLogistic g(u);
    const float zp = __builtin_fmaf(c2 * 3.0f * 0.044715f, u * u, c2);
    val = u * g.s;
    der = g.s * __builtin_fmaf(u * g.one_minus_s, zp, 1.0f);
}

}  // namespace zpp
