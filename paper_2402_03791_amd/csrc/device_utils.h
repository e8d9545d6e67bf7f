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

// tanh(y) = 1 - 2 / (1 + e^(2y)) on the hardware exp2 and reciprocal (about 10 instruction slots against
// about 30 for the library routine; the GEMM epilogues evaluate it for every output element while the
// matrix cores wait).  Saturates correctly to +-1; absolute error ~1e-7, which the GeLU forms below
// multiply by at most |u|/2.
__device__ __forceinline__ float fast_tanh(float y)
{
    const float e = __builtin_amdgcn_exp2f(y * 2.88539008177792681472f);  // e^(2y)
    return 1.0f - 2.0f * __builtin_amdgcn_rcpf(1.0f + e);
}
__device__ __forceinline__ float gelu_fwd(float u, int mode)
{
    if (mode == 1) return 0.5f * u * (1.0f + erff(u * 0.70710678118654752440f));
    const float c = 0.79788456080286535588f;
    return 0.5f * u * (1.0f + fast_tanh(c * (u + 0.044715f * u * u * u)));
}
__device__ __forceinline__ float gelu_bwd(float u, int mode)
{
    if (mode == 1) {
        const float phi = expf(-0.5f * u * u) * 0.39894228040143267794f;
        return 0.5f * (1.0f + erff(u * 0.70710678118654752440f)) + u * phi;
    }
    const float c = 0.79788456080286535588f;
    const float th = fast_tanh(c * (u + 0.044715f * u * u * u));
    return 0.5f * (1.0f + th) + 0.5f * u * (1.0f - th * th) * c * (1.0f + 3.0f * 0.044715f * u * u);
}

}  // namespace zpp
