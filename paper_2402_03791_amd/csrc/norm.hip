// LayerNorm / RMSNorm forward and backward, and the column reductions that give the gradients of
// gains, offsets and biases.  One wavefront per row with wave-level reductions; statistics and all
// arithmetic in fp32, storage in the compute dtype.  HBM bound.
#include "device_utils.h"
#include "kernels.h"

#include <climits>
#include <type_traits>

namespace zpp {

constexpr int kRowsPerBlock = 4;  // 4 waves of 64 lanes

// A lane's share of a row is the 16-byte vectors lane, lane + 64, ...  Rows of up to 64 * RV vectors (RV = 4, 8 or
// 16: up to 8192 bf16 or 4096 fp32 elements) are read once and kept in registers; longer rows (RV = 0) are read
// again in every pass.  Either way a lane visits its vectors in ascending order, so the sums are the same bits.
// (Forward only: 20.6 -> 15.8 us per launch of 4096 rows x 4096.  The backward row part with its two operands
// per row held the same way needs 185 registers, and the column part of the same launch then runs at two waves
// per SIMD: 41.5 -> 53 us.)
constexpr int kRowVecsMax = 16;
static int row_vecs(int64_t nv)
{
    for (int rv = 4; rv <= kRowVecsMax; rv *= 2)
        if (nv <= 64 * rv) return rv;
    return 0;
}

template <int RV, class F>
__device__ __forceinline__ void for_each_vec(int lane, int64_t nv, F f)
{
    if constexpr (RV > 0) {
#pragma unroll
        for (int i = 0; i < RV; ++i) {
            const int64_t c = lane + 64 * i;
            if (c < nv) f(i, c);
        }
    } else {
        for (int64_t c = lane; c < nv; c += 64) f(0, c);
    }
}

// ------------------------------------------------------------------ forward
template <class T, int KIND, int RV>
__global__ __launch_bounds__(256) void norm_fwd_kernel(const T *__restrict__ x, const T *__restrict__ gamma,
                                                       const T *__restrict__ beta, int64_t rows, int64_t h,
                                                       float eps, T *__restrict__ n, float *__restrict__ mean,
                                                       float *__restrict__ rstd, T *__restrict__ xcopy)
{
    constexpr int VN = Vec16<T>::N;
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * kRowsPerBlock + (threadIdx.x >> 6);
    if (row >= rows) return;
    const T *xr = x + row * h;
    const int64_t nv = h / VN;
    Vec16<T> buf[RV > 0 ? RV : 1];
    if constexpr (RV > 0) for_each_vec<RV>(lane, nv, [&](int i, int64_t c) { buf[i] = load16(xr + c * VN); });
    auto xv = [&](int i, int64_t c) -> Vec16<T> {
        if constexpr (RV > 0) return buf[i];
        else return load16(xr + c * VN);
    };
    float mu = 0.0f;
    if (KIND == NORM_LAYER) {
        float s = 0.0f;
        for_each_vec<RV>(lane, nv, [&](int i, int64_t c) {
            const Vec16<T> v = xv(i, c);
#pragma unroll
            for (int k = 0; k < VN; ++k) s += v.get(k);
        });
        mu = wave_sum(s) / (float)h;
    }
    float q = 0.0f;
    for_each_vec<RV>(lane, nv, [&](int i, int64_t c) {
        const Vec16<T> v = xv(i, c);
#pragma unroll
        for (int k = 0; k < VN; ++k) {
            const float dlt = v.get(k) - mu;
            q += dlt * dlt;
        }
    });
    const float var = wave_sum(q) / (float)h;
    const float rs = 1.0f / sqrtf(var + eps);
    if (lane == 0) {
        if (mean) mean[row] = mu;
        rstd[row] = rs;
    }
    for_each_vec<RV>(lane, nv, [&](int i, int64_t c) {
        const Vec16<T> v = xv(i, c);
        const Vec16<T> g = load16(gamma + c * VN);
        Vec16<T> o;
        if (KIND == NORM_LAYER) {
            const Vec16<T> b = load16(beta + c * VN);
#pragma unroll
            for (int k = 0; k < VN; ++k) o.set(k, g.get(k) * ((v.get(k) - mu) * rs) + b.get(k));
        } else {
#pragma unroll
            for (int k = 0; k < VN; ++k) o.set(k, g.get(k) * (v.get(k) * rs));
        }
        store16(n + row * h + c * VN, o);
        if (xcopy) store16(xcopy + row * h + c * VN, v);
    });
}

hipError_t launch_norm_fwd(int dt, int kind, const void *x, const void *gamma, const void *beta, int64_t T,
                           int64_t h, float eps, void *n, float *mean, float *rstd, void *xcopy,
                           hipStream_t s)
{
    if (T == 0) return hipSuccess;
    const dim3 grid((unsigned)((T + kRowsPerBlock - 1) / kRowsPerBlock));
    const int rv = row_vecs(h / (dt == DT_BF16 ? 8 : 4));
#define ZPP_LAUNCH2(TT, KK, RR)                                                                              \
    norm_fwd_kernel<TT, KK, RR><<<grid, 256, 0, s>>>((const TT *)x, (const TT *)gamma, (const TT *)beta, T, h, \
                                                     eps, (TT *)n, mean, rstd, (TT *)xcopy)
#define ZPP_LAUNCH(TT, KK)                          \
    do {                                            \
        if (rv == 4) ZPP_LAUNCH2(TT, KK, 4);        \
        else if (rv == 8) ZPP_LAUNCH2(TT, KK, 8);   \
        else if (rv == 16) ZPP_LAUNCH2(TT, KK, 16); \
        else ZPP_LAUNCH2(TT, KK, 0);                \
    } while (0)
    if (dt == DT_BF16) {
        if (kind == NORM_LAYER) ZPP_LAUNCH(bf16, NORM_LAYER); else ZPP_LAUNCH(bf16, NORM_RMS);
    } else {
        if (kind == NORM_LAYER) ZPP_LAUNCH(float, NORM_LAYER); else ZPP_LAUNCH(float, NORM_RMS);
    }
#undef ZPP_LAUNCH
#undef ZPP_LAUNCH2
    return hipGetLastError();
}

// ------------------------------------------------------------------ backward (row part)
// ghat = dn*gamma; LayerNorm: dx = (ghat - mean(ghat) - xhat*mean(ghat*xhat))*rstd
//                  RMSNorm:   dx = (ghat - xhat*mean(ghat*xhat))*rstd          (+ resid)
template <class T, int KIND>
__device__ __forceinline__ void norm_bwd_rows(const T *__restrict__ dn, const T *__restrict__ x,
                                              const float *__restrict__ mean, const float *__restrict__ rstd,
                                              const T *__restrict__ gamma, const T *__restrict__ resid,
                                              T *__restrict__ dx, int64_t rows, int64_t h, int64_t block)
{
    constexpr int VN = Vec16<T>::N;
    const int lane = threadIdx.x & 63;
    const int64_t row = block * kRowsPerBlock + (threadIdx.x >> 6);
    if (row >= rows) return;
    const int64_t nv = h / VN;
    const float mu = (KIND == NORM_LAYER) ? mean[row] : 0.0f;
    const float rs = rstd[row];
    float s1 = 0.0f, s2 = 0.0f;
    for (int64_t c = lane; c < nv; c += 64) {
        const Vec16<T> d = load16(dn + row * h + c * VN);
        const Vec16<T> v = load16(x + row * h + c * VN);
        const Vec16<T> g = load16(gamma + c * VN);
#pragma unroll
        for (int k = 0; k < VN; ++k) {
            const float gh = d.get(k) * g.get(k);
            s1 += gh;
            s2 += gh * ((v.get(k) - mu) * rs);
        }
    }
    const float m1 = (KIND == NORM_LAYER) ? wave_sum(s1) / (float)h : 0.0f;
    const float m2 = wave_sum(s2) / (float)h;
    for (int64_t c = lane; c < nv; c += 64) {
        const Vec16<T> d = load16(dn + row * h + c * VN);
        const Vec16<T> v = load16(x + row * h + c * VN);
        const Vec16<T> g = load16(gamma + c * VN);
        Vec16<T> o;
        if (resid) {
            const Vec16<T> r = load16(resid + row * h + c * VN);
#pragma unroll
            for (int k = 0; k < VN; ++k) {
                const float xh = (v.get(k) - mu) * rs;
                o.set(k, r.get(k) + (d.get(k) * g.get(k) - m1 - xh * m2) * rs);
            }
        } else {
#pragma unroll
            for (int k = 0; k < VN; ++k) {
                const float xh = (v.get(k) - mu) * rs;
                o.set(k, (d.get(k) * g.get(k) - m1 - xh * m2) * rs);
            }
        }
        store16(dx + row * h + c * VN, o);
    }
}

template <class T, int KIND>
__global__ __launch_bounds__(256) void norm_bwd_kernel(const T *__restrict__ dn, const T *__restrict__ x,
                                                       const float *__restrict__ mean,
                                                       const float *__restrict__ rstd,
                                                       const T *__restrict__ gamma, const T *__restrict__ resid,
                                                       T *__restrict__ dx, int64_t rows, int64_t h)
{
    norm_bwd_rows<T, KIND>(dn, x, mean, rstd, gamma, resid, dx, rows, h, blockIdx.x);
}

hipError_t launch_norm_bwd(int dt, int kind, const void *dn, const void *x, const float *mean,
                           const float *rstd, const void *gamma, const void *resid, void *dx, int64_t T,
                           int64_t h, hipStream_t s)
{
    if (T == 0) return hipSuccess;
    const dim3 grid((unsigned)((T + kRowsPerBlock - 1) / kRowsPerBlock));
#define ZPP_LAUNCH(TT, KK)                                                                              \
    norm_bwd_kernel<TT, KK><<<grid, 256, 0, s>>>((const TT *)dn, (const TT *)x, mean, rstd,             \
                                                 (const TT *)gamma, (const TT *)resid, (TT *)dx, T, h)
    if (dt == DT_BF16) {
        if (kind == NORM_LAYER) ZPP_LAUNCH(bf16, NORM_LAYER); else ZPP_LAUNCH(bf16, NORM_RMS);
    } else {
        if (kind == NORM_LAYER) ZPP_LAUNCH(float, NORM_LAYER); else ZPP_LAUNCH(float, NORM_RMS);
    }
#undef ZPP_LAUNCH
    return hipGetLastError();
}

// ------------------------------------------------------------------ column reductions
// Stage 1: grid (ceil(C/64), RC); a block reduces kColRows rows x 64 columns to one partial row.
// Stage 2: sums the RC partial rows in a fixed order, so results are run-to-run identical.
constexpr int kColRows = 128;

uint64_t colreduce_scratch_floats(int64_t T, int64_t C)
{
    const int64_t rc = (T + kColRows - 1) / kColRows;
    return (uint64_t)(2 * rc * C);
}

template <class T, int MODE>
__device__ __forceinline__ void colreduce_tile(const T *__restrict__ a, const T *__restrict__ x,
                                               const float *__restrict__ mean, const float *__restrict__ rstd,
                                               int64_t rows, int64_t C, int64_t ld, float *__restrict__ partial,
                                               int bx, int by, int rc)
{
    __shared__ float red0[4][64];
    __shared__ float red1[4][64];
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    const int64_t c = (int64_t)bx * 64 + tx;
    const int64_t r0 = (int64_t)by * kColRows;
    const int64_t r1 = (r0 + kColRows < rows) ? r0 + kColRows : rows;
    float s0 = 0.0f, s1 = 0.0f;
    if (c < C) {
        for (int64_t r = r0 + ty; r < r1; r += 4) {
            const float av = to_f32(a[r * ld + c]);
            if (MODE == COLRED_SUM) {
                s0 += av;
            } else if (MODE == COLRED_LAYERNORM) {
                s0 += av * ((to_f32(x[r * ld + c]) - mean[r]) * rstd[r]);
                s1 += av;
            } else {
                s0 += av * (to_f32(x[r * ld + c]) * rstd[r]);
            }
        }
    }
    red0[ty][tx] = s0;
    red1[ty][tx] = s1;
    __syncthreads();
    if (ty == 0 && c < C) {
        partial[(int64_t)by * C + c] = (red0[0][tx] + red0[1][tx]) + (red0[2][tx] + red0[3][tx]);
        if (MODE == COLRED_LAYERNORM)
            partial[((int64_t)rc + by) * C + c] = (red1[0][tx] + red1[1][tx]) + (red1[2][tx] + red1[3][tx]);
    }
}

template <class T, int MODE>
__global__ __launch_bounds__(256) void colreduce_stage1(const T *__restrict__ a, const T *__restrict__ x,
                                                        const float *__restrict__ mean,
                                                        const float *__restrict__ rstd, int64_t rows, int64_t C,
                                                        int64_t ld, float *__restrict__ partial)
{
    colreduce_tile<T, MODE>(a, x, mean, rstd, rows, C, ld, partial, blockIdx.x, blockIdx.y, gridDim.y);
}

// The first level of the gain/offset reduction of a norm for bf16 matrices whose width is a multiple of 512, with
// 16-byte loads: a work-group takes kColRows rows x 512 columns, a lane eight adjacent columns, the four waves every
// fourth row; the four partial sums per column meet in LDS and one partial row (two for LayerNorm) goes out, in the
// layout of colreduce_tile.  (With one 2-byte element per lane the column part of the launch below cost more
// than its row part.)
template <int KIND>
__device__ __forceinline__ void norm_colreduce_wide_tile(const bf16 *__restrict__ dn, const bf16 *__restrict__ x,
                                                         const float *__restrict__ mean, const float *__restrict__ rstd,
                                                         int64_t rows, int64_t C, float *__restrict__ partial, int bx,
                                                         int by, int rc)
{
    __shared__ float red[2][4][512];
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    const int64_t c = (int64_t)bx * 512 + tx * 8;
    const int64_t r0 = (int64_t)by * kColRows;
    const int64_t r1 = (r0 + kColRows < rows) ? r0 + kColRows : rows;
    float s0[8], s1[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) s0[k] = s1[k] = 0.0f;
    for (int64_t r = r0 + ty; r < r1; r += 4) {
        const bf16x8 d = *reinterpret_cast<const bf16x8 *>(dn + r * C + c);
        const bf16x8 v = *reinterpret_cast<const bf16x8 *>(x + r * C + c);
        const float mu = KIND == NORM_LAYER ? mean[r] : 0.0f, rs = rstd[r];
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const float dk = (float)d[k];
            s0[k] += dk * (((float)v[k] - mu) * rs);
            s1[k] += dk;
        }
    }
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        red[0][ty][tx * 8 + k] = s0[k];
        if (KIND == NORM_LAYER) red[1][ty][tx * 8 + k] = s1[k];
    }
    __syncthreads();
    for (int i = threadIdx.x; i < 512; i += 256) {
        const int64_t at = (int64_t)by * C + (int64_t)bx * 512 + i;
        partial[at] = (red[0][0][i] + red[0][1][i]) + (red[0][2][i] + red[0][3][i]);
        if (KIND == NORM_LAYER) partial[(int64_t)rc * C + at] = (red[1][0][i] + red[1][1][i]) + (red[1][2][i] + red[1][3][i]);
    }
}

// Norm backward and the first level of its gain/offset gradient reduction in one launch: both read dn and
// x and neither depends on the other.  Work-groups [0, nrow) take rows, the rest column tiles (tiles_c of them per
// group of kColRows rows; wide: 512 columns each, through the 16-byte path).
template <class T, int KIND>
__global__ __launch_bounds__(256) void norm_bwd_colreduce_kernel(const T *__restrict__ dn, const T *__restrict__ x,
                                                                 const float *__restrict__ mean,
                                                                 const float *__restrict__ rstd,
                                                                 const T *__restrict__ gamma,
                                                                 const T *__restrict__ resid, T *__restrict__ dx,
                                                                 int64_t rows, int64_t h, int nrow, int tiles_c,
                                                                 int rc, float *__restrict__ partial, bool wide)
{
    const int id = blockIdx.x;
    if (id < nrow) {
        norm_bwd_rows<T, KIND>(dn, x, mean, rstd, gamma, resid, dx, rows, h, id);
    } else if constexpr (std::is_same<T, bf16>::value) {
        const int j = id - nrow;
        if (wide)
            norm_colreduce_wide_tile<KIND>(dn, x, mean, rstd, rows, h, partial, j % tiles_c, j / tiles_c, rc);
        else
            colreduce_tile<T, KIND == NORM_LAYER ? COLRED_LAYERNORM : COLRED_RMSNORM>(dn, x, mean, rstd, rows, h, h,
                                                                                      partial, j % tiles_c, j / tiles_c, rc);
    } else {
        const int j = id - nrow;
        colreduce_tile<T, KIND == NORM_LAYER ? COLRED_LAYERNORM : COLRED_RMSNORM>(dn, x, mean, rstd, rows, h, h,
                                                                                  partial, j % tiles_c, j / tiles_c, rc);
    }
}

// dx = resid + d(norm)/dx, and the deferred item for d(gamma) (and d(beta) for LayerNorm)
hipError_t launch_norm_bwd_colreduce(int dt, int kind, const void *dn, const void *x, const float *mean,
                                     const float *rstd, const void *gamma, const void *resid, void *dx, int64_t T,
                                     int64_t h, float *dgamma, float *dbeta, float *partial, FinishItem *defer,
                                     hipStream_t s)
{
    if (T == 0 || h == 0) return hipSuccess;
    if (!defer) return hipErrorInvalidValue;
    const int64_t nrow = (T + kRowsPerBlock - 1) / kRowsPerBlock;
    const bool wide = dt == DT_BF16 && h % 512 == 0 && reinterpret_cast<uintptr_t>(dn) % 16 == 0 &&
                      reinterpret_cast<uintptr_t>(x) % 16 == 0;
    const int64_t rc = (T + kColRows - 1) / kColRows, tiles_c = wide ? h / 512 : (h + 63) / 64;
    if (nrow + rc * tiles_c > INT32_MAX) return hipErrorInvalidValue;
    const unsigned grid = (unsigned)(nrow + rc * tiles_c);
#define ZPP_LAUNCH(TT, KK)                                                                                   \
    norm_bwd_colreduce_kernel<TT, KK><<<grid, 256, 0, s>>>((const TT *)dn, (const TT *)x, mean, rstd,        \
                                                           (const TT *)gamma, (const TT *)resid, (TT *)dx, T, h, \
                                                           (int)nrow, (int)tiles_c, (int)rc, partial, wide)
    if (dt == DT_BF16) {
        if (kind == NORM_LAYER) ZPP_LAUNCH(bf16, NORM_LAYER); else ZPP_LAUNCH(bf16, NORM_RMS);
    } else {
        if (kind == NORM_LAYER) ZPP_LAUNCH(float, NORM_LAYER); else ZPP_LAUNCH(float, NORM_RMS);
    }
#undef ZPP_LAUNCH
    const bool two = kind == NORM_LAYER;
    *defer = FinishItem{partial, two ? partial + rc * h : nullptr, dgamma, two ? dbeta : nullptr, (int32_t)rc, h};
    return hipGetLastError();
}

__global__ __launch_bounds__(256) void colreduce_stage2(const float *__restrict__ partial, int64_t rc, int64_t C,
                                                        float *__restrict__ out0, float *__restrict__ out1)
{
    const int64_t c = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= C) return;
    float s0 = 0.0f, s1 = 0.0f;
    for (int64_t r = 0; r < rc; ++r) {
        s0 += partial[r * C + c];
        if (out1) s1 += partial[(rc + r) * C + c];
    }
    out0[c] = s0;
    if (out1) out1[c] = s1;
}

// Column sums of a bf16 matrix with 16-byte loads (the bias gradient db = column sums of dY when the
// weight-gradient product reads dY in place and no transposing pass is there to produce them on the way): a
// work-group takes kColRows rows x 512 columns, a lane eight adjacent columns, the four waves every fourth row;
// the four partial sums per column meet in LDS and one partial row goes out, for the same second level as the
// other column reductions.  C must be a multiple of 512.
__global__ __launch_bounds__(256) void colsum_wide_kernel(const bf16 *__restrict__ a, int64_t rows, int64_t C, int64_t ld,
                                                          float *__restrict__ partial)
{
    __shared__ float red[4][512];
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    const int64_t c = (int64_t)blockIdx.x * 512 + tx * 8;
    const int64_t r0 = (int64_t)blockIdx.y * kColRows;
    const int64_t r1 = (r0 + kColRows < rows) ? r0 + kColRows : rows;
    float acc[8] = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};
    for (int64_t r = r0 + ty; r < r1; r += 4) {
        const bf16x8 v = *reinterpret_cast<const bf16x8 *>(a + r * ld + c);
#pragma unroll
        for (int k = 0; k < 8; ++k) acc[k] += (float)v[k];
    }
#pragma unroll
    for (int k = 0; k < 8; ++k) red[ty][tx * 8 + k] = acc[k];
    __syncthreads();
    for (int i = threadIdx.x; i < 512; i += 256)
        partial[(int64_t)blockIdx.y * C + (int64_t)blockIdx.x * 512 + i] = (red[0][i] + red[1][i]) + (red[2][i] + red[3][i]);
}

hipError_t launch_colreduce(int dt, int mode, const void *a, const void *x, const float *mean,
                            const float *rstd, int64_t T, int64_t C, int64_t ld, float *out0, float *out1,
                            float *partial, hipStream_t s, FinishItem *defer)
{
    if (T == 0 || C == 0) return hipSuccess;
    const int64_t rc = (T + kColRows - 1) / kColRows;
    if (dt == DT_BF16 && mode == COLRED_SUM && defer && C % 512 == 0 && ld % 8 == 0 &&
        reinterpret_cast<uintptr_t>(a) % 16 == 0) {
        colsum_wide_kernel<<<dim3((unsigned)(C / 512), (unsigned)rc), 256, 0, s>>>((const bf16 *)a, T, C, ld, partial);
        *defer = FinishItem{partial, nullptr, out0, nullptr, (int32_t)rc, C};
        return hipGetLastError();
    }
    const dim3 grid((unsigned)((C + 63) / 64), (unsigned)rc);
#define ZPP_LAUNCH(TT, MM)                                                                                 \
    colreduce_stage1<TT, MM><<<grid, 256, 0, s>>>((const TT *)a, (const TT *)x, mean, rstd, T, C, ld, partial)
    if (dt == DT_BF16) {
        if (mode == COLRED_SUM) ZPP_LAUNCH(bf16, COLRED_SUM);
        else if (mode == COLRED_LAYERNORM) ZPP_LAUNCH(bf16, COLRED_LAYERNORM);
        else ZPP_LAUNCH(bf16, COLRED_RMSNORM);
    } else {
        if (mode == COLRED_SUM) ZPP_LAUNCH(float, COLRED_SUM);
        else if (mode == COLRED_LAYERNORM) ZPP_LAUNCH(float, COLRED_LAYERNORM);
        else ZPP_LAUNCH(float, COLRED_RMSNORM);
    }
#undef ZPP_LAUNCH
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (defer) {
        const bool two = mode == COLRED_LAYERNORM;
        *defer = FinishItem{partial, two ? partial + rc * C : nullptr, out0, two ? out1 : nullptr, (int32_t)rc, C};
        return hipSuccess;
    }
    colreduce_stage2<<<(unsigned)((C + 255) / 256), 256, 0, s>>>(partial, rc, C, out0,
                                                                 mode == COLRED_LAYERNORM ? out1 : nullptr);
    return hipGetLastError();
}

}  // namespace zpp
