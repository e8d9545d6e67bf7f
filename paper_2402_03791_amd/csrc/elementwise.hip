// Small HBM-bound kernels: matrix transpose, rotary embedding, SwiGLU forward and backward.
#include "device_utils.h"
#include "kernels.h"

#include <climits>

namespace zpp {

// ------------------------------------------------------------------ transpose
// out[c, r] = in[r, c], 64x64 tiles staged in LDS, 16-byte global loads and stores on both sides
// (8 lanes cover one 128-byte row).  Optionally the same pass produces per-tile column sums of the
// input (partial[tile_row][c] = sum over the tile's 64 rows), which the caller reduces over tile rows:
// that is the bias gradient db = colsum(dY), for free while dY is being transposed for dW = dY^T X.
// Requires R % 64 == 0, C % 64 == 0, ld_in % 8 == 0, ld_out % 8 == 0 (bf16).
// One 64x64 tile: (cx, ry) = tile column / tile row of the input.
template <bool COLSUM>
__device__ __forceinline__ void transpose_tile(const bf16 *__restrict__ in, int64_t ld_in, bf16 *__restrict__ out,
                                               int64_t ld_out, float *__restrict__ partial, int64_t C, int cx, int ry,
                                               bf16 *tile)
{
    constexpr int LD = 66;  // 33 dwords: the column reads of 8 row-chunks fall into 8 different banks
    const int64_t r0 = (int64_t)ry * 64, c0 = (int64_t)cx * 64;
    const int t = threadIdx.x;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int q = t + i * 256;
        const int row = q >> 3, ch = q & 7;
        const u32x4 v = *reinterpret_cast<const u32x4 *>(in + (r0 + row) * ld_in + c0 + ch * 8);
        uint32_t *dst = reinterpret_cast<uint32_t *>(tile + row * LD + ch * 8);
        dst[0] = v[0];
        dst[1] = v[1];
        dst[2] = v[2];
        dst[3] = v[3];
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int q = t + i * 256;
        const int c = q >> 3, kc = q & 7;  // output row (input column) and chunk of 8 input rows
        bf16x8 o;
        float sum = 0.0f;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            o[j] = tile[(kc * 8 + j) * LD + c];
            if (COLSUM) sum += (float)o[j];
        }
        *reinterpret_cast<bf16x8 *>(out + (c0 + c) * ld_out + r0 + kc * 8) = o;
        if (COLSUM) {
            sum += __shfl_xor(sum, 1, 64);
            sum += __shfl_xor(sum, 2, 64);
            sum += __shfl_xor(sum, 4, 64);
            if (kc == 0) partial[(int64_t)ry * C + c0 + c] = sum;
        }
    }
}

template <bool COLSUM>
__global__ __launch_bounds__(256) void transpose_bf16_kernel(const bf16 *__restrict__ in, int64_t ld_in,
                                                             bf16 *__restrict__ out, int64_t ld_out,
                                                             float *__restrict__ partial, int64_t C)
{
    __shared__ bf16 tile[64 * 66];
    transpose_tile<COLSUM>(in, ld_in, out, ld_out, partial, C, blockIdx.x, blockIdx.y, tile);
}

// Two transposes in one launch (the two operands of a weight-gradient product): work-groups [0, n0) take
// the tiles of the first matrix, which also yields column sums; the rest take the second.
struct TransposeDesc {
    const bf16 *in;
    int64_t ld_in;
    bf16 *out;
    int64_t ld_out;
    int32_t tiles_c;  // tile columns (C / 64)
};
__global__ __launch_bounds__(256) void transpose_pair_kernel(TransposeDesc a, float *__restrict__ partial_a,
                                                             int64_t Ca, int32_t n0, TransposeDesc b)
{
    __shared__ bf16 tile[64 * 66];
    const int id = blockIdx.x;
    if (id < n0) {
        if (partial_a)
            transpose_tile<true>(a.in, a.ld_in, a.out, a.ld_out, partial_a, Ca, id % a.tiles_c, id / a.tiles_c, tile);
        else
            transpose_tile<false>(a.in, a.ld_in, a.out, a.ld_out, nullptr, Ca, id % a.tiles_c, id / a.tiles_c, tile);
    } else {
        const int j = id - n0;
        transpose_tile<false>(b.in, b.ld_in, b.out, b.ld_out, nullptr, 0, j % b.tiles_c, j / b.tiles_c, tile);
    }
}

// generic element-wise fallback for other types and ragged sizes
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
    if (dt == DT_BF16) {
        if (R % 64 == 0 && C % 64 == 0 && ld_in % 8 == 0 && ld_out % 8 == 0)
            transpose_bf16_kernel<false><<<grid, 256, 0, s>>>((const bf16 *)in, ld_in, (bf16 *)out, ld_out, nullptr, C);
        else
            transpose_kernel<bf16><<<grid, 256, 0, s>>>((const bf16 *)in, R, C, ld_in, (bf16 *)out, ld_out);
    } else {
        transpose_kernel<float><<<grid, 256, 0, s>>>((const float *)in, R, C, ld_in, (float *)out, ld_out);
    }
    return hipGetLastError();
}

// Column sums of in[R, C] over all rows, written to colsum[C], fused with the transpose.
__global__ __launch_bounds__(256) void colsum_finish_kernel(const float *__restrict__ partial, int64_t tiles,
                                                            int64_t C, float *__restrict__ colsum)
{
    const int64_t c = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= C) return;
    float s = 0.0f;
    for (int64_t r = 0; r < tiles; ++r) s += partial[r * C + c];  // fixed order: run-to-run identical
    colsum[c] = s;
}

uint64_t transpose_colsum_scratch_floats(int64_t R, int64_t C) { return (uint64_t)((R + 63) / 64) * C; }

hipError_t launch_transpose_colsum(const void *in, int64_t R, int64_t C, int64_t ld_in, void *out,
                                   int64_t ld_out, float *colsum, float *partial, hipStream_t s, FinishItem *defer)
{
    if (R == 0 || C == 0) return hipSuccess;
    if (R % 64 || C % 64 || ld_in % 8 || ld_out % 8) return hipErrorInvalidValue;
    const dim3 grid((unsigned)(C / 64), (unsigned)(R / 64));
    transpose_bf16_kernel<true><<<grid, 256, 0, s>>>((const bf16 *)in, ld_in, (bf16 *)out, ld_out, partial, C);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (defer) {
        *defer = FinishItem{partial, nullptr, colsum, nullptr, (int32_t)(R / 64), C};
        return hipSuccess;
    }
    colsum_finish_kernel<<<(unsigned)((C + 255) / 256), 256, 0, s>>>(partial, R / 64, C, colsum);
    return hipGetLastError();
}

// a: [Ra, Ca] -> a_out[Ca, Ra] with column sums when colsum != null (partial, defer as in
// launch_transpose_colsum; defer must be given then); b: [Rb, Cb] -> b_out[Cb, Rb].  bf16, all sizes
// multiples of 64, leading dimensions multiples of 8.
hipError_t launch_transpose_pair(const void *a, int64_t Ra, int64_t Ca, int64_t lda, void *a_out, int64_t lda_out,
                                 float *colsum, float *partial, FinishItem *defer, const void *b, int64_t Rb,
                                 int64_t Cb, int64_t ldb, void *b_out, int64_t ldb_out, hipStream_t s)
{
    if (Ra % 64 || Ca % 64 || Rb % 64 || Cb % 64 || lda % 8 || lda_out % 8 || ldb % 8 || ldb_out % 8 ||
        (colsum && !defer))
        return hipErrorInvalidValue;
    const int64_t n0 = (Ra / 64) * (Ca / 64), n1 = (Rb / 64) * (Cb / 64);
    if (n0 + n1 == 0) return hipSuccess;
    if (n0 == 0 || n1 == 0 || n0 + n1 > INT32_MAX) return hipErrorInvalidValue;
    const TransposeDesc da{(const bf16 *)a, lda, (bf16 *)a_out, lda_out, (int32_t)(Ca / 64)};
    const TransposeDesc db{(const bf16 *)b, ldb, (bf16 *)b_out, ldb_out, (int32_t)(Cb / 64)};
    transpose_pair_kernel<<<(unsigned)(n0 + n1), 256, 0, s>>>(da, colsum ? partial : nullptr, Ca, (int32_t)n0, db);
    if (colsum) *defer = FinishItem{partial, nullptr, colsum, nullptr, (int32_t)(Ra / 64), Ca};
    return hipGetLastError();
}

// Second level of up to kFinishMax column reductions in one launch; blocks [first[i], first[i+1]) work on
// item i, one thread per column, partial rows added in ascending order (run-to-run identical).
constexpr int kFinishMax = 32;
struct FinishBatch {
    FinishItem item[kFinishMax];
    int32_t first[kFinishMax + 1];
    int32_t n;
    int32_t accumulate;  // out <- out + scale * sum
    float scale;
};

__global__ __launch_bounds__(256) void finish_columns_kernel(FinishBatch b)
{
    int i = 0;
    while (i + 1 < b.n && (int)blockIdx.x >= b.first[i + 1]) ++i;
    const FinishItem &it = b.item[i];
    const int64_t c = (int64_t)((int)blockIdx.x - b.first[i]) * 256 + threadIdx.x;
    if (c >= it.C) return;
    float s0 = 0.0f, s1 = 0.0f;
    for (int r = 0; r < it.rows; ++r) {
        s0 += it.partial0[(int64_t)r * it.C + c];
        if (it.partial1) s1 += it.partial1[(int64_t)r * it.C + c];
    }
    it.out0[c] = b.accumulate ? grad_accum(it.out0[c], b.scale, s0) : s0;
    if (it.out1) it.out1[c] = b.accumulate ? grad_accum(it.out1[c], b.scale, s1) : s1;
}

hipError_t launch_finish_columns(const FinishItem *items, int n, hipStream_t s, bool accumulate, float scale)
{
    for (int base = 0; base < n; base += kFinishMax) {
        FinishBatch b;
        b.n = n - base < kFinishMax ? n - base : kFinishMax;
        b.accumulate = accumulate;
        b.scale = scale;
        int32_t blocks = 0;
        for (int i = 0; i < b.n; ++i) {
            b.item[i] = items[base + i];
            b.first[i] = blocks;
            blocks += (int32_t)((items[base + i].C + 255) / 256);
        }
        b.first[b.n] = blocks;
        if (blocks == 0) continue;
        finish_columns_kernel<<<(unsigned)blocks, 256, 0, s>>>(b);
        if (hipError_t e = hipGetLastError()) return e;
    }
    return hipSuccess;
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

// The same rotation, one 16-byte vector (VN/2 pairs of one head) per thread: the vector's cos/sin values are
// VN consecutive floats of the table.  Needs d % VN == 0 (a vector never straddles two heads).
template <class T>
__global__ __launch_bounds__(256) void rope_vec_kernel(T *__restrict__ qkv, const float *__restrict__ table,
                                                       int64_t rows, int64_t seq, int64_t h, int64_t d, float sign)
{
    constexpr int VN = Vec16<T>::N;
    const int64_t nvrow = 2 * h / VN;  // vectors in the Q and K parts of one row
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= rows * nvrow) return;
    const int64_t t = idx / nvrow, col = (idx % nvrow) * VN;
    const int64_t i0 = (col % d) / 2, p = t % seq;
    const float *cs = table + (p * (d / 2) + i0) * 2;
    T *e = qkv + t * 3 * h + col;
    const Vec16<T> v = load16(e);
    Vec16<T> o;
#pragma unroll
    for (int k = 0; k < VN; k += 4) {
        const f32x4 w = *reinterpret_cast<const f32x4 *>(cs + k);  // cos, sin of two pairs
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            const float c = w[2 * q], sn = sign * w[2 * q + 1];
            const float a = v.get(k + 2 * q), b = v.get(k + 2 * q + 1);
            o.set(k + 2 * q, a * c - b * sn);
            o.set(k + 2 * q + 1, a * sn + b * c);
        }
    }
    store16(e, o);
}

hipError_t launch_rope(int dt, void *qkv, const float *table, int64_t T, int64_t seq, int64_t nh, int64_t d,
                       int sign, hipStream_t s)
{
    const int64_t h = nh * d;
    const int64_t n = T * h;
    if (n == 0) return hipSuccess;
    const int vn = dt == DT_BF16 ? 8 : 4;
    if (d % vn == 0 && reinterpret_cast<uintptr_t>(qkv) % 16 == 0 && (3 * h) % vn == 0) {
        const unsigned grid = (unsigned)((2 * n / vn + 255) / 256);
        if (dt == DT_BF16)
            rope_vec_kernel<bf16><<<grid, 256, 0, s>>>((bf16 *)qkv, table, T, seq, h, d, (float)sign);
        else
            rope_vec_kernel<float><<<grid, 256, 0, s>>>((float *)qkv, table, T, seq, h, d, (float)sign);
        return hipGetLastError();
    }
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

// g = GeLU(u) element-wise on stored pre-activations: what the epilogue of the first MLP product computes
// from the value it stores, for selective recomputation (n elements, a multiple of the 16-byte vector).
template <class T>
__global__ __launch_bounds__(256) void gelu_fwd_kernel(const T *__restrict__ u, T *__restrict__ g, int64_t nv, int mode)
{
    constexpr int VN = Vec16<T>::N;
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= nv) return;
    const Vec16<T> x = load16(u + idx * VN);
    Vec16<T> o;
#pragma unroll
    for (int k = 0; k < VN; ++k) o.set(k, gelu_fwd(x.get(k), mode));
    store16(g + idx * VN, o);
}

hipError_t launch_gelu_fwd(int dt, const void *u, void *g, int64_t n, int gelu_mode, hipStream_t s)
{
    const int64_t nv = n / (dt == DT_BF16 ? 8 : 4);
    if (nv == 0) return hipSuccess;
    if (n % (dt == DT_BF16 ? 8 : 4)) return hipErrorInvalidValue;
    const unsigned grid = (unsigned)((nv + 255) / 256);
    if (dt == DT_BF16)
        gelu_fwd_kernel<bf16><<<grid, 256, 0, s>>>((const bf16 *)u, (bf16 *)g, nv, gelu_mode);
    else
        gelu_fwd_kernel<float><<<grid, 256, 0, s>>>((const float *)u, (float *)g, nv, gelu_mode);
    return hipGetLastError();
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
