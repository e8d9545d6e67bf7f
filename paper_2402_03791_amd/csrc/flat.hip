// Flat-buffer passes over the ZeRO-3-style shard: materialise (stand-in for the per-unit parameter
// all-gather), gradient accumulation (stand-in for the per-unit reduce-scatter) and the fused Adam
// step (the optimizer-step task).  All three are HBM-bandwidth bound: 16-byte accesses, 64-bit
// indexing (the flat buffers exceed 4 GiB at the wide configuration), one contiguous chunk per work-group.
#include "device_utils.h"
#include "kernels.h"

namespace zpp {

// Launch shape of the streaming passes: no persistent grid-stride loop.  Every work-group owns one
// contiguous chunk of VPT*256 16-byte vectors (16 KB per buffer at VPT = 4), issues all its loads
// before its first store, and uses non-temporal accesses (nothing is reused).  Measured on MI355X a
// huge grid of such small chunks sustains 6.0-6.1 TB/s on the accumulate pass where a persistent
// grid of 16 groups per CU reaches 4.7 TB/s (about what a device-to-device hipMemcpy gets).

template <class T> __device__ __forceinline__ T nt_load(const T *p) { return __builtin_nontemporal_load(p); }
template <class T> __device__ __forceinline__ void nt_store(T v, T *p) { __builtin_nontemporal_store(v, p); }

static inline unsigned flat_blocks(uint64_t nvec, int vpt)
{
    const uint64_t per = (uint64_t)vpt * 256;
    uint64_t b = (nvec + per - 1) / per;
    return (unsigned)(b ? b : 1);
}

// ---------------------------------------------------------------- materialise
template <int VPT>
__global__ __launch_bounds__(256) void materialize_bf16_kernel(const float *__restrict__ P,
                                                               bf16 *__restrict__ W, uint64_t n)
{
    const uint64_t nvec = n / 8;  // 8 elements per output vector
    const uint64_t base = (uint64_t)blockIdx.x * (VPT * 256) + threadIdx.x;
    f32x4 a[VPT], b[VPT];
#pragma unroll
    for (int u = 0; u < VPT; ++u) {
        const uint64_t i = base + u * 256;
        if (i < nvec) {
            a[u] = nt_load(reinterpret_cast<const f32x4 *>(P) + 2 * i);
            b[u] = nt_load(reinterpret_cast<const f32x4 *>(P) + 2 * i + 1);
        }
    }
#pragma unroll
    for (int u = 0; u < VPT; ++u) {
        const uint64_t i = base + u * 256;
        if (i < nvec) {
            bf16x8 o;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                o[k] = (bf16)a[u][k];
                o[k + 4] = (bf16)b[u][k];
            }
            nt_store(o, reinterpret_cast<bf16x8 *>(W) + i);
        }
    }
    if (blockIdx.x == 0)  // ragged tail
        for (uint64_t j = nvec * 8 + threadIdx.x; j < n; j += 256) W[j] = (bf16)P[j];
}

template <int VPT>
__global__ __launch_bounds__(256) void materialize_f32_kernel(const float *__restrict__ P,
                                                              float *__restrict__ W, uint64_t n)
{
    const uint64_t nvec = n / 4;
    const uint64_t base = (uint64_t)blockIdx.x * (VPT * 256) + threadIdx.x;
    f32x4 a[VPT];
#pragma unroll
    for (int u = 0; u < VPT; ++u)
        if (base + u * 256 < nvec) a[u] = nt_load(reinterpret_cast<const f32x4 *>(P) + base + u * 256);
#pragma unroll
    for (int u = 0; u < VPT; ++u)
        if (base + u * 256 < nvec) nt_store(a[u], reinterpret_cast<f32x4 *>(W) + base + u * 256);
    if (blockIdx.x == 0)
        for (uint64_t j = nvec * 4 + threadIdx.x; j < n; j += 256) W[j] = P[j];
}

hipError_t launch_materialize(const float *P, void *W, uint64_t n, int dt, hipStream_t s)
{
    if (n == 0) return hipSuccess;
    if (dt == DT_BF16)
        materialize_bf16_kernel<4><<<flat_blocks(n / 8, 4), 256, 0, s>>>(P, (bf16 *)W, n);
    else
        materialize_f32_kernel<4><<<flat_blocks(n / 4, 4), 256, 0, s>>>(P, (float *)W, n);
    return hipGetLastError();
}

// Wt[c, r] = bf16(P[r, c]), any shape: 64x64 tiles through LDS, element accesses (the ragged fallback).
__global__ __launch_bounds__(256) void transpose_cast_ragged_kernel(const float *__restrict__ P,
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

// The same for rows in multiples of 128 and cols in multiples of 64, at streaming speed: a work-group takes a
// tile of 128 rows x 64 columns with 16-byte loads (each thread four pairs of vertically adjacent 4-float
// pieces, all eight loads in flight before the first use), rounds to bf16, packs the two rows of a pair into
// one 32-bit word per column (the output is contiguous along rows) and writes the words transposed into LDS -
// row stride 65 words, so the 64 lanes of a wave hit 64 different banks both ways - then reads eight
// consecutive rows of a column back and stores them with one 16-byte non-temporal store per lane.  Both the
// reads and the writes touch memory in 256-byte runs.
__device__ __forceinline__ void transpose_cast_tile(const float *__restrict__ P, bf16 *__restrict__ Wt, uint64_t rows,
                                                    uint64_t cols, uint64_t r0, uint64_t c0)
{
    constexpr int S = 65;                  // words per LDS row (64 row pairs + 1)
    __shared__ uint32_t tile[64 * S];      // [column][row pair]
    const int t = threadIdx.x;
    const int col4 = t & 15, pair0 = t >> 4;   // row pairs pair0 + 16 u
    f32x4 top[4], bot[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const float *src = P + (r0 + 2 * (pair0 + 16 * u)) * cols + c0 + 4 * col4;
        top[u] = nt_load(reinterpret_cast<const f32x4 *>(src));
        bot[u] = nt_load(reinterpret_cast<const f32x4 *>(src + cols));
    }
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            bf16x2 w;
            w[0] = (bf16)top[u][k];
            w[1] = (bf16)bot[u][k];
            tile[(4 * col4 + k) * S + pair0 + 16 * u] = __builtin_bit_cast(uint32_t, w);
        }
    __syncthreads();
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int c = (t >> 4) + 16 * u, q = t & 15;   // rows 8q .. 8q+7 of output row c
        u32x4 o;
#pragma unroll
        for (int k = 0; k < 4; ++k) o[k] = tile[c * S + 4 * q + k];
        nt_store(o, reinterpret_cast<u32x4 *>(Wt + (c0 + c) * rows + r0 + 8 * q));
    }
}

__global__ __launch_bounds__(256) void transpose_cast_kernel(const float *__restrict__ P, bf16 *__restrict__ Wt,
                                                             uint64_t rows, uint64_t cols)
{
    transpose_cast_tile(P, Wt, rows, cols, (uint64_t)blockIdx.y * 128, (uint64_t)blockIdx.x * 64);
}

// All matrices of a stage in one launch (one kernel tail instead of one per matrix): a work-group finds its
// matrix in the table by a scalar search, then its tile inside the matrix, column tiles fastest.
__global__ __launch_bounds__(256) void transpose_cast_many_kernel(const float *__restrict__ P, bf16 *__restrict__ Wt,
                                                                  TransposeCastTable tab)
{
    int i = 0;
    while (i + 1 < tab.n && blockIdx.x >= tab.first_block[i + 1]) ++i;
    const uint32_t local = blockIdx.x - tab.first_block[i];
    const uint32_t tiles_c = (uint32_t)(tab.cols[i] / 64), tiles_r = (uint32_t)(tab.rows[i] / 128);
    uint32_t tr, tc;
    if (tiles_c % 8 == 0 && tiles_r % 8 == 0) {
        // Work-groups that run at the same time form 8 x 8 squares of tiles: their reads are 2 KB runs of P's rows
        // and their writes 2 KB runs of Wt's rows, so both sides find several accesses per open DRAM page (in
        // row-major tile order the writes of concurrent work-groups are isolated 256-byte pieces).
        const uint32_t sq = local >> 6, in = local & 63;
        tr = (sq / (tiles_c / 8)) * 8 + (in >> 3);
        tc = (sq % (tiles_c / 8)) * 8 + (in & 7);
    } else {
        tr = local / tiles_c;
        tc = local % tiles_c;
    }
    transpose_cast_tile(P + tab.src[i], Wt + tab.dst[i], tab.rows[i], tab.cols[i], (uint64_t)tr * 128, (uint64_t)tc * 64);
}

hipError_t launch_transpose_cast_many(const float *P, void *Wt, TransposeCastTable tab, hipStream_t s)
{
    if (tab.n <= 0) return hipSuccess;
    if (tab.n > kTransposeCastMax || (reinterpret_cast<uintptr_t>(P) | reinterpret_cast<uintptr_t>(Wt)) % 16)
        return hipErrorInvalidValue;
    uint64_t blocks = 0;
    for (int i = 0; i < tab.n; ++i) {
        if (tab.rows[i] % 128 || tab.cols[i] % 64 || tab.src[i] % 4 || tab.dst[i] % 8) return hipErrorInvalidValue;
        tab.first_block[i] = (uint32_t)blocks;
        blocks += (tab.rows[i] / 128) * (tab.cols[i] / 64);
    }
    if (blocks > 0x7fffffffull) return hipErrorInvalidValue;
    tab.first_block[tab.n] = (uint32_t)blocks;
    if (blocks == 0) return hipSuccess;
    transpose_cast_many_kernel<<<(unsigned)blocks, 256, 0, s>>>(P, (bf16 *)Wt, tab);
    return hipGetLastError();
}

hipError_t launch_transpose_cast(const float *P, void *Wt, uint64_t rows, uint64_t cols, hipStream_t s)
{
    if (rows == 0 || cols == 0) return hipSuccess;
    if (rows % 128 == 0 && cols % 64 == 0 && (reinterpret_cast<uintptr_t>(P) | reinterpret_cast<uintptr_t>(Wt)) % 16 == 0) {
        dim3 grid((unsigned)(cols / 64), (unsigned)(rows / 128));
        transpose_cast_kernel<<<grid, 256, 0, s>>>(P, (bf16 *)Wt, rows, cols);
    } else {
        dim3 grid((unsigned)((cols + 63) / 64), (unsigned)((rows + 63) / 64));
        transpose_cast_ragged_kernel<<<grid, 256, 0, s>>>(P, (bf16 *)Wt, rows, cols);
    }
    return hipGetLastError();
}

// ---------------------------------------------------------------- accumulate
// FIRST: G counts as zero and is not read (the first accumulation after an Adam step that released G instead of
// zeroing it): G <- 0 + scale * S, the bits that adding onto zeros gives, for 8 instead of 12 bytes per element.
template <int VPT, bool FIRST>
__global__ __launch_bounds__(256) void accumulate_kernel(float *__restrict__ G, const float *__restrict__ S,
                                                         uint64_t n, float scale)
{
    const uint64_t nvec = n / 4;
    const uint64_t base = (uint64_t)blockIdx.x * (VPT * 256) + threadIdx.x;
    f32x4 g[VPT], v[VPT];
#pragma unroll
    for (int u = 0; u < VPT; ++u) {
        const uint64_t i = base + u * 256;
        if (i < nvec) {
            g[u] = FIRST ? f32x4{0.0f, 0.0f, 0.0f, 0.0f} : nt_load(reinterpret_cast<const f32x4 *>(G) + i);
            v[u] = nt_load(reinterpret_cast<const f32x4 *>(S) + i);
        }
    }
#pragma unroll
    for (int u = 0; u < VPT; ++u) {
        const uint64_t i = base + u * 256;
        if (i < nvec) {
#pragma unroll
            for (int k = 0; k < 4; ++k) g[u][k] = grad_accum(g[u][k], scale, v[u][k]);
            nt_store(g[u], reinterpret_cast<f32x4 *>(G) + i);
        }
    }
    if (blockIdx.x == 0)
        for (uint64_t j = nvec * 4 + threadIdx.x; j < n; j += 256) G[j] = grad_accum(FIRST ? 0.0f : G[j], scale, S[j]);
}

hipError_t launch_accumulate(float *G, const float *S, uint64_t n, float scale, hipStream_t s, bool first)
{
    if (n == 0) return hipSuccess;
    if (first)
        accumulate_kernel<4, true><<<flat_blocks(n / 4, 4), 256, 0, s>>>(G, S, n, scale);
    else
        accumulate_kernel<4, false><<<flat_blocks(n / 4, 4), 256, 0, s>>>(G, S, n, scale);
    return hipGetLastError();
}

__global__ __launch_bounds__(256) void fill_zero_kernel(float *__restrict__ G, uint64_t n)
{
    const uint64_t nvec = n / 4;
    const uint64_t i = (uint64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < nvec) nt_store(f32x4{0.0f, 0.0f, 0.0f, 0.0f}, reinterpret_cast<f32x4 *>(G) + i);
    if (blockIdx.x == 0)
        for (uint64_t j = nvec * 4 + threadIdx.x; j < n; j += 256) G[j] = 0.0f;
}

hipError_t launch_fill_zero(float *G, uint64_t n, hipStream_t s)
{
    if (n == 0) return hipSuccess;
    fill_zero_kernel<<<flat_blocks(n / 4, 1), 256, 0, s>>>(G, n);
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

// Optional write-back of updated parameters into the working copy (element i of the shard, 4 elements):
// the cast the next materialise would do, done while the values are in registers.
__device__ __forceinline__ void adam_write_back(const AdamArgs &a, uint64_t vec, const f32x4 &p)
{
    if (!a.wb) return;
    if (a.wb_bf16) {
        bf16x4 o;
#pragma unroll
        for (int k = 0; k < 4; ++k) o[k] = (bf16)p[k];
        reinterpret_cast<bf16x4 *>(a.wb)[vec] = o;
    } else {
        reinterpret_cast<f32x4 *>(a.wb)[vec] = p;
    }
}

template <int VPT>
__global__ __launch_bounds__(256) void adam_kernel(float *__restrict__ P, float *__restrict__ M,
                                                   float *__restrict__ V, float *__restrict__ G, uint64_t n,
                                                   AdamArgs a)
{
    const uint64_t nvec = n / 4;
    const uint64_t base = (uint64_t)blockIdx.x * (VPT * 256) + threadIdx.x;
    f32x4 p[VPT], m[VPT], v[VPT], g[VPT];
#pragma unroll
    for (int u = 0; u < VPT; ++u) {
        const uint64_t i = base + u * 256;
        if (i < nvec) {
            p[u] = nt_load(reinterpret_cast<const f32x4 *>(P) + i);
            m[u] = nt_load(reinterpret_cast<const f32x4 *>(M) + i);
            v[u] = nt_load(reinterpret_cast<const f32x4 *>(V) + i);
            g[u] = nt_load(reinterpret_cast<const f32x4 *>(G) + i);
        }
    }
#pragma unroll
    for (int u = 0; u < VPT; ++u) {
        const uint64_t i = base + u * 256;
        if (i < nvec) {
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                float pp = p[u][k], mm = m[u][k], vv = v[u][k], gg = g[u][k];
                adam_one(pp, mm, vv, gg, a);
                p[u][k] = pp;
                m[u][k] = mm;
                v[u][k] = vv;
                g[u][k] = gg;
            }
            nt_store(p[u], reinterpret_cast<f32x4 *>(P) + i);
            nt_store(m[u], reinterpret_cast<f32x4 *>(M) + i);
            nt_store(v[u], reinterpret_cast<f32x4 *>(V) + i);
            if (a.zero_grad) nt_store(g[u], reinterpret_cast<f32x4 *>(G) + i);
            adam_write_back(a, i, p[u]);
        }
    }
    if (blockIdx.x == 0)
        for (uint64_t j = nvec * 4 + threadIdx.x; j < n; j += 256) {
            float pp = P[j], mm = M[j], vv = V[j], gg = G[j];
            adam_one(pp, mm, vv, gg, a);
            P[j] = pp;
            M[j] = mm;
            V[j] = vv;
            if (a.zero_grad) G[j] = gg;
            if (a.wb) {
                if (a.wb_bf16) reinterpret_cast<bf16 *>(a.wb)[j] = (bf16)pp;
                else reinterpret_cast<float *>(a.wb)[j] = pp;
            }
        }
}

// Several ranges in one launch: a block finds its range in the table (a scalar search over at most
// kAdamRanges entries), takes that range's learning rate and weight decay, and then does exactly what a
// block of adam_kernel<1> does on the range: 256 16-byte vectors per array.
__global__ __launch_bounds__(256) void adam_ranges_kernel(float *__restrict__ P, float *__restrict__ M,
                                                          float *__restrict__ V, float *__restrict__ G,
                                                          AdamRanges r, AdamArgs a)
{
    int i = 0;
    while (i + 1 < r.n && blockIdx.x >= r.first_block[i + 1]) ++i;
    a.lr = r.lr[i];
    a.wd = r.wd[i];
    const uint64_t v = (uint64_t)(blockIdx.x - r.first_block[i]) * 256 + threadIdx.x;
    if (v >= r.count[i] / 4) return;
    const uint64_t e = r.offset[i] / 4 + v;
    f32x4 p = nt_load(reinterpret_cast<const f32x4 *>(P) + e);
    f32x4 m = nt_load(reinterpret_cast<const f32x4 *>(M) + e);
    f32x4 vv = nt_load(reinterpret_cast<const f32x4 *>(V) + e);
    f32x4 g = nt_load(reinterpret_cast<const f32x4 *>(G) + e);
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        float pp = p[k], mm = m[k], v2 = vv[k], gg = g[k];
        adam_one(pp, mm, v2, gg, a);
        p[k] = pp;
        m[k] = mm;
        vv[k] = v2;
        g[k] = gg;
    }
    nt_store(p, reinterpret_cast<f32x4 *>(P) + e);
    nt_store(m, reinterpret_cast<f32x4 *>(M) + e);
    nt_store(vv, reinterpret_cast<f32x4 *>(V) + e);
    if (a.zero_grad) nt_store(g, reinterpret_cast<f32x4 *>(G) + e);
    adam_write_back(a, e, p);
}

hipError_t launch_adam_ranges(float *P, float *M, float *V, float *G, AdamRanges r, const AdamArgs &a, hipStream_t s)
{
    if (r.n <= 0) return hipSuccess;
    if (r.n > kAdamRanges) return hipErrorInvalidValue;
    uint64_t blocks = 0;
    for (int i = 0; i < r.n; ++i) {
        if (r.offset[i] % 4 || r.count[i] % 4) return hipErrorInvalidValue;
        r.first_block[i] = (uint32_t)blocks;
        blocks += (r.count[i] / 4 + 255) / 256;
    }
    if (blocks > 0x7fffffffull) return hipErrorInvalidValue;
    r.first_block[r.n] = (uint32_t)blocks;
    if (blocks == 0) return hipSuccess;
    adam_ranges_kernel<<<(unsigned)blocks, 256, 0, s>>>(P, M, V, G, r, a);
    return hipGetLastError();
}

hipError_t launch_adam(float *P, float *M, float *V, float *G, uint64_t n, const AdamArgs &a, hipStream_t s)
{
    if (n == 0) return hipSuccess;
    adam_kernel<1><<<flat_blocks(n / 4, 1), 256, 0, s>>>(P, M, V, G, n, a);
    return hipGetLastError();
}

}  // namespace zpp
