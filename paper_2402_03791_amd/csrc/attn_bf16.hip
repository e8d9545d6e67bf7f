// Fused causal attention for bf16, head dim 128, on gfx950 MFMA (v_mfma_f32_32x32x16_bf16).
//
// Forward: one work-group per (sample, head, block of 128 queries), four wavefronts of 32 queries
// each.  Keys/values stream through LDS in tiles of 64 rows (double buffered).  Scores are computed
// transposed, S^T = K Q^T, so that a lane owns one query column and the softmax row reductions are
// in-lane plus one exchange with the lane 32 away; the probabilities then feed the second product
// O^T = V^T P^T straight from the accumulator registers.  The value tile is read with the LDS
// transposing load (ds_read_b64_tr_b16), which hands each lane four consecutive key rows of one
// value column.  The softmax never leaves registers; only O and the log-sum-exp are written.
//
// Backward: two kernels without atomics.  dQ: same structure as forward (lane = query), loops over
// key tiles.  dK/dV: lane = key, loops over query tiles.  P is recomputed from the saved
// log-sum-exp; delta = rowsum(dO o O) is computed by a small kernel first.
#include "device_utils.h"
#include "kernels.h"

namespace zpp {

typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

constexpr int kD = 128;        // head dim
constexpr int kTile = 64;      // rows of a streamed tile
constexpr int kTileElems = kTile * kD;

// LDS layouts of a [64][128] bf16 tile (256-byte rows).
// "row" layout: read as MFMA operand with 8 consecutive columns per lane (16-byte chunks).
__device__ __forceinline__ int off_row(int row, int chunk16) { return row * kD + ((chunk16 ^ (row & 15)) << 3); }
// "tr" layout: read with the transposing load, 4 consecutive rows x 16 columns per 16 lanes.
__device__ __forceinline__ int off_tr(int row, int col)
{
    const int gran = col >> 4;  // 32-byte granule
    return row * kD + ((gran ^ ((row & 3) << 1)) << 4) + (col & 15);
}

// 8 operand values for one lane: rows k0a..k0a+3 and k0b..k0b+3 of column (col_base + lane%16),
// out of a tile in "tr" layout.
__device__ __forceinline__ bf16x8 read_tr8(const bf16 *tile, int k0a, int k0b, int col_base, int lane)
{
    const int i = lane & 15, e = i >> 2, q4 = i & 3;
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(tile + off_tr(k0a + e, col_base + 4 * q4)));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(tile + off_tr(k0b + e, col_base + 4 * q4)));
    typedef __attribute__((ext_vector_type(8))) short s16x8;
    const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, both);
}

struct TileLoader {
    // 64 rows x 16 chunks of 16 bytes = 1024 chunks, 4 per thread
    const bf16 *src[4];
    int dst_row[4], dst_tr[4];
    bf16x8 reg[4];
    __device__ __forceinline__ void init(const bf16 *base, int64_t ld, int tid)
    {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int q = tid + i * 256;
            const int row = q >> 4, ch = q & 15;
            src[i] = base + (int64_t)row * ld + ch * 8;
            dst_row[i] = off_row(row, ch);
            dst_tr[i] = off_tr(row, ch * 8);
        }
    }
    __device__ __forceinline__ void load(int64_t row_off_elems)
    {
#pragma unroll
        for (int i = 0; i < 4; ++i) reg[i] = *reinterpret_cast<const bf16x8 *>(src[i] + row_off_elems);
    }
    __device__ __forceinline__ void store_row(bf16 *tile) const
    {
#pragma unroll
        for (int i = 0; i < 4; ++i) *reinterpret_cast<bf16x8 *>(tile + dst_row[i]) = reg[i];
    }
    __device__ __forceinline__ void store_tr(bf16 *tile) const
    {
#pragma unroll
        for (int i = 0; i < 4; ++i) *reinterpret_cast<bf16x8 *>(tile + dst_tr[i]) = reg[i];
    }
};

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// ------------------------------------------------------------------------------------ forward
__global__ __launch_bounds__(256) void attn_fwd_mfma_kernel(const bf16 *__restrict__ qkv, bf16 *__restrict__ attn,
                                                            float *__restrict__ lse, int seq, int nh,
                                                            float scale_log2e)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    bf16 *Ks = reinterpret_cast<bf16 *>(smem_raw);  // [2][64*128], "row" layout
    bf16 *Vs = Ks + 2 * kTileElems;                 // [2][64*128], "tr" layout

    const int qb = gridDim.x - 1 - blockIdx.x;  // heavy (late) query blocks first
    const int n = blockIdx.y, bi = blockIdx.z;
    const int64_t h = (int64_t)nh * kD, ld = 3 * h;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int g = lane >> 5, c = lane & 31;
    const int q0 = qb * 128, qw0 = q0 + 32 * wave;
    const int64_t row0 = (int64_t)bi * seq;

    bf16x8 qf[8];
    {
        const bf16 *qp = qkv + (row0 + qw0 + c) * ld + (int64_t)n * kD + 8 * g;
#pragma unroll
        for (int st = 0; st < 8; ++st) qf[st] = *reinterpret_cast<const bf16x8 *>(qp + 16 * st);
    }

    TileLoader lk, lv;
    lk.init(qkv + row0 * ld + h + (int64_t)n * kD, ld, tid);
    lv.init(qkv + row0 * ld + 2 * h + (int64_t)n * kD, ld, tid);

    f32x16 oacc[4];
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) oacc[t][e] = 0.0f;
    float m_run = -INFINITY, l_run = 0.0f;

    const int n_tiles = (q0 + 128) / kTile;
    lk.load(0);
    lv.load(0);
    lk.store_row(Ks);
    lv.store_tr(Vs);
    __syncthreads();

    for (int jt = 0; jt < n_tiles; ++jt) {
        const int buf = jt & 1;
        if (jt + 1 < n_tiles) {
            lk.load((int64_t)(jt + 1) * kTile * ld);
            lv.load((int64_t)(jt + 1) * kTile * ld);
        }
        const int kv0 = jt * kTile;
        if (kv0 <= qw0 + 31) {  // wave-uniform: this wave has unmasked entries in the tile
            const bf16 *ks = Ks + buf * kTileElems;
            const bf16 *vs = Vs + buf * kTileElems;
            f32x16 sacc[2];
#pragma unroll
            for (int T = 0; T < 2; ++T) {
#pragma unroll
                for (int e = 0; e < 16; ++e) sacc[T][e] = 0.0f;
#pragma unroll
                for (int st = 0; st < 8; ++st) {
                    const bf16x8 kf = *reinterpret_cast<const bf16x8 *>(ks + off_row(32 * T + c, 2 * st + g));
                    sacc[T] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[st], sacc[T], 0, 0, 0);
                }
            }
            // sacc[T][e] of this lane: key kv0 + 32T + 8(e/4) + 4g + e%4, query qw0 + c
            const bool need_mask = kv0 + kTile - 1 > qw0;
            float mloc = -INFINITY;
#pragma unroll
            for (int T = 0; T < 2; ++T)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    float sv = sacc[T][e] * scale_log2e;
                    if (need_mask) {
                        const int kv = kv0 + 32 * T + 8 * (e >> 2) + 4 * g + (e & 3);
                        if (kv > qw0 + c) sv = -INFINITY;
                    }
                    sacc[T][e] = sv;
                    mloc = fmaxf(mloc, sv);
                }
            mloc = fmaxf(mloc, __shfl_xor(mloc, 32, 64));
            const float m_new = fmaxf(m_run, mloc);
            const float alpha = fast_exp2(m_run - m_new);
            float psum = 0.0f;
            bf16x8 pf[4];
#pragma unroll
            for (int T = 0; T < 2; ++T)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const float p = fast_exp2(sacc[T][e] - m_new);
                    psum += p;
                    pf[2 * T + (e >> 3)][e & 7] = (bf16)p;
                }
            l_run = l_run * alpha + psum;
            m_run = m_new;
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int e = 0; e < 16; ++e) oacc[t][e] *= alpha;
            // O^T[dv, q] += sum_kv V^T[dv, kv] P^T[kv, q]
#pragma unroll
            for (int st = 0; st < 4; ++st) {
                const int k0 = 32 * (st >> 1) + 16 * (st & 1) + 4 * g;
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const bf16x8 vf = read_tr8(vs, k0, k0 + 8, 32 * t + ((lane >> 4) & 1) * 16, lane);
                    oacc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[st], oacc[t], 0, 0, 0);
                }
            }
        }
        if (jt + 1 < n_tiles) {
            lk.store_row(Ks + (buf ^ 1) * kTileElems);
            lv.store_tr(Vs + (buf ^ 1) * kTileElems);
        }
        __syncthreads();
    }

    const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
    const float inv = 1.0f / l_tot;
    bf16 *op = attn + (row0 + qw0 + c) * h + (int64_t)n * kD;
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int e4 = 0; e4 < 4; ++e4) {
            bf16x4 o;
#pragma unroll
            for (int r = 0; r < 4; ++r) o[r] = (bf16)(oacc[t][e4 * 4 + r] * inv);
            *reinterpret_cast<bf16x4 *>(op + 32 * t + 8 * e4 + 4 * g) = o;
        }
    if (g == 0)
        lse[((int64_t)bi * nh + n) * seq + qw0 + c] = (m_run + __builtin_amdgcn_logf(l_tot)) * 0.69314718055994530942f;
}

bool attn_mfma_supported(int64_t seq, int64_t d) { return d == kD && seq % 128 == 0 && seq >= 128; }

hipError_t launch_attn_simple_bwd(int dt, const void *qkv, const void *attn, const void *dattn,
                                  const float *lse, float *delta, void *dqkv, int64_t b, int64_t seq,
                                  int64_t nh, int64_t d, hipStream_t s);

hipError_t launch_attn_fwd(int dt, const void *qkv, void *attn, float *lse, int64_t b, int64_t seq, int64_t nh,
                           int64_t d, hipStream_t s)
{
    if (dt != DT_BF16 || !attn_mfma_supported(seq, d)) return hipErrorInvalidValue;
    if (b * seq == 0) return hipSuccess;
    constexpr size_t lds = 4 * kTileElems * sizeof(bf16);  // 64 KB
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(attn_fwd_mfma_kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const float scale_log2e = (1.0f / sqrtf((float)d)) * 1.44269504088896340736f;
    const dim3 grid((unsigned)(seq / 128), (unsigned)nh, (unsigned)b);
    attn_fwd_mfma_kernel<<<grid, 256, lds, s>>>((const bf16 *)qkv, (bf16 *)attn, lse, (int)seq, (int)nh, scale_log2e);
    return hipGetLastError();
}

hipError_t launch_attn_bwd(int dt, const void *qkv, const void *attn, const void *dattn, const float *lse,
                           float *delta, void *dqkv, int64_t b, int64_t seq, int64_t nh, int64_t d, hipStream_t s)
{
    // the MFMA backward kernels are not in yet: the generic kernels compute the same thing
    return launch_attn_simple_bwd(dt, qkv, attn, dattn, lse, delta, dqkv, b, seq, nh, d, s);
}

}  // namespace zpp
