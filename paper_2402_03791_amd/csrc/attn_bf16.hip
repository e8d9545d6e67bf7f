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

// ------------------------------------------------------------------------------------ backward: dQ
// Lane = query.  Per key tile: S^T = K Q^T and dP^T = V dO^T (operands K, V row-wise from LDS; Q, dO
// in registers), P^T = exp2(S^T*c - lse), dS^T = P^T o (dP^T - delta), dQ^T += K^T dS^T with K^T
// taken from a second copy of the key tile through the transposing load.
__global__ __launch_bounds__(256) void attn_bwd_dq_mfma_kernel(const bf16 *__restrict__ qkv,
                                                               const bf16 *__restrict__ dattn,
                                                               const float *__restrict__ lse,
                                                               const float *__restrict__ delta,
                                                               bf16 *__restrict__ dqkv, int seq, int nh, float scale,
                                                               float scale_log2e)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    bf16 *Kr = reinterpret_cast<bf16 *>(smem_raw);  // [2][tile] row layout
    bf16 *Kt = Kr + 2 * kTileElems;                 // [2][tile] tr layout
    bf16 *Vr = Kt + 2 * kTileElems;                 // [2][tile] row layout

    const int qb = gridDim.x - 1 - blockIdx.x;
    const int n = blockIdx.y, bi = blockIdx.z;
    const int64_t h = (int64_t)nh * kD, ld = 3 * h;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int g = lane >> 5, c = lane & 31;
    const int q0 = qb * 128, qw0 = q0 + 32 * wave;
    const int64_t row0 = (int64_t)bi * seq;

    bf16x8 qf[8], dof[8];
    {
        const bf16 *qp = qkv + (row0 + qw0 + c) * ld + (int64_t)n * kD + 8 * g;
        const bf16 *dp = dattn + (row0 + qw0 + c) * h + (int64_t)n * kD + 8 * g;
#pragma unroll
        for (int st = 0; st < 8; ++st) {
            qf[st] = *reinterpret_cast<const bf16x8 *>(qp + 16 * st);
            dof[st] = *reinterpret_cast<const bf16x8 *>(dp + 16 * st);
        }
    }
    const int64_t stat = ((int64_t)bi * nh + n) * seq + qw0 + c;
    const float l2 = lse[stat] * 1.44269504088896340736f;
    const float dl = delta[stat];

    TileLoader lk, lv;
    lk.init(qkv + row0 * ld + h + (int64_t)n * kD, ld, tid);
    lv.init(qkv + row0 * ld + 2 * h + (int64_t)n * kD, ld, tid);

    f32x16 dqacc[4];
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) dqacc[t][e] = 0.0f;

    const int n_tiles = (q0 + 128) / kTile;
    lk.load(0);
    lv.load(0);
    lk.store_row(Kr);
    lk.store_tr(Kt);
    lv.store_row(Vr);
    __syncthreads();

    for (int jt = 0; jt < n_tiles; ++jt) {
        const int buf = jt & 1;
        if (jt + 1 < n_tiles) {
            lk.load((int64_t)(jt + 1) * kTile * ld);
            lv.load((int64_t)(jt + 1) * kTile * ld);
        }
        const int kv0 = jt * kTile;
        if (kv0 <= qw0 + 31) {
            const bf16 *kr = Kr + buf * kTileElems, *kt = Kt + buf * kTileElems, *vr = Vr + buf * kTileElems;
            f32x16 sacc[2], dpacc[2];
#pragma unroll
            for (int T = 0; T < 2; ++T) {
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    sacc[T][e] = 0.0f;
                    dpacc[T][e] = 0.0f;
                }
#pragma unroll
                for (int st = 0; st < 8; ++st) {
                    const bf16x8 kf = *reinterpret_cast<const bf16x8 *>(kr + off_row(32 * T + c, 2 * st + g));
                    sacc[T] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[st], sacc[T], 0, 0, 0);
                    const bf16x8 vf = *reinterpret_cast<const bf16x8 *>(vr + off_row(32 * T + c, 2 * st + g));
                    dpacc[T] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, dof[st], dpacc[T], 0, 0, 0);
                }
            }
            const bool need_mask = kv0 + kTile - 1 > qw0;
            bf16x8 dsf[4];
#pragma unroll
            for (int T = 0; T < 2; ++T)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    float p = fast_exp2(sacc[T][e] * scale_log2e - l2);
                    if (need_mask) {
                        const int kv = kv0 + 32 * T + 8 * (e >> 2) + 4 * g + (e & 3);
                        if (kv > qw0 + c) p = 0.0f;
                    }
                    dsf[2 * T + (e >> 3)][e & 7] = (bf16)(p * (dpacc[T][e] - dl));
                }
#pragma unroll
            for (int st = 0; st < 4; ++st) {
                const int k0 = 32 * (st >> 1) + 16 * (st & 1) + 4 * g;
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const bf16x8 ktf = read_tr8(kt, k0, k0 + 8, 32 * t + ((lane >> 4) & 1) * 16, lane);
                    dqacc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ktf, dsf[st], dqacc[t], 0, 0, 0);
                }
            }
        }
        if (jt + 1 < n_tiles) {
            lk.store_row(Kr + (buf ^ 1) * kTileElems);
            lk.store_tr(Kt + (buf ^ 1) * kTileElems);
            lv.store_row(Vr + (buf ^ 1) * kTileElems);
        }
        __syncthreads();
    }
    bf16 *op = dqkv + (row0 + qw0 + c) * ld + (int64_t)n * kD;
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int e4 = 0; e4 < 4; ++e4) {
            bf16x4 o;
#pragma unroll
            for (int r = 0; r < 4; ++r) o[r] = (bf16)(dqacc[t][e4 * 4 + r] * scale);
            *reinterpret_cast<bf16x4 *>(op + 32 * t + 8 * e4 + 4 * g) = o;
        }
}

// ------------------------------------------------------------------------------------ backward: dK, dV
// Lane = key.  Per query tile: S = Q K^T and dP = dO V^T (operands Q, dO row-wise from LDS; K, V in
// registers), P = exp2(S*c - lse[q]), dS = P o (dP - delta[q]); dV^T += dO^T P and dK^T += Q^T dS with
// dO^T, Q^T taken from second copies of the tiles through the transposing load.
__global__ __launch_bounds__(256) void attn_bwd_dkv_mfma_kernel(const bf16 *__restrict__ qkv,
                                                                const bf16 *__restrict__ dattn,
                                                                const float *__restrict__ lse,
                                                                const float *__restrict__ delta,
                                                                bf16 *__restrict__ dqkv, int seq, int nh, float scale,
                                                                float scale_log2e)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    bf16 *Qr = reinterpret_cast<bf16 *>(smem_raw);  // [2][tile]
    bf16 *Qt = Qr + 2 * kTileElems;
    bf16 *Dr = Qt + 2 * kTileElems;
    bf16 *Dt = Dr + 2 * kTileElems;

    const int kb = blockIdx.x;  // early key blocks see the most queries and come first
    const int n = blockIdx.y, bi = blockIdx.z;
    const int64_t h = (int64_t)nh * kD, ld = 3 * h;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int g = lane >> 5, c = lane & 31;
    const int kv0 = kb * 128, kvw0 = kv0 + 32 * wave;
    const int64_t row0 = (int64_t)bi * seq;

    bf16x8 kf[8], vf[8];
    {
        const bf16 *kp = qkv + (row0 + kvw0 + c) * ld + h + (int64_t)n * kD + 8 * g;
#pragma unroll
        for (int st = 0; st < 8; ++st) {
            kf[st] = *reinterpret_cast<const bf16x8 *>(kp + 16 * st);
            vf[st] = *reinterpret_cast<const bf16x8 *>(kp + h + 16 * st);
        }
    }
    TileLoader lq, ld_o;
    lq.init(qkv + row0 * ld + (int64_t)n * kD, ld, tid);
    ld_o.init(dattn + row0 * h + (int64_t)n * kD, h, tid);
    const float *lse_b = lse + ((int64_t)bi * nh + n) * seq;
    const float *del_b = delta + ((int64_t)bi * nh + n) * seq;

    f32x16 dkacc[4], dvacc[4];
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            dkacc[t][e] = 0.0f;
            dvacc[t][e] = 0.0f;
        }

    const int it0 = kv0 / kTile, n_tiles = seq / kTile;
    lq.load((int64_t)it0 * kTile * ld);
    ld_o.load((int64_t)it0 * kTile * h);
    lq.store_row(Qr);
    lq.store_tr(Qt);
    ld_o.store_row(Dr);
    ld_o.store_tr(Dt);
    __syncthreads();

    for (int it = it0; it < n_tiles; ++it) {
        const int buf = (it - it0) & 1;
        if (it + 1 < n_tiles) {
            lq.load((int64_t)(it + 1) * kTile * ld);
            ld_o.load((int64_t)(it + 1) * kTile * h);
        }
        const int qt0 = it * kTile;
        if (qt0 + kTile - 1 >= kvw0) {  // wave-uniform: some query of the tile sees some key of this wave
            const bf16 *qr = Qr + buf * kTileElems, *qt = Qt + buf * kTileElems;
            const bf16 *dr = Dr + buf * kTileElems, *dtp = Dt + buf * kTileElems;
            f32x16 sacc[2], dpacc[2];
#pragma unroll
            for (int T = 0; T < 2; ++T) {
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    sacc[T][e] = 0.0f;
                    dpacc[T][e] = 0.0f;
                }
#pragma unroll
                for (int st = 0; st < 8; ++st) {
                    const bf16x8 qf = *reinterpret_cast<const bf16x8 *>(qr + off_row(32 * T + c, 2 * st + g));
                    sacc[T] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf, kf[st], sacc[T], 0, 0, 0);
                    const bf16x8 df = *reinterpret_cast<const bf16x8 *>(dr + off_row(32 * T + c, 2 * st + g));
                    dpacc[T] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(df, vf[st], dpacc[T], 0, 0, 0);
                }
            }
            // sacc[T][e] of this lane: query qt0 + 32T + 8(e/4) + 4g + e%4, key kvw0 + c
            const bool need_mask = qt0 < kvw0 + 31;
            bf16x8 pf[4], dsf[4];
#pragma unroll
            for (int T = 0; T < 2; ++T)
#pragma unroll
                for (int e4 = 0; e4 < 4; ++e4) {
                    const int qrel = 32 * T + 8 * e4 + 4 * g;
                    const f32x4 l4 = *reinterpret_cast<const f32x4 *>(lse_b + qt0 + qrel);
                    const f32x4 d4 = *reinterpret_cast<const f32x4 *>(del_b + qt0 + qrel);
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const int e = e4 * 4 + r;
                        float p = fast_exp2(sacc[T][e] * scale_log2e - l4[r] * 1.44269504088896340736f);
                        if (need_mask && (kvw0 + c > qt0 + qrel + r)) p = 0.0f;
                        pf[2 * T + (e >> 3)][e & 7] = (bf16)p;
                        dsf[2 * T + (e >> 3)][e & 7] = (bf16)(p * (dpacc[T][e] - d4[r]));
                    }
                }
#pragma unroll
            for (int st = 0; st < 4; ++st) {
                const int k0 = 32 * (st >> 1) + 16 * (st & 1) + 4 * g;
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const int col = 32 * t + ((lane >> 4) & 1) * 16;
                    const bf16x8 dotf = read_tr8(dtp, k0, k0 + 8, col, lane);
                    dvacc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dotf, pf[st], dvacc[t], 0, 0, 0);
                    const bf16x8 qtf = read_tr8(qt, k0, k0 + 8, col, lane);
                    dkacc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qtf, dsf[st], dkacc[t], 0, 0, 0);
                }
            }
        }
        if (it + 1 < n_tiles) {
            lq.store_row(Qr + (buf ^ 1) * kTileElems);
            lq.store_tr(Qt + (buf ^ 1) * kTileElems);
            ld_o.store_row(Dr + (buf ^ 1) * kTileElems);
            ld_o.store_tr(Dt + (buf ^ 1) * kTileElems);
        }
        __syncthreads();
    }
    bf16 *okp = dqkv + (row0 + kvw0 + c) * ld + h + (int64_t)n * kD;
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int e4 = 0; e4 < 4; ++e4) {
            bf16x4 ok, ov;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                ok[r] = (bf16)(dkacc[t][e4 * 4 + r] * scale);
                ov[r] = (bf16)dvacc[t][e4 * 4 + r];
            }
            *reinterpret_cast<bf16x4 *>(okp + 32 * t + 8 * e4 + 4 * g) = ok;
            *reinterpret_cast<bf16x4 *>(okp + h + 32 * t + 8 * e4 + 4 * g) = ov;
        }
}

// delta[b, nh, s] = sum_e dattn * attn, one wavefront per (row, head): each lane owns two columns
__global__ __launch_bounds__(256) void attn_delta_mfma_kernel(const bf16 *__restrict__ attn,
                                                              const bf16 *__restrict__ dattn,
                                                              float *__restrict__ delta, int64_t rows, int seq, int nh)
{
    const int lane = threadIdx.x & 63;
    const int64_t item = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);  // (row, head)
    if (item >= rows * nh) return;
    const int64_t t = item / nh;
    const int n = (int)(item % nh);
    const int64_t base = t * ((int64_t)nh * kD) + (int64_t)n * kD + lane * 2;
    const bf16x2 a = *reinterpret_cast<const bf16x2 *>(attn + base);
    const bf16x2 d = *reinterpret_cast<const bf16x2 *>(dattn + base);
    float acc = (float)a[0] * (float)d[0] + (float)a[1] * (float)d[1];
    acc = wave_sum(acc);
    if (lane == 0) delta[((t / seq) * nh + n) * seq + (t % seq)] = acc;
}

bool attn_mfma_supported(int64_t seq, int64_t d) { return d == kD && seq % 128 == 0 && seq >= 128; }

template <class K>
static hipError_t set_lds(K kern, size_t lds, bool &done)
{
    if (done) return hipSuccess;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)lds);
    if (e == hipSuccess) done = true;
    return e;
}

hipError_t launch_attn_fwd(int dt, const void *qkv, void *attn, float *lse, int64_t b, int64_t seq, int64_t nh,
                           int64_t d, hipStream_t s)
{
    if (dt != DT_BF16 || !attn_mfma_supported(seq, d)) return hipErrorInvalidValue;
    if (b * seq == 0) return hipSuccess;
    constexpr size_t lds = 4 * kTileElems * sizeof(bf16);  // 64 KB
    static bool attr_set = false;
    if (hipError_t e = set_lds(attn_fwd_mfma_kernel, lds, attr_set)) return e;
    const float scale_log2e = (1.0f / sqrtf((float)d)) * 1.44269504088896340736f;
    const dim3 grid((unsigned)(seq / 128), (unsigned)nh, (unsigned)b);
    attn_fwd_mfma_kernel<<<grid, 256, lds, s>>>((const bf16 *)qkv, (bf16 *)attn, lse, (int)seq, (int)nh, scale_log2e);
    return hipGetLastError();
}

hipError_t launch_attn_bwd(int dt, const void *qkv, const void *attn, const void *dattn, const float *lse,
                           float *delta, void *dqkv, int64_t b, int64_t seq, int64_t nh, int64_t d, hipStream_t s)
{
    if (dt != DT_BF16 || !attn_mfma_supported(seq, d)) return hipErrorInvalidValue;
    if (b * seq == 0) return hipSuccess;
    static bool a1 = false, a2 = false;
    constexpr size_t lds_dq = 6 * kTileElems * sizeof(bf16);   // 96 KB
    constexpr size_t lds_dkv = 8 * kTileElems * sizeof(bf16);  // 128 KB
    if (hipError_t e = set_lds(attn_bwd_dq_mfma_kernel, lds_dq, a1)) return e;
    if (hipError_t e = set_lds(attn_bwd_dkv_mfma_kernel, lds_dkv, a2)) return e;
    const float scale = 1.0f / sqrtf((float)d);
    const float scale_log2e = scale * 1.44269504088896340736f;
    const int64_t rows = b * seq;
    attn_delta_mfma_kernel<<<(unsigned)((rows * nh + 3) / 4), 256, 0, s>>>((const bf16 *)attn, (const bf16 *)dattn,
                                                                            delta, rows, (int)seq, (int)nh);
    const dim3 grid((unsigned)(seq / 128), (unsigned)nh, (unsigned)b);
    attn_bwd_dq_mfma_kernel<<<grid, 256, lds_dq, s>>>((const bf16 *)qkv, (const bf16 *)dattn, lse, delta,
                                                      (bf16 *)dqkv, (int)seq, (int)nh, scale, scale_log2e);
    attn_bwd_dkv_mfma_kernel<<<grid, 256, lds_dkv, s>>>((const bf16 *)qkv, (const bf16 *)dattn, lse, delta,
                                                        (bf16 *)dqkv, (int)seq, (int)nh, scale, scale_log2e);
    return hipGetLastError();
}

}  // namespace zpp
