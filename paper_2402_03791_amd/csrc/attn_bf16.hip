// Fused causal attention for bf16, head dim 128, on gfx950 MFMA (v_mfma_f32_32x32x16_bf16).
//
// A wave owns 32 queries (forward, dQ) or 32 keys (dK, dV); a work-group covers 128 consecutive ones.  Under
// the causal mask a work-group's work grows with its position in the sequence; the heavy ones are dispatched
// first.  Keys/values (or queries/dO) stream through LDS in tiles of 64 rows, copied global -> LDS directly.
// Scores are computed transposed, S^T = K Q^T, so that a lane owns one query column and the softmax row
// reductions are in-lane plus one exchange with the lane 32 away; the probabilities then feed the second
// product O^T = V^T P^T straight from the accumulator registers.  The value tile is read with the LDS
// transposing load (ds_read_b64_tr_b16), which hands each lane four consecutive key rows of one value
// column.  The softmax never leaves registers; only O and the log-sum-exp are written.
//
// Work-group shapes.  Forward and dQ: four waves, each taking every tile of its 32 rows, two stages of one tile
// pair in LDS (64 KB), two work-groups per CU.  dK/dV: four waves, one per SIMD, with all 512 registers each
// and four stages of tiles in LDS; see the kernel.  Every kernel serves every launch size: what a launch computes
// for a sample does not depend on how many samples it holds.
//
// Backward: two launches without atomics.  dQ: lane = query, loops over key tiles.  dK and dV: lane = key,
// loop over query tiles.  P is recomputed from the saved log-sum-exp; delta = rowsum(dO o O) and the
// log-sum-exp in base-2 units are computed by the dQ kernel and handed to the dK/dV kernel.
//
// What a wave can issue bounds these kernels as much as the matrix unit does: a SIMD issues one vector
// instruction per four cycles, the element-wise part of a tile is as long as its matrix part (about 130
// instructions against 32 of 32 cycles each in the forward kernel), and matrix and vector work of two waves on a
// SIMD overlap only in part (measured on a synthetic mix: 16 matrix instructions and a softmax-sized block of
// vector work take 455 ns on one SIMD when two waves each do one kind, 570 ns one after the other, 290 ns each
// alone).  Hence the trimming of the element-wise parts below.
#include "device_utils.h"
#include "kernels.h"

#include <type_traits>

namespace zpp {

typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

constexpr int kD = 128;        // head dim
constexpr int kTile = 64;      // rows of a streamed tile
constexpr int kTileBytes = kTile * kD * 2;  // 16 KB

// One LDS layout serves both ways a [64][128] bf16 tile (256-byte rows, 16 chunks of 16 bytes) is
// read: chunk c of row r sits at chunk position c ^ g(r), g(r) = ((r & 3) << 2) | ((r >> 2) & 3).
//  - row-wise MFMA operand (16 consecutive rows, same chunk): g takes 16 different values;
//  - transposing load (4 consecutive rows x 4 consecutive chunks): bits 2..3 of the position follow
//    the row, bits 0..1 the chunk, again 16 different positions.
__device__ __forceinline__ int swz(int row) { return ((row & 3) << 2) | ((row >> 2) & 3); }

// Global -> LDS copy of a tile, 16 load instructions shared by the NW waves of the work-group (4 rows of
// 256 bytes each): lane i of a load lands at byte 16*i of the 1 KB slot, so it fetches the chunk the
// swizzle assigns to that place.
template <int NW>
struct TileCopy {
    static constexpr int NL = 16 / NW;  // loads per wave per tile
    uint32_t voff[NL];
    __device__ __forceinline__ void init(int lane, int wave, int64_t ld_elems)
    {
#pragma unroll
        for (int j = 0; j < NL; ++j) {
            const int row = wave * (64 / NW) + j * 4 + (lane >> 4);
            const int c = (lane & 15) ^ swz(row);
            voff[j] = (uint32_t)((row * ld_elems + c * 8) * 2);
        }
    }
    // base: first byte of the tile's row 0 (uniform); lds_tile: LDS byte address of the tile (uniform)
    __device__ __forceinline__ void issue(const char *base, uint32_t lds_tile, int wave) const
    {
#pragma unroll
        for (int j = 0; j < NL; ++j) {
            const uint32_t dst = lds_tile + wave * (16384 / NW) + j * 1024;
            asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                         :
                         : "s"(dst), "v"(voff[j]), "s"(base)
                         : "memory");
        }
    }
};

// Per-lane LDS byte offsets (inside a tile) for the two read patterns.
struct TileAddr {
    uint32_t row[8];    // row-wise operand: rows lane%32 (+32 per MFMA tile), K sub-step st = 0..7
    uint32_t tr[4][2];  // transposing load: column tile t = 0..3, first/second group of 4 rows
    __device__ __forceinline__ void init(int lane)
    {
        const int r = lane & 31, gh = lane >> 5;
#pragma unroll
        for (int st = 0; st < 8; ++st) row[st] = r * 256 + (((2 * st + gh) ^ swz(r)) << 4);
        const int i = lane & 15, e = i >> 2, q4 = i & 3, half = (lane >> 4) & 1;
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int hi = 0; hi < 2; ++hi) {
                // row = k0 + e with k0 = (compile-time multiple of 16) + 4*gh + 8*hi
                const int rr = 4 * gh + 8 * hi + e;
                const int c = 4 * t + 2 * half + (q4 >> 1);
                tr[t][hi] = (4 * gh + e) * 256 + ((c ^ swz(rr)) << 4) + (q4 & 1) * 8;
            }
    }
};

// MFMA operand rows (32*T + lane%32), K sub-step st, from a tile at LDS byte address `tile`
__device__ __forceinline__ bf16x8 rd_row(const unsigned char *tile, const TileAddr &a, int T, int st)
{
    return *reinterpret_cast<const bf16x8 *>(tile + a.row[st] + T * 8192);
}
// MFMA operand gathered down the rows: column 32*t + lane%32 (as the operand's row index), K slots =
// tile rows 16*st + 8*(lane/32) .. +7 in the order the accumulator layout of S^T / S produces them:
// (4*gh + 0..3) then (8 + 4*gh + 0..3) inside each group of 16 rows.
__device__ __forceinline__ bf16x8 rd_tr(const unsigned char *tile, const TileAddr &a, int t, int st)
{
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(tile + a.tr[t][0] + st * 4096));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(tile + a.tr[t][1] + st * 4096 + 2048));
    return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
}

// Work-group -> (block of the sequence, head, sample) for a 1-D grid of nblk * nh * nb work-groups whose
// work grows with the block index.  The (sample, head) pairs are taken in chunks of about two residencies of
// the chip (1024 work-groups); inside a chunk the heaviest blocks of all its pairs come first, then the next
// lighter ones: a CU takes its next work-group when it has finished one, so this order packs the unequal
// work-groups tightly, and the light tail of one chunk runs beside the heavy head of the next.  Work-groups are
// dealt round-robin over the 8 XCDs, each with a private L2: all work-groups of one pair go to the same XCD, and
// an XCD works on chunk / 8 pairs at a time, so a pair's K/V (or Q/dO) rows are still near when the pair's other
// blocks want them, however many samples the launch has (one chunk over everything, the order used before, loses
// a quarter of the forward kernel's speed at 16 samples of 32 heads, and chunks of one residency start the
// last chunk's long work-groups too late).  chunk = 0: the whole grid is one chunk.  The last chunk may be
// shorter than the others.
__device__ __forceinline__ void decode_heavy_first(int id, int nblk, int nh, int nb, int chunk, int &blk, int &n, int &bi)
{
    const int nv = nh * nb;
    int k, v;
    if (chunk > 0) {
        const int per = nblk * chunk, ch = id / per, r = id - ch * per;
        const int cs = min(chunk, nv - ch * chunk);  // pairs of this chunk
        const int x = r & 7, j = r >> 3, ppx = cs >> 3;
        k = j / ppx;
        v = ch * chunk + (j - k * ppx) * 8 + x;
    } else if ((nv & 7) == 0) {
        const int j = id >> 3, per = nv >> 3;
        k = j / per;
        v = (j % per) * 8 + (id & 7);
    } else {
        k = id / nv;
        v = id % nv;
    }
    blk = nblk - 1 - k;
    n = v % nh;
    bi = v / nh;
}

// pairs per chunk for a launch over nv (sample, head) pairs: about 1024 work-groups per chunk, a multiple of 16;
// 0 (one chunk) when there is no more than a chunk of them or they cannot be dealt evenly to the XCDs
static int chunk_slots(int64_t nblk, int64_t nv)
{
    int64_t c = (1024 / nblk) / 16 * 16;
    if (c < 16) c = 16;
    return (nv % 8 == 0 && nv > c) ? (int)c : 0;
}

// depth of the register rings that carry LDS operands to the matrix instructions of the backward kernels
// (what fits beside the accumulators at two waves per SIMD)
constexpr int kRingDq = 4;

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// The tile copies are issued from inline assembly, so the compiler's own bookkeeping of outstanding global loads
// does not know about them.  If ordinary loads (the operands a wave keeps in registers) are still pending, by
// that bookkeeping, when the main loop is entered, the compiler puts its waits for them at their first use
// inside the loop, where on every later iteration they wait for the tile copies in flight instead and undo
// the overlap of copying and computing.  Naming a register as the input of an (empty) assembly statement makes
// the compiler wait for its load here, before the loop.
__device__ __forceinline__ void loaded_before_here(const bf16x8 &v)
{
    asm volatile("" : : "v"(__builtin_bit_cast(u32x4, v)));
}

__device__ __forceinline__ uint32_t lds_addr_of(const void *p)
{
    return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const unsigned char *)p;
}

// max over the two lanes that share a query column (lane and lane ^ 32), without a trip through LDS:
// v_permlane32_swap exchanges the upper half of one register with the lower half of another.
__device__ __forceinline__ float max_with_lane32(float v)
{
    const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
}
__device__ __forceinline__ float sum_with_lane32(float v)
{
    const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return __uint_as_float(sw[0]) + __uint_as_float(sw[1]);
}

// One step of the online softmax for a lane's 32 scores of a key tile (two accumulator blocks of S^T):
// p = 2^(s*c - m*c) as bf16 operands for the second product, row sum added to l_run.  The running maximum
// m_run only has to bound the scores to within what the arithmetic tolerates, so it is raised (and the output
// accumulator rescaled) only when some query of the wave sees a score more than 2^8 above it in the exponent:
// after the first tiles of a row that almost never happens, and the 64 multiplications of the accumulator and
// their wait for the previous tile's matrix instructions fall away.  The final division by the row sum makes the
// result independent of which m was used.
__device__ __forceinline__ void online_softmax_step(const f32x16 (&sacc)[2], float &m_run, float &l_run, f32x16 (&oacc)[4],
                                                    bf16x8 (&pf)[4], float scale_log2e, float lazy)
{
    float mloc = sacc[0][0];
#pragma unroll
    for (int T = 0; T < 2; ++T)
#pragma unroll
        for (int e = 0; e < 16; ++e) mloc = fmaxf(mloc, sacc[T][e]);
    mloc = max_with_lane32(mloc);
    if (__builtin_amdgcn_ballot_w64(mloc > m_run + lazy) != 0) {
        const float m_new = fmaxf(m_run, mloc);
        const float alpha = fast_exp2((m_run - m_new) * scale_log2e);
        l_run *= alpha;
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int e = 0; e < 16; ++e) oacc[t][e] *= alpha;
        m_run = m_new;
    }
    const float mc = m_run * scale_log2e;
    float psum = 0.0f;
#pragma unroll
    for (int T = 0; T < 2; ++T)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const float pe = fast_exp2(__builtin_fmaf(sacc[T][e], scale_log2e, -mc));
            psum += pe;
            pf[2 * T + (e >> 3)][e & 7] = (bf16)pe;
        }
    l_run += psum;
}

// A wave's 32 x 128 result block (accumulator layout: lane = row, registers along d) goes out through a
// wave-private 8 KB of LDS so that every store instruction writes four whole 256-byte rows: straight from the
// accumulator layout a store would touch 32 rows with 8 bytes each.  `w` must not be in use by anyone else.
__device__ __forceinline__ void store_rows_via_lds(const f32x16 (&acc)[4], float mul, unsigned char *w, bf16 *row0_ptr,
                                                  int64_t ld_elems, int lane)
{
    const int c = lane & 31, g = lane >> 5;
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int e4 = 0; e4 < 4; ++e4) {
            bf16x4 o;
#pragma unroll
            for (int r = 0; r < 4; ++r) o[r] = (bf16)(acc[t][e4 * 4 + r] * mul);
            *reinterpret_cast<bf16x4 *>(w + c * 256 + (((4 * t + e4) ^ (c & 15)) << 4) + g * 8) = o;
        }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int r = 4 * i + (lane >> 4), pos = lane & 15;
        const bf16x8 v = *reinterpret_cast<const bf16x8 *>(w + r * 256 + (pos << 4));
        *reinterpret_cast<bf16x8 *>(row0_ptr + r * ld_elems + ((pos ^ (r & 15)) << 3)) = v;
    }
}

// ------------------------------------------------------------------------------------ forward
// Four waves on 128 consecutive queries: every wave takes all key tiles of its 32 queries, tiles streamed one by
// one through two stages of 32 KB, so two work-groups fit a CU and run out of step with each other (one's matrix
// phase against the other's softmax phase, one's prologue and epilogue behind the other's tiles).  Work-groups are
// as heavy as their position in the sequence; the heavy ones are dispatched first.  One kernel for every launch
// size, so that a sample's result does not depend on how many samples the launch holds (an eight-wave form whose
// two waves per SIMD split a query group's key tiles and merged at the end was 5 % faster on launches of at most
// two work-groups per CU, 54 against 57 us at 32 heads x 2048, and gave other bits).
__global__ __launch_bounds__(256, 2) void attn_fwd_w4_kernel(const bf16 *__restrict__ qkv, bf16 *__restrict__ attn,
                                                             float *__restrict__ lse, int seq, int nh, int nb,
                                                             int chunk, float scale_log2e)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];  // [2 stages][K tile | V tile]
    int qb, n, bi;
    decode_heavy_first(blockIdx.x, seq / 128, nh, nb, chunk, qb, n, bi);
    const int64_t h = (int64_t)nh * kD, ld = 3 * h;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 5, c = lane & 31;
    const int qw0 = 128 * qb + 32 * wave;
    const int64_t row0 = (int64_t)bi * seq;

    bf16x8 qf[8];
    {
        const bf16 *qp = qkv + (row0 + qw0 + c) * ld + (int64_t)n * kD + 8 * g;
#pragma unroll
        for (int st = 0; st < 8; ++st) qf[st] = *reinterpret_cast<const bf16x8 *>(qp + 16 * st);
    }
    TileCopy<4> cp;
    cp.init(lane, wave, ld);
    TileAddr ad;
    ad.init(lane);
    const char *kbase = reinterpret_cast<const char *>(qkv + row0 * ld + h + (int64_t)n * kD);
    const char *vbase = kbase + h * 2;
    const int64_t tile_stride = (int64_t)kTile * ld * 2;
    const uint32_t lds0 = lds_addr_of(smem);

    f32x16 oacc[4];
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) oacc[t][e] = 0.0f;
    float m_run = -INFINITY, l_run = 0.0f;
    const float lazy = 8.0f / scale_log2e;  // 2^8 in the exponent, in units of the raw scores

    const int n_tiles = 2 * (qb + 1);
    const int my_tiles = qw0 / kTile + 1;
    auto issue_tile = [&](int jt) {
        const uint32_t dst = lds0 + (jt & 1) * 2 * kTileBytes;
        cp.issue(kbase + jt * tile_stride, dst, wave);
        cp.issue(vbase + jt * tile_stride, dst + kTileBytes, wave);
    };
    issue_tile(0);
#pragma unroll
    for (int st = 0; st < 8; ++st) loaded_before_here(qf[st]);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();

    for (int jt = 0; jt < n_tiles; ++jt) {
        if (jt + 1 < n_tiles) issue_tile(jt + 1);
        if (jt < my_tiles) {
            const int kv0 = jt * kTile;
            const unsigned char *ks = smem + (jt & 1) * 2 * kTileBytes;
            const unsigned char *vs = ks + kTileBytes;
            f32x16 sacc[2] = {};
            bf16x8 kr[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) kr[i] = rd_row(ks, ad, 0, i);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                sacc[i >> 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kr[i & 3], qf[i & 7], sacc[i >> 3], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
                if (i + 4 < 16) {
                    kr[i & 3] = rd_row(ks, ad, (i + 4) >> 3, (i + 4) & 7);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            bf16x8 vr[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) vr[i] = rd_tr(vs, ad, i & 3, i >> 2);
            __builtin_amdgcn_sched_barrier(0);
            if (kv0 + kTile - 1 > qw0) {
#pragma unroll
                for (int T = 0; T < 2; ++T)
#pragma unroll
                    for (int e = 0; e < 16; ++e) {
                        const int kv = kv0 + 32 * T + 8 * (e >> 2) + 4 * g + (e & 3);
                        if (kv > qw0 + c) sacc[T][e] = -INFINITY;
                    }
            }
            bf16x8 pf[4];
            online_softmax_step(sacc, m_run, l_run, oacc, pf, scale_log2e, lazy);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                oacc[i & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vr[i & 3], pf[i >> 2], oacc[i & 3], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
                if (i + 4 < 16) {
                    vr[i & 3] = rd_tr(vs, ad, (i + 4) & 3, (i + 4) >> 2);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
    }
    const float l_tot = sum_with_lane32(l_run);
    const float inv = 1.0f / l_tot;
    // (the loop's last barrier has every wave out of the stages)
    store_rows_via_lds(oacc, inv, smem + wave * 8192, attn + (row0 + qw0) * h + (int64_t)n * kD, h, lane);
    if (g == 0)
        lse[((int64_t)bi * nh + n) * seq + qw0 + c] =
            (m_run * scale_log2e + __builtin_amdgcn_logf(l_tot)) * 0.69314718055994530942f;
}

// ------------------------------------------------------------------------------------ backward: dQ
// Lane = query.  Per key tile: S^T = K Q^T and dP^T = V dO^T (operands K, V row-wise from LDS; Q, dO
// in registers), P^T = exp2(S^T*c - lse), dS^T = P^T o (dP^T - delta), dQ^T += K^T dS^T with K^T
// gathered from the same key tile through the transposing load.  It also computes
// delta[q] = sum_e dO[q,e] * O[q,e] for its queries and stores it for the dK kernel, which runs after it.
// Four waves per work-group on 128 consecutive queries: every wave all key tiles of its 32 queries, tiles
// streamed one by one through two stages, two work-groups per CU.
__global__ __launch_bounds__(256, 2) void attn_bwd_dq_w4_kernel(const bf16 *__restrict__ qkv, const bf16 *__restrict__ attn,
                                                                const bf16 *__restrict__ dattn,
                                                                const float *__restrict__ lse, float *__restrict__ delta,
                                                                bf16 *__restrict__ dqkv, int seq, int nh, int nb,
                                                                int chunk, float scale, float scale_log2e)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];  // [2 stages][K tile | V tile]
    int qb, n, bi;
    decode_heavy_first(blockIdx.x, seq / 128, nh, nb, chunk, qb, n, bi);
    const int64_t h = (int64_t)nh * kD, ld = 3 * h;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 5, c = lane & 31;
    const int qw0 = 128 * qb + 32 * wave;
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
    float dl = 0.0f;
    {
        const bf16 *op = attn + (row0 + qw0 + c) * h + (int64_t)n * kD + 8 * g;
#pragma unroll
        for (int st = 0; st < 8; ++st) {
            const bf16x8 of = *reinterpret_cast<const bf16x8 *>(op + 16 * st);
#pragma unroll
            for (int k = 0; k < 8; ++k) dl = __builtin_fmaf((float)dof[st][k], (float)of[k], dl);
        }
        dl = sum_with_lane32(dl);
        if (g == 0) {
            delta[stat] = dl;
            delta[(int64_t)nb * nh * seq + stat] = l2;  // the statistic in the units the exponentials use
        }
    }
    TileCopy<4> cp;
    cp.init(lane, wave, ld);
    TileAddr ad;
    ad.init(lane);
    const char *kbase = reinterpret_cast<const char *>(qkv + row0 * ld + h + (int64_t)n * kD);
    const char *vbase = kbase + h * 2;
    const int64_t tile_stride = (int64_t)kTile * ld * 2;
    const uint32_t lds0 = lds_addr_of(smem);

    f32x16 dqacc[4];
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) dqacc[t][e] = 0.0f;

    const int n_tiles = 2 * (qb + 1);
    const int my_tiles = qw0 / kTile + 1;
    auto issue_tile = [&](int jt) {
        const uint32_t dst = lds0 + (jt & 1) * 2 * kTileBytes;
        cp.issue(kbase + jt * tile_stride, dst, wave);
        cp.issue(vbase + jt * tile_stride, dst + kTileBytes, wave);
    };
    issue_tile(0);
#pragma unroll
    for (int st = 0; st < 8; ++st) {
        loaded_before_here(qf[st]);
        loaded_before_here(dof[st]);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();

    for (int jt = 0; jt < n_tiles; ++jt) {
        if (jt + 1 < n_tiles) issue_tile(jt + 1);
        if (jt < my_tiles) {
            const int kv0 = jt * kTile;
            const unsigned char *ks = smem + (jt & 1) * 2 * kTileBytes;
            const unsigned char *vs = ks + kTileBytes;
            const bool diag = kv0 + kTile - 1 > qw0;
            // Half a tile (32 keys) at a time: its 16 score and dP instructions, its element-wise part, then the
            // 8 dQ instructions that consume its dS, so that only two operand registers of dS are live.  LDS
            // operands go through small rings of registers, requested kRingDq steps ahead of their use, order pinned.
#pragma unroll
            for (int T = 0; T < 2; ++T) {
                f32x16 sacc, dpacc;
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    sacc[e] = 0.0f;
                    dpacc[e] = 0.0f;
                }
                bf16x8 kr[kRingDq], vr[kRingDq];
#pragma unroll
                for (int i = 0; i < kRingDq; ++i) {
                    kr[i] = rd_row(ks, ad, T, i);
                    vr[i] = rd_row(vs, ad, T, i);
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int st = 0; st < 8; ++st) {
                    sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kr[st % kRingDq], qf[st], sacc, 0, 0, 0);
                    __builtin_amdgcn_sched_barrier(0);
                    if (st + kRingDq < 8) {
                        kr[st % kRingDq] = rd_row(ks, ad, T, st + kRingDq);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                    dpacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vr[st % kRingDq], dof[st], dpacc, 0, 0, 0);
                    __builtin_amdgcn_sched_barrier(0);
                    if (st + kRingDq < 8) {
                        vr[st % kRingDq] = rd_row(vs, ad, T, st + kRingDq);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
                // the first K^T operands of the dQ product travel during the element-wise part
                bf16x8 tr[kRingDq];
#pragma unroll
                for (int i = 0; i < kRingDq; ++i) tr[i] = rd_tr(ks, ad, i & 3, 2 * T + (i >> 2));
                __builtin_amdgcn_sched_barrier(0);
                if (diag) {
#pragma unroll
                    for (int e = 0; e < 16; ++e) {
                        const int kv = kv0 + 32 * T + 8 * (e >> 2) + 4 * g + (e & 3);
                        if (kv > qw0 + c) sacc[e] = -INFINITY;
                    }
                }
                bf16x8 dsf[2];
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const float pe = fast_exp2(__builtin_fmaf(sacc[e], scale_log2e, -l2));
                    dsf[e >> 3][e & 7] = (bf16)(pe * (dpacc[e] - dl));
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int i = 0; i < 8; ++i) {  // i = 4 * (step of 16 keys) + t
                    dqacc[i & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tr[i % kRingDq], dsf[i >> 2], dqacc[i & 3], 0, 0, 0);
                    __builtin_amdgcn_sched_barrier(0);
                    if (i + kRingDq < 8) {
                        tr[i % kRingDq] = rd_tr(ks, ad, (i + kRingDq) & 3, 2 * T + ((i + kRingDq) >> 2));
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
            }
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
    }
    // (the loop's last barrier has every wave out of the stages)
    store_rows_via_lds(dqacc, scale, smem + wave * 8192, dqkv + (row0 + qw0) * ld + (int64_t)n * kD, ld, lane);
}

// ------------------------------------------------------------------------------------ backward: dK and dV
// One wave per SIMD (four per work-group, 128 consecutive keys, lane = key) with all 512 registers: K and V
// fragments and both accumulators stay in registers, and S and P are computed once for both products: 64 matrix
// instructions per tile of 64 queries (split in a dK and a dV body, each small enough for two waves per SIMD, the
// kernel needs 80 and three times the exponentials).  The element-wise part of one half tile (32 queries) is issued
// between the matrix instructions of the next half tile's S and dP products, one element per instruction, so
// that the vector unit works in the shadow of the matrix unit:
//     [S, dP of half u+1  ||  P, dS of half u]   [dV, dK of half u]   ...
// Query tiles (Q rows, dO rows, and the two per-query statistics) stream through four LDS stages, copied two
// tiles ahead.  All four waves walk all tiles of the key block (the first tile is fully masked for the upper two
// waves: uniform control flow is worth more than the skipped half tile).  With one wave per SIMD nothing hides
// a work-group's start and end, so the key block's own K and V rows arrive through LDS with coalesced copies
// and the results leave through LDS in whole rows.  Measured per work-group (timestamps in the kernel, 32
// heads x 2048, two samples): about 3950 cycles per tile against 2048 of matrix instructions - a lone wave
// issues its ~590 instructions per tile (64 matrix, 112 LDS reads, 160 element-wise, 64 accumulator reads, waits
// and addresses) at one per 6-7 cycles - and 9400 + 8800 cycles before and after the tiles with plain loads and
// stores from the accumulator layout, which the LDS paths cut.  Against the two-body kernel: 6 to 9 % less time
// for the backward pass.
constexpr int kFStages = 4;
constexpr int kFStageBytes = 2 * kTileBytes + 512;  // Q tile | dO tile | 64 log-sum-exp | 64 delta
constexpr int kFRingA = 4, kFRingB = 4;

// S and dP of half tile TA of the tile at `ta` into (sa, da); between its matrix instructions the element-wise
// part of half TV of the tile whose statistics lie at `stat`, from its scores and dP in (sv, dv), to the operands
// (pf, dsf) of the second products.  MASK (the first two tiles of a key block): elements with in-tile query index
// (less 4 g) below qlim are masked.
// A matrix instruction whose accumulator is kept in ordinary vector registers.  In a kernel that may use more than
// 256 registers the compiler gives every matrix instruction an accumulator in the second register file, and the
// element-wise code then pays one copy instruction per value it reads; written out, the S and dP accumulators stay
// where the vector unit reads them.  The compiler inserts no wait states around these, so results may only be
// read a phase (sixteen matrix instructions) later, which is how the kernel below is arranged anyway.
__device__ __forceinline__ void mfma_v_first(f32x16 &acc, const bf16x8 &a, const bf16x8 &b)
{
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(acc) : "v"(a), "v"(b));
}
__device__ __forceinline__ void mfma_v(f32x16 &acc, const bf16x8 &a, const bf16x8 &b)
{
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(acc) : "v"(a), "v"(b));
}

template <bool WITH_A, bool MASK, int TA, int TV>
__device__ __forceinline__ void dkv_scores_and_elementwise(f32x16 &sa, f32x16 &da, const f32x16 &sv, const f32x16 &dv,
                                                           bf16x8 (&pf)[2], bf16x8 (&dsf)[2], const unsigned char *ta,
                                                           const TileAddr &ad, const bf16x8 (&kf)[8],
                                                           const bf16x8 (&vf)[8], const float *stat, float scale_log2e,
                                                           int qlim, int g)
{
    // the statistics of four queries at a time, requested one group ahead
    f32x4 l4[2], d4[2];
    l4[0] = *reinterpret_cast<const f32x4 *>(stat + 32 * TV + 4 * g);
    d4[0] = *reinterpret_cast<const f32x4 *>(stat + 64 + 32 * TV + 4 * g);
    bf16x8 qr[kFRingA], dr[kFRingA];
    if constexpr (WITH_A) {
#pragma unroll
        for (int i = 0; i < kFRingA; ++i) {
            qr[i] = rd_row(ta, ad, TA, i);
            dr[i] = rd_row(ta + kTileBytes, ad, TA, i);
        }
    }
    __builtin_amdgcn_sched_barrier(0);
    float x0 = 0.0f, x1 = 0.0f, e0 = 0.0f, t0 = 0.0f;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        if constexpr (WITH_A) {
            const int k = i >> 1;
            if ((i & 1) == 0) {
                if (k == 0) mfma_v_first(sa, qr[0], kf[0]);
                else mfma_v(sa, qr[k % kFRingA], kf[k]);
                __builtin_amdgcn_sched_barrier(0);
                if (k + kFRingA < 8) qr[k % kFRingA] = rd_row(ta, ad, TA, k + kFRingA);
            } else {
                if (k == 0) mfma_v_first(da, dr[0], vf[0]);
                else mfma_v(da, dr[k % kFRingA], vf[k]);
                __builtin_amdgcn_sched_barrier(0);
                if (k + kFRingA < 8) dr[k % kFRingA] = rd_row(ta + kTileBytes, ad, TA, k + kFRingA);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        // elements i - 1 and i (a pair) of half TV: query 32 TV + 8 (e / 4) + 4 g + e % 4 of the tile.  The pair's
        // work is spread over the two slots so that no instruction uses the result of the one before it.
        if ((i & 3) == 0 && i + 4 < 16) {
            l4[((i >> 2) + 1) & 1] = *reinterpret_cast<const f32x4 *>(stat + 32 * TV + 8 * ((i >> 2) + 1) + 4 * g);
            d4[((i >> 2) + 1) & 1] = *reinterpret_cast<const f32x4 *>(stat + 64 + 32 * TV + 8 * ((i >> 2) + 1) + 4 * g);
        }
        if ((i & 1) == 0) {
            float sm0 = sv[i], sm1 = sv[i + 1];
            if constexpr (MASK) {
                if (qlim > 32 * TV + 8 * (i >> 2) + (i & 3)) sm0 = -INFINITY;
                if (qlim > 32 * TV + 8 * (i >> 2) + (i & 3) + 1) sm1 = -INFINITY;
            }
            x0 = __builtin_fmaf(sm0, scale_log2e, -l4[(i >> 2) & 1][i & 3]);
            x1 = __builtin_fmaf(sm1, scale_log2e, -l4[(i >> 2) & 1][(i & 3) + 1]);
            t0 = dv[i] - d4[(i >> 2) & 1][i & 3];
            e0 = fast_exp2(x0);
        } else {
            const float e1 = fast_exp2(x1);
            const float t1 = dv[i] - d4[(i >> 2) & 1][i & 3];
            const float m0 = e0 * t0;
            pf[i >> 3][(i & 7) - 1] = (bf16)e0;
            pf[i >> 3][i & 7] = (bf16)e1;
            const float m1 = e1 * t1;
            dsf[i >> 3][(i & 7) - 1] = (bf16)m0;
            dsf[i >> 3][i & 7] = (bf16)m1;
        }
        __builtin_amdgcn_sched_barrier(0);
    }
}

// dV += dO^T P and dK += Q^T dS for half tile TB of the tile at `tb`
template <int TB>
__device__ __forceinline__ void dkv_second_products(const bf16x8 (&pf)[2], const bf16x8 (&dsf)[2], const unsigned char *tb,
                                                    const TileAddr &ad, f32x16 (&acck)[4], f32x16 (&accv)[4])
{
    bf16x8 rv[kFRingB], rk[kFRingB];
#pragma unroll
    for (int i = 0; i < kFRingB; ++i) {
        rv[i] = rd_tr(tb + kTileBytes, ad, i & 3, 2 * TB + (i >> 2));
        rk[i] = rd_tr(tb, ad, i & 3, 2 * TB + (i >> 2));
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < 8; ++i) {  // i = 4 * (step of 16 queries) + t
        accv[i & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(rv[i % kFRingB], pf[i >> 2], accv[i & 3], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        if (i + kFRingB < 8) rv[i % kFRingB] = rd_tr(tb + kTileBytes, ad, (i + kFRingB) & 3, 2 * TB + ((i + kFRingB) >> 2));
        __builtin_amdgcn_sched_barrier(0);
        acck[i & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(rk[i % kFRingB], dsf[i >> 2], acck[i & 3], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        if (i + kFRingB < 8) rk[i % kFRingB] = rd_tr(tb, ad, (i + kFRingB) & 3, 2 * TB + ((i + kFRingB) >> 2));
        __builtin_amdgcn_sched_barrier(0);
    }
}

__global__ __launch_bounds__(256, 1) void attn_bwd_dkv_kernel(const bf16 *__restrict__ qkv,
                                                                    const bf16 *__restrict__ dattn,
                                                                    const float *__restrict__ delta,
                                                                    bf16 *__restrict__ dqkv, int seq, int nh, int nb,
                                                                    int chunk, float scale, float scale_log2e)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];  // [4 stages][Q tile | dO tile | statistics]
    int blk, n, bi;
    decode_heavy_first(blockIdx.x, seq / 128, nh, nb, chunk, blk, n, bi);
    const int kb = seq / 128 - 1 - blk;
    const int64_t h = (int64_t)nh * kD, ld = 3 * h;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 5, c = lane & 31;
    const int kvw0 = 128 * kb + 32 * wave;
    const int64_t row0 = (int64_t)bi * seq;

    TileCopy<4> cq, cd;
    cq.init(lane, wave, ld);
    cd.init(lane, wave, h);
    TileAddr ad;
    ad.init(lane);
    const char *qbase = reinterpret_cast<const char *>(qkv + row0 * ld + (int64_t)n * kD);
    const char *dbase = reinterpret_cast<const char *>(dattn + row0 * h + (int64_t)n * kD);
    const int64_t q_stride = (int64_t)kTile * ld * 2, d_stride = (int64_t)kTile * h * 2;
    const uint32_t lds0 = lds_addr_of(smem);
    const float *del_b = delta + ((int64_t)bi * nh + n) * seq;
    const float *lse_b = del_b + (int64_t)nb * nh * seq;  // log-sum-exp times log2(e), written by the dQ kernel
    const uint32_t lane4 = lane * 4;
    const int it0 = 2 * kb, n_tiles = 2 * (seq / 128 - kb);  // query tiles it0 + j, n_tiles >= 2
    // every wave issues the same nine copies per tile, so that one count serves all waits: waves 0 and 2 bring the
    // log-sum-exp values, waves 1 and 3 the deltas (twice the same bytes to the same place)
    auto issue_tile = [&](int j) {
        const int it = it0 + j;
        const uint32_t dst = lds0 + (j & (kFStages - 1)) * kFStageBytes;
        cq.issue(qbase + it * q_stride, dst, wave);
        cd.issue(dbase + it * d_stride, dst + kTileBytes, wave);
        const uint32_t sdst = dst + 2 * kTileBytes + (wave & 1) * 256;
        const float *src = ((wave & 1) ? del_b : lse_b) + it * kTile;
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2" : : "s"(sdst), "v"(lane4), "s"(src) : "memory");
    };

    f32x16 acck[4], accv[4];
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            acck[t][e] = 0.0f;
            accv[t][e] = 0.0f;
        }

    // The key block's own K and V rows come through LDS as well (stages 2 and 3, free until tile 2 is asked for):
    // coalesced copies and 16 LDS reads per wave instead of 16 loads that touch 32 rows each.
    bf16x8 kf[8], vf[8];
    {
        const char *kblk = reinterpret_cast<const char *>(qkv + (row0 + 128 * kb) * ld + h + (int64_t)n * kD);
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            const uint32_t dst = lds0 + (2 + half) * kFStageBytes;
            cq.issue(kblk + half * q_stride, dst, wave);
            cq.issue(kblk + half * q_stride + h * 2, dst + kTileBytes, wave);
        }
        issue_tile(0);
        issue_tile(1);
        asm volatile("s_waitcnt vmcnt(18)" ::: "memory");  // the sixteen K/V copies; tiles 0 and 1 may be in flight
        __syncthreads();
        const unsigned char *kv = smem + (2 + (wave >> 1)) * kFStageBytes;
#pragma unroll
        for (int s8 = 0; s8 < 8; ++s8) {
            kf[s8] = rd_row(kv, ad, wave & 1, s8);
            vf[s8] = rd_row(kv + kTileBytes, ad, wave & 1, s8);
        }
#pragma unroll
        for (int s8 = 0; s8 < 8; ++s8) {
            loaded_before_here(kf[s8]);
            loaded_before_here(vf[s8]);
        }
        __syncthreads();
        if (n_tiles > 2) {
            issue_tile(2);
            asm volatile("s_waitcnt vmcnt(18)" ::: "memory");  // tile 0 is there; tiles 1 and 2 may be in flight
        } else {
            asm volatile("s_waitcnt vmcnt(9)" ::: "memory");
        }
        __syncthreads();
    }

    f32x16 s0, p0, s1, p1;  // S and dP of the two half tiles in flight
    bf16x8 pf[2], dsf[2];
    {
        // S and dP of the first half tile, nothing to overlap with yet
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const bf16x8 qa = rd_row(smem, ad, 0, k), da = rd_row(smem + kTileBytes, ad, 0, k);
            if (k == 0) {
                mfma_v_first(s0, qa, kf[0]);
                mfma_v_first(p0, da, vf[0]);
            } else {
                mfma_v(s0, qa, kf[k]);
                mfma_v(p0, da, vf[k]);
            }
        }
        // these results are read sooner than a phase later (after the first barrier below): spell out the wait
        // states the compiler would put between a matrix instruction and a reader of its result
        asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
    }
    const int qlim0 = kvw0 + c - it0 * kTile - 4 * g;
    // one tile with the next tile's first half product inside it (the loop bodies), or without (the last tile)
    auto enter_tile = [&](int j) {
        // tile j + 1 has to be in LDS for this iteration; the copies of tile j + 2 (nine per wave) may still be in
        // flight; tile j + 3 goes into the stage of tile j - 1, which every wave has left once it is past the barrier
        if (j + 2 < n_tiles)
            asm volatile("s_waitcnt vmcnt(9)" ::: "memory");
        else
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (j + 3 < n_tiles) issue_tile(j + 3);
    };
    auto tile = [&](int j, auto mask, auto last) {
        constexpr bool MASK = decltype(mask)::value, LAST = decltype(last)::value;
        const unsigned char *tj = smem + (j & (kFStages - 1)) * kFStageBytes;
        const unsigned char *tn = smem + ((j + 1) & (kFStages - 1)) * kFStageBytes;
        const float *stat = reinterpret_cast<const float *>(tj + 2 * kTileBytes);
        const int qlim = qlim0 - j * kTile;
        dkv_scores_and_elementwise<true, MASK, 1, 0>(s1, p1, s0, p0, pf, dsf, tj, ad, kf, vf, stat, scale_log2e, qlim, g);
        dkv_second_products<0>(pf, dsf, tj, ad, acck, accv);
        dkv_scores_and_elementwise<!LAST, MASK, 0, 1>(s0, p0, s1, p1, pf, dsf, tn, ad, kf, vf, stat, scale_log2e, qlim, g);
        dkv_second_products<1>(pf, dsf, tj, ad, acck, accv);
    };
    using T_ = std::true_type;
    using F_ = std::false_type;
    // the first two tiles of a key block touch the diagonal, the others need no mask
    const int n_masked = n_tiles - 1 < 2 ? n_tiles - 1 : 2;
    for (int j = 0; j < n_masked; ++j) {
        enter_tile(j);
        tile(j, T_{}, F_{});
    }
    for (int j = 2; j + 1 < n_tiles; ++j) {
        enter_tile(j);
        tile(j, F_{}, F_{});
    }
    enter_tile(n_tiles - 1);
    if (n_tiles == 2)
        tile(n_tiles - 1, T_{}, T_{});
    else
        tile(n_tiles - 1, F_{}, T_{});
    __syncthreads();  // every wave has left the stages
    bf16 *outk = dqkv + (row0 + kvw0) * ld + h + (int64_t)n * kD;
    store_rows_via_lds(acck, scale, smem + wave * 16384, outk, ld, lane);
    store_rows_via_lds(accv, 1.0f, smem + wave * 16384 + 8192, outk + h, ld, lane);
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
    const float scale_log2e = (1.0f / sqrtf((float)d)) * 1.44269504088896340736f;
    const unsigned blocks = (unsigned)(seq / 128 * nh * b);
    const int chunk = chunk_slots(seq / 128, nh * b);
    constexpr size_t lds = 4 * kTileBytes;  // two stages of (K tile, V tile)
    static bool done = false;
    if (hipError_t e = set_lds(attn_fwd_w4_kernel, lds, done)) return e;
    attn_fwd_w4_kernel<<<dim3(blocks), 256, lds, s>>>((const bf16 *)qkv, (bf16 *)attn, lse, (int)seq, (int)nh, (int)b, chunk,
                                                      scale_log2e);
    return hipGetLastError();
}

hipError_t launch_attn_bwd(int dt, const void *qkv, const void *attn, const void *dattn, const float *lse,
                           float *delta, void *dqkv, int64_t b, int64_t seq, int64_t nh, int64_t d, hipStream_t s)
{
    if (dt != DT_BF16 || !attn_mfma_supported(seq, d)) return hipErrorInvalidValue;
    if (b * seq == 0) return hipSuccess;
    const float scale = 1.0f / sqrtf((float)d);
    const float scale_log2e = scale * 1.44269504088896340736f;
    constexpr size_t lds_dq = 4 * kTileBytes;            // two stages of (K tile, V tile)
    constexpr size_t lds_dkv = kFStages * kFStageBytes;  // four stages of (Q tile, dO tile, statistics)
    static bool a1 = false, a2 = false;
    if (hipError_t e = set_lds(attn_bwd_dq_w4_kernel, lds_dq, a1)) return e;
    if (hipError_t e = set_lds(attn_bwd_dkv_kernel, lds_dkv, a2)) return e;
    const unsigned blocks = (unsigned)(seq / 128 * nh * b);
    const int chunk = chunk_slots(seq / 128, nh * b);
    attn_bwd_dq_w4_kernel<<<dim3(blocks), 256, lds_dq, s>>>((const bf16 *)qkv, (const bf16 *)attn, (const bf16 *)dattn, lse,
                                                            delta, (bf16 *)dqkv, (int)seq, (int)nh, (int)b, chunk, scale,
                                                            scale_log2e);
    attn_bwd_dkv_kernel<<<dim3(blocks), 256, lds_dkv, s>>>((const bf16 *)qkv, (const bf16 *)dattn, delta, (bf16 *)dqkv,
                                                           (int)seq, (int)nh, (int)b, chunk, scale, scale_log2e);
    return hipGetLastError();
}

}  // namespace zpp
