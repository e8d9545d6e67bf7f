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
// Two work-group shapes.  Four waves, each taking every tile of its 32 rows, two stages of one tile pair in
// LDS (64 KB), two work-groups per CU: the default (all backward launches, forward launches of more than two
// work-groups per CU).  Eight waves, the two waves of a SIMD (w and w+4) sharing a group of 32 queries and
// splitting its key tiles even / odd, merged at the end, one work-group per CU: forward launches of at most
// two work-groups per CU, where the shorter chain of intervals per work-group wins.
//
// Backward: two launches without atomics.  dQ: lane = query, loops over key tiles.  dK and dV: lane = key,
// loop over query tiles.  P is recomputed from the saved log-sum-exp; delta = rowsum(dO o O) is computed by
// the dQ kernel and handed to the dK kernel.
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
// last chunk's long work-groups too late).  bodies = 2 (the dK/dV launch): each pair appears twice in a row on
// its XCD, once per body, and `chunk` counts those.  chunk = 0: the whole grid is one chunk.  The last chunk
// may be shorter than the others.
__device__ __forceinline__ void decode_heavy_first(int id, int nblk, int nh, int nb, int chunk, int bodies, int &blk,
                                                   int &n, int &bi, int &body)
{
    const int nv = nh * nb * bodies;
    int k, v;
    if (chunk > 0) {
        const int per = nblk * chunk, ch = id / per, r = id - ch * per;
        const int cs = min(chunk, nv - ch * chunk);  // (pair, body) slots of this chunk
        const int x = r & 7, j = r >> 3, ppx = cs >> 3;
        k = j / ppx;
        const int pi = j - k * ppx;
        if (bodies == 2) {
            // the chunk's slots on an XCD alternate between the two bodies of a pair
            body = pi & 1;
            v = ch * (chunk >> 1) + (pi >> 1) * 8 + x;
        } else {
            body = 0;
            v = ch * chunk + pi * 8 + x;
        }
    } else {
        if ((nv & 7) == 0) {
            const int j = id >> 3, per = nv >> 3;
            k = j / per;
            v = (j % per) * 8 + (id & 7);
        } else {
            k = id / nv;
            v = id % nv;
        }
        const int np = nh * nb;
        body = v >= np ? 1 : 0;
        v -= body * np;
    }
    blk = nblk - 1 - k;
    n = v % nh;
    bi = v / nh;
}

// (pair, body) slots per chunk for a launch over nv (sample, head) pairs: about 1024 work-groups per chunk, a
// multiple of 16; 0 (one chunk) when there is no more than a chunk of them or they cannot be dealt evenly to the
// XCDs
static int chunk_slots(int64_t nblk, int64_t nv, int bodies)
{
    int64_t c = (1024 / nblk) / 16 * 16;
    if (c < 16) c = 16;
    return (nv % 8 == 0 && nv * bodies > c) ? (int)c : 0;
}

// LDS holds two pairs of streamed tiles: a pair is copied in while the other is worked on.
constexpr int kStages = 4;

// depth of the register rings that carry LDS operands to the matrix instructions of the backward kernels
// (what fits beside the accumulators at two waves per SIMD)
constexpr int kRingDq = 4, kRingDkv = 3;

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

// ------------------------------------------------------------------------------------ forward
// Eight waves on 128 consecutive queries: waves w and w+4 (the two waves of a SIMD) own the same group of
// 32 queries and split its key tiles between them, wave w the even tiles, wave w+4 the odd ones, each with
// its own running maximum, row sum and output accumulator; at the end the second wave hands its three
// through LDS to the first, which merges them (the usual rescale by 2^(m_i - m)).  Key tiles are streamed
// in pairs, one barrier per pair, so in every interval both waves of a SIMD have a tile to work on and
// the SIMD interleaves the matrix phase of one with the softmax phase of the other; with one wave per
// query group the early (short) group of a SIMD leaves the late one running alone for most of the kernel.
// Work-groups are as heavy as their position in the sequence; the heavy ones are dispatched first.
__global__ __launch_bounds__(512, 2) void attn_fwd_split_kernel(const bf16 *__restrict__ qkv, bf16 *__restrict__ attn,
                                                                float *__restrict__ lse, int seq, int nh, int nb,
                                                                int chunk, float scale_log2e)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];  // [2 pairs][2 tiles][K tile | V tile]
    int qb, n, bi, body;
    decode_heavy_first(blockIdx.x, seq / 128, nh, nb, chunk, 1, qb, n, bi, body);
    const int64_t h = (int64_t)nh * kD, ld = 3 * h;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int half = wave >> 2, grp = wave & 3;
    const int g = lane >> 5, c = lane & 31;
    const int qw0 = 128 * qb + 32 * grp;
    const int64_t row0 = (int64_t)bi * seq;

    bf16x8 qf[8];
    {
        const bf16 *qp = qkv + (row0 + qw0 + c) * ld + (int64_t)n * kD + 8 * g;
#pragma unroll
        for (int st = 0; st < 8; ++st) qf[st] = *reinterpret_cast<const bf16x8 *>(qp + 16 * st);
    }
    TileCopy<8> cp;
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

    const int n_pairs = qb + 1;            // key tiles 2p, 2p+1 cover keys [128p, 128p + 128)
    const int my_tiles = qw0 / kTile + 1;  // tiles with unmasked entries for this wave's queries
    auto issue_pair = [&](int p) {
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const uint32_t dst = lds0 + ((p & 1) * 2 + t) * 2 * kTileBytes;
            cp.issue(kbase + (2 * p + t) * tile_stride, dst, wave);
            cp.issue(vbase + (2 * p + t) * tile_stride, dst + kTileBytes, wave);
        }
    };
    issue_pair(0);
#pragma unroll
    for (int st = 0; st < 8; ++st) loaded_before_here(qf[st]);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();

    for (int p = 0; p < n_pairs; ++p) {
        if (p + 1 < n_pairs) issue_pair(p + 1);  // into the buffer read in the previous interval
        const int jt = 2 * p + half;
        if (jt < my_tiles) {
            const int kv0 = jt * kTile;
            const unsigned char *ks = smem + ((p & 1) * 2 + half) * 2 * kTileBytes;
            const unsigned char *vs = ks + kTileBytes;
            f32x16 sacc[2] = {};
            // The 16 K operands come from LDS through a ring of four registers, each requested four MFMAs ahead
            // of its use and the order pinned (left to itself the compiler reads every operand into the same
            // register right before its MFMA and the matrix pipe waits out a whole LDS round trip each time).
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
            // the first V operands travel while the softmax is computed
            bf16x8 vr[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) vr[i] = rd_tr(vs, ad, i & 3, i >> 2);
            __builtin_amdgcn_sched_barrier(0);
            // sacc[T][e] of this lane: key kv0 + 32T + 8(e/4) + 4g + e%4, query qw0 + c; mask on the diagonal only
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
            for (int i = 0; i < 16; ++i) {  // i = 4 * st + t
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

    // merge the two halves of every query group: [64 accumulator values | m | l] x 64 lanes per group
    float *mg = reinterpret_cast<float *>(smem) + grp * (66 * 64);
    if (half == 1) {
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int e = 0; e < 16; ++e) mg[(t * 16 + e) * 64 + lane] = oacc[t][e];
        mg[64 * 64 + lane] = m_run;
        mg[65 * 64 + lane] = l_run;
    }
    __syncthreads();
    if (half == 1) return;
    {
        const float m_b = mg[64 * 64 + lane], l_b = mg[65 * 64 + lane];
        const float m = fmaxf(m_run, m_b);  // this wave always had tile 0, so m is finite
        const float a_a = fast_exp2((m_run - m) * scale_log2e), a_b = fast_exp2((m_b - m) * scale_log2e);
        l_run = l_run * a_a + l_b * a_b;
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int e = 0; e < 16; ++e) oacc[t][e] = oacc[t][e] * a_a + mg[(t * 16 + e) * 64 + lane] * a_b;
        m_run = m;
    }
    const float l_tot = sum_with_lane32(l_run);
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
        lse[((int64_t)bi * nh + n) * seq + qw0 + c] =
            (m_run * scale_log2e + __builtin_amdgcn_logf(l_tot)) * 0.69314718055994530942f;
}

// The same with four waves per work-group: every wave takes all key tiles of its 32 queries (no split, no merge),
// tiles streamed one by one through two stages of 32 KB, so two work-groups fit a CU and run out of step with
// each other.  Used when the grid has more than two work-groups per CU.
__global__ __launch_bounds__(256, 2) void attn_fwd_w4_kernel(const bf16 *__restrict__ qkv, bf16 *__restrict__ attn,
                                                             float *__restrict__ lse, int seq, int nh, int nb,
                                                             int chunk, float scale_log2e)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];  // [2 stages][K tile | V tile]
    int qb, n, bi, body;
    decode_heavy_first(blockIdx.x, seq / 128, nh, nb, chunk, 1, qb, n, bi, body);
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
    int qb, n, bi, body;
    decode_heavy_first(blockIdx.x, seq / 128, nh, nb, chunk, 1, qb, n, bi, body);
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
// Lane = key.  Per query tile: S = Q K^T (operands Q row-wise from LDS, K in registers),
// P = exp2(S*c - lse[q]).  Two instantiations, so that each fits two waves per SIMD:
//   DK = false: dV^T += dO^T P, with dO^T gathered from the dO tile through the transposing load;
//   DK = true:  dP = dO V^T (V in registers), dS = P o (dP - delta[q]), dK^T += Q^T dS.
// Recomputing S in both costs 16 of 80 MFMAs per tile and buys twice the occupancy (fused they need
// 434 VGPRs).  The per-query log-sum-exp and delta travel through LDS with the tiles (as ordinary loads
// inside the loop their in-order completion made every use wait behind the next tile's copies).
// Early key blocks see the most queries and are dispatched first; the dK and dV work-groups of a key
// block follow each other.
// Four waves per work-group on 128 consecutive keys: every wave all query tiles of its 32 keys (from the
// diagonal to the end of the sequence), streamed one by one through two stages, two work-groups per CU.
template <bool DK>
__device__ __forceinline__ void attn_bwd_dkv_w4_body(const bf16 *__restrict__ qkv, const bf16 *__restrict__ dattn,
                                                     const float *__restrict__ delta, bf16 *__restrict__ dqkv, int seq,
                                                     int nh, int nb, float scale, float scale_log2e, int kb, int n, int bi)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];  // [2][Q tile | dO tile], [2][lse | delta]
    const int64_t h = (int64_t)nh * kD, ld = 3 * h;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 5, c = lane & 31;
    const int kvw0 = 128 * kb + 32 * wave;
    const int64_t row0 = (int64_t)bi * seq;

    bf16x8 kf[8], vf[DK ? 8 : 1];
    {
        const bf16 *kp = qkv + (row0 + kvw0 + c) * ld + h + (int64_t)n * kD + 8 * g;
#pragma unroll
        for (int st = 0; st < 8; ++st) {
            kf[st] = *reinterpret_cast<const bf16x8 *>(kp + 16 * st);
            if constexpr (DK) vf[st] = *reinterpret_cast<const bf16x8 *>(kp + h + 16 * st);
        }
    }
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
    const uint32_t stat0 = lds0 + 2 * 2 * kTileBytes;
    const uint32_t lane4 = lane * 4;
    const int it0 = 2 * kb, n_tiles = 2 * (seq / 128 - kb);  // query tiles it0 + j
    auto issue_tile = [&](int j) {
        const int it = it0 + j, buf = j & 1;
        cq.issue(qbase + it * q_stride, lds0 + buf * 2 * kTileBytes, wave);
        cd.issue(dbase + it * d_stride, lds0 + buf * 2 * kTileBytes + kTileBytes, wave);
        if (wave == 0) {
            const uint32_t dst = stat0 + buf * 512;
            const float *src = lse_b + it * kTile;
            asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2" : : "s"(dst), "v"(lane4), "s"(src) : "memory");
        } else if (wave == 1 && DK) {
            const uint32_t dst = stat0 + buf * 512 + 256;
            const float *src = del_b + it * kTile;
            asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2" : : "s"(dst), "v"(lane4), "s"(src) : "memory");
        }
    };

    f32x16 acc[4];
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[t][e] = 0.0f;

    issue_tile(0);
#pragma unroll
    for (int st = 0; st < 8; ++st) {
        loaded_before_here(kf[st]);
        if constexpr (DK) loaded_before_here(vf[st]);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();

    for (int j = 0; j < n_tiles; ++j) {
        if (j + 1 < n_tiles) issue_tile(j + 1);
        const int buf = j & 1;
        const int qt0 = (it0 + j) * kTile;
        if (qt0 + kTile - 1 >= kvw0) {
            const unsigned char *qs = smem + buf * 2 * kTileBytes;
            const unsigned char *ds = qs + kTileBytes;
            const float *lse_s = reinterpret_cast<const float *>(smem + 2 * 2 * kTileBytes + buf * 512);
            const float *del_s = lse_s + 64;
            const bool diag = qt0 < kvw0 + 31;
            const unsigned char *src = DK ? qs : ds;
            // half a tile (32 queries) at a time, LDS operands through rings of registers, as in the dQ kernel
#pragma unroll
            for (int T = 0; T < 2; ++T) {
                f32x16 sacc, dpacc;
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    sacc[e] = 0.0f;
                    dpacc[e] = 0.0f;
                }
                bf16x8 qr[kRingDkv], dr[DK ? kRingDkv : 1];
#pragma unroll
                for (int i = 0; i < kRingDkv; ++i) {
                    qr[i] = rd_row(qs, ad, T, i);
                    if constexpr (DK) dr[i] = rd_row(ds, ad, T, i);
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int st = 0; st < 8; ++st) {
                    sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qr[st % kRingDkv], kf[st], sacc, 0, 0, 0);
                    __builtin_amdgcn_sched_barrier(0);
                    if (st + kRingDkv < 8) {
                        qr[st % kRingDkv] = rd_row(qs, ad, T, st + kRingDkv);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                    if constexpr (DK) {
                        dpacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dr[st % kRingDkv], vf[st], dpacc, 0, 0, 0);
                        __builtin_amdgcn_sched_barrier(0);
                        if (st + kRingDkv < 8) {
                            dr[st % kRingDkv] = rd_row(ds, ad, T, st + kRingDkv);
                            __builtin_amdgcn_sched_barrier(0);
                        }
                    }
                }
                // the first operands of the second product and the per-query statistics travel during the
                // element-wise part
                bf16x8 tr[kRingDkv];
#pragma unroll
                for (int i = 0; i < kRingDkv; ++i) tr[i] = rd_tr(src, ad, i & 3, 2 * T + (i >> 2));
                f32x4 l4[4], d4[DK ? 4 : 1];
#pragma unroll
                for (int e4 = 0; e4 < 4; ++e4) {
                    const int qrel = 32 * T + 8 * e4 + 4 * g;
                    l4[e4] = *reinterpret_cast<const f32x4 *>(lse_s + qrel);
                    if constexpr (DK) d4[e4] = *reinterpret_cast<const f32x4 *>(del_s + qrel);
                }
                __builtin_amdgcn_sched_barrier(0);
                if (diag) {
#pragma unroll
                    for (int e = 0; e < 16; ++e)
                        if (kvw0 + c > qt0 + 32 * T + 8 * (e >> 2) + 4 * g + (e & 3)) sacc[e] = -INFINITY;
                }
                bf16x8 frag[2];
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const float pe = fast_exp2(__builtin_fmaf(sacc[e], scale_log2e, -l4[e >> 2][e & 3]));
                    if constexpr (DK)
                        frag[e >> 3][e & 7] = (bf16)(pe * (dpacc[e] - d4[e >> 2][e & 3]));
                    else
                        frag[e >> 3][e & 7] = (bf16)pe;
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int i = 0; i < 8; ++i) {  // i = 4 * (step of 16 queries) + t
                    acc[i & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tr[i % kRingDkv], frag[i >> 2], acc[i & 3], 0, 0, 0);
                    __builtin_amdgcn_sched_barrier(0);
                    if (i + kRingDkv < 8) {
                        tr[i % kRingDkv] = rd_tr(src, ad, (i + kRingDkv) & 3, 2 * T + ((i + kRingDkv) >> 2));
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
            }
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
    }
    bf16 *out = dqkv + (row0 + kvw0 + c) * ld + (DK ? h : 2 * h) + (int64_t)n * kD;
    const float oscale = DK ? scale : 1.0f;
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int e4 = 0; e4 < 4; ++e4) {
            bf16x4 o;
#pragma unroll
            for (int r = 0; r < 4; ++r) o[r] = (bf16)(acc[t][e4 * 4 + r] * oscale);
            *reinterpret_cast<bf16x4 *>(out + 32 * t + 8 * e4 + 4 * g) = o;
        }
}

__global__ __launch_bounds__(256, 2) void attn_bwd_dkv_w4_kernel(const bf16 *__restrict__ qkv, const bf16 *__restrict__ dattn,
                                                                 const float *__restrict__ lse, const float *__restrict__ delta,
                                                                 bf16 *__restrict__ dqkv, int seq, int nh, int nb, int chunk,
                                                                 float scale, float scale_log2e)
{
    int blk, n, bi, body;
    decode_heavy_first(blockIdx.x, seq / 128, nh, nb, chunk, 2, blk, n, bi, body);
    const int kb = seq / 128 - 1 - blk;
    if (body == 0)
        attn_bwd_dkv_w4_body<true>(qkv, dattn, delta, dqkv, seq, nh, nb, scale, scale_log2e, kb, n, bi);
    else
        attn_bwd_dkv_w4_body<false>(qkv, dattn, delta, dqkv, seq, nh, nb, scale, scale_log2e, kb, n, bi);
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
    const int chunk = chunk_slots(seq / 128, nh * b, 1);
    // Up to two work-groups per CU's worth of work: the eight-wave kernel (a work-group's chain of intervals is
    // half as long); beyond: the four-wave kernel, two work-groups per CU, where one's prologue and epilogue
    // hide behind the other's tiles (measured at 32 heads x 2048: 54.0 against 57.0 us for 512 work-groups,
    // 106.8 against 95.2 us for 1024).
    if (blocks >= 768) {
        constexpr size_t lds = 4 * kTileBytes;  // two stages of (K tile, V tile)
        static bool done = false;
        if (hipError_t e = set_lds(attn_fwd_w4_kernel, lds, done)) return e;
        attn_fwd_w4_kernel<<<dim3(blocks), 256, lds, s>>>((const bf16 *)qkv, (bf16 *)attn, lse, (int)seq, (int)nh, (int)b,
                                                          chunk, scale_log2e);
    } else {
        constexpr size_t lds = kStages * 2 * kTileBytes;  // two pairs of (K tile, V tile)
        static bool done = false;
        if (hipError_t e = set_lds(attn_fwd_split_kernel, lds, done)) return e;
        attn_fwd_split_kernel<<<dim3(blocks), 512, lds, s>>>((const bf16 *)qkv, (bf16 *)attn, lse, (int)seq, (int)nh,
                                                             (int)b, 0, scale_log2e);
    }
    return hipGetLastError();
}

hipError_t launch_attn_bwd(int dt, const void *qkv, const void *attn, const void *dattn, const float *lse,
                           float *delta, void *dqkv, int64_t b, int64_t seq, int64_t nh, int64_t d, hipStream_t s)
{
    if (dt != DT_BF16 || !attn_mfma_supported(seq, d)) return hipErrorInvalidValue;
    if (b * seq == 0) return hipSuccess;
    const float scale = 1.0f / sqrtf((float)d);
    const float scale_log2e = scale * 1.44269504088896340736f;
    constexpr size_t lds_dq = 4 * kTileBytes;             // two stages of (K tile, V tile)
    constexpr size_t lds_dkv = 4 * kTileBytes + 2 * 512;  // two stages of (Q tile, dO tile) + lse/delta
    static bool a1 = false, a2 = false;
    if (hipError_t e = set_lds(attn_bwd_dq_w4_kernel, lds_dq, a1)) return e;
    if (hipError_t e = set_lds(attn_bwd_dkv_w4_kernel, lds_dkv, a2)) return e;
    const unsigned blocks = (unsigned)(seq / 128 * nh * b);
    attn_bwd_dq_w4_kernel<<<dim3(blocks), 256, lds_dq, s>>>((const bf16 *)qkv, (const bf16 *)attn, (const bf16 *)dattn, lse,
                                                            delta, (bf16 *)dqkv, (int)seq, (int)nh, (int)b,
                                                            chunk_slots(seq / 128, nh * b, 1), scale, scale_log2e);
    attn_bwd_dkv_w4_kernel<<<dim3(2 * blocks), 256, lds_dkv, s>>>((const bf16 *)qkv, (const bf16 *)dattn, lse, delta,
                                                                  (bf16 *)dqkv, (int)seq, (int)nh, (int)b,
                                                                  chunk_slots(seq / 128, nh * b, 2), scale, scale_log2e);
    return hipGetLastError();
}

}  // namespace zpp
