// bf16 MFMA GEMM for gfx950, fp32 accumulation in v_mfma_f32_16x16x32_bf16, fused epilogues (bias, residual,
// GeLU, GeLU', fp32 or bf16 output, in-place accumulation of fp32 output).
//
// One kernel template serves the three products of a linear layer (Section 2.3): each operand is read either
// with K contiguous or K-major, as it is stored, so nothing is transposed in memory.  A work-group computes a
// BM x BN tile (256x256 with two LDS slots of K = 64, or 128x256 / 256x128 with a ring of three, or 128x128);
// operands are copied global -> LDS directly, the K loop is rotated across its one barrier per K-step, and the
// order of every MFMA, LDS read and copy is written out and pinned, with no vector address arithmetic in the
// loop.  Work-group ids are remapped so that each XCD (one L2 each, ids are dealt round-robin over 8 XCDs)
// owns a compact group of neighbouring tiles; the epilogue transposes accumulators through LDS so that every
// global access is 16 bytes per lane.
#include "device_utils.h"
#include "kernels.h"

#include <mutex>
#include <type_traits>
#include <utility>

namespace zpp {

constexpr int kBK = 64;

struct EpiBf16 {
    const bf16 *bias, *resid, *aux;
    bf16 *out2;
    int act, gelu_mode, out_f32;  // out_f32 2: C (fp32) <- C + accum_scale * result
    float accum_scale;
};

__device__ __forceinline__ int lds_off(int row, int chunk)
{
    // element offset of 16-byte chunk `chunk` (0..7) of tile row `row`
    const int sw = (row & 7) ^ ((row >> 3) & 1);
    return row * kBK + ((chunk ^ sw) << 3);
}


// Compile-time loop: f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>), so that register
// arrays are only ever indexed with constants.
template <int... Is, class F>
__device__ __forceinline__ void static_for_impl(std::integer_sequence<int, Is...>, F &&f)
{
    (f(std::integral_constant<int, Is>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void static_for(F &&f)
{
    static_for_impl(std::make_integer_sequence<int, N>{}, static_cast<F &&>(f));
}

// Element-wise tail of the epilogue for one output element.
__device__ __forceinline__ void epi_store_one(float v, int64_t o_idx, void *__restrict__ Cv, const EpiBf16 &epi)
{
    if (epi.resid) v += (float)epi.resid[o_idx];
    if (epi.act == ACT_DGELU_MUL) v *= (float)(bf16)gelu_bwd((float)epi.aux[o_idx], epi.gelu_mode);
    if (epi.act == ACT_MUL_AUX) v *= (float)epi.aux[o_idx];
    if (epi.out_f32) {
        float *c = reinterpret_cast<float *>(Cv) + o_idx;
        *c = epi.out_f32 == 2 ? grad_accum(*c, epi.accum_scale, v) : v;
    } else {
        const bf16 o = (bf16)v;
        // the activation (and its derivative) is applied to the rounded pre-activation, the value that is stored
        // and re-read where it is kept
        if (epi.act == ACT_GELU_GRAD_DUAL) {
            float val, der;
            gelu_both((float)o, epi.gelu_mode, val, der);
            reinterpret_cast<bf16 *>(Cv)[o_idx] = (bf16)der;
            epi.out2[o_idx] = (bf16)val;
        } else {
            reinterpret_cast<bf16 *>(Cv)[o_idx] = o;
            if (epi.act == ACT_GELU_DUAL) epi.out2[o_idx] = (bf16)gelu_fwd((float)o, epi.gelu_mode);
        }
    }
}

// fp32 output without an element-wise tail (weight gradients): a lane owns 4 consecutive columns of a
// row, so that one store instruction of a wave writes whole rows of its 32-row slice (full 128-byte
// lines).  This is the lane geometry of that path, and the fetch of the old values of C when the product
// is accumulated in place (Section 3.1: G <- G + scale * dW).
template <int NT>
struct F32Rows {
    static constexpr int WN = NT * 32, CH4 = WN / 4, ROWS4 = 64 / CH4, PASSES4 = 32 / ROWS4;
    float *cf0;      // this lane's element of the wave tile's first pass
    int64_t pstep;   // elements between passes
    int64_t n4;      // first of the lane's 4 columns
    int rows_left;   // tile rows g*32 + p*ROWS4 below this are inside C
    int row4, c4;
    bool ok, accum, col_full, col_any;

    __device__ __forceinline__ void init(void *Cv, int64_t ldc, const EpiBf16 &epi, int64_t M, int64_t N,
                                         int64_t m_wave, int64_t n_wave, int lane)
    {
        ok = epi.out_f32 && (ldc % 8 == 0) && (reinterpret_cast<uintptr_t>(Cv) % 16 == 0) && !epi.resid &&
             epi.act == ACT_NONE;  // (the activation modes are for bf16 outputs)
        accum = ok && epi.out_f32 == 2;
        row4 = lane / CH4;
        c4 = lane % CH4;
        n4 = n_wave + c4 * 4;
        cf0 = reinterpret_cast<float *>(Cv) + (m_wave + row4) * ldc + n4;
        pstep = ROWS4 * ldc;
        const int64_t rl = M - m_wave - row4;
        rows_left = rl > 4096 ? 4096 : (int)rl;
        col_full = n4 + 4 <= N;
        col_any = n4 < N;
    }
    // old values of 32-row group G (zeros where the tile leaves C or the path is not taken)
    template <int G>
    __device__ __forceinline__ void fetch(f32x4 *dst) const
    {
#pragma unroll
        for (int p = 0; p < PASSES4; ++p) {
            dst[p] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
            if (accum && G * 32 + p * ROWS4 < rows_left && col_full)
                dst[p] = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(cf0 + (G * (32 / ROWS4) + p) * pstep));
        }
    }
};

// Epilogue shared by the GEMM kernels.  The accumulator layouts of the MFMAs give a lane one column and
// scattered rows, which would make every global store a 2-byte-per-lane scatter.  So each wave transposes
// its tile through its own slice of LDS, 32 rows at a time (fp32, bias already added; `put(i, stage)` deposits
// rows [32 i, 32 i + 32) of the wave tile, row stride epi_stride), and then every lane owns 8 consecutive
// columns of a row: residual / GeLU inputs are read and results written with 16-byte accesses, a full
// 128-byte line per 8 lanes.
// Must be entered after a work-group barrier that ends all use of the operand tiles in LDS.
constexpr int epi_stride(int NT) { return NT * 32 + 8; }  // floats; 4 rows apart = half the banks apart

template <int MT, int NT, class Put>
__device__ __forceinline__ void epilogue_rows(Put put, unsigned char *smem_raw, int n_waves, int wave, int lane,
                                              void *__restrict__ Cv, int64_t ldc, const EpiBf16 &epi, int64_t M,
                                              int64_t N, int64_t m_wave, int64_t n_wave)
{
    constexpr int WN = NT * 32;
    constexpr int STRIDE = epi_stride(NT);
    constexpr int CH = WN / 8;              // 8-column chunks per row
    constexpr int ROWS_PER_PASS = 64 / CH;  // rows covered by the 64 lanes at once
    constexpr int PASSES = 32 / ROWS_PER_PASS;
    float *stage = reinterpret_cast<float *>(smem_raw) + wave * (32 * STRIDE);
    const bool vec_ok = (ldc % 8 == 0) && (reinterpret_cast<uintptr_t>(Cv) % 16 == 0) &&
                        (!epi.resid || reinterpret_cast<uintptr_t>(epi.resid) % 16 == 0) &&
                        (!epi.aux || reinterpret_cast<uintptr_t>(epi.aux) % 16 == 0) &&
                        (!epi.out2 || reinterpret_cast<uintptr_t>(epi.out2) % 16 == 0);
    // The bf16 side input of the element-wise tail (the residual, or the pre-activation of the GeLU derivative)
    // is fetched one 32-row group ahead with direct-to-LDS copies, pass p of a group by the p-th copy, so that each
    // lane later reads back from LDS exactly the 16 bytes it asked for: the loop over the passes stays a loop (no
    // registers indexed by it), and the memory latency is met once per tile instead of once per pass (sixteen
    // times per wave tile, the bulk of what these epilogues cost before).  Two 32-row buffers per wave after the
    // staging slices.
    const bool mul_side = epi.act == ACT_DGELU_MUL || epi.act == ACT_MUL_AUX;
    const bf16 *side = mul_side ? epi.aux : epi.resid;
    const bool side_dma = side && vec_ok && !epi.out_f32 && !(mul_side && epi.resid) &&
                          m_wave + MT * 32 <= M && n_wave + WN <= N && 32 * ldc * 2 < ((int64_t)1 << 31);
    unsigned char *side_buf = smem_raw + n_waves * (32 * STRIDE * 4) + wave * (2 * 32 * WN * 2);
    const uint32_t side_lds = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)side_buf;
    const uint32_t side_voff = (uint32_t)(((lane / CH) * ldc + (lane % CH) * 8) * 2);
    const char *side_base = reinterpret_cast<const char *>(side + m_wave * ldc + n_wave);
    auto side_issue = [&](int grp) {
#pragma unroll
        for (int p = 0; p < PASSES; ++p) {
            const uint32_t dst = side_lds + (grp & 1) * (32 * WN * 2) + p * 1024;
            const char *src = side_base + (int64_t)(grp * 32 + p * ROWS_PER_PASS) * ldc * 2;
            asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                         :
                         : "s"(dst), "v"(side_voff), "s"(src)
                         : "memory");
        }
    };
    if (side_dma) side_issue(0);
    F32Rows<NT> fr;
    fr.init(Cv, ldc, epi, M, N, m_wave, n_wave, lane);
    constexpr int ROWS4 = F32Rows<NT>::ROWS4, PASSES4 = F32Rows<NT>::PASSES4;
    const bool f32_rows = fr.ok, accum = fr.accum;
    const int row4 = fr.row4, c4 = fr.c4;
    // Accumulating in place: the old values of a 32-row group are fetched one group ahead, so their
    // latency hides behind the previous group's transposition and stores.
    f32x4 old[2][PASSES4];
    fr.template fetch<0>(old[0]);
    // The loop over the passes is a real loop: unrolled, the element-wise tail (with its GeLU branches)
    // would be replicated MT * PASSES times and the epilogue would run at the speed of instruction
    // fetch.  The 32-row groups stay instantiated one by one, since accumulator registers can only be
    // indexed with constants.
    static_for<MT>([&](auto ii) {
        constexpr int i = decltype(ii)::value;
        if constexpr (i + 1 < MT)
            if (accum) fr.template fetch<i + 1>(old[(i + 1) & 1]);
        put(ii, stage);
        // the slice is private to this wave; LDS operations of a wave complete in order
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        if (side_dma) {
            // this group's side input has landed (and the stores of the group before are out); the next group's
            // goes into the other buffer while this one is worked on
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            if constexpr (i + 1 < MT) side_issue(i + 1);
        }
        if (accum) {
#pragma unroll
            for (int p = 0; p < PASSES4; ++p) {
                const int row = p * ROWS4 + row4;
                const f32x4 val = *reinterpret_cast<const f32x4 *>(stage + row * STRIDE + c4 * 4);
                if (i * 32 + p * ROWS4 >= fr.rows_left || !fr.col_any) continue;
                float *cf = fr.cf0 + (i * (32 / ROWS4) + p) * fr.pstep;
                if (fr.col_full) {
                    f32x4 g = old[i & 1][p];
#pragma unroll
                    for (int k = 0; k < 4; ++k) g[k] = grad_accum(g[k], epi.accum_scale, val[k]);
                    __builtin_nontemporal_store(g, reinterpret_cast<f32x4 *>(cf));
                } else {
                    for (int k = 0; k < 4 && fr.n4 + k < N; ++k)
                        cf[k] = grad_accum(cf[k], epi.accum_scale, stage[row * STRIDE + c4 * 4 + k]);
                }
            }
        } else if (f32_rows) {
#pragma unroll 1
            for (int p = 0; p < PASSES4; ++p) {
                const int row = p * ROWS4 + row4;
                const f32x4 val = *reinterpret_cast<const f32x4 *>(stage + row * STRIDE + c4 * 4);
                if (i * 32 + p * ROWS4 >= fr.rows_left || !fr.col_any) continue;
                float *cf = fr.cf0 + (i * (32 / ROWS4) + p) * fr.pstep;
                if (fr.col_full) {
                    // next read by the accumulate pass, long after: streamed past the caches
                    __builtin_nontemporal_store(val, reinterpret_cast<f32x4 *>(cf));
                } else {
                    for (int k = 0; k < 4 && fr.n4 + k < N; ++k) cf[k] = stage[row * STRIDE + c4 * 4 + k];
                }
            }
        } else
#pragma unroll 1
        for (int p = 0; p < PASSES; ++p) {
            const int row = p * ROWS_PER_PASS + lane / CH;
            const int c8 = lane % CH;
            const int64_t m = m_wave + i * 32 + row;
            const int64_t n = n_wave + c8 * 8;
            const f32x4 lo = *reinterpret_cast<const f32x4 *>(stage + row * STRIDE + c8 * 8);
            const f32x4 hi = *reinterpret_cast<const f32x4 *>(stage + row * STRIDE + c8 * 8 + 4);
            float v[8] = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
            if (m >= M || n >= N) continue;
            const int64_t o_idx = m * ldc + n;
            if (vec_ok && n + 8 <= N) {
                bf16x8 sv;
                if (side_dma) sv = *reinterpret_cast<const bf16x8 *>(side_buf + (i & 1) * (32 * WN * 2) + p * 1024 + lane * 16);
                if (epi.resid) {
                    const bf16x8 r = (side_dma && !mul_side) ? sv : *reinterpret_cast<const bf16x8 *>(epi.resid + o_idx);
#pragma unroll
                    for (int k = 0; k < 8; ++k) v[k] += (float)r[k];
                }
                if (mul_side) {
                    const bf16x8 u = side_dma ? sv : *reinterpret_cast<const bf16x8 *>(epi.aux + o_idx);
                    if (epi.act == ACT_MUL_AUX) {
#pragma unroll
                        for (int k = 0; k < 8; ++k) v[k] *= (float)u[k];
                    } else {
#pragma unroll
                        for (int k = 0; k < 8; ++k) v[k] *= (float)(bf16)gelu_bwd((float)u[k], epi.gelu_mode);
                    }
                }
                if (epi.out_f32) {
                    float *cf = reinterpret_cast<float *>(Cv) + o_idx;
                    *reinterpret_cast<f32x4 *>(cf) = f32x4{v[0], v[1], v[2], v[3]};
                    *reinterpret_cast<f32x4 *>(cf + 4) = f32x4{v[4], v[5], v[6], v[7]};
                } else {
                    bf16x8 o;
#pragma unroll
                    for (int k = 0; k < 8; ++k) o[k] = (bf16)v[k];
                    if (epi.act == ACT_GELU_GRAD_DUAL) {
                        bf16x8 g, d;
#pragma unroll
                        for (int k = 0; k < 8; ++k) {
                            float val, der;
                            gelu_both((float)o[k], epi.gelu_mode, val, der);
                            g[k] = (bf16)val;
                            d[k] = (bf16)der;
                        }
                        *reinterpret_cast<bf16x8 *>(reinterpret_cast<bf16 *>(Cv) + o_idx) = d;
                        *reinterpret_cast<bf16x8 *>(epi.out2 + o_idx) = g;
                    } else {
                        *reinterpret_cast<bf16x8 *>(reinterpret_cast<bf16 *>(Cv) + o_idx) = o;
                        if (epi.act == ACT_GELU_DUAL) {
                            bf16x8 g;
#pragma unroll
                            for (int k = 0; k < 8; ++k) g[k] = (bf16)gelu_fwd((float)o[k], epi.gelu_mode);
                            *reinterpret_cast<bf16x8 *>(epi.out2 + o_idx) = g;
                        }
                    }
                }
            } else {
                // ragged or unaligned edge: element by element (stage is re-read so that v[] is never
                // indexed with a loop variable)
#pragma unroll 1
                for (int k = 0; k < 8; ++k)
                    if (n + k < N) epi_store_one(stage[row * STRIDE + c8 * 8 + k], o_idx + k, Cv, epi);
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    });
}

// v_mfma_f32_16x16x32_bf16 accumulators: acc[i][j][e] of lane l is
// C[m_wave + i*16 + (l/16)*4 + e, n_wave + j*16 + l%16].
template <int MA, int NB>
__device__ __forceinline__ void epilogue16(f32x4 (&acc)[MA][NB], unsigned char *smem_raw, int n_waves, int wave, int lane,
                                           void *__restrict__ Cv, int64_t ldc, const EpiBf16 &epi, int64_t M,
                                           int64_t N, int64_t m_wave, int64_t n_wave)
{
    static_assert(MA % 2 == 0 && NB % 2 == 0, "whole 32x32 groups");
    constexpr int STRIDE = epi_stride(NB / 2);
    const int q16 = lane >> 4, c16 = lane & 15;
    float bias[NB];
#pragma unroll
    for (int j = 0; j < NB; ++j) {
        const int64_t n = n_wave + j * 16 + c16;
        bias[j] = (epi.bias && n < N) ? (float)epi.bias[n] : 0.0f;
    }
    epilogue_rows<MA / 2, NB / 2>(
        [&](auto ii, float *stage) {
            constexpr int i = decltype(ii)::value;
            static_for<2>([&](auto hh) {
                constexpr int h = decltype(hh)::value;
                static_for<NB>([&](auto jj) {
                    constexpr int j = decltype(jj)::value;
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        stage[(h * 16 + q16 * 4 + e) * STRIDE + j * 16 + c16] = acc[2 * i + h][j][e] + bias[j];
                });
            });
        },
        smem_raw, n_waves, wave, lane, Cv, ldc, epi, M, N, m_wave, n_wave);
}

// Which tile a work-group computes.  Work-group ids are dealt round-robin over the 8 XCDs (one L2 each):
// ids are first regrouped so that an XCD gets a contiguous run of tile numbers, and tile numbers walk the grid
// in bands of 8 tile rows, down a column of the band first, so that the tiles in flight on an XCD share their
// A rows and B columns in its L2.
__device__ __forceinline__ void tile_of_workgroup(int pid, int tiles_m, int tiles_n, int &tm, int &tn)
{
    const int total = tiles_m * tiles_n;
    if ((total & 7) == 0) pid = (pid & 7) * (total >> 3) + (pid >> 3);
    constexpr int GROUP_M = 8;
    const int per_group = GROUP_M * tiles_n;
    const int group = pid / per_group;
    const int first_m = group * GROUP_M;
    const int gsz = (tiles_m - first_m < GROUP_M) ? tiles_m - first_m : GROUP_M;
    tm = first_m + (pid % per_group) % gsz;
    tn = (pid % per_group) / gsz;
}

// ---------------------------------------------------------------------------------------------
// The kernel.  C[M,N] = sum_k A(m,k) B(n,k), each operand stored either with K contiguous ("row-major side": A
// [M, K], B [N, K]) or K-major (A [K, M], B [K, N]):
//   NT  (A row-major, B row-major)  forward  y = x . W^T
//   NN  (A row-major, B K-major)    input gradient  dX = dY . W  read from W[out, in] as stored
//   TN  (A K-major,  B K-major)     weight gradient dW = dY^T . X read from the token-major activations
// A ring of NS LDS slots of K = 64, operands global -> LDS directly, the K loop rotated across its one barrier
// per K-step.  The matrix instruction is v_mfma_f32_16x16x32_bf16: on this part the chip's power management
// sets the pace of a GEMM, and the 16x16x32 form delivers the same flops per cycle for less power than 32x32x16
// (a register-only loop runs at 2.0 against 1.75 GHz), which shows as a higher clock under the same kernel.
//   * A K-step is two sub-steps of 32 k.  A sub-step is MA groups; group G multiplies the 16-row block G of
//     the wave's A rows with the NB 16-column blocks of its B rows.  A blocks live in a ring of MA registers
//     and are read AHEAD = MA/2 groups before their group; the B blocks of the next sub-step (a second set of
//     registers) are read in groups AHEAD and AHEAD+1 together with its first A blocks.
//   * The LDS reads are written as asm and waited for by count (LDS reads return in order; at each group the
//     count of younger read instructions is a constant of the schedule; where it exceeds the 4-bit field the
//     wait covers a few blocks more).  Left to the compiler every wait is for all outstanding reads, which
//     exposes the full LDS latency twice per sub-step.
//   * Lane l of a 16x16x32 operand block holds row l%16 and eight consecutive k.  Which eight is free as long as
//     A and B agree; all sides use k-group (l/16 % 2) * 2 + l/32 (see the sides below for why).
//   * Copies: the copies of tile kt+NS are issued after the barrier of K-step kt, spread over the groups that
//     follow it, into the slot that barrier freed, so every copy has a whole K-step before it is waited for
//     (SPLIT: the second half of them in the first groups of the next K-step instead; better for the long-K
//     weight-gradient products, worse for the others); the wait before the barrier leaves (NS-2) K-steps of
//     copies in flight.
//   * The loop body is instantiated per slot, so all LDS addresses are a per-lane base register plus an
//     immediate, and the global addresses are a scalar base that advances per K-step plus a fixed per-lane
//     32-bit offset: no vector address arithmetic inside the loop.
template <int OFF>
__device__ __forceinline__ bf16x8 lds_read16(uint32_t addr)
{
    bf16x8 r;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(r) : "v"(addr), "n"(OFF));
    return r;
}

typedef __attribute__((ext_vector_type(4))) short s16x4_t;

template <int OFF>
__device__ __forceinline__ bf16x8 lds_read_tr8(uint32_t addr)
{
    // rows k .. k+3 at addr, rows k+4 .. k+7 four rows (2048 bytes) further
    s16x4_t lo, hi;
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(lo) : "v"(addr), "n"(OFF));
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(hi) : "v"(addr), "n"(OFF + 2048));
    return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
}

// k-group of lane l within a 32-k sub-step, the same on every side
__device__ __forceinline__ int k_group(int lane) { return ((lane >> 4) & 1) * 2 + (lane >> 5); }

// An operand stored with K contiguous ([rows, K]): ROWS rows of it per tile, NW waves copy them.  In LDS a
// slot is [ROWS][64 k] with 128-byte rows, the 16-byte chunk XORed with (row & 7) ^ (row >> 3 & 1) so that the
// row-wise 16-byte writes of a copy (8 rows x 128 bytes) and the 16-byte reads of an MFMA block (16 rows, one
// chunk per k-group) are free of bank conflicts.  A 16-byte LDS read serves lanes l and l+32 in the same pass:
// with k-group l/16 they would meet in the same banks (a two-way conflict on every read), with k_group() they
// take neighbouring chunks.  Rows past `limit` are clamped to the last valid row (their products are masked
// in the epilogue).
template <int ROWS, int NW>
struct RowMajorSide {
    static constexpr int COPIES = ROWS / 8 / NW;  // per wave per K-step, 8 rows each
    static constexpr int BUF = ROWS * kBK * 2;    // bytes per slot
    static constexpr int READ_INSTRS = 1;         // LDS instructions per operand block
    uint32_t voff[COPIES];
    const char *tile;    // first byte of the tile's first K-step
    int64_t kstep;       // bytes from one K-step to the next
    uint32_t ad[2][2];   // [offsets above 64 KB][sub-step]: LDS byte address of this lane's chunk in block 0, slot 0

    __device__ __forceinline__ void init(const bf16 *P, int64_t ld, int64_t origin, int64_t limit, int wave, int lane,
                                         int wave_row0, uint32_t lds_region)
    {
        const int lrow = lane >> 3, lch = lane & 7;
#pragma unroll
        for (int j = 0; j < COPIES; ++j) {
            const int row = (wave * COPIES + j) * 8 + lrow;
            const int sw = (row & 7) ^ ((row >> 3) & 1);
            int64_t r = row;
            if (origin + r > limit - 1) r = limit - 1 - origin;
            voff[j] = (uint32_t)((r * ld + ((lch ^ sw) << 3)) * 2);
        }
        tile = reinterpret_cast<const char *>(P + origin * ld);
        kstep = kBK * 2;
        const int row = wave_row0 + (lane & 15), kq = k_group(lane);
        const int sw = (row & 7) ^ ((row >> 3) & 1);
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            ad[0][s] = lds_region + row * 128 + (((s * 4 + kq) ^ sw) << 4);
            ad[1][s] = ad[0][s] + 65536;
        }
    }
    template <int BLK, int S, int SLOT>
    __device__ __forceinline__ bf16x8 read() const
    {
        constexpr int off = SLOT * BUF + BLK * 2048;
        return lds_read16<off % 65536>(ad[off / 65536][S]);
    }
};

// An operand stored K-major ([K, rows], rows contiguous), 256 rows of it per tile.  In LDS a slot is
// [64 k][256 rows] with 512-byte rows; a copy moves two k-rows (1 KB).  An MFMA block (one row, eight
// consecutive k per lane) is gathered down the k-rows with the transposing read ds_read_b64_tr_b16, two per
// block (four k each): within 16 lanes, lanes 4j+q point at k-row j, 8-byte piece q, and lane i receives
// element i%4 of the pieces of lanes i/4, 4+i/4, 8+i/4, 12+i/4, i.e. column i of four consecutive k-rows.
// The 16-byte chunk c of k-row k sits at chunk position c ^ (4 * (k % 4)) ^ (2 * (k / 16 % 2)): an 8-byte-per-lane
// access is served in two passes (lanes 0-31, lanes 32-63), a pass holds two k-groups (0 and 2, or 1 and 3) of
// four k-rows each, and the swizzle sends those eight 32-byte pieces to eight different bank groups.
template <int ROWS, int NW, int NBLK>
struct KMajorSide {
    static_assert(ROWS == 256, "512-byte k-rows");
    static constexpr int COPIES = kBK / 2 / NW;   // per wave per K-step, two k-rows each
    static constexpr int BUF = ROWS * kBK * 2;
    static constexpr int READ_INSTRS = 2;
    uint32_t voff[COPIES];
    const char *tile;
    int64_t kstep;
    uint32_t ad[2][NBLK];  // [offsets above 64 KB][block]: first transposing read of the block at sub-step 0, slot 0

    __device__ __forceinline__ void init(const bf16 *P, int64_t ld, int64_t origin, int64_t, int wave, int lane,
                                         int wave_row0, uint32_t lds_region)
    {
        // lane i of a copy writes bytes [16 i, 16 i + 16) of the 1 KB piece: k-row i/32, chunk position i%32
#pragma unroll
        for (int j = 0; j < COPIES; ++j) {
            const int row = 2 * (wave * COPIES + j) + (lane >> 5);
            const int chunk = (lane & 31) ^ (4 * (row & 3)) ^ (2 * ((row >> 4) & 1));
            voff[j] = (uint32_t)(((int64_t)row * ld + chunk * 8) * 2);
        }
        tile = reinterpret_cast<const char *>(P + origin);
        kstep = (int64_t)kBK * ld * 2;
        // k-row 8 kq + j of the sub-step, the 32-byte piece of 16-row block b at piece position b ^ (2 j) ^ (kq / 2)
        const int kq = k_group(lane), j = (lane & 15) >> 2, q = lane & 3;
        const int x = (2 * j) ^ (kq >> 1);
        const uint32_t rowoff = (uint32_t)((8 * kq + j) * 512 + 8 * q);
#pragma unroll
        for (int i = 0; i < NBLK; ++i) {
            ad[0][i] = lds_region + rowoff + 32 * ((wave_row0 / 16 + i) ^ x);
            ad[1][i] = ad[0][i] + 65536;
        }
    }
    template <int BLK, int S, int SLOT>
    __device__ __forceinline__ bf16x8 read() const
    {
        constexpr int off = SLOT * BUF + S * 16384;  // sub-step s is k-rows 32 s .. 32 s + 31
        return lds_read_tr8<off % 65536>(ad[off / 65536][BLK]);
    }
};

template <bool A_KMAJOR, bool B_KMAJOR, int BM, int BN, int WGM, int WGN, int NS, bool SPLIT>
__device__ __forceinline__ void gemm_bf16_tile(int64_t M, int64_t N, int64_t K, const bf16 *__restrict__ A, int64_t lda,
                                               const bf16 *__restrict__ B, int64_t ldb, void *__restrict__ Cv,
                                               int64_t ldc, const EpiBf16 &epi, int tiles_m, int tiles_n, int pid)
{
    constexpr int NW = WGM * WGN;
    constexpr int WM = BM / WGM, WN = BN / WGN;
    constexpr int MA = WM / 16, NB = WN / 16, NBH = NB / 2;
    constexpr int AHEAD = MA / 2;
    using ASide = typename std::conditional<A_KMAJOR, KMajorSide<BM, NW, MA>, RowMajorSide<BM, NW>>::type;
    using BSide = typename std::conditional<B_KMAJOR, KMajorSide<BN, NW, NB>, RowMajorSide<BN, NW>>::type;
    constexpr int A_I = ASide::COPIES, B_I = BSide::COPIES;
    constexpr int LPS = A_I + B_I;                       // global->LDS copies per wave per K-step
    constexpr int H1 = SPLIT ? LPS / 2 : LPS, H2 = LPS - H1;  // after the barrier / in the first groups of the next K-step
    constexpr int A_BUF = ASide::BUF, B_BUF = BSide::BUF;
    constexpr int B_REGION = NS * A_BUF;                 // byte offset of the B slots inside LDS
    constexpr int IA = ASide::READ_INSTRS, IB = BSide::READ_INSTRS;
    static_assert(A_I >= 1 && B_I >= 1 && MA >= 4 && MA % 2 == 0 && NB % 2 == 0, "tile/waves mismatch");
    static_assert((H1 + MA - AHEAD - 1) / (MA - AHEAD) <= NB && (H2 + AHEAD - 1) / AHEAD <= NB, "one copy per MFMA at most");
    static_assert(NS >= 2 && NS <= 3 && (NS - 2) * LPS < 64, "ring depth");
    static_assert(NS * A_BUF + MA * 2048 <= 2 * 65536 && NS * B_BUF + NB * 2048 <= 2 * 65536, "two base registers");

    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];

    int tm, tn;
    tile_of_workgroup(pid, tiles_m, tiles_n, tm, tn);
    const int64_t m0 = (int64_t)tm * BM, n0 = (int64_t)tn * BN;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WGN, wn = wave % WGN;

    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)smem_raw;
    ASide a;
    BSide b;
    a.init(A, lda, m0, M, wave, lane, wm * WM, lds_base);
    b.init(B, ldb, n0, N, wave, lane, wn * WN, lds_base + B_REGION);

    f32x4 acc[MA][NB];
#pragma unroll
    for (int i = 0; i < MA; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j) acc[i][j] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};

    const int nk = (int)(K / kBK);
    bf16x8 af[MA], bfr[2][NB];

    // copy n (0..LPS-1) of K-step kt into ring slot `slot`: scalar base (advances with the K-step) + fixed
    // per-lane 32-bit offset; M0 carries the LDS destination of the wave's 1 KB piece
    const uint32_t a_slot = lds_base + wave * A_I * 1024, b_slot = lds_base + B_REGION + wave * B_I * 1024;
    auto gll = [&](int n, int kt, int slot) {
        if (n < A_I) {
            const char *abase = a.tile + (int64_t)kt * a.kstep;
            const uint32_t dst = a_slot + slot * A_BUF + n * 1024;
            asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                         :
                         : "s"(dst), "v"(a.voff[n]), "s"(abase)
                         : "memory");
        } else {
            const int m = n - A_I;
            const char *bbase = b.tile + (int64_t)kt * b.kstep;
            const uint32_t dst = b_slot + slot * B_BUF + m * 1024;
            asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                         :
                         : "s"(dst), "v"(b.voff[m]), "s"(bbase)
                         : "memory");
        }
    };
    auto rd_a = [&](auto i_c, auto s_c, auto slot_c) {
        constexpr int i = decltype(i_c)::value;
        af[i] = a.template read<i, decltype(s_c)::value, decltype(slot_c)::value>();
    };
    auto rd_b = [&](auto j_c, auto s_c, auto slot_c) {
        constexpr int j = decltype(j_c)::value, s = decltype(s_c)::value;
        bfr[s][j] = b.template read<j, s, decltype(slot_c)::value>();
    };
    // One group: the NB MFMAs of A block G of sub-step S, preceded by the reads that keep the operands AHEAD
    // groups in front - A block G+AHEAD of this sub-step, or, in the second half of the sub-step, the first
    // A blocks and the B blocks of the next sub-step RS of slot RSLOT - and interleaved with copies
    // CP0 .. CP0+CPN-1 of K-step gkt into slot GSLOT.
    auto group = [&](auto s_c, auto g_c, auto slot_c, auto rs_c, auto rslot_c, auto cp0_c, auto cpn_c, auto gslot_c,
                     int gkt) {
        constexpr int S = decltype(s_c)::value, G = decltype(g_c)::value;
        constexpr int CP0 = decltype(cp0_c)::value, CPN = decltype(cpn_c)::value, GSLOT = decltype(gslot_c)::value;
        if constexpr (G < AHEAD) {
            rd_a(std::integral_constant<int, G + AHEAD>{}, s_c, slot_c);
        } else if constexpr (G == AHEAD) {
            rd_a(std::integral_constant<int, 0>{}, rs_c, rslot_c);
            __builtin_amdgcn_sched_barrier(0);
            static_for<NBH>([&](auto jj) {
                rd_b(jj, rs_c, rslot_c);
                __builtin_amdgcn_sched_barrier(0);
            });
        } else if constexpr (G == AHEAD + 1) {
            static_for<NBH>([&](auto jj) {
                rd_b(std::integral_constant<int, NBH + decltype(jj)::value>{}, rs_c, rslot_c);
                __builtin_amdgcn_sched_barrier(0);
            });
            rd_a(std::integral_constant<int, 1>{}, rs_c, rslot_c);
        } else {
            rd_a(std::integral_constant<int, G - AHEAD>{}, rs_c, rslot_c);
        }
        // LDS instructions younger than the last one this group needs (A block G; for G = 0 also the B blocks).
        // In issue order a sub-step reads A[AHEAD..MA-1] one per group, then {A'0, B'[0..NBH-1]},
        // {B'[NBH..NB-1], A'1}, A'2, ..., A'[AHEAD-1] of the next sub-step.
        constexpr int YOUNGER = AHEAD * IA + (G < AHEAD ? 0 : (G == AHEAD ? NBH * IB : NB * IB));
        asm volatile("s_waitcnt lgkmcnt(%0)" : : "n"(YOUNGER < 15 ? YOUNGER : 15));
        __builtin_amdgcn_sched_barrier(0);
        static_for<NB>([&](auto jj) {
            constexpr int j = decltype(jj)::value;
            acc[G][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[G], bfr[S][j], acc[G][j], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (j < CPN) {
                gll(CP0 + j, gkt, GSLOT);
                __builtin_amdgcn_sched_barrier(0);
            }
        });
    };
    using I0 = std::integral_constant<int, 0>;
    using I1 = std::integral_constant<int, 1>;

    // K-step kt out of ring slot SLOT.  On entry A blocks 0..AHEAD-1 and the B blocks of sub-step 0 are in
    // registers, tiles up to kt+NS-2 and the first H1 copies of tile kt+NS-1 have been requested.
    auto kstep = [&](auto slot_c, int kt) {
        constexpr int SLOT = decltype(slot_c)::value;
        using IS = std::integral_constant<int, SLOT>;
        using IN = std::integral_constant<int, (SLOT + 1) % NS>;
        using IF = std::integral_constant<int, (SLOT + NS - 1) % NS>;
        const int far1 = kt + NS - 1 < nk ? kt + NS - 1 : nk - 1;  // clamped: a surplus reload is never read
        const int far2 = kt + NS < nk ? kt + NS : nk - 1;
        static_for<MA>([&](auto gg) {
            constexpr int G = decltype(gg)::value;
            // the last H2 copies of tile kt+NS-1, spread over the first AHEAD groups
            constexpr int before = G < AHEAD ? (G * H2) / AHEAD : H2, after = G < AHEAD ? ((G + 1) * H2) / AHEAD : H2;
            group(I0{}, gg, IS{}, I1{}, IS{}, std::integral_constant<int, H1 + before>{},
                  std::integral_constant<int, after - before>{}, IF{}, far1);
        });
        static_for<MA>([&](auto gg) {
            constexpr int G = decltype(gg)::value;
            if constexpr (G == AHEAD) {
                // every read of this slot has been issued; tile kt+1 must have landed, (NS-2) K-steps of
                // copies may stay in flight
                asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" : : "n"((NS - 2) * LPS) : "memory");
                __builtin_amdgcn_s_barrier();
            }
            // the first H1 copies of tile kt+NS into the slot the barrier freed, spread over the groups after it
            constexpr int R = MA - AHEAD, Q = G - AHEAD;
            constexpr int before = G < AHEAD ? 0 : (Q * H1) / R, after = G < AHEAD ? 0 : ((Q + 1) * H1) / R;
            group(I1{}, gg, IS{}, I0{}, IN{}, std::integral_constant<int, before>{},
                  std::integral_constant<int, after - before>{}, IS{}, far2);
        });
    };

    // every slot is free at the start: request the first NS-1 K-steps and the first part of the next one at
    // once, then wait for the first only
    static_for<NS - 1>([&](auto ss) {
        constexpr int S = decltype(ss)::value;
        const int kt = S < nk ? S : nk - 1;
#pragma unroll
        for (int n = 0; n < LPS; ++n) gll(n, kt, S);
    });
    {
        const int kf = NS - 1 < nk ? NS - 1 : nk - 1;
#pragma unroll
        for (int n = 0; n < H1; ++n) gll(n, kf, NS - 1);
    }
    asm volatile("s_waitcnt vmcnt(%0)" : : "n"((NS - 2) * LPS + H1) : "memory");
    __syncthreads();
    static_for<AHEAD>([&](auto ii) { rd_a(ii, I0{}, I0{}); });
    static_for<NB>([&](auto jj) { rd_b(jj, I0{}, I0{}); });
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");

    for (int kt = 0; kt < nk; kt += NS)
        static_for<NS>([&](auto ii) {
            constexpr int I = decltype(ii)::value;
            if (kt + I < nk) kstep(ii, kt + I);
        });
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
    __syncthreads();  // nobody reads operand tiles any more: LDS becomes the epilogue's staging area

    epilogue16<MA, NB>(acc, smem_raw, WGM * WGN, wave, lane, Cv, ldc, epi, M, N, m0 + wm * WM, n0 + wn * WN);
}

template <bool A_KMAJOR, bool B_KMAJOR, int BM, int BN, int WGM, int WGN, int NS, bool SPLIT>
__global__ __launch_bounds__(WGM *WGN * 64) void gemm_bf16_kernel(
    int64_t M, int64_t N, int64_t K, const bf16 *__restrict__ A, int64_t lda, const bf16 *__restrict__ B,
    int64_t ldb, void *__restrict__ Cv, int64_t ldc, EpiBf16 epi, int tiles_m, int tiles_n)
{
    gemm_bf16_tile<A_KMAJOR, B_KMAJOR, BM, BN, WGM, WGN, NS, SPLIT>(M, N, K, A, lda, B, ldb, Cv, ldc, epi, tiles_m,
                                                                    tiles_n, (int)blockIdx.x);
}

// Several products with the same K and the same epilogue as one grid: the tiles of product p are the work-groups
// first[p] .. first[p+1]-1.  Every tile takes the same time, so CUs go from one product's last tiles straight to
// the next one's first, and the launch takes ceil(all tiles / 256) rounds of one tile per CU where one launch per
// product takes the sum of each product's rounded-up rounds (the four weight-gradient products of a block at
// hidden 5120, ffn 13824: 19 rounds instead of 21; at hidden 2048, ffn 8192: 3 instead of 4).
struct GemmGroupBf16 {
    int n;
    int first[kGemmGroupMax + 1];
    struct Problem {
        int64_t M, N;
        const bf16 *A, *B;
        void *C;
        int64_t lda, ldb, ldc;
        int tiles_m, tiles_n;
    } p[kGemmGroupMax];
};

template <bool A_KMAJOR, bool B_KMAJOR, int BM, int BN, int WGM, int WGN, int NS, bool SPLIT>
__global__ __launch_bounds__(WGM *WGN * 64) void gemm_bf16_group_kernel(GemmGroupBf16 g, int64_t K, EpiBf16 epi)
{
    const int id = (int)blockIdx.x;
    int p = 0;
    for (int i = 1; i < g.n; ++i)
        if (id >= g.first[i]) p = i;
    const GemmGroupBf16::Problem &q = g.p[p];
    gemm_bf16_tile<A_KMAJOR, B_KMAJOR, BM, BN, WGM, WGN, NS, SPLIT>(q.M, q.N, K, q.A, q.lda, q.B, q.ldb, q.C, q.ldc, epi,
                                                                    q.tiles_m, q.tiles_n, id - g.first[p]);
}

// One launch wrapper for every instantiation: raises the kernel's dynamic LDS limit once per process (guarded, so
// that host threads driving different stages may launch concurrently) and starts one work-group per tile.
template <class Kernel>
static hipError_t launch_tiles(Kernel kern, std::once_flag &once, hipError_t &attr_err, int BM, int BN, int threads,
                               size_t lds, int64_t M, int64_t N, int64_t K, const bf16 *A, int64_t lda, const bf16 *B,
                               int64_t ldb, void *C, int64_t ldc, const EpiBf16 &e, hipStream_t s)
{
    std::call_once(once, [&] {
        attr_err = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)lds);
    });
    if (attr_err != hipSuccess) return attr_err;
    const int tiles_m = (int)((M + BM - 1) / BM), tiles_n = (int)((N + BN - 1) / BN);
    kern<<<dim3((unsigned)(tiles_m * tiles_n)), threads, lds, s>>>(M, N, K, A, lda, B, ldb, C, ldc, e, tiles_m, tiles_n);
    return hipGetLastError();
}

// LDS of a work-group: the operand ring, or what the epilogue lays over it: per wave a 32-row staging slice of the
// wave tile in fp32 and two 32-row buffers of a bf16 side input
template <int BM, int BN, int WGM, int WGN, int NS>
static constexpr size_t gemm_lds_bytes()
{
    constexpr int WN = BN / WGN;
    constexpr size_t ring = (size_t)NS * (BM + BN) * kBK * sizeof(bf16);
    constexpr size_t epi = (size_t)WGM * WGN * (32 * epi_stride(WN / 32) * 4 + 2 * 32 * WN * 2);
    return ring > epi ? ring : epi;
}

template <bool A_KMAJOR, bool B_KMAJOR, int BM, int BN, int WGM, int WGN, int NS, bool SPLIT = false>
static hipError_t launch_kernel(int64_t M, int64_t N, int64_t K, const bf16 *A, int64_t lda, const bf16 *B, int64_t ldb,
                                void *C, int64_t ldc, const EpiBf16 &e, hipStream_t s)
{
    static std::once_flag once;
    static hipError_t attr_err = hipSuccess;
    return launch_tiles(gemm_bf16_kernel<A_KMAJOR, B_KMAJOR, BM, BN, WGM, WGN, NS, SPLIT>, once, attr_err, BM, BN,
                        WGM * WGN * 64, gemm_lds_bytes<BM, BN, WGM, WGN, NS>(), M, N, K, A, lda, B, ldb, C, ldc, e, s);
}

static EpiBf16 bf16_epilogue(const GemmEpi &epi)
{
    return EpiBf16{(const bf16 *)epi.bias, (const bf16 *)epi.resid, (const bf16 *)epi.aux, (bf16 *)epi.out2,
                   epi.act,                epi.gelu_mode,           epi.out_f32,           epi.accum_scale};
}

bool gemm_bf16_tt_supported(int64_t M, int64_t N, int64_t K, int64_t lda, int64_t ldb)
{
    return M > 0 && N > 0 && K > 0 && M % 256 == 0 && N % 256 == 0 && K % kBK == 0 && lda % 8 == 0 && ldb % 8 == 0 &&
           64 * lda * 2 < (int64_t)1 << 31 && 64 * ldb * 2 < (int64_t)1 << 31;
}

hipError_t launch_gemm_bf16_tt(int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *B, int64_t ldb,
                               void *C, int64_t ldc, const GemmEpi &epi, hipStream_t s)
{
    if (!gemm_bf16_tt_supported(M, N, K, lda, ldb)) return hipErrorInvalidValue;
    return launch_kernel<true, true, 256, 256, 2, 4, 2, true>(M, N, K, (const bf16 *)A, lda, (const bf16 *)B, ldb, C, ldc,
                                                              bf16_epilogue(epi), s);
}

hipError_t launch_gemm_bf16_tt_group(const GemmProblem *problems, int n, int64_t K, const GemmEpi &epi, hipStream_t s)
{
    if (n < 1 || n > kGemmGroupMax || epi.bias || epi.resid || epi.aux || epi.out2 || epi.act != ACT_NONE)
        return hipErrorInvalidValue;
    GemmGroupBf16 g;
    g.n = n;
    int64_t tiles = 0;
    for (int i = 0; i < n; ++i) {
        const GemmProblem &q = problems[i];
        if (!gemm_bf16_tt_supported(q.M, q.N, K, q.lda, q.ldb)) return hipErrorInvalidValue;
        g.first[i] = (int)tiles;
        g.p[i] = {q.M, q.N, (const bf16 *)q.A, (const bf16 *)q.B, q.C, q.lda, q.ldb, q.ldc, (int)(q.M / 256), (int)(q.N / 256)};
        tiles += (q.M / 256) * (q.N / 256);
        if (tiles >= (int64_t)1 << 31) return hipErrorInvalidValue;
    }
    for (int i = n; i <= kGemmGroupMax; ++i) g.first[i] = (int)tiles;
    for (int i = n; i < kGemmGroupMax; ++i) g.p[i] = g.p[0];
    static std::once_flag once;
    static hipError_t attr_err = hipSuccess;
    auto kern = gemm_bf16_group_kernel<true, true, 256, 256, 2, 4, 2, true>;
    constexpr size_t lds = gemm_lds_bytes<256, 256, 2, 4, 2>();
    std::call_once(once, [&] {
        attr_err = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)lds);
    });
    if (attr_err != hipSuccess) return attr_err;
    kern<<<dim3((unsigned)tiles), 512, lds, s>>>(g, K, bf16_epilogue(epi));
    return hipGetLastError();
}

bool gemm_bf16_nn_supported(int64_t M, int64_t N, int64_t K, int64_t lda, int64_t ldb)
{
    return M > 0 && N > 0 && K > 0 && N % 256 == 0 && K % kBK == 0 && lda % 8 == 0 && ldb % 8 == 0 &&
           64 * ldb * 2 < (int64_t)1 << 31 && 256 * lda * 2 < (int64_t)1 << 31;
}

hipError_t launch_gemm_bf16_nn(int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *B, int64_t ldb,
                               void *C, int64_t ldc, const GemmEpi &epi, hipStream_t s)
{
    if (!gemm_bf16_nn_supported(M, N, K, lda, ldb)) return hipErrorInvalidValue;
    const EpiBf16 e = bf16_epilogue(epi);
    // 256x256 tiles when they come in whole rounds of one per CU (or in many), else 128x256 with the deeper ring
    const int64_t t256 = ((M + 255) / 256) * (N / 256);
    if (t256 >= 256 && (t256 % 256 == 0 || t256 >= 1024))
        return launch_kernel<false, true, 256, 256, 2, 4, 2>(M, N, K, (const bf16 *)A, lda, (const bf16 *)B, ldb, C, ldc, e, s);
    return launch_kernel<false, true, 128, 256, 2, 4, 3>(M, N, K, (const bf16 *)A, lda, (const bf16 *)B, ldb, C, ldc, e, s);
}

bool gemm_bf16_supported(int64_t M, int64_t N, int64_t K)
{
    return M > 0 && N > 0 && K > 0 && (K % kBK) == 0;
}

hipError_t launch_gemm_bf16_nt(int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *B,
                               int64_t ldb, void *C, int64_t ldc, const GemmEpi &epi, hipStream_t s, int tile)
{
    if (M == 0 || N == 0) return hipSuccess;
    if (!gemm_bf16_supported(M, N, K) || (lda % 8) || (ldb % 8)) return hipErrorInvalidValue;
    // per-lane byte offsets inside a tile (up to 255 rows) are 32-bit
    if (256 * lda * 2 >= (int64_t)1 << 32 || 256 * ldb * 2 >= (int64_t)1 << 32) return hipErrorInvalidValue;
    const EpiBf16 e = bf16_epilogue(epi);
    const bf16 *a = (const bf16 *)A, *b = (const bf16 *)B;
    if (tile == GEMM_TILE_AUTO) {
        // 256x256 tiles, two LDS stages: lowest LDS and L2 traffic per flop, but one work-group per CU, so a
        // grid runs in rounds of 256 tiles; used when the rounds come out whole (or there are many).
        // Otherwise 256x128 / 128x256 tiles with three stages: twice as many tiles, and copies issued two
        // K-steps ahead, which the shorter K-step of a smaller tile needs (a T x h output at T = 2048 is 128
        // big tiles; T x 3h is 384, a round and a half).  Small problems: 128x128.
        const int64_t t256 = ((M + 255) / 256) * ((N + 255) / 256);
        if (t256 >= 256 && (t256 % 256 == 0 || t256 >= 1024)) {
            tile = GEMM_TILE_256x256;
        } else {
            const int64_t ta = ((M + 255) / 256) * ((N + 127) / 128), tb = ((M + 127) / 128) * ((N + 255) / 256);
            if (ta >= 192 || tb >= 192)
                tile = tb >= 192 ? GEMM_TILE_128x256 : GEMM_TILE_256x128;
            else
                tile = GEMM_TILE_128x128;
        }
    }
    switch (tile) {
    case GEMM_TILE_256x256: return launch_kernel<false, false, 256, 256, 2, 4, 2>(M, N, K, a, lda, b, ldb, C, ldc, e, s);
    case GEMM_TILE_128x128: return launch_kernel<false, false, 128, 128, 2, 2, 2>(M, N, K, a, lda, b, ldb, C, ldc, e, s);
    case GEMM_TILE_256x128: return launch_kernel<false, false, 256, 128, 4, 2, 3>(M, N, K, a, lda, b, ldb, C, ldc, e, s);
    case GEMM_TILE_128x256: return launch_kernel<false, false, 128, 256, 2, 4, 3>(M, N, K, a, lda, b, ldb, C, ldc, e, s);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace zpp
