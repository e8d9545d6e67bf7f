// Internal host-side launch API of the gfx950 kernels.  Everything is enqueued on the given
// stream; nothing allocates or synchronises.  Pointers are device pointers.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace zpp {

enum { DT_F32 = 0, DT_BF16 = 1 };
enum { NORM_LAYER = 0, NORM_RMS = 1 };
enum { COLRED_SUM = 0, COLRED_LAYERNORM = 1, COLRED_RMSNORM = 2 };
// ACT_GELU_DUAL: C receives the pre-activation u, out2 gelu(u).  ACT_DGELU_MUL: out = acc * gelu'(aux), aux = u.
// ACT_GELU_GRAD_DUAL (bf16 products): C receives gelu'(u) and out2 gelu(u), u being the pre-activation rounded to
// bf16 (it is not stored); ACT_MUL_AUX: out = acc * aux.  The pair moves the derivative's arithmetic from the
// backward epilogue, where it would be evaluated alone, into the forward one, where it shares the logistic function
// with the activation.  In bf16 ACT_DGELU_MUL multiplies by the derivative rounded to bf16, so that both pairs
// give the same bits.
enum { ACT_NONE = 0, ACT_GELU_DUAL = 1, ACT_DGELU_MUL = 2, ACT_GELU_GRAD_DUAL = 3, ACT_MUL_AUX = 4 };

inline size_t dt_size(int dt) { return dt == DT_BF16 ? 2 : 4; }

struct AdamArgs {
    float lr, beta1, beta2, eps, wd, grad_scale;
    float omb1, omb2;  // 1-beta1, 1-beta2, formed in double on the host and rounded once
    float c1, c2;      // bias corrections 1-beta1^t, 1-beta2^t
    int decoupled, zero_grad;
    void *wb = nullptr;  // optional write-back: bf16 (wb_bf16) or float copy of the new parameters, same indexing as P
    int wb_bf16 = 0;
};

// Up to kAdamRanges ranges of one flat shard updated by one launch, each with its own learning rate and
// weight decay (everything else from AdamArgs).  offset/count in elements, multiples of 4.
constexpr int kAdamRanges = 32;
struct AdamRanges {
    uint64_t offset[kAdamRanges], count[kAdamRanges];
    float lr[kAdamRanges], wd[kAdamRanges];
    uint32_t first_block[kAdamRanges + 1];  // blocks [first_block[i], first_block[i+1]) work on range i
    int32_t n;
};
hipError_t launch_adam_ranges(float *P, float *M, float *V, float *G, AdamRanges r, const AdamArgs &a, hipStream_t s);

// Epilogue of a GEMM: out = act(acc + bias[n] + resid[m,n]).
struct GemmEpi {
    const void *bias = nullptr;   // [N], element type of the compute dtype, or null
    const void *resid = nullptr;  // [M, ldc], element type of the compute dtype, or null
    void *out2 = nullptr;         // ACT_GELU_DUAL, ACT_GELU_GRAD_DUAL: receives gelu(u)
    const void *aux = nullptr;    // ACT_DGELU_MUL: pre-activation u[m,n]; ACT_MUL_AUX: the factor itself
    int act = ACT_NONE;
    int gelu_mode = 0;
    int out_f32 = 0;              // 1: C is float regardless of the compute dtype (weight gradients);
                                  // 2: as 1, and C <- C + accum_scale * result (accumulation in place)
    float accum_scale = 1.0f;
};

// ---- flat-buffer passes (HBM bound) ----
hipError_t launch_materialize(const float *P, void *W, uint64_t n, int dt, hipStream_t s);
// Wt[c, r] = bf16(P[r, c]) for a [rows, cols] matrix
hipError_t launch_transpose_cast(const float *P, void *Wt, uint64_t rows, uint64_t cols, hipStream_t s);
// The same for up to kTransposeCastMax matrices in one launch: matrix i is P[src[i] ...] of [rows[i], cols[i]]
// (rows a multiple of 128, cols of 64) and goes to Wt[dst[i] ...] (element offsets).
constexpr int kTransposeCastMax = 24;
struct TransposeCastTable {
    uint64_t src[kTransposeCastMax], dst[kTransposeCastMax], rows[kTransposeCastMax], cols[kTransposeCastMax];
    uint32_t first_block[kTransposeCastMax + 1];
    int32_t n;
};
hipError_t launch_transpose_cast_many(const float *P, void *Wt, TransposeCastTable tab, hipStream_t s);
// first: G counts as zero and is not read (G <- 0 + scale * S)
hipError_t launch_accumulate(float *G, const float *S, uint64_t n, float scale, hipStream_t s, bool first = false);
hipError_t launch_fill_zero(float *G, uint64_t n, hipStream_t s);
hipError_t launch_adam(float *P, float *M, float *V, float *G, uint64_t n, const AdamArgs &a, hipStream_t s);

// ---- norms ----
// n = gamma * xhat (+ beta); mean (LayerNorm only) and rstd are saved; xcopy (nullable) receives x.
hipError_t launch_norm_fwd(int dt, int kind, const void *x, const void *gamma, const void *beta, int64_t T,
                           int64_t h, float eps, void *n, float *mean, float *rstd, void *xcopy,
                           hipStream_t s);
// dx = resid + d(norm)/dx
hipError_t launch_norm_bwd(int dt, int kind, const void *dn, const void *x, const float *mean,
                           const float *rstd, const void *gamma, const void *resid, void *dx, int64_t T,
                           int64_t h, hipStream_t s);
// Column reductions over T rows of a [T, C] matrix with row stride ld:
//   COLRED_SUM: out0[c] = sum_t a[t,c]
//   COLRED_LAYERNORM: out0[c] = sum_t a[t,c]*(x[t,c]-mean[t])*rstd[t], out1[c] = sum_t a[t,c]
//   COLRED_RMSNORM:   out0[c] = sum_t a[t,c]*x[t,c]*rstd[t]
// partial: scratch of colreduce_scratch_floats(T, C) floats.
// A column reduction in two levels: the first-level kernels above/below leave `rows` partial rows of C
// floats each (two sets for COLRED_LAYERNORM, the second `rows * C` floats after the first); the second
// level adds them up in a fixed order.  The second level of many reductions can be batched into one
// launch (they are tiny and otherwise cost a launch each): pass `defer` to the first-level launchers,
// collect the items, and call launch_finish_columns once.  Partials must stay untouched until then.
struct FinishItem {
    const float *partial0, *partial1;  // partial1 may be null
    float *out0, *out1;
    int32_t rows;
    int64_t C;
};
// accumulate: out <- out + scale * sum instead of out <- sum
hipError_t launch_finish_columns(const FinishItem *items, int n, hipStream_t s, bool accumulate = false,
                                 float scale = 1.0f);
// Two bf16 transposes in one launch: a[Ra, Ca] -> a_out[Ca, Ra] (with column sums of a when colsum is
// given; then partial and defer as for launch_transpose_colsum, second level deferred), b likewise
// without sums.  All sizes multiples of 64.
hipError_t launch_transpose_pair(const void *a, int64_t Ra, int64_t Ca, int64_t lda, void *a_out, int64_t lda_out,
                                 float *colsum, float *partial, FinishItem *defer, const void *b, int64_t Rb,
                                 int64_t Cb, int64_t ldb, void *b_out, int64_t ldb_out, hipStream_t s);
uint64_t colreduce_scratch_floats(int64_t T, int64_t C);
// launch_norm_bwd and the first level of the COLRED_LAYERNORM / COLRED_RMSNORM reduction of (dn, x) in one
// launch; the second level is left in *defer.  partial: colreduce_scratch_floats(T, h) floats.
hipError_t launch_norm_bwd_colreduce(int dt, int kind, const void *dn, const void *x, const float *mean,
                                     const float *rstd, const void *gamma, const void *resid, void *dx, int64_t T,
                                     int64_t h, float *dgamma, float *dbeta, float *partial, FinishItem *defer,
                                     hipStream_t s);
hipError_t launch_colreduce(int dt, int mode, const void *a, const void *x, const float *mean,
                            const float *rstd, int64_t T, int64_t C, int64_t ld, float *out0, float *out1,
                            float *partial, hipStream_t s, FinishItem *defer = nullptr);

// ---- elementwise ----
// out[c, r] = in[r, c]; in has row stride ld_in, out row stride ld_out (elements)
hipError_t launch_transpose(int dt, const void *in, int64_t R, int64_t C, int64_t ld_in, void *out,
                            int64_t ld_out, hipStream_t s);
// bf16 only: transpose plus colsum[c] = sum_r in[r, c] in the same pass (R, C multiples of 64);
// partial: scratch of transpose_colsum_scratch_floats(R, C) floats.
uint64_t transpose_colsum_scratch_floats(int64_t R, int64_t C);
hipError_t launch_transpose_colsum(const void *in, int64_t R, int64_t C, int64_t ld_in, void *out,
                                   int64_t ld_out, float *colsum, float *partial, hipStream_t s,
                                   FinishItem *defer = nullptr);
// table[p, i] = (cos, sin)(p * base^(-2i/d)), p < seq, i < d/2
hipError_t launch_rope_table(float *table, int64_t seq, int64_t d, double base, hipStream_t s);
// rotates the Q and K parts of qkv[T, 3h] in place; sign = +1 forward, -1 inverse
hipError_t launch_rope(int dt, void *qkv, const float *table, int64_t T, int64_t seq, int64_t nh, int64_t d,
                       int sign, hipStream_t s);
// g[i] = GeLU(u[i]), n elements (a multiple of the 16-byte vector), as the epilogue of the first MLP product
hipError_t launch_gelu_fwd(int dt, const void *u, void *g, int64_t n, int gelu_mode, hipStream_t s);
// gu = [gate | up] of shape [T, 2f]; act[T, f] = silu(gate) * up
hipError_t launch_swiglu_fwd(int dt, const void *gu, void *act, int64_t T, int64_t f, hipStream_t s);
hipError_t launch_swiglu_bwd(int dt, const void *gu, const void *dact, void *dgu, int64_t T, int64_t f,
                             hipStream_t s);

// ---- GEMMs ----
// Generic strided fp32 GEMM: C[m,n] = sum_k A[m*sam + k*sak] * B[n*sbn + k*sbk], then the epilogue.
hipError_t launch_gemm_f32(int64_t M, int64_t N, int64_t K, const float *A, int64_t sam, int64_t sak,
                           const float *B, int64_t sbn, int64_t sbk, float *C, int64_t ldc,
                           const GemmEpi &epi, hipStream_t s);
// bf16 MFMA GEMM, both operands K-contiguous: C[M,N] = A[M,K] . B[N,K]^T with fp32 accumulation.
// Requires K % 64 == 0, lda/ldb % 8 == 0, 16-byte aligned bases.  tile: the work-group tile, chosen from
// the shape when GEMM_TILE_AUTO (256x256 and 128x128: two LDS stages; 256x128 and 128x256: a ring of three).
enum { GEMM_TILE_AUTO = -1, GEMM_TILE_256x256 = 0, GEMM_TILE_128x128 = 1, GEMM_TILE_256x128 = 2, GEMM_TILE_128x256 = 3,
       GEMM_TILE_LAST = 3 };
hipError_t launch_gemm_bf16_nt(int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *B,
                               int64_t ldb, void *C, int64_t ldc, const GemmEpi &epi, hipStream_t s,
                               int tile = GEMM_TILE_AUTO);
// The same product with both operands stored K-major: C[M,N] = A^T . B, A is [K, M] (row stride lda, M contiguous),
// B is [K, N] (row stride ldb): the weight-gradient product read from token-major activations in place.
// Only for shapes gemm_bf16_tt_supported accepts (M, N multiples of 256, K of 64).
bool gemm_bf16_tt_supported(int64_t M, int64_t N, int64_t K, int64_t lda, int64_t ldb);
hipError_t launch_gemm_bf16_tt(int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *B,
                               int64_t ldb, void *C, int64_t ldc, const GemmEpi &epi, hipStream_t s);
// Up to kGemmGroupMax K-major products with the same K and the same plain fp32 epilogue (write, or add into C
// in place) as one launch; each must be a shape gemm_bf16_tt_supported accepts.  Every C element is computed
// exactly as launch_gemm_bf16_tt computes it.
constexpr int kGemmGroupMax = 8;
struct GemmProblem {
    int64_t M, N;
    const void *A;
    int64_t lda;
    const void *B;
    int64_t ldb;
    void *C;
    int64_t ldc;
};
hipError_t launch_gemm_bf16_tt_group(const GemmProblem *problems, int n, int64_t K, const GemmEpi &epi, hipStream_t s);
// The same product with A K-contiguous ([M, K], row stride lda) and B stored [K, N] (row stride ldb): the
// input-gradient product read from the weights as stored.  Only for shapes gemm_bf16_nn_supported accepts
// (N a multiple of 256, K of 64).
bool gemm_bf16_nn_supported(int64_t M, int64_t N, int64_t K, int64_t lda, int64_t ldb);
hipError_t launch_gemm_bf16_nn(int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *B,
                               int64_t ldb, void *C, int64_t ldc, const GemmEpi &epi, hipStream_t s);
bool gemm_bf16_supported(int64_t M, int64_t N, int64_t K);

// ---- causal attention over packed qkv[T, 3h] (Q | K | V, head-major inside each) ----
// attn[T, h] (heads merged), lse[b, nh, s] = log-sum-exp of the scaled masked scores.
hipError_t launch_attn_fwd(int dt, const void *qkv, void *attn, float *lse, int64_t b, int64_t seq,
                           int64_t nh, int64_t d, hipStream_t s);
// delta is scratch of 2 * b * nh * s floats (sum_e dattn*attn per query, then the log-sum-exp times log2(e));
// dqkv[T, 3h] receives dQ | dK | dV.
hipError_t launch_attn_bwd(int dt, const void *qkv, const void *attn, const void *dattn, const float *lse,
                           float *delta, void *dqkv, int64_t b, int64_t seq, int64_t nh, int64_t d,
                           hipStream_t s);
bool attn_mfma_supported(int64_t seq, int64_t d);

}  // namespace zpp
