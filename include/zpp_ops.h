/*
 * zpp_ops.h — operator-level entry points of the same library, for per-kernel parity tests and
 * micro-benchmarks.  They launch exactly the kernels the stage calls in zpp.h use.  All pointers
 * are DEVICE pointers owned by the caller; work is enqueued on `hip_stream`; nothing allocates or
 * synchronises.  Errors are reported as in zpp.h.
 */
#ifndef ZPP_OPS_H
#define ZPP_OPS_H

#include "zpp.h"

#ifdef __cplusplus
extern "C" {
#endif

/* bf16 MFMA GEMM with fp32 accumulation: C[M,N] = A[M,K] . B[N,K]^T (+ bias[n]) (+ resid[m,n]).
 * This is the shape of every linear layer of the transformer block (Section 4.1) and, with
 * transposed operands, of the input- and weight-gradient products of Section 2.3.
 * A, B: bf16, K-contiguous, leading dimensions lda, ldb (elements, multiples of 8); K % 64 == 0.
 * C: bf16, or float when out_f32 != 0; leading dimension ldc.  bias, resid: bf16 or NULL.
 * out_f32 == 2: C is float and receives C + result (the in-place gradient accumulation of
 * stage_backward_accumulate, scale 1), so C must hold valid data on entry.
 * tile: -1 chosen from the shape; 0 256x256 and 1 128x128 work-group tiles (two LDS stages), 2 256x128 and
 * 3 128x256 (a ring of three LDS stages): the kernels the stage calls select among. */
zpp_status zpp_op_gemm_bf16_nt(int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *B,
                               int64_t ldb, void *C, int64_t ldc, const void *bias, const void *resid,
                               int32_t out_f32, int32_t tile, void *hip_stream);

/* The weight-gradient product of Section 2.3 without any transposition in memory: C[M,N] = A^T . B with A stored
 * [K, M] (M contiguous, leading dimension lda >= M) and B stored [K, N] (leading dimension ldb >= N), i.e.
 * dW[out,in] = dY[T,out]^T . X[T,in] read from the token-major activations where they lie.  bf16 operands, fp32
 * accumulation; C is bf16 (out_f32 == 0), float (1), or float and receives C + result (2).  M and N multiples
 * of 256, K a multiple of 64, lda and ldb multiples of 8 (ZPP_ERR_UNSUPPORTED otherwise; the stage then
 * transposes the operands and uses the product above). */
zpp_status zpp_op_gemm_bf16_tt(int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *B,
                               int64_t ldb, void *C, int64_t ldc, int32_t out_f32, void *hip_stream);

/* n (1..8) such products with the same K and the same kind of C as one launch: the weight-gradient products of
 * a block (Section 2.3) taken together, as the stage issues them, so that the grid is all their tiles back to
 * back and a product whose tiles do not fill the last round of one tile per CU shares that round with the next
 * product.  M, N, A, lda, B, ldb, C, ldc are host arrays of n entries (device pointers inside A, B, C); the
 * outputs must not overlap.  Each product's requirements and errors are those of zpp_op_gemm_bf16_tt, and every
 * C element gets the bits that call gives it. */
zpp_status zpp_op_gemm_bf16_tt_group(int32_t n, const int64_t *M, const int64_t *N, int64_t K, const void *const *A,
                                     const int64_t *lda, const void *const *B, const int64_t *ldb, void *const *C,
                                     const int64_t *ldc, int32_t out_f32, void *hip_stream);

/* The input-gradient product of Section 2.3 read from the weights as they are stored: C[M,N] = A . B with A
 * [M, K] (K contiguous, leading dimension lda >= K) and B [K, N] (N contiguous, leading dimension ldb >= N),
 * i.e. dX[T,in] = dY[T,out] . W[out,in] without a transposed copy of W.  bf16 operands, fp32 accumulation; C
 * as for the products above.  N a multiple of 256, K a multiple of 64, lda and ldb multiples of 8
 * (ZPP_ERR_UNSUPPORTED otherwise; the stage then keeps a transposed copy of that matrix). */
zpp_status zpp_op_gemm_bf16_nn(int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *B,
                               int64_t ldb, void *C, int64_t ldc, int32_t out_f32, void *hip_stream);

/* Causal attention over packed qkv[T, 3h] (Q | K | V, head-major inside each; T = b*seq, h = nh*d):
 * attn[T, h] = softmax(Q K^T / sqrt(d) + causal mask) V per (sample, head); lse[b, nh, seq] is the
 * log-sum-exp of the scaled, masked scores.  dtype: ZPP_DTYPE_*; impl 0 = generic kernel,
 * 1 = MFMA kernel (bf16, d = 128, seq % 128 == 0). */
zpp_status zpp_op_attention_fwd(int32_t dtype, int32_t impl, const void *qkv, void *attn, float *lse, int64_t b,
                                int64_t seq, int64_t nh, int64_t d, void *hip_stream);

/* Backward of the above: dqkv[T, 3h] = (dQ | dK | dV) from dattn[T, h]; delta is scratch of 2 * b * nh * seq
 * floats (per query the row sum of dattn o attn and the log-sum-exp in the units the exponentials use). */
zpp_status zpp_op_attention_bwd(int32_t dtype, int32_t impl, const void *qkv, const void *attn, const void *dattn,
                                const float *lse, float *delta, void *dqkv, int64_t b, int64_t seq, int64_t nh,
                                int64_t d, void *hip_stream);

/* For callers that cannot allocate device memory (HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc): zpp_op_attention_bwd without the `delta` argument.  The 2 * b * nh * seq floats of
 * scratch live in an 8 MiB array inside the library's device image (one copy per GPU the library runs on,
 * held until the process ends), so the call allocates nothing, and neither does anything it calls.
 * Limit: b * nh * seq <= zpp_op_attention_bwd_noalloc_max_rows() (2^20), ZPP_ERR_WORKSPACE beyond it.
 * The device of `hip_stream` must be the current device.  Every byte of scratch the kernels read is
 * written by the same call first, so nothing needs clearing between calls; but all calls on one GPU
 * share that GPU's array: calls that overlap in time on one GPU (different streams or host threads) race
 * and must be serialised by the caller.  Same kernels and same results as zpp_op_attention_bwd. */
uint64_t zpp_op_attention_bwd_noalloc_max_rows(void);
zpp_status zpp_op_attention_bwd_noalloc(int32_t dtype, int32_t impl, const void *qkv, const void *attn,
                                        const void *dattn, const float *lse, void *dqkv, int64_t b, int64_t seq,
                                        int64_t nh, int64_t d, void *hip_stream);

/* The flat-buffer passes on raw arrays of n elements (16-byte aligned): the optimizer step (zero_grad 0 or 1: there
 * is no stage here that could hold a released G), the gradient accumulation G += scale*S, and the fp32 ->
 * working-copy cast. */
zpp_status zpp_op_flat_adam(float *P, float *M, float *V, float *G, uint64_t n, const zpp_adam *hp, void *hip_stream);
zpp_status zpp_op_flat_accumulate(float *G, const float *S, uint64_t n, float scale, void *hip_stream);
zpp_status zpp_op_flat_materialize(const float *P, void *W, uint64_t n, int32_t dtype, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* ZPP_OPS_H */
