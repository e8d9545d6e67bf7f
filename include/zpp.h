/*
 * zpp.h — C ABI of the ZeroPP stage hot path on one MI355X (gfx950).
 *
 * What one GPU does under the ZeroPP schedule (the pipeline schedule of paper Section 3.1 and its
 * combination with ZeRO-3 and data parallelism in Section 3.2): the micro-batches of a pipeline stage run
 * back to back inside a scheduling unit of U micro-batches, so that the stage's parameters are
 * gathered once per unit (not once per micro-batch), its gradients are reduced once per unit, and
 * the optimizer step runs on the local partition of the model state.  With one GPU the gather is
 * a local cast/copy out of the flat fp32 master shard and the reduce-scatter is a local
 * accumulation into the flat fp32 gradient shard.
 *
 * Conventions
 *   - Every pointer named P, G, M, V, workspace, x, y, dy, dx is DEVICE memory owned by the caller.
 *     The library allocates no device memory, creates no streams and never synchronises; all work
 *     is enqueued on the `hip_stream` argument (a hipStream_t passed as void*, NULL = default
 *     stream).  Handles hold host metadata only.
 *   - Tensors are row-major.  Activations are [T, h] with T = micro_batch * seq tokens and the
 *     hidden axis contiguous; samples of a micro-batch are consecutive blocks of `seq` rows.
 *   - Activation element type: float when compute_dtype = ZPP_DTYPE_FP32, bf16 (upper half of an
 *     IEEE float, 2 bytes) when compute_dtype = ZPP_DTYPE_BF16.  P, G, M, V are always float.
 *   - Device pointers must be 256-byte aligned.
 *   - Every call returns a zpp_status; 0 is success.  Argument, state and alignment errors are
 *     found on the host before anything is launched.  zpp_last_error() returns a thread-local
 *     message for the last failing call.  No C++ exception crosses this boundary.
 *
 * Flat parameter layout (shared by P, G, M, V, the working copy and the staging gradients): blocks
 * concatenated without padding; inside a block, in this order, each matrix [out_features,
 * in_features] row-major so that y = x W^T + b:
 *   GPT   (arch 0): ln1.gamma[h] ln1.beta[h] attn.wqkv[3h,h] attn.bqkv[3h] attn.wo[h,h] attn.bo[h]
 *                   ln2.gamma[h] ln2.beta[h] mlp.w1[f,h] mlp.b1[f] mlp.w2[h,f] mlp.b2[h]
 *   LLaMA (arch 1): norm1.gamma[h] attn.wqkv[3h,h] attn.wo[h,h] norm2.gamma[h]
 *                   mlp.wgate[f,h] mlp.wup[f,h] mlp.wdown[h,f]
 * Rows of wqkv: all of Q (head n = rows n*d .. (n+1)*d-1), then K, then V.  A GPT block holds
 * 4h^2 + 2hf + 9h + f parameters, i.e. the roughly 12 h^2 per block that Section 4.1 counts with, when f = 4h.
 */
#ifndef ZPP_H
#define ZPP_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct zpp_stage zpp_stage; /* opaque; host-side metadata only */

typedef enum {
    ZPP_OK = 0,
    ZPP_ERR_ARG = -1,         /* null pointer, out-of-range index, inconsistent configuration */
    ZPP_ERR_STATE = -2,       /* call out of order (see the state machine below) */
    ZPP_ERR_ALIGN = -3,       /* device pointer not 256-byte aligned */
    ZPP_ERR_WORKSPACE = -4,   /* workspace smaller than zpp_stage_workspace_bytes() */
    ZPP_ERR_DEVICE = -5,      /* a kernel launch or HIP call failed */
    ZPP_ERR_UNSUPPORTED = -6  /* shape outside what the kernels support */
} zpp_status;

enum { ZPP_ARCH_GPT = 0, ZPP_ARCH_LLAMA = 1 };
enum { ZPP_DTYPE_FP32 = 0, ZPP_DTYPE_BF16 = 1 };
enum { ZPP_GELU_TANH = 0, ZPP_GELU_ERF = 1 };
enum { ZPP_RECOMPUTE_NONE = 0, ZPP_RECOMPUTE_FULL = 1, ZPP_RECOMPUTE_SELECTIVE = 2 };

typedef struct {
    int32_t arch;          /* ZPP_ARCH_GPT: pre-LN LayerNorm, biases, GeLU MLP.
                              ZPP_ARCH_LLAMA: RMSNorm, rotary embedding on Q and K, SwiGLU MLP, no biases */
    int32_t n_blocks;      /* transformer blocks in the stage (a stage is a run of consecutive layers, Section 2.1) */
    int32_t hidden;        /* h */
    int32_t n_heads;       /* head dim d = h / n_heads */
    int32_t ffn;           /* f, MLP width */
    int32_t seq;           /* s */
    int32_t micro_batch;   /* b, samples per micro-batch */
    int32_t unit_mbs;      /* U, micro-batches per scheduling unit (Section 3.1.2) */
    int32_t compute_dtype; /* ZPP_DTYPE_FP32: everything float.  ZPP_DTYPE_BF16: bf16 working copy and
                              activations, fp32 master / gradients / moments, fp32 accumulation */
    int32_t gelu_mode;     /* ZPP_GELU_TANH (default) or ZPP_GELU_ERF */
    float norm_eps;        /* epsilon inside the norm's square root */
    float rope_base;       /* rotary base (LLaMA only); angle = position * base^(-2i/d), adjacent pairs */
    int32_t split_backward; /* g >= 1: the workspace also holds, per (micro-batch, block), what the weight-gradient
                              task needs from the input-gradient task (each linear layer's dY), so that
                              stage_backward_input / stage_backward_weight may be used, and temporaries for
                              weight-gradient tasks of up to g micro-batches at once
                              (stage_backward_weight_group); 0: only the fused calls.  At most unit_mbs */
    int32_t recompute;      /* Activation recomputation (Section 3.3), full or selective.
                              ZPP_RECOMPUTE_FULL: stage_forward keeps only each block's input per micro-batch, and
                              the backward calls run a block's forward again (without its last linear layer,
                              whose output backward does not need) right before its backward.
                              ZPP_RECOMPUTE_SELECTIVE: the products and the attention output are kept, and only
                              what costs next to nothing to rebuild is dropped and rebuilt element-wise in
                              backward: the outputs of the two norms and of the activation function (6h of the
                              16h stored elements per token of a GPT block with f = 4h; the s x s attention
                              probabilities, the usual first choice, are never stored by the fused attention
                              kernels in any mode).
                              Same kernels on the same inputs either way, so results are bit-identical to
                              recompute = 0.  The fused backward calls rebuild once for both gradient tasks; with
                              split_backward each of the two tasks rebuilds for itself (twice the extra work:
                              the reason Section 3.3 recomputes only where the two tasks run back to back) */
    int32_t group_mbs;      /* g >= 2: the stage_*_group calls may take up to g consecutive micro-batches as one
                              matrix of g*T tokens (temporaries are sized for it); 0 or 1: one at a time.  A
                              split_backward = g' > 1 allows groups of g' too.  At most unit_mbs */
} zpp_stage_config;

typedef struct {
    float lr, beta1, beta2, eps, weight_decay;
    float grad_scale;      /* ghat = grad_scale * G */
    int32_t step;          /* t >= 1, used for bias correction */
    int32_t decoupled_wd;  /* 1: p -= lr*wd*p_old (AdamW form).  0: ghat += wd*p (L2 form) */
    int32_t zero_grad;     /* 1: G is zeroed in the same pass.  2 (a step over the whole shard only): G is released
                              instead - it counts as zero, its memory keeps the old gradients, and the first call
                              that adds into G afterwards (stage_accumulate_grads, or a gradient task that
                              accumulates in place) writes instead of adding: the same values as adding onto zeros
                              (an exact zero may differ in sign) without the 4 bytes per element of the zeroing and
                              the 4 of reading the zeros back.  Until then the contents of G mean nothing;
                              zpp_stage_bind forgets the release. */
    int32_t write_back;    /* 1: the updated parameters are also written into the stage's working copy (the bf16
                              round-to-nearest-even cast, or the float copy), so that the next
                              stage_materialize_params need not read P again for it (when the call, or the
                              ranges, covered the whole shard it only refreshes the transposed copies that
                              matrices of unusual shape need, see zpp_stage_workspace_bytes) */
} zpp_adam;

/* ---- handle, sizes, layout (host only; no device is touched) -------------------------------- */

/* Validates the configuration (positive sizes, hidden divisible by n_heads, shapes the kernels
 * support) and creates a handle.  Errors: ZPP_ERR_ARG, ZPP_ERR_UNSUPPORTED. */
zpp_status zpp_stage_create(const zpp_stage_config *cfg, zpp_stage **out);
void zpp_stage_destroy(zpp_stage *stage);

/* N, the number of parameters of the stage = elements of each of P, G, M, V. */
uint64_t zpp_stage_param_count(const zpp_stage *stage);

/* Bytes of caller-owned device workspace the stage needs: the materialised working copy of the
 * stage (one gathered stage, the L*M_w/(P*V) term of the memory formula in Section 4.2; in bf16 mode a
 * matrix [out, in] whose `in` is not a multiple of 256 or whose `out` is not a multiple of 64 also gets a
 * transposed copy there, which the input-gradient product of such a shape reads), the
 * fp32 staging buffer for one micro-batch's weight gradients, the activation stash of one
 * scheduling unit (the min(B,U)*L*M_a/P term; linear in unit_mbs; with split_backward it also
 * holds the output gradients kept between the two backward tasks) and per-call temporaries. */
uint64_t zpp_stage_workspace_bytes(const zpp_stage *stage);

/* Number of tensors in the flat layout, and the idx-th entry.  `name` points into the handle and
 * stays valid until zpp_stage_destroy.  offset is in elements. */
int32_t zpp_stage_layout_size(const zpp_stage *stage);
zpp_status zpp_stage_param_layout(const zpp_stage *stage, int32_t idx, const char **name,
                                  uint64_t *offset, uint64_t *rows, uint64_t *cols);

/* Binds caller-owned device memory.  P: fp32 master parameters [N]; G: fp32 gradient accumulator
 * [N] (the caller zeroes it before a training step, or uses zpp_adam.zero_grad); M, V: fp32 Adam
 * moments [N]; workspace: at least zpp_stage_workspace_bytes() bytes.  All 256-byte aligned.
 * May be called again to re-bind; resets the state machine. */
zpp_status zpp_stage_bind(zpp_stage *stage, float *P, float *G, float *M, float *V, void *workspace,
                          uint64_t workspace_bytes);

/* ---- the hot path ----------------------------------------------------------------------------
 *
 * State machine (from the task order of Section 3.1.1: forward pass, input/weight gradient
 * computation, optimizer step; and Section 3.2: gather -> U micro-batches -> reduce):
 *   bind -> stage_materialize_params -> stage_forward(mb) once per mb in [0,U), any order
 *        -> stage_backward(mb) only after stage_forward(mb), once
 *        -> stage_accumulate_grads(mb) only after stage_backward(mb), once; because the staging
 *           buffer is reused, stage_backward of another micro-batch before that is ZPP_ERR_STATE
 *           (stage_backward_accumulate(mb) stands for the pair backward + accumulate of one micro-batch;
 *           stage_backward_input(mb) then stage_backward_weight(mb) stand for stage_backward(mb) or,
 *           with in_place, for stage_backward_accumulate(mb); stage_backward_weight_group covers several
 *           micro-batches whose input-gradient tasks have run)
 *        -> shard_adam_step only when no micro-batch is half-done (forward without backward, input
 *           gradient without weight gradient, backward without accumulate)
 *        -> zpp_stage_end_unit, after which the next unit starts with forward (the working copy
 *           stays valid until P changes; after shard_adam_step a new stage_materialize_params is
 *           required, which is cheaper when the step wrote the parameters back).
 */

/* Stand-in for the per-unit parameter all-gather of Section 3.2: produces the working copy of the
 * whole stage from the flat fp32 master shard P (bf16 round-to-nearest-even cast, or a float
 * copy).  Idempotent; may be called again before the backward phase, mirroring the paper's second
 * gather, without changing results.  After an Adam step with write_back the first gather takes the
 * plain copy that step wrote instead of casting P again; a caller who writes P itself between such a
 * step and the gather (a checkpoint load, a re-initialisation) must call zpp_stage_params_changed
 * first.  Every other gather reads P. */
zpp_status stage_materialize_params(zpp_stage *stage, void *hip_stream);

/* Tells the stage that the caller has written P: the working copy is stale and the next
 * stage_materialize_params casts all of it from P.  Host only.  Errors: ZPP_ERR_STATE before bind. */
zpp_status zpp_stage_params_changed(zpp_stage *stage);

/* One micro-batch through all blocks of the stage (the forward task of Section 3.1.1).  Per block:
 * x1 = x + Attn(Norm1(x)); y = x1 + MLP(Norm2(x1)), causal attention, no dropout.  x, y: [T, h]
 * in the activation element type; x is only read during the call's enqueued work, y is written.
 * What backward needs is kept in the unit's activation stash, slot `micro_batch`. */
zpp_status stage_forward(zpp_stage *stage, int32_t micro_batch, const void *x, void *y, void *hip_stream);

/* Input-gradient and weight-gradient tasks of one micro-batch, fused (Sections 2.3 and 3.1.1): for
 * every linear layer dX = dY.W and dW = dY^T.X.  dy: gradient w.r.t. the stage output [T, h];
 * dx: gradient w.r.t. the stage input [T, h] (written).  The micro-batch's weight gradients g_mb
 * are written to the fp32 staging buffer (parameter layout) inside the workspace. */
zpp_status stage_backward(zpp_stage *stage, int32_t micro_batch, const void *dy, void *dx, void *hip_stream);

/* Stand-in for the per-unit gradient reduce-scatter of Section 3.2: G <- G + scale * g_mb over the
 * whole flat shard. */
zpp_status stage_accumulate_grads(zpp_stage *stage, int32_t micro_batch, float scale, void *hip_stream);

/* stage_backward followed by stage_accumulate_grads of the same micro-batch, as one call that never
 * materialises g_mb: every weight-gradient product adds scale * dW into its place in G from the
 * GEMM epilogue, and the bias and gain gradients are added by the reduction that sums them
 * (Section 2.3 for the products, Section 3.2 for the accumulation).  Each element of G receives the same
 * single fused multiply-add G + scale * g as in the two-call sequence, so the results are bit-identical
 * to it; the staging buffer is neither read nor written.  Arguments and errors as stage_backward;
 * afterwards the micro-batch counts as accumulated. */
zpp_status stage_backward_accumulate(zpp_stage *stage, int32_t micro_batch, const void *dy, void *dx,
                                     float scale, void *hip_stream);

/* The backward of a micro-batch as the two separate tasks of Section 3.1.1 (the split of Section 2.3:
 * the input-gradient computation dX = dY.W and the weight-gradient computation dW = dY^T.X), so that a
 * scheduler can run the weight-gradient task later, e.g. where the pipeline would otherwise idle.
 * Needs a stage created with split_backward = 1 (ZPP_ERR_STATE otherwise).
 *   stage_backward_input(mb): after stage_forward(mb), once.  Computes dx exactly as stage_backward
 *     and keeps each linear layer's dY (and the partial sums of the norm-gain reductions, which fall out of
 *     the pass that computes dx) in the unit's stash; dy is copied, so the caller may reuse it at once.
 *     Does not touch the staging buffer or G; input-gradient tasks of other micro-batches may follow
 *     before this one's weight-gradient task.
 *   stage_backward_weight(mb, in_place, scale): after stage_backward_input(mb), once.  Computes the
 *     weight, bias and gain gradients of the micro-batch from the stash.  in_place == 0: into the
 *     staging buffer, to be followed by stage_accumulate_grads(mb) like stage_backward (scale is
 *     ignored); in_place != 0: added into G as scale * g_mb like stage_backward_accumulate.
 * The two tasks launch the same kernels on the same operands as the fused calls: dx and the gradients
 * are bit-identical to theirs.  shard_adam_step and zpp_stage_end_unit refuse to run while a
 * micro-batch has its input gradient but not its weight gradient. */
zpp_status stage_backward_input(zpp_stage *stage, int32_t micro_batch, const void *dy, void *dx, void *hip_stream);
zpp_status stage_backward_weight(zpp_stage *stage, int32_t micro_batch, int32_t in_place, float scale,
                                 void *hip_stream);

/* The weight-gradient tasks of micro-batches [first, first + count) as one: since the gradient of the unit
 * is the sum over its micro-batches (Section 3.2.1 reduces it once per unit), each weight-gradient product
 * runs once over the concatenated tokens, dW += scale * [dY_first; ...]^T . [X_first; ...] with
 * K = count * T, so G is read and written once per group instead of once per micro-batch and the
 * product has a longer K loop.  Always in place (adds into G).  Needs every micro-batch of the group to
 * have had its input-gradient task (the group must cover grouped input-gradient tasks whole) and
 * count <= max(split_backward, group_mbs) of the configuration (ZPP_ERR_STATE otherwise).  The sum over
 * the group's micro-batches is formed inside the product's fp32 accumulation, so G differs from the
 * one-by-one result by summation order only (not bit-identical). */
zpp_status stage_backward_weight_group(zpp_stage *stage, int32_t first, int32_t count, float scale,
                                       void *hip_stream);

/* The micro-batches of a scheduling unit run back to back against one gathered copy of the stage's
 * parameters (Section 3.1, Section 3.1.2); these calls take `count` consecutive micro-batches
 * [first, first + count) of the unit as ONE task: every linear layer runs once over count * T tokens (a
 * larger product that reads the weights once per group instead of once per micro-batch), norms and
 * attention over count * micro_batch samples.  x, y, dy, dx: [count * T, h], micro-batch first + k in
 * rows [k*T, (k+1)*T).  Row by row the arithmetic is that of the one-micro-batch calls: y and dx are
 * bit-identical to theirs; weight, bias and gain gradients of the group are summed inside the products
 * and reductions (same value, another summation order).  count <= max(group_mbs, split_backward) of the
 * configuration (ZPP_ERR_STATE beyond); states and errors per micro-batch as for the one-micro-batch calls.
 *   stage_forward_group              = stage_forward of each micro-batch of the group
 *   stage_backward_input_group       = stage_backward_input of each; a later weight-gradient task
 *                                      (stage_backward_weight or _group) must cover the group whole
 *   stage_backward_accumulate_group  = stage_backward_accumulate of each (both tasks, added into G) */
zpp_status stage_forward_group(zpp_stage *stage, int32_t first, int32_t count, const void *x, void *y,
                               void *hip_stream);
zpp_status stage_backward_input_group(zpp_stage *stage, int32_t first, int32_t count, const void *dy, void *dx,
                                      void *hip_stream);
zpp_status stage_backward_accumulate_group(zpp_stage *stage, int32_t first, int32_t count, const void *dy,
                                           void *dx, float scale, void *hip_stream);

/* The optimizer-step task (Section 3.1.1; Section 3.2.2: each rank updates the parameters whose optimizer
 * states it holds): Adam on elements [offset, offset+count) of P, M, V using G.
 *   ghat = grad_scale*G (+ wd*p in L2 form); m <- b1 m + (1-b1) ghat; v <- b2 v + (1-b2) ghat^2;
 *   p <- p - lr*( (m/(1-b1^t)) / (sqrt(v/(1-b2^t)) + eps) + wd*p_old [decoupled form] ).
 * offset and count must be multiples of 4 elements except that offset+count may equal N.
 * Marks the working copy stale. */
zpp_status shard_adam_step(zpp_stage *stage, uint64_t offset, uint64_t count, const zpp_adam *hp,
                           void *hip_stream);

/* The same update over several ranges of the shard in one launch, each range with its own learning
 * rate and weight decay (the usual "no decay on norm gains, offsets and biases"; ZeRO-1-style
 * sub-ranges of Section 3.2.2 are ranges too).  Everything else (betas, eps, step, grad_scale, the decay
 * form, zero_grad) comes from *hp, whose lr and weight_decay are ignored.  Ranges: ascending, disjoint,
 * offset and count multiples of 4 elements; elements outside every range are left untouched (G included).
 * Errors as shard_adam_step; ZPP_ERR_ARG for overlapping or unordered ranges. */
typedef struct {
    uint64_t offset, count; /* elements */
    float lr, weight_decay;
} zpp_adam_range;
zpp_status shard_adam_step_ranges(zpp_stage *stage, const zpp_adam_range *ranges, int32_t n_ranges,
                                  const zpp_adam *hp, void *hip_stream);

/* Fills `out` (capacity entries) with ranges that cover the whole shard in layout order: matrices with
 * `weight_decay`, one-row tensors (gains, offsets, biases) with 0, all with `lr`; neighbours with equal
 * settings are merged.  Returns the number of ranges the shard needs (call with out = NULL to size the
 * array); host only. */
int32_t zpp_stage_decay_ranges(const zpp_stage *stage, float lr, float weight_decay, zpp_adam_range *out,
                               int32_t capacity);

/* Releases the unit's activation stash slots (a unit gives its memory back before the next unit starts,
 * Section 3.1.2) and resets the per-micro-batch states. */
zpp_status zpp_stage_end_unit(zpp_stage *stage);

/* ---- introspection (tests, benchmarks) ------------------------------------------------------- */

/* Number of times stage_materialize_params ran and bytes it read+wrote, since create. */
void zpp_stage_counters(const zpp_stage *stage, uint64_t *materialize_calls, uint64_t *materialize_bytes);

/* Device address and size of a named region inside the bound workspace:
 *   "W" working copy, "Wt" the transposed copies (may be empty), "S" staging gradients; stash tensors of (micro_batch, block) by name, e.g.
 *   "x", "n1", "qkv", "attn", "lse", "x1", "n2", "u", "g".  elem_bytes is 2 or 4.  ("u", the slot of the first MLP
 *   product: its pre-activation in fp32 stages and with selective recomputation, else the derivative of the
 *   activation at it, which is all the backward pass needs of it.)
 * Errors: ZPP_ERR_STATE before bind, ZPP_ERR_ARG for an unknown name or index. */
zpp_status zpp_stage_region(const zpp_stage *stage, const char *name, int32_t micro_batch, int32_t block,
                            void **ptr, uint64_t *elems, int32_t *elem_bytes);

/* Optional timing of the kernels the stage calls launch, by class, with HIP events recorded on the
 * caller's stream around each launch (process-wide switch; off by default; adds two event records
 * per launch).  zpp_profile_read waits for the recorded events and returns, for one class, the
 * number of bracketed launches, their summed duration and their summed algorithmic work (flops for
 * GEMM and attention with the causal convention 2*b*s^2*h forward and twice that backward; bytes
 * for the flat passes: 12 per element accumulate, 28 (+4 with zero_grad) Adam, read+write bytes
 * materialise; 0 for the rest), and for GEMMs also the minimum HBM bytes (each operand read once, the
 * result written once; a product accumulated in place also reads its result once). */
enum {
    ZPP_PROF_GEMM = 0, ZPP_PROF_ATTN_FWD = 1, ZPP_PROF_ATTN_BWD = 2, ZPP_PROF_ACCUMULATE = 3,
    ZPP_PROF_ADAM = 4, ZPP_PROF_MATERIALIZE = 5, ZPP_PROF_OTHER = 6,
    ZPP_PROF_GEMM_DW = 7, /* the weight-gradient products dY^T.X (fp32 output, written or accumulated in place);
                             ZPP_PROF_GEMM holds the forward and input-gradient products */
    ZPP_PROF_CLASSES = 8
};
zpp_status zpp_profile_enable(int32_t on);
void zpp_profile_reset(void);
zpp_status zpp_profile_read(int32_t cls, uint64_t *launches, double *total_ms, double *work, double *bytes);

const char *zpp_last_error(void);
const char *zpp_version(void);

#ifdef __cplusplus
}
#endif
#endif /* ZPP_H */
