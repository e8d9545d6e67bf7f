/*
 * zpp_device.h — several stages of one pipeline on one device.
 *
 * The schedule of Section 3.1 maps a multiple of the pipeline degree of stages onto the devices with a
 * looping placement, so a device holds V stages; inside a scheduling unit it runs them breadth-first:
 * all U micro-batches of one stage back to back, then the next stage (Section 3.1.1, Section 3.1.2),
 * and a stage's parameters are gathered only while it computes.  This header is that per-device
 * picture on one GPU: V stages of identical configuration share
 *   - one or two working-copy slots (one gathered stage each: the L*M_w/(P*V) term of the weight
 *     memory in Section 4.2; two slots when the next stage's gather is prefetched),
 *   - one scratch part (fp32 staging gradients, per-call temporaries),
 * and each owns the activation stash of its U micro-batches until its backward phase has run.
 * With `prefetch` the gather (stage_materialize_params) of the stage that computes next is enqueued on a
 * second stream while the current stage computes; the communication of this schedule overlaps with
 * computation easily (Section 4.1), and this is its one-GPU stand-in.  The library creates HIP events
 * (no device memory, no streams) to order the two streams.
 *
 * All device memory is the caller's: P, G, M, V hold V * N fp32 elements, stage v at
 * [v*N, (v+1)*N) with the flat layout of zpp.h; one workspace of zpp_device_workspace_bytes().
 * Pointers 256-byte aligned.  Errors and zpp_last_error() as in zpp.h.  Not thread-safe.
 */
#ifndef ZPP_DEVICE_H
#define ZPP_DEVICE_H

#include "zpp.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct zpp_device zpp_device; /* opaque; host-side metadata and HIP events only */

/* n_stages stages, each of configuration *cfg (unit_mbs = U micro-batches per unit).  prefetch != 0: two
 * working-copy slots and gathers on the side stream.  Errors: as zpp_stage_create; ZPP_ERR_ARG for
 * n_stages < 1. */
zpp_status zpp_device_create(const zpp_stage_config *cfg, int32_t n_stages, int32_t prefetch, zpp_device **out);
/* The same with a recomputation mode per stage (recompute[v] = ZPP_RECOMPUTE_*, overriding cfg->recompute;
 * NULL: cfg's for all).  Section 3.3 recomputes every stage mapped to a device except the last one: a stage
 * whose input- and weight-gradient tasks run back to back needs one recomputation for both, the last
 * stage's tasks are scheduled apart and it keeps its activations.  So a stage that recomputes runs the fused
 * backward call per micro-batch whatever cfg->split_backward says, and only the other stages split their
 * backward tasks; the stashes are sized stage by stage. */
zpp_status zpp_device_create_per_stage(const zpp_stage_config *cfg, int32_t n_stages, int32_t prefetch,
                                       const int32_t *recompute, zpp_device **out);
void zpp_device_destroy(zpp_device *dev);

int32_t zpp_device_stage_count(const zpp_device *dev);
/* V * N: elements of each of P, G, M, V. */
uint64_t zpp_device_param_count(const zpp_device *dev);
uint64_t zpp_device_workspace_bytes(const zpp_device *dev);
/* The three terms of the workspace in bytes: working-copy slots (1 or 2 gathered stages), scratch,
 * activation stashes of all V stages (the unit's min(B,U)*L*M_a/P term of Section 4.2). */
zpp_status zpp_device_memory_terms(const zpp_device *dev, uint64_t *working_copies, uint64_t *scratch,
                                   uint64_t *stash);
/* Borrowed handle of stage v for the host-side queries of zpp.h (layout, regions, counters); the hot-path
 * calls of zpp.h must not be mixed with the unit calls below on the same handle. */
zpp_stage *zpp_device_stage(zpp_device *dev, int32_t v);

zpp_status zpp_device_bind(zpp_device *dev, float *P, float *G, float *M, float *V, void *workspace,
                           uint64_t workspace_bytes);

/* Forward phase of one scheduling unit: for v = 0 .. V-1: gather stage v, then stage_forward of its U
 * micro-batches.  x, y: host arrays of V*U device pointers; entry v*U + m is the [T, h] input / output
 * of stage v for micro-batch m.  The caller wires the stages: on one GPU alone y of stage v is x of
 * stage v+1 (pass the same pointer); in a pipeline they come from and go to other ranks.
 * stream: the compute stream.  side_stream: where prefetched gathers run (ignored without prefetch;
 * NULL: gather on the compute stream). */
zpp_status device_forward_unit(zpp_device *dev, const void *const *x, void *const *y, void *stream,
                               void *side_stream);

/* Backward phase of the unit: for v = V-1 .. 0: gather stage v again unless its working copy is still in
 * a slot (the second gather of Section 3.2.1), then stage_backward_accumulate(scale) of its U
 * micro-batches; or, for a stage with split_backward = g > 0 that does not recompute, the stage's U
 * input-gradient tasks followed by its weight-gradient tasks in groups of g micro-batches
 * (stage_backward_weight_group).  dy, dx: as x, y. */
zpp_status device_backward_unit(zpp_device *dev, const void *const *dy, void *const *dx, float scale,
                                void *stream, void *side_stream);

/* shard_adam_step over every stage's whole shard. */
zpp_status device_adam_step(zpp_device *dev, const zpp_adam *hp, void *stream);

/* zpp_stage_end_unit for every stage: the stashes are free for the next unit. */
zpp_status zpp_device_end_unit(zpp_device *dev);

#ifdef __cplusplus
}
#endif
#endif /* ZPP_DEVICE_H */
