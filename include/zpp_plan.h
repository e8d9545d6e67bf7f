/*
 * zpp_plan.h — the closed-form cost model of Section 4 as host functions, and a small planner that
 * picks the scheduling-unit size U and the number of stages per device V under a memory limit.
 * Pure host arithmetic: no device, no allocation.  Symbols as in the paper's table of symbols.
 */
#ifndef ZPP_PLAN_H
#define ZPP_PLAN_H

#include "zpp.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct {
    int64_t L;  /* transformer layers of the whole model */
    int64_t h;  /* hidden size */
    int64_t s;  /* sequence length */
    int64_t b;  /* micro-batch size (samples) */
    int64_t B;  /* micro-batches on a single GPU per iteration */
    int64_t P;  /* pipeline-parallel size */
    int64_t D;  /* data-parallel size (the ZeRO-3 group) */
    double Mw;  /* weight memory of one transformer layer, any unit */
    double Ma;  /* activation memory of one transformer layer for one micro-batch, same unit */
} zpp_plan_model;

/* Section 4.1, per transformer block and iteration, in elements:
 *   tensor parallelism: four all-reduces in forward and backward, 8*B*b*s*h;
 *   ZeroPP: B/U units, each two all-gathers and one reduce-scatter of ~12h^2 parameters, 36*B*h^2/U.
 * zpp_plan_zeropp_wins: the paper's condition 2*s*U*b > 9*h under which the second is smaller. */
double zpp_plan_tp_comm(const zpp_plan_model *m);
double zpp_plan_zeropp_comm(const zpp_plan_model *m, int64_t U);
int32_t zpp_plan_zeropp_wins(const zpp_plan_model *m, int64_t U);

/* Section 4.2: pipeline bubbles of a unit of U micro-batches: 0 when U >= 2P-1 (enough active
 * micro-batches for the near-zero-bubble schedule), else B*(2P-1-U)/U. */
double zpp_plan_bubbles(const zpp_plan_model *m, int64_t U);

/* Section 4.2: maximum allocated memory = L*Mw/(P*D) + L*Mw/(P*V) + min(B,U)*L*Ma/P, and its three
 * terms (any of the pointers may be NULL): the partitioned weights, the one gathered stage, the
 * activations of one scheduling unit. */
double zpp_plan_max_memory(const zpp_plan_model *m, int64_t U, int64_t V, double *weights_partitioned,
                           double *weights_gathered, double *activations);

/* The rows of the paper's comparison of pipeline methods (Section 4.2): bubble ratio, weight memory and
 * activation memory as printed there ("near zero" is returned as 0).  V is used by the interleaved and
 * ZeroPP rows.  ZPP_ERR_ARG for an unknown method or non-positive sizes. */
enum { ZPP_PP_GPIPE = 0, ZPP_PP_1F1B = 1, ZPP_PP_INTERLEAVED_1F1B = 2, ZPP_PP_ZEROPP = 3, ZPP_PP_ZEROPP_RECOMPUTE = 4 };
zpp_status zpp_plan_pp_method(const zpp_plan_model *m, int32_t method, int64_t V, double *bubble_ratio,
                              double *weight_memory, double *activation_memory);

/* Planner: among U in the divisors of B and V in the divisors of L/P (whole layers per stage) whose
 * zpp_plan_max_memory is within memory_limit, the choice with the fewest bubbles, then the smallest
 * communication volume (the largest U), then the smallest memory (the largest V), then the smallest V.
 * ZPP_ERR_UNSUPPORTED if nothing fits, ZPP_ERR_ARG for sizes that are not positive or L not a multiple
 * of P. */
typedef struct {
    int64_t U, V;
    double memory, comm, bubbles;
} zpp_plan_choice;
zpp_status zpp_plan_choose(const zpp_plan_model *m, double memory_limit, zpp_plan_choice *out);

#ifdef __cplusplus
}
#endif
#endif /* ZPP_PLAN_H */
