// The cost model of Section 4 (include/zpp_plan.h): communication volume against tensor parallelism,
// pipeline bubbles, maximum allocated memory, the comparison table of pipeline methods, and a planner
// for U and V.  Host arithmetic only.
#include "../../include/zpp_plan.h"
#include "stage_internal.h"

#include <algorithm>
#include <vector>

using namespace zpp;

namespace {

bool valid(const zpp_plan_model *m)
{
    return m && m->L > 0 && m->h > 0 && m->s > 0 && m->b > 0 && m->B > 0 && m->P > 0 && m->D > 0 && m->Mw >= 0 &&
           m->Ma >= 0;
}

std::vector<int64_t> divisors(int64_t n)
{
    std::vector<int64_t> d;
    for (int64_t i = 1; i <= n; ++i)
        if (n % i == 0) d.push_back(i);
    return d;
}

}  // namespace

extern "C" {

double zpp_plan_tp_comm(const zpp_plan_model *m)
{
    return valid(m) ? 8.0 * (double)m->B * (double)m->b * (double)m->s * (double)m->h : 0.0;
}

double zpp_plan_zeropp_comm(const zpp_plan_model *m, int64_t U)
{
    // B/U units, each moving three times the ~12 h^2 parameters of a block
    return (valid(m) && U > 0) ? 3.0 * 12.0 * (double)m->h * (double)m->h * (double)m->B / (double)U : 0.0;
}

int32_t zpp_plan_zeropp_wins(const zpp_plan_model *m, int64_t U)
{
    return (valid(m) && U > 0) ? (2 * m->s * U * m->b > 9 * m->h) : 0;
}

double zpp_plan_bubbles(const zpp_plan_model *m, int64_t U)
{
    if (!valid(m) || U <= 0) return 0.0;
    const int64_t need = 2 * m->P - 1;
    return U >= need ? 0.0 : (double)m->B * (double)(need - U) / (double)U;
}

double zpp_plan_max_memory(const zpp_plan_model *m, int64_t U, int64_t V, double *weights_partitioned,
                           double *weights_gathered, double *activations)
{
    if (!valid(m) || U <= 0 || V <= 0) return 0.0;
    const double part = (double)m->L * m->Mw / ((double)m->P * (double)m->D);
    const double gath = (double)m->L * m->Mw / ((double)m->P * (double)V);
    const double act = (double)std::min(m->B, U) * (double)m->L * m->Ma / (double)m->P;
    if (weights_partitioned) *weights_partitioned = part;
    if (weights_gathered) *weights_gathered = gath;
    if (activations) *activations = act;
    return part + gath + act;
}

zpp_status zpp_plan_pp_method(const zpp_plan_model *m, int32_t method, int64_t V, double *bubble_ratio,
                              double *weight_memory, double *activation_memory)
{
    if (!valid(m) || V <= 0) return set_error(ZPP_ERR_ARG, "sizes must be positive");
    const double L = (double)m->L, P = (double)m->P, D = (double)m->D, B = (double)m->B, v = (double)V;
    double bub, w, a;
    switch (method) {
    case ZPP_PP_GPIPE:
        bub = (P - 1) / B;
        w = L * m->Mw / P;
        a = B * L * m->Ma / P;
        break;
    case ZPP_PP_1F1B:
        bub = (P - 1) / B;
        w = L * m->Mw / P;
        a = L * m->Ma;
        break;
    case ZPP_PP_INTERLEAVED_1F1B:
        bub = (P - 1) / (v * B);
        w = L * m->Mw / P;
        a = L * m->Ma * (1 + (P - 1) / (v * P));
        break;
    case ZPP_PP_ZEROPP:
        bub = 0;
        w = L * m->Mw * (1 / (P * D) + 1 / (P * v));
        a = L * m->Ma * (2 - 1 / P);
        break;
    case ZPP_PP_ZEROPP_RECOMPUTE:
        bub = 0;
        w = L * m->Mw * (1 / (P * D) + 1 / (P * v));
        a = L * m->Ma * (2 / v - 1 / (v * P));
        break;
    default:
        return set_error(ZPP_ERR_ARG, "unknown pipeline method %d", method);
    }
    if (bubble_ratio) *bubble_ratio = bub;
    if (weight_memory) *weight_memory = w;
    if (activation_memory) *activation_memory = a;
    return ZPP_OK;
}

zpp_status zpp_plan_choose(const zpp_plan_model *m, double memory_limit, zpp_plan_choice *out)
{
    if (!valid(m) || !out) return set_error(ZPP_ERR_ARG, "model sizes must be positive and out non-NULL");
    if (m->L % m->P) return set_error(ZPP_ERR_ARG, "L (%lld) is not a multiple of P (%lld)", (long long)m->L, (long long)m->P);
    bool found = false;
    zpp_plan_choice best{};
    for (int64_t U : divisors(m->B))
        for (int64_t V : divisors(m->L / m->P)) {
            zpp_plan_choice c{U, V, zpp_plan_max_memory(m, U, V, nullptr, nullptr, nullptr), zpp_plan_zeropp_comm(m, U),
                              zpp_plan_bubbles(m, U)};
            if (c.memory > memory_limit) continue;
            const bool better = !found || c.bubbles < best.bubbles ||
                                (c.bubbles == best.bubbles &&
                                 (c.comm < best.comm ||
                                  (c.comm == best.comm &&
                                   (c.memory < best.memory || (c.memory == best.memory && c.V < best.V)))));
            if (better) {
                best = c;
                found = true;
            }
        }
    if (!found)
        return set_error(ZPP_ERR_UNSUPPORTED, "no (U, V) keeps the maximum allocation within %.3g", memory_limit);
    *out = best;
    return ZPP_OK;
}

}  // extern "C"
