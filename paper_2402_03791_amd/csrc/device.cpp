// Several stages of one pipeline on one device (include/zpp_device.h): the per-device side of the
// paper's schedule.  A device holds V stages (looping placement, Section 3.1); inside a scheduling unit it
// runs the stages breadth-first - all U micro-batches of a stage back to back, then the next stage
// (Section 3.1.2) - and only the stage that computes (plus, with prefetch, the one that comes next) has its
// parameters gathered: the working copy is a slot that the stages take turns in, which is the
// L*M_w/(P*V) term of the weight memory in Section 4.2.  The gather of the next stage runs on a second
// stream while the current stage computes (the one-GPU stand-in for overlapping the all-gather).
// Host code only: every kernel is launched through the stage calls of stage.cpp.
#include "../../include/zpp_device.h"
#include "stage_internal.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <vector>

using namespace zpp;

struct zpp_device {
    zpp_stage_config cfg;
    int V = 0, U = 0, slots = 1;
    std::vector<zpp_stage *> st;
    uint64_t N = 0;
    StageParts parts{};
    uint64_t slot_off[2] = {0, 0}, scratch_off = 0, ws_bytes = 0;
    std::vector<uint64_t> stash_off, stash_bytes;
    std::vector<int> split;  // per stage: its split_backward (0: the fused backward call per micro-batch)
    bool bound = false;
    // working-copy slots: which stage's parameters a slot holds, and the two events that order its reuse
    int owner[2] = {-1, -1};
    hipEvent_t ready[2] = {nullptr, nullptr};  // recorded on the gathering stream when the copy is complete
    hipEvent_t freed[2] = {nullptr, nullptr};  // recorded on the compute stream after the slot's last reader
    bool ready_pending[2] = {false, false}, freed_valid[2] = {false, false};
    hipEvent_t unit_start = nullptr;           // compute-stream position at which P is final for this phase
};

namespace {

constexpr uint64_t kAlign = 256;
inline uint64_t align_up(uint64_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

zpp_status check(const zpp_device *d, bool need_bound)
{
    if (!d) return set_error(ZPP_ERR_ARG, "device is NULL");
    if (need_bound && !d->bound) return set_error(ZPP_ERR_STATE, "device has no bound memory (call zpp_device_bind)");
    return ZPP_OK;
}

#define DEV_HIP(expr)                                                                                      \
    do {                                                                                                   \
        hipError_t _e = (expr);                                                                            \
        if (_e != hipSuccess) return set_error(ZPP_ERR_DEVICE, "%s failed: %s", #expr, hipGetErrorString(_e)); \
    } while (0)

// Makes sure stage v's working copy is, or is being, written into its slot.  With a side stream the
// gather is enqueued there, after the slot's previous reader and after `unit_start`.
zpp_status gather(zpp_device *d, int v, hipStream_t main, hipStream_t side)
{
    const int slot = v % d->slots;
    if (d->owner[slot] == v && stage_has_working_copy(d->st[v])) return ZPP_OK;
    if (d->owner[slot] >= 0 && d->owner[slot] != v) stage_drop_working_copy(d->st[d->owner[slot]]);
    hipStream_t s = side ? side : main;
    if (side) {
        DEV_HIP(hipStreamWaitEvent(side, d->unit_start, 0));
        if (d->freed_valid[slot]) DEV_HIP(hipStreamWaitEvent(side, d->freed[slot], 0));
    }
    if (zpp_status e = stage_materialize_params(d->st[v], s)) return e;
    if (side) {
        DEV_HIP(hipEventRecord(d->ready[slot], side));
        d->ready_pending[slot] = true;
    }
    d->owner[slot] = v;
    return ZPP_OK;
}

// The compute stream may read stage v's working copy from here on.
zpp_status acquire(zpp_device *d, int v, hipStream_t main)
{
    const int slot = v % d->slots;
    if (d->ready_pending[slot]) {
        DEV_HIP(hipStreamWaitEvent(main, d->ready[slot], 0));
        d->ready_pending[slot] = false;
    }
    return ZPP_OK;
}

// The compute stream is done with stage v's working copy (for this phase).
zpp_status release(zpp_device *d, int v, hipStream_t main)
{
    const int slot = v % d->slots;
    DEV_HIP(hipEventRecord(d->freed[slot], main));
    d->freed_valid[slot] = true;
    return ZPP_OK;
}

// The events are created at the first phase (creating a handle touches no device).
zpp_status ensure_events(zpp_device *d)
{
    if (d->unit_start) return ZPP_OK;
    for (int i = 0; i < 2; ++i) {
        DEV_HIP(hipEventCreateWithFlags(&d->ready[i], hipEventDisableTiming));
        DEV_HIP(hipEventCreateWithFlags(&d->freed[i], hipEventDisableTiming));
    }
    DEV_HIP(hipEventCreateWithFlags(&d->unit_start, hipEventDisableTiming));
    return ZPP_OK;
}

// One phase of a unit: the stages in ascending or descending order, each with its U micro-batches back
// to back.
template <class PerMicroBatch, class PerStage>
zpp_status run_phase(zpp_device *d, bool descending, hipStream_t main, hipStream_t side, PerMicroBatch &&body,
                     PerStage &&after_stage)
{
    if (d->slots < 2) side = nullptr;
    if (zpp_status e = ensure_events(d)) return e;
    DEV_HIP(hipEventRecord(d->unit_start, main));
    const int first = descending ? d->V - 1 : 0, step = descending ? -1 : 1;
    if (zpp_status e = gather(d, first, main, side)) return e;
    for (int i = 0, v = first; i < d->V; ++i, v += step) {
        const int next = v + step;
        // with two slots the next stage's gather overlaps this stage's micro-batches
        if (d->slots == 2 && i + 1 < d->V)
            if (zpp_status e = gather(d, next, main, side)) return e;
        if (zpp_status e = acquire(d, v, main)) return e;
        for (int m = 0; m < d->U; ++m)
            if (zpp_status e = body(v, m)) return e;
        if (zpp_status e = after_stage(v)) return e;
        if (zpp_status e = release(d, v, main)) return e;
        if (d->slots == 1 && i + 1 < d->V)
            if (zpp_status e = gather(d, next, main, side)) return e;
    }
    return ZPP_OK;
}

}  // namespace

extern "C" {

zpp_status zpp_device_create_per_stage(const zpp_stage_config *cfg, int32_t n_stages, int32_t prefetch,
                                       const int32_t *recompute, zpp_device **out)
{
    if (!cfg || !out) return set_error(ZPP_ERR_ARG, "cfg/out is NULL");
    if (n_stages < 1 || n_stages > 4096) return set_error(ZPP_ERR_ARG, "n_stages must be in [1, 4096]");
    zpp_device *d = new (std::nothrow) zpp_device();
    if (!d) return set_error(ZPP_ERR_ARG, "out of host memory");
    d->cfg = *cfg;
    d->V = n_stages;
    d->U = cfg->unit_mbs;
    d->slots = (prefetch && n_stages > 1) ? 2 : 1;
    uint64_t scratch = 0;
    for (int v = 0; v < n_stages; ++v) {
        zpp_stage_config c = *cfg;
        if (recompute) c.recompute = recompute[v];
        // a stage that recomputes runs its two gradient tasks back to back so that one recomputation
        // serves both (Section 3.3); its stash needs no room for what the tasks hand to each other
        if (c.recompute != ZPP_RECOMPUTE_NONE) {
            c.group_mbs = std::max(c.group_mbs, c.split_backward);
            c.split_backward = 0;
        }
        zpp_stage *s = nullptr;
        if (zpp_status e = zpp_stage_create(&c, &s)) {
            zpp_device_destroy(d);
            return e;
        }
        d->st.push_back(s);
        d->split.push_back(c.split_backward);
        const StageParts p = stage_parts(s);
        if (v == 0) d->parts = p;
        scratch = std::max(scratch, p.scratch);
        d->stash_bytes.push_back(p.stash);
    }
    d->N = zpp_stage_param_count(d->st[0]);
    d->parts.scratch = scratch;
    uint64_t cur = 0;
    for (int i = 0; i < d->slots; ++i) {
        d->slot_off[i] = cur;
        cur = align_up(cur + d->parts.wcopy);
    }
    d->scratch_off = cur;
    cur = align_up(cur + d->parts.scratch);
    for (int v = 0; v < n_stages; ++v) {
        d->stash_off.push_back(cur);
        cur = align_up(cur + d->stash_bytes[v]);
    }
    d->ws_bytes = cur;
    *out = d;
    return ZPP_OK;
}

zpp_status zpp_device_create(const zpp_stage_config *cfg, int32_t n_stages, int32_t prefetch, zpp_device **out)
{
    return zpp_device_create_per_stage(cfg, n_stages, prefetch, nullptr, out);
}

void zpp_device_destroy(zpp_device *d)
{
    if (!d) return;
    for (zpp_stage *s : d->st) zpp_stage_destroy(s);
    for (int i = 0; i < 2; ++i) {
        if (d->ready[i]) (void)hipEventDestroy(d->ready[i]);
        if (d->freed[i]) (void)hipEventDestroy(d->freed[i]);
    }
    if (d->unit_start) (void)hipEventDestroy(d->unit_start);
    delete d;
}

int32_t zpp_device_stage_count(const zpp_device *d) { return d ? d->V : 0; }
uint64_t zpp_device_param_count(const zpp_device *d) { return d ? d->N * (uint64_t)d->V : 0; }
uint64_t zpp_device_workspace_bytes(const zpp_device *d) { return d ? d->ws_bytes : 0; }

zpp_status zpp_device_memory_terms(const zpp_device *d, uint64_t *working_copies, uint64_t *scratch, uint64_t *stash)
{
    if (zpp_status e = check(d, false)) return e;
    if (working_copies) *working_copies = d->scratch_off;  // the slots lie in front of the scratch part
    if (scratch) *scratch = d->stash_off[0] - d->scratch_off;
    if (stash) *stash = d->ws_bytes - d->stash_off[0];
    return ZPP_OK;
}

zpp_stage *zpp_device_stage(zpp_device *d, int32_t v)
{
    if (!d || v < 0 || v >= d->V) {
        set_error(ZPP_ERR_ARG, "stage index out of range");
        return nullptr;
    }
    return d->st[v];
}

zpp_status zpp_device_bind(zpp_device *d, float *P, float *G, float *M, float *V, void *workspace,
                           uint64_t workspace_bytes)
{
    if (zpp_status e = check(d, false)) return e;
    if (!P || !G || !M || !V || !workspace) return set_error(ZPP_ERR_ARG, "P, G, M, V and workspace must be non-NULL");
    if (workspace_bytes < d->ws_bytes)
        return set_error(ZPP_ERR_WORKSPACE, "workspace has %llu bytes, %llu needed", (unsigned long long)workspace_bytes,
                         (unsigned long long)d->ws_bytes);
    if ((d->N * 4) % kAlign && d->V > 1)
        return set_error(ZPP_ERR_ALIGN, "a stage's parameter count must be a multiple of 64 for stages to lie back to back");
    for (int v = 0; v < d->V; ++v) {
        const uint64_t o = (uint64_t)v * d->N;
        if (zpp_status e = stage_bind_parts(d->st[v], P + o, G + o, M + o, V + o, workspace, d->slot_off[v % d->slots],
                                            d->scratch_off, d->stash_off[v]))
            return e;
    }
    d->owner[0] = d->owner[1] = -1;
    d->ready_pending[0] = d->ready_pending[1] = false;
    d->freed_valid[0] = d->freed_valid[1] = false;
    d->bound = true;
    return ZPP_OK;
}

zpp_status device_forward_unit(zpp_device *d, const void *const *x, void *const *y, void *stream, void *side_stream)
{
    if (zpp_status e = check(d, true)) return e;
    if (!x || !y) return set_error(ZPP_ERR_ARG, "x/y is NULL");
    return run_phase(
        d, false, (hipStream_t)stream, (hipStream_t)side_stream,
        [&](int v, int m) {
            return stage_forward(d->st[v], m, x[(size_t)v * d->U + m], y[(size_t)v * d->U + m], stream);
        },
        [](int) { return ZPP_OK; });
}

zpp_status device_backward_unit(zpp_device *d, const void *const *dy, void *const *dx, float scale, void *stream,
                                void *side_stream)
{
    if (zpp_status e = check(d, true)) return e;
    if (!dy || !dx) return set_error(ZPP_ERR_ARG, "dy/dx is NULL");
    // A stage with split_backward = g: its input-gradient tasks first, then its weight-gradient tasks in groups
    // of g micro-batches; a stage without (and every stage that recomputes): the fused call per micro-batch.
    return run_phase(
        d, true, (hipStream_t)stream, (hipStream_t)side_stream,
        [&](int v, int m) {
            const void *dyp = dy[(size_t)v * d->U + m];
            void *dxp = dx[(size_t)v * d->U + m];
            return d->split[v] > 0 ? stage_backward_input(d->st[v], m, dyp, dxp, stream)
                                   : stage_backward_accumulate(d->st[v], m, dyp, dxp, scale, stream);
        },
        [&](int v) -> zpp_status {
            const int g = d->split[v];
            if (g <= 0) return ZPP_OK;
            for (int first = 0; first < d->U; first += g)
                if (zpp_status e = stage_backward_weight_group(d->st[v], first, std::min(g, d->U - first), scale, stream))
                    return e;
            return ZPP_OK;
        });
}

zpp_status device_adam_step(zpp_device *d, const zpp_adam *hp, void *stream)
{
    if (zpp_status e = check(d, true)) return e;
    for (int v = 0; v < d->V; ++v)
        if (zpp_status e = shard_adam_step(d->st[v], 0, d->N, hp, stream)) return e;
    return ZPP_OK;
}

zpp_status zpp_device_end_unit(zpp_device *d)
{
    if (zpp_status e = check(d, true)) return e;
    for (int v = 0; v < d->V; ++v)
        if (zpp_status e = zpp_stage_end_unit(d->st[v])) return e;
    return ZPP_OK;
}

}  // extern "C"
