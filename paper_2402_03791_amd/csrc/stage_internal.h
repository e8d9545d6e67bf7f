// Library-internal interface between the stage runtime (stage.cpp) and the per-device scheduler
// (device.cpp): placing a stage's three workspace parts at chosen offsets of a shared allocation, and the
// bookkeeping of which stage's working copy a shared slot holds.
#pragma once
#include "../../include/zpp.h"

namespace zpp {

struct StageParts {
    uint64_t wcopy;    // working copy of the stage's parameters (+ transposed copy, rotary table)
    uint64_t scratch;  // fp32 staging gradients and per-call temporaries
    uint64_t stash;    // activation stash of one scheduling unit
};
StageParts stage_parts(const zpp_stage *s);

// As zpp_stage_bind, with the three parts at byte offsets of `base` (each 256-byte aligned).  Stages that
// are never inside a call at the same time may share a scratch part; stages may share a working-copy
// part if stage_drop_working_copy is called on the loser whenever another one materialises into it.
zpp_status stage_bind_parts(zpp_stage *s, float *P, float *G, float *M, float *V, void *base, uint64_t wcopy_off,
                            uint64_t scratch_off, uint64_t stash_off);
void stage_drop_working_copy(zpp_stage *s);
bool stage_has_working_copy(const zpp_stage *s);

// Records the message zpp_last_error() returns and hands back `st`.
zpp_status set_error(zpp_status st, const char *fmt, ...);

}  // namespace zpp
