// What the opaque lcsa_cache handle of include/lcsa.h points to (host memory).  Internal: only the host layer
// of the library and the benchmark's measurement aids, which launch instrumented copies of the kernels on a
// cache the library manages, include this.
#pragma once
#include "../../include/lcsa.h"
#include "lcsa_kernels.h"

struct lcsa_cache {
    lcsa_geom geom;
    lcsa::KGeom kg;
    lcsa::KCache kc;
    size_t bytes;
    int start;             // sliding window: ring slot of the oldest visible group as enqueued so far (host mirror of
                           // the device words in kc.ring; replays of a captured append do not move it)
    int32_t policy;        // LCSA_EVICT_*
    int32_t *order;        // device [heads][cap]: visible group -> slot (importance-based policies)
    float *importance;     // device [heads][cap]: importance of the visible groups, from lcsa_block_importance
    float *row_group;      // device [heads][n_qb][cap]: scratch of lcsa_block_importance
    bool scored;           // `importance` was computed since the last append (the scores are used once)
};

