// Launch-free argument checks shared between the library's translation units, so
// that an entry point made of several launches (the two-stream runtime) can
// validate everything before it enqueues anything.  Not part of the C ABI.
#pragma once

#include <cstdint>

#include "pipesgd.h"

#define PIPESGD_HIDDEN __attribute__((visibility("hidden")))

// What pipesgd_allreduce_sim(ring, schedule, ..) would return without launching.
PIPESGD_HIDDEN int pipesgd_internal_check_allreduce(const pipesgd_ring *ring, int schedule);

// What pipesgd_apply_update_multi(..) would return without launching.
PIPESGD_HIDDEN int pipesgd_internal_check_update(int mode, int replicas, const void *const *g_sum_c,
                                                 const float *const *scales, uint64_t n, float *const *w,
                                                 float *const *v, float momentum);

// What pipesgd_synthetic_compute(..) would return without launching.
PIPESGD_HIDDEN int pipesgd_internal_check_standin(float duration_us, int workgroups);
