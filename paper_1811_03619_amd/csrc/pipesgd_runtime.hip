// The per-worker runtime of Algorithm 1 (arXiv 1811.03619) on one GPU: the
// paper's compute thread and communication thread become two HIP streams, its
// "ready" flags become HIP events.  Built on the library's public entry points
// (and their launch-free argument checks); the one kernel here is the stand-in
// for forward + backward.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <new>
#include <vector>

#include "pipesgd.h"
#include "pipesgd_internal.hpp"

namespace {

// Stand-in for "load a batch, forward pass, backward pass" (Alg. 1, compute
// thread lines 6-8): occupies `gridDim.x` workgroups for a given time and
// touches no memory.  The clock is the constant-rate 100 MHz counter.  Every
// wave leaves the loop: the counter only moves forward, and a hard cap on the
// number of polls bounds the wait even if it did not.
__global__ __launch_bounds__(64) void synthetic_compute_kernel(uint64_t ticks, unsigned *sink)
{
    const uint64_t t0 = wall_clock64();
    uint32_t polls = 0;
    while (wall_clock64() - t0 < ticks && polls < (1u << 24)) {
        __builtin_amdgcn_s_sleep(32);
        ++polls;
    }
    if (sink && ticks == ~0ull) *sink = polls;      // never true in practice; keeps the loop observable
}

constexpr int kEventRing = 8;
constexpr size_t kMaxTimed = 1u << 16;     // timed update launches kept until they are read out

}  // namespace

struct pipesgd_runtime {
    hipStream_t compute = nullptr;     // Alg. 1 "computation thread"
    hipStream_t comm = nullptr;        // Alg. 1 "communication thread"
    hipEvent_t local_ready[kEventRing];   // g_local[t] is ready   (compute -> comm)
    hipEvent_t sum_ready[kEventRing];     // g_sum[t] is ready     (comm -> compute)
    uint64_t t = 0;                    // iterations enqueued so far
    bool ok = false;
    // PIPESGD_RT_TIME_UPDATE: one (start, stop) pair of timing events per timed update launch,
    // reused after pipesgd_runtime_update_time has read them
    std::vector<hipEvent_t> timing;
    size_t timed = 0;                  // pairs recorded since the last read-out
};

extern "C" {

int pipesgd_runtime_create(pipesgd_runtime **out)
{
    if (!out) return PIPESGD_ERR_ARG;
    pipesgd_runtime *rt = new (std::nothrow) pipesgd_runtime();
    if (!rt) return PIPESGD_ERR_CAPACITY;
    bool good = hipStreamCreateWithFlags(&rt->compute, hipStreamNonBlocking) == hipSuccess &&
                hipStreamCreateWithFlags(&rt->comm, hipStreamNonBlocking) == hipSuccess;   // default priority
    for (int i = 0; i < kEventRing; ++i) { rt->local_ready[i] = nullptr; rt->sum_ready[i] = nullptr; }
    for (int i = 0; good && i < kEventRing; ++i)
        good = hipEventCreateWithFlags(&rt->local_ready[i], hipEventDisableTiming) == hipSuccess &&
               hipEventCreateWithFlags(&rt->sum_ready[i], hipEventDisableTiming) == hipSuccess;
    rt->ok = good;
    if (!good) { pipesgd_runtime_destroy(rt); return PIPESGD_ERR_HIP; }
    *out = rt;
    return PIPESGD_OK;
}

void pipesgd_runtime_destroy(pipesgd_runtime *rt)
{
    if (!rt) return;
    if (rt->compute) (void)hipStreamSynchronize(rt->compute);
    if (rt->comm) (void)hipStreamSynchronize(rt->comm);
    for (int i = 0; i < kEventRing; ++i) {
        if (rt->local_ready[i]) (void)hipEventDestroy(rt->local_ready[i]);
        if (rt->sum_ready[i]) (void)hipEventDestroy(rt->sum_ready[i]);
    }
    for (hipEvent_t e : rt->timing) (void)hipEventDestroy(e);
    if (rt->compute) (void)hipStreamDestroy(rt->compute);
    if (rt->comm) (void)hipStreamDestroy(rt->comm);
    delete rt;
}

void *pipesgd_runtime_stream(pipesgd_runtime *rt, int which)
{
    if (!rt) return nullptr;
    return which == 0 ? static_cast<void *>(rt->compute) : static_cast<void *>(rt->comm);
}

int pipesgd_runtime_sync(pipesgd_runtime *rt)
{
    if (!rt) return PIPESGD_ERR_ARG;
    if (hipStreamSynchronize(rt->compute) != hipSuccess) return PIPESGD_ERR_HIP;
    if (hipStreamSynchronize(rt->comm) != hipSuccess) return PIPESGD_ERR_HIP;
    return PIPESGD_OK;
}

int pipesgd_runtime_update_time(pipesgd_runtime *rt, double *total_ms, uint64_t *launches)
{
    if (!rt || !rt->ok || !total_ms || !launches) return PIPESGD_ERR_ARG;
    if (hipStreamSynchronize(rt->compute) != hipSuccess) return PIPESGD_ERR_HIP;
    double sum = 0.0;
    for (size_t i = 0; i < rt->timed; ++i) {
        float ms = 0.0f;
        if (hipEventElapsedTime(&ms, rt->timing[2 * i], rt->timing[2 * i + 1]) != hipSuccess) return PIPESGD_ERR_HIP;
        sum += static_cast<double>(ms);
    }
    *total_ms = sum;
    *launches = rt->timed;
    rt->timed = 0;
    return PIPESGD_OK;
}

int pipesgd_synthetic_compute(float duration_us, int workgroups, void *stream)
{
    const int rc = pipesgd_internal_check_standin(duration_us, workgroups);
    if (rc != PIPESGD_OK) return rc;
    if (duration_us == 0.0f) return PIPESGD_OK;
    const uint64_t ticks = static_cast<uint64_t>(static_cast<double>(duration_us) * 100.0);   // 100 MHz
    hipLaunchKernelGGL(synthetic_compute_kernel, dim3(workgroups), dim3(64), 0, static_cast<hipStream_t>(stream),
                       ticks, static_cast<unsigned *>(nullptr));
    return hipGetLastError() == hipSuccess ? PIPESGD_OK : PIPESGD_ERR_HIP;
}

int pipesgd_runtime_iteration(pipesgd_runtime *rt, const pipesgd_runtime_iter *it)
{
    if (!rt || !rt->ok || !it || !it->ring) return PIPESGD_ERR_ARG;
    if (it->width < 1 || it->width >= kEventRing || (it->flags & ~PIPESGD_RT_TIME_UPDATE) != 0) return PIPESGD_ERR_ARG;
    const int wg = it->compute_workgroups > 0 ? it->compute_workgroups : 1;
    // Everything is checked here, before the first launch or event record: a rejected call leaves both
    // streams, the events and the iteration count as they were, and the same iteration can be issued again.
    int rc = pipesgd_internal_check_allreduce(it->ring, it->schedule);
    if (rc == PIPESGD_OK) {
        const bool sync = it->width == 1;
        rc = pipesgd_internal_check_update(it->ring->mode, it->replicas, sync ? it->fresh_g_sum_c : it->stale_g_sum_c,
                                           sync ? it->fresh_scales : it->stale_scales, it->ring->n, it->w, it->v,
                                           it->momentum);
    }
    if (rc == PIPESGD_OK && it->width >= 2 && it->ring->n > 0) {
        // the update reads the stale slot set while the AllReduce on the other stream writes the ring's: they
        // must be different buffers (pointer identity; partial overlaps are the caller's to avoid)
        for (int r = 0; r < it->replicas && rc == PIPESGD_OK; ++r)
            for (int q = 0; q < it->ring->workers; ++q)
                if (it->stale_g_sum_c[r] == it->ring->g_sum_c[q]) { rc = PIPESGD_ERR_ARG; break; }
    }
    if (rc == PIPESGD_OK) rc = pipesgd_internal_check_standin(it->compute_us, wg);
    if (rc == PIPESGD_OK) rc = pipesgd_internal_check_standin(it->wire_us, 1);
    if (rc != PIPESGD_OK) return rc;
    hipEvent_t t_start = nullptr, t_stop = nullptr;     // host objects only; made before anything is enqueued
    if (it->flags & PIPESGD_RT_TIME_UPDATE) {
        if (rt->timed >= kMaxTimed) return PIPESGD_ERR_CAPACITY;       // read the times out first
        try {
            while (rt->timing.size() < 2 * (rt->timed + 1)) {
                hipEvent_t e;
                if (hipEventCreate(&e) != hipSuccess) return PIPESGD_ERR_HIP;
                rt->timing.push_back(e);
            }
        } catch (const std::bad_alloc &) {
            return PIPESGD_ERR_CAPACITY;
        }
        t_start = rt->timing[2 * rt->timed];
        t_stop = rt->timing[2 * rt->timed + 1];
    }
    // the update launch, bracketed by the timing events when asked for
    auto update = [&](const void *const *g_sum_c, const float *const *scales) -> int {
        if (t_start && hipEventRecord(t_start, rt->compute) != hipSuccess) return PIPESGD_ERR_HIP;
        const int urc = pipesgd_apply_update_multi(it->ring->mode, it->replicas, g_sum_c, scales, it->ring->n, it->w, it->v,
                                                   it->lr, it->momentum, it->grad_scale, rt->compute);
        if (urc != PIPESGD_OK) return urc;
        if (t_stop) {
            if (hipEventRecord(t_stop, rt->compute) != hipSuccess) return PIPESGD_ERR_HIP;
            ++rt->timed;
        }
        return PIPESGD_OK;
    };

    const uint64_t t = rt->t + 1;                       // this call is iteration t (1-based)
    hipEvent_t sum_ready = rt->sum_ready[t % kEventRing];

    if (it->width >= 2) {
        // Indexing: g[t] is the gradient evaluated at w[t-1]; A[t] = AllReduce(g[t]);
        // w[t] = Update(w[t-1], A[t-(K-1)]), K = width = Alg. 1's iteration dependency
        // (2 in the paper's optimal setting).  (Alg. 1 counts the same steps one later.)
        const uint64_t lag = static_cast<uint64_t>(it->width - 1);
        // communication thread: g[t] was marked ready by the previous call's compute part
        if (t > 1 && hipStreamWaitEvent(rt->comm, rt->local_ready[t % kEventRing], 0) != hipSuccess) return PIPESGD_ERR_HIP;
        rc = pipesgd_allreduce_sim(it->ring, it->schedule, rt->comm);
        if (rc != PIPESGD_OK) return rc;
        rc = pipesgd_synthetic_compute(it->wire_us, 1, rt->comm);          // time on the network
        if (rc != PIPESGD_OK) return rc;
        if (hipEventRecord(sum_ready, rt->comm) != hipSuccess) return PIPESGD_ERR_HIP;
        // computation thread, meanwhile: wait for A[t-(K-1)], decompress + update -> w[t], then the
        // stand-in for batch/forward/backward that yields g[t+1], and mark it ready
        if (t > lag && hipStreamWaitEvent(rt->compute, rt->sum_ready[(t - lag) % kEventRing], 0) != hipSuccess)
            return PIPESGD_ERR_HIP;
        rc = update(it->stale_g_sum_c, it->stale_scales);
        if (rc != PIPESGD_OK) return rc;
        rc = pipesgd_synthetic_compute(it->compute_us, wg, rt->compute);
        if (rc != PIPESGD_OK) return rc;
        if (hipEventRecord(rt->local_ready[(t + 1) % kEventRing], rt->compute) != hipSuccess) return PIPESGD_ERR_HIP;
    } else {
        // decentralised synchronous SGD: compute g[t], AllReduce it, update with this iteration's sum
        hipEvent_t local_ready = rt->local_ready[t % kEventRing];
        rc = pipesgd_synthetic_compute(it->compute_us, wg, rt->compute);
        if (rc != PIPESGD_OK) return rc;
        if (hipEventRecord(local_ready, rt->compute) != hipSuccess) return PIPESGD_ERR_HIP;
        if (hipStreamWaitEvent(rt->comm, local_ready, 0) != hipSuccess) return PIPESGD_ERR_HIP;
        rc = pipesgd_allreduce_sim(it->ring, it->schedule, rt->comm);
        if (rc != PIPESGD_OK) return rc;
        rc = pipesgd_synthetic_compute(it->wire_us, 1, rt->comm);          // time on the network
        if (rc != PIPESGD_OK) return rc;
        if (hipEventRecord(sum_ready, rt->comm) != hipSuccess) return PIPESGD_ERR_HIP;
        if (hipStreamWaitEvent(rt->compute, sum_ready, 0) != hipSuccess) return PIPESGD_ERR_HIP;
        rc = update(it->fresh_g_sum_c, it->fresh_scales);
        if (rc != PIPESGD_OK) return rc;
    }
    rt->t = t;
    return PIPESGD_OK;
}

}  // extern "C"

int pipesgd_internal_check_standin(float duration_us, int workgroups)
{
    if (!(duration_us >= 0.0f) || duration_us > 1.0e6f || workgroups < 1 || workgroups > 65535) return PIPESGD_ERR_ARG;
    return PIPESGD_OK;
}
