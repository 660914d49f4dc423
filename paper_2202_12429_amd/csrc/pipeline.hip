// bp_pipeline_*: cache maintenance overlapped with training (Section 3.2: prefetching runs ahead of the trainer;
// Section 3.4: the trainer's cache is maintained beside the training step, on slots the running batch does not
// touch).  Host-side scheduling only: the row copies are the launches of cache_apply.hip, enqueued on a
// maintenance stream of its own and tied to the caller's compute stream with events.
//
// Per batch i the compute stream runs  acquire(i) . forward . backward/update . release(i).  release(i) enqueues
//   A_i  stage the rows evicted after batch i, then fetch the LATE prefetches of batch i+1 (those whose slot was
//        freed by batch i's evictions)                                         -> batch i+1 may start
//   B_i  write the staged rows back and fetch the EARLY prefetches of batch i+2 (slots free since before batch
//        i+1), while batch i+1 trains.
// When batch i+1 has no late prefetches, A_i is empty and B_i is a single launch without staging
// (bp_cache_apply_handoff): an evicted row leaves and the row that takes its slot arrives through one lane group.
// A batch without late prefetches (the usual case when the plan keeps a reserve of free slots) is ready as soon as
// B of two batches earlier is done, so the compute stream never waits for the batch before it.
// Which prefetches are early follows from the ring order alone: the x-th miss of the trace takes ring position x,
// positions below C are the initial slots and position C + e is the slot of the e-th eviction, so the misses of
// batch j whose position lies below C + (evictions up to batch j-2) are a prefix of its (id-ordered) list.
// Reads of the backing table stay behind the write-backs they depend on because both are on the maintenance
// stream, in order; an early prefetch never meets a pending update because with L_eff >= 2 a row used by batch
// j-1 and again by batch j is kept, not fetched.  With L_eff == 1 nothing is early and the write-back precedes the
// fetches, as in the synchronous order.
#include <new>
#include <vector>

#include "common.h"

struct bp_pipeline {
    bp_config cfg;
    void *cache_w, *cache_s, *back_w, *back_s;
    const int64_t *p_ids, *e_ids;
    const int32_t *p_slots, *e_slots;
    std::vector<int64_t> p_off, e_off, early;
    int32_t T, L_eff;
    void* staging;
    size_t staging_bytes;
    hipStream_t maint;
    hipEvent_t ready[2], done[2], hand;
    int64_t grid_cap;     // workgroups per maintenance launch at most
    bool begun;
};

namespace bp {
namespace {

// Workgroups per maintenance launch: 2 per CU keeps ~2,000 wavefronts of 16-byte accesses in flight, enough for the
// host link and for a backing table in HBM, and leaves the rest of every CU to the training kernels.
constexpr int64_t kMaintenanceBlocks = 512;
// The one-launch step (no staging) runs narrower still.  While rows are in flight over the host link a training kernel
// beside them crawls, whatever CUs it runs on (the forward pass takes 0.2-0.3 ms instead of 0.03): the requests to
// host memory hold up everybody's requests somewhere on the way out of the GPU, and how much depends on how many
// of them are outstanding.  128 workgroups are the measured optimum on a Criteo-shaped step behind PCIe (a step of
// 0.345 ms; 0.378 with 256 or 512 workgroups, 0.396 with 64, 0.420 with 32).
constexpr int64_t kHandoffBlocks = 128;
// ... and only for steps of moderate size.  With ten times the rows per step (0.7 M rows of 256 bytes, a multi-hot
// workload) the staged path, whose second launch keeps both directions of the link busy at once, ends 10 % ahead of
// the one-launch step at any width (128, 256, 512 workgroups); with 47 K rows of 384 bytes per step it is 8 % behind.
constexpr int64_t kHandoffMaxRows = int64_t(1) << 17;

int prefetch_range(bp_pipeline* p, int64_t a, int64_t b) {      // cache <- backing for list entries [a, b)
    if (b <= a) return BP_OK;
    return cache_apply_impl(&p->cfg, p->cache_w, p->cache_s, p->back_w, p->back_s, nullptr, nullptr, 0, p->p_ids + a,
                            p->p_slots + a, b - a, p->maint, p->grid_cap);
}

int64_t late_count(const bp_pipeline* p, int j) {
    return j < p->T ? (p->p_off[j + 1] - p->p_off[j]) - p->early[j] : 0;
}

// A_i and B_i for i in [-1, T-1]; i == -1 is the start of the trace (nothing to write back).  Batch j is ready once
// its last fetch is enqueued: after A_{j-1} when it has late prefetches, else already after B_{j-2}, in which case
// it never waits for the batch before it.
int enqueue_after_batch(bp_pipeline* p, int i) {
    const int T = p->T;
    const int64_t ea = i >= 0 ? p->e_off[i] : 0, eb = i >= 0 ? p->e_off[i + 1] : 0;
    const int64_t ne = eb - ea;
    const int j1 = i + 1, j2 = i + 2;
    const int64_t p1a = j1 < T ? p->p_off[j1] + p->early[j1] : 0, p1b = j1 < T ? p->p_off[j1 + 1] : 0;   // late of i+1
    const int64_t p2a = j2 < T ? p->p_off[j2] : 0, p2b = j2 < T ? p->p_off[j2] + p->early[j2] : 0;       // early of i+2
    if (p->L_eff < 2) {
        // the synchronous order: every write-back of batch i before any fetch for batch i+1
        BP_TRY(cache_apply_impl(&p->cfg, p->cache_w, p->cache_s, p->back_w, p->back_s, p->e_ids + ea, p->e_slots + ea, ne,
                                p->p_ids + p1a, p->p_slots + p1a, p1b - p1a, p->maint, p->grid_cap));
        if (j1 < T) BP_HIP(hipEventRecord(p->ready[j1 & 1], p->maint));
        return BP_OK;
    }
    if (p->L_eff >= 3 && i >= 0 && late_count(p, j1) == 0 && ne + (p2b - p2a) <= kHandoffMaxRows) {
        // Nothing of batch i+1 waits for the slots freed now, so no staging: one launch writes the rows evicted after
        // batch i back and fetches the early prefetches of batch i+2.  By the ring order those of them whose slot was
        // not free before (miss ordinal x with x - C at or past batch i's first eviction) are the tail of the early
        // prefix, and they take the slots of batch i's evictions from the first one on, in order: the pairing that
        // bp_cache_apply_handoff moves through registers.  (With late prefetches of batch i+1 the first evictions
        // pair with those instead, and the staged path below is taken.)
        int64_t n_free = p->cfg.capacity + ea - p2a;          // early entries whose slot has been free since before
        if (n_free > p2b - p2a) n_free = p2b - p2a;
        if (n_free < 0) return fail(BP_ERR_INVALID_ARG, "internal: batch %d has no late prefetches but its successor's ring positions say otherwise", j1);
        const int64_t narrow = p->grid_cap < kHandoffBlocks ? p->grid_cap : kHandoffBlocks;
        BP_TRY(cache_apply_handoff_impl(&p->cfg, p->cache_w, p->cache_s, p->back_w, p->back_s, p->e_ids + ea,
                                        p->e_slots + ea, ne, p->p_ids + p2a, p->p_slots + p2a, p2b - p2a, n_free, nullptr,
                                        p->maint, narrow));
        if (j2 < T && late_count(p, j2) == 0) BP_HIP(hipEventRecord(p->ready[j2 & 1], p->maint));
        return BP_OK;
    }
    BP_TRY(cache_stage_impl(&p->cfg, p->cache_w, p->cache_s, p->e_slots + ea, ne, p->staging, p->staging_bytes, p->maint,
                            p->grid_cap));
    if (j1 < T && (i < 0 || late_count(p, j1) > 0)) {
        BP_TRY(prefetch_range(p, p1a, p1b));
        BP_HIP(hipEventRecord(p->ready[j1 & 1], p->maint));
    }
    if (p->L_eff >= 3) {     // rows evicted after batch i are not used by batch i+2: one launch, both directions
        BP_TRY(cache_apply_staged_impl(&p->cfg, p->cache_w, p->cache_s, p->back_w, p->back_s, p->e_ids + ea,
                                       p->e_slots + ea, ne, p->staging, p->staging_bytes, p->p_ids + p2a, p->p_slots + p2a,
                                       p2b - p2a, p->maint, p->grid_cap));
    } else {
        BP_TRY(cache_apply_staged_impl(&p->cfg, p->cache_w, p->cache_s, p->back_w, p->back_s, p->e_ids + ea,
                                       p->e_slots + ea, ne, p->staging, p->staging_bytes, nullptr, nullptr, 0, p->maint,
                                       p->grid_cap));
        BP_TRY(prefetch_range(p, p2a, p2b));
    }
    if (j2 < T && late_count(p, j2) == 0) BP_HIP(hipEventRecord(p->ready[j2 & 1], p->maint));
    return BP_OK;
}

}  // namespace
}  // namespace bp

using namespace bp;

BP_EXPORT int bp_pipeline_early_counts(const int64_t* prefetch_offsets, const int64_t* evict_offsets, int32_t n_iters,
                                       int64_t capacity, int32_t L_eff, int64_t* early) {
    if (!prefetch_offsets || !evict_offsets || !early) return fail(BP_ERR_INVALID_ARG, "NULL pointer");
    if (n_iters < 1 || capacity < 1) return fail(BP_ERR_INVALID_ARG, "n_iters or capacity < 1");
    for (int j = 0; j < n_iters; ++j) {
        int64_t e = 0;
        if (j >= 1 && L_eff >= 2) {
            const int64_t misses = prefetch_offsets[j + 1] - prefetch_offsets[j];
            e = capacity + evict_offsets[j - 1] - prefetch_offsets[j];   // free ring positions known before batch j-1
            if (e < 0) e = 0;
            if (e > misses) e = misses;
        }
        early[j] = e;
    }
    return BP_OK;
}

BP_EXPORT int bp_pipeline_create(const bp_config* cfg, void* cache_w, void* cache_state, void* backing_w,
                                 void* backing_state, const int64_t* prefetch_ids, const int32_t* prefetch_slots,
                                 const int64_t* prefetch_offsets, const int64_t* evict_ids, const int32_t* evict_slots,
                                 const int64_t* evict_offsets, int32_t n_iters, int32_t L_eff, void* staging,
                                 size_t staging_bytes, bp_pipeline** out) {
    BP_TRY(check_config(cfg));
    if (!out) return fail(BP_ERR_INVALID_ARG, "out is NULL");
    *out = nullptr;
    if (n_iters < 1 || L_eff < 1) return fail(BP_ERR_INVALID_ARG, "n_iters or L_eff < 1");
    if (!cache_w || !backing_w || !prefetch_offsets || !evict_offsets) return fail(BP_ERR_INVALID_ARG, "NULL pointer");
    if (cfg->optimizer != BP_SGD && (!cache_state || !backing_state))
        return fail(BP_ERR_INVALID_ARG, "optimizer state pointers are NULL");
    int64_t most = 0;
    for (int i = 0; i < n_iters; ++i) {
        if (prefetch_offsets[i + 1] < prefetch_offsets[i] || evict_offsets[i + 1] < evict_offsets[i])
            return fail(BP_ERR_INVALID_ARG, "list offsets decrease at batch %d", i);
        const int64_t ne = evict_offsets[i + 1] - evict_offsets[i];
        if (ne > most) most = ne;
    }
    if ((prefetch_offsets[n_iters] && (!prefetch_ids || !prefetch_slots)) ||
        (evict_offsets[n_iters] && (!evict_ids || !evict_slots)))
        return fail(BP_ERR_INVALID_ARG, "a list pointer is NULL");
    size_t need = 0;
    BP_TRY(bp_cache_apply_duplex_workspace_bytes(cfg, most, &need));
    if (most && L_eff >= 2) {
        if (!staging || ((uintptr_t)staging & 255)) return fail(BP_ERR_INVALID_ARG, "staging NULL or not 256-byte aligned");
        if (staging_bytes < need)
            return fail(BP_ERR_WORKSPACE_TOO_SMALL, "staging %zu < required %zu bytes", staging_bytes, need);
    }
    bp_pipeline* p = new (std::nothrow) bp_pipeline();
    if (!p) return fail(BP_ERR_INVALID_ARG, "out of host memory");
    p->cfg = *cfg;
    p->cache_w = cache_w; p->cache_s = cache_state; p->back_w = backing_w; p->back_s = backing_state;
    p->p_ids = prefetch_ids; p->p_slots = prefetch_slots; p->e_ids = evict_ids; p->e_slots = evict_slots;
    p->p_off.assign(prefetch_offsets, prefetch_offsets + n_iters + 1);
    p->e_off.assign(evict_offsets, evict_offsets + n_iters + 1);
    p->early.resize(n_iters);
    p->T = n_iters; p->L_eff = L_eff;
    p->staging = staging; p->staging_bytes = staging_bytes;
    p->maint = nullptr; p->hand = nullptr; p->begun = false;
    p->grid_cap = kMaintenanceBlocks;
    p->ready[0] = p->ready[1] = p->done[0] = p->done[1] = nullptr;
    int st = bp_pipeline_early_counts(prefetch_offsets, evict_offsets, n_iters, cfg->capacity, L_eff, p->early.data());
    hipError_t e = hipSuccess;
    if (st == BP_OK) e = hipStreamCreateWithFlags(&p->maint, hipStreamNonBlocking);     // default priority
    hipEvent_t* evs[5] = {&p->ready[0], &p->ready[1], &p->done[0], &p->done[1], &p->hand};
    for (int k = 0; k < 5 && st == BP_OK && e == hipSuccess; ++k) e = hipEventCreateWithFlags(evs[k], hipEventDisableTiming);
    if (st == BP_OK && e != hipSuccess) st = fail(BP_ERR_HIP, "creating the maintenance stream or its events failed: %s", hipGetErrorString(e));
    if (st != BP_OK) {
        bp_pipeline_destroy(p);
        return st;
    }
    *out = p;
    return BP_OK;
}

BP_EXPORT int bp_pipeline_destroy(bp_pipeline* p) {
    if (!p) return BP_OK;
    if (p->maint) (void)hipStreamSynchronize(p->maint);
    hipEvent_t evs[5] = {p->ready[0], p->ready[1], p->done[0], p->done[1], p->hand};
    for (hipEvent_t ev : evs)
        if (ev) (void)hipEventDestroy(ev);
    if (p->maint) (void)hipStreamDestroy(p->maint);
    delete p;
    return BP_OK;
}

BP_EXPORT int bp_pipeline_early(const bp_pipeline* p, int32_t batch, int64_t* early) {
    if (!p || !early || batch < 0 || batch >= p->T) return fail(BP_ERR_INVALID_ARG, "bad pipeline, batch or pointer");
    *early = p->early[batch];
    return BP_OK;
}

BP_EXPORT int bp_pipeline_begin(bp_pipeline* p, void* compute_stream) {
    if (!p) return fail(BP_ERR_INVALID_ARG, "pipeline is NULL");
    // whatever the compute stream has enqueued so far (the plan, the table) precedes the first fetch
    BP_HIP(hipEventRecord(p->hand, (hipStream_t)compute_stream));
    BP_HIP(hipStreamWaitEvent(p->maint, p->hand, 0));
    p->begun = true;
    return enqueue_after_batch(p, -1);
}

BP_EXPORT int bp_pipeline_acquire(bp_pipeline* p, int32_t batch, void* compute_stream) {
    if (!p || !p->begun) return fail(BP_ERR_INVALID_ARG, "pipeline is NULL or not begun");
    if (batch < 0 || batch >= p->T) return fail(BP_ERR_INVALID_ARG, "batch %d outside [0, %d)", batch, p->T);
    BP_HIP(hipStreamWaitEvent((hipStream_t)compute_stream, p->ready[batch & 1], 0));
    return BP_OK;
}

BP_EXPORT int bp_pipeline_release(bp_pipeline* p, int32_t batch, void* compute_stream) {
    if (!p || !p->begun) return fail(BP_ERR_INVALID_ARG, "pipeline is NULL or not begun");
    if (batch < 0 || batch >= p->T) return fail(BP_ERR_INVALID_ARG, "batch %d outside [0, %d)", batch, p->T);
    BP_HIP(hipEventRecord(p->done[batch & 1], (hipStream_t)compute_stream));
    BP_HIP(hipStreamWaitEvent(p->maint, p->done[batch & 1], 0));
    return enqueue_after_batch(p, batch);
}

BP_EXPORT int bp_pipeline_end(bp_pipeline* p, void* compute_stream) {
    if (!p) return fail(BP_ERR_INVALID_ARG, "pipeline is NULL");
    BP_HIP(hipEventRecord(p->hand, p->maint));
    BP_HIP(hipStreamWaitEvent((hipStream_t)compute_stream, p->hand, 0));
    p->begun = false;
    return BP_OK;
}
