// bp_cache_apply: trainer-side cache maintenance (Section 3.4 "Trainer"; ordering rule of Section 3.2,
// "Consistency with the Lookahead algorithm").  Two row-copy launches on one stream: write-backs of the
// evict list first, then loads of the prefetch list.  The backing table is addressed through a
// device-visible pointer, so when it lives in pinned host memory the copies run as zero-copy PCIe
// reads / writes issued straight from the wavefronts, 16 bytes per lane, one row per lane group.
#include "common.h"
#include "row_access.h"

namespace bp {

namespace {

// TO_BACKING: backing[id] <- cache[slot]; otherwise cache[slot] <- backing[id].
template <int GW, bool TO_BACKING>
__global__ __launch_bounds__(kRowBlock) void cache_copy_rows_kernel(uint4* __restrict__ cache_w, uint4* __restrict__ back_w,
                                                                    uint4* __restrict__ cache_s, uint4* __restrict__ back_s,
                                                                    const int64_t* __restrict__ ids,
                                                                    const int32_t* __restrict__ slots, int64_t n, int64_t R,
                                                                    int64_t C, int lpr, int slpr, int rowwise, int64_t wst, int64_t sst) {
    const int c = threadIdx.x % GW;
    const int64_t stride = (int64_t)gridDim.x * (kRowBlock / GW);
    for (int64_t e = ((int64_t)blockIdx.x * kRowBlock + threadIdx.x) / GW; e < n; e += stride) {
        const int64_t g = ids[e];
        const int64_t s = slots[e];
        if (g < 0 || g >= R || s < 0 || s >= C) continue;
        if (c < lpr) {
            if (TO_BACKING) back_w[g * lpr + c] = cache_w[s * wst + c];
            else cache_w[s * wst + c] = back_w[g * lpr + c];
        }
        for (int k = c; k < slpr; k += GW) {          // element-wise state: its own row of slpr pieces
            if (TO_BACKING) back_s[g * slpr + k] = cache_s[s * sst + k];
            else cache_s[s * sst + k] = back_s[g * slpr + k];
        }
        if (rowwise && c == 0) {                      // row-wise state: one fp32 per row
            float* cs = reinterpret_cast<float*>(cache_s);
            float* bs = reinterpret_cast<float*>(back_s);
            if (TO_BACKING) bs[g] = cs[s * sst]; else cs[s * sst] = bs[g];
        }
    }
}

// Duplex variant, step 1: evicted rows leave the cache for a staging area in HBM (entry e -> staging row e), which
// frees their slots at HBM speed.
template <int GW>
__global__ __launch_bounds__(kRowBlock) void cache_stage_rows_kernel(const uint4* __restrict__ cache_w,
                                                                     const uint4* __restrict__ cache_s,
                                                                     uint4* __restrict__ stage_w, uint4* __restrict__ stage_s,
                                                                     const int32_t* __restrict__ slots, int64_t n, int64_t C,
                                                                     int lpr, int slpr, int rowwise, int64_t wst, int64_t sst) {
    const int c = threadIdx.x % GW;
    const int64_t stride = (int64_t)gridDim.x * (kRowBlock / GW);
    for (int64_t e = ((int64_t)blockIdx.x * kRowBlock + threadIdx.x) / GW; e < n; e += stride) {
        const int64_t s = slots[e];
        if (s < 0 || s >= C) continue;
        if (c < lpr) stage_w[e * lpr + c] = cache_w[s * wst + c];
        for (int k = c; k < slpr; k += GW) stage_s[e * slpr + k] = cache_s[s * sst + k];
        if (rowwise && c == 0) reinterpret_cast<float*>(stage_s)[e] = reinterpret_cast<const float*>(cache_s)[s * sst];
    }
}

// Duplex variant, step 2: one launch moves rows in both directions at once, so writes to the backing table
// (staging -> backing) and reads from it (backing -> cache) share the link's two directions instead of taking
// turns.  Lane groups alternate between the two lists while both last.
template <int GW>
__global__ __launch_bounds__(kRowBlock) void cache_duplex_kernel(uint4* __restrict__ cache_w, uint4* __restrict__ cache_s,
                                                                 uint4* __restrict__ back_w, uint4* __restrict__ back_s,
                                                                 const uint4* __restrict__ stage_w,
                                                                 const uint4* __restrict__ stage_s,
                                                                 const int64_t* __restrict__ e_ids,
                                                                 const int32_t* __restrict__ e_slots, int64_t n_e,
                                                                 const int64_t* __restrict__ p_ids,
                                                                 const int32_t* __restrict__ p_slots, int64_t n_p, int64_t R,
                                                                 int64_t C, int lpr, int slpr, int rowwise, int64_t wst, int64_t sst) {
    const int c = threadIdx.x % GW;
    const int64_t stride = (int64_t)gridDim.x * (kRowBlock / GW);
    const int64_t both = 2 * (n_e < n_p ? n_e : n_p);
    for (int64_t x = ((int64_t)blockIdx.x * kRowBlock + threadIdx.x) / GW; x < n_e + n_p; x += stride) {
        bool evict;
        int64_t k;
        if (x < both) {
            evict = (x & 1) == 0;
            k = x >> 1;
        } else {
            evict = n_e > n_p;
            k = x - both / 2;
        }
        if (evict) {
            const int64_t g = e_ids[k];
            const int64_t s = e_slots[k];
            if (g < 0 || g >= R || s < 0 || s >= C) continue;        // same entries the staging step skipped
            if (c < lpr) back_w[g * lpr + c] = stage_w[k * lpr + c];
            for (int q = c; q < slpr; q += GW) back_s[g * slpr + q] = stage_s[k * slpr + q];
            if (rowwise && c == 0) reinterpret_cast<float*>(back_s)[g] = reinterpret_cast<const float*>(stage_s)[k];
        } else {
            const int64_t g = p_ids[k];
            const int64_t s = p_slots[k];
            if (g < 0 || g >= R || s < 0 || s >= C) continue;
            if (c < lpr) cache_w[s * wst + c] = back_w[g * lpr + c];
            for (int q = c; q < slpr; q += GW) cache_s[s * sst + q] = back_s[g * slpr + q];
            if (rowwise && c == 0) reinterpret_cast<float*>(cache_s)[s * sst] = reinterpret_cast<const float*>(back_s)[g];
        }
    }
}

// Maintenance in one launch without a staging area.  With the FIFO ring the prefetches of a step that land in slots
// freed by the same step's evictions are the tail of the prefetch list, and they take those slots in the evictions'
// own order: prefetch entry n_early + k gets the slot of evict entry k.  Lane group k therefore moves the evicted row
// out and the fetched row in, one after the other, through its registers; nobody else touches that slot in this
// step.  The other evictions (k >= n_late) and the early prefetches (slots that were free before) are plain copies.
template <int GW>
__global__ __launch_bounds__(kRowBlock) void cache_handoff_kernel(uint4* __restrict__ cache_w, uint4* __restrict__ cache_s,
                                                                  uint4* __restrict__ back_w, uint4* __restrict__ back_s,
                                                                  const int64_t* __restrict__ e_ids,
                                                                  const int32_t* __restrict__ e_slots, int64_t n_e,
                                                                  const int64_t* __restrict__ p_ids,
                                                                  const int32_t* __restrict__ p_slots, int64_t n_p,
                                                                  int64_t n_early, int64_t R, int64_t C, int lpr, int slpr,
                                                                  int rowwise, int64_t wst, int64_t sst,
                                                                  uint32_t* __restrict__ mismatch) {
    const int c = threadIdx.x % GW;
    const int64_t stride = (int64_t)gridDim.x * (kRowBlock / GW);
    const int64_t n_late = n_p - n_early;
    // units: [0, n_e) the evictions (the first n_late of them followed by their paired fetch), then the early fetches
    for (int64_t x = ((int64_t)blockIdx.x * kRowBlock + threadIdx.x) / GW; x < n_e + n_early; x += stride) {
        if (x < n_e) {
            const int64_t g = e_ids[x];
            const int64_t s = e_slots[x];
            const bool ok = g >= 0 && g < R && s >= 0 && s < C;
            if (ok) {
                if (c < lpr) back_w[g * lpr + c] = cache_w[s * wst + c];
                for (int q = c; q < slpr; q += GW) back_s[g * slpr + q] = cache_s[s * sst + q];
                if (rowwise && c == 0) reinterpret_cast<float*>(back_s)[g] = reinterpret_cast<const float*>(cache_s)[s * sst];
            }
            if (x >= n_late) continue;
            const int64_t g2 = p_ids[n_early + x];
            const int64_t s2 = p_slots[n_early + x];
            if (s2 != s) {                       // not the pairing of a FIFO plan: leave the slot alone and say so
                if (c == 0 && mismatch) atomicOr(mismatch, 1u);
                continue;
            }
            if (g2 < 0 || g2 >= R || !ok) continue;
            // the reads of the evicted row above have returned before these writes are issued: same lanes, same addresses
            if (c < lpr) cache_w[s * wst + c] = back_w[g2 * lpr + c];
            for (int q = c; q < slpr; q += GW) cache_s[s * sst + q] = back_s[g2 * slpr + q];
            if (rowwise && c == 0) reinterpret_cast<float*>(cache_s)[s * sst] = reinterpret_cast<const float*>(back_s)[g2];
        } else {
            const int64_t m = x - n_e;
            const int64_t g = p_ids[m];
            const int64_t s = p_slots[m];
            if (g < 0 || g >= R || s < 0 || s >= C) continue;
            if (c < lpr) cache_w[s * wst + c] = back_w[g * lpr + c];
            for (int q = c; q < slpr; q += GW) cache_s[s * sst + q] = back_s[g * slpr + q];
            if (rowwise && c == 0) reinterpret_cast<float*>(cache_s)[s * sst] = reinterpret_cast<const float*>(back_s)[g];
        }
    }
}

inline dim3 capped_grid(int64_t threads, int64_t max_blocks) {
    int64_t blocks = ceil_div(threads, kRowBlock);
    if (max_blocks > 0 && blocks > max_blocks) blocks = max_blocks;
    return dim3((unsigned)(blocks > 0 ? blocks : 1));
}

struct DuplexLaunch {
    const bp_config* cfg;
    void *cache_w, *cache_s, *back_w, *back_s, *stage_w, *stage_s;
    const int64_t* e_ids;
    const int32_t* e_slots;
    int64_t n_e;
    const int64_t* p_ids;
    const int32_t* p_slots;
    int64_t n_p;
    hipStream_t stream;
    bool stage, apply;     // which of the two steps to launch
    int64_t max_blocks;    // 0: one lane group per entry; otherwise the grid is capped and the lane groups stride
    template <int GW, bool BF16>
    int run() {
        const int lpr = (int)(row_bytes(cfg) / 16);
        const int slpr = cfg->optimizer == BP_ADAGRAD ? cfg->dim / 4 : 0;
        const int rowwise = cfg->optimizer == BP_ADAGRAD_ROWWISE;
        if (stage && n_e)
            BP_LAUNCH(K_CACHE_STAGE, (cache_stage_rows_kernel<GW>), capped_grid(n_e * GW, max_blocks),
                      dim3(kRowBlock), 0, stream, (const uint4*)cache_w, (const uint4*)cache_s, (uint4*)stage_w,
                      (uint4*)stage_s, e_slots, n_e, cfg->capacity, lpr, slpr, rowwise, cache_w_stride16(cfg), cache_s_stride(cfg));
        if (apply && n_e + n_p)
            BP_LAUNCH(K_CACHE_DUPLEX, (cache_duplex_kernel<GW>), capped_grid((n_e + n_p) * GW, max_blocks),
                      dim3(kRowBlock), 0, stream, (uint4*)cache_w, (uint4*)cache_s, (uint4*)back_w, (uint4*)back_s,
                      (const uint4*)stage_w, (const uint4*)stage_s, e_ids, e_slots, n_e, p_ids, p_slots, n_p,
                      cfg->total_rows, cfg->capacity, lpr, slpr, rowwise, cache_w_stride16(cfg), cache_s_stride(cfg));
        return BP_OK;
    }
};

size_t stage_w_bytes(const bp_config* cfg, int64_t n_evict) {
    return (((size_t)(n_evict > 0 ? n_evict : 1) * row_bytes(cfg)) + 255) & ~size_t(255);
}
size_t stage_s_bytes(const bp_config* cfg, int64_t n_evict) {
    return (((size_t)(n_evict > 0 ? n_evict : 1) * state_row_bytes(cfg)) + 255) & ~size_t(255);
}

struct CopyLaunch {
    const bp_config* cfg;
    void *cache_w, *cache_s, *back_w, *back_s;
    const int64_t* ids;
    const int32_t* slots;
    int64_t n;
    bool to_backing;
    hipStream_t stream;
    int64_t max_blocks;
    template <int GW, bool BF16>
    int run() {
        const int lpr = (int)(row_bytes(cfg) / 16);
        const int slpr = cfg->optimizer == BP_ADAGRAD ? cfg->dim / 4 : 0;
        const int rowwise = cfg->optimizer == BP_ADAGRAD_ROWWISE;
        const dim3 grid = capped_grid(n * GW, max_blocks);
        if (to_backing)
            BP_LAUNCH(K_CACHE_EVICT, (cache_copy_rows_kernel<GW, true>), grid, dim3(kRowBlock), 0, stream, (uint4*)cache_w,
                      (uint4*)back_w, (uint4*)cache_s, (uint4*)back_s, ids, slots, n, cfg->total_rows, cfg->capacity, lpr,
                      slpr, rowwise, cache_w_stride16(cfg), cache_s_stride(cfg));
        else
            BP_LAUNCH(K_CACHE_PREFETCH, (cache_copy_rows_kernel<GW, false>), grid, dim3(kRowBlock), 0, stream,
                      (uint4*)cache_w, (uint4*)back_w, (uint4*)cache_s, (uint4*)back_s, ids, slots, n, cfg->total_rows,
                      cfg->capacity, lpr, slpr, rowwise, cache_w_stride16(cfg), cache_s_stride(cfg));
        return BP_OK;
    }
};

}  // namespace
}  // namespace bp

using namespace bp;

namespace bp {
int cache_apply_impl(const bp_config* cfg, void* cache_w, void* cache_state, void* backing_w, void* backing_state,
                              const int64_t* evict_ids, const int32_t* evict_slots, int64_t n_evict,
                              const int64_t* prefetch_ids, const int32_t* prefetch_slots, int64_t n_prefetch,
                              void* stream, int64_t grid_cap) {
    BP_TRY(check_config(cfg));
    if (n_evict < 0 || n_prefetch < 0) return fail(BP_ERR_INVALID_ARG, "negative list length");
    if (n_evict + n_prefetch == 0) return BP_OK;
    if (!cache_w || !backing_w) return fail(BP_ERR_INVALID_ARG, "cache_w or backing_w is NULL");
    if (cfg->optimizer != BP_SGD && (!cache_state || !backing_state))
        return fail(BP_ERR_INVALID_ARG, "optimizer state pointers are NULL");
    if (((uintptr_t)cache_w | (uintptr_t)backing_w | (uintptr_t)cache_state | (uintptr_t)backing_state) & 15)
        return fail(BP_ERR_INVALID_ARG, "row pointers must be 16-byte aligned");
    if ((n_evict && (!evict_ids || !evict_slots)) || (n_prefetch && (!prefetch_ids || !prefetch_slots)))
        return fail(BP_ERR_INVALID_ARG, "a list pointer is NULL");
    const int lpr = (int)(row_bytes(cfg) / 16);
    if (n_evict) {
        CopyLaunch l{cfg, cache_w, cache_state, backing_w, backing_state, evict_ids, evict_slots, n_evict, true,
                     (hipStream_t)stream, grid_cap};
        BP_TRY(dispatch_row(lpr, false, l));
    }
    if (n_prefetch) {
        CopyLaunch l{cfg, cache_w, cache_state, backing_w, backing_state, prefetch_ids, prefetch_slots, n_prefetch, false,
                     (hipStream_t)stream, grid_cap};
        BP_TRY(dispatch_row(lpr, false, l));
    }
    return BP_OK;
}
}  // namespace bp

BP_EXPORT int bp_cache_apply(const bp_config* cfg, void* cache_w, void* cache_state, void* backing_w, void* backing_state,
                              const int64_t* evict_ids, const int32_t* evict_slots, int64_t n_evict,
                              const int64_t* prefetch_ids, const int32_t* prefetch_slots, int64_t n_prefetch,
                              void* stream) {
    return bp::cache_apply_impl(cfg, cache_w, cache_state, backing_w, backing_state, evict_ids, evict_slots, n_evict, prefetch_ids,
                                prefetch_slots, n_prefetch, stream, 0);
}

BP_EXPORT int bp_cache_apply_duplex_workspace_bytes(const bp_config* cfg, int64_t n_evict, size_t* bytes) {
    if (!bytes) return fail(BP_ERR_INVALID_ARG, "bytes is NULL");
    BP_TRY(check_config(cfg));
    if (n_evict < 0) return fail(BP_ERR_INVALID_ARG, "negative list length");
    *bytes = stage_w_bytes(cfg, n_evict) + stage_s_bytes(cfg, n_evict);
    return BP_OK;
}

BP_EXPORT int bp_cache_apply_duplex(const bp_config* cfg, void* cache_w, void* cache_state, void* backing_w,
                                    void* backing_state, const int64_t* evict_ids, const int32_t* evict_slots,
                                    int64_t n_evict, const int64_t* prefetch_ids, const int32_t* prefetch_slots,
                                    int64_t n_prefetch, void* workspace, size_t workspace_bytes, void* stream) {
    BP_TRY(check_config(cfg));
    if (n_evict < 0 || n_prefetch < 0) return fail(BP_ERR_INVALID_ARG, "negative list length");
    if (n_evict + n_prefetch == 0) return BP_OK;
    if (!cache_w || !backing_w) return fail(BP_ERR_INVALID_ARG, "cache_w or backing_w is NULL");
    if (cfg->optimizer != BP_SGD && (!cache_state || !backing_state))
        return fail(BP_ERR_INVALID_ARG, "optimizer state pointers are NULL");
    if (((uintptr_t)cache_w | (uintptr_t)backing_w | (uintptr_t)cache_state | (uintptr_t)backing_state) & 15)
        return fail(BP_ERR_INVALID_ARG, "row pointers must be 16-byte aligned");
    if ((n_evict && (!evict_ids || !evict_slots)) || (n_prefetch && (!prefetch_ids || !prefetch_slots)))
        return fail(BP_ERR_INVALID_ARG, "a list pointer is NULL");
    const size_t need = stage_w_bytes(cfg, n_evict) + stage_s_bytes(cfg, n_evict);
    if (n_evict && (!workspace || ((uintptr_t)workspace & 255)))
        return fail(BP_ERR_INVALID_ARG, "workspace NULL or not 256-byte aligned");
    if (n_evict && workspace_bytes < need)
        return fail(BP_ERR_WORKSPACE_TOO_SMALL, "workspace %zu < required %zu bytes", workspace_bytes, need);
    DuplexLaunch l{cfg, cache_w, cache_state, backing_w, backing_state, workspace,
                   workspace ? (char*)workspace + stage_w_bytes(cfg, n_evict) : nullptr, evict_ids, evict_slots, n_evict,
                   prefetch_ids, prefetch_slots, n_prefetch, (hipStream_t)stream, true, true, 0};
    return dispatch_row((int)(row_bytes(cfg) / 16), false, l);
}

namespace bp {
namespace {
int check_staging(const bp_config* cfg, int64_t n_evict, const void* staging, size_t staging_bytes) {
    if (n_evict == 0) return BP_OK;
    const size_t need = stage_w_bytes(cfg, n_evict) + stage_s_bytes(cfg, n_evict);
    if (!staging || ((uintptr_t)staging & 255)) return fail(BP_ERR_INVALID_ARG, "staging NULL or not 256-byte aligned");
    if (staging_bytes < need)
        return fail(BP_ERR_WORKSPACE_TOO_SMALL, "staging %zu < required %zu bytes", staging_bytes, need);
    return BP_OK;
}
}  // namespace
}  // namespace bp

namespace bp {
int cache_stage_impl(const bp_config* cfg, const void* cache_w, const void* cache_state, const int32_t* evict_slots,
                             int64_t n_evict, void* staging, size_t staging_bytes, void* stream, int64_t grid_cap) {
    BP_TRY(check_config(cfg));
    if (n_evict < 0) return fail(BP_ERR_INVALID_ARG, "negative list length");
    if (n_evict == 0) return BP_OK;
    if (!cache_w || !evict_slots) return fail(BP_ERR_INVALID_ARG, "cache_w or evict_slots is NULL");
    if (cfg->optimizer != BP_SGD && !cache_state) return fail(BP_ERR_INVALID_ARG, "cache_state is NULL");
    if (((uintptr_t)cache_w | (uintptr_t)cache_state) & 15) return fail(BP_ERR_INVALID_ARG, "row pointers must be 16-byte aligned");
    BP_TRY(check_staging(cfg, n_evict, staging, staging_bytes));
    DuplexLaunch l{cfg, const_cast<void*>(cache_w), const_cast<void*>(cache_state), nullptr, nullptr, staging,
                   (char*)staging + stage_w_bytes(cfg, n_evict), nullptr, evict_slots, n_evict, nullptr, nullptr, 0,
                   (hipStream_t)stream, true, false, grid_cap};
    return dispatch_row((int)(row_bytes(cfg) / 16), false, l);
}
}  // namespace bp

BP_EXPORT int bp_cache_stage(const bp_config* cfg, const void* cache_w, const void* cache_state, const int32_t* evict_slots,
                             int64_t n_evict, void* staging, size_t staging_bytes, void* stream) {
    return bp::cache_stage_impl(cfg, cache_w, cache_state, evict_slots, n_evict, staging, staging_bytes, stream, 0);
}

namespace bp {
int cache_apply_staged_impl(const bp_config* cfg, void* cache_w, void* cache_state, void* backing_w,
                                    void* backing_state, const int64_t* evict_ids, const int32_t* evict_slots,
                                    int64_t n_evict, const void* staging, size_t staging_bytes, const int64_t* prefetch_ids,
                                    const int32_t* prefetch_slots, int64_t n_prefetch, void* stream, int64_t grid_cap) {
    BP_TRY(check_config(cfg));
    if (n_evict < 0 || n_prefetch < 0) return fail(BP_ERR_INVALID_ARG, "negative list length");
    if (n_evict + n_prefetch == 0) return BP_OK;
    if (!backing_w || (n_prefetch && !cache_w)) return fail(BP_ERR_INVALID_ARG, "cache_w or backing_w is NULL");
    if (cfg->optimizer != BP_SGD && (!backing_state || (n_prefetch && !cache_state)))
        return fail(BP_ERR_INVALID_ARG, "optimizer state pointers are NULL");
    if (((uintptr_t)cache_w | (uintptr_t)backing_w | (uintptr_t)cache_state | (uintptr_t)backing_state) & 15)
        return fail(BP_ERR_INVALID_ARG, "row pointers must be 16-byte aligned");
    if ((n_evict && (!evict_ids || !evict_slots)) || (n_prefetch && (!prefetch_ids || !prefetch_slots)))
        return fail(BP_ERR_INVALID_ARG, "a list pointer is NULL");
    BP_TRY(check_staging(cfg, n_evict, staging, staging_bytes));
    void* st = const_cast<void*>(staging);
    DuplexLaunch l{cfg, cache_w, cache_state, backing_w, backing_state, st,
                   st ? (char*)st + stage_w_bytes(cfg, n_evict) : nullptr, evict_ids, evict_slots, n_evict, prefetch_ids,
                   prefetch_slots, n_prefetch, (hipStream_t)stream, false, true, grid_cap};
    return dispatch_row((int)(row_bytes(cfg) / 16), false, l);
}
}  // namespace bp

BP_EXPORT int bp_cache_apply_staged(const bp_config* cfg, void* cache_w, void* cache_state, void* backing_w,
                                    void* backing_state, const int64_t* evict_ids, const int32_t* evict_slots,
                                    int64_t n_evict, const void* staging, size_t staging_bytes, const int64_t* prefetch_ids,
                                    const int32_t* prefetch_slots, int64_t n_prefetch, void* stream) {
    return bp::cache_apply_staged_impl(cfg, cache_w, cache_state, backing_w, backing_state, evict_ids, evict_slots, n_evict,
                                       staging, staging_bytes, prefetch_ids, prefetch_slots, n_prefetch, stream, 0);
}

namespace bp {
namespace {
struct HandoffLaunch {
    const bp_config* cfg;
    void *cache_w, *cache_s, *back_w, *back_s;
    const int64_t* e_ids;
    const int32_t* e_slots;
    int64_t n_e;
    const int64_t* p_ids;
    const int32_t* p_slots;
    int64_t n_p, n_early;
    uint32_t* mismatch;
    hipStream_t stream;
    int64_t grid_cap;
    template <int GW, bool BF16>
    int run() {
        const int lpr = (int)(row_bytes(cfg) / 16);
        const int slpr = cfg->optimizer == BP_ADAGRAD ? cfg->dim / 4 : 0;
        const int rowwise = cfg->optimizer == BP_ADAGRAD_ROWWISE;
        BP_LAUNCH(K_CACHE_DUPLEX, (cache_handoff_kernel<GW>), capped_grid((n_e + n_early) * GW, grid_cap),
                  dim3(kRowBlock), 0, stream, (uint4*)cache_w, (uint4*)cache_s, (uint4*)back_w, (uint4*)back_s, e_ids,
                  e_slots, n_e, p_ids, p_slots, n_p, n_early, cfg->total_rows, cfg->capacity, lpr, slpr, rowwise,
                  cache_w_stride16(cfg), cache_s_stride(cfg), mismatch);
        return BP_OK;
    }
};
}  // namespace
}  // namespace bp

namespace bp {
int cache_apply_handoff_impl(const bp_config* cfg, void* cache_w, void* cache_state, void* backing_w,
                                     void* backing_state, const int64_t* evict_ids, const int32_t* evict_slots,
                                     int64_t n_evict, const int64_t* prefetch_ids, const int32_t* prefetch_slots,
                                     int64_t n_prefetch, int64_t n_early, uint32_t* mismatch_flag, void* stream, int64_t grid_cap) {
    BP_TRY(check_config(cfg));
    if (n_evict < 0 || n_prefetch < 0) return fail(BP_ERR_INVALID_ARG, "negative list length");
    if (n_early < 0 || n_early > n_prefetch || n_prefetch - n_early > n_evict)
        return fail(BP_ERR_INVALID_ARG, "n_early %lld: need 0 <= n_early <= n_prefetch and n_prefetch - n_early <= n_evict",
                    (long long)n_early);
    if (n_evict + n_prefetch == 0) return BP_OK;
    if (!cache_w || !backing_w) return fail(BP_ERR_INVALID_ARG, "cache_w or backing_w is NULL");
    if (cfg->optimizer != BP_SGD && (!cache_state || !backing_state))
        return fail(BP_ERR_INVALID_ARG, "optimizer state pointers are NULL");
    if (((uintptr_t)cache_w | (uintptr_t)backing_w | (uintptr_t)cache_state | (uintptr_t)backing_state) & 15)
        return fail(BP_ERR_INVALID_ARG, "row pointers must be 16-byte aligned");
    if ((n_evict && (!evict_ids || !evict_slots)) || (n_prefetch && (!prefetch_ids || !prefetch_slots)))
        return fail(BP_ERR_INVALID_ARG, "a list pointer is NULL");
    HandoffLaunch l{cfg, cache_w, cache_state, backing_w, backing_state, evict_ids, evict_slots, n_evict, prefetch_ids,
                    prefetch_slots, n_prefetch, n_early, mismatch_flag, (hipStream_t)stream, grid_cap};
    return dispatch_row((int)(row_bytes(cfg) / 16), false, l);
}
}  // namespace bp

BP_EXPORT int bp_cache_apply_handoff(const bp_config* cfg, void* cache_w, void* cache_state, void* backing_w,
                                     void* backing_state, const int64_t* evict_ids, const int32_t* evict_slots,
                                     int64_t n_evict, const int64_t* prefetch_ids, const int32_t* prefetch_slots,
                                     int64_t n_prefetch, int64_t n_early, uint32_t* mismatch_flag, void* stream) {
    return bp::cache_apply_handoff_impl(cfg, cache_w, cache_state, backing_w, backing_state, evict_ids, evict_slots, n_evict,
                                        prefetch_ids, prefetch_slots, n_prefetch, n_early, mismatch_flag, stream, 0);
}
