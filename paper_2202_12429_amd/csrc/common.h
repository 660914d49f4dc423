// Shared host-side plumbing of the library: status/error text, launch + profiling helpers,
// workspace carving.  No device code here.
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include <cstdarg>
#include <cstddef>
#include <cstdint>
#include <cstdio>

#include "../../include/bagpipe.h"

// Entry points of the C ABI: the only symbols the shared library exports (built with -fvisibility=hidden).
#define BP_EXPORT extern "C" __attribute__((visibility("default")))

namespace bp {

constexpr int kWave = 64;   // gfx950 wavefront

// ---- error reporting ---------------------------------------------------------------------------
void set_error(const char* fmt, ...) __attribute__((format(printf, 1, 2)));
int fail(int status, const char* fmt, ...) __attribute__((format(printf, 2, 3)));

#define BP_HIP(expr)                                                                              \
    do {                                                                                          \
        hipError_t e_ = (expr);                                                                   \
        if (e_ != hipSuccess)                                                                     \
            return ::bp::fail(BP_ERR_HIP, "%s failed: %s (%s:%d)", #expr, hipGetErrorString(e_), \
                              __FILE__, __LINE__);                                                \
    } while (0)

#define BP_TRY(expr)              \
    do {                          \
        int s_ = (expr);          \
        if (s_ != BP_OK) return s_; \
    } while (0)

int check_config(const bp_config* cfg);

// The cache maintenance entry points with an explicit cap on the grid of their launches (0 = one lane group per
// list entry): the overlapped schedule keeps its copies narrow so that they leave most of the GPU to the training
// kernels running beside them; a few hundred wavefronts already keep the host link busy.
int cache_apply_impl(const bp_config* cfg, void* cache_w, void* cache_state, void* backing_w, void* backing_state,
                     const int64_t* evict_ids, const int32_t* evict_slots, int64_t n_evict, const int64_t* prefetch_ids,
                     const int32_t* prefetch_slots, int64_t n_prefetch, void* stream, int64_t grid_cap);
int cache_stage_impl(const bp_config* cfg, const void* cache_w, const void* cache_state, const int32_t* evict_slots,
                     int64_t n_evict, void* staging, size_t staging_bytes, void* stream, int64_t grid_cap);
int cache_apply_staged_impl(const bp_config* cfg, void* cache_w, void* cache_state, void* backing_w, void* backing_state,
                            const int64_t* evict_ids, const int32_t* evict_slots, int64_t n_evict, const void* staging,
                            size_t staging_bytes, const int64_t* prefetch_ids, const int32_t* prefetch_slots,
                            int64_t n_prefetch, void* stream, int64_t grid_cap);
int cache_apply_handoff_impl(const bp_config* cfg, void* cache_w, void* cache_state, void* backing_w, void* backing_state,
                             const int64_t* evict_ids, const int32_t* evict_slots, int64_t n_evict,
                             const int64_t* prefetch_ids, const int32_t* prefetch_slots, int64_t n_prefetch,
                             int64_t n_early, uint32_t* mismatch_flag, void* stream, int64_t grid_cap);

inline size_t elem_bytes(int dtype) { return dtype == BP_F32 ? 4 : 2; }
inline size_t row_bytes(const bp_config* c) { return (size_t)c->dim * elem_bytes(c->weight_dtype); }
inline size_t state_row_bytes(const bp_config* c) {
    return c->optimizer == BP_ADAGRAD ? (size_t)c->dim * 4 : c->optimizer == BP_ADAGRAD_ROWWISE ? 4 : 0;
}

// The cache arrays may be laid out with a stride wider than a row (bp_config.cache_w_stride / cache_state_stride: a
// caller that keeps a row's optimizer state right behind its weights passes the record size for both).  Stride of a
// cache row in 16-byte pieces; stride of its state in 16-byte pieces (element-wise state) or in floats (one float
// per row).
inline int64_t cache_w_stride16(const bp_config* c) {
    return (int64_t)((c->cache_w_stride ? (size_t)c->cache_w_stride : row_bytes(c)) / 16);
}
inline int64_t cache_s_stride(const bp_config* c) {
    const size_t b = c->cache_state_stride ? (size_t)c->cache_state_stride : state_row_bytes(c);
    return (int64_t)(c->optimizer == BP_ADAGRAD ? b / 16 : b / 4);
}

// ---- workspace carving -------------------------------------------------------------------------
// Hands out 256-byte aligned pieces of one caller-owned buffer; with base == nullptr it only counts.
class Carver {
  public:
    Carver(void* base, size_t bytes) : base_((char*)base), cap_(bytes) {}
    template <typename T>
    T* take(size_t count) {
        size_t off = (used_ + 255) & ~size_t(255);
        used_ = off + count * sizeof(T);
        return base_ ? (T*)(base_ + off) : nullptr;
    }
    size_t used() const { return (used_ + 255) & ~size_t(255); }
    bool fits() const { return used() <= cap_; }

  private:
    char* base_;
    size_t cap_;
    size_t used_ = 0;
};

// ---- kernel ids for profiling ------------------------------------------------------------------
enum KernelId {
    K_SORT_UPSWEEP = 0,
    K_SORT_SCAN,
    K_SORT_DOWNSWEEP,
    K_SCAN_REDUCE,
    K_SCAN_SPINE,
    K_SCAN_APPLY,
    K_PLAN_KEYS,
    K_PLAN_PAIRS,
    K_PLAN_HIST,
    K_PLAN_OCC,
    K_PLAN_FLAGS,
    K_PLAN_LISTS,
    K_PLAN_JUMP,
    K_PLAN_SLOTS,
    K_PLAN_GROUP,
    K_CACHE_EVICT,
    K_CACHE_PREFETCH,
    K_CACHE_STAGE,
    K_CACHE_DUPLEX,
    K_FWD,
    K_BWD_KEYS,
    K_BWD_ITEMS,
    K_BWD_REDUCE_UPDATE,
    K_FILL,
    K_COPY,
    K_NUM_KERNELS
};

extern bool g_profile_on;
extern uint64_t g_profile_mask;
bool profile_events(int id, hipEvent_t* start, hipEvent_t* stop);

// Launch `kernel`; when profiling is on, the launch carries a start and a stop event of its own (the runtime stamps
// them with the kernel's begin and end, so the reading holds no launch gap and no neighbouring work).
#define BP_LAUNCH(id, kernel, grid, block, shmem, stream, ...)                      \
    do {                                                                             \
        hipEvent_t ea_ = nullptr, eb_ = nullptr;                                     \
        if (::bp::g_profile_on && ((::bp::g_profile_mask >> (id)) & 1) && ::bp::profile_events((id), &ea_, &eb_))  \
            hipExtLaunchKernelGGL(kernel, grid, block, shmem, stream, ea_, eb_, 0, __VA_ARGS__);  \
        else                                                                         \
            hipLaunchKernelGGL(kernel, grid, block, shmem, stream, __VA_ARGS__);    \
        hipError_t le_ = hipGetLastError();                                          \
        if (le_ != hipSuccess)                                                       \
            return ::bp::fail(BP_ERR_HIP, "launch of %s failed: %s", #kernel, hipGetErrorString(le_)); \
    } while (0)

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
inline int bits_for(int64_t n) {   // bits needed to represent values in [0, n)
    int b = 1;
    while (b < 63 && (int64_t(1) << b) < n) ++b;
    return b;
}

}  // namespace bp
