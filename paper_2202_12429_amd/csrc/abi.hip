// Status text, argument checks shared by all entry points, and the event-based kernel profiler.
#include <cstring>
#include <algorithm>
#include <vector>

#include "common.h"
#include "row_access.h"

namespace bp {

static thread_local char t_error[512] = "";

void set_error(const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(t_error, sizeof(t_error), fmt, ap);
    va_end(ap);
}

int fail(int status, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(t_error, sizeof(t_error), fmt, ap);
    va_end(ap);
    return status;
}

int check_config(const bp_config* cfg) {
    if (!cfg) return fail(BP_ERR_INVALID_ARG, "cfg is NULL");
    if (cfg->total_rows < 1) return fail(BP_ERR_INVALID_ARG, "total_rows %lld < 1", (long long)cfg->total_rows);
    if (cfg->capacity < 1 || cfg->capacity >= (int64_t(1) << 31) - 1)
        return fail(BP_ERR_INVALID_ARG, "capacity %lld outside [1, 2^31 - 1)", (long long)cfg->capacity);
    if (cfg->weight_dtype != BP_F32 && cfg->weight_dtype != BP_BF16)
        return fail(BP_ERR_INVALID_ARG, "unknown weight_dtype %d", cfg->weight_dtype);
    if (cfg->optimizer != BP_SGD && cfg->optimizer != BP_ADAGRAD && cfg->optimizer != BP_ADAGRAD_ROWWISE)
        return fail(BP_ERR_INVALID_ARG, "unknown optimizer %d", cfg->optimizer);
    if (cfg->reserve < 0 || cfg->reserve >= cfg->capacity)
        return fail(BP_ERR_INVALID_ARG, "reserve %lld outside [0, capacity)", (long long)cfg->reserve);
    if (cfg->lookahead < 0) return fail(BP_ERR_INVALID_ARG, "lookahead %d < 0", cfg->lookahead);
    if (cfg->dim < 1) return fail(BP_ERR_INVALID_ARG, "dim %d < 1", cfg->dim);
    const size_t rb = row_bytes(cfg);
    if (rb % 16 != 0) return fail(BP_ERR_INVALID_ARG, "row of %zu bytes is not a multiple of 16 bytes", rb);
    if (rb > 1024) return fail(BP_ERR_UNSUPPORTED, "row of %zu bytes exceeds 1024 bytes", rb);
    if (cfg->cache_w_stride && (cfg->cache_w_stride < (int64_t)rb || cfg->cache_w_stride % 16 != 0))
        return fail(BP_ERR_INVALID_ARG, "cache_w_stride %lld: 0, or a multiple of 16 bytes >= the row's %zu bytes",
                    (long long)cfg->cache_w_stride, rb);
    const size_t sb = state_row_bytes(cfg);
    if (cfg->cache_state_stride &&
        (sb == 0 || cfg->cache_state_stride < (int64_t)sb || cfg->cache_state_stride % (cfg->optimizer == BP_ADAGRAD ? 16 : 4) != 0))
        return fail(BP_ERR_INVALID_ARG, "cache_state_stride %lld: 0, or a multiple of %d bytes >= the state's %zu bytes",
                    (long long)cfg->cache_state_stride, cfg->optimizer == BP_ADAGRAD ? 16 : 4, sb);
    return BP_OK;
}

// ---- profiler --------------------------------------------------------------------------------
bool g_profile_on = false;
uint64_t g_profile_mask = ~uint64_t(0);

namespace {
struct Span {
    int id;
    hipEvent_t a, b;
};
std::vector<Span> g_spans;          // recorded, not yet collected
std::vector<hipEvent_t> g_free;     // recycled events
int64_t g_count[K_NUM_KERNELS];
double g_ms[K_NUM_KERNELS];
std::vector<float> g_samples[K_NUM_KERNELS];     // every recorded launch's duration, for the spread

hipEvent_t get_event() {
    if (!g_free.empty()) {
        hipEvent_t e = g_free.back();
        g_free.pop_back();
        return e;
    }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}

const char* const kKernelNames[K_NUM_KERNELS] = {
    "sort_upsweep", "sort_scan", "sort_downsweep", "scan_reduce", "scan_spine", "scan_apply",
    "plan_keys", "plan_pairs", "plan_hist", "plan_occupancy", "plan_flags", "plan_lists", "plan_ring_jump",
    "plan_slots", "plan_group", "cache_evict", "cache_prefetch", "cache_stage", "cache_duplex", "embbag_fwd", "bwd_keys", "bwd_items", "bwd_reduce_update",
    "fill", "copy_calibration"};
}  // namespace

bool profile_events(int id, hipEvent_t* start, hipEvent_t* stop) {
    hipEvent_t a = get_event(), b = get_event();
    if (!a || !b) {
        if (a) g_free.push_back(a);
        if (b) g_free.push_back(b);
        return false;
    }
    g_spans.push_back(Span{id, a, b});
    *start = a;
    *stop = b;
    return true;
}

// A plain streaming copy of known size: the yardstick for byte counters (what FETCH_SIZE / WRITE_SIZE read for
// exactly `bytes` read and `bytes` written) and for the copy bandwidth this GPU sustains.
__global__ __launch_bounds__(256) void copy_calibration_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst,
                                                               size_t n16) {
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;      // one 16-byte piece per lane, exact grid
    if (i < n16) dst[i] = src[i];
}

// Randomly placed rows fetched U at a time per lane group (four is how the backward pass reads gradient rows), and
// folded into one word per lane so that the loads cannot be dropped.
template <int GW, int U>
__global__ __launch_bounds__(256) void gather_calibration_kernel(const uint4* __restrict__ table, uint32_t table_rows,
                                                                 int lpr, const uint32_t* __restrict__ rows, uint32_t n,
                                                                 uint4* __restrict__ sink) {
    const uint32_t t = blockIdx.x * 256u + threadIdx.x;
    const uint32_t group = t / GW;
    const int c = (int)(t % GW);
    uint4 acc = make_uint4(0, 0, 0, 0);
    const uint64_t first = (uint64_t)group * U;
    if (c < lpr && first < n) {
        uint32_t r[U];
#pragma unroll
        for (int j = 0; j < U; ++j) r[j] = first + j < n ? min(rows[first + j], table_rows - 1u) : 0u;
        uint4 v[U];
#pragma unroll
        for (int j = 0; j < U; ++j) v[j] = first + j < n ? table[(size_t)r[j] * lpr + c] : make_uint4(0, 0, 0, 0);
#pragma unroll
        for (int j = 0; j < U; ++j) {
            acc.x ^= v[j].x; acc.y ^= v[j].y; acc.z ^= v[j].z; acc.w ^= v[j].w;
        }
    }
#pragma unroll
    for (int off = GW / 2; off >= 1; off >>= 1) {     // one word per lane group leaves: the writes stay negligible
        acc.x ^= __shfl_xor(acc.x, off, GW); acc.y ^= __shfl_xor(acc.y, off, GW);
        acc.z ^= __shfl_xor(acc.z, off, GW); acc.w ^= __shfl_xor(acc.w, off, GW);
    }
    if (c == 0) sink[group] = acc;
}

struct GatherLaunch {
    const void* table;
    int64_t table_rows;
    int lpr;
    const uint32_t* rows;
    int64_t n;
    void* sink;
    hipStream_t stream;
    int in_flight;
    template <int GW, int U>
    int launch() {
        const int64_t threads = ceil_div(n, U) * GW;
        const int64_t blocks = ceil_div(threads, 256);
        if (blocks >= (int64_t(1) << 24)) return fail(BP_ERR_UNSUPPORTED, "gather of %lld rows is too large for one launch", (long long)n);
        BP_LAUNCH(K_COPY, (gather_calibration_kernel<GW, U>), dim3((unsigned)blocks), dim3(256), 0, stream,
                  (const uint4*)table, (uint32_t)table_rows, lpr, rows, (uint32_t)n, (uint4*)sink);
        return BP_OK;
    }
    template <int GW, bool BF16>
    int run() {
        switch (in_flight) {
            case 1: return launch<GW, 1>();
            case 2: return launch<GW, 2>();
            case 4: return launch<GW, 4>();
            case 8: return launch<GW, 8>();
            default: return fail(BP_ERR_INVALID_ARG, "rows_in_flight %d: 1, 2, 4 or 8", in_flight);
        }
    }
};

// The mirror image: rows written to randomly chosen places, U per lane group, with nothing read but the row numbers
// (how the forward pass over the plan's grouping writes the output rows of one-lookup bags).  A piece says which row,
// which piece and which list entry wrote it.
constexpr uint32_t kScatterMark = 0x5ca77e25u;
template <int GW, int U>
__global__ __launch_bounds__(256) void scatter_calibration_kernel(uint4* __restrict__ table, uint32_t table_rows, int lpr,
                                                                  const uint32_t* __restrict__ rows, uint32_t n) {
    const uint32_t t = blockIdx.x * 256u + threadIdx.x;
    const uint32_t group = t / GW;
    const int c = (int)(t % GW);
    const uint64_t first = (uint64_t)group * U;
    if (c >= lpr || first >= n) return;
    uint32_t r[U];
#pragma unroll
    for (int j = 0; j < U; ++j) r[j] = first + j < n ? rows[first + j] : table_rows;
#pragma unroll
    for (int j = 0; j < U; ++j)
        if (r[j] < table_rows) table[(size_t)r[j] * lpr + c] = make_uint4(r[j], (uint32_t)c, (uint32_t)(first + j), kScatterMark);
}

struct ScatterLaunch {
    void* table;
    int64_t table_rows;
    int lpr;
    const uint32_t* rows;
    int64_t n;
    hipStream_t stream;
    int in_flight;
    template <int GW, int U>
    int launch() {
        const int64_t threads = ceil_div(n, U) * GW;
        const int64_t blocks = ceil_div(threads, 256);
        if (blocks >= (int64_t(1) << 24)) return fail(BP_ERR_UNSUPPORTED, "scatter of %lld rows is too large for one launch", (long long)n);
        BP_LAUNCH(K_COPY, (scatter_calibration_kernel<GW, U>), dim3((unsigned)blocks), dim3(256), 0, stream, (uint4*)table,
                  (uint32_t)table_rows, lpr, rows, (uint32_t)n);
        return BP_OK;
    }
    template <int GW, bool BF16>
    int run() {
        switch (in_flight) {
            case 1: return launch<GW, 1>();
            case 2: return launch<GW, 2>();
            case 4: return launch<GW, 4>();
            default: return fail(BP_ERR_INVALID_ARG, "rows_in_flight %d: 1, 2 or 4", in_flight);
        }
    }
};

// Does nothing: what a pair of bracketing events reads around it is the cost of the bracket itself.
__global__ __launch_bounds__(64) void bracket_probe_kernel() {}

}  // namespace bp

using namespace bp;

BP_EXPORT const char* bp_error_string(int status) {
    switch (status) {
        case BP_OK: return "ok";
        case BP_ERR_INVALID_ARG: return "invalid argument";
        case BP_ERR_CAPACITY: return "cache capacity below one batch's unique rows";
        case BP_ERR_WORKSPACE_TOO_SMALL: return "workspace or list capacity too small";
        case BP_ERR_ID_OUT_OF_RANGE: return "id out of range";
        case BP_ERR_HIP: return "HIP runtime error";
        case BP_ERR_UNSUPPORTED: return "size beyond a documented limit";
        default: return "unknown status";
    }
}

BP_EXPORT const char* bp_last_error_message(void) { return t_error; }

BP_EXPORT int bp_version(void) { return 100; }

BP_EXPORT int bp_profile_bracket_overhead(void* stream_, int32_t reps, double* median_us) {
    hipStream_t stream = (hipStream_t)stream_;
    if (!median_us || reps < 1 || reps > 4096) return fail(BP_ERR_INVALID_ARG, "median_us is NULL or reps outside [1, 4096]");
    std::vector<hipEvent_t> ev(2 * (size_t)reps, nullptr);
    int st = BP_OK;
    for (auto& e : ev)
        if (hipEventCreate(&e) != hipSuccess) st = fail(BP_ERR_HIP, "hipEventCreate failed");
    if (st == BP_OK) {
        for (int r = 0; r < reps; ++r) {
            hipExtLaunchKernelGGL(bracket_probe_kernel, dim3(1), dim3(64), 0, stream, ev[2 * r], ev[2 * r + 1], 0);
        }
        if (hipStreamSynchronize(stream) != hipSuccess) st = fail(BP_ERR_HIP, "hipStreamSynchronize failed");
    }
    if (st == BP_OK) {
        std::vector<float> ms((size_t)reps, 0.f);
        for (int r = 0; r < reps; ++r) (void)hipEventElapsedTime(&ms[r], ev[2 * r], ev[2 * r + 1]);
        std::nth_element(ms.begin(), ms.begin() + reps / 2, ms.end());
        *median_us = (double)ms[reps / 2] * 1e3;
    }
    for (auto e : ev)
        if (e) (void)hipEventDestroy(e);
    return st;
}

BP_EXPORT int bp_copy_calibration(void* dst, const void* src, size_t bytes, void* stream) {
    if (!dst || !src || bytes % 16 != 0 || (((uintptr_t)dst | (uintptr_t)src) & 15))
        return fail(BP_ERR_INVALID_ARG, "copy needs 16-byte aligned pointers and a multiple of 16 bytes");
    if (bytes == 0) return BP_OK;
    const size_t n16 = bytes / 16;
    const size_t blocks = (n16 + 255) / 256;
    if (blocks >= (size_t(1) << 31)) return fail(BP_ERR_UNSUPPORTED, "copy of %zu bytes is too large for one launch", bytes);
    BP_LAUNCH(K_COPY, copy_calibration_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream,
              (const uint4*)src, (uint4*)dst, n16);
    return BP_OK;
}

BP_EXPORT int bp_gather_calibration(void* sink, const void* table, int64_t table_rows, int32_t row_bytes,
                                    const uint32_t* rows, int64_t n, int32_t rows_in_flight, void* stream) {
    if (!sink || !table || !rows || (((uintptr_t)sink | (uintptr_t)table) & 15))
        return fail(BP_ERR_INVALID_ARG, "gather needs 16-byte aligned table and sink and a row list");
    if (row_bytes < 16 || row_bytes > 1024 || row_bytes % 16 != 0)
        return fail(BP_ERR_INVALID_ARG, "row_bytes %d: a multiple of 16 in [16, 1024]", row_bytes);
    if (table_rows < 1 || table_rows >= (int64_t(1) << 32) || n < 0 || n >= (int64_t(1) << 31))
        return fail(BP_ERR_INVALID_ARG, "table_rows or n out of range");
    if (n == 0) return BP_OK;
    if (rows_in_flight != 1 && rows_in_flight != 2 && rows_in_flight != 4 && rows_in_flight != 8)
        return fail(BP_ERR_INVALID_ARG, "rows_in_flight %d: 1, 2, 4 or 8", rows_in_flight);
    GatherLaunch l{table, table_rows, row_bytes / 16, rows, n, sink, (hipStream_t)stream, rows_in_flight};
    return dispatch_row(row_bytes / 16, false, l);
}

BP_EXPORT int bp_scatter_calibration(void* table, int64_t table_rows, int32_t row_bytes, const uint32_t* rows, int64_t n,
                                     int32_t rows_in_flight, void* stream) {
    if (!table || !rows || ((uintptr_t)table & 15))
        return fail(BP_ERR_INVALID_ARG, "scatter needs a 16-byte aligned table and a row list");
    if (row_bytes < 16 || row_bytes > 1024 || row_bytes % 16 != 0)
        return fail(BP_ERR_INVALID_ARG, "row_bytes %d: a multiple of 16 in [16, 1024]", row_bytes);
    if (table_rows < 1 || table_rows >= (int64_t(1) << 32) || n < 0 || n >= (int64_t(1) << 31))
        return fail(BP_ERR_INVALID_ARG, "table_rows or n out of range");
    if (n == 0) return BP_OK;
    if (rows_in_flight != 1 && rows_in_flight != 2 && rows_in_flight != 4)
        return fail(BP_ERR_INVALID_ARG, "rows_in_flight %d: 1, 2 or 4", rows_in_flight);
    ScatterLaunch l{table, table_rows, row_bytes / 16, rows, n, (hipStream_t)stream, rows_in_flight};
    return dispatch_row(row_bytes / 16, false, l);
}

BP_EXPORT int bp_profile_enable(int on) {
    if (on) {
        for (auto& s : g_spans) {
            g_free.push_back(s.a);
            g_free.push_back(s.b);
        }
        g_spans.clear();
        std::memset(g_count, 0, sizeof(g_count));
        std::memset(g_ms, 0, sizeof(g_ms));
        for (auto& v : g_samples) v.clear();
    }
    g_profile_on = on != 0;
    return BP_OK;
}

BP_EXPORT int bp_profile_select(uint64_t kernel_mask) {
    g_profile_mask = kernel_mask;
    return BP_OK;
}

BP_EXPORT int bp_profile_collect(void) {
    for (auto& s : g_spans) {
        BP_HIP(hipEventSynchronize(s.b));
        float ms = 0.f;
        BP_HIP(hipEventElapsedTime(&ms, s.a, s.b));
        g_count[s.id] += 1;
        g_ms[s.id] += ms;
        g_samples[s.id].push_back(ms);
        g_free.push_back(s.a);
        g_free.push_back(s.b);
    }
    g_spans.clear();
    return BP_OK;
}

BP_EXPORT int bp_profile_spread(int id, double* min_ms, double* median_ms, double* max_ms) {
    if (id < 0 || id >= K_NUM_KERNELS) return fail(BP_ERR_INVALID_ARG, "kernel id %d out of range", id);
    std::vector<float> v = g_samples[id];
    if (v.empty()) return fail(BP_ERR_INVALID_ARG, "no recorded launch of kernel %d", id);
    std::sort(v.begin(), v.end());
    if (min_ms) *min_ms = v.front();
    if (max_ms) *max_ms = v.back();
    if (median_ms) *median_ms = v.size() % 2 ? v[v.size() / 2] : 0.5 * (v[v.size() / 2 - 1] + v[v.size() / 2]);
    return BP_OK;
}

BP_EXPORT int bp_profile_num_kernels(void) { return K_NUM_KERNELS; }

BP_EXPORT const char* bp_profile_kernel_name(int id) {
    return id >= 0 && id < K_NUM_KERNELS ? kKernelNames[id] : "";
}

BP_EXPORT int bp_profile_get(int id, int64_t* launches, double* total_ms) {
    if (id < 0 || id >= K_NUM_KERNELS) return fail(BP_ERR_INVALID_ARG, "kernel id %d out of range", id);
    if (launches) *launches = g_count[id];
    if (total_ms) *total_ms = g_ms[id];
    return BP_OK;
}
