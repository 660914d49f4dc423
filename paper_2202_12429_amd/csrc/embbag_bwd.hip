// bp_embbag_bwd_update: deterministic backward + fused sparse optimizer step on cached rows.
//
// Gradients, not embeddings, are combined (Section 6), so any per-row optimizer can follow; the update
// rules are SGD, element-wise Adagrad and row-wise Adagrad.
//
//   1. keys = slot of every lookup, payload = its bag; stable LSD radix sort on the slot bits, so the
//      lookups of a slot end up adjacent and in lookup order.
//   2. the sorted array is cut into work items: a new item starts at every change of slot and at every
//      multiple of kChunk positions (so a slot hit thousands of times by a skewed batch is shared by
//      many lane groups); item starts are compacted with a scan.
//   3. one lane group per item adds its gradient rows in order (fp64 accumulators).  An item that covers its whole
//      slot applies the update at once; so does the first item of a slot that crosses a single cut (it carries on
//      to the slot's end and the second item steps aside); otherwise the sum goes to a partial row addressed by
//      the chunk boundary it touches.
//   4. for slots split over several items, one wavefront adds the partial rows (lane groups round-robin,
//      then a butterfly across the groups) and applies the update.
// Every order of addition is fixed by the data, never by timing: results are bit-identical run to run.
// The summed gradient is rounded to fp32 once; the optimizer step itself is fp32 arithmetic.
#include "common.h"
#include "device_prims.h"
#include "row_access.h"

namespace bp {
namespace {

constexpr int kChunk = kBwdChunk;  // sorted positions per work item at most
constexpr int kMaxGridBlocks = 8192;

// ---- 1. keys ---------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void bwd_keys_kernel(const int32_t* __restrict__ slots, const int64_t* __restrict__ bag_off,
                                                       int64_t n, int64_t bags, int64_t C, uint32_t* __restrict__ keys,
                                                       uint32_t* __restrict__ vals) {
    const int64_t k = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (k >= n) return;
    const uint32_t s = (uint32_t)slots[k];
    keys[k] = s < (uint64_t)C ? s : (uint32_t)C;     // out-of-range slots sort behind every real one
    uint32_t bag = (uint32_t)k;
    if (bag_off) {                                   // largest b with bag_off[b] <= k
        int64_t lo = 0, hi = bags;                   // bag_off[lo] <= k < bag_off[hi]
        while (hi - lo > 1) {
            const int64_t mid = (lo + hi) >> 1;
            if (bag_off[mid] <= k) lo = mid; else hi = mid;
        }
        bag = (uint32_t)lo;
    }
    vals[k] = bag;
}

// Grouped variant: the plan lists lookup positions grouped by row; the gradient row of a position is its bag.
// First every bag writes its number over its own stretch of positions (neighbouring lanes write neighbouring
// stretches), then the grouped positions pick their bag up from that map, which stays in L2.
__global__ __launch_bounds__(256) void bwd_bag_of_lookup_kernel(const int64_t* __restrict__ bag_off, int64_t bags, int64_t n,
                                                                uint32_t* __restrict__ bag_of_lookup) {
    const int64_t b = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (b >= bags) return;
    int64_t k = bag_off[b], end = bag_off[b + 1];
    if (k < 0) k = 0;
    if (end > n) end = n;
    for (; k < end; ++k) bag_of_lookup[k] = (uint32_t)b;
}

__global__ __launch_bounds__(256) void bwd_bags_of_positions_kernel(const int32_t* __restrict__ positions,
                                                                    const uint32_t* __restrict__ bag_of_lookup, int64_t n,
                                                                    int64_t bags, uint32_t* __restrict__ bag_of) {
    const int64_t p = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (p >= n) return;
    const uint32_t k = (uint32_t)positions[p];
    const uint32_t b = k < (uint64_t)n ? bag_of_lookup[k] : 0u;
    bag_of[p] = b < (uint64_t)bags ? b : 0u;      // offsets that do not cover every lookup leave holes in the map
}

// ---- 2. work items ---------------------------------------------------------------------------
struct ItemStartIn {
    const uint32_t* keys;
    __device__ __forceinline__ uint32_t operator()(int64_t p) const {
        return (p == 0 || (p % kChunk) == 0 || keys[p] != keys[p - 1]) ? 1u : 0u;
    }
};
// An item record is the position of the item's first sorted lookup, with bit 31 set when that lookup is the first
// of its slot.  Everything else a kernel needs to know about an item follows from its neighbours' records: the item
// ends where the next one starts, and it is the last of its slot iff the next item is a first.
constexpr uint32_t kItemHead = 0x80000000u, kItemPos = 0x7fffffffu;

struct ItemStartOut {
    const uint32_t* keys;
    uint32_t* item_start;
    __device__ __forceinline__ void operator()(int64_t p, uint32_t exc, uint32_t inc) const {
        if (inc != exc) item_start[exc] = (uint32_t)p | ((p == 0 || keys[p] != keys[p - 1]) ? kItemHead : 0u);
    }
};

// ---- 3./4. reduce and update -----------------------------------------------------------------
struct UpdateParams {
    int optimizer;
    float lr, eps;
    int lpr;
    int dim;
    uint32_t bags;      // rows of the upstream gradient: a bag number beyond them reads row 0 instead
};

// Running sum of one 16-byte piece of gradient rows.  Sums are carried in fp64 and rounded to fp32 once,
// which makes the result independent of how a slot's lookups were cut into items (fp64 addition of
// fp32 values is exact until the partial sums outgrow 53 bits); everything after the sum is fp32.
template <int N>
struct SumPiece {
    double v[N];
    __device__ __forceinline__ void zero() {
#pragma unroll
        for (int i = 0; i < N; ++i) v[i] = 0.0;
    }
    template <bool BF16>
    __device__ __forceinline__ void add(const Piece<BF16>& p) {
#pragma unroll
        for (int i = 0; i < N; ++i) v[i] += (double)p.v[i];
    }
    __device__ __forceinline__ void add(const SumPiece& o) {
#pragma unroll
        for (int i = 0; i < N; ++i) v[i] += o.v[i];
    }
    // fp64 [.. D] partial rows: the piece of lane c starts at element c * N
    __device__ __forceinline__ void load(const double* row, int c) {
        const double2* p = reinterpret_cast<const double2*>(row + (size_t)c * N);
#pragma unroll
        for (int i = 0; i < N / 2; ++i) {
            const double2 t = p[i];
            v[2 * i] = t.x; v[2 * i + 1] = t.y;
        }
    }
    __device__ __forceinline__ void store(double* row, int c) const {
        double2* p = reinterpret_cast<double2*>(row + (size_t)c * N);
#pragma unroll
        for (int i = 0; i < N / 2; ++i) p[i] = make_double2(v[2 * i], v[2 * i + 1]);
    }
    template <bool BF16>
    __device__ __forceinline__ Piece<BF16> rounded() const {
        Piece<BF16> p;
#pragma unroll
        for (int i = 0; i < N; ++i) p.v[i] = (float)v[i];
        return p;
    }
};

template <int GW>
__device__ __forceinline__ double group_sum(double x) {
#pragma unroll
    for (int off = GW / 2; off >= 1; off >>= 1) x += __shfl_xor(x, off, GW);
    return x;
}

// The piece of lane c of row `slot` and of its optimizer state, loaded ahead of the gradient sum so that the row's
// latency hides behind the gradient loads.
template <bool BF16>
struct RowPiece {
    uint4 w_raw;
    Piece<BF16> s;       // element-wise Adagrad state
    float s_row;         // row-wise Adagrad state
};

template <bool BF16>
__device__ __forceinline__ RowPiece<BF16> load_row(const UpdateParams& u, const uint4* cache_w, const float* cache_s,
                                                   int64_t slot, int c, bool active) {
    RowPiece<BF16> r;
    r.w_raw = make_uint4(0, 0, 0, 0);
    r.s.zero();
    r.s_row = 0.f;
    if (active) {
        r.w_raw = cache_w[slot * u.lpr + c];
        if (u.optimizer == BP_ADAGRAD) r.s.load_f32(cache_s + slot * u.dim, c);
    }
    if (u.optimizer == BP_ADAGRAD_ROWWISE) r.s_row = cache_s[slot];
    return r;
}

// Applies one optimizer step to the piece of lane c of row `slot`; g is the row's summed gradient in fp32, r the
// piece as loaded by load_row.  All lanes of the group call this (the row-wise rule reduces over the group); lanes
// with c >= lpr carry zeros and touch no memory, and neither do the lanes of a group that is not the writer.
// One fp32 operation per statement: step = lr*g, then for Adagrad s += g*g, den = sqrt(s) + eps, step /= den,
// and w -= step.
template <int GW, bool BF16>
__device__ __forceinline__ void finish_update(const UpdateParams& u, uint4* cache_w, float* cache_s, int64_t slot, int c,
                                              const RowPiece<BF16>& r, const Piece<BF16>& g, bool active) {
    constexpr int N = Piece<BF16>::N;
    Piece<BF16> w;
    w.decode(r.w_raw);
    if (u.optimizer == BP_SGD) {
#pragma unroll
        for (int i = 0; i < N; ++i) {
            const float step = u.lr * g.v[i];
            w.v[i] = w.v[i] - step;
        }
    } else if (u.optimizer == BP_ADAGRAD) {
        Piece<BF16> s = r.s;
#pragma unroll
        for (int i = 0; i < N; ++i) {
            const float gg = g.v[i] * g.v[i];
            s.v[i] = s.v[i] + gg;
            const float den = sqrtf(s.v[i]) + u.eps;
            const float step = (u.lr * g.v[i]) / den;
            w.v[i] = w.v[i] - step;
        }
        if (active) s.store_f32(cache_s + slot * u.dim, c);
    } else {
        double ss = 0.0;                       // mean of squares over the row: an fp64 sum, rounded once
#pragma unroll
        for (int i = 0; i < N; ++i) ss += (double)g.v[i] * (double)g.v[i];
        ss = group_sum<GW>(ss);
        const float mean = (float)(ss / (double)u.dim);
        const float s = r.s_row + mean;
        const float den = sqrtf(s) + u.eps;
#pragma unroll
        for (int i = 0; i < N; ++i) {
            const float step = (u.lr * g.v[i]) / den;
            w.v[i] = w.v[i] - step;
        }
        if (c == 0 && active) cache_s[slot] = s;
    }
    if (active) cache_w[slot * u.lpr + c] = w.encode();
}

template <int GW, bool BF16>
__device__ __forceinline__ void apply_update(const UpdateParams& u, uint4* cache_w, float* cache_s, int64_t slot, int c,
                                             const Piece<BF16>& g, bool writer = true) {
    const bool active = c < u.lpr && writer;
    const RowPiece<BF16> r = load_row<BF16>(u, cache_w, cache_s, slot, c, active);
    finish_update<GW, BF16>(u, cache_w, cache_s, slot, c, r, g, active);
}

// One lane group per work item.  Loads are issued as early as their addresses are known: the item's records
// together, then its slot and the first gradient indices together, then the cache row and the gradient rows.
template <int GW, bool BF16>
__global__ __launch_bounds__(kRowBlock) void bwd_reduce_update_kernel(const uint32_t* __restrict__ keys,
                                                                     const uint32_t* __restrict__ bag_of,
                                                                     const uint32_t* __restrict__ item_start,
                                                                     const uint32_t* __restrict__ n_items_ptr,
                                                                     uint32_t n_items_host, uint32_t n, int64_t C,
                                                                     const float* __restrict__ grad,
                                                                     uint4* cache_w, float* cache_s, double* partial,
                                                                     UpdateParams u) {
    constexpr int N = Piece<BF16>::N;
    const uint32_t W = n_items_ptr ? *n_items_ptr : n_items_host;   // counted on the device, or known to the host
    const int c = threadIdx.x % GW;
    const bool active = c < u.lpr;
    const uint32_t groups = gridDim.x * (kRowBlock / GW);
    for (uint32_t w = (blockIdx.x * kRowBlock + threadIdx.x) / GW; w < W; w += groups) {
        const uint32_t rp = item_start[w > 0 ? w - 1 : 0];
        const uint32_t r0 = item_start[w];
        const uint32_t r1 = w + 1 < W ? item_start[w + 1] : (n | kItemHead);
        const uint32_t r2 = w + 2 < W ? item_start[w + 2] : (n | kItemHead);
        const uint32_t start = r0 & kItemPos, end = r1 & kItemPos;
        const bool head = (r0 & kItemHead) != 0, tail = (r1 & kItemHead) != 0;
        // A row that crosses exactly one cut (it starts in one chunk and ends in the next) is finished by its first
        // item alone: that item carries on to the row's end, the second item steps aside.  Only rows that cross two
        // cuts or more go through partial sums.
        const bool takes_next = head && !tail && (r2 & kItemHead);     // the row's second item is its last
        const bool steps_aside = !head && tail && (rp & kItemHead);    // second of two: the first item does it all
        const uint32_t last = takes_next ? (r2 & kItemPos) : end;
        const bool whole = (head && tail) || takes_next;
        if (start >= n || last > n || last < start) continue;           // a malformed record reads nothing
        const uint32_t slot = keys[start];
        uint32_t idx[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) idx[j] = start + j < last ? bag_of[start + j] : 0u;
        if (steps_aside || (int64_t)slot >= C) continue;               // slot C: sentinel of out-of-range slots
        RowPiece<BF16> row;
        if (whole) row = load_row<BF16>(u, cache_w, cache_s, (int64_t)slot, c, active);
        SumPiece<N> acc;
        acc.zero();
        if (active) {
            // bursts of four rows; the indices of the next burst are loaded while the rows of this one arrive
            for (uint32_t p = start; p < last; p += 4) {
                Piece<BF16> t[4];
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (p + j < last) t[j].load_f32(grad + (size_t)min(idx[j], u.bags - 1u) * u.dim, c);   // clamped where it is used: the index load stays in flight until then
#pragma unroll
                for (int j = 0; j < 4; ++j) idx[j] = p + 4 + j < last ? bag_of[p + 4 + j] : 0u;
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (p + j < last) acc.add(t[j]);
            }
        }
        if (whole) {
            finish_update<GW, BF16>(u, cache_w, cache_s, (int64_t)slot, c, row, acc.template rounded<BF16>(), active);
        } else if (active) {
            // head item of a split slot ends on a chunk boundary b*kChunk: row 2b; a later item starts on
            // boundary b*kChunk: row 2b+1
            const size_t prow = head ? 2 * (size_t)(end / kChunk) : 2 * (size_t)(start / kChunk) + 1;
            acc.store(partial + prow * u.dim, c);
        }
    }
}

// Split slots: one wavefront per slot.  Its 64/GW lane groups take the slot's partial rows round-robin
// (row 2b of the head item goes to group 0, row 2b'+1 of the item starting at boundary b' to group
// (b' - b) mod groups), each adds its share in order with four loads in flight, and the group sums are added
// across the wavefront by a butterfly whose order is fixed by the lane numbers.  Every group then holds the
// slot's gradient; group 0 writes the update.
template <int GW, bool BF16>
__global__ __launch_bounds__(kRowBlock) void bwd_combine_update_kernel(const uint32_t* __restrict__ keys,
                                                                      const uint32_t* __restrict__ item_start,
                                                                      const uint32_t* __restrict__ n_items_ptr,
                                                                      uint32_t n_items_host, uint32_t n, int64_t C,
                                                                      uint4* cache_w, float* cache_s,
                                                                      const double* __restrict__ partial, UpdateParams u) {
    constexpr int N = Piece<BF16>::N;
    constexpr int G = kWave / GW;                     // lane groups per wavefront
    const uint32_t W = n_items_ptr ? *n_items_ptr : n_items_host;   // counted on the device, or known to the host
    const int lane = threadIdx.x % kWave;
    const int c = lane % GW, j = lane / GW;
    const bool active = c < u.lpr;
    const uint32_t waves = gridDim.x * (kRowBlock / kWave);
    for (uint32_t w = (blockIdx.x * kRowBlock + threadIdx.x) / kWave; w < W; w += waves) {
        const uint32_t r0 = item_start[w];
        const uint32_t r1 = w + 1 < W ? item_start[w + 1] : (n | kItemHead);
        if (!(r0 & kItemHead) || (r1 & kItemHead)) continue;   // only the first item of a split slot works here
        const uint32_t r2 = w + 2 < W ? item_start[w + 2] : (n | kItemHead);
        if (r2 & kItemHead) continue;                           // crosses one cut only: done by the reduce kernel
        const uint32_t start = r0 & kItemPos, end = r1 & kItemPos;
        const uint32_t slot = keys[start];
        if ((int64_t)slot >= C) continue;
        SumPiece<N> acc;
        acc.zero();
        const uint32_t b0 = end / kChunk;             // end is a chunk boundary because the slot goes on
        if (active && j == 0) acc.load(partial + 2 * (size_t)b0 * u.dim, c);
        // the item starting at boundary b belongs to this slot iff b*kChunk < n and keys[b*kChunk] == slot
        for (uint64_t b = (uint64_t)b0 + j;; b += 4 * G) {
            bool ok[4];
            SumPiece<N> t[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const uint64_t bb = b + (uint64_t)k * G;
                // the key test and the partial row are loaded side by side (row 2bb+1 exists whenever
                // bb*kChunk < n; a row that turns out not to belong to the slot is dropped): one latency per round
                const bool inb = bb * kChunk < n;
                const uint32_t key = inb ? keys[bb * kChunk] : ~0u;
                t[k].zero();
                if (inb && active) t[k].load(partial + (2 * bb + 1) * u.dim, c);
                ok[k] = inb && key == slot;
            }
#pragma unroll
            for (int k = 0; k < 4; ++k)
                if (ok[k]) acc.add(t[k]);
            if (!ok[3]) break;                        // the slot's boundaries are consecutive
        }
#pragma unroll
        for (int off = GW; off < kWave; off <<= 1) {
#pragma unroll
            for (int i = 0; i < N; ++i) acc.v[i] += __shfl_xor(acc.v[i], off, kWave);
        }
        apply_update<GW, BF16>(u, cache_w, cache_s, (int64_t)slot, c, acc.template rounded<BF16>(), j == 0);
    }
}

// Split rows when the plan lists them: one workgroup per split row.  Its 256/GW lane groups take the row's partial
// sums round-robin as above; the group sums meet in LDS and every group adds them in group order, so all hold the
// row's gradient and group 0 writes the update.  No idle wavefronts: the grid is the list.
template <int GW, bool BF16>
__global__ __launch_bounds__(kRowBlock) void bwd_combine_split_kernel(const uint32_t* __restrict__ keys,
                                                                     const uint32_t* __restrict__ split_starts, uint32_t n,
                                                                     int64_t C, uint4* cache_w, float* cache_s,
                                                                     const double* __restrict__ partial, UpdateParams u) {
    constexpr int N = Piece<BF16>::N;
    constexpr int G = kRowBlock / GW;                 // lane groups per workgroup
    constexpr int U = G >= 64 ? 1 : (G >= 32 ? 2 : 4);  // partial rows in flight per group: about 64 per round
    __shared__ double red[G][N][GW];
    const int c = threadIdx.x % GW, j = threadIdx.x / GW;
    const bool active = c < u.lpr;
    const uint32_t start = split_starts[blockIdx.x];
    if (start >= n) return;
    const uint32_t slot = keys[start];
    if ((int64_t)slot >= C) return;
    const uint32_t b0 = start / kChunk + 1;           // the row's first item ends at the next cut after `start`
    // the row itself is asked for now, so that it arrives while the partial sums are added up
    const bool writer = active && j == 0;
    const RowPiece<BF16> row = load_row<BF16>(u, cache_w, cache_s, (int64_t)slot, c, writer);
    SumPiece<N> acc;
    acc.zero();
    if (active && j == 0) acc.load(partial + 2 * (size_t)b0 * u.dim, c);
    for (uint64_t b = (uint64_t)b0 + j;; b += U * G) {
        bool ok[U];
        SumPiece<N> t[U];
#pragma unroll
        for (int k = 0; k < U; ++k) {
            const uint64_t bb = b + (uint64_t)k * G;
            // the key test and the partial row are loaded side by side (row 2bb+1 exists whenever
            // bb*kChunk < n; a row that turns out not to belong to the slot is dropped): one latency per round
            const bool inb = bb * kChunk < n;
            const uint32_t key = inb ? keys[bb * kChunk] : ~0u;
            t[k].zero();
            if (inb && active) t[k].load(partial + (2 * bb + 1) * u.dim, c);
            ok[k] = inb && key == slot;
        }
#pragma unroll
        for (int k = 0; k < U; ++k)
            if (ok[k]) acc.add(t[k]);
        if (!ok[U - 1]) break;
    }
#pragma unroll
    for (int i = 0; i < N; ++i) red[j][i][c] = acc.v[i];
    __syncthreads();
    acc.zero();
    for (int g = 0; g < G; ++g) {
#pragma unroll
        for (int i = 0; i < N; ++i) acc.v[i] += red[g][i][c];
    }
    finish_update<GW, BF16>(u, cache_w, cache_s, (int64_t)slot, c, row, acc.template rounded<BF16>(), writer);
}

// ---- workspace -------------------------------------------------------------------------------
constexpr int kSmallIPT = 4, kLargeIPT = 16;
constexpr int64_t kLargeSort = int64_t(1) << 21;

struct BwdWorkspace {
    uint32_t *keys_a, *keys_b, *vals_a, *vals_b, *sort_temp, *item_start, *scan_partials;
    double* partial;
    size_t bytes;
};

BwdWorkspace carve_bwd(void* base, size_t cap, int64_t n, int dim) {
    Carver c(base, cap);
    BwdWorkspace w{};
    const size_t m = (size_t)(n > 0 ? n : 1);
    w.keys_a = c.take<uint32_t>(m);
    w.keys_b = c.take<uint32_t>(m);
    w.vals_a = c.take<uint32_t>(m);
    w.vals_b = c.take<uint32_t>(m);
    w.sort_temp = c.take<uint32_t>(n >= kLargeSort ? sort_temp_words<kLargeIPT>(n) : sort_temp_words<kSmallIPT>(n));
    w.item_start = c.take<uint32_t>(m + 1);
    w.scan_partials = c.take<uint32_t>(scan_partials(n));
    w.partial = c.take<double>((2 * (m / kChunk + 2)) * (size_t)dim);
    w.bytes = c.used();
    return w;
}

struct BwdLaunch {
    const bp_config* cfg;
    double* partial;
    const uint32_t *skeys, *sbags, *item_start;
    const uint32_t* n_items;       // device count, or NULL when n_items_host is given
    uint32_t n_items_host;
    const uint32_t* split_starts;  // list of split rows (grouped path), or NULL: find them item by item
    uint32_t n_split;
    int64_t n;
    const float* grad;
    void* cache_w;
    void* cache_s;
    hipStream_t stream;
    int64_t bags;
    template <int GW, bool BF16>
    int run() {
        UpdateParams u{cfg->optimizer, cfg->lr, cfg->eps, (int)(row_bytes(cfg) / 16), cfg->dim,
                       (uint32_t)(bags > 0 ? bags : 1)};
        const int groups_per_block = kRowBlock / GW;
        const int64_t items_bound = n_items ? n : (int64_t)n_items_host;     // at most one item per lookup
        int64_t blocks = ceil_div(items_bound, groups_per_block);
        if (blocks > kMaxGridBlocks) blocks = kMaxGridBlocks;
        if (blocks < 1) blocks = 1;
        BP_LAUNCH(K_BWD_REDUCE_UPDATE, (bwd_reduce_update_kernel<GW, BF16>), dim3((unsigned)blocks), dim3(kRowBlock), 0, stream,
                  skeys, sbags, item_start, n_items, n_items_host, (uint32_t)n, cfg->capacity, grad, (uint4*)cache_w,
                  (float*)cache_s, partial, u);
        if (n_items == nullptr) {                                            // grouped path: the plan lists the split rows
            if (n_split)
                BP_LAUNCH(K_BWD_COMBINE_UPDATE, (bwd_combine_split_kernel<GW, BF16>), dim3(n_split), dim3(kRowBlock), 0,
                          stream, skeys, split_starts, (uint32_t)n, cfg->capacity, (uint4*)cache_w, (float*)cache_s,
                          (const double*)partial, u);
            return BP_OK;
        }
        int64_t cblocks = ceil_div(items_bound, kRowBlock / kWave);          // one wavefront per item
        if (cblocks < 1) cblocks = 1;
        if (cblocks > kMaxGridBlocks) cblocks = kMaxGridBlocks;
        BP_LAUNCH(K_BWD_COMBINE_UPDATE, (bwd_combine_update_kernel<GW, BF16>), dim3((unsigned)cblocks), dim3(kRowBlock), 0,
                  stream, skeys, item_start, n_items, n_items_host, (uint32_t)n, cfg->capacity, (uint4*)cache_w,
                  (float*)cache_s, (const double*)partial, u);
        return BP_OK;
    }
};

int check_bwd_args(const bp_config* cfg, int64_t n, int64_t bags) {
    BP_TRY(check_config(cfg));
    if (n < 0 || bags < 0) return fail(BP_ERR_INVALID_ARG, "negative size");
    if (n >= (int64_t(1) << 31) || bags >= (int64_t(1) << 31)) return fail(BP_ERR_UNSUPPORTED, "size >= 2^31");
    return BP_OK;
}

}  // namespace
}  // namespace bp

using namespace bp;

BP_EXPORT int bp_embbag_bwd_update_workspace_bytes(const bp_config* cfg, int64_t n_lookups, int64_t bags, size_t* bytes) {
    if (!bytes) return fail(BP_ERR_INVALID_ARG, "bytes is NULL");
    BP_TRY(check_bwd_args(cfg, n_lookups, bags));
    *bytes = carve_bwd(nullptr, 0, n_lookups, cfg->dim).bytes;
    return BP_OK;
}

BP_EXPORT int bp_embbag_bwd_update(const bp_config* cfg, void* cache_w, void* cache_state, const int32_t* lookup_slots,
                                    const int64_t* bag_offsets, int64_t n_lookups, int64_t bags, const float* grad_out,
                                    void* workspace, size_t workspace_bytes, void* stream_) {
    hipStream_t stream = (hipStream_t)stream_;
    const int64_t n = n_lookups;
    BP_TRY(check_bwd_args(cfg, n, bags));
    if (n == 0) return BP_OK;
    if (!bag_offsets && n != bags)
        return fail(BP_ERR_INVALID_ARG, "bag_offsets is NULL but n_lookups %lld != bags %lld", (long long)n, (long long)bags);
    if (!cache_w || !lookup_slots || !grad_out) return fail(BP_ERR_INVALID_ARG, "NULL pointer");
    if (cfg->optimizer != BP_SGD && !cache_state) return fail(BP_ERR_INVALID_ARG, "cache_state is NULL");
    if (((uintptr_t)cache_w | (uintptr_t)cache_state | (uintptr_t)grad_out) & 15)
        return fail(BP_ERR_INVALID_ARG, "cache_w, cache_state and grad_out must be 16-byte aligned");
    if (!workspace || ((uintptr_t)workspace & 255)) return fail(BP_ERR_INVALID_ARG, "workspace NULL or not 256-byte aligned");
    BwdWorkspace w = carve_bwd(workspace, workspace_bytes, n, cfg->dim);
    if (w.bytes > workspace_bytes)
        return fail(BP_ERR_WORKSPACE_TOO_SMALL, "workspace %zu < required %zu bytes", workspace_bytes, w.bytes);

    BP_LAUNCH(K_BWD_KEYS, bwd_keys_kernel, dim3((unsigned)ceil_div(n, 256)), dim3(256), 0, stream, lookup_slots, bag_offsets, n,
              bags, cfg->capacity, w.keys_a, w.vals_a);
    bool in_b = false;
    const int key_bits = bits_for(cfg->capacity + 1);
    if (n >= kLargeSort)
        BP_TRY((radix_sort_pairs<uint32_t, kLargeIPT>(w.keys_a, w.keys_b, w.vals_a, w.vals_b, n, 0, key_bits, w.sort_temp,
                                                      stream, &in_b)));
    else
        BP_TRY((radix_sort_pairs<uint32_t, kSmallIPT>(w.keys_a, w.keys_b, w.vals_a, w.vals_b, n, 0, key_bits, w.sort_temp,
                                                      stream, &in_b)));
    const uint32_t* skeys = in_b ? w.keys_b : w.keys_a;
    const uint32_t* sbags = in_b ? w.vals_b : w.vals_a;

    BP_TRY((device_scan<uint32_t, AddOp, ItemStartIn, ItemStartOut>(ItemStartIn{skeys}, ItemStartOut{skeys, w.item_start}, n,
                                                                    w.scan_partials, AddOp(), 0u, stream)));
    const uint32_t* n_items = w.scan_partials + scan_num_tiles(n);

    BwdLaunch l{cfg, w.partial, skeys, sbags, w.item_start, n_items, 0u, nullptr, 0u, n, grad_out, cache_w, cache_state, stream, bags};
    return dispatch_row((int)(row_bytes(cfg) / 16), cfg->weight_dtype == BP_BF16, l);
}

// ---- grouped variant: the plan already lists the batch's lookups grouped by row ---------------------------------
namespace bp {
namespace {
struct GroupedWorkspace {
    uint32_t* bag_of;          // bag of every grouped position
    uint32_t* bag_of_lookup;   // bag of every lookup, in lookup order
    double* partial;
    size_t bytes;
};
GroupedWorkspace carve_grouped(void* base, size_t cap, int64_t n, int dim, bool multi_hot) {
    Carver c(base, cap);
    GroupedWorkspace w{};
    const size_t m = (size_t)(n > 0 ? n : 1);
    w.bag_of = multi_hot ? c.take<uint32_t>(m) : nullptr;
    w.bag_of_lookup = multi_hot ? c.take<uint32_t>(m) : nullptr;
    w.partial = c.take<double>((2 * (m / kChunk + 2)) * (size_t)dim);
    w.bytes = c.used();
    return w;
}
}  // namespace
}  // namespace bp

BP_EXPORT int bp_embbag_bwd_update_grouped_workspace_bytes(const bp_config* cfg, int64_t n_lookups, int64_t bags,
                                                           int32_t multi_hot, size_t* bytes) {
    if (!bytes) return fail(BP_ERR_INVALID_ARG, "bytes is NULL");
    BP_TRY(check_bwd_args(cfg, n_lookups, bags));
    *bytes = carve_grouped(nullptr, 0, n_lookups, cfg->dim, multi_hot != 0).bytes;
    return BP_OK;
}

BP_EXPORT int bp_embbag_bwd_update_grouped(const bp_config* cfg, void* cache_w, void* cache_state,
                                           const int32_t* grouped_slots, const int32_t* grouped_lookups,
                                           const uint32_t* item_starts, int64_t n_items, const uint32_t* split_starts,
                                           int64_t n_split, const int64_t* bag_offsets,
                                           int64_t n_lookups, int64_t bags, const float* grad_out, void* workspace,
                                           size_t workspace_bytes, void* stream_) {
    hipStream_t stream = (hipStream_t)stream_;
    const int64_t n = n_lookups;
    BP_TRY(check_bwd_args(cfg, n, bags));
    if (n == 0) return BP_OK;
    if (n_items < 1 || n_items > n) return fail(BP_ERR_INVALID_ARG, "n_items %lld outside [1, n_lookups]", (long long)n_items);
    if (n_split < 0 || n_split > n_items || (n_split && !split_starts))
        return fail(BP_ERR_INVALID_ARG, "n_split %lld outside [0, n_items] or split_starts is NULL", (long long)n_split);
    if (!bag_offsets && n != bags)
        return fail(BP_ERR_INVALID_ARG, "bag_offsets is NULL but n_lookups %lld != bags %lld", (long long)n, (long long)bags);
    if (!cache_w || !grouped_slots || !grouped_lookups || !item_starts || !grad_out) return fail(BP_ERR_INVALID_ARG, "NULL pointer");
    if (cfg->optimizer != BP_SGD && !cache_state) return fail(BP_ERR_INVALID_ARG, "cache_state is NULL");
    if (((uintptr_t)cache_w | (uintptr_t)cache_state | (uintptr_t)grad_out) & 15)
        return fail(BP_ERR_INVALID_ARG, "cache_w, cache_state and grad_out must be 16-byte aligned");
    if (!workspace || ((uintptr_t)workspace & 255)) return fail(BP_ERR_INVALID_ARG, "workspace NULL or not 256-byte aligned");
    GroupedWorkspace w = carve_grouped(workspace, workspace_bytes, n, cfg->dim, bag_offsets != nullptr);
    if (w.bytes > workspace_bytes)
        return fail(BP_ERR_WORKSPACE_TOO_SMALL, "workspace %zu < required %zu bytes", workspace_bytes, w.bytes);
    const uint32_t* bag_of = reinterpret_cast<const uint32_t*>(grouped_lookups);   // one lookup per bag: position == bag
    if (bag_offsets) {
        BP_LAUNCH(K_BWD_KEYS, bwd_bag_of_lookup_kernel, dim3((unsigned)ceil_div(bags > 0 ? bags : 1, 256)), dim3(256), 0,
                  stream, bag_offsets, bags, n, w.bag_of_lookup);
        BP_LAUNCH(K_BWD_KEYS, bwd_bags_of_positions_kernel, dim3((unsigned)ceil_div(n, 256)), dim3(256), 0, stream,
                  grouped_lookups, (const uint32_t*)w.bag_of_lookup, n, bags, w.bag_of);
        bag_of = w.bag_of;
    }
    BwdLaunch l{cfg, w.partial, reinterpret_cast<const uint32_t*>(grouped_slots), bag_of, item_starts, nullptr,
                (uint32_t)n_items, split_starts, (uint32_t)n_split, n, grad_out, cache_w, cache_state, stream, bags};
    return dispatch_row((int)(row_bytes(cfg) / 16), cfg->weight_dtype == BP_BF16, l);
}
