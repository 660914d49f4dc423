// bp_oracle_plan: the lookahead planner (Algorithm 1, Section 3.2) as data-parallel passes.
//
// Algorithm 1 walks the batches with a dictionary and a set.  The same decisions follow from one fact
// per (id, batch) pair — the gap to the id's next use:
//   kept after batch i   <=>  gap < L_eff            (its TTL lies beyond i)
//   prefetched at i      <=>  first use, or not kept after the previous use
//   TTL                   =   last use inside [i, i + L_eff - 1]
// so the planner sorts (id, batch) keys, dedupes them into unique pairs, reads gaps off neighbouring
// pairs, and derives everything else with scans:
//   1. one 64-bit word per lookup, (id | batch | place inside the batch), made by the first pass of a stable LSD
//      radix sort on the id bits as it reads the caller's ids (the input is batch-major, so equal ids stay in batch
//      and lookup order)
//   2. head flags + scan  -> unique pairs (sorted by id, then batch), pair index of every lookup
//   3. histogram H[gap][batch] and per-batch unique counts -> occupancy for every candidate lookahead
//      -> L_eff = largest lookahead whose peak occupancy fits the capacity
//   4. per-pair flags (miss / evict), TTL, and the pair that fetched the row (max-scan of miss indices)
//   5. regroup pairs by batch (stable sort on the batch bits) -> lists ascending in id inside a batch,
//      miss / evict ordinals by one packed scan
//   6. FIFO free ring without a walk over batches: the x-th miss takes ring position x; positions below
//      C are the initial slots, position C + e holds the slot freed by the e-th eviction, i.e. the slot
//      of an earlier miss.  Every miss follows those links to the end of its chain (plan_ring_resolve_kernel).
//   7. slots of pairs -> list slots and the per-lookup slot map
//   8. (optional) one more stable pass on the batch bits, with the slot in place of the id in every word, lists every
//      batch's lookups grouped by row, with the work-item cuts the grouped backward pass uses, so that the backward
//      pass need not sort
#include <algorithm>
#include <cstring>
#include <vector>

#include "common.h"
#include "bwd_records.h"
#include "device_prims.h"

namespace bp {
namespace {

constexpr int kPlanSortIPT = 16;       // 4096 keys per tile for the big (id, batch) sort
constexpr int kBlock = 256;
constexpr uint32_t kGapInf = 0x7fffffffu;
constexpr int kMaxIters = 8192;
constexpr int kMaxTrainers = 64;

struct PlanScalars {
    uint32_t error_flags;   // bit 0: id out of range
    int32_t L_eff;          // 0 = no feasible lookahead
    int32_t L_sel;          // min(L_eff, Lcap): index into peak[]
    int32_t L_requested;    // configured lookahead, or the start-up rule's value when none is configured
    int64_t peak;
    int64_t min_capacity;
    uint32_t n_pairs;       // unique (id, batch) pairs
    uint32_t ring_open;     // bit k: the k-th launch of the ring's chain walk left a chain short of its end
};

// ---- 1. keys ---------------------------------------------------------------------------------
// A lookup travels through the sort as one 64-bit word: (id << (ib + pb)) | (batch << pb) | place, `place` being the
// lookup's position inside its batch (pb bits).  The word is made where the first sort pass reads its input, from the
// caller's ids, so no array of keys and positions is written beforehand and none of positions is carried along.
// Chunked planning: the rows resident at the chunk boundary form a batch 0 of their own in front of the chunk's
// batches (which then count from 1), so that everything downstream sees them as rows fetched before the chunk.
// Batch of a position (in the lookups' own order, and equally in the batch-grouped order, which has the same batch
// stretches).  The host lists the batch of every kPosTile-th position; from there a lane walks on, which it hardly
// ever has to.  Nothing here depends on a loaded key, so these reads run beside the key's own.
constexpr int kPosTileShift = 12;
struct BatchOfPos {
    const int32_t* tile_batch;     // batch of position t << kPosTileShift
    const int64_t* iter_off;       // batch offsets as the planner counts them, [T + 1]
    int T;
    __device__ __forceinline__ int find(int64_t p) const {
        int b = tile_batch[p >> kPosTileShift];
        while (b + 1 < T && iter_off[b + 1] <= p) ++b;
        return b;
    }
};

__global__ __launch_bounds__(kBlock) void plan_tile_batch_kernel(const int64_t* __restrict__ iter_off, int T, int64_t tiles,
                                                                 int32_t* __restrict__ tile_batch) {
    const int64_t t = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (t >= tiles) return;
    const int64_t p = t << kPosTileShift;
    int lo = 0, hi = T;                                   // the last batch that starts at or before p
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (iter_off[mid] <= p) lo = mid; else hi = mid;
    }
    tile_batch[t] = lo;
}

struct PlanKeySource {
    const int64_t* ids;            // the lookups, batch after batch
    const int64_t* resident_ids;   // the carried rows (elements [0, first)), or NULL
    int64_t first;
    BatchOfPos where;
    int ib, pb;
    int64_t R;
    PlanScalars* sc;
    typedef int64_t Raw;
    __device__ __forceinline__ int64_t load(uint32_t i) const {
        return *((int64_t)i < first ? resident_ids + i : ids + ((int64_t)i - first));
    }
    struct Cursor {
        const PlanKeySource& s;
        int b;                     // batch of the last element asked for
        int64_t lo, hi;            // its stretch
        __device__ __forceinline__ Cursor(const PlanKeySource& src, uint32_t i) : s(src) {
            b = s.where.find((int64_t)i);
            lo = s.where.iter_off[b];
            hi = s.where.iter_off[b + 1];
        }
        __device__ __forceinline__ uint64_t key(uint32_t i, int64_t g) {
            while ((int64_t)i >= hi && b + 1 < s.where.T) {      // elements are asked for in ascending order
                ++b;
                lo = hi;
                hi = s.where.iter_off[b + 1];
            }
            if (g < 0 || g >= s.R) {
                atomicOr(&s.sc->error_flags, 1u);
                g = 0;
            }
            return ((uint64_t)g << (s.ib + s.pb)) | ((uint64_t)b << s.pb) | (uint64_t)((int64_t)i - lo);
        }
    };
};

// ---- 2. unique pairs -------------------------------------------------------------------------
struct HeadFlagIn {
    const uint64_t* keys;
    int pb;
    __device__ __forceinline__ uint32_t operator()(int64_t p) const {
        return (p == 0 || (keys[p] >> pb) != (keys[p - 1] >> pb)) ? 1u : 0u;
    }
};
struct PairOut {
    const uint64_t* keys;
    int pb;
    uint64_t* ukey;           // (id << ib) | batch of every pair
    uint32_t* uq;
    uint32_t* pair_start;     // where the pair's lookups begin in the sorted order
    __device__ __forceinline__ void operator()(int64_t p, uint32_t exc, uint32_t inc) const {
        uq[p] = inc - 1u;
        if (inc != exc) {
            ukey[exc] = keys[p] >> pb;
            pair_start[exc] = (uint32_t)p;
        }
    }
};

// With the grouping asked for, the regrouping sort at the end of the plan reads these same sorted words for its first
// histogram (the batch bits).  One kernel then makes both: a workgroup takes one tile of that sort, which is a whole
// number of the scan's tiles, counts the heads of each of them (what scan_reduce_kernel would leave in `partials`)
// and the tile's batch digits (what sort_upsweep_kernel would leave in `counts`).  Elements are dealt to lanes as in
// the scan, so a lane's left neighbour is the lane below it, the round before, or one word fetched per wavefront.
template <int RB>
__global__ __launch_bounds__(kSortBlock) void plan_head_hist_kernel(const uint64_t* __restrict__ keys, uint32_t n, int pb,
                                                                    uint32_t* __restrict__ partials, uint32_t scan_tiles,
                                                                    uint32_t mask, uint32_t* __restrict__ counts,
                                                                    uint32_t ntiles) {
    constexpr int RADIX = 1 << RB;
    constexpr int TILE = kSortBlock * kPlanSortIPT;
    constexpr int PARTS = TILE / kScanTile;
    constexpr int WAVES = kSortBlock / kWave;
    static_assert(kSortBlock == kScanBlock && TILE % kScanTile == 0, "a tile of the sort is a whole number of scan tiles");
    __shared__ uint32_t hist[RADIX];
    __shared__ uint32_t wave_tot[PARTS][WAVES];
    const uint32_t tile = blockIdx.x;
    const int w = threadIdx.x / kWave, lane = lane_id();
    for (int d = threadIdx.x; d < RADIX; d += kSortBlock) hist[d] = 0;
    __syncthreads();
#pragma unroll
    for (int h = 0; h < PARTS; ++h) {
        const int64_t first = (int64_t)tile * TILE + h * kScanTile + w * kScanWaveStretch;      // of this wavefront
        uint64_t k[kScanRounds];
#pragma unroll
        for (int r = 0; r < kScanRounds; ++r) {
            const int64_t i = first + r * kWave + lane;
            k[r] = i < (int64_t)n ? keys[i] : 0;
        }
        uint64_t before = first > 0 && first <= (int64_t)n ? keys[first - 1] : 0;               // left of lane 0, round 0
        uint32_t heads = 0;
#pragma unroll
        for (int r = 0; r < kScanRounds; ++r) {
            const int64_t i = first + r * kWave + lane;
            uint64_t left = __shfl_up(k[r], 1, kWave);
            if (lane == 0) left = before;
            before = __shfl(k[r], kWave - 1, kWave);
            if (i < (int64_t)n) {
                heads += (i == 0 || (k[r] >> pb) != (left >> pb)) ? 1u : 0u;
                // as in sort_upsweep_kernel: the lanes that share the first active lane's digit count themselves at once
                const uint32_t d = (uint32_t)(k[r] >> pb) & mask;
                const uint32_t d0 = __builtin_amdgcn_readfirstlane(d);
                const uint64_t same = __ballot(d == d0);
                if (d != d0) atomicAdd(&hist[d], 1u);
                else if ((same & lanemask_lt()) == 0) atomicAdd(&hist[d0], (uint32_t)__popcll(same));
            }
        }
        heads = wave_reduce(heads, AddOp());
        if (lane == 0) wave_tot[h][w] = heads;
    }
    __syncthreads();
    if (threadIdx.x < PARTS) {
        const uint32_t st = tile * PARTS + threadIdx.x;
        uint32_t total = 0;
#pragma unroll
        for (int i = 0; i < WAVES; ++i) total += wave_tot[threadIdx.x][i];
        if (st < scan_tiles) partials[st] = total;
    }
    for (int d = threadIdx.x; d < RADIX; d += kSortBlock) counts[(size_t)d * ntiles + tile] = hist[d];
}

// ---- 3. gaps, histogram, occupancy -----------------------------------------------------------
__device__ __forceinline__ uint32_t pair_gap(const uint64_t* ukey, uint32_t q, uint32_t M, int ib, uint64_t imask) {
    if (q + 1 >= M) return kGapInf;
    const uint64_t a = ukey[q], b = ukey[q + 1];
    return (a >> ib) == (b >> ib) ? (uint32_t)((b & imask) - (a & imask)) : kGapInf;
}

// Each workgroup walks a contiguous stretch of pairs and keeps its counts in LDS: the per-batch unique counts and
// the histogram rows of the small gaps [2, 2 + lds_gaps), which take nearly all the hits; larger gaps go to global
// atomics.  Integer atomics only: the sums do not depend on the order.
// The number of pairs is read from the device (the host has not fetched it yet: it comes back together with the
// lookahead, in one synchronisation instead of two); the grid is sized for the lookups, an upper bound.
__global__ __launch_bounds__(kBlock) void plan_hist_kernel(const uint64_t* __restrict__ ukey,
                                                           const uint32_t* __restrict__ n_pairs, int ib, int T,
                                                           int Lcap, int lds_gaps,
                                                           uint32_t* __restrict__ H, uint32_t* __restrict__ ucount,
                                                           uint32_t* __restrict__ first_use, int chunk,
                                                           uint32_t* __restrict__ V) {
    const uint32_t M = *n_pairs;
    const uint32_t per_block = (M + gridDim.x - 1) / gridDim.x;
    if ((uint64_t)blockIdx.x * per_block >= M) return;
    extern __shared__ uint32_t lds[];   // [T] unique counts, [T] first uses, then [lds_gaps][T] histogram rows
    uint32_t* lds_u = lds;
    uint32_t* lds_f = lds + T;
    uint32_t* lds_h = lds + 2 * T;
    const int cells = (2 + lds_gaps) * T;
    for (int i = threadIdx.x; i < cells; i += kBlock) lds[i] = 0;
    __syncthreads();
    const uint64_t imask = (uint64_t(1) << ib) - 1;
    const uint64_t begin = (uint64_t)blockIdx.x * per_block;
    const uint64_t end = begin + per_block < M ? begin + per_block : M;
    // four pairs per thread and round, their keys and both neighbours' requested before any of them is counted
    constexpr int kPairsInFlight = 4;
    for (uint64_t q0 = begin + threadIdx.x; q0 < end; q0 += kBlock * kPairsInFlight) {
        uint64_t key[kPairsInFlight], prev[kPairsInFlight], next[kPairsInFlight];
#pragma unroll
        for (int r = 0; r < kPairsInFlight; ++r) {
            const uint64_t q = q0 + (uint64_t)r * kBlock;
            const bool in = q < end;
            key[r] = in ? ukey[q] : 0;
            prev[r] = in && q > 0 ? ukey[q - 1] : ~uint64_t(0);        // no id has all bits set
            next[r] = in && q + 1 < M ? ukey[q + 1] : ~uint64_t(0);
        }
#pragma unroll
        for (int r = 0; r < kPairsInFlight; ++r) {
            if (q0 + (uint64_t)r * kBlock >= end) break;
            const uint64_t a = key[r];
            const uint32_t i = (uint32_t)(a & imask);
            atomicAdd(&lds_u[i], 1u);
            if ((prev[r] >> ib) != (a >> ib)) atomicAdd(&lds_f[i], 1u);   // the id's first batch
            const uint32_t gap = (a >> ib) == (next[r] >> ib) ? (uint32_t)((next[r] & imask) - i) : kGapInf;
            if (chunk && i == 0) {      // a carried resident stays until its next use, whatever the lookahead
                atomicAdd(&V[gap == kGapInf ? (uint32_t)T : gap], 1u);
                continue;
            }
            if (gap >= 2u && gap < (uint32_t)Lcap) {
                if (gap < 2u + (uint32_t)lds_gaps) atomicAdd(&lds_h[(gap - 2u) * T + i], 1u);
                else atomicAdd(&H[(size_t)gap * T + i], 1u);
            }
        }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < T; i += kBlock) {
        if (lds_u[i]) atomicAdd(&ucount[i], lds_u[i]);
        if (lds_f[i]) atomicAdd(&first_use[i], lds_f[i]);
    }
    for (int x = threadIdx.x; x < lds_gaps * T; x += kBlock)
        if (lds_h[x]) atomicAdd(&H[(size_t)2 * T + x], lds_h[x]);      // row (2 + x / T), column x % T
}

// H[gap][.] -> inclusive prefix over batches, one wavefront per gap row
__global__ __launch_bounds__(kBlock) void plan_occ_prefix_kernel(uint32_t* H, int T, int Lcap) {
    const int gap = blockIdx.x * (kBlock / kWave) + threadIdx.x / kWave;
    if (gap < 2 || gap >= Lcap) return;
    uint32_t* row = H + (size_t)gap * T;
    uint32_t run = 0;
    for (int base = 0; base < T; base += kWave) {
        const int i = base + lane_id();
        const uint32_t inc = wave_inclusive_scan(i < T ? row[i] : 0u, AddOp());
        if (i < T) row[i] = run + inc;
        run += __shfl(inc, kWave - 1);
    }
}

// Carried residents not yet used again at batch j: vcover[j] = residents - (those whose next use is batch <= j);
// batch 0 holds them as its own rows.  One thread.
__global__ void plan_vcover_kernel(const uint32_t* __restrict__ V, uint32_t R0, int T, uint32_t* __restrict__ vcover) {
    if (blockIdx.x != 0 || threadIdx.x != 0) return;
    uint32_t run = R0;
    vcover[0] = 0;
    for (int j = 1; j < T; ++j) {
        run -= V[j];
        vcover[j] = run;
    }
}

// rows resident but unused at batch j because of pairs with exactly this gap: batches i in (j - gap, j), and only
// pairs of batches <= last_deciding (a chunk asks what its own decisions leave in the cache of the batches after it)
__device__ __forceinline__ uint32_t covering(const uint32_t* Hc, int T, int gap, int j, int last_deciding) {
    if (j < 1) return 0;
    const int top = j - 1 < last_deciding ? j - 1 : last_deciding;
    if (j - gap >= top) return 0;
    const uint32_t* row = Hc + (size_t)gap * T;
    const uint32_t hi = row[top];
    const uint32_t lo = j - gap >= 0 ? row[j - gap] : 0u;
    return hi - lo;
}

// peak[L'] = max_j occupancy(j, L') for L' = 1..Lcap.  One workgroup per batch j: occupancy(j, L') is the unique
// count of j plus the prefix sum over gap < L' of covering(gap, j), taken with a workgroup scan over the gaps.
__global__ __launch_bounds__(kBlock) void plan_occ_peak_kernel(const uint32_t* __restrict__ Hc,
                                                               const uint32_t* __restrict__ ucount,
                                                               const uint32_t* __restrict__ vcover, int j_first,
                                                               int j_last, int T, int Lcap, uint32_t* __restrict__ peak) {
    __shared__ uint32_t wave_tot[kBlock / kWave];
    // A chunk's peak is taken over the batches it emits and, for the batches after them, over what its decisions
    // alone leave there (their own rows, the carried rows, the rows this chunk keeps): if that fits, the following
    // chunk can be planned at least with a lookahead of one.
    const int j = blockIdx.x;
    if (j < j_first) return;
    uint32_t carry = ucount[j] + (vcover ? vcover[j] : 0u);
    if (threadIdx.x == 0) {
        atomicMax(&peak[1], carry);
        if (Lcap >= 2) atomicMax(&peak[2], carry);       // L' = 2 keeps gap 1 only: nothing is resident unused
    }
    for (int base = 2; base < Lcap; base += kBlock) {     // gap = L' - 1 for L' = 3..Lcap
        const int gap = base + threadIdx.x;
        const uint32_t v = gap < Lcap ? covering(Hc, T, gap, j, j_last) : 0u;
        uint32_t exc, inc, total;
        block_scan<kBlock>(v, AddOp(), 0u, wave_tot, &exc, &inc, &total);
        if (gap < Lcap) atomicMax(&peak[gap + 1], carry + inc);
        carry += total;
    }
}

// One wavefront: pick L_eff, exclusive scan of the per-batch unique counts.  64 candidates, or 64 batches, per step.
__global__ __launch_bounds__(kWave) void plan_choose_kernel(const uint32_t* __restrict__ peak,
                                                            const uint32_t* __restrict__ ucount,
                                                            const uint32_t* __restrict__ first_use, int T, int Lcap,
                                                            int lookahead, int64_t budget, int carried_batches,
                                                            const uint32_t* __restrict__ n_pairs, PlanScalars* sc,
                                                            uint32_t* __restrict__ pair_off) {
    if (blockIdx.x != 0) return;
    const int lane = lane_id();
    int requested = lookahead, top = Lcap;
    if (lookahead == 0) {
        // no lookahead configured (Section 4): batches are prefetched at start-up until the cache is full; the
        // distinct rows of batches 0..k-1 are the ids whose first use lies in those batches.  The running total
        // never falls, so the batches that fit are a prefix and counting them finds its end.
        int64_t held = 0;
        int k = 0;
        for (int i0 = 0; i0 < T; i0 += kWave) {
            const int i = i0 + lane;
            const int64_t inc = held + wave_inclusive_scan<int64_t>(i < T ? (int64_t)first_use[i] : 0, AddOp());
            k += (int)__popcll(__ballot(i < T && inc <= budget));
            held = __shfl(inc, kWave - 1, kWave);
            if (held > budget) break;
        }
        requested = k - carried_batches;             // a chunk's batch 0 holds the carried residents, not lookups
        if (requested < 0) requested = 0;
        top = requested < Lcap ? requested : Lcap;
    }
    int sel = 0;                                     // the largest candidate whose peak occupancy fits
    for (int hi = top; hi >= 1 && sel == 0; hi -= kWave) {
        const int Lp = hi - lane;
        const uint64_t fits = __ballot(Lp >= 1 && (int64_t)peak[Lp >= 1 ? Lp : 1] <= budget);
        if (fits) sel = hi - (__ffsll((unsigned long long)fits) - 1);
    }
    uint32_t run = 0;
    for (int i0 = 0; i0 <= T; i0 += kWave) {
        const int i = i0 + lane;
        const uint32_t x = i < T ? ucount[i] : 0u;
        const uint32_t inc = run + wave_inclusive_scan<uint32_t>(x, AddOp());
        if (i <= T) pair_off[i] = inc - x;
        run = __shfl(inc, kWave - 1, kWave);
    }
    if (lane == 0) {
        sc->n_pairs = *n_pairs;          // comes back to the host with the lookahead, in one copy
        sc->L_sel = sel;
        sc->L_eff = (sel == top && sel > 0) ? requested : sel;   // windows of T or more batches are all alike
        sc->L_requested = requested;
        sc->peak = sel ? peak[sel] : 0;
        sc->min_capacity = peak[1];
    }
}

__global__ void plan_occ_final_kernel(const uint32_t* __restrict__ Hc, const uint32_t* __restrict__ ucount,
                                      const uint32_t* __restrict__ vcover, int T, const PlanScalars* sc,
                                      int64_t* __restrict__ occ) {
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= T) return;
    uint32_t run = ucount[j] + (vcover ? vcover[j] : 0u);
    for (int gap = 2; gap < sc->L_sel; ++gap) run += covering(Hc, T, gap, j, T);
    occ[j] = run;
}

// ---- 4. per-pair decisions -------------------------------------------------------------------
// Everything the lists need about a pair travels in one 64-bit record, which is also the key of the regroup sort
// (sorted on its lowest iter_bits only):  id | ttl | evict | miss | batch.
constexpr uint64_t kMiss = 1, kEvict = 2;

struct PairRecord {
    int ib;
    __device__ __forceinline__ uint64_t pack(uint64_t g, uint32_t ttl, uint64_t flags, uint32_t i) const {
        return (g << (2 * ib + 2)) | ((uint64_t)ttl << (ib + 2)) | (flags << ib) | i;
    }
    __device__ __forceinline__ uint32_t batch(uint64_t r) const { return (uint32_t)(r & ((uint64_t(1) << ib) - 1)); }
    __device__ __forceinline__ uint64_t flags(uint64_t r) const { return (r >> ib) & 3; }
    __device__ __forceinline__ uint32_t ttl(uint64_t r) const { return (uint32_t)((r >> (ib + 2)) & ((uint64_t(1) << ib) - 1)); }
    __device__ __forceinline__ int64_t id(uint64_t r) const { return (int64_t)(r >> (2 * ib + 2)); }
};

// The search for the TTL probes up to L_eff - 1 pairs ahead, one probe behind the other: the workgroup first copies
// its own pairs (kFlagsPerThread per thread), the one before them and the next kFlagsWindow into LDS, where a probe
// costs a fraction of a trip to L2 (probes beyond that window go to memory as before).
constexpr int kFlagsWindow = 1024;
constexpr int kFlagsPerThread = 4;
constexpr int kFlagsTile = kBlock * kFlagsPerThread;
__global__ __launch_bounds__(kBlock) void plan_flags_kernel(const uint64_t* __restrict__ ukey, uint32_t M, int ib,
                                                            const PlanScalars* sc, int chunk, uint64_t* __restrict__ rec) {
    __shared__ uint64_t win[kFlagsTile + 1 + kFlagsWindow];
    const uint64_t imask = (uint64_t(1) << ib) - 1;
    const int64_t Leff = sc->L_eff;
    const int64_t win_first = (int64_t)blockIdx.x * kFlagsTile - 1;             // pair number of win[0]
    const int ahead = (int)(Leff - 1 < kFlagsWindow ? (Leff > 1 ? Leff - 1 : 0) : kFlagsWindow);
    const int span = kFlagsTile + 1 + ahead;
    for (int t = threadIdx.x; t < span; t += kBlock) {
        const int64_t p = win_first + t;
        win[t] = p >= 0 && p < (int64_t)M ? ukey[p] : ~uint64_t(0);
    }
    __syncthreads();
    const auto key_at = [&](int64_t p) -> uint64_t {                            // first pair of the tile - 1 <= p < M
        const int64_t t = p - win_first;
        return t < span ? win[t] : ukey[p];
    };
#pragma unroll
    for (int e = 0; e < kFlagsPerThread; ++e) {
        const uint32_t q = blockIdx.x * kFlagsTile + e * kBlock + threadIdx.x;
        if (q >= M) break;
        const uint64_t k = key_at(q);
        const uint64_t g = k >> ib;
        const int64_t i = (int64_t)(k & imask);
        uint32_t gap = kGapInf;
        if (q + 1 < M) {
            const uint64_t kn = key_at((int64_t)q + 1);
            if ((kn >> ib) == g) gap = (uint32_t)((kn & imask) - (k & imask));
        }
        const bool carried = chunk && i == 0;              // resident since before the chunk: stays until its next use
        const bool keep = carried || (int64_t)gap < Leff;
        bool miss = true;
        if (q > 0) {
            const uint64_t kp = key_at((int64_t)q - 1);
            if ((kp >> ib) == g && ((chunk && (kp & imask) == 0) || i - (int64_t)(kp & imask) < Leff)) miss = false;
        }
        uint32_t t = (uint32_t)i;
        if (keep && !carried) {
            // last pair of this id whose batch is <= i + L_eff - 1: it lies within L_eff - 1 pairs of q
            const int64_t last_iter = i + Leff - 1 < (int64_t)imask ? i + Leff - 1 : (int64_t)imask;
            const uint64_t bound = (g << ib) | (uint64_t)last_iter;
            int64_t lo = q, hi = (int64_t)q + Leff - 1;     // pair lo <= bound; answer in [lo, hi]
            if (hi > (int64_t)M - 1) hi = (int64_t)M - 1;
            while (lo < hi) {
                const int64_t mid = (lo + hi + 1) >> 1;
                if (key_at(mid) <= bound) lo = mid; else hi = mid - 1;
            }
            t = (uint32_t)(key_at(lo) & imask);
        }
        rec[q] = PairRecord{ib}.pack(g, t, (miss ? kMiss : 0) | (keep ? 0 : kEvict), (uint32_t)i);
    }
}

struct MissIndexIn {
    const uint64_t* rec;
    int ib;
    __device__ __forceinline__ uint32_t operator()(int64_t q) const {
        return (PairRecord{ib}.flags(rec[q]) & kMiss) ? (uint32_t)q : 0u;
    }
};
struct StoreInclusiveU32 {
    uint32_t* p;
    __device__ __forceinline__ void operator()(int64_t i, uint32_t, uint32_t inc) const { p[i] = inc; }
};

// ---- 5. lists in (batch, id) order -----------------------------------------------------------
struct ListCountIn {
    const uint64_t* srec;     // records sorted by batch (stable: id order inside a batch)
    int ib;
    __device__ __forceinline__ uint64_t operator()(int64_t k) const {
        const uint64_t f = PairRecord{ib}.flags(srec[k]);
        return (f & kMiss) | (((f & kEvict) >> 1) << 32);
    }
};
struct ListOut {
    const uint64_t* srec;
    const uint32_t* ord;      // what travelled with the k-th sorted record: its pair's number (numbered) or the
                              // number of the pair that fetched its row, which for a miss is the pair itself
    const uint32_t* pair_off;
    int ib;
    int64_t* keep_ids;
    int32_t* keep_ttl;
    int64_t* prefetch_ids;
    int64_t* evict_ids;
    uint32_t* missord;
    uint32_t* evict_pair;    // for every eviction, the pair that fetched the evicted row
    int64_t* prefetch_off;   // device copies of the CSR offsets, [T+1], pre-filled with -1
    int64_t* evict_off;
    int32_t ttl_shift;       // 1 in chunk mode: the chunk's batches count from 1 inside the planner
    // optional marking of the trainers that use a row (keep_owner == NULL: off)
    int32_t* keep_owner;
    const uint64_t* ukey;     // pairs in (id, batch) order
    uint32_t M;
    const uint32_t* pair_start;
    uint32_t n_sorted;        // lookups in the sorted order (carried rows included)
    const uint64_t* skeys;    // the sorted lookups' words: the low pb bits are the place inside the batch
    int pb;
    const int64_t* cuts;      // device [real batches][P + 1]
    int P;
    const uint32_t* chain;    // the pair that fetched the row a pair uses
    bool numbered;
    __device__ __forceinline__ int trainer_of(const int64_t* c, int64_t rel) const {
        int lo = 0, hi = P;                               // largest t < P with c[t] <= rel
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (c[mid] <= rel) lo = mid; else hi = mid;
        }
        return lo;
    }
    __device__ __forceinline__ int32_t owner_of(uint32_t q, uint32_t i) const {
        if (ttl_shift && i == 0) return -1;               // a chunk's carried rows: no lookups
        const uint32_t a = pair_start[q], b = q + 1 < M ? pair_start[q + 1] : n_sorted;
        const uint64_t pmask = (uint64_t(1) << pb) - 1;
        const int64_t* c = cuts + (size_t)(i - ttl_shift) * (P + 1);
        // the pair's lookups are in position order and a trainer owns a stretch of positions: first and last decide
        const int t0 = trainer_of(c, (int64_t)(skeys[a] & pmask)), t1 = trainer_of(c, (int64_t)(skeys[b - 1] & pmask));
        if (t0 == t1) return t0;
        const uint64_t imask = (uint64_t(1) << ib) - 1;
        const bool next = q + 1 < M && (ukey[q + 1] >> ib) == (ukey[q] >> ib) && (ukey[q + 1] & imask) == (uint64_t)i + 1;
        return next ? -2 : -1;
    }
    __device__ __forceinline__ void operator()(int64_t k, uint64_t exc, uint64_t) const {
        const PairRecord pr{ib};
        const uint64_t r = srec[k];
        const uint32_t q = ord[k];           // not numbered: the pair's own number only where the pair is a miss
        const int64_t g = pr.id(r);
        const uint32_t i = pr.batch(r);
        const uint32_t x = (uint32_t)exc, e = (uint32_t)(exc >> 32);
        const uint64_t f = pr.flags(r);
        keep_ids[k] = g;
        keep_ttl[k] = (int32_t)pr.ttl(r) - ttl_shift;
        if (keep_owner) keep_owner[k] = owner_of(q, i);
        if (f & kMiss) {
            prefetch_ids[x] = g;
            missord[q] = x;
        }
        if (f & kEvict) {
            evict_ids[e] = g;
            evict_pair[e] = numbered ? chain[q] : q;       // the pair that fetched the row: same residency, same slot
        }
        if ((uint32_t)k == pair_off[i]) {
            prefetch_off[i] = x;
            evict_off[i] = e;
        }
    }
};

// ---- 6. FIFO ring: chains of links ------------------------------------------------------------
__global__ __launch_bounds__(kBlock) void plan_ring_init_kernel(const uint64_t* __restrict__ totals, int64_t C,
                                                                const uint32_t* __restrict__ evict_pair,
                                                                const uint32_t* __restrict__ missord,
                                                                uint32_t* __restrict__ par) {
    const uint32_t n_miss = (uint32_t)*totals, n_evict = (uint32_t)(*totals >> 32);
    const uint32_t x = blockIdx.x * kBlock + threadIdx.x;
    if (x >= n_miss) return;
    if ((int64_t)x < C) {
        par[x] = x;                                   // initial ring content: slot x at position x
    } else {
        const uint32_t e = (uint32_t)((int64_t)x - C);   // ring position C + e was pushed by eviction e
        par[x] = e < n_evict ? missord[evict_pair[e]] : 0u;
    }
}

// Every miss walks its own chain towards the ring position below C it ends at, kRingHops hops per launch at most,
// and leaves with a link to where it got.  A hop goes back at least one batch, so a chain has at most T hops and
// ceil(log_kRingHops(T + 1)) launches resolve everything whatever the trace (in practice a slot changes hands a few
// times over a trace and the first launch does it all).  Lanes read entries that other lanes may have advanced
// already: either value lies on the same chain, the newer one nearer to its end.
constexpr int kRingHops = 64;
// A launch that follows one which brought every chain to its end has nothing to do and says so at once.
__global__ __launch_bounds__(kBlock) void plan_ring_resolve_kernel(const uint64_t* __restrict__ totals, int max_hops,
                                                                   uint32_t* par, PlanScalars* sc, int launch) {
    if (launch > 0 && ((sc->ring_open >> (launch - 1)) & 1u) == 0u) return;
    const uint32_t n_miss = (uint32_t)*totals;
    for (uint64_t x64 = (uint64_t)blockIdx.x * kBlock + threadIdx.x; x64 < n_miss; x64 += (uint64_t)gridDim.x * kBlock) {
        const uint32_t x = (uint32_t)x64;
        uint32_t p = par[x];
        bool ended = false;
        for (int hop = 0; hop < max_hops; ++hop) {
            const uint32_t pp = p < n_miss ? par[p] : 0u;
            if (pp == p) {
                ended = true;
                break;
            }
            p = pp;
        }
        par[x] = p;
        if (!ended) atomicOr(&sc->ring_open, 1u << launch);
    }
}

// ---- 7. slots --------------------------------------------------------------------------------
// par resolves a miss to a ring position below C, and ring0 (NULL: the identity) is what that position held when
// planning started.  Only while the occupancy stays within C, though: in chunk mode the batches past the emitted ones
// are planned with the chunk's lookahead without any bound on their occupancy, so their misses may ask for slots
// that are freed only later; such a miss resolves to nothing below C and gets no slot (-1).  Those batches are never
// reported.
__device__ __forceinline__ int32_t resolved_slot(uint32_t p0, const int32_t* __restrict__ ring0, int64_t C) {
    if ((int64_t)p0 >= C) return -1;
    return ring0 ? ring0[p0] : (int32_t)p0;
}

__global__ __launch_bounds__(kBlock) void plan_pair_slots_kernel(uint32_t M, const uint32_t* __restrict__ chain,
                                                                 const uint32_t* __restrict__ missord,
                                                                 const uint32_t* __restrict__ par,
                                                                 const int32_t* __restrict__ ring0, int64_t C,
                                                                 int32_t* __restrict__ slot_of_pair) {
    const uint32_t q = blockIdx.x * kBlock + threadIdx.x;
    if (q >= M) return;
    slot_of_pair[q] = resolved_slot(par[missord[chain[q]]], ring0, C);
}

__global__ __launch_bounds__(kBlock) void plan_list_slots_kernel(const uint64_t* __restrict__ totals,
                                                                 const uint32_t* __restrict__ par,
                                                                 const uint32_t* __restrict__ evict_pair,
                                                                 const int32_t* __restrict__ slot_of_pair,
                                                                 const int32_t* __restrict__ ring0, int64_t C,
                                                                 int32_t* __restrict__ prefetch_slots,
                                                                 int32_t* __restrict__ evict_slots,
                                                                 uint64_t* __restrict__ totals_out) {
    const uint32_t n_miss = (uint32_t)*totals, n_evict = (uint32_t)(*totals >> 32);
    const uint32_t x = blockIdx.x * kBlock + threadIdx.x;
    if (x == 0) *totals_out = *totals;               // where the host's one copy at the end finds them
    if (x < n_miss) prefetch_slots[x] = resolved_slot(par[x], ring0, C);
    if (x < n_evict) {
        // The x-th eviction pushed ring position C + x.  Where a later miss took that position, its resolved link is
        // the evicted row's own slot, read in list order; only the evictions nobody reused go through their pair.
        const int64_t pos = C + (int64_t)x;
        evict_slots[x] = pos < (int64_t)n_miss ? resolved_slot(par[pos], ring0, C) : slot_of_pair[evict_pair[x]];
    }
}

// Workgroups are handed to the eight XCDs round-robin, and each XCD has an L2 of its own.  The kernels below write
// 4-byte values to scattered places of a stretch of memory; when the workgroups that share a stretch run on one XCD
// the stores meet in its L2 and leave as full lines.  This maps blockIdx so that XCD x walks the x-th eighth of the
// virtual blocks in order.
constexpr uint32_t kXcds = 8;
__device__ __forceinline__ int64_t xcd_contiguous_block(uint32_t per_xcd) {
    return (int64_t)(blockIdx.x % kXcds) * per_xcd + blockIdx.x / kXcds;
}
inline uint32_t blocks_per_xcd(int64_t n) { return (uint32_t)ceil_div(n > 0 ? ceil_div(n, kBlock) : 1, (int64_t)kXcds); }

__global__ __launch_bounds__(kBlock) void plan_lookup_slots_kernel(int64_t N, int64_t first, int ib, int pb,
                                                                   const uint64_t* __restrict__ skeys,
                                                                   const int64_t* __restrict__ iter_off,
                                                                   const uint32_t* __restrict__ uq,
                                                                   const int32_t* __restrict__ slot_of_pair,
                                                                   int32_t* __restrict__ lookup_slots) {
    const int64_t p = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (p >= N) return;
    const uint64_t k = skeys[p];
    const int64_t pos = iter_off[(k >> pb) & ((uint64_t(1) << ib) - 1)] + (int64_t)(k & ((uint64_t(1) << pb) - 1));
    if (pos >= first) lookup_slots[pos - first] = slot_of_pair[uq[p]];   // below first: carried rows
}

// ---- 8. lookups of every batch grouped by row (optional) ---------------------------------------
// The id bits of every sorted word are replaced by the slot of its pair, in the id-major order (where the pair
// indices, and so the reads of the pairs' slots, ascend): word = (slot << (ib + pb)) | (batch << pb) | place.  A
// stable sort on the batch bits then lists every batch's lookups grouped by id and in lookup order inside a group.
// Inside one batch a change of slot is a change of row.
struct GroupWord {
    int ib, pb;
    __device__ __forceinline__ uint32_t slot(uint64_t k) const { return (uint32_t)(k >> (ib + pb)); }
    __device__ __forceinline__ uint32_t batch(uint64_t k) const { return (uint32_t)(k >> pb) & ((1u << ib) - 1u); }
    __device__ __forceinline__ uint32_t place(uint64_t k) const { return (uint32_t)(k & ((uint64_t(1) << pb) - 1)); }
};
// The regrouping sort's scatter makes these words as it reads its input (its histogram only needs the batch bits,
// which the sorted words already hold).
struct GroupWordSource {
    const uint64_t* skeys;
    const uint32_t* uq;
    const int32_t* slot_of_pair;
    int low;                                  // ib + pb: the bits kept from the sorted word
    struct Raw {
        uint64_t k;
        uint32_t q;
    };
    __device__ __forceinline__ Raw load(uint32_t i) const { return Raw{skeys[i], uq[i]}; }
    struct Cursor {
        const GroupWordSource& s;
        __device__ __forceinline__ Cursor(const GroupWordSource& src, uint32_t) : s(src) {}
        __device__ __forceinline__ uint64_t key(uint32_t, Raw raw) {
            return ((uint64_t)(uint32_t)s.slot_of_pair[raw.q] << s.low) | (raw.k & ((uint64_t(1) << s.low) - 1));
        }
    };
};

// Rows of the grouped order.  A row starts where (slot, batch) changes; the kernel that scatters the slot map reads
// every grouped word anyway and leaves these starts as bit masks, 64 lookups a word.  A scan over the words
// (population counts) then numbers the rows, and every word writes the first grouped positions of its rows to row_pos.
struct RowMaskIn {
    const uint64_t* head_mask;
    __device__ __forceinline__ uint32_t operator()(int64_t w) const { return (uint32_t)__popcll(head_mask[w]); }
};
// A wavefront takes 64 mask words and goes through them one by one: lane b owns bit b of the word in hand, and the
// lanes whose bit is set write their positions side by side, behind the rows that the scan counted before the word.
// (Every word writing its own rows from one lane, inside the scan's last pass, scatters 64 short runs per store.)
__global__ __launch_bounds__(kBlock) void plan_row_starts_kernel(const uint64_t* __restrict__ head_mask,
                                                                 const uint32_t* __restrict__ rows_before, int64_t n_words,
                                                                 uint32_t* __restrict__ row_pos) {
    const int lane = lane_id();
    const int64_t w0 = ((int64_t)blockIdx.x * (kBlock / kWave) + threadIdx.x / kWave) * kWave;    // wave-uniform
    if (w0 >= n_words) return;
    const int64_t mine = w0 + lane;
    const uint64_t m = mine < n_words ? head_mask[mine] : 0;
    const uint32_t before = mine < n_words ? rows_before[mine] : 0u;
    uint64_t left = __ballot(m != 0);                                // words of this wavefront that hold a row start
    while (left) {
        const int t = __ffsll((unsigned long long)left) - 1;
        left &= left - 1;
        const uint64_t word = __shfl(m, t, kWave);
        const uint32_t base = __shfl(before, t, kWave);
        if ((word >> lane) & 1u)
            row_pos[base + (uint32_t)__popcll(word & lanemask_lt())] = (uint32_t)((w0 + t) * 64 + lane);
    }
}

// Second scan, over the rows (RowPiecesIn counts the pieces): every row writes its record beside its keep-list
// entry (the carried residents of a chunk own the first `first` entries), a long row its piece records, and the
// first row of a batch the batch's offsets.  A piece's `partial` is counted through the whole trace here and made
// relative to its batch afterwards; until then its first reserved word holds the batch.
struct GroupRecordOut {
    const uint32_t* row_pos;
    const uint32_t* n_rows;
    uint32_t n;
    const uint64_t* gkeys;
    GroupWord gw;
    const int64_t* iter_off;
    int64_t first;
    uint4* row_recs;
    uint4* piece_recs;
    int64_t* piece_off;    // device copies of the CSR offsets, [T+1] each, pre-filled with -1
    int64_t* multi_off;
    __device__ __forceinline__ void operator()(int64_t r, uint64_t exc, uint64_t inc) const {
        const uint32_t R = *n_rows;
        if (r >= (int64_t)R) return;
        const uint32_t p = row_pos[r];
        const uint32_t count = (r + 1 < (int64_t)R ? row_pos[r + 1] : n) - p;
        const uint64_t k = gkeys[p];
        const uint32_t b = gw.batch(k), slot = gw.slot(k);
        const int64_t base = iter_off[b];
        const uint32_t rel = (uint32_t)((int64_t)p - base);
        const uint32_t pc = pieces_of(count);
        row_recs[first + r] = make_uint4(rel | (pc ? kLongRow : 0u), count, slot, gw.place(k));
        if (pc) write_pieces(piece_recs, (uint32_t)exc, pc, rel, count, slot, (uint32_t)(exc >> 32), b);
        if ((int64_t)p == base) {
            piece_off[b] = (int64_t)(uint32_t)exc;
            multi_off[b] = (int64_t)(exc >> 32);
        }
    }
};
__global__ __launch_bounds__(kBlock) void plan_piece_partial_kernel(uint4* __restrict__ piece_recs,
                                                                    const uint32_t* __restrict__ n_pieces, int T,
                                                                    const int64_t* __restrict__ multi_off,
                                                                    uint64_t* __restrict__ totals_out) {
    const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i == 0) *totals_out = *reinterpret_cast<const uint64_t*>(n_pieces);    // pieces | pieces of rows of several
    if (i >= (int64_t)*n_pieces) return;
    uint4 r = piece_recs[2 * i + 1];
    if (r.z < (uint32_t)T) r.y -= (uint32_t)multi_off[r.z];
    r.z = 0u;
    piece_recs[2 * i + 1] = r;
}

// The per-lookup slot map (when the caller wants one) written from the batch-grouped order: the targets of neighbouring grouped lookups lie in
// their batch's stretch of the map (a few MB at most).  The same pass over the grouped words writes each lookup's
// place to grouped_lookups and the row starts as bit masks (a wavefront holds 64 consecutive grouped positions
// starting at a multiple of 64, lane = position % 64; positions outside [first, N) start no row).
__global__ __launch_bounds__(kBlock) void plan_lookup_slots_grouped_kernel(int64_t N, uint32_t per_xcd, GroupWord gw,
                                                                           int64_t first,
                                                                           const uint64_t* __restrict__ gkeys,
                                                                           BatchOfPos where,
                                                                           int32_t* __restrict__ lookup_slots,
                                                                           int32_t* __restrict__ grouped_lookups,
                                                                           uint64_t* __restrict__ head_mask) {
    const int64_t p = xcd_contiguous_block(per_xcd) * kBlock + threadIdx.x;
    const bool real = p >= first && p < N;
    const uint64_t k = real ? gkeys[p] : 0;
    // the word before: the lane below holds it, only a wavefront's first lane has to load it
    uint64_t before = __shfl_up(k, 1, kWave);
    if (lane_id() == 0 && real && p > first) before = gkeys[p - 1];
    bool head = false;
    if (real) {
        const uint32_t place = gw.place(k);
        if (lookup_slots) lookup_slots[where.iter_off[gw.batch(k)] + place - first] = (int32_t)gw.slot(k);
        grouped_lookups[p - first] = (int32_t)place;
        head = p == first || (k >> gw.pb) != (before >> gw.pb);
    }
    const uint64_t m = __ballot(head);
    if ((p & 63) == 0 && p < ((N + 63) & ~int64_t(63))) head_mask[p >> 6] = m;
}

template <typename T>
__global__ __launch_bounds__(kBlock) void fill_kernel(T* p, int64_t n, T v) {
    const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i < n) p[i] = v;
}

// ---- 9. carried state of chunked planning ------------------------------------------------------
// Rows resident after batch e: for every id, its last pair with batch <= e, if that pair keeps the row (a carried
// resident not used up to e, or a gap to the next use below L_eff).  Pairs are in (id, batch) order, so the output is
// ascending in id.
struct ResidentFlagIn {
    const uint64_t* ukey;
    uint32_t M;
    int ib;
    uint32_t e;
    const PlanScalars* sc;
    __device__ __forceinline__ uint32_t operator()(int64_t q) const {
        const uint64_t imask = (uint64_t(1) << ib) - 1;
        const uint64_t k = ukey[q];
        const uint32_t i = (uint32_t)(k & imask);
        if (i > e) return 0u;
        const uint32_t gap = pair_gap(ukey, (uint32_t)q, M, ib, imask);
        const bool last_seen = gap == kGapInf || i + gap > e;            // no later use at or before batch e
        const bool kept = i == 0 || (int64_t)gap < (int64_t)sc->L_eff;
        return last_seen && kept ? 1u : 0u;
    }
};
struct ResidentOut {
    const uint64_t* ukey;
    const int32_t* slot_of_pair;
    int ib;
    int64_t* resident_ids;
    int32_t* ring;
    __device__ __forceinline__ void operator()(int64_t q, uint32_t exc, uint32_t inc) const {
        if (inc != exc) {
            resident_ids[exc] = (int64_t)(ukey[q] >> ib);
            ring[exc] = slot_of_pair[q];
        }
    }
};

// The free slots in FIFO order behind the residents: ring positions [n_miss, C + n_evict) as of batch e.
__global__ __launch_bounds__(kBlock) void plan_state_queue_kernel(int64_t n_miss, int64_t n_evict, int64_t C,
                                                                  const int32_t* __restrict__ ring0,
                                                                  const int32_t* __restrict__ evict_slots,
                                                                  int64_t n_resident, int32_t* __restrict__ ring_out) {
    const int64_t x = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    const int64_t pos = n_miss + x;
    if (pos >= C + n_evict) return;
    const int32_t slot = pos < C ? (ring0 ? ring0[pos] : (int32_t)pos) : evict_slots[pos - C];
    ring_out[n_resident + x] = slot;
}

// ---- workspace layout ------------------------------------------------------------------------
struct PlanWorkspace {
    uint64_t *keys_a, *keys_b;
    uint32_t* uq;            // pair of every sorted lookup
    int32_t* tile_batch;     // batch of every 4096-th position
    uint32_t* sort_temp;
    uint32_t* scan_partials32;   // head scan, chain scan
    uint64_t* scan_partials64;   // list scan
    uint32_t *H, *ucount, *first_use, *peak, *pair_off, *V, *vcover;
    PlanScalars* scalars;
    int64_t *occ, *offsets, *prefetch_off, *evict_off, *iter_off;
    uint64_t *rec_a, *rec_b;
    uint32_t *chain, *val2_a, *val2_b, *missord, *evict_pair, *par, *pair_start;
    int64_t* cuts;           // trainer cuts of every batch, [T][kMaxTrainers + 1] at most
    int32_t* slot_of_pair;
    uint64_t* keys_c;      // grouping only: the other half of the regrouping sort's ping-pong
    uint32_t* group_counts;   // grouping only: the regrouping sort's first histogram, made by the head scan's first pass
    int64_t* piece_off;
    int64_t* multi_off;
    size_t bytes;
};

PlanWorkspace carve_plan(void* base, size_t cap, int64_t N, int T, int Lcap, bool grouping) {
    Carver c(base, cap);
    PlanWorkspace w{};
    const size_t n = (size_t)(N > 0 ? N : 1);
    w.keys_a = c.take<uint64_t>(n);
    w.keys_b = c.take<uint64_t>(n);
    w.uq = c.take<uint32_t>(n < 64 ? 64 : n);      // later the rows' first positions of the grouping step
    w.tile_batch = c.take<int32_t>((n >> kPosTileShift) + 2);
    w.sort_temp = c.take<uint32_t>(sort_temp_words<kPlanSortIPT>(N));
    w.scan_partials32 = c.take<uint32_t>(scan_partials(N));
    w.scan_partials64 = c.take<uint64_t>(scan_partials(N));
    w.H = c.take<uint32_t>((size_t)(Lcap + 1) * T);
    w.ucount = c.take<uint32_t>(T);
    w.first_use = c.take<uint32_t>(T);
    w.V = c.take<uint32_t>(T + 1);
    w.vcover = c.take<uint32_t>(T + 1);
    w.peak = c.take<uint32_t>(Lcap + 2);
    w.scalars = c.take<PlanScalars>(1);
    w.occ = c.take<int64_t>(T);
    // the per-batch offsets the host reads at the end, side by side so that one copy fetches them all
    w.offsets = c.take<int64_t>(5 * (size_t)(T + 1) + 2);       // + the totals of the lists and of the pieces
    w.prefetch_off = w.offsets;
    w.evict_off = w.offsets + (T + 1);
    w.piece_off = w.offsets + 2 * (size_t)(T + 1);
    w.multi_off = w.offsets + 3 * (size_t)(T + 1);
    w.pair_off = reinterpret_cast<uint32_t*>(w.offsets + 4 * (size_t)(T + 1));
    w.iter_off = c.take<int64_t>(T + 1);
    w.rec_a = c.take<uint64_t>(n);
    w.rec_b = c.take<uint64_t>(n);
    w.chain = c.take<uint32_t>(n);
    w.val2_a = c.take<uint32_t>(n);
    w.val2_b = c.take<uint32_t>(n);
    w.missord = c.take<uint32_t>(n);
    w.evict_pair = c.take<uint32_t>(n);
    w.par = c.take<uint32_t>(n);
    w.pair_start = c.take<uint32_t>(n + 1);
    w.cuts = c.take<int64_t>((size_t)T * (kMaxTrainers + 1));
    w.slot_of_pair = c.take<int32_t>(n);
    if (grouping) {
        w.keys_c = c.take<uint64_t>(n);
        w.group_counts = c.take<uint32_t>((size_t)kMaxRadix * sort_num_tiles<kPlanSortIPT>(N));
    }
    w.bytes = c.used();
    return w;
}

int check_plan_args(const bp_config* cfg, int64_t N, int32_t T) {
    BP_TRY(check_config(cfg));
    if (N < 0 || N >= (int64_t(1) << 31)) return fail(BP_ERR_UNSUPPORTED, "n_lookups %lld outside [0, 2^31)", (long long)N);
    if (T < 1 || T > kMaxIters) return fail(BP_ERR_UNSUPPORTED, "n_iters %d outside [1, %d]", T, kMaxIters);
    if (bits_for(cfg->total_rows) + 2 * bits_for(T) + 2 > 64)
        return fail(BP_ERR_UNSUPPORTED, "id bits + 2 * batch bits + 2 exceed 64");
    return BP_OK;
}

inline dim3 grid_for(int64_t n) { return dim3((unsigned)(n > 0 ? ceil_div(n, kBlock) : 1)); }

}  // namespace
}  // namespace bp

using namespace bp;

BP_EXPORT int bp_oracle_plan_workspace_bytes(const bp_config* cfg, int64_t n_lookups, int32_t n_iters, int32_t with_grouping,
                                             size_t* bytes) {
    if (!bytes) return fail(BP_ERR_INVALID_ARG, "bytes is NULL");
    BP_TRY(check_plan_args(cfg, n_lookups, n_iters));
    const int Lcap = cfg->lookahead > 0 && cfg->lookahead < n_iters ? cfg->lookahead : n_iters;
    *bytes = carve_plan(nullptr, 0, n_lookups, n_iters, Lcap, with_grouping != 0).bytes;
    return BP_OK;
}

namespace bp {
namespace {

struct ChunkArgs {              // chunked planning: emit the first n_emit batches, carry the cache state across
    int n_emit;
    const bp_plan_state* in;    // NULL: the cache is empty and the ring holds slots 0..C-1 in order
    bp_plan_state* out;
};

__global__ __launch_bounds__(kBlock) void iota_slots_kernel(int32_t* p, int64_t n) {
    const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i < n) p[i] = (int32_t)i;
}

// The planner proper.  T_in batches of lookups; in chunk mode (ch != NULL) the rows resident at the chunk boundary
// are put in front of them as a batch 0 of their own, the lists of the first n_emit real batches are reported, and
// the state after the last of them is written out.
int plan_impl(const bp_config* cfg, const int64_t* ids, const int64_t* iter_offsets, int32_t T_in, bp_plan* plan,
              void* workspace, size_t workspace_bytes, hipStream_t stream, const ChunkArgs* ch) {
    if (!plan || !iter_offsets) return fail(BP_ERR_INVALID_ARG, "plan or iter_offsets is NULL");
    if (T_in < 1) return fail(BP_ERR_UNSUPPORTED, "n_iters %d < 1", T_in);
    BP_TRY(check_config(cfg));
    const bool chunk = ch != nullptr;
    const int shift = chunk ? 1 : 0;
    const int T = T_in + shift;                         // batches as the planner counts them
    const int n_emit = chunk ? ch->n_emit : T_in;
    const int64_t C = cfg->capacity;
    const int64_t R0 = chunk && ch->in ? ch->in->n_resident : 0;
    if (chunk) {
        if (n_emit < 1 || n_emit > T_in) return fail(BP_ERR_INVALID_ARG, "n_emit %d outside [1, n_iters]", n_emit);
        if (!ch->out || !ch->out->resident_ids || !ch->out->ring) return fail(BP_ERR_INVALID_ARG, "the output state is NULL");
        if (R0 < 0 || R0 > C) return fail(BP_ERR_INVALID_ARG, "n_resident %lld outside [0, capacity]", (long long)R0);
        if (ch->in && (!ch->in->ring || (R0 && !ch->in->resident_ids))) return fail(BP_ERR_INVALID_ARG, "the input state is NULL");
        if (ch->in && (ch->in->ring == ch->out->ring || (R0 && ch->in->resident_ids == ch->out->resident_ids)))
            return fail(BP_ERR_INVALID_ARG, "input and output state must be different buffers");
    }
    const int64_t N_real = iter_offsets[T_in];
    const int64_t N = N_real + R0;                      // carried residents come first, then the lookups
    BP_TRY(check_plan_args(cfg, N, T));
    if (iter_offsets[0] != 0) return fail(BP_ERR_INVALID_ARG, "iter_offsets[0] != 0");
    for (int i = 0; i < T_in; ++i)
        if (iter_offsets[i + 1] < iter_offsets[i]) return fail(BP_ERR_INVALID_ARG, "iter_offsets decreases at %d", i);
    if (!plan->prefetch_offsets || !plan->evict_offsets || !plan->keep_offsets || !plan->occupancy)
        return fail(BP_ERR_INVALID_ARG, "a host output array of the plan is NULL");
    if (N > 0 && ((N_real > 0 && (!ids || (!plan->lookup_slots && !plan->grouped_lookups))) || !plan->prefetch_ids || !plan->prefetch_slots ||
                  !plan->evict_ids || !plan->evict_slots || !plan->keep_ids || !plan->keep_ttl))
        return fail(BP_ERR_INVALID_ARG, "a device array of the plan is NULL");
    if (!workspace || ((uintptr_t)workspace & 255)) return fail(BP_ERR_INVALID_ARG, "workspace NULL or not 256-byte aligned");

    const int Lcap = cfg->lookahead > 0 && cfg->lookahead < T ? cfg->lookahead : T;   // 0: not configured, any window
    const bool grouping = plan->grouped_lookups || plan->row_recs || plan->piece_recs || plan->piece_offsets;
    if (grouping && !(plan->grouped_lookups && plan->row_recs && plan->piece_recs && plan->piece_offsets))
        return fail(BP_ERR_INVALID_ARG, "the grouping outputs of the plan must be all set or all NULL");
    if (grouping && (((uintptr_t)plan->row_recs | (uintptr_t)plan->piece_recs) & 15))
        return fail(BP_ERR_INVALID_ARG, "row_recs and piece_recs must be 16-byte aligned");
    PlanWorkspace w = carve_plan(workspace, workspace_bytes, N, T, Lcap, grouping);
    if (w.bytes > workspace_bytes)
        return fail(BP_ERR_WORKSPACE_TOO_SMALL, "workspace %zu < required %zu bytes", workspace_bytes, w.bytes);
    const int32_t* ring0 = chunk && ch->in ? ch->in->ring : nullptr;
    const bool owners = plan->keep_owner || plan->trainer_cuts;
    const int P = plan->n_trainers;
    if (owners) {
        if (!plan->keep_owner || !plan->trainer_cuts || P < 1 || P > kMaxTrainers)
            return fail(BP_ERR_INVALID_ARG, "keep_owner, trainer_cuts and n_trainers in [1, %d] go together", kMaxTrainers);
        for (int i = 0; i < T_in; ++i) {
            const int64_t* c = plan->trainer_cuts + (size_t)i * (P + 1);
            bool ok = c[0] == 0 && c[P] == iter_offsets[i + 1] - iter_offsets[i];
            for (int t = 0; t < P && ok; ++t) ok = c[t] <= c[t + 1];
            if (!ok) return fail(BP_ERR_INVALID_ARG, "trainer_cuts of batch %d do not run from 0 to the batch's size", i);
        }
    }

    plan->L_eff = 0;
    plan->L_requested = cfg->lookahead;
    plan->peak_occupancy = 0;
    plan->min_capacity = 0;
    plan->n_unique_pairs = 0;
    if (N == 0) {   // nothing is ever looked up: empty lists, the full requested lookahead is feasible
        for (int i = 0; i <= n_emit; ++i) plan->prefetch_offsets[i] = plan->evict_offsets[i] = plan->keep_offsets[i] = 0;
        for (int i = 0; i < n_emit; ++i) plan->occupancy[i] = 0;
        plan->L_eff = plan->L_requested = cfg->lookahead ? cfg->lookahead : T_in;
        if (grouping)
            for (int i = 0; i <= n_emit; ++i) plan->piece_offsets[i] = 0;
        if (chunk) {                                      // the ring passes through unchanged
            ch->out->n_resident = 0;
            if (ring0) BP_HIP(hipMemcpyAsync(ch->out->ring, ring0, sizeof(int32_t) * C, hipMemcpyDeviceToDevice, stream));
            else BP_LAUNCH(K_FILL, iota_slots_kernel, grid_for(C), dim3(kBlock), 0, stream, ch->out->ring, C);
            BP_HIP(hipStreamSynchronize(stream));
        }
        return BP_OK;
    }

    const int ib = bits_for(T), gb = bits_for(cfg->total_rows);
    std::vector<int64_t> voff((size_t)T + 1);            // batch offsets as the planner counts them
    voff[0] = 0;
    for (int i = 0; i <= T_in; ++i) voff[(size_t)i + shift] = R0 + iter_offsets[i];
    int64_t largest = 1;
    for (int i = 0; i < T; ++i) largest = std::max(largest, voff[(size_t)i + 1] - voff[(size_t)i]);
    const int pb = bits_for(largest);                    // bits of a lookup's place inside its batch
    if (gb + ib + pb > 64 || 32 + ib + pb > 64)
        return fail(BP_ERR_UNSUPPORTED, "id or slot bits (%d / 32) + batch bits (%d) + bits of the largest batch (%d) exceed 64",
                    gb, ib, pb);

    // ---- 1. keys + sort
    BP_HIP(hipMemcpyAsync(w.iter_off, voff.data(), sizeof(int64_t) * (T + 1), hipMemcpyHostToDevice, stream));
    BP_LAUNCH(K_PLAN_KEYS, plan_tile_batch_kernel, grid_for((N >> kPosTileShift) + 1), dim3(kBlock), 0, stream,
              (const int64_t*)w.iter_off, T, (N >> kPosTileShift) + 1, w.tile_batch);
    BP_HIP(hipMemsetAsync(w.scalars, 0, sizeof(PlanScalars), stream));
    if (owners)
        BP_HIP(hipMemcpyAsync(w.cuts, plan->trainer_cuts, sizeof(int64_t) * (size_t)T_in * (P + 1), hipMemcpyHostToDevice,
                              stream));
    // the lookups arrive batch by batch, so a stable sort on the id bits alone leaves every id's words in batch order
    // and, inside a batch, in lookup order
    const BatchOfPos where{w.tile_batch, w.iter_off, T};
    const PlanKeySource source{ids, chunk && ch->in ? ch->in->resident_ids : nullptr, R0, where, ib, pb, cfg->total_rows,
                               w.scalars};
    uint64_t* const kbuf[2] = {w.keys_a, w.keys_b};
    uint32_t* const no_vals[2] = {nullptr, nullptr};
    int sorted_in = -1;
    BP_TRY((radix_sort_from<uint64_t, kPlanSortIPT, PlanKeySource, PlanKeySource, false>(
        source, source, kbuf, no_vals, N, ib + pb, ib + pb + gb, w.sort_temp, stream, &sorted_in)));
    const uint64_t* skeys = kbuf[sorted_in];
    uint64_t* ukey = kbuf[sorted_in ^ 1];          // the other ping-pong buffer is free now
    uint32_t* uq = w.uq;

    // ---- 2. unique pairs
    const int group_bits = grouping ? radix_first_pass_bits(pb, pb + ib) : 0;     // of the regrouping sort's first pass
    if (grouping) {
        const uint32_t ntiles = sort_num_tiles<kPlanSortIPT>(N);
        const uint32_t mask = (1u << group_bits) - 1u;
        if (group_bits > 8)
            BP_LAUNCH(K_SCAN_REDUCE, plan_head_hist_kernel<9>, dim3(ntiles), dim3(kSortBlock), 0, stream, skeys, (uint32_t)N, pb,
                      w.scan_partials32, (uint32_t)scan_num_tiles(N), mask, w.group_counts, ntiles);
        else
            BP_LAUNCH(K_SCAN_REDUCE, plan_head_hist_kernel<8>, dim3(ntiles), dim3(kSortBlock), 0, stream, skeys, (uint32_t)N, pb,
                      w.scan_partials32, (uint32_t)scan_num_tiles(N), mask, w.group_counts, ntiles);
        BP_TRY((device_scan_reduced<uint32_t, AddOp, HeadFlagIn, PairOut>(
            HeadFlagIn{skeys, pb}, PairOut{skeys, pb, ukey, uq, w.pair_start}, N, w.scan_partials32, AddOp(), 0u, stream)));
    } else {
        BP_TRY((device_scan<uint32_t, AddOp, HeadFlagIn, PairOut>(HeadFlagIn{skeys, pb}, PairOut{skeys, pb, ukey, uq, w.pair_start},
                                                                  N, w.scan_partials32, AddOp(), 0u, stream)));
    }
    const uint32_t* n_pairs_dev = w.scan_partials32 + scan_num_tiles(N);     // stays valid until the next 32-bit scan

    // ---- 3. occupancy for every candidate lookahead, L_eff
    // H, ucount, first_use, V, vcover and peak lie one after the other in the workspace: one clear for all of them
    BP_HIP(hipMemsetAsync(w.H, 0, (size_t)((char*)(w.peak + (Lcap + 2)) - (char*)w.H), stream));
    {
        int lds_gaps = (int)((48 * 1024 / 4 - 2 * T) / T);              // histogram rows that fit in 48 KiB next to 2 x [T]
        if (lds_gaps > Lcap - 2) lds_gaps = Lcap - 2;
        if (lds_gaps < 0) lds_gaps = 0;
        int64_t blocks = ceil_div(N, 4 * 32 * 1024);                     // >= 32 Ki pairs per workgroup amortise the flush
        if (blocks > 1024) blocks = 1024;                                // (about one lookup in four starts a pair)
        if (blocks < 1) blocks = 1;
        BP_LAUNCH(K_PLAN_HIST, plan_hist_kernel, dim3((unsigned)blocks), dim3(kBlock),
                  sizeof(uint32_t) * (size_t)(2 + lds_gaps) * T, stream, (const uint64_t*)ukey, n_pairs_dev, ib, T, Lcap,
                  lds_gaps, w.H, w.ucount, w.first_use, (int)chunk, w.V);
    }
    const uint32_t* vcover = nullptr;
    if (chunk) {
        BP_LAUNCH(K_PLAN_OCC, plan_vcover_kernel, dim3(1), dim3(64), 0, stream, (const uint32_t*)w.V, (uint32_t)R0, T, w.vcover);
        vcover = w.vcover;
    }
    const int j_first = shift, j_last = shift + n_emit - 1;      // the batches whose occupancy counts
    BP_LAUNCH(K_PLAN_OCC, plan_occ_prefix_kernel, dim3((unsigned)ceil_div(Lcap, kBlock / kWave)), dim3(kBlock), 0, stream, w.H,
              T, Lcap);
    BP_LAUNCH(K_PLAN_OCC, plan_occ_peak_kernel, dim3(T), dim3(kBlock), 0, stream, (const uint32_t*)w.H,
              (const uint32_t*)w.ucount, vcover, j_first, j_last, T, Lcap, w.peak);
    BP_LAUNCH(K_PLAN_OCC, plan_choose_kernel, dim3(1), dim3(64), 0, stream, (const uint32_t*)w.peak,
              (const uint32_t*)w.ucount, (const uint32_t*)w.first_use, T, Lcap, cfg->lookahead, C - cfg->reserve, shift,
              n_pairs_dev, w.scalars, w.pair_off);
    BP_LAUNCH(K_PLAN_OCC, plan_occ_final_kernel, grid_for(T), dim3(kBlock), 0, stream, (const uint32_t*)w.H,
              (const uint32_t*)w.ucount, vcover, T, (const PlanScalars*)w.scalars, w.occ);
    // the scalars and the occupancies lie side by side: one copy (every copy to pageable memory holds the host up
    // until the stream has drained, and the stream then idles until the next launch arrives)
    const size_t report_bytes = (size_t)((const char*)(w.occ + T) - (const char*)w.scalars);
    std::vector<char> report(report_bytes);
    BP_HIP(hipMemcpyAsync(report.data(), w.scalars, report_bytes, hipMemcpyDeviceToHost, stream));
    BP_HIP(hipStreamSynchronize(stream));
    PlanScalars hs;
    std::memcpy(&hs, report.data(), sizeof(hs));
    const int64_t* hocc = reinterpret_cast<const int64_t*>(report.data() + ((const char*)w.occ - (const char*)w.scalars));
    const uint32_t M = hs.n_pairs;
    if (hs.error_flags & 1u) return fail(BP_ERR_ID_OUT_OF_RANGE, "an id lies outside [0, %lld)", (long long)cfg->total_rows);
    plan->n_unique_pairs = M;
    if ((int64_t)M > plan->list_capacity)
        return fail(BP_ERR_WORKSPACE_TOO_SMALL, "list_capacity %lld < %u unique (id, batch) pairs",
                    (long long)plan->list_capacity, M);
    for (int i = 0; i < n_emit; ++i) plan->occupancy[i] = hocc[(size_t)i + shift];
    plan->min_capacity = hs.min_capacity;
    plan->L_requested = hs.L_requested;
    if (hs.L_eff < 1)
        return fail(BP_ERR_CAPACITY, "capacity %lld - reserve %lld < %lld rows one batch needs in the cache", (long long)C,
                    (long long)cfg->reserve, (long long)hs.min_capacity);
    plan->L_eff = hs.L_eff;
    plan->peak_occupancy = hs.peak;

    // ---- 4. flags, TTL, fetching pair of every pair
    BP_LAUNCH(K_PLAN_FLAGS, plan_flags_kernel, dim3((unsigned)(M > 0 ? ceil_div((int64_t)M, kFlagsTile) : 1)), dim3(kBlock), 0,
              stream, (const uint64_t*)ukey, M, ib,
              (const PlanScalars*)w.scalars, (int)chunk, w.rec_a);
    BP_TRY((device_scan<uint32_t, MaxOp, MissIndexIn, StoreInclusiveU32>(MissIndexIn{w.rec_a, ib}, StoreInclusiveU32{w.chain},
                                                                         M, w.scan_partials32, MaxOp(), 0u, stream)));

    // ---- 5. regroup by batch (the records travel as keys), lists
    // What travels with a record: the number of the pair that fetched its row (for a miss that is the pair itself,
    // which is all the lists need); with the trainer marking asked for, the pair's own number instead, and the list
    // pass then looks the fetching pair up.
    bool ord_in_b = false;
    if (owners) {
        BP_TRY((radix_sort_numbered<uint64_t, kPlanSortIPT>(w.rec_a, w.rec_b, w.val2_a, w.val2_b, M, 0, ib, w.sort_temp,
                                                            stream, &ord_in_b)));
    } else {
        uint64_t* const rbuf[2] = {w.rec_b, w.rec_a};
        uint32_t* const vbuf[2] = {w.val2_b, w.val2_a};
        const SortArrays<uint64_t> rup{w.rec_a, nullptr}, rsrc{w.rec_a, w.chain};
        int r_in = -1;
        BP_TRY((radix_sort_from<uint64_t, kPlanSortIPT, SortArrays<uint64_t>, SortArrays<uint64_t>, true>(
            rup, rsrc, rbuf, vbuf, M, 0, ib, w.sort_temp, stream, &r_in)));
        ord_in_b = r_in == 0;
    }
    const uint64_t* srec = ord_in_b ? w.rec_b : w.rec_a;
    const uint32_t* ord = ord_in_b ? w.val2_b : w.val2_a;
    // prefetch, evict, piece and several-piece offsets start at -1 ("this batch owns no entry")
    BP_LAUNCH(K_FILL, fill_kernel<int64_t>, grid_for(4 * (T + 1)), dim3(kBlock), 0, stream, w.offsets, (int64_t)(4 * (T + 1)),
              (int64_t)-1);
    BP_TRY((device_scan<uint64_t, AddOp, ListCountIn, ListOut>(
        ListCountIn{srec, ib},
        ListOut{srec, ord, w.pair_off, ib, plan->keep_ids, plan->keep_ttl, plan->prefetch_ids, plan->evict_ids, w.missord,
                w.evict_pair, w.prefetch_off, w.evict_off, shift, owners ? plan->keep_owner : nullptr, ukey, M,
                w.pair_start, (uint32_t)N, skeys, pb, w.cuts, P, w.chain, owners},
        M, w.scan_partials64, AddOp(), uint64_t(0), stream)));
    const uint64_t* totals = w.scan_partials64 + scan_num_tiles(M);

    // ---- 6. ring
    BP_LAUNCH(K_PLAN_JUMP, plan_ring_init_kernel, grid_for(M), dim3(kBlock), 0, stream, totals, C,
              (const uint32_t*)w.evict_pair, (const uint32_t*)w.missord, w.par);
    int ring_launch = 0;
    // the first launch one thread per miss; the others, which as a rule find nothing left and are over at once, a
    // small grid that strides over the misses
    const int64_t ring_blocks = M > 0 ? ceil_div((int64_t)M, kBlock) : 1;
    for (int64_t reach = 1; reach < (int64_t)T + 1; reach *= kRingHops) {
        const dim3 ring_grid((unsigned)(ring_launch == 0 ? ring_blocks : std::min<int64_t>(ring_blocks, 2048)));
        BP_LAUNCH(K_PLAN_JUMP, plan_ring_resolve_kernel, ring_grid, dim3(kBlock), 0, stream, totals, kRingHops, w.par,
                  w.scalars, ring_launch);
        ++ring_launch;
    }

    // ---- 7. slots
    BP_LAUNCH(K_PLAN_SLOTS, plan_pair_slots_kernel, grid_for(M), dim3(kBlock), 0, stream, M, (const uint32_t*)w.chain,
              (const uint32_t*)w.missord, (const uint32_t*)w.par, ring0, C, w.slot_of_pair);
    BP_LAUNCH(K_PLAN_SLOTS, plan_list_slots_kernel, grid_for(M), dim3(kBlock), 0, stream, totals, (const uint32_t*)w.par,
              (const uint32_t*)w.evict_pair, (const int32_t*)w.slot_of_pair, ring0, C, plan->prefetch_slots,
              plan->evict_slots, reinterpret_cast<uint64_t*>(w.offsets + 5 * (size_t)(T + 1)));
    if (!grouping && N_real)      // with grouping the slot map is written from the batch-grouped order (step 8)
        BP_LAUNCH(K_PLAN_SLOTS, plan_lookup_slots_kernel, grid_for(N), dim3(kBlock), 0, stream, N, R0, ib, pb, skeys,
                  (const int64_t*)w.iter_off, (const uint32_t*)uq, (const int32_t*)w.slot_of_pair, plan->lookup_slots);

    // ---- 8. grouping for the backward pass
    if (grouping) {
        // one pass as a rule (batch bits <= 9): out of the sorted words into the spare buffer; a second pass would
        // come back into the sorted words' own buffer, which nobody reads any more by then
        const GroupWordSource gsrc{skeys, uq, w.slot_of_pair, ib + pb};
        const SortArrays<uint64_t> gup{skeys, nullptr};
        uint64_t* const gbuf[2] = {w.keys_c, const_cast<uint64_t*>(skeys)};
        int g_in = -1;
        BP_TRY((radix_sort_from<uint64_t, kPlanSortIPT, SortArrays<uint64_t>, GroupWordSource, false>(
            gup, gsrc, gbuf, no_vals, N, pb, pb + ib, w.sort_temp, stream, &g_in, w.group_counts)));
        const uint64_t* gkeys = gbuf[g_in];
        const GroupWord gw{ib, pb};
        // one pass over the grouped words: slot map, grouped_lookups, row starts as bit masks (the masks go to a
        // pair-level buffer that nobody reads any more); then the rows' first positions, into the buffer of the
        // sorted lookups' pair numbers, which is free as well
        const uint32_t per_xcd = blocks_per_xcd(N);
        uint64_t* head_mask = reinterpret_cast<uint64_t*>(w.par);
        uint32_t* row_pos = w.uq;
        const int64_t n_words = (N + 63) / 64;
        BP_LAUNCH(K_PLAN_SLOTS, plan_lookup_slots_grouped_kernel, dim3(per_xcd * kXcds), dim3(kBlock), 0, stream, N, per_xcd,
                  gw, R0, gkeys, where, plan->lookup_slots, plan->grouped_lookups, head_mask);
        uint32_t* rows_before = w.val2_a;                      // free since the lists were written
        BP_TRY((device_scan<uint32_t, AddOp, RowMaskIn, StoreExclusiveU32>(RowMaskIn{head_mask}, StoreExclusiveU32{rows_before},
                                                                          n_words, w.scan_partials32, AddOp(), 0u, stream)));
        BP_LAUNCH(K_PLAN_GROUP, plan_row_starts_kernel, dim3((unsigned)ceil_div(n_words, (int64_t)kBlock)), dim3(kBlock), 0,
                  stream, (const uint64_t*)head_mask, (const uint32_t*)rows_before, n_words, row_pos);
        const uint32_t* n_rows = w.scan_partials32 + scan_num_tiles(n_words);
        // at most one row per pair (fewer only where the look-ahead batches of a chunk hold rows without a slot)
        const int64_t rows_bound = (int64_t)M - R0 > 0 ? (int64_t)M - R0 : 1;
        BP_TRY((device_scan<uint64_t, AddOp, RowPiecesIn, GroupRecordOut>(
            RowPiecesIn{row_pos, n_rows, (uint32_t)N},
            GroupRecordOut{row_pos, n_rows, (uint32_t)N, gkeys, gw, (const int64_t*)w.iter_off, R0,
                           reinterpret_cast<uint4*>(plan->row_recs), reinterpret_cast<uint4*>(plan->piece_recs),
                           w.piece_off, w.multi_off},
            rows_bound, w.scan_partials64, AddOp(), uint64_t(0), stream)));
        const uint32_t* n_pieces_dev = reinterpret_cast<const uint32_t*>(w.scan_partials64 + scan_num_tiles(rows_bound));
        BP_LAUNCH(K_PLAN_GROUP, plan_piece_partial_kernel, grid_for((int64_t)piece_capacity_for(N_real)), dim3(kBlock), 0,
                  stream, reinterpret_cast<uint4*>(plan->piece_recs), n_pieces_dev, T, (const int64_t*)w.multi_off,
                  reinterpret_cast<uint64_t*>(w.offsets + 5 * (size_t)(T + 1) + 1));
    }

    // ---- CSR offsets to the host (in chunk mode: of the emitted batches; positions in the device lists, so the
    // first offset is where the carried residents' own entries end)
    std::vector<int64_t> hoffsets(5 * (size_t)(T + 1) + 2);     // one copy: the five arrays and the totals lie side by side
    BP_HIP(hipMemcpyAsync(hoffsets.data(), w.offsets, sizeof(int64_t) * hoffsets.size(), hipMemcpyDeviceToHost, stream));
    BP_HIP(hipStreamSynchronize(stream));
    int64_t* const hpre = hoffsets.data();
    int64_t* const hev = hpre + (T + 1);
    int64_t* const hpiece = hpre + 2 * (size_t)(T + 1);
    const uint32_t* const hpair = reinterpret_cast<const uint32_t*>(hpre + 4 * (size_t)(T + 1));
    const uint64_t htot = (uint64_t)hoffsets[5 * (size_t)(T + 1)];
    const uint64_t n_pieces_multi = grouping ? (uint64_t)hoffsets[5 * (size_t)(T + 1) + 1] : 0;
    const int64_t n_miss = (int64_t)(uint32_t)htot, n_evict = (int64_t)(htot >> 32);
    hpre[T] = n_miss;
    hev[T] = n_evict;
    for (int i = T - 1; i >= 0; --i) {   // batches without lookups own no pair: their lists are empty
        if (hpre[i] < 0) hpre[i] = hpre[i + 1];
        if (hev[i] < 0) hev[i] = hev[i + 1];
    }
    for (int i = 0; i <= n_emit; ++i) {
        plan->prefetch_offsets[i] = hpre[(size_t)i + shift];
        plan->evict_offsets[i] = hev[(size_t)i + shift];
        plan->keep_offsets[i] = (int64_t)hpair[(size_t)i + shift];
    }
    if (grouping) {
        hpiece[T] = (int64_t)(uint32_t)n_pieces_multi;          // pieces of the long rows of all batches
        for (int i = T - 1; i >= 0; --i)
            if (hpiece[i] < 0) hpiece[i] = hpiece[i + 1];
        for (int i = 0; i <= n_emit; ++i) plan->piece_offsets[i] = hpiece[(size_t)i + shift];
    }
    if (!chunk) {
        if (n_miss != n_evict) return fail(BP_ERR_HIP, "internal: %lld prefetches but %lld evictions", (long long)n_miss, (long long)n_evict);
        return BP_OK;
    }

    // ---- 9. the state after the last emitted batch
    const uint32_t e = (uint32_t)j_last;
    const int64_t miss_e = hpre[(size_t)e + 1], evict_e = hev[(size_t)e + 1];       // misses / evictions through batch e
    BP_TRY((device_scan<uint32_t, AddOp, ResidentFlagIn, ResidentOut>(
        ResidentFlagIn{ukey, M, ib, e, w.scalars},
        ResidentOut{ukey, (const int32_t*)w.slot_of_pair, ib, ch->out->resident_ids, ch->out->ring}, M, w.scan_partials32,
        AddOp(), 0u, stream)));
    uint32_t n_res = 0;
    BP_HIP(hipMemcpyAsync(&n_res, w.scan_partials32 + scan_num_tiles(M), sizeof(uint32_t), hipMemcpyDeviceToHost, stream));
    BP_HIP(hipStreamSynchronize(stream));
    if ((int64_t)n_res != miss_e - evict_e)
        return fail(BP_ERR_HIP, "internal: %u resident rows but %lld misses - %lld evictions", n_res, (long long)miss_e,
                    (long long)evict_e);
    const int64_t n_free = C + evict_e - miss_e;
    if (n_free > 0)
        BP_LAUNCH(K_PLAN_SLOTS, plan_state_queue_kernel, grid_for(n_free), dim3(kBlock), 0, stream, miss_e, evict_e, C, ring0,
                  (const int32_t*)plan->evict_slots, (int64_t)n_res, ch->out->ring);
    BP_HIP(hipStreamSynchronize(stream));
    ch->out->n_resident = n_res;
    return BP_OK;
}

}  // namespace
}  // namespace bp

BP_EXPORT int bp_oracle_plan(const bp_config* cfg, const int64_t* ids, const int64_t* iter_offsets, int32_t n_iters,
                              bp_plan* plan, void* workspace, size_t workspace_bytes, void* stream) {
    return plan_impl(cfg, ids, iter_offsets, n_iters, plan, workspace, workspace_bytes, (hipStream_t)stream, nullptr);
}

BP_EXPORT int bp_oracle_plan_chunk_workspace_bytes(const bp_config* cfg, int64_t n_lookups, int32_t n_iters,
                                                   int32_t with_grouping, size_t* bytes) {
    if (!bytes) return fail(BP_ERR_INVALID_ARG, "bytes is NULL");
    BP_TRY(check_config(cfg));
    if (n_lookups < 0 || n_iters < 1) return fail(BP_ERR_INVALID_ARG, "n_lookups < 0 or n_iters < 1");
    BP_TRY(check_plan_args(cfg, n_lookups + cfg->capacity, n_iters + 1));
    const int T = n_iters + 1;
    const int Lcap = cfg->lookahead > 0 && cfg->lookahead < T ? cfg->lookahead : T;
    *bytes = carve_plan(nullptr, 0, n_lookups + cfg->capacity, T, Lcap, with_grouping != 0).bytes;
    return BP_OK;
}

BP_EXPORT int bp_oracle_plan_chunk(const bp_config* cfg, const int64_t* ids, const int64_t* iter_offsets, int32_t n_iters,
                                    int32_t n_emit, const bp_plan_state* state_in, bp_plan_state* state_out, bp_plan* plan,
                                    void* workspace, size_t workspace_bytes, void* stream) {
    const ChunkArgs ch{n_emit, state_in, state_out};
    return plan_impl(cfg, ids, iter_offsets, n_iters, plan, workspace, workspace_bytes, (hipStream_t)stream, &ch);
}
