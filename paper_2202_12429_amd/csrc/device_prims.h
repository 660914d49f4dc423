// Wavefront- and workgroup-level building blocks for gfx950 (64-wide wavefronts) and the two device-wide
// primitives the planner and the backward pass share: a tiled scan and a stable LSD radix sort.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

#include "common.h"

namespace bp {

// ---------------------------------------------------------------------------------------------
// wavefront helpers
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ int lane_id() { return threadIdx.x & (kWave - 1); }

__device__ __forceinline__ uint64_t lanemask_lt() { return (uint64_t(1) << lane_id()) - 1; }

struct AddOp {
    template <typename T>
    __device__ __forceinline__ T operator()(T a, T b) const { return a + b; }
};
struct MaxOp {
    template <typename T>
    __device__ __forceinline__ T operator()(T a, T b) const { return a > b ? a : b; }
};

template <typename T, typename Op>
__device__ __forceinline__ T wave_inclusive_scan(T x, Op op) {
    const int lane = lane_id();
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
        T y = __shfl_up(x, off, kWave);
        if (lane >= off) x = op(y, x);
    }
    return x;
}

// Scan of one value per thread over a workgroup of BLOCK threads (BLOCK % 64 == 0), thread order.
// `wave_tot` is LDS scratch of BLOCK/64 entries.  Writes the exclusive and inclusive values and the
// reduction over the whole workgroup.  Ends with a barrier, so wave_tot can be reused at once.
template <int BLOCK, typename T, typename Op>
__device__ __forceinline__ void block_scan(T x, Op op, T identity, T* wave_tot, T* exclusive, T* inclusive,
                                           T* block_total) {
    constexpr int WAVES = BLOCK / kWave;
    const int w = threadIdx.x / kWave, lane = lane_id();
    T inc = wave_inclusive_scan(x, op);
    T exc = __shfl_up(inc, 1, kWave);
    if (lane == 0) exc = identity;
    if (lane == kWave - 1) wave_tot[w] = inc;
    __syncthreads();
    T prefix = identity, total = identity;
#pragma unroll
    for (int i = 0; i < WAVES; ++i) {
        T t = wave_tot[i];
        if (i < w) prefix = op(prefix, t);
        total = op(total, t);
    }
    __syncthreads();
    *exclusive = op(prefix, exc);
    *inclusive = op(prefix, inc);
    *block_total = total;
}

// ---------------------------------------------------------------------------------------------
// device-wide scan:  out(i, exclusive_prefix_i, inclusive_prefix_i)  for value_i = in(i), i in [0, n)
//   pass 1  per-tile reduction                   -> partials[tile]
//   pass 2  one workgroup scans the partials in place (exclusive) and appends the grand total
//   pass 3  per-tile scan seeded with its partial
// A tile is kScanTile consecutive elements; each wavefront owns a contiguous stretch of it and takes it in
// kScanRounds rounds of 64 consecutive elements (lane l holds element r*64 + l of the stretch), so loads coalesce
// and a round is scanned with lane shuffles alone; the workgroup meets at one barrier per tile.
// Op must be associative and commutative (add, max).
// ---------------------------------------------------------------------------------------------
constexpr int kScanBlock = 256;
constexpr int kScanRounds = 8;
constexpr int kScanTile = kScanBlock * kScanRounds;
constexpr int kScanWaveStretch = kWave * kScanRounds;

template <typename T, typename Op>
__device__ __forceinline__ T wave_reduce(T x, Op op) {
#pragma unroll
    for (int off = kWave / 2; off >= 1; off >>= 1) x = op(x, __shfl_xor(x, off, kWave));
    return x;
}

template <typename T, typename Op, typename In>
__global__ __launch_bounds__(kScanBlock) void scan_reduce_kernel(In in, int64_t n, T* partials, Op op, T identity) {
    __shared__ T wave_tot[kScanBlock / kWave];
    const int w = threadIdx.x / kWave, lane = lane_id();
    const int64_t base = (int64_t)blockIdx.x * kScanTile + w * kScanWaveStretch + lane;
    T acc = identity;
#pragma unroll
    for (int r = 0; r < kScanRounds; ++r) {
        const int64_t i = base + r * kWave;
        if (i < n) acc = op(acc, in(i));
    }
    acc = wave_reduce(acc, op);
    if (lane == 0) wave_tot[w] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        T total = identity;
#pragma unroll
        for (int k = 0; k < kScanBlock / kWave; ++k) total = op(total, wave_tot[k]);
        partials[blockIdx.x] = total;
    }
}

// One workgroup: it is the serial part of every scan.  A thread takes kSpinePerThread consecutive partials per round
// and moves them in 16-byte accesses: with one 4-byte access per partial and thread the kernel's time follows the
// number of memory instructions, whatever the rounds (41,600 partials, the spine of a scan over 85 M elements: 42 us
// element by element, 12 us this way).
constexpr int kSpinePerThread = 8;
template <typename T, typename Op>
__global__ __launch_bounds__(1024) void scan_spine_kernel(T* partials, int64_t nparts, Op op, T identity) {
    constexpr int VEC = kSpinePerThread * (int)sizeof(T) / 16;
    static_assert(kSpinePerThread * sizeof(T) % 16 == 0, "a thread's partials are a whole number of 16-byte pieces");
    __shared__ T wave_tot[1024 / kWave];
    const bool aligned = (reinterpret_cast<uintptr_t>(partials) & 15) == 0;
    T carry = identity;
    for (int64_t base = 0; base < nparts; base += 1024 * kSpinePerThread) {
        const int64_t i0 = base + (int64_t)threadIdx.x * kSpinePerThread;
        const bool whole = aligned && i0 + kSpinePerThread <= nparts;
        union {
            T v[kSpinePerThread];
            uint4 q[VEC];
        } mine;
        if (whole) {
            const uint4* src = reinterpret_cast<const uint4*>(partials + i0);
#pragma unroll
            for (int k = 0; k < VEC; ++k) mine.q[k] = src[k];
        } else {
#pragma unroll
            for (int k = 0; k < kSpinePerThread; ++k) mine.v[k] = i0 + k < nparts ? partials[i0 + k] : identity;
        }
        T sum = identity;
#pragma unroll
        for (int k = 0; k < kSpinePerThread; ++k) sum = op(sum, mine.v[k]);
        T exc, inc, total;
        block_scan<1024>(sum, op, identity, wave_tot, &exc, &inc, &total);
        T run = op(carry, exc);
#pragma unroll
        for (int k = 0; k < kSpinePerThread; ++k) {       // every partial becomes the scan of those before it
            const T next = op(run, mine.v[k]);
            mine.v[k] = run;
            run = next;
        }
        if (whole) {
            uint4* dst = reinterpret_cast<uint4*>(partials + i0);
#pragma unroll
            for (int k = 0; k < VEC; ++k) dst[k] = mine.q[k];
        } else {
#pragma unroll
            for (int k = 0; k < kSpinePerThread; ++k)
                if (i0 + k < nparts) partials[i0 + k] = mine.v[k];
        }
        carry = op(carry, total);
    }
    if (threadIdx.x == 0) partials[nparts] = carry;
}

template <typename T, typename Op, typename In, typename Out>
__global__ __launch_bounds__(kScanBlock) void scan_apply_kernel(In in, Out out, int64_t n, const T* partials, Op op,
                                                                T identity) {
    __shared__ T wave_tot[kScanBlock / kWave];
    const int w = threadIdx.x / kWave, lane = lane_id();
    const int64_t base = (int64_t)blockIdx.x * kScanTile + w * kScanWaveStretch + lane;
    T v[kScanRounds];
    T mine = identity;
#pragma unroll
    for (int r = 0; r < kScanRounds; ++r) {
        const int64_t i = base + r * kWave;
        v[r] = i < n ? in(i) : identity;
        mine = op(mine, v[r]);
    }
    mine = wave_reduce(mine, op);
    if (lane == 0) wave_tot[w] = mine;
    __syncthreads();
    T carry = partials[blockIdx.x];                       // everything before this wavefront's stretch
    for (int k = 0; k < w; ++k) carry = op(carry, wave_tot[k]);
#pragma unroll
    for (int r = 0; r < kScanRounds; ++r) {
        const int64_t i = base + r * kWave;
        const T inc = wave_inclusive_scan(v[r], op);
        T exc = __shfl_up(inc, 1, kWave);
        if (lane == 0) exc = identity;
        if (i < n) out(i, op(carry, exc), op(carry, inc));
        carry = op(carry, __shfl(inc, kWave - 1, kWave));
    }
}

inline int64_t scan_num_tiles(int64_t n) { return n > 0 ? ceil_div(n, kScanTile) : 1; }
// partials needed by device_scan: one per tile plus the grand total
inline size_t scan_partials(int64_t n) { return (size_t)scan_num_tiles(n) + 1; }

// Runs the three passes on `stream`.  partials[scan_num_tiles(n)] holds the grand total afterwards.  The per-tile
// reduction reads its values through `in_reduce`, the final pass through `in_apply`: the same values, but the first
// may leave notes for the second (flags that are costly to derive twice).
template <typename T, typename Op, typename InReduce, typename InApply, typename Out>
int device_scan2(InReduce in_reduce, InApply in_apply, Out out, int64_t n, T* partials, Op op, T identity,
                 hipStream_t stream) {
    const int64_t tiles = scan_num_tiles(n);
    BP_LAUNCH(K_SCAN_REDUCE, (scan_reduce_kernel<T, Op, InReduce>), dim3((unsigned)tiles), dim3(kScanBlock), 0, stream,
              in_reduce, n, partials, op, identity);
    BP_LAUNCH(K_SCAN_SPINE, (scan_spine_kernel<T, Op>), dim3(1), dim3(1024), 0, stream, partials, tiles, op, identity);
    BP_LAUNCH(K_SCAN_APPLY, (scan_apply_kernel<T, Op, InApply, Out>), dim3((unsigned)tiles), dim3(kScanBlock), 0, stream,
              in_apply, out, n, (const T*)partials, op, identity);
    return BP_OK;
}
// Passes 2 and 3 alone, for a caller whose own kernel has left the per-tile reductions in `partials`.
template <typename T, typename Op, typename InApply, typename Out>
int device_scan_reduced(InApply in_apply, Out out, int64_t n, T* partials, Op op, T identity, hipStream_t stream) {
    const int64_t tiles = scan_num_tiles(n);
    BP_LAUNCH(K_SCAN_SPINE, (scan_spine_kernel<T, Op>), dim3(1), dim3(1024), 0, stream, partials, tiles, op, identity);
    BP_LAUNCH(K_SCAN_APPLY, (scan_apply_kernel<T, Op, InApply, Out>), dim3((unsigned)tiles), dim3(kScanBlock), 0, stream,
              in_apply, out, n, (const T*)partials, op, identity);
    return BP_OK;
}
template <typename T, typename Op, typename In, typename Out>
int device_scan(In in, Out out, int64_t n, T* partials, Op op, T identity, hipStream_t stream) {
    return device_scan2<T, Op, In, In, Out>(in, in, out, n, partials, op, identity, stream);
}

// ---------------------------------------------------------------------------------------------
// stable LSD radix sort of (key, 32-bit value) pairs, RB = 8 or 9 bits per pass
//   upsweep    per-tile digit histogram              -> counts[digit][tile]
//   scan       exclusive scan of counts (digit-major) -> global base of every (digit, tile)
//   downsweep  per-tile stable ranking in LDS, coalesced scatter
// Ranking inside a tile: each wavefront owns a contiguous 64*IPT stretch, lane l holds elements
// j*64+l; for every j the lanes that share a digit find each other with ballots (one per digit bit),
// rank = running per-wave digit count + number of lower lanes among the peers.
// The bits to sort are spread evenly over the fewest passes of at most 9 bits (34 bits: 9+9+8+8).
// ---------------------------------------------------------------------------------------------
constexpr int kSortBlock = 256;
// Tile of this workgroup.  Workgroups go to the eight XCDs round-robin; with the mapping below XCD x takes the x-th
// eighth of the tiles in order, so the tiles whose scattered runs are neighbours in memory meet in one L2.
__device__ __forceinline__ uint32_t sort_tile_of_block(uint32_t ntiles) {
    const uint32_t per = (ntiles + 7u) / 8u;
    return (blockIdx.x % 8u) * per + blockIdx.x / 8u;
}
inline uint32_t sort_grid(uint32_t ntiles) { return (ntiles + 7u) / 8u * 8u; }
constexpr int kMaxRadixBits = 9;
constexpr int kMaxRadix = 1 << kMaxRadixBits;

// Where a pass reads its elements.  Plain arrays are the common case; a pass may also make its keys on the fly from
// something else (and so save writing them out first).  A source loads what it needs for element i with load(i),
// which depends on nothing but i, so a thread's loads all go out together; a cursor per thread then turns what was
// loaded into the key, for element numbers in ascending order.
template <typename K>
struct SortArrays {
    const K* keys;
    const uint32_t* vals;     // NULL for a sort of keys alone
    typedef K Raw;
    __device__ __forceinline__ K load(uint32_t i) const { return keys[i]; }
    __device__ __forceinline__ uint32_t val(uint32_t i) const { return vals[i]; }
    struct Cursor {
        __device__ __forceinline__ Cursor(const SortArrays&, uint32_t) {}
        __device__ __forceinline__ K key(uint32_t, K raw) { return raw; }
    };
};

// Keys whose values are their own places in the array (a sort that is to return the permutation it applied).
template <typename K>
struct SortKeysNumbered {
    const K* keys;
    typedef K Raw;
    __device__ __forceinline__ K load(uint32_t i) const { return keys[i]; }
    __device__ __forceinline__ uint32_t val(uint32_t i) const { return i; }
    struct Cursor {
        __device__ __forceinline__ Cursor(const SortKeysNumbered&, uint32_t) {}
        __device__ __forceinline__ K key(uint32_t, K raw) { return raw; }
    };
};

template <typename K, int IPT, int RB, typename Src>
__global__ __launch_bounds__(kSortBlock) void sort_upsweep_kernel(Src src, uint32_t n, int shift, uint32_t mask,
                                                                  uint32_t* __restrict__ counts, uint32_t ntiles) {
    constexpr int RADIX = 1 << RB;
    __shared__ uint32_t hist[RADIX];
    const uint32_t tile = sort_tile_of_block(ntiles);
    if (tile >= ntiles) return;
    for (int d = threadIdx.x; d < RADIX; d += kSortBlock) hist[d] = 0;
    __syncthreads();
    const uint32_t base = tile * (kSortBlock * IPT);
    if (base + threadIdx.x < n) {
        typename Src::Raw raw[IPT];
#pragma unroll
        for (int j = 0; j < IPT; ++j) {
            uint32_t i = base + j * kSortBlock + threadIdx.x;
            raw[j] = src.load(i < n ? i : n - 1u);
        }
        typename Src::Cursor cur(src, base + threadIdx.x);
#pragma unroll
        for (int j = 0; j < IPT; ++j) {
            uint32_t i = base + j * kSortBlock + threadIdx.x;
            if (i < n) {
                // skewed keys put many lanes on one counter: the lanes that share the first active lane's digit count
                // themselves with one addition, the others add one by one
                const uint32_t d = (uint32_t)(cur.key(i, raw[j]) >> shift) & mask;
                const uint32_t d0 = __builtin_amdgcn_readfirstlane(d);
                const uint64_t same = __ballot(d == d0);
                if (d != d0) atomicAdd(&hist[d], 1u);
                else if ((same & lanemask_lt()) == 0) atomicAdd(&hist[d0], (uint32_t)__popcll(same));
            }
        }
    }
    __syncthreads();
    for (int d = threadIdx.x; d < RADIX; d += kSortBlock) counts[(size_t)d * ntiles + tile] = hist[d];
}

template <typename K, int IPT, int RB, typename Src, bool VALS>
__global__ __launch_bounds__(kSortBlock) void sort_downsweep_kernel(Src src, K* __restrict__ kout,
                                                                    uint32_t* __restrict__ vout, uint32_t n, int shift,
                                                                    uint32_t mask, const uint32_t* __restrict__ bases,
                                                                    uint32_t ntiles) {
    constexpr int RADIX = 1 << RB;
    constexpr int DPT = RADIX / kSortBlock;    // consecutive digits owned by a thread in the digit scan (1 or 2)
    constexpr int WAVES = kSortBlock / kWave;
    constexpr int TILE = kSortBlock * IPT;
    constexpr int WTILE = kWave * IPT;
    static_assert(RADIX % kSortBlock == 0, "radix must be a multiple of the workgroup size");
    __shared__ uint32_t wcnt[WAVES][RADIX];    // per-wave digit counts, then per-wave exclusive offsets
    __shared__ uint32_t dstart[RADIX];         // tile-local start of each digit
    __shared__ uint32_t gbase[RADIX];          // global base of the digit for this tile, minus dstart
    __shared__ uint32_t wave_tot[WAVES];
    __shared__ K skeys[TILE];
    __shared__ uint32_t svals[VALS ? TILE : 1];

    const int tid = threadIdx.x, lane = tid & (kWave - 1), w = tid / kWave;
    const uint32_t tile = sort_tile_of_block(ntiles);
    if (tile >= ntiles) return;
    for (int d = tid; d < WAVES * RADIX; d += kSortBlock) (&wcnt[0][0])[d] = 0;
    __syncthreads();

    const uint32_t tile_base = tile * TILE;
    const uint32_t wbase = tile_base + w * WTILE;
    K key[IPT];
    uint32_t val[VALS ? IPT : 1];
    uint32_t rank[IPT];
    {
        typename Src::Raw raw[IPT];
#pragma unroll
        for (int j = 0; j < IPT; ++j) {
            uint32_t i = wbase + j * kWave + lane;
            raw[j] = src.load(i < n ? i : n - 1u);
            if constexpr (VALS) val[j] = i < n ? src.val(i) : 0u;
        }
        typename Src::Cursor cur(src, wbase + lane < n ? wbase + lane : 0u);
#pragma unroll
        for (int j = 0; j < IPT; ++j) {
            uint32_t i = wbase + j * kWave + lane;
            key[j] = i < n ? cur.key(i, raw[j]) : K(~K(0));
        }
    }
    const uint64_t lt = lanemask_lt();
#pragma unroll
    for (int j = 0; j < IPT; ++j) {
        const bool valid = wbase + j * kWave + lane < n;
        const uint32_t d = (uint32_t)(key[j] >> shift) & mask;
        uint64_t peers = __ballot(valid);
#pragma unroll
        for (int b = 0; b < RB; ++b) {
            const bool bit = (d >> b) & 1u;
            const uint64_t m = __ballot(bit);
            peers &= bit ? m : ~m;
        }
        const uint32_t before = wcnt[w][d];
        rank[j] = before + (uint32_t)__popcll(peers & lt);
        __builtin_amdgcn_wave_barrier();
        if (valid && (peers & lt) == 0) wcnt[w][d] = before + (uint32_t)__popcll(peers);   // lowest peer lane
        __builtin_amdgcn_wave_barrier();
    }
    __syncthreads();

    {   // thread tid owns digits tid*DPT .. tid*DPT+DPT-1: offsets of the waves inside each digit, then digit starts
        uint32_t tot[DPT];
        uint32_t sum = 0;
#pragma unroll
        for (int k = 0; k < DPT; ++k) {
            const int d = tid * DPT + k;
            uint32_t run = 0;
#pragma unroll
            for (int i = 0; i < WAVES; ++i) {
                uint32_t c = wcnt[i][d];
                wcnt[i][d] = run;
                run += c;
            }
            tot[k] = run;
            sum += run;
        }
        uint32_t exc, inc, total;
        block_scan<kSortBlock>(sum, AddOp(), 0u, wave_tot, &exc, &inc, &total);
#pragma unroll
        for (int k = 0; k < DPT; ++k) {
            const int d = tid * DPT + k;
            dstart[d] = exc;
            gbase[d] = bases[(size_t)d * ntiles + tile] - exc;
            exc += tot[k];
        }
    }
    __syncthreads();

#pragma unroll
    for (int j = 0; j < IPT; ++j) {
        if (wbase + j * kWave + lane < n) {
            const uint32_t d = (uint32_t)(key[j] >> shift) & mask;
            const uint32_t pos = dstart[d] + wcnt[w][d] + rank[j];
            skeys[pos] = key[j];
            if constexpr (VALS) svals[pos] = val[j];
        }
    }
    __syncthreads();

    const uint32_t tile_n = n - tile_base < (uint32_t)TILE ? n - tile_base : (uint32_t)TILE;
#pragma unroll
    for (int j = 0; j < IPT; ++j) {
        const uint32_t pos = j * kSortBlock + tid;
        if (pos < tile_n) {
            const K k = skeys[pos];
            const uint32_t dst = gbase[(uint32_t)(k >> shift) & mask] + pos;
            kout[dst] = k;
            if constexpr (VALS) vout[dst] = svals[pos];
        }
    }
}

struct LoadU32 {
    const uint32_t* p;
    __device__ __forceinline__ uint32_t operator()(int64_t i) const { return p[i]; }
};
struct StoreExclusiveU32 {
    uint32_t* p;
    __device__ __forceinline__ void operator()(int64_t i, uint32_t exc, uint32_t) const { p[i] = exc; }
};

template <int IPT>
inline uint32_t sort_num_tiles(int64_t n) { return (uint32_t)(n > 0 ? ceil_div(n, kSortBlock * IPT) : 1); }

// uint32 words of temporary storage for radix_sort_pairs<.., IPT> of n elements
template <int IPT>
inline size_t sort_temp_words(int64_t n) {
    size_t counts = (size_t)kMaxRadix * sort_num_tiles<IPT>(n);
    return counts + 64 + scan_partials((int64_t)counts) + 64;
}

// One pass.  The histogram reads `up`, the scatter reads `src`: the same elements, but a source that has to fetch
// more than the digit needs may leave that to the scatter alone.
// `ready`: the pass's histogram (counts[digit][tile], as the upsweep writes it) made by a kernel of the caller's that
// read the same elements anyway; NULL: the upsweep makes it.
template <typename K, int IPT, int RB, typename Up, typename Src, bool VALS>
int radix_sort_pass(const Up& up, const Src& src, K* kout, uint32_t* vout, int64_t n, int bit, int nb, uint32_t* counts,
                    uint32_t* partials, uint32_t ntiles, hipStream_t stream, const uint32_t* ready) {
    const int64_t ncounts = (int64_t)(1 << RB) * ntiles;
    const uint32_t mask = (1u << nb) - 1u;
    if (!ready)
        BP_LAUNCH(K_SORT_UPSWEEP, (sort_upsweep_kernel<K, IPT, RB, Up>), dim3(sort_grid(ntiles)), dim3(kSortBlock), 0, stream,
                  up, (uint32_t)n, bit, mask, counts, ntiles);
    BP_TRY((device_scan<uint32_t, AddOp, LoadU32, StoreExclusiveU32>(LoadU32{ready ? ready : counts}, StoreExclusiveU32{counts},
                                                                     ncounts, partials, AddOp(), 0u, stream)));
    BP_LAUNCH(K_SORT_DOWNSWEEP, (sort_downsweep_kernel<K, IPT, RB, Src, VALS>), dim3(sort_grid(ntiles)), dim3(kSortBlock), 0,
              stream, src, kout, vout, (uint32_t)n, bit, mask, (const uint32_t*)counts, ntiles);
    return BP_OK;
}

template <typename K, int IPT, typename Up, typename Src, bool VALS>
int radix_sort_one_pass(const Up& up, const Src& src, K* kout, uint32_t* vout, int64_t n, int bit, int nb,
                        uint32_t* counts, uint32_t* partials, uint32_t ntiles, hipStream_t stream,
                        const uint32_t* ready = nullptr) {
    if (nb > 8)
        return radix_sort_pass<K, IPT, 9, Up, Src, VALS>(up, src, kout, vout, n, bit, nb, counts, partials, ntiles, stream,
                                                         ready);
    return radix_sort_pass<K, IPT, 8, Up, Src, VALS>(up, src, kout, vout, n, bit, nb, counts, partials, ntiles, stream, ready);
}

// Bits the first pass of a sort over [begin_bit, end_bit) takes (the passes share the bits evenly).
inline int radix_first_pass_bits(int begin_bit, int end_bit) {
    const int total = end_bit - begin_bit;
    if (total <= 0) return 0;
    const int passes = (total + kMaxRadixBits - 1) / kMaxRadixBits;
    return (total + passes - 1) / passes;
}

// Stable sort of n elements by key bits [begin_bit, end_bit).  The first pass reads `first` (any source; its
// histogram reads `first_up`, which must give the same sorted bits) and writes buffer 0, every later pass reads the
// buffer the one before wrote and writes the other one; *result says which buffer holds the sorted output (-1: no
// pass ran, nothing was written).  VALS: 32-bit values travel with the keys.  n < 2^32 - kSortBlock*IPT.
// first_counts: the first pass's histogram where a kernel of the caller's has made it already (radix_sort_pass).
template <typename K, int IPT, typename Up, typename Src, bool VALS>
int radix_sort_from(const Up& first_up, const Src& first, K* const kbuf[2], uint32_t* const vbuf[2], int64_t n,
                    int begin_bit, int end_bit, uint32_t* temp, hipStream_t stream, int* result,
                    const uint32_t* first_counts = nullptr) {
    *result = -1;
    if (n <= 0 || end_bit <= begin_bit) return BP_OK;
    const uint32_t ntiles = sort_num_tiles<IPT>(n);
    uint32_t* counts = temp;
    uint32_t* partials = temp + (((size_t)kMaxRadix * ntiles + 63) & ~size_t(63));
    const int total = end_bit - begin_bit;
    const int passes = (total + kMaxRadixBits - 1) / kMaxRadixBits;
    int bit = begin_bit;
    for (int p = 0; p < passes; ++p) {
        const int left = end_bit - bit;
        const int nb = (left + (passes - p) - 1) / (passes - p);      // spread the remaining bits evenly
        const int out = p & 1;
        if (p == 0) {
            BP_TRY((radix_sort_one_pass<K, IPT, Up, Src, VALS>(first_up, first, kbuf[out], VALS ? vbuf[out] : nullptr, n, bit,
                                                               nb, counts, partials, ntiles, stream, first_counts)));
        } else {
            const SortArrays<K> in{kbuf[out ^ 1], VALS ? vbuf[out ^ 1] : nullptr};
            BP_TRY((radix_sort_one_pass<K, IPT, SortArrays<K>, SortArrays<K>, VALS>(in, in, kbuf[out],
                                                                                    VALS ? vbuf[out] : nullptr, n, bit, nb,
                                                                                    counts, partials, ntiles, stream)));
        }
        bit += nb;
        *result = out;
    }
    return BP_OK;
}

// Sorts n (key, value) pairs by key bits [begin_bit, end_bit), stable.  The data ping-pongs between
// (keys_a, vals_a) and (keys_b, vals_b); input is in the `a` buffers; *result_in_b tells where the
// sorted output ended up.  n < 2^32 - kSortBlock*IPT.
template <typename K, int IPT>
int radix_sort_pairs(K* keys_a, K* keys_b, uint32_t* vals_a, uint32_t* vals_b, int64_t n, int begin_bit, int end_bit,
                     uint32_t* temp, hipStream_t stream, bool* result_in_b) {
    K* const kbuf[2] = {keys_b, keys_a};
    uint32_t* const vbuf[2] = {vals_b, vals_a};
    int result = -1;
    const SortArrays<K> in{keys_a, vals_a};
    BP_TRY((radix_sort_from<K, IPT, SortArrays<K>, SortArrays<K>, true>(in, in, kbuf, vbuf, n, begin_bit, end_bit, temp, stream,
                                                                        &result)));
    *result_in_b = result == 0;
    return BP_OK;
}

// The same with the values 0 .. n-1 in the order of the input: vals_a is scratch, nobody has to fill it.
template <typename K, int IPT>
int radix_sort_numbered(K* keys_a, K* keys_b, uint32_t* vals_a, uint32_t* vals_b, int64_t n, int begin_bit, int end_bit,
                        uint32_t* temp, hipStream_t stream, bool* result_in_b) {
    K* const kbuf[2] = {keys_b, keys_a};
    uint32_t* const vbuf[2] = {vals_b, vals_a};
    int result = -1;
    const SortArrays<K> up{keys_a, nullptr};
    const SortKeysNumbered<K> in{keys_a};
    BP_TRY((radix_sort_from<K, IPT, SortArrays<K>, SortKeysNumbered<K>, true>(up, in, kbuf, vbuf, n, begin_bit, end_bit, temp,
                                                                              stream, &result)));
    *result_in_b = result == 0;
    return BP_OK;
}

// The same for keys alone.
template <typename K, int IPT>
int radix_sort_keys(K* keys_a, K* keys_b, int64_t n, int begin_bit, int end_bit, uint32_t* temp, hipStream_t stream,
                    bool* result_in_b) {
    K* const kbuf[2] = {keys_b, keys_a};
    uint32_t* const vbuf[2] = {nullptr, nullptr};
    int result = -1;
    const SortArrays<K> in{keys_a, nullptr};
    BP_TRY((radix_sort_from<K, IPT, SortArrays<K>, SortArrays<K>, false>(in, in, kbuf, vbuf, n, begin_bit, end_bit, temp, stream,
                                                                         &result)));
    *result_in_b = result == 0;
    return BP_OK;
}

}  // namespace bp
