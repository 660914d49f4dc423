// bp_embbag_bwd_update: deterministic backward + fused sparse optimizer step on cached rows.
//
// Gradients, not embeddings, are combined (Section 6), so any per-row optimizer can follow; the update
// rules are SGD, element-wise Adagrad and row-wise Adagrad.
//
// The work of a batch is described by two lists of records (the planner emits them with its optional grouping;
// bp_embbag_bwd_update builds them itself after a stable sort of the lookups by slot):
//   row records    one per distinct row: where its lookups start in the grouped order, how many they are, its
//                  slot, its first lookup.  A row of up to BP_BWD_ROW_MAX lookups is summed (fp64) and updated by
//                  one lane group, which needs nothing but its record to ask for the cache row and the first
//                  gradient row.
//   piece records  a row with more lookups is cut into pieces of BP_BWD_PIECE lookups; one workgroup takes a piece,
//                  its lane groups add their shares and meet in LDS.  A one-piece row is updated at once.  For a
//                  row of several pieces the workgroup stores the piece's sum, and the one that finds, by a counter,
//                  that all the others have stored theirs adds the sums in piece order and updates the row.
// ONE launch does all of it: workgroups [0, piece_blocks) take pieces, the rest take rows.
// Every order of addition is fixed by the records, never by timing: results are bit-identical run to run.
// The summed gradient is rounded to fp32 once; the optimizer step itself is fp32 arithmetic.
#include "bwd_records.h"
#include "common.h"
#include "device_prims.h"
#include "row_access.h"

namespace bp {
namespace {

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
// First every bag writes its number over its own stretch of positions -- a wavefront takes 64 bags and goes through
// them one by one, its lanes writing side by side (one lane per bag would scatter 64 short runs per store) --, then
// the grouped positions pick their bag up from that map, which stays in L2.
__global__ __launch_bounds__(256) void bwd_bag_of_lookup_kernel(const int64_t* __restrict__ bag_off, int64_t bags, int64_t n,
                                                                uint32_t* __restrict__ bag_of_lookup) {
    const int lane = threadIdx.x % kWave;
    const int64_t b0 = ((int64_t)blockIdx.x * (256 / kWave) + threadIdx.x / kWave) * kWave;      // wave-uniform
    if (b0 >= bags) return;
    const int64_t b = b0 + lane;
    int64_t k = b < bags ? bag_off[b] : 0, end = b < bags ? bag_off[b + 1] : 0;
    if (k < 0) k = 0;
    if (end > n) end = n;
    const int here = (int)(bags - b0 < kWave ? bags - b0 : kWave);
    for (int t = 0; t < here; ++t) {
        const int64_t first = __shfl(k, t, kWave), stop = __shfl(end, t, kWave);
        for (int64_t q = first + lane; q < stop; q += kWave) bag_of_lookup[q] = (uint32_t)(b0 + t);
    }
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

// ---- 3./4. reduce and update -----------------------------------------------------------------
struct UpdateParams {
    int optimizer;
    float lr, eps;
    int lpr;
    int dim;
    uint32_t bags;      // rows of the upstream gradient: a bag number beyond them reads row 0 instead
    int64_t wst;        // stride of a cache row, in 16-byte pieces
    int64_t sst;        // stride of a row's optimizer state, in floats
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
    // The same through device-coherent accesses: written through to memory and read from it, past the caches that
    // the GPU's dies do not share, so that a sum stored by one workgroup can be read by any other without either of
    // them writing back or dropping everything else its cache holds (what a device-wide fence would cost).
    __device__ __forceinline__ void store_device(double* row, int c) const {
        uint64_t* p = reinterpret_cast<uint64_t*>(row + (size_t)c * N);
#pragma unroll
        for (int i = 0; i < N; ++i)
            __hip_atomic_store(p + i, (uint64_t)__double_as_longlong(v[i]), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __device__ __forceinline__ void load_device(const double* row, int c) {
        const uint64_t* p = reinterpret_cast<const uint64_t*>(row + (size_t)c * N);
#pragma unroll
        for (int i = 0; i < N; ++i)
            v[i] = __longlong_as_double((long long)__hip_atomic_load(p + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
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
        r.w_raw = cache_w[slot * u.wst + c];
        if (u.optimizer == BP_ADAGRAD) r.s.load_f32(cache_s + slot * u.sst, c);
    }
    if (u.optimizer == BP_ADAGRAD_ROWWISE) r.s_row = cache_s[slot * u.sst];
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
        if (active) s.store_f32(cache_s + slot * u.sst, c);
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
        if (c == 0 && active) cache_s[slot * u.sst] = s;
    }
    if (active) cache_w[slot * u.wst + c] = w.encode();
}

// Adds the gradient rows of the grouped lookups [p0, p1) into acc: bursts of four rows, the indices of the next
// burst loaded while the rows of this one arrive.  idx holds the bag numbers of the first four lookups.
template <bool BF16, int N>
__device__ __forceinline__ void add_gradient_rows(SumPiece<N>& acc, uint32_t (&idx)[4], uint32_t p0, uint32_t p1,
                                                  const uint32_t* __restrict__ bag_of, const float* __restrict__ grad,
                                                  const UpdateParams& u, int c) {
    for (uint32_t p = p0; p < p1; p += 4) {
        Piece<BF16> t[4];
#pragma unroll
        for (int j = 0; j < 4; ++j)     // the bag number is clamped where it is used: its load stays in flight until then
            if (p + j < p1) t[j].load_f32(grad + (size_t)min(idx[j], u.bags - 1u) * u.dim, c);
#pragma unroll
        for (int j = 0; j < 4; ++j) idx[j] = p + 4 + j < p1 ? bag_of[p + 4 + j] : 0u;
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (p + j < p1) acc.add(t[j]);
    }
}

// Sum over the lane groups of a workgroup, in group order: every group leaves its sum in LDS, group 0 adds them up.
// Two barriers; `red` may be reused after the call.
template <int G, int GW, int N>
__device__ __forceinline__ void workgroup_sum(SumPiece<N>& acc, double (*red)[N][GW], int j, int c) {
#pragma unroll
    for (int i = 0; i < N; ++i) red[j][i][c] = acc.v[i];
    __syncthreads();
    if (j == 0) {
        acc.zero();
        for (int g = 0; g < G; ++g) {
#pragma unroll
            for (int i = 0; i < N; ++i) acc.v[i] += red[g][i][c];
        }
    }
    __syncthreads();
}

// counts: the numbers of row and piece records when they were made on the device (bp_embbag_bwd_update), else NULL
// and the host's numbers hold.  use_first: a row record's `first` is the bag of its first lookup (one lookup per bag,
// or records made from sorted bag numbers); otherwise every bag number comes from bag_of.
// Rows a lane group takes per round.  Two would have their requests in flight together, but at eight wavefronts per
// SIMD their state spills (50.7 us), and with the registers for it only six wavefronts fit (40.8 us).
constexpr int kBwdRows = 1;
template <int GW, bool BF16>
__global__ __launch_bounds__(kRowBlock, BF16 ? 4 : 8) void bwd_rows_kernel(const uint4* __restrict__ row_recs,
                                                            const uint4* __restrict__ piece_recs,
                                                            const uint32_t* __restrict__ n_rows_ptr,
                                                            const uint32_t* __restrict__ n_pieces_ptr,
                                                            uint32_t n_rows_host, uint32_t n_pieces_host,
                                                            uint32_t piece_blocks, const uint32_t* __restrict__ bag_of,
                                                            int use_first, uint32_t n, int64_t C,
                                                            const float* __restrict__ grad, uint4* cache_w, float* cache_s,
                                                            double* partial, uint32_t partial_rows, uint32_t* tickets,
                                                            UpdateParams u) {
    constexpr int N = Piece<BF16>::N;
    constexpr int G = kRowBlock / GW;                 // lane groups per workgroup
    const int c = threadIdx.x % GW, j = threadIdx.x / GW;
    const bool active = c < u.lpr;

    if (blockIdx.x >= piece_blocks) {
        // ---- rows of up to kRowMax lookups: kBwdRows per lane group and round.  First every request that needs
        // nothing but the record -- the cache row, its state, the first bag numbers -- then the sums.  The record's
        // test is a value, not a branch in front of the requests: behind an early `continue` the compiler fetches
        // the record word by word, each word behind the test of the one before, and the row's requests leave two
        // round trips later (39.4 instead of 37.3 us on a Criteo-shaped batch).
        const uint32_t R = n_rows_ptr ? *n_rows_ptr : n_rows_host;
        const uint32_t groups = (gridDim.x - piece_blocks) * G;
        for (uint32_t w0 = ((blockIdx.x - piece_blocks) * G + j) * kBwdRows; w0 < R; w0 += groups * kBwdRows) {
            uint4 rec[kBwdRows];
            bool ok[kBwdRows];
            RowPiece<BF16> row[kBwdRows];
            uint32_t idx[kBwdRows][4];
#pragma unroll
            for (int r = 0; r < kBwdRows; ++r) rec[r] = w0 + r < R ? row_recs[w0 + r] : make_uint4(0, 0, 0, 0);
#pragma unroll
            for (int r = 0; r < kBwdRows; ++r) {
                const uint32_t start = rec[r].x & kPosMask, count = rec[r].y, slot = rec[r].z;
                ok[r] = !(rec[r].x & kLongRow) && (int64_t)slot < C && count != 0 && start < n && count <= n - start;
                row[r] = load_row<BF16>(u, cache_w, cache_s, ok[r] ? (int64_t)slot : 0, c, active && ok[r]);
                idx[r][0] = use_first ? rec[r].w : (ok[r] ? bag_of[start] : 0u);
#pragma unroll
                for (int k = 1; k < 4; ++k) idx[r][k] = ok[r] && (uint32_t)k < count ? bag_of[start + k] : 0u;
            }
#pragma unroll
            for (int r = 0; r < kBwdRows; ++r) {
                if (!ok[r]) continue;
                const uint32_t start = rec[r].x & kPosMask, count = rec[r].y;
                SumPiece<N> acc;
                acc.zero();
                if (active) add_gradient_rows<BF16, N>(acc, idx[r], start, start + count, bag_of, grad, u, c);
                finish_update<GW, BF16>(u, cache_w, cache_s, (int64_t)rec[r].z, c, row[r], acc.template rounded<BF16>(), active);
            }
        }
        return;
    }

    // ---- pieces of longer rows: one workgroup each
    __shared__ double red[G][N][GW];
    __shared__ uint32_t s_last;
    const uint32_t P = n_pieces_ptr ? *n_pieces_ptr : n_pieces_host;
    const bool writer = active && j == 0;
    for (uint32_t pi = blockIdx.x; pi < P; pi += piece_blocks) {
        const uint4 r0 = piece_recs[2 * (size_t)pi], r1 = piece_recs[2 * (size_t)pi + 1];
        const uint32_t start = r0.x, count = r0.y, slot = r0.z, index = r0.w, pieces = r1.x, pbase = r1.y;
        // a record that points outside the batch or the workspace does nothing (the test is the same in every lane)
        if ((int64_t)slot >= C || count == 0 || start >= n || count > n - start || pieces == 0 || index >= pieces) continue;
        const bool direct = pieces == 1;
        if (!direct && (pbase >= partial_rows || pieces > partial_rows - pbase)) continue;
        // lane group j takes the j-th stretch of the piece
        const uint32_t per = (count + G - 1) / G;
        const uint32_t p0 = start + min((uint32_t)j * per, count), p1 = start + min((uint32_t)(j + 1) * per, count);
        uint32_t idx[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) idx[k] = p0 + k < p1 ? bag_of[p0 + k] : 0u;
        SumPiece<N> acc;
        acc.zero();
        if (active) add_gradient_rows<BF16, N>(acc, idx, p0, p1, bag_of, grad, u, c);
        workgroup_sum<G, GW, N>(acc, red, j, c);
        if (direct) {      // the row is asked for only now: one more round trip after a few hundred gradient rows
            if (j == 0) {
                const RowPiece<BF16> row = load_row<BF16>(u, cache_w, cache_s, (int64_t)slot, c, writer);
                finish_update<GW, BF16>(u, cache_w, cache_s, (int64_t)slot, c, row, acc.template rounded<BF16>(), writer);
            }
            continue;
        }
        // one of several pieces: leave the sum where the last workgroup of the row will find it, then take a ticket
        // (device-coherent stores, complete before the barrier lets thread 0 count this piece; the workgroup that
        // counts the last piece then reads all the sums with device-coherent loads)
        if (writer) acc.store_device(partial + (size_t)(pbase + index) * u.dim, c);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        __syncthreads();
        if (threadIdx.x == 0)
            s_last = __hip_atomic_fetch_add(&tickets[pbase], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + 1u == pieces ? 1u : 0u;
        __syncthreads();
        const bool last = s_last != 0u;
        __syncthreads();                               // everybody has read s_last before a later piece rewrites it
        if (!last) continue;
        acc.zero();
        for (uint32_t b = (uint32_t)j; b < pieces; b += 2 * G) {      // lane groups take the pieces round-robin
            SumPiece<N> t[2];
#pragma unroll
            for (int k = 0; k < 2; ++k) {
                t[k].zero();
                if (active && b + (uint32_t)k * G < pieces) t[k].load_device(partial + (size_t)(pbase + b + k * G) * u.dim, c);
            }
#pragma unroll
            for (int k = 0; k < 2; ++k) acc.add(t[k]);
        }
        workgroup_sum<G, GW, N>(acc, red, j, c);
        if (j == 0) {
            const RowPiece<BF16> row = load_row<BF16>(u, cache_w, cache_s, (int64_t)slot, c, writer);
            finish_update<GW, BF16>(u, cache_w, cache_s, (int64_t)slot, c, row, acc.template rounded<BF16>(), writer);
        }
        if (threadIdx.x == 0)                          // the counter is zero again for the next call
            __hip_atomic_store(&tickets[pbase], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// ---- records made on the device (bp_embbag_bwd_update: one batch, lookups sorted by slot) -------------------------
// First scan, over the sorted lookups: a row starts where the slot changes; row r's first sorted position goes to
// row_pos[r].
struct RowHeadIn {
    const uint32_t* keys;
    __device__ __forceinline__ uint32_t operator()(int64_t p) const { return (p == 0 || keys[p] != keys[p - 1]) ? 1u : 0u; }
};
struct RowHeadOut {
    uint32_t* row_pos;
    __device__ __forceinline__ void operator()(int64_t p, uint32_t exc, uint32_t inc) const {
        if (inc != exc) row_pos[exc] = (uint32_t)p;
    }
};
// Second scan, over the rows (RowPiecesIn): every row writes its record, a long row its piece records.
struct RowRecordOut {
    const uint32_t* row_pos;
    const uint32_t* n_rows;
    uint32_t n;
    const uint32_t* keys;      // sorted slots
    const uint32_t* bags;      // bag of every sorted lookup
    uint4* row_recs;
    uint4* piece_recs;
    __device__ __forceinline__ void operator()(int64_t r, uint64_t exc, uint64_t inc) const {
        const uint32_t R = *n_rows;
        if (r >= (int64_t)R) return;
        const uint32_t start = row_pos[r];
        const uint32_t count = (r + 1 < (int64_t)R ? row_pos[r + 1] : n) - start;
        const uint32_t slot = keys[start];
        const uint32_t pc = pieces_of(count);
        row_recs[r] = make_uint4(start | (pc ? kLongRow : 0u), count, slot, bags[start]);
        if (pc) write_pieces(piece_recs, (uint32_t)exc, pc, start, count, slot, (uint32_t)(exc >> 32), 0u);
    }
};

// ---- workspace -------------------------------------------------------------------------------
constexpr int kSmallIPT = 4, kLargeIPT = 16;
constexpr int64_t kLargeSort = int64_t(1) << 21;

struct ReduceScratch {      // what the reduce kernel itself needs, in both entry points
    uint32_t* tickets;      // the caller's counters, one per partial row, zero between calls
    double* partial;
    uint32_t partial_rows;
};
ReduceScratch carve_reduce(Carver& c, int64_t n, int dim) {
    ReduceScratch r{};
    r.partial_rows = (uint32_t)partial_rows_for(n);
    r.partial = c.take<double>((size_t)r.partial_rows * (size_t)dim);
    return r;
}

struct BwdWorkspace {
    ReduceScratch red;
    uint32_t *keys_a, *keys_b, *vals_a, *vals_b, *sort_temp, *row_pos, *scan_partials32;
    uint64_t* scan_partials64;
    uint4 *row_recs, *piece_recs;
    size_t bytes;
};

BwdWorkspace carve_bwd(void* base, size_t cap, int64_t n, int dim) {
    Carver c(base, cap);
    BwdWorkspace w{};
    const size_t m = (size_t)(n > 0 ? n : 1);
    w.red = carve_reduce(c, n, dim);
    w.keys_a = c.take<uint32_t>(m);
    w.keys_b = c.take<uint32_t>(m);
    w.vals_a = c.take<uint32_t>(m);
    w.vals_b = c.take<uint32_t>(m);
    w.sort_temp = c.take<uint32_t>(n >= kLargeSort ? sort_temp_words<kLargeIPT>(n) : sort_temp_words<kSmallIPT>(n));
    w.row_pos = c.take<uint32_t>(m);
    w.scan_partials32 = c.take<uint32_t>(scan_partials(n));
    w.scan_partials64 = c.take<uint64_t>(scan_partials(n));
    w.row_recs = c.take<uint4>(m);
    w.piece_recs = c.take<uint4>(2 * piece_capacity_for(n));
    w.bytes = c.used();
    return w;
}

struct BwdLaunch {
    const bp_config* cfg;
    ReduceScratch red;
    const uint4 *row_recs, *piece_recs;
    const uint32_t *n_rows_ptr, *n_pieces_ptr;     // device counts, or NULL when the host's numbers hold
    uint32_t n_rows, n_pieces;                     // host counts, or upper bounds when the device counts
    const uint32_t* bag_of;
    int use_first;
    int64_t n;
    const float* grad;
    void* cache_w;
    void* cache_s;
    hipStream_t stream;
    int64_t bags;
    template <int GW, bool BF16>
    int run() {
        const size_t sbytes = cfg->cache_state_stride ? (size_t)cfg->cache_state_stride : state_row_bytes(cfg);
        UpdateParams u{cfg->optimizer, cfg->lr, cfg->eps, (int)(row_bytes(cfg) / 16), cfg->dim,
                       (uint32_t)(bags > 0 ? bags : 1), cache_w_stride16(cfg), (int64_t)(sbytes / 4)};
        const int groups_per_block = kRowBlock / GW;
        int64_t piece_blocks = n_pieces, row_blocks = ceil_div((int64_t)n_rows, (int64_t)groups_per_block * kBwdRows);
        if (piece_blocks > kMaxGridBlocks / 4) piece_blocks = kMaxGridBlocks / 4;
        if (row_blocks > kMaxGridBlocks) row_blocks = kMaxGridBlocks;
        if (row_blocks < 1) row_blocks = 1;
        BP_LAUNCH(K_BWD_REDUCE_UPDATE, (bwd_rows_kernel<GW, BF16>), dim3((unsigned)(piece_blocks + row_blocks)),
                  dim3(kRowBlock), 0, stream, row_recs, piece_recs, n_rows_ptr, n_pieces_ptr, n_rows, n_pieces,
                  (uint32_t)piece_blocks, bag_of, use_first, (uint32_t)n, cfg->capacity, grad, (uint4*)cache_w,
                  (float*)cache_s, red.partial, red.partial_rows, red.tickets, u);
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

BP_EXPORT size_t bp_embbag_bwd_ticket_bytes(int64_t n_lookups) { return partial_rows_for(n_lookups) * sizeof(uint32_t); }

BP_EXPORT int bp_embbag_bwd_update_workspace_bytes(const bp_config* cfg, int64_t n_lookups, int64_t bags, size_t* bytes) {
    if (!bytes) return fail(BP_ERR_INVALID_ARG, "bytes is NULL");
    BP_TRY(check_bwd_args(cfg, n_lookups, bags));
    *bytes = carve_bwd(nullptr, 0, n_lookups, cfg->dim).bytes;
    return BP_OK;
}

BP_EXPORT int bp_embbag_bwd_update(const bp_config* cfg, void* cache_w, void* cache_state, const int32_t* lookup_slots,
                                    const int64_t* bag_offsets, int64_t n_lookups, int64_t bags, const float* grad_out,
                                    void* workspace, size_t workspace_bytes, uint32_t* tickets, void* stream_) {
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
    if (!tickets || ((uintptr_t)tickets & 3)) return fail(BP_ERR_INVALID_ARG, "tickets NULL or not 4-byte aligned");
    BwdWorkspace w = carve_bwd(workspace, workspace_bytes, n, cfg->dim);
    if (w.bytes > workspace_bytes)
        return fail(BP_ERR_WORKSPACE_TOO_SMALL, "workspace %zu < required %zu bytes", workspace_bytes, w.bytes);
    w.red.tickets = tickets;

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

    // rows, then their records; the counts stay on the device
    BP_TRY((device_scan<uint32_t, AddOp, RowHeadIn, RowHeadOut>(RowHeadIn{skeys}, RowHeadOut{w.row_pos}, n, w.scan_partials32,
                                                               AddOp(), 0u, stream)));
    const uint32_t* n_rows = w.scan_partials32 + scan_num_tiles(n);
    BP_TRY((device_scan<uint64_t, AddOp, RowPiecesIn, RowRecordOut>(
        RowPiecesIn{w.row_pos, n_rows, (uint32_t)n},
        RowRecordOut{w.row_pos, n_rows, (uint32_t)n, skeys, sbags, w.row_recs, w.piece_recs}, n, w.scan_partials64, AddOp(),
        uint64_t(0), stream)));
    const uint32_t* n_pieces = reinterpret_cast<const uint32_t*>(w.scan_partials64 + scan_num_tiles(n));   // low word

    BwdLaunch l{cfg, w.red, w.row_recs, w.piece_recs, n_rows, n_pieces, (uint32_t)n, (uint32_t)piece_capacity_for(n), sbags,
                1, n, grad_out, cache_w, cache_state, stream, bags};
    return dispatch_row((int)(row_bytes(cfg) / 16), cfg->weight_dtype == BP_BF16, l);
}

// ---- grouped variant: the plan already lists the batch's lookups grouped by row ---------------------------------
namespace bp {
namespace {
struct GroupedWorkspace {
    ReduceScratch red;
    uint32_t* bag_of;          // bag of every grouped position
    uint32_t* bag_of_lookup;   // bag of every lookup, in lookup order
    size_t bytes;
};
GroupedWorkspace carve_grouped(void* base, size_t cap, int64_t n, int dim, bool multi_hot) {
    Carver c(base, cap);
    GroupedWorkspace w{};
    const size_t m = (size_t)(n > 0 ? n : 1);
    w.red = carve_reduce(c, n, dim);
    w.bag_of = multi_hot ? c.take<uint32_t>(m) : nullptr;
    w.bag_of_lookup = multi_hot ? c.take<uint32_t>(m) : nullptr;
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
                                           const int32_t* grouped_lookups, const bp_row_rec* row_recs, int64_t n_rows,
                                           const bp_piece_rec* piece_recs, int64_t n_pieces, const int64_t* bag_offsets,
                                           int64_t n_lookups, int64_t bags, const float* grad_out, void* workspace,
                                           size_t workspace_bytes, uint32_t* tickets, void* stream_) {
    hipStream_t stream = (hipStream_t)stream_;
    const int64_t n = n_lookups;
    BP_TRY(check_bwd_args(cfg, n, bags));
    if (n == 0) return BP_OK;
    if (n_rows < 1 || n_rows > n) return fail(BP_ERR_INVALID_ARG, "n_rows %lld outside [1, n_lookups]", (long long)n_rows);
    if (n_pieces < 0 || n_pieces > (int64_t)piece_capacity_for(n) || (n_pieces && !piece_recs))
        return fail(BP_ERR_INVALID_ARG, "n_pieces %lld outside [0, %lld] or piece_recs is NULL", (long long)n_pieces,
                    (long long)piece_capacity_for(n));
    if (!bag_offsets && n != bags)
        return fail(BP_ERR_INVALID_ARG, "bag_offsets is NULL but n_lookups %lld != bags %lld", (long long)n, (long long)bags);
    if (!cache_w || !grouped_lookups || !row_recs || !grad_out) return fail(BP_ERR_INVALID_ARG, "NULL pointer");
    if (cfg->optimizer != BP_SGD && !cache_state) return fail(BP_ERR_INVALID_ARG, "cache_state is NULL");
    if (((uintptr_t)cache_w | (uintptr_t)cache_state | (uintptr_t)grad_out | (uintptr_t)row_recs | (uintptr_t)piece_recs) & 15)
        return fail(BP_ERR_INVALID_ARG, "cache_w, cache_state, grad_out and the records must be 16-byte aligned");
    if (!workspace || ((uintptr_t)workspace & 255)) return fail(BP_ERR_INVALID_ARG, "workspace NULL or not 256-byte aligned");
    if (!tickets || ((uintptr_t)tickets & 3)) return fail(BP_ERR_INVALID_ARG, "tickets NULL or not 4-byte aligned");
    GroupedWorkspace w = carve_grouped(workspace, workspace_bytes, n, cfg->dim, bag_offsets != nullptr);
    if (w.bytes > workspace_bytes)
        return fail(BP_ERR_WORKSPACE_TOO_SMALL, "workspace %zu < required %zu bytes", workspace_bytes, w.bytes);
    w.red.tickets = tickets;
    const uint32_t* bag_of = reinterpret_cast<const uint32_t*>(grouped_lookups);   // one lookup per bag: position == bag
    if (bag_offsets) {
        BP_LAUNCH(K_BWD_KEYS, bwd_bag_of_lookup_kernel, dim3((unsigned)ceil_div(bags > 0 ? bags : 1, 256)), dim3(256), 0,
                  stream, bag_offsets, bags, n, w.bag_of_lookup);
        BP_LAUNCH(K_BWD_KEYS, bwd_bags_of_positions_kernel, dim3((unsigned)ceil_div(n, 256)), dim3(256), 0, stream,
                  grouped_lookups, (const uint32_t*)w.bag_of_lookup, n, bags, w.bag_of);
        bag_of = w.bag_of;
    }
    BwdLaunch l{cfg, w.red, reinterpret_cast<const uint4*>(row_recs), reinterpret_cast<const uint4*>(piece_recs), nullptr,
                nullptr, (uint32_t)n_rows, (uint32_t)n_pieces, bag_of, bag_offsets == nullptr, n, grad_out, cache_w,
                cache_state, stream, bags};
    return dispatch_row((int)(row_bytes(cfg) / 16), cfg->weight_dtype == BP_BF16, l);
}

// ---- the grouped variant for callers that cannot allocate ---------------------------------------------------------
// Same kernels; the scratch (counters, partial sums, the bag numbers of the grouped positions) lives in a fixed array
// in device memory that belongs to the library.  Every GPU the library runs on holds its own copy of the array at
// its own address, found once per device with that device current.
namespace bp {
namespace {
constexpr size_t kStaticScratchBytes = size_t(16) << 20;
// The counters own a stretch of fixed size at the array's start, whatever the batch: partial sums of one call must
// never land where a later, larger call expects zeroed counters.
constexpr size_t kStaticTickets = size_t(1) << 16;
constexpr size_t kStaticTicketBytes = kStaticTickets * sizeof(uint32_t);
static __device__ __align__(256) unsigned char g_static_scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
unsigned char* g_scratch_ptr[kMaxDevices] = {};     // per device: where its copy of the array lives

__global__ __launch_bounds__(256) void bwd_clear_words_kernel(uint32_t* p, size_t n) {
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) p[i] = 0u;
}

// The current device's copy of the scratch array.  On the first call for a device the address is looked up and the
// array cleared once (the counters at its start must be zero; every call leaves them zero).
int static_scratch(hipStream_t stream, unsigned char** out) {
    int dev = -1;
    BP_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return fail(BP_ERR_UNSUPPORTED, "device %d outside [0, %d)", dev, kMaxDevices);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        BP_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(g_static_scratch)));
        if (!ptr) return fail(BP_ERR_HIP, "the scratch array has no address on device %d", dev);
        const size_t words = kStaticScratchBytes / sizeof(uint32_t);
        BP_LAUNCH(K_FILL, bwd_clear_words_kernel, dim3((unsigned)ceil_div((int64_t)words, 256)), dim3(256), 0, stream,
                  (uint32_t*)ptr, words);
        g_scratch_ptr[dev] = (unsigned char*)ptr;
    }
    *out = g_scratch_ptr[dev];
    return BP_OK;
}
}  // namespace
}  // namespace bp

BP_EXPORT size_t bp_embbag_bwd_update_grouped_static_max_bytes(void) { return kStaticScratchBytes; }

BP_EXPORT int bp_embbag_bwd_update_grouped_static_bytes(const bp_config* cfg, int64_t n_lookups, int64_t bags,
                                                        int32_t multi_hot, size_t* bytes) {
    if (!bytes) return fail(BP_ERR_INVALID_ARG, "bytes is NULL");
    BP_TRY(check_bwd_args(cfg, n_lookups, bags));
    if (partial_rows_for(n_lookups) > kStaticTickets)
        return fail(BP_ERR_UNSUPPORTED, "a batch of %lld lookups needs %zu counters, the library's fixed array holds %zu",
                    (long long)n_lookups, partial_rows_for(n_lookups), kStaticTickets);
    *bytes = kStaticTicketBytes + carve_grouped(nullptr, 0, n_lookups, cfg->dim, multi_hot != 0).bytes;
    return BP_OK;
}

BP_EXPORT int bp_embbag_bwd_update_grouped_static(const bp_config* cfg, void* cache_w, void* cache_state,
                                                  const int32_t* grouped_lookups, const bp_row_rec* row_recs,
                                                  int64_t n_rows, const bp_piece_rec* piece_recs, int64_t n_pieces,
                                                  const int64_t* bag_offsets, int64_t n_lookups, int64_t bags,
                                                  const float* grad_out, void* stream) {
    size_t need = 0;
    BP_TRY(bp_embbag_bwd_update_grouped_static_bytes(cfg, n_lookups, bags, bag_offsets != nullptr, &need));
    if (need > kStaticScratchBytes)
        return fail(BP_ERR_UNSUPPORTED, "a batch of %lld lookups needs %zu bytes of scratch, the library's fixed array holds %zu",
                    (long long)n_lookups, need, kStaticScratchBytes);
    if (n_lookups == 0) return BP_OK;
    unsigned char* base = nullptr;
    BP_TRY(static_scratch((hipStream_t)stream, &base));
    return bp_embbag_bwd_update_grouped(cfg, cache_w, cache_state, grouped_lookups, row_recs, n_rows, piece_recs, n_pieces,
                                        bag_offsets, n_lookups, bags, grad_out, base + kStaticTicketBytes,
                                        kStaticScratchBytes - kStaticTicketBytes, reinterpret_cast<uint32_t*>(base), stream);
}
