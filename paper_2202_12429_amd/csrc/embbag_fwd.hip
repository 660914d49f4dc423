// bp_embbag_fwd: EmbeddingBag-sum forward over cache slots (the trainer's embedding lookup, Section 2.1,
// served from the GPU-resident cache of Section 3.2).
//  - bags of several lookups: one lane group per bag; every lane owns a 16-byte piece of the row, accumulates in
//    fp32 in lookup order and writes its piece of the pooled row;
//  - one lookup per bag (a row copy): the output is a flat array of 16-byte pieces, one per lane with no idle
//    lanes, several pieces per lane in flight; a wavefront's stores are one contiguous kilobyte.
// bp_embbag_fwd_grouped: the same row copies walked by the plan's row and piece records instead of a slot per
// lookup: every distinct row is fetched once and written to the bags that look it up.
#include "bwd_records.h"
#include "common.h"
#include "row_access.h"

namespace bp {
namespace {

template <int GW, bool BF16>
__global__ __launch_bounds__(kRowBlock) void embbag_fwd_kernel(const uint4* __restrict__ cache_w,
                                                               const int32_t* __restrict__ slots,
                                                               const int64_t* __restrict__ bag_off, int64_t bags,
                                                               int64_t n, int64_t C, int lpr, int64_t wst, int dim,
                                                               float* __restrict__ out) {
    const int64_t bag = ((int64_t)blockIdx.x * kRowBlock + threadIdx.x) / GW;
    const int c = threadIdx.x % GW;
    if (bag >= bags || c >= lpr) return;
    Piece<BF16> acc;
    acc.zero();
    {
        int64_t k = bag_off[bag];
        int64_t end = bag_off[bag + 1];
        if (k < 0) k = 0;                           // offsets that point outside the lookups read nothing there
        if (end > n) end = n;
        for (; k + 4 <= end; k += 4) {              // four independent row loads in flight, added in order
            uint32_t s[4];
            uint4 raw[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) s[j] = (uint32_t)slots[k + j];
#pragma unroll
            for (int j = 0; j < 4; ++j) raw[j] = s[j] < (uint64_t)C ? cache_w[(int64_t)s[j] * wst + c] : make_uint4(0, 0, 0, 0);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                Piece<BF16> p;
                p.decode(raw[j]);
                acc.add(p);
            }
        }
        for (; k < end; ++k) {
            const uint32_t s = (uint32_t)slots[k];
            if (s < (uint64_t)C) {
                Piece<BF16> p;
                p.decode(cache_w[(int64_t)s * wst + c]);
                acc.add(p);
            }
        }
    }
    acc.store_f32_stream(out + bag * dim, c);
}

// One lookup per bag.  Piece p of the output belongs to bag p / lpr, piece p % lpr of its row.  A workgroup owns
// kRowBlock * U consecutive pieces; the division by lpr uses inv = floor(2^32 / lpr) + 1, exact for the dividends
// that occur here (below 2^32 / lpr).
constexpr int kFlatPieces = 4;
template <bool BF16, int U>
__global__ __launch_bounds__(kRowBlock) void embbag_fwd_onehot_kernel(const uint4* __restrict__ cache_w,
                                                                      const int32_t* __restrict__ slots, int64_t bags,
                                                                      int64_t C, uint32_t lpr, uint32_t inv, int64_t wst,
                                                                      int dim, float* __restrict__ out) {
    const int64_t base = (int64_t)blockIdx.x * (kRowBlock * U);
    const int64_t bag0 = base / lpr;
    const uint32_t r0 = (uint32_t)(base - bag0 * lpr);
    int64_t bag[U];
    uint32_t c[U], s[U];
    uint4 raw[U];
#pragma unroll
    for (int j = 0; j < U; ++j) {
        const uint32_t q = r0 + j * kRowBlock + threadIdx.x;
        const uint32_t dq = lpr == 1 ? q : __umulhi(q, inv);
        c[j] = q - dq * lpr;
        bag[j] = bag0 + dq;
        s[j] = bag[j] < bags ? (uint32_t)slots[bag[j]] : 0xffffffffu;
    }
#pragma unroll
    for (int j = 0; j < U; ++j)
        raw[j] = s[j] < (uint64_t)C ? cache_w[(int64_t)s[j] * wst + c[j]] : make_uint4(0, 0, 0, 0);
#pragma unroll
    for (int j = 0; j < U; ++j) {
        if (bag[j] >= bags) continue;
        Piece<BF16> p;
        p.decode(raw[j]);
        p.store_f32_stream(out + bag[j] * dim, (int)c[j]);
    }
}

// One lookup per bag, from the plan's grouping: the bag of the grouped lookup at position p is grouped[p].  The output
// rows are written one here, one there, and a 128-byte line is often shared by two of them: plain stores, which meet
// in L2, are quicker here than non-temporal ones (27 against 30 us on a Criteo-shaped batch of 192-byte rows; 183
// against 253 us on 1.3 M rows of 512 bytes, whole lines).  Workgroups
// [0, piece_blocks) take the pieces of long rows (every lane group fetches the row and writes it to its share of the
// piece's bags), the others take one row of up to kRowMax lookups per lane group.
constexpr int kFwdRows = 2;
template <int GW, bool BF16>
__global__ __launch_bounds__(kRowBlock) void embbag_fwd_rows_kernel(const uint4* __restrict__ row_recs,
                                                                    const uint4* __restrict__ piece_recs, uint32_t n_rows,
                                                                    uint32_t n_pieces, uint32_t piece_blocks,
                                                                    const uint32_t* __restrict__ grouped, uint32_t n,
                                                                    int64_t C, const uint4* __restrict__ cache_w, int lpr,
                                                                    int64_t wst, int dim, float* __restrict__ out) {
    constexpr int G = kRowBlock / GW;
    static_assert(kPiece <= (uint32_t)kRowBlock, "a lane group's share of a piece is at most one lookup per lane");
    const int c = threadIdx.x % GW, j = threadIdx.x / GW;
    const bool active = c < lpr;
    if (blockIdx.x >= piece_blocks) {
        if (!active) return;
        // kFwdRows consecutive rows per lane group and round: their records first, then their rows and the bags of
        // their first lookups, all in flight together, then the stores
        const uint32_t groups = (gridDim.x - piece_blocks) * G;
        for (uint32_t w0 = ((blockIdx.x - piece_blocks) * G + j) * kFwdRows; w0 < n_rows; w0 += groups * kFwdRows) {
            uint4 rec[kFwdRows], raw[kFwdRows];
            uint32_t start[kFwdRows], count[kFwdRows], bag[kFwdRows][4];
#pragma unroll
            for (int r = 0; r < kFwdRows; ++r) rec[r] = w0 + r < n_rows ? row_recs[w0 + r] : make_uint4(0, 0, 0, 0);
#pragma unroll
            for (int r = 0; r < kFwdRows; ++r) {
                start[r] = rec[r].x & kPosMask;
                count[r] = rec[r].y;
                const uint32_t slot = rec[r].z;
                if ((rec[r].x & kLongRow) || (int64_t)slot >= C || start[r] >= n || count[r] > n - start[r]) count[r] = 0;
                raw[r] = count[r] ? cache_w[(int64_t)slot * wst + c] : make_uint4(0, 0, 0, 0);
                bag[r][0] = rec[r].w;                     // the row's first lookup: its position is its bag
#pragma unroll
                for (int k = 1; k < 4; ++k) bag[r][k] = (uint32_t)k < count[r] ? grouped[start[r] + k] : n;
            }
#pragma unroll
            for (int r = 0; r < kFwdRows; ++r) {
                if (count[r] == 0) continue;
                Piece<BF16> p;
                p.decode(raw[r]);
#pragma unroll
                for (int k = 0; k < 4; ++k)
                    if ((uint32_t)k < count[r] && bag[r][k] < n) p.store_f32(out + (size_t)bag[r][k] * dim, c);
                for (uint32_t k = 4; k < count[r]; k += 4) {      // the few rows of 5 .. kRowMax lookups
                    uint32_t more[4];
#pragma unroll
                    for (int q = 0; q < 4; ++q) more[q] = k + q < count[r] ? grouped[start[r] + k + q] : n;
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        if (more[q] < n) p.store_f32(out + (size_t)more[q] * dim, c);
                }
            }
        }
        return;
    }
    // a piece: lane group j writes the row to the j-th stretch of the piece's bags.  A stretch has at most GW lookups
    // (kPiece <= G * GW), so every lane of the group, idle ones included, fetches one bag number and the group hands
    // them round by lane shuffle: one coalesced load instead of a round trip per bag.
    for (uint32_t pi = blockIdx.x; pi < n_pieces; pi += piece_blocks) {
        const uint4 r0 = piece_recs[2 * (size_t)pi];
        const uint32_t start = r0.x, count = r0.y, slot = r0.z;
        if ((int64_t)slot >= C || count == 0 || count > kPiece || start >= n || count > n - start) continue;
        const uint32_t per = (count + G - 1) / G;
        const uint32_t p0 = min((uint32_t)j * per, count), share = min(per, count - p0);
        const uint32_t mine = (uint32_t)c < share ? grouped[start + p0 + c] : n;
        Piece<BF16> p;
        if (active) p.decode(cache_w[(int64_t)slot * wst + c]);
#pragma unroll
        for (int t = 0; t < GW; ++t) {
            const uint32_t bag = __shfl(mine, t, GW);
            if (active && bag < n) p.store_f32(out + (size_t)bag * dim, c);
        }
    }
}

struct FwdRowsLaunch {
    const bp_config* cfg;
    const void* cache_w;
    const uint32_t* grouped;
    const uint4* row_recs;
    const uint4* piece_recs;
    int64_t n_rows, n_pieces, bags;
    float* out;
    hipStream_t stream;
    template <int GW, bool BF16>
    int run() {
        int64_t piece_blocks = n_pieces, row_blocks = ceil_div(n_rows, (int64_t)(kRowBlock / GW) * kFwdRows);
        if (piece_blocks > kMaxGridBlocks / 4) piece_blocks = kMaxGridBlocks / 4;
        if (row_blocks > kMaxGridBlocks) row_blocks = kMaxGridBlocks;
        if (row_blocks < 1) row_blocks = 1;
        BP_LAUNCH(K_FWD, (embbag_fwd_rows_kernel<GW, BF16>), dim3((unsigned)(piece_blocks + row_blocks)), dim3(kRowBlock), 0,
                  stream, row_recs, piece_recs, (uint32_t)n_rows, (uint32_t)n_pieces, (uint32_t)piece_blocks, grouped,
                  (uint32_t)bags, cfg->capacity, (const uint4*)cache_w, (int)(row_bytes(cfg) / 16), cache_w_stride16(cfg),
                  cfg->dim, out);
        return BP_OK;
    }
};

struct FwdLaunch {
    const bp_config* cfg;
    const void* cache_w;
    const int32_t* slots;
    const int64_t* bag_off;
    int64_t bags, n_lookups;
    float* out;
    hipStream_t stream;
    template <int GW, bool BF16>
    int run() {
        const int lpr = (int)(row_bytes(cfg) / 16);
        if (bag_off == nullptr) {
            const uint32_t inv = lpr == 1 ? 0u : (uint32_t)((uint64_t(1) << 32) / (uint32_t)lpr + 1);
            const dim3 flat((unsigned)ceil_div(bags * lpr, (int64_t)kRowBlock * kFlatPieces));
            BP_LAUNCH(K_FWD, (embbag_fwd_onehot_kernel<BF16, kFlatPieces>), flat, dim3(kRowBlock), 0, stream,
                      (const uint4*)cache_w, slots, bags, cfg->capacity, (uint32_t)lpr, inv, cache_w_stride16(cfg), cfg->dim, out);
            return BP_OK;
        }
        const dim3 grid((unsigned)ceil_div(bags * GW, kRowBlock));
        BP_LAUNCH(K_FWD, (embbag_fwd_kernel<GW, BF16>), grid, dim3(kRowBlock), 0, stream, (const uint4*)cache_w, slots,
                  bag_off, bags, n_lookups, cfg->capacity, lpr, cache_w_stride16(cfg), cfg->dim, out);
        return BP_OK;
    }
};

}  // namespace
}  // namespace bp

using namespace bp;

BP_EXPORT int bp_embbag_fwd(const bp_config* cfg, const void* cache_w, const int32_t* lookup_slots,
                             const int64_t* bag_offsets, int64_t n_lookups, int64_t bags, float* out, void* stream) {
    BP_TRY(check_config(cfg));
    if (bags < 0 || n_lookups < 0) return fail(BP_ERR_INVALID_ARG, "negative size");
    if (bags >= (int64_t(1) << 31) || n_lookups >= (int64_t(1) << 31)) return fail(BP_ERR_UNSUPPORTED, "size >= 2^31");
    if (bags == 0) return BP_OK;
    if (!bag_offsets && n_lookups != bags)
        return fail(BP_ERR_INVALID_ARG, "bag_offsets is NULL but n_lookups %lld != bags %lld", (long long)n_lookups, (long long)bags);
    if (!cache_w || !out || (n_lookups && !lookup_slots)) return fail(BP_ERR_INVALID_ARG, "NULL pointer");
    if (((uintptr_t)cache_w | (uintptr_t)out) & 15) return fail(BP_ERR_INVALID_ARG, "cache_w and out must be 16-byte aligned");
    FwdLaunch l{cfg, cache_w, lookup_slots, bag_offsets, bags, n_lookups, out, (hipStream_t)stream};
    return dispatch_row((int)(row_bytes(cfg) / 16), cfg->weight_dtype == BP_BF16, l);
}

BP_EXPORT int bp_embbag_fwd_grouped(const bp_config* cfg, const void* cache_w, const int32_t* grouped_lookups,
                                     const bp_row_rec* row_recs, int64_t n_rows, const bp_piece_rec* piece_recs,
                                     int64_t n_pieces, int64_t bags, float* out, void* stream) {
    BP_TRY(check_config(cfg));
    if (bags < 0 || n_rows < 0 || n_pieces < 0) return fail(BP_ERR_INVALID_ARG, "negative size");
    if (bags >= (int64_t(1) << 31)) return fail(BP_ERR_UNSUPPORTED, "size >= 2^31");
    if (n_rows > bags || n_pieces > bags) return fail(BP_ERR_INVALID_ARG, "more rows or pieces than lookups");
    if (bags == 0 || n_rows == 0) return BP_OK;
    if (!cache_w || !out || !grouped_lookups || !row_recs || (n_pieces && !piece_recs))
        return fail(BP_ERR_INVALID_ARG, "NULL pointer");
    if (((uintptr_t)cache_w | (uintptr_t)out | (uintptr_t)row_recs | (uintptr_t)piece_recs) & 15)
        return fail(BP_ERR_INVALID_ARG, "cache_w, out, row_recs and piece_recs must be 16-byte aligned");
    FwdRowsLaunch l{cfg, cache_w, reinterpret_cast<const uint32_t*>(grouped_lookups), reinterpret_cast<const uint4*>(row_recs),
                    reinterpret_cast<const uint4*>(piece_recs), n_rows, n_pieces, bags, out, (hipStream_t)stream};
    return dispatch_row((int)(row_bytes(cfg) / 16), cfg->weight_dtype == BP_BF16, l);
}
