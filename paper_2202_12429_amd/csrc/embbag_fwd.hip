// bp_embbag_fwd: EmbeddingBag-sum forward over cache slots (the trainer's embedding lookup, Section 2.1,
// served from the GPU-resident cache of Section 3.2).
//  - bags of several lookups: one lane group per bag; every lane owns a 16-byte piece of the row, accumulates in
//    fp32 in lookup order and writes its piece of the pooled row;
//  - one lookup per bag (a row copy): the output is a flat array of 16-byte pieces, one per lane with no idle
//    lanes, several pieces per lane in flight; a wavefront's stores are one contiguous kilobyte.
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
