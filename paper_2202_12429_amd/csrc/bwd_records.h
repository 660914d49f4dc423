// Row and piece records of a batch grouped by row (bp_row_rec / bp_piece_rec of the C header): what both makers of
// them, the planner's grouping step and bp_embbag_bwd_update's own scans, and the kernels that walk them share.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

#include "common.h"

namespace bp {

constexpr uint32_t kRowMax = BP_BWD_ROW_MAX;   // lookups of a row one lane group takes at most
constexpr uint32_t kPiece = BP_BWD_PIECE;      // lookups per piece of a longer row
constexpr uint32_t kLongRow = 0x80000000u, kPosMask = 0x7fffffffu;
constexpr int kMaxGridBlocks = 8192;             // workgroups of a launch that walks the records, at most

static_assert(sizeof(bp_row_rec) == 16 && sizeof(bp_piece_rec) == 32, "records are read and written as 16-byte words");

// Rows of several pieces have more than kPiece lookups each, so a batch of n lookups holds fewer than n / kPiece +
// n / (kPiece + 1) + 1 pieces of such rows: that many partial sums and tickets at most.
inline size_t partial_rows_for(int64_t n) { return (size_t)(n > 0 ? n : 0) / kPiece * 2 + 2; }
// Long rows have more than kRowMax lookups each and a row of m lookups has at most m / kPiece + 1 pieces.
inline size_t piece_capacity_for(int64_t n) {
    return (size_t)(n > 0 ? n : 0) / (kRowMax + 1) + (size_t)(n > 0 ? n : 0) / kPiece + 2;
}

__device__ __forceinline__ uint32_t pieces_of(uint32_t count) { return count > kRowMax ? (count + kPiece - 1) / kPiece : 0u; }

// The records of the `pieces` pieces of one long row: lookups [start, start + count) of the grouped order; `partial`
// numbers the row's first piece among the pieces of rows of several pieces; `tag` goes to the first reserved word.
__device__ __forceinline__ void write_pieces(uint4* piece_recs, uint32_t first_piece, uint32_t pieces, uint32_t start,
                                             uint32_t count, uint32_t slot, uint32_t partial, uint32_t tag) {
    for (uint32_t k = 0; k < pieces; ++k) {
        const uint32_t off = k * kPiece;
        piece_recs[2 * (size_t)(first_piece + k)] = make_uint4(start + off, min(kPiece, count - off), slot, k);
        piece_recs[2 * (size_t)(first_piece + k) + 1] = make_uint4(pieces, partial, tag, 0u);
    }
}

// Scan over the rows, whose first grouped positions are row_pos[0 .. *n_rows): pieces of the long rows in the low
// word, pieces of the rows of several pieces in the high word.  The rows end where the next one starts, the last one
// at n.
struct RowPiecesIn {
    const uint32_t* row_pos;
    const uint32_t* n_rows;
    uint32_t n;
    __device__ __forceinline__ uint64_t operator()(int64_t r) const {
        const uint32_t R = *n_rows;
        if (r >= (int64_t)R) return 0;
        const uint32_t count = (r + 1 < (int64_t)R ? row_pos[r + 1] : n) - row_pos[r];
        const uint32_t pc = pieces_of(count);
        return (uint64_t)pc | ((uint64_t)(pc > 1 ? pc : 0u) << 32);
    }
};

}  // namespace bp
