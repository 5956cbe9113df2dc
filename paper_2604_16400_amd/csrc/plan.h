// Device plan of one mixed batch: plain-old-data shared by the host planner and the kernels.
//
// The plan is the integer half of the layer.  It turns the caller's segment table into
//   * the per-token map (segment, adapter, training flag),
//   * two row orders -- all tokens, and training tokens only -- each grouped by adapter
//     (stable, so tokens of one adapter stay in ascending order) and padded with -1 rows,
//   * work items for the skinny (rank-wide) passes: runs of rows that share one adapter,
//   * for every row tile of the big GEMMs, the list of 16-wide K-steps of the low-rank
//     extension [x | s h] [W ; B_a] with the rows each step applies to,
//   * one gradient item per trained adapter (its run of training rows).
// Everything lives in one int32 block that is built on the host and copied to the GPU.
#pragma once
#include <stdint.h>

#include <vector>

namespace collm {

constexpr int kWideRows = 128;  // rows of an item of the rank-wide pass for long runs of one adapter
constexpr int kRowPad = 256;   // row orders are padded to a multiple of the largest GEMM tile
constexpr int kMaxRank = 256;  // largest adapter rank the kernels accept
constexpr int kSkinnyRows = 16;  // rows of one MFMA tile of the skinny passes; an item holds 1 or 2 tiles
constexpr int kSkinnyMaxSplit = 32;  // K slices a skinny pass may be cut into (partial sums in a workspace)
constexpr int kKStep = 16;       // K extent of one low-rank extension step (one MFMA K)

// Run of rows of one adapter inside a row order (never crosses an adapter boundary).
struct SkinnyItem {
    int32_t adapter;
    int32_t row_lo;  // first row (index into the row order)
    int32_t n_rows;  // 1..item_rows of the row order
    int32_t rank;    // rank of the adapter
};

// One 16-wide K-step of the low-rank extension inside a GEMM row tile.  Self-contained (no
// lookups through the adapter index) so that a kernel can fetch a step, and everything needed to
// address its operands, with one 16-byte scalar load.
struct ExtStep {
    uint32_t koff_rank;  // first rank index of the step (multiple of 16) | rank of the adapter << 16
    uint32_t rows;       // row_lo | row_hi << 16: rows [row_lo, row_hi) of the tile use this adapter
    uint64_t tab;        // device address of the adapter's table for this GEMM (B_a forward, A_a backward)
};
constexpr int kExtBatch = 4;  // steps a kernel fetches at a time; the step array is padded by as many
constexpr int kExtGroup = 64;  // rank indices of a group (kExtBatch steps): the steps of a tile are listed group by group

// Training rows of one trained adapter inside the training row order.
struct GradItem {
    int32_t adapter;
    int32_t row_lo, row_hi;  // rows of the training row order
    int32_t rank;
};

// Offsets (in int32 units) into the plan block, and counts.  Host-side description.
struct RowOrderLayout {
    int32_t n_rows = 0, n_rows_pad = 0;
    int32_t off_row_tok = 0;      // [n_rows_pad] token index or -1
    int32_t off_row_adapter = 0;  // [n_rows_pad] adapter or -1
    int32_t n_items = 0, off_items = 0;  // SkinnyItem[n_items]
    int32_t item_rows = kSkinnyRows;     // most rows an item holds (16 or 32)
    int32_t n_wide = 0, off_wide = 0;    // SkinnyItem[n_wide] of up to kWideRows rows: long runs, taken by the tiled pass
    int32_t bm = 0, n_tiles_m = 0;       // GEMM row tile the extension tables were built for
    int32_t off_ext_off = 0;             // [n_tiles_m + 1]
    int32_t off_ext = 0, n_ext = 0;      // ExtStep[n_ext]
    int32_t max_ext_per_tile = 0;
    // the same for row tiles of half the size (built when bm is 256): a GEMM may run its last rows on
    // smaller tiles
    int32_t n_tiles_m_half = 0, off_ext_off_half = 0, off_ext_half = 0;
    // host only: the adapter of every extension step (both tables), so that the table addresses inside the
    // steps can be replaced when only the adapter tables of a batch change
    std::vector<int32_t> ext_adapter, ext_adapter_half;
};

struct PlanLayout {
    int32_t n_tokens = 0, n_segments = 0, n_adapters = 0;
    int32_t rpad = 16;            // largest rank of the adapter table, rounded up to 16
    int32_t off_tok_segment = 0;  // [T]
    int32_t off_tok_adapter = 0;  // [T]
    int32_t off_tok_train = 0;    // [T] 0/1
    int32_t off_rank = 0;         // [N]
    int32_t off_A_ptr = 0;        // [N] 64-bit device pointers (8-byte aligned offset)
    int32_t off_B_ptr = 0;        // [N]
    int32_t off_dA_ptr = 0;       // [N] (backward only)
    int32_t off_dB_ptr = 0;       // [N]
    RowOrderLayout all;           // every token (forward)
    RowOrderLayout train;         // training tokens (backward)
    int32_t n_grad = 0, off_grad = 0;        // GradItem[n_grad]
    int32_t max_grad_rows = 0;               // most training rows of one trained adapter
    int32_t total_ints = 0;
};

}  // namespace collm
