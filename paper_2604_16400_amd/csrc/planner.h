// Host-side planner interface (integer bookkeeping of the mixed batch).
#pragma once
#include <stddef.h>
#include <stdint.h>

#include <vector>

#include "collm_lora.h"
#include "plan.h"

namespace collm {

// Checks sizes, segment boundaries, adapter indices and ranks.  Returns a COLLM_* status.
int validate_batch(const collm_shape *s, const int32_t *rank, const int32_t *seg_start,
                   const int32_t *seg_adapter, const uint8_t *seg_is_train, int max_rank);

// Every token inherits the adapter and training flag of the segment that contains it.
void token_map(const collm_shape *s, const int32_t *seg_start, const int32_t *seg_adapter,
               const uint8_t *seg_is_train, int32_t *tok_segment, int32_t *tok_adapter,
               uint8_t *tok_is_train);

struct PlanRequest {
    const collm_shape *shape = nullptr;
    const int32_t *rank = nullptr;
    const int32_t *rank_ext_all = nullptr;  // ranks for the extension steps over all rows, if other than `rank`
                                            // (sibling projections: `rank` holds the sum over the siblings)
    const int32_t *seg_start = nullptr;
    const int32_t *seg_adapter = nullptr;
    const uint8_t *seg_is_train = nullptr;
    const void *const *A = nullptr;  // device pointers to store in the plan (may be null)
    const void *const *B = nullptr;
    float *const *dA = nullptr;
    float *const *dB = nullptr;
    int bm_all = 256;    // GEMM row tile of the forward GEMM
    int bm_train = 256;  // GEMM row tile of the dX GEMM
    int max_row_tiles = 1;  // most 16-row tiles a skinny item may hold (what the kernels for this rank width take)
    // > 0: runs of at least this many rows of an adapter whose rank is a multiple of 8 become items of up to
    // kWideRows rows for the tiled rank-wide pass; one value for the order of all rows, one for the training rows
    int wide_min_rows_all = 0, wide_min_rows_train = 0;
};

// Builds the plan block for a batch that passed validate_batch.
int build_plan(const PlanRequest &rq, std::vector<int32_t> &blk, PlanLayout &L);

// Upper bound of the plan size for a context's maxima (int32 units).
size_t plan_ints_upper_bound(int max_tokens, int max_segments, int max_adapters, int max_rank);

}  // namespace collm
