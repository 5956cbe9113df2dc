// Kernel argument blocks and launchers (device side of the library).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

#include "plan.h"

namespace collm {

// Timing of the calling thread's next launches through COLLM_LAUNCH: `start` is recorded when the first of them
// begins on the GPU, `stop` when the last one launched so far ends (the kernels' own time stamps, as a profiler
// reads them: no marker is added to the stream, and the time between the two events holds no event latency).
struct LaunchEvents {
    hipEvent_t start = nullptr, stop = nullptr;
    int launches = 0;
};
extern thread_local LaunchEvents g_launch_events;
#define COLLM_LAUNCH(kern, grid, block, smem, st, ...)                                                            \
    do {                                                                                                          \
        ::collm::LaunchEvents &le_ = ::collm::g_launch_events;                                                    \
        if (le_.stop) {                                                                                           \
            hipExtLaunchKernelGGL(kern, grid, block, smem, st, le_.launches == 0 ? le_.start : nullptr, le_.stop, \
                                  0, __VA_ARGS__);                                                                \
            ++le_.launches;                                                                                       \
        } else {                                                                                                  \
            hipLaunchKernelGGL(kern, grid, block, smem, st, __VA_ARGS__);                                         \
        }                                                                                                         \
    } while (0)

enum { kTile256x256 = 0, kTile128x128 = 2 };  // GEMM tile shapes (rows x columns of the output)

// out[tok(m)][n] = sum_k a[tok(m)][k] * b(k, n)  +  sum over the row tile's extension steps
struct GemmArgs {
    const void *a;      // rows gathered through row_tok, K contiguous
    int64_t lda;
    const void *b;      // [K][N] (row length ldb) or, K-major, [N][K]
    int64_t ldb;
    void *out;          // rows scattered through row_tok
    int64_t ldo;
    int N, K;
    uint32_t a_bytes, b_bytes;  // sizes of the two operand tensors (each below 2 GiB)
    int tiles_m, tiles_n;
    int tile_m_base;          // first row tile of this launch (a GEMM may be split over launches by rows)
    int band_m;               // row tiles per band of the tile order (0 = one band); set by the launcher
    int n_base;               // first output column of this launch (... or by columns); a multiple of 8
    const int32_t *row_tok;   // [tiles_m * BM]
    const int32_t *ext_off;   // [tiles_m + 1]
    const ExtStep *ext;
    const void *hs;           // low-rank activations of the rows, [rows][hs_ld], row order
    int hs_ld;
    uint32_t hs_bytes;        // size of hs
    int64_t ext_ld;           // row length of a [rank][N] table (forward)
    const void *zeros;        // at least 16 bytes of zeros, 16-byte aligned (source of masked 16-byte loads)
    // sibling projections side by side in the output columns (forward GEMM): a column tile of sibling j (columns
    // from sib_col[j - 1] on) takes columns j * rank .. of hs for its extension steps, rank = that of the step
    int n_sib;                // 0 or 1: a single projection
    int sib_col[3];
    // gate/up pair with the SwiGLU epilogue (launch_gemm_swiglu): N = d_ff output columns; the up sibling's columns
    // of b and of the expand tables start at act_col; pre_act (optional, [tokens][pre_ld]) receives both
    // pre-activations of the rows of training tokens (tok_train: token -> 0/1)
    int act_col;
    void *pre_act;
    int64_t pre_ld;
    const int32_t *tok_train;
    // rank-wide pass over long runs of one adapter (launch_wide): one row tile per item, second operand =
    // the item's adapter table ([K][rank] or, K-major, [rank][K]), K cut into slices of k_per_split,
    // fp32 sums of slice s for row r of the row order at part[(s * part_rows + r) * part_ld + q]
    const SkinnyItem *items;
    const uint64_t *tab;
    float *part;
    int part_rows, part_ld;
    int k_per_split;          // multiple of 64
    int n_rows, row_base;     // launch_gemm_splitk: the launch covers rows row_base .. row_base + n_rows of the row order
                              // (row_base = 128 tile_m_base); part row = row - row_base
    int part_n_sib;           // as SkinnyArgs::n_sib (0 or 1: ranks as the items give them)
    int64_t tab_ld, tab_off;  // as SkinnyArgs
    // launch_wide: warm-up of the GEMM that follows, as in SkinnyArgs (extra blocks behind the n_items items)
    const void *warm_base;
    uint64_t warm_bytes;
    int warm_blocks, n_items;
};

// out[m][q] = sum_k in[tok(m)][k] * tab_a(k, q), one SkinnyItem per blockIdx.x
struct SkinnyArgs {
    const void *in;
    int64_t ld_in;
    uint32_t in_bytes;        // size of the streamed tensor (below 2 GiB)
    int K;
    const uint64_t *tab;      // adapter -> table; [K][rank] or, K-major, [rank][K]
    const SkinnyItem *items;
    const int32_t *row_tok;
    const int32_t *tok_train;
    float *f32_out;           // optional fp32 result
    int64_t f32_ld;
    int f32_cols;             // columns written per row (zero beyond the rank)
    int f32_by_token;         // 1: row = token index, training tokens only; 0: row order
    float f32_mult;
    void *bf_out;             // optional scaled copy in the element type, row order
    int bf_ld;
    float bf_mult;
    // K split over several blocks (bf16 kernels): sums of the slices, [slice][part_rows][part_ld]
    float *part;
    int part_rows, part_ld;
    // One of n_sib sibling projections whose low-rank activations lie side by side (K-major tables only): the
    // items' ranks are n_sib times the adapter's, the pass reads columns tab_off .. tab_off + K of table rows
    // of length tab_ld and writes result columns sib * rank .. of each row; the last sibling also zero-fills
    // the row from n_sib * rank on.  n_sib 0 or 1: none of this (tab_ld = K, tab_off = 0).
    int n_sib, sib;
    int64_t tab_ld, tab_off;
    // Warm-up of the GEMM that follows this pass (bf16 kernels): warm_blocks extra blocks behind the items (block
    // index n_items ..) read warm_bytes at warm_base once and drop them, so that the weight is in the last-level cache
    // when the GEMM asks for it.  The pass itself leaves most of the memory bandwidth idle.  0 blocks: none of this.
    const void *warm_base;
    uint64_t warm_bytes;
    int warm_blocks, n_items;
};

// out_a(q, n) = sum_t small[t][q] * big[tok(t)][n] over one adapter's training rows
struct GradArgs {
    const void *big;          // [T][N] gathered through row_tok
    int64_t ld_big;
    uint32_t big_bytes;       // size of `big` (below 2 GiB)
    int N;
    const float *small_;      // fp32 [.][ld_small]; row = token (small_by_token) or row order
    int64_t ld_small;
    int small_by_token;
    float small_mult;
    const void *small_bf;     // bf16 kernels: if set, the small operand as a bf16 copy [row order][ld_small_bf],
    int ld_small_bf;          // already scaled, zeros from the rank up to the next multiple of 16 (fp32 one unused)
    const int32_t *row_tok;   // training row order
    const GradItem *items;    // one per trained adapter
    const uint64_t *out_tab;  // adapter -> fp32 output
    int out_transposed;       // 0: out[q][n] (row length N); 1: out[n][q] (row length rank)
    int accumulate;
    // one of n_sib sibling projections (bf16 copy of the small operand, out_transposed = 0 only): the items'
    // ranks are n_sib times the adapter's, the small operand is columns sib * rank .. of the copy, and the
    // result goes to out[q][out_off + n] with row length ld_out.  n_sib 0 or 1: none of this.
    int n_sib, sib;
    int64_t ld_out, out_off;
};

// One read of the training rows of dy for both dh and dB_a (narrow ranks: every rank at most 16).
//   dh[t][q]   = sum_n dy[tok(t)][n] * B_a[q][n]      -> unscaled fp32 partial sums, one slice per group of kDualCols columns:
//                part_dh[(group * part_rows + t) * part_ld + q]; launch_skinny_finish adds the groups, scales and stores
//   dB_a[q][n] = sum_t hs[t][q] * dy[tok(t)][n]       (hs = s h as bf16, row order, zero from the rank up to 16)
// The rows of a trained adapter are cut into pieces of piece_rows rows (a multiple of 32, at most kDualMaxPieceRows); an adapter
// of one piece gets dB_a written (or added to, `accumulate`) directly, one of more pieces gets per-piece sums
// part_dB[((item * max_pieces + piece) * 16 + q) * N + n], which launch_dual_sum adds in piece order.
constexpr int kDualCols = 512, kDualMaxPieceRows = 512;
struct DualArgs {
    const void *dy;           // [T][N] bf16, rows gathered through row_tok
    int64_t ld_dy;
    uint32_t dy_bytes;
    int N;
    const void *hs;           // bf16 [row order][ld_hs]
    int ld_hs;
    uint32_t hs_bytes;        // size of hs (the kernel reads it through a buffer resource)
    const int32_t *row_tok;   // training row order
    const GradItem *items;    // one per trained adapter
    int n_grad;
    const uint64_t *tab_b;    // adapter -> B_a [rank][N] bf16
    const uint64_t *out_tab;  // adapter -> dB_a fp32 [rank][N]
    int accumulate;
    int piece_rows, max_pieces;
    float *part_dh;
    int part_rows, part_ld;
    float *part_dB;
    // extra rows of blocks that read `warm_bytes` bytes at warm_base once and drop them (the weight of the GEMM that follows)
    const void *warm_base;
    uint64_t warm_bytes;
    int warm_rows;
};
hipError_t launch_dual(const DualArgs &a, hipStream_t st);
hipError_t launch_dual_sum(const DualArgs &a, hipStream_t st);
// The GEMM kernels' tile order: (row tile, column tile) of workgroup id 0 .. tiles_m * tiles_n - 1 with bands of `band`
// row tiles (0 = none), and the band the launchers choose for a tile height and contraction length (host only).
void host_tile_order(int tiles_m, int tiles_n, int band, int32_t *tm, int32_t *tn);
int gemm_band_rows(int tile_rows, int K, int tiles_m);
hipError_t launch_gemm(const GemmArgs &a, int tile_cfg, bool b_kmajor, hipStream_t st);
// The GEMM with K cut into n_split slices of k_per_split (128x128 tiles): fp32 sums of slice s for row r of the row order at
// part[(s * part_rows + r) * part_ld + n] (part_ld >= N, a multiple of 4), then launch_gemm_finish adds the slices, rounds
// and scatters the rows through row_tok.
hipError_t launch_gemm_splitk(const GemmArgs &a, int n_split, bool b_kmajor, hipStream_t st);
hipError_t launch_gemm_finish(const GemmArgs &a, int n_split, hipStream_t st);
// tile_cfg kTile256x256 or kTile128x128; tiles_n counts tiles of half as many output columns as the tile has
hipError_t launch_gemm_swiglu(const GemmArgs &a, int tile_cfg, hipStream_t st);
// a, lda, K, a_bytes, row_tok and the fields of the rank-wide pass; everything else is ignored.  Items hold up
// to kWideRows rows; ranks must be multiples of 8.  The caller adds the slices with launch_skinny_finish.
hipError_t launch_wide(const GemmArgs &a, int n_items, int rpad, int n_split, bool t_kmajor, hipStream_t st);
hipError_t launch_skinny_finish(const SkinnyArgs &a, int n_items, int item_rows, int n_split, hipStream_t st);
int gemm_tile_rows(int tile_cfg);
int gemm_tile_cols(int tile_cfg);
// items hold up to 16 * row_tiles rows (row_tiles <= skinny_max_row_tiles(rpad)); n_split slices of K
hipError_t launch_skinny(const SkinnyArgs &a, int n_items, int rpad, int row_tiles, int n_split, bool t_kmajor,
                         hipStream_t st);
int skinny_max_row_tiles(int rpad);
int skinny_waves(int rpad);  // waves of a block, which split the block's K slice
int skinny_chunk(int rpad);  // K values a wave fetches at a time
int skinny_depth(int rpad, int row_tiles);  // chunks a wave keeps in flight
hipError_t launch_grad(const GradArgs &a, int n_grad, int rpad, hipStream_t st);
// dst[t][q] = bf16(mult * src[row_tok[t]][q]) for n_rows rows and ld_dst (multiple of 8) columns; columns from
// src_cols on are zero
hipError_t launch_pack_rows(const float *src, int64_t ld_src, int src_cols, const int32_t *row_tok, int n_rows,
                            float mult, void *dst, int ld_dst, hipStream_t st);

// copies ints [first_int, first_int + n_ints) (rounded outwards to 16 bytes) of a pinned host
// block into the device plan, in stream order, then stores `seq` to the pinned word
// `done_host_dev`; `counter` is a device int that is zero between uploads
hipError_t launch_plan_copy(const int32_t *src_pinned, int32_t *dst, size_t first_int, size_t n_ints, int *counter,
                            uint32_t *done_host_dev, uint32_t seq, hipStream_t st);

// copies n_ints ints (a multiple of 4) from HOST memory `src` to device memory `dst` in stream order without any
// staging buffer: the words travel inside the arguments of as many small kernels as it takes (3.5 KiB each)
hipError_t launch_plan_words(const int32_t *src_host, int32_t *dst, size_t n_ints, hipStream_t st);
// clears `bytes` (a multiple of 16) bytes at dst with a small kernel
hipError_t launch_fill_zero(void *dst, size_t bytes, hipStream_t st);

// dst[i] = (1/n_copies) sum_k src[k][i]; element type bf16 or fp32, fp32 sums in copy order
constexpr int kMaxFedAvgCopies = 16;
struct FedAvgArgs {
    const void *src[kMaxFedAvgCopies];
    void *dst;
    int64_t n;
    int n_copies;
};
// one AdamW step: param (element type), optional fp32 master copy, fp32 grad and moments
struct AdamWArgs {
    void *param;
    float *master;
    const float *grad;
    float *m, *v;
    int64_t n;
    float lr, beta1, beta2, eps, weight_decay;
    float bias1;        // 1 - beta1^step
    float rsqrt_bias2;  // 1 / sqrt(1 - beta2^step)
};
// Backward of out = silu(g) * u for the rows of up to kSwigluSegs training segments: pre holds g in columns
// 0 .. d_ff and u in columns d_ff .. 2 d_ff of a row, dy receives d out / d g and d out / d u in the same places.
constexpr int kSwigluSegs = 64;
struct SwigluBwdArgs {
    const void *pre;
    const void *dout;
    void *dy;
    int d_ff;
    int64_t ld_pre, ld_dout, ld_dy;
    int n_seg;
    int32_t row0[kSwigluSegs + 1];  // rows of the launch before segment k
    int32_t tok0[kSwigluSegs];      // first token of segment k
};
hipError_t launch_swiglu_bwd(const SwigluBwdArgs &a, hipStream_t st);
hipError_t launch_fedavg(const FedAvgArgs &a, bool bf16, hipStream_t st);
hipError_t launch_adamw(const AdamWArgs &a, bool bf16, hipStream_t st);

// fp32 element type: same argument blocks, plain fp32 FMA kernels
hipError_t launch_gemm_f32(const GemmArgs &a, bool b_kmajor, hipStream_t st);
hipError_t launch_skinny_f32(const SkinnyArgs &a, int n_items, bool t_kmajor, hipStream_t st);
hipError_t launch_grad_f32(const GradArgs &a, int n_grad, hipStream_t st);

}  // namespace collm
