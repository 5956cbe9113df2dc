/*
 * collm_lora.h -- C ABI of the mixed-batch LoRA linear layer for AMD MI355X (gfx950).
 *
 * The layer is the LoRA-instrumented linear layer of the paper's section 4.2 (a frozen
 * base weight W_pre plus a trainable low-rank update Delta W = B_g A_g; only the adapters
 * train), evaluated the way the paper's model sharing runs it (section 2.1, "CoLLM's model
 * sharing"; section 7, "Concurrent Inference and Fine-tuning via Model Sharing"): inference
 * requests and fine-tuning sequences use ONE copy of the base weight and of the adapters at
 * the same time.  Here the two kinds of work arrive as one batch of tokens cut into
 * segments; a segment names its adapter and says whether it trains.  The inference batch b
 * and the training batch B of the paper's coordinator (section 5) are the inference-token
 * and training-token counts of that batch.
 *
 * Row-vector convention, all matrices row-major and dense:
 *     x  [T, d_in]        batch of tokens
 *     W  [d_in, d_out]    base weight (= W_pre^T), frozen
 *     A[a] [d_in, r_a]    down-projection of adapter a (= A_g^T)
 *     B[a] [r_a, d_out]   up-projection of adapter a   (= B_g^T)
 * For token t of a segment with adapter a:
 *     h[t,:] = x[t,:] A[a]                       y[t,:] = x[t,:] W + scale * h[t,:] B[a]
 * and for a token of a training segment, given dy = dL/dy:
 *     dh[t,:] = scale * dy[t,:] B[a]^T           dx[t,:] = dy[t,:] W^T + dh[t,:] A[a]^T
 *     dA[a] += x[t,:]^T dh[t,:]                  dB[a] += scale * h[t,:]^T dy[t,:]
 * There is no gradient for W.
 *
 * Element types: COLLM_BF16 (x, W, A, B, y, dy, dx are bfloat16; every product is
 * accumulated in fp32 and y / dx are rounded to bfloat16 once, on the final store) or
 * COLLM_F32 (all fp32, plain fp32 fused multiply-add).  h_save, dA and dB are always fp32.
 *
 * Conventions common to all entry points
 *   - "dev" pointers are device memory on the context's GPU, 16-byte aligned; "HOST"
 *     pointers are ordinary host memory.  The caller owns every buffer; the library owns
 *     only the context and its workspace and keeps no caller pointer after a call returns.
 *   - The compute calls are asynchronous: they enqueue work on `stream` (a hipStream_t, NULL
 *     = the default stream) and return.  Host arrays are copied before the call returns and
 *     may be reused at once.  One context serves one stream at a time; calls on the same
 *     context must not overlap on different streams, and a context is not thread-safe.
 *   - Every call returns a status: COLLM_OK (0) or a negative error.  All validation is done
 *     on the host before anything is launched; on an error no output buffer is touched.
 *   - d_in and d_out must be multiples of 8 (bf16) or 4 (fp32); x, dy and W must each stay
 *     below 2 GiB (COLLM_E_SHAPE otherwise).  Ranks may be any value in 1..max_rank.  Empty
 *     segments and an empty batch are legal.
 */
#ifndef COLLM_LORA_H
#define COLLM_LORA_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct collm_ctx collm_ctx; /* opaque: pinned staging, device plan and workspace */

typedef enum { COLLM_F32 = 0, COLLM_BF16 = 1 } collm_dtype;

/*
 * How the weight and the adapter tables lie in memory.  The mathematics is the same; with
 * COLLM_LAYOUT_OUT_IN every one of them, and every adapter gradient, is the transpose of the
 * array described at the calls below (the convention of module weights that store
 * [out_features, in_features]):
 *
 *                           W               A[i]              B[i]              dA[i]  dB[i]
 *   COLLM_LAYOUT_IN_OUT     [d_in, d_out]   [d_in, rank]      [rank, d_out]     as A   as B
 *   COLLM_LAYOUT_OUT_IN     [d_out, d_in]   [rank, d_in]      [d_out, rank]     as A   as B
 *
 * x, y, dy, dx and h_save do not change.
 */
typedef enum { COLLM_LAYOUT_IN_OUT = 0, COLLM_LAYOUT_OUT_IN = 1 } collm_layout;

enum {
    COLLM_OK = 0,
    COLLM_E_NULL = -1,     /* a required pointer is NULL                                    */
    COLLM_E_SHAPE = -2,    /* non-positive or unsupported size, or beyond the context maxima */
    COLLM_E_SEGMENTS = -3, /* seg_start[0] != 0, decreasing, or seg_start[S] != n_tokens     */
    COLLM_E_ADAPTER = -4,  /* adapter index outside [-1, N), training segment without an     */
                           /* adapter, NULL table of a used adapter, NULL dA/dB of a trained */
    COLLM_E_RANK = -5,     /* rank outside 1..max_rank                                       */
    COLLM_E_DTYPE = -6,    /* unknown element type                                           */
    COLLM_E_ALIGN = -7,    /* a device pointer is not 16-byte aligned                        */
    COLLM_E_HIP = -8,      /* a HIP call failed; see collm_last_error()                      */
    COLLM_E_NOMEM = -9     /* host or device allocation failed                               */
};

typedef struct {
    int32_t d_in, d_out;
    int32_t n_tokens;   /* T */
    int32_t n_segments; /* S */
    int32_t n_adapters; /* N */
    int32_t dtype;      /* collm_dtype */
    float scale;        /* multiplies the low-rank term */
    int32_t layout;     /* collm_layout of W, A, B, dA, dB */
} collm_shape;

/* Create a context on GPU `device` able to serve calls with n_tokens <= max_tokens,
 * n_segments <= max_segments, n_adapters <= max_adapters, every rank <= max_rank
 * (max_rank <= 256) and d_in, d_out <= max_d.  Allocates pinned staging and the device
 * workspace once; the compute calls allocate nothing.  *out is NULL on failure. */
int collm_ctx_create(collm_ctx **out, int device, int32_t max_tokens, int32_t max_segments,
                     int32_t max_adapters, int32_t max_rank, int32_t max_d);
/* Waits for the device to finish the context's work, then frees everything it owns. */
int collm_ctx_destroy(collm_ctx *ctx);
/* Bytes of device workspace the context holds. */
int64_t collm_ctx_workspace_bytes(const collm_ctx *ctx);

const char *collm_status_string(int status);
/* Text of the last HIP failure seen by this thread ("" if none). */
const char *collm_last_error(void);

/*
 * Forward (the definition above; paper section 4.2 for the parameterisation, section 2.1
 * for inference and training tokens sharing W and the adapters).
 *
 * Steps, all in the library's kernels: the host turns the segment table into a device plan
 * (token -> segment/adapter map, rows grouped by adapter, tile tables); a segmented shrink
 * computes h = x A[a] in fp32; one GEMM computes x W and adds scale * h B[a] as extra
 * K-steps before the single rounding of y.
 *
 *   x            dev  [T, d_in]
 *   W            dev  [d_in, d_out]  (shapes of W, A, B as for COLLM_LAYOUT_IN_OUT; see collm_layout)
 *   A, B         HOST arrays [N] of dev pointers, A[i]: [d_in, rank[i]], B[i]: [rank[i], d_out];
 *                an entry may be NULL if no segment uses adapter i
 *   rank         HOST [N]
 *   seg_start    HOST [S+1], seg_start[0] = 0, non-decreasing, seg_start[S] = T
 *   seg_adapter  HOST [S], 0..N-1, or -1 = base weight only (inference segments only)
 *   seg_is_train HOST [S], 0 or 1
 *   y            dev  [T, d_out]; every row is written
 *   h_save       dev  fp32 [T, max_rank] (row stride = the context's max_rank) or NULL.
 *                Rows of training tokens receive h (unscaled), zero-filled from rank[a] up
 *                to max_rank; rows of inference tokens are not touched.
 */
int collm_lora_linear_fwd(collm_ctx *ctx, const collm_shape *shape, const void *x, const void *W,
                          const void *const *A, const void *const *B, const int32_t *rank,
                          const int32_t *seg_start, const int32_t *seg_adapter,
                          const uint8_t *seg_is_train, void *y, float *h_save, void *stream);

/*
 * Backward for the training segments (only adapters train: paper section 4.2).
 *
 *   x, W, A, B, rank, seg_*   as in the forward call (same batch)
 *   dy           dev  [T, d_out]; only rows of training tokens are read
 *   h_save       dev  fp32 [T, max_rank] as written by the forward call, or NULL to recompute
 *   dx           dev  [T, d_in] or NULL; only rows of training tokens are written
 *   dA, dB       HOST arrays [N] of dev fp32 pointers, dA[i]: [d_in, rank[i]],
 *                dB[i]: [rank[i], d_out].  Only adapters that own a training segment are
 *                written (their entries must be non-NULL); all others are ignored.
 *                Both arrays may be NULL to skip the adapter gradients.
 *   accumulate   0: overwrite dA/dB of the trained adapters; 1: add to what they hold
 *                (gradient accumulation over micro-batches, paper section 2.2 footnote)
 *
 * Gradients of one adapter are summed over its training tokens in ascending token order in
 * fixed-size partial sums that are then added in order: no floating-point atomics, so two
 * runs give the same bits.
 */
int collm_lora_linear_bwd(collm_ctx *ctx, const collm_shape *shape, const void *x, const void *W,
                          const void *const *A, const void *const *B, const int32_t *rank,
                          const int32_t *seg_start, const int32_t *seg_adapter,
                          const uint8_t *seg_is_train, const void *dy, const float *h_save,
                          void *dx, float *const *dA, float *const *dB, int accumulate,
                          void *stream);

/*
 * collm_lora_linear_fwd for callers that cannot allocate: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments and results as collm_lora_linear_fwd, but there is no
 * context: the workspace (plan, scaled low-rank activations, partial sums) is a static array of 16 MiB in the
 * library's device image, one copy per GPU, held until the process ends, and the plan reaches it inside kernel
 * arguments instead of pinned staging memory.  The call allocates no device or pinned memory and calls no
 * allocating HIP routine, at the first call or later; the first call on a device looks up the array's address on
 * that device and clears the 256 bytes of it that must be zero.
 *   device       GPU to run on (made current); 0 <= device < 64
 *   h_save       dev fp32 [T, 64] (row stride 64) or NULL
 *   everything else as for collm_lora_linear_fwd.
 * Limits: n_tokens <= 2048, n_segments <= 2048, n_adapters <= 64, every rank <= 64, d_in and d_out <= 16384.
 * Beyond them: COLLM_E_SHAPE (COLLM_E_RANK for a rank), collm_last_error() names the limits, nothing is launched.
 * All calls on one GPU share that GPU's array: a call must not overlap in time with another call of this entry
 * point on the same GPU (other stream or other thread); calls on one stream are ordered and safe.
 */
int collm_lora_linear_fwd_noalloc(int device, const collm_shape *shape, const void *x, const void *W,
                                  const void *const *A, const void *const *B, const int32_t *rank,
                                  const int32_t *seg_start, const int32_t *seg_adapter,
                                  const uint8_t *seg_is_train, void *y, float *h_save, void *stream);

/*
 * Sibling projections: several projections of the same x (gate and up of an MLP; q, k, v of an
 * attention block), each with its own base weight and its own adapter pair of the same rank
 * (paper section 4.2 parameterisation, applied per projection; the batch, the segments and the
 * adapter of a token are shared).  The caller stores them side by side:
 *
 *   W     dev [d_in, D]          columns of sibling 0, then of sibling 1, ...; D = sum of d_out[j]
 *   A[i]  dev [d_in, P rank[i]]  columns j rank[i] .. (j + 1) rank[i]: the shrink table of sibling j
 *   B[i]  dev [rank[i], D]       columns as in W: the expand table of sibling j in its columns
 *   y, dy dev [T, D]             dA[i], dB[i] fp32, shaped as A[i], B[i]
 *   h_save dev fp32 [T, max_rank]: h of sibling j in columns j rank[a] .. of a row
 *
 * so that, for sibling j with columns C_j:  y[t, C_j] = x[t] W[:, C_j] + scale (x[t] A_j[a]) B[a][:, C_j].
 * One pass over x serves all shrink tables, one GEMM all siblings (the backward GEMM contracts
 * over all D columns at once, which also sums the siblings' contributions to dx).
 *
 * Limits: bf16, COLLM_LAYOUT_IN_OUT, shape->d_out = D, 1..COLLM_MAX_SIBLINGS siblings, every
 * d_out[j] a multiple of 8 and all but the last multiples of 256; with more than one sibling
 * every rank a multiple of 8; P * rank <= the context's max_rank (COLLM_E_RANK otherwise),
 * D <= its max_d.  All other arguments, statuses and guarantees as for collm_lora_linear_fwd /
 * collm_lora_linear_bwd.
 *
 * activation = COLLM_ACT_SWIGLU (forward call; two siblings of equal width d_ff, gate then up;
 * ranks multiples of 16): the forward call combines the pair before its single rounding,
 *     y[t, j] = silu(g) u,  g = y_gate[t, j], u = y_up[t, j], silu(g) = g / (1 + exp(-g)),
 * and y is dev [T, d_ff].  If pre_act (dev [T, D]) is not NULL, rows of training tokens receive
 * both pre-activations (g in columns 0 .. d_ff, u after them, each rounded to bf16): what
 * collm_swiglu_bwd needs; rows of inference tokens are not touched.  The backward call ignores
 * `activation` and pre_act: its dy is the gradient with respect to the pre-activations.
 */
#define COLLM_MAX_SIBLINGS 4
typedef enum { COLLM_ACT_NONE = 0, COLLM_ACT_SWIGLU = 1 } collm_activation;
typedef struct {
    int32_t n_siblings;                 /* P */
    int32_t d_out[COLLM_MAX_SIBLINGS];  /* output width of each sibling */
    int32_t activation;                 /* collm_activation */
    void *pre_act;                      /* COLLM_ACT_SWIGLU: dev [T, D] or NULL (see above) */
} collm_siblings;

/*
 * Backward of y = silu(g) u for the rows of training tokens (bf16): from dout = dL/dy, dev
 * [T, d_ff], and the pre-activations the forward call kept (pre_act, dev [T, 2 d_ff]),
 *     dy[t, j]        = dout[t, j] u sigma(g) (1 + g (1 - sigma(g)))      (dL/dg)
 *     dy[t, d_ff + j] = dout[t, j] g sigma(g)                              (dL/du)
 * in fp32, rounded once.  dy is dev [T, 2 d_ff]: the dy of collm_lora_siblings_bwd.  Rows of
 * inference tokens are neither read nor written.  seg_start, seg_is_train: HOST, as in the
 * other calls (checked the same way); d_ff a multiple of 8; pointers 16-byte aligned.
 */
int collm_swiglu_bwd(int device, int32_t n_tokens, int32_t d_ff, int32_t n_segments,
                     const int32_t *seg_start, const uint8_t *seg_is_train, const void *pre_act,
                     const void *dout, void *dy, void *stream);

int collm_lora_siblings_fwd(collm_ctx *ctx, const collm_shape *shape, const collm_siblings *siblings,
                            const void *x, const void *W, const void *const *A, const void *const *B,
                            const int32_t *rank, const int32_t *seg_start, const int32_t *seg_adapter,
                            const uint8_t *seg_is_train, void *y, float *h_save, void *stream);
int collm_lora_siblings_bwd(collm_ctx *ctx, const collm_shape *shape, const collm_siblings *siblings,
                            const void *x, const void *W, const void *const *A, const void *const *B,
                            const int32_t *rank, const int32_t *seg_start, const int32_t *seg_adapter,
                            const uint8_t *seg_is_train, const void *dy, const float *h_save, void *dx,
                            float *const *dA, float *const *dB, int accumulate, void *stream);

/*
 * Integer bookkeeping on the host (no GPU needed): per-token segment index, adapter index
 * and training flag.  All pointers HOST; outputs have n_tokens entries.  Uses only
 * n_tokens, n_segments and n_adapters of `shape`.
 */
int collm_token_map(const collm_shape *shape, const int32_t *seg_start,
                    const int32_t *seg_adapter, const uint8_t *seg_is_train,
                    int32_t *tok_segment, int32_t *tok_adapter, uint8_t *tok_is_train);

/*
 * Debug: read back the plan the DEVICE holds from the context's last compute call and undo
 * its row grouping, giving the token map the kernels actually used.  Synchronises the
 * context's last stream.  Outputs HOST, n_tokens entries of the last call.
 */
int collm_debug_device_token_map(collm_ctx *ctx, int32_t *tok_segment, int32_t *tok_adapter,
                                 uint8_t *tok_is_train);

/*
 * Debug, HOST only (no GPU): how the library would cut a GEMM of `rows` x `cols` outputs with
 * contraction length K into tiles: *tile = 0 (256x256) or 2 (128x128) for the first
 * *big_tiles_m row tiles, then *tail_tiles_m row tiles of 128 rows as 128x128 tiles (0: none).
 * *tail_cols (0: none; only with 256x256 tiles and no row tail): that many 256-wide tile columns
 * at the right edge run as 128x128 tiles over all rows in a second launch.
 * can_split: whether few 128x128 tiles may cut K into slices (see collm_debug_set_gemm_split).
 */
int collm_debug_host_tiling(int rows, int cols, int K, int can_split, int32_t *tile, int32_t *big_tiles_m,
                            int32_t *tail_tiles_m, int32_t *tail_cols);

/*
 * Debug, HOST only (no GPU): the order in which the workgroups of a GEMM launch of tiles_m x tiles_n tiles take
 * the tiles.  Workgroup ids go round-robin to the GPU's 8 XCDs (each with an L2 of its own); every XCD gets a
 * contiguous run of an order that walks groups of 8 row tiles column by column, and the grid is walked in bands
 * of *band_used row tiles (0 = one band), so that a band's rows of the first operand stay in the last-level cache
 * while the column tiles stream.  band = -1: the band the library chooses for tiles of tile_rows (128 or 256) rows
 * and contraction length K; band >= 0 (a multiple of 8): that band.  tile_m, tile_n: HOST, tiles_m * tiles_n
 * entries, the tile of workgroup id 0, 1, ...  Every tile appears exactly once.
 */
int collm_debug_host_tile_order(int tile_rows, int tiles_m, int tiles_n, int K, int band, int32_t *band_used,
                                int32_t *tile_m, int32_t *tile_n);

/*
 * Debug, HOST only (no GPU): the order in which the plan lists the rows of a batch for the GEMM
 * over all rows (training_rows_only = 0) or over the training rows (1), and the number of
 * 16-wide low-rank K-steps every row tile of tile_rows (64, 128 or 256) rows carries.
 * row_tok receives the token of every row (n_tokens entries at most), tile_steps one entry per
 * row tile.  Returns the number of rows (>= 0) or a negative status.
 */
int collm_debug_host_row_order(const collm_shape *shape, const int32_t *rank, const int32_t *seg_start,
                               const int32_t *seg_adapter, const uint8_t *seg_is_train, int tile_rows,
                               int training_rows_only, int32_t *row_tok, int32_t *tile_steps);

/*
 * Debug/tuning: force the tile shape of the forward GEMM and of the dX GEMM
 * (0: 256x256, 2: 128x128 rows x columns of the output; -1: let the library choose from the
 * problem size; anything else: COLLM_E_SHAPE).  Affects only speed, never results beyond
 * rounding order.
 */
int collm_debug_set_tiles(collm_ctx *ctx, int fwd_tile, int bwd_tile);

/*
 * Debug/tuning: into how many slices of K a GEMM with few rows (fewer than 256 tiles of
 * 128x128) is cut across blocks; the slices' fp32 sums are added by a second kernel before the
 * single rounding.  -1: let the library choose; 1: never; 2..64: that many (as far as K and
 * the workspace allow).  bf16 only.  Affects only speed and rounding order.
 */
int collm_debug_set_gemm_split(collm_ctx *ctx, int n_slices);

/*
 * Debug/tuning: which rows the rank-wide passes (h = x A, dh = dy B^T) run as 128-row tiles
 * rather than 16-row items: runs of at least min_rows rows of one adapter whose rank is a
 * multiple of 8.  0: never; -1: let the library choose (every such adapter when the widest
 * rank of the batch is at least 49; for the training rows already from 17).  bf16 only.
 * Affects only speed and rounding order.
 */
int collm_debug_set_wide_pass(collm_ctx *ctx, int min_rows);

/*
 * Debug/tuning: whether the backward call takes dh and dB from ONE pass over the training rows of dy.
 * That pass applies to bf16, COLLM_LAYOUT_IN_OUT, no siblings, every rank of the batch at most 16, adapter gradients
 * requested, partial sums within the context's workspace.  -1 (default): where it applies and the training rows of dy
 * are at least 192 MiB (below that the second read of dy comes from the last-level cache and is cheaper than the
 * partial sums); 1: wherever it applies;
 * 0: never, dh and dB each read dy (what every other case does).  Affects only speed and rounding order.
 */
int collm_debug_set_dual_pass(collm_ctx *ctx, int mode);

/*
 * What the HIP runtime reports for GPU `device`: compute units, the highest engine clock and memory clock in
 * kHz, the width of the memory bus in bits and the size of the L2 cache in bytes.  For reports; touches no context.
 */
int collm_device_info(int device, int32_t *compute_units, int32_t *clock_khz, int32_t *memory_clock_khz,
                      int32_t *memory_bus_bits, int64_t *l2_bytes);

/*
 * Debug/profiling, HOST only: what the plan of the context's last compute call cost on the host.
 * *mode = 0: the plan on the device was reused as it is; 1: built anew from the segment table; 2: same
 * batch, other adapter tables (their addresses replaced in place); 3: only the dA/dB pointer tables were new.
 * *build_us: host time spent building or patching; *upload_us: host time spent copying it into pinned
 * staging and enqueueing the copy kernel; *bytes: bytes sent to the device.
 */
int collm_debug_plan_stats(const collm_ctx *ctx, float *build_us, float *upload_us, int32_t *bytes, int32_t *mode);

/*
 * Debug/profiling: duration in milliseconds of each pass (one kernel, or the few kernels of
 * a pass) launched by the context's last compute call, from the start of its first kernel to
 * the end of its last by the kernels' own time stamps (HIP events attached to the launches on
 * the call's own stream; no event latency inside the interval; 0 for a pass that launched
 * nothing).  collm_profile_enable(ctx, 1) makes every later call time its passes this way,
 * all on the call's stream, one after the other;
 * collm_profile_read synchronises, fills names[i] (static strings) and ms[i] for up to
 * `cap` passes and returns how many there were (or a negative status).
 */
int collm_profile_enable(collm_ctx *ctx, int enable);
int collm_profile_read(collm_ctx *ctx, const char **names, float *ms, int cap);

/*
 * The step after the backward pass.  Both calls are element-wise over one adapter table of n_elems
 * elements (A_i: d_in * rank, B_i: rank * d_out), asynchronous on `stream`, allocate nothing and need
 * no context; `device` is made current.  Device buffers must be 16-byte aligned.
 *
 * collm_adapter_fedavg: aggregation of the adapter copies of the participating replicas (paper
 * section 4.2, the equation for the aggregated B and A): dst[i] = (1/n_copies) sum_k src[k][i].
 *   src       HOST array [n_copies] of dev pointers, element type `dtype`; 1 <= n_copies <= 16
 *   dst       dev, element type `dtype`; may be one of the sources
 * Sums are fp32 in copy order, one rounding to `dtype`.  COLLM_E_SHAPE for n_copies out of range.
 *
 * collm_adapter_adamw: one AdamW update (decoupled weight decay, bias-corrected moments; only the
 * adapters train, paper section 4.2; the optimizer itself is this library's reading) from the fp32
 * gradient that collm_lora_linear_bwd produced:
 *   m = beta1 m + (1 - beta1) g;  v = beta2 v + (1 - beta2) g^2
 *   w = w (1 - lr wd) - lr / (1 - beta1^step) * m / (sqrt(v) / sqrt(1 - beta2^step) + eps)
 *   param     dev, element type `dtype`: read (unless `master` is given) and written
 *   master    dev fp32 copy of the parameters or NULL; when given it is the one updated and
 *             `param` receives its rounded value
 *   grad      dev fp32, read; m, v: dev fp32, updated in place
 *   step      1 for the first update.  COLLM_E_SHAPE for step < 1 or n_elems < 0.
 */
typedef struct {
    float lr, beta1, beta2, eps, weight_decay;
    int32_t step;
} collm_adamw;

int collm_adapter_fedavg(int device, collm_dtype dtype, int32_t n_copies, const void *const *src, void *dst,
                         int64_t n_elems, void *stream);
int collm_adapter_adamw(int device, collm_dtype dtype, void *param, float *master, const float *grad,
                        float *m, float *v, int64_t n_elems, const collm_adamw *hp, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* COLLM_LORA_H */
