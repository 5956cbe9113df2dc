// C ABI of the mixed-batch LoRA linear layer: context, validation, plan upload, launches.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <chrono>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <thread>
#include <vector>

#include "collm_lora.h"
#include "kernels.h"
#include "planner.h"

using namespace collm;

namespace collm {
thread_local LaunchEvents g_launch_events;
}

namespace {

thread_local std::string g_last_error;

int hip_fail(hipError_t e, const char *what)
{
    char buf[256];
    std::snprintf(buf, sizeof buf, "%s: %s", what, hipGetErrorString(e));
    g_last_error = buf;
    return COLLM_E_HIP;
}

#define HIP_TRY(expr)                                     \
    do {                                                  \
        hipError_t e_ = (expr);                           \
        if (e_ != hipSuccess) return hip_fail(e_, #expr); \
    } while (0)

constexpr int kSlots = 16;             // pinned staging ring: the host may run this many uploads ahead
constexpr uint64_t kWarmMaxBytes = (uint64_t)40 << 20;  // largest weight a rank-wide pass fetches ahead of its GEMM
constexpr int kMaxProfile = 16;

inline int round_up(int v, int m) { return (v + m - 1) / m * m; }
inline bool aligned16(const void *p) { return ((uintptr_t)p & 15u) == 0; }

}  // namespace

struct collm_ctx {
    int device = 0;
    bool static_scratch = false;  // the workspace is the library's static device array; plans travel as kernel arguments
    int max_tokens = 0, max_segments = 0, max_adapters = 0, max_rank = 0, max_d = 0;
    int rows_cap = 0;   // padded row capacity
    int rpad_cap = 0;   // max_rank rounded up to 16

    size_t plan_cap = 0;  // int32 units
    int32_t *h_stage[kSlots] = {};      // pinned, device-visible
    int32_t *h_stage_dev[kSlots] = {};  // the same memory as the GPU addresses it
    uint32_t stage_seq[kSlots] = {};    // sequence number of the upload that last used the slot (0: none)
    uint32_t seq = 0;                   // uploads issued so far
    uint32_t *h_done = nullptr;         // pinned word: sequence number of the last finished upload
    uint32_t *h_done_dev = nullptr;
    int *d_copy_counter = nullptr;
    void *d_zeros = nullptr;  // 256 bytes of zeros for masked 16-byte loads
    float *d_part = nullptr;  // sums of the K slices of a skinny pass  [slices][rows][rpad]
    size_t part_bytes = 0;
    int slot = 0;
    int32_t *d_plan = nullptr;

    void *d_hs = nullptr;     // scaled low-rank activations, forward row order  [rows][rpad]
    void *d_dhs = nullptr;    // dh in the element type, training row order      [rows][rpad]
    float *d_h32 = nullptr;   // recomputed h, training row order                [rows][rpad]
    float *d_dh32 = nullptr;  // dh in fp32, training row order                  [rows][rpad]
    int64_t workspace_bytes = 0;

    std::vector<int32_t> plan;
    PlanLayout L;
    bool plan_valid = false;
    // what the cached plan was built from
    collm_shape key_shape{};
    int key_bm_all = 0, key_bm_train = 0;
    std::vector<int32_t> key_seg_start, key_seg_adapter, key_rank;
    std::vector<uint8_t> key_seg_train;
    std::vector<uint64_t> key_A, key_B;

    int tile_fwd = -1, tile_bwd = -1;  // forced GEMM tile shapes (-1 = choose)
    int wide_min_rows = -1;            // forced threshold of the tiled rank-wide pass (-1 = choose, 0 = never)
    int dual_pass = -1;                // dh and dB from one pass over dy: -1 = where it pays, 0 = never, 1 = wherever it applies
    int gemm_split = -1;               // forced number of K slices of a GEMM with few rows (-1 = choose, 1 = never)
    int n_cus = 0;                     // compute units of the device
    int key_wide = 0, key_nsib = 0;
    std::vector<int32_t> sum_rank;     // sibling calls: ranks summed over the siblings
    hipStream_t last_stream = nullptr;
    // the adapter gradients run beside dh and the dX GEMM on a second stream
    hipStream_t side = nullptr;
    hipEvent_t ev_fork = nullptr, ev_dh = nullptr, ev_join = nullptr;

    // host cost of the plan of the last compute call (collm_debug_plan_stats)
    float plan_build_us = 0.f, plan_upload_us = 0.f;
    int plan_mode = 0;       // 0: reused as it is, 1: built anew, 2: table addresses replaced, 3: gradient pointers only
    int plan_bytes_up = 0;   // bytes the call sent to the device

    bool profile = false;
    int n_prof = 0;
    const char *prof_name[kMaxProfile] = {};
    hipEvent_t prof_ev[kMaxProfile][2] = {};
    int prof_launches[kMaxProfile] = {};  // kernels each entry timed (0: nothing ran, the events were not recorded)
    bool prof_ev_made = false;
};

namespace {

// How a GEMM's tiles are cut: `tile` for the first `big_tiles_m` row tiles (all of them when
// tail_tiles_m is 0), then 128x128 tiles for `tail_tiles_m` row tiles of 128 rows.  Or (tail_cols > 0, 256x256
// tiles, no row tail): the last tail_cols tile columns of all rows run as 128x128 tiles in a second launch.
struct Tiling {
    int tile;
    int big_tiles_m;
    int tail_tiles_m;
    int tail_cols = 0;
};

// can_split: the 128x128 tiles behind the large ones may have K cut into slices (see run_gemm), which lets a few
// such tiles use the whole GPU
Tiling pick_tiling(int rows, int cols, int K, bool can_split)
{
    // Two shapes are worth choosing between: 256x256 run by four waves (one block per CU, the most
    // efficient inner loop) and 128x128 (two blocks per CU, four times as many tiles).  The cost of
    // a choice is the time its tiles take over the 256 CUs in units of one full round of 256x256
    // tiles; the constants are read off measurements on 4096- to 13824-wide layers:
    //  - 256x256: a GPU that is not filled once clocks higher (0.5 + 0.5 x); after whole rounds a last
    //    round that keeps a fraction f of the CUs busy costs 0.6 + 0.7 f, at most 1;
    //  - 128x128: a round of 512 tiles costs 0.65, one that leaves every CU a single block 0.39; from
    //    two rounds on the blocks' different speeds smooth the rounds out (0.62 per round, 0.3 for a
    //    nearly empty last one);
    //  - whole rounds of 256x256 tiles over the first rows and 128x128 tiles over the rest, as two
    //    launches: the sum of both plus 0.1 for the idle CUs at the boundary between them; fewer than 448
    //    small tiles with K in slices cost their share of a full round plus the kernel that adds the slices.
    auto cost_large = [](double tiles) {
        const double x = tiles / 256.0, whole = std::floor(x), part = x - whole;
        if (x <= 1.0) return 0.5 + 0.5 * x;
        return whole + (part == 0.0 ? 0.0 : std::min(1.0, 0.6 + 0.7 * part));
    };
    auto cost_small = [](double tiles) {
        const double x = tiles / 512.0, whole = std::floor(x), part = x - whole;
        if (whole >= 2.0) return 0.62 * whole + (part == 0.0 ? 0.0 : (part <= 0.1 ? 0.3 : 0.62 * part + 0.1));
        if (whole == 0.0) return part <= 0.5 ? 0.39 : 0.65;
        return 0.65 + (part == 0.0 ? 0.0 : (part <= 0.1 ? 0.3 : 0.65));
    };
    const int rp = round_up(std::max(rows, 1), kRowPad);
    const int tm = rp / 256, tn = (cols + 255) / 256, tn128 = (cols + 127) / 128;
    const int rows128 = (std::max(rows, 1) + 127) / 128;
    const double cost256 = cost_large((double)tm * tn), cost128 = cost_small((double)rows128 * tn128);
    Tiling best = cost256 <= cost128 ? Tiling{kTile256x256, tm, 0} : Tiling{kTile128x128, rows128, 0};
    double best_cost = std::min(cost256, cost128);
    const int rounds = tm * tn / 256;
    if (rounds >= 1 && (tm * tn) % 256 != 0) {
        const int m = std::min(tm - 1, rounds * 256 / tn);
        const int tail = (std::max(rows, 1) - 256 * m + 127) / 128;
        if (m >= 1 && tail >= 1) {
            const double tail_tiles = (double)tail * tn128;
            const double tail_cost = (can_split && K >= 1024 && tail_tiles < 448) ? 0.65 * tail_tiles / 512.0 + 0.05
                                                                                 : cost_small(tail_tiles);
            const double cost = cost_large((double)m * tn) + tail_cost + 0.1;
            if (cost < best_cost) {
                best = Tiling{kTile256x256, m, tail};
                best_cost = cost;
            }
        }
    }
    // ... or whole rounds over the first tile columns and the last columns of all rows as at most one round of
    // 128x128 tiles (two per CU) in a second launch: a last round that fills part of the CUs with large tiles
    // costs most of a round, 512 small tiles cost 0.65.
    if (rounds >= 1 && (tm * tn) % 256 != 0) {
        const int c = tn - rounds * 256 / tm;  // tile columns that do not fit the whole rounds
        const int cols_tail = cols - 256 * (tn - c);
        const long small = (long)rows128 * ((cols_tail + 127) / 128);
        if (c >= 1 && c < tn && small <= 512) {
            const double cost = cost_large((double)tm * (tn - c)) + cost_small((double)small) + 0.05;
            if (cost < best_cost - 0.05) best = Tiling{kTile256x256, tm, 0, c};
        }
    }
    return best;
}

// One GEMM over the row order `R`: a single launch, or whole rounds of large tiles followed by
// small tiles over the remaining rows.
hipError_t run_gemm(collm_ctx *c, GemmArgs g, const RowOrderLayout &R, int rows, int cols, int forced_tile,
                    bool b_kmajor, hipStream_t st, bool swiglu = false)
{
    // SwiGLU epilogue: `cols` counts gate and up columns; a tile holds half as many output columns as it is wide
    auto launch = [&](int tile) {
        g.tiles_n = (cols + gemm_tile_cols(tile) - 1) / gemm_tile_cols(tile);
        return swiglu ? launch_gemm_swiglu(g, tile, st) : launch_gemm(g, tile, b_kmajor, st);
    };
    const bool can_split = !swiglu && c->gemm_split != 1;
    const Tiling t = forced_tile >= 0 ? Tiling{forced_tile, R.n_rows_pad / gemm_tile_rows(forced_tile), 0}
                                      : pick_tiling(rows, cols, g.K, can_split);
    g.tile_m_base = 0;
    g.tiles_m = t.big_tiles_m;
    g.ext_off = c->d_plan + R.off_ext_off;
    g.ext = reinterpret_cast<const ExtStep *>(c->d_plan + R.off_ext);
    // Few tiles against a long contraction (decode-sized batches, or the small tiles behind whole rounds of large
    // ones): too few blocks to fill the GPU, each walking all of K with one tile of loads in flight.  Cut K into
    // slices so that up to two blocks per CU exist, as long as a slice keeps 512 K values and the fp32 partial sums
    // fit the workspace; a second kernel adds the slices.  Returns false if the launch should be a plain one.
    auto try_split = [&](int tiles_m, int row_base, int n_rows_here, hipError_t &err) -> bool {
        if (!can_split || forced_tile >= 0) return false;
        const int tiles_n = (cols + 127) / 128;
        const long tiles = (long)tiles_m * tiles_n;
        const long per_slice = (long)tiles_m * 128 * cols * 4;
        long want = c->gemm_split > 1 ? c->gemm_split : (tiles < 448 ? (448 + tiles - 1) / tiles : 1);
        want = std::min<long>({want, c->gemm_split > 1 ? g.K / 64 : g.K / 512, (long)c->part_bytes / per_slice, 64L});
        if (want < 2) return false;
        GemmArgs gs = g;
        gs.tiles_m = tiles_m;
        gs.tiles_n = tiles_n;
        gs.k_per_split = round_up((int)((g.K + want - 1) / want), 64);
        const int n_split = (g.K + gs.k_per_split - 1) / gs.k_per_split;
        gs.part = c->d_part;
        gs.part_rows = tiles_m * 128;
        gs.part_ld = cols;
        gs.row_base = row_base;
        gs.n_rows = n_rows_here;
        err = launch_gemm_splitk(gs, n_split, b_kmajor, st);
        if (err == hipSuccess) err = launch_gemm_finish(gs, n_split, st);
        return true;
    };
    hipError_t e = hipSuccess;
    if (t.tile == kTile128x128 && t.tail_tiles_m == 0 && try_split(t.big_tiles_m, 0, rows, e)) return e;
    if (t.tail_cols > 0 && !swiglu) {
        // whole rounds of large tiles over the first columns, small tiles over the other columns of all rows
        const int tn_big = (cols + 255) / 256 - t.tail_cols;
        g.tiles_n = tn_big;
        e = launch_gemm(g, kTile256x256, b_kmajor, st);
        if (e != hipSuccess) return e;
        g.n_base = 256 * tn_big;
        g.tiles_n = (cols - g.n_base + 127) / 128;
        g.tiles_m = (rows + 127) / 128;
        g.ext_off = c->d_plan + R.off_ext_off_half;
        g.ext = reinterpret_cast<const ExtStep *>(c->d_plan + R.off_ext_half);
        return launch_gemm(g, kTile128x128, b_kmajor, st);
    }
    e = launch(t.tile);
    if (e != hipSuccess || t.tail_tiles_m == 0) return e;
    g.tile_m_base = 2 * t.big_tiles_m;
    g.tiles_m = t.tail_tiles_m;
    g.ext_off = c->d_plan + R.off_ext_off_half;
    g.ext = reinterpret_cast<const ExtStep *>(c->d_plan + R.off_ext_half);
    if (try_split(t.tail_tiles_m, 256 * t.big_tiles_m, rows - 256 * t.big_tiles_m, e)) return e;
    return launch(kTile128x128);
}

// Times the kernels launched while it lives (profile mode): from the start of the first to the end of the last,
// by the kernels' own time stamps (see LaunchEvents).
struct Prof {
    collm_ctx *c;
    int idx = -1;
    Prof(collm_ctx *c_, hipStream_t, const char *name) : c(c_)
    {
        if (name && c->profile && c->n_prof < kMaxProfile) {
            idx = c->n_prof++;
            c->prof_name[idx] = name;
            c->prof_launches[idx] = 0;
            g_launch_events = LaunchEvents{c->prof_ev[idx][0], c->prof_ev[idx][1], 0};
        }
    }
    ~Prof()
    {
        if (idx >= 0) {
            c->prof_launches[idx] = g_launch_events.launches;
            g_launch_events = LaunchEvents{};
        }
    }
    Prof(const Prof &) = delete;
    Prof &operator=(const Prof &) = delete;
};

int check_common(collm_ctx *ctx, const collm_shape *s, const void *x, const void *W,
                 const void *const *A, const void *const *B, const int32_t *rank,
                 const int32_t *seg_start, const int32_t *seg_adapter, const uint8_t *seg_is_train)
{
    if (!ctx || !s) return COLLM_E_NULL;
    if (s->dtype != COLLM_F32 && s->dtype != COLLM_BF16) return COLLM_E_DTYPE;
    const int q = s->dtype == COLLM_BF16 ? 8 : 4;
    if (s->d_in <= 0 || s->d_out <= 0 || s->d_in % q || s->d_out % q) return COLLM_E_SHAPE;
    if (s->layout != COLLM_LAYOUT_IN_OUT && s->layout != COLLM_LAYOUT_OUT_IN) return COLLM_E_SHAPE;
    if (s->d_in > ctx->max_d || s->d_out > ctx->max_d) return COLLM_E_SHAPE;
    if (s->n_tokens < 0 || s->n_tokens > ctx->max_tokens) return COLLM_E_SHAPE;
    {
        // the kernels address each operand tensor with 32-bit byte offsets below 2 GiB
        const int64_t lim = (int64_t)1 << 31, e = s->dtype == COLLM_BF16 ? 2 : 4;
        const int64_t dmax = std::max(s->d_in, s->d_out), dmin = std::min(s->d_in, s->d_out);
        if (((int64_t)s->n_tokens + 1) * dmax * e >= lim || (dmax + 128) * dmin * e >= lim) return COLLM_E_SHAPE;
    }
    if (s->n_segments < 0 || s->n_segments > ctx->max_segments) return COLLM_E_SHAPE;
    if (s->n_adapters < 0 || s->n_adapters > ctx->max_adapters) return COLLM_E_SHAPE;
    if (!seg_start) return COLLM_E_NULL;
    if (s->n_adapters > 0 && (!rank || !A || !B)) return COLLM_E_NULL;
    int rc = validate_batch(s, rank, seg_start, seg_adapter, seg_is_train, ctx->max_rank);
    if (rc != COLLM_OK) return rc;
    if (s->n_tokens > 0 && (!x || !W)) return COLLM_E_NULL;
    if (!aligned16(x) || !aligned16(W)) return COLLM_E_ALIGN;
    for (int k = 0; k < s->n_segments; ++k) {
        const int a = seg_adapter[k];
        if (a < 0 || seg_start[k + 1] == seg_start[k]) continue;
        if (!A[a] || !B[a]) return COLLM_E_ADAPTER;
        if (!aligned16(A[a]) || !aligned16(B[a])) return COLLM_E_ALIGN;
    }
    return COLLM_OK;
}

bool same_key(collm_ctx *c, const collm_shape *s, const void *const *A, const void *const *B,
              const int32_t *rank, const int32_t *seg_start, const int32_t *seg_adapter,
              const uint8_t *seg_is_train, int bm_all, int bm_train, int wide)
{
    if (!c->plan_valid) return false;
    const collm_shape &k = c->key_shape;
    if (k.d_in != s->d_in || k.d_out != s->d_out || k.n_tokens != s->n_tokens ||
        k.n_segments != s->n_segments || k.n_adapters != s->n_adapters || k.dtype != s->dtype)
        return false;
    if (bm_all != c->key_bm_all || bm_train != c->key_bm_train || wide != c->key_wide) return false;
    const int S = s->n_segments, N = s->n_adapters;
    if (std::memcmp(c->key_seg_start.data(), seg_start, sizeof(int32_t) * (S + 1))) return false;
    if (S && std::memcmp(c->key_seg_adapter.data(), seg_adapter, sizeof(int32_t) * S)) return false;
    if (S && std::memcmp(c->key_seg_train.data(), seg_is_train, S)) return false;
    if (N && std::memcmp(c->key_rank.data(), rank, sizeof(int32_t) * N)) return false;
    (void)A;
    (void)B;
    return true;
}

bool same_tables(collm_ctx *c, int N, const void *const *A, const void *const *B)
{
    for (int a = 0; a < N; ++a)
        if (c->key_A[a] != (uint64_t)(uintptr_t)A[a] || c->key_B[a] != (uint64_t)(uintptr_t)B[a]) return false;
    return true;
}

// Same batch, other adapter tables (another layer or projection of the model): the plan keeps its shape; the
// two pointer tables and the table address inside every extension step are replaced.
void patch_tables(collm_ctx *c, int N, const void *const *A, const void *const *B)
{
    PlanLayout &L = c->L;
    for (int a = 0; a < N; ++a) {
        const uint64_t va = (uint64_t)(uintptr_t)A[a], vb = (uint64_t)(uintptr_t)B[a];
        std::memcpy(c->plan.data() + L.off_A_ptr + 2 * a, &va, 8);
        std::memcpy(c->plan.data() + L.off_B_ptr + 2 * a, &vb, 8);
        c->key_A[a] = va;
        c->key_B[a] = vb;
    }
    auto patch = [&](int32_t off_ext, const std::vector<int32_t> &step_adapter, const void *const *tab) {
        ExtStep *ext = reinterpret_cast<ExtStep *>(c->plan.data() + off_ext);
        for (size_t k = 0; k < step_adapter.size(); ++k)
            if (step_adapter[k] >= 0) ext[k].tab = (uint64_t)(uintptr_t)tab[step_adapter[k]];  // (empty steps have no table)
    };
    patch(L.all.off_ext, L.all.ext_adapter, B);            // forward: expand tables
    patch(L.all.off_ext_half, L.all.ext_adapter_half, B);
    patch(L.train.off_ext, L.train.ext_adapter, A);        // backward: shrink tables
    patch(L.train.off_ext_half, L.train.ext_adapter_half, A);
}

// Copy ints [lo, hi) of the host plan to the device plan through a pinned staging slot.
int upload(collm_ctx *c, size_t lo, size_t hi, hipStream_t st)
{
    if (hi <= lo) return COLLM_OK;
    const auto t0 = std::chrono::steady_clock::now();
    if (c->static_scratch) {
        // no pinned staging exists: the words travel inside the arguments of a few small kernels
        const size_t lo4 = lo & ~(size_t)3, hi4 = std::min((hi + 3) & ~(size_t)3, c->plan.size());
        HIP_TRY(launch_plan_words(c->plan.data() + lo4, c->d_plan + lo4, hi4 - lo4, st));
        c->last_stream = st;
        c->plan_upload_us += std::chrono::duration<float, std::micro>(std::chrono::steady_clock::now() - t0).count();
        c->plan_bytes_up += (int)((hi4 - lo4) * sizeof(int32_t));
        return COLLM_OK;
    }
    const int sl = c->slot;
    c->slot = (c->slot + 1) % kSlots;
    if (c->stage_seq[sl] != 0) {
        // the slot is free once the upload that used it has been copied by the GPU
        const volatile uint32_t *done = c->h_done;
        int spins = 0;
        while ((int32_t)(*done - c->stage_seq[sl]) < 0) {
            if (++spins > 2000) {  // far behind: let the stream drain instead of spinning
                HIP_TRY(hipStreamSynchronize(c->last_stream));
                break;
            }
            std::this_thread::yield();
        }
    }
    // rounded outwards to 16 bytes (the plan vector is padded to a multiple of 64 ints)
    const size_t lo4 = lo & ~(size_t)3, hi4 = std::min((hi + 3) & ~(size_t)3, c->plan.size());
    std::memcpy(c->h_stage[sl] + lo4, c->plan.data() + lo4, (hi4 - lo4) * sizeof(int32_t));
    const uint32_t seq = ++c->seq == 0 ? ++c->seq : c->seq;
    HIP_TRY(launch_plan_copy(c->h_stage_dev[sl], c->d_plan, lo4, hi4 - lo4, c->d_copy_counter, c->h_done_dev, seq, st));
    c->stage_seq[sl] = seq;
    c->last_stream = st;
    c->plan_upload_us += std::chrono::duration<float, std::micro>(std::chrono::steady_clock::now() - t0).count();
    c->plan_bytes_up += (int)((hi4 - lo4) * sizeof(int32_t));
    return COLLM_OK;
}

// Build (or reuse) the plan of this batch and put it on the device.
int prepare_plan(collm_ctx *c, const collm_shape *s, const void *const *A, const void *const *B,
                 const int32_t *rank, const int32_t *seg_start, const int32_t *seg_adapter,
                 const uint8_t *seg_is_train, float *const *dA, float *const *dB, bool allow_reuse,
                 hipStream_t st, const int32_t *rank_ext_all = nullptr, int n_sib = 1)
{
    const bool f32 = s->dtype == COLLM_F32;
    int n_train = 0;
    for (int k = 0; k < s->n_segments; ++k)
        if (seg_is_train[k]) n_train += seg_start[k + 1] - seg_start[k];
    const bool can_split = !f32 && c->gemm_split != 1;
    const int tile_fwd = c->tile_fwd >= 0 ? c->tile_fwd : pick_tiling(s->n_tokens, s->d_out, s->d_in, can_split && n_sib < 16).tile;
    const int tile_bwd = c->tile_bwd >= 0 ? c->tile_bwd : pick_tiling(n_train, s->d_in, s->d_out, can_split).tile;
    const int bm_all = f32 ? 64 : gemm_tile_rows(tile_fwd);
    const int bm_train = f32 ? 64 : gemm_tile_rows(tile_bwd);
    int rmax = 1;
    for (int a = 0; a < s->n_adapters; ++a) rmax = std::max(rmax, rank[a]);
    // All rows of an adapter take the tiled rank-wide pass when ranks reach 64: there an adapter's table
    // outweighs 16 or 32 rows of activations several times, and the tiled pass fetches it once per 128 rows.
    // Narrow ranks waste its 128 columns of matrix work; measured, it still pays for the dh pass (tables
    // with K contiguous) from rank 32 up.  Encoded as all-rows threshold + 65536 * training-rows threshold.
    const int rpad_max = round_up(rmax, kKStep);
    const int wide_all = f32 ? 0 : (c->wide_min_rows >= 0 ? c->wide_min_rows : (rpad_max >= 64 ? 1 : 0));
    const int wide_train = f32 ? 0 : (c->wide_min_rows >= 0 ? c->wide_min_rows : (rpad_max >= 32 ? 1 : 0));
    const int wide = wide_all + 65536 * wide_train;

    // A batch whose segment table, ranks, adapter tables and sizes equal those of the plan the device holds
    // reuses it (every layer and projection of a model sees the same batch): only a call on another stream
    // than the one the plan was uploaded on builds it again, since nothing orders the two streams.
    const bool reuse = allow_reuse && st == c->last_stream && n_sib == c->key_nsib &&
                       same_key(c, s, A, B, rank, seg_start, seg_adapter, seg_is_train, bm_all, bm_train, wide);
    bool upload_all = false;
    c->plan_build_us = c->plan_upload_us = 0.f;
    c->plan_mode = c->plan_bytes_up = 0;
    const auto t_plan = std::chrono::steady_clock::now();
    auto built = [&](int mode) {
        c->plan_mode = mode;
        c->plan_build_us = std::chrono::duration<float, std::micro>(std::chrono::steady_clock::now() - t_plan).count();
    };
    if (reuse && !same_tables(c, s->n_adapters, A, B)) {
        patch_tables(c, s->n_adapters, A, B);
        upload_all = true;
        built(2);
    }
    if (!reuse) {
        PlanRequest rq;
        rq.shape = s;
        rq.rank = rank;
        rq.rank_ext_all = rank_ext_all;
        rq.seg_start = seg_start;
        rq.seg_adapter = seg_adapter;
        rq.seg_is_train = seg_is_train;
        rq.A = A;
        rq.B = B;
        rq.dA = dA;
        rq.dB = dB;
        rq.bm_all = bm_all;
        rq.bm_train = bm_train;
        rq.max_row_tiles = f32 ? 1 : skinny_max_row_tiles(round_up(rmax, kKStep));
        rq.wide_min_rows_all = wide_all;
        rq.wide_min_rows_train = wide_train;
        c->plan_valid = false;
        int rc = build_plan(rq, c->plan, c->L);
        if (rc != COLLM_OK) return rc;
        if ((size_t)c->L.total_ints > c->plan_cap) {
            g_last_error = "the plan of this batch is larger than the context's plan buffer";
            return COLLM_E_SHAPE;
        }
        built(1);
        rc = upload(c, 0, c->L.total_ints, st);
        if (rc != COLLM_OK) return rc;
        // remember what this plan was built from
        const int S = s->n_segments, N = s->n_adapters;
        c->key_shape = *s;
        c->key_bm_all = bm_all;
        c->key_bm_train = bm_train;
        c->key_wide = wide;
        c->key_nsib = n_sib;
        c->key_seg_start.assign(seg_start, seg_start + S + 1);
        c->key_seg_adapter.assign(seg_adapter, seg_adapter + S);
        c->key_seg_train.assign(seg_is_train, seg_is_train + S);
        c->key_rank.assign(rank, rank + N);
        c->key_A.resize(N);
        c->key_B.resize(N);
        for (int a = 0; a < N; ++a) {
            c->key_A[a] = (uint64_t)(uintptr_t)A[a];
            c->key_B[a] = (uint64_t)(uintptr_t)B[a];
        }
        c->plan_valid = true;
    } else if (dA || dB || upload_all) {
        // same batch as the plan on the device: at most the pointer tables are new
        const int N = s->n_adapters;
        bool changed = false;
        for (int a = 0; a < N; ++a) {
            const uint64_t va = dA ? (uint64_t)(uintptr_t)dA[a] : 0, vb = dB ? (uint64_t)(uintptr_t)dB[a] : 0;
            changed |= std::memcmp(c->plan.data() + c->L.off_dA_ptr + 2 * a, &va, 8) != 0;
            changed |= std::memcmp(c->plan.data() + c->L.off_dB_ptr + 2 * a, &vb, 8) != 0;
            std::memcpy(c->plan.data() + c->L.off_dA_ptr + 2 * a, &va, 8);
            std::memcpy(c->plan.data() + c->L.off_dB_ptr + 2 * a, &vb, 8);
        }
        if (upload_all) {
            int rc = upload(c, 0, c->L.total_ints, st);
            if (rc != COLLM_OK) return rc;
        } else if (changed) {
            c->plan_mode = 3;
            int rc = upload(c, c->L.off_dA_ptr, (size_t)c->L.off_dB_ptr + 2 * (size_t)std::max(N, 1), st);
            if (rc != COLLM_OK) return rc;
        }
    }
    c->last_stream = st;
    return COLLM_OK;
}

// A rank-wide pass restricted to one of several sibling projections that lie side by side in the columns of
// dy and of the K-major tables: columns col0 .. col0 + K of rows of length ld.
struct SiblingPass {
    int n_sib = 0, sib = 0;
    int64_t ld = 0, col0 = 0;
    int rpad = 0;  // padded width of the widest single rank
};

// Partial sums of a rank-wide pass that another kernel has left in the layout of the pass's own K slices
// (part[(slice * part_rows + row) * part_ld + q]): run_skinny then only adds them up and stores.
struct SliceSums {
    float *part;
    int part_rows, part_ld, n_slices;
};

// One skinny pass over a row order.
int run_skinny(collm_ctx *c, const collm_shape *s, const RowOrderLayout &R, const void *in, int K,
               int32_t off_tab, bool t_kmajor, float *f32_out, int64_t f32_ld, int f32_cols,
               int f32_by_token, float f32_mult, void *bf_out, float bf_mult, const char *name,
               hipStream_t st, const SiblingPass *sp = nullptr, const void *warm = nullptr, uint64_t warm_bytes = 0,
               const SliceSums *sums = nullptr)
{
    if (R.n_items == 0 && R.n_wide == 0) return COLLM_OK;
    SkinnyArgs a{};
    // The weight of the GEMM that follows, fetched into the last-level cache by extra blocks of this pass (one per
    // compute unit) - if the weight is small (a GEMM of so few K tiles per block cannot hide the memory's latency:
    // 4096x4096 runs a fifth longer on a weight that comes from memory, 69 instead of 59 us) and this pass streams
    // less than the weight (it is then bound by latency and leaves the memory system idle; the fetch, about 12 us for
    // 33 MB, makes it 4 us longer).  Larger passes lose more than the GEMM gains (5120x5120, 8192 rows: +13 us / -11 us).
    const uint64_t pass_bytes = (uint64_t)R.n_rows * (uint64_t)K * (s->dtype == COLLM_BF16 ? 2 : 4);
    if (warm && warm_bytes <= kWarmMaxBytes && pass_bytes <= warm_bytes && c->n_cus > 0) {
        a.warm_base = warm;
        a.warm_bytes = warm_bytes;
        a.warm_blocks = c->n_cus;
    }
    const int64_t esz = s->dtype == COLLM_BF16 ? 2 : 4;
    a.in = in;
    a.ld_in = K;
    a.in_bytes = (uint32_t)((int64_t)s->n_tokens * K * esz);
    if (sp) {
        a.in = reinterpret_cast<const uint8_t *>(in) + sp->col0 * esz;
        a.ld_in = sp->ld;
        a.in_bytes = (uint32_t)((int64_t)s->n_tokens * sp->ld * esz - sp->col0 * esz);
        a.n_sib = sp->n_sib;
        a.sib = sp->sib;
        a.tab_ld = sp->ld;
        a.tab_off = sp->col0;
    }
    const int rpad = sp ? sp->rpad : c->L.rpad;
    a.K = K;
    a.tab = reinterpret_cast<const uint64_t *>(c->d_plan + off_tab);
    a.items = reinterpret_cast<const SkinnyItem *>(c->d_plan + R.off_items);
    a.row_tok = c->d_plan + R.off_row_tok;
    a.tok_train = c->d_plan + c->L.off_tok_train;
    a.f32_out = f32_out;
    a.f32_ld = f32_ld;
    a.f32_cols = f32_cols;
    a.f32_by_token = f32_by_token;
    a.f32_mult = f32_mult;
    a.bf_out = bf_out;
    a.bf_ld = c->L.rpad;
    a.bf_mult = bf_mult;
    // A wave keeps `depth` chunks of K in flight and so needs K / (waves * chunk * depth) round trips to
    // memory; cutting K into slices across blocks shortens that chain at the price of a second kernel that
    // adds the slices (about 6 us with its launch).  Cut only when the chain is longer than about six round
    // trips and the items alone give fewer than 8 waves per CU (with more, the pass is bound by bandwidth and
    // more, shorter blocks only scatter the stream), up to that many waves or down to about three trips, as
    // long as a wave keeps one chunk and the partial sums stay well below the bytes streamed (and inside the
    // workspace).
    int n_split = 1;
    if (s->dtype == COLLM_BF16) {
        const int kw = skinny_waves(rpad);
        const int per_trip = kw * skinny_chunk(rpad) * skinny_depth(rpad, R.item_rows / kSkinnyRows);
        const long trips = (K + per_trip - 1) / per_trip;
        const long per_split = (long)c->rows_cap * c->rpad_cap * 4;
        long lim = std::min<long>(kSkinnyMaxSplit, (long)c->part_bytes / per_split);
        lim = std::min<long>(lim, K / (4L * rpad));
        lim = std::min<long>(lim, K / ((long)skinny_chunk(rpad) * kw));
        const long waves = (long)R.n_items * kw;
        if (trips > 6 && waves > 0 && waves < 2048)
            n_split = (int)std::max<long>(1, std::min<long>({lim, (2048 + waves - 1) / waves, (trips + 2) / 3}));
    }
    a.part = c->d_part;
    a.part_rows = c->rows_cap;
    a.part_ld = c->rpad_cap;
    if (sums) {
        // the slices are there already: only the kernel that adds them and does this pass's stores
        if (R.n_wide > 0 || s->dtype != COLLM_BF16) return COLLM_E_SHAPE;
        a.part = sums->part;
        a.part_rows = sums->part_rows;
        a.part_ld = sums->part_ld;
        HIP_TRY(launch_skinny_finish(a, R.n_items, R.item_rows, sums->n_slices, st));
        return COLLM_OK;
    }
    Prof prof(c, st, name);
    if (s->dtype == COLLM_F32) {
        HIP_TRY(launch_skinny_f32(a, R.n_items, t_kmajor, st));
        return COLLM_OK;
    }
    if (R.n_wide > 0) {
        // Long runs: 128-row tiles through the GEMM machinery.  A block fills a CU (four LDS stages), so K is cut
        // so that at most one block per CU exists, as long as a slice keeps 512 K values and the partial sums fit
        // the workspace; the small kernel that adds the slices also does this pass's stores.
        GemmArgs g{};
        g.a = a.in;
        g.lda = a.ld_in;
        g.K = K;
        g.a_bytes = a.in_bytes;
        g.row_tok = a.row_tok;
        g.items = reinterpret_cast<const SkinnyItem *>(c->d_plan + R.off_wide);
        g.tab = a.tab;
        g.part = a.part;
        g.part_rows = a.part_rows;
        g.part_ld = a.part_ld;
        g.part_n_sib = a.n_sib;
        g.tab_ld = a.tab_ld;
        g.tab_off = a.tab_off;
        // (the warm-up rides with the tiled pass when there is one, else with the 16-row items)
        g.warm_base = a.warm_base;
        g.warm_bytes = a.warm_bytes;
        g.warm_blocks = a.warm_blocks;
        a.warm_blocks = 0;
        const long blocks = (long)R.n_wide * ((rpad + 127) / 128);
        const long per_split = (long)c->rows_cap * c->rpad_cap * 4;
        // (one block per CU with K-major tables, two with tables as they lie in memory: see launch_wide)
        long ns = std::min<long>({(t_kmajor ? 256 : 512) / blocks, std::max(1, K / 512), (long)c->part_bytes / per_split,
                                  (long)kSkinnyMaxSplit});
        ns = std::max<long>(ns, 1);
        g.k_per_split = round_up((int)((K + ns - 1) / ns), 64);
        const int n_wsplit = (K + g.k_per_split - 1) / g.k_per_split;
        HIP_TRY(launch_wide(g, R.n_wide, rpad, n_wsplit, t_kmajor, st));
        SkinnyArgs w = a;
        w.items = g.items;
        HIP_TRY(launch_skinny_finish(w, R.n_wide, kWideRows, n_wsplit, st));
    }
    if (R.n_items > 0)
        HIP_TRY(launch_skinny(a, R.n_items, rpad, R.item_rows / kSkinnyRows, n_split, t_kmajor, st));
    return COLLM_OK;
}


// Sibling projections (several projections of the same x side by side in the columns of W, y and dy).  Checks
// the description and fills c->sum_rank with the ranks summed over the siblings, which is what the rank-wide
// passes over all siblings, the plan and the context's limits see.
int prepare_siblings(collm_ctx *c, const collm_shape *s, const collm_siblings *sib, const int32_t *rank)
{
    if (!c || !s || !sib) return COLLM_E_NULL;
    if (s->dtype != COLLM_BF16) return COLLM_E_DTYPE;
    if (s->layout != COLLM_LAYOUT_IN_OUT) return COLLM_E_SHAPE;
    const bool swiglu = sib->activation == COLLM_ACT_SWIGLU;
    if (sib->activation != COLLM_ACT_NONE && !swiglu) return COLLM_E_SHAPE;
    const int P = sib->n_siblings;
    if (P < 1 || P > COLLM_MAX_SIBLINGS) return COLLM_E_SHAPE;
    if (swiglu && (P != 2 || sib->d_out[0] != sib->d_out[1])) return COLLM_E_SHAPE;
    if (!aligned16(sib->pre_act)) return COLLM_E_ALIGN;
    int64_t sum = 0;
    for (int j = 0; j < P; ++j) {
        if (sib->d_out[j] <= 0 || sib->d_out[j] % 8) return COLLM_E_SHAPE;
        if (j + 1 < P && sib->d_out[j] % 256) return COLLM_E_SHAPE;  // a column tile belongs to one sibling
        sum += sib->d_out[j];
    }
    if (sum != s->d_out) return COLLM_E_SHAPE;
    if (s->n_adapters < 0 || s->n_adapters > c->max_adapters) return COLLM_E_SHAPE;
    if (s->n_adapters > 0 && !rank) return COLLM_E_NULL;
    c->sum_rank.resize((size_t)std::max(s->n_adapters, 1));
    for (int a = 0; a < s->n_adapters; ++a) {
        if (rank[a] < 1 || rank[a] > c->max_rank || (P > 1 && rank[a] % 8) || (swiglu && rank[a] % 16))
            return COLLM_E_RANK;
        c->sum_rank[a] = rank[a] * P;
    }
    return COLLM_OK;
}

}  // namespace

// -----------------------------------------------------------------------------------------
// Workspace of collm_lora_linear_fwd_noalloc: one array per GPU the library is loaded on, held until the
// process ends.  The name is a host-side stand-in, not a device address: the address on a device comes from
// hipGetSymbolAddress with that device current, once per device, and is what the kernels receive.
namespace {
constexpr size_t kScratchBytes = (size_t)16 << 20;
constexpr int kScratchMaxTokens = 2048, kScratchMaxSegments = 2048, kScratchMaxAdapters = 64, kScratchMaxRank = 64,
              kScratchMaxD = 16384;
constexpr size_t kScratchZerosOff = 0, kScratchPlanOff = 4096, kScratchPlanBytes = (size_t)256 << 10,
                 kScratchHsOff = kScratchPlanOff + kScratchPlanBytes,
                 kScratchHsBytes = (size_t)kScratchMaxTokens * kScratchMaxRank * 4,
                 kScratchPartOff = kScratchHsOff + kScratchHsBytes, kScratchPartBytes = kScratchBytes - kScratchPartOff;
static_assert(kScratchMaxTokens % kRowPad == 0 && kScratchMaxRank % kKStep == 0, "limits are padded sizes already");
static_assert(kScratchPartOff % 256 == 0 && kScratchHsOff % 256 == 0, "every region is 256-byte aligned");
constexpr int kMaxDevices = 64;
}  // namespace
static __device__ __align__(256) unsigned char scratch[kScratchBytes];
namespace {
std::mutex g_scratch_mutex;
collm_ctx *g_scratch_ctx[kMaxDevices] = {};

// The per-device context of the entry point that allocates nothing: host bookkeeping only, every device pointer
// lies inside that device's copy of `scratch`.  Set up at the first call on the device.
int scratch_context(int device, hipStream_t st, collm_ctx **out)
{
    if (device < 0 || device >= kMaxDevices) return COLLM_E_SHAPE;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ctx[device]) {
        HIP_TRY(hipSetDevice(device));
        unsigned char *ptr = nullptr;
        HIP_TRY(hipGetSymbolAddress((void **)&ptr, HIP_SYMBOL(scratch)));
        if (!ptr || ((uintptr_t)ptr & 255u)) {
            g_last_error = "address of the static scratch array is null or misaligned";
            return COLLM_E_HIP;
        }
        collm_ctx *c = new (std::nothrow) collm_ctx();
        if (!c) return COLLM_E_NOMEM;
        c->device = device;
        c->static_scratch = true;
        c->max_tokens = kScratchMaxTokens;
        c->max_segments = kScratchMaxSegments;
        c->max_adapters = kScratchMaxAdapters;
        c->max_rank = kScratchMaxRank;
        c->max_d = kScratchMaxD;
        c->rows_cap = kScratchMaxTokens;
        c->rpad_cap = kScratchMaxRank;
        c->plan_cap = kScratchPlanBytes / sizeof(int32_t);
        c->d_zeros = ptr + kScratchZerosOff;
        c->d_plan = reinterpret_cast<int32_t *>(ptr + kScratchPlanOff);
        c->d_hs = ptr + kScratchHsOff;
        c->d_part = reinterpret_cast<float *>(ptr + kScratchPartOff);
        c->part_bytes = kScratchPartBytes;
        if (hipDeviceGetAttribute(&c->n_cus, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess) c->n_cus = 0;
        c->workspace_bytes = (int64_t)kScratchBytes;
        // host vectors at their largest size, so that later calls do not grow them
        c->plan.reserve(c->plan_cap);
        c->key_seg_start.reserve(kScratchMaxSegments + 1);
        c->key_seg_adapter.reserve(kScratchMaxSegments);
        c->key_seg_train.reserve(kScratchMaxSegments);
        c->key_rank.reserve(kScratchMaxAdapters);
        c->key_A.reserve(kScratchMaxAdapters);
        c->key_B.reserve(kScratchMaxAdapters);
        // the block of zeros that masked 16-byte loads read (a small fill kernel, in stream order before any use)
        hipError_t e = launch_fill_zero(c->d_zeros, 256, st);
        if (e != hipSuccess) {
            delete c;
            return hip_fail(e, "launch_fill_zero");
        }
        g_scratch_ctx[device] = c;
    }
    *out = g_scratch_ctx[device];
    return COLLM_OK;
}
}  // namespace

// -----------------------------------------------------------------------------------------
extern "C" {

const char *collm_status_string(int status)
{
    switch (status) {
    case COLLM_OK: return "ok";
    case COLLM_E_NULL: return "a required pointer is NULL";
    case COLLM_E_SHAPE: return "unsupported size, or beyond what the context was created for";
    case COLLM_E_SEGMENTS: return "bad segment table";
    case COLLM_E_ADAPTER: return "bad adapter index or missing adapter table";
    case COLLM_E_RANK: return "rank out of range";
    case COLLM_E_DTYPE: return "unknown element type";
    case COLLM_E_ALIGN: return "device pointer not 16-byte aligned";
    case COLLM_E_HIP: return "HIP call failed";
    case COLLM_E_NOMEM: return "allocation failed";
    default: return "unknown status";
    }
}

const char *collm_last_error(void) { return g_last_error.c_str(); }

int collm_token_map(const collm_shape *shape, const int32_t *seg_start, const int32_t *seg_adapter,
                    const uint8_t *seg_is_train, int32_t *tok_segment, int32_t *tok_adapter,
                    uint8_t *tok_is_train)
{
    if (!shape || !seg_start) return COLLM_E_NULL;
    int rc = validate_batch(shape, nullptr, seg_start, seg_adapter, seg_is_train, kMaxRank);
    if (rc != COLLM_OK) return rc;
    if (shape->n_tokens > 0 && (!tok_segment || !tok_adapter || !tok_is_train)) return COLLM_E_NULL;
    token_map(shape, seg_start, seg_adapter, seg_is_train, tok_segment, tok_adapter, tok_is_train);
    return COLLM_OK;
}

int collm_ctx_create(collm_ctx **out, int device, int32_t max_tokens, int32_t max_segments,
                     int32_t max_adapters, int32_t max_rank, int32_t max_d)
{
    if (!out) return COLLM_E_NULL;
    *out = nullptr;
    if (max_tokens < 1 || max_segments < 1 || max_adapters < 0 || max_d < 1) return COLLM_E_SHAPE;
    if (max_rank < 1 || max_rank > kMaxRank) return COLLM_E_RANK;
    HIP_TRY(hipSetDevice(device));
    collm_ctx *c = new (std::nothrow) collm_ctx();
    if (!c) return COLLM_E_NOMEM;
    c->device = device;
    c->max_tokens = max_tokens;
    c->max_segments = max_segments;
    c->max_adapters = max_adapters;
    c->max_rank = max_rank;
    c->max_d = max_d;
    c->rows_cap = round_up(max_tokens, kRowPad);
    c->rpad_cap = round_up(max_rank, kKStep);
    c->plan_cap = plan_ints_upper_bound(max_tokens, max_segments, max_adapters, max_rank);
    if (hipDeviceGetAttribute(&c->n_cus, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess) c->n_cus = 0;

    auto fail = [&](int rc) {
        collm_ctx_destroy(c);
        return rc;
    };
    int64_t ws = 0;
    auto dev_alloc = [&](void **p, size_t bytes) -> hipError_t {
        ws += (int64_t)bytes;
        return hipMalloc(p, bytes);
    };
    for (int i = 0; i < kSlots; ++i) {
        if (hipHostMalloc((void **)&c->h_stage[i], c->plan_cap * sizeof(int32_t), hipHostMallocMapped) != hipSuccess)
            return fail(COLLM_E_NOMEM);
        if (hipHostGetDevicePointer((void **)&c->h_stage_dev[i], c->h_stage[i], 0) != hipSuccess) return fail(COLLM_E_HIP);
    }
    if (hipHostMalloc((void **)&c->h_done, 64, hipHostMallocMapped) != hipSuccess) return fail(COLLM_E_NOMEM);
    *c->h_done = 0;
    if (hipHostGetDevicePointer((void **)&c->h_done_dev, c->h_done, 0) != hipSuccess) return fail(COLLM_E_HIP);
    const size_t act = (size_t)c->rows_cap * c->rpad_cap;
    // partial sums of the K slices: room for kSkinnyMaxSplit slices, but no more than 64 MiB (at least one)
    c->part_bytes = std::max(act * 4, std::min(act * 4 * kSkinnyMaxSplit, (size_t)64 << 20));
    // ... and of a GEMM with few rows: up to 8 slices of 512 rows of the widest output
    c->part_bytes = std::max(c->part_bytes, std::min((size_t)std::min(c->rows_cap, 512) * (size_t)max_d * 4 * 8, (size_t)64 << 20));
    if (dev_alloc((void **)&c->d_plan, c->plan_cap * sizeof(int32_t)) != hipSuccess ||
        dev_alloc(&c->d_hs, act * 4) != hipSuccess || dev_alloc(&c->d_dhs, act * 4) != hipSuccess ||
        dev_alloc((void **)&c->d_h32, act * 4) != hipSuccess ||
        dev_alloc((void **)&c->d_dh32, act * 4) != hipSuccess ||
        dev_alloc((void **)&c->d_copy_counter, 64) != hipSuccess || dev_alloc(&c->d_zeros, 256) != hipSuccess ||
        dev_alloc((void **)&c->d_part, c->part_bytes) != hipSuccess)
        return fail(COLLM_E_NOMEM);
    if (hipMemset(c->d_copy_counter, 0, 64) != hipSuccess) return fail(COLLM_E_HIP);
    if (hipMemset(c->d_zeros, 0, 256) != hipSuccess) return fail(COLLM_E_HIP);
    if (hipStreamCreateWithFlags(&c->side, hipStreamNonBlocking) != hipSuccess ||
        hipEventCreateWithFlags(&c->ev_fork, hipEventDisableTiming) != hipSuccess ||
        hipEventCreateWithFlags(&c->ev_dh, hipEventDisableTiming) != hipSuccess ||
        hipEventCreateWithFlags(&c->ev_join, hipEventDisableTiming) != hipSuccess)
        return fail(COLLM_E_HIP);
    if (hipDeviceSynchronize() != hipSuccess) return fail(COLLM_E_HIP);
    c->workspace_bytes = ws;
    *out = c;
    return COLLM_OK;
}

int collm_ctx_destroy(collm_ctx *c)
{
    if (!c) return COLLM_OK;
    (void)hipSetDevice(c->device);
    (void)hipDeviceSynchronize();
    for (int i = 0; i < kSlots; ++i) {
        if (c->h_stage[i]) (void)hipHostFree(c->h_stage[i]);
    }
    if (c->h_done) (void)hipHostFree(c->h_done);
    if (c->side) (void)hipStreamDestroy(c->side);
    for (hipEvent_t e : {c->ev_fork, c->ev_dh, c->ev_join})
        if (e) (void)hipEventDestroy(e);
    if (c->prof_ev_made)
        for (int i = 0; i < kMaxProfile; ++i) {
            (void)hipEventDestroy(c->prof_ev[i][0]);
            (void)hipEventDestroy(c->prof_ev[i][1]);
        }
    void *bufs[] = {c->d_plan, c->d_hs, c->d_dhs, c->d_h32, c->d_dh32, c->d_copy_counter, c->d_zeros, c->d_part};
    for (void *b : bufs)
        if (b) (void)hipFree(b);
    delete c;
    return COLLM_OK;
}

int64_t collm_ctx_workspace_bytes(const collm_ctx *c) { return c ? c->workspace_bytes : 0; }

int collm_debug_host_tile_order(int tile_rows, int tiles_m, int tiles_n, int K, int band, int32_t *band_used,
                                int32_t *tile_m, int32_t *tile_n)
{
    if (!band_used || !tile_m || !tile_n) return COLLM_E_NULL;
    if (tiles_m <= 0 || tiles_n <= 0 || K <= 0 || (tile_rows != 128 && tile_rows != 256) ||
        (int64_t)tiles_m * tiles_n > (1 << 24) || (band >= 0 && band % 8 != 0))
        return COLLM_E_SHAPE;
    *band_used = band >= 0 ? band : gemm_band_rows(tile_rows, K, tiles_m);
    host_tile_order(tiles_m, tiles_n, *band_used, tile_m, tile_n);
    return COLLM_OK;
}

int collm_debug_host_tiling(int rows, int cols, int K, int can_split, int32_t *tile, int32_t *big_tiles_m,
                            int32_t *tail_tiles_m, int32_t *tail_cols)
{
    if (!tile || !big_tiles_m || !tail_tiles_m || !tail_cols) return COLLM_E_NULL;
    if (rows < 0 || cols <= 0 || K <= 0) return COLLM_E_SHAPE;
    const Tiling t = pick_tiling(rows, cols, K, can_split != 0);
    *tile = t.tile;
    *big_tiles_m = t.big_tiles_m;
    *tail_tiles_m = t.tail_tiles_m;
    *tail_cols = t.tail_cols;
    return COLLM_OK;
}

int collm_debug_host_row_order(const collm_shape *s, const int32_t *rank, const int32_t *seg_start,
                               const int32_t *seg_adapter, const uint8_t *seg_is_train, int tile_rows,
                               int training_rows_only, int32_t *row_tok, int32_t *tile_steps)
{
    if (!s || !seg_start || !row_tok || !tile_steps) return COLLM_E_NULL;
    if (tile_rows != 64 && tile_rows != 128 && tile_rows != 256) return COLLM_E_SHAPE;
    int rc = validate_batch(s, rank, seg_start, seg_adapter, seg_is_train, 256);
    if (rc != COLLM_OK) return rc;
    PlanRequest rq;
    rq.shape = s;
    rq.rank = rank;
    rq.seg_start = seg_start;
    rq.seg_adapter = seg_adapter;
    rq.seg_is_train = seg_is_train;
    rq.bm_all = rq.bm_train = tile_rows;
    std::vector<int32_t> plan;
    PlanLayout L;
    rc = build_plan(rq, plan, L);
    if (rc != COLLM_OK) return rc;
    const RowOrderLayout &R = training_rows_only ? L.train : L.all;
    for (int i = 0; i < R.n_rows; ++i) row_tok[i] = plan[R.off_row_tok + i];
    const int n_tiles = (R.n_rows + tile_rows - 1) / tile_rows;
    for (int t = 0; t < n_tiles; ++t) tile_steps[t] = plan[R.off_ext_off + t + 1] - plan[R.off_ext_off + t];
    return R.n_rows;
}

int collm_debug_set_tiles(collm_ctx *c, int fwd_tile, int bwd_tile)
{
    if (!c) return COLLM_E_NULL;
    auto ok = [](int t) { return t == -1 || t == kTile256x256 || t == kTile128x128; };
    if (!ok(fwd_tile) || !ok(bwd_tile)) return COLLM_E_SHAPE;
    c->tile_fwd = fwd_tile;
    c->tile_bwd = bwd_tile;
    return COLLM_OK;
}

int collm_debug_set_gemm_split(collm_ctx *c, int n_slices)
{
    if (!c) return COLLM_E_NULL;
    if (n_slices < -1 || n_slices == 0 || n_slices > 64) return COLLM_E_SHAPE;
    c->gemm_split = n_slices;
    return COLLM_OK;
}

int collm_debug_set_dual_pass(collm_ctx *c, int mode)
{
    if (!c) return COLLM_E_NULL;
    if (mode < -1 || mode > 1) return COLLM_E_SHAPE;
    c->dual_pass = mode;
    return COLLM_OK;
}

int collm_debug_set_wide_pass(collm_ctx *c, int min_rows)
{
    if (!c) return COLLM_E_NULL;
    if (min_rows < -1 || min_rows > 65535) return COLLM_E_SHAPE;
    c->wide_min_rows = min_rows;
    return COLLM_OK;
}

int collm_device_info(int device, int32_t *compute_units, int32_t *clock_khz, int32_t *memory_clock_khz,
                      int32_t *memory_bus_bits, int64_t *l2_bytes)
{
    if (!compute_units || !clock_khz || !memory_clock_khz || !memory_bus_bits || !l2_bytes) return COLLM_E_NULL;
    hipDeviceProp_t pr;
    HIP_TRY(hipGetDeviceProperties(&pr, device));
    *compute_units = pr.multiProcessorCount;
    *clock_khz = pr.clockRate;
    *memory_clock_khz = pr.memoryClockRate;
    *memory_bus_bits = pr.memoryBusWidth;
    *l2_bytes = pr.l2CacheSize;
    return COLLM_OK;
}

int collm_debug_plan_stats(const collm_ctx *c, float *build_us, float *upload_us, int32_t *bytes, int32_t *mode)
{
    if (!c || !build_us || !upload_us || !bytes || !mode) return COLLM_E_NULL;
    *build_us = c->plan_build_us;
    *upload_us = c->plan_upload_us;
    *bytes = c->plan_bytes_up;
    *mode = c->plan_mode;
    return COLLM_OK;
}

int collm_profile_enable(collm_ctx *c, int enable)
{
    if (!c) return COLLM_E_NULL;
    if (enable && !c->prof_ev_made) {
        for (int i = 0; i < kMaxProfile; ++i) {
            HIP_TRY(hipEventCreate(&c->prof_ev[i][0]));
            HIP_TRY(hipEventCreate(&c->prof_ev[i][1]));
        }
        c->prof_ev_made = true;
    }
    c->profile = enable != 0;
    c->n_prof = 0;
    return COLLM_OK;
}

int collm_profile_read(collm_ctx *c, const char **names, float *ms, int cap)
{
    if (!c || !names || !ms) return COLLM_E_NULL;
    const int n = std::min(c->n_prof, cap);
    for (int i = 0; i < n; ++i) {
        names[i] = c->prof_name[i];
        ms[i] = 0.f;
        if (c->prof_launches[i] == 0) continue;
        HIP_TRY(hipEventSynchronize(c->prof_ev[i][1]));
        HIP_TRY(hipEventElapsedTime(&ms[i], c->prof_ev[i][0], c->prof_ev[i][1]));
    }
    return n;
}

static int fwd_impl(collm_ctx *c, const collm_shape *s, const collm_siblings *sib, const void *x, const void *W,
                    const void *const *A, const void *const *B, const int32_t *rank1,
                    const int32_t *seg_start, const int32_t *seg_adapter,
                    const uint8_t *seg_is_train, void *y, float *h_save, void *stream)
{
    // with siblings, `rank` is the sum over the siblings and rank1 the adapter's own
    const int P = sib ? sib->n_siblings : 1;
    int rc = sib ? prepare_siblings(c, s, sib, rank1) : COLLM_OK;
    if (rc != COLLM_OK) return rc;
    const int32_t *rank = P > 1 ? c->sum_rank.data() : rank1;
    const bool swiglu = sib && sib->activation == COLLM_ACT_SWIGLU;
    rc = check_common(c, s, x, W, A, B, rank, seg_start, seg_adapter, seg_is_train);
    if (rc != COLLM_OK) return rc;
    if (s->n_tokens > 0 && !y) return COLLM_E_NULL;
    if (!aligned16(y) || !aligned16(h_save)) return COLLM_E_ALIGN;
    if (s->n_tokens == 0) return COLLM_OK;
    hipStream_t st = (hipStream_t)stream;
    HIP_TRY(hipSetDevice(c->device));
    c->n_prof = 0;
    // (with the SwiGLU epilogue the extension steps run over both siblings' ranks, as in the backward GEMM)
    {
        Prof prof(c, st, "plan_copy");
        rc = prepare_plan(c, s, A, B, rank, seg_start, seg_adapter, seg_is_train, nullptr, nullptr, true, st,
                          P > 1 && !swiglu ? rank1 : nullptr, swiglu ? 16 + P : P);
    }
    if (rc != COLLM_OK) return rc;
    const PlanLayout &L = c->L;
    const bool f32 = s->dtype == COLLM_F32;

    // shrink: h = x A_a (fp32), kept as s*h in the element type for the GEMM's extra K-steps
    // COLLM_LAYOUT_OUT_IN: every table is the transpose, so each pass takes the kernel variant its
    // counterpart in the other direction uses
    const bool tr = s->layout == COLLM_LAYOUT_OUT_IN;
    rc = run_skinny(c, s, L.all, x, s->d_in, L.off_A_ptr, tr, h_save, c->max_rank, c->max_rank, 1, 1.0f,
                    c->d_hs, s->scale, "shrink", st, nullptr, f32 ? nullptr : W, (uint64_t)s->d_in * s->d_out * 2);
    if (rc != COLLM_OK) return rc;

    GemmArgs g{};
    g.a = x;
    g.lda = s->d_in;
    g.b = W;
    g.ldb = tr ? s->d_in : s->d_out;
    g.out = y;
    g.ldo = s->d_out;
    g.N = s->d_out;
    g.K = s->d_in;
    g.a_bytes = (uint32_t)((int64_t)s->n_tokens * s->d_in * 2);
    g.b_bytes = (uint32_t)((int64_t)s->d_in * s->d_out * 2);
    g.tiles_m = L.all.n_tiles_m;
    g.row_tok = c->d_plan + L.all.off_row_tok;
    g.ext_off = c->d_plan + L.all.off_ext_off;
    g.ext = reinterpret_cast<const ExtStep *>(c->d_plan + L.all.off_ext);
    g.hs = c->d_hs;
    g.hs_ld = L.rpad;
    g.hs_bytes = (uint32_t)((size_t)c->rows_cap * c->rpad_cap * 4);
    g.ext_ld = tr ? 0 : s->d_out;
    g.zeros = c->d_zeros;
    g.n_sib = swiglu ? 0 : P;
    for (int j = 0, col = 0; j + 1 < P; ++j) g.sib_col[j] = (col += sib->d_out[j]);
    if (swiglu) {
        // y is [T, d_ff]; W and the expand tables keep their 2 d_ff columns
        g.N = g.ldo = g.act_col = sib->d_out[0];
        g.pre_act = sib->pre_act;
        g.pre_ld = s->d_out;
        g.tok_train = c->d_plan + L.off_tok_train;
    }
    {
        Prof prof(c, st, "gemm_fwd");
        if (f32) {
            HIP_TRY(launch_gemm_f32(g, tr, st));
        } else {
            HIP_TRY(run_gemm(c, g, L.all, s->n_tokens, s->d_out, c->tile_fwd, tr, st, swiglu));
        }
    }
    return COLLM_OK;
}

int collm_lora_linear_fwd(collm_ctx *c, const collm_shape *s, const void *x, const void *W,
                          const void *const *A, const void *const *B, const int32_t *rank,
                          const int32_t *seg_start, const int32_t *seg_adapter,
                          const uint8_t *seg_is_train, void *y, float *h_save, void *stream)
{
    return fwd_impl(c, s, nullptr, x, W, A, B, rank, seg_start, seg_adapter, seg_is_train, y, h_save, stream);
}

int collm_lora_linear_fwd_noalloc(int device, const collm_shape *s, const void *x, const void *W,
                                  const void *const *A, const void *const *B, const int32_t *rank,
                                  const int32_t *seg_start, const int32_t *seg_adapter,
                                  const uint8_t *seg_is_train, void *y, float *h_save, void *stream)
{
    if (!s) return COLLM_E_NULL;
    if (s->n_tokens > kScratchMaxTokens || s->n_segments > kScratchMaxSegments || s->n_adapters > kScratchMaxAdapters ||
        s->d_in > kScratchMaxD || s->d_out > kScratchMaxD) {
        char buf[200];
        std::snprintf(buf, sizeof buf,
                      "collm_lora_linear_fwd_noalloc serves at most %d tokens, %d segments, %d adapters of rank <= %d and "
                      "d_in, d_out <= %d (static workspace of %zu MiB)",
                      kScratchMaxTokens, kScratchMaxSegments, kScratchMaxAdapters, kScratchMaxRank, kScratchMaxD,
                      kScratchBytes >> 20);
        g_last_error = buf;
        return COLLM_E_SHAPE;
    }
    collm_ctx *c = nullptr;
    int rc = scratch_context(device, (hipStream_t)stream, &c);
    if (rc != COLLM_OK) return rc;
    rc = fwd_impl(c, s, nullptr, x, W, A, B, rank, seg_start, seg_adapter, seg_is_train, y, h_save, stream);
    if (rc == COLLM_E_RANK)
        g_last_error = "collm_lora_linear_fwd_noalloc: a rank is outside 1..64 (the static workspace's limit)";
    return rc;
}

int collm_lora_siblings_fwd(collm_ctx *c, const collm_shape *s, const collm_siblings *sib, const void *x,
                            const void *W, const void *const *A, const void *const *B, const int32_t *rank,
                            const int32_t *seg_start, const int32_t *seg_adapter, const uint8_t *seg_is_train,
                            void *y, float *h_save, void *stream)
{
    if (!sib) return COLLM_E_NULL;
    return fwd_impl(c, s, sib, x, W, A, B, rank, seg_start, seg_adapter, seg_is_train, y, h_save, stream);
}

static int bwd_impl(collm_ctx *c, const collm_shape *s, const collm_siblings *sib, const void *x, const void *W,
                    const void *const *A, const void *const *B, const int32_t *rank1,
                    const int32_t *seg_start, const int32_t *seg_adapter,
                    const uint8_t *seg_is_train, const void *dy, const float *h_save, void *dx,
                    float *const *dA, float *const *dB, int accumulate, void *stream)
{
    const int P = sib ? sib->n_siblings : 1;
    int rc = sib ? prepare_siblings(c, s, sib, rank1) : COLLM_OK;
    if (rc != COLLM_OK) return rc;
    const int32_t *rank = P > 1 ? c->sum_rank.data() : rank1;
    rc = check_common(c, s, x, W, A, B, rank, seg_start, seg_adapter, seg_is_train);
    if (rc != COLLM_OK) return rc;
    if ((dA == nullptr) != (dB == nullptr)) return COLLM_E_NULL;
    int n_train = 0;
    for (int k = 0; k < s->n_segments; ++k) {
        if (!seg_is_train[k] || seg_start[k + 1] == seg_start[k]) continue;
        n_train += seg_start[k + 1] - seg_start[k];
        const int a = seg_adapter[k];
        if (dA) {
            if (!dA[a] || !dB[a]) return COLLM_E_ADAPTER;
            if (!aligned16(dA[a]) || !aligned16(dB[a])) return COLLM_E_ALIGN;
        }
    }
    if (n_train > 0 && !dy) return COLLM_E_NULL;
    if (!aligned16(dy) || !aligned16(dx) || !aligned16(h_save)) return COLLM_E_ALIGN;
    if (n_train == 0) return COLLM_OK;
    hipStream_t st = (hipStream_t)stream;
    HIP_TRY(hipSetDevice(c->device));
    c->n_prof = 0;
    {
        Prof prof(c, st, "plan_copy");
        rc = prepare_plan(c, s, A, B, rank, seg_start, seg_adapter, seg_is_train, dA, dB, true, st,
                          P > 1 ? rank1 : nullptr, P);
    }
    if (rc != COLLM_OK) return rc;
    // siblings: widest single rank, padded, for the passes that take one sibling at a time
    int rpad1 = c->L.rpad;
    if (P > 1) {
        int r1 = 1;
        for (int a = 0; a < s->n_adapters; ++a) r1 = std::max(r1, rank1[a]);
        rpad1 = round_up(r1, kKStep);
    }
    const PlanLayout &L = c->L;
    const bool f32 = s->dtype == COLLM_F32;
    const bool tr = s->layout == COLLM_LAYOUT_OUT_IN;

    // h of the training rows, if the forward call did not keep it
    if (!h_save && dA) {
        rc = run_skinny(c, s, L.train, x, s->d_in, L.off_A_ptr, tr, c->d_h32, L.rpad, L.rpad, 0, 1.0f,
                        c->d_hs, s->scale, "shrink_recompute", st);
        if (rc != COLLM_OK) return rc;
    }
    // The adapter gradients depend on little (dB_a: h and dy; dA_a: dh and x) and are bound by memory
    // latency, as is dh: they run on a second stream beside dh and the dX GEMM, which joins the
    // caller's stream again before the call returns.  (Serial when kernels are being timed.)
    const bool overlap = dA && !c->profile;
    hipStream_t gs = overlap ? c->side : st;
    GradArgs ga{};
    const int64_t esz = f32 ? 4 : 2;
    ga.row_tok = c->d_plan + L.train.off_row_tok;
    ga.items = reinterpret_cast<const GradItem *>(c->d_plan + L.off_grad);
    ga.accumulate = accumulate ? 1 : 0;

    // Narrow ranks (all at most 16), tables as [rank][d_out]: dh and dB_a both come from ONE pass over the training
    // rows of dy (kernels.h, DualArgs), which is the largest operand of the backward pass beside W.  The rows of
    // every trained adapter are cut into pieces so that two blocks per CU exist (pieces of 512 rows down to 64), as
    // long as the per-group slices of dh and the per-piece sums of dB fit the workspace of partial sums.  It pays where
    // the training rows of dy do not fit the last-level cache (256 MB): 8192 rows of 28672 columns (470 MB) take 153 us
    // against 94 + 122 for the two passes and the step is 1 % shorter; 8192 x 8192 (134 MB) 65 against 31 + 43 with
    // no gain for the step (the two passes run side by side on two streams and the second reader finds dy in the
    // cache); on 8192 x 1024 (34 against 10 + 15) and 1792 x 4096 (28 against 14 + 10) the partial sums and the two
    // kernels that add them cost more than the second read.
    constexpr int64_t kDualMinBytes = (int64_t)192 << 20;
    DualArgs du{};
    bool dual = false;
    if (!f32 && !tr && P == 1 && dA && c->dual_pass != 0 && L.rpad == kKStep && L.train.n_wide == 0 && L.n_grad > 0 &&
        (c->dual_pass == 1 || (int64_t)L.train.n_rows * s->d_out * 2 >= kDualMinBytes)) {
        const int groups = (s->d_out + kDualCols - 1) / kDualCols;
        auto pieces_of = [&](int rows) { return (L.max_grad_rows + rows - 1) / rows; };
        auto fits = [&](int rows) {
            const size_t dh_floats = (size_t)round_up(groups * L.train.n_rows_pad * kKStep, 64);
            // (pieces are the grid's second dimension, with the rows of blocks that fetch the weight behind them)
            return (long)L.n_grad * pieces_of(rows) + c->n_cus < 65536 &&
                   (dh_floats + (size_t)L.n_grad * pieces_of(rows) * kKStep * s->d_out) * 4 <= c->part_bytes;
        };
        int rows = kDualMaxPieceRows;
        while (rows > 64 && (long)groups * L.n_grad * pieces_of(rows) < 2L * std::max(c->n_cus, 1)) rows >>= 1;
        while (rows < kDualMaxPieceRows && !fits(rows)) rows <<= 1;
        if (fits(rows)) {
            dual = true;
            du.dy = dy;
            du.ld_dy = s->d_out;
            du.dy_bytes = (uint32_t)((int64_t)s->n_tokens * s->d_out * 2);
            du.N = s->d_out;
            du.hs = c->d_hs;
            du.ld_hs = L.rpad;
            du.hs_bytes = (uint32_t)((size_t)L.train.n_rows_pad * L.rpad * 2);
            du.row_tok = ga.row_tok;
            du.items = ga.items;
            du.n_grad = L.n_grad;
            du.tab_b = reinterpret_cast<const uint64_t *>(c->d_plan + L.off_B_ptr);
            du.out_tab = reinterpret_cast<const uint64_t *>(c->d_plan + L.off_dB_ptr);
            du.accumulate = ga.accumulate;
            du.piece_rows = rows;
            du.max_pieces = pieces_of(rows);
            du.part_dh = c->d_part;
            du.part_rows = L.train.n_rows_pad;
            du.part_ld = kKStep;
            du.part_dB = c->d_part + round_up(groups * L.train.n_rows_pad * kKStep, 64);
            // (the weight of the dX GEMM, as the dh pass would fetch it: see run_skinny)
            const uint64_t w_bytes = (uint64_t)s->d_in * s->d_out * 2;
            if (dx && w_bytes <= kWarmMaxBytes && (uint64_t)L.train.n_rows * s->d_out * 2 <= w_bytes && c->n_cus > 0) {
                du.warm_base = W;
                du.warm_bytes = w_bytes;
                du.warm_rows = (c->n_cus + groups - 1) / groups;
            }
        }
    }
    if (dual) {
        Prof prof(c, st, "dh_dB");
        // s h as bf16 in training row order: left by the recomputing pass, or packed from h_save here
        if (h_save)
            HIP_TRY(launch_pack_rows(h_save, c->max_rank, c->max_rank, c->d_plan + L.train.off_row_tok, L.train.n_rows,
                                     s->scale, c->d_hs, L.rpad, st));
        HIP_TRY(launch_dual(du, st));
        const SliceSums sums{du.part_dh, du.part_rows, du.part_ld, (s->d_out + kDualCols - 1) / kDualCols};
        rc = run_skinny(c, s, L.train, dy, s->d_out, L.off_B_ptr, true, c->d_dh32, L.rpad, L.rpad, 0, s->scale, c->d_dhs,
                        s->scale, nullptr, st, nullptr, nullptr, 0, &sums);
        if (rc != COLLM_OK) return rc;
        HIP_TRY(launch_dual_sum(du, st));
    }
    if (dA && !dual) {
        if (overlap) {
            HIP_TRY(hipEventRecord(c->ev_fork, st));
            HIP_TRY(hipStreamWaitEvent(c->side, c->ev_fork, 0));
        }
        // dB_a = s h^T dy
        ga.big = dy;
        ga.ld_big = s->d_out;
        ga.big_bytes = (uint32_t)((int64_t)s->n_tokens * s->d_out * esz);
        ga.N = s->d_out;
        if (h_save) {
            ga.small_ = h_save;
            ga.ld_small = c->max_rank;
            ga.small_by_token = 1;
        } else {
            ga.small_ = c->d_h32;
            ga.ld_small = L.rpad;
            ga.small_by_token = 0;
        }
        ga.small_mult = s->scale;
        if (!f32) {
            // the small operand as a scaled bf16 copy in training row order (half the bytes of the fp32 one, no
            // conversion in the kernel): left by the recomputing pass, or packed from h_save here.  The forward
            // call's copy of s h (all rows) in the same buffer is dead once that call's GEMM has run.
            if (h_save)
                HIP_TRY(launch_pack_rows(h_save, c->max_rank, c->max_rank, c->d_plan + L.train.off_row_tok,
                                         L.train.n_rows, s->scale, c->d_hs, L.rpad, gs));
            ga.small_bf = c->d_hs;
            ga.ld_small_bf = L.rpad;
        }
        ga.out_tab = reinterpret_cast<const uint64_t *>(c->d_plan + L.off_dB_ptr);
        ga.out_transposed = tr ? 1 : 0;
        {
            Prof prof(c, gs, "grad_dB");
            if (f32) {
                HIP_TRY(launch_grad_f32(ga, L.n_grad, gs));
            } else if (P == 1) {
                HIP_TRY(launch_grad(ga, L.n_grad, L.rpad, gs));
            } else {
                // one launch per sibling: its columns of dy against its columns of s h
                for (int j = 0, col = 0; j < P; col += sib->d_out[j], ++j) {
                    GradArgs gj = ga;
                    gj.big = reinterpret_cast<const uint8_t *>(dy) + (int64_t)col * 2;
                    gj.big_bytes = ga.big_bytes - (uint32_t)col * 2u;
                    gj.N = sib->d_out[j];
                    gj.n_sib = P;
                    gj.sib = j;
                    gj.ld_out = s->d_out;
                    gj.out_off = col;
                    HIP_TRY(launch_grad(gj, L.n_grad, rpad1, gs));
                }
            }
        }
    }

    // dh = s dy B_a^T: fp32 for dA, element type for the dX GEMM's extra K-steps
    if (dual) {
        // dh came out of the pass over dy above, together with dB
    } else if (P == 1) {
        rc = run_skinny(c, s, L.train, dy, s->d_out, L.off_B_ptr, !tr, c->d_dh32, L.rpad, L.rpad, 0, s->scale,
                        c->d_dhs, s->scale, "dh", st, nullptr, (f32 || !dx) ? nullptr : W, (uint64_t)s->d_in * s->d_out * 2);
        if (rc != COLLM_OK) return rc;
    } else {
        // one pass per sibling over its columns of dy and of the tables, each writing its columns of dh
        for (int j = 0, col = 0; j < P; col += sib->d_out[j], ++j) {
            SiblingPass sp;
            sp.n_sib = P;
            sp.sib = j;
            sp.ld = s->d_out;
            sp.col0 = col;
            sp.rpad = rpad1;
            rc = run_skinny(c, s, L.train, dy, sib->d_out[j], L.off_B_ptr, true, c->d_dh32, L.rpad, L.rpad, 0,
                            s->scale, c->d_dhs, s->scale, "dh", st, &sp);
            if (rc != COLLM_OK) return rc;
        }
    }

    if (dA) {
        if (overlap) {
            HIP_TRY(hipEventRecord(c->ev_dh, st));
            HIP_TRY(hipStreamWaitEvent(c->side, c->ev_dh, 0));
        }
        // dA_a = x^T dh
        ga.big = x;
        ga.ld_big = s->d_in;
        ga.big_bytes = (uint32_t)((int64_t)s->n_tokens * s->d_in * esz);
        ga.N = s->d_in;
        ga.small_ = c->d_dh32;
        ga.ld_small = L.rpad;
        ga.small_by_token = 0;
        ga.small_mult = 1.0f;
        if (!f32) {
            ga.small_bf = c->d_dhs;  // dh in the element type, as the dh pass left it for the dX GEMM
            ga.ld_small_bf = L.rpad;
        }
        ga.out_tab = reinterpret_cast<const uint64_t *>(c->d_plan + L.off_dA_ptr);
        ga.out_transposed = tr ? 0 : 1;
        {
            Prof prof(c, gs, "grad_dA");
            if (f32) HIP_TRY(launch_grad_f32(ga, L.n_grad, gs));
            else HIP_TRY(launch_grad(ga, L.n_grad, L.rpad, gs));
        }
        if (overlap) HIP_TRY(hipEventRecord(c->ev_join, c->side));
    }

    if (dx) {
        GemmArgs g{};
        g.a = dy;
        g.lda = s->d_out;
        g.b = W;
        g.ldb = tr ? s->d_in : s->d_out;
        g.out = dx;
        g.ldo = s->d_in;
        g.N = s->d_in;
        g.K = s->d_out;
        g.a_bytes = (uint32_t)((int64_t)s->n_tokens * s->d_out * 2);
        g.b_bytes = (uint32_t)((int64_t)s->d_in * s->d_out * 2);
        g.tiles_m = L.train.n_tiles_m;
        g.row_tok = c->d_plan + L.train.off_row_tok;
        g.ext_off = c->d_plan + L.train.off_ext_off;
        g.ext = reinterpret_cast<const ExtStep *>(c->d_plan + L.train.off_ext);
        g.hs = c->d_dhs;
        g.hs_ld = L.rpad;
        g.hs_bytes = (uint32_t)((size_t)c->rows_cap * c->rpad_cap * 4);
        g.ext_ld = tr ? s->d_in : 0;
        g.zeros = c->d_zeros;
        Prof prof(c, st, "gemm_dx");
        if (f32) {
            HIP_TRY(launch_gemm_f32(g, !tr, st));
        } else {
            HIP_TRY(run_gemm(c, g, L.train, n_train, s->d_in, c->tile_bwd, !tr, st));
        }
    }
    if (overlap) HIP_TRY(hipStreamWaitEvent(st, c->ev_join, 0));
    return COLLM_OK;
}

int collm_lora_linear_bwd(collm_ctx *c, const collm_shape *s, const void *x, const void *W,
                          const void *const *A, const void *const *B, const int32_t *rank,
                          const int32_t *seg_start, const int32_t *seg_adapter,
                          const uint8_t *seg_is_train, const void *dy, const float *h_save, void *dx,
                          float *const *dA, float *const *dB, int accumulate, void *stream)
{
    return bwd_impl(c, s, nullptr, x, W, A, B, rank, seg_start, seg_adapter, seg_is_train, dy, h_save, dx, dA, dB,
                    accumulate, stream);
}

int collm_lora_siblings_bwd(collm_ctx *c, const collm_shape *s, const collm_siblings *sib, const void *x,
                            const void *W, const void *const *A, const void *const *B, const int32_t *rank,
                            const int32_t *seg_start, const int32_t *seg_adapter, const uint8_t *seg_is_train,
                            const void *dy, const float *h_save, void *dx, float *const *dA, float *const *dB,
                            int accumulate, void *stream)
{
    if (!sib) return COLLM_E_NULL;
    return bwd_impl(c, s, sib, x, W, A, B, rank, seg_start, seg_adapter, seg_is_train, dy, h_save, dx, dA, dB,
                    accumulate, stream);
}

int collm_swiglu_bwd(int device, int32_t n_tokens, int32_t d_ff, int32_t n_segments, const int32_t *seg_start,
                     const uint8_t *seg_is_train, const void *pre_act, const void *dout, void *dy, void *stream)
{
    if (n_tokens < 0 || n_segments < 0 || d_ff <= 0 || d_ff % 8) return COLLM_E_SHAPE;
    if (n_segments > 0 && (!seg_start || !seg_is_train)) return COLLM_E_NULL;
    if (n_segments > 0 && seg_start[0] != 0) return COLLM_E_SEGMENTS;
    bool any = false;
    for (int k = 0; k < n_segments; ++k) {
        if (seg_start[k + 1] < seg_start[k]) return COLLM_E_SEGMENTS;
        any = any || (seg_is_train[k] && seg_start[k + 1] > seg_start[k]);
    }
    if (n_segments > 0 && seg_start[n_segments] != n_tokens) return COLLM_E_SEGMENTS;
    if (!any) return COLLM_OK;
    if (!pre_act || !dout || !dy) return COLLM_E_NULL;
    if (!aligned16(pre_act) || !aligned16(dout) || !aligned16(dy)) return COLLM_E_ALIGN;
    HIP_TRY(hipSetDevice(device));
    SwigluBwdArgs a{};
    a.pre = pre_act;
    a.dout = dout;
    a.dy = dy;
    a.d_ff = d_ff;
    a.ld_pre = a.ld_dy = 2 * (int64_t)d_ff;
    a.ld_dout = d_ff;
    for (int k = 0; k < n_segments; ++k) {
        const int n = seg_start[k + 1] - seg_start[k];
        if (seg_is_train[k] && n > 0) {
            a.tok0[a.n_seg] = seg_start[k];
            a.row0[a.n_seg + 1] = a.row0[a.n_seg] + n;
            ++a.n_seg;
        }
        if (a.n_seg == kSwigluSegs || (k + 1 == n_segments && a.n_seg > 0)) {
            HIP_TRY(launch_swiglu_bwd(a, (hipStream_t)stream));
            a.n_seg = 0;
        }
    }
    return COLLM_OK;
}

int collm_adapter_fedavg(int device, collm_dtype dtype, int32_t n_copies, const void *const *src, void *dst,
                         int64_t n_elems, void *stream)
{
    if (dtype != COLLM_F32 && dtype != COLLM_BF16) return COLLM_E_DTYPE;
    if (n_copies < 1 || n_copies > kMaxFedAvgCopies || n_elems < 0) return COLLM_E_SHAPE;
    if (!src || (n_elems > 0 && !dst)) return COLLM_E_NULL;
    if (!aligned16(dst)) return COLLM_E_ALIGN;
    FedAvgArgs a{};
    for (int k = 0; k < n_copies; ++k) {
        if (n_elems > 0 && !src[k]) return COLLM_E_NULL;
        if (!aligned16(src[k])) return COLLM_E_ALIGN;
        a.src[k] = src[k];
    }
    if (n_elems == 0) return COLLM_OK;
    a.dst = dst;
    a.n = n_elems;
    a.n_copies = n_copies;
    HIP_TRY(hipSetDevice(device));
    HIP_TRY(launch_fedavg(a, dtype == COLLM_BF16, (hipStream_t)stream));
    return COLLM_OK;
}

int collm_adapter_adamw(int device, collm_dtype dtype, void *param, float *master, const float *grad,
                        float *m, float *v, int64_t n_elems, const collm_adamw *hp, void *stream)
{
    if (dtype != COLLM_F32 && dtype != COLLM_BF16) return COLLM_E_DTYPE;
    if (!hp) return COLLM_E_NULL;
    if (n_elems < 0 || hp->step < 1) return COLLM_E_SHAPE;
    if (n_elems == 0) return COLLM_OK;
    if (!param || !grad || !m || !v) return COLLM_E_NULL;
    if (!aligned16(param) || !aligned16(master) || !aligned16(grad) || !aligned16(m) || !aligned16(v)) return COLLM_E_ALIGN;
    AdamWArgs a{};
    a.param = param;
    a.master = master;
    a.grad = grad;
    a.m = m;
    a.v = v;
    a.n = n_elems;
    a.lr = hp->lr;
    a.beta1 = hp->beta1;
    a.beta2 = hp->beta2;
    a.eps = hp->eps;
    a.weight_decay = hp->weight_decay;
    a.bias1 = (float)(1.0 - std::pow((double)hp->beta1, (double)hp->step));
    a.rsqrt_bias2 = (float)(1.0 / std::sqrt(1.0 - std::pow((double)hp->beta2, (double)hp->step)));
    HIP_TRY(hipSetDevice(device));
    HIP_TRY(launch_adamw(a, dtype == COLLM_BF16, (hipStream_t)stream));
    return COLLM_OK;
}

int collm_debug_device_token_map(collm_ctx *c, int32_t *tok_segment, int32_t *tok_adapter,
                                 uint8_t *tok_is_train)
{
    if (!c) return COLLM_E_NULL;
    if (!c->plan_valid) return COLLM_E_SHAPE;
    const PlanLayout &L = c->L;
    if (L.n_tokens > 0 && (!tok_segment || !tok_adapter || !tok_is_train)) return COLLM_E_NULL;
    HIP_TRY(hipSetDevice(c->device));
    HIP_TRY(hipStreamSynchronize(c->last_stream));
    std::vector<int32_t> dev((size_t)L.total_ints);
    HIP_TRY(hipMemcpy(dev.data(), c->d_plan, dev.size() * sizeof(int32_t), hipMemcpyDeviceToHost));
    // Undo the adapter grouping: row r of the forward row order is token row_tok[r] and was
    // given adapter row_adapter[r]; segment and training flag come from the per-token arrays
    // the kernels read.
    for (int t = 0; t < L.n_tokens; ++t) tok_adapter[t] = -2;
    for (int r = 0; r < L.all.n_rows_pad; ++r) {
        const int tok = dev[L.all.off_row_tok + r];
        if (tok < 0) continue;
        if (tok >= L.n_tokens) return COLLM_E_SHAPE;
        tok_adapter[tok] = dev[L.all.off_row_adapter + r];
    }
    for (int t = 0; t < L.n_tokens; ++t) {
        tok_segment[t] = dev[L.off_tok_segment + t];
        tok_is_train[t] = (uint8_t)dev[L.off_tok_train + t];
        // the per-token adapter array must agree with the row order
        if (dev[L.off_tok_adapter + t] != tok_adapter[t]) tok_adapter[t] = -3;
    }
    // training rows must be exactly the training tokens
    std::vector<uint8_t> seen((size_t)std::max(L.n_tokens, 1), 0);
    for (int r = 0; r < L.train.n_rows_pad; ++r) {
        const int tok = dev[L.train.off_row_tok + r];
        if (tok >= 0 && tok < L.n_tokens) seen[tok] = 1;
    }
    for (int t = 0; t < L.n_tokens; ++t)
        if (seen[t] != tok_is_train[t]) tok_is_train[t] = 0xEE;
    return COLLM_OK;
}

}  // extern "C"
