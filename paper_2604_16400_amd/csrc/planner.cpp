// Host-side planner: segment table -> device plan (see plan.h).  Integer work only.
#include "planner.h"

#include <algorithm>
#include <cstring>

namespace collm {

int validate_batch(const collm_shape *s, const int32_t *rank, const int32_t *seg_start,
                   const int32_t *seg_adapter, const uint8_t *seg_is_train, int max_rank)
{
    if (!s || !seg_start) return COLLM_E_NULL;
    if (s->n_tokens < 0 || s->n_segments < 0 || s->n_adapters < 0) return COLLM_E_SHAPE;
    if (s->n_segments > 0 && (!seg_adapter || !seg_is_train)) return COLLM_E_NULL;
    if (s->n_adapters > 0 && rank) {
        for (int a = 0; a < s->n_adapters; ++a)
            if (rank[a] < 1 || rank[a] > max_rank) return COLLM_E_RANK;
    }
    if (seg_start[0] != 0) return COLLM_E_SEGMENTS;
    for (int k = 0; k < s->n_segments; ++k)
        if (seg_start[k + 1] < seg_start[k]) return COLLM_E_SEGMENTS;
    if (seg_start[s->n_segments] != s->n_tokens) return COLLM_E_SEGMENTS;
    for (int k = 0; k < s->n_segments; ++k) {
        const int a = seg_adapter[k];
        if (a < -1 || a >= s->n_adapters) return COLLM_E_ADAPTER;
        if (seg_is_train[k] > 1) return COLLM_E_SEGMENTS;
        if (seg_is_train[k] && a < 0) return COLLM_E_ADAPTER;
    }
    return COLLM_OK;
}

void token_map(const collm_shape *s, const int32_t *seg_start, const int32_t *seg_adapter,
               const uint8_t *seg_is_train, int32_t *tok_segment, int32_t *tok_adapter,
               uint8_t *tok_is_train)
{
    for (int k = 0; k < s->n_segments; ++k) {
        const int lo = seg_start[k], hi = seg_start[k + 1];
        std::fill(tok_segment + lo, tok_segment + hi, k);
        std::fill(tok_adapter + lo, tok_adapter + hi, seg_adapter[k]);
        std::fill(tok_is_train + lo, tok_is_train + hi, seg_is_train[k]);
    }
}

static inline int round_up(int v, int m) { return (v + m - 1) / m * m; }

namespace {

struct Builder {
    std::vector<int32_t> &blk;
    explicit Builder(std::vector<int32_t> &b) : blk(b) {}
    int32_t alloc(size_t n_ints, int align_ints = 4)
    {
        size_t off = (blk.size() + align_ints - 1) / align_ints * align_ints;
        blk.resize(off + n_ints, 0);
        return (int32_t)off;
    }
};

// Rows (token indices, already filtered) sorted by adapter, stable; items; extension tables.
void build_row_order(Builder &b, RowOrderLayout &L, const std::vector<int32_t> &tokens,
                     const int32_t *tok_adapter, const int32_t *rank, int n_adapters, int bm,
                     const void *const *ext_tab, int max_row_tiles, int rpad, int wide_min_rows,
                     const int32_t *rank_ext, bool split_runs)
{
    const int n = (int)tokens.size();
    L.n_rows = n;
    L.n_rows_pad = round_up(std::max(n, 1), kRowPad);
    L.off_row_tok = b.alloc(L.n_rows_pad);
    L.off_row_adapter = b.alloc(L.n_rows_pad);

    // Rows in runs of one adapter, stable in token order inside an adapter; base-only rows first.  Where the
    // runs lie is free, and it decides how the extension steps spread over the GEMM row tiles: every adapter
    // that reaches into a tile costs that tile its K-steps, and the tiles with the most steps finish last.
    // With adapters of very different popularity, listing them by index would pile the many rare ones into
    // the last tiles.  So (split_runs): the adapters with less than a tile of rows are dealt out over the
    // tiles in proportion to the rows passed, each as one run, and the rows of the larger adapters fill
    // what is left of every tile (they reach into several tiles anyway).  Without split_runs every adapter
    // is one run (what the gradient items need), larger adapters first.
    std::vector<int32_t> count(n_adapters + 1, 0);  // [0]: base-only rows
    for (int i = 0; i < n; ++i) count[tok_adapter[tokens[i]] + 1]++;
    struct Run {
        int32_t adapter, lo, len;
    };
    std::vector<Run> runs;  // in row order
    {
        std::vector<int32_t> big, small_;
        for (int a = 0; a < n_adapters; ++a) {
            if (count[a + 1] >= bm) big.push_back(a);
            else if (count[a + 1] > 0) small_.push_back(a);
        }
        auto larger = [&](int32_t x, int32_t y) { return count[x + 1] > count[y + 1]; };
        std::stable_sort(big.begin(), big.end(), larger);
        std::stable_sort(small_.begin(), small_.end(), larger);
        int32_t pos = count[0];
        const int64_t adapter_rows = n - count[0];
        size_t dealt = 0, bi = 0;
        int32_t rem = big.empty() ? 0 : count[big[0] + 1];
        auto put = [&](int32_t a, int32_t len) {
            if (!runs.empty() && runs.back().adapter == a) runs.back().len += len;
            else runs.push_back({a, pos, len});
            pos += len;
        };
        while (pos < n) {
            const int32_t tile_end = std::min(n, (pos / bm + 1) * bm);
            size_t due = bi < big.size() ? (size_t)((int64_t)small_.size() * (tile_end - count[0]) / adapter_rows)
                                         : small_.size();
            if (!split_runs) due = bi < big.size() ? 0 : small_.size();
            while (dealt < due && dealt < small_.size()) {
                put(small_[dealt], count[small_[dealt] + 1]);
                ++dealt;
            }
            const int32_t fill_end = split_runs ? tile_end : n;
            while (pos < fill_end && bi < big.size()) {
                const int32_t take = std::min(rem, fill_end - pos);
                put(big[bi], take);
                rem -= take;
                if (rem == 0 && ++bi < big.size()) rem = count[big[bi] + 1];
            }
        }
    }
    {
        int32_t *row_tok = b.blk.data() + L.off_row_tok;
        int32_t *row_ad = b.blk.data() + L.off_row_adapter;
        // the tokens of an adapter fill its runs in row order
        std::vector<std::vector<int32_t>> runs_of(n_adapters);
        for (size_t k = 0; k < runs.size(); ++k) runs_of[runs[k].adapter].push_back((int32_t)k);
        std::vector<int32_t> which(n_adapters, 0), used(n_adapters, 0);
        int32_t base_pos = 0;
        for (int i = 0; i < n; ++i) {
            const int a = tok_adapter[tokens[i]];
            int32_t pos_i;
            if (a < 0) {
                pos_i = base_pos++;
            } else {
                if (used[a] == runs[runs_of[a][which[a]]].len) {
                    ++which[a];
                    used[a] = 0;
                }
                pos_i = runs[runs_of[a][which[a]]].lo + used[a]++;
            }
            row_tok[pos_i] = tokens[i];
            row_ad[pos_i] = a;
        }
        for (int i = n; i < L.n_rows_pad; ++i) {
            row_tok[i] = -1;
            row_ad[i] = -1;
        }
    }

    // skinny items: runs of one adapter, cut into pieces of at most item_rows rows.  Two row tiles per
    // item halve the fetches of an adapter's table (which weigh as much as the rows for rank 16 and
    // several times as much for larger ranks) but also halve the waves in flight, and these passes are
    // bound by memory latency on small batches: measured, pairs pay from about 4096 rows on.
    // (for ranks above 64, where the table outweighs the rows eight times and more, from 2048 rows on)
    const int tiles = (max_row_tiles >= 2 && (n >= 4096 || (rpad >= 128 && n >= 2048))) ? 2 : 1;
    L.item_rows = kSkinnyRows * tiles;
    // Long runs go to the tiled pass instead (items of up to kWideRows rows: an adapter's table is fetched
    // once per 128 rows); what a run leaves over below the threshold stays a skinny item.
    std::vector<SkinnyItem> items, wide;
    for (const Run &run : runs) {
        const int32_t a = run.adapter;
        int lo = run.lo;
        const int hi = run.lo + run.len;
        if (wide_min_rows > 0 && rank[a] % 8 == 0) {
            while (hi - lo >= wide_min_rows) {
                const int m = std::min(kWideRows, hi - lo);
                wide.push_back({a, lo, m, rank[a]});
                lo += m;
            }
        }
        for (int r = lo; r < hi; r += L.item_rows)
            items.push_back({a, r, std::min(L.item_rows, hi - r), rank[a]});
    }
    L.n_items = (int)items.size();
    L.off_items = b.alloc(items.size() * 4 + 4);
    if (!items.empty())
        std::memcpy(b.blk.data() + L.off_items, items.data(), items.size() * sizeof(SkinnyItem));
    L.n_wide = (int)wide.size();
    L.off_wide = b.alloc(wide.size() * 4 + 4);
    if (!wide.empty())
        std::memcpy(b.blk.data() + L.off_wide, wide.data(), wide.size() * sizeof(SkinnyItem));

    // low-rank extension steps of every GEMM row tile
    auto build_ext = [&](int tile_rows, int32_t &n_tiles, int32_t &off_ext_off, int32_t &off_ext, int32_t *n_ext,
                         int32_t *max_per_tile, std::vector<int32_t> &step_adapter) {
        step_adapter.clear();
        n_tiles = L.n_rows_pad / tile_rows;
        std::vector<int32_t> ext_off(n_tiles + 1, 0);
        std::vector<ExtStep> ext;
        int most = 0;
        for (int t = 0; t < n_tiles; ++t) {
            ext_off[t] = (int)ext.size();
            const int r0 = t * tile_rows, r1 = std::min(n, r0 + tile_rows);
            // The steps of a tile are listed by 64-wide groups of rank indices (all runs' steps below 64, then
            // those of 64..127, ...), and a group that is not the tile's last is filled up to whole batches with
            // empty steps: a batch then lies inside one group, which is what a kernel that keeps one group of
            // every row's low-rank activations in LDS needs.  (Ranks up to 64: one group, nothing changes.)
            for (int g0 = 0, more = 1; more; g0 += kExtGroup) {
                more = 0;
                if (g0 > 0)
                    while (((int)ext.size() - ext_off[t]) % kExtBatch != 0) {
                        ext.push_back({0u, 0u, 0});
                        step_adapter.push_back(-1);
                    }
                int r = r0;
                while (r < r1) {
                    const int a = b.blk[L.off_row_adapter + r];
                    int e = r + 1;
                    while (e < r1 && b.blk[L.off_row_adapter + e] == a) ++e;
                    if (a >= 0) {
                        const uint64_t tab = ext_tab ? (uint64_t)(uintptr_t)ext_tab[a] : 0;
                        for (int k = g0; k < std::min(rank_ext[a], g0 + kExtGroup); k += kKStep) {
                            ext.push_back({(uint32_t)k | ((uint32_t)rank_ext[a] << 16), (uint32_t)(r - r0) | ((uint32_t)(e - r0) << 16), tab});
                            step_adapter.push_back(a);
                        }
                        if (rank_ext[a] > g0 + kExtGroup) more = 1;
                    }
                    r = e;
                }
            }
            most = std::max(most, (int)ext.size() - ext_off[t]);
        }
        ext_off[n_tiles] = (int)ext.size();
        off_ext_off = b.alloc(ext_off.size());
        std::memcpy(b.blk.data() + off_ext_off, ext_off.data(), ext_off.size() * 4);
        off_ext = b.alloc((ext.size() + kExtBatch) * 4);  // padded: a kernel reads whole batches
        if (!ext.empty()) std::memcpy(b.blk.data() + off_ext, ext.data(), ext.size() * sizeof(ExtStep));
        if (n_ext) *n_ext = (int)ext.size();
        if (max_per_tile) *max_per_tile = most;
    };
    L.bm = bm;
    build_ext(bm, L.n_tiles_m, L.off_ext_off, L.off_ext, &L.n_ext, &L.max_ext_per_tile, L.ext_adapter);
    L.ext_adapter_half.clear();
    if (bm == 256) build_ext(128, L.n_tiles_m_half, L.off_ext_off_half, L.off_ext_half, nullptr, nullptr, L.ext_adapter_half);
}

}  // namespace

int build_plan(const PlanRequest &rq, std::vector<int32_t> &blk, PlanLayout &L)
{
    const collm_shape *s = rq.shape;
    const int T = s->n_tokens, N = s->n_adapters;
    blk.clear();
    blk.reserve((size_t)T * 8 + 4096);
    Builder b(blk);
    L = PlanLayout();
    L.n_tokens = T;
    L.n_segments = s->n_segments;
    L.n_adapters = N;
    int rmax = 1;
    for (int a = 0; a < N; ++a) rmax = std::max(rmax, rq.rank[a]);
    L.rpad = round_up(rmax, kKStep);

    L.off_tok_segment = b.alloc(std::max(T, 1));
    L.off_tok_adapter = b.alloc(std::max(T, 1));
    L.off_tok_train = b.alloc(std::max(T, 1));
    {
        std::vector<uint8_t> tr((size_t)std::max(T, 1));
        token_map(s, rq.seg_start, rq.seg_adapter, rq.seg_is_train, blk.data() + L.off_tok_segment,
                  blk.data() + L.off_tok_adapter, tr.data());
        for (int t = 0; t < T; ++t) blk[L.off_tok_train + t] = tr[t];
    }
    L.off_rank = b.alloc(std::max(N, 1));
    for (int a = 0; a < N; ++a) blk[L.off_rank + a] = rq.rank[a];
    L.off_A_ptr = b.alloc((size_t)std::max(N, 1) * 2);
    L.off_B_ptr = b.alloc((size_t)std::max(N, 1) * 2);
    L.off_dA_ptr = b.alloc((size_t)std::max(N, 1) * 2);
    L.off_dB_ptr = b.alloc((size_t)std::max(N, 1) * 2);
    auto put_ptrs = [&](int32_t off, const void *const *p) {
        if (!p) return;
        for (int a = 0; a < N; ++a) {
            const uint64_t v = (uint64_t)(uintptr_t)p[a];
            std::memcpy(blk.data() + off + 2 * a, &v, 8);
        }
    };
    put_ptrs(L.off_A_ptr, rq.A);
    put_ptrs(L.off_B_ptr, rq.B);
    put_ptrs(L.off_dA_ptr, (const void *const *)rq.dA);
    put_ptrs(L.off_dB_ptr, (const void *const *)rq.dB);

    std::vector<int32_t> all((size_t)T), train;
    for (int t = 0; t < T; ++t) all[t] = t;
    train.reserve(T);
    for (int t = 0; t < T; ++t)
        if (blk[L.off_tok_train + t]) train.push_back(t);

    // the vector may reallocate inside build_row_order: always index through blk.data()
    {
        std::vector<int32_t> tok_adapter(blk.begin() + L.off_tok_adapter,
                                         blk.begin() + L.off_tok_adapter + T);
        build_row_order(b, L.all, all, tok_adapter.data(), rq.rank, N, rq.bm_all, rq.B, rq.max_row_tiles, L.rpad, rq.wide_min_rows_all,
                        rq.rank_ext_all ? rq.rank_ext_all : rq.rank, true);
        build_row_order(b, L.train, train, tok_adapter.data(), rq.rank, N, rq.bm_train, rq.A, rq.max_row_tiles, L.rpad, rq.wide_min_rows_train,
                        rq.rank, false);
    }

    // gradient items: one per trained adapter, rows contiguous in the training row order
    std::vector<GradItem> grad;
    {
        const int32_t *row_ad = blk.data() + L.train.off_row_adapter;
        int r = 0;
        while (r < L.train.n_rows) {
            const int a = row_ad[r];
            int e = r + 1;
            while (e < L.train.n_rows && row_ad[e] == a) ++e;
            GradItem g{};
            g.adapter = a;
            g.row_lo = r;
            g.row_hi = e;
            g.rank = rq.rank[a];
            grad.push_back(g);
            L.max_grad_rows = std::max(L.max_grad_rows, e - r);
            r = e;
        }
    }
    L.n_grad = (int)grad.size();
    L.off_grad = b.alloc(grad.size() * 4 + 4);
    if (!grad.empty()) std::memcpy(blk.data() + L.off_grad, grad.data(), grad.size() * sizeof(GradItem));
    b.alloc(0, 64);
    L.total_ints = (int32_t)blk.size();
    return COLLM_OK;
}

size_t plan_ints_upper_bound(int max_tokens, int max_segments, int max_adapters, int max_rank)
{
    (void)max_segments;
    const size_t Tp = (size_t)round_up(std::max(max_tokens, 1), kRowPad);
    const size_t N = (size_t)std::max(max_adapters, 1);
    const size_t steps = (size_t)round_up(max_rank, kKStep) / kKStep;
    size_t n = 0;
    n += 3 * Tp;                         // token map
    n += 9 * N + 64;                     // rank + four pointer tables
    for (int k = 0; k < 2; ++k) {
        n += 2 * Tp;                     // row_tok, row_adapter
        n += 4 * (Tp / kSkinnyRows + N) + 8;          // skinny items
        n += 4 * (Tp / 8 + N) + 8;                    // items of the tiled pass (runs of 8 rows at least)
        n += 2 * (Tp / 64 + 8);          // ext_off (smallest tile 64 rows), two tile sizes
        n += 2 * (4 * steps * (Tp / 64 + N) + 4 * kExtBatch + 8);  // ext steps: (tiles + adapter runs) x steps, two tile sizes
    }
    n += 4 * N + 8;                      // grad items
    return n + 1024;
}

}  // namespace collm
