// Host-only driver for a sanitizer build of the planner (tests/test_host_abi.py compiles it together with
// csrc/planner.cpp under -fsanitize=address,undefined and runs it): random batches through build_plan with every
// option, each plan checked against what the segment table fixes.  Prints "planner ok <cases>" and returns 0.
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <random>
#include <vector>

#include "planner.h"

using namespace collm;

#define REQUIRE(cond)                                                                      \
    do {                                                                                   \
        if (!(cond)) {                                                                     \
            std::fprintf(stderr, "case %d: check failed: %s (line %d)\n", g_case, #cond, __LINE__); \
            std::exit(1);                                                                  \
        }                                                                                  \
    } while (0)
static int g_case = 0;

static void check_order(const std::vector<int32_t> &plan, const RowOrderLayout &R, const std::vector<int32_t> &want_tokens,
                        const std::vector<int32_t> &tok_adapter, const std::vector<int32_t> &rank,
                        const std::vector<int32_t> &rank_ext, int n_tokens, bool one_run_per_adapter)
{
    REQUIRE(R.n_rows == (int)want_tokens.size());
    REQUIRE(R.n_rows_pad % kRowPad == 0 && R.n_rows_pad >= R.n_rows && R.n_rows_pad >= kRowPad);
    std::vector<int> seen((size_t)n_tokens + 1, 0);
    std::vector<int32_t> last_tok(rank.size() + 1, -1);
    std::vector<int> runs(rank.size() + 1, 0);
    int prev_ad = -2;
    for (int r = 0; r < R.n_rows_pad; ++r) {
        const int tok = plan[R.off_row_tok + r], ad = plan[R.off_row_adapter + r];
        if (r >= R.n_rows) {
            REQUIRE(tok == -1 && ad == -1);
            continue;
        }
        REQUIRE(tok >= 0 && tok < n_tokens && !seen[tok]);
        seen[tok] = 1;
        REQUIRE(ad == tok_adapter[tok]);
        REQUIRE(tok > last_tok[ad + 1]);  // ascending token order inside an adapter
        last_tok[ad + 1] = tok;
        if (ad != prev_ad) ++runs[ad + 1];
        prev_ad = ad;
    }
    for (int tok : want_tokens) REQUIRE(seen[tok]);
    if (one_run_per_adapter)
        for (size_t a = 0; a < runs.size(); ++a) REQUIRE(runs[a] <= 1);
    // items: every row with an adapter belongs to exactly one item (skinny or tiled), inside one run
    std::vector<int> covered((size_t)R.n_rows_pad, 0);
    auto items = [&](int32_t off, int n, int max_rows) {
        for (int i = 0; i < n; ++i) {
            SkinnyItem it;
            std::memcpy(&it, plan.data() + off + 4 * i, sizeof it);
            REQUIRE(it.n_rows >= 1 && it.n_rows <= max_rows && it.row_lo >= 0 && it.row_lo + it.n_rows <= R.n_rows);
            REQUIRE(it.adapter >= 0 && it.adapter < (int)rank.size() && it.rank == rank[it.adapter]);
            for (int r = it.row_lo; r < it.row_lo + it.n_rows; ++r) {
                REQUIRE(plan[R.off_row_adapter + r] == it.adapter);
                ++covered[r];
            }
        }
    };
    items(R.off_items, R.n_items, R.item_rows);
    items(R.off_wide, R.n_wide, kWideRows);
    for (int r = 0; r < R.n_rows; ++r) REQUIRE(covered[r] == (plan[R.off_row_adapter + r] >= 0 ? 1 : 0));
    // extension steps: per tile, every (row, rank index) of a row with an adapter is covered exactly once
    auto ext = [&](int tile_rows, int n_tiles, int32_t off_ext_off, int32_t off_ext) {
        REQUIRE(n_tiles == R.n_rows_pad / tile_rows);
        for (int t = 0; t < n_tiles; ++t) {
            const int e0 = plan[off_ext_off + t], e1 = plan[off_ext_off + t + 1];
            REQUIRE(e0 <= e1);
            std::vector<int> hit((size_t)tile_rows * (kMaxRank / kKStep), 0);
            int group = 0;
            for (int e = e0; e < e1; ++e) {
                ExtStep s;
                std::memcpy(&s, plan.data() + off_ext + 4 * e, sizeof s);
                const int koff = (int)(s.koff_rank & 0xffffu), rk = (int)(s.koff_rank >> 16);
                const int lo = (int)(s.rows & 0xffffu), hi = (int)(s.rows >> 16);
                if (rk == 0) {  // an empty step that fills a group up to whole batches
                    REQUIRE(s.rows == 0 && s.tab == 0);
                    continue;
                }
                REQUIRE(koff % kKStep == 0 && koff < rk && lo < hi && hi <= tile_rows);
                REQUIRE(koff / kExtGroup >= group);
                if (koff / kExtGroup > group) {
                    REQUIRE((e - e0) % kExtBatch == 0);  // a batch lies inside one group
                    group = koff / kExtGroup;
                }
                for (int r = lo; r < hi; ++r) {
                    const int ad = plan[R.off_row_adapter + t * tile_rows + r];
                    REQUIRE(ad >= 0 && rank_ext[ad] == rk);
                    ++hit[(size_t)r * (kMaxRank / kKStep) + koff / kKStep];
                }
            }
            for (int r = 0; r < tile_rows; ++r) {
                const int row = t * tile_rows + r;
                const int ad = row < R.n_rows ? plan[R.off_row_adapter + row] : -1;
                for (int k = 0; k < kMaxRank / kKStep; ++k)
                    REQUIRE(hit[(size_t)r * (kMaxRank / kKStep) + k] == ((ad >= 0 && k * kKStep < rank_ext[ad]) ? 1 : 0));
            }
        }
    };
    ext(R.bm, R.n_tiles_m, R.off_ext_off, R.off_ext);
    if (R.bm == 256) ext(128, R.n_tiles_m_half, R.off_ext_off_half, R.off_ext_half);
}

int main(int argc, char **argv)
{
    const int n_cases = argc > 1 ? std::atoi(argv[1]) : 10000;
    std::mt19937 rng(20260416u);
    auto uni = [&](int lo, int hi) { return (int)(rng() % (uint32_t)(hi - lo + 1)) + lo; };
    std::vector<int32_t> plan;
    for (g_case = 0; g_case < n_cases; ++g_case) {
        const int N = uni(0, 12), S = uni(0, 40);
        std::vector<int32_t> rank((size_t)N), rank_ext;
        for (int a = 0; a < N; ++a) rank[a] = uni(0, 3) ? uni(1, 32) * 8 : uni(1, 256);
        std::vector<int32_t> seg_start(1, 0), seg_adapter, tok_adapter, tok_seg;
        std::vector<uint8_t> seg_train, tok_train;
        for (int k = 0; k < S; ++k) {
            const int kind = uni(0, 9);
            const int len = kind == 0 ? 0 : (kind < 6 ? 1 : (kind < 9 ? uni(2, 60) : uni(60, 700)));
            const int ad = (N == 0 || uni(0, 9) == 0) ? -1 : uni(0, N - 1);
            const int tr = ad >= 0 && uni(0, 2) == 0;
            seg_start.push_back(seg_start.back() + len);
            seg_adapter.push_back(ad);
            seg_train.push_back((uint8_t)tr);
            for (int i = 0; i < len; ++i) {
                tok_adapter.push_back(ad);
                tok_seg.push_back(k);
                tok_train.push_back((uint8_t)tr);
            }
        }
        const int T = seg_start.back();
        collm_shape sh{};
        sh.d_in = 64;
        sh.d_out = 128;
        sh.n_tokens = T;
        sh.n_segments = S;
        sh.n_adapters = N;
        sh.dtype = COLLM_BF16;
        REQUIRE(validate_batch(&sh, rank.data(), seg_start.data(), seg_adapter.data(), seg_train.data(), kMaxRank) == COLLM_OK);
        // the host token map against the definition
        std::vector<int32_t> ts((size_t)T + 1, -9), ta((size_t)T + 1, -9);
        std::vector<uint8_t> tt((size_t)T + 1, 9);
        token_map(&sh, seg_start.data(), seg_adapter.data(), seg_train.data(), ts.data(), ta.data(), tt.data());
        for (int t = 0; t < T; ++t) REQUIRE(ts[t] == tok_seg[t] && ta[t] == tok_adapter[t] && tt[t] == tok_train[t]);
        REQUIRE(ts[T] == -9 && ta[T] == -9 && tt[T] == 9);

        PlanRequest rq;
        rq.shape = &sh;
        rq.rank = rank.data();
        const bool siblings = N > 0 && uni(0, 5) == 0;  // extension steps over other ranks than the items' (sibling calls)
        rank_ext = rank;
        if (siblings) {
            bool halves = true;
            for (int a = 0; a < N; ++a) halves = halves && rank[a] % 16 == 0;
            if (halves) {
                for (int a = 0; a < N; ++a) rank_ext[a] = rank[a] / 2;
                rq.rank_ext_all = rank_ext.data();
            }
        }
        rq.seg_start = seg_start.data();
        rq.seg_adapter = seg_adapter.data();
        rq.seg_is_train = seg_train.data();
        const int tiles[3] = {64, 128, 256};
        rq.bm_all = tiles[uni(0, 2)];
        rq.bm_train = tiles[uni(0, 2)];
        rq.max_row_tiles = uni(1, 2);
        rq.wide_min_rows_all = uni(0, 2) ? 0 : uni(1, 200);
        rq.wide_min_rows_train = uni(0, 2) ? 0 : uni(1, 200);
        PlanLayout L;
        REQUIRE(build_plan(rq, plan, L) == COLLM_OK);
        REQUIRE(L.total_ints == (int)plan.size() && L.total_ints % 64 == 0);
        REQUIRE((size_t)L.total_ints <= plan_ints_upper_bound(std::max(T, 1), std::max(S, 1), N, kMaxRank));
        for (int t = 0; t < T; ++t)
            REQUIRE(plan[L.off_tok_segment + t] == tok_seg[t] && plan[L.off_tok_adapter + t] == tok_adapter[t] &&
                    plan[L.off_tok_train + t] == tok_train[t]);
        for (int a = 0; a < N; ++a) REQUIRE(plan[L.off_rank + a] == rank[a]);
        std::vector<int32_t> all, train;
        for (int t = 0; t < T; ++t) {
            all.push_back(t);
            if (tok_train[t]) train.push_back(t);
        }
        check_order(plan, L.all, all, tok_adapter, rank, rq.rank_ext_all ? rank_ext : rank, T, false);
        check_order(plan, L.train, train, tok_adapter, rank, rank, T, true);
        // gradient items: one per trained adapter, its run of the training order
        std::vector<int> trained((size_t)N + 1, 0);
        for (int i = 0; i < L.n_grad; ++i) {
            GradItem g;
            std::memcpy(&g, plan.data() + L.off_grad + 4 * i, sizeof g);
            REQUIRE(g.adapter >= 0 && g.adapter < N && !trained[g.adapter] && g.rank == rank[g.adapter]);
            trained[g.adapter] = 1;
            REQUIRE(g.row_lo >= 0 && g.row_lo < g.row_hi && g.row_hi <= L.train.n_rows);
            for (int r = g.row_lo; r < g.row_hi; ++r) REQUIRE(plan[L.train.off_row_adapter + r] == g.adapter);
            REQUIRE(g.row_lo == 0 || plan[L.train.off_row_adapter + g.row_lo - 1] != g.adapter);
            REQUIRE(g.row_hi == L.train.n_rows || plan[L.train.off_row_adapter + g.row_hi] != g.adapter);
        }
        for (int t = 0; t < T; ++t)
            if (tok_train[t]) REQUIRE(trained[tok_adapter[t]]);
    }
    std::printf("planner ok %d\n", n_cases);
    return 0;
}
