"""GPU parity: the C-ABI library against the fp64 CPU oracle on the same seeded inputs.

Tolerances (max|got - ref| / max|ref| per output tensor): 1e-2 for bf16 inputs with fp32
accumulation, 1e-5 for fp32.  Index work (token -> segment / adapter) is compared bit for bit.
"""
import numpy as np
import pytest

import oracle
from paper_2604_16400_amd import binding
from paper_2604_16400_amd import workloads as wl

from gpu_util import TOL, DeviceLayer, check_full, make_ctx, maxrel, to_dev, to_host

pytestmark = pytest.mark.gpu


def _run_full(w, tol=None, h_save=True, transposed=False, wide_min_rows=None, gemm_split=None, dual_pass=None, **kw):
    t = wl.make_tensors(w)
    ctx = make_ctx(w, **kw)
    if dual_pass is not None:
        ctx.set_dual_pass(dual_pass)
    if wide_min_rows is not None:
        ctx.set_wide_pass(wide_min_rows)
    if gemm_split is not None:
        ctx.set_gemm_split(gemm_split)
    layer = DeviceLayer(w, t, ctx, transposed=transposed)
    layer.fwd(h_save=h_save)
    layer.bwd(h_save=h_save)
    errs = check_full(layer, TOL[w.dtype] if tol is None else tol, check_h=h_save)
    # the plan the device holds encodes exactly the oracle's token map
    ts, ta, tt = ctx.device_token_map(w.n_tokens)
    rs, ra, rt = oracle.token_map(w.seg_start, w.seg_adapter, w.seg_is_train)
    assert np.array_equal(ts, rs) and np.array_equal(ta, ra) and np.array_equal(tt, rt)
    ctx.close()
    return errs


# ------------------------------------------------------------------ the five configurations
def test_config1_fp32_every_element():
    errs = _run_full(wl.make_config(1))
    print("config 1 errors", errs)


def test_config2_bf16_every_element():
    errs = _run_full(wl.make_config(2))
    print("config 2 errors", errs)
    # one bf16 rounding of the output is ~2^-9 of the row scale; anything near 1e-2 is a bug
    assert errs["y"] < 6e-3 and errs["dx"] < 6e-3


def _sampled_projection(cfg, proj_index, max_rows=None):
    """Full-size run in the launch configuration the benchmark times.  The two W-sized
    contractions are checked on the row sample (first, last and two interior tokens of every
    segment plus every token of the shortest training segment), all columns: the oracle computes
    exactly those rows from its definition.  h, dA and dB are checked on every element."""
    import torch

    w = wl.make_config(cfg)
    p = w.projections[proj_index]
    t = wl.make_tensors(w, proj_index)
    ctx = make_ctx(w)
    layer = DeviceLayer(w, t, ctx, proj_index)
    layer.fwd()
    layer.bwd()
    torch.cuda.synchronize()
    tol = TOL[w.dtype]
    ta, tt = layer.tok_adapter, layer.tok_train
    rows = wl.sample_rows(w, seed=proj_index)
    if max_rows is not None and len(rows) > max_rows:
        # cap the rows, never the columns: keep every segment's first token, thin out the rest evenly
        firsts = np.intersect1d(rows, w.seg_start[:-1])
        rest = np.setdiff1d(rows, firsts)
        keep = max(0, max_rows - len(firsts))
        rest = rest[np.linspace(0, len(rest) - 1, keep).astype(np.int64)] if keep else rest[:0]
        rows = np.union1d(firsts, rest)

    # forward: y[rows, :]
    y_ref, h_rows = oracle.lora_linear_fwd(t.x[rows], t.W, t.A, t.B, ta[rows], w.scale)
    y = to_host(layer.y)
    assert np.all(np.isfinite(y))
    e_y = maxrel(y[rows], y_ref)
    # backward: dx[training rows of the sample, :]
    trs = rows[tt[rows] != 0]
    dx_ref, _, _ = oracle.lora_linear_bwd(t.x[trs], t.W, t.A, t.B, ta[trs], np.ones(len(trs), np.uint8), w.scale,
                                          t.dy[trs], want_dab=False)
    dx = to_host(layer.dx)
    assert np.all(np.isnan(dx[tt == 0])) and np.all(np.isfinite(dx[tt != 0]))
    e_dx = maxrel(dx[trs], dx_ref)
    # low-rank terms in full
    _, dA_ref, dB_ref = oracle.lora_linear_bwd(t.x, None, t.A, t.B, ta, tt, w.scale, t.dy, want_dx=False)
    errs = {"y": e_y, "dx": e_dx}
    for a in range(w.n_adapters):
        dA, dB = to_host(layer.dA[a]), to_host(layer.dB[a])
        if dA_ref[a] is None:
            assert np.all(np.isnan(dA)) and np.all(np.isnan(dB))
        else:
            errs[f"dA{a}"] = maxrel(dA, dA_ref[a])
            errs[f"dB{a}"] = maxrel(dB, dB_ref[a])
    hs = to_host(layer.h_save)
    tr = tt != 0
    assert np.all(np.isnan(hs[~tr]))
    # h of every training token, from the oracle's forward pass on those rows against a weight of one column
    # (h does not depend on W)
    tr_tok = np.flatnonzero(tr)
    _, h_tr = oracle.lora_linear_fwd(t.x[tr_tok], t.W[:, :1], t.A, [b[:, :1] for b in t.B], ta[tr_tok], w.scale)
    h_ref = np.zeros((len(tr_tok), hs.shape[1]))
    for k, tok in enumerate(tr_tok):
        h_ref[k, : w.ranks[ta[tok]]] = h_tr[k, : w.ranks[ta[tok]]]
    errs["h"] = maxrel(hs[tr], h_ref)
    for tok in tr_tok[:: max(1, len(tr_tok) // 256)]:
        assert np.all(hs[tok, w.ranks[ta[tok]]:] == 0.0)
    ts, ta_d, tt_d = ctx.device_token_map(w.n_tokens)
    rs, ra, rt = oracle.token_map(w.seg_start, w.seg_adapter, w.seg_is_train)
    assert np.array_equal(ts, rs) and np.array_equal(ta_d, ra) and np.array_equal(tt_d, rt)
    ctx.close()
    print(f"config {cfg} {p.name}: {len(rows)} rows ({len(trs)} training) x all {p.d_out}/{p.d_in} columns, errors",
          {k: float("%.3g" % v) for k, v in errs.items() if k in ("y", "dx", "h")},
          "max dA/dB", max([v for k, v in errs.items() if k[0] == "d" and k != "dx"], default=0.0))
    bad = {k: v for k, v in errs.items() if not v <= tol}
    assert not bad, bad
    return errs


@pytest.mark.parametrize("proj", [0, 1, 2])
def test_config3_sampled(proj):
    _sampled_projection(3, proj)


@pytest.mark.parametrize("proj", [0, 1])
def test_config4_sampled(proj):
    _sampled_projection(4, proj)


@pytest.mark.parametrize("proj", [0, 1, 2])
def test_config5_sampled(proj):
    _sampled_projection(5, proj)


# ------------------------------------------------------------------ edge cases
def _adhoc(dtype, d_in, d_out, ranks, lens, adapters, train, scale=2.0, seed=7):
    return wl.make_adhoc("adhoc", dtype, d_in, d_out, ranks, lens, adapters, train, scale=scale, seed=seed)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_ragged_shapes_odd_ranks_empty_segments(dtype):
    # sizes that are no multiple of any tile, ranks that are no multiple of 8, empty segments,
    # base-only segments, two training segments on one adapter, an adapter used by both kinds
    q = 8 if dtype == "bf16" else 4
    w = _adhoc(dtype, 25 * q, 41 * q, [3, 5, 17, 8, 1, 24], [5, 0, 37, 1, 130, 0, 70, 2, 64, 301],
               [0, 1, -1, 2, 2, 3, 5, -1, 4, 2], [0, 0, 0, 0, 1, 0, 1, 0, 0, 1], scale=0.3)
    _run_full(w)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_shuffled_segment_order(dtype):
    w = _adhoc(dtype, 256, 192, [16, 8, 32], [40, 1, 1, 1, 90, 33, 1, 260], [0, 1, 2, 0, 1, 2, 1, 0],
               [0, 0, 0, 0, 1, 0, 0, 1])
    ws, _ = wl.shuffled_segments(w, seed=3)
    _run_full(ws)


def test_all_inference_batch_and_all_training_batch():
    w = _adhoc("bf16", 128, 256, [16, 16], [10, 20, 30], [0, 1, -1], [0, 0, 0])
    t = wl.make_tensors(w)
    ctx = make_ctx(w)
    layer = DeviceLayer(w, t, ctx)
    layer.fwd()
    layer.bwd()  # nothing trains: a no-op that must leave every output untouched
    check_full(layer, TOL["bf16"])
    ctx.close()
    w = _adhoc("bf16", 128, 256, [16, 16], [100, 200], [1, 0], [1, 1])
    _run_full(w)


def test_single_token_and_empty_batch():
    _run_full(_adhoc("bf16", 64, 64, [8], [1], [0], [1]))
    _run_full(_adhoc("f32", 64, 64, [8], [1], [0], [0]))
    w = _adhoc("bf16", 64, 64, [8], [0, 0], [0, -1], [0, 0])
    t = wl.make_tensors(w)
    ctx = make_ctx(w)
    layer = DeviceLayer(w, t, ctx)
    layer.fwd()
    layer.bwd()
    ctx.close()


def test_many_adapters_in_one_tile_and_large_rank():
    # 300 one-token decode segments over 40 adapters (many adapters per GEMM row tile), ranks
    # up to the largest supported (256), plus training segments
    rng = np.random.default_rng(1)
    ranks = rng.choice([8, 16, 64, 256], size=40)
    lens = [1] * 300 + [150, 90]
    ads = list(rng.integers(0, 40, size=300)) + [3, 17]
    w = _adhoc("bf16", 512, 384, ranks, lens, ads, [0] * 300 + [1, 1])
    _run_full(w)


def test_few_rows_long_contraction_and_many_trained_adapters_in_one_tile():
    # 20 training rows against an 8192-long contraction: the rank-wide passes cut K into many slices
    # across blocks (partial sums added by the second kernel); the dh pass (K = 64) uses a single one
    _run_full(_adhoc("bf16", 8192, 64, [16, 8], [20, 3], [0, 1], [1, 0]))
    _run_full(_adhoc("bf16", 64, 8192, [16, 8], [20, 3], [0, 1], [1, 0]))
    # six trained adapters inside one GEMM row tile, ranks that are and are not multiples of 8: several
    # batches of extension steps in the dX GEMM, some loaded element by element and some directly
    w = _adhoc("bf16", 320, 192, [3, 16, 40, 16, 9, 64], [30, 20, 25, 35, 10, 40, 12], [0, 1, 2, 3, 4, 5, -1],
               [1, 1, 1, 1, 1, 1, 0], scale=0.3)
    _run_full(w)


@pytest.mark.parametrize("wide_side", ["d_out", "d_in", "d_out_long_k"])
def test_rows_split_between_large_and_small_tiles(wide_side):
    # 2300 rows x 7424 columns is 9 x 29 tiles of 256x256, five more than one round over 256 CUs: the
    # first 8 row tiles run as 256x256, rows 2048.. as 128x128 tiles in a second launch.  Segments and
    # adapters (one with a rank that is no multiple of 8) straddle row 2048 and row 2176; every element
    # is compared.  d_out wide: the forward GEMM is the split one; d_in wide: the dX GEMM.
    lens = [700, 1, 1, 500, 300, 1, 600, 197]
    ads = [0, 1, 2, 1, -1, 0, 2, 3]
    if wide_side == "d_out_long_k":
        # K = 1024: the small tiles of the last rows also cut K into slices (second kernel adds them)
        w = _adhoc("bf16", 1024, 7424, [16, 8, 12, 32], lens, ads, [1, 0, 0, 1, 0, 0, 1, 0], scale=0.5)
    elif wide_side == "d_out":
        w = _adhoc("bf16", 64, 7424, [16, 8, 12, 32], lens, ads, [1, 0, 0, 1, 0, 0, 1, 0], scale=0.5)
    else:
        lens[4], lens[6], lens[7] = 30, 800, 297   # 2300 training rows beside 30 base-only ones
        w = _adhoc("bf16", 7424, 64, [16, 8, 12, 32], lens, ads, [1, 1, 1, 1, 0, 1, 1, 1], scale=0.5)
    _run_full(w)


@pytest.mark.parametrize("wide_side", ["d_out", "d_in"])
def test_columns_split_between_large_and_small_tiles(wide_side):
    # 5000 rows x 7000 columns is 20 x 28 tiles of 256x256, 48 more than two rounds over 256 CUs: the first 25
    # tile columns run as 256x256 tiles, columns 6400.. of all rows as 128x128 tiles in a second launch (five
    # tile columns, the last 88 columns wide; the last row tile 8 rows high).  Adapters with ranks that are and
    # are not multiples of 8, one above 64 (two groups of extension steps); every element is compared.
    assert binding.host_tiling(5000, 7000, 64) == (binding.TILE_256x256, 20, 0, 3)
    lens = [1500, 1, 1, 1100, 400, 1, 1300, 697]
    ads = [0, 1, 2, 1, -1, 0, 2, 3]
    if wide_side == "d_out":
        w = _adhoc("bf16", 64, 7000, [16, 8, 12, 72], lens, ads, [1, 0, 0, 1, 0, 0, 1, 0], scale=0.5)
    else:
        lens[4], lens[7] = 30, 1097    # 5000 training rows beside 30 base-only ones
        w = _adhoc("bf16", 7000, 64, [16, 8, 12, 72], lens, ads, [1, 1, 1, 1, 0, 1, 1, 1], scale=0.5)
    _run_full(w)


@pytest.mark.parametrize("transposed", [False, True])
def test_gemm_with_few_rows_cut_into_k_slices(transposed):
    # decode-sized batches: the library cuts K of both GEMMs into slices by itself (forward: 37 rows against
    # K = 2048; dX: 21 training rows against K = 1536), partial sums added by the second kernel before the one rounding
    lens = [1] * 16 + [9, 12]
    ads = list(np.arange(16) % 3) + [1, 2]
    w = _adhoc("bf16", 2048, 1536, [16, 8, 24], lens, ads, [0] * 16 + [1, 1], scale=0.5)
    _run_full(w, transposed=transposed)
    _run_full(w, transposed=transposed, gemm_split=1)      # and the same batch without slices
    # forced: 3 slices of a K that is no multiple of 3 x 64, ragged everything, rows of several adapters and
    # base-only rows in one tile, more than one row tile
    w = _adhoc("bf16", 328, 200, [16, 5, 40], [60, 1, 130, 0, 70, 2, 64], [0, 1, 2, 2, -1, 1, 0], [1, 0, 1, 0, 0, 0, 1],
               scale=0.3)
    _run_full(w, transposed=transposed, gemm_split=3)
    _run_full(w, transposed=transposed, gemm_split=64)     # clamped to one K tile per slice
    _run_full(_adhoc("bf16", 8192, 64, [16], [1], [0], [0]), transposed=transposed)   # one token


@pytest.mark.parametrize("transposed", [False, True])
def test_rank_wide_passes_as_row_tiles(transposed):
    # Runs of at least 8 rows of an adapter whose rank is a multiple of 8 go through the tiled pass (128-row
    # items, K cut into slices, partial sums added by the second kernel); the other rows stay on the 16-row
    # items.  Ragged everything: K = 200 and 328 (no multiple of 64), ranks 8..136 and two that are no
    # multiple of 8, runs of 8, 129, 300 and 7 rows, an adapter shared by a decode token and a training run.
    lens = [300, 1, 129, 7, 8, 40, 1, 1, 260, 33]
    ads = [0, 0, 1, 2, 2, 3, 4, -1, 5, 6]
    trn = [1, 0, 1, 0, 1, 0, 0, 0, 1, 1]
    w = _adhoc("bf16", 200, 328, [64, 136, 8, 12, 16, 40, 3], lens, ads, trn, scale=0.3)
    _run_full(w, transposed=transposed, wide_min_rows=8)
    _run_full(w, transposed=transposed, wide_min_rows=8, h_save=False)
    # many slices: 40 rows against K = 8192, both directions
    _run_full(_adhoc("bf16", 8192, 64, [64, 16], [40, 3], [0, 1], [1, 0]), transposed=transposed, wide_min_rows=8)
    _run_full(_adhoc("bf16", 64, 8192, [64, 16], [40, 3], [0, 1], [1, 0]), transposed=transposed, wide_min_rows=8)
    # the choice the library makes by itself (ranks from 49 up) against the same batch with the pass off
    w = _adhoc("bf16", 512, 384, [64, 128, 256, 56], [200, 1, 1, 90, 150, 31, 500], [0, 1, 2, 3, 1, 2, 2],
               [1, 0, 0, 0, 1, 0, 1])
    _run_full(w, transposed=transposed)
    _run_full(w, transposed=transposed, wide_min_rows=0)


def test_two_contexts_on_two_streams_interleaved():
    # Two contexts with different batches, each on a stream of its own, called alternately without waiting in
    # between (forward A, forward B, backward A, backward B, twice): a context's plan, workspace and gradient
    # stream are its own, and nothing in the library is shared between them but read-only code.
    import torch

    wa = _adhoc("bf16", 512, 384, [16, 64, 8], [300, 1, 1, 90, 150, 31], [0, 1, 2, 1, -1, 0], [1, 0, 0, 1, 0, 0], scale=0.3)
    wb = _adhoc("bf16", 256, 640, [32, 128], [40, 200, 7, 260], [1, 0, -1, 1], [0, 1, 0, 1], scale=0.3, seed=11)
    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
    ca, cb = make_ctx(wa), make_ctx(wb)
    la, lb = DeviceLayer(wa, wl.make_tensors(wa), ca), DeviceLayer(wb, wl.make_tensors(wb), cb, transposed=True)
    torch.cuda.synchronize()

    def call(layer, stream, fwd):
        w = layer.w
        if fwd:
            layer.ctx.collm_lora_linear_fwd(layer.x, layer.W, layer.A, layer.B, w.ranks, w.seg_start, w.seg_adapter,
                                            w.seg_is_train, w.scale, layer.y, layer.h_save, stream=stream,
                                            layout=layer.layout)
        else:
            layer.ctx.collm_lora_linear_bwd(layer.x, layer.W, layer.A, layer.B, w.ranks, w.seg_start, w.seg_adapter,
                                            w.seg_is_train, w.scale, layer.dy, layer.h_save, layer.dx, layer.dA, layer.dB,
                                            False, stream=stream, layout=layer.layout)

    for _ in range(2):
        call(la, sa, True)
        call(lb, sb, True)
        call(la, sa, False)
        call(lb, sb, False)
    torch.cuda.synchronize()
    check_full(la, TOL["bf16"])
    check_full(lb, TOL["bf16"])
    ca.close()
    cb.close()


@pytest.mark.parametrize("transposed", [False, True])
def test_many_extension_steps_in_one_row_tile(transposed):
    # Twelve adapters of ranks 128 and 256 with 20 rows each share one 256-row tile: 144 extension steps in four
    # groups of 64 rank indices, more than the 64 step records a kernel keeps in registers (the later batches come
    # through the scalar cache), the rows' operand loaded again for every group; forward (all rows) and backward
    # (the training rows of eight of the adapters), every tile shape.
    ranks = [128, 256] * 6
    lens = [20] * 12 + [9]
    ads = list(range(12)) + [-1]
    trn = [1, 1, 0, 1, 1, 0, 1, 1, 0, 1, 1, 0, 0]
    w = _adhoc("bf16", 256, 320, ranks, lens, ads, trn, scale=0.2)
    _, steps = binding.host_row_order(w.ranks, w.seg_start, w.seg_adapter, w.seg_is_train, 256)
    assert steps.max() >= 144
    for tile in (None, binding.TILE_256x256, binding.TILE_128x128):
        t = wl.make_tensors(w)
        ctx = make_ctx(w)
        if tile is not None:
            ctx.set_tiles(tile, tile)
        layer = DeviceLayer(w, t, ctx, transposed=transposed)
        layer.fwd(h_save=True)
        layer.bwd(h_save=True)
        check_full(layer, TOL[w.dtype])
        ctx.close()


@pytest.mark.parametrize("seed", range(12))
def test_random_batches_every_element(seed):
    # Seeded random batches through every path at once: ranks 1..256 (multiples of 8 or not, above 64: several
    # groups of extension steps), up to 40 adapters with skewed popularity, decode tokens, long and empty segments,
    # base-only segments, either layout, every tile shape, with and without h_save.  Every element is compared.
    rng = np.random.default_rng(1000 + seed)
    n_ad = int(rng.integers(1, 41))
    top = [16, 64, 128, 256][seed % 4]
    ranks = [int(rng.integers(1, top + 1)) if rng.random() < 0.4 else int(rng.integers(1, top // 8 + 1)) * 8 for _ in range(n_ad)]
    n_seg = int(rng.integers(1, 60))
    lens, ads, trn = [], [], []
    for _ in range(n_seg):
        kind = rng.random()
        lens.append(0 if kind < 0.05 else (1 if kind < 0.5 else int(rng.integers(2, 400 if kind > 0.9 else 60))))
        a = -1 if rng.random() < 0.1 else int(min(n_ad - 1, rng.zipf(1.5) - 1))
        ads.append(a)
        trn.append(int(a >= 0 and rng.random() < 0.4))
    if sum(lens) == 0:
        lens[0] = 5
    d_in, d_out = int(rng.integers(1, 80)) * 8, int(rng.integers(1, 80)) * 8
    w = _adhoc("bf16", d_in, d_out, ranks, lens, ads, trn, scale=0.3, seed=seed)
    tile = [None, binding.TILE_256x256, binding.TILE_128x128][seed % 3]
    t = wl.make_tensors(w)
    ctx = make_ctx(w)
    if tile is not None:
        ctx.set_tiles(tile, tile)
    layer = DeviceLayer(w, t, ctx, transposed=bool(seed % 2))
    layer.fwd(h_save=seed % 3 != 0)
    layer.bwd(h_save=seed % 3 != 0)
    check_full(layer, TOL[w.dtype], check_h=seed % 3 != 0)
    ctx.close()


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_transposed_weight_and_table_layout(dtype):
    # W [d_out, d_in], A [rank, d_in], B [d_out, rank], gradients likewise: the same mathematics, so the
    # oracle is fed the transposes back.  Ragged sizes, ranks that are and are not multiples of 8,
    # decode and training rows sharing tiles; then config 2 (bf16) in full.
    q = 8 if dtype == "bf16" else 4
    w = _adhoc(dtype, 25 * q, 41 * q, [3, 5, 17, 8, 1, 24], [5, 0, 37, 1, 130, 0, 70, 2, 64, 301],
               [0, 1, -1, 2, 2, 3, 5, -1, 4, 2], [0, 0, 0, 0, 1, 0, 1, 0, 0, 1], scale=0.3)
    _run_full(w, transposed=True)
    _run_full(w, transposed=True, h_save=False)
    w = _adhoc(dtype, 64 * q, 24 * q, [16, 64, 40], [1] * 40 + [300, 200, 150], list(np.arange(40) % 3) + [0, 1, 2],
               [0] * 40 + [1, 1, 0])
    _run_full(w, transposed=True)
    if dtype == "bf16":
        errs = _run_full(wl.make_config(2), transposed=True)
        assert errs["y"] < 6e-3 and errs["dx"] < 6e-3


@pytest.mark.parametrize("tile", [binding.TILE_256x256, binding.TILE_128x128])
@pytest.mark.parametrize("dims", [(64, 192), (320, 64), (192, 448), (136, 328)])
def test_odd_tile_counts_and_unpaired_extension_steps(tile, dims):
    # The GEMM tiles multiply two 16-wide extension steps per MFMA and walk K in tiles of 64: contractions of 1, 2, 3, 5
    # and 7 tiles (forward: d_in, backward: d_out), ranks of one, two and three steps (the last pair of a batch
    # half empty), ranks that are no multiple of 8, adapters that change inside a 16-row block, columns that end
    # inside a 16-column block; both layouts.  Every element is compared.
    d_in, d_out = dims
    lens = [5, 3, 9, 1, 1, 70, 130, 2, 40, 200, 7]
    ads = [0, 1, 2, 3, 0, 1, 2, -1, 3, 0, 2]
    trn = [0, 1, 0, 0, 0, 1, 1, 0, 1, 1, 0]
    w = _adhoc("bf16", d_in, d_out, [16, 40, 8, 20], lens, ads, trn, scale=0.4, seed=11)
    for transposed in (False, True):
        t = wl.make_tensors(w)
        ctx = make_ctx(w)
        ctx.set_tiles(tile, tile)
        layer = DeviceLayer(w, t, ctx, transposed=transposed)
        layer.fwd()
        layer.bwd()
        check_full(layer, TOL["bf16"])
        ctx.close()


@pytest.mark.parametrize("tile", [binding.TILE_256x256, binding.TILE_128x128])
def test_every_gemm_tile_shape(tile):
    w = _adhoc("bf16", 448, 584, [16, 32, 8], [1] * 50 + [300, 77, 200], list(np.arange(50) % 3) + [0, 1, 2],
               [0] * 50 + [1, 0, 1])
    t = wl.make_tensors(w)
    ctx = make_ctx(w)
    ctx.set_tiles(tile, tile)
    layer = DeviceLayer(w, t, ctx)
    layer.fwd()
    layer.bwd()
    check_full(layer, TOL["bf16"])
    ctx.close()


def test_same_batch_other_adapter_tables_reuses_the_plan():
    # Every layer and projection of a model sees the same batch with its own weight and adapter tables: the plan
    # on the device keeps its shape and only the table addresses inside it are replaced.  Two sets of tensors
    # (same segments, different values and buffers) through one context, calls interleaved; each checked in full.
    for shape in ((512, 384, [16, 64, 8], [40, 1, 1, 1, 300, 90, 33, 1, 260], [0, 1, 2, 0, 1, 1, 2, 1, 0],
                   [0, 0, 0, 0, 1, 1, 0, 0, 1]),
                  (64, 7424, [16, 8, 12, 32], [700, 1, 1, 500, 300, 1, 600, 197], [0, 1, 2, 1, -1, 0, 2, 3],
                   [1, 0, 0, 1, 0, 0, 1, 0])):
        d_in, d_out, ranks, lens, ads, trn = shape
        w1 = _adhoc("bf16", d_in, d_out, ranks, lens, ads, trn, scale=0.5, seed=7)
        w2 = _adhoc("bf16", d_in, d_out, ranks, lens, ads, trn, scale=0.5, seed=8)
        ctx = make_ctx(w1)
        l1 = DeviceLayer(w1, wl.make_tensors(w1), ctx)
        l2 = DeviceLayer(w2, wl.make_tensors(w2), ctx)
        l1.fwd()
        l2.fwd()
        l1.fwd()
        l2.bwd()
        l1.bwd()
        l2.fwd()
        check_full(l1, TOL["bf16"])
        check_full(l2, TOL["bf16"])
        ctx.close()


def test_weight_fetch_beside_the_rank_wide_passes():
    # A small weight is read once by extra blocks of the rank-wide pass that runs before each GEMM (the pass must
    # stream fewer bytes than the weight).  Those blocks compute nothing: results are as the oracle's, on the
    # 16-row items (rank 16), on the tiled pass (rank 64, long runs) and with both in one launch sequence; ragged
    # K so that the last share of the weight is a partial one.
    for ranks, lens, ads, trn in (([16, 16], [300, 40, 1, 171], [0, 1, 1, 0], [1, 0, 0, 0]),
                                  ([64, 64], [300, 40, 1, 171], [0, 1, 1, 0], [1, 0, 0, 1]),
                                  ([64, 16, 8], [260, 30, 1, 190, 31], [0, 1, 2, 0, 1], [1, 1, 0, 0, 0])):
        w = _adhoc("bf16", 1096, 2056, ranks, lens, ads, trn, scale=0.7)
        assert w.n_tokens * 1096 * 2 < 1096 * 2056 * 2  # the condition under which the weight is fetched
        _run_full(w)
        _run_full(w, transposed=True)
        _run_full(w, h_save=False)


def test_dh_and_dB_from_one_pass_over_dy():
    # Ranks up to 16: the backward call may take dh and dB from one pass over the training rows of dy (forced here,
    # since the library only chooses it for large dy).  Ragged everything: d_out no multiple of the 512-column groups
    # or of 64, ranks 16, 8, 12 and 5, adapters of 1, 33, 70, 600 and 1100 training rows (one piece, several pieces,
    # pieces that end inside a 32-row chunk), an adapter shared by inference and training segments, accumulate on and
    # off, h recomputed; each against the oracle, and the forced pass against the two separate passes.
    cases = [(264, 1096, [16, 8, 12, 5], [600, 1, 33, 9, 70, 1, 1100, 17], [0, 1, 1, 2, 3, 0, 2, 3], [1, 0, 1, 0, 1, 1, 1, 0]),
             (128, 2048, [16, 16], [512, 64, 5], [0, 1, 1], [1, 1, 0]),
             (64, 40, [16], [3, 200], [0, 0], [0, 1])]
    for d_in, d_out, ranks, lens, ads, trn in cases:
        w = _adhoc("bf16", d_in, d_out, ranks, lens, ads, trn, scale=0.6)
        for h_save in (True, False):
            e1 = _run_full(w, h_save=h_save, dual_pass=1)
            e0 = _run_full(w, h_save=h_save, dual_pass=0)
            assert set(e1) == set(e0)
    # gradient accumulation through the one-pass path (pieces summed by the second kernel, and the direct write)
    w = _adhoc("bf16", 128, 1032, [16, 8], [700, 40, 3], [0, 1, 1], [1, 1, 0])
    t = wl.make_tensors(w)
    ctx = make_ctx(w)
    ctx.set_dual_pass(1)
    layer = DeviceLayer(w, t, ctx)
    layer.fwd()
    layer.bwd()
    first = [to_host(g).copy() for g in layer.dB]
    layer.bwd(accumulate=True)
    for g, f in zip(layer.dB, first):
        assert maxrel(to_host(g), 2.0 * f) < 1e-6
    ctx.close()


def test_plan_statistics_and_device_info():
    info = binding.device_info(0)
    assert info["compute_units"] > 0 and info["clock_mhz"] > 0 and info["memory_bus_bits"] > 0
    w1 = _adhoc("bf16", 256, 128, [16, 8], [40, 1, 30, 9], [0, 1, 1, 0], [1, 0, 0, 0])
    w2 = _adhoc("bf16", 256, 128, [16, 8], [40, 1, 30, 9], [1, 0, 0, 1], [1, 0, 0, 0])
    ctx = make_ctx(w1)
    l1 = DeviceLayer(w1, wl.make_tensors(w1), ctx)
    l2 = DeviceLayer(w2, wl.make_tensors(w2), ctx)
    l1.fwd()
    st = ctx.plan_stats()
    assert st["mode"] == 1 and st["build_us"] > 0 and st["upload_us"] > 0 and st["bytes"] > 0   # built and uploaded
    l1.fwd()
    assert ctx.plan_stats()["mode"] == 0                                                          # reused as it is
    l2.fwd()
    assert ctx.plan_stats()["mode"] == 1                                                          # another batch
    l2.bwd()
    check_full(l2, TOL["bf16"])
    ctx.close()


# ------------------------------------------------------------------ contracts
def test_recompute_h_and_accumulate_and_run_to_run():
    import torch

    w = wl.make_config(2)
    t = wl.make_tensors(w)
    ctx = make_ctx(w)
    layer = DeviceLayer(w, t, ctx)
    layer.fwd()
    layer.bwd()
    torch.cuda.synchronize()
    y1, dx1 = layer.y.clone(), layer.dx.clone()
    dA1 = [a.clone() for a in layer.dA]
    dB1 = [b.clone() for b in layer.dB]
    # run to run: same bits (no floating-point atomics anywhere)
    layer.fwd()
    layer.bwd()
    torch.cuda.synchronize()
    eq = lambda a, b: torch.equal(a.view(torch.int16 if a.dtype == torch.bfloat16 else torch.int32),
                                  b.view(torch.int16 if b.dtype == torch.bfloat16 else torch.int32))
    assert eq(layer.y, y1) and eq(layer.dx, dx1)
    tr_ad = int(w.seg_adapter[-1])
    assert eq(layer.dA[tr_ad], dA1[tr_ad]) and eq(layer.dB[tr_ad], dB1[tr_ad])
    # h recomputed inside the backward call gives the same gradients as the saved one.  dA and dx do
    # not depend on h: same bits.  The recomputed h may be summed in another order than the saved one
    # (the pass over the training rows may cut K into a different number of slices than the pass over
    # all rows), so a few of its values can round to the neighbouring bf16 value before dB is formed.
    layer.bwd(h_save=False)
    torch.cuda.synchronize()
    assert eq(layer.dA[tr_ad], dA1[tr_ad]) and eq(layer.dx, dx1)
    err = (layer.dB[tr_ad] - dB1[tr_ad]).abs().max().item() / dB1[tr_ad].abs().max().item()
    assert err <= 1e-3, err
    # and the recomputing call is itself reproducible
    dB2 = layer.dB[tr_ad].clone()
    layer.bwd(h_save=False)
    torch.cuda.synchronize()
    assert eq(layer.dB[tr_ad], dB2)
    layer.bwd()
    torch.cuda.synchronize()
    assert eq(layer.dB[tr_ad], dB1[tr_ad])
    # accumulate adds to what the buffers hold
    layer.bwd(accumulate=True)
    torch.cuda.synchronize()
    assert torch.allclose(layer.dA[tr_ad], 2 * dA1[tr_ad], rtol=1e-6, atol=0)
    assert torch.allclose(layer.dB[tr_ad], 2 * dB1[tr_ad], rtol=1e-6, atol=0)
    ctx.close()


def test_backward_without_dx_or_without_adapter_gradients():
    import torch

    w = _adhoc("bf16", 256, 128, [16, 8], [30, 100, 60], [0, 1, 0], [0, 1, 1])
    t = wl.make_tensors(w)
    ctx = make_ctx(w)
    full = DeviceLayer(w, t, ctx)
    full.fwd()
    full.bwd()
    a = DeviceLayer(w, t, ctx)
    a.fwd()
    a.bwd(dx=False)
    b = DeviceLayer(w, t, ctx)
    b.fwd()
    b.bwd(dab=False)
    torch.cuda.synchronize()
    assert torch.isnan(a.dx).all()
    assert all(torch.equal(p, q) for p, q in zip(a.dA, full.dA))
    assert all(torch.isnan(p).all() for p in b.dA + b.dB)
    tr = torch.from_numpy(full.tok_train != 0).cuda()
    assert torch.equal(b.dx[tr].view(torch.int16), full.dx[tr].view(torch.int16))
    ctx.close()


def test_error_statuses_touch_nothing():
    import torch

    w = _adhoc("bf16", 64, 64, [8, 8], [10, 20], [0, 1], [0, 1])
    t = wl.make_tensors(w)
    ctx = make_ctx(w)
    layer = DeviceLayer(w, t, ctx)

    def expect(status, fn):
        with pytest.raises(binding.CollmError) as e:
            fn()
        assert e.value.status == status, e.value

    c = ctx.collm_lora_linear_fwd
    args = lambda **k: dict(dict(x=layer.x, W=layer.W, A=layer.A, B=layer.B, rank=w.ranks, seg_start=w.seg_start,
                                 seg_adapter=w.seg_adapter, seg_is_train=w.seg_is_train, scale=2.0, y=layer.y), **k)
    expect(-3, lambda: c(**args(seg_start=[0, 10, 29])))
    expect(-3, lambda: c(**args(seg_start=[1, 10, 30])))
    expect(-4, lambda: c(**args(seg_adapter=[0, 2])))
    expect(-4, lambda: c(**args(seg_adapter=[0, -1])))          # training segment without adapter
    expect(-4, lambda: c(**args(A=[layer.A[0], None])))        # used adapter without table
    expect(-5, lambda: c(**args(rank=[8, 9])))                 # beyond the context's max_rank
    expect(-5, lambda: c(**args(rank=[8, 0])))
    odd = layer.x.view(-1)[4:][: 29 * 64].view(29, 64)  # 8 bytes off a 16-byte boundary
    expect(-7, lambda: c(**args(x=odd, seg_start=[0, 10, 29])))
    big = torch.zeros((31, 64), dtype=torch.bfloat16, device="cuda")
    expect(-2, lambda: c(**args(x=big, seg_start=[0, 10, 31])))  # more tokens than the context holds
    expect(-2, lambda: c(**args(x=layer.x[:, :60].contiguous())))  # d_in not a multiple of 8
    expect(-2, lambda: c(**args(layout=2)))                      # unknown layout
    torch.cuda.synchronize()
    assert torch.isnan(layer.y).all()
    # backward: trained adapter without gradient buffers
    expect(-4, lambda: ctx.collm_lora_linear_bwd(layer.x, layer.W, layer.A, layer.B, w.ranks, w.seg_start,
                                                 w.seg_adapter, w.seg_is_train, 2.0, layer.dy, None, layer.dx,
                                                 [layer.dA[0], None], [layer.dB[0], None]))
    assert torch.isnan(layer.dx).all()
    ctx.close()


# ---------------------------------------------------------------------------------------------
# the step after the backward pass: AdamW update of an adapter table, aggregation of the copies
# ---------------------------------------------------------------------------------------------
def _rounded(a, dtype):
    return wl.bf16_round(a) if dtype == "bf16" else a


@pytest.mark.gpu
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("shape", [(4096, 16), (16, 4096), (1037, 5), (1, 3), (11008, 64)])
def test_adapter_fedavg_matches_oracle(dtype, shape):
    import torch

    rng = np.random.default_rng(20260416 + shape[0])
    K = 5 if shape[0] != 11008 else 16
    host = [_rounded(rng.normal(0.0, 0.02, size=shape).astype(np.float32), dtype) for _ in range(K)]
    ref = oracle.adapter_fedavg(host)
    dev = [to_dev(h, dtype) for h in host]
    dst = torch.full_like(dev[0], float("nan"))
    binding.collm_adapter_fedavg(dev, dst)
    torch.cuda.synchronize()
    got = dst.float().cpu().numpy().astype(np.float64)
    err = np.max(np.abs(got - ref)) / np.max(np.abs(ref))
    assert err <= TOL[dtype], err
    # in place (dst is one of the sources) gives the same bits
    binding.collm_adapter_fedavg(dev, dev[2])
    torch.cuda.synchronize()
    assert torch.equal(dev[2].view(torch.int16 if dtype == "bf16" else torch.int32),
                       dst.view(torch.int16 if dtype == "bf16" else torch.int32))


@pytest.mark.gpu
@pytest.mark.parametrize("dtype,use_master", [("bf16", True), ("bf16", False), ("f32", False)])
def test_adapter_adamw_matches_oracle(dtype, use_master):
    import torch

    rng = np.random.default_rng(7)
    shape = (4099, 16)  # not a multiple of four elements: exercises the tail
    p0 = _rounded(rng.normal(0.0, 0.02, size=shape).astype(np.float32), dtype)
    # the C ABI takes fp32 hyper-parameters: the oracle gets exactly those values
    lr, b1, b2, eps, wd = (float(np.float32(h)) for h in (1e-3, 0.9, 0.999, 1e-8, 0.01))
    param = to_dev(p0, dtype)
    master = torch.tensor(p0, dtype=torch.float32, device="cuda") if use_master else None
    m = torch.zeros(shape, dtype=torch.float32, device="cuda")
    v = torch.zeros(shape, dtype=torch.float32, device="cuda")
    rp, rm, rv = p0.astype(np.float64), np.zeros(shape), np.zeros(shape)
    for step in range(1, 4):
        g = rng.normal(0.0, 1e-2, size=shape).astype(np.float32)
        binding.collm_adapter_adamw(param, torch.tensor(g, device="cuda"), m, v, lr, b1, b2, eps, wd, step,
                                    master=master)
        torch.cuda.synchronize()
        # without a master copy the parameter a step starts from is the rounded result of the step before
        start = rp if (use_master or dtype == "f32" or step == 1) else param_prev
        rp, rm, rv = oracle.adamw_step(start, g, rm, rv, lr, b1, b2, eps, wd, step)
        param_prev = param.float().cpu().numpy().astype(np.float64)
        ref_w = rp
        got_w = (master if use_master else param).float().cpu().numpy().astype(np.float64)
        tol_w = 1e-5 if (use_master or dtype == "f32") else TOL["bf16"]
        assert np.max(np.abs(got_w - ref_w)) / np.max(np.abs(ref_w)) <= tol_w
        assert np.max(np.abs(m.cpu().numpy() - rm)) / np.max(np.abs(rm)) <= 1e-5
        assert np.max(np.abs(v.cpu().numpy() - rv)) / np.max(np.abs(rv)) <= 1e-5
        # the element-type copy is the rounded master
        if use_master:
            assert torch.equal(param, master.to(torch.bfloat16))


@pytest.mark.gpu
def test_adapter_update_error_statuses():
    import torch

    a = torch.zeros(64, dtype=torch.bfloat16, device="cuda")
    f = torch.zeros(64, dtype=torch.float32, device="cuda")
    with pytest.raises(binding.CollmError) as e:
        binding.collm_adapter_fedavg([a] * 17, a)
    assert e.value.status == -2
    with pytest.raises(binding.CollmError) as e:
        binding.collm_adapter_adamw(a, f, f.clone(), f.clone(), 1e-3, 0.9, 0.999, 1e-8, 0.0, 0)
    assert e.value.status == -2
    with pytest.raises(binding.CollmError) as e:
        binding.collm_adapter_fedavg([a, a[1:33]], a[:32])
    assert e.value.status == -7
