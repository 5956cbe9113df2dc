"""CPU-side checks of the C-ABI library: it loads, exports what the header declares, and its
host-only integer bookkeeping equals the oracle's bit for bit."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
from paper_2604_16400_amd import binding
from paper_2604_16400_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    lib = binding.load_library()
    hdr = open(os.path.join(ROOT, "include", "collm_lora.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    names = re.findall(r"\b(collm_[a-z_0-9]+)\s*\(", hdr)
    assert len(set(names)) >= 11
    for n in set(names):
        assert hasattr(lib, n), n
    assert lib.collm_status_string(0) == b"ok"
    assert lib.collm_status_string(-3) != lib.collm_status_string(-4)


def test_token_map_matches_oracle_bit_for_bit_fuzz():
    rng = np.random.default_rng(20260416)
    for it in range(10000):
        S = int(rng.integers(0, 40))
        kind = it % 4
        if kind == 0:
            lens = rng.integers(0, 4, size=S)
        elif kind == 1:
            lens = rng.integers(1, 300, size=S)
        elif kind == 2:
            lens = (rng.random(S) < 0.3) * rng.integers(0, 2000, size=S)
        else:
            lens = np.ones(S, dtype=np.int64)
        seg_start = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
        tr = rng.integers(0, 2, size=S).astype(np.uint8)
        ad = rng.integers(-1, 7, size=S).astype(np.int32)
        ad[(tr != 0) & (ad < 0)] = 0
        got = binding.collm_token_map(seg_start, ad, tr, n_adapters=7)
        ref = oracle.token_map(seg_start, ad, tr)
        for g, r in zip(got, ref):
            assert g.dtype == r.dtype and np.array_equal(g, r)


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
def test_token_map_configs(cfg):
    w = wl.make_config(cfg)
    got = binding.collm_token_map(w.seg_start, w.seg_adapter, w.seg_is_train, n_adapters=w.n_adapters)
    ref = oracle.token_map(w.seg_start, w.seg_adapter, w.seg_is_train)
    for g, r in zip(got, ref):
        assert np.array_equal(g, r)
    assert int(np.count_nonzero(got[2])) == w.n_train_tokens


def test_token_map_rejects_bad_tables():
    f = binding.collm_token_map
    with pytest.raises(binding.CollmError) as e:
        f([1, 3], [0], [0])  # does not start at 0
    assert e.value.status == -3
    with pytest.raises(binding.CollmError) as e:
        f([0, 3, 2], [0, 0], [0, 0])  # decreasing
    assert e.value.status == -3
    with pytest.raises(binding.CollmError) as e:
        f([0, 3], [0], [0], n_tokens=4)  # does not end at T
    assert e.value.status == -3
    with pytest.raises(binding.CollmError) as e:
        f([0, 3], [5], [0], n_adapters=5)  # adapter out of range
    assert e.value.status == -4
    with pytest.raises(binding.CollmError) as e:
        f([0, 3], [-1], [1], n_adapters=5)  # training segment without adapter
    assert e.value.status == -4
    with pytest.raises(binding.CollmError) as e:
        f([0, 3], [-2], [0], n_adapters=5)
    assert e.value.status == -4


# ---------------------------------------------------------------------------------------------
# the plan's row order (host logic): rows in runs of one adapter, low-rank K-steps per row tile
# ---------------------------------------------------------------------------------------------
def _steps_from_rows(row_tok, tok_adapter, ranks, tile_rows):
    """K-steps per row tile, counted from the row order: every maximal run of one adapter inside a
    tile costs ceil(rank / 16) steps; the steps are listed by groups of 64 rank indices, and every group
    but the tile's last is filled up to a multiple of four steps."""
    out = []
    for t0 in range(0, len(row_tok), tile_rows):
        ads = tok_adapter[row_tok[t0:t0 + tile_rows]]
        run_ranks = [int(ranks[a]) for i, a in enumerate(ads) if a >= 0 and (i == 0 or ads[i - 1] != a)]
        n, g = 0, 0
        while True:
            n += sum((min(r, g + 64) - g + 15) // 16 for r in run_ranks if r > g)
            g += 64
            if not any(r > g for r in run_ranks):
                break
            n = (n + 3) // 4 * 4
        out.append(n)
    return np.array(out, dtype=np.int32)


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
@pytest.mark.parametrize("tile_rows", [128, 256])
def test_plan_row_order_is_a_grouping_and_counts_its_steps(cfg, tile_rows):
    w = wl.make_config(cfg)
    _, ta, tt = oracle.token_map(w.seg_start, w.seg_adapter, w.seg_is_train)
    row_tok, steps = binding.host_row_order(w.ranks, w.seg_start, w.seg_adapter, w.seg_is_train, tile_rows)
    assert sorted(row_tok.tolist()) == list(range(w.n_tokens))           # every token exactly once
    ads = ta[row_tok]
    n_base = int((ta < 0).sum())
    assert np.all(ads[:n_base] < 0) and np.all(ads[n_base:] >= 0)        # base-only rows first
    for a in range(w.n_adapters):                                         # token order kept inside an adapter
        toks = row_tok[ads == a]
        assert np.all(np.diff(toks) > 0)
    assert np.array_equal(steps, _steps_from_rows(row_tok, ta, w.ranks, tile_rows))
    # training rows: one run per adapter (the gradient items are runs)
    row_tr, steps_tr = binding.host_row_order(w.ranks, w.seg_start, w.seg_adapter, w.seg_is_train, tile_rows, True)
    assert sorted(row_tr.tolist()) == np.flatnonzero(tt).tolist()
    ads_tr = ta[row_tr]
    changes = int((np.diff(ads_tr) != 0).sum()) + 1 if len(ads_tr) else 0
    assert changes == len(np.unique(ads_tr))
    assert np.array_equal(steps_tr, _steps_from_rows(row_tr, ta, w.ranks, tile_rows))


def test_plan_spreads_rare_adapters_over_the_row_tiles():
    # configuration 3: 32 adapters of rank 64 with Zipf popularity.  Listed by adapter index, the rare ones
    # would share the last tiles (11 adapters = 44 steps in one of them); dealt out, no tile carries more than
    # a few adapters beside the large ones that fill it.
    w = wl.make_config(3)
    _, ta, _ = oracle.token_map(w.seg_start, w.seg_adapter, w.seg_is_train)
    _, steps = binding.host_row_order(w.ranks, w.seg_start, w.seg_adapter, w.seg_is_train, 256)
    by_index = _steps_from_rows(np.argsort(ta, kind="stable").astype(np.int32), ta, w.ranks, 256)
    assert by_index.max() >= 40
    assert steps.max() <= 20 and steps.max() <= by_index.max() // 2
    assert steps.sum() <= by_index.sum() + 4 * len(steps)   # at most one more run per tile, of rank 64


def test_gemm_tiling_covers_the_rows_and_matches_the_measured_choices():
    rng = np.random.default_rng(5)
    for _ in range(2000):
        rows = int(rng.integers(1, 40000))
        cols = int(rng.integers(1, 4000)) * 8
        K = int(rng.integers(1, 2000)) * 8
        tile, big, tail, tail_cols = binding.host_tiling(rows, cols, K, bool(rng.integers(0, 2)))
        assert tile in (binding.TILE_256x256, binding.TILE_128x128) and big >= 1 and tail >= 0 and tail_cols >= 0
        tr = 256 if tile == binding.TILE_256x256 else 128
        assert tr * big + 128 * tail >= rows                      # every row is in some tile
        if tail:
            assert tile == binding.TILE_256x256 and 256 * big < rows          # the tail starts inside the rows
            assert 256 * big + 128 * (tail - 1) < rows                        # and has no empty row tile
        else:
            assert tr * (big - 1) < rows or rows <= tr
        if tail_cols:
            # large tiles over whole rounds of the 256 CUs, then at most one round of small tiles (two per CU)
            tn = (cols + 255) // 256
            assert tile == binding.TILE_256x256 and tail == 0 and 0 < tail_cols < tn
            assert big * (tn - tail_cols) <= 256 * (big * tn // 256)
            assert ((rows + 127) // 128) * ((cols - 256 * (tn - tail_cols) + 127) // 128) <= 512
    # choices the measurements on the five configurations gave
    assert binding.host_tiling(2048, 4096, 4096) == (binding.TILE_128x128, 16, 0, 0)    # c2 forward: one round of 512 small tiles
    assert binding.host_tiling(16384, 8192, 8192) == (binding.TILE_256x256, 64, 0, 0)   # c5: whole rounds of large tiles
    assert binding.host_tiling(3277, 5120, 5120) == (binding.TILE_256x256, 12, 2, 0)    # c4 dX: 240 large tiles + the last 205 rows
    assert binding.host_tiling(8192, 5120, 5120) == (binding.TILE_256x256, 32, 0, 4)    # c4 forward: 2 rounds + 512 tiles of 128x128
    assert binding.host_tiling(4096, 11008, 4096) == (binding.TILE_256x256, 16, 0, 0)   # c3 forward: 2.7 rounds, no split pays
    assert binding.host_tiling(64, 4096, 4096)[0] == binding.TILE_128x128               # decode-sized


def _sanitizer_run(tmp_path, compiler, std, sources, args):
    """Builds the sources with the address and undefined-behaviour sanitizers (static runtimes, so that nothing
    preloaded into this process matters) and runs the result."""
    import subprocess

    exe = str(tmp_path / "sanitized")
    cmd = [compiler, std, "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan",
           "-static-libubsan", "-I", os.path.join(ROOT, "include"), "-I", os.path.join(ROOT, "paper_2604_16400_amd", "csrc"),
           *sources, "-lm", "-o", exe]
    subprocess.run(cmd, check=True, capture_output=True, text=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", LD_PRELOAD="")
    r = subprocess.run([exe, *args], capture_output=True, text=True, env=env, timeout=240)
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-4000:]
    return r.stdout


def test_planner_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    # 10^4 random segment tables through build_plan with every option (tile sizes, item sizes, the tiled pass,
    # sibling ranks), each plan checked against what the table fixes: csrc/planner.cpp is offset arithmetic into
    # one int32 block
    out = _sanitizer_run(tmp_path, "g++", "-std=c++17",
                         [os.path.join(ROOT, "tests", "sanitize_planner.cpp"),
                          os.path.join(ROOT, "paper_2604_16400_amd", "csrc", "planner.cpp")], ["10000"])
    assert "planner ok 10000" in out


def test_oracle_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    out = _sanitizer_run(tmp_path, "gcc", "-std=c11",
                         [os.path.join(ROOT, "tests", "sanitize_oracle.c"), os.path.join(ROOT, "oracle", "collm_oracle.c")],
                         ["300"])
    assert "oracle ok 300" in out


def test_gemm_tile_order_visits_every_tile_once_and_keeps_bands_together():
    # The workgroup id -> tile map of the GEMM kernels, run on the host: a bijection for every grid and band, a band's
    # tiles contiguous in workgroup ids, and the walk of every XCD through a band.
    rng = np.random.default_rng(5)
    shapes = [(64, 112, 32), (64, 32, 32), (64, 4, 0), (13, 20, 0), (13, 20, 8), (40, 7, 16), (33, 5, 24), (1, 1, 0), (7, 3, 8)]
    shapes += [(int(rng.integers(1, 70)), int(rng.integers(1, 40)), int(rng.integers(0, 5)) * 8) for _ in range(60)]
    for tiles_m, tiles_n, band in shapes:
        used, tm, tn = binding.host_tile_order(256, tiles_m, tiles_n, 8192, band)
        assert used == band
        seen = np.zeros((tiles_m, tiles_n), dtype=np.int32)
        np.add.at(seen, (tm, tn), 1)
        assert (seen == 1).all(), (tiles_m, tiles_n, band)
        if 0 < band < tiles_m:
            ids = np.arange(tiles_m * tiles_n)
            assert np.array_equal(tm // band, ids // (band * tiles_n)), (tiles_m, tiles_n, band)
        # an XCD (workgroup ids 8 i + x) walks the groups of 8 row tiles of a band in ascending order, and inside a
        # group column by column
        b = band if 0 < band < tiles_m else tiles_m
        for x in range(8):
            m, n = tm[x::8].astype(np.int64), tn[x::8].astype(np.int64)
            key = ((m // b) * (tiles_m + 8) + (m % b) // 8) * tiles_n + n
            assert (np.diff(key) >= 0).all(), (tiles_m, tiles_n, band, x)
    # the band the library chooses: the rows of configuration 5 (16384 x 8192) in bands of 32 row tiles; none where all
    # rows fit the cache anyway (few row tiles) or where not even 16 row tiles do (K = 28672)
    assert binding.host_tile_order(256, 64, 112, 8192)[0] == 32
    assert binding.host_tile_order(256, 64, 32, 8192)[0] == 32
    assert binding.host_tile_order(256, 32, 54, 5120)[0] == 0
    assert binding.host_tile_order(256, 32, 32, 28672)[0] == 0
    assert binding.host_tile_order(128, 16, 32, 4096)[0] == 0

