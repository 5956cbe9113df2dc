"""GPU parity of the sibling-projection calls (several projections of the same x stored side by side)
against the fp64 oracle, element by element.  Tolerance as for the single projection: 1e-2 of the
largest reference entry per output tensor (bf16 inputs, fp32 accumulation)."""
import numpy as np
import pytest

import oracle
from paper_2604_16400_amd import binding
from paper_2604_16400_amd import workloads as wl

from gpu_util import TOL, maxrel, to_dev, to_host

pytestmark = pytest.mark.gpu


class SiblingCase:
    def __init__(self, d_in, d_outs, ranks, lens, adapters, train, scale=2.0, seed=11):
        rng = np.random.default_rng(seed)
        self.d_in, self.d_outs, self.scale = d_in, list(d_outs), scale
        self.P, self.D = len(d_outs), int(sum(d_outs))
        self.ranks = np.asarray(ranks, dtype=np.int32)
        self.seg_start = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
        self.seg_adapter = np.asarray(adapters, dtype=np.int32)
        self.seg_is_train = np.asarray(train, dtype=np.uint8)
        T = int(self.seg_start[-1])
        self.T = T
        r32 = lambda *s: rng.standard_normal(s).astype(np.float32)
        self.x = wl.bf16_round(r32(T, d_in))
        self.W = wl.bf16_round(r32(d_in, self.D) * 0.02)
        self.A = [wl.bf16_round(r32(d_in, self.P * int(r)) * d_in ** -0.5) for r in ranks]
        self.B = [wl.bf16_round(r32(int(r), self.D) * 0.05) for r in ranks]
        self.dy = wl.bf16_round(r32(T, self.D))
        _, self.tok_adapter, self.tok_train = oracle.token_map(self.seg_start, self.seg_adapter, self.seg_is_train)


def _run(case: SiblingCase, h_save=True, accumulate=False):
    import torch

    P, T, D = case.P, case.T, case.D
    max_rank = P * int(case.ranks.max())
    ctx = binding.Context(max(T, 1), len(case.seg_adapter), len(case.ranks), max_rank, max(case.d_in, D))
    nan = float("nan")
    x, W, dy = to_dev(case.x, "bf16"), to_dev(case.W, "bf16"), to_dev(np.where(case.tok_train[:, None] != 0, case.dy, np.nan).astype(np.float32), "bf16")
    A, B = [to_dev(a, "bf16") for a in case.A], [to_dev(b, "bf16") for b in case.B]
    y = torch.full((T, D), nan, dtype=torch.bfloat16, device="cuda")
    dx = torch.full((T, case.d_in), nan, dtype=torch.bfloat16, device="cuda")
    hs = torch.full((T, max_rank), nan, dtype=torch.float32, device="cuda")
    base = 1.5 if accumulate else nan
    dA = [torch.full(a.shape, base, dtype=torch.float32, device="cuda") for a in case.A]
    dB = [torch.full(b.shape, base, dtype=torch.float32, device="cuda") for b in case.B]
    seg = (case.ranks, case.seg_start, case.seg_adapter, case.seg_is_train, case.scale)
    ctx.collm_lora_siblings_fwd(case.d_outs, x, W, A, B, *seg, y, hs if h_save else None)
    ctx.collm_lora_siblings_bwd(case.d_outs, x, W, A, B, *seg, dy, hs if h_save else None, dx, dA, dB, accumulate)
    torch.cuda.synchronize()

    ta, tt = case.tok_adapter, case.tok_train
    y_ref, h_ref = oracle.lora_siblings_fwd(case.x, case.W, case.A, case.B, case.d_outs, ta, case.scale)
    dx_ref, dA_ref, dB_ref = oracle.lora_siblings_bwd(case.x, case.W, case.A, case.B, case.d_outs, ta, tt, case.scale,
                                                      case.dy)
    errs = {}
    yh = to_host(y)
    assert np.all(np.isfinite(yh))
    errs["y"] = maxrel(yh, y_ref)
    tr = tt != 0
    dxh = to_host(dx)
    assert np.all(np.isnan(dxh[~tr]))
    if tr.any():
        assert np.all(np.isfinite(dxh[tr]))
        errs["dx"] = maxrel(dxh[tr], dx_ref[tr])
    if h_save:
        hh = to_host(hs)
        assert np.all(np.isnan(hh[~tr]))
        if tr.any():
            ref = np.zeros((int(tr.sum()), max_rank))
            ref[:, : h_ref.shape[1]] = h_ref[tr]
            errs["h"] = maxrel(hh[tr], ref)
            for tok in np.flatnonzero(tr):  # zero beyond the P ranks of the token's adapter
                assert np.all(hh[tok, P * case.ranks[ta[tok]]:] == 0.0)
    for a in range(len(case.ranks)):
        gA, gB = to_host(dA[a]), to_host(dB[a])
        if dA_ref[a] is None:
            if accumulate:
                assert np.all(gA == 1.5) and np.all(gB == 1.5)
            else:
                assert np.all(np.isnan(gA)) and np.all(np.isnan(gB))
        else:
            off = 1.5 if accumulate else 0.0
            errs[f"dA{a}"] = maxrel(gA - off, dA_ref[a])
            errs[f"dB{a}"] = maxrel(gB - off, dB_ref[a])
    ts, ta_d, tt_d = ctx.device_token_map(T)
    rs, ra, rt = oracle.token_map(case.seg_start, case.seg_adapter, case.seg_is_train)
    assert np.array_equal(ts, rs) and np.array_equal(ta_d, ra) and np.array_equal(tt_d, rt)
    ctx.close()
    bad = {k: v for k, v in errs.items() if not v <= TOL["bf16"]}
    assert not bad, f"beyond tolerance: {bad} (all: {errs})"
    return errs


LENS = [5, 0, 37, 1, 130, 0, 70, 2, 64, 301]
ADS = [0, 1, -1, 2, 2, 3, 3, -1, 1, 2]
TRN = [0, 0, 0, 0, 1, 0, 1, 0, 0, 1]


def test_two_siblings_ragged():
    # gate/up-like pair; the second sibling's width is no multiple of a tile; ranks 8..64 (24 and 40 leave the
    # last 16-wide step of a sibling half empty); decode, base-only, empty and training segments
    c = SiblingCase(320, (256, 200), [8, 16, 24, 40], LENS, ADS, TRN, scale=0.3)
    _run(c)
    _run(c, h_save=False)
    _run(c, accumulate=True)


def test_three_siblings_qkv_like():
    c = SiblingCase(512, (512, 256, 128), [16, 8, 32], [40, 1, 1, 1, 90, 33, 1, 260], [0, 1, 2, 0, 1, 2, 1, 0],
                    [0, 0, 0, 0, 1, 0, 0, 1])
    _run(c)
    _run(c, h_save=False)


def test_two_siblings_wide_ranks_and_large_tiles():
    # rank 64 per sibling (128 side by side: the tiled rank-wide passes, per sibling on the dh side),
    # enough rows and columns for 256x256 tiles, rows of several adapters inside one row tile
    c = SiblingCase(1024, (1536, 1280), [64, 32, 64], [300, 1, 1, 200, 150, 9, 260], [0, 1, 2, 1, 2, -1, 0],
                    [1, 0, 0, 1, 0, 0, 1])
    _run(c)
    _run(c, h_save=False)


def test_one_sibling_equals_the_single_projection_call():
    import torch

    c = SiblingCase(256, (192,), [12, 16], [30, 50, 7], [0, 1, 0], [1, 0, 1], scale=0.5)
    _run(c)  # ranks need not be multiples of 8 with a single sibling
    ctx = binding.Context(c.T, 3, 2, 16, 256)
    x, W = to_dev(c.x, "bf16"), to_dev(c.W, "bf16")
    A, B = [to_dev(a, "bf16") for a in c.A], [to_dev(b, "bf16") for b in c.B]
    seg = (c.ranks, c.seg_start, c.seg_adapter, c.seg_is_train, c.scale)
    y1 = torch.empty((c.T, 192), dtype=torch.bfloat16, device="cuda")
    y2 = torch.empty_like(y1)
    ctx.collm_lora_siblings_fwd((192,), x, W, A, B, *seg, y1)
    ctx.collm_lora_linear_fwd(x, W, A, B, *seg, y2)
    torch.cuda.synchronize()
    assert torch.equal(y1, y2)
    ctx.close()


def test_sibling_error_statuses():
    import torch

    c = SiblingCase(64, (256, 64), [8, 16], [10, 20], [0, 1], [0, 1])
    ctx = binding.Context(c.T, 2, 2, 32, 320)
    x, W = to_dev(c.x, "bf16"), to_dev(c.W, "bf16")
    A, B = [to_dev(a, "bf16") for a in c.A], [to_dev(b, "bf16") for b in c.B]
    y = torch.full((c.T, c.D), float("nan"), dtype=torch.bfloat16, device="cuda")
    seg = [c.ranks, c.seg_start, c.seg_adapter, c.seg_is_train, c.scale]

    def expect(status, fn):
        with pytest.raises(binding.CollmError) as e:
            fn()
        assert e.value.status == status, e.value

    f = ctx.collm_lora_siblings_fwd
    expect(-2, lambda: f((256, 32), x, W, A, B, *seg, y))            # widths do not add up to W's columns
    expect(-2, lambda: f((64, 256), x, W, A, B, *seg, y))            # a sibling but the last is no multiple of 256
    expect(-5, lambda: f((256, 64), x, W, A, B, [8, 12], *seg[1:], y))   # rank no multiple of 8
    expect(-5, lambda: f((256, 64), x, W, A, B, [8, 24], *seg[1:], y))   # 2 x 24 beyond the context's max_rank
    xf = torch.zeros((c.T, 64), dtype=torch.float32, device="cuda")
    expect(-6, lambda: f((256, 64), xf, W, A, B, *seg, y))           # fp32 is not served
    torch.cuda.synchronize()
    assert torch.isnan(y).all()
    ctx.close()


# ---------------------------------------------------------------------------------------------
# gate/up pair with the SwiGLU epilogue, and the gradient through it
# ---------------------------------------------------------------------------------------------
def _run_swiglu(case: SiblingCase, tile=None, keep_pre=True):
    import torch

    assert case.P == 2 and case.d_outs[0] == case.d_outs[1]
    T, D, d_ff = case.T, case.D, case.d_outs[0]
    max_rank = 2 * int(case.ranks.max())
    ctx = binding.Context(max(T, 1), len(case.seg_adapter), len(case.ranks), max_rank, max(case.d_in, D))
    if tile is not None:
        ctx.set_tiles(tile, tile)
    x, W = to_dev(case.x, "bf16"), to_dev(case.W, "bf16")
    A, B = [to_dev(a, "bf16") for a in case.A], [to_dev(b, "bf16") for b in case.B]
    y = torch.full((T, d_ff), float("nan"), dtype=torch.bfloat16, device="cuda")
    pre = torch.full((T, D), float("nan"), dtype=torch.bfloat16, device="cuda")
    hs = torch.full((T, max_rank), float("nan"), dtype=torch.float32, device="cuda")
    seg = (case.ranks, case.seg_start, case.seg_adapter, case.seg_is_train, case.scale)
    ctx.collm_lora_siblings_fwd(case.d_outs, x, W, A, B, *seg, y, hs, activation=binding.ACT_SWIGLU,
                                pre_act=pre if keep_pre else None)
    torch.cuda.synchronize()
    y_pre_ref, h_ref = oracle.lora_siblings_fwd(case.x, case.W, case.A, case.B, case.d_outs, case.tok_adapter, case.scale)
    out_ref = oracle.swiglu(y_pre_ref)
    yh = to_host(y)
    assert np.all(np.isfinite(yh))
    errs = {"y": maxrel(yh, out_ref)}
    tr = case.tok_train != 0
    ph = to_host(pre)
    if keep_pre:
        assert np.all(np.isnan(ph[~tr]))
        if tr.any():
            assert np.all(np.isfinite(ph[tr]))
            errs["pre"] = maxrel(ph[tr], y_pre_ref[tr])
    else:
        assert np.all(np.isnan(ph))
    hh = to_host(hs)
    if tr.any():
        ref = np.zeros((int(tr.sum()), max_rank))
        ref[:, : h_ref.shape[1]] = h_ref[tr]
        errs["h"] = maxrel(hh[tr], ref)
    ctx.close()
    bad = {k: v for k, v in errs.items() if not v <= TOL["bf16"]}
    assert not bad, f"beyond tolerance: {bad} (all: {errs})"
    return pre


@pytest.mark.parametrize("tile", [None, binding.TILE_256x256, binding.TILE_128x128])
def test_swiglu_epilogue(tile):
    # d_ff = 256 + 40 columns per sibling would break the multiple-of-256 rule for the first sibling, so: 512
    # (two 256-wide or four 128-wide column pairs); ranks 16..64; decode, base-only and training rows mixed
    c = SiblingCase(320, (512, 512), [16, 32, 48, 64], LENS, ADS, TRN, scale=0.3)
    _run_swiglu(c, tile)
    _run_swiglu(c, tile, keep_pre=False)


def test_swiglu_epilogue_large_tiles_and_tail():
    # 2300 rows x (2 x 3840) columns: whole rounds of 256x256 tiles, then 128x128 tiles over the last rows
    lens = [700, 1, 1, 500, 300, 1, 600, 197]
    ads = [0, 1, 2, 1, -1, 0, 2, 2]
    c = SiblingCase(64, (3840, 3840), [16, 32, 16], lens, ads, [1, 0, 0, 1, 0, 0, 1, 0], scale=0.5)
    _run_swiglu(c)


def test_swiglu_backward_kernel_and_chain():
    import torch

    # the gradient kernel alone, then the chain: forward with epilogue -> gradient kernel -> sibling backward
    c = SiblingCase(320, (512, 512), [16, 32, 48, 64], LENS, ADS, TRN, scale=0.3)
    pre = _run_swiglu(c)
    rng = np.random.default_rng(3)
    d_ff, T = 512, c.T
    dout_h = wl.bf16_round(rng.standard_normal((T, d_ff)).astype(np.float32))
    tr = c.tok_train != 0
    dout = to_dev(np.where(tr[:, None], dout_h, np.nan).astype(np.float32), "bf16")  # inference rows must not be read
    dy = torch.full((T, 2 * d_ff), float("nan"), dtype=torch.bfloat16, device="cuda")
    binding.collm_swiglu_bwd(c.seg_start, c.seg_is_train, pre, dout, dy)
    torch.cuda.synchronize()
    dyh, preh = to_host(dy), to_host(pre)
    assert np.all(np.isnan(dyh[~tr])) and np.all(np.isfinite(dyh[tr]))
    ref = oracle.swiglu_bwd(preh[tr], dout_h[tr])
    assert maxrel(dyh[tr], ref) <= TOL["bf16"]
    # chain: the sibling backward on that dy.  Every link is compared at the stated tolerance with the oracle fed
    # the values the link before it really produced (the rounded pre-activations above, the rounded dy here), so
    # that no link's rounding is charged to the next one.
    dy_ref = np.zeros((T, 2 * d_ff))
    dy_ref[tr] = dyh[tr]
    dx_ref, dA_ref, dB_ref = oracle.lora_siblings_bwd(c.x, c.W, c.A, c.B, c.d_outs, c.tok_adapter, c.tok_train, c.scale, dy_ref)
    ctx = binding.Context(T, len(c.seg_adapter), len(c.ranks), 128, 1024)
    x, W = to_dev(c.x, "bf16"), to_dev(c.W, "bf16")
    A, B = [to_dev(a, "bf16") for a in c.A], [to_dev(b, "bf16") for b in c.B]
    dx = torch.full((T, c.d_in), float("nan"), dtype=torch.bfloat16, device="cuda")
    dA = [torch.full(a.shape, float("nan"), dtype=torch.float32, device="cuda") for a in c.A]
    dB = [torch.full(b.shape, float("nan"), dtype=torch.float32, device="cuda") for b in c.B]
    ctx.collm_lora_siblings_bwd(c.d_outs, x, W, A, B, c.ranks, c.seg_start, c.seg_adapter, c.seg_is_train, c.scale,
                                dy, None, dx, dA, dB)
    torch.cuda.synchronize()
    errs = {"dx": maxrel(to_host(dx)[tr], dx_ref[tr])}
    for a in range(len(c.ranks)):
        if dA_ref[a] is not None:
            errs[f"dA{a}"] = maxrel(to_host(dA[a]), dA_ref[a])
            errs[f"dB{a}"] = maxrel(to_host(dB[a]), dB_ref[a])
    ctx.close()
    bad = {k: v for k, v in errs.items() if not v <= TOL["bf16"]}
    assert not bad, f"beyond tolerance: {bad} (all: {errs})"


def test_swiglu_backward_more_rows_than_a_grid_dimension():
    import torch

    # 70000 training rows in one segment (beyond 65535) between two inference segments
    d_ff, lens, trn = 64, [300, 70000, 17], [0, 1, 0]
    T = sum(lens)
    seg_start = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    rng = np.random.default_rng(11)
    pre_h = wl.bf16_round(rng.standard_normal((T, 2 * d_ff)).astype(np.float32))
    dout_h = wl.bf16_round(rng.standard_normal((T, d_ff)).astype(np.float32))
    tr = np.repeat(np.array(trn), lens) != 0
    pre, dout = to_dev(pre_h, "bf16"), to_dev(np.where(tr[:, None], dout_h, np.nan).astype(np.float32), "bf16")
    dy = torch.full((T, 2 * d_ff), float("nan"), dtype=torch.bfloat16, device="cuda")
    binding.collm_swiglu_bwd(seg_start, np.array(trn, np.uint8), pre, dout, dy)
    torch.cuda.synchronize()
    dyh = to_host(dy)
    assert np.all(np.isnan(dyh[~tr])) and np.all(np.isfinite(dyh[tr]))
    assert maxrel(dyh[tr], oracle.swiglu_bwd(pre_h[tr], dout_h[tr])) <= TOL["bf16"]


def test_swiglu_error_statuses():
    import torch

    c = SiblingCase(64, (256, 256), [16, 8], [10, 20], [0, 1], [0, 1])
    ctx = binding.Context(c.T, 2, 2, 64, 512)
    x, W = to_dev(c.x, "bf16"), to_dev(c.W, "bf16")
    A, B = [to_dev(a, "bf16") for a in c.A], [to_dev(b, "bf16") for b in c.B]
    y = torch.full((c.T, 256), float("nan"), dtype=torch.bfloat16, device="cuda")
    seg = [c.ranks, c.seg_start, c.seg_adapter, c.seg_is_train, c.scale]
    with pytest.raises(binding.CollmError) as e:   # rank 8 is no multiple of 16
        ctx.collm_lora_siblings_fwd((256, 256), x, W, A, B, *seg, y, activation=binding.ACT_SWIGLU)
    assert e.value.status == -5
    with pytest.raises(binding.CollmError) as e:   # unknown activation
        ctx.collm_lora_siblings_fwd((256, 256), x, W, A, B, *seg, y, activation=7)
    assert e.value.status == -2
    torch.cuda.synchronize()
    assert torch.isnan(y).all()
    ctx.close()


def test_sibling_edge_batches():
    import torch

    # one token; inference only (the backward call is a no-op); training only; widest rank the context takes
    _run(SiblingCase(256, (256, 64), [8], [1], [0], [1]))
    c = SiblingCase(256, (256, 64), [8, 16], [3, 40, 9], [0, 1, -1], [0, 0, 0])
    _run(c)
    _run(SiblingCase(256, (256, 64), [8, 16], [30, 41], [1, 0], [1, 1]))
    _run(SiblingCase(128, (256, 256), [128], [70, 9], [0, 0], [1, 0]))   # 2 x 128 = 256 rank columns side by side
    # empty batch
    ctx = binding.Context(8, 2, 1, 16, 512)
    e = SiblingCase(64, (256, 64), [8], [0, 0], [0, -1], [0, 0])
    x = torch.zeros((0, 64), dtype=torch.bfloat16, device="cuda")
    W = to_dev(e.W, "bf16")
    y = torch.zeros((0, 320), dtype=torch.bfloat16, device="cuda")
    ctx.collm_lora_siblings_fwd((256, 64), x, W, [to_dev(e.A[0], "bf16")], [to_dev(e.B[0], "bf16")], e.ranks, e.seg_start,
                                e.seg_adapter, e.seg_is_train, 1.0, y)
    ctx.close()


def test_swiglu_single_token_and_decode_batch():
    # decode-sized batches take the K-sliced GEMM in the plain sibling call; the epilogue version keeps whole tiles
    c = SiblingCase(2048, (256, 256), [16, 32], [1], [1], [0])
    _run_swiglu(c)
    _run(c)
    lens = [1] * 24 + [8]
    c = SiblingCase(2048, (512, 512), [16, 32, 16], lens, list(np.arange(24) % 3) + [2], [0] * 24 + [1], scale=0.5)
    _run_swiglu(c)
    _run(c)
    _run(c, h_save=False)
