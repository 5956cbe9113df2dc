"""The forward entry point that allocates nothing (static device workspace) against the context-based one."""
import numpy as np
import pytest

from paper_2604_16400_amd import binding
from paper_2604_16400_amd import workloads as wl

from gpu_util import TOL, maxrel, to_dev, to_host

pytestmark = pytest.mark.gpu


def _both(w, transposed=False):
    import torch

    t = wl.make_tensors(w)
    p = w.projections[0]
    tp = (lambda a: np.ascontiguousarray(np.asarray(a).T)) if transposed else (lambda a: a)
    layout = binding.LAYOUT_OUT_IN if transposed else binding.LAYOUT_IN_OUT
    x, W = to_dev(t.x, w.dtype), to_dev(tp(t.W), w.dtype)
    A, B = [to_dev(tp(a), w.dtype) for a in t.A], [to_dev(tp(b), w.dtype) for b in t.B]
    T = w.n_tokens
    dt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    mr = binding.NOALLOC_MAX_RANK
    outs = []
    for static in (False, True):
        y = torch.full((T, p.d_out), float("nan"), dtype=dt, device="cuda")
        hs = torch.full((T, mr), float("nan"), dtype=torch.float32, device="cuda")
        args = (x, W, A, B, w.ranks, w.seg_start, w.seg_adapter, w.seg_is_train, w.scale, y, hs)
        if static:
            binding.collm_lora_linear_fwd_noalloc(*args, layout=layout)
        else:
            ctx = binding.Context(max(T, 1), max(w.n_segments, 1), w.n_adapters, mr, max(p.d_in, p.d_out))
            ctx.collm_lora_linear_fwd(*args, layout=layout)
            torch.cuda.synchronize()
            ctx.close()
        torch.cuda.synchronize()
        outs.append((to_host(y), to_host(hs)))
    (y0, h0), (y1, h1) = outs
    tr = np.repeat(w.seg_is_train, np.diff(w.seg_start)) != 0
    assert np.all(np.isfinite(y1)) and np.all(np.isfinite(y0))
    assert np.array_equal(np.isnan(h0), np.isnan(h1)) and np.all(np.isnan(h1[~tr]))
    tol = TOL[w.dtype]
    assert maxrel(y1, y0) <= tol, maxrel(y1, y0)
    if tr.any():
        assert maxrel(h1[tr], h0[tr]) <= tol
    return maxrel(y1, y0)


def test_noalloc_forward_matches_the_context_call_twice_second_smaller():
    big = wl.make_adhoc("noalloc_big", "bf16", 1024, 1536, [16, 8, 64, 24],
                        [1] * 90 + [400, 33, 512, 0, 700], list(np.arange(90) % 4) + [0, 1, -1, 2, 3],
                        [0] * 90 + [1, 0, 0, 0, 1], scale=0.5, seed=21)
    small = wl.make_adhoc("noalloc_small", "bf16", 256, 328, [16, 40], [1] * 9 + [70, 21], list(np.arange(9) % 2) + [1, 0],
                          [0] * 9 + [1, 0], scale=2.0, seed=22)
    e_big = _both(big)
    e_small = _both(small)          # smaller input right after: nothing of the larger call may leak in
    e_tr = _both(small, transposed=True)
    e_f32 = _both(wl.make_config(1))
    print("noalloc vs context: max-normalised differences", e_big, e_small, e_tr, e_f32)


def test_noalloc_rejects_sizes_beyond_its_workspace():
    import torch

    x = torch.zeros((4096, 64), dtype=torch.bfloat16, device="cuda")
    W = torch.zeros((64, 64), dtype=torch.bfloat16, device="cuda")
    y = torch.full((4096, 64), float("nan"), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(binding.CollmError) as e:
        binding.collm_lora_linear_fwd_noalloc(x, W, [], [], [], [0, 4096], [-1], [0], 1.0, y)
    assert e.value.status == -2 and "2048 tokens" in str(e.value)
    A = [torch.zeros((64, 128), dtype=torch.bfloat16, device="cuda")]
    B = [torch.zeros((128, 64), dtype=torch.bfloat16, device="cuda")]
    with pytest.raises(binding.CollmError) as e:   # rank 128 > 64
        binding.collm_lora_linear_fwd_noalloc(x[:100], W, A, B, [128], [0, 100], [0], [0], 1.0, y[:100])
    assert e.value.status == -5
    torch.cuda.synchronize()
    assert torch.isnan(y).all()
