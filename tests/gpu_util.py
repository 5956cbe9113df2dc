"""Helpers of the GPU parity tests: run the library and the oracle on the same seeded inputs."""
from __future__ import annotations

import numpy as np

import oracle
from paper_2604_16400_amd import binding
from paper_2604_16400_amd import workloads as wl

TOL = {"bf16": 1e-2, "f32": 1e-5}  # max|got - ref| / max|ref| per output tensor


to_dev = wl.to_device


def to_host(t) -> np.ndarray:
    return t.float().cpu().numpy().astype(np.float64)


def maxrel(got, ref) -> float:
    got, ref = np.asarray(got, dtype=np.float64), np.asarray(ref, dtype=np.float64)
    if ref.size == 0:
        return 0.0
    return float(np.max(np.abs(got - ref)) / max(float(np.max(np.abs(ref))), 1e-300))


class DeviceLayer:
    """Inputs of one projection on the GPU plus the output buffers, sentinel-filled.  With
    transposed=True the weight, the adapter tables and the adapter gradients live on the device as
    transposes (LAYOUT_OUT_IN); the host-side tensors in `t` keep the paper's layout."""

    def __init__(self, w: wl.Workload, t: wl.Tensors, ctx: binding.Context, proj_index: int = 0,
                 dy_poison_inference: bool = True, transposed: bool = False):
        import torch

        self.w, self.t, self.ctx = w, t, ctx
        self.layout = binding.LAYOUT_OUT_IN if transposed else binding.LAYOUT_IN_OUT
        tp = (lambda a: np.ascontiguousarray(np.asarray(a).T)) if transposed else (lambda a: a)
        p = w.projections[proj_index]
        self.p = p
        dt = w.dtype
        self.tdtype = torch.bfloat16 if dt == "bf16" else torch.float32
        self.x = to_dev(t.x, dt)
        self.W = to_dev(tp(t.W), dt)
        self.A = [to_dev(tp(a), dt) for a in t.A]
        self.B = [to_dev(tp(b), dt) for b in t.B]
        _, self.tok_adapter, self.tok_train = oracle.token_map(w.seg_start, w.seg_adapter, w.seg_is_train)
        dy = np.array(t.dy, dtype=np.float32)
        if dy_poison_inference:
            dy[self.tok_train == 0] = np.nan  # rows of inference tokens must never be read
        self.dy = to_dev(dy, dt)
        T = w.n_tokens
        self.y = torch.full((T, p.d_out), float("nan"), dtype=self.tdtype, device="cuda")
        self.dx = torch.full((T, p.d_in), float("nan"), dtype=self.tdtype, device="cuda")
        self.h_save = torch.full((T, ctx.max_rank), float("nan"), dtype=torch.float32, device="cuda")
        sh = (lambda a, b: (b, a)) if transposed else (lambda a, b: (a, b))
        self.dA = [torch.full(sh(p.d_in, int(r)), float("nan"), dtype=torch.float32, device="cuda") for r in w.ranks]
        self.dB = [torch.full(sh(int(r), p.d_out), float("nan"), dtype=torch.float32, device="cuda") for r in w.ranks]

    def fwd(self, h_save=True):
        w = self.w
        self.ctx.collm_lora_linear_fwd(self.x, self.W, self.A, self.B, w.ranks, w.seg_start, w.seg_adapter,
                                       w.seg_is_train, w.scale, self.y, self.h_save if h_save else None,
                                       layout=self.layout)

    def bwd(self, h_save=True, accumulate=False, dx=True, dab=True):
        w = self.w
        self.ctx.collm_lora_linear_bwd(self.x, self.W, self.A, self.B, w.ranks, w.seg_start, w.seg_adapter,
                                       w.seg_is_train, w.scale, self.dy, self.h_save if h_save else None,
                                       self.dx if dx else None, self.dA if dab else None,
                                       self.dB if dab else None, accumulate, layout=self.layout)


def make_ctx(w: wl.Workload, max_rank=None) -> binding.Context:
    d = max(max(p.d_in, p.d_out) for p in w.projections)
    mr = int(max_rank if max_rank is not None else max(int(w.ranks.max()) if len(w.ranks) else 1, 1))
    return binding.Context(max(w.n_tokens, 1), max(w.n_segments, 1), max(w.n_adapters, 0), mr, d)


def check_full(layer: DeviceLayer, tol: float, check_h=True):
    """Element-by-element comparison of every output with the oracle (small problems)."""
    import torch

    w, t = layer.w, layer.t
    torch.cuda.synchronize()
    ta, tt = layer.tok_adapter, layer.tok_train
    y_ref, h_ref = oracle.lora_linear_fwd(t.x, t.W, t.A, t.B, ta, w.scale)
    dy = np.array(t.dy, dtype=np.float64)
    dx_ref, dA_ref, dB_ref = oracle.lora_linear_bwd(t.x, t.W, t.A, t.B, ta, tt, w.scale, dy)
    errs = {}
    y = to_host(layer.y)
    assert np.all(np.isfinite(y)), "y has unwritten or non-finite entries"
    errs["y"] = maxrel(y, y_ref)
    tr = tt != 0
    dx = to_host(layer.dx)
    assert np.all(np.isnan(dx[~tr])), "dx rows of inference tokens were written"
    if tr.any():
        assert np.all(np.isfinite(dx[tr]))
        errs["dx"] = maxrel(dx[tr], dx_ref[tr])
    if check_h:
        hs = to_host(layer.h_save)
        assert np.all(np.isnan(hs[~tr])), "h_save rows of inference tokens were written"
        if tr.any():
            href = np.zeros((int(tr.sum()), hs.shape[1]))
            href[:, : h_ref.shape[1]] = h_ref[tr]
            errs["h"] = maxrel(hs[tr], href)
            # beyond the adapter's rank the row is zero-filled
            for tok in np.flatnonzero(tr):
                assert np.all(hs[tok, w.ranks[ta[tok]]:] == 0.0)
    for a in range(w.n_adapters):
        dA, dB = to_host(layer.dA[a]), to_host(layer.dB[a])
        if layer.layout == binding.LAYOUT_OUT_IN:
            dA, dB = dA.T, dB.T
        if dA_ref[a] is None:
            assert np.all(np.isnan(dA)) and np.all(np.isnan(dB)), f"untrained adapter {a} was written"
        else:
            assert np.all(np.isfinite(dA)) and np.all(np.isfinite(dB))
            errs[f"dA{a}"] = maxrel(dA, dA_ref[a])
            errs[f"dB{a}"] = maxrel(dB, dB_ref[a])
    bad = {k: v for k, v in errs.items() if not v <= tol}
    assert not bad, f"beyond tolerance {tol}: {bad} (all: {errs})"
    return errs
