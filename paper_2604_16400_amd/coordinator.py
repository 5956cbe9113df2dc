"""Interference-aware batch sizing on measured timings of the mixed-batch LoRA layer (host logic).

The paper's Coordinator (section 5) fits, for a replica that runs fine-tuning and inference together,
two planes over the training batch size B and the inference batch size b,
    T_train(B, b) = a_t B + b_t b + c_t        T_infer(B, b) = a_i b + b_i B + c_i,
then for every candidate B takes the largest b whose predicted inference latency meets the latency
budget tau', and keeps the pair that maximises
    GOODPUT(B, b) = B / T_train(B, b) * (a p l + B0) / (a p l + B)
(throughput times the efficiency term with gradient noise p, loss reduction l, scaling constant a
and initial batch size B0).  Here B and b are the training and inference token counts of one
mixed batch and the latencies are those of this library's layer, measured on the GPU:
  * fused     one forward + backward call over the mixed batch (T_train = T_infer = the step);
  * streams   the paper's own arrangement: the inference tokens as one forward call on one stream,
              the training tokens as forward + backward on another, sharing W and the adapters.
`python -m paper_2604_16400_amd.coordinator` measures both over a grid of (B, b), fits the planes and
prints the chosen pair as JSON.  The fitting and the search need no GPU.
"""
from __future__ import annotations

import json
import sys
import time
from dataclasses import dataclass
from typing import Iterable, Optional, Sequence, Tuple

import numpy as np


@dataclass
class LatencyModel:
    """T(B, b) = own * (own batch) + other * (other batch) + const, as in the paper's two planes."""
    coef_B: float
    coef_b: float
    const: float

    def __call__(self, B, b):
        return self.coef_B * B + self.coef_b * b + self.const


def fit_latency_model(B: Sequence[float], b: Sequence[float], T: Sequence[float]) -> Tuple[LatencyModel, float]:
    """Least-squares plane through the samples (B_k, b_k, T_k); returns the model and R^2."""
    B, b, T = (np.asarray(v, dtype=np.float64) for v in (B, b, T))
    if not (B.shape == b.shape == T.shape) or B.ndim != 1 or B.size < 3:
        raise ValueError("need at least three samples (B, b, T) of equal length")
    X = np.stack([B, b, np.ones_like(B)], axis=1)
    coef, *_ = np.linalg.lstsq(X, T, rcond=None)
    resid = T - X @ coef
    tot = T - T.mean()
    r2 = 1.0 - float(resid @ resid) / float(tot @ tot) if float(tot @ tot) > 0 else 1.0
    return LatencyModel(float(coef[0]), float(coef[1]), float(coef[2])), r2


def infer_batch_limit(infer: LatencyModel, B: float, tau: float, b_max: int) -> int:
    """b*(B): the largest inference batch 0 <= b <= b_max with T_infer(B, b) <= tau (-1 if none)."""
    ok = lambda b: infer.coef_B * B + infer.coef_b * b + infer.const <= tau
    if infer.coef_b <= 0:
        # (a plane fitted to noisy timings may slope the wrong way: the largest batch is then the easiest one)
        return int(b_max) if ok(b_max) else -1
    if not ok(0):
        return -1
    b = int(min(b_max, max(0.0, np.floor((tau - infer.coef_B * B - infer.const) / infer.coef_b))))
    # the division is only a first guess: settle on the predicate itself
    while b < b_max and ok(b + 1):
        b += 1
    while b > 0 and not ok(b):
        b -= 1
    return b


def goodput(train: LatencyModel, B: float, b: float, a: float, p: float, l: float, B0: float) -> float:
    if B <= 0:
        return 0.0
    t = train(B, b)
    if t <= 0:
        return 0.0
    return (B / t) * (a * p * l + B0) / (a * p * l + B)


def choose_batch_sizes(train: LatencyModel, infer: LatencyModel, tau: float, B_grid: Iterable[int], b_max: int,
                       a: float, p: float, l: float, B0: float) -> Optional[Tuple[int, int, float]]:
    """(B*, b*, goodput): grid search over B with b = b*(B); None when no B meets the budget.
    Ties go to the smaller B (first in grid order)."""
    best = None
    for B in B_grid:
        bs = infer_batch_limit(infer, B, tau, b_max)
        if bs < 0:
            continue
        g = goodput(train, B, bs, a, p, l, B0)
        if best is None or g > best[2]:
            best = (int(B), int(bs), float(g))
    return best


# ---------------------------------------------------------------------------------------------
# measurement on the GPU
# ---------------------------------------------------------------------------------------------
def _make_batch(n_train: int, n_infer: int, n_adapters: int, rank: int, seed: int):
    """Segment table of a mixed batch: n_infer decode tokens (adapter round-robin), then one training
    segment of n_train tokens on adapter 0."""
    lens = [1] * n_infer + ([n_train] if n_train > 0 else [])
    adapters = [i % n_adapters for i in range(n_infer)] + ([0] if n_train > 0 else [])
    train = [0] * n_infer + ([1] if n_train > 0 else [])
    seg_start = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    return seg_start, np.asarray(adapters, np.int32), np.asarray(train, np.uint8)


def measure(d_in=8192, d_out=8192, n_adapters=16, rank=16, B_grid=(1024, 2048, 4096, 8192),
            b_grid=(256, 1024, 2048, 4096), iters=20, log=None):
    """Latencies of the layer over a grid of (B, b).  The layer and the batches are large enough that the GPU,
    not the host that enqueues the calls (about 60 us per call), sets the time."""
    import torch

    from . import binding

    dev = "cuda"
    g = torch.Generator(device=dev)
    g.manual_seed(20260416)
    rn = lambda shape, std: (torch.randn(shape, generator=g, device=dev) * std).to(torch.bfloat16)
    T_max = max(B_grid) + max(b_grid)
    W = rn((d_in, d_out), 0.02)
    A = binding.PointerTable([rn((d_in, rank), d_in ** -0.5) for _ in range(n_adapters)])
    Bt = binding.PointerTable([rn((rank, d_out), 0.01) for _ in range(n_adapters)])
    dA = binding.PointerTable([torch.empty((d_in, rank), device=dev) for _ in range(n_adapters)])
    dB = binding.PointerTable([torch.empty((rank, d_out), device=dev) for _ in range(n_adapters)])
    ranks = np.full(n_adapters, rank, np.int32)
    x, dy = rn((T_max, d_in), 1.0), rn((T_max, d_out), 1.0)
    y, dx = torch.empty_like(dy), torch.empty_like(x)
    h = torch.empty((T_max, rank), device=dev)
    ctx_f = binding.Context(T_max, T_max + 1, n_adapters, rank, max(d_in, d_out))
    ctx_t = binding.Context(T_max, T_max + 1, n_adapters, rank, max(d_in, d_out))
    ctx_i = binding.Context(T_max, T_max + 1, n_adapters, rank, max(d_in, d_out))
    s_train, s_infer = torch.cuda.Stream(), torch.cuda.Stream()

    def fused(nB, nb):
        ss, sa, st = _make_batch(nB, nb, n_adapters, rank, 0)
        T = nB + nb
        ctx_f.collm_lora_linear_fwd(x[:T], W, A, Bt, ranks, ss, sa, st, 2.0, y[:T], h[:T])
        ctx_f.collm_lora_linear_bwd(x[:T], W, A, Bt, ranks, ss, sa, st, 2.0, dy[:T], h[:T], dx[:T], dA, dB, False)

    def train_only(nB, stream):
        ss, sa, st = _make_batch(nB, 0, n_adapters, rank, 0)
        ctx_t.collm_lora_linear_fwd(x[:nB], W, A, Bt, ranks, ss, sa, st, 2.0, y[:nB], h[:nB], stream=stream)
        ctx_t.collm_lora_linear_bwd(x[:nB], W, A, Bt, ranks, ss, sa, st, 2.0, dy[:nB], h[:nB], dx[:nB], dA, dB, False,
                                    stream=stream)

    def infer_only(nB, nb, stream):
        ss, sa, st = _make_batch(0, nb, n_adapters, rank, 0)
        ctx_i.collm_lora_linear_fwd(x[nB:nB + nb], W, A, Bt, ranks, ss, sa, st, 2.0, y[nB:nB + nb], None, stream=stream)

    def wall(fn):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(iters):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / iters

    # the HIP runtime stalls once, for tens of milliseconds, near a process's 1024th dispatch: get past it
    # (on every stream that will be used)
    for _ in range(150):
        fused(B_grid[0], b_grid[0])
        train_only(B_grid[0], s_train)
        infer_only(B_grid[0], b_grid[0], s_infer)
        infer_only(B_grid[0], b_grid[0], s_infer)
        infer_only(B_grid[0], b_grid[0], s_infer)
    torch.cuda.synchronize()
    rows = []
    for nB in B_grid:
        for nb in b_grid:
            t_fused = wall(lambda: fused(nB, nb))
            # two streams: every call is bracketed by events on its own stream while the other stream runs, so the
            # averages are the latencies of one training iteration and of one inference batch under contention
            for _ in range(3):
                train_only(nB, s_train)
                infer_only(nB, nb, s_infer)
            torch.cuda.synchronize()
            ev_t = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(iters)]
            ev_i = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(iters)]
            t0 = time.perf_counter()
            for k in range(iters):
                ev_t[k][0].record(s_train)
                train_only(nB, s_train)
                ev_t[k][1].record(s_train)
                ev_i[k][0].record(s_infer)
                infer_only(nB, nb, s_infer)
                ev_i[k][1].record(s_infer)
            torch.cuda.synchronize()
            t_both = (time.perf_counter() - t0) / iters
            t_train = sum(a.elapsed_time(b) for a, b in ev_t) * 1e-3 / iters
            t_infer = sum(a.elapsed_time(b) for a, b in ev_i) * 1e-3 / iters
            rows.append({"B": nB, "b": nb, "fused_s": t_fused, "streams_train_s": t_train, "streams_infer_s": t_infer,
                         "streams_both_s": t_both})
            if log:
                print(f"B={nB:5d} b={nb:5d} fused {t_fused*1e6:8.1f} us | two streams: train {t_train*1e6:8.1f} us "
                      f"infer {t_infer*1e6:8.1f} us, both {t_both*1e6:8.1f} us", file=log, flush=True)
    for c in (ctx_f, ctx_t, ctx_i):
        c.close()
    return rows


def main(argv=None):
    rows = measure(log=sys.stderr)
    Bv, bv = [r["B"] for r in rows], [r["b"] for r in rows]
    out = {"layer": "8192->8192 bf16, 16 adapters of rank 16; B = training tokens (one segment), b = decode tokens",
           "samples": rows, "models": {}}
    fits = {}
    for key in ("fused_s", "streams_train_s", "streams_infer_s"):
        m, r2 = fit_latency_model(Bv, bv, [r[key] for r in rows])
        fits[key] = m
        out["models"][key] = {"coef_B_us_per_token": m.coef_B * 1e6, "coef_b_us_per_token": m.coef_b * 1e6,
                              "const_us": m.const * 1e6, "r2": r2}
    # batch sizing with the paper's objective: budget = twice the latency of the smallest fused batch; p l and a
    # are inputs of the training job (here a p l = 2048, B0 = 1024)
    tau = 2.0 * min(r["fused_s"] for r in rows)
    grid = list(range(512, 8193, 256))
    for name, train, infer in (("fused", fits["fused_s"], fits["fused_s"]),
                               ("streams", fits["streams_train_s"],
                                LatencyModel(fits["streams_infer_s"].coef_B, fits["streams_infer_s"].coef_b,
                                             fits["streams_infer_s"].const))):
        best = choose_batch_sizes(train, infer, tau, grid, 4096, 1.0, 2048.0, 1.0, 1024.0)
        out["models"][name + "_choice"] = {"tau_us": tau * 1e6, "B": None if best is None else best[0],
                                           "b": None if best is None else best[1],
                                           "goodput_tokens_per_s": None if best is None else best[2]}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
