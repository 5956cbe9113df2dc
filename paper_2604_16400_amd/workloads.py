"""Seeded synthetic workloads for the mixed-batch LoRA linear layer.

This module only *draws inputs*: segment tables, adapter ranks and random tensors.  It holds
none of the layer's arithmetic and is the one module that both the GPU tests/benchmark and
the CPU oracle's tests may share.  numpy only (to_device, the upload helper, also uses torch).

The paper evaluates on ShareGPT / Alpaca request lengths replayed on Azure-Code and
Azure-Conv arrival traces (section 8.1) with LLaMA-3.1-8B and LLaMA-2-13B replicas.  None
of that data is used here; the five configurations below are synthetic stand-ins with the
same structure: LLaMA-shaped projection sizes, a mix of one-token decode segments, prefill
chunks with log-normal lengths and whole training sequences, and adapters picked uniformly
or by a Zipf law.  The inference batch b and the training batch B of the paper's
coordinator (section 5) appear here as the number of inference and training tokens.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Tuple

import numpy as np

BASE_SEED = 20260416


# --------------------------------------------------------------------------------------
# bf16 helpers (input preparation only: round-to-nearest-even of fp32 to 16 bits)
# --------------------------------------------------------------------------------------
def bf16_bits(a: np.ndarray) -> np.ndarray:
    """fp32 array -> uint16 array of bf16 bit patterns (round to nearest even)."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_widen(bits: np.ndarray) -> np.ndarray:
    """uint16 bf16 bit patterns -> the exactly equal fp32 values."""
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_round(a: np.ndarray) -> np.ndarray:
    """fp32 array -> fp32 array holding bf16-representable values."""
    return bf16_widen(bf16_bits(a))


def to_device(a: np.ndarray, dtype: str):
    """Host array -> tensor on the current GPU in the element type of a workload ("bf16": the
    array's values rounded to nearest even, which is exact for the tensors make_tensors draws)."""
    import torch

    if dtype == "bf16":
        bits = bf16_bits(a).view(np.int16)
        return torch.from_numpy(bits).view(torch.bfloat16).reshape(a.shape).cuda()
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


# --------------------------------------------------------------------------------------
@dataclass
class Projection:
    name: str
    d_in: int
    d_out: int


@dataclass
class Workload:
    name: str
    index: int                 # 1..5 for the five configurations, 0 for ad-hoc cases
    dtype: str                 # "f32" or "bf16"
    n_tokens: int
    ranks: np.ndarray          # int32 [N]
    scale: float
    seg_start: np.ndarray      # int32 [S+1]
    seg_adapter: np.ndarray    # int32 [S]
    seg_is_train: np.ndarray   # uint8 [S]
    projections: List[Projection]
    seed: int
    std_x: float = 1.0
    std_w: float = 0.02
    std_a: float | None = None  # None -> 1/sqrt(d_in)
    std_b: float = 0.01
    std_dy: float = 1.0
    notes: str = ""

    @property
    def n_adapters(self) -> int:
        return int(len(self.ranks))

    @property
    def n_segments(self) -> int:
        return int(len(self.seg_adapter))

    @property
    def n_train_tokens(self) -> int:
        lens = np.diff(self.seg_start)
        return int(lens[self.seg_is_train != 0].sum())

    def flops(self, proj: Projection) -> Tuple[float, float]:
        """Algorithmic flops (forward, backward) of one projection of this workload."""
        lens = np.diff(self.seg_start).astype(np.float64)
        r_seg = np.where(self.seg_adapter >= 0, self.ranks[np.maximum(self.seg_adapter, 0)], 0)
        r_seg = r_seg.astype(np.float64)
        tr = self.seg_is_train != 0
        f_fwd = 2.0 * self.n_tokens * proj.d_in * proj.d_out
        f_fwd += float((lens * 2.0 * r_seg).sum()) * (proj.d_in + proj.d_out)
        f_bwd = 2.0 * self.n_train_tokens * proj.d_in * proj.d_out
        f_bwd += float((lens[tr] * 4.0 * r_seg[tr]).sum()) * (proj.d_in + proj.d_out)
        return f_fwd, f_bwd


def _segments(lens, adapters, train):
    lens = np.asarray(lens, dtype=np.int64)
    seg_start = np.zeros(len(lens) + 1, dtype=np.int32)
    seg_start[1:] = np.cumsum(lens)
    return (seg_start, np.asarray(adapters, dtype=np.int32), np.asarray(train, dtype=np.uint8))


def _zipf_p(n: int, alpha: float) -> np.ndarray:
    p = (np.arange(n, dtype=np.float64) + 1.0) ** (-alpha)
    return p / p.sum()


def _lognormal_chunks(rng, total: int, mu: float, sigma: float, lo: int, hi: int) -> List[int]:
    """Chunk lengths drawn until `total` tokens are covered; the last one is cut to fit."""
    out: List[int] = []
    left = total
    while left > 0:
        n = int(np.clip(np.rint(rng.lognormal(mu, sigma)), lo, hi))
        n = min(n, left)
        out.append(n)
        left -= n
    if len(out) > 1 and out[-1] < lo:
        out[-2] += out[-1]
        out.pop()
    return out


def _largest_remainder(weights: np.ndarray, total: int, minimum: int) -> np.ndarray:
    """Integers >= minimum, proportional to `weights`, summing to exactly `total`."""
    n = len(weights)
    spare = total - minimum * n
    assert spare >= 0
    q = weights / weights.sum() * spare
    base = np.floor(q).astype(np.int64)
    rem = int(spare - base.sum())
    order = np.argsort(-(q - base), kind="stable")
    base[order[:rem]] += 1
    return base + minimum


def make_config(index: int) -> Workload:
    """The five benchmark configurations (1-based)."""
    seed = BASE_SEED + index
    rng = np.random.Generator(np.random.Philox(key=seed))
    if index == 1:
        ss, sa, st = _segments([20, 12, 32], [0, 3, 1], [0, 0, 1])
        return Workload("c1_fp32_256", 1, "f32", 64, np.full(4, 8, np.int32), 2.0, ss, sa, st,
                        [Projection("linear", 256, 256)], seed,
                        std_x=0.02, std_w=0.02, std_a=0.02, std_b=0.01,
                        notes="3 segments: 20 tok a0 inf, 12 tok a3 inf, 32 tok a1 train")
    if index == 2:
        dec = rng.integers(0, 16, size=256)
        train_adapter = int(rng.integers(0, 16))
        ss, sa, st = _segments([1] * 256 + [1792], list(dec) + [train_adapter], [0] * 256 + [1])
        return Workload("c2_llama7b_qproj", 2, "bf16", 2048, np.full(16, 16, np.int32), 2.0,
                        ss, sa, st, [Projection("q_proj", 4096, 4096)], seed,
                        notes="256 decode tokens + one 1792-token training segment")
    if index == 3:
        n_ad = 32
        p = _zipf_p(n_ad, 1.2)
        chunks = _lognormal_chunks(rng, 3072 - 256, 5.0, 1.0, 16, 1024)
        lens = [1] * 256 + chunks + [512, 512]
        n_inf = 256 + len(chunks)
        inf_ad = rng.choice(n_ad, size=n_inf, p=p)
        tr_ad = rng.choice(n_ad, size=2, replace=False, p=p)
        ss, sa, st = _segments(lens, list(inf_ad) + list(tr_ad), [0] * n_inf + [1, 1])
        return Workload("c3_llama7b_mlp", 3, "bf16", 4096, np.full(n_ad, 64, np.int32), 2.0,
                        ss, sa, st,
                        [Projection("gate_proj", 4096, 11008), Projection("up_proj", 4096, 11008),
                         Projection("down_proj", 11008, 4096)], seed,
                        notes="256 decode + lognormal(5,1) prefill chunks + 2x512 train")
    if index == 4:
        n_ad = 64
        p = _zipf_p(n_ad, 1.1)
        ranks = rng.choice(np.array([8, 16, 32, 128], dtype=np.int32), size=n_ad).astype(np.int32)
        n_train = 3 * 1024 + 205
        n_inf_tok = 8192 - n_train
        w = rng.lognormal(3.5, 1.0, size=96)
        chunks = _largest_remainder(w, n_inf_tok - 200, 2)
        lens = [1] * 200 + [int(c) for c in chunks] + [1024, 1024, 1024, 205]
        inf_ad = rng.choice(n_ad, size=296, p=p)
        tr_ad = rng.choice(n_ad, size=4, replace=False, p=p)
        ss, sa, st = _segments(lens, list(inf_ad) + list(tr_ad), [0] * 296 + [1] * 4)
        return Workload("c4_llama13b", 4, "bf16", 8192, ranks, 2.0, ss, sa, st,
                        [Projection("attn_proj", 5120, 5120), Projection("gate_up_proj", 5120, 13824)],
                        seed, notes="200 decode + 96 prefill + (3x1024+205) train, mixed ranks")
    if index == 5:
        n_ad = 128
        lens = [1] * 1024 + [256] * 28 + [2048] * 4
        inf_ad = rng.integers(0, n_ad, size=1024 + 28)
        tr_ad = rng.choice(n_ad, size=4, replace=False)
        ss, sa, st = _segments(lens, list(inf_ad) + list(tr_ad), [0] * 1052 + [1] * 4)
        return Workload("c5_llama70b", 5, "bf16", 16384, np.full(n_ad, 16, np.int32), 2.0,
                        ss, sa, st,
                        [Projection("o_proj", 8192, 8192), Projection("kv_proj", 8192, 1024),
                         Projection("gate_up_proj", 8192, 28672)], seed,
                        notes="1024 decode + 28x256 prefill + 4x2048 train")
    raise ValueError("config index must be 1..5")


def make_adhoc(name: str, dtype: str, d_in: int, d_out: int, ranks, lens, adapters, train,
               scale: float = 2.0, seed: int = 1234, **std) -> Workload:
    """A hand-specified segmentation (edge-case and parity tests)."""
    ss, sa, st = _segments(lens, adapters, train)
    return Workload(name, 0, dtype, int(ss[-1]), np.asarray(ranks, dtype=np.int32), scale,
                    ss, sa, st, [Projection("linear", d_in, d_out)], seed, **std)


def shuffled_segments(w: Workload, seed: int):
    """The same segments in a random order (order-invariance checks).  Returns the new
    workload and `tok_perm` such that new token t is old token tok_perm[t]."""
    rng = np.random.Generator(np.random.Philox(key=seed))
    perm = rng.permutation(w.n_segments)
    lens = np.diff(w.seg_start)[perm]
    ss, sa, st = _segments(lens, w.seg_adapter[perm], w.seg_is_train[perm])
    tok_perm = np.concatenate(
        [np.arange(w.seg_start[k], w.seg_start[k + 1], dtype=np.int64) for k in perm]
        + [np.zeros(0, dtype=np.int64)])
    ws = Workload(w.name + "_shuffled", w.index, w.dtype, w.n_tokens, w.ranks, w.scale, ss, sa,
                  st, w.projections, w.seed, w.std_x, w.std_w, w.std_a, w.std_b, w.std_dy,
                  w.notes)
    return ws, tok_perm


# --------------------------------------------------------------------------------------
@dataclass
class Tensors:
    """Inputs of one projection.  Every array is fp32; for a bf16 workload every value is
    bf16-representable, so both sides of a parity test start from identical numbers."""
    x: np.ndarray
    W: np.ndarray
    A: List[np.ndarray] = field(default_factory=list)
    B: List[np.ndarray] = field(default_factory=list)
    dy: np.ndarray | None = None


def _normal(seed: int, stream: int, shape, std: float, bf16: bool) -> np.ndarray:
    rng = np.random.Generator(np.random.Philox(key=seed, counter=[0, 0, stream, 0]))
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.float32)
    step = 1 << 24
    for lo in range(0, n, step):
        hi = min(n, lo + step)
        blk = rng.standard_normal(hi - lo, dtype=np.float32) * np.float32(std)
        out[lo:hi] = bf16_round(blk) if bf16 else blk
    return out.reshape(shape)


def make_tensors(w: Workload, proj_index: int = 0, with_dy: bool = True) -> Tensors:
    """x ~ N(0, std_x), W ~ N(0, std_w), A ~ N(0, 1/sqrt(d_in)), B ~ N(0, std_b),
    dy ~ N(0, std_dy); standard deviations, drawn in fp32 and (bf16 workloads) rounded."""
    p = w.projections[proj_index]
    bf = w.dtype == "bf16"
    seed = w.seed * 16 + proj_index
    std_a = w.std_a if w.std_a is not None else 1.0 / np.sqrt(p.d_in)
    t = Tensors(
        x=_normal(seed, 1, (w.n_tokens, p.d_in), w.std_x, bf),
        W=_normal(seed, 2, (p.d_in, p.d_out), w.std_w, bf),
    )
    for a, r in enumerate(w.ranks):
        t.A.append(_normal(seed, 1000 + 2 * a, (p.d_in, int(r)), std_a, bf))
        t.B.append(_normal(seed, 1001 + 2 * a, (int(r), p.d_out), w.std_b, bf))
    if with_dy:
        t.dy = _normal(seed, 3, (w.n_tokens, p.d_out), w.std_dy, bf)
    return t


def sample_rows(w: Workload, seed: int = 0, interior: int = 2) -> np.ndarray:
    """Token rows on which the W-sized contractions are checked at full size: first and last
    token of every segment, `interior` random interior tokens per segment, and every token
    of the shortest training segment."""
    rng = np.random.Generator(np.random.Philox(key=w.seed * 7 + seed))
    rows = set()
    lens = np.diff(w.seg_start)
    for k in range(w.n_segments):
        lo, hi = int(w.seg_start[k]), int(w.seg_start[k + 1])
        if hi <= lo:
            continue
        rows.add(lo)
        rows.add(hi - 1)
        if hi - lo > 2:
            for t in rng.integers(lo + 1, hi - 1, size=interior):
                rows.add(int(t))
    tr = [k for k in range(w.n_segments) if w.seg_is_train[k] and lens[k] > 0]
    if tr:
        k = min(tr, key=lambda k: (lens[k], k))
        rows.update(range(int(w.seg_start[k]), int(w.seg_start[k + 1])))
    return np.array(sorted(rows), dtype=np.int64)
