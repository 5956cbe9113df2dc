"""CPU oracle for the mixed-batch LoRA linear layer -- TEST INFRASTRUCTURE ONLY.

Thin ctypes wrapper around ``collm_oracle.c`` (plain fp64 loops).  Only the tests, the
smoke check and the benchmark's CPU-baseline leg may import this package; the GPU library
and its Python binding never do, and this package imports nothing from them.

The operation is the LoRA-instrumented linear layer of the paper's section 4.2
(frozen W_pre plus Delta W = B_g A_g) evaluated on one batch that mixes inference and
training segments sharing one weight copy (section 2.1, "model sharing").  Row-vector
convention: ``x [T, d_in]``, ``W [d_in, d_out]``, ``A[a] [d_in, r_a]``, ``B[a] [r_a, d_out]``.

Pins (tests/test_oracle_pins.py): a hand-worked one-token example, numpy's matmul for the
base term and for the merged weight X (W + s A B), segment independence, permutation
invariance, closed-form gradients, and central finite differences.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "collm_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None

_f64p = ctypes.POINTER(ctypes.c_double)
_i32p = ctypes.POINTER(ctypes.c_int32)
_u8p = ctypes.POINTER(ctypes.c_uint8)


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (OpenMP over independent tokens / output entries)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-o", tmp, _SRC]
        )
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.oracle_num_threads.restype = ctypes.c_int
    return _lib


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float64)


def _ptr_table(arrs):
    tab = (ctypes.c_void_p * max(1, len(arrs)))()
    for k, a in enumerate(arrs):
        tab[k] = None if a is None else a.ctypes.data
    return tab


def token_map(seg_start, seg_adapter, seg_is_train):
    """Per-token (segment, adapter, is_train) arrays from the segment description."""
    seg_start = np.ascontiguousarray(seg_start, dtype=np.int32)
    seg_adapter = np.ascontiguousarray(seg_adapter, dtype=np.int32)
    seg_is_train = np.ascontiguousarray(seg_is_train, dtype=np.uint8)
    S = len(seg_adapter)
    T = int(seg_start[S]) if S > 0 else 0
    tok_seg = np.full(T, -7, dtype=np.int32)
    tok_adapter = np.full(T, -7, dtype=np.int32)
    tok_train = np.full(T, 7, dtype=np.uint8)
    _load().oracle_token_map(
        ctypes.c_int32(S),
        seg_start.ctypes.data_as(_i32p),
        seg_adapter.ctypes.data_as(_i32p),
        seg_is_train.ctypes.data_as(_u8p),
        tok_seg.ctypes.data_as(_i32p),
        tok_adapter.ctypes.data_as(_i32p),
        tok_train.ctypes.data_as(_u8p),
    )
    return tok_seg, tok_adapter, tok_train


def base_matmul(x, W):
    x, W = _f64(x), _f64(W)
    T, d_in = x.shape
    d_out = W.shape[1]
    assert W.shape[0] == d_in
    y = np.empty((T, d_out), dtype=np.float64)
    _load().oracle_base_matmul(
        ctypes.c_int32(T), ctypes.c_int32(d_in), ctypes.c_int32(d_out),
        x.ctypes.data_as(_f64p), W.ctypes.data_as(_f64p), y.ctypes.data_as(_f64p),
    )
    return y


def lora_linear_fwd(x, W, A, B, tok_adapter, scale):
    """Returns (y [T, d_out], h [T, r_max]) in fp64; h = x A_a, unscaled."""
    x, W = _f64(x), _f64(W)
    A = [_f64(a) for a in A]
    B = [_f64(b) for b in B]
    T, d_in = x.shape
    d_out = W.shape[1]
    assert W.shape[0] == d_in
    rank = np.array([a.shape[1] for a in A], dtype=np.int32)
    for a, b, r in zip(A, B, rank):
        assert a.shape == (d_in, r) and b.shape == (r, d_out)
    tok_adapter = np.ascontiguousarray(tok_adapter, dtype=np.int32)
    assert tok_adapter.shape == (T,)
    assert tok_adapter.size == 0 or (tok_adapter.min() >= -1 and tok_adapter.max() < len(A))
    rmax = int(rank.max()) if len(rank) else 1
    y = np.empty((T, d_out), dtype=np.float64)
    h = np.empty((T, rmax), dtype=np.float64)
    _load().oracle_lora_linear_fwd(
        ctypes.c_int32(T), ctypes.c_int32(d_in), ctypes.c_int32(d_out),
        x.ctypes.data_as(_f64p), W.ctypes.data_as(_f64p),
        _ptr_table(A), _ptr_table(B),
        rank.ctypes.data_as(_i32p), tok_adapter.ctypes.data_as(_i32p),
        ctypes.c_double(scale), y.ctypes.data_as(_f64p), h.ctypes.data_as(_f64p),
        ctypes.c_int32(rmax),
    )
    return y, h


def lora_linear_bwd(x, W, A, B, tok_adapter, tok_is_train, scale, dy, want_dx=True,
                    want_dab=True):
    """Returns (dx or None, dA list, dB list).

    dx rows of inference tokens are NaN (never written); dA[a]/dB[a] is None for an adapter
    without a training token.
    """
    x = _f64(x)
    A = [_f64(a) for a in A]
    B = [_f64(b) for b in B]
    dy = _f64(dy)
    T, d_in = x.shape
    d_out = dy.shape[1]
    rank = np.array([a.shape[1] for a in A], dtype=np.int32)
    tok_adapter = np.ascontiguousarray(tok_adapter, dtype=np.int32)
    tok_is_train = np.ascontiguousarray(tok_is_train, dtype=np.uint8)
    assert tok_adapter.shape == (T,) and tok_is_train.shape == (T,) and dy.shape[0] == T
    trained = sorted(set(int(a) for a in tok_adapter[tok_is_train != 0]))
    assert all(0 <= a < len(A) for a in trained), "training tokens need an adapter"
    dx = None
    Wp = None
    if want_dx:
        W = _f64(W)
        assert W.shape == (d_in, d_out)
        Wp = W.ctypes.data_as(_f64p)
        dx = np.full((T, d_in), np.nan, dtype=np.float64)
    dA = [None] * len(A)
    dB = [None] * len(A)
    if want_dab:
        for a in trained:
            dA[a] = np.full((d_in, rank[a]), np.nan, dtype=np.float64)
            dB[a] = np.full((rank[a], d_out), np.nan, dtype=np.float64)
    _load().oracle_lora_linear_bwd(
        ctypes.c_int32(T), ctypes.c_int32(d_in), ctypes.c_int32(d_out), ctypes.c_int32(len(A)),
        x.ctypes.data_as(_f64p), Wp, _ptr_table(A), _ptr_table(B),
        rank.ctypes.data_as(_i32p), tok_adapter.ctypes.data_as(_i32p),
        tok_is_train.ctypes.data_as(_u8p), ctypes.c_double(scale),
        dy.ctypes.data_as(_f64p),
        None if dx is None else dx.ctypes.data_as(_f64p),
        _ptr_table(dA) if want_dab else None,
        _ptr_table(dB) if want_dab else None,
    )
    return dx, dA, dB


# ---------------------------------------------------------------------------------------------
# The step after the backward pass: update of the trained adapter tables and their aggregation.
# ---------------------------------------------------------------------------------------------
def _sibling_slices(A, B, d_outs):
    """Column ranges of the siblings in W / B_i, and for every sibling the adapters' own tables."""
    P = len(d_outs)
    cols = np.concatenate([[0], np.cumsum(d_outs)]).astype(int)
    per = []
    for j in range(P):
        Aj, Bj = [], []
        for a, b in zip(A, B):
            r = b.shape[0]
            assert a.shape[1] == P * r and b.shape[1] == cols[-1]
            Aj.append(np.ascontiguousarray(a[:, j * r:(j + 1) * r]))
            Bj.append(np.ascontiguousarray(b[:, cols[j]:cols[j + 1]]))
        per.append((Aj, Bj))
    return cols, per


def lora_siblings_fwd(x, W, A, B, d_outs, tok_adapter, scale):
    """Sibling projections of the same x stored side by side (W [d_in, D], A_i [d_in, P r_i], B_i [r_i, D]):
    each sibling is a LoRA projection of its own (paper section 4.2, applied per projection), so the result
    is the per-projection forward on the sibling's slices, written into its columns.  Returns
    (y [T, D], h [T, P r_max]); a row of h holds sibling j's x A_j in columns j r_a .. (j + 1) r_a, r_a the
    rank of the token's adapter, and zeros elsewhere."""
    x, W = _f64(x), _f64(W)
    A = [_f64(a) for a in A]
    B = [_f64(b) for b in B]
    cols, per = _sibling_slices(A, B, d_outs)
    P, T = len(d_outs), x.shape[0]
    rmax = max([b.shape[0] for b in B], default=1)
    y = np.empty((T, cols[-1]))
    h = np.zeros((T, P * rmax))
    tok_adapter = np.asarray(tok_adapter)
    for j, (Aj, Bj) in enumerate(per):
        yj, hj = lora_linear_fwd(x, np.ascontiguousarray(W[:, cols[j]:cols[j + 1]]), Aj, Bj, tok_adapter, scale)
        y[:, cols[j]:cols[j + 1]] = yj
        for t in range(T):
            a = tok_adapter[t]
            if a >= 0:
                r = B[a].shape[0]
                h[t, j * r:(j + 1) * r] = hj[t, :r]
    return y, h


def lora_siblings_bwd(x, W, A, B, d_outs, tok_adapter, tok_is_train, scale, dy):
    """Backward of lora_siblings_fwd: every sibling's per-projection backward on its slices; dx is the sum over
    the siblings (x feeds all of them), dA_i and dB_i are assembled in the layout of A_i and B_i."""
    x, W, dy = _f64(x), _f64(W), _f64(dy)
    A = [_f64(a) for a in A]
    B = [_f64(b) for b in B]
    cols, per = _sibling_slices(A, B, d_outs)
    dx = None
    dA = [None] * len(A)
    dB = [None] * len(B)
    for j, (Aj, Bj) in enumerate(per):
        sl = slice(cols[j], cols[j + 1])
        dxj, dAj, dBj = lora_linear_bwd(x, np.ascontiguousarray(W[:, sl]), Aj, Bj, tok_adapter, tok_is_train, scale,
                                        np.ascontiguousarray(dy[:, sl]))
        dx = dxj if dx is None else dx + dxj
        for i in range(len(A)):
            if dAj[i] is None:
                continue
            r = B[i].shape[0]
            if dA[i] is None:
                dA[i] = np.zeros_like(A[i])
                dB[i] = np.zeros_like(B[i])
            dA[i][:, j * r:(j + 1) * r] = dAj[i]
            dB[i][:, sl] = dBj[i]
    return dx, dA, dB


def swiglu(pre):
    """Gated activation of a gate/up pair stored side by side (pre [T, 2 d_ff]: gate columns, then up columns):
    out[t, j] = silu(g) u with silu(g) = g / (1 + exp(-g)) (Shazeer 2020, the SwiGLU feed-forward variant of the
    Llama models the paper serves)."""
    pre = _f64(pre)
    d = pre.shape[1] // 2
    g, u = pre[:, :d], pre[:, d:]
    return g / (1.0 + np.exp(-g)) * u


def swiglu_bwd(pre, dout):
    """Gradient of swiglu with respect to pre: [dL/dg | dL/du] from dout = dL/dout, term by term:
    d silu / dg = sigma(g) (1 + g (1 - sigma(g)))."""
    pre, dout = _f64(pre), _f64(dout)
    d = pre.shape[1] // 2
    g, u = pre[:, :d], pre[:, d:]
    sg = 1.0 / (1.0 + np.exp(-g))
    return np.concatenate([dout * u * sg * (1.0 + g * (1.0 - sg)), dout * g * sg], axis=1)


def adapter_fedavg(copies) -> np.ndarray:
    """Aggregation of the adapter copies of the |K| participating replicas (paper section 4.2, the
    equation for the aggregated B and A): the element-wise mean, copies added in index order."""
    copies = [_f64(c) for c in copies]
    assert len(copies) >= 1 and all(c.shape == copies[0].shape for c in copies)
    acc = np.zeros_like(copies[0])
    for c in copies:
        acc = acc + c
    return acc / float(len(copies))


def adamw_step(p, g, m, v, lr, beta1, beta2, eps, weight_decay, step):
    """One AdamW update (Loshchilov & Hutter 2019, decoupled weight decay, bias-corrected moments) of
    one adapter table in fp64.  The paper trains only the adapters (section 4.2) and keeps "gradients
    and optimizer state" with the fine-tuning task (section 2.1) without naming the optimizer; AdamW
    is this library's reading.  `step` counts from 1.  Returns (p, m, v)."""
    p, g, m, v = _f64(p).copy(), _f64(g), _f64(m).copy(), _f64(v).copy()
    assert step >= 1
    it = np.nditer([p, g, m, v], op_flags=[["readwrite"], ["readonly"], ["readwrite"], ["readwrite"]])
    c1 = 1.0 - beta1 ** step
    c2 = 1.0 - beta2 ** step
    for pi, gi, mi, vi in it:
        gval = float(gi)
        m_new = beta1 * float(mi) + (1.0 - beta1) * gval
        v_new = beta2 * float(vi) + (1.0 - beta2) * gval * gval
        p_dec = float(pi) * (1.0 - lr * weight_decay)
        denom = (v_new ** 0.5) / (c2 ** 0.5) + eps
        pi[...] = p_dec - (lr / c1) * m_new / denom
        mi[...] = m_new
        vi[...] = v_new
    return p, m, v


# ---------------------------------------------------------------------------------------------
# The Coordinator's batch sizing (paper section 5), written out step by step.
# ---------------------------------------------------------------------------------------------
def fit_plane(B, b, T):
    """Least-squares plane T ~ c0 B + c1 b + c2: normal equations solved by Gaussian elimination with
    partial pivoting, in fp64 loops."""
    B, b, T = [float(v) for v in B], [float(v) for v in b], [float(v) for v in T]
    n = len(T)
    cols = [B, b, [1.0] * n]
    M = [[sum(cols[i][k] * cols[j][k] for k in range(n)) for j in range(3)] + [sum(cols[i][k] * T[k] for k in range(n))]
         for i in range(3)]
    for c in range(3):
        piv = max(range(c, 3), key=lambda r: abs(M[r][c]))
        M[c], M[piv] = M[piv], M[c]
        for r in range(c + 1, 3):
            f = M[r][c] / M[c][c]
            for k in range(c, 4):
                M[r][k] -= f * M[c][k]
    sol = [0.0, 0.0, 0.0]
    for c in (2, 1, 0):
        sol[c] = (M[c][3] - sum(M[c][k] * sol[k] for k in range(c + 1, 3))) / M[c][c]
    return tuple(sol)


def coordinator_choice(train, infer, tau, B_grid, b_max, a, p, l, B0):
    """(B*, b*, goodput) by brute force.  `train` = (coefficient of B, of b, constant) of T_train,
    `infer` the same triple of T_infer (coefficient of B first).  For every B of the grid, b*(B) is found
    by trying every b from b_max down to 0; GOODPUT = B / T_train(B, b*) * (a p l + B0) / (a p l + B);
    the first B with the largest GOODPUT wins; None if no (B, b) meets the budget."""
    best = None
    for B in B_grid:
        b_star = None
        for b in range(int(b_max), -1, -1):
            if infer[0] * B + infer[1] * b + infer[2] <= tau:
                b_star = b
                break
        if b_star is None:
            continue
        t_train = train[0] * B + train[1] * b_star + train[2]
        g = 0.0 if (B <= 0 or t_train <= 0) else (B / t_train) * (a * p * l + B0) / (a * p * l + B)
        if best is None or g > best[2]:
            best = (int(B), int(b_star), g)
    return best
