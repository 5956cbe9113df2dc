"""Python face of libcollm_lora.so: argument marshalling only.

Every step of the layer (plan, shrink, GEMM with fused expand, gradients) runs inside the
C-ABI library; this module turns torch tensors into pointers, sizes and a stream handle.
PyTorch is used for device memory and streams and for nothing else.  There is no fallback:
if the library cannot be loaded, or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcollm_lora.so")

COLLM_F32 = 0
COLLM_BF16 = 1
ACT_NONE, ACT_SWIGLU = 0, 1
LAYOUT_IN_OUT, LAYOUT_OUT_IN = 0, 1  # W [d_in, d_out] (paper, row vectors) / W [d_out, d_in] (module weights)

TILE_AUTO, TILE_256x256, TILE_128x128 = -1, 0, 2


class CollmError(RuntimeError):
    def __init__(self, status: int, where: str, detail: str = ""):
        self.status = status
        super().__init__(f"{where}: status {status} ({detail})")


class collm_shape(ctypes.Structure):
    _fields_ = [
        ("d_in", ctypes.c_int32), ("d_out", ctypes.c_int32), ("n_tokens", ctypes.c_int32),
        ("n_segments", ctypes.c_int32), ("n_adapters", ctypes.c_int32), ("dtype", ctypes.c_int32),
        ("scale", ctypes.c_float), ("layout", ctypes.c_int32),
    ]


class collm_siblings(ctypes.Structure):
    _fields_ = [("n_siblings", ctypes.c_int32), ("d_out", ctypes.c_int32 * 4), ("activation", ctypes.c_int32),
                ("pre_act", ctypes.c_void_p)]


class collm_adamw(ctypes.Structure):
    _fields_ = [
        ("lr", ctypes.c_float), ("beta1", ctypes.c_float), ("beta2", ctypes.c_float), ("eps", ctypes.c_float),
        ("weight_decay", ctypes.c_float), ("step", ctypes.c_int32),
    ]


_lib = None
_i32p = ctypes.POINTER(ctypes.c_int32)
_u8p = ctypes.POINTER(ctypes.c_uint8)
_vpp = ctypes.POINTER(ctypes.c_void_p)


def load_library(build_if_missing: bool = True) -> ctypes.CDLL:
    """Loads libcollm_lora.so (building it first only if it does not exist)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        if not build_if_missing:
            raise FileNotFoundError(LIB_PATH)
        from . import build as _build

        _build.build()
    try:
        # the HIP runtime PyTorch has loaded must be the one this library binds to
        import torch  # noqa: F401
    except Exception:  # pragma: no cover - torch is only needed for device memory
        pass
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, sp = ctypes.c_void_p, ctypes.c_int32, ctypes.POINTER(collm_shape)
    lib.collm_ctx_create.argtypes = [_vpp, ctypes.c_int, i32, i32, i32, i32, i32]
    lib.collm_ctx_create.restype = ctypes.c_int
    lib.collm_ctx_destroy.argtypes = [vp]
    lib.collm_ctx_destroy.restype = ctypes.c_int
    lib.collm_ctx_workspace_bytes.argtypes = [vp]
    lib.collm_ctx_workspace_bytes.restype = ctypes.c_int64
    lib.collm_status_string.argtypes = [ctypes.c_int]
    lib.collm_status_string.restype = ctypes.c_char_p
    lib.collm_last_error.argtypes = []
    lib.collm_last_error.restype = ctypes.c_char_p
    lib.collm_lora_linear_fwd.argtypes = [vp, sp, vp, vp, _vpp, _vpp, _i32p, _i32p, _i32p, _u8p, vp, vp, vp]
    lib.collm_lora_linear_fwd.restype = ctypes.c_int
    lib.collm_lora_linear_bwd.argtypes = [vp, sp, vp, vp, _vpp, _vpp, _i32p, _i32p, _i32p, _u8p, vp, vp, vp,
                                          _vpp, _vpp, ctypes.c_int, vp]
    lib.collm_lora_linear_bwd.restype = ctypes.c_int
    lib.collm_lora_linear_fwd_noalloc.argtypes = [ctypes.c_int, sp, vp, vp, _vpp, _vpp, _i32p, _i32p, _i32p, _u8p, vp, vp, vp]
    lib.collm_lora_linear_fwd_noalloc.restype = ctypes.c_int
    sbp = ctypes.POINTER(collm_siblings)
    lib.collm_lora_siblings_fwd.argtypes = [vp, sp, sbp, vp, vp, _vpp, _vpp, _i32p, _i32p, _i32p, _u8p, vp, vp, vp]
    lib.collm_lora_siblings_fwd.restype = ctypes.c_int
    lib.collm_lora_siblings_bwd.argtypes = [vp, sp, sbp, vp, vp, _vpp, _vpp, _i32p, _i32p, _i32p, _u8p, vp, vp, vp,
                                            _vpp, _vpp, ctypes.c_int, vp]
    lib.collm_lora_siblings_bwd.restype = ctypes.c_int
    lib.collm_swiglu_bwd.argtypes = [ctypes.c_int, i32, i32, i32, _i32p, _u8p, vp, vp, vp, vp]
    lib.collm_swiglu_bwd.restype = ctypes.c_int
    lib.collm_token_map.argtypes = [sp, _i32p, _i32p, _u8p, _i32p, _i32p, _u8p]
    lib.collm_token_map.restype = ctypes.c_int
    lib.collm_debug_device_token_map.argtypes = [vp, _i32p, _i32p, _u8p]
    lib.collm_debug_device_token_map.restype = ctypes.c_int
    lib.collm_debug_host_tiling.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, _i32p, _i32p, _i32p,
                                            _i32p]
    lib.collm_debug_host_tiling.restype = ctypes.c_int
    lib.collm_debug_host_tile_order.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, _i32p,
                                                _i32p, _i32p]
    lib.collm_debug_host_tile_order.restype = ctypes.c_int
    lib.collm_debug_host_row_order.argtypes = [sp, _i32p, _i32p, _i32p, _u8p, ctypes.c_int, ctypes.c_int, _i32p, _i32p]
    lib.collm_debug_host_row_order.restype = ctypes.c_int
    lib.collm_debug_set_tiles.argtypes = [vp, ctypes.c_int, ctypes.c_int]
    lib.collm_debug_set_tiles.restype = ctypes.c_int
    lib.collm_debug_set_gemm_split.argtypes = [vp, ctypes.c_int]
    lib.collm_debug_set_gemm_split.restype = ctypes.c_int
    lib.collm_debug_set_wide_pass.argtypes = [vp, ctypes.c_int]
    lib.collm_debug_set_wide_pass.restype = ctypes.c_int
    lib.collm_debug_set_dual_pass.argtypes = [vp, ctypes.c_int]
    lib.collm_debug_set_dual_pass.restype = ctypes.c_int
    lib.collm_device_info.argtypes = [ctypes.c_int, _i32p, _i32p, _i32p, _i32p, ctypes.POINTER(ctypes.c_int64)]
    lib.collm_device_info.restype = ctypes.c_int
    lib.collm_debug_plan_stats.argtypes = [vp, ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_float), _i32p, _i32p]
    lib.collm_debug_plan_stats.restype = ctypes.c_int
    lib.collm_profile_enable.argtypes = [vp, ctypes.c_int]
    lib.collm_profile_enable.restype = ctypes.c_int
    lib.collm_profile_read.argtypes = [vp, ctypes.POINTER(ctypes.c_char_p), ctypes.POINTER(ctypes.c_float),
                                       ctypes.c_int]
    lib.collm_profile_read.restype = ctypes.c_int
    lib.collm_adapter_fedavg.argtypes = [ctypes.c_int, ctypes.c_int, i32, _vpp, vp, ctypes.c_int64, vp]
    lib.collm_adapter_fedavg.restype = ctypes.c_int
    lib.collm_adapter_adamw.argtypes = [ctypes.c_int, ctypes.c_int, vp, vp, vp, vp, vp, ctypes.c_int64,
                                        ctypes.POINTER(collm_adamw), vp]
    lib.collm_adapter_adamw.restype = ctypes.c_int
    _lib = lib
    return lib


def _check(status: int, where: str):
    if status != 0:
        lib = load_library()
        detail = lib.collm_status_string(status).decode()
        if status == -8 or where.endswith("_noalloc"):
            detail += ": " + lib.collm_last_error().decode()
        raise CollmError(status, where, detail)


def _seg_arrays(seg_start, seg_adapter, seg_is_train):
    ss = np.ascontiguousarray(seg_start, dtype=np.int32)
    sa = np.ascontiguousarray(seg_adapter, dtype=np.int32)
    st = np.ascontiguousarray(seg_is_train, dtype=np.uint8)
    if len(ss) != len(sa) + 1 or len(st) != len(sa):
        raise ValueError("seg_start needs S+1 entries, seg_adapter and seg_is_train S")
    return ss, sa, st


def collm_token_map(seg_start, seg_adapter, seg_is_train, n_tokens: Optional[int] = None,
                    n_adapters: int = 1 << 30):
    """Host-only integer bookkeeping: per-token (segment, adapter, is_train)."""
    lib = load_library()
    ss, sa, st = _seg_arrays(seg_start, seg_adapter, seg_is_train)
    T = int(ss[-1]) if n_tokens is None else int(n_tokens)
    sh = collm_shape(8, 8, T, len(sa), n_adapters, COLLM_BF16, 1.0, LAYOUT_IN_OUT)
    ts = np.full(max(T, 0), -9, np.int32)
    ta = np.full(max(T, 0), -9, np.int32)
    tt = np.full(max(T, 0), 9, np.uint8)
    _check(lib.collm_token_map(ctypes.byref(sh), ss.ctypes.data_as(_i32p), sa.ctypes.data_as(_i32p),
                               st.ctypes.data_as(_u8p), ts.ctypes.data_as(_i32p), ta.ctypes.data_as(_i32p),
                               tt.ctypes.data_as(_u8p)), "collm_token_map")
    return ts, ta, tt


def host_tiling(rows: int, cols: int, K: int, can_split: bool = True):
    """(tile, big_tiles_m, tail_tiles_m, tail_cols) the library would use for a GEMM of this size (host logic,
    no GPU)."""
    lib = load_library()
    out = [ctypes.c_int32(-9) for _ in range(4)]
    _check(lib.collm_debug_host_tiling(rows, cols, K, 1 if can_split else 0, *[ctypes.byref(o) for o in out]),
           "collm_debug_host_tiling")
    return tuple(o.value for o in out)


def host_tile_order(tile_rows: int, tiles_m: int, tiles_n: int, K: int, band: int = -1):
    """(band_used, tile_m, tile_n): the tile every workgroup id of a GEMM launch takes (host logic, no GPU)."""
    lib = load_library()
    used = ctypes.c_int32(-9)
    tm = np.empty(tiles_m * tiles_n, dtype=np.int32)
    tn = np.empty(tiles_m * tiles_n, dtype=np.int32)
    _check(lib.collm_debug_host_tile_order(tile_rows, tiles_m, tiles_n, K, band, ctypes.byref(used),
                                           tm.ctypes.data_as(_i32p), tn.ctypes.data_as(_i32p)),
           "collm_debug_host_tile_order")
    return used.value, tm, tn


def host_row_order(rank, seg_start, seg_adapter, seg_is_train, tile_rows: int = 256, training_rows_only: bool = False):
    """(row_tok, tile_steps) of the plan for this batch, built on the host (no GPU needed)."""
    lib = load_library()
    ss, sa, st = _seg_arrays(seg_start, seg_adapter, seg_is_train)
    rk = np.ascontiguousarray(rank, dtype=np.int32)
    T = int(ss[-1])
    sh = collm_shape(8, 8, T, len(sa), len(rk), COLLM_BF16, 1.0, LAYOUT_IN_OUT)
    row_tok = np.full(max(T, 1), -7, np.int32)
    steps = np.full((T + tile_rows - 1) // tile_rows + 1, -7, np.int32)
    n = lib.collm_debug_host_row_order(ctypes.byref(sh), rk.ctypes.data_as(_i32p), ss.ctypes.data_as(_i32p),
                                       sa.ctypes.data_as(_i32p), st.ctypes.data_as(_u8p), tile_rows,
                                       1 if training_rows_only else 0, row_tok.ctypes.data_as(_i32p),
                                       steps.ctypes.data_as(_i32p))
    _check(min(n, 0), "collm_debug_host_row_order")
    return row_tok[:n], steps[: (n + tile_rows - 1) // tile_rows]


def device_info(device: int = 0):
    """dict(compute_units, clock_mhz, memory_clock_mhz, memory_bus_bits, l2_bytes) of a GPU, as the runtime reports it."""
    lib = load_library()
    v = [ctypes.c_int32() for _ in range(4)]
    l2 = ctypes.c_int64()
    _check(lib.collm_device_info(device, *[ctypes.byref(x) for x in v], ctypes.byref(l2)), "collm_device_info")
    return {"compute_units": v[0].value, "clock_mhz": v[1].value / 1e3, "memory_clock_mhz": v[2].value / 1e3,
            "memory_bus_bits": v[3].value, "l2_bytes": l2.value}


class PointerTable:
    """A HOST array of device pointers built once from a list of tensors (entries may be
    None).  Passing the same PointerTable to many calls skips rebuilding the array; the
    tensors are kept alive by the table."""

    def __init__(self, tensors: Sequence):
        self.tensors = list(tensors)
        self.array = (ctypes.c_void_p * max(len(self.tensors), 1))()
        for i, t in enumerate(self.tensors):
            self.array[i] = None if t is None else t.data_ptr()

    def __len__(self):
        return len(self.tensors)


def _ptr_table(tensors, n: int):
    if isinstance(tensors, PointerTable):
        return tensors.array
    return PointerTable(tensors if tensors is not None else [None] * n).array


class Context:
    """Owns one collm_ctx (pinned staging + device workspace) on one GPU."""

    def __init__(self, max_tokens: int, max_segments: int, max_adapters: int, max_rank: int, max_d: int,
                 device: int = 0):
        self._lib = load_library()
        self._h = ctypes.c_void_p()
        self.max_rank = int(max_rank)
        _check(self._lib.collm_ctx_create(ctypes.byref(self._h), device, max_tokens, max_segments,
                                          max_adapters, max_rank, max_d), "collm_ctx_create")

    def close(self):
        if getattr(self, "_h", None) is not None and self._h.value:
            self._lib.collm_ctx_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @property
    def workspace_bytes(self) -> int:
        return int(self._lib.collm_ctx_workspace_bytes(self._h))

    def set_tiles(self, fwd_tile: int = TILE_AUTO, bwd_tile: int = TILE_AUTO):
        _check(self._lib.collm_debug_set_tiles(self._h, fwd_tile, bwd_tile), "collm_debug_set_tiles")

    def set_gemm_split(self, n_slices: int = -1):
        _check(self._lib.collm_debug_set_gemm_split(self._h, n_slices), "collm_debug_set_gemm_split")

    def set_wide_pass(self, min_rows: int = -1):
        _check(self._lib.collm_debug_set_wide_pass(self._h, min_rows), "collm_debug_set_wide_pass")

    def set_dual_pass(self, mode: int = -1):
        """-1: dh and dB from one pass over dy where that pays; 1: wherever it applies; 0: never."""
        _check(self._lib.collm_debug_set_dual_pass(self._h, mode), "collm_debug_set_dual_pass")

    def plan_stats(self):
        """Host cost of the plan of the last compute call: dict(build_us, upload_us, bytes, mode)."""
        b, u = ctypes.c_float(), ctypes.c_float()
        n, m = ctypes.c_int32(), ctypes.c_int32()
        _check(self._lib.collm_debug_plan_stats(self._h, ctypes.byref(b), ctypes.byref(u), ctypes.byref(n),
                                                ctypes.byref(m)), "collm_debug_plan_stats")
        return {"build_us": b.value, "upload_us": u.value, "bytes": n.value, "mode": m.value}

    def profile_enable(self, on: bool):
        _check(self._lib.collm_profile_enable(self._h, 1 if on else 0), "collm_profile_enable")

    def profile_read(self):
        names = (ctypes.c_char_p * 16)()
        ms = (ctypes.c_float * 16)()
        n = self._lib.collm_profile_read(self._h, names, ms, 16)
        if n < 0:
            _check(n, "collm_profile_read")
        return [(names[i].decode(), float(ms[i])) for i in range(n)]

    def device_token_map(self, n_tokens: int):
        ts = np.full(n_tokens, -9, np.int32)
        ta = np.full(n_tokens, -9, np.int32)
        tt = np.full(n_tokens, 9, np.uint8)
        _check(self._lib.collm_debug_device_token_map(self._h, ts.ctypes.data_as(_i32p),
                                                      ta.ctypes.data_as(_i32p), tt.ctypes.data_as(_u8p)),
               "collm_debug_device_token_map")
        return ts, ta, tt

    # ------------------------------------------------------------------------------------
    def _shape(self, x, W, n_seg, n_adapters, scale, layout):
        import torch

        if x.dtype == torch.bfloat16:
            dt = COLLM_BF16
        elif x.dtype == torch.float32:
            dt = COLLM_F32
        else:
            raise TypeError("x must be bfloat16 or float32")
        d_out = W.shape[0] if layout == LAYOUT_OUT_IN else W.shape[1]
        return collm_shape(int(x.shape[1]), int(d_out), int(x.shape[0]), n_seg, n_adapters, dt, float(scale),
                           int(layout))

    @staticmethod
    def _stream(stream):
        import torch

        s = torch.cuda.current_stream() if stream is None else stream
        return ctypes.c_void_p(s.cuda_stream)

    def collm_lora_linear_fwd(self, x, W, A: List, B: List, rank, seg_start, seg_adapter, seg_is_train,
                              scale: float, y, h_save=None, stream=None, layout: int = 0):
        """y <- x W + scale (x A_a) B_a per segment; h_save (optional) <- x A_a on training rows.
        layout LAYOUT_OUT_IN: W, A_a, B_a are given transposed ([d_out, d_in], [rank, d_in], [d_out, rank])."""
        ss, sa, st = _seg_arrays(seg_start, seg_adapter, seg_is_train)
        rk = np.ascontiguousarray(rank, dtype=np.int32)
        sh = self._shape(x, W, len(sa), len(rk), scale, layout)
        At, Bt = _ptr_table(A, len(rk)), _ptr_table(B, len(rk))
        _check(self._lib.collm_lora_linear_fwd(
            self._h, ctypes.byref(sh), x.data_ptr(), W.data_ptr(), At, Bt, rk.ctypes.data_as(_i32p),
            ss.ctypes.data_as(_i32p), sa.ctypes.data_as(_i32p), st.ctypes.data_as(_u8p), y.data_ptr(),
            None if h_save is None else h_save.data_ptr(), self._stream(stream)), "collm_lora_linear_fwd")
        return y

    def collm_lora_linear_bwd(self, x, W, A: List, B: List, rank, seg_start, seg_adapter, seg_is_train,
                              scale: float, dy, h_save=None, dx=None, dA: Optional[List] = None,
                              dB: Optional[List] = None, accumulate: bool = False, stream=None, layout: int = 0):
        """Training rows: dx <- dy W^T + dh A_a^T; dA_a, dB_a (fp32) summed over the adapter's tokens.
        layout LAYOUT_OUT_IN: W, A_a, B_a, dA_a, dB_a are all transposed."""
        ss, sa, st = _seg_arrays(seg_start, seg_adapter, seg_is_train)
        rk = np.ascontiguousarray(rank, dtype=np.int32)
        sh = self._shape(x, W, len(sa), len(rk), scale, layout)
        At, Bt = _ptr_table(A, len(rk)), _ptr_table(B, len(rk))
        dAt = _ptr_table(dA, len(rk)) if dA is not None else None
        dBt = _ptr_table(dB, len(rk)) if dB is not None else None
        _check(self._lib.collm_lora_linear_bwd(
            self._h, ctypes.byref(sh), x.data_ptr(), W.data_ptr(), At, Bt, rk.ctypes.data_as(_i32p),
            ss.ctypes.data_as(_i32p), sa.ctypes.data_as(_i32p), st.ctypes.data_as(_u8p), dy.data_ptr(),
            None if h_save is None else h_save.data_ptr(), None if dx is None else dx.data_ptr(),
            dAt, dBt, 1 if accumulate else 0, self._stream(stream)), "collm_lora_linear_bwd")


    @staticmethod
    def _siblings(d_outs, activation=0, pre_act=None):
        d = [int(v) for v in d_outs]
        if not 1 <= len(d) <= 4:
            raise ValueError("1 to 4 sibling projections")
        sb = collm_siblings()
        sb.n_siblings = len(d)
        for j, v in enumerate(d):
            sb.d_out[j] = v
        sb.activation = int(activation)
        sb.pre_act = None if pre_act is None else pre_act.data_ptr()
        return sb

    def collm_lora_siblings_fwd(self, d_outs, x, W, A: List, B: List, rank, seg_start, seg_adapter, seg_is_train,
                                scale: float, y, h_save=None, stream=None, activation: int = ACT_NONE, pre_act=None):
        """Sibling projections of x stored side by side (W [d_in, sum d_outs], A_i [d_in, P rank_i],
        B_i [rank_i, sum d_outs]): y[:, C_j] <- x W[:, C_j] + scale (x A_i,j) B_i[:, C_j].
        activation ACT_SWIGLU (gate, up): y [T, d_ff] <- silu(gate) * up; pre_act (optional, [T, 2 d_ff])
        keeps both pre-activations of training rows."""
        ss, sa, st = _seg_arrays(seg_start, seg_adapter, seg_is_train)
        rk = np.ascontiguousarray(rank, dtype=np.int32)
        sh = self._shape(x, W, len(sa), len(rk), scale, LAYOUT_IN_OUT)
        sb = self._siblings(d_outs, activation, pre_act)
        At, Bt = _ptr_table(A, len(rk)), _ptr_table(B, len(rk))
        _check(self._lib.collm_lora_siblings_fwd(
            self._h, ctypes.byref(sh), ctypes.byref(sb), x.data_ptr(), W.data_ptr(), At, Bt,
            rk.ctypes.data_as(_i32p), ss.ctypes.data_as(_i32p), sa.ctypes.data_as(_i32p), st.ctypes.data_as(_u8p),
            y.data_ptr(), None if h_save is None else h_save.data_ptr(), self._stream(stream)),
            "collm_lora_siblings_fwd")
        return y

    def collm_lora_siblings_bwd(self, d_outs, x, W, A: List, B: List, rank, seg_start, seg_adapter, seg_is_train,
                                scale: float, dy, h_save=None, dx=None, dA: Optional[List] = None,
                                dB: Optional[List] = None, accumulate: bool = False, stream=None):
        """Backward of collm_lora_siblings_fwd; dA_i, dB_i (fp32) shaped as A_i, B_i."""
        ss, sa, st = _seg_arrays(seg_start, seg_adapter, seg_is_train)
        rk = np.ascontiguousarray(rank, dtype=np.int32)
        sh = self._shape(x, W, len(sa), len(rk), scale, LAYOUT_IN_OUT)
        sb = self._siblings(d_outs)
        At, Bt = _ptr_table(A, len(rk)), _ptr_table(B, len(rk))
        dAt = _ptr_table(dA, len(rk)) if dA is not None else None
        dBt = _ptr_table(dB, len(rk)) if dB is not None else None
        _check(self._lib.collm_lora_siblings_bwd(
            self._h, ctypes.byref(sh), ctypes.byref(sb), x.data_ptr(), W.data_ptr(), At, Bt,
            rk.ctypes.data_as(_i32p), ss.ctypes.data_as(_i32p), sa.ctypes.data_as(_i32p), st.ctypes.data_as(_u8p),
            dy.data_ptr(), None if h_save is None else h_save.data_ptr(), None if dx is None else dx.data_ptr(),
            dAt, dBt, 1 if accumulate else 0, self._stream(stream)), "collm_lora_siblings_bwd")


NOALLOC_MAX_RANK = 64  # row stride of h_save in collm_lora_linear_fwd_noalloc


def collm_lora_linear_fwd_noalloc(x, W, A: List, B: List, rank, seg_start, seg_adapter, seg_is_train, scale: float, y,
                                  h_save=None, stream=None, layout: int = 0):
    """collm_lora_linear_fwd without a context: the workspace is the library's static device array (h_save, if
    given, has row stride 64)."""
    import torch

    lib = load_library()
    ss, sa, st = _seg_arrays(seg_start, seg_adapter, seg_is_train)
    rk = np.ascontiguousarray(rank, dtype=np.int32)
    dt = COLLM_BF16 if x.dtype == torch.bfloat16 else COLLM_F32
    d_out = W.shape[0] if layout == LAYOUT_OUT_IN else W.shape[1]
    sh = collm_shape(int(x.shape[1]), int(d_out), int(x.shape[0]), len(sa), len(rk), dt, float(scale), int(layout))
    At, Bt = _ptr_table(A, len(rk)), _ptr_table(B, len(rk))
    _check(lib.collm_lora_linear_fwd_noalloc(
        x.device.index or 0, ctypes.byref(sh), x.data_ptr(), W.data_ptr(), At, Bt, rk.ctypes.data_as(_i32p),
        ss.ctypes.data_as(_i32p), sa.ctypes.data_as(_i32p), st.ctypes.data_as(_u8p), y.data_ptr(),
        None if h_save is None else h_save.data_ptr(), _stream_handle(stream)), "collm_lora_linear_fwd_noalloc")
    return y


def _dtype_of(t):
    import torch

    if t.dtype == torch.bfloat16:
        return COLLM_BF16
    if t.dtype == torch.float32:
        return COLLM_F32
    raise TypeError("tensor must be bfloat16 or float32")


def _stream_handle(stream):
    import torch

    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def collm_swiglu_bwd(seg_start, seg_is_train, pre_act, dout, dy, stream=None):
    """Training rows: dy [T, 2 d_ff] <- gradient of silu(gate) * up with respect to the pre-activations pre_act,
    from dout [T, d_ff]."""
    lib = load_library()
    ss = np.ascontiguousarray(seg_start, dtype=np.int32)
    st = np.ascontiguousarray(seg_is_train, dtype=np.uint8)
    _check(lib.collm_swiglu_bwd(dout.device.index or 0, int(dout.shape[0]), int(dout.shape[1]), len(st),
                                ss.ctypes.data_as(_i32p), st.ctypes.data_as(_u8p), pre_act.data_ptr(),
                                dout.data_ptr(), dy.data_ptr(), _stream_handle(stream)), "collm_swiglu_bwd")
    return dy


def collm_adapter_fedavg(copies: Sequence, dst, stream=None):
    """dst <- mean of the adapter copies (same shape and element type), summed in list order."""
    lib = load_library()
    tab = copies if isinstance(copies, PointerTable) else PointerTable(copies)
    _check(lib.collm_adapter_fedavg(dst.device.index or 0, _dtype_of(dst), len(tab), tab.array, dst.data_ptr(),
                                    dst.numel(), _stream_handle(stream)), "collm_adapter_fedavg")
    return dst


def collm_adapter_adamw(param, grad, m, v, lr: float, beta1: float, beta2: float, eps: float,
                        weight_decay: float, step: int, master=None, stream=None):
    """One AdamW step on `param` (and its optional fp32 `master` copy) from the fp32 `grad`."""
    lib = load_library()
    hp = collm_adamw(lr, beta1, beta2, eps, weight_decay, int(step))
    _check(lib.collm_adapter_adamw(param.device.index or 0, _dtype_of(param), param.data_ptr(),
                                   None if master is None else master.data_ptr(), grad.data_ptr(), m.data_ptr(),
                                   v.data_ptr(), param.numel(), ctypes.byref(hp), _stream_handle(stream)),
           "collm_adapter_adamw")
    return param
