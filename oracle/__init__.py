"""CPU oracle for MoE dispatch/combine -- TEST INFRASTRUCTURE, not product code.

`ep_oracle.c` holds the plain sequential definitions; this module compiles it
with gcc and wraps it for numpy arrays.  Only tests, the smoke check and the
benchmark's CPU-baseline leg may import it.  It imports nothing from the HIP
package.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ep_oracle.c")
_LIB = os.path.join(_HERE, "libep_oracle.so")

LAYOUT_CONCAT = 0
LAYOUT_PADDED = 1


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no fast-math, no FMA contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-shared", "-fPIC",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.ep_oracle_double_to_bf16.restype = ctypes.c_uint16
        _lib.ep_oracle_double_to_bf16.argtypes = [ctypes.c_double]
        _lib.ep_oracle_bf16_to_float.restype = ctypes.c_float
        _lib.ep_oracle_bf16_to_float.argtypes = [ctypes.c_uint16]
        _lib.ep_oracle_msg_header_bytes.restype = ctypes.c_int64
        _lib.ep_oracle_msg_header_bytes.argtypes = [ctypes.c_int]
        for fn in (_lib.ep_oracle_footprint_per_expert,):
            fn.restype = ctypes.c_int64
            fn.argtypes = [ctypes.c_int64] * 3
        _lib.ep_oracle_footprint_optimised.restype = ctypes.c_int64
        _lib.ep_oracle_footprint_optimised.argtypes = [ctypes.c_int64] * 4
        _lib.ep_oracle_e4m3_to_float.restype = ctypes.c_float
        _lib.ep_oracle_e4m3_to_float.argtypes = [ctypes.c_uint8]
        _lib.ep_oracle_double_to_e4m3.restype = ctypes.c_uint8
        _lib.ep_oracle_double_to_e4m3.argtypes = [ctypes.c_double]
        _lib.ep_oracle_quantize_row.restype = None
        _lib.ep_oracle_dispatch_fp8.restype = None
        _lib.ep_oracle_layout.restype = None
        _lib.ep_oracle_dispatch.restype = None
        _lib.ep_oracle_combine.restype = None
        _lib.ep_oracle_combine_hier.restype = None
        _lib.ep_oracle_dedup_send.restype = None
        _lib.ep_oracle_dedup_recv.restype = None
    return _lib


def _p(a: Optional[np.ndarray]):
    if a is None:
        return ctypes.c_void_p(0)
    return ctypes.c_void_p(a.ctypes.data)


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


@dataclass
class Layout:
    T: int
    K: int
    E: int
    R: int
    layout: int
    C: int
    C_rank: int
    expert_count: np.ndarray
    expert_kept: np.ndarray
    expert_offset: np.ndarray
    slot: np.ndarray
    dst_row: np.ndarray
    sorted_token: np.ndarray
    sorted_k: np.ndarray
    sorted_row: np.ndarray
    rank_pair_count: np.ndarray
    rank_token_count: np.ndarray
    rank_offset: np.ndarray
    rank_row: np.ndarray
    kept: int
    dropped: int
    masked: int
    invalid: int
    n_sorted: int
    n_msgs: int


def layout(topk_idx: np.ndarray, E: int, R: int, layout: int = LAYOUT_CONCAT, C: int = 0,
           C_rank: int = 0, expert_base: Optional[np.ndarray] = None) -> Layout:
    topk_idx = _i32(topk_idx)
    T, K = topk_idx.shape
    if E % R != 0:
        raise ValueError("E must be a multiple of R")
    if layout == LAYOUT_PADDED and C <= 0:
        raise ValueError("padded layout needs C > 0")
    if C_rank <= 0:
        C_rank = T
    n = T * K
    out = dict(
        expert_count=np.zeros(E, np.int32), expert_kept=np.zeros(E, np.int32),
        expert_offset=np.zeros(E + 1, np.int32), slot=np.full((T, K), -7, np.int32),
        dst_row=np.full((T, K), -7, np.int32), sorted_token=np.full(n, -1, np.int32),
        sorted_k=np.full(n, -1, np.int32), sorted_row=np.full(n, -1, np.int32),
        rank_pair_count=np.zeros(R, np.int32), rank_token_count=np.zeros(R, np.int32),
        rank_offset=np.zeros(R + 1, np.int32), rank_row=np.full((T, K), -7, np.int32))
    totals = np.zeros(6, np.int64)
    base = None if expert_base is None else _i32(expert_base)
    lib().ep_oracle_layout(
        _p(topk_idx), ctypes.c_int(T), ctypes.c_int(K), ctypes.c_int(E), ctypes.c_int(R),
        ctypes.c_int(layout), ctypes.c_int(C), ctypes.c_int(C_rank), _p(base),
        _p(out["expert_count"]), _p(out["expert_kept"]), _p(out["expert_offset"]), _p(out["slot"]),
        _p(out["dst_row"]), _p(out["sorted_token"]), _p(out["sorted_k"]), _p(out["sorted_row"]),
        _p(out["rank_pair_count"]), _p(out["rank_token_count"]), _p(out["rank_offset"]),
        _p(out["rank_row"]), _p(totals))
    return Layout(T=T, K=K, E=E, R=R, layout=layout, C=C, C_rank=C_rank, kept=int(totals[0]),
                  dropped=int(totals[1]), masked=int(totals[2]), invalid=int(totals[3]),
                  n_sorted=int(totals[4]), n_msgs=int(totals[5]), **out)


def _strides(layout_mode: int, C: int, H: int, stride0: Optional[int], stride1: Optional[int]):
    if layout_mode == LAYOUT_PADDED:
        s1 = H if stride1 is None else stride1
        s0 = C * s1 if stride0 is None else stride0
    else:
        s0 = H if stride0 is None else stride0
        s1 = 0
    return int(s0), int(s1)


def dispatch(x_bits: np.ndarray, w: Optional[np.ndarray], lay: Layout, recv_x: np.ndarray,
             recv_w: Optional[np.ndarray] = None, recv_src: Optional[np.ndarray] = None,
             stride0: Optional[int] = None, stride1: Optional[int] = None) -> None:
    """Scatter rows of x into recv_x (uint16 storage, modified in place)."""
    assert x_bits.dtype == np.uint16 and recv_x.dtype == np.uint16
    T, H = x_bits.shape
    s0, s1 = _strides(lay.layout, lay.C, H, stride0, stride1)
    wc = None if w is None else np.ascontiguousarray(w, dtype=np.float32)
    lib().ep_oracle_dispatch(
        _p(x_bits), ctypes.c_int64(x_bits.strides[0] // 2), _p(wc), _p(lay.dst_row),
        ctypes.c_int(T), ctypes.c_int(lay.K), ctypes.c_int(H), ctypes.c_int(lay.layout),
        ctypes.c_int(max(lay.C, 1)), ctypes.c_int64(s0), ctypes.c_int64(s1), _p(recv_x),
        _p(recv_w), _p(recv_src))


def combine(y_bits: np.ndarray, w: Optional[np.ndarray], lay: Layout, H: int,
            acc: str = "f64", stride0: Optional[int] = None,
            stride1: Optional[int] = None, T: Optional[int] = None) -> np.ndarray:
    """Gather + weighted reduce; returns uint16 [T, H] bf16 bit patterns."""
    assert y_bits.dtype == np.uint16
    T = lay.T if T is None else T
    s0, s1 = _strides(lay.layout, lay.C, H, stride0, stride1)
    out = np.zeros((T, H), np.uint16)
    wc = None if w is None else np.ascontiguousarray(w, dtype=np.float32)
    lib().ep_oracle_combine(
        _p(y_bits), ctypes.c_int(lay.layout), ctypes.c_int(max(lay.C, 1)), ctypes.c_int64(s0),
        ctypes.c_int64(s1), _p(wc), _p(lay.dst_row), ctypes.c_int(T), ctypes.c_int(lay.K),
        ctypes.c_int(H), _p(out), ctypes.c_int64(H), ctypes.c_int({"f64": 0, "f32": 1}[acc]))
    return out


def combine_hier(y_bits: np.ndarray, w: Optional[np.ndarray], lay: Layout, topk_idx: np.ndarray, H: int,
                 ranks_per_node: int, stride0: Optional[int] = None, stride1: Optional[int] = None) -> np.ndarray:
    """Combine with the two-level (per node, then across nodes) float32 summation order."""
    assert y_bits.dtype == np.uint16
    s0, s1 = _strides(lay.layout, lay.C, H, stride0, stride1)
    out = np.zeros((lay.T, H), np.uint16)
    wc = None if w is None else np.ascontiguousarray(w, dtype=np.float32)
    lib().ep_oracle_combine_hier(
        _p(y_bits), ctypes.c_int(lay.layout), ctypes.c_int(max(lay.C, 1)), ctypes.c_int64(s0),
        ctypes.c_int64(s1), _p(wc), _p(lay.dst_row), _p(_i32(topk_idx)), ctypes.c_int(lay.T),
        ctypes.c_int(lay.K), ctypes.c_int(H), ctypes.c_int(lay.E // lay.R), ctypes.c_int(lay.R),
        ctypes.c_int(ranks_per_node), _p(out), ctypes.c_int64(H))
    return out


def msg_header_bytes(K: int) -> int:
    return int(lib().ep_oracle_msg_header_bytes(ctypes.c_int(K)))


def dedup_send(x_bits: np.ndarray, topk_idx: np.ndarray, w: Optional[np.ndarray], lay: Layout,
               n_slots: int) -> np.ndarray:
    """Once-per-destination-rank messages; returns the staging windows as bytes [n_slots, msg]."""
    T, H = x_bits.shape
    msg = msg_header_bytes(lay.K) + 2 * H
    win = np.full((n_slots, msg), 0xA5, np.uint8)
    wc = None if w is None else np.ascontiguousarray(w, dtype=np.float32)
    lib().ep_oracle_dedup_send(
        _p(x_bits), ctypes.c_int64(x_bits.strides[0] // 2), _p(_i32(topk_idx)), _p(wc),
        _p(lay.rank_row), ctypes.c_int(T), ctypes.c_int(lay.K), ctypes.c_int(H), _p(win))
    return win


def dedup_recv(win: np.ndarray, lay: Layout, H: int, recv_x: np.ndarray,
               recv_w: Optional[np.ndarray] = None, recv_src: Optional[np.ndarray] = None,
               expert_base: Optional[np.ndarray] = None, stride0: Optional[int] = None,
               stride1: Optional[int] = None):
    """Receiver fan-out over all simulated destination ranks; returns (recv_count[E], dropped)."""
    s0, s1 = _strides(lay.layout, lay.C, H, stride0, stride1)
    recv_count = np.zeros(lay.E, np.int32)
    dropped = ctypes.c_int64(0)
    base = None if expert_base is None else _i32(expert_base)
    lib().ep_oracle_dedup_recv(
        _p(win), _p(lay.rank_offset), _p(lay.rank_token_count), ctypes.c_int(lay.K),
        ctypes.c_int(H), ctypes.c_int(lay.E), ctypes.c_int(lay.R), ctypes.c_int(lay.layout),
        ctypes.c_int(max(lay.C, 1)), _p(base), ctypes.c_int64(s0), ctypes.c_int64(s1),
        _p(recv_x), _p(recv_w), _p(recv_src), _p(recv_count), ctypes.byref(dropped))
    return recv_count, int(dropped.value)


def double_to_e4m3(v: float) -> int:
    return int(lib().ep_oracle_double_to_e4m3(ctypes.c_double(v)))


def e4m3_to_float(c: int) -> float:
    return float(lib().ep_oracle_e4m3_to_float(ctypes.c_uint8(c)))


def quantize_row(x_bits_row: np.ndarray):
    """One token row (uint16 bf16 bits, H % 128 == 0) -> (uint8 [H] E4M3 codes, float32 [H/128] scales)."""
    x = np.ascontiguousarray(x_bits_row, dtype=np.uint16)
    H = x.shape[0]
    assert H % 128 == 0
    q = np.zeros(H, np.uint8)
    sc = np.zeros(H // 128, np.float32)
    lib().ep_oracle_quantize_row(_p(x), ctypes.c_int(H), _p(q), _p(sc))
    return q, sc


def dispatch_fp8(x_bits: np.ndarray, lay: Layout, recv_q: np.ndarray, recv_scales: np.ndarray,
                 stride0: Optional[int] = None, stride1: Optional[int] = None) -> None:
    """Quantising dispatch: recv_q uint8 windows, recv_scales float32 [rows, H/128] (in place)."""
    assert x_bits.dtype == np.uint16 and recv_q.dtype == np.uint8 and recv_scales.dtype == np.float32
    T, H = x_bits.shape
    s0, s1 = _strides(lay.layout, lay.C, H, stride0, stride1)
    lib().ep_oracle_dispatch_fp8(
        _p(x_bits), ctypes.c_int64(x_bits.strides[0] // 2), _p(lay.dst_row), ctypes.c_int(T),
        ctypes.c_int(lay.K), ctypes.c_int(H), ctypes.c_int(lay.layout), ctypes.c_int(max(lay.C, 1)),
        ctypes.c_int64(s0), ctypes.c_int64(s1), _p(recv_q), _p(recv_scales))


def footprint_per_expert(E: int, B: int, P: int) -> int:
    return int(lib().ep_oracle_footprint_per_expert(E, B, P))


def footprint_optimised(N: int, B: int, K: int, P: int) -> int:
    return int(lib().ep_oracle_footprint_optimised(N, B, K, P))


def double_to_bf16(v: float) -> int:
    return int(lib().ep_oracle_double_to_bf16(ctypes.c_double(v)))
