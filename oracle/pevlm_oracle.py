"""ctypes front end of the fp64 CPU oracle in ``pevlm_oracle.c``.  TEST INFRASTRUCTURE ONLY.

It only marshals numpy arrays into the C routines (which hold all the arithmetic) and chains them
in the order the method states: sequential positions -> rotary embedding of Q and K at those
positions (Sec. "Position Encoding") -> masked softmax attention with the explicit PEVLM mask
(Sec. "Formulations", Eq. 3-5, on top of Eq. 1).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "pevlm_oracle.c")
_LIB = os.path.join(_HERE, "libpevlm_oracle.so")

F32, BF16, F64 = 0, 1, 2


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (plain -O2 + OpenMP).  Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        )
    return _LIB


class _CLayout(ctypes.Structure):
    _fields_ = [
        ("num_seqs", ctypes.c_int32),
        ("cu_seqlens", ctypes.POINTER(ctypes.c_int32)),
        ("sink_len", ctypes.POINTER(ctypes.c_int32)),
        ("block_len", ctypes.POINTER(ctypes.c_int32)),
        ("ctx_len", ctypes.POINTER(ctypes.c_int32)),
        ("query_len", ctypes.POINTER(ctypes.c_int32)),
        ("window_blocks", ctypes.POINTER(ctypes.c_int32)),
    ]


_lib = None


def _load():
    global _lib
    if _lib is None:
        # PEVLM_ORACLE_LIB: load another build of the oracle (the mutation tests plant a mistake in
        # a copy of the C source and check that the pins notice)
        _lib = ctypes.CDLL(os.environ.get("PEVLM_ORACLE_LIB") or build())
        _lib.pevlm_oracle_check_layout.restype = ctypes.c_int
        _lib.pevlm_oracle_visible.restype = ctypes.c_int
        _lib.pevlm_oracle_visible.argtypes = [ctypes.c_int64] * 5
        _lib.pevlm_oracle_visible_blockwise.restype = ctypes.c_int
        _lib.pevlm_oracle_visible_blockwise.argtypes = [ctypes.c_int64] * 6
        _lib.pevlm_oracle_threads.restype = ctypes.c_int
        _lib.pevlm_oracle_mask_row.restype = None
        _lib.pevlm_oracle_positions.restype = None
        _lib.pevlm_oracle_rope.restype = None
        _lib.pevlm_oracle_rope_mrope.restype = None
        _lib.pevlm_oracle_attn.restype = None
    return _lib


@dataclass
class Layout:
    """Partition of each packed sequence: [sink S | context C in blocks of B | question Q]."""

    cu_seqlens: Sequence[int]
    sink_len: Sequence[int]
    block_len: Sequence[int]
    ctx_len: Sequence[int]
    query_len: Sequence[int]
    window_blocks: Optional[Sequence[int]] = None  # question sees sink + last W blocks (None / <0: all)

    def __post_init__(self):
        self._cu = np.ascontiguousarray(self.cu_seqlens, dtype=np.int32)
        self._s = np.ascontiguousarray(self.sink_len, dtype=np.int32)
        self._b = np.ascontiguousarray(self.block_len, dtype=np.int32)
        self._c = np.ascontiguousarray(self.ctx_len, dtype=np.int32)
        self._q = np.ascontiguousarray(self.query_len, dtype=np.int32)
        p = lambda a: a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))
        self._w = None if self.window_blocks is None else np.ascontiguousarray(self.window_blocks, dtype=np.int32)
        self._c_struct = _CLayout(len(self._s), p(self._cu), p(self._s), p(self._b), p(self._c), p(self._q),
                                  None if self._w is None else p(self._w))

    @property
    def num_seqs(self) -> int:
        return len(self._s)

    @property
    def total_tokens(self) -> int:
        return int(self._cu[-1])

    def ref(self):
        return ctypes.byref(self._c_struct)


def check_layout(lay: Layout) -> int:
    return int(_load().pevlm_oracle_check_layout(lay.ref()))


def threads() -> int:
    return int(_load().pevlm_oracle_threads())


def visible(S: int, B: int, C: int, i: int, j: int) -> bool:
    return bool(_load().pevlm_oracle_visible(S, B, C, i, j))


def positions(lay: Layout, pos_offset: Optional[Sequence[int]] = None) -> np.ndarray:
    pos = np.zeros(lay.total_tokens, dtype=np.int32)
    off = None
    offp = None
    if pos_offset is not None:
        off = np.ascontiguousarray(pos_offset, dtype=np.int32)
        offp = off.ctypes.data_as(ctypes.c_void_p)
    _load().pevlm_oracle_positions(lay.ref(), offp, pos.ctypes.data_as(ctypes.c_void_p))
    return pos


def mask_row(lay: Layout, t: int, causal: bool = True) -> np.ndarray:
    vis = np.zeros(lay.total_tokens, dtype=np.uint8)
    _load().pevlm_oracle_mask_row(lay.ref(), ctypes.c_int64(t), ctypes.c_int(int(causal)),
                                  vis.ctypes.data_as(ctypes.c_void_p))
    return vis


def mask_matrix(lay: Layout, causal: bool = True) -> np.ndarray:
    """Explicit [T, T] visibility matrix (small layouts only)."""
    T = lay.total_tokens
    return np.stack([mask_row(lay, t, causal) for t in range(T)]) if T else np.zeros((0, 0), np.uint8)


def _dtype_code(a: np.ndarray) -> int:
    if a.dtype == np.float32:
        return F32
    if a.dtype == np.float64:
        return F64
    if a.dtype == np.uint16:
        return BF16  # raw bf16 bit patterns
    raise TypeError(f"unsupported dtype {a.dtype}: pass float32, float64 or uint16 (bf16 bits)")


def _rows_arg(rows, T):
    if rows is None:
        return None, None, T
    r = np.ascontiguousarray(rows, dtype=np.int64)
    return r, r.ctypes.data_as(ctypes.c_void_p), len(r)


def rope(x: np.ndarray, pos: np.ndarray, rope_base: float, rows=None) -> np.ndarray:
    """Rotate x[T, H, D] at positions pos[T]; returns fp64 [n_rows, H, D]."""
    x = np.ascontiguousarray(x)
    T, H, D = x.shape
    pos = np.ascontiguousarray(pos, dtype=np.int32)
    r, rp, n = _rows_arg(rows, T)
    out = np.empty((n, H, D), dtype=np.float64)
    _load().pevlm_oracle_rope(x.ctypes.data_as(ctypes.c_void_p), ctypes.c_int(_dtype_code(x)),
                              ctypes.c_int64(T), ctypes.c_int32(H), ctypes.c_int32(D),
                              pos.ctypes.data_as(ctypes.c_void_p), ctypes.c_double(rope_base),
                              rp, ctypes.c_int64(n), out.ctypes.data_as(ctypes.c_void_p))
    return out


def rope_mrope(x: np.ndarray, pos3: np.ndarray, section, rope_base: float, rows=None) -> np.ndarray:
    """Rotate x[T, H, D] with three position axes pos3[3, T]; pair indices are split into
    section = (temporal, height, width) consecutive groups.  Returns fp64 [n_rows, H, D]."""
    x = np.ascontiguousarray(x)
    T, H, D = x.shape
    pos3 = np.ascontiguousarray(pos3, dtype=np.int32)
    sec = np.ascontiguousarray(section, dtype=np.int32)
    assert pos3.shape == (3, T) and sec.shape == (3,) and int(sec.sum()) == D // 2 and (sec >= 0).all()
    r, rp, n = _rows_arg(rows, T)
    out = np.empty((n, H, D), dtype=np.float64)
    _load().pevlm_oracle_rope_mrope(x.ctypes.data_as(ctypes.c_void_p), ctypes.c_int(_dtype_code(x)),
                                    ctypes.c_int64(T), ctypes.c_int32(H), ctypes.c_int32(D),
                                    pos3.ctypes.data_as(ctypes.c_void_p), sec.ctypes.data_as(ctypes.c_void_p),
                                    ctypes.c_double(rope_base), rp, ctypes.c_int64(n),
                                    out.ctypes.data_as(ctypes.c_void_p))
    return out


def attn(q_rot: np.ndarray, k_rot: np.ndarray, v: np.ndarray, lay: Layout, rows=None,
         kv_head_of_q=None, softmax_scale: float = 0.0, key_range=None, causal: bool = True,
         skip_masked: bool = True):
    """Masked softmax attention for the selected rows.  q_rot [n_rows, Hq, D] fp64 (already
    rotated), k_rot [T, Hkv, D] fp64, v [T, Hkv, D] (float32 / float64 / uint16 bf16 bits).
    Returns (out [n_rows, Hq, D], lse [n_rows, Hq]) in fp64."""
    q_rot = np.ascontiguousarray(q_rot, dtype=np.float64)
    k_rot = np.ascontiguousarray(k_rot, dtype=np.float64)
    v = np.ascontiguousarray(v)
    T, Hkv, D = k_rot.shape
    assert T == lay.total_tokens and v.shape == k_rot.shape
    r, rp, n = _rows_arg(rows, T)
    assert q_rot.shape[0] == n and q_rot.shape[2] == D
    Hq = q_rot.shape[1]
    hm = None
    hmp = None
    if kv_head_of_q is not None:
        hm = np.ascontiguousarray(kv_head_of_q, dtype=np.int32)
        hmp = hm.ctypes.data_as(ctypes.c_void_p)
    lo, hi = (0, T) if key_range is None else key_range
    out = np.empty((n, Hq, D), dtype=np.float64)
    lse = np.empty((n, Hq), dtype=np.float64)
    _load().pevlm_oracle_attn(q_rot.ctypes.data_as(ctypes.c_void_p), k_rot.ctypes.data_as(ctypes.c_void_p),
                              v.ctypes.data_as(ctypes.c_void_p), ctypes.c_int(_dtype_code(v)), lay.ref(),
                              ctypes.c_int32(Hq), ctypes.c_int32(Hkv), ctypes.c_int32(D), hmp,
                              ctypes.c_double(softmax_scale), rp, ctypes.c_int64(n),
                              ctypes.c_int64(lo), ctypes.c_int64(hi), ctypes.c_int(int(causal)),
                              ctypes.c_int(int(skip_masked)), out.ctypes.data_as(ctypes.c_void_p),
                              lse.ctypes.data_as(ctypes.c_void_p))
    return out, lse


def forward(q: np.ndarray, k: np.ndarray, v: np.ndarray, lay: Layout, rope_base: float, rows=None,
            kv_head_of_q=None, softmax_scale: float = 0.0, pos_offset=None, skip_masked: bool = True,
            pos: Optional[np.ndarray] = None):
    """Whole path for the selected rows: positions -> RoPE(Q rows, all K) -> masked attention.
    `pos` overrides the sequential positions (used only by tests that show re-based positions
    give a different answer)."""
    if pos is None:
        pos = positions(lay, pos_offset)
    k_rot = rope(k, pos, rope_base)
    q_rot = rope(q, pos, rope_base, rows)
    return attn(q_rot, k_rot, v, lay, rows, kv_head_of_q, softmax_scale, skip_masked=skip_masked)
