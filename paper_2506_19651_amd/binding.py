"""ctypes binding of libpevlm.so: same names as the C entry points, argument marshalling only.

Tensors are torch tensors in device memory (torch is used to allocate memory and to name the
stream); their data pointers go straight to the C ABI.  Descriptor arrays stay on the host.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_PKG, "libpevlm.so")

PEVLM_OK, PEVLM_ERR_INVALID_ARG, PEVLM_ERR_UNSUPPORTED, PEVLM_ERR_WORKSPACE_TOO_SMALL, PEVLM_ERR_HIP = range(5)
PEVLM_F32, PEVLM_BF16 = 0, 1
PEVLM_MAX_SPLITS = 64


class PevlmError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"pevlm status {status}: {message}")
        self.status = status


class _CLayout(ctypes.Structure):
    _fields_ = [("num_seqs", ctypes.c_int32)] + [
        (n, ctypes.POINTER(ctypes.c_int32)) for n in ("cu_seqlens", "sink_len", "block_len", "ctx_len", "query_len")]


class _CHeads(ctypes.Structure):
    _fields_ = [("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("kv_head_of_q", ctypes.POINTER(ctypes.c_int32)), ("dtype", ctypes.c_int32),
                ("softmax_scale", ctypes.c_float)]


class WorkItem(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("q_start", "q_rows", "full_start", "full_len", "diag_start",
                                              "diag_len", "seq", "reserved")]


class _StreamSlot(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("q_start", "q_rows", "head", "reserved")]


class StreamItem(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("full_start", "full_len", "diag_start", "diag_len", "kv_head",
                                              "n_full_tiles", "n_tiles", "seq")] + [("slot", _StreamSlot * 8)]


class Fp8Plan(ctypes.Structure):
    _fields_ = [("n_items", ctypes.c_int64), ("n_key_tiles", ctypes.c_int64)] + \
               [(n, ctypes.c_size_t) for n in ("items", "key_tiles", "kv_amax", "q_scales", "q_codes", "k_tiles", "v_tiles", "total")]


_lib = None


def lib_path() -> str:
    return _LIB_PATH


def load_library():
    """Loads libpevlm.so.  Raises if it has not been built: there is no other path."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError(f"{_LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                              "(or paper_2506_19651_amd/build.py) first; there is no fallback path")
        lib = ctypes.CDLL(_LIB_PATH)
        vp, i32, f32p = ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p
        LP, HP = ctypes.POINTER(_CLayout), ctypes.POINTER(_CHeads)
        lib.pevlm_rope_seq.restype = ctypes.c_int
        lib.pevlm_rope_seq.argtypes = [vp, vp, LP, HP, ctypes.c_double, vp, vp]
        lib.pevlm_block_prefill_workspace_bytes.restype = ctypes.c_size_t
        lib.pevlm_block_prefill_workspace_bytes.argtypes = [LP, HP]
        lib.pevlm_block_prefill_attn.restype = ctypes.c_int
        lib.pevlm_block_prefill_attn.argtypes = [vp, vp, vp, vp, f32p, LP, HP, vp, ctypes.c_size_t, vp]
        lib.pevlm_query_workspace_bytes.restype = ctypes.c_size_t
        lib.pevlm_query_workspace_bytes.argtypes = [LP, HP, i32]
        lib.pevlm_query_attn.restype = ctypes.c_int
        lib.pevlm_query_attn.argtypes = [vp, vp, vp, vp, f32p, LP, HP, i32, vp, ctypes.c_size_t, vp]
        lib.pevlm_query_attn_static.restype = ctypes.c_int
        lib.pevlm_query_attn_static.argtypes = [vp, vp, vp, vp, f32p, LP, HP, i32, vp]
        lib.pevlm_block_prefill_rope_workspace_bytes.restype = ctypes.c_size_t
        lib.pevlm_block_prefill_rope_workspace_bytes.argtypes = [LP, HP]
        lib.pevlm_block_prefill_attn_rope.restype = ctypes.c_int
        lib.pevlm_block_prefill_attn_rope.argtypes = [vp, vp, vp, vp, f32p, LP, HP, ctypes.c_double, vp, i32, vp, ctypes.c_size_t, vp]
        lib.pevlm_query_rope_workspace_bytes.restype = ctypes.c_size_t
        lib.pevlm_query_rope_workspace_bytes.argtypes = [LP, HP, i32]
        lib.pevlm_query_attn_rope.restype = ctypes.c_int
        lib.pevlm_query_attn_rope.argtypes = [vp, vp, vp, vp, f32p, LP, HP, i32, ctypes.c_double, vp, vp, ctypes.c_size_t, vp]
        i32p = ctypes.POINTER(ctypes.c_int32)
        lib.pevlm_block_prefill_attn_blocks.restype = ctypes.c_int
        lib.pevlm_block_prefill_attn_blocks.argtypes = [vp, vp, vp, vp, f32p, LP, HP, i32p, i32p, i32, vp, ctypes.c_size_t, vp]
        lib.pevlm_query_window_workspace_bytes.restype = ctypes.c_size_t
        lib.pevlm_query_window_workspace_bytes.argtypes = [LP, HP, i32]
        lib.pevlm_query_attn_window.restype = ctypes.c_int
        lib.pevlm_query_attn_window.argtypes = [vp, vp, vp, vp, f32p, LP, HP, i32p, i32, vp, ctypes.c_size_t, vp]
        lib.pevlm_prefill_worklist_blocks_host.restype = ctypes.c_int64
        lib.pevlm_prefill_worklist_blocks_host.argtypes = [LP, i32, i32p, i32p, i32, ctypes.POINTER(WorkItem), ctypes.c_int64]
        lib.pevlm_query_worklist_window_host.restype = ctypes.c_int64
        lib.pevlm_query_worklist_window_host.argtypes = [LP, i32, i32, i32p, ctypes.POINTER(WorkItem), ctypes.c_int64]
        lib.pevlm_block_prefill_attn_mrope.restype = ctypes.c_int
        lib.pevlm_block_prefill_attn_mrope.argtypes = [vp, vp, vp, vp, f32p, LP, HP, ctypes.c_double, vp, i32p, i32, vp,
                                                       ctypes.c_size_t, vp]
        lib.pevlm_query_attn_mrope.restype = ctypes.c_int
        lib.pevlm_query_attn_mrope.argtypes = [vp, vp, vp, vp, f32p, LP, HP, i32, ctypes.c_double, vp, i32p, vp, ctypes.c_size_t, vp]
        lib.pevlm_block_prefill_fp8_plan.restype = ctypes.c_int
        lib.pevlm_block_prefill_fp8_plan.argtypes = [LP, HP, ctypes.POINTER(Fp8Plan)]
        lib.pevlm_block_prefill_fp8_workspace_bytes.restype = ctypes.c_size_t
        lib.pevlm_block_prefill_fp8_workspace_bytes.argtypes = [LP, HP]
        lib.pevlm_block_prefill_attn_fp8.restype = ctypes.c_int
        lib.pevlm_block_prefill_attn_fp8.argtypes = [vp, vp, vp, vp, f32p, LP, HP, vp, ctypes.c_size_t, i32, vp]
        lib.pevlm_last_error.restype = ctypes.c_char_p
        lib.pevlm_version.restype = i32
        lib.pevlm_prefill_tile_rows.restype = i32
        lib.pevlm_prefill_tile_rows.argtypes = [HP]
        lib.pevlm_query_tile_rows.restype = i32
        lib.pevlm_query_tile_rows.argtypes = [HP]
        lib.pevlm_prefill_uses_stream_kernel.restype = ctypes.c_int32
        lib.pevlm_prefill_uses_stream_kernel.argtypes = [LP, HP]
        lib.pevlm_set_prefill_kernel.restype = ctypes.c_int32
        lib.pevlm_set_prefill_kernel.argtypes = [i32]
        lib.pevlm_prefill_stream_items_host.restype = ctypes.c_int64
        lib.pevlm_prefill_stream_items_host.argtypes = [LP, HP, ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int32), i32,
                                                        ctypes.POINTER(StreamItem), ctypes.c_int64]
        lib.pevlm_prefill_worklist_host.restype = ctypes.c_int64
        lib.pevlm_prefill_worklist_host.argtypes = [LP, i32, ctypes.POINTER(WorkItem), ctypes.c_int64]
        lib.pevlm_query_worklist_host.restype = ctypes.c_int64
        lib.pevlm_query_worklist_host.argtypes = [LP, i32, i32, ctypes.POINTER(WorkItem), ctypes.c_int64]
        lib.pevlm_rope_mrope.restype = ctypes.c_int
        lib.pevlm_rope_mrope.argtypes = [vp, vp, ctypes.c_int64, HP, ctypes.c_double, vp, ctypes.POINTER(ctypes.c_int32), vp]
        lib.pevlm_probe_mfma_bf16.restype = ctypes.c_int
        lib.pevlm_probe_mfma_bf16.argtypes = [vp, i32, i32, ctypes.POINTER(ctypes.c_double), vp]
        lib.pevlm_probe_tile_loop_bf16.restype = ctypes.c_int
        lib.pevlm_probe_tile_loop_bf16.argtypes = [vp, vp, ctypes.c_size_t, i32, i32, i32, ctypes.POINTER(ctypes.c_double), vp]
        lib.pevlm_probe_copy.restype = ctypes.c_int
        lib.pevlm_probe_copy.argtypes = [vp, vp, ctypes.c_size_t, vp]
        lib.pevlm_visible_pairs.restype = ctypes.c_int
        lib.pevlm_visible_pairs.argtypes = [LP] + [ctypes.POINTER(ctypes.c_int64)] * 3
        _lib = lib
    return _lib


def _i32p(a: np.ndarray):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


class Layout:
    """Host-side partition descriptor: per sequence sink S, block length B, context length C,
    question length Q; sequences are packed back to back (cu_seqlens)."""

    def __init__(self, cu_seqlens: Sequence[int], sink_len, block_len, ctx_len, query_len):
        self.cu = np.ascontiguousarray(cu_seqlens, dtype=np.int32)
        self.s = np.ascontiguousarray(sink_len, dtype=np.int32)
        self.b = np.ascontiguousarray(block_len, dtype=np.int32)
        self.c = np.ascontiguousarray(ctx_len, dtype=np.int32)
        self.q = np.ascontiguousarray(query_len, dtype=np.int32)
        self.struct = _CLayout(len(self.s), _i32p(self.cu), _i32p(self.s), _i32p(self.b), _i32p(self.c), _i32p(self.q))

    @classmethod
    def from_seqs(cls, seqs):
        a = np.asarray(seqs, dtype=np.int64).reshape(-1, 4)
        cu = np.concatenate([[0], np.cumsum(a[:, 0] + a[:, 2] + a[:, 3])])
        return cls(cu, a[:, 0], a[:, 1], a[:, 2], a[:, 3])

    @property
    def total_tokens(self) -> int:
        return int(self.cu[-1]) if len(self.cu) else 0

    def ref(self):
        return ctypes.byref(self.struct)


class Heads:
    def __init__(self, n_q_heads: int, n_kv_heads: int, head_dim: int, dtype: str,
                 kv_head_of_q: Optional[Sequence[int]] = None, softmax_scale: float = 0.0):
        self.map = None if kv_head_of_q is None else np.ascontiguousarray(kv_head_of_q, dtype=np.int32)
        code = {"f32": PEVLM_F32, "bf16": PEVLM_BF16}.get(dtype, dtype)
        self.struct = _CHeads(n_q_heads, n_kv_heads, head_dim, None if self.map is None else _i32p(self.map),
                              int(code), float(softmax_scale))
        self.n_q_heads, self.n_kv_heads, self.head_dim, self.dtype = n_q_heads, n_kv_heads, head_dim, dtype

    def ref(self):
        return ctypes.byref(self.struct)


def _check(status: int):
    if status != PEVLM_OK:
        raise PevlmError(status, pevlm_last_error())


def _ptr(t):
    if t is None:
        return None
    if hasattr(t, "data_ptr"):
        return ctypes.c_void_p(t.data_ptr())
    return ctypes.c_void_p(int(t))


def _stream_ptr(stream):
    if stream is None:
        import torch
        return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    if hasattr(stream, "cuda_stream"):
        return ctypes.c_void_p(stream.cuda_stream)
    return ctypes.c_void_p(int(stream))


def _workspace(nbytes: int, like):
    import torch
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=like.device)


def pevlm_last_error() -> str:
    return load_library().pevlm_last_error().decode()


def pevlm_probe_mfma_bf16(scratch, workgroups: int, iters: int, stream=None) -> float:
    """Enqueues the register-resident bf16 MFMA loop; returns the floating-point operations of the launch."""
    flops = ctypes.c_double(0.0)
    _check(load_library().pevlm_probe_mfma_bf16(_ptr(scratch), int(workgroups), int(iters), ctypes.byref(flops), _stream_ptr(stream)))
    return float(flops.value)


def pevlm_probe_tile_loop_bf16(scratch, kv, workgroups: int, iters: int, with_softmax: bool = True, stream=None) -> float:
    """Enqueues the tile-loop probe on `kv` (a device tensor of finite bf16 data); returns the FLOPs of its MFMAs."""
    flops = ctypes.c_double(0.0)
    _check(load_library().pevlm_probe_tile_loop_bf16(_ptr(scratch), _ptr(kv), int(kv.numel() * kv.element_size()), int(workgroups),
                                                     int(iters), int(bool(with_softmax)), ctypes.byref(flops), _stream_ptr(stream)))
    return float(flops.value)


def pevlm_probe_copy(dst, src, nbytes: int, stream=None) -> None:
    _check(load_library().pevlm_probe_copy(_ptr(dst), _ptr(src), int(nbytes), _stream_ptr(stream)))


def pevlm_version() -> int:
    return int(load_library().pevlm_version())


def pevlm_prefill_tile_rows(heads: "Heads") -> int:
    return int(load_library().pevlm_prefill_tile_rows(heads.ref()))


def pevlm_query_tile_rows(heads: "Heads") -> int:
    return int(load_library().pevlm_query_tile_rows(heads.ref()))


def pevlm_rope_seq(q, k, layout: Layout, heads: Heads, rope_base: float, pos_offset=None, stream=None):
    off = None if pos_offset is None else np.ascontiguousarray(pos_offset, dtype=np.int32)
    offp = None if off is None else off.ctypes.data_as(ctypes.c_void_p)
    _check(load_library().pevlm_rope_seq(_ptr(q), _ptr(k), layout.ref(), heads.ref(), float(rope_base), offp,
                                         _stream_ptr(stream)))


def _offsets(pos_offset):
    off = None if pos_offset is None else np.ascontiguousarray(pos_offset, dtype=np.int32)
    return off, (None if off is None else off.ctypes.data_as(ctypes.c_void_p))


def pevlm_block_prefill_rope_workspace_bytes(layout: Layout, heads: Heads) -> int:
    return int(load_library().pevlm_block_prefill_rope_workspace_bytes(layout.ref(), heads.ref()))


def pevlm_block_prefill_attn_rope(q, k, v, out, layout: Layout, heads: Heads, rope_base: float, pos_offset=None,
                                  k_is_rotated: bool = False, lse=None, workspace=None, stream=None):
    if workspace is None:
        workspace = _workspace(pevlm_block_prefill_rope_workspace_bytes(layout, heads), q)
    _off, offp = _offsets(pos_offset)
    _check(load_library().pevlm_block_prefill_attn_rope(_ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(lse), layout.ref(),
                                                        heads.ref(), float(rope_base), offp, int(bool(k_is_rotated)),
                                                        _ptr(workspace), workspace.numel(), _stream_ptr(stream)))


def pevlm_query_rope_workspace_bytes(layout: Layout, heads: Heads, num_splits: int = 0) -> int:
    return int(load_library().pevlm_query_rope_workspace_bytes(layout.ref(), heads.ref(), int(num_splits)))


def pevlm_query_attn_rope(q, k, v, out, layout: Layout, heads: Heads, rope_base: float, pos_offset=None, num_splits: int = 0,
                          lse=None, workspace=None, stream=None):
    if workspace is None:
        workspace = _workspace(pevlm_query_rope_workspace_bytes(layout, heads, num_splits), q)
    _off, offp = _offsets(pos_offset)
    _check(load_library().pevlm_query_attn_rope(_ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(lse), layout.ref(), heads.ref(),
                                                int(num_splits), float(rope_base), offp, _ptr(workspace),
                                                workspace.numel(), _stream_ptr(stream)))


def pevlm_block_prefill_attn_mrope(q, k, v, out, layout: Layout, heads: Heads, rope_base: float, pos_ids, section,
                                   k_is_rotated: bool = False, lse=None, workspace=None, stream=None):
    if workspace is None:
        workspace = _workspace(pevlm_block_prefill_rope_workspace_bytes(layout, heads), q)
    _s, sp = _i32_array(section)
    _check(load_library().pevlm_block_prefill_attn_mrope(_ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(lse), layout.ref(),
                                                         heads.ref(), float(rope_base), _ptr(pos_ids), sp,
                                                         int(bool(k_is_rotated)), _ptr(workspace), workspace.numel(),
                                                         _stream_ptr(stream)))


def pevlm_query_attn_mrope(q, k, v, out, layout: Layout, heads: Heads, rope_base: float, pos_ids, section, num_splits: int = 0,
                           lse=None, workspace=None, stream=None):
    if workspace is None:
        workspace = _workspace(pevlm_query_rope_workspace_bytes(layout, heads, num_splits), q)
    _s, sp = _i32_array(section)
    _check(load_library().pevlm_query_attn_mrope(_ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(lse), layout.ref(), heads.ref(),
                                                 int(num_splits), float(rope_base), _ptr(pos_ids), sp, _ptr(workspace),
                                                 workspace.numel(), _stream_ptr(stream)))


def pevlm_rope_mrope(q, k, num_tokens: int, heads: Heads, rope_base: float, pos_ids, section, stream=None):
    """pos_ids: device int32 tensor [3, num_tokens]; section: three host ints adding up to head_dim/2."""
    sec = (ctypes.c_int32 * 3)(*[int(x) for x in section])
    _check(load_library().pevlm_rope_mrope(_ptr(q), _ptr(k), int(num_tokens), heads.ref(), float(rope_base), _ptr(pos_ids),
                                           sec, _stream_ptr(stream)))


def pevlm_block_prefill_workspace_bytes(layout: Layout, heads: Heads) -> int:
    return int(load_library().pevlm_block_prefill_workspace_bytes(layout.ref(), heads.ref()))


def pevlm_block_prefill_attn(q, k, v, out, layout: Layout, heads: Heads, lse=None, workspace=None, stream=None):
    if workspace is None:
        workspace = _workspace(pevlm_block_prefill_workspace_bytes(layout, heads), q)
    _check(load_library().pevlm_block_prefill_attn(_ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(lse), layout.ref(),
                                                   heads.ref(), _ptr(workspace), workspace.numel(),
                                                   _stream_ptr(stream)))
    return workspace


FP8_QUANTISE, FP8_ATTEND = 1, 2


def pevlm_block_prefill_fp8_plan(layout: Layout, heads: Heads) -> Fp8Plan:
    plan = Fp8Plan()
    _check(load_library().pevlm_block_prefill_fp8_plan(layout.ref(), heads.ref(), ctypes.byref(plan)))
    return plan


def pevlm_block_prefill_fp8_workspace_bytes(layout: Layout, heads: Heads) -> int:
    return int(load_library().pevlm_block_prefill_fp8_workspace_bytes(layout.ref(), heads.ref()))


def pevlm_block_prefill_attn_fp8(q, k, v, out, layout: Layout, heads: Heads, lse=None, workspace=None, stages: int = 0,
                                 stream=None):
    if workspace is None:
        workspace = _workspace(pevlm_block_prefill_fp8_workspace_bytes(layout, heads), q)
    _check(load_library().pevlm_block_prefill_attn_fp8(_ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(lse), layout.ref(),
                                                       heads.ref(), _ptr(workspace), workspace.numel(), int(stages),
                                                       _stream_ptr(stream)))
    return workspace


def pevlm_query_workspace_bytes(layout: Layout, heads: Heads, num_splits: int = 0) -> int:
    return int(load_library().pevlm_query_workspace_bytes(layout.ref(), heads.ref(), int(num_splits)))


def pevlm_query_attn(q, k, v, out, layout: Layout, heads: Heads, num_splits: int = 0, lse=None, workspace=None,
                     stream=None):
    if workspace is None:
        workspace = _workspace(pevlm_query_workspace_bytes(layout, heads, num_splits), q)
    _check(load_library().pevlm_query_attn(_ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(lse), layout.ref(),
                                           heads.ref(), int(num_splits), _ptr(workspace), workspace.numel(),
                                           _stream_ptr(stream)))
    return workspace


def pevlm_query_attn_static(q, k, v, out, layout: Layout, heads: Heads, num_splits: int = 0, lse=None, stream=None):
    _check(load_library().pevlm_query_attn_static(_ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(lse), layout.ref(),
                                                  heads.ref(), int(num_splits), _stream_ptr(stream)))


def _i32_array(values):
    a = np.ascontiguousarray(values, dtype=np.int32)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def pevlm_block_prefill_attn_blocks(q, k, v, out, layout: Layout, heads: Heads, first_block, num_blocks, with_sink: bool,
                                    lse=None, workspace=None, stream=None):
    if workspace is None:
        workspace = _workspace(pevlm_block_prefill_workspace_bytes(layout, heads), q)
    _fb, fbp = _i32_array(first_block)
    _nb, nbp = _i32_array(num_blocks)
    _check(load_library().pevlm_block_prefill_attn_blocks(_ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(lse), layout.ref(),
                                                          heads.ref(), fbp, nbp, int(bool(with_sink)), _ptr(workspace),
                                                          workspace.numel(), _stream_ptr(stream)))
    return workspace


def pevlm_query_window_workspace_bytes(layout: Layout, heads: Heads, num_splits: int = 0) -> int:
    return int(load_library().pevlm_query_window_workspace_bytes(layout.ref(), heads.ref(), int(num_splits)))


def pevlm_query_attn_window(q, k, v, out, layout: Layout, heads: Heads, window_blocks, num_splits: int = 0, lse=None,
                            workspace=None, stream=None):
    if workspace is None:
        workspace = _workspace(pevlm_query_window_workspace_bytes(layout, heads, num_splits), q)
    _w, wp = _i32_array(window_blocks)
    _check(load_library().pevlm_query_attn_window(_ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(lse), layout.ref(), heads.ref(),
                                                  wp, int(num_splits), _ptr(workspace), workspace.numel(),
                                                  _stream_ptr(stream)))
    return workspace


def pevlm_prefill_worklist_blocks_host(layout: Layout, tile_rows: int, first_block, num_blocks, with_sink: bool):
    lib = load_library()
    _fb, fbp = _i32_array(first_block)
    _nb, nbp = _i32_array(num_blocks)
    n = lib.pevlm_prefill_worklist_blocks_host(layout.ref(), tile_rows, fbp, nbp, int(bool(with_sink)), None, 0)
    if n < 0:
        raise PevlmError(PEVLM_ERR_INVALID_ARG, pevlm_last_error())
    items = (WorkItem * max(n, 1))()
    lib.pevlm_prefill_worklist_blocks_host(layout.ref(), tile_rows, fbp, nbp, int(bool(with_sink)), items, n)
    return [items[i] for i in range(n)]


def pevlm_query_worklist_window_host(layout: Layout, tile_rows: int, num_splits: int, window_blocks):
    lib = load_library()
    _w, wp = _i32_array(window_blocks)
    n = lib.pevlm_query_worklist_window_host(layout.ref(), tile_rows, num_splits, wp, None, 0)
    if n < 0:
        raise PevlmError(PEVLM_ERR_INVALID_ARG, pevlm_last_error())
    items = (WorkItem * max(n, 1))()
    lib.pevlm_query_worklist_window_host(layout.ref(), tile_rows, num_splits, wp, items, n)
    return [items[i] for i in range(n)]


def pevlm_prefill_worklist_host(layout: Layout, tile_rows: int):
    lib = load_library()
    n = lib.pevlm_prefill_worklist_host(layout.ref(), tile_rows, None, 0)
    if n < 0:
        raise PevlmError(PEVLM_ERR_INVALID_ARG, pevlm_last_error())
    items = (WorkItem * max(n, 1))()
    lib.pevlm_prefill_worklist_host(layout.ref(), tile_rows, items, n)
    return [items[i] for i in range(n)]


def pevlm_prefill_uses_stream_kernel(layout: Layout, heads: Heads) -> bool:
    return bool(load_library().pevlm_prefill_uses_stream_kernel(layout.ref(), heads.ref()))


def pevlm_set_prefill_kernel(mode) -> int:
    """mode: 0 / "auto", 1 / "classic", 2 / "stream"; returns the previous mode (int)."""
    code = {"auto": 0, "classic": 1, "stream": 2}.get(mode, mode)
    prev = int(load_library().pevlm_set_prefill_kernel(int(code)))
    if prev < 0:
        raise PevlmError(PEVLM_ERR_INVALID_ARG, "prefill kernel mode must be 0, 1 or 2")
    return prev


def pevlm_prefill_stream_items_host(layout: Layout, heads: Heads, first_block=None, num_blocks=None, with_sink: bool = True):
    lib = load_library()
    fbp = nbp = None
    if first_block is not None:
        _fb, fbp = _i32_array(first_block)
        _nb, nbp = _i32_array(num_blocks)
    n = lib.pevlm_prefill_stream_items_host(layout.ref(), heads.ref(), fbp, nbp, int(bool(with_sink)), None, 0)
    if n < 0:
        raise PevlmError(PEVLM_ERR_INVALID_ARG, pevlm_last_error())
    items = (StreamItem * max(n, 1))()
    lib.pevlm_prefill_stream_items_host(layout.ref(), heads.ref(), fbp, nbp, int(bool(with_sink)), items, n)
    return [items[i] for i in range(n)]


def pevlm_query_worklist_host(layout: Layout, tile_rows: int, num_splits: int):
    lib = load_library()
    n = lib.pevlm_query_worklist_host(layout.ref(), tile_rows, num_splits, None, 0)
    if n < 0:
        raise PevlmError(PEVLM_ERR_INVALID_ARG, pevlm_last_error())
    items = (WorkItem * max(n, 1))()
    lib.pevlm_query_worklist_host(layout.ref(), tile_rows, num_splits, items, n)
    return [items[i] for i in range(n)]


def pevlm_visible_pairs(layout: Layout):
    a, b, c = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int64()
    _check(load_library().pevlm_visible_pairs(layout.ref(), ctypes.byref(a), ctypes.byref(b), ctypes.byref(c)))
    return a.value, b.value, c.value
