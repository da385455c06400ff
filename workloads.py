"""Seeded synthetic video-token workloads shared by the tests, the smoke check and the benchmark.

This module only describes shapes and draws random tensors; it contains none of the method's
arithmetic (no positions, no rotation, no masks, no attention).  Both the GPU library and the CPU
oracle are fed from the arrays produced here.

The workloads stand in for the paper's video inputs (Sec. "Experiments": 128-768 frames, 26k-100k
text+video tokens, sink and context blocks given in frames): they have the same structure
(a sink of prompt + first frames, frame-aligned context blocks, a short trailing question; GQA head
shapes of the 7B models evaluated) but random contents.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Tuple

import numpy as np

GLOBAL_SEED = 250619651
TENSOR_Q, TENSOR_K, TENSOR_V, TENSOR_OFFSET, TENSOR_ROWS = 0, 1, 2, 3, 4


@dataclass
class Workload:
    name: str
    config_id: int
    dtype: str  # "f32" or "bf16"
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    rope_base: float
    seqs: List[Tuple[int, int, int, int]]  # per sequence (sink S, block B, context C, question Q)
    value_scale: float = 1.0
    key_offset_scale: float = 0.0  # std of a per-KV-head mean added to every key (sink skew)
    note: str = ""
    qk_scale: float = 1.0  # extra factor on Q and K only (peaky softmax)
    key_ramp: float = 1.0  # keys grow linearly to this factor along each sequence (rising maxima)

    @property
    def cu_seqlens(self) -> np.ndarray:
        lens = [s + c + q for (s, _b, c, q) in self.seqs]
        return np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)

    @property
    def total_tokens(self) -> int:
        return int(self.cu_seqlens[-1])

    def layout_arrays(self) -> Dict[str, np.ndarray]:
        a = np.asarray(self.seqs, dtype=np.int32).reshape(-1, 4)
        return dict(cu_seqlens=self.cu_seqlens, sink_len=a[:, 0].copy(), block_len=a[:, 1].copy(),
                    ctx_len=a[:, 2].copy(), query_len=a[:, 3].copy())


def _frames(n_frames: int, tokens_per_frame: int) -> int:
    return n_frames * tokens_per_frame


def _configs() -> Dict[str, Workload]:
    w: Dict[str, Workload] = {}
    # c1: tiny fp32 sanity. sink 32, 4 frames x 16 tokens, 1 frame per block, 8 question tokens.
    w["c1"] = Workload("c1", 1, "f32", 2, 1, 64, 1.0e4, [(32, 16, 64, 8)], 1.0)
    # c2: Qwen2-VL-7B-shaped layer. sink 256, 64 frames x 256 tokens in 16 blocks of 4 frames, 64 q.
    w["c2"] = Workload("c2", 2, "bf16", 28, 4, 128, 1.0e6, [(256, 1024, _frames(64, 256), 64)], 0.5)
    # c3: headline. 256 frames x 256 tokens in 64 blocks of 1024, 128 q, per-head key mean offset.
    w["c3"] = Workload("c3", 3, "bf16", 28, 4, 128, 1.0e6, [(256, 1024, _frames(256, 256), 128)], 0.5,
                       key_offset_scale=0.3)
    # c4: larger GQA, block-length sweep over 2/4/8/16 frames of 196 tokens; sink 392 is extra.
    for tag, fpb in (("a", 2), ("b", 4), ("c", 8), ("d", 16)):
        w["c4" + tag] = Workload("c4" + tag, 4, "bf16", 32, 8, 128, 1.0e6,
                                 [(392, fpb * 196, _frames(512, 196), 256)], 0.5,
                                 note=f"block = {fpb} frames")
    # c5a: ragged batch taken literally (all blocks full); c5b: one frame off so the last block of
    # every sequence is partial.
    w["c5a"] = Workload("c5a", 5, "bf16", 28, 4, 128, 1.0e6,
                        [(256, 1024, _frames(f, 256), 64) for f in (32, 96, 160, 256)], 0.5)
    w["c5b"] = Workload("c5b", 5, "bf16", 28, 4, 128, 1.0e6,
                        [(256, 1024, _frames(f, 256), 64) for f in (33, 97, 161, 255)], 0.5,
                        note="partial last blocks")
    # Same token sequence as c3 laid out as one dense causal block: the full-attention comparison.
    w["c3_full_causal"] = Workload("c3_full_causal", 3, "bf16", 28, 4, 128, 1.0e6,
                                   [(0, 65920, 65920, 0)], 0.5, key_offset_scale=0.3,
                                   note="c3 tokens, no sink, one block, no question")
    return w


CONFIGS: Dict[str, Workload] = _configs()


def small_variant(w: Workload, name: str, seqs, **kw) -> Workload:
    """Same head shape / dtype / distribution as `w` on a smaller partition (parity cases that the
    oracle finishes in seconds)."""
    d = dict(name=name, config_id=w.config_id, dtype=w.dtype, n_q_heads=w.n_q_heads,
             n_kv_heads=w.n_kv_heads, head_dim=w.head_dim, rope_base=w.rope_base, seqs=list(seqs),
             value_scale=w.value_scale, key_offset_scale=w.key_offset_scale)
    d.update(kw)
    return Workload(**d)


# ----------------------------------------------------------------------------- storage rounding
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even float32 -> bf16 bit patterns (uint16), in slabs to bound temporaries."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    out = np.empty(x.shape, dtype=np.uint16)
    xf, of = x.reshape(-1), out.reshape(-1)
    step = 1 << 22
    for lo in range(0, xf.size, step):
        u = xf[lo:lo + step].view(np.uint32)
        r = (u >> np.uint32(16)) & np.uint32(1)
        r += np.uint32(0x7FFF)
        r += u
        r >>= np.uint32(16)
        of[lo:lo + step] = r
    return out


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


# ----------------------------------------------------------------------------- tensors
def _rng(config_id: int, seq_idx: int, tensor_id: int, seed: int) -> np.random.Generator:
    ss = np.random.SeedSequence(entropy=seed, spawn_key=(config_id, seq_idx, tensor_id))
    return np.random.Generator(np.random.Philox(ss))


def generate(w: Workload, seed: int = GLOBAL_SEED) -> Dict[str, np.ndarray]:
    """Draw Q [T,Hq,D], K, V [T,Hkv,D] i.i.d. N(0,1) * value_scale (keys additionally shifted by a
    per-KV-head mean when key_offset_scale > 0), one Philox stream per (config, sequence, tensor).
    Returns float32 arrays for f32 workloads and uint16 bf16 bit patterns for bf16 workloads: the
    values handed to the GPU and to the oracle are identical."""
    T, D = w.total_tokens, w.head_dim
    store = np.float32 if w.dtype == "f32" else np.uint16
    out = {"q": np.empty((T, w.n_q_heads, D), store), "k": np.empty((T, w.n_kv_heads, D), store),
           "v": np.empty((T, w.n_kv_heads, D), store)}
    cu = w.cu_seqlens
    for si in range(len(w.seqs)):
        lo, hi = int(cu[si]), int(cu[si + 1])
        n = hi - lo
        for name, tid, H in (("q", TENSOR_Q, w.n_q_heads), ("k", TENSOR_K, w.n_kv_heads),
                             ("v", TENSOR_V, w.n_kv_heads)):
            x = _rng(w.config_id, si, tid, seed).standard_normal((n, H, D), dtype=np.float32)
            x *= np.float32(w.value_scale)
            if name in ("q", "k") and w.qk_scale != 1.0:
                x *= np.float32(w.qk_scale)
            if name == "k" and w.key_ramp != 1.0:
                x *= np.linspace(1.0, w.key_ramp, n, dtype=np.float32)[:, None, None]
            if name == "k" and w.key_offset_scale > 0.0:
                mu = _rng(w.config_id, si, TENSOR_OFFSET, seed).standard_normal((1, H, D), dtype=np.float32)
                x += mu * np.float32(w.key_offset_scale)
            out[name][lo:hi] = x if w.dtype == "f32" else f32_to_bf16_bits(x)
    return out


def as_float32(a: np.ndarray) -> np.ndarray:
    return a if a.dtype == np.float32 else bf16_bits_to_f32(a)


# ----------------------------------------------------------------------------- 3-axis position ids
def mrope_position_ids(w: Workload, frame_tokens: int, grid_w: int) -> np.ndarray:
    """Three-axis (temporal, height, width) position ids [3, T] of a video prompt, an INPUT of the
    multimodal-RoPE call (no rotation arithmetic here).  Each sequence is read as: text prefix
    (the sink minus its last `frame_tokens` tokens, if it is that long), then video frames of
    `frame_tokens` tokens laid out row-major on a grid `grid_w` wide (end of sink + all context
    tokens; a trailing partial frame is a truncated grid), then the question as text.  A text token
    takes the running counter on all three axes; a run of frames that starts at counter n0 gives
    frame f, row r, column c the ids (n0 + f, n0 + r, n0 + c); the counter then continues after the
    largest id used.  Ids are those of the whole prompt: nothing restarts at a block boundary."""
    ids = np.zeros((3, w.total_tokens), dtype=np.int32)
    t0 = 0
    for (S, _B, C, Q) in w.seqs:
        n_text = S - frame_tokens if S >= frame_tokens else S
        n_video = (S - n_text) + C
        n = 0
        ids[:, t0:t0 + n_text] = np.arange(n_text, dtype=np.int32)[None, :]
        n += n_text
        if n_video > 0:
            j = np.arange(n_video, dtype=np.int32)
            f, rem = j // frame_tokens, j % frame_tokens
            r, c = rem // grid_w, rem % grid_w
            v0 = t0 + n_text
            ids[0, v0:v0 + n_video] = n + f
            ids[1, v0:v0 + n_video] = n + r
            ids[2, v0:v0 + n_video] = n + c
            n += int(max(f.max(), r.max(), c.max())) + 1
        q0 = t0 + S + C
        ids[:, q0:q0 + Q] = n + np.arange(Q, dtype=np.int32)[None, :]
        t0 += S + C + Q
    return ids


# ----------------------------------------------------------------------------- row samples
def sample_rows(w: Workload, n_random: int = 512, tile: int = 128, seed: int = GLOBAL_SEED,
                max_question_rows: Optional[int] = None) -> np.ndarray:
    """Deterministic sample of packed rows on which large workloads are compared with the oracle:
    per sequence the first and last row of every region; both sides of every block boundary of the
    first, a middle and the last block; both sides of every `tile`-row edge inside the first block;
    all question rows; plus n_random seeded-random rows over the whole batch."""
    rows: List[int] = []
    cu = w.cu_seqlens
    for si, (S, B, C, Q) in enumerate(w.seqs):
        base = int(cu[si])
        L = S + C + Q
        add = lambda p: rows.append(base + p) if 0 <= p < L else None
        for lo, n in ((0, S), (S, C), (S + C, Q)):
            if n > 0:
                add(lo), add(lo + n - 1)
        nb = (C + B - 1) // B if C > 0 else 0
        for b in sorted({0, nb // 2, nb - 1}) if nb else []:
            b0 = S + b * B
            b1 = min(S + C, b0 + B)
            for p in (b0 - 1, b0, b0 + 1, b1 - 2, b1 - 1, b1):
                add(p)
        if nb:
            for e in range(S + tile, min(S + B, S + C), tile):
                add(e - 1), add(e)
        for e in range(tile, S, tile):
            add(e - 1), add(e)
        qrows = range(S + C, L)
        if max_question_rows is not None and Q > max_question_rows:
            step = Q / max_question_rows
            qrows = sorted({S + C + int(i * step) for i in range(max_question_rows)} | {L - 1})
        for p in qrows:
            add(p)
    T = w.total_tokens
    if n_random > 0 and T > 0:
        r = _rng(w.config_id, 0, TENSOR_ROWS, seed).integers(0, T, size=n_random)
        rows.extend(int(x) for x in r)
    return np.unique(np.asarray(rows, dtype=np.int64))
