"""Useful-FLOP accounting from the paper's operation counts (Sec. "Formulations", Eq. 6-10).

The paper counts 2*H operations per (query, key) pair with H = n_q_heads * head_dim (one GEMM).
Here both GEMMs (Q K^T and P V) are counted at 2 FLOP per multiply-add, i.e. 4 * head_dim per
visible pair per query head, and only pairs the mask keeps are counted (causal inside regions)."""
from __future__ import annotations

from .binding import Heads, Layout, pevlm_visible_pairs


def useful_flops(layout: Layout, heads: Heads):
    """Returns (prefill_flops, question_flops): sink + context-block rows, question rows."""
    sink, blocks, question = pevlm_visible_pairs(layout)
    per_pair = 4 * heads.head_dim * heads.n_q_heads
    return (sink + blocks) * per_pair, question * per_pair


# ---------------------------------------------------------------------------------------------
# Time model of the block-prefill call and the choice of sink and block size under a latency cap.
# The paper observes that both sizes trade accuracy against attention time and leaves their choice to
# tuning (Sec. on sink and block size; cost side: Eq. 7, Eq. 8 and Eq. 10, quadratic in both).
#
# Streaming kernel (one resident workgroup of 8 wavefronts per compute unit, items dealt round robin
# inside each XCD's eighth of the list): a workgroup needs
#     STREAM_US_PER_ITEM * items + STREAM_US_PER_TILE * key tiles of its items,
# and the launch takes as long as its slowest workgroup.  One-item-per-workgroup kernel (two
# workgroups of 4 wavefronts per compute unit, dispatched as slots free up):
#     time * (2 * CUs) = US_PER_WORKGROUP * workgroups + US_PER_WORKGROUP_TILE * sum of key tiles.
# The constants are fitted to measured runs on one MI355X (profiles/block_prefill_sweep.md); the
# predictions stay within +-12 % of them (head_dim 128).
STREAM_US_PER_ITEM = 3.48
STREAM_US_PER_TILE = 1.778
US_PER_WORKGROUP = 6.1
US_PER_WORKGROUP_TILE = 1.865
_TILE_ROWS, _KEY_TILE = 128, 64


def prefill_work(layout: Layout, heads: Heads):
    """(workgroups, workgroup key tiles) of the one-item-per-workgroup kernel, from the same host
    enumeration the library offers (items of <= 64 rows are taken for 2 or 4 heads of a KV group by
    one workgroup)."""
    from .binding import pevlm_prefill_worklist_host

    G = heads.n_q_heads // heads.n_kv_heads
    packs = G > 1 and heads.map is None
    n_wg = n_tiles = 0
    for it in pevlm_prefill_worklist_host(layout, _TILE_ROWS):
        tiles = -(-it.full_len // _KEY_TILE) + -(-it.diag_len // _KEY_TILE)
        groups32 = -(-it.q_rows // 32)
        hpw = (4 if groups32 <= 1 else 2 if groups32 <= 2 else 1) if packs else 1
        wgs = heads.n_kv_heads * -(-G // hpw)
        n_wg += wgs
        n_tiles += wgs * tiles
    return n_wg, n_tiles


def stream_work(layout: Layout, heads: Heads, compute_units: int = 256):
    """Per workgroup of the streaming kernel: (items, key tiles), as two arrays, following the
    kernel's own assignment (XCD x takes items [x * ceil(n/8), ...), its workgroups take them round
    robin)."""
    import ctypes

    import numpy as np

    from .binding import StreamItem, load_library

    lib = load_library()
    n = lib.pevlm_prefill_stream_items_host(layout.ref(), heads.ref(), None, None, 1, None, 0)
    if n <= 0:
        return np.zeros(0), np.zeros(0)
    items = (StreamItem * n)()
    lib.pevlm_prefill_stream_items_host(layout.ref(), heads.ref(), None, None, 1, items, n)
    words = ctypes.sizeof(StreamItem) // 4
    tiles = np.frombuffer(items, dtype=np.int32).reshape(n, words)[:, 6].astype(np.int64)  # n_tiles
    per_xcd = (n + 7) // 8
    wgs = min(max(compute_units // 8, 1), per_xcd)
    cnt, til = [], []
    for x in range(8):
        t = tiles[x * per_xcd:min(n, (x + 1) * per_xcd)]
        for j in range(wgs):
            cnt.append(len(t[j::wgs]))
            til.append(int(t[j::wgs].sum()))
    return np.asarray(cnt), np.asarray(til)


def predict_block_prefill_ms(layout: Layout, heads: Heads, compute_units: int = 256) -> float:
    from .binding import pevlm_prefill_uses_stream_kernel

    if pevlm_prefill_uses_stream_kernel(layout, heads):
        cnt, til = stream_work(layout, heads, compute_units)
        return float((STREAM_US_PER_ITEM * cnt + STREAM_US_PER_TILE * til).max()) * 1e-3
    n_wg, n_tiles = prefill_work(layout, heads)
    return (US_PER_WORKGROUP * n_wg + US_PER_WORKGROUP_TILE * n_tiles) / (2 * compute_units) * 1e-3


def choose_block_len(sink_len: int, ctx_len: int, query_len: int, heads: Heads, candidates, max_ms: float,
                     compute_units: int = 256):
    """Largest candidate block length (the paper's accuracy grows with the block size) whose
    predicted block-prefill time stays within max_ms; None if none does.  Returns (B, predicted_ms)."""
    best = None
    for B in sorted(candidates):
        lay = Layout.from_seqs([(sink_len, B, ctx_len, query_len)])
        ms = predict_block_prefill_ms(lay, heads, compute_units)
        if ms <= max_ms:
            best = (B, ms)
    return best


def video_layout(prefix_tokens: int, tokens_per_frame: int, n_frames: int, query_len: int, sink_frames: int,
                 block_frames: int):
    """(S, B, C, Q) of a video prompt partitioned as in Sec. "Partitioning Strategy": the sink is the
    text prefix plus the first sink_frames frames, the remaining frames form context blocks of
    block_frames frames (the last one may be shorter), the question follows."""
    sink_frames = min(sink_frames, n_frames)
    S = prefix_tokens + sink_frames * tokens_per_frame
    C = (n_frames - sink_frames) * tokens_per_frame
    return S, max(block_frames * tokens_per_frame, 1), C, query_len


def choose_sink_and_block(prefix_tokens: int, tokens_per_frame: int, n_frames: int, query_len: int, heads: Heads,
                          sink_frames, block_frames, max_ms: float, compute_units: int = 256):
    """Both knobs at once.  For every (sink frames, block frames) of the two candidate lists the
    block-prefill time is predicted; among the pairs within max_ms the one that keeps the most
    (query, key) pairs visible is returned -- the pair closest to full attention, which is the direction
    in which the paper's accuracy grows for both sizes -- ties going to the larger block.
    Returns (best, table): best = (sink_frames, block_frames, predicted_ms, visible_pairs) or None,
    table = that tuple for every candidate pair."""
    table = []
    for sf in sink_frames:
        for bf in block_frames:
            lay = Layout.from_seqs([video_layout(prefix_tokens, tokens_per_frame, n_frames, query_len, sf, bf)])
            sink, blocks, _question = pevlm_visible_pairs(lay)
            table.append((sf, bf, predict_block_prefill_ms(lay, heads, compute_units), sink + blocks))
    ok = [r for r in table if r[2] <= max_ms]
    best = max(ok, key=lambda r: (r[3], r[1])) if ok else None
    return best, table
