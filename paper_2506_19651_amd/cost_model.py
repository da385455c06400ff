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
# Time model of the block-prefill call and a block-length chooser (the paper's observation that the
# sink / block sizes trade accuracy against attention cost and "should be adaptively tuned",
# Sec. on sink and block size; cost side: Eq. 8 and Eq. 10).
#
# The bf16 kernel keeps two workgroups per compute unit busy; a launch's time is well described
# (+-10 % over all measured configurations, head_dim 128, MI355X) by
#     time * (2 * CUs) = US_PER_WORKGROUP * workgroups + US_PER_WORKGROUP_TILE * sum of key tiles,
# the first term being the per-item part (loads before the first tile, unpipelined first tile,
# epilogue), the second the steady-state tile loop.  Both constants are fitted to measured runs.
US_PER_WORKGROUP = 6.1
US_PER_WORKGROUP_TILE = 1.865
_TILE_ROWS, _KEY_TILE = 128, 64


def prefill_work(layout: Layout, heads: Heads):
    """(workgroups, workgroup key tiles) of pevlm_block_prefill_attn for bf16 tensors, from the same
    host enumeration the library offers (items of <= 64 rows are taken for 2 or 4 heads of a KV
    group by one workgroup)."""
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


def predict_block_prefill_ms(layout: Layout, heads: Heads, compute_units: int = 256) -> float:
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
