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
