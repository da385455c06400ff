"""pevlm_query_attn_static (the question call whose scratch memory is an array inside the library,
for callers that cannot allocate): its output must equal pevlm_query_attn's bit for bit, on two
calls in a row, the second on a smaller input, and sizes beyond the built-in array are rejected."""
import numpy as np
import pytest
import torch

import paper_2506_19651_amd as P
import workloads as W
from gpu_util import DEV, layout_heads, oracle_layout, to_device, to_host_f32

pytestmark = pytest.mark.gpu


def _both(w, splits):
    data = W.generate(w)
    lay, heads = layout_heads(w)
    q, k, v = to_device(data["q"]), to_device(data["k"]), to_device(data["v"])
    P.pevlm_rope_seq(q, k, lay, heads, w.rope_base)
    ref = torch.full_like(q, float("nan"))
    ref_lse = torch.full((w.total_tokens, w.n_q_heads), float("nan"), device=DEV)
    P.pevlm_query_attn(q, k, v, ref, lay, heads, num_splits=splits, lse=ref_lse)
    out = torch.full_like(q, float("nan"))
    lse = torch.full((w.total_tokens, w.n_q_heads), float("nan"), device=DEV)
    before = torch.cuda.memory_allocated()
    P.pevlm_query_attn_static(q, k, v, out, lay, heads, num_splits=splits, lse=lse)
    assert torch.cuda.memory_allocated() == before  # nothing taken from torch's allocator either
    torch.cuda.synchronize()
    return data, q, k, ref, ref_lse, out, lse


def _same(a, b):
    bits = torch.int16 if a.dtype == torch.bfloat16 else torch.int32
    return torch.equal(a.view(bits), b.view(bits))  # NaN-poisoned untouched rows compare equal as bits


def test_static_scratch_call_equals_workspace_call_on_two_calls_in_a_row(oracle):
    big = W.Workload("static_big", 31, "bf16", 8, 2, 128, 1.0e6, [(300, 392, 3000, 200), (0, 128, 700, 70)], 0.5)
    small = W.Workload("static_small", 32, "bf16", 8, 2, 128, 1.0e6, [(64, 100, 450, 33)], 0.5)
    for w, splits in ((big, 6), (small, 3)):  # the second call finds the first call's partials in the scratch
        data, q, k, ref, ref_lse, out, lse = _both(w, splits)
        assert _same(out, ref) and _same(lse, ref_lse)
        # and against the oracle (question rows)
        a = w.layout_arrays()
        qrows = np.concatenate([np.arange(c0 + S + C, c0 + S + C + Q) for c0, (S, B, C, Q) in zip(a["cu_seqlens"], w.seqs)])
        want, _ = oracle.forward(data["q"], data["k"], data["v"], oracle_layout(oracle, w), w.rope_base, rows=qrows)
        got = to_host_f32(out[torch.from_numpy(qrows).to(DEV)])
        d = np.abs(got - want)
        assert np.isfinite(got).all() and d.max() <= 2e-2 and d.mean() <= 2e-3
    # fp32 tensors, automatic split count, then a smaller one again
    for seqs in ([(40, 33, 150, 21), (3, 16, 64, 7)], [(5, 8, 24, 6)]):
        w = W.Workload("static_f32", 33, "f32", 4, 2, 64, 1.0e4, seqs, 1.0)
        _d, q, k, ref, ref_lse, out, lse = _both(w, 0)
        assert _same(out, ref) and _same(lse, ref_lse)


def test_static_scratch_call_rejects_what_does_not_fit():
    # 512 question rows x 32 heads x 64 splits of fp32 partials: far beyond the built-in array
    w = W.Workload("static_too_big", 34, "bf16", 32, 8, 128, 1.0e6, [(0, 64, 64, 512)], 0.5)
    lay, heads = layout_heads(w)
    assert P.pevlm_query_workspace_bytes(lay, heads, 64) > (64 << 20)
    q = torch.zeros((w.total_tokens, 32, 128), dtype=torch.bfloat16, device=DEV)
    k = torch.zeros((w.total_tokens, 8, 128), dtype=torch.bfloat16, device=DEV)
    out = torch.full_like(q, float("nan"))
    with pytest.raises(P.PevlmError, match="scratch"):
        P.pevlm_query_attn_static(q, k, k, out, lay, heads, num_splits=64)
    torch.cuda.synchronize()
    assert torch.isnan(out).all()  # nothing was enqueued
    # the same layout with few splits fits and runs
    P.pevlm_query_attn_static(q, k, k, out, lay, heads, num_splits=2)
    torch.cuda.synchronize()
    assert torch.isfinite(out[64:].float()).all()
