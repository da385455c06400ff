"""Helpers of the GPU parity tests: move seeded host arrays to the device, run the three library
calls through the Python binding (which forwards to the C ABI), bring results back."""
import numpy as np
import torch

import paper_2506_19651_amd as P
import workloads as W

DEV = "cuda:0"


def to_device(a: np.ndarray) -> torch.Tensor:
    if a.dtype == np.uint16:  # bf16 bit patterns
        return torch.from_numpy(a.view(np.int16)).to(DEV).view(torch.bfloat16)
    return torch.from_numpy(a).to(DEV)


def to_host_f32(t: torch.Tensor) -> np.ndarray:
    return t.float().cpu().numpy()


def layout_heads(w: W.Workload, kv_head_of_q=None, softmax_scale=0.0):
    return P.Layout.from_seqs(w.seqs), P.Heads(w.n_q_heads, w.n_kv_heads, w.head_dim, w.dtype, kv_head_of_q,
                                               softmax_scale)


def run_path(w: W.Workload, data, num_splits=0, pos_offset=None, kv_head_of_q=None, want_lse=False,
             softmax_scale=0.0, poison=True):
    """rope -> block prefill -> question attention.  Returns dict(out, lse, q_rot, k_rot) on host."""
    lay, heads = layout_heads(w, kv_head_of_q, softmax_scale)
    q, k, v = to_device(data["q"]), to_device(data["k"]), to_device(data["v"])
    out = torch.full_like(q, float("nan")) if poison else torch.zeros_like(q)
    lse = torch.full((w.total_tokens, w.n_q_heads), float("nan"), device=DEV) if want_lse else None
    P.pevlm_rope_seq(q, k, lay, heads, w.rope_base, pos_offset)
    P.pevlm_block_prefill_attn(q, k, v, out, lay, heads, lse=lse)
    after_prefill = out.clone() if poison else None
    P.pevlm_query_attn(q, k, v, out, lay, heads, num_splits=num_splits, lse=lse)
    torch.cuda.synchronize()
    return dict(out=out, lse=lse, q_rot=q, k_rot=k, v=v, after_prefill=after_prefill, lay=lay, heads=heads)


def oracle_layout(oracle, w: W.Workload):
    a = w.layout_arrays()
    return oracle.Layout(a["cu_seqlens"], a["sink_len"], a["block_len"], a["ctx_len"], a["query_len"])


def error_stats(got: np.ndarray, want: np.ndarray):
    d = np.abs(got.astype(np.float64) - want)
    rel = np.sqrt((d ** 2).sum(-1)) / np.maximum(np.sqrt((want ** 2).sum(-1)), 1e-30)
    return dict(max_abs=float(d.max()), mean_abs=float(d.mean()), max_rel_l2=float(rel.max()))
