#!/usr/bin/env python3
"""Benchmark of the PEVLM prefill attention path on one MI355X.

A step is one pass of the whole hot path over the 64K-token workload (c3): sequential RoPE of Q and
K, block-parallel prefill attention (sink + 64 context blocks), split-KV question attention + merge.
Inputs are resident in HBM before the timed region.  Prints ONE JSON line:
  value      useful TFLOP/s of the whole path (only unmasked FLOPs: 4*D per visible pair per head)
  roofline   the dominant kernel (block-prefill attention) against the bf16 MFMA peak, its duration
             measured with HIP events on the launch stream inside the timed region
  cpu_baseline  the fp64 CPU oracle timed on a bounded row sample of the same workload
and, as context, ms per kernel (mean, median, min), this build's own dense full-causal attention on
the same tokens and the resulting attention speedup (the paper reports up to 7.47x on one H20-96G),
the question kernel with its K/V flushed out of the caches first ("cold"), and what the device
sustains on a register-resident bf16 MFMA loop and on a 1 GiB streaming copy ("measured_peaks").
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 matrix peak
MFMA_FP8_PEAK_TFLOPS = 5000.0   # ... dense fp8
# HBM bytes per block-prefill launch from the FETCH_SIZE / WRITE_SIZE passes recorded in
# profiles/attn_bf16_prefill_c3_counters.md (scaled by the same counters on a 1 GiB device copy)
MEASURED_PREFILL_TRAFFIC_BYTES = {("c3", "attn_bf16_stream_kernel<128>"): 1.280e9}
HBM_PEAK_GBS = 8000.0


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="c3")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-full-causal", action="store_true")
    ap.add_argument("--num-splits", type=int, default=0)
    ap.add_argument("--no-probes", action="store_true", help="skip the MFMA-rate / copy / cold-cache side measurements")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the widened calls (RoPE folded into attention, streaming, three-axis RoPE): profiler runs "
                         "use this so that every kernel name stands for one kind of launch")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU only: this path uses no collectives and every GPU box here has one "
              "GPU; run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2506_19651_amd as P
    import workloads as W

    if not os.path.exists(P.lib_path()):
        from paper_2506_19651_amd.build import build_library
        build_library()
    P.load_library()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    w = W.CONFIGS[args.workload]
    assert w.dtype == "bf16"
    data = W.generate(w)

    def to_dev(a):
        return torch.from_numpy(a.view(np.int16)).to(dev).view(torch.bfloat16)

    lay = P.Layout.from_seqs(w.seqs)
    heads = P.Heads(w.n_q_heads, w.n_kv_heads, w.head_dim, w.dtype)
    q0, k0, v = to_dev(data["q"]), to_dev(data["k"]), to_dev(data["v"])
    # q, k: rotated once (what the attention calls of every step read); qs, ks: the tensors the timed
    # RoPE call rotates in place step after step (its time does not depend on the values)
    q, k = q0.clone(), k0.clone()
    qs, ks = q0.clone(), k0.clone()
    P.pevlm_rope_seq(q, k, lay, heads, w.rope_base)
    out = torch.zeros_like(q)
    ws_p = torch.empty(P.pevlm_block_prefill_workspace_bytes(lay, heads), dtype=torch.uint8, device=dev)
    ws_q = torch.empty(P.pevlm_query_workspace_bytes(lay, heads, args.num_splits), dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream()

    def step(ev=None):
        if ev:
            ev[0].record(stream)
        P.pevlm_rope_seq(qs, ks, lay, heads, w.rope_base, stream=stream)
        if ev:
            ev[1].record(stream)
        P.pevlm_block_prefill_attn(q, k, v, out, lay, heads, workspace=ws_p, stream=stream)
        if ev:
            ev[2].record(stream)
        P.pevlm_query_attn(q, k, v, out, lay, heads, num_splits=args.num_splits, workspace=ws_q, stream=stream)
        if ev:
            ev[3].record(stream)

    def timed(fn, reps):
        fn()
        torch.cuda.synchronize()
        ts = []
        for _ in range(reps):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(stream)
            fn()
            b.record(stream)
            torch.cuda.synchronize()
            ts.append(a.elapsed_time(b))
        return float(np.median(ts))

    peaks = None
    if not args.no_probes:
        # What the device sustains, measured BEFORE the steps: bf16 MFMA issue (two workgroups per CU, as
        # the attention kernel runs), a 1 GiB streaming copy (also the known-size kernel that scales the
        # FETCH_SIZE / WRITE_SIZE counters of a profiler pass over this same command) and the kernels' own
        # tile step in a bare loop (no per-item work, no masks; the K tensor of the workload as data), with
        # and without the softmax arithmetic.  Running them first also means that the warm-up steps start
        # on a device that has been under load for ~0.1 s: after an idle stretch the first ~35 launches of
        # any kernel run 5-30 % slow while the clocks settle, which 5 warm-up steps alone do not cover.
        scratch = torch.zeros(64, dtype=torch.float32, device=dev)
        n_cu = torch.cuda.get_device_properties(0).multi_processor_count
        flops = P.pevlm_probe_mfma_bf16(scratch, 2 * n_cu, 8000, stream=stream)
        ms_m = timed(lambda: P.pevlm_probe_mfma_bf16(scratch, 2 * n_cu, 8000, stream=stream), 5)
        gib = 1 << 30
        src = torch.empty(gib, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty(gib, dtype=torch.uint8, device=dev)
        ms_c = timed(lambda: P.pevlm_probe_copy(dst, src, gib, stream=stream), 5)
        peaks = {"mfma_bf16_tflops": flops / (ms_m * 1e-3) / 1e12, "hbm_copy_gbs": 2 * gib / (ms_c * 1e-3) / 1e9}
        kv_probe = k[: 40 * 64].contiguous() if w.head_dim == 128 else None
        if kv_probe is not None and kv_probe.numel() * 2 >= 4 * 16384:
            fl_t = P.pevlm_probe_tile_loop_bf16(scratch, kv_probe, 2 * n_cu, 2000, True, stream=stream)
            ms_t = timed(lambda: P.pevlm_probe_tile_loop_bf16(scratch, kv_probe, 2 * n_cu, 2000, True, stream=stream), 5)
            ms_t0 = timed(lambda: P.pevlm_probe_tile_loop_bf16(scratch, kv_probe, 2 * n_cu, 2000, False, stream=stream), 5)
            peaks["tile_loop"] = (fl_t / (ms_t * 1e-3) / 1e12, fl_t / (ms_t0 * 1e-3) / 1e12)

    # first pass: kept for the accuracy figures reported next to the timing (every later pass
    # computes the same output from the same once-rotated q, k)
    step()
    torch.cuda.synchronize()
    first_out = out.clone()

    for _ in range(args.warmup):
        step()
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(events[i])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_step = (t1 - t0) * 1e3 / args.steps
    t_rope = np.array([e[0].elapsed_time(e[1]) for e in events])
    t_prefill = np.array([e[1].elapsed_time(e[2]) for e in events])
    t_query = np.array([e[2].elapsed_time(e[3]) for e in events])
    ms_rope, ms_prefill, ms_query = float(t_rope.mean()), float(t_prefill.mean()), float(t_query.mean())

    f_prefill, f_query = P.useful_flops(lay, heads)
    # which of the two block-prefill kernels the library ran for this layout (its own per-call choice)
    prefill_kernel_name = (f"attn_bf16_stream_kernel<{w.head_dim}>" if P.pevlm_prefill_uses_stream_kernel(lay, heads)
                           else f"attn_bf16_kernel<{w.head_dim},false,false>")
    T = w.total_tokens
    rope_bytes = 2 * T * (w.n_q_heads + w.n_kv_heads) * w.head_dim * 2
    kv_bytes = 2 * T * w.n_kv_heads * w.head_dim * 2

    result = {
        "metric": "pevlm_prefill_attention_useful_tflops",
        "value": round((f_prefill + f_query) / (ms_step * 1e-3) / 1e12, 3),
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": f"{w.name}: {len(w.seqs)} sequence(s), sink {w.seqs[0][0]}, blocks of {w.seqs[0][1]} "
                               f"({', '.join(str(-(-c // b)) for (_s, b, c, _q) in w.seqs)} per sequence), "
                               f"question {w.seqs[0][3]}, T={T}, {w.n_q_heads}/{w.n_kv_heads} heads x {w.head_dim}",
                   "tokens": T, "num_splits": args.num_splits},
        "ms_per_layer": round(ms_rope + ms_prefill + ms_query, 4),
        "ms_rope": round(ms_rope, 4),
        "ms_block_prefill": round(ms_prefill, 4),
        "ms_query_attn": round(ms_query, 4),
        "ms_median_min": {"rope": [round(float(np.median(t_rope)), 4), round(float(t_rope.min()), 4)],
                          "block_prefill": [round(float(np.median(t_prefill)), 4), round(float(t_prefill.min()), 4)],
                          "query_attn": [round(float(np.median(t_query)), 4), round(float(t_query.min()), 4)]},
        "block_prefill_useful_tflops": round(f_prefill / (ms_prefill * 1e-3) / 1e12, 2),
        "query_attn_useful_tflops": round(f_query / (ms_query * 1e-3) / 1e12, 2),
        "rope_gbs": round(rope_bytes / (ms_rope * 1e-3) / 1e9, 1),
        "query_kv_gbs": round(kv_bytes / (ms_query * 1e-3) / 1e9, 1),
        "roofline": {
            "kernel": prefill_kernel_name + " (block-prefill)",
            "bound": "mfma",
            "achieved": round(f_prefill / (ms_prefill * 1e-3) / 1e12, 2),
            "peak": MFMA_BF16_PEAK_TFLOPS,
            "unit": "TFLOP/s",
            "frac": round(f_prefill / (ms_prefill * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
            "traffic": MEASURED_PREFILL_TRAFFIC_BYTES.get((args.workload, prefill_kernel_name)),
        },
        "paper_context": "paper reports up to 7.47x attention speedup on one NVIDIA H20-96G (bf16, ~100k tokens)",
    }

    if not args.no_extras:
        # the same step with RoPE folded into the attention calls (the prefill call rotates K in place and
        # fills the cos/sin table; q0 stays un-rotated); outputs are bit-identical to the three-call path
        ws_pf = torch.empty(P.pevlm_block_prefill_rope_workspace_bytes(lay, heads), dtype=torch.uint8, device=dev)
        ws_qf = torch.empty(P.pevlm_query_rope_workspace_bytes(lay, heads, args.num_splits), dtype=torch.uint8, device=dev)
        out_f = torch.zeros_like(q0)

        def step_fused(ev=None):
            if ev:
                ev[0].record(stream)
            if ev:
                ev[1].record(stream)
            P.pevlm_block_prefill_attn_rope(q0, kf, v, out_f, lay, heads, w.rope_base, workspace=ws_pf, stream=stream)
            if ev:
                ev[2].record(stream)
            P.pevlm_query_attn_rope(q0, kf, v, out_f, lay, heads, w.rope_base, num_splits=args.num_splits, workspace=ws_qf,
                                    stream=stream)
            if ev:
                ev[3].record(stream)

        kf = k0.clone()  # rotated in place by every fused step (timing only; the first pass is the checked one)
        step_fused()
        torch.cuda.synchronize()
        fused_matches = bool(torch.equal(out_f.view(torch.int16), first_out.view(torch.int16)))
        for _ in range(args.warmup):
            step_fused()
        events_f = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
        torch.cuda.synchronize()
        tf0 = time.perf_counter()
        for i in range(args.steps):
            step_fused(events_f[i])
        torch.cuda.synchronize()
        tf1 = time.perf_counter()
        ms_step_f = (tf1 - tf0) * 1e3 / args.steps
        result["fused_rope"] = {
            "ms_per_step": round(ms_step_f, 4),
            "value": round((f_prefill + f_query) / (ms_step_f * 1e-3) / 1e12, 3),
            "ms_block_prefill_incl_k_rope": round(float(np.mean([e[1].elapsed_time(e[2]) for e in events_f])), 4),
            "ms_query_attn": round(float(np.mean([e[2].elapsed_time(e[3]) for e in events_f])), 4),
            "bit_identical_to_three_call_path": fused_matches,
        }

    if not args.no_extras:
        # fp8 (E4M3) variant of the block-prefill call: quantise stage (bf16 -> codes, K/V re-tiled) and
        # attention stage timed separately and together; judged against the fp8 matrix peak
        ws_8 = torch.empty(P.pevlm_block_prefill_fp8_workspace_bytes(lay, heads), dtype=torch.uint8, device=dev)
        out_8 = torch.zeros_like(q)

        def timed_stage(stages):
            P.pevlm_block_prefill_attn_fp8(q, k, v, out_8, lay, heads, workspace=ws_8, stages=stages, stream=stream)
            torch.cuda.synchronize()
            ts = []
            for _ in range(max(5, args.steps // 2)):
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record(stream)
                P.pevlm_block_prefill_attn_fp8(q, k, v, out_8, lay, heads, workspace=ws_8, stages=stages, stream=stream)
                b.record(stream)
                torch.cuda.synchronize()
                ts.append(a.elapsed_time(b))
            return float(np.mean(ts))

        ms_8q, ms_8a, ms_8 = timed_stage(P.FP8_QUANTISE), timed_stage(P.FP8_ATTEND), timed_stage(0)
        a_ = w.layout_arrays()
        pre_rows = torch.cat([torch.arange(int(c0), int(c0) + s_ + c_, device=dev)
                              for c0, (s_, _b, c_, _q) in zip(a_["cu_seqlens"], w.seqs)])
        diff8 = (out_8[pre_rows].float() - first_out[pre_rows].float()).abs()
        result["fp8_block_prefill"] = {
            "ms_quantise": round(ms_8q, 4), "ms_attend": round(ms_8a, 4), "ms_both": round(ms_8, 4),
            "attend_useful_tflops": round(f_prefill / (ms_8a * 1e-3) / 1e12, 2),
            "roofline": {"kernel": f"attn_fp8_kernel<{w.head_dim}>", "bound": "mfma", "peak": MFMA_FP8_PEAK_TFLOPS, "unit": "TFLOP/s",
                         "achieved": round(f_prefill / (ms_8a * 1e-3) / 1e12, 2),
                         "frac": round(f_prefill / (ms_8a * 1e-3) / 1e12 / MFMA_FP8_PEAK_TFLOPS, 4)},
            "speedup_of_attend_over_bf16_kernel": round(ms_prefill / ms_8a, 3),
            "max_abs_diff_to_bf16_path": float(diff8.max()), "mean_abs_diff_to_bf16_path": float(diff8.mean()),
        }
        del ws_8, out_8

    if not args.no_probes:
        mfma_rate, copy_rate = peaks["mfma_bf16_tflops"], peaks["hbm_copy_gbs"]
        result["measured_peaks"] = {"mfma_bf16_tflops": round(mfma_rate, 1), "hbm_copy_gbs": round(copy_rate, 1),
                                    "how": "register-resident v_mfma_f32_32x32x16_bf16 loop, 2 workgroups/CU; 1 GiB device copy (read+write bytes)"}
        result["roofline"]["frac_of_measured_mfma_rate"] = round(result["roofline"]["achieved"] / mfma_rate, 4)
        if "tile_loop" in peaks:
            tile_rate, tile_rate0 = peaks["tile_loop"]
            result["measured_peaks"]["tile_loop_bf16_tflops"] = round(tile_rate, 1)
            result["measured_peaks"]["tile_loop_bf16_tflops_without_softmax"] = round(tile_rate0, 1)
            result["measured_peaks"]["tile_loop_how"] = ("the kernels' tile routines in a bare loop on workload data, 2 workgroups/CU: MFMAs, "
                                                         "LDS fragment reads, global->LDS tile loads, barrier (+ weights arithmetic)")
            # the real kernel's useful rate against the bare loop
            result["roofline"]["frac_of_tile_loop_rate"] = round(result["roofline"]["achieved"] / tile_rate, 4)
        result["rope_frac_of_measured_copy_rate"] = round(result["rope_gbs"] / copy_rate, 4)
        # question attention with K/V evicted: the 1 GiB copy (4x the 256 MB last-level cache) runs
        # right before each timed launch
        cold = []
        for _ in range(5):
            P.pevlm_probe_copy(dst, src, gib, stream=stream)
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(stream)
            P.pevlm_query_attn(q, k, v, out, lay, heads, num_splits=args.num_splits, workspace=ws_q, stream=stream)
            b.record(stream)
            torch.cuda.synchronize()
            cold.append(a.elapsed_time(b))
        result["ms_query_attn_cold"] = round(float(np.median(cold)), 4)
        result["query_kv_gbs_cold"] = round(kv_bytes / (float(np.median(cold)) * 1e-3) / 1e9, 1)
        del src, dst
        # streaming calls: one more context block appended to the prompt (rows of the last block only),
        # and the question restricted to the sink plus the newest quarter of the blocks
        nblk = [(-(-c // b) if c else 0) for (_s, b, c, _q) in w.seqs]
        if min(nblk) >= 4 and not args.no_extras:
            first, one = [n - 1 for n in nblk], [1] * len(nblk)
            ms_blk = timed(lambda: P.pevlm_block_prefill_attn_blocks(q, k, v, out, lay, heads, first, one, False,
                                                                     workspace=ws_p, stream=stream), 10)
            win = [n // 4 for n in nblk]
            ws_w = torch.empty(P.pevlm_query_window_workspace_bytes(lay, heads, 0), dtype=torch.uint8, device=dev)
            ms_win = timed(lambda: P.pevlm_query_attn_window(q, k, v, out, lay, heads, win, workspace=ws_w, stream=stream), 10)
            result["streaming"] = {"ms_prefill_one_appended_block_per_sequence": round(ms_blk, 4),
                                   "ms_query_attn_window_quarter": round(ms_win, 4), "window_blocks": win}
        if not args.no_extras:
            # three-axis RoPE on the same tensors (ids of a video prompt with 16x16 / 14x14 tokens per frame)
            ft, gw = (196, 14) if w.seqs[0][1] % 196 == 0 else (256, 16)
            ids = torch.from_numpy(W.mrope_position_ids(w, ft, gw)).to(dev)
            half = w.head_dim // 2
            sec = (half // 4, (half - half // 4) // 2, half - half // 4 - (half - half // 4) // 2)
            ms_mr = timed(lambda: P.pevlm_rope_mrope(qs, ks, T, heads, w.rope_base, ids, sec, stream=stream), 10)
            result["ms_rope_mrope"] = round(ms_mr, 4)
            result["rope_mrope_gbs"] = round((rope_bytes + 12 * T) / (ms_mr * 1e-3) / 1e9, 1)

    if not args.no_full_causal:
        wf = W.CONFIGS["c3_full_causal"] if args.workload == "c3" else W.small_variant(
            w, w.name + "_full_causal", [(0, s + c + qq, s + c + qq, 0) for (s, b, c, qq) in w.seqs])
        layf = P.Layout.from_seqs(wf.seqs)
        ws_f = torch.empty(P.pevlm_block_prefill_workspace_bytes(layf, heads), dtype=torch.uint8, device=dev)
        outf = torch.empty_like(q)
        P.pevlm_block_prefill_attn(q, k, v, outf, layf, heads, workspace=ws_f, stream=stream)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = 3
        e0.record(stream)
        for _ in range(reps):
            P.pevlm_block_prefill_attn(q, k, v, outf, layf, heads, workspace=ws_f, stream=stream)
        e1.record(stream)
        torch.cuda.synchronize()
        ms_full = e0.elapsed_time(e1) / reps
        ff, _ = P.useful_flops(layf, heads)
        result["ms_full_causal"] = round(ms_full, 3)
        result["full_causal_useful_tflops"] = round(ff / (ms_full * 1e-3) / 1e12, 2)
        result["attn_speedup_vs_full_causal"] = round(ms_full / (ms_prefill + ms_query), 2)
        del outf

    if not args.no_cpu_baseline:
        import oracle
        oracle.build()
        a = w.layout_arrays()
        olay = oracle.Layout(a["cu_seqlens"], a["sink_len"], a["block_len"], a["ctx_len"], a["query_len"])
        rows = W.sample_rows(w, n_random=8192)
        pairs = int(sum(int(oracle.mask_row(olay, int(t)).sum()) for t in rows))
        tc0 = time.perf_counter()
        want, _ = oracle.forward(data["q"], data["k"], data["v"], olay, w.rope_base, rows=rows)
        tc1 = time.perf_counter()
        cpu_flops = 4 * w.head_dim * w.n_q_heads * pairs
        got = first_out[torch.from_numpy(rows).to(dev)].float().cpu().numpy()
        err = np.abs(got - want)
        result["cpu_baseline"] = {
            "value": round(cpu_flops / (tc1 - tc0) / 1e12, 6),
            "unit": "TFLOP/s",
            "cores": oracle.threads(),
            "kind": "oracle",
            "sample": f"{len(rows)} of {T} rows of {w.name} (region/block/tile edges, all question rows, 8192 seeded "
                      f"random rows) x all heads, {pairs} visible pairs/head, {tc1 - tc0:.1f} s incl. fp64 RoPE of all keys",
        }
        result["max_abs_err_vs_oracle"] = float(err.max())
        result["mean_abs_err_vs_oracle"] = float(err.mean())

    print(json.dumps(result))


if __name__ == "__main__":
    main()
