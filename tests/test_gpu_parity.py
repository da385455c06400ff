"""Parity of the HIP path with the CPU oracle, element by element on the same seeded inputs.
Every call goes through the C ABI of libpevlm.so (via the thin ctypes binding).

Tolerances (from the benchmark spec): bf16 storage with fp32 accumulation -> max-abs <= 2e-2 and
mean-abs <= 2e-3; fp32 path -> 1e-5.  Sharper self-imposed checks ride along (relative L2 error per
row, exact leak tests, bitwise run-to-run reproducibility)."""
import ctypes

import numpy as np
import pytest
import torch

import paper_2506_19651_amd as P
import workloads as W
from gpu_util import DEV, error_stats, layout_heads, oracle_layout, run_path, to_device, to_host_f32

pytestmark = pytest.mark.gpu

BF16_MAX, BF16_MEAN, BF16_REL = 2e-2, 2e-3, 3e-2
F32_TOL = 1e-5


@pytest.fixture(params=["auto", "stream"])
def prefill_kernel(request):
    """Runs a test under the library's own choice of block-prefill kernel and with the streaming kernel
    forced (small layouts would otherwise never reach it)."""
    prev = P.pevlm_set_prefill_kernel(request.param)
    yield request.param
    P.pevlm_set_prefill_kernel(prev)


def oracle_rows(oracle, w, data, rows, **kw):
    return oracle.forward(data["q"], data["k"], data["v"], oracle_layout(oracle, w), w.rope_base, rows=rows, **kw)


def check_bf16(got, want, tag):
    st = error_stats(got, want)
    print(f"[{tag}] rows={got.shape[0]} max_abs={st['max_abs']:.3e} mean_abs={st['mean_abs']:.3e} "
          f"max_rel_l2={st['max_rel_l2']:.3e}", flush=True)
    assert np.isfinite(got).all()
    assert st["max_abs"] <= BF16_MAX and st["mean_abs"] <= BF16_MEAN and st["max_rel_l2"] <= BF16_REL, st


# ------------------------------------------------------------------------------------ fp32 path
def test_c1_fp32_all_rows(oracle):
    w = W.CONFIGS["c1"]
    data = W.generate(w)
    r = run_path(w, data, want_lse=True)
    want, want_lse = oracle_rows(oracle, w, data, None)
    got = to_host_f32(r["out"])
    assert np.isfinite(got).all()
    assert np.max(np.abs(got - want)) <= F32_TOL
    assert np.max(np.abs(to_host_f32(r["lse"]) - want_lse)) <= 1e-4
    # rotated q/k against the oracle's fp64 rotation
    olay = oracle_layout(oracle, w)
    pos = oracle.positions(olay)
    assert np.max(np.abs(to_host_f32(r["q_rot"]) - oracle.rope(data["q"], pos, w.rope_base))) <= 2e-6
    assert np.max(np.abs(to_host_f32(r["k_rot"]) - oracle.rope(data["k"], pos, w.rope_base))) <= 2e-6
    # the prefill call left the question rows alone, the question call left the others alone
    ap = to_host_f32(r["after_prefill"])
    S, B, C, Q = w.seqs[0]
    assert np.isnan(ap[S + C:]).all() and np.array_equal(ap[:S + C], got[:S + C])


F32_CASES = [
    ("ragged_batch", 4, 2, 64, [(5, 7, 31, 3), (0, 16, 50, 9), (12, 9, 0, 5), (3, 4, 10, 0)], None, 0),
    ("d128_splits3", 4, 1, 128, [(40, 33, 150, 21)], None, 3),
    ("head_map", 4, 2, 64, [(9, 8, 40, 6)], [1, 0, 1, 0], 2),
    ("no_sink_one_block", 2, 2, 64, [(0, 90, 90, 0)], None, 0),
    ("question_only", 2, 1, 64, [(0, 1, 0, 70)], None, 5),
]


@pytest.mark.parametrize("name,Hq,Hkv,D,seqs,hmap,splits", F32_CASES, ids=[c[0] for c in F32_CASES])
def test_fp32_layouts(oracle, name, Hq, Hkv, D, seqs, hmap, splits):
    w = W.Workload(name, 11, "f32", Hq, Hkv, D, 1.0e4, seqs, 1.0)
    data = W.generate(w)
    offs = [100 * i + 7 for i in range(len(seqs))]
    r = run_path(w, data, num_splits=splits, pos_offset=offs, kv_head_of_q=hmap, want_lse=True)
    want, want_lse = oracle_rows(oracle, w, data, None, kv_head_of_q=hmap, pos_offset=offs)
    got = to_host_f32(r["out"])
    assert np.isfinite(got).all()
    assert np.max(np.abs(got - want)) <= F32_TOL
    assert np.max(np.abs(to_host_f32(r["lse"]) - want_lse)) <= 1e-4


# ------------------------------------------------------------------------------------ bf16 path
BF16_SMALL = [
    # several 128-row tiles, ragged tails, sink not a multiple of the key tile, partial last block
    ("tiles_ragged", 8, 2, 128, [(300, 392, 1000, 70)], 0),
    ("aligned", 4, 4, 128, [(256, 512, 1024, 64)], 4),
    ("batch_mixed", 4, 2, 128, [(130, 200, 777, 129), (0, 64, 320, 5), (17, 1000, 250, 0), (5, 3, 0, 200)], 3),
    ("d64", 4, 1, 64, [(100, 160, 500, 33)], 2),
    ("tiny_everything", 2, 1, 128, [(1, 1, 3, 1), (0, 1, 0, 1), (2, 5, 5, 0)], 1),
    ("one_block_full_causal", 2, 1, 128, [(0, 700, 700, 0)], 0),
]


@pytest.mark.parametrize("name,Hq,Hkv,D,seqs,splits", BF16_SMALL, ids=[c[0] for c in BF16_SMALL])
def test_bf16_small_all_rows(oracle, name, Hq, Hkv, D, seqs, splits, prefill_kernel):
    w = W.Workload(name, 12, "bf16", Hq, Hkv, D, 1.0e6, seqs, 0.5, key_offset_scale=0.3)
    data = W.generate(w)
    r = run_path(w, data, num_splits=splits, want_lse=True)
    want, want_lse = oracle_rows(oracle, w, data, None)
    got = to_host_f32(r["out"])
    check_bf16(got, want, name)
    assert np.max(np.abs(to_host_f32(r["lse"]) - want_lse)) <= 2e-2
    # sequential RoPE alone: one rounding to bf16 of the exact rotation
    olay = oracle_layout(oracle, w)
    pos = oracle.positions(olay)
    for key in ("q", "k"):
        exact = oracle.rope(data[key], pos, w.rope_base)
        err = np.abs(to_host_f32(r[key + "_rot"]) - exact)
        assert np.all(err <= np.abs(exact) * 2.0 ** -8 + 1e-6)
    # attention alone ("stage" check): oracle attention fed with the GPU's own rotated bf16 q/k
    q_rot, k_rot = to_host_f32(r["q_rot"]).astype(np.float64), to_host_f32(r["k_rot"]).astype(np.float64)
    stage, _ = oracle.attn(q_rot, k_rot, data["v"], olay)
    check_bf16(got, stage, name + "/attention-only")


HARD = [
    # nearly one-hot softmax (scaled scores of ~10 in base-2 units)
    ("peaky", dict(qk_scale=2.5), [(200, 300, 900, 40)], 0),
    # the row maximum keeps rising tile after tile: the reference maximum must follow
    ("rising_max", dict(qk_scale=1.5, key_ramp=6.0), [(128, 640, 1280, 64)], 3),
    # weights overflow bf16/fp32 range against a stale reference inside one tile
    ("huge_scores", dict(qk_scale=6.0, key_ramp=3.0), [(64, 256, 512, 32)], 2),
]


@pytest.mark.parametrize("name,extra,seqs,splits", HARD, ids=[c[0] for c in HARD])
def test_bf16_hard_softmax_cases(oracle, name, extra, seqs, splits, prefill_kernel):
    """Inputs that drive the rare paths of the online softmax (reference maximum raised after the
    fact, overflow of the first-pass weights).  Compared with the oracle fed with the GPU's own
    rotated bf16 Q/K, so that only the attention arithmetic is under test."""
    w = W.Workload(name, 15, "bf16", 4, 2, 128, 1.0e6, seqs, 0.5, **extra)
    data = W.generate(w)
    r = run_path(w, data, num_splits=splits, want_lse=True)
    olay = oracle_layout(oracle, w)
    q_rot, k_rot = to_host_f32(r["q_rot"]).astype(np.float64), to_host_f32(r["k_rot"]).astype(np.float64)
    want, want_lse = oracle.attn(q_rot, k_rot, data["v"], olay)
    got = to_host_f32(r["out"])
    st = error_stats(got, want)
    print(f"[{name}] max_abs={st['max_abs']:.3e} mean_abs={st['mean_abs']:.3e} lse_err={np.max(np.abs(to_host_f32(r['lse']) - want_lse)):.3e}", flush=True)
    assert np.isfinite(got).all()
    assert st["max_abs"] <= BF16_MAX and st["mean_abs"] <= BF16_MEAN, st
    lse_err = np.abs(to_host_f32(r["lse"]) - want_lse)
    assert np.all(lse_err <= 2e-2 + 1e-4 * np.abs(want_lse))


TAILS = [(128, 1), (128, 31), (128, 32), (128, 33), (128, 63), (64, 8), (64, 40)]


@pytest.mark.parametrize("D,tail", TAILS, ids=[f"D{d}_tail{t}" for d, t in TAILS])
def test_bf16_sink_that_does_not_fill_a_key_tile(oracle, D, tail, prefill_kernel):
    """Sinks of 64 n + tail keys (the last key tile of the sink is ragged, the block's own keys start in
    a fresh tile): blocks shorter and longer than a tile, a sink smaller than a tile, several
    sequences.  Oracle fed with the GPU's rotated bf16 Q/K; exactness of the mask is covered by the
    zero-weight test below."""
    seqs = [(64 + tail, 150, 700, 20), (tail, 40, 130, 0), (128 + tail, 64 - tail, 300, 7)]
    w = W.Workload(f"tail{tail}", 40 + tail, "bf16", 4, 2, D, 1.0e6, seqs, 0.5)
    data = W.generate(w)
    r = run_path(w, data, num_splits=2, want_lse=True)
    olay = oracle_layout(oracle, w)
    q_rot, k_rot = to_host_f32(r["q_rot"]).astype(np.float64), to_host_f32(r["k_rot"]).astype(np.float64)
    want, want_lse = oracle.attn(q_rot, k_rot, data["v"], olay)
    got = to_host_f32(r["out"])
    st = error_stats(got, want)
    print(f"[tail {tail} D {D}] max_abs={st['max_abs']:.3e} mean_abs={st['mean_abs']:.3e}", flush=True)
    assert np.isfinite(got).all()
    assert st["max_abs"] <= BF16_MAX and st["mean_abs"] <= BF16_MEAN, st
    lse_err = np.abs(to_host_f32(r["lse"]) - want_lse)
    assert np.all(lse_err <= 2e-2 + 1e-4 * np.abs(want_lse))


def prefill_list_on_device(ws, lay, heads):
    """True if the work list the block-prefill call left in its workspace equals the host enumeration
    (stream items for the streaming bf16 kernel, plain work items otherwise)."""
    if P.pevlm_prefill_uses_stream_kernel(lay, heads):
        host = P.pevlm_prefill_stream_items_host(lay, heads)
        size = ctypes.sizeof(P.StreamItem)
        host_bytes = b"".join(bytes(it) for it in host)
    else:
        host = P.pevlm_prefill_worklist_host(lay, P.pevlm_prefill_tile_rows(heads))
        size = ctypes.sizeof(P.WorkItem)
        host_bytes = b"".join(bytes(it) for it in host)
    assert len(host) > 0
    return ws.cpu().numpy()[: len(host) * size].tobytes() == host_bytes


def test_bf16_gpu_worklist_equals_host_enumeration(prefill_kernel):
    seqs = [(130, 200, 777, 129), (0, 64, 320, 5), (17, 1000, 250, 0), (5, 3, 0, 200)]
    w = W.Workload("wl", 13, "bf16", 4, 2, 128, 1.0e6, seqs, 0.5)
    data = W.generate(w)
    lay, heads = layout_heads(w)
    q, k, v = to_device(data["q"]), to_device(data["k"]), to_device(data["v"])
    out = torch.zeros_like(q)
    ws = P.pevlm_block_prefill_attn(q, k, v, out, lay, heads)
    torch.cuda.synchronize()
    assert prefill_list_on_device(ws, lay, heads)
    ws = P.pevlm_query_attn(q, k, v, out, lay, heads, num_splits=5)
    torch.cuda.synchronize()
    host = P.pevlm_query_worklist_host(lay, P.pevlm_query_tile_rows(heads), 5)
    n = len(host)
    dev_items = ws.cpu().numpy()[: n * 32].view(np.int32).reshape(n, 8)
    host_items = np.array([[getattr(it, f) for f, _ in P.WorkItem._fields_] for it in host], np.int32)
    assert np.array_equal(dev_items, host_items)


def test_bf16_no_cross_block_leak_and_reproducible(prefill_kernel):
    """Exact checks: perturbing another block's K/V leaves a block's rows bit-identical; two runs
    give bit-identical outputs; keys a row must not see have exactly zero weight (V = 0 on visible
    keys, 1 elsewhere -> output exactly 0)."""
    S, B, C, Q = 200, 300, 1200, 40
    w = W.Workload("leak", 14, "bf16", 4, 2, 128, 1.0e6, [(S, B, C, Q)], 0.5)
    data = W.generate(w)
    a = run_path(w, data)["out"].view(torch.int16).cpu().numpy()
    b = run_path(w, data)["out"].view(torch.int16).cpu().numpy()
    assert np.array_equal(a, b)
    d2 = {k_: v_.copy() for k_, v_ in data.items()}
    big = W.f32_to_bf16_bits(np.full((B, 2, 128), 3.0, np.float32))
    d2["k"][S + B:S + 2 * B] = big
    d2["v"][S + B:S + 2 * B] = big
    c = run_path(w, d2)["out"].view(torch.int16).cpu().numpy()
    keep = np.r_[0:S + B, S + 2 * B:S + C]
    assert np.array_equal(c[keep], a[keep])
    assert not np.array_equal(c[S + B:S + 2 * B], a[S + B:S + 2 * B])
    assert not np.array_equal(c[S + C:], a[S + C:])
    # zero-weight test for the rows of one block: V = 1 on every key the block must not see
    d3 = {k_: v_.copy() for k_, v_ in data.items()}
    one = W.f32_to_bf16_bits(np.ones((1,), np.float32))[0]
    d3["v"][:] = one
    d3["v"][:S] = 0
    d3["v"][S + 2 * B:S + 3 * B] = 0
    o = to_host_f32(run_path(w, d3)["out"])
    assert np.all(o[S + 2 * B:S + 3 * B] == 0.0)
    assert np.all(o[:S] == 0.0)
    later = o[S + 3 * B:S + C]  # later blocks: sink has V=0, own block V=1 -> strictly inside (0, 1]
    assert np.all((later > 0.0) & (later <= 1.0))


FULL = [("c2", 512), ("c3", 384), ("c4a", 256), ("c4b", 128), ("c4c", 128), ("c4d", 256), ("c5a", 128), ("c5b", 256)]


@pytest.mark.parametrize("name,n_random", FULL, ids=[c[0] for c in FULL])
def test_bf16_full_size_sampled_rows(oracle, name, n_random):
    """The benchmark's own configurations at full size, in the launch configuration bench.py times;
    the oracle evaluates a deterministic row sample (region edges, block boundaries, tile edges,
    question rows, seeded random rows)."""
    w = W.CONFIGS[name]
    data = W.generate(w)
    r = run_path(w, data, poison=True)
    rows = W.sample_rows(w, n_random=n_random, max_question_rows=48)
    want, _ = oracle_rows(oracle, w, data, rows)
    out = r["out"]
    got = to_host_f32(out[torch.from_numpy(rows).to(DEV)])
    check_bf16(got, want, name)
    # properties that hold at any size: every row written, finite, inside the hull of V
    assert torch.isfinite(out.float()).all()
    vmax = float(to_host_f32(r["v"].float().abs().max()))
    assert float(out.float().abs().max()) <= vmax * 1.01


def test_bf16_full_causal_c3_sampled_rows(oracle):
    """The dense causal layout bench.py times as the comparison (one 65 920-row block, no sink, up to
    1030 key tiles per work item): first and last rows, both sides of 128-row tile edges spread over
    the sequence, and seeded random rows against the oracle."""
    w = W.CONFIGS["c3_full_causal"]
    data = W.generate(w)
    lay, heads = layout_heads(w)
    q, k, v = to_device(data["q"]), to_device(data["k"]), to_device(data["v"])
    out = torch.full_like(q, float("nan"))
    P.pevlm_rope_seq(q, k, lay, heads, w.rope_base)
    P.pevlm_block_prefill_attn(q, k, v, out, lay, heads)
    torch.cuda.synchronize()
    T = w.total_tokens
    edges = [128 * e for e in (1, 2, 3, 17, 100, 255, 256, 400, 511, 514)]
    rows = [0, 1, 2, 63, 64, T - 2, T - 1] + [e - 1 for e in edges] + edges
    rows += [int(x) for x in np.random.default_rng(3).integers(0, T, 130)]
    rows = np.unique(np.asarray(rows, dtype=np.int64))
    want, _ = oracle_rows(oracle, w, data, rows)
    check_bf16(to_host_f32(out[torch.from_numpy(rows).to(DEV)]), want, "c3_full_causal")
    assert torch.isfinite(out.float()).all()


SCALE_CASES = [
    ("f32_d64", "f32", 4, 2, 64, [(12, 9, 50, 5), (3, 16, 64, 7)], 0.05, 3),
    ("f32_d128", "f32", 2, 1, 128, [(40, 33, 150, 21)], 0.2, 2),
    ("bf16_d128", "bf16", 8, 2, 128, [(300, 392, 1000, 70)], 0.05, 4),
    ("bf16_d128_sharp", "bf16", 4, 2, 128, [(130, 200, 777, 129), (0, 64, 320, 5)], 0.2, 0),
    ("bf16_d64", "bf16", 4, 1, 64, [(100, 160, 500, 33)], 0.2, 3),
]


@pytest.mark.parametrize("name,dtype,Hq,Hkv,D,seqs,scale,splits", SCALE_CASES, ids=[c[0] for c in SCALE_CASES])
def test_caller_chosen_softmax_scale(oracle, name, dtype, Hq, Hkv, D, seqs, scale, splits, prefill_kernel):
    """Eq. 1 with the caller's factor in place of 1/sqrt(d): all three calls (and the pair with RoPE
    folded in), out and lse, against the oracle evaluated with the same factor; and the result
    differs from the default-scale one (the factor really is used)."""
    w = W.Workload("scale_" + name, 21, dtype, Hq, Hkv, D, 1.0e6, seqs, 0.5 if dtype == "bf16" else 1.0)
    data = W.generate(w)
    r = run_path(w, data, num_splits=splits, want_lse=True, softmax_scale=scale)
    want, want_lse = oracle_rows(oracle, w, data, None, softmax_scale=scale)
    got, got_lse = to_host_f32(r["out"]), to_host_f32(r["lse"])
    if dtype == "f32":
        assert np.isfinite(got).all() and np.max(np.abs(got - want)) <= F32_TOL
        assert np.max(np.abs(got_lse - want_lse)) <= 1e-4
    else:
        check_bf16(got, want, name)
        assert np.max(np.abs(got_lse - want_lse)) <= 2e-2
        lay, heads = layout_heads(w, None, scale)
        q, k, v = to_device(data["q"]), to_device(data["k"]), to_device(data["v"])
        out = torch.full_like(q, float("nan"))
        P.pevlm_block_prefill_attn_rope(q, k, v, out, lay, heads, w.rope_base)
        P.pevlm_query_attn_rope(q, k, v, out, lay, heads, w.rope_base, num_splits=splits)
        torch.cuda.synchronize()
        assert torch.equal(out.view(torch.int16), r["out"].view(torch.int16))
    default, _ = oracle_rows(oracle, w, data, None)
    assert np.max(np.abs(default - want)) > 10 * (F32_TOL if dtype == "f32" else 1e-3)
    # the default written out explicitly gives the default result
    r2 = run_path(w, data, num_splits=splits, softmax_scale=float(1.0 / np.sqrt(D)))
    r3 = run_path(w, data, num_splits=splits)
    assert np.max(np.abs(to_host_f32(r2["out"]) - to_host_f32(r3["out"]))) <= (1e-6 if dtype == "f32" else 2.0 ** -8)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_rotated_tensors_under_position_offsets(oracle, dtype):
    """pevlm_rope_seq with per-sequence starting positions: rotated Q and K element by element
    against the oracle's rotation at positions o_s + n (fp32: 2e-6; bf16: one rounding)."""
    seqs = [(130, 200, 777, 129), (0, 64, 320, 5), (17, 100, 250, 0)]
    offs = [37, 100000, 4096]
    w = W.Workload("offs_" + dtype, 22, dtype, 4, 2, 128, 1.0e6, seqs, 0.5 if dtype == "bf16" else 1.0)
    data = W.generate(w)
    r = run_path(w, data, pos_offset=offs)
    pos = oracle.positions(oracle_layout(oracle, w), offs)
    for key in ("q", "k"):
        exact = oracle.rope(data[key], pos, w.rope_base)
        err = np.abs(to_host_f32(r[key + "_rot"]) - exact)
        if dtype == "bf16":
            assert np.all(err <= np.abs(exact) * 2.0 ** -8 + 1e-6)
        else:
            assert err.max() <= 5e-6
    # and the rotation without offsets is a different tensor (the offsets are really used)
    r0 = run_path(w, data)
    assert not torch.equal(r0["k_rot"], r["k_rot"])


def test_roofline_probes_run_and_copy_is_exact():
    """The measurement-only entry points: the copy moves every byte, the MFMA loop reports its
    operation count, bad arguments are rejected before any launch."""
    n = (1 << 20) + 4096
    src = torch.randint(0, 255, (n,), dtype=torch.uint8, device=DEV)
    dst = torch.zeros_like(src)
    P.pevlm_probe_copy(dst, src, n)
    torch.cuda.synchronize()
    assert torch.equal(dst, src)
    scratch = torch.zeros(16, dtype=torch.float32, device=DEV)
    flops = P.pevlm_probe_mfma_bf16(scratch, 8, 10)
    torch.cuda.synchronize()
    assert flops == 8 * 4 * 10 * 4 * 32768 and float(scratch.abs().sum()) == 0.0
    with pytest.raises(P.PevlmError):
        P.pevlm_probe_copy(dst, src, 24)
    with pytest.raises(P.PevlmError):
        P.pevlm_probe_mfma_bf16(scratch, 0, 10)
    # the tile-loop probe: reads only inside the buffer it is given (guard bands around it stay intact and
    # the buffer itself is never written), reports its operation count, rejects a buffer below four tiles
    tiles = 5
    buf = torch.full((4096 + tiles * 16384 + 4096,), 0x3C, dtype=torch.uint8, device=DEV)
    kv = buf[4096: 4096 + tiles * 16384].view(torch.bfloat16)
    before = buf.clone()
    for soft in (True, False):
        flops = P.pevlm_probe_tile_loop_bf16(scratch, kv, 16, 7, soft)
        torch.cuda.synchronize()
        assert flops == 16 * 4 * 7 * 32 * 32768
    assert torch.equal(buf, before) and float(scratch.abs().sum()) == 0.0
    with pytest.raises(P.PevlmError):
        P.pevlm_probe_tile_loop_bf16(scratch, kv[: 3 * 8192], 16, 7, True)


# ------------------------------------------------------------------------------------ multimodal RoPE
MROPE_CASES = [
    # name, dtype, Hq, Hkv, D, seqs, frame_tokens, grid_w, section
    ("f32_d64", "f32", 4, 2, 64, [(40, 32, 96, 9), (3, 16, 40, 5)], 16, 4, (8, 12, 12)),
    ("bf16_d128_qwen_split", "bf16", 8, 2, 128, [(300, 512, 1536, 70)], 256, 16, (16, 24, 24)),
    ("bf16_d128_ragged_sections", "bf16", 4, 1, 128, [(100, 196, 700, 33)], 196, 14, (5, 20, 39)),
    ("bf16_d64_one_axis_empty", "bf16", 4, 4, 64, [(64, 64, 320, 8)], 64, 8, (12, 20, 0)),
]


@pytest.mark.parametrize("name,dtype,Hq,Hkv,D,seqs,ft,gw,section", MROPE_CASES, ids=[c[0] for c in MROPE_CASES])
def test_mrope_against_oracle(oracle, name, dtype, Hq, Hkv, D, seqs, ft, gw, section):
    """pevlm_rope_mrope element by element against the oracle's three-axis rotation, and the whole
    path (three-axis RoPE -> block prefill -> question attention) against the oracle's attention
    over its own rotated tensors."""
    w = W.Workload(name, 13, dtype, Hq, Hkv, D, 1.0e6, seqs, 0.5 if dtype == "bf16" else 1.0)
    data = W.generate(w)
    ids = W.mrope_position_ids(w, ft, gw)
    lay, heads = layout_heads(w)
    q, k, v = to_device(data["q"]), to_device(data["k"]), to_device(data["v"])
    ids_d = torch.from_numpy(ids).to(DEV)
    P.pevlm_rope_mrope(q, k, w.total_tokens, heads, w.rope_base, ids_d, section)
    out = torch.full_like(q, float("nan"))
    P.pevlm_block_prefill_attn(q, k, v, out, lay, heads)
    P.pevlm_query_attn(q, k, v, out, lay, heads)
    torch.cuda.synchronize()
    q_exact = oracle.rope_mrope(data["q"], ids, section, w.rope_base)
    k_exact = oracle.rope_mrope(data["k"], ids, section, w.rope_base)
    for got, exact in ((to_host_f32(q), q_exact), (to_host_f32(k), k_exact)):
        err = np.abs(got - exact)
        if dtype == "bf16":
            assert np.all(err <= np.abs(exact) * 2.0 ** -8 + 1e-6)  # one rounding of the exact rotation
        else:
            assert err.max() <= 2e-6
    want, _ = oracle.attn(q_exact, k_exact, data["v"], oracle_layout(oracle, w))
    got = to_host_f32(out)
    if dtype == "bf16":
        check_bf16(got, want, name)
    else:
        assert np.max(np.abs(got - want)) <= F32_TOL


def test_mrope_with_equal_axes_is_sequential_rope_bitwise():
    w = W.small_variant(W.CONFIGS["c2"], "mrope_eq", [(256, 512, 1024, 64), (0, 128, 300, 7)])
    data = W.generate(w)
    lay, heads = layout_heads(w)
    q1, k1 = to_device(data["q"]), to_device(data["k"])
    q2, k2 = q1.clone(), k1.clone()
    offs = [11, 4000]
    P.pevlm_rope_seq(q1, k1, lay, heads, w.rope_base, offs)
    pos = np.concatenate([np.arange(S + C + Q, dtype=np.int32) + o for (S, _b, C, Q), o in zip(w.seqs, offs)])
    ids = torch.from_numpy(np.stack([pos, pos, pos])).to(DEV)
    P.pevlm_rope_mrope(q2, k2, w.total_tokens, heads, w.rope_base, ids, (16, 24, 24))
    torch.cuda.synchronize()
    assert torch.equal(q1.view(torch.int16), q2.view(torch.int16)) and torch.equal(k1.view(torch.int16), k2.view(torch.int16))


def test_mrope_full_size_c3_sampled_rows(oracle):
    """The 64K-token workload with the ids of a 16x16-token-per-frame video prompt."""
    w = W.CONFIGS["c3"]
    data = W.generate(w)
    ids = W.mrope_position_ids(w, 256, 16)
    _lay, heads = layout_heads(w)
    q, k = to_device(data["q"]), to_device(data["k"])
    P.pevlm_rope_mrope(q, k, w.total_tokens, heads, w.rope_base, torch.from_numpy(ids).to(DEV), (16, 24, 24))
    torch.cuda.synchronize()
    rows = W.sample_rows(w, n_random=256, max_question_rows=16)
    idx = torch.from_numpy(rows).to(DEV)
    for t, key in ((q, "q"), (k, "k")):
        exact = oracle.rope_mrope(data[key], ids, (16, 24, 24), w.rope_base, rows=rows)
        err = np.abs(to_host_f32(t[idx]) - exact)
        assert np.all(err <= np.abs(exact) * 2.0 ** -8 + 1e-6)


# ------------------------------------------------------------------------------------ fused query rotation
FUSED_CASES = [
    ("tiles_ragged", 8, 2, 128, [(300, 392, 1000, 70)], 0, None),
    ("batch_mixed_offsets", 4, 2, 128, [(130, 200, 777, 129), (0, 64, 320, 5), (17, 1000, 250, 0), (5, 3, 0, 200)], 3,
     [7, 0, 100000, 31]),
    ("d64", 4, 1, 64, [(100, 160, 500, 33)], 2, None),
]


@pytest.mark.parametrize("name,Hq,Hkv,D,seqs,splits,offs", FUSED_CASES, ids=[c[0] for c in FUSED_CASES])
def test_fused_query_rotation_equals_unfused_bitwise_and_oracle(oracle, name, Hq, Hkv, D, seqs, splits, offs):
    """pevlm_*_attn_rope on un-rotated q (+ K rotated alone) must reproduce the three-call path bit for
    bit, and therefore the oracle within the bf16 tolerances; q itself stays untouched."""
    w = W.Workload(name, 14, "bf16", Hq, Hkv, D, 1.0e6, seqs, 0.5, key_offset_scale=0.3)
    data = W.generate(w)
    ref = run_path(w, data, num_splits=splits, pos_offset=offs, want_lse=True)
    lay, heads = layout_heads(w)
    q, k, v = to_device(data["q"]), to_device(data["k"]), to_device(data["v"])
    q_before = q.clone()
    out = torch.full_like(q, float("nan"))
    lse = torch.full((w.total_tokens, Hq), float("nan"), device=DEV)
    # keys rotated in place by the prefill call itself
    P.pevlm_block_prefill_attn_rope(q, k, v, out, lay, heads, w.rope_base, offs, lse=lse)
    P.pevlm_query_attn_rope(q, k, v, out, lay, heads, w.rope_base, offs, num_splits=splits, lse=lse)
    torch.cuda.synchronize()
    assert torch.equal(q, q_before)
    assert torch.equal(k.view(torch.int16), ref["k_rot"].view(torch.int16))
    assert torch.equal(out.view(torch.int16), ref["out"].view(torch.int16))
    assert torch.equal(lse.view(torch.int32), ref["lse"].view(torch.int32))
    # keys rotated beforehand by pevlm_rope_seq
    k2 = to_device(data["k"])
    out2 = torch.full_like(q, float("nan"))
    P.pevlm_rope_seq(None, k2, lay, heads, w.rope_base, offs)
    P.pevlm_block_prefill_attn_rope(q, k2, v, out2, lay, heads, w.rope_base, offs, k_is_rotated=True)
    P.pevlm_query_attn_rope(q, k2, v, out2, lay, heads, w.rope_base, offs, num_splits=splits)
    torch.cuda.synchronize()
    assert torch.equal(k2.view(torch.int16), ref["k_rot"].view(torch.int16))
    assert torch.equal(out2.view(torch.int16), ref["out"].view(torch.int16))
    want, _ = oracle_rows(oracle, w, data, None, pos_offset=offs)
    check_bf16(to_host_f32(out), want, name + "/fused")


def test_fused_query_rotation_full_size_c3(oracle):
    w = W.CONFIGS["c3"]
    data = W.generate(w)
    ref = run_path(w, data, poison=True)
    lay, heads = layout_heads(w)
    q, k, v = to_device(data["q"]), to_device(data["k"]), to_device(data["v"])
    out = torch.full_like(q, float("nan"))
    P.pevlm_block_prefill_attn_rope(q, k, v, out, lay, heads, w.rope_base)
    P.pevlm_query_attn_rope(q, k, v, out, lay, heads, w.rope_base)
    torch.cuda.synchronize()
    assert torch.equal(out.view(torch.int16), ref["out"].view(torch.int16))
    rows = W.sample_rows(w, n_random=128, max_question_rows=16)
    want, _ = oracle_rows(oracle, w, data, rows)
    check_bf16(to_host_f32(out[torch.from_numpy(rows).to(DEV)]), want, "c3/fused")


def test_fused_query_rotation_rejects_fp32():
    w = W.CONFIGS["c1"]
    data = W.generate(w)
    lay, heads = layout_heads(w)
    q, k, v = to_device(data["q"]), to_device(data["k"]), to_device(data["v"])
    out = torch.zeros_like(q)
    with pytest.raises(P.PevlmError):
        P.pevlm_block_prefill_attn_rope(q, k, v, out, lay, heads, w.rope_base)
    with pytest.raises(P.PevlmError):
        P.pevlm_query_attn_rope(q, k, v, out, lay, heads, w.rope_base)


def test_fused_prefill_with_no_prefill_rows_still_rotates_keys():
    w = W.small_variant(W.CONFIGS["c2"], "question_only_bf16", [(0, 1, 0, 70)])
    data = W.generate(w)
    ref = run_path(w, data)
    lay, heads = layout_heads(w)
    q, k, v = to_device(data["q"]), to_device(data["k"]), to_device(data["v"])
    out = torch.full_like(q, float("nan"))
    P.pevlm_block_prefill_attn_rope(q, k, v, out, lay, heads, w.rope_base)
    P.pevlm_query_attn_rope(q, k, v, out, lay, heads, w.rope_base)
    torch.cuda.synchronize()
    assert torch.equal(k.view(torch.int16), ref["k_rot"].view(torch.int16))
    assert torch.equal(out.view(torch.int16), ref["out"].view(torch.int16))


# ------------------------------------------------------------------------------------ many sequences
def _many_seqs(n, seed):
    rng = np.random.default_rng(seed)
    seqs = []
    for _ in range(n):
        S, B = int(rng.integers(0, 40)), int(rng.integers(1, 50))
        C = int(rng.integers(0, 120)) if rng.random() < 0.8 else 0
        Q = int(rng.integers(0, 20))
        if S + C + Q == 0:
            Q = 1
        seqs.append((S, B, C, Q))
    return seqs


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_batches_larger_than_one_sequence_table(oracle, dtype, prefill_kernel):
    """130 packed sequences: the host hands the sequence table to the kernels in pieces of 48, so
    work-list offsets, compact question rows and RoPE rows cross piece boundaries."""
    seqs = _many_seqs(130, 5)
    w = W.Workload("many_" + dtype, 15, dtype, 4, 2, 64 if dtype == "f32" else 128, 1.0e4, seqs, 1.0 if dtype == "f32" else 0.5)
    data = W.generate(w)
    offs = [int(x) for x in np.random.default_rng(6).integers(0, 5000, len(seqs))]
    r = run_path(w, data, num_splits=2, pos_offset=offs, want_lse=True)
    want, want_lse = oracle_rows(oracle, w, data, None, pos_offset=offs)
    got = to_host_f32(r["out"])
    if dtype == "f32":
        assert np.isfinite(got).all() and np.max(np.abs(got - want)) <= F32_TOL
        assert np.max(np.abs(to_host_f32(r["lse"]) - want_lse)) <= 1e-4
    else:
        check_bf16(got, want, "many_bf16")
        lay, heads = layout_heads(w)
        q, k, v = to_device(data["q"]), to_device(data["k"]), to_device(data["v"])
        out = torch.full_like(q, float("nan"))
        P.pevlm_block_prefill_attn_rope(q, k, v, out, lay, heads, w.rope_base, offs)
        P.pevlm_query_attn_rope(q, k, v, out, lay, heads, w.rope_base, offs, num_splits=2)
        torch.cuda.synchronize()
        assert torch.equal(out.view(torch.int16), r["out"].view(torch.int16))
    # device-built work lists equal the host enumeration across the pieces
    lay, heads = layout_heads(w)
    q, k, v = to_device(data["q"]), to_device(data["k"]), to_device(data["v"])
    out = torch.zeros_like(q)
    ws = P.pevlm_block_prefill_attn(q, k, v, out, lay, heads)
    torch.cuda.synchronize()
    assert prefill_list_on_device(ws, lay, heads)
    ws = P.pevlm_query_attn(q, k, v, out, lay, heads, num_splits=3)
    host = P.pevlm_query_worklist_host(lay, P.pevlm_query_tile_rows(heads), 3)
    torch.cuda.synchronize()
    n = len(host)
    assert n > 100
    dev_items = ws.cpu().numpy()[: n * 32].view(np.int32).reshape(n, 8)
    host_items = np.array([[getattr(it, f) for f, _ in P.WorkItem._fields_] for it in host], np.int32)
    assert np.array_equal(dev_items, host_items)


# ------------------------------------------------------------------------------------ seeded sweep
def _random_case(rng):
    D = int(rng.choice([64, 128]))
    Hkv = int(rng.choice([1, 2, 4]))
    G = int(rng.choice([1, 2, 4, 7]))
    n_seq = int(rng.integers(1, 4))
    seqs = []
    for _ in range(n_seq):
        S = int(rng.choice([0, 1, 31, 64, 65, 130, 200]))
        B = int(rng.choice([1, 7, 32, 64, 100, 128, 129, 300]))
        C = int(rng.choice([0, B, 2 * B, 2 * B + 1, 3 * B - 1, 333])) if rng.random() < 0.85 else 0
        C = min(C, 500)
        Q = int(rng.choice([0, 1, 5, 32, 33, 64, 65, 129, 140]))
        if S + C + Q == 0:
            S = 3
        seqs.append((S, B, C, Q))
    hmap = None
    if rng.random() < 0.25:
        hmap = [int(x) for x in rng.integers(0, Hkv, Hkv * G)]
    return D, Hkv, G, seqs, hmap, int(rng.integers(0, 6))


@pytest.mark.parametrize("dtype,seed", [("bf16", 101), ("bf16", 102), ("bf16", 103), ("f32", 104), ("bf16", 105), ("bf16", 106), ("f32", 107), ("bf16", 108)])
def test_seeded_sweep_of_small_layouts(oracle, dtype, seed, prefill_kernel):
    """Twelve random small layouts per seed (ragged tiles, 1-token blocks, missing regions, GQA widths
    1/2/4/7, explicit head maps, split counts 0-5) through all three calls, every row against the
    oracle; the bf16 cases also through the calls with RoPE folded in."""
    rng = np.random.default_rng(seed)
    for case in range(12):
        D, Hkv, G, seqs, hmap, splits = _random_case(rng)
        tag = f"{dtype}/{seed}/{case}: D={D} Hq={Hkv * G} Hkv={Hkv} seqs={seqs} map={hmap} splits={splits}"
        print(tag, flush=True)
        w = W.Workload(f"sweep{seed}_{case}", 16, dtype, Hkv * G, Hkv, D, 1.0e6, seqs, 0.5 if dtype == "bf16" else 1.0,
                       key_offset_scale=0.2)
        data = W.generate(w)
        r = run_path(w, data, num_splits=splits, kv_head_of_q=hmap, want_lse=True)
        want, want_lse = oracle_rows(oracle, w, data, None, kv_head_of_q=hmap)
        got = to_host_f32(r["out"])
        if dtype == "f32":
            assert np.isfinite(got).all() and np.max(np.abs(got - want)) <= F32_TOL, tag
            assert np.max(np.abs(to_host_f32(r["lse"]) - want_lse)) <= 1e-4, tag
            continue
        check_bf16(got, want, tag)
        assert np.max(np.abs(to_host_f32(r["lse"]) - want_lse)) <= 2e-2, tag
        lay, heads = layout_heads(w, hmap)
        q, k, v = to_device(data["q"]), to_device(data["k"]), to_device(data["v"])
        out = torch.full_like(q, float("nan"))
        P.pevlm_block_prefill_attn_rope(q, k, v, out, lay, heads, w.rope_base)
        P.pevlm_query_attn_rope(q, k, v, out, lay, heads, w.rope_base, num_splits=splits)
        torch.cuda.synchronize()
        assert torch.equal(out.view(torch.int16), r["out"].view(torch.int16)), tag


# ------------------------------------------------------------------------------------ streaming calls
STREAM_CASES = [
    ("bf16_ragged", "bf16", 8, 2, 128, [(300, 392, 1500, 70), (0, 128, 700, 40)]),
    ("bf16_d64_tiny_blocks", "bf16", 4, 1, 64, [(17, 5, 43, 9)]),
    ("f32", "f32", 4, 2, 64, [(12, 9, 50, 5), (3, 16, 64, 7)]),
]


@pytest.mark.parametrize("name,dtype,Hq,Hkv,D,seqs", STREAM_CASES, ids=[c[0] for c in STREAM_CASES])
def test_blocks_arriving_in_pieces_reproduce_the_one_shot_prefill(oracle, name, dtype, Hq, Hkv, D, seqs, prefill_kernel):
    """Sink + first blocks, then the remaining blocks two at a time: every call writes exactly its
    rows, the pieces add up to pevlm_block_prefill_attn bit for bit, and equal the oracle's rows."""
    w = W.Workload(name, 17, dtype, Hq, Hkv, D, 1.0e6, seqs, 0.5 if dtype == "bf16" else 1.0)
    data = W.generate(w)
    lay, heads = layout_heads(w)
    q, k, v = to_device(data["q"]), to_device(data["k"]), to_device(data["v"])
    P.pevlm_rope_seq(q, k, lay, heads, w.rope_base)
    ref = torch.full_like(q, float("nan"))
    P.pevlm_block_prefill_attn(q, k, v, ref, lay, heads)
    out = torch.full_like(q, float("nan"))
    nb = [(-(-C // B) if C else 0) for (S, B, C, Q) in seqs]
    done = [0] * len(seqs)
    first_call = True
    while first_call or any(d < n for d, n in zip(done, nb)):
        count = [min(2, n - d) for d, n in zip(done, nb)]
        before = out.clone()
        P.pevlm_block_prefill_attn_blocks(q, k, v, out, lay, heads, done, count, with_sink=first_call)
        torch.cuda.synchronize()
        t0 = 0
        for si, (S, B, C, Q) in enumerate(seqs):
            sel = torch.zeros(w.total_tokens, dtype=torch.bool, device=DEV)
            if first_call:
                sel[t0:t0 + S] = True
            sel[t0 + S + done[si] * B: min(t0 + S + C, t0 + S + (done[si] + count[si]) * B)] = True
            rows = slice(t0, t0 + S + C + Q)
            m = sel[rows]
            assert torch.equal(out[rows][m].view(torch.int32 if dtype == "f32" else torch.int16),
                               ref[rows][m].view(torch.int32 if dtype == "f32" else torch.int16))
            untouched = ~m
            assert torch.equal(torch.isnan(out[rows][untouched]), torch.isnan(before[rows][untouched]))
            t0 += S + C + Q
        done = [d + c for d, c in zip(done, count)]
        first_call = False
    both_nan = torch.isnan(out) & torch.isnan(ref)
    assert torch.equal(torch.nan_to_num(out), torch.nan_to_num(ref)) and torch.equal(torch.isnan(out), both_nan)
    # the rows written by the piecewise calls, directly against the oracle
    data_rows = np.concatenate([np.arange(c0, c0 + S + C) for c0, (S, B, C, Q) in zip(w.cu_seqlens, seqs)])
    want, _ = oracle_rows(oracle, w, data, data_rows)
    got = to_host_f32(out[torch.from_numpy(data_rows).to(DEV)])
    if dtype == "bf16":
        check_bf16(got, want, name + "/pieces")
    else:
        assert np.isfinite(got).all() and np.max(np.abs(got - want)) <= F32_TOL


WINDOW_CASES = [
    ("bf16_ragged", "bf16", 8, 2, 128, [(300, 392, 1500, 70), (0, 128, 700, 40)], [2, 0], 0),
    ("bf16_all_and_one", "bf16", 4, 4, 128, [(64, 256, 1024, 130), (200, 100, 950, 33)], [-1, 1], 5),
    ("bf16_d64", "bf16", 4, 1, 64, [(17, 5, 43, 9)], [3], 2),
    ("f32", "f32", 4, 2, 64, [(12, 9, 50, 5), (3, 16, 64, 7)], [1, 2], 3),
    ("f32_window_wider_than_context", "f32", 2, 1, 64, [(5, 8, 24, 6)], [7], 1),
]


@pytest.mark.parametrize("name,dtype,Hq,Hkv,D,seqs,windows,splits", WINDOW_CASES, ids=[c[0] for c in WINDOW_CASES])
def test_windowed_question_against_oracle(oracle, name, dtype, Hq, Hkv, D, seqs, windows, splits):
    w = W.Workload(name, 18, dtype, Hq, Hkv, D, 1.0e6, seqs, 0.5 if dtype == "bf16" else 1.0)
    data = W.generate(w)
    lay, heads = layout_heads(w)
    q, k, v = to_device(data["q"]), to_device(data["k"]), to_device(data["v"])
    out = torch.full_like(q, float("nan"))
    lse = torch.full((w.total_tokens, Hq), float("nan"), device=DEV)
    P.pevlm_rope_seq(q, k, lay, heads, w.rope_base)
    P.pevlm_query_attn_window(q, k, v, out, lay, heads, windows, num_splits=splits, lse=lse)
    torch.cuda.synchronize()
    a = w.layout_arrays()
    olay = oracle.Layout(a["cu_seqlens"], a["sink_len"], a["block_len"], a["ctx_len"], a["query_len"], window_blocks=windows)
    qrows = np.concatenate([np.arange(c0 + S + C, c0 + S + C + Q) for c0, (S, B, C, Q) in zip(a["cu_seqlens"], seqs)])
    want, want_lse = oracle.forward(data["q"], data["k"], data["v"], olay, w.rope_base, rows=qrows)
    idx = torch.from_numpy(qrows).to(DEV)
    got = to_host_f32(out[idx])
    if dtype == "bf16":
        check_bf16(got, want, name)
        assert np.max(np.abs(to_host_f32(lse[idx]) - want_lse)) <= 2e-2
    else:
        assert np.max(np.abs(got - want)) <= F32_TOL and np.max(np.abs(to_host_f32(lse[idx]) - want_lse)) <= 1e-4
    other = torch.ones(w.total_tokens, dtype=torch.bool, device=DEV)
    other[idx] = False
    assert torch.isnan(out[other]).all()  # only question rows are written


def test_windowed_question_full_size_c3(oracle):
    """64K-token workload, the question keeps the sink and the 16 newest of its 64 blocks."""
    w = W.CONFIGS["c3"]
    data = W.generate(w)
    lay, heads = layout_heads(w)
    q, k, v = to_device(data["q"]), to_device(data["k"]), to_device(data["v"])
    out = torch.full_like(q, float("nan"))
    P.pevlm_rope_seq(q, k, lay, heads, w.rope_base)
    P.pevlm_query_attn_window(q, k, v, out, lay, heads, [16])
    torch.cuda.synchronize()
    (S, B, C, Q), = w.seqs
    qrows = np.arange(S + C, S + C + Q, 5)
    a = w.layout_arrays()
    olay = oracle.Layout(a["cu_seqlens"], a["sink_len"], a["block_len"], a["ctx_len"], a["query_len"], window_blocks=[16])
    want, _ = oracle.forward(data["q"], data["k"], data["v"], olay, w.rope_base, rows=qrows)
    check_bf16(to_host_f32(out[torch.from_numpy(qrows).to(DEV)]), want, "c3/window16")


# ------------------------------------------------------------------------------------ time model
def test_time_model_against_fresh_measurements():
    """The block-prefill time model behind the sink / block-size chooser, against launches timed here.
    Boxes differ by several per cent in sustained clock, so the check is in two parts: every predicted
    time within 20 % of the measured one, and -- with the box's speed taken out through one reference
    point -- every predicted ratio to the reference within 12 % of the measured ratio."""
    from paper_2506_19651_amd.cost_model import choose_sink_and_block, predict_block_prefill_ms, video_layout
    heads = P.Heads(28, 4, 128, "bf16")
    grid = [(1, 4), (2, 8), (4, 2), (4, 16), (8, 8)]  # (sink frames, block frames); the first is the reference
    n_cu = torch.cuda.get_device_properties(0).multi_processor_count
    meas, pred = [], []
    for sf, bf in grid:
        S, B, C, Q = video_layout(0, 256, 256, 128, sf, bf)
        lay = P.Layout.from_seqs([(S, B, C, Q)])
        T = S + C + Q
        g = torch.Generator(device=DEV).manual_seed(5)
        q = (torch.randn(T, 28, 128, device=DEV, generator=g) * 0.5).bfloat16()
        k = (torch.randn(T, 4, 128, device=DEV, generator=g) * 0.5).bfloat16()
        v = (torch.randn(T, 4, 128, device=DEV, generator=g) * 0.5).bfloat16()
        out = torch.empty_like(q)
        ws = torch.empty(P.pevlm_block_prefill_workspace_bytes(lay, heads), dtype=torch.uint8, device=DEV)
        # untimed launches first: after an idle stretch the first few dozen launches of any kernel run slow
        # while the clocks settle
        for _ in range(40 if not meas else 10):
            P.pevlm_block_prefill_attn(q, k, v, out, lay, heads, workspace=ws)
        torch.cuda.synchronize()
        ts = []
        for _ in range(3):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(8):
                P.pevlm_block_prefill_attn(q, k, v, out, lay, heads, workspace=ws)
            e1.record()
            torch.cuda.synchronize()
            ts.append(e0.elapsed_time(e1) / 8)
        meas.append(sorted(ts)[1])
        pred.append(predict_block_prefill_ms(lay, heads, n_cu))
        print(f"[time model] sink {sf} frames, block {bf} frames: measured {meas[-1]:.3f} ms, predicted {pred[-1]:.3f} ms", flush=True)
    for m, p_ in zip(meas, pred):
        assert abs(p_ / m - 1.0) <= 0.20, (meas, pred)
        assert abs((p_ / pred[0]) / (m / meas[0]) - 1.0) <= 0.12, (meas, pred)
    # the chooser's pick under a cap set between two measured points really fits that cap here
    cap = 0.5 * (sorted(meas)[1] + sorted(meas)[2])
    best, _table = choose_sink_and_block(0, 256, 256, 128, heads, [sf for sf, _ in grid], [bf for _, bf in grid], cap, n_cu)
    assert best is not None and best[2] <= cap


# ------------------------------------------------------------------------------------ guard bands
def _guarded(nbytes, guard=4096):
    """A device byte range of exactly `nbytes` with `guard` bytes of a known pattern on both sides."""
    pad = (-nbytes) % 256
    buf = torch.full((guard + nbytes + pad + guard,), 0xA5, dtype=torch.uint8, device=DEV)
    return buf, buf[guard:guard + nbytes]


def _guards_intact(buf, nbytes, guard=4096):
    return bool((buf[:guard] == 0xA5).all()) and bool((buf[guard + nbytes:] == 0xA5).all())


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_nothing_is_written_outside_out_lse_and_the_workspaces(dtype, prefill_kernel):
    """out, lse and both workspaces sit between guard bands (workspaces sized exactly as the
    *_workspace_bytes queries say); after all calls every guard byte still holds its pattern."""
    seqs = [(130, 200, 777, 129), (0, 64, 320, 5), (17, 1000, 250, 0), (5, 3, 0, 200)]
    w = W.Workload("guards_" + dtype, 23, dtype, 8, 2, 128 if dtype == "bf16" else 64, 1.0e6, seqs, 0.5)
    data = W.generate(w)
    lay, heads = layout_heads(w)
    q, k, v = to_device(data["q"]), to_device(data["k"]), to_device(data["v"])
    esz = 2 if dtype == "bf16" else 4
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    n_out = q.numel() * esz
    n_lse = w.total_tokens * w.n_q_heads * 4
    sizes = dict(out=n_out, lse=n_lse,
                 wp=P.pevlm_block_prefill_workspace_bytes(lay, heads), wq=P.pevlm_query_workspace_bytes(lay, heads, 5))
    if dtype == "bf16":
        sizes["wpr"] = P.pevlm_block_prefill_rope_workspace_bytes(lay, heads)
        sizes["wqr"] = P.pevlm_query_rope_workspace_bytes(lay, heads, 5)
    bufs = {name: _guarded(n) for name, n in sizes.items()}
    out = bufs["out"][1].view(tdt).view(q.shape)
    lse = bufs["lse"][1].view(torch.float32).view(w.total_tokens, w.n_q_heads)
    P.pevlm_rope_seq(q, k, lay, heads, w.rope_base)
    P.pevlm_block_prefill_attn(q, k, v, out, lay, heads, lse=lse, workspace=bufs["wp"][1])
    P.pevlm_query_attn(q, k, v, out, lay, heads, num_splits=5, lse=lse, workspace=bufs["wq"][1])
    torch.cuda.synchronize()
    ref = out.clone()
    if dtype == "bf16":
        q2, k2 = to_device(data["q"]), to_device(data["k"])
        P.pevlm_block_prefill_attn_rope(q2, k2, v, out, lay, heads, w.rope_base, lse=lse, workspace=bufs["wpr"][1])
        P.pevlm_query_attn_rope(q2, k2, v, out, lay, heads, w.rope_base, num_splits=5, lse=lse, workspace=bufs["wqr"][1])
        torch.cuda.synchronize()
        assert torch.equal(out.view(torch.int16), ref.view(torch.int16))
    for name, n in sizes.items():
        assert _guards_intact(bufs[name][0], n), f"guard band of {name} overwritten"
    assert torch.isfinite(out.float()).all() and torch.isfinite(lse).all()


# ------------------------------------------------------------------------------------ graph capture
def test_calls_can_be_captured_in_a_graph_and_replayed(prefill_kernel):
    """The library neither allocates nor synchronises nor clears memory with memset nodes, so the
    three calls can be recorded into a HIP graph.  Replays (with eager work and synchronisation in
    between, on fresh inputs each time) must reproduce the eager result bit for bit."""
    w = W.small_variant(W.CONFIGS["c2"], "graph", [(256, 512, 2048, 64), (0, 128, 500, 20)])
    lay, heads = layout_heads(w)
    datas = [W.generate(W.small_variant(w, f"graph{i}", w.seqs, config_id=40 + i)) for i in range(3)]
    q, k, v = to_device(datas[0]["q"]), to_device(datas[0]["k"]), to_device(datas[0]["v"])
    out = torch.zeros_like(q)
    ws_p = torch.empty(P.pevlm_block_prefill_workspace_bytes(lay, heads), dtype=torch.uint8, device=DEV)
    ws_q = torch.empty(P.pevlm_query_workspace_bytes(lay, heads, 0), dtype=torch.uint8, device=DEV)

    def run():
        P.pevlm_rope_seq(q, k, lay, heads, w.rope_base)
        P.pevlm_block_prefill_attn(q, k, v, out, lay, heads, workspace=ws_p)
        P.pevlm_query_attn(q, k, v, out, lay, heads, workspace=ws_q)

    # eager references
    refs = []
    for d in datas:
        q.copy_(to_device(d["q"])); k.copy_(to_device(d["k"])); v.copy_(to_device(d["v"]))
        out.zero_()
        run()
        torch.cuda.synchronize()
        refs.append(out.clone())
    # capture once (warm-up on a side stream first, as torch asks)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run()
    for rep in range(2):
        for d, ref in zip(datas, refs):
            q.copy_(to_device(d["q"])); k.copy_(to_device(d["k"])); v.copy_(to_device(d["v"]))
            out.fill_(float("nan"))
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(out.view(torch.int16), ref.view(torch.int16)), (rep,)
            (out.float().sum() + 1).item()  # eager work between replays


@pytest.mark.parametrize("k_is_rotated", [False, True])
def test_folded_rope_with_three_axis_ids_equals_three_call_path_bitwise(oracle, k_is_rotated):
    w = W.Workload("mrope_fused", 19, "bf16", 8, 2, 128, 1.0e6, [(300, 512, 1536, 70), (256, 256, 900, 33)], 0.5)
    data = W.generate(w)
    ids = W.mrope_position_ids(w, 256, 16)
    section = (16, 24, 24)
    lay, heads = layout_heads(w)
    ids_d = torch.from_numpy(ids).to(DEV)
    # three calls
    q1, k1, v = to_device(data["q"]), to_device(data["k"]), to_device(data["v"])
    ref = torch.full_like(q1, float("nan"))
    P.pevlm_rope_mrope(q1, k1, w.total_tokens, heads, w.rope_base, ids_d, section)
    P.pevlm_block_prefill_attn(q1, k1, v, ref, lay, heads)
    P.pevlm_query_attn(q1, k1, v, ref, lay, heads, num_splits=3)
    # folded
    q2, k2 = to_device(data["q"]), to_device(data["k"])
    if k_is_rotated:
        P.pevlm_rope_mrope(None, k2, w.total_tokens, heads, w.rope_base, ids_d, section)
    out = torch.full_like(q2, float("nan"))
    P.pevlm_block_prefill_attn_mrope(q2, k2, v, out, lay, heads, w.rope_base, ids_d, section, k_is_rotated=k_is_rotated)
    P.pevlm_query_attn_mrope(q2, k2, v, out, lay, heads, w.rope_base, ids_d, section, num_splits=3)
    torch.cuda.synchronize()
    assert torch.equal(k2.view(torch.int16), k1.view(torch.int16))
    assert torch.equal(out.view(torch.int16), ref.view(torch.int16))
    assert torch.equal(q2.view(torch.int16), to_device(data["q"]).view(torch.int16))
    # and against the oracle
    q_exact = oracle.rope_mrope(data["q"], ids, section, w.rope_base)
    k_exact = oracle.rope_mrope(data["k"], ids, section, w.rope_base)
    want, _ = oracle.attn(q_exact, k_exact, data["v"], oracle_layout(oracle, w))
    check_bf16(to_host_f32(out), want, "mrope_fused")
