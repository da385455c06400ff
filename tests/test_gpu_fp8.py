"""Parity of the fp8 (E4M3) variant of the block-prefill call with the CPU oracle, through the C ABI.

Two things are checked separately, as the header of the call states them:
  * the quantised operands (an integer decision): codes, scales and tile images in the workspace are
    compared BIT FOR BIT with oracle/fp8_e4m3.py on the same bf16 inputs;
  * the attention over those operands: the oracle's exact (fp64) attention over the de-quantised
    tensors, against which the kernel differs only by the rounding of its weights to E4M3 and of its
    output to bf16.  Bound used below, element by element: with weights p_j = (1 + d_j) p*_j,
    |d_j| <= 2^-4 for weights at or above the smallest normal E4M3 number (2^-6, i.e. 2^-13 of the
    largest weight of the row or more), smaller ones are off by at most half a subnormal step 2^-10,
    i.e. 2^-17 of the largest weight each; the kernel divides by the sum of the UNROUNDED weights, so
        |out - out*| <= 2^-4 * A(|v|) + N 2^-17 max|v| + 2^-8 |out*|,
    A(|v|) being the same attention applied to |v| (computed by the oracle), N the number of visible
    keys, and the last term the bf16 rounding of the output."""
import numpy as np
import pytest
import torch

import paper_2506_19651_amd as P
import workloads as W
from gpu_util import DEV, error_stats, layout_heads, oracle_layout, to_device, to_host_f32
from oracle import fp8_e4m3 as F8

pytestmark = pytest.mark.gpu


def bf16_bits_to_f64(a):
    return (a.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def rotated_inputs(w, data):
    """bf16 Q, K (rotated on the device by the library's RoPE call) and V, as device tensors."""
    lay, heads = layout_heads(w)
    q, k, v = to_device(data["q"]), to_device(data["k"]), to_device(data["v"])
    P.pevlm_rope_seq(q, k, lay, heads, w.rope_base)
    torch.cuda.synchronize()
    return lay, heads, q, k, v


def host_bits(t):
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


def prefill_rows(w):
    a = w.layout_arrays()
    rows = [np.arange(c0, c0 + S + C) for c0, (S, B, C, Q) in zip(a["cu_seqlens"], w.seqs)]
    return np.concatenate(rows) if rows else np.zeros(0, np.int64)


def unswizzle_k(tiles, D):
    """[n, Hkv, 64 * D] tile images -> [n, Hkv, 64, D] codes."""
    n, Hkv, _ = tiles.shape
    cpr = D // 16
    img = tiles.reshape(n, Hkv, 64, cpr, 16)
    out = np.empty_like(img)
    for r in range(64):
        for c in range(cpr):
            out[:, :, r, c] = img[:, :, r, c ^ ((r // (16 // cpr)) % cpr)]
    return out.reshape(n, Hkv, 64, D)


def unswizzle_v(tiles, D):
    """[n, Hkv, D * 64] tile images -> [n, Hkv, 64 keys, D] codes."""
    n, Hkv, _ = tiles.shape
    img = tiles.reshape(n, Hkv, D, 4, 16)
    lin = np.empty_like(img)
    for d in range(D):
        for c in range(4):
            lin[:, :, d, c] = img[:, :, d, c ^ ((d // 4) % 4)]
    lin = lin.reshape(n, Hkv, D, 64)
    j = np.arange(64)
    key = ((j % 32) // 16) * 32 + ((j % 16) // 4) * 8 + (j // 32) * 4 + j % 4
    out = np.empty((n, Hkv, 64, D), np.uint8)
    out[:, :, key, :] = lin.transpose(0, 1, 3, 2)
    return out


QUANT_CASES = [("d128", 4, 2, 128, [(130, 200, 777, 9), (0, 64, 320, 5), (17, 100, 250, 0)]),
               ("d64", 6, 3, 64, [(70, 33, 150, 4), (5, 64, 64, 0)])]


@pytest.mark.parametrize("name,Hq,Hkv,D,seqs", QUANT_CASES, ids=[c[0] for c in QUANT_CASES])
def test_fp8_codes_scales_and_tile_images_bit_for_bit(name, Hq, Hkv, D, seqs):
    w = W.Workload("fp8q_" + name, 31, "bf16", Hq, Hkv, D, 1.0e6, seqs, 0.5)
    data = W.generate(w)
    # wide range of magnitudes, exact zeros, a negative zero and one dominant value per tensor
    rng = np.random.default_rng(5)
    for key_ in ("q", "k", "v"):
        x = bf16_bits_to_f64(data[key_]) * 2.0 ** rng.integers(-12, 6, data[key_].shape)
        x[rng.random(x.shape) < 0.01] = 0.0
        x[3, 0, 1] = -0.0
        x[11, 1, 5] = 300.0
        data[key_] = W.f32_to_bf16_bits(x.astype(np.float32))
    lay, heads = layout_heads(w)
    q, k, v = to_device(data["q"]), to_device(data["k"]), to_device(data["v"])
    out = torch.zeros_like(q)
    ws = P.pevlm_block_prefill_attn_fp8(q, k, v, out, lay, heads, stages=P.FP8_QUANTISE)
    torch.cuda.synchronize()
    assert torch.count_nonzero(out) == 0  # the quantise stage alone writes no output
    plan = P.pevlm_block_prefill_fp8_plan(lay, heads)
    raw = ws.cpu().numpy()
    T = w.total_tokens
    ref = F8.quantise_qkv(bf16_bits_to_f64(data["q"]), bf16_bits_to_f64(data["k"]), bf16_bits_to_f64(data["v"]), F8.q_factor(0.0, D))
    q_codes = raw[plan.q_codes: plan.q_codes + T * Hq * D].reshape(T, Hq, D)
    q_scales = raw[plan.q_scales: plan.q_scales + T * Hq * 4].view(np.float32).reshape(T, Hq)
    assert np.array_equal(q_codes, ref["q_codes"])
    assert np.array_equal(q_scales.astype(np.float64), np.ldexp(1.0, ref["q_exp"]))
    amax = raw[plan.kv_amax: plan.kv_amax + 2 * Hkv * 4].view(np.float32).reshape(2, Hkv).astype(np.float64)
    assert np.array_equal(amax[0], np.abs(bf16_bits_to_f64(data["k"])).max(axis=(0, 2)))
    assert np.array_equal(amax[1], np.abs(bf16_bits_to_f64(data["v"])).max(axis=(0, 2)))
    # the key tiles are the 64-row tiles of the regions, in the order of the host enumeration
    tiles = P.pevlm_prefill_worklist_host(lay, 64)
    n = len(tiles)
    assert n == plan.n_key_tiles
    dev_tiles = raw[plan.key_tiles: plan.key_tiles + n * 32].view(np.int32).reshape(n, 8)
    assert np.array_equal(dev_tiles[:, :2], np.array([[t.q_start, t.q_rows] for t in tiles], np.int32))
    kt = unswizzle_k(raw[plan.k_tiles: plan.k_tiles + n * Hkv * 64 * D].reshape(n, Hkv, 64 * D), D)
    vt = unswizzle_v(raw[plan.v_tiles: plan.v_tiles + n * Hkv * 64 * D].reshape(n, Hkv, 64 * D), D)
    for i, t in enumerate(tiles):
        rows = slice(t.q_start, t.q_start + t.q_rows)
        assert np.array_equal(kt[i, :, :t.q_rows], ref["k_codes"][rows].transpose(1, 0, 2)), i
        assert np.array_equal(vt[i, :, :t.q_rows], ref["v_codes"][rows].transpose(1, 0, 2)), i
        assert not kt[i, :, t.q_rows:].any() and not vt[i, :, t.q_rows:].any()  # padding rows are zero codes


ATTN_CASES = [
    ("d128", 4, 2, 128, [(130, 200, 777, 9), (0, 64, 320, 5), (17, 100, 250, 0), (5, 3, 0, 20)], {}),
    ("d64", 6, 3, 64, [(70, 33, 150, 4), (200, 300, 900, 0)], {}),
    ("d128_gqa7", 28, 4, 128, [(256, 1024, 2048, 16)], {}),
    ("d128_peaky", 4, 2, 128, [(200, 300, 900, 40)], dict(qk_scale=2.5)),
    ("d128_rising", 4, 2, 128, [(128, 640, 1280, 64)], dict(qk_scale=1.5, key_ramp=6.0)),
]


def fp8_reference(oracle, w, q_bits, k_bits, v_bits, rows):
    """Exact attention over the de-quantised tensors, and the same attention applied to |v|."""
    qd, kd, vd = F8.dequantised_qkv(bf16_bits_to_f64(q_bits), bf16_bits_to_f64(k_bits), bf16_bits_to_f64(v_bits),
                                    F8.q_factor(0.0, w.head_dim))
    olay = oracle_layout(oracle, w)
    want, want_lse = oracle.attn(qd[rows], kd, vd, olay, rows=rows)
    mean_abs_v, _ = oracle.attn(qd[rows], kd, np.abs(vd), olay, rows=rows)
    return want, want_lse, mean_abs_v, float(np.abs(vd).max())


def check_fp8(got, got_lse, want, want_lse, mean_abs_v, vmax, n_keys, tag):
    bound = 2.0 ** -4 * mean_abs_v + n_keys * 2.0 ** -17 * vmax + 2.0 ** -8 * np.abs(want) + 1e-30
    err = np.abs(got - want)
    st = error_stats(got, want)
    print(f"[fp8 {tag}] max_abs={st['max_abs']:.3e} mean_abs={st['mean_abs']:.3e} max_rel_l2={st['max_rel_l2']:.3e} "
          f"worst err/bound={float((err / bound).max()):.3f} lse_err={float(np.abs(got_lse - want_lse).max()):.2e}", flush=True)
    assert np.isfinite(got).all()
    assert np.all(err <= bound)
    # the sum of the weights is kept unrounded: lse carries only fp32 rounding and the exp2 approximation
    assert np.max(np.abs(got_lse - want_lse)) <= 2e-3 + 1e-5 * np.abs(want_lse).max()


@pytest.mark.parametrize("name,Hq,Hkv,D,seqs,extra", ATTN_CASES, ids=[c[0] for c in ATTN_CASES])
def test_fp8_attention_against_oracle_over_the_quantised_tensors(oracle, name, Hq, Hkv, D, seqs, extra):
    w = W.Workload("fp8a_" + name, 32, "bf16", Hq, Hkv, D, 1.0e6, seqs, 0.5, **extra)
    data = W.generate(w)
    lay, heads, q, k, v = rotated_inputs(w, data)
    out = torch.full_like(q, float("nan"))
    lse = torch.full((w.total_tokens, Hq), float("nan"), device=DEV)
    ws = P.pevlm_block_prefill_attn_fp8(q, k, v, out, lay, heads, lse=lse)
    torch.cuda.synchronize()
    rows = prefill_rows(w)
    want, want_lse, mean_abs_v, vmax = fp8_reference(oracle, w, host_bits(q), host_bits(k), host_bits(v), rows)
    ridx = torch.from_numpy(rows).to(DEV)
    n_keys = max(S + B for (S, B, C, Q) in seqs)
    check_fp8(to_host_f32(out[ridx]), to_host_f32(lse[ridx]), want, want_lse, mean_abs_v, vmax, n_keys, name)
    # question rows are not this call's: untouched
    other = np.setdiff1d(np.arange(w.total_tokens), rows)
    if other.size:
        assert torch.isnan(out[torch.from_numpy(other).to(DEV)].float()).all()
    # the attend stage alone, from the workspace the first call filled, reproduces the result bit for bit
    out2 = torch.full_like(q, float("nan"))
    P.pevlm_block_prefill_attn_fp8(q, k, v, out2, lay, heads, workspace=ws, stages=P.FP8_ATTEND)
    torch.cuda.synchronize()
    assert torch.equal(out2[ridx].view(torch.int16), out[ridx].view(torch.int16))
    # end to end against the unquantised operands (what a user of the variant gives up): reported, loosely bounded
    olay = oracle_layout(oracle, w)
    exact, _ = oracle.attn(bf16_bits_to_f64(host_bits(q))[rows], bf16_bits_to_f64(host_bits(k)), data["v"], olay, rows=rows)
    st = error_stats(to_host_f32(out[ridx]), exact)
    print(f"[fp8 {name}] against unquantised operands: max_abs={st['max_abs']:.3e} mean_abs={st['mean_abs']:.3e} "
          f"max_rel_l2={st['max_rel_l2']:.3e}", flush=True)
    assert st["mean_abs"] <= 2e-2


def test_fp8_with_a_head_map_and_a_caller_scale(oracle):
    """Query heads mapped to KV heads out of order (unequal use would be legal too) and a softmax factor
    other than 1/sqrt(d): both reach the fp8 kernel through the per-lane exponent constant and the head tables."""
    seqs = [(100, 160, 500, 7), (30, 64, 200, 0)]
    kv_map = [1, 0, 0, 1, 1, 0, 1, 0]
    w = W.Workload("fp8_map", 34, "bf16", 8, 2, 128, 1.0e6, seqs, 0.5)
    data = W.generate(w)
    lay, heads = layout_heads(w, kv_map, 0.2)
    q, k, v = to_device(data["q"]), to_device(data["k"]), to_device(data["v"])
    P.pevlm_rope_seq(q, k, lay, heads, w.rope_base)
    out = torch.full_like(q, float("nan"))
    lse = torch.full((w.total_tokens, 8), float("nan"), device=DEV)
    P.pevlm_block_prefill_attn_fp8(q, k, v, out, lay, heads, lse=lse)
    torch.cuda.synchronize()
    rows = prefill_rows(w)
    qd, kd, vd = F8.dequantised_qkv(bf16_bits_to_f64(host_bits(q)), bf16_bits_to_f64(host_bits(k)), bf16_bits_to_f64(host_bits(v)),
                                    F8.q_factor(0.2, 128))
    olay = oracle_layout(oracle, w)
    s32 = float(np.float32(0.2))
    want, want_lse = oracle.attn(qd[rows], kd, vd, olay, rows=rows, kv_head_of_q=kv_map, softmax_scale=s32)
    mean_abs_v, _ = oracle.attn(qd[rows], kd, np.abs(vd), olay, rows=rows, kv_head_of_q=kv_map, softmax_scale=s32)
    ridx = torch.from_numpy(rows).to(DEV)
    check_fp8(to_host_f32(out[ridx]), to_host_f32(lse[ridx]), want, want_lse, mean_abs_v, float(np.abs(vd).max()),
              max(S + B for (S, B, C, Q) in seqs), "head map, scale 0.2")
    plain, _ = oracle.attn(qd[rows], kd, vd, olay, rows=rows)  # default map and scale: must differ
    assert np.max(np.abs(plain - want)) > 0.05


def test_fp8_batch_larger_than_one_sequence_table(oracle):
    """130 packed sequences (the sequence table travels to the kernels in pieces of 48): the key-tile
    numbering and the work list run on across the pieces; sequences without sink, without context,
    blocks shorter than a tile."""
    rng = np.random.default_rng(5)
    seqs = []
    for _ in range(130):
        S, B = int(rng.integers(0, 40)), int(rng.integers(1, 50))
        C = int(rng.integers(0, 120)) if rng.random() < 0.8 else 0
        Q = int(rng.integers(0, 20))
        seqs.append((S, B, C, Q if S + C + Q else 1))
    w = W.Workload("fp8_many", 35, "bf16", 4, 2, 64, 1.0e4, seqs, 0.5)
    data = W.generate(w)
    lay, heads, q, k, v = rotated_inputs(w, data)
    out = torch.full_like(q, float("nan"))
    lse = torch.full((w.total_tokens, 4), float("nan"), device=DEV)
    ws = P.pevlm_block_prefill_attn_fp8(q, k, v, out, lay, heads, lse=lse)
    torch.cuda.synchronize()
    rows = prefill_rows(w)
    want, want_lse, mean_abs_v, vmax = fp8_reference(oracle, w, host_bits(q), host_bits(k), host_bits(v), rows)
    ridx = torch.from_numpy(rows).to(DEV)
    check_fp8(to_host_f32(out[ridx]), to_host_f32(lse[ridx]), want, want_lse, mean_abs_v, vmax, max(S + B for (S, B, C, Q) in seqs), "130 sequences")
    plan = P.pevlm_block_prefill_fp8_plan(lay, heads)
    tiles = P.pevlm_prefill_worklist_host(lay, 64)
    dev_tiles = ws.cpu().numpy()[plan.key_tiles: plan.key_tiles + len(tiles) * 32].view(np.int32).reshape(len(tiles), 8)
    assert len(tiles) == plan.n_key_tiles > 130
    assert np.array_equal(dev_tiles[:, :2], np.array([[t.q_start, t.q_rows] for t in tiles], np.int32))


@pytest.mark.parametrize("cfg,n_random", [("c3", 100), ("c4a", 64), ("c5b", 64)])
def test_fp8_full_size_sampled_rows(oracle, cfg, n_random):
    """Full-size configurations (c3: the one bench.py times; c4a: 392-token sink and blocks, ragged tiles;
    c5b: four sequences with partial last blocks): sampled sink and context rows (region and block edges,
    tile edges, seeded random rows) against the oracle over the de-quantised operands."""
    w = W.CONFIGS[cfg]
    data = W.generate(w)
    lay, heads, q, k, v = rotated_inputs(w, data)
    out = torch.full_like(q, float("nan"))
    lse = torch.full((w.total_tokens, w.n_q_heads), float("nan"), device=DEV)
    P.pevlm_block_prefill_attn_fp8(q, k, v, out, lay, heads, lse=lse)
    torch.cuda.synchronize()
    pre = prefill_rows(w)
    rows = np.intersect1d(W.sample_rows(w, n_random=n_random, max_question_rows=1), pre)
    assert rows.size >= 60
    want, want_lse, mean_abs_v, vmax = fp8_reference(oracle, w, host_bits(q), host_bits(k), host_bits(v), rows)
    ridx = torch.from_numpy(rows).to(DEV)
    check_fp8(to_host_f32(out[ridx]), to_host_f32(lse[ridx]), want, want_lse, mean_abs_v, vmax,
              max(S + B for (S, B, C, Q) in w.seqs), cfg)
    assert torch.isfinite(out[torch.from_numpy(pre).to(DEV)].float()).all()


def test_fp8_rejects_what_it_does_not_cover():
    lay = P.Layout.from_seqs([(8, 8, 16, 0)])
    with pytest.raises(Exception):
        P.pevlm_block_prefill_fp8_plan(lay, P.Heads(2, 1, 64, "f32"))
    heads = P.Heads(2, 1, 64, "bf16")
    q = torch.zeros((24, 2, 64), dtype=torch.bfloat16, device=DEV)
    k = torch.zeros((24, 1, 64), dtype=torch.bfloat16, device=DEV)
    small = torch.zeros(256, dtype=torch.uint8, device=DEV)
    with pytest.raises(Exception):
        P.pevlm_block_prefill_attn_fp8(q, k, k, q.clone(), lay, heads, workspace=small)
    with pytest.raises(Exception):
        P.pevlm_block_prefill_attn_fp8(q, k, k, q.clone(), lay, heads, stages=4)
