"""Pins for the CPU oracle: every check here takes its expected value from somewhere other than
the oracle -- brute-force loops over the three formulas (Eq. 3-5), torch's CPU attention routine,
the paper's closed-form operation counts (Eq. 6-10), closed forms and analytic identities."""
import itertools
import cmath
import math

import numpy as np
import pytest
import torch

RNG = np.random.default_rng(12345)


def make_layout(oracle, seqs):
    lens = [s + c + q for (s, b, c, q) in seqs]
    cu = np.concatenate([[0], np.cumsum(lens)])
    a = np.asarray(seqs).reshape(-1, 4)
    return oracle.Layout(cu, a[:, 0], a[:, 1], a[:, 2], a[:, 3])


def rand_qkv(T, Hq, Hkv, D, rng=RNG):
    return (rng.standard_normal((T, Hq, D)), rng.standard_normal((T, Hkv, D)),
            rng.standard_normal((T, Hkv, D)))


# ------------------------------------------------------------------ brute force (tiny inputs)
def brute_rope_complex(x, pos, base):
    """Rotation written as a complex multiplication: (x_i + i x_{i+D/2}) * exp(i pos base^(-2i/D))."""
    T, H, D = x.shape
    half = D // 2
    z = x[..., :half] + 1j * x[..., half:]
    freq = np.array([base ** (-2.0 * i / D) for i in range(half)])
    rot = np.exp(1j * pos[:, None, None] * freq[None, None, :])
    z = z * rot
    return np.concatenate([z.real, z.imag], axis=-1)


def brute_causal_attention(q_rows, k_rows, v_rows):
    """Plain loops: the last len(q_rows) positions of a causal attention over len(k_rows) keys.
    q_rows [n, D], k_rows/v_rows [m, D], n <= m; query r sits at key position m - n + r."""
    n, D = len(q_rows), len(q_rows[0])
    m = len(k_rows)
    out = []
    for r in range(n):
        last = m - n + r
        scores = []
        for j in range(last + 1):
            dot = 0.0
            for d in range(D):
                dot += q_rows[r][d] * k_rows[j][d]
            scores.append(dot / math.sqrt(D))
        mx = max(scores)
        ws = [math.exp(s - mx) for s in scores]
        tot = sum(ws)
        out.append([sum(ws[j] * v_rows[j][d] for j in range(last + 1)) / tot for d in range(D)])
    return out


def brute_pevlm(q, k, v, seqs, base, Hq, Hkv):
    """Eq. 3, 4 and 5 evaluated one at a time, each on its own gathered key set."""
    T, _, D = q.shape
    out = np.zeros((T, Hq, D))
    start = 0
    for (S, B, C, Q) in seqs:
        L = S + C + Q
        pos = np.arange(L, dtype=np.float64)  # sequential positions, never re-based
        qs = brute_rope_complex(q[start:start + L], pos, base)
        ks = brute_rope_complex(k[start:start + L], pos, base)
        vs = v[start:start + L]
        for h in range(Hq):
            g = h // (Hq // Hkv)
            Qh, Kh, Vh = qs[:, h].tolist(), ks[:, g].tolist(), vs[:, g].tolist()
            # Eq. 3: sink attends to itself
            if S:
                out[start:start + S, h] = brute_causal_attention(Qh[:S], Kh[:S], Vh[:S])
            # Eq. 4: block c_i attends to sink + c_i
            nb = (C + B - 1) // B if C else 0
            for b in range(nb):
                b0, b1 = S + b * B, min(S + C, S + (b + 1) * B)
                out[start + b0:start + b1, h] = brute_causal_attention(
                    Qh[b0:b1], Kh[:S] + Kh[b0:b1], Vh[:S] + Vh[b0:b1])
            # Eq. 5: question attends to sink + all blocks + itself
            if Q:
                out[start + S + C:start + L, h] = brute_causal_attention(Qh[S + C:], Kh, Vh)
        start += L
    return out


TINY = [
    [(0, 1, 0, 1)],
    [(3, 2, 6, 4)],
    [(1, 5, 13, 0)],          # partial last block (5,5,3), no question
    [(0, 2, 6, 1)],           # no sink: block-attention mask
    [(3, 1, 3, 1)],           # blocks of one token
    [(4, 5, 0, 4)],           # no context: sink + question
    [(3, 5, 7, 4), (0, 2, 5, 0), (2, 3, 3, 1)],  # packed batch, ragged
]


@pytest.mark.parametrize("seqs", TINY)
@pytest.mark.parametrize("heads", [(1, 1, 2), (2, 1, 4), (4, 2, 4)])
def test_p1_brute_force(oracle, seqs, heads):
    Hq, Hkv, D = heads
    lay = make_layout(oracle, seqs)
    T = lay.total_tokens
    q, k, v = rand_qkv(T, Hq, Hkv, D)
    want = brute_pevlm(q, k, v, seqs, 10000.0, Hq, Hkv)
    for skip in (True, False):
        got, _ = oracle.forward(q, k, v, lay, 10000.0, skip_masked=skip)
        assert np.max(np.abs(got - want)) <= 1e-12


# ------------------------------------------------------------------ library routine on the pieces
def sdpa_last_rows(q, k, v, n_last, Hq, Hkv):
    """torch CPU causal attention over a gathered sequence; returns its last n_last rows."""
    G = Hq // Hkv
    qt = torch.from_numpy(q).permute(1, 0, 2)[None]                      # [1,Hq,m,D]
    kt = torch.from_numpy(k).permute(1, 0, 2).repeat_interleave(G, 0)[None]
    vt = torch.from_numpy(v).permute(1, 0, 2).repeat_interleave(G, 0)[None]
    o = torch.nn.functional.scaled_dot_product_attention(qt, kt, vt, is_causal=True)
    return o[0].permute(1, 0, 2).numpy()[-n_last:] if n_last else np.zeros((0, Hq, q.shape[-1]))


@pytest.mark.parametrize("seqs", [[(16, 8, 40, 6)], [(5, 7, 31, 3)], [(0, 16, 50, 9)], [(12, 9, 0, 5)]])
def test_p2_pieces_equal_library_causal_attention(oracle, seqs):
    Hq, Hkv, D, base = 4, 2, 16, 1.0e6
    (S, B, C, Q), = seqs
    L = S + C + Q
    lay = make_layout(oracle, seqs)
    q, k, v = rand_qkv(L, Hq, Hkv, D)
    got, _ = oracle.forward(q, k, v, lay, base)
    pos = np.arange(L, dtype=np.float64)
    qr, kr = brute_rope_complex(q, pos, base), brute_rope_complex(k, pos, base)
    if S:
        np.testing.assert_allclose(got[:S], sdpa_last_rows(qr[:S], kr[:S], v[:S], S, Hq, Hkv), atol=1e-10, rtol=0)
    nb = (C + B - 1) // B if C else 0
    for b in range(nb):
        b0, b1 = S + b * B, min(S + C, S + (b + 1) * B)
        idx = np.r_[0:S, b0:b1]
        want = sdpa_last_rows(qr[idx], kr[idx], v[idx], b1 - b0, Hq, Hkv)
        np.testing.assert_allclose(got[b0:b1], want, atol=1e-10, rtol=0)
    if Q:
        np.testing.assert_allclose(got[S + C:], sdpa_last_rows(qr, kr, v, Q, Hq, Hkv), atol=1e-10, rtol=0)


# ------------------------------------------------------------------ closed-form pair counts
def eq10_pairs(S, B, N, Q):
    """Operation count of Eq. 10 without the 2H factor."""
    return S * S + Q * Q + N * B * B + Q * S + N * Q * B + N * S * B


@pytest.mark.parametrize("S,B,N,Q", [(32, 16, 4, 8), (3, 2, 5, 4), (0, 4, 3, 2), (7, 1, 6, 0), (5, 9, 0, 3),
                                     (256, 1024, 2, 64)])
def test_p3_blockwise_mask_sums_to_eq10(oracle, S, B, N, Q):
    lay = make_layout(oracle, [(S, B, N * B, Q)])
    total = sum(int(oracle.mask_row(lay, t, causal=False).sum()) for t in range(lay.total_tokens))
    assert total == eq10_pairs(S, B, N, Q)


def causal_pairs(S, B, C, Q):
    blocks = [B] * (C // B) + ([C % B] if C % B else [])
    return (S * (S + 1) // 2 + sum(b * S + b * (b + 1) // 2 for b in blocks)
            + Q * (S + C) + Q * (Q + 1) // 2)


@pytest.mark.parametrize("S,B,C,Q,expect", [
    (32, 16, 64, 8, 3924),            # tiny sanity config: 528 + 2592 + 804
    (3, 5, 13, 2, None), (0, 4, 10, 0, None), (256, 1024, 2048 + 256, 64, None)])
def test_p3_causal_mask_pair_count(oracle, S, B, C, Q, expect):
    lay = make_layout(oracle, [(S, B, C, Q)])
    total = sum(int(oracle.mask_row(lay, t).sum()) for t in range(lay.total_tokens))
    assert total == causal_pairs(S, B, C, Q)
    if expect is not None:
        assert total == expect


def test_p3_golden_pair_counts(oracle):
    """Per-region visible pairs per head at the 16K-token config, from the closed forms
    (tests/golden/pair_counts.txt), against the oracle's explicit mask rows."""
    import os
    path = os.path.join(os.path.dirname(__file__), "golden", "pair_counts.txt")
    want = {}
    for line in open(path):
        if line.startswith("#") or not line.strip():
            continue
        name, sink, blocks, question = line.split()
        want[name] = (int(sink), int(blocks), int(question))
    S, B, C, Q = 256, 1024, 16384, 64
    lay = make_layout(oracle, [(S, B, C, Q)])
    sums = [0, 0, 0]
    for t in range(lay.total_tokens):
        sums[0 if t < S else (1 if t < S + C else 2)] += int(oracle.mask_row(lay, t).sum())
    assert tuple(sums) == want["c2"]


def test_mask_matrix_structure(oracle):
    """Independent construction of the mask from the prose: causal; sink keys visible to all later
    rows; context rows see no other block; question rows see everything before them; sequences of
    a packed batch are isolated."""
    seqs = [(3, 4, 10, 2), (2, 3, 6, 1)]
    lay = make_layout(oracle, seqs)
    M = oracle.mask_matrix(lay)
    T = lay.total_tokens
    want = np.zeros((T, T), np.uint8)
    base = 0
    for (S, B, C, Q) in seqs:
        L = S + C + Q
        region = ["s"] * S + [("c", p // B) for p in range(C)] + ["q"] * Q
        for i in range(L):
            for j in range(i + 1):
                ok = region[j] == "s" or region[i] == "q" or region[i] == region[j]
                want[base + i, base + j] = ok
        base += L
    assert np.array_equal(M, want)
    assert np.all(np.diag(M) == 1)  # every row sees itself: no empty softmax


# ------------------------------------------------------------------ degenerate layouts
def test_p4_degenerate_layouts_reduce_to_causal(oracle):
    Hq, Hkv, D, base, L = 4, 2, 8, 1.0e4, 37
    q, k, v = rand_qkv(L, Hq, Hkv, D)
    pos = np.arange(L, dtype=np.float64)
    qr, kr = brute_rope_complex(q, pos, base), brute_rope_complex(k, pos, base)
    full = sdpa_last_rows(qr, kr, v, L, Hq, Hkv)
    for seqs in ([(0, L, L, 0)],      # one block, no sink
                 [(20, 5, 0, 17)],    # no context
                 [(L, 1, 0, 0)],      # sink only
                 [(0, 1, 0, L)]):     # question only
        got, _ = oracle.forward(q, k, v, make_layout(oracle, seqs), base)
        np.testing.assert_allclose(got, full, atol=1e-12, rtol=0)
    # no sink: block-diagonal causal
    B = 10
    got, _ = oracle.forward(q, k, v, make_layout(oracle, [(0, B, L, 0)]), base)
    for b0 in range(0, L, B):
        b1 = min(L, b0 + B)
        np.testing.assert_allclose(got[b0:b1], sdpa_last_rows(qr[b0:b1], kr[b0:b1], v[b0:b1], b1 - b0, Hq, Hkv),
                                   atol=1e-12, rtol=0)


# ------------------------------------------------------------------ convexity, constant V, zero Q
def test_p5_convex_constant_zeroq(oracle):
    seqs = [(6, 5, 17, 4), (0, 3, 7, 2)]
    Hq, Hkv, D = 4, 2, 8
    lay = make_layout(oracle, seqs)
    T = lay.total_tokens
    q, k, v = rand_qkv(T, Hq, Hkv, D)
    M = oracle.mask_matrix(lay).astype(bool)
    got, _ = oracle.forward(q, k, v, lay, 1.0e4)
    for t in range(T):
        for h in range(Hq):
            vv = v[M[t], h // 2]
            assert np.all(got[t, h] <= vv.max(0) + 1e-12) and np.all(got[t, h] >= vv.min(0) - 1e-12)
    vc = np.broadcast_to(RNG.standard_normal((1, Hkv, D)), (T, Hkv, D)).copy()
    got, _ = oracle.forward(q, k, vc, lay, 1.0e4)
    np.testing.assert_allclose(got, np.repeat(vc, 2, axis=1), atol=1e-12, rtol=0)
    got, lse = oracle.forward(np.zeros_like(q), k, v, lay, 1.0e4)
    for t in range(T):
        for h in range(Hq):
            np.testing.assert_allclose(got[t, h], v[M[t], h // 2].mean(0), atol=1e-12, rtol=0)
            assert abs(lse[t, h] - math.log(M[t].sum())) <= 1e-12


# ------------------------------------------------------------------ leaks / masked contribution
def test_p6_masked_keys_contribute_exactly_zero(oracle):
    seqs = [(5, 4, 14, 3), (2, 6, 6, 2)]
    Hq, Hkv, D = 2, 1, 8
    lay = make_layout(oracle, seqs)
    T = lay.total_tokens
    q, k, v = rand_qkv(T, Hq, Hkv, D)
    M = oracle.mask_matrix(lay).astype(bool)
    # (i) literal -inf mask == masked keys bypassed, bit for bit
    a, la = oracle.forward(q, k, v, lay, 1.0e4, skip_masked=False)
    b, lb = oracle.forward(q, k, v, lay, 1.0e4, skip_masked=True)
    assert np.array_equal(a, b) and np.array_equal(la, lb)
    # (ii) V = 0 on visible keys and 1 on invisible ones -> exactly 0
    pos = oracle.positions(lay)
    kr = oracle.rope(k, pos, 1.0e4)
    for t in range(T):
        vv = np.where(M[t][:, None, None], 0.0, 1.0) * np.ones((T, Hkv, D))
        qr = oracle.rope(q, pos, 1.0e4, rows=[t])
        o, _ = oracle.attn(qr, kr, vv, lay, rows=[t])
        assert np.all(o == 0.0)
    # (iii) perturbing another block's K/V leaves a block's rows bitwise unchanged
    S, B, C, Q = seqs[0]
    k2, v2 = k.copy(), v.copy()
    k2[S + B:S + 2 * B] += 3.0
    v2[S + B:S + 2 * B] -= 5.0
    c, _ = oracle.forward(q, k2, v2, lay, 1.0e4)
    keep = np.r_[0:S + B, S + 2 * B:S + C, S + C + Q:T]
    assert np.array_equal(c[keep], b[keep])
    assert not np.array_equal(c[S + B:S + 2 * B], b[S + B:S + 2 * B])
    assert not np.array_equal(c[S + C:S + C + Q], b[S + C:S + C + Q])  # the question does see it


# ------------------------------------------------------------------ RoPE identities
def test_p7_rope_identities(oracle):
    T, H, D, base = 9, 3, 16, 1.0e4
    x = RNG.standard_normal((T, H, D))
    pos = np.array([0, 1, 2, 5, 100, 1000, 65535, 100999, 7], dtype=np.int32)
    y = oracle.rope(x, pos, base)
    np.testing.assert_array_equal(y[0], x[0])                       # p = 0 is the identity
    half = D // 2
    n_in = x[..., :half] ** 2 + x[..., half:] ** 2
    n_out = y[..., :half] ** 2 + y[..., half:] ** 2
    np.testing.assert_allclose(n_out, n_in, rtol=1e-13)            # each pair keeps its norm
    # pair 0 turns by exactly pos radians: spot values at p = 1
    np.testing.assert_allclose(y[1, :, 0], x[1, :, 0] * math.cos(1.0) - x[1, :, half] * math.sin(1.0), atol=1e-15)
    np.testing.assert_allclose(y[1, :, half], x[1, :, half] * math.cos(1.0) + x[1, :, 0] * math.sin(1.0), atol=1e-15)
    # last pair turns by pos * base^(-(D-2)/D)
    th = 5 * base ** (-(D - 2) / D)
    np.testing.assert_allclose(y[3, :, half - 1], x[3, :, half - 1] * math.cos(th) - x[3, :, D - 1] * math.sin(th),
                               atol=1e-15)
    np.testing.assert_allclose(y, brute_rope_complex(x, pos.astype(np.float64), base), atol=1e-11, rtol=0)
    # <R_m q, R_n k> depends on m - n only
    qv, kv = RNG.standard_normal((1, 1, D)), RNG.standard_normal((1, 1, D))
    dots = []
    for m, n in ((10, 3), (1007, 1000), (50007, 50000)):
        dots.append(float(np.sum(oracle.rope(qv, np.array([m], np.int32), base) *
                                 oracle.rope(kv, np.array([n], np.int32), base))))
    assert max(dots) - min(dots) <= 1e-9
    # inputs in float32 and bf16 bits are widened exactly
    xf = x.astype(np.float32)
    np.testing.assert_array_equal(oracle.rope(xf, pos, base), oracle.rope(xf.astype(np.float64), pos, base))
    bits = (xf.view(np.uint32) >> 16).astype(np.uint16)
    xb = (bits.astype(np.uint32) << 16).view(np.float32)
    np.testing.assert_array_equal(oracle.rope(bits, pos, base), oracle.rope(xb.astype(np.float64), pos, base))


def test_p7_constant_position_offset_changes_nothing(oracle):
    seqs = [(4, 5, 12, 3), (3, 4, 4, 2)]
    lay = make_layout(oracle, seqs)
    q, k, v = rand_qkv(lay.total_tokens, 2, 2, 8)
    a, _ = oracle.forward(q, k, v, lay, 1.0e4)
    b, _ = oracle.forward(q, k, v, lay, 1.0e4, pos_offset=[1234, 77])
    assert np.max(np.abs(a - b)) <= 1e-9


def test_p7_position_offsets_written_out(oracle):
    """Sequential positions with a per-sequence start: token n of sequence s sits at o_s + n
    (Sec. "Position Encoding": the ids of the whole prompt are kept), spelt out by hand."""
    seqs = [(2, 2, 3, 1), (1, 3, 3, 0), (0, 1, 0, 2)]
    lay = make_layout(oracle, seqs)
    assert oracle.positions(lay).tolist() == [0, 1, 2, 3, 4, 5, 0, 1, 2, 3, 0, 1]
    assert oracle.positions(lay, [100, 7, 50000]).tolist() == [100, 101, 102, 103, 104, 105, 7, 8, 9, 10, 50000, 50001]
    # offsets of distinct sequences are independent of each other
    assert oracle.positions(lay, [0, 9, 0]).tolist() == [0, 1, 2, 3, 4, 5, 9, 10, 11, 12, 0, 1]


def test_p7_rotation_under_position_offsets_matches_complex_multiplication(oracle):
    """The whole path with non-zero starts: rotated Q/K equal the complex-multiplication brute force
    at positions o_s + n, and the attention output equals the brute force evaluated at those
    positions.  Distinct per-sequence offsets; the path is not invariant to a dropped or shared
    offset in its rotated tensors even though attention outputs are (relative property)."""
    seqs = [(3, 4, 9, 2), (2, 3, 5, 3)]
    offs = [37, 1201]
    Hq, Hkv, D, base = 2, 1, 8, 1.0e4
    lay = make_layout(oracle, seqs)
    T = lay.total_tokens
    q, k, v = rand_qkv(T, Hq, Hkv, D)
    want_pos = np.concatenate([np.arange(3 + 9 + 2) + 37, np.arange(2 + 5 + 3) + 1201]).astype(np.float64)
    pos = oracle.positions(lay, offs)
    np.testing.assert_array_equal(pos, want_pos.astype(np.int32))
    np.testing.assert_allclose(oracle.rope(k, pos, base), brute_rope_complex(k, want_pos, base), atol=1e-11, rtol=0)
    np.testing.assert_allclose(oracle.rope(q, pos, base, rows=[1, 15, 20]),
                               brute_rope_complex(q, want_pos, base)[[1, 15, 20]], atol=1e-11, rtol=0)
    # rotated keys under an offset differ from the ones without (the offset really enters the angle)
    assert np.max(np.abs(oracle.rope(k, pos, base) - oracle.rope(k, oracle.positions(lay), base))) > 0.1


# ------------------------------------------------------------------ caller-chosen softmax scale (Eq. 1)
def brute_scaled_attention(q_rows, k_rows, v_rows, visible, scale):
    """Plain loops: softmax(scale * q.k over the visible keys) V, for each query row r and its key set
    visible[r] (indices into k_rows)."""
    out, lse = [], []
    for r, keys in enumerate(visible):
        scores = [scale * sum(q_rows[r][d] * k_rows[j][d] for d in range(len(q_rows[r]))) for j in keys]
        mx = max(scores)
        ws = [math.exp(s - mx) for s in scores]
        tot = sum(ws)
        out.append([sum(w * v_rows[j][d] for w, j in zip(ws, keys)) / tot for d in range(len(v_rows[0]))])
        lse.append(mx + math.log(tot))
    return out, lse


@pytest.mark.parametrize("scale", [0.05, 0.2, 1.7])
def test_p13_custom_softmax_scale_against_brute_force(oracle, scale):
    """Eq. 1 with the caller's factor in place of 1/sqrt(d): out and lse against plain loops over the
    visible keys of each row (visibility written out from Eq. 3-5, not taken from the oracle)."""
    (S, B, C, Q) = (3, 4, 10, 3)
    L = S + C + Q
    Hq, Hkv, D, base = 2, 1, 6, 1.0e4
    lay = make_layout(oracle, [(S, B, C, Q)])
    q, k, v = rand_qkv(L, Hq, Hkv, D)
    posf = np.arange(L, dtype=np.float64)
    qr, kr = brute_rope_complex(q, posf, base), brute_rope_complex(k, posf, base)
    visible = []
    for i in range(L):
        if i < S or i >= S + C:
            visible.append(list(range(i + 1)))
        else:
            b0 = S + ((i - S) // B) * B
            visible.append(list(range(S)) + list(range(b0, i + 1)))
    got, got_lse = oracle.forward(q, k, v, lay, base, softmax_scale=scale)
    for h in range(Hq):
        want, want_lse = brute_scaled_attention(qr[:, h].tolist(), kr[:, 0].tolist(), v[:, 0].tolist(), visible, scale)
        assert np.max(np.abs(got[:, h] - np.asarray(want))) <= 1e-12
        assert np.max(np.abs(got_lse[:, h] - np.asarray(want_lse))) <= 1e-12


def test_p13_explicit_default_scale_and_scale_sensitivity(oracle):
    """Passing 1/sqrt(D) explicitly is the default (same arithmetic up to one rounding of the factor);
    another factor gives another answer; a huge factor tends to the hard maximum (one-hot weights)."""
    (S, B, C, Q) = (4, 5, 10, 2)
    L = S + C + Q
    Hq, Hkv, D, base = 2, 2, 16, 1.0e4
    lay = make_layout(oracle, [(S, B, C, Q)])
    q, k, v = rand_qkv(L, Hq, Hkv, D)
    a, la = oracle.forward(q, k, v, lay, base)
    b, lb = oracle.forward(q, k, v, lay, base, softmax_scale=1.0 / math.sqrt(D))
    assert np.max(np.abs(a - b)) <= 1e-14 and np.max(np.abs(la - lb)) <= 1e-14
    c, _ = oracle.forward(q, k, v, lay, base, softmax_scale=2.0 / math.sqrt(D))
    assert np.max(np.abs(a - c)) > 1e-3
    # scale -> large: every row returns the value of its best visible key
    posf = np.arange(L, dtype=np.float64)
    qr, kr = brute_rope_complex(q, posf, base), brute_rope_complex(k, posf, base)
    hard, _ = oracle.forward(q, k, v, lay, base, softmax_scale=1.0e4)
    i = L - 1  # a question row: all keys visible
    for h in range(Hq):
        best = int(np.argmax(kr[:, h] @ qr[i, h]))
        np.testing.assert_allclose(hard[i, h], v[best, h], atol=1e-9)


# ------------------------------------------------------------------ multimodal RoPE (three axes)
def brute_mrope_complex(x, pos3, section, base):
    """Independent evaluation: pair (i, i+D/2) as one complex number, turned by exp(j * angle), the
    angle taken from the axis whose consecutive section holds pair index i."""
    T, H, D = x.shape
    half = D // 2
    bounds = np.cumsum([0] + list(section))
    out = np.empty((T, H, D), dtype=np.float64)
    for t in range(T):
        for i in range(half):
            axis = [a for a in range(3) if bounds[a] <= i < bounds[a + 1]][0]
            w = cmath.exp(1j * float(pos3[axis][t]) * base ** (-2.0 * i / D))
            for h in range(H):
                z = complex(x[t, h, i], x[t, h, i + half]) * w
                out[t, h, i], out[t, h, i + half] = z.real, z.imag
    return out


def test_p11_mrope_against_brute_force_and_1d_rope(oracle):
    T, H, D, base = 11, 2, 16, 1.0e4
    x = RNG.standard_normal((T, H, D))
    pos3 = np.stack([RNG.integers(0, 3000, T), RNG.integers(0, 40, T), RNG.integers(0, 40, T)]).astype(np.int32)
    for section in [(2, 3, 3), (8, 0, 0), (0, 0, 8), (1, 6, 1), (3, 5, 0)]:
        y = oracle.rope_mrope(x, pos3, section, base)
        np.testing.assert_allclose(y, brute_mrope_complex(x, pos3, section, base), atol=1e-11, rtol=0)
    # three equal axes: the one-dimensional rotation (pinned above), bit for bit
    p = pos3[0]
    np.testing.assert_array_equal(oracle.rope_mrope(x, np.stack([p, p, p]), (2, 3, 3), base), oracle.rope(x, p, base))
    # rows subset
    rows = np.array([7, 0, 3], dtype=np.int64)
    np.testing.assert_array_equal(oracle.rope_mrope(x, pos3, (2, 3, 3), base, rows=rows),
                                  oracle.rope_mrope(x, pos3, (2, 3, 3), base)[rows])


def test_p11_mrope_axis_touches_only_its_section_and_is_relative_per_axis(oracle):
    T, H, D, base = 6, 2, 32, 1.0e6
    half, section = D // 2, (4, 6, 6)
    x = RNG.standard_normal((T, H, D))
    pos3 = np.stack([np.arange(T) + 5, np.arange(T) % 3, (np.arange(T) * 2) % 5]).astype(np.int32)
    y = oracle.rope_mrope(x, pos3, section, base)
    for axis, (lo, hi) in enumerate(((0, 4), (4, 10), (10, 16))):
        moved = pos3.copy()
        moved[axis] += 17
        z = oracle.rope_mrope(x, moved, section, base)
        idx = np.zeros(D, bool)
        idx[lo:hi] = True
        idx[half + lo:half + hi] = True
        np.testing.assert_array_equal(z[..., ~idx], y[..., ~idx])      # other sections untouched, exactly
        assert np.all(np.abs(z[..., idx] - y[..., idx]).max(axis=(1, 2)) > 1e-3)
    # pair norms kept; pair 0 (temporal) turns by exactly pos_t radians
    np.testing.assert_allclose(y[..., :half] ** 2 + y[..., half:] ** 2, x[..., :half] ** 2 + x[..., half:] ** 2, rtol=1e-13)
    th = float(pos3[0][2])
    np.testing.assert_allclose(y[2, :, 0], x[2, :, 0] * math.cos(th) - x[2, :, half] * math.sin(th), atol=1e-14)
    # first pair of the height section: frequency index continues (i = 4), it does not restart at 0
    th = float(pos3[1][4]) * base ** (-2.0 * 4 / D)
    np.testing.assert_allclose(y[4, :, 4], x[4, :, 4] * math.cos(th) - x[4, :, half + 4] * math.sin(th), atol=1e-14)
    # <R_m q, R_n k> depends on m - n per axis: shift both tokens by the same (dt, dh, dw)
    qv, kv = RNG.standard_normal((1, 1, D)), RNG.standard_normal((1, 1, D))
    dots = []
    for shift in ((0, 0, 0), (900, 3, 11), (50000, 20, 0)):
        pq = np.array([[10 + shift[0]], [2 + shift[1]], [7 + shift[2]]], np.int32)
        pk = np.array([[4 + shift[0]], [5 + shift[1]], [1 + shift[2]]], np.int32)
        dots.append(float(np.sum(oracle.rope_mrope(qv, pq, section, base) * oracle.rope_mrope(kv, pk, section, base))))
    assert max(dots) - min(dots) <= 1e-9


def test_p11_mrope_position_ids_of_a_video_prompt():
    """The input recipe: text counts on all axes, frames share a temporal id per frame and walk the
    grid on the other two, the counter resumes after the largest id, nothing restarts per block."""
    import workloads as W
    w = W.Workload("m", 9, "f32", 2, 1, 16, 1.0e4, [(10, 8, 20, 3), (2, 4, 5, 2)], 1.0)
    ids = W.mrope_position_ids(w, frame_tokens=6, grid_w=3)
    # sequence 0: 4 text tokens, then 26 video tokens = 4 frames of 2x3 + 2 tokens, then 3 text tokens
    np.testing.assert_array_equal(ids[:, :4], np.tile(np.arange(4), (3, 1)))
    np.testing.assert_array_equal(ids[0, 4:30], 4 + np.arange(26) // 6)
    np.testing.assert_array_equal(ids[1, 4:30], 4 + (np.arange(26) % 6) // 3)
    np.testing.assert_array_equal(ids[2, 4:30], 4 + (np.arange(26) % 6) % 3)
    np.testing.assert_array_equal(ids[:, 30:33], np.tile(9 + np.arange(3), (3, 1)))  # largest id was 4 + 4
    # sequence 1 (sink shorter than a frame: all text) starts again from 0
    np.testing.assert_array_equal(ids[:, 33:35], np.tile(np.arange(2), (3, 1)))
    np.testing.assert_array_equal(ids[0, 35:40], 2 + np.arange(5) // 6)
    np.testing.assert_array_equal(ids[2, 35:40], 2 + np.arange(5) % 3)
    np.testing.assert_array_equal(ids[:, 40:42], np.tile(5 + np.arange(2), (3, 1)))  # largest id was 2 + 2 (column)


# ------------------------------------------------------------------ sliding window for the question
def make_window_layout(oracle, seqs, windows):
    lens = [s + c + q for (s, b, c, q) in seqs]
    cu = np.concatenate([[0], np.cumsum(lens)])
    a = np.asarray(seqs).reshape(-1, 4)
    return oracle.Layout(cu, a[:, 0], a[:, 1], a[:, 2], a[:, 3], window_blocks=windows)


@pytest.mark.parametrize("seqs,windows", [
    ([(3, 4, 14, 5)], [2]), ([(3, 4, 14, 5)], [0]), ([(0, 5, 15, 4)], [1]), ([(6, 3, 9, 2)], [9]),
    ([(2, 4, 9, 3), (5, 2, 8, 0), (1, 3, 3, 4)], [1, 0, -1]),
])
def test_p12_window_mask_against_explicit_rule(oracle, seqs, windows):
    """Mask matrix with a window, entry by entry, against the rule written out here: rows outside the
    question are unchanged; a question row keeps a context key only if its block is among the last W."""
    lay_w = make_window_layout(oracle, seqs, windows)
    lay = make_layout(oracle, seqs)
    Mw, M = oracle.mask_matrix(lay_w), oracle.mask_matrix(lay)
    t0 = 0
    for (S, B, C, Q), W_ in zip(seqs, windows):
        L = S + C + Q
        n_blocks = -(-C // B) if C else 0
        for i in range(L):
            for j in range(L):
                want = int(M[t0 + i, t0 + j])
                if W_ >= 0 and i >= S + C and S <= j < S + C and (j - S) // B < n_blocks - W_:
                    want = 0
                assert int(Mw[t0 + i, t0 + j]) == want, (i, j)
        # nothing leaks across sequences either
        assert not Mw[t0:t0 + L, :t0].any() and not Mw[t0:t0 + L, t0 + L:].any()
        t0 += L


@pytest.mark.parametrize("S,B,C,Q,W_", [(6, 4, 14, 5, 2), (0, 5, 15, 4, 1), (7, 3, 9, 3, 0), (4, 8, 20, 6, 1)])
def test_p12_windowed_question_equals_causal_attention_over_kept_keys(oracle, S, B, C, Q, W_):
    """Question rows under a window = the last Q rows of ordinary causal attention (torch CPU) over
    [sink ; last W blocks ; question], every token rotated at its ORIGINAL position.  Sink and
    context rows are those of the method without a window."""
    Hq, Hkv, D, base = 4, 2, 16, 1.0e4
    L = S + C + Q
    lay_w = make_window_layout(oracle, [(S, B, C, Q)], [W_])
    q, k, v = rand_qkv(L, Hq, Hkv, D)
    got, _ = oracle.forward(q, k, v, lay_w, base)
    plain, _ = oracle.forward(q, k, v, make_layout(oracle, [(S, B, C, Q)]), base)
    np.testing.assert_array_equal(got[:S + C], plain[:S + C])
    pos = np.arange(L, dtype=np.float64)
    qr, kr = brute_rope_complex(q, pos, base), brute_rope_complex(k, pos, base)
    n_blocks = -(-C // B)
    first_kept = max(0, n_blocks - W_)
    idx = np.r_[0:S, S + first_kept * B:S + C, S + C:L]
    np.testing.assert_allclose(got[S + C:], sdpa_last_rows(qr[idx], kr[idx], v[idx], Q, Hq, Hkv), atol=1e-10, rtol=0)
    # a window that covers every block changes nothing; lse of a windowed row is never larger
    full, lse_full = oracle.forward(q, k, v, make_window_layout(oracle, [(S, B, C, Q)], [n_blocks]), base)
    np.testing.assert_array_equal(full, plain)
    _, lse_w = oracle.forward(q, k, v, lay_w, base)
    assert np.all(lse_w[S + C:] <= lse_full[S + C:] + 1e-12)


# ------------------------------------------------------------------ log-sum-exp merge identity
def test_p8_lse_merge_identity(oracle):
    seqs = [(6, 7, 20, 5)]
    lay = make_layout(oracle, seqs)
    T = lay.total_tokens
    Hq, Hkv, D = 4, 2, 8
    q, k, v = rand_qkv(T, Hq, Hkv, D)
    pos = oracle.positions(lay)
    kr, qr = oracle.rope(k, pos, 1.0e4), oracle.rope(q, pos, 1.0e4)
    whole, lse = oracle.attn(qr, kr, v, lay)
    for cuts in ([0, 9, T], [0, 3, 4, 17, 30, T], [0, T - 1, T]):
        parts = [oracle.attn(qr, kr, v, lay, key_range=(a, b)) for a, b in zip(cuts[:-1], cuts[1:])]
        lses = np.stack([p[1] for p in parts])                    # [n_parts, T, Hq]
        mx = lses.max(0)
        wts = np.exp(lses - mx)                                   # exp(-inf) = 0 for empty parts
        merged = sum(w[..., None] * p[0] for w, p in zip(wts, parts)) / wts.sum(0)[..., None]
        np.testing.assert_allclose(merged, whole, atol=1e-12, rtol=0)
        np.testing.assert_allclose(mx + np.log(wts.sum(0)), lse, atol=1e-12, rtol=0)
    # lse against its definition through brute scores on one row
    t, h = T - 1, 1
    s = np.array([np.dot(qr[t, h], kr[j, h // 2]) / math.sqrt(D) for j in range(T)])
    assert abs(lse[t, h] - (s.max() + math.log(np.exp(s - s.max()).sum()))) <= 1e-12


# ------------------------------------------------------------------ sequential vs re-based positions
def test_p9_sequential_positions_are_not_rebased(oracle):
    S, B, C, Q = 4, 6, 18, 3
    lay = make_layout(oracle, [(S, B, C, Q)])
    L = S + C + Q
    q, k, v = rand_qkv(L, 2, 1, 16)
    seq, _ = oracle.forward(q, k, v, lay, 1.0e4)
    assert np.array_equal(oracle.positions(lay), np.arange(L))
    rebased = np.arange(L, dtype=np.int32)
    for b in range(C // B):
        rebased[S + b * B:S + (b + 1) * B] = S + np.arange(B)     # every block restarts after the sink
    rb, _ = oracle.forward(q, k, v, lay, 1.0e4, pos=rebased)
    np.testing.assert_allclose(rb[:S + B], seq[:S + B], atol=1e-12)  # sink and first block unchanged
    assert np.max(np.abs(rb[S + B:S + C] - seq[S + B:S + C])) > 1e-3  # later blocks differ
    # without a sink only relative positions inside a block matter: re-basing changes nothing there
    lay0 = make_layout(oracle, [(0, B, C, 0)])
    a, _ = oracle.forward(q[:C], k[:C], v[:C], lay0, 1.0e4)
    rb0 = np.tile(np.arange(B, dtype=np.int32), C // B)
    b, _ = oracle.forward(q[:C], k[:C], v[:C], lay0, 1.0e4, pos=rb0)
    np.testing.assert_allclose(a, b, atol=1e-9)


def test_p10_cost_model_brackets_reported_speedup():
    """Pair-count ratio full / PEVLM at the paper's own performance setting (about 100k tokens,
    sink = block = 16 frames ~ 4096 tokens) sits above the attention speedups it reports
    (7.47x-7.79x at that setting), as a cost model that ignores fixed overheads should."""
    S = B = 4096
    N, Q = 23, 64
    L = S + N * B + Q
    ratio = L * L / eq10_pairs(S, B, N, Q)
    assert 7.79 < ratio < 20


def test_layout_check(oracle):
    assert oracle.check_layout(make_layout(oracle, [(3, 2, 6, 4)])) == 0
    bad = oracle.Layout([0, 10], [3], [2], [6], [4])
    assert oracle.check_layout(bad) != 0
    assert oracle.check_layout(oracle.Layout([0, 5], [3], [0], [2], [0])) != 0


def test_gqa_head_map(oracle):
    lay = make_layout(oracle, [(2, 3, 6, 2)])
    q, k, v = rand_qkv(lay.total_tokens, 4, 2, 4)
    a, _ = oracle.forward(q, k, v, lay, 1.0e4)
    b, _ = oracle.forward(q, k, v, lay, 1.0e4, kv_head_of_q=[0, 0, 1, 1])
    assert np.array_equal(a, b)
    c, _ = oracle.forward(q, k, v, lay, 1.0e4, kv_head_of_q=[1, 0, 1, 0])
    d, _ = oracle.forward(q[:, [1, 0, 3, 2]], k, v, lay, 1.0e4, kv_head_of_q=[0, 1, 0, 1])
    np.testing.assert_allclose(c, d[:, [1, 0, 3, 2]], atol=1e-14)
