"""Host-side logic of libpevlm that needs no GPU: exported symbols, argument validation, the
tile work lists (expanded back to a boolean mask and compared with the oracle's explicit mask),
and the closed-form pair counts."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2506_19651_amd as P

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    lib = P.load_library()
    header = open(os.path.join(ROOT, "include", "pevlm.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    names = set(re.findall(r"\b(pevlm_[a-z_0-9]+)\s*\(", header))
    assert {"pevlm_rope_seq", "pevlm_block_prefill_attn", "pevlm_query_attn"} <= names
    for n in sorted(names):
        assert hasattr(lib, n), f"{n} declared in include/pevlm.h but not exported"
    assert P.pevlm_version() >= 100


LAYOUTS = [
    [(0, 1, 0, 1)],
    [(3, 2, 6, 4)],
    [(1, 5, 13, 0)],
    [(0, 2, 6, 1)],
    [(4, 5, 0, 4)],
    [(300, 392, 1000, 70)],
    [(256, 128, 1024, 64)],
    [(130, 200, 777, 129), (0, 64, 320, 5), (17, 1000, 250, 0), (5, 3, 0, 200)],
]


def expand_items(items, T):
    M = np.zeros((T, T), np.uint8)
    owner = np.zeros(T, np.int32)
    for it in items:
        assert it.q_rows >= 1
        for r in range(it.q_start, it.q_start + it.q_rows):
            owner[r] += 1
            M[r, it.full_start:it.full_start + it.full_len] += 1
            hi = min(it.diag_start + it.diag_len, r + 1)
            if hi > it.diag_start:
                M[r, it.diag_start:hi] += 1
    return M, owner


@pytest.mark.parametrize("seqs", LAYOUTS)
@pytest.mark.parametrize("tile_rows", [1, 16, 128, 256])
def test_prefill_worklist_expands_to_oracle_mask(oracle, seqs, tile_rows):
    lay = P.Layout.from_seqs(seqs)
    T = lay.total_tokens
    olay = oracle.Layout(lay.cu, lay.s, lay.b, lay.c, lay.q)
    want = oracle.mask_matrix(olay)
    items = P.pevlm_prefill_worklist_host(lay, tile_rows)
    got, owner = expand_items(items, T)
    is_question = np.zeros(T, bool)
    for si, (S, B, C, Q) in enumerate(seqs):
        is_question[lay.cu[si] + S + C: lay.cu[si + 1]] = True
    assert np.all(owner[~is_question] == 1) and np.all(owner[is_question] == 0)  # each row exactly once
    assert np.array_equal(got[~is_question], want[~is_question])                 # and exactly its keys, once
    for it in items:  # a tile never leaves its region and never exceeds the tile size
        assert it.q_rows <= tile_rows
    n_expected = 0
    for (S, B, C, Q) in seqs:
        n_expected += -(-S // tile_rows)
        nb = -(-C // B) if C else 0
        for b in range(nb):
            n_expected += -(-min(B, C - b * B) // tile_rows)
    assert len(items) == n_expected


def expand_stream_items(items, T, Hq):
    """cover[row, head] = how many slots own it; M[head][row, key] = how often the key is offered to the row."""
    cover = np.zeros((T, Hq), np.int32)
    M = np.zeros((Hq, T, T), np.uint8)
    for it in items:
        assert it.n_full_tiles == -(-it.full_len // 64) and it.n_tiles == it.n_full_tiles + -(-it.diag_len // 64)
        assert it.n_tiles >= 1
        used = [sl for sl in it.slot if sl.q_rows > 0]
        assert used and all(1 <= sl.q_rows <= 32 for sl in used)
        # the item's diagonal range reaches exactly its last row
        assert it.diag_start + it.diag_len == max(sl.q_start + sl.q_rows for sl in used)
        for sl in used:
            for r in range(sl.q_start, sl.q_start + sl.q_rows):
                cover[r, sl.head] += 1
                M[sl.head, r, it.full_start:it.full_start + it.full_len] += 1
                hi = min(it.diag_start + it.diag_len, r + 1)
                assert hi > it.diag_start
                M[sl.head, r, it.diag_start:hi] += 1
    return cover, M


STREAM_HEADS = [(4, 2, None), (7, 1, None), (8, 2, [1, 0, 0, 1, 1, 0, 1, 0]), (3, 3, None)]


@pytest.mark.parametrize("seqs", LAYOUTS)
@pytest.mark.parametrize("Hq,Hkv,hmap", STREAM_HEADS)
def test_stream_items_expand_to_oracle_mask(oracle, seqs, Hq, Hkv, hmap):
    lay = P.Layout.from_seqs(seqs)
    heads = P.Heads(Hq, Hkv, 128, "bf16", hmap)
    T = lay.total_tokens
    olay = oracle.Layout(lay.cu, lay.s, lay.b, lay.c, lay.q)
    want = oracle.mask_matrix(olay)
    items = P.pevlm_prefill_stream_items_host(lay, heads)
    cover, M = expand_stream_items(items, T, Hq)
    G = Hq // Hkv
    kv = hmap if hmap is not None else [h // G for h in range(Hq)]
    for it in items:
        assert all(kv[sl.head] == it.kv_head for sl in it.slot if sl.q_rows > 0)
    t0 = 0
    for (S, B, C, Q) in seqs:
        assert np.all(cover[t0:t0 + S + C] == 1) and np.all(cover[t0 + S + C:t0 + S + C + Q] == 0)
        for h in range(Hq):
            assert np.array_equal(M[h, t0:t0 + S + C], want[t0:t0 + S + C])
        t0 += S + C + Q


def test_stream_items_of_a_block_selection_and_unequal_groups():
    seqs = [(70, 100, 350, 9), (0, 33, 99, 0)]
    lay = P.Layout.from_seqs(seqs)
    heads = P.Heads(4, 2, 128, "bf16")
    full = P.pevlm_prefill_stream_items_host(lay, heads)
    key = lambda it: (it.seq, it.diag_start, it.kv_head, it.slot[0].q_start, it.slot[0].head)
    sel = P.pevlm_prefill_stream_items_host(lay, heads, [1, 0], [3, 2], with_sink=False)
    fullmap = {key(it): bytes(it) for it in full}
    assert len(sel) > 0 and all(fullmap[key(it)] == bytes(it) for it in sel)
    rows = sorted({r for it in sel for sl in it.slot if sl.q_rows for r in range(sl.q_start, sl.q_start + sl.q_rows)})
    assert rows == list(range(70 + 100, 70 + 350)) + list(range(429, 429 + 66))
    # unequal groups per KV head, fp32 tensors, short lists: the one-item kernel is used instead
    uneven = P.Heads(4, 2, 128, "bf16", [0, 0, 0, 1])
    with pytest.raises(P.PevlmError):
        P.pevlm_prefill_stream_items_host(lay, uneven)
    big = P.Layout.from_seqs([(256, 1024, 65536, 128)])
    prev = P.pevlm_set_prefill_kernel("auto")
    try:
        assert P.pevlm_prefill_uses_stream_kernel(big, P.Heads(28, 4, 128, "bf16"))
        assert not P.pevlm_prefill_uses_stream_kernel(big, P.Heads(28, 4, 128, "f32"))
        assert not P.pevlm_prefill_uses_stream_kernel(big, P.Heads(4, 2, 128, "bf16", [0, 0, 0, 1]))
        assert not P.pevlm_prefill_uses_stream_kernel(lay, heads)  # a few dozen items for 256 compute units
        assert P.pevlm_set_prefill_kernel("stream") == 0
        assert P.pevlm_prefill_uses_stream_kernel(lay, heads) and not P.pevlm_prefill_uses_stream_kernel(lay, uneven)
        assert P.pevlm_set_prefill_kernel("classic") == 2
        assert not P.pevlm_prefill_uses_stream_kernel(big, P.Heads(28, 4, 128, "bf16"))
        with pytest.raises(P.PevlmError):
            P.pevlm_set_prefill_kernel(7)
    finally:
        P.pevlm_set_prefill_kernel(prev)


@pytest.mark.parametrize("seqs", LAYOUTS)
@pytest.mark.parametrize("tile_rows,num_splits", [(16, 1), (16, 3), (128, 4), (128, 64), (1, 2)])
def test_query_worklist_expands_to_oracle_mask(oracle, seqs, tile_rows, num_splits):
    lay = P.Layout.from_seqs(seqs)
    T = lay.total_tokens
    olay = oracle.Layout(lay.cu, lay.s, lay.b, lay.c, lay.q)
    want = oracle.mask_matrix(olay)
    items = P.pevlm_query_worklist_host(lay, tile_rows, num_splits)
    got, owner = expand_items(items, T)
    total_q = sum(q for (_, _, _, q) in seqs)
    slots = set()
    for it in items:  # every (split, question row) owns a distinct slot of the partial buffers
        for r in range(it.q_rows):
            slot = it.reserved + r
            assert 0 <= slot < num_splits * total_q and slot not in slots
            slots.add(slot)
    assert len(slots) == num_splits * total_q
    for si, (S, B, C, Q) in enumerate(seqs):
        lo, hi = lay.cu[si] + S + C, lay.cu[si + 1]
        assert np.all(owner[lo:hi] == num_splits)
        assert np.array_equal(got[lo:hi], want[lo:hi])  # splits partition each row's keys exactly
        assert np.all(got[lay.cu[si]:lo] == 0)


STREAM_LAYOUTS = [
    [(3, 2, 6, 4)],
    [(0, 5, 13, 3)],
    [(300, 392, 1000, 70)],
    [(130, 200, 777, 129), (0, 64, 320, 5), (17, 1000, 250, 0), (5, 3, 0, 200)],
]


@pytest.mark.parametrize("seqs", STREAM_LAYOUTS)
@pytest.mark.parametrize("tile_rows", [1, 16, 128])
def test_block_range_worklist_is_the_matching_slice_of_the_mask(oracle, seqs, tile_rows):
    """Items of a block range cover exactly the rows of those blocks (and the sink if asked), each
    once, with exactly the keys the oracle's mask gives those rows."""
    lay = P.Layout.from_seqs(seqs)
    T = lay.total_tokens
    want = oracle.mask_matrix(oracle.Layout(lay.cu, lay.s, lay.b, lay.c, lay.q))
    rng = np.random.default_rng(len(seqs) * 100 + tile_rows)
    for with_sink in (False, True):
        first, count = [], []
        for (S, B, C, Q) in seqs:
            nb = -(-C // B) if C else 0
            f = int(rng.integers(0, nb + 1))
            first.append(f)
            count.append(int(rng.integers(0, nb - f + 1)))
        items = P.pevlm_prefill_worklist_blocks_host(lay, tile_rows, first, count, with_sink)
        got, owner = expand_items(items, T) if items else (np.zeros((T, T), np.uint8), np.zeros(T, np.int32))
        selected = np.zeros(T, bool)
        for si, (S, B, C, Q) in enumerate(seqs):
            b0 = lay.cu[si]
            if with_sink:
                selected[b0:b0 + S] = True
            lo = b0 + S + first[si] * B
            hi = min(b0 + S + C, b0 + S + (first[si] + count[si]) * B)
            selected[lo:hi] = True
        assert np.array_equal(owner, selected.astype(np.int32))
        assert np.array_equal(got[selected], want[selected]) and not got[~selected].any()
    # the whole range is the plain work list
    nb_all = [(-(-C // B) if C else 0) for (S, B, C, Q) in seqs]
    full = P.pevlm_prefill_worklist_blocks_host(lay, tile_rows, [0] * len(seqs), nb_all, True)
    plain = P.pevlm_prefill_worklist_host(lay, tile_rows)
    as_rows = lambda its: [[getattr(it, f) for f, _ in P.WorkItem._fields_] for it in its]
    assert as_rows(full) == as_rows(plain)
    with pytest.raises(P.PevlmError):
        P.pevlm_prefill_worklist_blocks_host(lay, tile_rows, [0] * len(seqs), [n + 1 for n in nb_all], True)


@pytest.mark.parametrize("seqs", STREAM_LAYOUTS)
@pytest.mark.parametrize("tile_rows,num_splits", [(16, 2), (16, 5), (128, 3), (1, 2)])
def test_window_worklist_expands_to_oracle_window_mask(oracle, seqs, tile_rows, num_splits):
    lay = P.Layout.from_seqs(seqs)
    T = lay.total_tokens
    rng = np.random.default_rng(num_splits * 7 + tile_rows)
    for trial in range(3):
        windows = []
        for (S, B, C, Q) in seqs:
            nb = -(-C // B) if C else 0
            windows.append(int(rng.integers(-1, nb + 2)))
        want = oracle.mask_matrix(oracle.Layout(lay.cu, lay.s, lay.b, lay.c, lay.q, window_blocks=windows))
        items = P.pevlm_query_worklist_window_host(lay, tile_rows, num_splits, windows)
        got, owner = expand_items_allow_empty(items, T)
        total_q = sum(q for (_, _, _, q) in seqs)
        slots = set()
        for it in items:
            for r in range(it.q_rows):
                slot = it.reserved + r
                assert 0 <= slot < num_splits * total_q and slot not in slots
                slots.add(slot)
        assert len(slots) == num_splits * total_q
        for si, (S, B, C, Q) in enumerate(seqs):
            lo, hi = lay.cu[si] + S + C, lay.cu[si + 1]
            assert np.all(owner[lo:hi] == num_splits)
            assert np.array_equal(got[lo:hi], want[lo:hi])
            assert np.all(got[lay.cu[si]:lo] == 0)


def expand_items_allow_empty(items, T):
    return expand_items(items, T) if items else (np.zeros((T, T), np.uint8), np.zeros(T, np.int32))


def test_visible_pairs_match_oracle_mask_and_golden(oracle):
    for seqs in LAYOUTS:
        lay = P.Layout.from_seqs(seqs)
        olay = oracle.Layout(lay.cu, lay.s, lay.b, lay.c, lay.q)
        M = oracle.mask_matrix(olay)
        sums = [0, 0, 0]
        for si, (S, B, C, Q) in enumerate(seqs):
            b = lay.cu[si]
            sums[0] += int(M[b:b + S].sum())
            sums[1] += int(M[b + S:b + S + C].sum())
            sums[2] += int(M[b + S + C:b + S + C + Q].sum())
        assert P.pevlm_visible_pairs(lay) == tuple(sums)
    golden = {}
    for line in open(os.path.join(ROOT, "tests", "golden", "pair_counts.txt")):
        if line.strip() and not line.startswith("#"):
            n, a, b, c = line.split()
            golden[n] = (int(a), int(b), int(c))
    import workloads as W
    for name, want in golden.items():
        w = W.CONFIGS[name]
        assert P.pevlm_visible_pairs(P.Layout.from_seqs(w.seqs)) == want
    # headline config: useful FLOPs of the block-prefill path
    w = W.CONFIGS["c3"]
    pre, que = P.useful_flops(P.Layout.from_seqs(w.seqs), P.Heads(28, 4, 128, "bf16"))
    assert pre == 4 * 128 * 28 * (32896 + 50364416) and que == 4 * 128 * 28 * 8429632


def test_argument_validation_without_gpu():
    """Invalid arguments are rejected before anything touches the device."""
    lib = P.load_library()
    lay = P.Layout.from_seqs([(3, 2, 6, 4)])
    heads = P.Heads(4, 2, 64, "f32")
    fake = ctypes.c_void_p(0x1000)  # aligned, never dereferenced on these paths
    call = lambda l, h, q=fake: lib.pevlm_block_prefill_attn(q, fake, fake, fake, None, l.ref(), h.ref(), None, 0, None)
    bad_sum = P.Layout([0, 10], [3], [2], [6], [4])
    assert call(bad_sum, heads) == P.binding.PEVLM_ERR_INVALID_ARG and "sink+ctx+query" in P.pevlm_last_error()
    assert call(P.Layout([0, 13], [3], [0], [6], [4]), heads) == P.binding.PEVLM_ERR_INVALID_ARG
    assert call(P.Layout([0, 5], [-1], [2], [2], [4]), heads) == P.binding.PEVLM_ERR_INVALID_ARG
    assert call(lay, P.Heads(4, 3, 64, "f32")) == P.binding.PEVLM_ERR_INVALID_ARG
    assert call(lay, P.Heads(4, 2, 64, "f32", kv_head_of_q=[0, 1, 2, 0])) == P.binding.PEVLM_ERR_INVALID_ARG
    assert call(lay, P.Heads(4, 2, 96, "f32")) == P.binding.PEVLM_ERR_UNSUPPORTED
    assert call(lay, P.Heads(4, 2, 64, 7)) == P.binding.PEVLM_ERR_UNSUPPORTED
    assert call(lay, heads, None) == P.binding.PEVLM_ERR_INVALID_ARG
    assert call(lay, heads, ctypes.c_void_p(0x1004)) == P.binding.PEVLM_ERR_INVALID_ARG
    assert call(lay, heads) == P.binding.PEVLM_ERR_WORKSPACE_TOO_SMALL
    assert "workspace" in P.pevlm_last_error()
    q = lambda ns: lib.pevlm_query_attn(fake, fake, fake, fake, None, lay.ref(), heads.ref(), ns, None, 0, None)
    assert q(-1) == P.binding.PEVLM_ERR_INVALID_ARG and q(65) == P.binding.PEVLM_ERR_INVALID_ARG
    assert q(0) == P.binding.PEVLM_ERR_WORKSPACE_TOO_SMALL
    assert lib.pevlm_rope_seq(fake, fake, lay.ref(), heads.ref(), -1.0, None, None) == P.binding.PEVLM_ERR_INVALID_ARG
    sec = lambda *v: (ctypes.c_int32 * 3)(*v)
    mr = lambda n, section, ids=fake, base=1e4: lib.pevlm_rope_mrope(fake, fake, n, heads.ref(), base, ids, section, None)
    assert mr(10, sec(8, 12, 11)) == P.binding.PEVLM_ERR_INVALID_ARG and "section" in P.pevlm_last_error()
    assert mr(10, sec(-1, 21, 12)) == P.binding.PEVLM_ERR_INVALID_ARG
    assert mr(10, None) == P.binding.PEVLM_ERR_INVALID_ARG
    assert mr(10, sec(8, 12, 12), None) == P.binding.PEVLM_ERR_INVALID_ARG
    assert mr(-1, sec(8, 12, 12)) == P.binding.PEVLM_ERR_INVALID_ARG
    assert mr(10, sec(8, 12, 12), fake, 0.0) == P.binding.PEVLM_ERR_INVALID_ARG
    assert mr(0, sec(8, 12, 12)) == P.binding.PEVLM_OK  # nothing to do, nothing launched
    assert P.pevlm_block_prefill_workspace_bytes(bad_sum, heads) == 0
    assert P.pevlm_query_workspace_bytes(lay, heads, 0) > 0


def test_workspace_sizes_cover_items_and_partials():
    lay = P.Layout.from_seqs([(256, 1024, 65536, 128)])
    heads = P.Heads(28, 4, 128, "bf16")
    n = len(P.pevlm_prefill_worklist_host(lay, P.pevlm_prefill_tile_rows(heads)))
    assert P.pevlm_block_prefill_workspace_bytes(lay, heads) >= n * ctypes.sizeof(P.WorkItem)
    for ns in (1, 8, 64):
        need = ns * 128 * 28 * (128 + 2) * 4 + 128 * 4 + ns * ctypes.sizeof(P.WorkItem)
        assert P.pevlm_query_workspace_bytes(lay, heads, ns) >= need


def test_time_model_tracks_measured_runs_and_sink_block_choice():
    """The model against the measured grid kept under profiles/ (product timings, not oracle values),
    then the choosers: feasibility under a cap, preference for the most visible pairs."""
    from paper_2506_19651_amd.cost_model import (choose_block_len, choose_sink_and_block, predict_block_prefill_ms,
                                                 prefill_work, stream_work, video_layout)
    prev = P.pevlm_set_prefill_kernel("auto")
    try:
        n = 0
        for line in open(os.path.join(ROOT, "profiles", "block_prefill_sweep.md")):
            f = line.split()
            if len(f) != 7 or f[0] not in ("q7b", "g32"):
                continue
            S, B, C, Q, ms, stream = int(f[1]), int(f[2]), int(f[3]), int(f[4]), float(f[5]), int(f[6])
            heads = P.Heads(28, 4, 128, "bf16") if f[0] == "q7b" else P.Heads(32, 8, 128, "bf16")
            lay = P.Layout.from_seqs([(S, B, C, Q)])
            assert int(P.pevlm_prefill_uses_stream_kernel(lay, heads)) == stream
            pred = predict_block_prefill_ms(lay, heads)
            assert abs(pred / ms - 1.0) <= 0.12, (line, pred)
            n += 1
        assert n >= 30
        # work of the headline config under both kernels
        lay3, h3 = P.Layout.from_seqs([(256, 1024, 65536, 128)]), P.Heads(28, 4, 128, "bf16")
        assert prefill_work(lay3, h3)[0] == 514 * 28
        cnt, til = stream_work(lay3, h3)
        assert len(cnt) == 256 and cnt.sum() == (7 + 64 * 28) * 4 and 28 <= cnt.min() <= cnt.max() <= 29
        # one knob: block-length sweep of the 100K-token configuration (2/4/8/16 frames of 196 tokens)
        heads = P.Heads(32, 8, 128, "bf16")
        pick = lambda cap: choose_block_len(392, 100352, 256, heads, [392, 784, 1568, 3136], cap)
        assert pick(1.0) is None
        assert pick(1.8)[0] == 784 and pick(2.5)[0] == 1568 and pick(10.0)[0] == 3136
        # both knobs: 256 frames of 256 tokens behind a 64-token prefix
        assert video_layout(64, 256, 256, 128, 2, 4) == (64 + 512, 1024, 254 * 256, 128)
        best, table = choose_sink_and_block(64, 256, 256, 128, h3, [1, 2, 4, 8, 16], [2, 4, 8, 16], 1.5)
        assert len(table) == 20 and best is not None and best[2] <= 1.5
        feasible = [r for r in table if r[2] <= 1.5]
        assert best[3] == max(r[3] for r in feasible)            # most visible pairs within the cap
        assert any(r[2] > 1.5 and r[3] > best[3] for r in table)  # and something better was too slow
        assert choose_sink_and_block(64, 256, 256, 128, h3, [1, 2], [2, 4], 0.2)[0] is None
        # the cost grows with either knob (Eq. 7 and Eq. 8 are quadratic in S and B)
        t = {(r[0], r[1]): r[2] for r in table}
        assert t[(1, 2)] < t[(1, 16)] and t[(1, 2)] < t[(16, 2)] and t[(4, 4)] < t[(8, 8)]
    finally:
        P.pevlm_set_prefill_kernel(prev)


def test_fp8_plan_offsets_and_counts():
    """Host side of the fp8 variant: the plan's counts equal the host enumerations, its parts are
    256-byte aligned, in order, large enough and do not overlap; unsupported dtypes are refused."""
    for (Hq, Hkv, D, seqs) in [(4, 2, 128, [(130, 200, 777, 9), (0, 64, 320, 5), (17, 100, 250, 0)]),
                               (6, 3, 64, [(70, 33, 150, 4), (5, 64, 64, 0)]), (28, 4, 128, [(256, 1024, 65536, 128)])]:
        lay = P.Layout.from_seqs(seqs)
        heads = P.Heads(Hq, Hkv, D, "bf16")
        plan = P.pevlm_block_prefill_fp8_plan(lay, heads)
        T = sum(s + c + q for (s, b, c, q) in seqs)
        assert plan.n_items == len(P.pevlm_prefill_worklist_host(lay, 128))
        assert plan.n_key_tiles == len(P.pevlm_prefill_worklist_host(lay, 64))
        parts = [("items", plan.n_items * 32), ("key_tiles", plan.n_key_tiles * 32), ("kv_amax", 2 * Hkv * 4),
                 ("q_scales", T * Hq * 4), ("q_codes", T * Hq * D), ("k_tiles", plan.n_key_tiles * Hkv * 64 * D),
                 ("v_tiles", plan.n_key_tiles * Hkv * 64 * D)]
        end = 0
        for name, size in parts:
            off = getattr(plan, name)
            assert off % 256 == 0 and off >= end, name
            end = off + size
        assert end <= plan.total - 256 and plan.total == P.pevlm_block_prefill_fp8_workspace_bytes(lay, heads)
    with pytest.raises(P.PevlmError):
        P.pevlm_block_prefill_fp8_plan(P.Layout.from_seqs([(8, 8, 16, 0)]), P.Heads(2, 1, 64, "f32"))
    assert P.pevlm_block_prefill_fp8_workspace_bytes(P.Layout.from_seqs([(8, 8, 16, 0)]), P.Heads(2, 1, 64, "f32")) == 0

