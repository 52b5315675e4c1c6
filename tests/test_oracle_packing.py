"""Pins for the packing / work-list oracle: closed cases of first-fit, a replay
proof of the first-fit rule, brute-force coverage of the work lists and
closed-form item counts."""
import numpy as np
import pytest

from oracle import packing as op


def test_first_fit_closed_cases():
    b, p, n = op.first_fit([25] * 12, 100)           # exactly 4 per bin
    assert n == 3 and list(b) == [0] * 4 + [1] * 4 + [2] * 4 and list(p) == [0, 1, 2, 3] * 3
    b, p, n = op.first_fit([100] * 5, 100)           # one per bin
    assert n == 5 and list(b) == [0, 1, 2, 3, 4] and list(p) == [0] * 5
    # textbook first-fit example: 60 40 | 70 30 ... small items fall back into early bins
    b, p, n = op.first_fit([60, 70, 40, 30, 50, 50], 100)
    assert list(b) == [0, 1, 0, 1, 2, 2] and list(p) == [0, 0, 1, 1, 0, 1] and n == 3
    b, p, n = op.first_fit([0, 0, 7], 7)             # zero-length samples are legal
    assert list(b) == [0, 0, 0] and n == 1
    with pytest.raises(ValueError):
        op.first_fit([5, 11], 10)


def test_first_fit_replay_proof():
    r = np.random.default_rng(0)
    lens = r.integers(0, 400, size=300)
    budget = 1000
    b, p, n = op.first_fit(lens, budget)
    fill = np.zeros(n, dtype=np.int64)
    seen = np.zeros(n, dtype=np.int64)
    for i, L in enumerate(lens):
        # at arrival time the sample fits nowhere earlier and fits where placed
        assert all(fill[e] + L > budget for e in range(b[i]) if True)
        assert fill[b[i]] + L <= budget
        assert p[i] == seen[b[i]]
        fill[b[i]] += L
        seen[b[i]] += 1
    assert fill.sum() == lens.sum() and fill.max() <= budget
    # bins open in order: bin e+1 only exists once bin e is non-empty
    assert sorted(set(b.tolist())) == list(range(n))


def test_bin_layout():
    cu, pl, mx = op.bin_layout([3, 0, 5], [1, 0, 5])
    assert list(cu) == [0, 3, 3, 8] and list(pl) == [1, 0, 5] and mx == 5
    cu, pl, mx = op.bin_layout([], None)
    assert list(cu) == [0] and pl is None and mx == 0


@pytest.mark.parametrize("mode", [op.MASK_CAUSAL, op.MASK_PREFIX_BIDIR_SUFFIX, op.MASK_PREFIX_CAUSAL_SUFFIX])
@pytest.mark.parametrize("bm,bn", [(4, 4), (8, 4), (4, 8), (16, 8)])
def test_worklists_cover_every_allowed_pair_exactly_once(mode, bm, bn):
    lens = [1, 13, 0, 8, 21, 4]
    cu, _, _ = op.bin_layout(lens)
    prefix = None if mode == op.MASK_CAUSAL else np.array([0, 5, 0, 8, 9, 0], dtype=np.int32)
    want_pairs = sum(op.allowed_pairs(L, 0 if prefix is None else int(prefix[s]), mode) for s, L in enumerate(lens))
    for pass_id in (op.PASS_FWD, op.PASS_BWD_DKDV, op.PASS_BWD_DQ):
        items = op.build_worklist(cu, prefix, pass_id, bm, bn, mode)
        assert op.check_coverage(items, cu, prefix, pass_id, bm, bn, mode) == want_pairs
        work = items[:, 5] if pass_id != op.PASS_BWD_DKDV else items[:, 4]
        assert np.all(np.diff(work) <= 0)            # heaviest first
    # a planted defect is caught: dropping the last key tile of the heaviest item
    items = op.build_worklist(cu, prefix, op.PASS_FWD, bm, bn, mode)
    if items[0, 5] > 1:
        broken = items.copy()
        broken[0, 5] -= 1
        broken[0, 4] = min(broken[0, 4], broken[0, 5])
        with pytest.raises(AssertionError):
            op.check_coverage(broken, cu, prefix, op.PASS_FWD, bm, bn, mode)


@pytest.mark.parametrize("bm,bn", [(4, 4), (8, 4), (4, 8), (16, 8)])
def test_three_block_worklists_cover_every_allowed_pair_exactly_once(bm, bn):
    lens = [1, 13, 0, 8, 21, 4, 30]
    cu, _, _ = op.bin_layout(lens)
    ends = np.array([[0, 1], [5, 9], [0, 0], [8, 8], [0, 13], [0, 0], [11, 30]], dtype=np.int32)
    mode = op.MASK_THREE_BLOCK
    # pairs by block sizes a, b, c: a^2 + b (a + b) + c (a + b + c)
    want_pairs = sum(P * P + (P2 - P) * P2 + (L - P2) * L for L, (P, P2) in zip(lens, ends.tolist()))
    assert want_pairs == sum(op.allowed_pairs(L, P, mode, P2) for L, (P, P2) in zip(lens, ends.tolist()))
    for pass_id in (op.PASS_FWD, op.PASS_BWD_DKDV, op.PASS_BWD_DQ):
        items = op.build_worklist(cu, ends, pass_id, bm, bn, mode)
        assert op.check_coverage(items, cu, ends, pass_id, bm, bn, mode) == want_pairs
        assert np.all(items[:, 6] >= 0) and np.all(items[:, 5 if pass_id == op.PASS_BWD_DKDV else 3] >= items[:, 6])
    # a planted defect is caught: the second boundary of one sample moved by one row
    items = op.build_worklist(cu, ends, op.PASS_FWD, bm, bn, mode)
    wrong = ends.copy()
    wrong[1, 1] += 1
    with pytest.raises(AssertionError):
        op.check_coverage(items, cu, wrong, op.PASS_FWD, bm, bn, mode)


@pytest.mark.parametrize("bm,bn", [(4, 4), (8, 4), (4, 8), (16, 8)])
def test_sliding_window_worklists_cover_every_allowed_pair_exactly_once(bm, bn):
    lens = [1, 13, 0, 8, 21, 4, 30]
    cu, _, _ = op.bin_layout(lens)
    W = np.array([1, 5, 3, 8, 1, 100, 11], dtype=np.int32)
    mode = op.MASK_SLIDING_WINDOW
    # a band of width W under the diagonal: full rows W, the first W - 1 rows shorter
    want_pairs = sum(min(L, w) * (min(L, w) + 1) // 2 + max(0, L - w) * w for L, w in zip(lens, W.tolist()))
    assert want_pairs == sum(op.allowed_pairs(L, w, mode) for L, w in zip(lens, W.tolist()))
    for pass_id in (op.PASS_FWD, op.PASS_BWD_DKDV, op.PASS_BWD_DQ):
        items = op.build_worklist(cu, W, pass_id, bm, bn, mode)
        assert op.check_coverage(items, cu, W, pass_id, bm, bn, mode) == want_pairs
    # no item visits more tiles than the window can touch: ceil((rows + W - 1) / tile) + 1
    fwd = op.build_worklist(cu, W, op.PASS_FWD, bm, bn, mode)
    for q_row0, q_rows, c, _, n_full, n_tiles, w, L in fwd.tolist():
        first = max(0, q_row0 - c + 1 - w) // bn
        assert n_tiles - first <= -(-(q_rows + w - 1) // bn) + 1
    dk = op.build_worklist(cu, W, op.PASS_BWD_DKDV, bm, bn, mode)
    for kv_row0, kv_rows, c, qt_first, qt_count, _, w, L in dk.tolist():
        assert qt_first == (kv_row0 - c) // bm and qt_count <= -(-(kv_rows + w - 1) // bm) + 1
    # planted defects are caught: a window one wider than the lists were built for, and a dropped query tile
    wrong = W.copy()
    wrong[4] += 1
    with pytest.raises(AssertionError):
        op.check_coverage(fwd, cu, wrong, op.PASS_FWD, bm, bn, mode)
    broken = dk.copy()
    row = int(np.argmax(broken[:, 4]))
    if broken[row, 4] > 1:
        broken[row, 4] -= 1
        with pytest.raises(AssertionError):
            op.check_coverage(broken, cu, W, op.PASS_BWD_DKDV, bm, bn, mode)


def test_closed_form_counts_causal():
    # causal: items = sum ceil(L/bm); key tiles of the query tile starting at row r0 with `rows`
    # rows = ceil((r0 + rows) / bn); full tiles = floor((r0 + 1) / bn)
    lens = [37, 5, 64, 100]
    cu, _, _ = op.bin_layout(lens)
    bm, bn = 16, 8
    items = op.build_worklist(cu, None, op.PASS_FWD, bm, bn)
    assert len(items) == sum(-(-L // bm) for L in lens)
    for q_row0, q_rows, c, P2, n_full, n_tiles, P, L in items.tolist():
        r0 = q_row0 - c
        assert P2 == -1 and n_tiles == -(-(r0 + q_rows) // bn) and n_full == (r0 + 1) // bn and P == -1
    assert items[:, 5].sum() == sum(-(-min(L, (t + 1) * bm) // bn) for L in lens for t in range(-(-L // bm)))
    dk = op.build_worklist(cu, None, op.PASS_BWD_DKDV, bm, bn)
    assert len(dk) == sum(-(-L // bn) for L in lens)
    for kv_row0, kv_rows, c, qt_first, qt_count, _, P, L in dk.tolist():
        assert qt_first == (kv_row0 - c) // bm and qt_first + qt_count == -(-L // bm)


def test_closed_form_counts_prefix_lm():
    # prefix rows see exactly P keys, suffix rows see all L
    L, P, bm, bn = 50, 23, 8, 8
    cu, _, _ = op.bin_layout([L])
    items = op.build_worklist(cu, [P], op.PASS_FWD, bm, bn)
    by_row0 = {it[0]: it for it in items.tolist()}
    for t in range(-(-L // bm)):
        it = by_row0[t * bm]
        last_row = min(L, (t + 1) * bm) - 1
        first_row = t * bm
        want_len = P if last_row < P else L
        min_vis = P if first_row < P else L
        assert it[3] == -1 and it[5] == -(-want_len // bn) and it[4] == min_vis // bn and it[6] == P
    assert op.allowed_pairs(L, P, op.MASK_PREFIX_BIDIR_SUFFIX) == P * P + (L - P) * L
    assert op.allowed_pairs(L, P, op.MASK_CAUSAL) == L * (L + 1) // 2
    assert op.allowed_pairs(L, P, op.MASK_PREFIX_CAUSAL_SUFFIX) == P * P + sum(i + 1 for i in range(P, L))


def test_workload_bins_match_the_stored_summary():
    # tests/golden/workload_bins.json is written by tests/golden/make_workload_bins.py (oracle only).
    # Its token / sample / pair counts for the first bins were also derived independently when the
    # workloads were specified: vlm 30 samples / 16319 tokens, pi05 35 / 32227, longtail 87 / 65516
    # tokens with a longest sample of 3638, tiny 176 tokens and 6793 pairs.
    import json
    import os
    from paper_2603_11101_amd import workloads as wl
    with open(os.path.join(os.path.dirname(__file__), "golden", "workload_bins.json")) as f:
        gold = json.load(f)
    assert (gold["vlm"]["bin0_samples"], gold["vlm"]["bin0_tokens"]) == (30, 16319)
    assert (gold["pi05"]["bin0_samples"], gold["pi05"]["bin0_tokens"]) == (35, 32227)
    assert (gold["longtail"]["bin0_samples"], gold["longtail"]["bin0_tokens"], gold["longtail"]["bin0_max_len"]) == (87, 65516, 3638)
    assert (gold["tiny"]["bin0_tokens"], gold["tiny"]["bin0_pairs_per_head"]) == (176, 6793)
    for name, w in wl.WORKLOADS.items():
        lens, prefix = wl.sample_lengths(name)
        bin_of, pos, nb = op.first_fit(lens, w.budget)
        idx = op.bin_members(bin_of, pos, 0)
        g = gold[name]
        assert nb == g["num_bins"] and len(idx) == g["bin0_samples"]
        assert int(lens[idx].sum()) == g["bin0_tokens"] and int(lens[idx].max()) == g["bin0_max_len"]
