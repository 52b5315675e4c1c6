"""CPU-only tests of the built library: it loads, exports every symbol the
header declares, and its host-side integer work (first-fit packing, layout,
work lists, E4M3 quantiser) equals the oracle's bit for bit.  Device entry
points are only driven into their host-side validation errors here."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import e4m3 as oe
from oracle import packing as op
from paper_2603_11101_amd import binding as va
from paper_2603_11101_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "varlen_attn.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(va_\w+|varlen_attn_\w+)\s*\(", header))
    assert declared == set(va.EXPORTS)
    lib = ctypes.CDLL(va.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), name


def test_first_fit_and_layout_equal_oracle_on_every_workload():
    for name, w in wl.WORKLOADS.items():
        lens, prefix = wl.sample_lengths(name)
        b, p, n = va.va_pack_first_fit(lens, w.budget)
        ob, opos, on = op.first_fit(lens, w.budget)
        assert n == on and np.array_equal(b, ob) and np.array_equal(p, opos)
        for bin_id in (0, n - 1):
            idx = op.bin_members(ob, opos, bin_id)
            cu, pl, mx = va.va_bin_layout(lens[idx], None if prefix is None else prefix[idx])
            ocu, opl, omx = op.bin_layout(lens[idx], None if prefix is None else prefix[idx])
            assert np.array_equal(cu, ocu) and mx == omx and cu.dtype == np.int32
            assert (pl is None and opl is None) or np.array_equal(pl, opl)


def test_first_fit_random_and_edge_cases():
    r = np.random.default_rng(5)
    for trial in range(20):
        budget = int(r.integers(1, 500))
        lens = r.integers(0, budget + 1, size=int(r.integers(0, 200)))
        b, p, n = va.va_pack_first_fit(lens, budget)
        ob, opos, on = op.first_fit(lens, budget)
        assert n == on and np.array_equal(b, ob) and np.array_equal(p, opos)
    with pytest.raises(va.VarlenAttnError) as e:
        va.va_pack_first_fit([5, 11], 10)
    assert e.value.code == va.VA_ESIZE and "exceeds the budget" in str(e.value)
    with pytest.raises(va.VarlenAttnError) as e:
        va.va_pack_first_fit([5, -1], 10)
    assert e.value.code == va.VA_EINVAL
    with pytest.raises(va.VarlenAttnError) as e:
        va.va_bin_layout([5, 3], [2, 4])
    assert e.value.code == va.VA_EINVAL


HEADS = [(2, 2, 64), (16, 8, 128), (8, 1, 256), (4, 1, 64), (6, 2, 128), (4, 4, 80), (2, 1, 192)]


@pytest.mark.parametrize("mode", [va.VA_MASK_CAUSAL, va.VA_MASK_PREFIX_LM, va.VA_MASK_PREFIX_LM_CAUSAL, va.VA_MASK_THREE_BLOCK,
                                  va.VA_MASK_SLIDING_WINDOW])
@pytest.mark.parametrize("Hq,Hkv,D", HEADS)
def test_worklists_equal_oracle_and_cover(mode, Hq, Hkv, D):
    r = np.random.default_rng(Hq * 1000 + D + mode)
    lens = np.concatenate([[1, 0, 300, 129, 64, 17], r.integers(1, 260, size=5)]).astype(np.int32)
    cu, _, _ = va.va_bin_layout(lens)
    prefix = None if mode == va.VA_MASK_CAUSAL else np.array([int(r.integers(0, L + 1)) for L in lens], dtype=np.int32)
    if mode == va.VA_MASK_THREE_BLOCK:
        prefix = wl.random_block_ends(Hq * 1000 + D, lens)
        prefix[2], prefix[3], prefix[4] = (300, 300), (0, 0), (0, 64)    # one block only, three ways
    elif mode == va.VA_MASK_SLIDING_WINDOW:
        prefix = r.integers(1, 200, size=len(lens)).astype(np.int32)
        prefix[2], prefix[3], prefix[4] = 70, 1, 1000    # a band; self only; wider than the sample
    elif prefix is not None:
        prefix[2], prefix[3] = 300, 0    # degenerate: whole sample is prefix / no prefix at all
    for pass_id in (va.VA_PASS_FWD, va.VA_PASS_BWD_DKDV, va.VA_PASS_BWD_DQ):
        rows, cols = va.va_tile_shape(pass_id, D, Hq, Hkv)
        got = va.va_build_worklist(cu, prefix, mode, pass_id, D, Hq, Hkv)
        header, items = got[0], va.worklist_items(got)
        assert header[1] == pass_id and header[2] == rows and header[3] == cols and header[4] == D
        assert header[5] == mode and header[6] == len(items) and header[7] == cu[-1]
        # the schedule assigns every work (item x head chunk) to exactly one persistent workgroup
        table, ids = va.worklist_schedule(got)
        per_item = Hkv if pass_id == va.VA_PASS_BWD_DKDV else got[1, 2]
        assert got[1, 1] == len(items) * per_item and sorted(ids.tolist()) == list(range(len(ids)))
        assert table[0, 0] == 0 and np.array_equal(table[1:, 0], np.cumsum(table[:-1, 1])) and table[:, 1].sum() == len(ids)
        if pass_id == va.VA_PASS_BWD_DKDV:
            # one work per workgroup: the id array is the launch order, the item order unless the list says otherwise
            assert got[1, 3] in (0, 1) and (got[1, 3] == 1 or np.array_equal(ids, np.arange(len(ids))))
            assert got[1, 7] == 0 and np.all(items[:, 1] >> 8 == 0)       # few works per workgroup slot: nothing is split
        else:
            # longest-processing-time-first: no workgroup exceeds the mean load by more than the heaviest work
            steps = items[:, 5]
            if mode == va.VA_MASK_SLIDING_WINDOW:   # tiles below the window are not visited
                steps = items[:, 5] - np.maximum(0, items[:, 0] - items[:, 2] + 1 - items[:, 6]) // cols
            cost = np.repeat(steps, per_item) + 2
            loads = np.array([cost[ids[a:a + n]].sum() for a, n in table])
            assert loads.max() <= cost.sum() / len(table) + cost.max()
        # the oracle names tile sizes by role: bm = query rows, bn = key rows
        bm, bn = (cols, rows) if pass_id == va.VA_PASS_BWD_DKDV else (rows, cols)
        want = op.build_worklist(cu, prefix, pass_id, bm, bn, mode)
        assert np.array_equal(items, want)
    # brute-force coverage of the library's own lists on a smaller stream (quadratic check)
    small = np.array([1, 70, 33, 130], dtype=np.int32)
    cu_s, _, _ = va.va_bin_layout(small)
    pre_s = None if mode == va.VA_MASK_CAUSAL else np.array([1, 40, 0, 97], dtype=np.int32)
    if mode == va.VA_MASK_THREE_BLOCK:
        pre_s = np.array([[0, 1], [10, 40], [0, 0], [64, 97]], dtype=np.int32)
    if mode == va.VA_MASK_SLIDING_WINDOW:
        pre_s = np.array([3, 40, 1, 65], dtype=np.int32)
    for pass_id in (va.VA_PASS_FWD, va.VA_PASS_BWD_DKDV, va.VA_PASS_BWD_DQ):
        rows, cols = va.va_tile_shape(pass_id, D, Hq, Hkv)
        bm, bn = (cols, rows) if pass_id == va.VA_PASS_BWD_DKDV else (rows, cols)
        items = va.worklist_items(va.va_build_worklist(cu_s, pre_s, mode, pass_id, D, Hq, Hkv))
        op.check_coverage(items, cu_s, pre_s, pass_id, bm, bn, mode)


def whole_tiles(worklist):
    """Item records of a dK/dV list with the pieces of every split key tile put together again; checks on the
    way that the pieces of a tile occupy consecutive partial slots and follow each other without gap or overlap."""
    items = va.worklist_items(worklist)
    slot = (items[:, 1] >> 8) - 1
    whole = [it.copy() for it, s in zip(items, slot) if s < 0]
    taken = set()
    for rec in va.worklist_merges(worklist):
        row0, w1, first, pieces, qt_first, qt_count = (int(x) for x in rec[:6])
        assert pieces >= 2 and w1 >> 8 == 0
        at = qt_first
        for j in range(pieces):
            (i,) = np.nonzero(slot == first + j)[0]
            assert i not in taken and items[i, 0] == row0 and items[i, 1] & 0xff == w1 and items[i, 3] == at and items[i, 4] > 0
            taken.add(int(i))
            at += int(items[i, 4])
        assert at == qt_first + qt_count
        it = items[i].copy()
        it[1], it[3], it[4] = w1, qt_first, qt_count
        whole.append(it)
    assert len(taken) == int((slot >= 0).sum())
    return np.array(whole, dtype=np.int32).reshape(-1, 8)


def sorted_rows(a):
    return a[np.lexsort(a.T[::-1])]


def replay_dispatch(cost_in_launch_order, slots):
    """Finish time when workgroup b runs on XCD b % 8 and every XCD gives its works, in order, to the
    least-loaded of its slots / 8 workgroup slots."""
    import heapq
    heaps = [[0] * (slots // 8) for _ in range(8)]
    finish = 0
    for pos, c in enumerate(cost_in_launch_order):
        h = heaps[pos % 8]
        t = heapq.heappop(h) + int(c)
        heapq.heappush(h, t)
        finish = max(finish, t)
    return finish


def test_heavy_key_tiles_are_split_where_the_last_round_would_idle():
    # pi05, bin 0: 257 heavy dK/dV works (8 query heads x 27-32 query tiles each) for 256 workgroup slots
    w = wl.WORKLOADS["pi05"]
    lens, prefix = wl.sample_lengths("pi05")
    b, p, n = va.va_pack_first_fit(lens, w.budget)
    idx = op.bin_members(b, p, 0)
    cu, pl, mx = va.va_bin_layout(lens[idx], prefix[idx])
    rows, cols = va.va_tile_shape(va.VA_PASS_BWD_DKDV, w.head_dim, w.num_q_heads, w.num_kv_heads)
    got = va.va_build_worklist(cu, pl, va.VA_MASK_PREFIX_LM, va.VA_PASS_BWD_DKDV, w.head_dim, w.num_q_heads, w.num_kv_heads)
    items = va.worklist_items(got)
    assert got[1, 7] >= 1 and int((items[:, 1] >> 8 > 0).sum()) >= 2
    assert np.all(np.diff(items[:, 4]) <= 0)                              # still heaviest first
    # put together again, the list is the oracle's
    want = op.build_worklist(cu, pl, va.VA_PASS_BWD_DKDV, cols, rows, va.VA_MASK_PREFIX_LM)
    assert np.array_equal(sorted_rows(whole_tiles(got)), sorted_rows(want))
    # and the replayed dispatch ends within 10 % of the lower bound, where the unsplit list needs two rounds
    G = w.num_q_heads // w.num_kv_heads
    slots = int(got[1, 0])
    cost = np.repeat(items[:, 4] * G + 2, w.num_kv_heads)
    bound = max(cost.sum() / slots, np.repeat(want[:, 4] * G + 2, w.num_kv_heads).max())
    assert replay_dispatch(cost, slots) <= 1.1 * bound
    assert replay_dispatch(np.repeat(want[:, 4] * G + 2, w.num_kv_heads), slots) > 1.5 * bound
    # the library accepts its own list and refuses one whose pieces leave a gap
    Hq, Hkv, D = w.num_q_heads, w.num_kv_heads, w.head_dim
    shape = va.make_shape(int(cu[-1]), len(cu) - 1, Hq, Hkv, D, mx, va.VA_MASK_PREFIX_LM)
    need = va.varlen_attn_bwd_workspace_bytes(shape)
    assert need >= 2 * int(cu[-1]) * Hq * 4 + 2 * rows * D * 4 * Hkv * 4
    # the validation of the device calls: the library accepts its own list and refuses lists whose pieces leave
    # a gap, overlap, share a slot, or whose merge record names another tile
    va.va_check_worklist(got, va.VA_PASS_BWD_DKDV, cu, pl, shape)

    def call(dkdv_list):
        try:
            va.va_check_worklist(dkdv_list, va.VA_PASS_BWD_DKDV, cu, pl, shape)
        except va.VarlenAttnError as e:
            return e.code
        return va.VA_OK

    pieces = np.nonzero(items[:, 1] >> 8 > 0)[0] + 2            # records of the pieces
    merge = int(got[1, 6]) - int(got[1, 7])                      # record of the first merge record
    gap, overlap, shared, other_tile, lost = (got.copy() for _ in range(5))
    gap[pieces[1], 3] += 1                                       # second piece starts one query tile late
    overlap[pieces[1], 4] += 1                                   # ... or covers one tile too many
    shared[pieces[1], 1] = shared[pieces[0], 1]                  # two pieces, one slot
    other_tile[merge, 0] += rows                                 # merge record of a different key tile
    lost[1, 7] = 0                                               # pieces without their merge record
    for bad in (gap, overlap, shared, other_tile, lost):
        assert call(bad) == va.VA_EINVAL, va.va_last_error()


def test_split_pieces_cover_every_pair_once():
    # 65 samples x 4 KV heads = 260 equal works for 256 slots at head_dim 256: the last tile is cut in two
    Hq, Hkv, D = 4, 4, 256
    lens = np.full(65, 64, dtype=np.int32)
    cu, _, _ = va.va_bin_layout(lens)
    rows, cols = va.va_tile_shape(va.VA_PASS_BWD_DKDV, D, Hq, Hkv)
    got = va.va_build_worklist(cu, None, va.VA_MASK_CAUSAL, va.VA_PASS_BWD_DKDV, D, Hq, Hkv)
    items = va.worklist_items(got)
    assert got[1, 7] == 1 and int((items[:, 1] >> 8 > 0).sum()) == 2
    whole = whole_tiles(got)
    op.check_coverage(whole, cu, None, va.VA_PASS_BWD_DKDV, cols, rows, va.VA_MASK_CAUSAL)
    assert np.array_equal(sorted_rows(whole), sorted_rows(op.build_worklist(cu, None, va.VA_PASS_BWD_DKDV, cols, rows, va.VA_MASK_CAUSAL)))


def test_in_step_launch_order_keeps_a_sample_on_one_xcd():
    # heavy-tailed lengths, many works per slot: the id array of the dK/dV list is the launch order, and the
    # key tiles of one (sample, KV head) sit at positions of one XCD (position % 8), next to each other
    w = wl.WORKLOADS["longtail"]
    lens, _ = wl.sample_lengths("longtail")
    b, p, n = va.va_pack_first_fit(lens, w.budget)
    cu, _, mx = va.va_bin_layout(lens[op.bin_members(b, p, 0)])
    got = va.va_build_worklist(cu, None, va.VA_MASK_CAUSAL, va.VA_PASS_BWD_DKDV, w.head_dim, w.num_q_heads, w.num_kv_heads)
    assert got[1, 3] == 1
    items = va.worklist_items(got)
    _, ids = va.worklist_schedule(got)
    assert sorted(ids.tolist()) == list(range(len(items) * w.num_kv_heads))
    group = {}
    for pos, wid in enumerate(ids.tolist()):
        group.setdefault((int(items[wid // w.num_kv_heads, 2]), wid % w.num_kv_heads), []).append(pos)
    on_one_xcd = sum(len({pos % 8 for pos in g}) == 1 for g in group.values())
    assert on_one_xcd >= 0.95 * len(group)
    adjacent = sum(max(g) - min(g) == 8 * (len(g) - 1) for g in group.values() if len({pos % 8 for pos in g}) == 1)
    assert adjacent >= 0.9 * on_one_xcd
    # and the replay of the dispatch says it ends within 3 % of the item order
    G = w.num_q_heads // w.num_kv_heads
    cost = np.repeat(items[:, 4] * G + 2, w.num_kv_heads)
    assert replay_dispatch(cost[ids], int(got[1, 0])) <= 1.03 * replay_dispatch(cost, int(got[1, 0]))


@pytest.mark.parametrize("trial", range(24))
def test_builder_and_validator_agree_on_random_streams(trial):
    # random head shapes, masks and length mixes, some with many equal works per workgroup slot so that tiles are
    # split: every list the builder returns passes the validation of the device calls; put together again, the
    # dK/dV list is the oracle's; its id array is a permutation; single-word damage anywhere in the items, the
    # schedule or the merge records is refused or leaves a list that is still safe to follow (it passes again)
    r = np.random.default_rng(9000 + trial)
    Hkv = int(r.choice([1, 2, 4, 8]))
    G = int(r.choice([1, 2, 4, 8]))
    D = int(r.choice([64, 128, 256]))
    mode = int(r.choice([va.VA_MASK_CAUSAL, va.VA_MASK_PREFIX_LM, va.VA_MASK_PREFIX_LM_CAUSAL, va.VA_MASK_THREE_BLOCK,
                         va.VA_MASK_SLIDING_WINDOW]))
    slots = 512 if D <= 128 else 256
    kind = trial % 3
    if kind == 0:       # a few samples of mixed length
        lens = r.integers(0, 700, size=int(r.integers(1, 12)))
    elif kind == 1:     # just more equal works than slots: the case the split is for
        per_sample = Hkv
        n = slots // per_sample + int(r.integers(1, 4))
        lens = np.full(n, int(r.choice([64, 100, 128])))
    else:               # many works per slot
        lens = r.integers(1, 400, size=int(r.integers(200, 500)))
    lens = lens.astype(np.int32)
    cu, _, mx = va.va_bin_layout(lens)
    if mode == va.VA_MASK_CAUSAL:
        prefix = None
    elif mode == va.VA_MASK_THREE_BLOCK:
        prefix = wl.random_block_ends(trial, lens)
    elif mode == va.VA_MASK_SLIDING_WINDOW:
        prefix = r.integers(1, 300, size=len(lens)).astype(np.int32)
    else:
        prefix = np.array([int(r.integers(0, L + 1)) for L in lens], dtype=np.int32)
    if kind == 1 and prefix is not None:
        prefix[:] = prefix[0]          # equal samples, equal masks
    Hq = G * Hkv
    shape = va.make_shape(int(cu[-1]), len(lens), Hq, Hkv, D, mx, mode)
    for pass_id in (va.VA_PASS_FWD, va.VA_PASS_BWD_DKDV, va.VA_PASS_BWD_DQ):
        got = va.va_build_worklist(cu, prefix, mode, pass_id, D, Hq, Hkv)
        va.va_check_worklist(got, pass_id, cu, prefix, shape)
        _, ids = va.worklist_schedule(got)
        assert sorted(ids.tolist()) == list(range(int(got[1, 1])))
        used = got[:int(got[1, 6])]
        if pass_id == va.VA_PASS_BWD_DKDV and (int(cu[-1]) <= 6000 or kind == 1):
            rows, cols = va.va_tile_shape(pass_id, D, Hq, Hkv)
            if kind == 1:    # equal samples: the oracle's (quadratic, brute-force) list of one sample, moved along the stream
                one = op.build_worklist(cu[:2], None if prefix is None else prefix[:1], pass_id, cols, rows, mode)
                want = np.concatenate([one + np.array([c, 0, c, 0, 0, 0, 0, 0], dtype=np.int32) for c in cu[:-1]])
            else:
                want = op.build_worklist(cu, prefix, pass_id, cols, rows, mode)
            if kind == 1 and want[:, 4].max() >= 2:      # a tile with one query tile cannot be cut
                assert got[1, 7] >= 1, "this case is meant to split a tile"
            assert np.array_equal(sorted_rows(whole_tiles(got)), sorted_rows(want))
        for _ in range(40):
            bad = got.copy()
            rec, word = int(r.integers(0, len(used))), int(r.integers(0, 8))
            bad[rec, word] += int(r.choice([-3, -1, 1, 2, 64, 1 << 8, 1 << 20]))
            try:
                va.va_check_worklist(bad, pass_id, cu, prefix, shape)
            except va.VarlenAttnError as e:
                assert e.code in (va.VA_EINVAL, va.VA_EUNSUPPORTED)


def test_worklist_counts_on_the_workloads():
    # closed-form item and key-tile counts for the first bin of each workload
    for name in ("vlm", "pi05", "longtail", "vit"):
        w = wl.WORKLOADS[name]
        lens, prefix = wl.sample_lengths(name)
        b, p, n = va.va_pack_first_fit(lens, w.budget)
        idx = op.bin_members(b, p, 0)
        cu, pl, mx = va.va_bin_layout(lens[idx], None if prefix is None else prefix[idx])
        mode = va.VA_MASK_PREFIX_LM if w.prefix_lm else va.VA_MASK_CAUSAL
        rows, cols = va.va_tile_shape(va.VA_PASS_FWD, w.head_dim, w.num_q_heads, w.num_kv_heads)
        items = va.worklist_items(va.va_build_worklist(cu, pl, mode, va.VA_PASS_FWD, w.head_dim, w.num_q_heads, w.num_kv_heads))
        assert len(items) == sum(-(-int(L) // rows) for L in lens[idx])
        if not w.prefix_lm:
            want_tiles = sum(-(-min(int(L), (t + 1) * rows) // cols) for L in lens[idx] for t in range(-(-int(L) // rows)))
            assert int(items[:, 5].sum()) == want_tiles
        assert np.all(np.diff(items[:, 5]) <= 0)


def test_tile_shape_errors():
    assert va.va_tile_shape(va.VA_PASS_BWD_DKDV, 80, 4, 4) == va.va_tile_shape(va.VA_PASS_BWD_DKDV, 128, 4, 4)
    for bad in ((va.VA_PASS_FWD, 112, 4, 2), (va.VA_PASS_FWD, 32, 4, 2), (va.VA_PASS_FWD, 128, 5, 2), (7, 128, 4, 2)):
        with pytest.raises(va.VarlenAttnError) as e:
            va.va_tile_shape(*bad)
        assert e.value.code == va.VA_EUNSUPPORTED


def test_e4m3_quantiser_equals_oracle_bit_for_bit():
    r = np.random.default_rng(9)
    x = wl.round_to_bf16((r.standard_normal((300, 5, 64)) * np.array([1e-3, 0.1, 1.0, 30.0, 0.0])[None, :, None]).astype(np.float32))
    codes, descale = va.va_quantize_e4m3_per_head(wl.bf16_bits(x))
    ocodes, odescale = oe.quantize_per_head(x)
    assert np.array_equal(descale, odescale) and np.array_equal(codes, ocodes)
    # every representable magnitude and every midpoint, scaled so that descale = 1
    vals = [oe.decode_scalar(c) for c in range(0x7F)]
    mids = [(vals[i] + vals[i + 1]) / 2 for i in range(0x7E)]
    probe = np.array(vals + mids + [448.0], dtype=np.float32)
    probe = probe[wl.round_to_bf16(probe) == probe]           # keep those bf16 can hold exactly
    probe = np.concatenate([probe, -probe]).reshape(-1, 1, 1)
    probe = np.concatenate([probe, np.full((1, 1, 1), 448.0, dtype=np.float32)])
    codes, descale = va.va_quantize_e4m3_per_head(wl.bf16_bits(probe))
    assert descale[0] == 1.0 and np.array_equal(codes, oe.encode(probe))


def with_non_finite(seed, T, H, D):
    """bf16 bit patterns [T, H, D] with a NaN of either sign planted in head 0 and infinities in head 1;
    returns (bits, mask of the NaN positions)"""
    r = np.random.default_rng(seed)
    x = wl.bf16_bits(wl.round_to_bf16(r.standard_normal((T, H, D)).astype(np.float32) * 3.0)).copy()
    nan = np.zeros(x.shape, dtype=bool)
    nan[T // 3, 0, 5] = nan[T - 1, 0, D - 1] = True
    x[T // 3, 0, 5], x[T - 1, 0, D - 1] = 0x7fc0, 0xffc1
    x[1, 1, 0], x[T // 2, 1, 7] = 0x7f80, 0xff80
    return x, nan


def test_quantisers_keep_a_nan_out_of_the_scale():
    # A NaN becomes the NaN code at its own place and does not touch the scale of its head or block: every
    # other element is quantised as if the NaN were a zero (the oracle's quantiser on the cleaned array).
    # An infinity makes the scale of its head infinite: finite values go to code 0, the infinity itself to NaN.
    T, H, D = 40, 3, 16
    x, nan = with_non_finite(3, T, H, D)
    cleaned = x.copy()
    cleaned[nan] = 0
    codes, descale = va.va_quantize_e4m3_per_head(x)
    with np.errstate(invalid="ignore"):      # the infinities of head 1 divide to NaN in the oracle as well
        ocodes, odescale = oe.quantize_per_head(wl.bits_to_f32(cleaned))
    assert np.all(codes[nan] == 0x7F)
    assert np.array_equal(codes[:, 0][~nan[:, 0]], ocodes[:, 0][~nan[:, 0]]) and descale[0] == odescale[0]
    assert np.array_equal(codes[:, 2], ocodes[:, 2]) and descale[2] == odescale[2]
    inf = (x[:, 1] & 0x7fff) == 0x7f80
    assert np.isinf(descale[1]) and np.all(codes[:, 1][inf] == 0x7F) and np.all(codes[:, 1][~inf] & 0x7f == 0)
    # block-wise: the same per block
    cu = np.array([0, 13, 40], dtype=np.int32)
    bcodes, bdescale = va.va_quantize_e4m3_blockwise(x, cu)
    with np.errstate(invalid="ignore"):
        ocodes, odescale = oe.quantize_blockwise(wl.bits_to_f32(cleaned), cu)
    assert np.all(bcodes[nan] == 0x7F) and np.array_equal(bcodes[:, 0][~nan[:, 0]], ocodes[:, 0][~nan[:, 0]])
    assert np.array_equal(bcodes[:, 2], ocodes[:, 2])


def expand_block_descale(descale, cu, H):
    """The oracle's [num_blocks, H] block scales, one row per token (the library's layout)."""
    starts = oe.block_starts(cu)
    out = np.zeros((int(cu[-1]), H), dtype=np.float32)
    for s in range(len(cu) - 1):
        for t in range(int(cu[s]), int(cu[s + 1])):
            out[t] = descale[int(starts[s]) + (t - int(cu[s])) // oe.BLOCK_TOKENS]
    return out


def test_blockwise_e4m3_quantiser_equals_oracle_bit_for_bit():
    r = np.random.default_rng(19)
    lens = [5, 128, 0, 129, 300, 1, 256]
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    T, H, D = int(cu[-1]), 3, 48
    x = r.standard_normal((T, H, D)).astype(np.float32)
    x *= np.exp2(r.integers(-12, 8, size=(T // 50 + 1,)))[np.arange(T) // 50][:, None, None]   # magnitude drifts along the stream
    x[128 + 5:128 + 5 + 128, 1] = 0.0      # an all-zero block (sample 1, head 1): descale 1
    x = wl.round_to_bf16(x)
    codes, descale_tok = va.va_quantize_e4m3_blockwise(wl.bf16_bits(x), cu)
    ocodes, odescale = oe.quantize_blockwise(x, cu)
    want = expand_block_descale(odescale, cu, H)
    assert np.array_equal(descale_tok.view(np.uint32), want.view(np.uint32)) and np.array_equal(codes, ocodes)
    assert np.all(descale_tok[133:261, 1] == 1.0)
    # one sample shorter than a block equals the per-head quantiser on that sample
    c1, d1 = va.va_quantize_e4m3_blockwise(wl.bf16_bits(x[:5]), np.array([0, 5], dtype=np.int32))
    c2, d2 = va.va_quantize_e4m3_per_head(wl.bf16_bits(x[:5]))
    assert np.array_equal(c1, c2) and np.all(d1 == d2[None, :])
    # bad sample boundaries are refused
    with pytest.raises(va.VarlenAttnError):
        va.va_quantize_e4m3_blockwise(wl.bf16_bits(x[:5]), np.array([1, 5], dtype=np.int32))
    bad = np.array([0, 4, 3, 5], dtype=np.int32)
    with pytest.raises(va.VarlenAttnError):
        va.va_quantize_e4m3_blockwise(wl.bf16_bits(x[:5]), bad)


def _fake(n=1 << 12):
    return np.zeros(n, dtype=np.uint8)


def test_device_entry_points_reject_bad_arguments_on_the_host():
    Hq, Hkv, D = 4, 2, 64
    cu = np.array([0, 40, 100], dtype=np.int32)
    wl_h = va.va_build_worklist(cu, None, va.VA_MASK_CAUSAL, va.VA_PASS_FWD, D, Hq, Hkv)
    buf = _fake()
    lse = np.zeros(1024, dtype=np.float32)

    def call(shape, cu_=cu, wl_=wl_h, q=buf, scale=0.125, prefix=None):
        # stream pointer 0 is never reached: validation fails first
        rc = va._lib.varlen_attn_fwd(va._ptr(q), va._ptr(buf), va._ptr(buf), va._ptr(cu_), va._ptr(prefix), va._ptr(wl_),
                                     va._ptr(wl_), ctypes.byref(shape), ctypes.c_float(scale), va._ptr(buf),
                                     va._ptr(lse), ctypes.c_void_p(0))
        return rc, va.va_last_error()

    ok = dict(total_tokens=100, num_seqs=2, num_q_heads=Hq, num_kv_heads=Hkv, head_dim=D, max_seqlen=60,
              mask_mode=va.VA_MASK_CAUSAL)
    assert call(va.make_shape(**{**ok, "head_dim": 112}))[0] == va.VA_EUNSUPPORTED
    assert call(va.make_shape(**{**ok, "num_q_heads": 3}))[0] == va.VA_EUNSUPPORTED
    assert call(va.make_shape(**{**ok, "max_seqlen": 59}))[0] == va.VA_ESIZE
    assert call(va.make_shape(**{**ok, "max_seqlen": 1 << 29}))[0] == va.VA_ESIZE       # 32-bit buffer offsets
    assert call(va.make_shape(**{**ok, "total_tokens": 101}))[0] == va.VA_EINVAL
    assert call(va.make_shape(**ok), cu_=np.array([0, 60, 40], dtype=np.int32))[0] == va.VA_EINVAL
    assert call(va.make_shape(**ok), cu_=np.array([1, 40, 100], dtype=np.int32))[0] == va.VA_EINVAL
    assert call(va.make_shape(**ok), scale=0.0)[0] == va.VA_EINVAL
    assert call(va.make_shape(**ok), scale=float("nan"))[0] == va.VA_EINVAL
    assert call(va.make_shape(**{**ok, "mask_mode": va.VA_MASK_PREFIX_LM}))[0] == va.VA_EINVAL      # no prefix_lens
    assert call(va.make_shape(**{**ok, "mask_mode": va.VA_MASK_PREFIX_LM}),
                prefix=np.array([41, 0], dtype=np.int32))[0] == va.VA_EINVAL
    rc, msg = call(va.make_shape(**ok), q=buf[1:])
    assert rc == va.VA_EALIGN and "aligned" in msg
    # a work list built for another stream, pass or head_dim is refused
    other = va.va_build_worklist(np.array([0, 50, 100], dtype=np.int32), None, va.VA_MASK_CAUSAL, va.VA_PASS_FWD, D, Hq, Hkv)
    tampered = wl_h.copy()
    tampered[2, 1] = 1000
    wrong_pass = va.va_build_worklist(cu, None, va.VA_MASK_CAUSAL, va.VA_PASS_BWD_DKDV, D, Hq, Hkv)
    bad_table = wl_h.copy()
    bad_table[wl_h[1, 4] + 1, 3] += 1                  # first workgroup claims one work too many
    bad_flag = wl_h.copy()
    bad_flag[1, 3] = 1                                 # the in-step flag belongs to dK/dV lists
    bad_copy = wl_h.copy()
    bad_copy[wl_h[1, 4], 1] += 1                       # its copy of its first item differs from the item
    bad_id = wl_h.copy()
    bad_id[wl_h[1, 5], 0] = wl_h[1, 1]                 # a work id past the end
    # words near the end of the int32 range: refused by comparisons that cannot wrap around
    huge_len = wl_h.copy()
    huge_len[2, 2], huge_len[2, 7] = 2**31 - 5, 2**31 - 1   # first row of the sample, its length
    huge_row = wl_h.copy()
    huge_row[2, 0] = 2**31 - 1                               # first row of the item
    for bad in (other, tampered, wrong_pass, bad_table, bad_copy, bad_id, bad_flag, huge_len, huge_row):
        assert call(va.make_shape(**ok), wl_=np.ascontiguousarray(bad))[0] == va.VA_EINVAL
    dkdv = va.va_build_worklist(cu, None, va.VA_MASK_CAUSAL, va.VA_PASS_BWD_DKDV, D, Hq, Hkv)
    huge_range = dkdv.copy()
    huge_range[2, 3], huge_range[2, 4] = 2**31 - 1, 2**31 - 1   # first query tile and count of the first item
    with pytest.raises(va.VarlenAttnError) as e:
        va.va_check_worklist(huge_range, va.VA_PASS_BWD_DKDV, cu, None, va.make_shape(**ok))
    assert e.value.code == va.VA_EINVAL
    assert va.varlen_attn_bwd_workspace_bytes(va.make_shape(**ok)) >= 100 * Hq * 4


def test_three_block_ends_are_validated():
    cu = np.array([0, 10, 30], dtype=np.int32)
    for bad in ([[4, 3], [0, 0]], [[0, 11], [0, 0]], [[-1, 5], [0, 0]], [[0, 0], [5, 21]]):
        with pytest.raises(va.VarlenAttnError) as e:
            va.va_build_worklist(cu, np.array(bad, dtype=np.int32), va.VA_MASK_THREE_BLOCK, va.VA_PASS_FWD, 64, 2, 2)
        assert e.value.code == va.VA_EINVAL and "block ends" in str(e.value)
    with pytest.raises(ValueError):      # one entry per sample is not enough for this mask
        va.va_build_worklist(cu, np.array([3, 4], dtype=np.int32), va.VA_MASK_THREE_BLOCK, va.VA_PASS_FWD, 64, 2, 2)
    with pytest.raises(va.VarlenAttnError) as e:
        va.va_build_worklist(cu, np.array([3, 4], dtype=np.int32), 5, va.VA_PASS_FWD, 64, 2, 2)
    assert e.value.code == va.VA_EUNSUPPORTED
    # both boundaries land in the items: P in word 6, P2 in word 3 (forward, dQ) or 5 (dK/dV)
    ends = np.array([[2, 7], [20, 20]], dtype=np.int32)
    for pass_id, word in ((va.VA_PASS_FWD, 3), (va.VA_PASS_BWD_DQ, 3), (va.VA_PASS_BWD_DKDV, 5)):
        items = va.worklist_items(va.va_build_worklist(cu, ends, va.VA_MASK_THREE_BLOCK, pass_id, 64, 2, 2))
        for it in items:
            s = 0 if it[2] == 0 else 1
            assert (it[6], it[word]) == tuple(ends[s])


def test_fp8_entry_points_reject_bad_arguments_on_the_host():
    # every call fails in validation, before any stream or device pointer is used
    Hq, Hkv = 4, 2
    cu = np.array([0, 40, 100], dtype=np.int32)
    buf, lse = _fake(), np.zeros(1024, dtype=np.float32)
    f32 = np.zeros(1024, dtype=np.float32)

    def fwd(fn, D=128, qd=f32, q=buf):
        wl_h = va.va_build_worklist(cu, None, va.VA_MASK_CAUSAL, va.VA_PASS_FWD, D, Hq, Hkv)
        shape = va.make_shape(100, 2, Hq, Hkv, D, 60, va.VA_MASK_CAUSAL)
        rc = fn(va._ptr(q), va._ptr(buf), va._ptr(buf), va._ptr(qd), va._ptr(f32), va._ptr(f32), va._ptr(cu),
                ctypes.c_void_p(0), va._ptr(wl_h), va._ptr(wl_h), ctypes.byref(shape), ctypes.c_float(0.1),
                va._ptr(buf), va._ptr(lse), ctypes.c_void_p(0))
        return rc, va.va_last_error()

    for fn in (va._lib.varlen_attn_fwd_fp8, va._lib.varlen_attn_fwd_fp8_blockwise):
        rc, msg = fwd(fn, D=96)                       # a head dimension the bf16 kernels take and the FP8 forward does not
        assert rc == va.VA_EUNSUPPORTED and "64, 128 and 256" in msg
        assert fwd(fn, q=None)[0] == va.VA_EINVAL
        assert fwd(fn, qd=None)[0] == va.VA_EINVAL
        assert fwd(fn, q=buf[8:])[0] == va.VA_EALIGN
    assert fwd(va._lib.varlen_attn_fwd_fp8_blockwise, qd=f32.view(np.uint8)[2:].view(np.uint8))[0] == va.VA_EALIGN

    def quant(cu_=cu, cu_dev=cu, H=2, D=64, x=buf, codes=buf, d=f32):
        rc = va._lib.va_quantize_e4m3_blockwise_device(va._ptr(x), va._ptr(cu_), va._ptr(cu_dev), ctypes.c_int32(len(cu) - 1),
                                                       ctypes.c_int32(H), ctypes.c_int32(D), va._ptr(codes), va._ptr(d),
                                                       ctypes.c_void_p(0))
        return rc, va.va_last_error()

    assert quant(D=12)[0] == va.VA_EINVAL and quant(H=0)[0] == va.VA_EINVAL
    assert quant(cu_=np.array([0, 50, 40], dtype=np.int32))[0] == va.VA_EINVAL
    assert quant(cu_=np.array([1, 50, 60], dtype=np.int32))[0] == va.VA_EINVAL
    assert quant(cu_dev=None)[0] == va.VA_EINVAL and quant(x=None)[0] == va.VA_EINVAL
    assert quant(x=buf[8:])[0] == va.VA_EALIGN and quant(codes=buf[4:])[0] == va.VA_EALIGN
    assert quant(cu_=np.array([0, 0, 0], dtype=np.int32), x=None, codes=None, d=None)[0] == va.VA_OK   # nothing to do


def test_window_widths_are_validated():
    cu = np.array([0, 10, 30], dtype=np.int32)
    for bad in ([0, 5], [4, -1]):
        with pytest.raises(va.VarlenAttnError) as e:
            va.va_build_worklist(cu, np.array(bad, dtype=np.int32), va.VA_MASK_SLIDING_WINDOW, va.VA_PASS_FWD, 64, 2, 2)
        assert e.value.code == va.VA_EINVAL
    with pytest.raises(va.VarlenAttnError):
        va.va_build_worklist(cu, None, va.VA_MASK_SLIDING_WINDOW, va.VA_PASS_FWD, 64, 2, 2)
    # a window as long as the sample lists what the causal mask lists, apart from the W word
    wide = va.worklist_items(va.va_build_worklist(cu, np.array([10, 99], dtype=np.int32), va.VA_MASK_SLIDING_WINDOW, va.VA_PASS_FWD, 64, 2, 2))
    causal = va.worklist_items(va.va_build_worklist(cu, None, va.VA_MASK_CAUSAL, va.VA_PASS_FWD, 64, 2, 2))
    assert np.array_equal(np.delete(wide, 6, axis=1), np.delete(causal, 6, axis=1))


def test_forward_schedule_keeps_the_works_of_a_sample_and_kv_head_on_one_xcd():
    # causal stream: workgroup b runs on XCD b % 8; the works that stream the same K and V rows should
    # share an XCD (groups heavier than a sixteenth of an XCD's share may be cut), and stay balanced
    r = np.random.default_rng(5)
    lens = r.integers(200, 900, size=40).astype(np.int32)
    cu, _, _ = va.va_bin_layout(lens)
    Hq, Hkv, D = 16, 8, 128
    for pass_id in (va.VA_PASS_FWD, va.VA_PASS_BWD_DQ):
        got = va.va_build_worklist(cu, None, va.VA_MASK_CAUSAL, pass_id, D, Hq, Hkv)
        items = va.worklist_items(got)
        table, ids = va.worklist_schedule(got)
        per_item = int(got[1, 2])
        chunks_per_head = per_item // Hkv
        xcds = {}
        for b, (first, count) in enumerate(table.tolist()):
            for wid in ids[first:first + count].tolist():
                key = (int(items[wid // per_item, 2]), (wid % per_item) // chunks_per_head)
                xcds.setdefault(key, set()).add(b % 8)
        assert len(xcds) == len(lens) * Hkv
        assert sum(len(v) == 1 for v in xcds.values()) >= 0.9 * len(xcds)
        cost = np.repeat(items[:, 5], per_item) + 2
        loads = np.array([cost[ids[a:a + n]].sum() for a, n in table])
        assert loads.max() <= 1.1 * cost.sum() / len(table) + cost.max()
    # whole samples visible to every row: every query tile of a sample costs the same and the plain
    # heaviest-first order is used, which hands consecutive works to consecutive workgroups
    full = va.va_build_worklist(cu, lens, va.VA_MASK_PREFIX_LM, va.VA_PASS_FWD, D, Hq, Hkv)
    table, ids = va.worklist_schedule(full)
    assert ids[table[0, 0]] == 0 and ids[table[1, 0]] == 1 and ids[table[7, 0]] == 7


def test_bench_refuses_more_than_one_gpu():
    # the benchmark is a one-GPU program: asking for more must end with a message, before any device is touched
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "one GPU" in (r.stdout + r.stderr)
