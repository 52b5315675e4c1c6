"""Oracle for the host-side integer work: first-fit packing, the per-bin layout
and the per-tile work lists.

TEST INFRASTRUCTURE ONLY.  Plain Python loops, written from the rule, sharing
nothing with the C++ packer of the library.

Packing (paper section 2.2.1 (2), "Data Packing"): samples are concatenated end
to end into sequences close to a token budget.  The paper does not name the
bin-packing rule; the reading taken is online first-fit in arrival order: bins
are opened in order, each sample goes to the lowest-numbered bin that still has
room for it, nothing is sorted or reordered, and the order inside a bin is the
placement order.

Work lists: one item per tile of rows, listing only the key tiles that hold at
least one allowed (query, key) pair, so fully masked tiles are never visited
and no tile spans two samples.  Items are 8 int32 words:

  forward / dQ pass (one item per query tile of ``bm`` token rows)
    0 q_row0      absolute first row of the tile in the stream
    1 q_rows      valid rows in the tile (<= bm)
    2 seq_row0    first row of the sample (cu_seqlens[s])
    3 block2_end  P2_s under the three-block mask, else -1
    4 n_full      leading key tiles in which every (row, key) pair is allowed
    5 n_tiles     key tiles visited = ceil(kv_len / bn), kv_len = keys visible
                  to at least one row of the tile
    6 prefix_len  P_s, or -1 when the stream is causal
    7 seq_len     L_s

  dK/dV pass (one item per key tile of ``bn`` token rows)
    0 kv_row0     absolute first key row of the tile
    1 kv_rows     valid key rows (<= bn)
    2 seq_row0    cu_seqlens[s]
    3 qt_first    index (within the sample) of the first query tile, of ``bm``
                  rows, that holds a row seeing a key of this tile
    4 qt_count    number of query tiles from qt_first to the end of the sample
    5 block2_end  P2_s under the three-block mask, else -1
    6 prefix_len  P_s or -1
    7 seq_len     L_s

Order: descending amount of work (n_tiles, resp. qt_count), ties in ascending
(sample, tile) order.

Sliding window (prefix_len holds the window W): n_full and n_tiles are those of
the causal mask on the same rows; an item visits the key tiles from the first
one that holds an allowed pair up to n_tiles, and treats as mask-free those from
the first one fully inside the window of its last row up to n_full; its amount
of work is the number of tiles it visits.  qt_count of a dK/dV item ends with
the last query tile that holds a row seeing a key of the item.
"""
import numpy as np

PASS_FWD = 0
PASS_BWD_DKDV = 1
PASS_BWD_DQ = 2

MASK_CAUSAL = 0
MASK_PREFIX_BIDIR_SUFFIX = 1
MASK_PREFIX_CAUSAL_SUFFIX = 2
MASK_THREE_BLOCK = 3      # prefix_lens holds [num_seqs, 2]: the ends (P, P2) of the first two blocks
MASK_SLIDING_WINDOW = 4   # causal, at most the W most recent keys; prefix_lens holds W >= 1 per sample


def first_fit(lens, budget):
    """Online first-fit.  Returns (bin_of_sample, pos_in_bin, num_bins)."""
    free = []
    count = []
    bin_of = []
    pos_in = []
    for L in lens:
        L = int(L)
        if L < 0 or L > budget:
            raise ValueError("sample length outside [0, budget]")
        placed = None
        for b in range(len(free)):
            if free[b] >= L:
                placed = b
                break
        if placed is None:
            free.append(budget)
            count.append(0)
            placed = len(free) - 1
        free[placed] -= L
        bin_of.append(placed)
        pos_in.append(count[placed])
        count[placed] += 1
    return (np.array(bin_of, dtype=np.int32), np.array(pos_in, dtype=np.int32), len(free))


def bin_members(bin_of, pos_in, b):
    """Original sample indices of bin ``b`` in placement order."""
    idx = [i for i in range(len(bin_of)) if bin_of[i] == b]
    idx.sort(key=lambda i: pos_in[i])
    return np.array(idx, dtype=np.int32)


def bin_layout(lens, prefix=None):
    """cu_seqlens (exclusive prefix sums), prefix_lens and max_seqlen of one bin."""
    cu = [0]
    for L in lens:
        cu.append(cu[-1] + int(L))
    mx = max([int(L) for L in lens], default=0)
    # one entry per sample, or the pair of block ends of the three-block mask
    pl = None if prefix is None else np.array([[int(x) for x in np.atleast_1d(p)] for p in prefix], dtype=np.int32)
    if pl is not None and pl.shape[1:] == (1,):
        pl = pl[:, 0]
    return np.array(cu, dtype=np.int32), pl, mx


def visible(i, L, P, mode, P2=-1):
    """Number of keys local query row i may attend to."""
    if mode in (MASK_CAUSAL, MASK_SLIDING_WINDOW):
        return i + 1
    if i < P:
        return P
    if mode == MASK_PREFIX_BIDIR_SUFFIX:
        return L
    if mode == MASK_THREE_BLOCK:
        return P2 if i < P2 else L
    return i + 1


def allowed(i, j, L, P, mode, P2=-1):
    if mode == MASK_SLIDING_WINDOW:        # P holds the window
        return 0 <= i - j < P
    return 0 <= j < visible(i, L, P, mode, P2)


def block_ends(prefix_lens, mode, s):
    """(P, P2) of sample s as stored in an item: -1 where the mask has no such boundary."""
    if mode == MASK_CAUSAL:
        return -1, -1
    if mode == MASK_THREE_BLOCK:
        pair = np.asarray(prefix_lens).reshape(-1, 2)[s]
        return int(pair[0]), int(pair[1])
    return int(prefix_lens[s]), -1


def _mode(prefix_lens, mask_mode):
    if mask_mode is None:
        return MASK_CAUSAL if prefix_lens is None else MASK_PREFIX_BIDIR_SUFFIX
    return mask_mode


def build_worklist(cu_seqlens, prefix_lens, pass_id, bm, bn, mask_mode=None):
    """Canonical work list as an [n_items, 8] int32 array, by brute force over
    rows and keys (no closed forms: every count is obtained by looking at every
    (row, key) pair of the tile)."""
    mode = _mode(prefix_lens, mask_mode)
    n = len(cu_seqlens) - 1
    items = []
    for s in range(n):
        c = int(cu_seqlens[s])
        L = int(cu_seqlens[s + 1]) - c
        P, P2 = block_ends(prefix_lens, mode, s)
        if pass_id in (PASS_FWD, PASS_BWD_DQ):
            for t in range((L + bm - 1) // bm):
                rows = range(t * bm, min(L, (t + 1) * bm))
                kv_len = 0
                for i in rows:
                    for j in range(L):
                        if allowed(i, j, L, P, mode, P2):
                            kv_len = max(kv_len, j + 1)
                n_tiles = (kv_len + bn - 1) // bn
                upper = MASK_CAUSAL if mode == MASK_SLIDING_WINDOW else mode   # n_full looks at the upper edge only
                n_full = 0
                for kt in range(n_tiles):
                    if kt != n_full:
                        break
                    ok = (kt + 1) * bn <= L
                    for i in rows:
                        for j in range(kt * bn, min(L, (kt + 1) * bn)):
                            ok = ok and allowed(i, j, L, P, upper, P2)
                    if ok:
                        n_full += 1
                visited = sum(1 for kt in range(n_tiles)
                              if any(allowed(i, j, L, P, mode, P2) for i in rows for j in range(kt * bn, min(L, (kt + 1) * bn))))
                items.append(((visited, s, t), [c + t * bm, len(rows), c, P2, n_full, n_tiles, P, L]))
        else:
            for kt in range((L + bn - 1) // bn):
                keys = range(kt * bn, min(L, (kt + 1) * bn))
                first_row = None
                for i in range(L):
                    if any(allowed(i, j, L, P, mode, P2) for j in keys):
                        first_row = i
                        break
                assert first_row is not None  # every key is seen by its own row
                qt_first = first_row // bm
                last_row = max(i for i in range(L) if any(allowed(i, j, L, P, mode, P2) for j in keys))
                qt_count = (L + bm - 1) // bm - qt_first
                if mode == MASK_SLIDING_WINDOW:
                    qt_count = last_row // bm - qt_first + 1
                items.append(((qt_count, s, kt), [c + kt * bn, len(keys), c, qt_first, qt_count, P2, P, L]))
    items.sort(key=lambda e: (-e[0][0], e[0][1], e[0][2]))
    if not items:
        return np.zeros((0, 8), dtype=np.int32)
    return np.array([e[1] for e in items], dtype=np.int32)


def check_coverage(items, cu_seqlens, prefix_lens, pass_id, bm, bn, mask_mode=None):
    """Brute-force proof that a work list visits every allowed (query, key) pair
    exactly once, visits no fully masked tile, marks as 'full' only tiles with
    no masked pair, and never lets a tile cross a sample boundary.  Raises
    AssertionError with the reason otherwise."""
    mode = _mode(prefix_lens, mask_mode)
    n = len(cu_seqlens) - 1
    T = int(cu_seqlens[n])
    sample_of_row = np.full(T, -1, dtype=np.int64)
    for s in range(n):
        sample_of_row[int(cu_seqlens[s]):int(cu_seqlens[s + 1])] = s
    seen = {}
    for it in np.asarray(items).reshape(-1, 8):
        a, rows, c, w3, w4, w5, P, L = [int(x) for x in it]
        assert rows > 0, "empty tile listed"
        s = int(sample_of_row[a])
        assert s >= 0 and int(cu_seqlens[s]) == c and int(cu_seqlens[s + 1]) - c == L, "wrong sample fields"
        assert a + rows <= c + L, "tile crosses the end of its sample"
        wantP, wantP2 = block_ends(prefix_lens, mode, s)
        assert P == wantP, "wrong prefix"
        if pass_id in (PASS_FWD, PASS_BWD_DQ):
            assert (a - c) % bm == 0 and rows <= bm
            P2, n_full, n_tiles = w3, w4, w5
            assert P2 == wantP2, "wrong end of the second block"
            assert n_full <= n_tiles and (n_tiles - 1) * bn < L
            kt_first, kt_plain = 0, 0
            if mode == MASK_SLIDING_WINDOW:   # the lower edge as the interface states it, from W
                kt_first = max(0, (a - c) + 1 - P) // bn
                kt_plain = -(-max(0, (a - c + rows - 1) + 1 - P) // bn)
            for kt in range(kt_first, n_tiles):
                pairs = 0
                masked = 0
                for i in range(a - c, a - c + rows):
                    for j in range(kt * bn, (kt + 1) * bn):
                        if j < L and allowed(i, j, L, P, mode, P2):
                            pairs += 1
                            key = (s, i, j)
                            seen[key] = seen.get(key, 0) + 1
                        else:
                            masked += 1
                assert pairs > 0, "fully masked tile listed"
                if kt_plain <= kt < n_full:
                    assert masked == 0, "tile marked full holds a masked pair"
        else:
            assert (a - c) % bn == 0 and rows <= bn
            qt_first, qt_count, P2 = w3, w4, w5
            assert P2 == wantP2, "wrong end of the second block"
            if mode == MASK_SLIDING_WINDOW:
                assert 0 < qt_count and qt_first + qt_count <= (L + bm - 1) // bm
            else:
                assert qt_first + qt_count == (L + bm - 1) // bm
            pairs_first = 0
            pairs_last = 0
            for qt in range(qt_first, qt_first + qt_count):
                for i in range(qt * bm, min(L, (qt + 1) * bm)):
                    for j in range(a - c, a - c + rows):
                        if allowed(i, j, L, P, mode, P2):
                            key = (s, i, j)
                            seen[key] = seen.get(key, 0) + 1
                            if qt == qt_first:
                                pairs_first += 1
                            if qt == qt_first + qt_count - 1:
                                pairs_last += 1
            assert pairs_first > 0, "first listed query tile sees nothing of this key tile"
            if mode == MASK_SLIDING_WINDOW:
                assert pairs_last > 0, "last listed query tile sees nothing of this key tile"
    total = 0
    for s in range(n):
        c = int(cu_seqlens[s])
        L = int(cu_seqlens[s + 1]) - c
        P, P2 = block_ends(prefix_lens, mode, s)
        for i in range(L):
            for j in range(L):
                if allowed(i, j, L, P, mode, P2):
                    total += 1
                    assert seen.get((s, i, j), 0) == 1, f"pair {(s, i, j)} visited {seen.get((s, i, j), 0)} times"
    assert total == len(seen), "a pair outside the mask was visited"
    return total


def allowed_pairs(L, P, mode, P2=-1):
    """Number of allowed (query, key) pairs of one sample, by counting."""
    if mode == MASK_SLIDING_WINDOW:
        return sum(min(i + 1, P) for i in range(L))
    return sum(visible(i, L, P, mode, P2) for i in range(L))
