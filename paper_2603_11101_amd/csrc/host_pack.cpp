// Host-side integer work of the packed variable-length attention library:
// first-fit packing, per-bin layout, tile shapes, per-tile work lists and the
// per-head E4M3 quantiser.  Pure host code; nothing here touches the GPU.
//
// Paper: section 2.2.1 (2) "Data Packing" (samples are concatenated into
// sequences close to the maximum context length, no padding tokens) and
// section 2.2.1 (1) (compute on valid tokens only).  The paper names no bin
// rule; online first-fit in arrival order is this library's reading.
#include "common.h"

#include <algorithm>
#include <cmath>
#include <cstring>
#include <functional>
#include <map>
#include <utility>
#include <vector>

namespace va {

thread_local char g_error[512] = "";

int fail(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_error, sizeof(g_error), fmt, ap);
    va_end(ap);
    return code;
}

// Heads of one KV group that a forward / dQ workgroup stacks on its 128 rows.
int heads_per_block(int32_t Hq, int32_t Hkv) {
    const int G = Hq / Hkv;
    int hpb = 1;
    while (hpb * 2 <= 8 && G % (hpb * 2) == 0) hpb *= 2;
    return hpb;
}

int tile_shape(int32_t pass, int32_t D, int32_t Hq, int32_t Hkv, int32_t* rows, int32_t* cols) {
    if (!head_dim_supported(D)) return fail(VA_EUNSUPPORTED, "head_dim %d not in {48,64,80,96,128,160,192,256}", D);
    if (Hq <= 0 || Hkv <= 0 || Hq % Hkv != 0)
        return fail(VA_EUNSUPPORTED, "num_q_heads %d is not a positive multiple of num_kv_heads %d", Hq, Hkv);
    switch (pass) {
        case VA_PASS_FWD:
            *rows = kFwdBlockRows / heads_per_block(Hq, Hkv);
            *cols = kFwdKvTile;
            return VA_OK;
        case VA_PASS_BWD_DQ:
            *rows = kDqBlockRows / heads_per_block(Hq, Hkv);
            *cols = kDqKvTile;
            return VA_OK;
        case VA_PASS_BWD_DKDV:
            *rows = kDkdvKvRows;
            *cols = dkdv_q_tile(D);
            return VA_OK;
        default:
            return fail(VA_EUNSUPPORTED, "unknown pass %d", pass);
    }
}

int works_per_item(int32_t pass, int32_t Hq, int32_t Hkv) {
    if (pass == VA_PASS_BWD_DKDV) return Hkv;
    return Hkv * ((Hq / Hkv) / heads_per_block(Hq, Hkv));
}

WorklistLayout worklist_layout(int32_t pass, int32_t D, int32_t Hq, int32_t Hkv, int32_t num_items, int32_t num_merges) {
    WorklistLayout l;
    l.num_workgroups = persistent_workgroups(pass, D);
    l.works_per_item = works_per_item(pass, Hq, Hkv);
    l.num_works = num_items * l.works_per_item;
    l.num_items = num_items;
    l.item_rec = 2;
    l.table_rec = l.item_rec + num_items;
    l.id_rec = l.table_rec + l.num_workgroups * (kTableWordsPerWorkgroup / 8);
    l.num_merges = num_merges;
    l.flags = 0;
    l.merge_rec = l.id_rec + (l.num_works + 7) / 8;
    l.total_recs = l.merge_rec + num_merges;
    return l;
}

}  // namespace va

using namespace va;

namespace {

struct Keyed {
    int32_t work;  // inner-loop steps of the item per head (the order of the list)
    WorkItem it;
};

// dK/dV pass: one workgroup runs one work, and the hardware hands the works to free workgroup slots in list
// order (heaviest first).  With few heavy works per slot the last round can leave most slots idle (257 equal
// works on 256 slots take two rounds).  This routine replays that dispatch on `slots` slots and, while the
// work that finishes last ends later than 1.04 times the lower bound max(mean load, heaviest work) (and, to
// begin with, later than 1.1 times), cuts the query tiles of its key tile into pieces of about an eighth of
// the lower bound each.  A piece is an item of its own with a partial-sum slot; `merges` receives one record
// per split tile.  At most max_slots pieces in all.
void split_late_tiles(std::vector<Keyed>& items, std::vector<WorkItem>& merges, int32_t G, int32_t Hkv,
                      int32_t slots, int32_t max_slots) {
    auto cost = [&](const Keyed& k) { return (int64_t)k.work * G + kWorkFixedCost; };
    auto heavier = [](const Keyed& a, const Keyed& b) { return a.work > b.work; };
    int32_t used = 0;
    std::vector<int64_t> heap;
    for (int32_t round = 0; round < max_slots; ++round) {
        std::stable_sort(items.begin(), items.end(), heavier);
        int64_t total = 0, heaviest = 0, last_finish = 0;
        int32_t last_item = -1;
        heap.assign((size_t)slots, 0);  // min-heap of slot loads (all zero: already a heap)
        for (size_t i = 0; i < items.size(); ++i)
            for (int32_t g = 0; g < Hkv; ++g) {
                const int64_t c = cost(items[i]);
                std::pop_heap(heap.begin(), heap.end(), std::greater<int64_t>());
                const int64_t finish = heap.back() + c;
                heap.back() = finish;
                std::push_heap(heap.begin(), heap.end(), std::greater<int64_t>());
                total += c;
                heaviest = std::max(heaviest, c);
                if (finish > last_finish) {
                    last_finish = finish;
                    last_item = (int32_t)i;
                }
            }
        if (last_item < 0) return;
        const int64_t bound = std::max((total + slots - 1) / slots, heaviest);
        if (last_finish * 100 <= bound * (used == 0 ? 110 : 104)) return;
        Keyed& k = items[(size_t)last_item];
        if (dkdv_item_slot(k.it.w[1]) >= 0) return;  // a piece is not split again
        const int32_t n = k.it.w[4];                  // query tiles of the item
        const int32_t per = (int32_t)std::max<int64_t>(1, bound / 8 / G);
        const int32_t pieces = std::min({(n + per - 1) / per, kMaxPiecesPerTile, max_slots - used});
        if (pieces < 2) return;
        const Keyed whole = k;
        merges.push_back({{whole.it.w[0], whole.it.w[1], used, pieces, whole.it.w[3], whole.it.w[4], 0, 0}});
        int32_t at = whole.it.w[3];
        for (int32_t j = 0; j < pieces; ++j) {
            const int32_t count = n / pieces + (j < n % pieces ? 1 : 0);
            Keyed piece = whole;
            piece.work = count;
            piece.it.w[1] = whole.it.w[1] | (used + j + 1) << 8;
            piece.it.w[3] = at;
            piece.it.w[4] = count;
            at += count;
            if (j == 0) items[(size_t)last_item] = piece;
            else items.push_back(piece);
        }
        used += pieces;
    }
}

}  // namespace

extern "C" {

const char* va_last_error(void) { return g_error; }

int va_pack_first_fit(const int32_t* lens, int32_t N, int32_t budget,
                      int32_t* bin_of_sample, int32_t* pos_in_bin, int32_t* num_bins) {
    if (N < 0 || budget < 0 || !num_bins || (N > 0 && (!lens || !bin_of_sample || !pos_in_bin)))
        return fail(VA_EINVAL, "va_pack_first_fit: null pointer or negative size");
    for (int32_t i = 0; i < N; ++i) {
        if (lens[i] < 0) return fail(VA_EINVAL, "va_pack_first_fit: lens[%d] = %d is negative", i, lens[i]);
        if (lens[i] > budget)
            return fail(VA_ESIZE, "va_pack_first_fit: lens[%d] = %d exceeds the budget %d", i, lens[i], budget);
    }
    std::vector<int32_t> free_tokens, count;
    for (int32_t i = 0; i < N; ++i) {
        size_t b = 0;
        while (b < free_tokens.size() && free_tokens[b] < lens[i]) ++b;
        if (b == free_tokens.size()) {
            free_tokens.push_back(budget);
            count.push_back(0);
        }
        free_tokens[b] -= lens[i];
        bin_of_sample[i] = (int32_t)b;
        pos_in_bin[i] = count[b]++;
    }
    *num_bins = (int32_t)free_tokens.size();
    return VA_OK;
}

int va_bin_layout(const int32_t* lens, const int32_t* prefix, int32_t n,
                  int32_t* cu_seqlens, int32_t* prefix_lens, int32_t* max_seqlen) {
    if (n < 0 || !cu_seqlens || !max_seqlen || (n > 0 && !lens) || (prefix && !prefix_lens))
        return fail(VA_EINVAL, "va_bin_layout: null pointer or negative size");
    int64_t sum = 0;
    int32_t mx = 0;
    for (int32_t s = 0; s < n; ++s) {
        if (lens[s] < 0) return fail(VA_EINVAL, "va_bin_layout: lens[%d] is negative", s);
        if (prefix && (prefix[s] < 0 || prefix[s] > lens[s]))
            return fail(VA_EINVAL, "va_bin_layout: prefix[%d] = %d outside [0, %d]", s, prefix[s], lens[s]);
        sum += lens[s];
        if (sum > INT32_MAX) return fail(VA_ESIZE, "va_bin_layout: more than 2^31-1 tokens");
        mx = std::max(mx, lens[s]);
    }
    cu_seqlens[0] = 0;
    for (int32_t s = 0; s < n; ++s) {
        cu_seqlens[s + 1] = cu_seqlens[s] + lens[s];
        if (prefix) prefix_lens[s] = prefix[s];
    }
    *max_seqlen = mx;
    return VA_OK;
}

int va_tile_shape(int32_t pass, int32_t head_dim, int32_t num_q_heads, int32_t num_kv_heads,
                  int32_t* rows, int32_t* cols) {
    if (!rows || !cols) return fail(VA_EINVAL, "va_tile_shape: null pointer");
    return tile_shape(pass, head_dim, num_q_heads, num_kv_heads, rows, cols);
}

static int check_cu(const int32_t* cu, int32_t n, const char* who) {
    if (n < 0 || !cu) return fail(VA_EINVAL, "%s: null cu_seqlens or negative num_seqs", who);
    if (cu[0] != 0) return fail(VA_EINVAL, "%s: cu_seqlens[0] = %d, expected 0", who, cu[0]);
    for (int32_t s = 0; s < n; ++s)
        if (cu[s + 1] < cu[s]) return fail(VA_EINVAL, "%s: cu_seqlens decreases at %d", who, s);
    return VA_OK;
}

int va_worklist_size(const int32_t* cu, int32_t n, int32_t pass, int32_t D,
                      int32_t Hq, int32_t Hkv, size_t* bytes) {
    if (!bytes) return fail(VA_EINVAL, "va_worklist_size: null pointer");
    int rc = check_cu(cu, n, "va_worklist_size");
    if (rc) return rc;
    int32_t rows, cols;
    rc = tile_shape(pass, D, Hq, Hkv, &rows, &cols);
    if (rc) return rc;
    int64_t items = 0;
    for (int32_t s = 0; s < n; ++s) items += (cu[s + 1] - cu[s] + rows - 1) / rows;
    // a dK/dV list may hold split key tiles: every piece is one more item, every split tile one merge record
    const int32_t extra = pass == VA_PASS_BWD_DKDV ? max_partial_slots(D, Hkv) : 0;
    if ((items + extra) * works_per_item(pass, Hq, Hkv) > INT32_MAX / 2) return fail(VA_ESIZE, "va_worklist_size: too many works");
    *bytes = (size_t)worklist_layout(pass, D, Hq, Hkv, (int32_t)items + extra, extra / 2).total_recs * sizeof(WorkItem);
    return VA_OK;
}

int va_build_worklist(const int32_t* cu, const int32_t* prefix_lens, int32_t n,
                      int32_t mask_mode, int32_t pass, int32_t D, int32_t Hq, int32_t Hkv,
                      void* host_out, size_t bytes, int32_t* num_items) {
    if (!host_out || !num_items) return fail(VA_EINVAL, "va_build_worklist: null pointer");
    if (mask_mode < VA_MASK_CAUSAL || mask_mode > VA_MASK_SLIDING_WINDOW)
        return fail(VA_EUNSUPPORTED, "va_build_worklist: unknown mask mode %d", mask_mode);
    if (mask_mode != VA_MASK_CAUSAL && !prefix_lens)
        return fail(VA_EINVAL, "va_build_worklist: prefix mask needs prefix_lens");
    size_t need;
    int rc = va_worklist_size(cu, n, pass, D, Hq, Hkv, &need);
    if (rc) return rc;
    if (bytes < need) return fail(VA_ESIZE, "va_build_worklist: buffer of %zu bytes, need %zu", bytes, need);
    int32_t bm, bn;  // rows of an item, rows of the tiles it loops over
    tile_shape(pass, D, Hq, Hkv, &bm, &bn);

    std::vector<Keyed> items;
    std::vector<WorkItem> merges;
    for (int32_t s = 0; s < n; ++s) {
        const int32_t c = cu[s], L = cu[s + 1] - c;
        int32_t P, P2;
        block_ends(prefix_lens, mask_mode, s, &P, &P2);
        if (!block_ends_valid(P, P2, L, mask_mode))
            return fail(VA_EINVAL, "va_build_worklist: block ends (%d, %d) of sample %d outside [0, %d] or out of order, or a window below 1",
                        P, P2, s, L);
        const int32_t Pm = P < 0 ? 0 : P, P2m = P2 < 0 ? 0 : P2;
        if (pass == VA_PASS_BWD_DKDV) {
            // item rows are key rows (bm), inner tiles are query tiles (bn)
            const int32_t q_tiles = (L + bn - 1) / bn;
            for (int32_t j0 = 0; j0 < L; j0 += bm) {
                int32_t first_row;  // first query row that sees key j0
                if (mask_mode == VA_MASK_CAUSAL || mask_mode == VA_MASK_SLIDING_WINDOW) first_row = j0;
                else if (j0 < Pm) first_row = 0;
                else if (mask_mode == VA_MASK_PREFIX_LM) first_row = Pm;
                else if (mask_mode == VA_MASK_THREE_BLOCK) first_row = j0 < P2m ? Pm : P2m;
                else first_row = j0;
                const int32_t qt_first = first_row / bn;
                int32_t qt_end = q_tiles;  // one past the last query tile with a row that sees a key of the tile
                if (mask_mode == VA_MASK_SLIDING_WINDOW) {
                    const int64_t last_row = std::min<int64_t>(L - 1, (int64_t)j0 + std::min(bm, L - j0) - 1 + Pm - 1);
                    qt_end = (int32_t)(last_row / bn) + 1;
                }
                WorkItem it = {{c + j0, std::min(bm, L - j0), c, qt_first, qt_end - qt_first, P2, P, L}};
                items.push_back({it.w[4], it});
            }
        } else {
            for (int32_t r0 = 0; r0 < L; r0 += bm) {
                const int32_t rows = std::min(bm, L - r0);
                const int32_t kv_len = visible(r0 + rows - 1, L, Pm, P2m, mask_mode);
                const int32_t n_tiles = (kv_len + bn - 1) / bn;
                const int32_t n_full = visible(r0, L, Pm, P2m, mask_mode) / bn;
                WorkItem it = {{c + r0, rows, c, P2, n_full, n_tiles, P, L}};
                // under the sliding window the key tiles below the first row's window are not visited
                items.push_back({n_tiles - first_visible(r0, Pm, mask_mode) / bn, it});
            }
        }
    }
    if (pass == VA_PASS_BWD_DKDV)
        split_late_tiles(items, merges, Hq / Hkv, Hkv, persistent_workgroups(pass, D), max_partial_slots(D, Hkv));
    std::stable_sort(items.begin(), items.end(), [](const Keyed& a, const Keyed& b) { return a.work > b.work; });
    const WorklistLayout lay = worklist_layout(pass, D, Hq, Hkv, (int32_t)items.size(), (int32_t)merges.size());
    WorkItem* out = static_cast<WorkItem*>(host_out);
    std::memset(out, 0, need);
    out[0] = {{kWorklistMagic, pass, bm, bn, D, mask_mode, lay.num_items, cu[n]}};
    out[1] = {{lay.num_workgroups, lay.num_works, lay.works_per_item, 0 /* flags, set below */, lay.table_rec, lay.id_rec,
               lay.total_recs, lay.num_merges}};
    for (size_t i = 0; i < items.size(); ++i) out[lay.item_rec + i] = items[i].it;
    for (size_t i = 0; i < merges.size(); ++i) out[lay.merge_rec + i] = merges[i];

    // Assignment of the works to the persistent workgroups.  cost(work) = its inner-loop steps plus a fixed
    // part; items are sorted by cost and every work of an item costs the same, so id order is cost order.
    const int32_t G = Hq / Hkv;
    const int32_t P = lay.num_workgroups;
    std::vector<int64_t> load((size_t)P, 0);
    std::vector<std::vector<int32_t>> mine((size_t)P);
    auto cost_of = [&](int32_t id) {
        return (int64_t)items[id / lay.works_per_item].work * (pass == VA_PASS_BWD_DKDV ? G : 1) + kWorkFixedCost;
    };
    // Where every query tile of a sample costs the same (no causal structure: whole samples visible), the
    // plain order below already walks the tiles of a sample one after the other, i.e. is local by itself.
    bool tiles_differ = false;
    {
        std::map<int32_t, int32_t> cost_of_sample;  // first row of the sample -> cost of the first of its items seen
        for (const Keyed& k : items) {
            const auto at = cost_of_sample.emplace(k.it.w[2], k.work).first;
            tiles_differ = tiles_differ || at->second != k.work;
        }
    }
    if (tiles_differ && pass != VA_PASS_BWD_DKDV && P % kXcds == 0) {
        // Forward and dQ: all works of one (sample, KV head) stream the same K and V rows.  Workgroup b runs
        // on XCD b % 8, and each XCD has an L2 of its own, so those works are given to workgroups of one XCD
        // and placed at about the same position of their queues: they then run at about the same time and
        // the rows are fetched into that L2 once instead of once per work.  Groups go to the XCDs, and
        // the works of a group to the workgroups of its XCD, longest processing time first; groups heavier
        // than a sixteenth of an XCD's share are cut into runs of consecutive query tiles first, so that
        // few heavy groups (one KV head, long samples) still balance.
        struct Group {
            int64_t cost = 0;
            std::vector<int32_t> works;
        };
        const int32_t chunks_per_head = lay.works_per_item / Hkv;  // head chunks that share one KV head
        int64_t total = 0;
        for (int32_t id = 0; id < lay.num_works; ++id) total += cost_of(id);
        const int64_t cap = std::max<int64_t>(1, total / (kXcds * 16));
        std::vector<Group> groups;
        {
            std::map<std::pair<int32_t, int32_t>, int32_t> open;  // (sample's first row, KV head) -> its current group
            for (int32_t id = 0; id < lay.num_works; ++id) {
                const int32_t g = (id % lay.works_per_item) / chunks_per_head;
                const std::pair<int32_t, int32_t> key(items[id / lay.works_per_item].it.w[2], g);
                auto at = open.find(key);
                if (at == open.end() || groups[at->second].cost + cost_of(id) > cap) {
                    open[key] = (int32_t)groups.size();
                    groups.emplace_back();
                    at = open.find(key);
                }
                groups[at->second].cost += cost_of(id);
                groups[at->second].works.push_back(id);
            }
        }
        std::vector<int32_t> order(groups.size());
        for (size_t i = 0; i < order.size(); ++i) order[i] = (int32_t)i;
        std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) { return groups[a].cost > groups[b].cost; });
        int64_t xcd_load[kXcds] = {};
        std::vector<int32_t> of_xcd[kXcds];
        for (int32_t gi : order) {
            int32_t x = 0;
            for (int32_t c = 1; c < kXcds; ++c)
                if (xcd_load[c] < xcd_load[x]) x = c;
            xcd_load[x] += groups[gi].cost;
            of_xcd[x].push_back(gi);
        }
        auto heavier = [&](int32_t a, int32_t b) { return load[a] != load[b] ? load[a] > load[b] : a > b; };
        for (int32_t x = 0; x < kXcds; ++x) {
            std::vector<int32_t> heap;  // min-heap on (load, index) over the workgroups of this XCD
            for (int32_t w = x; w < P; w += kXcds) heap.push_back(w);
            for (int32_t gi : of_xcd[x])
                for (int32_t id : groups[gi].works) {
                    std::pop_heap(heap.begin(), heap.end(), heavier);
                    const int32_t w = heap.back();
                    load[w] += cost_of(id);
                    mine[w].push_back(id);
                    std::push_heap(heap.begin(), heap.end(), heavier);
                }
        }
    } else if (pass == VA_PASS_BWD_DKDV) {
        // One work per workgroup; workgroup b of the launch runs on XCD b % 8 and takes the work at position b
        // of the id array.  Item order (heaviest first) balances best but spreads the key tiles of a sample
        // over all XCDs and over the run of the kernel, so that every tile fetches the sample's Q and dO rows
        // again (measured: 3.4 times the rows on heavy-tailed lengths).  The other order keeps the tiles of
        // one (sample, KV head) on one XCD, next to each other, heaviest sample first; the kernel walks the
        // query tiles downwards, so those tiles then read the same rows at the same time.  It is taken
        // where every workgroup slot runs at least four works (with one or two works per slot the tiles of a
        // sample run at the same time in either order, and item order measured 5 % faster) and a replay of the
        // hardware's dispatch says it ends within 3 % of the item order.
        std::vector<int32_t> order((size_t)lay.num_works);
        for (int32_t id = 0; id < lay.num_works; ++id) order[id] = id;
        if (P % kXcds == 0 && lay.num_works >= 4 * P) {
            struct Group {
                int64_t cost = 0;
                std::vector<int32_t> works;
            };
            std::map<std::pair<int32_t, int32_t>, int32_t> index;  // (sample's first row, KV head) -> group
            std::vector<Group> groups;
            for (int32_t id = 0; id < lay.num_works; ++id) {
                const std::pair<int32_t, int32_t> key(items[id / lay.works_per_item].it.w[2], id % lay.works_per_item);
                auto at = index.find(key);
                if (at == index.end()) {
                    at = index.emplace(key, (int32_t)groups.size()).first;
                    groups.emplace_back();
                }
                groups[at->second].cost += cost_of(id);
                groups[at->second].works.push_back(id);
            }
            std::vector<int32_t> by_cost(groups.size());
            for (size_t i = 0; i < by_cost.size(); ++i) by_cost[i] = (int32_t)i;
            std::stable_sort(by_cost.begin(), by_cost.end(), [&](int32_t a, int32_t b) { return groups[a].cost > groups[b].cost; });
            int64_t xcd_load[kXcds] = {};
            std::vector<int32_t> queue[kXcds];
            for (int32_t gi : by_cost) {
                int32_t x = 0;
                for (int32_t c = 1; c < kXcds; ++c)
                    if (xcd_load[c] < xcd_load[x]) x = c;
                xcd_load[x] += groups[gi].cost;
                queue[x].insert(queue[x].end(), groups[gi].works.begin(), groups[gi].works.end());
            }
            // position 8 k + x is the k-th work of XCD x; an XCD that has run out takes from the end of the
            // queue that has most left
            std::vector<int32_t> local;
            size_t head[kXcds] = {}, tail[kXcds];
            for (int32_t x = 0; x < kXcds; ++x) tail[x] = queue[x].size();
            for (int32_t pos = 0; pos < lay.num_works; ++pos) {
                const int32_t x = pos % kXcds;
                if (head[x] < tail[x]) {
                    local.push_back(queue[x][head[x]++]);
                    continue;
                }
                int32_t most = -1;
                for (int32_t c = 0; c < kXcds; ++c)
                    if (head[c] < tail[c] && (most < 0 || tail[c] - head[c] > tail[most] - head[most])) most = c;
                local.push_back(queue[most][--tail[most]]);
            }
            // replay of the dispatch: every XCD hands its positions, in order, to the least-loaded of its slots
            auto finish_time = [&](const std::vector<int32_t>& ord) {
                const int32_t per_xcd = P / kXcds;
                std::vector<int64_t> heap((size_t)P, 0);  // kXcds min-heaps of per_xcd slot loads
                int64_t finish = 0;
                for (int32_t pos = 0; pos < lay.num_works; ++pos) {
                    const auto first = heap.begin() + (pos % kXcds) * per_xcd, last = first + per_xcd;
                    std::pop_heap(first, last, std::greater<int64_t>());
                    *(last - 1) += cost_of(ord[pos]);
                    finish = std::max(finish, *(last - 1));
                    std::push_heap(first, last, std::greater<int64_t>());
                }
                return finish;
            };
            if (finish_time(local) * 100 <= finish_time(order) * 103) {
                order.swap(local);
                out[1].w[3] |= kListFlagInStep;
            }
        }
        // the table is not used by this pass; it holds the order in equal runs so that it still partitions the ids
        const int32_t per = std::max(1, (lay.num_works + P - 1) / P);
        for (int32_t i = 0; i < lay.num_works; ++i) mine[i / per].push_back(order[i]);
    } else {
        // Longest processing time first: works in descending cost order (ties: ascending id), each to the
        // least-loaded workgroup (ties: lowest index).
        auto heavier = [&](int32_t a, int32_t b) { return load[a] != load[b] ? load[a] > load[b] : a > b; };
        std::vector<int32_t> heap((size_t)P);
        for (int32_t w = 0; w < P; ++w) heap[w] = w;  // min-heap on (load, index); all loads 0: already a heap
        for (int32_t id = 0; id < lay.num_works; ++id) {
            std::pop_heap(heap.begin(), heap.end(), heavier);
            const int32_t w = heap.back();
            load[w] += cost_of(id);
            mine[w].push_back(id);
            std::push_heap(heap.begin(), heap.end(), heavier);
        }
    }
    int32_t* table = out[lay.table_rec].w;
    int32_t* ids = out[lay.id_rec].w;
    int32_t at = 0;
    for (int32_t w = 0; w < P; ++w) {
        int32_t* e = table + kTableWordsPerWorkgroup * w;
        const int32_t count = (int32_t)mine[w].size();
        for (int32_t i = 0; i < kTableWordsPerWorkgroup; ++i) e[i] = 0;
        if (count > 0) {
            const WorkItem& first = items[mine[w][0] / lay.works_per_item].it;
            for (int32_t i = 0; i < 8; ++i) e[i] = first.w[i];
            e[8] = mine[w][0];
            e[9] = mine[w][count > 1 ? 1 : 0];
        }
        e[10] = at;
        e[11] = count;
        for (int32_t id : mine[w]) ids[at++] = id;
    }
    *num_items = lay.num_items;
    return VA_OK;
}

// bfloat16 bits -> float
static inline float bf16_to_float(uint16_t b) {
    uint32_t u = (uint32_t)b << 16;
    float f;
    std::memcpy(&f, &u, 4);
    return f;
}

// Round-to-nearest-even E4M3 (OCP, "fn": no infinities, NaN = 0x7F), saturating.
static inline uint8_t encode_e4m3(float x) {
    if (std::isnan(x)) return 0x7F;
    const uint8_t sign = std::signbit(x) ? 0x80 : 0x00;
    const float a = std::fabs(x);
    if (a >= 448.0f) return sign | 0x7E;
    if (a < 0.015625f) {  // below 2^-6: subnormal spacing 2^-9; a result of 8 is the first normal
        return sign | (uint8_t)std::nearbyintf(a * 512.0f);
    }
    int e;
    const float frac = std::frexp(a, &e);  // a = frac * 2^e, frac in [0.5, 1)
    int m = (int)std::nearbyintf((frac * 2.0f - 1.0f) * 8.0f);
    e -= 1;
    if (m == 8) {
        m = 0;
        e += 1;
    }
    return sign | (uint8_t)(((e + 7) << 3) | m);
}

int va_quantize_e4m3_per_head(const uint16_t* x, int32_t T, int32_t H, int32_t D,
                              uint8_t* codes, float* descale) {
    if (T < 0 || H <= 0 || D <= 0 || !descale || (T > 0 && (!x || !codes)))
        return fail(VA_EINVAL, "va_quantize_e4m3_per_head: null pointer or bad size");
    std::vector<float> amax((size_t)H, 0.0f);
    for (int64_t t = 0; t < T; ++t)
        for (int32_t h = 0; h < H; ++h) {
            const uint16_t* row = x + ((size_t)t * H + h) * D;
            float m = amax[h];
            for (int32_t d = 0; d < D; ++d) m = std::max(m, std::fabs(bf16_to_float(row[d])));
            amax[h] = m;
        }
    for (int32_t h = 0; h < H; ++h) {
        const float s = amax[h] / 448.0f;
        descale[h] = s > 0.0f ? s : 1.0f;
    }
    for (int64_t t = 0; t < T; ++t)
        for (int32_t h = 0; h < H; ++h) {
            const size_t base = ((size_t)t * H + h) * D;
            for (int32_t d = 0; d < D; ++d) codes[base + d] = encode_e4m3(bf16_to_float(x[base + d]) / descale[h]);
        }
    return VA_OK;
}

int va_quantize_e4m3_blockwise(const uint16_t* x, const int32_t* cu_seqlens, int32_t num_seqs, int32_t H, int32_t D,
                               uint8_t* codes, float* descale_tok) {
    const char* who = "va_quantize_e4m3_blockwise";
    if (!cu_seqlens || num_seqs < 0 || H <= 0 || D <= 0) return fail(VA_EINVAL, "%s: null pointer or bad size", who);
    if (cu_seqlens[0] != 0) return fail(VA_EINVAL, "%s: cu_seqlens[0] must be 0", who);
    for (int32_t s = 0; s < num_seqs; ++s)
        if (cu_seqlens[s + 1] < cu_seqlens[s]) return fail(VA_EINVAL, "%s: cu_seqlens decreases at %d", who, s);
    const int32_t T = cu_seqlens[num_seqs];
    if (T > 0 && (!x || !codes || !descale_tok)) return fail(VA_EINVAL, "%s: null buffer", who);
    for (int32_t s = 0; s < num_seqs; ++s)
        for (int32_t r0 = cu_seqlens[s]; r0 < cu_seqlens[s + 1]; r0 += VA_FP8_BLOCK_TOKENS) {
            const int32_t r1 = std::min(cu_seqlens[s + 1], r0 + VA_FP8_BLOCK_TOKENS);
            for (int32_t h = 0; h < H; ++h) {
                float amax = 0.0f;
                for (int32_t t = r0; t < r1; ++t) {
                    const uint16_t* row = x + ((size_t)t * H + h) * D;
                    for (int32_t d = 0; d < D; ++d) amax = std::max(amax, std::fabs(bf16_to_float(row[d])));
                }
                const float sc = amax / 448.0f;
                const float descale = sc > 0.0f ? sc : 1.0f;
                for (int32_t t = r0; t < r1; ++t) {
                    const size_t base = ((size_t)t * H + h) * D;
                    descale_tok[(size_t)t * H + h] = descale;
                    for (int32_t d = 0; d < D; ++d) codes[base + d] = encode_e4m3(bf16_to_float(x[base + d]) / descale);
                }
            }
        }
    return VA_OK;
}

}  // extern "C"
