// Shared declarations of the library's translation units (host side).
#pragma once

#include <cstdarg>
#include <cstdint>
#include <cstdio>

#include "../../include/varlen_attn.h"

namespace va {

// One work-list record: 8 int32 words (see include/varlen_attn.h for the fields).
struct WorkItem {
    int32_t w[8];
};
static_assert(sizeof(WorkItem) == 32, "work items are 32 bytes");

constexpr int32_t kWorklistMagic = 0x56415734;  // "VAW4"

// Work-list layout, in 32-byte records:
//   record 0   {magic, pass, rows, cols, head_dim, mask_mode, num_items, total_tokens}
//   record 1   {num_workgroups, num_works, works_per_item, flags, first table record,
//               first work-id record, total records, number of merge records}
//              (items start at record 2; flags: kListFlagInStep)
//   items      num_items records, heaviest first
//   table      two records per persistent workgroup: the item of its first work; then {id of that work,
//              id of its second work, first schedule position, number of works, 0, 0, 0, 0}
//   work ids   num_works words, 8 per record: item * works_per_item + head chunk, grouped by workgroup
//   merges     (dK/dV lists only) one record per key tile whose query tiles were split over several items:
//              {kv_row0, kv_rows, first partial slot, number of pieces, qt_first, qt_count, 0, 0}
// A work is one item for one head chunk (forward, dQ: the query heads a workgroup stacks; dK/dV: one
// KV head).  The kernels are launched with num_workgroups persistent workgroups; the table is a
// longest-processing-time-first assignment of the works to them, computed on the host.
constexpr int32_t kTableWordsPerWorkgroup = 16;
// dK/dV list: workgroup b runs the work at position b of the id array (not work b): the order that keeps the
// key tiles of one (sample, KV head) next to each other on one XCD
constexpr int32_t kListFlagInStep = 1;

struct WorklistLayout {
    int32_t num_workgroups, num_works, works_per_item, num_items;
    int32_t item_rec, table_rec, id_rec, total_recs;
    int32_t num_merges, merge_rec;
    int32_t flags;  // of the list at hand (filled when a list is checked)
};

// Tile geometry.  A forward / dQ workgroup owns kFwdBlockRows rows of the
// (head, token) product: the query heads of one KV group are stacked on the
// row axis, so a group of G heads (up to 8 per workgroup) covers
// kFwdBlockRows / G token rows.  Keys are visited kFwdKvTile rows at a time.
constexpr int32_t kFwdBlockRows = 128;
constexpr int32_t kFwdKvTile = 64;
constexpr int32_t kDqBlockRows = 128;
constexpr int32_t kDqKvTile = 64;
// A dK/dV workgroup owns kDkdvKvRows key rows of one KV head and visits the
// query rows that see them kDkdvQTile rows at a time, for every head of the group.
constexpr int32_t kDkdvKvRows = 128;
// Split key tiles of the dK/dV pass.  Where a few heavy works would leave most of the chip idle at the end
// of the kernel, the host cuts the query tiles of a key tile into pieces; every piece is an item of its
// own whose workgroups write float32 partial sums of dK and dV into a slot of the caller's workspace, and
// a merge kernel adds the pieces of a tile in slot order.  Word 1 of a dK/dV item is
// kv_rows | (slot + 1) << 8, slot + 1 = 0 for an item that writes dK and dV itself.
// A slot holds dK then dV of one key tile for every KV head: Hkv * 2 * kDkdvKvRows * geometry floats.
constexpr int64_t kPartialBudgetBytes = 16 << 20;
constexpr int32_t kMinPartialSlots = 4, kMaxPartialSlots = 64, kMaxPiecesPerTile = 16;
constexpr int32_t dkdv_item_rows(int32_t w1) { return w1 & 0xff; }
constexpr int32_t dkdv_item_slot(int32_t w1) { return (w1 >> 8) - 1; }

// Head dimensions the kernels exist for, and the geometry (values per row of the LDS tiles and register
// blocks) each runs on: 80, the head dimension of the vision encoder the paper trains (section 2.2.1 (1)),
// uses the geometry of 128 with 5 of 8 contraction steps and 3 of 4 output blocks; the other values in
// between work the same way.
constexpr bool head_dim_supported(int32_t D) {
    return D == 48 || D == 64 || D == 80 || D == 96 || D == 128 || D == 160 || D == 192 || D == 256;
}
constexpr int32_t tile_geometry(int32_t D) { return D <= 64 ? 64 : D <= 128 ? 128 : 256; }
constexpr int32_t dkdv_q_tile(int32_t D) { return tile_geometry(D) >= 128 ? 32 : 64; }
constexpr int64_t partial_slot_bytes(int32_t D, int32_t Hkv) {
    return (int64_t)Hkv * 2 * kDkdvKvRows * tile_geometry(D) * (int64_t)sizeof(float);
}
constexpr int32_t max_partial_slots(int32_t D, int32_t Hkv) {
    const int64_t fit = kPartialBudgetBytes / partial_slot_bytes(D, Hkv);
    return (int32_t)(fit < kMinPartialSlots ? kMinPartialSlots : fit > kMaxPartialSlots ? kMaxPartialSlots : fit);
}

// Whether the dQ kernel computes delta = rowsum(dO * O) and LSE * log2(e) itself (and then runs before
// the dK/dV kernel, which reads both) instead of a separate pass over O and dO.
constexpr bool dq_computes_delta(int32_t D) { return D <= 128; }

// Persistent workgroups launched for a pass: CUs of an MI355X times the workgroups a CU holds.
constexpr int32_t persistent_workgroups(int32_t /*pass*/, int32_t D) { return D <= 128 ? 512 : 256; }
// XCDs of an MI355X: workgroup b of a launch runs on XCD b % kXcds, each with its own L2.
constexpr int32_t kXcds = 8;
// Cost of a work in units of inner-loop steps: its steps plus a fixed part for the item switch.
constexpr int32_t kWorkFixedCost = 2;

// Number of keys local query row i of a sample may see: length L, block ends P and P2 (values below 0
// stand for "no such boundary" and are taken as 0).
inline int32_t visible(int32_t i, int32_t L, int32_t P, int32_t P2, int32_t mode) {
    if (mode == VA_MASK_CAUSAL || mode == VA_MASK_SLIDING_WINDOW) return i + 1;
    if (i < P) return P;
    if (mode == VA_MASK_PREFIX_LM) return L;
    if (mode == VA_MASK_THREE_BLOCK) return i < P2 ? P2 : L;
    return i + 1;
}
// First key local query row i may see: 0, except under the sliding window, whose width W travels in P.
inline int32_t first_visible(int32_t i, int32_t P, int32_t mode) {
    return mode == VA_MASK_SLIDING_WINDOW && i + 1 - P > 0 ? i + 1 - P : 0;
}
// Block ends of sample s as stored in the work items (-1 where the mask has no such boundary), from the
// caller's prefix_lens: one entry per sample, or the pair (P, P2) under VA_MASK_THREE_BLOCK.
inline void block_ends(const int32_t* prefix_lens, int32_t mode, int32_t s, int32_t* P, int32_t* P2) {
    *P = -1;
    *P2 = -1;
    if (mode == VA_MASK_THREE_BLOCK) {
        *P = prefix_lens[2 * s];
        *P2 = prefix_lens[2 * s + 1];
    } else if (mode != VA_MASK_CAUSAL) {
        *P = prefix_lens[s];
    }
}
// 0 <= P <= L, and P <= P2 <= L under VA_MASK_THREE_BLOCK; a window width is at least 1
inline bool block_ends_valid(int32_t P, int32_t P2, int32_t L, int32_t mode) {
    if (mode == VA_MASK_CAUSAL) return true;
    if (mode == VA_MASK_SLIDING_WINDOW) return P >= 1;
    if (P < 0 || P > L) return false;
    return mode != VA_MASK_THREE_BLOCK || (P2 >= P && P2 <= L);
}

extern thread_local char g_error[512];
int works_per_item(int32_t pass, int32_t Hq, int32_t Hkv);
WorklistLayout worklist_layout(int32_t pass, int32_t D, int32_t Hq, int32_t Hkv, int32_t num_items, int32_t num_merges = 0);
int fail(int code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));
int heads_per_block(int32_t Hq, int32_t Hkv);
int tile_shape(int32_t pass, int32_t D, int32_t Hq, int32_t Hkv, int32_t* rows, int32_t* cols);

}  // namespace va
