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

constexpr int32_t kWorklistMagic = 0x56415731;  // "VAW1"

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
constexpr int32_t dkdv_q_tile(int32_t D) { return D >= 128 ? 32 : 64; }

extern thread_local char g_error[512];
int fail(int code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));
int heads_per_block(int32_t Hq, int32_t Hkv);
int tile_shape(int32_t pass, int32_t D, int32_t Hq, int32_t Hkv, int32_t* rows, int32_t* cols);

}  // namespace va
