// Work descriptors of the persistent kernels, fetched two works ahead.
//
// A persistent workgroup runs the works table[b] .. of the schedule one after the other.  The
// descriptor of a work sits behind two dependent loads (schedule position -> work id -> item record).
// Fetched when needed, that chain costs two memory round trips at every work switch; here the id is
// requested three works ahead and the item record two works ahead, each a whole work before its value
// is needed, so a switch never waits for memory.  What is in flight travels in one vector register:
// lanes 0..7 the item's words and lane 8 the id of the next work, lane 9 the id of the work after it.
#pragma once

#include "kernels.h"
#include "mfma_util.h"

namespace va {

// One work of the forward or dQ kernel: an item and the query heads the workgroup stacks (all wave-uniform).
struct RowWork {
    int q_row0, q_rows, seq_row0, P2, n_full, n_tiles, P, L, g, h0;
};

template <int HPB>
struct RowWorkStream {
    const AttnParams& p;
    int lane;
    int work, work_end;  // schedule positions of the current work and past the last one
    int ahead;           // lanes 0..8: descriptor of work + 1; lane 9: id of work + 2

    // descriptor of the work with this id (wave-uniform) in lanes 0..8, id of schedule position `pos` in lane 9
    VA_DEV int load_ahead(int id, int pos) const {
        const int32_t* words = p.items[id / p.works_per_item].w;
        const int32_t* src = lane < 8 ? words + lane : p.work_ids + min(pos, work_end - 1);
        const int v = lane == 8 ? id : *src;
        return v;
    }
    VA_DEV RowWork unpack(int v) const {
        const int id = __builtin_amdgcn_readlane(v, 8);
        const int hc = id % p.works_per_item;
        const int G = p.Hq / p.Hkv;
        const int chunks_per_group = G / HPB;
        RowWork w;
        w.q_row0 = __builtin_amdgcn_readlane(v, 0);
        w.q_rows = __builtin_amdgcn_readlane(v, 1);
        w.seq_row0 = __builtin_amdgcn_readlane(v, 2);
        w.P2 = __builtin_amdgcn_readlane(v, 3);
        w.n_full = __builtin_amdgcn_readlane(v, 4);
        w.n_tiles = __builtin_amdgcn_readlane(v, 5);
        w.P = __builtin_amdgcn_readlane(v, 6);
        w.L = __builtin_amdgcn_readlane(v, 7);
        w.g = hc / chunks_per_group;
        w.h0 = w.g * G + (hc % chunks_per_group) * HPB;
        return w;
    }

    // Positions first .. end - 1 (end > first).  Returns the first work; the next two are on their way.
    VA_DEV RowWork start(int first, int end) {
        work = first;
        work_end = end;
        const int id0 = __builtin_amdgcn_readfirstlane(p.work_ids[first]);
        const int id1 = __builtin_amdgcn_readfirstlane(p.work_ids[min(first + 1, end - 1)]);
        const int cur_v = load_ahead(id0, first);
        ahead = load_ahead(id1, first + 2);
        return unpack(cur_v);
    }
    VA_DEV bool has_next() const { return work + 1 < work_end; }
    // Call once at the top of every work: returns the descriptor of work + 1 (meaningless unless
    // has_next()) and requests what lies further ahead.
    VA_DEV RowWork peek_next() {
        const RowWork nxt = unpack(ahead);
        ahead = load_ahead(__builtin_amdgcn_readlane(ahead, 9), work + 3);
        return nxt;
    }
    VA_DEV void advance() { ++work; }
};

}  // namespace va
