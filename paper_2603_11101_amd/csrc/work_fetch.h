// Work descriptors of the persistent kernels, fetched two works ahead.
//
// A persistent workgroup runs the works table[b] .. of the schedule one after the other.  The
// descriptor of a work sits behind two dependent loads (schedule position -> work id -> item record).
// Fetched when needed, that chain costs two memory round trips at every work switch; here the id is
// requested three works ahead and the item record two works ahead, each a whole work before its value
// is needed, so a switch never waits for memory.  What is in flight travels in one vector register:
// lanes 0..7 the item's words and lane 8 the id of the next work, lane 9 the id of the work after it.
// The table entry of a workgroup holds its first descriptor in that very form (plus the id of its second
// work and its range of schedule positions), so the kernel's first loads of Q, K and V are one round
// trip away from its start instead of three.
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

    // Reads the table entry of workgroup b: words 0..7 the item of its first work, 8 that work's id, 9 the
    // id of its second work, 10 and 11 its first schedule position and its number of works.  Returns false
    // if the workgroup has nothing to do; else `first` is its first work and the next two are on their way.
    VA_DEV bool start(int b, RowWork* first) {
        const int v = p.wg_table[kTableWordsPerWorkgroup * b + (lane & 15)];
        work = __builtin_amdgcn_readlane(v, 10);
        work_end = work + __builtin_amdgcn_readlane(v, 11);
        if (work_end <= work) return false;
        ahead = load_ahead(__builtin_amdgcn_readlane(v, 9), work + 2);
        *first = unpack(v);
        return true;
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
