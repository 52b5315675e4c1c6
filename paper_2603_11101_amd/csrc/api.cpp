// C-ABI device entry points: argument validation on the host, then kernel
// launches on the caller's stream.  No device allocation, no synchronisation.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <vector>

#include "kernels.h"

using namespace va;

namespace {

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int check_shape(const va_shape* s, const int32_t* cu, const int32_t* prefix_lens, const char* who) {
    if (!s || !cu) return fail(VA_EINVAL, "%s: null shape or cu_seqlens", who);
    if (s->mask_mode != VA_MASK_CAUSAL && !prefix_lens)
        return fail(VA_EINVAL, "%s: a prefix mask needs prefix_lens", who);
    if (!head_dim_supported(s->head_dim))
        return fail(VA_EUNSUPPORTED, "%s: head_dim %d not in {48,64,80,96,128,160,192,256}", who, s->head_dim);
    if (s->num_q_heads <= 0 || s->num_kv_heads <= 0 || s->num_q_heads % s->num_kv_heads != 0)
        return fail(VA_EUNSUPPORTED, "%s: num_q_heads %d is not a positive multiple of num_kv_heads %d", who,
                    s->num_q_heads, s->num_kv_heads);
    if (s->mask_mode < VA_MASK_CAUSAL || s->mask_mode > VA_MASK_SLIDING_WINDOW)
        return fail(VA_EUNSUPPORTED, "%s: unknown mask mode %d", who, s->mask_mode);
    if (s->num_seqs < 0 || s->total_tokens < 0) return fail(VA_EINVAL, "%s: negative sizes", who);
    if (cu[0] != 0) return fail(VA_EINVAL, "%s: cu_seqlens[0] = %d, expected 0", who, cu[0]);
    for (int32_t i = 0; i < s->num_seqs; ++i) {
        const int32_t L = cu[i + 1] - cu[i];
        if (L < 0) return fail(VA_EINVAL, "%s: cu_seqlens decreases at sample %d", who, i);
        if (L > s->max_seqlen)
            return fail(VA_ESIZE, "%s: sample %d has %d tokens, max_seqlen is %d", who, i, L, s->max_seqlen);
        int32_t P, P2;
        block_ends(prefix_lens, s->mask_mode, i, &P, &P2);
        if (!block_ends_valid(P, P2, L, s->mask_mode))
            return fail(VA_EINVAL, "%s: block ends (%d, %d) of sample %d outside [0, %d] or out of order, or a window below 1", who, P, P2, i, L);
    }
    if (cu[s->num_seqs] != s->total_tokens)
        return fail(VA_EINVAL, "%s: cu_seqlens ends at %d, total_tokens is %d", who, cu[s->num_seqs], s->total_tokens);
    // Element offsets are computed in size_t on the device, but the kernels address the rows of one sample
    // (and the LSE rows of one block of heads) through buffers with 32-bit byte offsets.
    if ((int64_t)s->max_seqlen * s->num_q_heads * s->head_dim * 2 >= (int64_t)1 << 31)
        return fail(VA_ESIZE, "%s: max_seqlen * num_q_heads * head_dim * 2 must stay below 2^31 bytes", who);
    if ((int64_t)s->total_tokens * 8 * 4 >= (int64_t)1 << 31)
        return fail(VA_ESIZE, "%s: total_tokens must stay below 2^26", who);
    return VA_OK;
}

// The host copy of a work list is checked against the stream it claims to
// describe: headers, every item must lie inside one sample of cu_seqlens, and
// the workgroup table must partition the works.
int check_worklist(const void* dev, const void* host, const va_shape* s, const int32_t* cu, const int32_t* prefix_lens,
                   int32_t pass, const char* who, WorklistLayout* layout) {
    if (!dev || !host) return fail(VA_EINVAL, "%s: null work list", who);
    const WorkItem* w = static_cast<const WorkItem*>(host);
    int32_t rows, cols;
    int rc = tile_shape(pass, s->head_dim, s->num_q_heads, s->num_kv_heads, &rows, &cols);
    if (rc) return rc;
    const int32_t* h = w[0].w;
    if (h[0] != kWorklistMagic || h[1] != pass || h[2] != rows || h[3] != cols || h[4] != s->head_dim ||
        h[5] != s->mask_mode || h[6] < 0 || h[7] != s->total_tokens)
        return fail(VA_EINVAL, "%s: work list header does not match this call (pass %d, tile %dx%d, head_dim %d, mask %d, T %d)",
                    who, pass, rows, cols, s->head_dim, s->mask_mode, s->total_tokens);
    const int32_t n = h[6];
    int64_t expect = 0;
    for (int32_t i = 0; i < s->num_seqs; ++i) expect += (cu[i + 1] - cu[i] + rows - 1) / rows;
    const int32_t* h1 = w[1].w;
    // split key tiles (dK/dV lists only): every piece is an item more, every split tile has a merge record
    const int32_t max_slots = pass == VA_PASS_BWD_DKDV ? max_partial_slots(s->head_dim, s->num_kv_heads) : 0;
    const int32_t num_merges = h1[7];
    if (num_merges < 0 || num_merges > max_slots / 2 || n < expect || n > expect + max_slots)
        return fail(VA_EINVAL, "%s: work list holds %d items and %d merge records, this stream has %lld tiles", who, n,
                    num_merges, (long long)expect);
    const WorklistLayout lay = worklist_layout(pass, s->head_dim, s->num_q_heads, s->num_kv_heads, n, num_merges);
    if (h1[0] != lay.num_workgroups || h1[1] != lay.num_works || h1[2] != lay.works_per_item ||
        (h1[3] & ~(pass == VA_PASS_BWD_DKDV ? kListFlagInStep : 0)) != 0 ||
        h1[4] != lay.table_rec || h1[5] != lay.id_rec || h1[6] != lay.total_recs)
        return fail(VA_EINVAL, "%s: work list schedule header does not match this call", who);
    // pieces by partial slot: first query tile, number of query tiles, first key row (-1: slot not used)
    int32_t piece_first[kMaxPartialSlots], piece_count[kMaxPartialSlots], piece_row0[kMaxPartialSlots];
    for (int32_t i = 0; i < kMaxPartialSlots; ++i) piece_row0[i] = -1;
    int32_t num_pieces = 0;
    for (int32_t i = 0; i < n; ++i) {
        const int32_t* it = w[lay.item_rec + i].w;
        const int32_t row0 = it[0], seq0 = it[2], L = it[7];
        const int32_t nrows = pass == VA_PASS_BWD_DKDV ? dkdv_item_rows(it[1]) : it[1];
        const int32_t slot = pass == VA_PASS_BWD_DKDV ? dkdv_item_slot(it[1]) : -1;
        const int32_t P = it[6], P2 = it[pass == VA_PASS_BWD_DKDV ? 5 : 3];
        // (sums in 64 bits: the words of a list that was tampered with may be anything)
        const bool ok = nrows > 0 && nrows <= rows && seq0 >= 0 && L > 0 && row0 >= seq0 &&
                        (int64_t)row0 + nrows <= (int64_t)seq0 + L && (int64_t)seq0 + L <= s->total_tokens &&
                        (row0 - seq0) % rows == 0 && it[1] >= 0 && slot < max_slots &&
                        (s->mask_mode == VA_MASK_CAUSAL ? P == -1 : block_ends_valid(P, P2, L, s->mask_mode)) &&
                        (s->mask_mode == VA_MASK_THREE_BLOCK || P2 == -1);
        if (!ok) return fail(VA_EINVAL, "%s: work item %d is out of bounds", who, i);
        // (seq0, L) must be one of the samples of cu_seqlens
        const int32_t* lo = std::lower_bound(cu, cu + s->num_seqs, seq0);
        while (lo < cu + s->num_seqs && lo[0] == seq0 && lo[1] == seq0) ++lo;  // skip empty samples at this row
        if (lo >= cu + s->num_seqs || lo[0] != seq0 || lo[1] - lo[0] != L)
            return fail(VA_EINVAL, "%s: work item %d does not match a sample of cu_seqlens", who, i);
        // the kernels take the mask from the item words alone: they must be those of this call's prefix_lens
        int32_t Ps, P2s;
        block_ends(prefix_lens, s->mask_mode, (int32_t)(lo - cu), &Ps, &P2s);
        if (P != Ps || P2 != P2s)
            return fail(VA_EINVAL, "%s: work item %d was built for other block ends (or another window) than prefix_lens holds", who, i);
        const int32_t Pm = P < 0 ? 0 : P, P2m = P2 < 0 ? 0 : P2;
        if (pass == VA_PASS_BWD_DKDV) {
            int32_t qt_end = (L + cols - 1) / cols;
            if (s->mask_mode == VA_MASK_SLIDING_WINDOW)
                qt_end = (int32_t)(std::min<int64_t>(L - 1, (int64_t)(row0 - seq0) + nrows - 1 + Pm - 1) / cols) + 1;
            const int64_t qt_last = (int64_t)it[3] + it[4];
            if (it[3] < 0 || it[4] <= 0 || (slot < 0 ? qt_last != qt_end : qt_last > qt_end))
                return fail(VA_EINVAL, "%s: work item %d has a bad query-tile range", who, i);
            if (slot >= 0) {
                if (piece_row0[slot] >= 0) return fail(VA_EINVAL, "%s: partial slot %d is used by two items", who, slot);
                piece_first[slot] = it[3];
                piece_count[slot] = it[4];
                piece_row0[slot] = row0;
                ++num_pieces;
                // the last piece of a tile must end where the whole tile ends: checked with the merge record below
                if (qt_last == qt_end) piece_count[slot] |= 1 << 30;
            }
        } else {
            const int32_t r0 = row0 - seq0;
            const int32_t kv_len = visible(r0 + nrows - 1, L, Pm, P2m, s->mask_mode);
            if (it[5] != (kv_len + cols - 1) / cols || it[4] < 0 || it[4] > visible(r0, L, Pm, P2m, s->mask_mode) / cols)
                return fail(VA_EINVAL, "%s: work item %d has a bad key range", who, i);
        }
    }
    // Merge records: the pieces of a tile occupy consecutive slots, follow each other without gap or overlap from
    // the tile's first query tile to its last, and share the tile's first key row; every piece belongs to one.
    int32_t merged = 0;
    for (int32_t m = 0; m < num_merges; ++m) {
        const int32_t* r = w[lay.merge_rec + m].w;
        const int32_t first = r[2], pieces = r[3];
        if (pieces < 2 || first < 0 || first > max_slots - pieces || dkdv_item_slot(r[1]) != -1)
            return fail(VA_EINVAL, "%s: merge record %d is out of bounds", who, m);
        int32_t at = r[4];
        for (int32_t j = 0; j < pieces; ++j) {
            const int32_t sl = first + j;
            const bool last = j == pieces - 1;
            if (piece_row0[sl] != r[0] || piece_first[sl] != at || (piece_count[sl] >> 30 & 1) != (last ? 1 : 0))
                return fail(VA_EINVAL, "%s: the pieces of merge record %d do not tile its query range", who, m);
            at += piece_count[sl] & ((1 << 30) - 1);
            piece_row0[sl] = -2;  // taken
        }
        if (at != r[4] + r[5] || dkdv_item_rows(r[1]) <= 0 || dkdv_item_rows(r[1]) > rows)
            return fail(VA_EINVAL, "%s: merge record %d has a bad range", who, m);
        merged += pieces;
    }
    if (merged != num_pieces || n - num_pieces + num_merges != expect)
        return fail(VA_EINVAL, "%s: work list holds %d items (%d pieces, %d merge records), this stream has %lld tiles", who,
                    n, num_pieces, num_merges, (long long)expect);
    const int32_t* table = w[lay.table_rec].w;
    const int32_t* ids = w[lay.id_rec].w;
    // one bit per work; the buffer belongs to the thread and only ever grows, so a launch allocates nothing
    // once the thread has seen its largest list
    thread_local std::vector<uint64_t> listed;
    const size_t words = ((size_t)lay.num_works + 63) / 64;
    if (listed.size() < words) listed.resize(words);
    std::fill(listed.begin(), listed.begin() + words, 0ull);
    for (int32_t i = 0; i < lay.num_works; ++i) {
        if (ids[i] < 0 || ids[i] >= lay.num_works) return fail(VA_EINVAL, "%s: work id %d out of range", who, i);
        uint64_t& word = listed[(size_t)ids[i] >> 6];
        const uint64_t bit = 1ull << (ids[i] & 63);
        if (word & bit) return fail(VA_EINVAL, "%s: work %d is listed twice", who, ids[i]);
        word |= bit;
    }
    int32_t at = 0;
    for (int32_t g = 0; g < lay.num_workgroups; ++g) {
        const int32_t* e = table + kTableWordsPerWorkgroup * g;
        const int32_t count = e[11];
        if (e[10] != at || count < 0 || count > lay.num_works - at)
            return fail(VA_EINVAL, "%s: workgroup table does not partition the works", who);
        if (count > 0) {  // the entry repeats the first descriptor of the workgroup: it must be the validated one
            const int32_t id0 = ids[at], id1 = ids[at + (count > 1 ? 1 : 0)];
            if (e[8] != id0 || e[9] != id1 ||
                std::memcmp(e, w[lay.item_rec + id0 / lay.works_per_item].w, 8 * sizeof(int32_t)) != 0)
                return fail(VA_EINVAL, "%s: table entry of workgroup %d does not repeat its first work", who, g);
        }
        at += count;
    }
    if (at != lay.num_works) return fail(VA_EINVAL, "%s: workgroup table does not partition the works", who);
    *layout = lay;
    layout->flags = h1[3];
    return VA_OK;
}

void set_worklist(AttnParams* p, const void* dev, const WorklistLayout& lay) {
    const WorkItem* recs = static_cast<const WorkItem*>(dev);
    p->items = recs + lay.item_rec;
    p->wg_table = recs[lay.table_rec].w;
    p->work_ids = recs[lay.id_rec].w;
    p->num_items = lay.num_items;
    p->num_workgroups = lay.num_workgroups;
    p->works_per_item = lay.works_per_item;
    p->merges = recs + lay.merge_rec;
    p->num_merges = lay.num_merges;
    p->dkdv_by_ids = (lay.flags & kListFlagInStep) ? 1 : 0;
}

int check_scale(float scale, const char* who) {
    if (!(scale > 0.0f) || !std::isfinite(scale)) return fail(VA_EINVAL, "%s: scale must be positive and finite", who);
    return VA_OK;
}

AttnParams base_params(const va_shape* s, float scale) {
    AttnParams p;
    std::memset(&p, 0, sizeof(p));
    p.T = s->total_tokens;
    p.Hq = s->num_q_heads;
    p.Hkv = s->num_kv_heads;
    p.D = s->head_dim;
    p.mask_mode = s->mask_mode;
    p.scale = scale;
    return p;
}

size_t round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// bytes of the two per-row arrays at the start of the backward workspace
size_t row_stats_bytes(const va_shape* s) {
    return 2 * round_up((size_t)s->total_tokens * (size_t)s->num_q_heads * sizeof(float), 256);
}

}  // namespace

extern "C" {

size_t varlen_attn_bwd_workspace_bytes(const va_shape* s) {
    if (!s || s->total_tokens < 0 || s->num_q_heads <= 0) return 0;
    if (s->num_kv_heads <= 0 || !head_dim_supported(s->head_dim)) return 0;
    // delta = rowsum(dO * O) and LSE * log2(e), float32 [Hq, T] each, then the partial-sum slots of split key tiles
    return row_stats_bytes(s) + (size_t)max_partial_slots(s->head_dim, s->num_kv_heads) *
                                    (size_t)partial_slot_bytes(s->head_dim, s->num_kv_heads);
}

int varlen_attn_fwd(const void* q, const void* k, const void* v,
                    const int32_t* cu_seqlens, const int32_t* prefix_lens,
                    const void* worklist, const void* worklist_host,
                    const va_shape* shape, float scale,
                    void* out, float* lse, void* stream) {
    const char* who = "varlen_attn_fwd";
    int rc = check_shape(shape, cu_seqlens, prefix_lens, who);
    if (rc) return rc;
    if ((rc = check_scale(scale, who))) return rc;
    if (shape->total_tokens == 0) return VA_OK;
    if (!q || !k || !v || !out || !lse) return fail(VA_EINVAL, "%s: null tensor pointer", who);
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out) || !aligned16(lse))
        return fail(VA_EALIGN, "%s: tensor pointers must be 16-byte aligned", who);
    WorklistLayout lay;
    if ((rc = check_worklist(worklist, worklist_host, shape, cu_seqlens, prefix_lens, VA_PASS_FWD, who, &lay))) return rc;
    AttnParams p = base_params(shape, scale);
    p.q = q;
    p.k = k;
    p.v = v;
    p.out = out;
    p.lse = lse;
    set_worklist(&p, worklist, lay);
    hipError_t e = launch_fwd_bf16(p, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return fail(VA_EHIP, "%s: launch failed: %s", who, hipGetErrorString(e));
    return VA_OK;
}

// Validation shared by the backward entry points; fills the kernel parameters.
static int prepare_bwd(const char* who, const void* q, const void* k, const void* v, const void* out, const float* lse,
                       const void* dout, const int32_t* cu_seqlens, const int32_t* prefix_lens,
                       const void* worklist_dkdv, const void* worklist_dkdv_host,
                       const void* worklist_dq, const void* worklist_dq_host,
                       const va_shape* shape, float scale, void* dq, void* dk, void* dv,
                       void* workspace, size_t workspace_bytes,
                       AttnParams* p, WorklistLayout* lay_dkdv, WorklistLayout* lay_dq, bool* empty) {
    int rc = check_shape(shape, cu_seqlens, prefix_lens, who);
    if (rc) return rc;
    if ((rc = check_scale(scale, who))) return rc;
    *empty = shape->total_tokens == 0;
    if (*empty) return VA_OK;
    if (!q || !k || !v || !out || !lse || !dout || !dq || !dk || !dv || !workspace)
        return fail(VA_EINVAL, "%s: null tensor pointer", who);
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out) || !aligned16(lse) || !aligned16(dout) ||
        !aligned16(dq) || !aligned16(dk) || !aligned16(dv))
        return fail(VA_EALIGN, "%s: tensor pointers must be 16-byte aligned", who);
    if ((reinterpret_cast<uintptr_t>(workspace) & 255u) != 0)
        return fail(VA_EALIGN, "%s: workspace must be 256-byte aligned", who);
    if (workspace_bytes < varlen_attn_bwd_workspace_bytes(shape))
        return fail(VA_ESIZE, "%s: workspace of %zu bytes, need %zu", who, workspace_bytes,
                    varlen_attn_bwd_workspace_bytes(shape));
    if ((rc = check_worklist(worklist_dkdv, worklist_dkdv_host, shape, cu_seqlens, prefix_lens, VA_PASS_BWD_DKDV, who, lay_dkdv))) return rc;
    if ((rc = check_worklist(worklist_dq, worklist_dq_host, shape, cu_seqlens, prefix_lens, VA_PASS_BWD_DQ, who, lay_dq))) return rc;
    *p = base_params(shape, scale);
    p->q = q;
    p->k = k;
    p->v = v;
    p->out = const_cast<void*>(out);
    p->lse = const_cast<float*>(lse);
    p->dout = dout;
    p->dq = dq;
    p->dk = dk;
    p->dv = dv;
    p->delta = static_cast<float*>(workspace);
    p->lse2 = reinterpret_cast<float*>(static_cast<char*>(workspace) + row_stats_bytes(shape) / 2);
    p->partials = reinterpret_cast<float*>(static_cast<char*>(workspace) + row_stats_bytes(shape));
    return VA_OK;
}

// The kernels of one backward call, on one stream, restricted to `stages`.  Where the dQ kernel computes
// delta and the rescaled LSE itself it runs first and the dK/dV kernel, which reads both, after it;
// otherwise a pass over O and dO comes first.
static hipError_t launch_backward(AttnParams* p, hipStream_t st, const void* worklist_dkdv, const WorklistLayout& lay_dkdv,
                                  const void* worklist_dq, const WorklistLayout& lay_dq, uint32_t stages) {
    hipError_t e = hipSuccess;
    const bool fused = dq_computes_delta(p->D);
    const bool dq_first = fused && (stages & VA_BWD_STAGE_DQ);
    if ((stages & VA_BWD_STAGE_DELTA) && !dq_first) e = launch_bwd_delta(*p, st);
    if (e == hipSuccess && dq_first) {
        set_worklist(p, worklist_dq, lay_dq);
        e = launch_bwd_dq(*p, st);
    }
    if (e == hipSuccess && (stages & VA_BWD_STAGE_DKDV)) {
        set_worklist(p, worklist_dkdv, lay_dkdv);
        e = launch_bwd_dkdv(*p, st);
    }
    if (e == hipSuccess && (stages & VA_BWD_STAGE_DQ) && !dq_first) {
        set_worklist(p, worklist_dq, lay_dq);
        e = launch_bwd_dq(*p, st);
    }
    return e;
}

int varlen_attn_bwd_stages(const void* q, const void* k, const void* v, const void* out, const float* lse,
                           const void* dout, const int32_t* cu_seqlens, const int32_t* prefix_lens,
                           const void* worklist_dkdv, const void* worklist_dkdv_host,
                           const void* worklist_dq, const void* worklist_dq_host,
                           const va_shape* shape, float scale,
                           void* dq, void* dk, void* dv,
                           void* workspace, size_t workspace_bytes, void* stream, uint32_t stages) {
    const char* who = "varlen_attn_bwd";
    if (stages == 0 || (stages & ~(uint32_t)VA_BWD_STAGE_ALL) != 0)
        return fail(VA_EINVAL, "%s: stages must be a non-empty combination of VA_BWD_STAGE_*", who);
    AttnParams p;
    WorklistLayout lay_dkdv, lay_dq;
    bool empty = false;
    int rc = prepare_bwd(who, q, k, v, out, lse, dout, cu_seqlens, prefix_lens, worklist_dkdv, worklist_dkdv_host,
                         worklist_dq, worklist_dq_host, shape, scale, dq, dk, dv, workspace, workspace_bytes,
                         &p, &lay_dkdv, &lay_dq, &empty);
    if (rc || empty) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const hipError_t e = launch_backward(&p, st, worklist_dkdv, lay_dkdv, worklist_dq, lay_dq, stages);
    if (e != hipSuccess) return fail(VA_EHIP, "%s: launch failed: %s", who, hipGetErrorString(e));
    return VA_OK;
}

int varlen_attn_bwd(const void* q, const void* k, const void* v, const void* out, const float* lse,
                    const void* dout, const int32_t* cu_seqlens, const int32_t* prefix_lens,
                    const void* worklist_dkdv, const void* worklist_dkdv_host,
                    const void* worklist_dq, const void* worklist_dq_host,
                    const va_shape* shape, float scale,
                    void* dq, void* dk, void* dv,
                    void* workspace, size_t workspace_bytes, void* stream) {
    return varlen_attn_bwd_stages(q, k, v, out, lse, dout, cu_seqlens, prefix_lens, worklist_dkdv, worklist_dkdv_host,
                                  worklist_dq, worklist_dq_host, shape, scale, dq, dk, dv, workspace, workspace_bytes,
                                  stream, VA_BWD_STAGE_ALL);
}

int va_bwd_has_delta_kernel(int32_t head_dim) { return dq_computes_delta(head_dim) ? 0 : 1; }

int va_check_worklist(const void* worklist_host, int32_t pass, const int32_t* cu_seqlens, const int32_t* prefix_lens,
                      const va_shape* shape) {
    const char* who = "va_check_worklist";
    if (pass != VA_PASS_FWD && pass != VA_PASS_BWD_DKDV && pass != VA_PASS_BWD_DQ)
        return fail(VA_EUNSUPPORTED, "%s: unknown pass %d", who, pass);
    int rc = check_shape(shape, cu_seqlens, prefix_lens, who);
    if (rc) return rc;
    WorklistLayout lay;
    // the device copy is not looked at by the check: the host copy stands in for it
    return check_worklist(worklist_host, worklist_host, shape, cu_seqlens, prefix_lens, pass, who, &lay);
}

int va_quantize_e4m3_per_head_device(const void* x, int32_t T, int32_t H, int32_t D, void* codes, float* descale,
                                     void* stream) {
    const char* who = "va_quantize_e4m3_per_head_device";
    if (T < 0 || H <= 0 || D <= 0 || D % 8 != 0 || !descale || (T > 0 && (!x || !codes)))
        return fail(VA_EINVAL, "%s: null pointer or bad size (D must be a multiple of 8)", who);
    if (!aligned16(x) || (reinterpret_cast<uintptr_t>(codes) & 7u) != 0 || (reinterpret_cast<uintptr_t>(descale) & 3u) != 0)
        return fail(VA_EALIGN, "%s: x must be 16-byte, codes 8-byte, descale 4-byte aligned", who);
    const hipError_t e = launch_quantize_e4m3(x, T, H, D, codes, descale, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return fail(VA_EHIP, "%s: launch failed: %s", who, hipGetErrorString(e));
    return VA_OK;
}

}  // extern "C"

namespace {

int fwd_fp8_entry(const char* who, bool blockwise, const void* q8, const void* k8, const void* v8,
                  const float* q_descale, const float* k_descale, const float* v_descale,
                  const int32_t* cu_seqlens, const int32_t* prefix_lens, const void* worklist, const void* worklist_host,
                  const va_shape* shape, float scale, void* out, float* lse, void* stream) {
    int rc = check_shape(shape, cu_seqlens, prefix_lens, who);
    if (rc) return rc;
    if (shape->head_dim != 64 && shape->head_dim != 128 && shape->head_dim != 256)
        return fail(VA_EUNSUPPORTED, "%s: head_dim %d, the FP8 forward exists for 64, 128 and 256", who, shape->head_dim);
    if ((rc = check_scale(scale, who))) return rc;
    if (shape->total_tokens == 0) return VA_OK;
    if (!q8 || !k8 || !v8 || !q_descale || !k_descale || !v_descale || !out || !lse)
        return fail(VA_EINVAL, "%s: null tensor pointer", who);
    if (!aligned16(q8) || !aligned16(k8) || !aligned16(v8) || !aligned16(out) || !aligned16(lse))
        return fail(VA_EALIGN, "%s: tensor pointers must be 16-byte aligned", who);
    if (blockwise) {
        if (((reinterpret_cast<uintptr_t>(q_descale) | reinterpret_cast<uintptr_t>(k_descale) |
              reinterpret_cast<uintptr_t>(v_descale)) & 3u) != 0)
            return fail(VA_EALIGN, "%s: descale arrays must be 4-byte aligned", who);
        // the kernel addresses the per-token descales through 32-bit byte offsets
        if ((int64_t)shape->total_tokens * shape->num_q_heads * 4 > INT32_MAX)
            return fail(VA_ESIZE, "%s: total_tokens * num_q_heads * 4 exceeds 2^31 - 1", who);
    }
    WorklistLayout lay;
    if ((rc = check_worklist(worklist, worklist_host, shape, cu_seqlens, prefix_lens, VA_PASS_FWD, who, &lay))) return rc;
    AttnParams p = base_params(shape, scale);
    p.q = q8;
    p.k = k8;
    p.v = v8;
    p.q_descale = q_descale;
    p.k_descale = k_descale;
    p.v_descale = v_descale;
    p.out = out;
    p.lse = lse;
    set_worklist(&p, worklist, lay);
    hipError_t e = launch_fwd_fp8(p, blockwise, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return fail(VA_EHIP, "%s: launch failed: %s", who, hipGetErrorString(e));
    return VA_OK;
}

}  // namespace

extern "C" {

int varlen_attn_fwd_fp8(const void* q8, const void* k8, const void* v8,
                        const float* q_descale, const float* k_descale, const float* v_descale,
                        const int32_t* cu_seqlens, const int32_t* prefix_lens,
                        const void* worklist, const void* worklist_host,
                        const va_shape* shape, float scale,
                        void* out, float* lse, void* stream) {
    return fwd_fp8_entry("varlen_attn_fwd_fp8", false, q8, k8, v8, q_descale, k_descale, v_descale, cu_seqlens,
                         prefix_lens, worklist, worklist_host, shape, scale, out, lse, stream);
}

int varlen_attn_fwd_fp8_blockwise(const void* q8, const void* k8, const void* v8,
                                  const float* q_descale_tok, const float* k_descale_tok, const float* v_descale_tok,
                                  const int32_t* cu_seqlens, const int32_t* prefix_lens,
                                  const void* worklist, const void* worklist_host,
                                  const va_shape* shape, float scale,
                                  void* out, float* lse, void* stream) {
    return fwd_fp8_entry("varlen_attn_fwd_fp8_blockwise", true, q8, k8, v8, q_descale_tok, k_descale_tok, v_descale_tok,
                         cu_seqlens, prefix_lens, worklist, worklist_host, shape, scale, out, lse, stream);
}

int va_quantize_e4m3_blockwise_device(const void* x, const int32_t* cu_seqlens, const int32_t* cu_seqlens_device,
                                      int32_t num_seqs, int32_t H, int32_t D, void* codes, float* descale_tok,
                                      void* stream) {
    const char* who = "va_quantize_e4m3_blockwise_device";
    if (!cu_seqlens || !cu_seqlens_device || num_seqs < 0 || H <= 0 || D <= 0 || D % 8 != 0)
        return fail(VA_EINVAL, "%s: null pointer or bad size (D must be a multiple of 8)", who);
    if (cu_seqlens[0] != 0) return fail(VA_EINVAL, "%s: cu_seqlens[0] must be 0", who);
    int64_t blocks = 0;
    for (int32_t s = 0; s < num_seqs; ++s) {
        if (cu_seqlens[s + 1] < cu_seqlens[s]) return fail(VA_EINVAL, "%s: cu_seqlens decreases at %d", who, s);
        blocks += (cu_seqlens[s + 1] - cu_seqlens[s] + VA_FP8_BLOCK_TOKENS - 1) / VA_FP8_BLOCK_TOKENS;
    }
    const int32_t T = cu_seqlens[num_seqs];
    if (T == 0) return VA_OK;
    if (!x || !codes || !descale_tok) return fail(VA_EINVAL, "%s: null buffer", who);
    if (!aligned16(x) || (reinterpret_cast<uintptr_t>(codes) & 7u) != 0 || (reinterpret_cast<uintptr_t>(descale_tok) & 3u) != 0 ||
        (reinterpret_cast<uintptr_t>(cu_seqlens_device) & 3u) != 0)
        return fail(VA_EALIGN, "%s: x must be 16-byte, codes 8-byte, descale_tok and cu_seqlens_device 4-byte aligned", who);
    if ((H + 3) / 4 > 65535) return fail(VA_ESIZE, "%s: more than 262140 heads", who);
    const hipError_t e = launch_quantize_e4m3_blockwise(x, cu_seqlens_device, num_seqs, T, (int32_t)blocks, H, D, codes,
                                                        descale_tok, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return fail(VA_EHIP, "%s: launch failed: %s", who, hipGetErrorString(e));
    return VA_OK;
}

}  // extern "C"
