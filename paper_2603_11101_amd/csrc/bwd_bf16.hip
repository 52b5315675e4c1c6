// Backward kernels, bf16.  The probabilities are recomputed from the saved LSE
// instead of being stored by the forward (paper section 2.2.1 (1) relies on the
// FlashAttention scheme for this; the schedule below is this library's own):
//
//   1. delta[h, r] = sum_d dO[r,h,d] * O[r,h,d] and LSE * log2(e).  At D <= 128 the dQ kernel
//      computes both for the rows of each of its works (it holds their dO rows anyway and fetches the
//      O rows while dQ of the previous work is being staged), so it runs first; at D = 256, where it
//      has no registers left for the O rows, a memory-bound pass of its own comes first.
//   2. dK/dV: one workgroup per (key tile of 128 rows, KV head).  The K
//      fragments of the tile stay in registers (the V fragments too at D = 64;
//      at D >= 128 the V tile stays in LDS); the workgroup walks over the
//      query tiles that see the key tile, for every query head of the group,
//      and accumulates dV^T += dO^T P and dK^T += Q^T dS in registers.
//   3. dQ: one workgroup per (query tile, head group), the mirror image of the
//      forward: walks over the visible key tiles and accumulates
//      dQ^T += K^T dS^T.
// No atomics anywhere: every output element is written by exactly one lane, so
// results do not depend on scheduling.
//
// With p = exp(scale * s - LSE):  dP = dO V^T,  dS = p * (dP - delta),
// dQ = scale * dS K,  dK = scale * dS^T Q,  dV = p^T dO.
#include <type_traits>

#include "kernels.h"
#include "mfma_util.h"
#include "work_fetch.h"

namespace va {

namespace {

constexpr float kLog2e = 1.4426950408889634f;
constexpr int kPrefetch = 4;  // LDS fragment reads in flight ahead of the MFMA that uses them

// ------------------------------------------------------------------ delta

// One group of D/8 lanes per (token, head) row; each lane multiplies 8 pairs per row and handles
// kDeltaRowsPerGroup rows, all of whose loads are issued before the first is used.
constexpr int kDeltaRowsPerGroup = 4;

// DR <= D is the head dimension in memory: the lanes of a group past DR / 8 load nothing and add zero.
template <int D, int DR>
__global__ __launch_bounds__(256) void bwd_delta_kernel(const __bf16* __restrict__ o, const __bf16* __restrict__ dout,
                                                        const float* __restrict__ lse, float* __restrict__ delta,
                                                        float* __restrict__ lse2, int T, int Hq) {
    constexpr int LPR = D / 8;  // lanes per row
    constexpr int GROUPS = 256 / LPR;
    constexpr int R = kDeltaRowsPerGroup;
    const size_t rows = (size_t)T * Hq;
    const size_t row0 = ((size_t)blockIdx.x * GROUPS + threadIdx.x / LPR) * R;
    const int c = threadIdx.x % LPR;
    bf16x8 a[R], b[R];
#pragma unroll
    for (int i = 0; i < R; ++i) {
        const size_t row = row0 + i < rows ? row0 + i : rows - 1;
        const u32x4 zero = {0u, 0u, 0u, 0u};
        a[i] = __builtin_bit_cast(bf16x8, zero);
        b[i] = __builtin_bit_cast(bf16x8, zero);
        if (DR == D || c < DR / 8) {
            a[i] = *reinterpret_cast<const bf16x8*>(o + row * DR + c * 8);
            b[i] = *reinterpret_cast<const bf16x8*>(dout + row * DR + c * 8);
        }
    }
#pragma unroll
    for (int i = 0; i < R; ++i) {
        float acc = 0.0f;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc += (float)a[i][e] * (float)b[i][e];
#pragma unroll
        for (int off = LPR / 2; off > 0; off >>= 1) acc += __shfl_xor(acc, off);
        const size_t row = row0 + i;
        if (row < rows && c == 0) {
            const size_t t = row / Hq, h = row % Hq;
            delta[h * T + t] = -acc;  // stored negated: the dK/dV kernel starts its dP sums from it
            lse2[h * T + t] = lse[h * T + t] * kLog2e;  // the other kernels work with base-2 exponentials
        }
    }
}

// ------------------------------------------------------------------ dK / dV

// What one workgroup needs to know about a dK/dV work (all wave-uniform).
struct DkdvWork {
    int kv_row0, kv_rows, seq_row0, qt_first, qt_count, P2, P, L, g;
    int slot;  // partial-sum slot of a piece of a split key tile, -1 for a work that writes dK and dV itself
};

VA_DEV DkdvWork fetch_dkdv_work(const AttnParams& p, int id) {
    const WorkItem it = p.items[id / p.works_per_item];
    DkdvWork w;
    w.kv_row0 = it.w[0];
    w.kv_rows = dkdv_item_rows(it.w[1]);
    w.slot = dkdv_item_slot(it.w[1]);
    w.seq_row0 = it.w[2];
    w.qt_first = it.w[3];
    w.qt_count = it.w[4];
    w.P2 = it.w[5];
    w.P = it.w[6];
    w.L = it.w[7];
    w.g = id % p.works_per_item;
    return w;
}

// This wave's 32 key rows of dK or dV (KV head g of the tile starting at row kv_row0), from the transposed
// accumulator through `stage` (32 * D * 2 bytes of LDS of the wave's own) out as whole rows; rows past
// kv_rows are dropped by the buffer's range check.
template <int D, int DR, int DT = (DR + 31) / 32>
VA_DEV void store_kv_rows(const AttnParams& p, char* stage, void* tensor, float factor, int kv_row0, int kv_rows, int g,
                          int wave, int lane, const f32x16 (&acc)[DT]) {
    using Rows = RowBlock<D, DR>;
    const int rows_here = min(max(kv_rows - 32 * wave, 0), 32);
    const size_t off = ((size_t)(kv_row0 + 32 * wave) * p.Hkv + g) * DR;
    const int row_bytes = p.Hkv * DR * 2;
    const unsigned bytes = rows_here > 0 ? (unsigned)(rows_here - 1) * row_bytes + DR * 2 : 0u;
    const int lane_off = Rows::lane_offset(lane, row_bytes);
    auto soff = [&](int j) { return j * Rows::RPI * row_bytes; };
    store_block_rows<D, DT>(stage, acc, factor, lane, Rows::rows(static_cast<__bf16*>(tensor) + off, bytes), lane_off, soff);
    __builtin_amdgcn_sched_barrier(0);
}
template <int D, int DR, int DT = (DR + 31) / 32>
VA_DEV void store_dkdv_rows(const AttnParams& p, char* stage, int kv_row0, int kv_rows, int g, int wave, int lane,
                            const f32x16 (&dk)[DT], const f32x16 (&dv)[DT]) {
    store_kv_rows<D, DR>(p, stage, p.dk, p.scale, kv_row0, kv_rows, g, wave, lane, dk);
    store_kv_rows<D, DR>(p, stage, p.dv, 1.0f, kv_row0, kv_rows, g, wave, lane, dv);
}

// Partial sums of a split key tile.  A slot holds, per KV head, dK then dV of the tile in the order the
// accumulators hold them: [wave][32-column block dt][register quad q][lane] float4, so that a wave
// instruction moves 1 KiB of consecutive memory.  The merge kernel reads with the same mapping.
template <int D>
VA_DEV float* partial_slot(const AttnParams& p, int slot, int g) {
    return p.partials + ((size_t)slot * p.Hkv + g) * (2 * kDkdvKvRows * D);
}
template <int D, int DT>
VA_DEV void store_partial(float* slot, int wave, int lane, const f32x16 (&dk)[DT], const f32x16 (&dv)[DT]) {
#pragma unroll
    for (int which = 0; which < 2; ++which)
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const f32x16& a = which ? dv[dt] : dk[dt];
                const f32x4 v = {a[4 * q], a[4 * q + 1], a[4 * q + 2], a[4 * q + 3]};
                float* dst = slot + which * (kDkdvKvRows * D) + ((wave * (D / 32) + dt) * 4 + q) * 256 + lane * 4;
                *reinterpret_cast<f32x4*>(dst) = v;
            }
}
// acc = (first ? 0 : acc) + one tensor (which: 0 dK, 1 dV) of one wave's share of the slot
template <int D, int DT>
VA_DEV void add_partial(const float* slot, int which, int wave, int lane, bool first, f32x16 (&acc)[DT]) {
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const float* src = slot + which * (kDkdvKvRows * D) + ((wave * (D / 32) + dt) * 4 + q) * 256 + lane * 4;
            const f32x4 v = *reinterpret_cast<const f32x4*>(src);
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[dt][4 * q + e] = first ? v[e] : acc[dt][4 * q + e] + v[e];
        }
}

// dK/dV kernel, one work per workgroup: in item order (heaviest first), or, where the list says so
// (dkdv_by_ids), in the order of its id array, which places the key tiles of one (sample, KV head) next to
// each other on one XCD.  A work is one key tile of 128 rows of
// one KV head; each wave owns 32 key rows and keeps their K fragments in registers.  The workgroup walks
// over the query tiles that see the key tile, for every query head of the group, staging Q, dO, LSE and
// delta in two LDS stages that are filled asynchronously one step ahead.  (A persistent form that
// prefetched across works kept K and both accumulators live across the switch and spilled; a two-pass
// form for D = 256, dV then dK, cost a fifth product and a second launch.)
//   V_LDS  the V rows of the key tile live in LDS (second operand of dP = dO V^T) instead of registers:
//          that buys the register room for two workgroups per CU at D = 128 and for both accumulators
//          (256 registers per lane, in the accumulation registers) at D = 256
//   DR     head dimension of the tensors in memory (a multiple of 16, D / 2 < DR <= D); D is then the
//          geometry of the LDS tiles and register blocks only
// FAMILY selects the mask code: 0 the masks with one boundary, 1 the three-block mask, 2 the sliding window
// (the P word of the work holds the width W; query rows past the window of a key block skip it, and
// blocks cut by the window's lower edge carry the mask like the diagonal ones).
template <int D, bool V_LDS, int FAMILY, int DR>
__global__ __launch_bounds__(256, D <= 128 ? 2 : 1) void bwd_dkdv_kernel(AttnParams p) {
    constexpr bool THREE = FAMILY == 1, WINDOW = FAMILY == 2;
    static_assert(DR % 16 == 0 && DR <= D && DR > D / 2, "head dimension and geometry do not match");
    constexpr bool V_IN_LDS = V_LDS, V_REGS = !V_LDS;
    constexpr int BMQ = dkdv_q_tile(D);  // query rows staged per step
    constexpr int QB = BMQ / 32;         // 32-row query blocks per step
    constexpr int KSTEPS = DR / 16;
    constexpr int DT = (DR + 31) / 32;
    constexpr int PF = D >= 128 ? 2 : kPrefetch;  // fragment reads in flight; D >= 128 has no registers to spare
    constexpr int TILE_BYTES = BMQ * D * 2;
    constexpr int STAGE_BYTES = 2 * TILE_BYTES + 2 * 64 * (int)sizeof(float);  // Q, dO, LSE2[64], delta[64]
    constexpr int AUX = 2 * STAGE_BYTES;  // V tile of the work; output staging at the end of the work
    static_assert(TILE_BYTES % FragAddr<D>::kTileAlign == 0 && STAGE_BYTES % FragAddr<D>::kTileAlign == 0,
                  "fragment addresses take tile offsets in multiples of the tile alignment");
    extern __shared__ __attribute__((aligned(16))) char smem[];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform: say so, it selects pointers and LDS slices
    const int hf = lane >> 5, l32 = lane & 31;

    const int G = p.Hq / p.Hkv;
    const float c = p.scale * kLog2e;
    const int q_row_bytes = p.Hq * DR * 2;
    const int kv_row_bytes = p.Hkv * DR * 2;
    const unsigned smem_lds = lds_addr(smem);
    AsyncTile<D, BMQ, 4, DR> loader;
    loader.init(wave, lane, q_row_bytes);
    const FragAddr<D> fa(lane);

    // Step n of a work is query tile qt_first + qt_count - 1 - n / G of head g * G + n % G.  Q and dO rows
    // of (sample, head) and the LSE / delta rows are raw buffers: anything past the sample reads as zero.
    struct StageSource {
        i32x4 q, dout, aux;  // aux: LSE rows for wave 0, delta rows for wave 1
        int qt, in_group;    // query tile (from qt_first) and head inside the group of the stage issued last
        int head;
    };
    auto head_buffers = [&](const DkdvWork& w, StageSource& src) {
        const size_t off = ((size_t)w.seq_row0 * p.Hq + src.head) * DR;
        const unsigned q_bytes = (unsigned)(w.L - 1) * q_row_bytes + DR * 2;
        src.q = make_rsrc(static_cast<const __bf16*>(p.q) + off, q_bytes);
        src.dout = make_rsrc(static_cast<const __bf16*>(p.dout) + off, q_bytes);
        src.aux = make_rsrc((wave == 0 ? p.lse2 : p.delta) + (size_t)src.head * p.T + w.seq_row0, (unsigned)w.L * 4);
    };
    // issues the stage after the one issued last (the first call issues step 0); returns its first query row
    auto issue_next_stage = [&](const DkdvWork& w, StageSource& src, int st_index) {
        // Query tiles from the last one down, every head of the group at each tile: the key tiles of one
        // sample, where they run next to each other on one XCD, then read the same Q and dO rows at about the
        // same time, whatever their number of query tiles.  One order for every list, so that the sums do not
        // depend on how a list was scheduled.
        if (++src.in_group == G) {  // counters instead of a division by the group size at every step
            src.in_group = 0;
            --src.qt;
        }
        src.head = w.g * G + src.in_group;
        head_buffers(w, src);
        const int qt = src.qt;
        const unsigned st = smem_lds + st_index * STAGE_BYTES;
        const int q0 = (w.qt_first + qt) * BMQ;
        loader.issue(src.q, st, q0 * q_row_bytes);
        loader.issue(src.dout, st + TILE_BYTES, q0 * q_row_bytes);
        if (wave < 2)  // 64 floats each: lane i fetches row q0 + i
            buffer_load_lds_4(st + 2 * TILE_BYTES + wave * 256, lane * 4, src.aux, q0 * 4);
        return q0;
    };
    auto issue_v = [&](const DkdvWork& w) {
        if (V_IN_LDS) {
            AsyncTile<D, kDkdvKvRows, 4, DR> v_loader;  // rebuilt per work: not worth registers across the step loop
            v_loader.init(wave, lane, kv_row_bytes);
            const __bf16* v_seq = static_cast<const __bf16*>(p.v) + ((size_t)w.seq_row0 * p.Hkv + w.g) * DR;
            v_loader.issue(make_rsrc(v_seq, (unsigned)(w.L - 1) * kv_row_bytes + DR * 2), smem_lds + AUX,
                           (w.kv_row0 - w.seq_row0) * kv_row_bytes);
        }
    };
    // K (and V) fragments of the lane's key row: k-slots d = 16 t + 8 hf + 0..7
    bf16x8 kf[KSTEPS], vf[V_REGS ? KSTEPS : 1];
    auto load_k = [&](const DkdvWork& w) {
        const bool valid = 32 * wave + l32 < w.kv_rows;
        const size_t off = ((size_t)(w.kv_row0 + 32 * wave + l32) * p.Hkv + w.g) * DR;
        const __bf16* krow = static_cast<const __bf16*>(p.k) + off;
        const __bf16* vrow = static_cast<const __bf16*>(p.v) + off;
#pragma unroll
        for (int t = 0; t < KSTEPS; ++t) {
            u32x4 a = {0u, 0u, 0u, 0u}, b = {0u, 0u, 0u, 0u};
            if (valid) {
                a = *reinterpret_cast<const u32x4*>(krow + 16 * t + 8 * hf);
                if (V_REGS) b = *reinterpret_cast<const u32x4*>(vrow + 16 * t + 8 * hf);
            }
            kf[t] = __builtin_bit_cast(bf16x8, a);
            if (V_REGS) vf[t] = __builtin_bit_cast(bf16x8, b);
        }
    };

    const DkdvWork cur = fetch_dkdv_work(p, p.dkdv_by_ids ? p.work_ids[blockIdx.x] : (int)blockIdx.x);
    int stage = 0;
    StageSource src;
    src.in_group = G - 1;  // the first stage wraps to head 0 of the last query tile
    src.qt = cur.qt_count;
    src.head = cur.g * G;
    head_buffers(cur, src);
    int q0_next = issue_next_stage(cur, src, 0);  // first query row of the stage in flight
    issue_v(cur);
    load_k(cur);

    {
        const int n_steps = G * cur.qt_count;
        const RowMask mask(cur.P, cur.P2, cur.L, p.mask_mode);
        const int L = cur.L;
        // keys local query row i sees: [lo_of(i), vis_of(i))
        auto vis_of = [&](int i) { return WINDOW ? i + 1 : mask.vis<THREE>(i); };
        auto lo_of = [&](int i) { return WINDOW ? max(0, i + 1 - cur.P) : 0; };
        // this wave's 32 key rows; the lane owns key row jw + l32 (local index in the sample)
        const int jw = cur.kv_row0 - cur.seq_row0 + 32 * wave;

        f32x16 dk[DT], dv[DT];
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                dk[dt][r] = 0.0f;
                dv[dt][r] = 0.0f;
            }
#pragma unroll
        for (int t = 0; t < KSTEPS; ++t) {
            settle(kf[t]);
            if (V_REGS) settle(vf[t]);
        }
        wait_async_loads();
        __syncthreads();

        // One step; the last one is a separate instantiation that prefetches nothing and ends without a barrier.
        auto step = [&](const int n, auto last_tag) {
            constexpr bool last = decltype(last_tag)::value;
            const int q0 = q0_next;
            if constexpr (!last) q0_next = issue_next_stage(cur, src, stage ^ 1);
            const int q_tile = stage * STAGE_BYTES;  // byte offsets of this stage's tiles
            const int do_tile = q_tile + TILE_BYTES;
            const float* lse_s = reinterpret_cast<const float*>(smem + q_tile + 2 * TILE_BYTES);
            const float* delta_s = lse_s + 64;
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) {
                const int i0 = q0 + 32 * qb;  // first query row of the block (local index in the sample)
                if (i0 >= L) break;
                const int i1 = min(i0 + 31, L - 1);
                if (vis_of(i1) <= jw) continue;  // nothing of this key block is visible
                if (WINDOW && lo_of(i0) >= jw + 32) continue;  // the window of every row has moved past it
                // rows past the sample read as zeros and must get p = 0: they count as seeing no key
                const bool need_mask = vis_of(i0) < jw + 32 || i0 + 32 > L || (WINDOW && lo_of(i1) > jw);

                // S = Q K^T and dP = dO V^T: rows = query rows (registers), columns = key rows (lanes).
                // MFMAs alternate between the two accumulators so that none waits on the one just issued.
                // The dP sums start from -delta of their rows (the workspace holds delta negated; registers
                // 4 r4 .. 4 r4 + 3 of the accumulator are four consecutive rows, one 16-byte read), so that
                // dP - delta comes out of the matrix unit and dS costs one multiplication per element.
                f32x16 s, dp;
#pragma unroll
                for (int r = 0; r < 16; ++r) s[r] = 0.0f;
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    const f32x4 d4 = *reinterpret_cast<const f32x4*>(delta_s + 32 * qb + 8 * r4 + 4 * hf);
#pragma unroll
                    for (int e = 0; e < 4; ++e) dp[4 * r4 + e] = d4[e];
                }
                {
                    constexpr int NS = 2 * KSTEPS;  // step i: product i % 2 (0: S, 1: dP), k-step i / 2
                    auto prod = [&](int i) { return i % 2; };
                    auto kstep = [&](int i) { return i / 2; };
                    bf16x8 ring[PF], vring[V_IN_LDS ? PF : 1];
                    auto fetch = [&](int i) {
                        ring[i % PF] = fa.rowmajor(smem, prod(i) ? do_tile : q_tile, qb, kstep(i));
                        if (V_IN_LDS && prod(i)) vring[i % PF] = fa.rowmajor(smem, AUX, wave, kstep(i));
                    };
#pragma unroll
                    for (int i = 0; i < PF; ++i) fetch(i);
#pragma unroll
                    for (int i = 0; i < NS; ++i) {
                        const bf16x8 a = ring[i % PF];
                        const bf16x8 bv = V_IN_LDS ? vring[i % PF] : vf[V_REGS ? kstep(i) : 0];
                        if (i + PF < NS) fetch(i + PF);
                        if (prod(i)) dp = mfma32(a, bv, dp);
                        else s = mfma32(a, kf[kstep(i)], s);
                    }
                    __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);  // the four reads of -delta above
#pragma unroll
                    for (int i = 0; i < PF; ++i) {
                        if (V_IN_LDS && (i % 2)) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
                        else __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                    }
#pragma unroll
                    for (int i = 0; i < NS; ++i) {
                        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                        if (i + PF < NS) {
                            if (V_IN_LDS && ((i + PF) % 2)) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
                            else __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                        }
                    }
                }
                // first transposed fragments on their way while the elementwise part runs.
                // Step i of the last products: which = i % NW (dV from dO^T, dK from Q^T), block (i / NW) % DT,
                // query rows 16 (i / (NW DT)) .. + 15 of the block.
                constexpr int NW = 2;
                constexpr int NT = 2 * DT * NW;
                auto tfrag = [&](int i) {
                    const bool is_dk = (i % NW) == 1;
                    return fa.transposed(smem, is_dk ? q_tile : do_tile, 2 * qb + i / (NW * DT), (i / NW) % DT);
                };
                bf16x8 tring[PF];
#pragma unroll
                for (int i = 0; i < PF; ++i) tring[i] = tfrag(i);

#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    const int rb = 32 * qb + 8 * r4 + 4 * hf;  // tile row of registers 4 r4 .. 4 r4 + 3
                    const f32x4 l4 = *reinterpret_cast<const f32x4*>(lse_s + rb);
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int r = 4 * r4 + e;
                        const float pv = __builtin_amdgcn_exp2f(__builtin_fmaf(s[r], c, -l4[e]));
                        s[r] = pv;
                        dp[r] = pv * dp[r];  // dp holds dP - delta
                    }
                }
                if (need_mask) {
                    // A branch of its own: folded into the loop above, the visibility arithmetic and the
                    // selects would run in every block, masked or not.  Passing the key row through an
                    // opaque statement ties everything below to this side of the branch.
                    int key = jw + l32;  // key row of this lane, local to the sample
                    asm volatile("" : "+v"(key));
                    const int row_base = q0 + 32 * qb + 4 * hf;  // query row of register 0, local to the sample
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int step = 8 * (r / 4) + r % 4;  // query row of register r is row_base + step
                        bool hidden;
                        if constexpr (WINDOW) {
                            // visible iff 0 <= row - key < W and the row lies inside the sample: one unsigned
                            // comparison on a per-lane difference, one on wave-uniform values
                            hidden = (unsigned)(row_base - key + step) >= (unsigned)cur.P || step >= L - row_base;
                        } else {
                            hidden = key >= mask.vis_in_sample<THREE>(row_base + step);
                        }
                        if (hidden) {
                            s[r] = 0.0f;
                            dp[r] = 0.0f;
                        }
                    }
                }
                bf16x8 pb[2], dsb[2];
#pragma unroll
                for (int x = 0; x < 2; ++x) {
                    pb[x] = to_bf16x8(s[8 * x], s[8 * x + 1], s[8 * x + 2], s[8 * x + 3], s[8 * x + 4], s[8 * x + 5],
                                          s[8 * x + 6], s[8 * x + 7]);
                    dsb[x] = to_bf16x8(dp[8 * x], dp[8 * x + 1], dp[8 * x + 2], dp[8 * x + 3], dp[8 * x + 4],
                                           dp[8 * x + 5], dp[8 * x + 6], dp[8 * x + 7]);
                }
                // dV^T += dO^T P ; dK^T += Q^T dS  (rows = d, columns = key rows): consecutive MFMAs go to
                // different accumulators
#pragma unroll
                for (int i = 0; i < NT; ++i) {
                    const bf16x8 a = tring[i % PF];
                    if (i + PF < NT) tring[i % PF] = tfrag(i + PF);
                    const bool is_dk = (i % NW) == 1;
                    const int dt = (i / NW) % DT, x = i / (NW * DT);
                    if (is_dk) dk[dt] = mfma32(a, dsb[x], dk[dt]);
                    else dv[dt] = mfma32(a, pb[x], dv[dt]);
                }
#pragma unroll
                for (int i = 0; i < NT; ++i) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 1);
                    if (i + PF < NT) __builtin_amdgcn_sched_group_barrier(0x100, 2, 1);
                }
            }
            stage ^= 1;
            if constexpr (!last) {
                wait_async_loads();
                __syncthreads();
            }
        };
        for (int n = 0; n + 1 < n_steps; ++n) step(n, std::false_type{});
        step(n_steps - 1, std::true_type{});

        // dK and dV leave as whole rows through the V-tile region; every wave must be done with it first
        __syncthreads();
        if (cur.slot < 0) {
            store_dkdv_rows<D, DR>(p, smem + AUX + wave * (32 * D * 2), cur.kv_row0, cur.kv_rows, cur.g, wave, lane, dk, dv);
        } else {
            // a piece of a split key tile: the accumulators as they are, float32, into its slot
            store_partial<D, DT>(partial_slot<D>(p, cur.slot, cur.g), wave, lane, dk, dv);
        }
    }
}

// Merge kernel of the split key tiles: one wave per (merge record, KV head, 32 key rows, dK or dV) adds the
// pieces of the tile in slot order, every lane the registers it would have held in the dK/dV kernel, and
// writes the rows the way that kernel does.  The order is fixed, so the sums do not depend on scheduling.
template <int D, int DR>
__global__ __launch_bounds__(64) void bwd_dkdv_merge_kernel(AttnParams p) {
    constexpr int DT = (DR + 31) / 32;
    extern __shared__ __attribute__((aligned(16))) char smem[];  // 32 * D * 2 bytes: the wave's staging slice
    const int lane = threadIdx.x;
    const int part = (int)blockIdx.x % 8, mg = (int)blockIdx.x / 8;
    const int which = part & 1, wave = part >> 1;  // the 32-row slice a wave of the dK/dV kernel owns
    const int m = mg / p.Hkv, g = mg % p.Hkv;
    const WorkItem rec = p.merges[m];
    const int kv_row0 = rec.w[0], kv_rows = dkdv_item_rows(rec.w[1]), first = rec.w[2], pieces = rec.w[3];
    f32x16 acc[DT];
    add_partial<D, DT>(partial_slot<D>(p, first, g), which, wave, lane, true, acc);
    for (int j = 1; j < pieces; ++j) add_partial<D, DT>(partial_slot<D>(p, first + j, g), which, wave, lane, false, acc);
    store_kv_rows<D, DR>(p, smem, which ? p.dv : p.dk, which ? 1.0f : p.scale, kv_row0, kv_rows, g, wave, lane, acc);
}

// One work per workgroup, in item order (heaviest first).
template <int D, int DR = D>
hipError_t launch_dkdv_d(const AttnParams& p, hipStream_t stream) {
    if (p.num_items == 0) return hipSuccess;
    constexpr bool V_LDS = D >= 128;
    // two stages of (Q tile, dO tile, LSE, delta), then the V tile / output staging region
    constexpr size_t smem = 2 * (2 * dkdv_q_tile(D) * D * 2 + 2 * 64 * sizeof(float)) + kDkdvKvRows * D * 2;
    const unsigned grid = (unsigned)(p.num_items * p.works_per_item);
    // one instantiation per mask family: the masks without a second block or a lower edge do not pay for them
    auto launch = [&](auto family) -> hipError_t {
        constexpr int FAMILY = decltype(family)::value;
        const hipError_t attr = VA_ALLOW_DYNAMIC_LDS((&bwd_dkdv_kernel<D, V_LDS, FAMILY, DR>), smem);
        if (attr != hipSuccess) return attr;
        hipLaunchKernelGGL((bwd_dkdv_kernel<D, V_LDS, FAMILY, DR>), dim3(grid), dim3(256), smem, stream, p);
        return hipSuccess;
    };
    hipError_t e;
    if (p.mask_mode == VA_MASK_THREE_BLOCK) {
        e = launch(std::integral_constant<int, 1>{});
    } else if (p.mask_mode == VA_MASK_SLIDING_WINDOW) {
        e = launch(std::integral_constant<int, 2>{});
    } else {
        e = launch(std::integral_constant<int, 0>{});
    }
    if (e != hipSuccess) return e;
    e = hipGetLastError();
    if (e != hipSuccess || p.num_merges == 0) return e;
    constexpr size_t merge_smem = 32 * D * 2;  // one staging slice
    hipLaunchKernelGGL((bwd_dkdv_merge_kernel<D, DR>), dim3((unsigned)(p.num_merges * p.Hkv * 8)), dim3(64), merge_smem, stream, p);
    return hipGetLastError();
}

template <int D, int DR = D>
hipError_t launch_delta_d(const AttnParams& p, hipStream_t stream) {
    const size_t rows = (size_t)p.T * p.Hq;
    constexpr int RPB = 256 / (D / 8) * kDeltaRowsPerGroup;
    const unsigned grid = (unsigned)((rows + RPB - 1) / RPB);
    if (grid == 0) return hipSuccess;
    hipLaunchKernelGGL((bwd_delta_kernel<D, DR>), dim3(grid), dim3(256), 0, stream, static_cast<const __bf16*>(p.out),
                       static_cast<const __bf16*>(p.dout), p.lse, p.delta, p.lse2, p.T, p.Hq);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_bwd_delta(const AttnParams& p, hipStream_t stream) {
    switch (p.D) {
        case 48: return launch_delta_d<64, 48>(p, stream);
        case 64: return launch_delta_d<64>(p, stream);
        case 80: return launch_delta_d<128, 80>(p, stream);
        case 96: return launch_delta_d<128, 96>(p, stream);
        case 128: return launch_delta_d<128>(p, stream);
        case 160: return launch_delta_d<256, 160>(p, stream);
        case 192: return launch_delta_d<256, 192>(p, stream);
        case 256: return launch_delta_d<256>(p, stream);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_bwd_dkdv(const AttnParams& p, hipStream_t stream) {
    switch (p.D) {
        case 48: return launch_dkdv_d<64, 48>(p, stream);
        case 64: return launch_dkdv_d<64>(p, stream);
        case 80: return launch_dkdv_d<128, 80>(p, stream);
        case 96: return launch_dkdv_d<128, 96>(p, stream);
        case 128: return launch_dkdv_d<128>(p, stream);
        case 160: return launch_dkdv_d<256, 160>(p, stream);
        case 192: return launch_dkdv_d<256, 192>(p, stream);
        case 256: return launch_dkdv_d<256>(p, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace va
