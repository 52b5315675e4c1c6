// Backward, bf16: the dQ kernel (step 3 of the schedule described at the top of bwd_bf16.hip, and step 1 as
// well at head dimensions up to 128, where it computes delta and LSE * log2(e) for its own rows).  A
// translation unit of its own so that it compiles alongside the dK/dV kernel.
#include <type_traits>

#include "kernels.h"
#include "mfma_util.h"
#include "work_fetch.h"

namespace va {

namespace {

constexpr float kLog2e = 1.4426950408889634f;
constexpr int kPrefetch = 4;  // LDS fragment reads in flight ahead of the MFMA that uses them

// ------------------------------------------------------------------ dQ

using DqWork = RowWork;

// Persistent, like the forward: workgroup b runs the works the host assigned to it; the first K/V tile and
// the Q / dO fragments of the next work are fetched while the last key tile of the current one is processed.
//   FUSE   the kernel computes delta = rowsum(dO * O) and LSE * log2(e) of its own rows (every row of every
//          head belongs to exactly one work of this kernel) and writes both for the dK/dV kernel, which
//          then runs after this one; the separate pass over O and dO is not launched.
//   DR     head dimension of the tensors in memory (a multiple of 16, D / 2 < DR <= D); D is then the
//          geometry of the LDS tiles and register blocks only
// WINDOW: the sliding-window mask, as in the forward kernel (key tiles below the window of the work's first
// row are not visited, those reaching below the window of its last row carry the mask).
template <int D, int HPB, bool FUSE, int DR, bool WINDOW>
__global__ __launch_bounds__(256, D <= 128 ? 2 : 1) void bwd_dq_kernel(AttnParams p) {
    static_assert(DR % 16 == 0 && DR <= D && DR > D / 2, "head dimension and geometry do not match");
    using Rows = RowBlock<D, DR>;
    constexpr int NQ = D / 16;  // row fragments a block of rows is fetched as (the first KSTEPS are used)
    constexpr int BMT = kDqBlockRows / HPB;
    constexpr int BN = kDqKvTile;
    constexpr int KSTEPS = DR / 16;
    constexpr int DT = (DR + 31) / 32;
    constexpr int TILE_BYTES = BN * D * 2;
    static_assert(TILE_BYTES % FragAddr<D>::kTileAlign == 0 && (32 * D * 2) % FragAddr<D>::kTileAlign == 0,
                  "fragment addresses take tile and slice offsets in multiples of the tile alignment");
    constexpr int PF = D == 128 ? 2 : kPrefetch;  // fragment reads in flight; D = 128 has no registers to spare
    extern __shared__ __attribute__((aligned(16))) char smem[];  // two stages, each a K tile then a V tile

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int hf = lane >> 5, l32 = lane & 31;
    RowWorkStream<HPB> works{p, lane};
    DqWork cur;
    if (!works.start((int)blockIdx.x, &cur)) return;

    const int kv_row_bytes = p.Hkv * DR * 2;
    const int tile_step = __builtin_amdgcn_readfirstlane(BN * kv_row_bytes);
    const unsigned smem_lds = lds_addr(smem);
    AsyncTile<D, BN, 4, DR> loader;
    loader.init(wave, lane, kv_row_bytes);
    const FragAddr<D> fa(lane);
    const float c = p.scale * kLog2e;

    auto kv_rsrc = [&](const void* base, const DqWork& w) {
        return make_rsrc(static_cast<const __bf16*>(base) + ((size_t)w.seq_row0 * p.Hkv + w.g) * DR,
                         (unsigned)(w.L - 1) * kv_row_bytes + DR * 2);
    };
    // Q and dO rows of the wave's 32 stacked rows, whole rows per group of lanes (to_fragments() turns them
    // into the fragments of the row this lane owns, k-slots d = 16 t + 8 hf + 0..7), and its LSE and delta
    const int row = wave * 32 + l32;
    bf16x8 qf[NQ], dof[NQ];
    float lse2, delta;  // FUSE: lse2 holds the natural-log LSE until finish_rows() rescales it
    // Stacked row rr = wave * 32 + r is token rr % BMT of head h0 + rr / BMT; seen from the first row of
    // the work's first head, tokens past q_rows lie beyond the end of the buffer and read as zero.
    const int q_tok_bytes = p.Hq * DR * 2;
    auto block_rows = [&](const void* tensor, const DqWork& w) {
        return Rows::rows(static_cast<const __bf16*>(tensor) + ((size_t)w.q_row0 * p.Hq + w.h0) * DR,
                          (unsigned)(w.q_rows - 1) * q_tok_bytes + HPB * DR * 2);
    };
    auto block_soff = [&](int j) {
        const int rr = __builtin_amdgcn_readfirstlane(wave * 32 + j * Rows::RPI);
        return (rr % BMT) * q_tok_bytes + (rr / BMT) * (DR * 2);
    };
    // the dQ rows that leave at the end of a work: vector memory operations younger than the loads of the
    // next work's first tile
    constexpr int kEpilogueStores = Rows::N + (FUSE ? 2 : 0);
    auto load_rows = [&](const DqWork& w) {
        const int lane_off = Rows::lane_offset(lane, q_tok_bytes);
        Rows::load(qf, block_rows(p.q, w), lane_off, block_soff);
        Rows::load(dof, block_rows(p.dout, w), lane_off, block_soff);
        // LSE and delta of the row this lane owns, through raw buffers as well; the offset is derived from
        // the lane number on the spot (see RowBlock::lane_offset)
        int l = lane;
        asm volatile("" : "+v"(l));
        const int rr = wave * 32 + (l & 31), tok = rr % BMT;
        const size_t first = (size_t)w.h0 * p.T + w.q_row0;
        const unsigned bytes = (unsigned)((HPB - 1) * p.T + w.q_rows) * 4u;
        // Rows past the item aim beyond the buffer and read LSE = delta = 0 like their Q and dO rows:
        // s = 0, p = 1, dP = 0, dS = 0, so they stay finite and contribute nothing (and are never stored).
        const int off = tok < w.q_rows ? ((rr / BMT) * p.T + tok) * 4 : 0x7ffffff0;
        lse2 = __builtin_bit_cast(
            float, __builtin_amdgcn_raw_buffer_load_b32(Rows::rows((FUSE ? p.lse : p.lse2) + first, bytes), off, 0, 0));
        if constexpr (!FUSE)
            delta = -__builtin_bit_cast(  // stored negated
                float, __builtin_amdgcn_raw_buffer_load_b32(Rows::rows(p.delta + first, bytes), off, 0, 0));
    };
    // FUSE: the O rows of the block, requested where the registers of the tile loop are free
    bf16x8 of[FUSE ? NQ : 1];
    auto load_o = [&](const DqWork& w) {
        if constexpr (FUSE)
            Rows::load(of, block_rows(p.out, w), Rows::lane_offset(lane, q_tok_bytes), block_soff);
    };
    // Q, dO (and O) rows -> fragments of the row this lane owns, through the wave's LDS slice; FUSE: delta
    // from the fragments (each lane sums its half of the row, the halves meet across lane 32), LSE rescaled,
    // and both written where the dK/dV kernel reads them.  Exactly two stores when FUSE.
    auto finish_rows = [&](const DqWork& w, int slice) {
        Rows::to_fragments(qf, smem, slice, fa, lane);
        Rows::to_fragments(dof, smem, slice, fa, lane);
        if constexpr (FUSE) {
            Rows::to_fragments(of, smem, slice, fa, lane);
            // delta of row i is element (i, i) of dO O^T over the wave's 32 rows: KSTEPS MFMAs instead of
            // 16 KSTEPS conversions and multiply-adds per lane.  Lane (column i, half hf) holds rows
            // 8 (r / 4) + 4 hf + r % 4 in its registers, so the diagonal sits in register
            // 4 (i / 8) + i % 4 of the lane whose half is (i / 4) % 2; the other half contributes zero.
            f32x16 dd;
#pragma unroll
            for (int r = 0; r < 16; ++r) dd[r] = 0.0f;
#pragma unroll
            for (int t = 0; t < KSTEPS; ++t) dd = mfma32(dof[t], of[t], dd);
            int l = lane;
            asm volatile("" : "+v"(l));  // lane constants below are derived here, not kept across the kernel
            const int want = (l & 31) - 4 * (l >> 5);
            float acc = 0.0f;
#pragma unroll
            for (int r = 0; r < 16; ++r) acc = (8 * (r / 4) + r % 4 == want) ? dd[r] : acc;
            delta = acc + __shfl_xor(acc, 32);
            lse2 *= kLog2e;
            const int rr = wave * 32 + (l & 31), tok = rr % BMT;
            const size_t first = (size_t)w.h0 * p.T + w.q_row0;
            const unsigned bytes = (unsigned)((HPB - 1) * p.T + w.q_rows) * 4u;
            const int off = (tok < w.q_rows && l < 32) ? ((rr / BMT) * p.T + tok) * 4 : 0x7ffffff0;
            // the workspace holds delta negated (the dK/dV kernel starts its dP sums from it)
            __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, -delta), Rows::rows(p.delta + first, bytes), off, 0, 0);
            __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, lse2), Rows::rows(p.lse2 + first, bytes), off, 0, 0);
        }
    };
    const int slice_in_stage = wave * (32 * D * 2);  // this wave's private part of a stage

    // first key tile a work visits: 0 unless the window has moved past it
    auto first_tile = [&](const DqWork& w) {
        return WINDOW ? max(0, w.q_row0 - w.seq_row0 + 1 - w.P) / BN : 0;
    };
    int stage = 0;
    loader.issue(kv_rsrc(p.k, cur), smem_lds, first_tile(cur) * tile_step);
    loader.issue(kv_rsrc(p.v, cur), smem_lds + TILE_BYTES, first_tile(cur) * tile_step);
    load_rows(cur);
    load_o(cur);
    finish_rows(cur, 2 * TILE_BYTES + slice_in_stage);  // stage 1 is still free
    // Every ordinary load is consumed before the loop head, here and at the end of a work, so that the
    // compiler has no wait of its own to place at the top of a work, where output rows are still leaving.
    asm volatile("" ::"v"(lse2), "v"(delta));

    for (;;) {
        const bool has_next = works.has_next();
        const DqWork nxt = works.peek_next();
        const i32x4 k_rsrc = kv_rsrc(p.k, cur), v_rsrc = kv_rsrc(p.v, cur);
        const int tok = row % BMT;
        const int row_in_sample = cur.q_row0 - cur.seq_row0 + tok;
        const int vis = WINDOW ? row_in_sample + 1 : RowMask(cur.P, cur.P2, cur.L, p.mask_mode).vis(row_in_sample);
        const int lo = WINDOW ? max(0, row_in_sample + 1 - cur.P) : 0;

        f32x16 dq[DT];
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int r = 0; r < 16; ++r) dq[dt][r] = 0.0f;

#pragma unroll
        for (int t = 0; t < KSTEPS; ++t) {
            settle(qf[t]);
            settle(dof[t]);
        }
        const float my_lse2 = lse2, my_delta = delta;
        wait_async_loads_except<kEpilogueStores>();  // the first tile has landed; the last work's dQ may still be leaving
        __syncthreads();

        // One key tile; the last tile of a work is a separate instantiation that alone prefetches for the
        // next work, so the loop over the other tiles holds no ordinary global load.
        auto tile = [&](const int kt, auto last_tag, auto masked_tag) {
            constexpr bool last = decltype(last_tag)::value;
            constexpr bool need_mask = decltype(masked_tag)::value;
            const int j0 = kt * BN;
            const int k_tile = stage * 2 * TILE_BYTES;
            const int v_tile = k_tile + TILE_BYTES;
            {
                const unsigned nk = smem_lds + (stage ^ 1) * 2 * TILE_BYTES;
                if constexpr (!last) {
                    loader.issue(k_rsrc, nk, (kt + 1) * tile_step);
                    loader.issue(v_rsrc, nk + TILE_BYTES, (kt + 1) * tile_step);
                } else if (has_next) {
                    loader.issue(kv_rsrc(p.k, nxt), nk, first_tile(nxt) * tile_step);
                    loader.issue(kv_rsrc(p.v, nxt), nk + TILE_BYTES, first_tile(nxt) * tile_step);
                }
            }
            // One 32-key block at a time: S^T and dP^T (rows = key rows in registers, columns = query rows in
            // lanes), the elementwise part, then dQ^T += K^T dS^T for these 32 keys.  MFMAs alternate between
            // independent accumulators so that none waits on the one just issued.
#pragma unroll
            for (int b = 0; b < 2; ++b) {
                // A block none of the wave's rows sees (the upper half of a diagonal tile for the rows of its
                // lower half, a block wholly below the window) has P = 0 and dS = 0: its products are not issued.
                bool seen = true;
                if constexpr (need_mask) {
                    const int jb = j0 + 32 * b;
                    seen = __builtin_amdgcn_ballot_w64(vis > jb && (!WINDOW || lo < jb + 32)) != 0;
                }
                f32x16 s, dp;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    s[r] = 0.0f;
                    dp[r] = 0.0f;
                }
                if (seen) {
                    constexpr int NS = 2 * KSTEPS;  // step i: product i % 2 (0: S from K, 1: dP from V), k-step i / 2
                    auto frag = [&](int i) { return fa.rowmajor(smem, (i % 2) ? v_tile : k_tile, b, i / 2); };
                    bf16x8 ring[PF];
#pragma unroll
                    for (int i = 0; i < PF; ++i) ring[i] = frag(i);
#pragma unroll
                    for (int i = 0; i < NS; ++i) {
                        const bf16x8 a = ring[i % PF];
                        if (i + PF < NS) ring[i % PF] = frag(i + PF);
                        if (i % 2) dp = mfma32(a, dof[i / 2], dp);
                        else s = mfma32(a, qf[i / 2], s);
                    }
#pragma unroll
                    for (int i = 0; i < PF; ++i) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
#pragma unroll
                    for (int i = 0; i < NS; ++i) {
                        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                        if (i + PF < NS) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                    }
                }
                if (b == 1) {
                    // the row fragments are free now: those of the next work can start loading
                    if constexpr (last) {
                        if (has_next) load_rows(nxt);
                    }
                }
                if (!seen) continue;
                // first K^T fragments on their way while the elementwise part runs.
                // Step i of the last product: keys 32 b + 16 (i / DT) .. + 15, dQ^T block i % DT.
                bf16x8 kring[PF];
#pragma unroll
                for (int i = 0; i < PF; ++i) kring[i] = fa.transposed(smem, k_tile, 2 * b + i / DT, i % DT);
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    float pv = __builtin_amdgcn_exp2f(__builtin_fmaf(s[r], c, -my_lse2));
                    if (need_mask && (j0 + 32 * b + acc_row(r, hf) >= vis || (WINDOW && j0 + 32 * b + acc_row(r, hf) < lo)))
                        pv = 0.0f;
                    dp[r] = pv * (dp[r] - my_delta);
                }
                bf16x8 dsb[2];
#pragma unroll
                for (int x = 0; x < 2; ++x)
                    dsb[x] = to_bf16x8(dp[8 * x], dp[8 * x + 1], dp[8 * x + 2], dp[8 * x + 3],
                                       dp[8 * x + 4], dp[8 * x + 5], dp[8 * x + 6], dp[8 * x + 7]);
                {
                    constexpr int NS = 2 * DT;
#pragma unroll
                    for (int i = 0; i < NS; ++i) {
                        const bf16x8 a = kring[i % PF];
                        if (i + PF < NS) kring[i % PF] = fa.transposed(smem, k_tile, 2 * b + (i + PF) / DT, (i + PF) % DT);
                        dq[i % DT] = mfma32(a, dsb[i / DT], dq[i % DT]);
                    }
#pragma unroll
                    for (int i = 0; i < NS; ++i) {
                        __builtin_amdgcn_sched_group_barrier(0x008, 1, 1);
                        if (i + PF < NS) __builtin_amdgcn_sched_group_barrier(0x100, 2, 1);
                    }
                }
            }
            stage ^= 1;
            if constexpr (!last) {
                wait_async_loads();
                __syncthreads();
            }
        };
        // Tiles every row of the block sees completely come first and carry no mask code at all (as a
        // run-time condition inside one tile body the mask turns into selects that every tile pays for).
        // The last tile is always treated as masked: it is the ragged one.
        {
            const int n_plain = min(cur.n_full, cur.n_tiles - 1);
            int kt = first_tile(cur);
            if constexpr (WINDOW) {
                // tiles that reach below the window of the work's last row
                const int low_end = (max(0, cur.q_row0 - cur.seq_row0 + cur.q_rows - cur.P) + BN - 1) / BN;
                for (; kt < min(low_end, cur.n_tiles - 1); ++kt) tile(kt, std::false_type{}, std::true_type{});
            }
            for (; kt < n_plain; ++kt) tile(kt, std::false_type{}, std::false_type{});
            for (; kt + 1 < cur.n_tiles; ++kt) tile(kt, std::false_type{}, std::true_type{});
            tile(cur.n_tiles - 1, std::true_type{}, std::true_type{});
        }

        // dQ leaves through the LDS stage that was just processed; every wave must be done reading it first
        __syncthreads();
        const int out_slice = (stage ^ 1) * 2 * TILE_BYTES + slice_in_stage;
        if (has_next) load_o(nxt);  // on its way while dQ is staged
        store_block_rows<D, DT>(smem + out_slice, dq, p.scale, lane, block_rows(p.dq, cur),
                            Rows::lane_offset(lane, q_tok_bytes), block_soff);
        if (!has_next) break;
        // the next Q and dO rows have arrived meanwhile; the same slice turns them into fragments
        finish_rows(nxt, out_slice);
        asm volatile("" ::"v"(lse2), "v"(delta));
        works.advance();
        cur = nxt;
    }
}

template <int D, int HPB, int DR, bool WINDOW>
hipError_t launch_dq_dhw(const AttnParams& p, hipStream_t stream, unsigned grid) {
    constexpr size_t smem = 2 * 2 * kDqKvTile * D * 2;  // two stages of (K tile, V tile)
    constexpr bool FUSE = dq_computes_delta(D);
    const hipError_t attr = VA_ALLOW_DYNAMIC_LDS((&bwd_dq_kernel<D, HPB, FUSE, DR, WINDOW>), smem);
    if (attr != hipSuccess) return attr;
    hipLaunchKernelGGL((bwd_dq_kernel<D, HPB, FUSE, DR, WINDOW>), dim3(grid), dim3(256), smem, stream, p);
    return hipGetLastError();
}

template <int D, int HPB, int DR>
hipError_t launch_dq_dh(const AttnParams& p, hipStream_t stream, unsigned grid) {
    if (p.mask_mode != VA_MASK_SLIDING_WINDOW) return launch_dq_dhw<D, HPB, DR, false>(p, stream, grid);
    return launch_dq_dhw<D, HPB, DR, true>(p, stream, grid);
}

template <int D, int DR = D>
hipError_t launch_dq_d(const AttnParams& p, hipStream_t stream) {
    const int hpb = heads_per_block(p.Hq, p.Hkv);
    const unsigned grid = (unsigned)p.num_workgroups;
    if (p.num_items == 0) return hipSuccess;
    switch (hpb) {
        case 1: return launch_dq_dh<D, 1, DR>(p, stream, grid);
        case 2: return launch_dq_dh<D, 2, DR>(p, stream, grid);
        case 4: return launch_dq_dh<D, 4, DR>(p, stream, grid);
        default: return launch_dq_dh<D, 8, DR>(p, stream, grid);
    }
}

}  // namespace

hipError_t launch_bwd_dq(const AttnParams& p, hipStream_t stream) {
    switch (p.D) {
        case 48: return launch_dq_d<64, 48>(p, stream);
        case 64: return launch_dq_d<64>(p, stream);
        case 80: return launch_dq_d<128, 80>(p, stream);
        case 96: return launch_dq_d<128, 96>(p, stream);
        case 128: return launch_dq_d<128>(p, stream);
        case 160: return launch_dq_d<256, 160>(p, stream);
        case 192: return launch_dq_d<256, 192>(p, stream);
        case 256: return launch_dq_d<256>(p, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace va
