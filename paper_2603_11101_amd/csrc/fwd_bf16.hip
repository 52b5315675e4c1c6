// Forward kernel, bf16: fused scores -> running softmax -> weighted values.
//
// What it computes (paper section 2.2.1 (1), variable-length attention on the
// valid tokens of a packed stream, and (2), packing): for every query row of a
// work item, O = softmax(scale * q K^T) V over the keys of its own sample that
// the mask lets it see, and LSE = ln sum exp(scale * q k).
//
// Shape of the work.  One workgroup (4 waves) owns 128 rows of the stacked
// (query head, token) axis: HPB heads of one KV group times 128 / HPB
// consecutive tokens of one sample, so all rows share the same K/V tiles.
// Each wave owns 32 of those rows.  Keys are visited 64 at a time; the work
// item lists how many key tiles hold a visible key, so masked tiles are never
// touched, and how many leading tiles need no mask at all.
//
// Both products are computed transposed so that a lane owns one query row
// throughout: S^T = K Q^T puts query row (lane % 32) in every accumulator
// register of the lane, the row maximum and sum are reductions over the lane's
// own registers plus one exchange with lane + 32, and O^T = V^T P^T takes P^T
// straight from those registers as its second operand.  V^T fragments come
// from the row-major LDS tile through the transposing LDS read.
#include <type_traits>

#include "kernels.h"
#include "mfma_util.h"
#include "work_fetch.h"

namespace va {

namespace {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr int kPrefetch = 4;       // LDS fragment reads in flight ahead of the MFMA that uses them
constexpr float kMaxLag = 8.0f;  // the softmax reference may trail a row's true maximum by this many powers of two

using FwdWork = RowWork;

// Persistent kernel: workgroup b runs the works the host assigned to it, one after the other.  While the
// last key tile of a work is being processed, the first K/V tile of the next work is already on its way
// into the free LDS stage and the next Q fragments are being loaded, so a work switch costs no memory
// round trip.
// D is the geometry of the LDS tiles and register blocks (64, 128 or 256 values per row); DR <= D the
// head dimension of the tensors in memory, a multiple of 16: products run over DR / 16 k-steps and
// (DR + 31) / 32 output blocks only, and the chunks of a row from DR / 8 on are neither fetched nor stored.
// WINDOW: the sliding-window mask (the P word of a work holds the width W): the keys of local row i start
// at lo(i) = max(0, i + 1 - W), the key tiles below lo(first row) are not visited, and those below
// lo(last row), rounded up to a tile, carry the mask like the diagonal ones.  A separate instantiation, so
// that the other masks pay nothing for the lower edge.
template <int D, int HPB, int DR, bool WINDOW>
__global__ __launch_bounds__(256, D <= 128 ? 2 : 1) void fwd_bf16_kernel(AttnParams p) {
    static_assert(DR % 16 == 0 && DR <= D && DR > D / 2, "head dimension and geometry do not match");
    constexpr int BMT = kFwdBlockRows / HPB;  // token rows of the work item
    constexpr int BN = kFwdKvTile;
    constexpr int KSTEPS = DR / 16;        // MFMA steps over the head dimension
    constexpr int DT = (DR + 31) / 32;     // 32-row blocks of O^T
    constexpr int NQ = D / 16;             // row fragments a block of rows is fetched as (the first KSTEPS are used)
    using Rows = RowBlock<D, DR>;
    constexpr int TILE_BYTES = BN * D * 2;
    static_assert(TILE_BYTES % FragAddr<D>::kTileAlign == 0 && (32 * D * 2) % FragAddr<D>::kTileAlign == 0,
                  "fragment addresses take tile and slice offsets in multiples of the tile alignment");
    extern __shared__ __attribute__((aligned(16))) char smem[];  // two stages, each a K tile then a V tile

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int hf = lane >> 5, l32 = lane & 31;
    RowWorkStream<HPB> works{p, lane};
    FwdWork cur;
    if (!works.start((int)blockIdx.x, &cur)) return;

    const int kv_row_bytes = p.Hkv * DR * 2;
    const int tile_step = __builtin_amdgcn_readfirstlane(BN * kv_row_bytes);
    const unsigned smem_lds = lds_addr(smem);
    AsyncTile<D, BN, 4, DR> loader;
    loader.init(wave, lane, kv_row_bytes);
    const FragAddr<D> fa(lane);
    const float c = p.scale * kLog2e;

    // K and V rows of one sample and KV head as raw buffers: rows >= L read as zero
    auto kv_rsrc = [&](const void* base, const FwdWork& w) {
        return make_rsrc(static_cast<const __bf16*>(base) + ((size_t)w.seq_row0 * p.Hkv + w.g) * DR,
                         (unsigned)(w.L - 1) * kv_row_bytes + DR * 2);
    };
    // Q rows of the wave's 32 stacked rows, whole rows per group of lanes; to_fragments() turns them into
    // the fragments of the row this lane owns (k-slots d = 16 t + 8 hf + 0..7)
    const int row = wave * 32 + l32;
    // Stacked row rr = wave * 32 + r is token rr % BMT of head h0 + rr / BMT; seen from the first row of
    // the work's first head, tokens past q_rows lie beyond the end of the buffer and read as zero.
    const int q_tok_bytes = p.Hq * DR * 2;
    auto block_rows = [&](const void* tensor, const FwdWork& w) {
        return Rows::rows(static_cast<const __bf16*>(tensor) + ((size_t)w.q_row0 * p.Hq + w.h0) * DR,
                          (unsigned)(w.q_rows - 1) * q_tok_bytes + HPB * DR * 2);
    };
    auto block_soff = [&](int j) {
        const int rr = __builtin_amdgcn_readfirstlane(wave * 32 + j * Rows::RPI);
        return (rr % BMT) * q_tok_bytes + (rr / BMT) * (DR * 2);
    };
    auto load_q = [&](bf16x8 (&qf)[NQ], const FwdWork& w) {
        Rows::load(qf, block_rows(p.q, w), Rows::lane_offset(lane, q_tok_bytes), block_soff);
    };
    // output rows and the LSE store that leave at the end of a work: vector memory operations younger than
    // the loads of the next work's first tile
    constexpr int kEpilogueStores = Rows::N + 1;
    const int slice_in_stage = wave * (32 * D * 2);  // this wave's private part of a stage

    // first key tile a work visits: 0 unless the window has moved past it
    auto first_tile = [&](const FwdWork& w) {
        return WINDOW ? max(0, w.q_row0 - w.seq_row0 + 1 - w.P) / BN : 0;
    };
    int stage = 0;  // LDS stage that holds (or will hold) the tile about to be processed
    loader.issue(kv_rsrc(p.k, cur), smem_lds, first_tile(cur) * tile_step);
    loader.issue(kv_rsrc(p.v, cur), smem_lds + TILE_BYTES, first_tile(cur) * tile_step);
    bf16x8 qf[NQ];
    load_q(qf, cur);
    Rows::to_fragments(qf, smem, 2 * TILE_BYTES + slice_in_stage, fa, lane);  // stage 1 is still free

    for (;;) {
        const bool has_next = works.has_next();
        const FwdWork nxt = works.peek_next();
        const i32x4 k_rsrc = kv_rsrc(p.k, cur), v_rsrc = kv_rsrc(p.v, cur);
        const int tok = row % BMT;
        const bool row_valid = tok < cur.q_rows;
        const int row_in_sample = cur.q_row0 - cur.seq_row0 + tok;
        const int vis = WINDOW ? row_in_sample + 1 : RowMask(cur.P, cur.P2, cur.L, p.mask_mode).vis(row_in_sample);
        const int lo = WINDOW ? max(0, row_in_sample + 1 - cur.P) : 0;

        f32x16 o[DT];
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int r = 0; r < 16; ++r) o[dt][r] = 0.0f;
        // Reference point of the exponentials, in units of scale * log2(e) * s.  It only moves when some
        // row of the wave would otherwise exceed 2^kMaxLag, so most tiles skip the rescaling of O;
        // the probabilities are then at most 2^kMaxLag instead of 1, which float32 sums and bf16 P absorb.
        float m = -INFINITY;
        float lsum = 0.0f;  // this lane's share of the running sum (other share in lane + 32)

#pragma unroll
        for (int t = 0; t < KSTEPS; ++t) settle(qf[t]);
        wait_async_loads_except<kEpilogueStores>();  // the first tile has landed; the last work's output may still be leaving
        __syncthreads();

        // One key tile.  The last tile of a work is a separate instantiation: it alone prefetches for the
        // next work, so the loop over the other tiles contains no ordinary global load and the compiler
        // has no reason to wait for memory inside it.
        auto tile = [&](const int kt, auto last_tag, auto masked_tag) {
            constexpr bool last = decltype(last_tag)::value;
            constexpr bool masked = decltype(masked_tag)::value;
            const int j0 = kt * BN;
            const int k_tile = stage * 2 * TILE_BYTES;  // byte offsets of this stage's tiles
            const int v_tile = k_tile + TILE_BYTES;
            {
                // next tile of this work, or the first tile of the next work, into the other stage
                const unsigned nk = smem_lds + (stage ^ 1) * 2 * TILE_BYTES;
                if constexpr (!last) {
                    loader.issue(k_rsrc, nk, (kt + 1) * tile_step);
                    loader.issue(v_rsrc, nk + TILE_BYTES, (kt + 1) * tile_step);
                } else if (has_next) {
                    loader.issue(kv_rsrc(p.k, nxt), nk, first_tile(nxt) * tile_step);
                    loader.issue(kv_rsrc(p.v, nxt), nk + TILE_BYTES, first_tile(nxt) * tile_step);
                }
            }

            // S^T: two blocks of 32 keys x 32 query rows.  The K fragments are fetched from LDS kPrefetch
            // steps ahead of the MFMA that consumes them; consecutive MFMAs alternate between the two
            // blocks so that none waits for the result of the one just issued.
            f32x16 s[2];
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int r = 0; r < 16; ++r) s[b][r] = 0.0f;
            {
                constexpr int NS = 2 * KSTEPS;  // step i: block i % 2, k-step i / 2
                bf16x8 ring[kPrefetch];
#pragma unroll
                for (int i = 0; i < kPrefetch; ++i) ring[i] = fa.rowmajor(smem, k_tile, i % 2, i / 2);
#pragma unroll
                for (int i = 0; i < NS; ++i) {
                    const bf16x8 a = ring[i % kPrefetch];
                    if (i + kPrefetch < NS) ring[i % kPrefetch] = fa.rowmajor(smem, k_tile, (i + kPrefetch) % 2, (i + kPrefetch) / 2);
                    s[i % 2] = mfma32(a, qf[i / 2], s[i % 2]);
                }
                // pin the issue order: kPrefetch reads up front, then one read per MFMA
#pragma unroll
                for (int i = 0; i < kPrefetch; ++i) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
#pragma unroll
                for (int i = 0; i < NS; ++i) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    if (i + kPrefetch < NS) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                }
            }
            // the Q fragments are free now: those of the next work can start loading
            if constexpr (last) {
                if (has_next) load_q(qf, nxt);
            }

            if constexpr (masked) {
#pragma unroll
                for (int b = 0; b < 2; ++b)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        if (j0 + 32 * b + acc_row(r, hf) >= vis || (WINDOW && j0 + 32 * b + acc_row(r, hf) < lo))
                            s[b][r] = -INFINITY;
            }
            // first V^T fragments on their way while the softmax runs.  Step i: keys 16 (i / DT) .. + 15,
            // O^T block i % DT, so consecutive MFMAs go to different accumulators.
            bf16x8 vring[kPrefetch];
#pragma unroll
            for (int i = 0; i < kPrefetch; ++i) vring[i] = fa.transposed(smem, v_tile, i / DT, i % DT);
            float mx = s[0][0];
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[b][r]);
            mx = pair_max(mx) * c;
            if (__builtin_amdgcn_ballot_w64(mx > m + kMaxLag) != 0) {  // wave-uniform: some row needs a new reference
                asm volatile("");  // keep this a branch: folded into a select, its multiplications would run on every tile
                const float m_new = fmaxf(m, mx);
                // m = -inf on the first tile: alpha = 0, O = 0.  Under the window a row may see no key of the
                // first tiles it visits: it keeps m = -inf and takes the reference 0 until it sees one.
                const float alpha = __builtin_amdgcn_exp2f(m - (WINDOW && m_new == -INFINITY ? 0.0f : m_new));
                m = m_new;
                lsum *= alpha;
#pragma unroll
                for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                    for (int r = 0; r < 16; ++r) o[dt][r] *= alpha;
            }
            float psum = 0.0f;
            const float m_ref = WINDOW && m == -INFINITY ? 0.0f : m;
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float pv = __builtin_amdgcn_exp2f(__builtin_fmaf(s[b][r], c, -m_ref));
                    s[b][r] = pv;
                    psum += pv;
                }
            lsum += psum;

            // P^T as second operand: registers 8 x .. 8 x + 7 of a block are the k-slots of step x
            bf16x8 pf[4];
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int x = 0; x < 2; ++x)
                    pf[2 * b + x] = to_bf16x8(s[b][8 * x + 0], s[b][8 * x + 1], s[b][8 * x + 2], s[b][8 * x + 3],
                                              s[b][8 * x + 4], s[b][8 * x + 5], s[b][8 * x + 6], s[b][8 * x + 7]);
            {
                constexpr int NS = 4 * DT;
#pragma unroll
                for (int i = 0; i < NS; ++i) {
                    const bf16x8 a = vring[i % kPrefetch];
                    if (i + kPrefetch < NS)
                        vring[i % kPrefetch] = fa.transposed(smem, v_tile, (i + kPrefetch) / DT, (i + kPrefetch) % DT);
                    o[i % DT] = mfma32(a, pf[i / DT], o[i % DT]);
                }
#pragma unroll
                for (int i = 0; i < NS; ++i) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 1);
                    if (i + kPrefetch < NS) __builtin_amdgcn_sched_group_barrier(0x100, 2, 1);
                }
            }

            stage ^= 1;
            if constexpr (!last) {
                // the next tile has landed and every wave is done reading this one
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

        lsum = pair_sum(lsum);
        // O leaves through the LDS stage that was just processed (the other one may already be receiving
        // the first tile of the next work); every wave must be done reading it first
        __syncthreads();
        const int out_slice = (stage ^ 1) * 2 * TILE_BYTES + slice_in_stage;
        store_block_rows<D, DT>(smem + out_slice, o, 1.0f / lsum, lane, block_rows(p.out, cur),
                                Rows::lane_offset(lane, q_tok_bytes), block_soff);
        {
            // LSE of the row this lane owns, from the lanes of the lower half; the others aim past the buffer
            const __amdgpu_buffer_rsrc_t lse_rows =
                Rows::rows(p.lse + (size_t)cur.h0 * p.T + cur.q_row0, (unsigned)((HPB - 1) * p.T + cur.q_rows) * 4u);
            const int off = (row_valid && hf == 0) ? ((row / BMT) * p.T + tok) * 4 : 0x7ffffff0;
            __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, (m + __builtin_amdgcn_logf(lsum)) * kLn2), lse_rows,
                                                  off, 0, 0);
        }
        if (!has_next) break;
        // the next Q rows have arrived meanwhile; the same slice turns them into fragments
        Rows::to_fragments(qf, smem, out_slice, fa, lane);
        works.advance();
        cur = nxt;
    }
}

template <int D, int HPB, int DR, bool WINDOW>
hipError_t launch_dhw(const AttnParams& p, hipStream_t stream, unsigned grid) {
    constexpr size_t smem = 2 * 2 * kFwdKvTile * D * 2;  // two stages of (K tile, V tile)
    const hipError_t attr = VA_ALLOW_DYNAMIC_LDS((&fwd_bf16_kernel<D, HPB, DR, WINDOW>), smem);
    if (attr != hipSuccess) return attr;
    hipLaunchKernelGGL((fwd_bf16_kernel<D, HPB, DR, WINDOW>), dim3(grid), dim3(256), smem, stream, p);
    return hipGetLastError();
}

template <int D, int HPB, int DR>
hipError_t launch_dh(const AttnParams& p, hipStream_t stream, unsigned grid) {
    if (p.mask_mode != VA_MASK_SLIDING_WINDOW) return launch_dhw<D, HPB, DR, false>(p, stream, grid);
    return launch_dhw<D, HPB, DR, true>(p, stream, grid);
}

template <int D, int DR = D>
hipError_t launch_d(const AttnParams& p, hipStream_t stream) {
    const int hpb = heads_per_block(p.Hq, p.Hkv);
    const unsigned grid = (unsigned)p.num_workgroups;
    if (p.num_items == 0) return hipSuccess;
    switch (hpb) {
        case 1: return launch_dh<D, 1, DR>(p, stream, grid);
        case 2: return launch_dh<D, 2, DR>(p, stream, grid);
        case 4: return launch_dh<D, 4, DR>(p, stream, grid);
        default: return launch_dh<D, 8, DR>(p, stream, grid);
    }
}

}  // namespace

hipError_t launch_fwd_bf16(const AttnParams& p, hipStream_t stream) {
    switch (p.D) {
        case 48: return launch_d<64, 48>(p, stream);
        case 64: return launch_d<64>(p, stream);
        case 80: return launch_d<128, 80>(p, stream);
        case 96: return launch_d<128, 96>(p, stream);
        case 128: return launch_d<128>(p, stream);
        case 160: return launch_d<256, 160>(p, stream);
        case 192: return launch_d<256, 192>(p, stream);
        case 256: return launch_d<256>(p, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace va
