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
#include "kernels.h"
#include "mfma_util.h"

namespace va {

namespace {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr int kPrefetch = 4;       // LDS fragment reads in flight ahead of the MFMA that uses them
constexpr float kMaxLag = 8.0f;  // the softmax reference may trail a row's true maximum by this many powers of two

template <int D, int HPB>
__global__ __launch_bounds__(256, D <= 128 ? 2 : 1) void fwd_bf16_kernel(AttnParams p) {
    constexpr int BMT = kFwdBlockRows / HPB;  // token rows of the work item
    constexpr int BN = kFwdKvTile;
    constexpr int KSTEPS = D / 16;  // MFMA steps over the head dimension
    constexpr int DT = D / 32;      // 32-row blocks of O^T
    constexpr int TILE_BYTES = BN * D * 2;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    // two stages, each a K tile followed by a V tile

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int hf = lane >> 5, l32 = lane & 31;
    const int G = p.Hq / p.Hkv;
    const int chunks_per_group = G / HPB;
    const int nhc = p.Hkv * chunks_per_group;
    const int hc = blockIdx.x % nhc;
    const WorkItem it = p.items[blockIdx.x / nhc];
    const int q_row0 = it.w[0], q_rows = it.w[1], seq_row0 = it.w[2];
    const int n_full = it.w[4], n_tiles = it.w[5], P = it.w[6], L = it.w[7];
    const int g = hc / chunks_per_group;
    const int h0 = g * G + (hc % chunks_per_group) * HPB;

    // K and V rows of this sample and KV head as raw buffers: rows >= L read as zero
    const int kv_row_bytes = p.Hkv * D * 2;
    const unsigned kv_bytes = (unsigned)(L - 1) * kv_row_bytes + D * 2;
    const i32x4 k_rsrc = make_rsrc(static_cast<const __bf16*>(p.k) + ((size_t)seq_row0 * p.Hkv + g) * D, kv_bytes);
    const i32x4 v_rsrc = make_rsrc(static_cast<const __bf16*>(p.v) + ((size_t)seq_row0 * p.Hkv + g) * D, kv_bytes);
    AsyncTile<D, BN, 4> loader;
    loader.init(wave, lane, kv_row_bytes);
    const unsigned smem_lds = lds_addr(smem);
    const int tile_step = __builtin_amdgcn_readfirstlane(BN * kv_row_bytes);

    // first K/V tile on its way before anything else
    loader.issue(k_rsrc, smem_lds, 0);
    loader.issue(v_rsrc, smem_lds + TILE_BYTES, 0);

    // the stacked row this lane owns
    const int row = wave * 32 + l32;
    const int head = h0 + row / BMT;
    const int tok = row % BMT;
    const bool row_valid = tok < q_rows;
    const int vis = RowMask(P, L, p.mask_mode).vis(q_row0 - seq_row0 + tok);

    // Q fragments stay in registers for the whole item: k-slots d = 16 t + 8 hf + 0..7
    bf16x8 qf[KSTEPS];
    {
        const __bf16* qrow = static_cast<const __bf16*>(p.q) + ((size_t)(q_row0 + tok) * p.Hq + head) * D;
#pragma unroll
        for (int t = 0; t < KSTEPS; ++t) {
            u32x4 raw = {0u, 0u, 0u, 0u};
            if (row_valid) raw = *reinterpret_cast<const u32x4*>(qrow + 16 * t + 8 * hf);
            qf[t] = __builtin_bit_cast(bf16x8, raw);
        }
    }

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
    const float c = p.scale * kLog2e;

#pragma unroll
    for (int t = 0; t < KSTEPS; ++t) settle(qf[t]);
    wait_async_loads();
    __syncthreads();

    const FragAddr<D> fa(lane);
    for (int kt = 0; kt < n_tiles; ++kt) {
        const int j0 = kt * BN;
        const int k_tile = (kt & 1) * 2 * TILE_BYTES;  // byte offsets of this stage's tiles
        const int v_tile = k_tile + TILE_BYTES;
#ifndef VA_EXP_NO_PREFETCH
        if (kt + 1 < n_tiles) {
            const unsigned nk = smem_lds + ((kt + 1) & 1) * 2 * TILE_BYTES;
            loader.issue(k_rsrc, nk, (kt + 1) * tile_step);
            loader.issue(v_rsrc, nk + TILE_BYTES, (kt + 1) * tile_step);
        }
#endif

        // S^T: two blocks of 32 keys x 32 query rows.  The K fragments are fetched from LDS kPrefetch
        // steps ahead of the MFMA that consumes them so the matrix pipe never waits on an LDS read.
        f32x16 s[2];
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) s[b][r] = 0.0f;
        {
            constexpr int NS = 2 * KSTEPS;
            bf16x8 ring[kPrefetch];
#pragma unroll
            for (int i = 0; i < kPrefetch; ++i) ring[i] = fa.rowmajor(smem, k_tile, i / KSTEPS, i % KSTEPS);
#pragma unroll
            for (int i = 0; i < NS; ++i) {
                const bf16x8 a = ring[i % kPrefetch];
                if (i + kPrefetch < NS)
                    ring[i % kPrefetch] = fa.rowmajor(smem, k_tile, (i + kPrefetch) / KSTEPS, (i + kPrefetch) % KSTEPS);
                s[i / KSTEPS] = mfma32(a, qf[i % KSTEPS], s[i / KSTEPS]);
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
        if (kt >= n_full) {
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    if (j0 + 32 * b + acc_row(r, hf) >= vis) s[b][r] = -INFINITY;
        }
        // first V^T fragments on their way while the softmax runs
        bf16x8 vring[kPrefetch];
#pragma unroll
        for (int i = 0; i < kPrefetch; ++i) 
#if defined(VA_EXP_V_ROWMAJOR)
            vring[i] = fa.rowmajor(smem, v_tile, i % 2, i / 4);
#else
            vring[i] = fa.transposed(smem, v_tile, i % 4, i / 4);
#endif

        float mx = s[0][0];
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[b][r]);
        mx = pair_max(mx) * c;
        if (__builtin_amdgcn_ballot_w64(mx > m + kMaxLag) != 0) {  // wave-uniform: some row needs a new reference
            const float m_new = fmaxf(m, mx);
            const float alpha = __builtin_amdgcn_exp2f(m - m_new);  // m = -inf on the first tile: alpha = 0, O = 0
            m = m_new;
            lsum *= alpha;
#pragma unroll
            for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                for (int r = 0; r < 16; ++r) o[dt][r] *= alpha;
        }
        float psum = 0.0f;
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
#ifdef VA_EXP_NO_EXP
                const float pv = s[b][r];
#else
                const float pv = __builtin_amdgcn_exp2f(__builtin_fmaf(s[b][r], c, -m));
#endif
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
            constexpr int NS = 4 * DT;  // step i: O^T block i / 4, keys 16 (i % 4) .. + 15
#pragma unroll
            for (int i = 0; i < NS; ++i) {
                const bf16x8 a = vring[i % kPrefetch];
                if (i + kPrefetch < NS)
                    {
#if defined(VA_EXP_V_ROWMAJOR)
                    vring[i % kPrefetch] = fa.rowmajor(smem, v_tile, (i + kPrefetch) % 2, (i + kPrefetch) / 4);
#elif defined(VA_EXP_V_NOREAD)
                    vring[i % kPrefetch] = a;
#else
                    vring[i % kPrefetch] = fa.transposed(smem, v_tile, (i + kPrefetch) % 4, (i + kPrefetch) / 4);
#endif
                }
                o[i / 4] = mfma32(a, pf[i % 4], o[i / 4]);
            }
#pragma unroll
            for (int i = 0; i < NS; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 1);
                if (i + kPrefetch < NS) __builtin_amdgcn_sched_group_barrier(0x100, 2, 1);
            }
        }

        // the next tile has landed and every wave is done reading this one
        wait_async_loads();
#ifndef VA_EXP_NO_BARRIER
        __syncthreads();
#endif
    }

    lsum = pair_sum(lsum);
    if (row_valid) {
        const float inv = 1.0f / lsum;
        __bf16* orow = static_cast<__bf16*>(p.out) + ((size_t)(q_row0 + tok) * p.Hq + head) * D;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
                f32x4 f = {o[dt][4 * r4] * inv, o[dt][4 * r4 + 1] * inv, o[dt][4 * r4 + 2] * inv, o[dt][4 * r4 + 3] * inv};
                bf16x4 h = __builtin_convertvector(f, bf16x4);
                *reinterpret_cast<bf16x4*>(orow + 32 * dt + 8 * r4 + 4 * hf) = h;
            }
        if (hf == 0) p.lse[(size_t)head * p.T + q_row0 + tok] = (m + __builtin_amdgcn_logf(lsum)) * kLn2;
    }
}

template <int D, int HPB>
hipError_t launch_dh(const AttnParams& p, hipStream_t stream, unsigned grid) {
    constexpr size_t smem = 2 * 2 * kFwdKvTile * D * 2;  // two stages of (K tile, V tile)
    static const hipError_t attr = allow_dynamic_lds(reinterpret_cast<const void*>(&fwd_bf16_kernel<D, HPB>), smem);
    if (attr != hipSuccess) return attr;
    hipLaunchKernelGGL((fwd_bf16_kernel<D, HPB>), dim3(grid), dim3(256), smem, stream, p);
    return hipGetLastError();
}

template <int D>
hipError_t launch_d(const AttnParams& p, hipStream_t stream) {
    const int G = p.Hq / p.Hkv;
    const int hpb = heads_per_block(p.Hq, p.Hkv);
    const unsigned grid = (unsigned)p.num_items * (unsigned)(p.Hkv * (G / hpb));
    if (grid == 0) return hipSuccess;
    switch (hpb) {
        case 1: return launch_dh<D, 1>(p, stream, grid);
        case 2: return launch_dh<D, 2>(p, stream, grid);
        case 4: return launch_dh<D, 4>(p, stream, grid);
        default: return launch_dh<D, 8>(p, stream, grid);
    }
}

}  // namespace

hipError_t launch_fwd_bf16(const AttnParams& p, hipStream_t stream) {
    switch (p.D) {
        case 64: return launch_d<64>(p, stream);
        case 128: return launch_d<128>(p, stream);
        case 256: return launch_d<256>(p, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace va
