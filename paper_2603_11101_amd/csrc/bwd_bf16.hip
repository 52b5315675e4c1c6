// Backward kernels, bf16.  The probabilities are recomputed from the saved LSE
// instead of being stored by the forward (paper section 2.2.1 (1) relies on the
// FlashAttention scheme for this; the schedule below is this library's own):
//
//   1. delta[h, r] = sum_d dO[r,h,d] * O[r,h,d]                (memory bound)
//   2. dK/dV: one workgroup per (key tile of 128 rows, KV head).  The K and V
//      fragments of the tile stay in registers; the workgroup walks over the
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
#include "kernels.h"
#include "mfma_util.h"

namespace va {

namespace {

constexpr float kLog2e = 1.4426950408889634f;

// ------------------------------------------------------------------ delta

// One group of D/8 lanes per (token, head) row; each lane multiplies 8 pairs.
template <int D>
__global__ __launch_bounds__(256) void bwd_delta_kernel(const __bf16* __restrict__ o, const __bf16* __restrict__ dout,
                                                        const float* __restrict__ lse, float* __restrict__ delta,
                                                        float* __restrict__ lse2, int T, int Hq) {
    constexpr int LPR = D / 8;  // lanes per row
    constexpr int RPB = 256 / LPR;
    const size_t row = (size_t)blockIdx.x * RPB + threadIdx.x / LPR;
    const int c = threadIdx.x % LPR;
    const size_t rows = (size_t)T * Hq;
    float acc = 0.0f;
    if (row < rows) {
        const bf16x8 a = *reinterpret_cast<const bf16x8*>(o + row * D + c * 8);
        const bf16x8 b = *reinterpret_cast<const bf16x8*>(dout + row * D + c * 8);
#pragma unroll
        for (int e = 0; e < 8; ++e) acc += (float)a[e] * (float)b[e];
    }
#pragma unroll
    for (int off = LPR / 2; off > 0; off >>= 1) acc += __shfl_xor(acc, off);
    if (row < rows && c == 0) {
        const size_t t = row / Hq, h = row % Hq;
        delta[h * T + t] = acc;
        lse2[h * T + t] = lse[h * T + t] * kLog2e;  // the other kernels work with base-2 exponentials
    }
}

// ------------------------------------------------------------------ dK / dV

// V_LDS: the V rows of the key tile live in LDS (read as second operand of dP = dO V^T) instead of in
// registers, which buys the register room for two workgroups per CU at D = 128 and avoids spilling at
// D = 256.
// PART: 0 = dK and dV in one pass; 1 = dV only; 2 = dK only.  At D = 256 the two accumulators together
// (256 registers per lane) leave no room for anything else, so the kernel is launched once per part
// there, at the price of recomputing the scores (5 products instead of 4).
template <int D, bool V_LDS, int PART>
__global__ __launch_bounds__(256, D <= 128 ? 2 : 1) void bwd_dkdv_kernel(AttnParams p) {
    constexpr bool DO_DV = PART != 2, DO_DK = PART != 1;
    constexpr int BMQ = dkdv_q_tile(D);  // query rows staged per step
    constexpr int QB = BMQ / 32;         // 32-row query blocks per step
    constexpr int KSTEPS = D / 16;
    constexpr int DT = D / 32;
    constexpr int TILE_BYTES = BMQ * D * 2;
    constexpr int STAGE_BYTES = 2 * TILE_BYTES + 2 * 64 * (int)sizeof(float);  // Q, dO, LSE2[64], delta[64]
    extern __shared__ __attribute__((aligned(16))) char smem[];  // two stages, then the V tile if V_LDS
    constexpr int v_tile = 2 * STAGE_BYTES;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int hf = lane >> 5, l32 = lane & 31;
    const int g = blockIdx.x % p.Hkv;
    const WorkItem it = p.items[blockIdx.x / p.Hkv];
    const int kv_row0 = it.w[0], kv_rows = it.w[1], seq_row0 = it.w[2];
    const int qt_first = it.w[3], qt_count = it.w[4], P = it.w[6], L = it.w[7];
    const int G = p.Hq / p.Hkv;
    const float c = p.scale * kLog2e;
    const RowMask mask(P, L, p.mask_mode);

    // Stage n holds query tile qt_first + n % qt_count of head g * G + n / qt_count.  Q and dO rows of
    // (sample, head) and the LSE / delta rows are raw buffers: anything past the sample reads as zero.
    const int n_steps = G * qt_count;
    const int q_row_bytes = p.Hq * D * 2;
    const unsigned q_bytes = (unsigned)(L - 1) * q_row_bytes + D * 2;
    AsyncTile<D, BMQ, 4> loader;
    loader.init(wave, lane, q_row_bytes);
    const unsigned smem_lds = lds_addr(smem);
    auto issue = [&](int n) {
        const unsigned st = smem_lds + (n & 1) * STAGE_BYTES;
        const int head = g * G + n / qt_count;
        const int q0 = (qt_first + n % qt_count) * BMQ;
        const size_t off = ((size_t)seq_row0 * p.Hq + head) * D;
        loader.issue(make_rsrc(static_cast<const __bf16*>(p.q) + off, q_bytes), st, q0 * q_row_bytes);
        loader.issue(make_rsrc(static_cast<const __bf16*>(p.dout) + off, q_bytes), st + TILE_BYTES, q0 * q_row_bytes);
        if (wave < 2) {  // 64 floats each: lane i fetches row q0 + i
            const float* src = (wave == 0 ? p.lse2 : p.delta) + (size_t)head * p.T + seq_row0;
            buffer_load_lds_4(st + 2 * TILE_BYTES + wave * 256, lane * 4, make_rsrc(src, (unsigned)L * 4), q0 * 4);
        }
    };
    issue(0);
    if (V_LDS && DO_DK) {
        const int kv_row_bytes = p.Hkv * D * 2;
        AsyncTile<D, kDkdvKvRows, 4> v_loader;
        v_loader.init(wave, lane, kv_row_bytes);
        const __bf16* v_seq = static_cast<const __bf16*>(p.v) + ((size_t)seq_row0 * p.Hkv + g) * D;
        v_loader.issue(make_rsrc(v_seq, (unsigned)(L - 1) * kv_row_bytes + D * 2), smem_lds + 2 * STAGE_BYTES,
                       (kv_row0 - seq_row0) * kv_row_bytes);
    }

    // this wave's 32 key rows; the lane owns key row jw + l32 (local index in the sample)
    const int jw = kv_row0 - seq_row0 + 32 * wave;
    const int kv_local = jw + l32;
    const bool kv_valid = 32 * wave + l32 < kv_rows;

    // K and V fragments of the lane's key row: k-slots d = 16 t + 8 hf + 0..7
    constexpr bool V_REGS = !V_LDS && DO_DK;
    bf16x8 kf[KSTEPS], vf[V_REGS ? KSTEPS : 1];
    {
        const size_t off = ((size_t)(kv_row0 + 32 * wave + l32) * p.Hkv + g) * D;
        const __bf16* krow = static_cast<const __bf16*>(p.k) + off;
        const __bf16* vrow = static_cast<const __bf16*>(p.v) + off;
#pragma unroll
        for (int t = 0; t < KSTEPS; ++t) {
            u32x4 a = {0u, 0u, 0u, 0u}, b = {0u, 0u, 0u, 0u};
            if (kv_valid) {
                a = *reinterpret_cast<const u32x4*>(krow + 16 * t + 8 * hf);
                if (V_REGS) b = *reinterpret_cast<const u32x4*>(vrow + 16 * t + 8 * hf);
            }
            kf[t] = __builtin_bit_cast(bf16x8, a);
            if (V_REGS) vf[t] = __builtin_bit_cast(bf16x8, b);
        }
    }

    f32x16 dk[DO_DK ? DT : 1], dv[DO_DV ? DT : 1];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            if (DO_DK) dk[dt][r] = 0.0f;
            if (DO_DV) dv[dt][r] = 0.0f;
        }

#pragma unroll
    for (int t = 0; t < KSTEPS; ++t) {
        settle(kf[t]);
        if (V_REGS) settle(vf[t]);
    }
    wait_async_loads();
    __syncthreads();

    const FragAddr<D> fa(lane);
    for (int n = 0; n < n_steps; ++n) {
        if (n + 1 < n_steps) issue(n + 1);
        const int q_tile = (n & 1) * STAGE_BYTES;  // byte offsets of this stage's tiles
        const int do_tile = q_tile + TILE_BYTES;
        const float* lse_s = reinterpret_cast<const float*>(smem + q_tile + 2 * TILE_BYTES);
        const float* delta_s = lse_s + 64;
        const int q0 = (qt_first + n % qt_count) * BMQ;
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            const int i0 = q0 + 32 * qb;  // first query row of the block (local index in the sample)
            if (i0 >= L) break;
            const int i1 = min(i0 + 31, L - 1);
            if (mask.vis(i1) <= jw) continue;  // nothing of this key block is visible
            // rows past the sample read as zeros and must get p = 0: they count as seeing no key
            const bool need_mask = mask.vis(i0) < jw + 32 || i0 + 32 > L;

            // S = Q K^T : rows = query rows (registers), columns = key rows (lanes)
            f32x16 s, dp;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                s[r] = 0.0f;
                dp[r] = 0.0f;
            }
#pragma unroll
            for (int t = 0; t < KSTEPS; ++t) s = mfma32(fa.rowmajor(smem, q_tile, qb, t), kf[t], s);
            __builtin_amdgcn_sched_barrier(0);  // keep the fragment reads of one product from piling up ahead of another
            if (DO_DK) {
#pragma unroll
                for (int t = 0; t < KSTEPS; ++t)
                    dp = mfma32(fa.rowmajor(smem, do_tile, qb, t),
                                V_LDS ? fa.rowmajor(smem, v_tile, wave, t) : vf[V_REGS ? t : 0], dp);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
                const int rb = 32 * qb + 8 * r4 + 4 * hf;  // tile row of registers 4 r4 .. 4 r4 + 3
                const f32x4 l4 = *reinterpret_cast<const f32x4*>(lse_s + rb);
                const f32x4 d4 = *reinterpret_cast<const f32x4*>(delta_s + rb);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int r = 4 * r4 + e;
                    float pv = __builtin_amdgcn_exp2f(__builtin_fmaf(s[r], c, -l4[e]));
                    if (need_mask && kv_local >= mask.vis_in_sample(q0 + rb + e)) pv = 0.0f;
                    s[r] = pv;
                    if (DO_DK) dp[r] = pv * (dp[r] - d4[e]);
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
            __builtin_amdgcn_sched_barrier(0);
            // dV^T += dO^T P ; dK^T += Q^T dS  (rows = d, columns = key rows)
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) {
#pragma unroll
                for (int x = 0; x < 2; ++x) {
                    if (DO_DV) dv[dt] = mfma32(fa.transposed(smem, do_tile, 2 * qb + x, dt), pb[x], dv[dt]);
                    if (DO_DK) dk[dt] = mfma32(fa.transposed(smem, q_tile, 2 * qb + x, dt), dsb[x], dk[dt]);
                }
                if (D == 256 && (dt & 1)) __builtin_amdgcn_sched_barrier(0);
            }
        }
        wait_async_loads();
        __syncthreads();
    }

    if (kv_valid) {
        const size_t off = ((size_t)(kv_row0 + 32 * wave + l32) * p.Hkv + g) * D;
        __bf16* dk_row = static_cast<__bf16*>(p.dk) + off;
        __bf16* dv_row = static_cast<__bf16*>(p.dv) + off;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
                if (DO_DK) {
                    f32x4 a = {dk[dt][4 * r4] * p.scale, dk[dt][4 * r4 + 1] * p.scale, dk[dt][4 * r4 + 2] * p.scale,
                               dk[dt][4 * r4 + 3] * p.scale};
                    *reinterpret_cast<bf16x4*>(dk_row + 32 * dt + 8 * r4 + 4 * hf) = __builtin_convertvector(a, bf16x4);
                }
                if (DO_DV) {
                    f32x4 b = {dv[dt][4 * r4], dv[dt][4 * r4 + 1], dv[dt][4 * r4 + 2], dv[dt][4 * r4 + 3]};
                    *reinterpret_cast<bf16x4*>(dv_row + 32 * dt + 8 * r4 + 4 * hf) = __builtin_convertvector(b, bf16x4);
                }
            }
    }
}

// ------------------------------------------------------------------ dQ

template <int D, int HPB>
__global__ __launch_bounds__(256, D <= 128 ? 2 : 1) void bwd_dq_kernel(AttnParams p) {
    constexpr int BMT = kDqBlockRows / HPB;
    constexpr int BN = kDqKvTile;
    constexpr int KSTEPS = D / 16;
    constexpr int DT = D / 32;
    constexpr int TILE_BYTES = BN * D * 2;
    extern __shared__ __attribute__((aligned(16))) char smem[];

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

    const int kv_row_bytes = p.Hkv * D * 2;
    const unsigned kv_bytes = (unsigned)(L - 1) * kv_row_bytes + D * 2;
    const i32x4 k_rsrc = make_rsrc(static_cast<const __bf16*>(p.k) + ((size_t)seq_row0 * p.Hkv + g) * D, kv_bytes);
    const i32x4 v_rsrc = make_rsrc(static_cast<const __bf16*>(p.v) + ((size_t)seq_row0 * p.Hkv + g) * D, kv_bytes);
    AsyncTile<D, BN, 4> loader;
    loader.init(wave, lane, kv_row_bytes);
    const unsigned smem_lds = lds_addr(smem);
    const int tile_step = __builtin_amdgcn_readfirstlane(BN * kv_row_bytes);
    loader.issue(k_rsrc, smem_lds, 0);
    loader.issue(v_rsrc, smem_lds + TILE_BYTES, 0);

    const int row = wave * 32 + l32;
    const int head = h0 + row / BMT;
    const int tok = row % BMT;
    const bool row_valid = tok < q_rows;
    const int vis = RowMask(P, L, p.mask_mode).vis(q_row0 - seq_row0 + tok);
    const float c = p.scale * kLog2e;

    bf16x8 qf[KSTEPS], dof[KSTEPS];
    float lse2 = INFINITY, delta = 0.0f;  // rows past the sample: p = exp2(-inf) = 0
    {
        const size_t off = ((size_t)(q_row0 + tok) * p.Hq + head) * D;
        const __bf16* qrow = static_cast<const __bf16*>(p.q) + off;
        const __bf16* dorow = static_cast<const __bf16*>(p.dout) + off;
#pragma unroll
        for (int t = 0; t < KSTEPS; ++t) {
            u32x4 a = {0u, 0u, 0u, 0u}, b = {0u, 0u, 0u, 0u};
            if (row_valid) {
                a = *reinterpret_cast<const u32x4*>(qrow + 16 * t + 8 * hf);
                b = *reinterpret_cast<const u32x4*>(dorow + 16 * t + 8 * hf);
            }
            qf[t] = __builtin_bit_cast(bf16x8, a);
            dof[t] = __builtin_bit_cast(bf16x8, b);
        }
        if (row_valid) {
            lse2 = p.lse2[(size_t)head * p.T + q_row0 + tok];
            delta = p.delta[(size_t)head * p.T + q_row0 + tok];
        }
    }

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
    asm volatile("" ::"v"(lse2), "v"(delta));
    wait_async_loads();
    __syncthreads();

    const FragAddr<D> fa(lane);
    for (int kt = 0; kt < n_tiles; ++kt) {
        const int j0 = kt * BN;
        const int k_tile = (kt & 1) * 2 * TILE_BYTES;  // byte offsets of this stage's tiles
        const int v_tile = k_tile + TILE_BYTES;
        if (kt + 1 < n_tiles) {
            const unsigned nk = smem_lds + ((kt + 1) & 1) * 2 * TILE_BYTES;
            loader.issue(k_rsrc, nk, (kt + 1) * tile_step);
            loader.issue(v_rsrc, nk + TILE_BYTES, (kt + 1) * tile_step);
        }
        bf16x8 dsb[4];
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            // S^T and dP^T blocks: rows = key rows (registers), columns = query rows (lanes)
            f32x16 s, dp;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                s[r] = 0.0f;
                dp[r] = 0.0f;
            }
#pragma unroll
            for (int t = 0; t < KSTEPS; ++t) s = mfma32(fa.rowmajor(smem, k_tile, b, t), qf[t], s);
#pragma unroll
            for (int t = 0; t < KSTEPS; ++t) dp = mfma32(fa.rowmajor(smem, v_tile, b, t), dof[t], dp);
            const bool need_mask = kt >= n_full;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                float pv = __builtin_amdgcn_exp2f(__builtin_fmaf(s[r], c, -lse2));
                if (need_mask && j0 + 32 * b + acc_row(r, hf) >= vis) pv = 0.0f;
                dp[r] = pv * (dp[r] - delta);
            }
#pragma unroll
            for (int x = 0; x < 2; ++x)
                dsb[2 * b + x] = to_bf16x8(dp[8 * x], dp[8 * x + 1], dp[8 * x + 2], dp[8 * x + 3], dp[8 * x + 4],
                                           dp[8 * x + 5], dp[8 * x + 6], dp[8 * x + 7]);
        }
        // dQ^T += K^T dS^T
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int x = 0; x < 4; ++x)
                dq[dt] = mfma32(fa.transposed(smem, k_tile, x, dt), dsb[x], dq[dt]);
        wait_async_loads();
        __syncthreads();
    }

    if (row_valid) {
        __bf16* dq_row = static_cast<__bf16*>(p.dq) + ((size_t)(q_row0 + tok) * p.Hq + head) * D;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
                f32x4 f = {dq[dt][4 * r4] * p.scale, dq[dt][4 * r4 + 1] * p.scale, dq[dt][4 * r4 + 2] * p.scale,
                           dq[dt][4 * r4 + 3] * p.scale};
                *reinterpret_cast<bf16x4*>(dq_row + 32 * dt + 8 * r4 + 4 * hf) = __builtin_convertvector(f, bf16x4);
            }
    }
}

template <int D, int HPB>
hipError_t launch_dq_dh(const AttnParams& p, hipStream_t stream, unsigned grid) {
    constexpr size_t smem = 2 * 2 * kDqKvTile * D * 2;  // two stages of (K tile, V tile)
    static const hipError_t attr = allow_dynamic_lds(reinterpret_cast<const void*>(&bwd_dq_kernel<D, HPB>), smem);
    if (attr != hipSuccess) return attr;
    hipLaunchKernelGGL((bwd_dq_kernel<D, HPB>), dim3(grid), dim3(256), smem, stream, p);
    return hipGetLastError();
}

template <int D>
hipError_t launch_dq_d(const AttnParams& p, hipStream_t stream) {
    const int G = p.Hq / p.Hkv;
    const int hpb = heads_per_block(p.Hq, p.Hkv);
    const unsigned grid = (unsigned)p.num_items * (unsigned)(p.Hkv * (G / hpb));
    if (grid == 0) return hipSuccess;
    switch (hpb) {
        case 1: return launch_dq_dh<D, 1>(p, stream, grid);
        case 2: return launch_dq_dh<D, 2>(p, stream, grid);
        case 4: return launch_dq_dh<D, 4>(p, stream, grid);
        default: return launch_dq_dh<D, 8>(p, stream, grid);
    }
}

template <int D, int PART>
hipError_t launch_dkdv_part(const AttnParams& p, hipStream_t stream, unsigned grid) {
    constexpr bool V_LDS = D >= 128;
    constexpr size_t smem = 2 * (2 * dkdv_q_tile(D) * D * 2 + 2 * 64 * sizeof(float)) + (V_LDS ? kDkdvKvRows * D * 2 : 0);
    static const hipError_t attr = allow_dynamic_lds(reinterpret_cast<const void*>(&bwd_dkdv_kernel<D, V_LDS, PART>), smem);
    if (attr != hipSuccess) return attr;
    hipLaunchKernelGGL((bwd_dkdv_kernel<D, V_LDS, PART>), dim3(grid), dim3(256), smem, stream, p);
    return hipGetLastError();
}

template <int D>
hipError_t launch_dkdv_d(const AttnParams& p, hipStream_t stream) {
    const unsigned grid = (unsigned)p.num_items * (unsigned)p.Hkv;
    if (grid == 0) return hipSuccess;
    if constexpr (D <= 128) {
        return launch_dkdv_part<D, 0>(p, stream, grid);
    } else {
        const hipError_t e = launch_dkdv_part<D, 1>(p, stream, grid);
        return e != hipSuccess ? e : launch_dkdv_part<D, 2>(p, stream, grid);
    }
}

template <int D>
hipError_t launch_delta_d(const AttnParams& p, hipStream_t stream) {
    const size_t rows = (size_t)p.T * p.Hq;
    constexpr int RPB = 256 / (D / 8);
    const unsigned grid = (unsigned)((rows + RPB - 1) / RPB);
    if (grid == 0) return hipSuccess;
    hipLaunchKernelGGL((bwd_delta_kernel<D>), dim3(grid), dim3(256), 0, stream, static_cast<const __bf16*>(p.out),
                       static_cast<const __bf16*>(p.dout), p.lse, p.delta, p.lse2, p.T, p.Hq);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_bwd_delta(const AttnParams& p, hipStream_t stream) {
    switch (p.D) {
        case 64: return launch_delta_d<64>(p, stream);
        case 128: return launch_delta_d<128>(p, stream);
        case 256: return launch_delta_d<256>(p, stream);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_bwd_dkdv(const AttnParams& p, hipStream_t stream) {
    switch (p.D) {
        case 64: return launch_dkdv_d<64>(p, stream);
        case 128: return launch_dkdv_d<128>(p, stream);
        case 256: return launch_dkdv_d<256>(p, stream);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_bwd_dq(const AttnParams& p, hipStream_t stream) {
    switch (p.D) {
        case 64: return launch_dq_d<64>(p, stream);
        case 128: return launch_dq_d<128>(p, stream);
        case 256: return launch_dq_d<256>(p, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace va
