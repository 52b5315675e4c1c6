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

VA_DEV int visible_keys(int i, int L, int P, int mode) {
    if (mode == VA_MASK_CAUSAL) return i + 1;
    if (i < P) return P;
    return mode == VA_MASK_PREFIX_LM ? L : i + 1;
}

template <int D, int HPB>
__global__ __launch_bounds__(256) void fwd_bf16_kernel(AttnParams p) {
    constexpr int BMT = kFwdBlockRows / HPB;  // token rows of the work item
    constexpr int BN = kFwdKvTile;
    constexpr int KSTEPS = D / 16;  // MFMA steps over the head dimension
    constexpr int DT = D / 32;      // 32-row blocks of O^T
    extern __shared__ __attribute__((aligned(16))) char smem[];
    char* k_tile = smem;
    char* v_tile = smem + BN * D * 2;

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

    // the stacked row this lane owns
    const int row = wave * 32 + l32;
    const int head = h0 + row / BMT;
    const int tok = row % BMT;
    const bool row_valid = tok < q_rows;
    const int vis = visible_keys(q_row0 - seq_row0 + tok, L, P, p.mask_mode);

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
    float m = -INFINITY;  // running maximum of scale * log2(e) * s
    float lsum = 0.0f;    // this lane's share of the running sum (other share in lane + 32)
    const float c = p.scale * kLog2e;

    const size_t kv_stride = (size_t)p.Hkv * D;
    const __bf16* k_base = static_cast<const __bf16*>(p.k) + ((size_t)seq_row0 * p.Hkv + g) * D;
    const __bf16* v_base = static_cast<const __bf16*>(p.v) + ((size_t)seq_row0 * p.Hkv + g) * D;

    for (int kt = 0; kt < n_tiles; ++kt) {
        const int j0 = kt * BN;
        __syncthreads();
        load_tile<D, BN, 256>(k_tile, k_base + (size_t)j0 * kv_stride, kv_stride, L - j0, tid);
        load_tile<D, BN, 256>(v_tile, v_base + (size_t)j0 * kv_stride, kv_stride, L - j0, tid);
        __syncthreads();

        // S^T: two blocks of 32 keys x 32 query rows
        f32x16 s[2];
#pragma unroll
        for (int b = 0; b < 2; ++b) {
#pragma unroll
            for (int r = 0; r < 16; ++r) s[b][r] = 0.0f;
#pragma unroll
            for (int t = 0; t < KSTEPS; ++t)
                s[b] = mfma32(frag_rowmajor<D>(k_tile, 32 * b + l32, t, hf), qf[t], s[b]);
        }
        if (kt >= n_full) {
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    if (j0 + 32 * b + acc_row(r, hf) >= vis) s[b][r] = -INFINITY;
        }
        float mx = s[0][0];
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[b][r]);
        mx = pair_max(mx);
        const float m_new = fmaxf(m, mx * c);
        const float m_use = m_new == -INFINITY ? 0.0f : m_new;
        const float alpha = __builtin_amdgcn_exp2f(m - m_use);
        m = m_new;
        float psum = 0.0f;
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float pv = __builtin_amdgcn_exp2f(__builtin_fmaf(s[b][r], c, -m_use));
                s[b][r] = pv;
                psum += pv;
            }
        lsum = lsum * alpha + psum;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int r = 0; r < 16; ++r) o[dt][r] *= alpha;

        // P^T as second operand: registers 8 x .. 8 x + 7 of a block are the k-slots of step x
        bf16x8 pf[4];
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int x = 0; x < 2; ++x)
                pf[2 * b + x] = to_bf16x8(s[b][8 * x + 0], s[b][8 * x + 1], s[b][8 * x + 2], s[b][8 * x + 3],
                                          s[b][8 * x + 4], s[b][8 * x + 5], s[b][8 * x + 6], s[b][8 * x + 7]);
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int x = 0; x < 4; ++x)
                o[dt] = mfma32(frag_transposed<D>(v_tile, 16 * x, 32 * dt, lane), pf[x], o[dt]);
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

template <int D>
hipError_t launch_d(const AttnParams& p, hipStream_t stream) {
    const int G = p.Hq / p.Hkv;
    const int hpb = heads_per_block(p.Hq, p.Hkv);
    const unsigned grid = (unsigned)p.num_items * (unsigned)(p.Hkv * (G / hpb));
    const size_t smem = 2 * kFwdKvTile * D * 2;
    if (grid == 0) return hipSuccess;
    switch (hpb) {
        case 1: hipLaunchKernelGGL((fwd_bf16_kernel<D, 1>), dim3(grid), dim3(256), smem, stream, p); break;
        case 2: hipLaunchKernelGGL((fwd_bf16_kernel<D, 2>), dim3(grid), dim3(256), smem, stream, p); break;
        case 4: hipLaunchKernelGGL((fwd_bf16_kernel<D, 4>), dim3(grid), dim3(256), smem, stream, p); break;
        default: hipLaunchKernelGGL((fwd_bf16_kernel<D, 8>), dim3(grid), dim3(256), smem, stream, p); break;
    }
    return hipGetLastError();
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
