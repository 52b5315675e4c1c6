// Forward kernel, FP8: Q, K, V are OCP E4M3 bytes with one float32 descale per
// head; both products run on v_mfma_f32_32x32x64_f8f6f4 (64 contraction slots
// per instruction, twice the bf16 rate); scores, softmax, row sums and LSE are
// float32; the probabilities are requantised to E4M3 for the second product.
//
// The paper's FP8 material (section 2.2.3) concerns weight quantisation and
// only supplies the scaling vocabulary; the per-head scale is its per-channel
// rule applied along the head axis.  Everything else here is this library's.
//
// Same decomposition as the bf16 forward: one workgroup = 128 stacked
// (head, token) rows of one KV group, 4 waves x 32 rows, 64 keys per step,
// S^T = K Q^T then O^T = V^T P^T so a lane owns one query row throughout.
//
// Row order inside a key tile.  An accumulator register r of lane half hf of
// the block b product holds the key that A-lane i = 8 (r / 4) + 4 hf + r % 4
// loaded.  A-lane i of block b loads tile row 32 * (bit 2 of i) + 16 b +
// 4 * (i / 8) + i % 4, so register r of half hf holds tile row
// 32 hf + 16 b + r: the 32 probabilities of a lane are 32 consecutive keys,
// in register order, which is exactly the byte order the second product wants
// when its V^T operand comes from four 8-row transposing byte reads.
#include "kernels.h"
#include "mfma_util.h"

namespace va {

namespace {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kPShift = 8.0f;  // probabilities are stored as p * 2^8 in E4M3 (largest value 256 <= 448)

typedef int i32x8 __attribute__((ext_vector_type(8)));
typedef int i32x2 __attribute__((ext_vector_type(2)));
typedef int i32x4 __attribute__((ext_vector_type(4)));

VA_DEV f32x16 mfma_f8(i32x8 a, i32x8 b, f32x16 c) {
    // formats 0 = E4M3 for both operands; block scales 127 = 2^0
    return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, c, 0, 0, 0, 127, 0, 127);
}

// LDS tile of 64 rows x 128 bytes, 16-byte chunks, chunk c of row r stored at
// c ^ swz(r).  Conflict free for (1) 16 lanes reading one chunk of the rows
// {x, 32 + x : x in 0..7} (+ 16 b), and (2) 32 lanes reading 8 consecutive rows
// by 32 bytes with the transposing byte read.
VA_DEV int swz8(int r) { return (((r >> 1) & 3) << 1) | ((r >> 5) & 1); }
VA_DEV int off8(int r, int c) { return r * 128 + ((c ^ swz8(r)) << 4); }

template <int HPB>
__global__ __launch_bounds__(256) void fwd_fp8_kernel(AttnParams p) {
    constexpr int D = 128;
    constexpr int BMT = kFwdBlockRows / HPB;
    constexpr int BN = kFwdKvTile;
    constexpr int KSTEPS = D / 64;
    constexpr int DT = D / 32;
    __shared__ __attribute__((aligned(16))) char k_tile[BN * D];
    __shared__ __attribute__((aligned(16))) char v_tile[BN * D];

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

    const int row = wave * 32 + l32;
    const int head = h0 + row / BMT;
    const int tok = row % BMT;
    const bool row_valid = tok < q_rows;
    const int vis = RowMask(P, L, p.mask_mode).vis(q_row0 - seq_row0 + tok);

    // Q fragments: contraction slots d = 64 t + 32 hf + 0..31
    i32x8 qf[KSTEPS];
    {
        const char* qrow = static_cast<const char*>(p.q) + ((size_t)(q_row0 + tok) * p.Hq + head) * D;
#pragma unroll
        for (int t = 0; t < KSTEPS; ++t) {
            i32x4 lo = {0, 0, 0, 0}, hi = {0, 0, 0, 0};
            if (row_valid) {
                lo = *reinterpret_cast<const i32x4*>(qrow + 64 * t + 32 * hf);
                hi = *reinterpret_cast<const i32x4*>(qrow + 64 * t + 32 * hf + 16);
            }
            qf[t] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        }
    }
    // scores in base 2: s2 = acc * scale * q_descale[h] * k_descale[g] * log2(e)
    const float c = p.scale * p.q_descale[head] * p.k_descale[g] * kLog2e;
    const float v_descale = p.v_descale[g];

    f32x16 o[DT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[dt][r] = 0.0f;
    float m = -INFINITY;
    float lsum = 0.0f;  // sum of p * 2^8, this lane's share

    const size_t kv_stride = (size_t)p.Hkv * D;
    const char* k_base = static_cast<const char*>(p.k) + ((size_t)seq_row0 * p.Hkv + g) * D;
    const char* v_base = static_cast<const char*>(p.v) + ((size_t)seq_row0 * p.Hkv + g) * D;

    // tile row this lane loads as A-lane l32 of block 0 (block 1: + 16)
    const int a_row = 32 * ((l32 >> 2) & 1) + 4 * (l32 >> 3) + (l32 & 3);

    for (int kt = 0; kt < n_tiles; ++kt) {
        const int j0 = kt * BN;
        __syncthreads();
#pragma unroll
        for (int i = 0; i < (BN * D / 16) / 256; ++i) {
            const int cid = tid + i * 256;
            const int r = cid >> 3, ch = cid & 7;
            i32x4 kk = {0, 0, 0, 0}, vv = {0, 0, 0, 0};
            if (j0 + r < L) {
                kk = *reinterpret_cast<const i32x4*>(k_base + (size_t)(j0 + r) * kv_stride + ch * 16);
                vv = *reinterpret_cast<const i32x4*>(v_base + (size_t)(j0 + r) * kv_stride + ch * 16);
            }
            *reinterpret_cast<i32x4*>(k_tile + off8(r, ch)) = kk;
            *reinterpret_cast<i32x4*>(v_tile + off8(r, ch)) = vv;
        }
        __syncthreads();

        f32x16 s[2];
#pragma unroll
        for (int b = 0; b < 2; ++b) {
#pragma unroll
            for (int r = 0; r < 16; ++r) s[b][r] = 0.0f;
            const int kr = a_row + 16 * b;
#pragma unroll
            for (int t = 0; t < KSTEPS; ++t) {
                const i32x4 lo = *reinterpret_cast<const i32x4*>(k_tile + off8(kr, 4 * t + 2 * hf));
                const i32x4 hi = *reinterpret_cast<const i32x4*>(k_tile + off8(kr, 4 * t + 2 * hf + 1));
                s[b] = mfma_f8(__builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7), qf[t], s[b]);
            }
        }
        if (kt >= n_full) {
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    if (j0 + 32 * hf + 16 * b + r >= vis) s[b][r] = -INFINITY;
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
        const float shift = kPShift - m_use;
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float pv = __builtin_amdgcn_exp2f(__builtin_fmaf(s[b][r], c, shift));
                s[b][r] = pv;
                psum += pv;
            }
        lsum = lsum * alpha + psum;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int r = 0; r < 16; ++r) o[dt][r] *= alpha;

        // P^T operand: byte e of the lane = register e % 16 of block e / 16 = key 32 hf + e
        i32x8 pf;
#pragma unroll
        for (int w = 0; w < 8; ++w) {
            const int b = w >> 2, r = (w & 3) * 4;
            int word = __builtin_amdgcn_cvt_pk_fp8_f32(s[b][r], s[b][r + 1], 0, false);
            word = __builtin_amdgcn_cvt_pk_fp8_f32(s[b][r + 2], s[b][r + 3], word, true);
            pf[w] = word;
        }
        // V^T operand: column d = 32 dt + l32, keys 32 hf + 0..31 through four transposing byte reads.
        // In a group of 16 lanes, lane i receives byte (i % 8) of the 8 bytes addressed by lane 2 e + i / 8 as
        // element e (measured); lane s of the group therefore points at row s / 2, columns 8 (s % 2) .. + 7.
        const int s16 = lane & 15;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
            const int col = 32 * dt + 16 * ((lane >> 4) & 1) + 8 * (s16 & 1);
            i32x8 vf;
#pragma unroll
            for (int x = 0; x < 4; ++x) {
                const int vr = 32 * hf + 8 * x + (s16 >> 1);
                typedef __attribute__((address_space(3))) i32x2* lds_i32x2;
                const i32x2 two = __builtin_amdgcn_ds_read_tr8_b64_v2i32(
                    (lds_i32x2)(lds_char*)(v_tile + off8(vr, col >> 4) + (col & 8)));
                vf[2 * x] = two[0];
                vf[2 * x + 1] = two[1];
            }
            o[dt] = mfma_f8(vf, pf, o[dt]);
        }
    }

    lsum = pair_sum(lsum);
    if (row_valid) {
        // O = v_descale * (V8^T P8) / sum(p * 2^8): the 2^8 of the stored probabilities cancels
        const float inv = v_descale / lsum;
        __bf16* orow = static_cast<__bf16*>(p.out) + ((size_t)(q_row0 + tok) * p.Hq + head) * D;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
                f32x4 f = {o[dt][4 * r4] * inv, o[dt][4 * r4 + 1] * inv, o[dt][4 * r4 + 2] * inv, o[dt][4 * r4 + 3] * inv};
                *reinterpret_cast<bf16x4*>(orow + 32 * dt + 8 * r4 + 4 * hf) = __builtin_convertvector(f, bf16x4);
            }
        if (hf == 0)
            p.lse[(size_t)head * p.T + q_row0 + tok] = (m + __builtin_amdgcn_logf(lsum) - kPShift) * kLn2;
    }
}

}  // namespace

hipError_t launch_fwd_fp8(const AttnParams& p, hipStream_t stream) {
    if (p.D != 128) return hipErrorNotSupported;
    const int G = p.Hq / p.Hkv;
    const int hpb = heads_per_block(p.Hq, p.Hkv);
    const unsigned grid = (unsigned)p.num_items * (unsigned)(p.Hkv * (G / hpb));
    if (grid == 0) return hipSuccess;
    switch (hpb) {
        case 1: hipLaunchKernelGGL((fwd_fp8_kernel<1>), dim3(grid), dim3(256), 0, stream, p); break;
        case 2: hipLaunchKernelGGL((fwd_fp8_kernel<2>), dim3(grid), dim3(256), 0, stream, p); break;
        case 4: hipLaunchKernelGGL((fwd_fp8_kernel<4>), dim3(grid), dim3(256), 0, stream, p); break;
        default: hipLaunchKernelGGL((fwd_fp8_kernel<8>), dim3(grid), dim3(256), 0, stream, p); break;
    }
    return hipGetLastError();
}

}  // namespace va
