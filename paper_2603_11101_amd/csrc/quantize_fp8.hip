// Per-head OCP E4M3 quantisation on the device, bit-identical to the host
// routine va_quantize_e4m3_per_head: descale[h] = amax_h / 448 (1 for an
// all-zero head), code = round-to-nearest-even E4M3 of x / descale[h],
// saturating at +-448.  (The scaling vocabulary is that of section 2.2.3;
// applying it per attention head is this library's choice.)
//
// Four small kernels on the caller's stream: clear the per-head maxima, reduce
// |x| per head, encode, turn the maxima into descales.  The descale array holds
// the maxima (as float bits: for non-negative floats the integer order is the
// float order) until the last kernel; nothing else is needed, nothing is
// allocated.
//
// The block-wise quantiser (one scale per 128 tokens of one sample and one
// head, bit-identical to va_quantize_e4m3_blockwise) is one kernel further down.
#include "kernels.h"
#include "mfma_util.h"

namespace va {

namespace {

constexpr int kMaxHeadsInLds = 256;

__global__ void quant_clear_kernel(unsigned* amax_bits, int H) {
    const int h = blockIdx.x * blockDim.x + threadIdx.x;
    if (h < H) amax_bits[h] = 0u;
}

VA_DEV float bf16_bits_to_float(unsigned bits16) { return __builtin_bit_cast(float, bits16 << 16); }

typedef int i32x2 __attribute__((ext_vector_type(2)));

// |bf16| of the 8 values of a chunk as float bits, their maximum.  NaN patterns (above the bits of infinity)
// count as zero, as in the host routine, whose maximum drops them: a NaN in the input turns into the NaN
// code at its own place and leaves the scale of its head or block alone.
VA_DEV unsigned chunk_amax_bits(u32x4 raw) {
    unsigned m = 0u;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        // clear the sign, move the 16 bits to the top half
        const unsigned lo = (raw[w] & 0x7fffu) << 16, hi = raw[w] & 0x7fff0000u;
        m = max(m, lo > 0x7f800000u ? 0u : lo);
        m = max(m, hi > 0x7f800000u ? 0u : hi);
    }
    return m;
}

VA_DEV float descale_of(unsigned amax_bits) {
    const float s = __builtin_bit_cast(float, amax_bits) / 448.0f;
    return s > 0.0f ? s : 1.0f;
}

// Eight bf16 values -> eight E4M3 codes of value / descale.
VA_DEV i32x2 encode_chunk(u32x4 raw, float descale) {
    float v[8];
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        v[2 * w] = bf16_bits_to_float(raw[w] & 0xffffu) / descale;
        v[2 * w + 1] = bf16_bits_to_float(raw[w] >> 16) / descale;
    }
    // The conversion instruction rounds to nearest even, subnormals included, but turns magnitudes of
    // 464 and more into NaN instead of saturating: clamp first (448 is representable).  The clamp would
    // also turn a NaN into -448; a NaN (the value itself, or infinity over an infinite scale) gets the
    // NaN code 0x7F of the host routine instead.
    unsigned nan_lo = 0u, nan_hi = 0u;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        if (v[e] != v[e]) (e < 4 ? nan_lo : nan_hi) |= 0xffu << (8 * (e & 3));
        v[e] = fminf(fmaxf(v[e], -448.0f), 448.0f);
    }
    int lo = __builtin_amdgcn_cvt_pk_fp8_f32(v[0], v[1], 0, false);
    lo = __builtin_amdgcn_cvt_pk_fp8_f32(v[2], v[3], lo, true);
    int hi = __builtin_amdgcn_cvt_pk_fp8_f32(v[4], v[5], 0, false);
    hi = __builtin_amdgcn_cvt_pk_fp8_f32(v[6], v[7], hi, true);
    lo = (int)(((unsigned)lo & ~nan_lo) | (0x7f7f7f7fu & nan_lo));
    hi = (int)(((unsigned)hi & ~nan_hi) | (0x7f7f7f7fu & nan_hi));
    return i32x2{lo, hi};
}

// x is [rows = T * H, D] bf16; a thread takes 8 consecutive values (16 bytes) at a time.
__global__ __launch_bounds__(256) void quant_amax_kernel(const uint16_t* x, size_t chunks, int chunks_per_row, int H,
                                                         unsigned* amax_bits) {
    __shared__ unsigned lds_max[kMaxHeadsInLds];
    const bool use_lds = H <= kMaxHeadsInLds;
    if (use_lds) {
        for (int h = threadIdx.x; h < H; h += blockDim.x) lds_max[h] = 0u;
        __syncthreads();
    }
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < chunks; i += (size_t)gridDim.x * blockDim.x) {
        const u32x4 raw = *reinterpret_cast<const u32x4*>(x + i * 8);
        const unsigned m = chunk_amax_bits(raw);
        const int h = (int)((i / chunks_per_row) % H);
        if (use_lds) atomicMax(&lds_max[h], m);
        else atomicMax(&amax_bits[h], m);
    }
    if (use_lds) {
        __syncthreads();
        for (int h = threadIdx.x; h < H; h += blockDim.x)
            if (lds_max[h] != 0u) atomicMax(&amax_bits[h], lds_max[h]);
    }
}


__global__ __launch_bounds__(256) void quant_encode_kernel(const uint16_t* x, size_t chunks, int chunks_per_row, int H,
                                                           const unsigned* amax_bits, unsigned char* codes) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < chunks; i += (size_t)gridDim.x * blockDim.x) {
        const int h = (int)((i / chunks_per_row) % H);
        const float descale = descale_of(amax_bits[h]);
        *reinterpret_cast<i32x2*>(codes + i * 8) = encode_chunk(*reinterpret_cast<const u32x4*>(x + i * 8), descale);
    }
}

__global__ void quant_descale_kernel(float* descale, int H) {
    const int h = blockIdx.x * blockDim.x + threadIdx.x;
    if (h < H) {
        const float s = descale[h] / 448.0f;  // still the maximum here
        descale[h] = s > 0.0f ? s : 1.0f;
    }
}

// Block-wise variant: a block is up to kBlockTokens consecutive tokens of one sample, one head.
constexpr int kBlockTokens = 128;

// Rows [r0, r1) of block number b in sample order, found by a prefix sum over the samples' block counts,
// 64 samples at a time; every lane of the wave returns the same pair.  An empty range means "no such
// block".  The range is clipped to [0, T), whatever cu holds.
VA_DEV void find_block(const int* cu, int n, int T, int b, int lane, int* r0_out, int* r1_out) {
    int r0 = 0, r1 = 0;
    for (int base = 0; base < n; base += 64) {
        const int s = base + lane;
        int c0 = 0, c1 = 0;
        if (s < n) {
            c0 = cu[s];
            c1 = cu[s + 1];
        }
        const int nb = c1 > c0 ? (c1 - c0 + kBlockTokens - 1) / kBlockTokens : 0;
        int incl = nb;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int up = __shfl_up(incl, d);
            if (lane >= d) incl += up;
        }
        const int total = __shfl(incl, 63);
        if (b < total) {
            const int src = __ffsll((unsigned long long)__ballot(b < incl)) - 1;  // the sample that holds block b
            const int first = __shfl(incl - nb, src);
            r0 = __shfl(c0, src) + (b - first) * kBlockTokens;
            r1 = min(__shfl(c1, src), r0 + kBlockTokens);
            break;
        }
        b -= total;
    }
    *r0_out = max(r0, 0);
    *r1_out = min(r1, T);
}

// Head dimensions up to 256.  Workgroup (b, h): block number b in sample order, head h; wave w takes the
// rows 32 w .. 32 w + 31 of the block and keeps them in registers (J chunks of 8 values per lane), so x is
// read once: maximum per wave, the four maxima meet in LDS, then every wave encodes what it holds.
template <int J>
__global__ __launch_bounds__(256) void quant_blockwise_kernel(const uint16_t* x, const int* cu, int n, int T, int H,
                                                              int chunks_per_row, unsigned char* codes,
                                                              float* descale_tok) {
    __shared__ unsigned wave_max[4];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int h = (int)blockIdx.y;
    int r0, r1;
    find_block(cu, n, T, (int)blockIdx.x, lane, &r0, &r1);
    if (r0 >= r1) return;  // the same for the whole workgroup
    const int w0 = r0 + 32 * wave;
    const int wrows = max(0, min(32, r1 - w0));  // rows of this wave
    const int chunks = wrows * chunks_per_row;
    const int row_bytes = H * chunks_per_row * 16;
    const size_t first = ((size_t)w0 * H + h) * chunks_per_row;  // first chunk of this wave, in chunks
    // the ranges end with the wave's last row of this head: nothing outside them can be touched
    const unsigned span = wrows > 0 ? (unsigned)(wrows - 1) * row_bytes + chunks_per_row * 16 : 0u;
    const __amdgpu_buffer_rsrc_t src = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<char*>(reinterpret_cast<const char*>(x)) + (wrows > 0 ? first * 16 : 0), 0, (int)span, 0x00020000);
    const __amdgpu_buffer_rsrc_t dst =
        __builtin_amdgcn_make_buffer_rsrc(codes + (wrows > 0 ? first * 8 : 0), 0, (int)(span / 2), 0x00020000);
    u32x4 raw[J];
    int at[J];  // byte offset of the lane's chunk j in x (half of it in codes), out of range where it has none
    unsigned m = 0u;
#pragma unroll
    for (int j = 0; j < J; ++j) {
        const int i = lane + 64 * j;
        at[j] = i < chunks ? (i / chunks_per_row) * row_bytes + (i % chunks_per_row) * 16 : (int)0x7ffffff0;
        raw[j] = __builtin_amdgcn_raw_buffer_load_b128(src, at[j], 0, 0);  // zero where out of range
    }
#pragma unroll
    for (int j = 0; j < J; ++j) m = max(m, chunk_amax_bits(raw[j]));
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) m = max(m, (unsigned)__shfl_xor((int)m, d));
    if (lane == 0) wave_max[wave] = m;
    __syncthreads();
    const float descale = descale_of(max(max(wave_max[0], wave_max[1]), max(wave_max[2], wave_max[3])));
#pragma unroll
    for (int j = 0; j < J; ++j) {
        typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
        const int off = at[j] == (int)0x7ffffff0 ? at[j] : at[j] / 2;
        __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(u32x2, encode_chunk(raw[j], descale)), dst, off, 0, 0);
    }
    const int r = r0 + 64 * (wave & 1) + lane;  // waves 0 and 1 write the scales of the block's rows
    if (wave < 2 && r < r1) descale_tok[(size_t)r * H + h] = descale;
}

// Any head dimension: workgroup (b, y), wave w takes head 4 y + w and the whole block, reads it twice
// (maximum, then encoding).  Waves do not interact.

__global__ __launch_bounds__(256) void quant_blockwise_two_pass_kernel(const uint16_t* x, const int* cu, int n, int T,
                                                                       int H, int chunks_per_row, unsigned char* codes,
                                                                       float* descale_tok) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int h = blockIdx.y * 4 + wave;
    if (h >= H) return;
    int r0, r1;
    find_block(cu, n, T, (int)blockIdx.x, lane, &r0, &r1);
    if (r0 >= r1) return;
    const int rows = r1 - r0, chunks = rows * chunks_per_row;
    const size_t row_chunks = (size_t)H * chunks_per_row;  // chunks from one token row to the next
    const uint16_t* xb = x + ((size_t)r0 * H + h) * chunks_per_row * 8;
    unsigned m = 0u;
    for (int i = lane; i < chunks; i += 64) {
        const size_t at = ((size_t)(i / chunks_per_row) * row_chunks + i % chunks_per_row) * 8;
        m = max(m, chunk_amax_bits(*reinterpret_cast<const u32x4*>(xb + at)));
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) m = max(m, (unsigned)__shfl_xor((int)m, d));
    const float descale = descale_of(m);
    unsigned char* cb = codes + ((size_t)r0 * H + h) * chunks_per_row * 8;
    for (int i = lane; i < chunks; i += 64) {
        const size_t at = ((size_t)(i / chunks_per_row) * row_chunks + i % chunks_per_row) * 8;
        *reinterpret_cast<i32x2*>(cb + at) = encode_chunk(*reinterpret_cast<const u32x4*>(xb + at), descale);
    }
    for (int r = lane; r < rows; r += 64) descale_tok[(size_t)(r0 + r) * H + h] = descale;
}

}  // namespace

hipError_t launch_quantize_e4m3(const void* x, int32_t T, int32_t H, int32_t D, void* codes, float* descale,
                                hipStream_t stream) {
    const size_t chunks = (size_t)T * H * (D / 8);
    const unsigned hb = (unsigned)((H + 255) / 256);
    unsigned* bits = reinterpret_cast<unsigned*>(descale);
    hipLaunchKernelGGL(quant_clear_kernel, dim3(hb), dim3(256), 0, stream, bits, H);
    if (chunks > 0) {
        const unsigned grid = (unsigned)std::min<size_t>((chunks + 255) / 256, 256 * 8);
        hipLaunchKernelGGL(quant_amax_kernel, dim3(grid), dim3(256), 0, stream, static_cast<const uint16_t*>(x), chunks,
                           D / 8, H, bits);
        hipLaunchKernelGGL(quant_encode_kernel, dim3(grid), dim3(256), 0, stream, static_cast<const uint16_t*>(x), chunks,
                           D / 8, H, bits, static_cast<unsigned char*>(codes));
    }
    hipLaunchKernelGGL(quant_descale_kernel, dim3(hb), dim3(256), 0, stream, descale, H);
    return hipGetLastError();
}

hipError_t launch_quantize_e4m3_blockwise(const void* x, const int32_t* cu_device, int32_t num_seqs, int32_t T,
                                          int32_t num_blocks, int32_t H, int32_t D, void* codes, float* descale_tok,
                                          hipStream_t stream) {
    if (num_blocks == 0) return hipSuccess;
    const uint16_t* xs = static_cast<const uint16_t*>(x);
    unsigned char* cs = static_cast<unsigned char*>(codes);
    const int cpr = D / 8;
    const dim3 grid((unsigned)num_blocks, (unsigned)H);
    // a wave holds 32 rows: 32 * cpr chunks over 64 lanes
    if (cpr <= 8 && H <= 65535)
        hipLaunchKernelGGL(quant_blockwise_kernel<4>, grid, dim3(256), 0, stream, xs, cu_device, num_seqs, T, H, cpr, cs, descale_tok);
    else if (cpr <= 16 && H <= 65535)
        hipLaunchKernelGGL(quant_blockwise_kernel<8>, grid, dim3(256), 0, stream, xs, cu_device, num_seqs, T, H, cpr, cs, descale_tok);
    else if (cpr <= 32 && H <= 65535)
        hipLaunchKernelGGL(quant_blockwise_kernel<16>, grid, dim3(256), 0, stream, xs, cu_device, num_seqs, T, H, cpr, cs, descale_tok);
    else
        hipLaunchKernelGGL(quant_blockwise_two_pass_kernel, dim3((unsigned)num_blocks, (unsigned)((H + 3) / 4)), dim3(256), 0,
                           stream, xs, cu_device, num_seqs, T, H, cpr, cs, descale_tok);
    return hipGetLastError();
}

}  // namespace va
