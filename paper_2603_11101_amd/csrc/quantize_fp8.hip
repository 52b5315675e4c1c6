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
#include "kernels.h"
#include "mfma_util.h"

namespace va {

namespace {

constexpr int kMaxHeadsInLds = 256;

__global__ void quant_clear_kernel(unsigned* amax_bits, int H) {
    const int h = blockIdx.x * blockDim.x + threadIdx.x;
    if (h < H) amax_bits[h] = 0u;
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
        unsigned m = 0u;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            // |bf16| as float bits: clear the sign, move the 16 bits to the top half
            m = max(m, (raw[w] & 0x7fffu) << 16);
            m = max(m, raw[w] & 0x7fff0000u);
        }
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

VA_DEV float bf16_bits_to_float(unsigned bits16) { return __builtin_bit_cast(float, bits16 << 16); }

__global__ __launch_bounds__(256) void quant_encode_kernel(const uint16_t* x, size_t chunks, int chunks_per_row, int H,
                                                           const unsigned* amax_bits, unsigned char* codes) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < chunks; i += (size_t)gridDim.x * blockDim.x) {
        const int h = (int)((i / chunks_per_row) % H);
        const float amax = __builtin_bit_cast(float, amax_bits[h]);
        const float s = amax / 448.0f;
        const float descale = s > 0.0f ? s : 1.0f;
        const u32x4 raw = *reinterpret_cast<const u32x4*>(x + i * 8);
        float v[8];
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            v[2 * w] = bf16_bits_to_float(raw[w] & 0xffffu) / descale;
            v[2 * w + 1] = bf16_bits_to_float(raw[w] >> 16) / descale;
        }
        // The conversion instruction rounds to nearest even, subnormals included, but turns magnitudes of
        // 464 and more into NaN instead of saturating: clamp first (448 is representable).
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = fminf(fmaxf(v[e], -448.0f), 448.0f);
        int lo = __builtin_amdgcn_cvt_pk_fp8_f32(v[0], v[1], 0, false);
        lo = __builtin_amdgcn_cvt_pk_fp8_f32(v[2], v[3], lo, true);
        int hi = __builtin_amdgcn_cvt_pk_fp8_f32(v[4], v[5], 0, false);
        hi = __builtin_amdgcn_cvt_pk_fp8_f32(v[6], v[7], hi, true);
        typedef int i32x2 __attribute__((ext_vector_type(2)));
        *reinterpret_cast<i32x2*>(codes + i * 8) = i32x2{lo, hi};
    }
}

__global__ void quant_descale_kernel(float* descale, int H) {
    const int h = blockIdx.x * blockDim.x + threadIdx.x;
    if (h < H) {
        const float s = descale[h] / 448.0f;  // still the maximum here
        descale[h] = s > 0.0f ? s : 1.0f;
    }
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

}  // namespace va
