// Device helpers shared by the attention kernels: vector types, the MFMA
// wrappers, the LDS tile layout and the fragment loads that go with it.
//
// Register layouts of v_mfma_f32_32x32x16_bf16 on gfx950 (wave64), as measured
// on the hardware with one-hot operands:
//   A[i][k]  lane l holds row i = l % 32 and the 8 k-slots of group l / 32
//   B[k][j]  lane l holds column j = l % 32 and the 8 k-slots of group l / 32
//            (slot (group, e) of A meets slot (group, e) of B)
//   D[i][j]  lane l holds column j = l % 32; register r holds row
//            i = 8 * (r / 4) + 4 * (l / 32) + r % 4
// Because the k-slots of A and B pair up one to one, any assignment of the
// contraction index to slots is valid as long as both operands use the same.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace va {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

#define VA_DEV __device__ __forceinline__

VA_DEV f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// Row of D held by accumulator register r of a lane in half hf (= lane / 32).
VA_DEV int acc_row(int r, int hf) { return 8 * (r >> 2) + 4 * hf + (r & 3); }

// v_permlane32_swap exchanges the upper 32 lanes of its first operand with the
// lower 32 lanes of its second (measured); with both equal to x, result[0] is
// the lower half's value and result[1] the upper half's, in both lanes of a
// pair (l, l + 32).
VA_DEV float pair_max(float x) {
    u32x2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
VA_DEV float pair_sum(float x) {
    u32x2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// ---------------------------------------------------------------- LDS tiles
//
// A tile is ROWS token rows of D bf16 values, row-major, cut into 16-byte
// chunks (8 values).  Chunk c of row r is stored at chunk position
// c ^ swizzle(r) of the same row.  The swizzle is chosen so that both access
// patterns of the MFMA fragments are free of bank conflicts (64 banks of
// 4 bytes): (1) 16 lanes reading the same chunk of 16 consecutive rows, and
// (2) 32 lanes reading 4 consecutive rows by 4 consecutive chunks with the
// transposing read.
template <int D>
VA_DEV int swizzle(int r) {
    if (D == 64) return (((r >> 1) & 1) << 2) | ((r >> 2) & 3);
    return ((r & 3) << 2) | ((r >> 2) & 3);
}

// Byte offset inside a tile of the 16-byte chunk c of row r.
template <int D>
VA_DEV int tile_off(int r, int c) {
    return r * (D * 2) + ((c ^ swizzle<D>(r)) << 4);
}

typedef __attribute__((address_space(3))) char lds_char;

VA_DEV bf16x8 lds_read_chunk(const char* tile, int off) {
    return *reinterpret_cast<const bf16x8*>(tile + off);
}

// Operand fragment "rows x k" for a row-major tile whose contraction index is
// the column (the D axis): lane holds row `row`, k-slots d = 16*t + 8*hf + 0..7.
template <int D>
VA_DEV bf16x8 frag_rowmajor(const char* tile, int row, int t, int hf) {
    return lds_read_chunk(tile, tile_off<D>(row, 2 * t + hf));
}

// Operand fragment for a row-major tile whose contraction index is the ROW
// (token) axis: the lane wants column `col` (a D index) and the 8 token rows
// row0 + {4*hf + 0..3, 8 + 4*hf + 0..3}, which is exactly the order in which a
// 32x32 accumulator holds its rows (see acc_row), so a product whose other
// operand comes straight out of an accumulator lines up.
//
// ds_read_b64_tr_b16 works on groups of 16 lanes: lane i of a group receives,
// as element e, the 16-bit word (i % 4) of the 8 bytes addressed by lane
// 4 * e + i / 4 of the group (measured).  Pointing lane s of a group at row
// (s / 4), columns 4 * (s % 4) .. + 3 of a 4 x 16 block therefore hands lane i
// the column i of that block, rows 0..3.
template <int D>
VA_DEV bf16x8 frag_transposed(const char* tile, int row0, int col_base32, int lane) {
    const int hf = lane >> 5;
    const int s = lane & 15;
    const int col = col_base32 + ((lane >> 4) & 1) * 16 + (s & 3) * 4;  // first of the 4 columns this lane addresses
    const int r0 = row0 + 4 * hf + (s >> 2);
    const int r1 = r0 + 8;
    const int chunk = col >> 3;
    const int half = (col & 4) << 1;  // 0 or 8 bytes
    typedef __attribute__((address_space(3))) s16x4* lds_s16x4;
    s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4)(lds_char*)(tile + tile_off<D>(r0, chunk) + half));
    s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4)(lds_char*)(tile + tile_off<D>(r1, chunk) + half));
    typedef short s16x8 __attribute__((ext_vector_type(8)));
    s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, both);
}

// Copy ROWS x D bf16 values from global memory (row stride `gstride` elements)
// into a swizzled LDS tile with 16-byte accesses; rows >= valid_rows are filled
// with zeros and never read from memory.
template <int D, int ROWS, int THREADS>
VA_DEV void load_tile(char* tile, const __bf16* g, size_t gstride, int valid_rows, int tid) {
    constexpr int CPR = D / 8;
    constexpr int CHUNKS = ROWS * CPR;
    static_assert(CHUNKS % THREADS == 0, "tile must divide among the threads");
#pragma unroll
    for (int i = 0; i < CHUNKS / THREADS; ++i) {
        const int cid = tid + i * THREADS;
        const int r = cid / CPR, c = cid % CPR;
        u32x4 val = {0u, 0u, 0u, 0u};
        if (r < valid_rows) val = *reinterpret_cast<const u32x4*>(g + (size_t)r * gstride + c * 8);
        *reinterpret_cast<u32x4*>(tile + tile_off<D>(r, c)) = val;
    }
}

// Asynchronous copy of ROWS x D bf16 values from global memory straight into a
// swizzled LDS tile (global_load_lds_dwordx4: every lane fetches 16 bytes and
// the hardware writes them to LDS at base + 16 * lane, no registers involved).
// One wave instruction fills 1 KiB of the tile; the NWAVES waves of the
// workgroup share the tile's instructions.  The swizzle is applied on the
// global side: the lane that fills chunk position pc of row r fetches chunk
// pc ^ swizzle(r) of that row.  Rows >= valid_rows (>= 1) are filled with a copy
// of the last valid row instead of being read: callers make sure such rows meet
// a zero probability, so a finite stand-in is as good as zero.
// The caller must wait (wait_async_loads) and then barrier before reading.
template <int D, int ROWS, int NWAVES>
VA_DEV void async_load_tile(char* tile, const __bf16* g, size_t gstride, int valid_rows, int wave, int lane) {
    constexpr int CPR = D / 8;
    constexpr int RPI = 64 / CPR;  // rows per wave instruction
    constexpr int INSTR = ROWS / RPI;
    static_assert(INSTR % NWAVES == 0, "tile must divide among the waves");
    typedef __attribute__((address_space(3))) void lds_void;
    typedef __attribute__((address_space(1))) const void glb_void;
    const int pc = lane % CPR;
#pragma unroll
    for (int j = 0; j < INSTR / NWAVES; ++j) {
        const int inst = wave * (INSTR / NWAVES) + j;
        const int r = inst * RPI + lane / CPR;
        const int rc = min(r, valid_rows - 1);
        const __bf16* src = g + (size_t)rc * gstride + ((pc ^ swizzle<D>(r)) << 3);
        __builtin_amdgcn_global_load_lds((glb_void*)src, (lds_void*)(tile + inst * 1024), 16, 0, 0);
    }
}

VA_DEV void wait_async_loads() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// float pairs -> packed bf16 (round to nearest even)
VA_DEV bf16x8 to_bf16x8(float a0, float a1, float a2, float a3, float a4, float a5, float a6, float a7) {
    f32x8 f = {a0, a1, a2, a3, a4, a5, a6, a7};
    return __builtin_convertvector(f, bf16x8);
}

}  // namespace va
