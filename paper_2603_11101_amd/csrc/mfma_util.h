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

#include "../../include/varlen_attn.h"

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

// ---------------------------------------------------------------- masks
//
// Every mask of the library has the form "local query row i sees keys j < vis(i)" with vis
// non-decreasing: causal i + 1; prefix-LM P for i < P, else L; prefix-LM with causal suffix P for
// i < P, else i + 1.  Branch-free so that it can sit in per-element code.
struct RowMask {
    int P;   // end of the first block (0 when causal)
    int P2;  // end of the second block (0 unless the mask has three blocks)
    int SF;  // L when the rows behind the blocks see the whole sample, else 0
    int L;
    VA_DEV RowMask(int item_P, int item_P2, int item_L, int mode)
        : P(item_P < 0 ? 0 : item_P),
          P2(item_P2 < 0 ? 0 : item_P2),
          SF(mode == VA_MASK_PREFIX_LM || mode == VA_MASK_THREE_BLOCK ? item_L : 0),
          L(item_L) {}
    // Every arm is computed before it is chosen, so that these stay selects and never become branches.
    // THREE = false leaves the second block out: for kernels instantiated per mask family, where the
    // extra select per row would be paid by the masks that have no second block.
    template <bool THREE = true>
    VA_DEV int vis(int i) const {  // any i >= 0
        const int behind = max(i + 1, SF);
        const int second = (THREE && i < P2) ? P2 : behind;
        return i < P ? P : second;
    }
    template <bool THREE = true>
    VA_DEV int vis_in_sample(int i) const {  // rows past the sample see nothing
        const int v = vis<THREE>(i);
        return i < L ? v : 0;
    }
};

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
__host__ __device__ constexpr int swizzle(int r) {
    return D == 64 ? ((((r >> 1) & 1) << 2) | ((r >> 2) & 3)) : (((r & 3) << 2) | ((r >> 2) & 3));
}

// Byte offset inside a tile of the 16-byte chunk c of row r.
template <int D>
__host__ __device__ constexpr int tile_off(int r, int c) {
    return r * (D * 2) + ((c ^ swizzle<D>(r)) << 4);
}

typedef __attribute__((address_space(3))) char lds_char;

// Per-lane constants of the two fragment patterns, so that the address of a fragment is one XOR
// (plus an immediate) away from a value computed once per kernel.
//
// Row-major fragment (contraction over D): the lane reads row 32 b + lane % 32, k-slots
// d = 16 t + 8 hf + 0..7, i.e. chunk 2 t + hf.  The swizzle of that row only depends on lane % 32 and
// only touches chunk bits, so   offset(b, t) = (rm ^ (t << 5)) + b * 32 rows.
//
// Transposed fragment (contraction over token rows): the lane wants column 32 dt + lane % 32 and the
// 8 token rows 16 x + {4 hf + 0..3, 8 + 4 hf + 0..3}, the order in which a 32x32 accumulator holds
// its rows (acc_row), so a product whose other operand comes straight out of an accumulator lines up.
// ds_read_b64_tr_b16 works on groups of 16 lanes: lane i of a group receives, as element e, the
// 16-bit word (i % 4) of the 8 bytes addressed by lane 4 e + i / 4 of the group (measured).  Lane s of
// a group therefore points at row s / 4, columns 4 (s % 4) .. + 3 of a 4 x 16 block, and lane i gets
// column i of the block, rows 0..3.  Two reads (rows + 0 and + 8) make one fragment:
//   offset(j, x, dt) = (tr ^ (j << 5) ^ (dt << 6)) + (8 j + 16 x) rows.
template <int D>
struct FragAddr {
    int rm;
    int tr;

    static __host__ __device__ constexpr int rm_base(int lane) {
        const int l32 = lane & 31, hf = lane >> 5, sw = swizzle<D>(l32);
        return l32 * (D * 2) + ((hf ^ (sw & 1)) << 4) + ((sw >> 1) << 5);
    }
    static __host__ __device__ constexpr int tr_base(int lane, int j) {
        const int hf = lane >> 5, s = lane & 15;
        const int r = 4 * hf + (s >> 2) + 8 * j;
        const int sw = swizzle<D>(r);
        const int cl = 2 * ((lane >> 4) & 1) + ((s & 3) >> 1);  // chunk of the lane's 4 columns inside a 32-column block
        const int half = (s & 1) << 3;                          // which 8 bytes of the chunk
        return r * (D * 2) + half + ((cl ^ (sw & 3)) << 4) + ((sw >> 2) << 6);
    }
    static __host__ __device__ constexpr int rm_off(int lane, int b, int t) {
        return (rm_base(lane) ^ (t << 5)) + b * 32 * (D * 2);
    }
    // The second read (rows + 8) needs no base of its own: eight rows further down the swizzle differs
    // in one chunk bit, so its offset is that of the first read XOR 32, plus eight rows.
    static __host__ __device__ constexpr int tr_off(int lane, int j, int x, int dt) {
        return ((tr_base(lane, 0) ^ (j << 5)) ^ (dt << 6)) + j * 8 * (D * 2) + x * 16 * (D * 2);
    }
    // the closed forms against the plain definition, every lane and step
    static constexpr bool self_check() {
        for (int lane = 0; lane < 64; ++lane) {
            const int l32 = lane & 31, hf = lane >> 5, s = lane & 15;
            for (int b = 0; b < 4; ++b)
                for (int t = 0; t < D / 16; ++t)
                    if (rm_off(lane, b, t) != tile_off<D>(32 * b + l32, 2 * t + hf)) return false;
            for (int j = 0; j < 2; ++j)
                for (int x = 0; x < 8; ++x)
                    for (int dt = 0; dt < D / 32; ++dt) {
                        const int row = 16 * x + 4 * hf + (s >> 2) + 8 * j;
                        const int col = 32 * dt + ((lane >> 4) & 1) * 16 + (s & 3) * 4;
                        if (tr_off(lane, j, x, dt) != tile_off<D>(row, col >> 3) + ((col & 4) << 1)) return false;
                    }
        }
        return true;
    }
    static_assert(self_check(), "fragment address closed forms disagree with the tile layout");

    VA_DEV explicit FragAddr(int lane) : rm(rm_base(lane)), tr(tr_base(lane, 0)) {}

    // `lds` is the base of dynamic shared memory, `tile` the byte offset of the tile inside it: a multiple of
    // kTileAlign.  The compile-time chunk bits (below kTileAlign) are XOR-ed into the lane constant, not into
    // lane constant + tile: those values do not change from tile to tile, so the compiler keeps them in
    // registers and a tile costs one addition per fragment address instead of an addition and an XOR.
    static constexpr int kTileAlign = 512;
    static_assert((15 << 5) < kTileAlign && ((7 << 6) ^ 32) < kTileAlign, "chunk bits must stay below the tile alignment");
    VA_DEV bf16x8 rowmajor(const char* lds, int tile, int b, int t) const {
        return *reinterpret_cast<const bf16x8*>(lds + (((rm ^ (t << 5)) + tile) + b * 32 * (D * 2)));
    }
    VA_DEV bf16x8 transposed(const char* lds, int tile, int x, int dt) const {
        typedef __attribute__((address_space(3))) s16x4* lds_s16x4;
        typedef short s16x8 __attribute__((ext_vector_type(8)));
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (lds_s16x4)(lds_char*)(lds + (((tr ^ (dt << 6)) + tile) + x * 16 * (D * 2))));
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (lds_s16x4)(lds_char*)(lds + (((tr ^ ((dt << 6) ^ 32)) + tile) + 8 * (D * 2) + x * 16 * (D * 2))));
        return __builtin_bit_cast(bf16x8, (s16x8)__builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    }
};

// ---------------------------------------------------------------- asynchronous tile loads
//
// Tiles travel from global memory straight into LDS (buffer_load_dwordx4 ... lds:
// every lane fetches 16 bytes and the hardware writes them to LDS at
// M0 + 16 * lane, no registers involved).  The loads are issued from inline
// assembly so that the compiler does not see them as LDS writes: it would
// otherwise wait for them before the next LDS read that might alias, which
// defeats prefetching into the other stage.  The kernels order them by hand:
// wait_async_loads() and a barrier before the first read of a stage.
//
// The global side is a raw buffer resource covering exactly the rows of one
// sample for one head, so rows past the sample read as zero and are never
// touched in memory.

typedef int i32x4 __attribute__((ext_vector_type(4)));

// Buffer resource for `bytes` bytes starting at `base` (wave-uniform).
VA_DEV i32x4 make_rsrc(const void* base, unsigned bytes) {
    const unsigned long long a = reinterpret_cast<unsigned long long>(base);
    i32x4 r;
    r[0] = __builtin_amdgcn_readfirstlane((int)(a & 0xffffffffu));
    r[1] = __builtin_amdgcn_readfirstlane((int)((a >> 32) & 0xffffu));  // stride 0: raw buffer
    r[2] = __builtin_amdgcn_readfirstlane((int)bytes);
    r[3] = 0x00020000;
    return r;
}

// LDS byte address of a pointer into shared memory (wave-uniform).
VA_DEV unsigned lds_addr(const void* p) {
    return __builtin_amdgcn_readfirstlane((unsigned)(size_t)(lds_char*)p);
}

// lds_dst, rsrc and soffset must be wave-uniform; readfirstlane makes that explicit to the compiler
VA_DEV void buffer_load_lds_16(unsigned lds_dst, int voffset, i32x4 rsrc, int soffset) {
    lds_dst = __builtin_amdgcn_readfirstlane(lds_dst);
    soffset = __builtin_amdgcn_readfirstlane(soffset);
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                 :: "s"(lds_dst), "v"(voffset), "s"(rsrc), "s"(soffset) : "memory");
}
VA_DEV void buffer_load_lds_4(unsigned lds_dst, int voffset, i32x4 rsrc, int soffset) {
    lds_dst = __builtin_amdgcn_readfirstlane(lds_dst);
    soffset = __builtin_amdgcn_readfirstlane(soffset);
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dword %1, %2, %3 offen lds"
                 :: "s"(lds_dst), "v"(voffset), "s"(rsrc), "s"(soffset) : "memory");
}

// A fragment that was loaded from global memory by ordinary loads before a loop that also issues
// asynchronous tile loads: touching it here makes the compiler place its own wait for those ordinary
// loads now, instead of a conservative wait-for-everything at the first use inside the loop (which
// would also wait for the freshly issued tile loads it knows nothing about).
VA_DEV void settle(const bf16x8& f) { asm volatile("" ::"v"(f)); }

VA_DEV void wait_async_loads() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }
// Vector memory operations of a wave complete in issue order: waiting until at most YOUNGER are outstanding
// waits for everything issued before the YOUNGER most recent ones (output rows on their way, say).
template <int YOUNGER>
VA_DEV void wait_async_loads_except() {
    static_assert(YOUNGER >= 0 && YOUNGER < 64, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(YOUNGER) : "memory");
}

// Copy plan of one swizzled ROWS x D bf16 tile shared by NWAVES waves.  One
// wave instruction fills 1 KiB of the tile (64 / (D/8) rows); the lane that
// fills chunk position pc of row r fetches chunk pc ^ swizzle(r) of that row, so
// the swizzle costs nothing.  The per-lane offsets do not depend on which tile
// of the sample is fetched: that goes into the scalar offset of the load.
//
// DR < D: the rows in memory hold DR values (DR * 2 bytes, a multiple of 32) and the tile keeps the
// geometry of D: chunk positions from DR / 8 on are not fetched (their lanes aim past the buffer and the
// hardware writes zeros).  Row bytes are then no multiple of the tile's row size, so the chunk can no
// longer be XOR-ed inside the byte offset and travels in a register of its own.
template <int D, int ROWS, int NWAVES, int DR = D>
struct AsyncTile {
    static constexpr int CPR = D / 8;
    static constexpr int RPI = 64 / CPR;
    static constexpr int INSTR = ROWS / RPI;
    static constexpr int PER_WAVE = INSTR / NWAVES;
    static_assert(INSTR % NWAVES == 0, "tile must divide among the waves");
    // Instruction j of a wave fetches rows RPI * j further down than instruction 0.  Their swizzles differ
    // from those of instruction 0 by the same constant for every lane and wave, so one per-lane offset
    // serves all instructions: offset(j) = (voff0 ^ (swizzle(RPI j) << 4)) + RPI j rows.
    static constexpr bool self_check() {
        for (int w = 0; w < NWAVES; ++w)
            for (int j = 0; j < PER_WAVE; ++j)
                for (int x = 0; x < RPI; ++x)
                    if ((swizzle<D>((w * PER_WAVE + j) * RPI + x) ^ swizzle<D>(w * PER_WAVE * RPI + x)) != swizzle<D>(j * RPI))
                        return false;
        return true;
    }
    static_assert(self_check(), "the swizzle does not separate into a lane part and an instruction part");
    int voff0;
    int chunk0;    // DR < D only: chunk fetched by instruction 0 (voff0 then holds the row part alone)
    int first;     // first instruction of this wave
    int row_step;  // bytes between the rows of consecutive instructions

    VA_DEV void init(int wave, int lane, int row_bytes) {
        first = __builtin_amdgcn_readfirstlane(wave * PER_WAVE);
        row_step = __builtin_amdgcn_readfirstlane(RPI * row_bytes);
        const int pc = lane % CPR;
        const int r = wave * PER_WAVE * RPI + lane / CPR;
        if constexpr (DR == D) {
            voff0 = r * row_bytes + ((pc ^ swizzle<D>(r)) << 4);
            chunk0 = 0;
        } else {
            voff0 = r * row_bytes;
            chunk0 = pc ^ swizzle<D>(r);
        }
    }
    // tile_lds: LDS address of the tile; soffset: byte offset of the tile's first row in the buffer, which
    // must lie inside the buffer: the range check compares the per-lane offset with the buffer size minus
    // the scalar offset in unsigned arithmetic, so rows past the end are only caught through the per-lane part
    VA_DEV void issue(i32x4 rsrc, unsigned tile_lds, int soffset) const {
        int v = voff0;
        asm volatile("" : "+v"(v));  // derive the offsets here instead of keeping PER_WAVE of them in registers
#pragma unroll
        for (int j = 0; j < PER_WAVE; ++j) {
            if constexpr (DR == D) {
                buffer_load_lds_16(tile_lds + (first + j) * 1024, (v ^ (swizzle<D>(j * RPI) << 4)) + j * row_step, rsrc, soffset);
            } else {
                const int c = chunk0 ^ swizzle<D>(j * RPI);
                const int off = c < DR / 8 ? v + j * row_step + (c << 4) : 0x7ffffff0;
                buffer_load_lds_16(tile_lds + (first + j) * 1024, off, rsrc, soffset);
            }
        }
    }
};

// ---------------------------------------------------------------- operand blocks that stay in registers
//
// A wave's 32 x D operand block (Q and dO of the forward and dQ kernels) lives in registers as
// row-major fragments for a whole work.  Fetching the fragments directly makes every wave instruction
// touch 32 rows with 32 bytes each, and the address path of the vector cache handles one row (cache
// line) at a time.  So the block is fetched with whole rows per group of lanes (64 / (D/8) rows per
// instruction) and turned into fragments through a wave-private, swizzled 32 x D LDS slice.
// DR < D: rows of DR values in memory, geometry of D in LDS and registers; the lanes of the chunks from
// DR / 8 on aim past the buffer (they load zeros and store nothing).
template <int D, int DR = D>
struct RowBlock {
    static constexpr int CPR = D / 8;     // 16-byte chunks of a row
    static constexpr int RPI = 64 / CPR;  // rows per wave instruction
    static constexpr int N = 32 / RPI;    // instructions per block = fragments per lane (D / 16)

    // Per-lane byte offset of the lane's piece in instruction 0: row lane / CPR, chunk lane % CPR.  Meant to
    // be called where it is used: the lane number is made opaque so that the offset is derived on the spot
    // instead of occupying a register for the whole kernel.
    VA_DEV static int lane_offset(int lane, int row_bytes) {
        asm volatile("" : "+v"(lane));
        const int off = (lane / CPR) * row_bytes + (lane % CPR) * 16;
        if constexpr (DR == D) return off;
        return lane % CPR < DR / 8 ? off : 0x7ffffff0;
    }

    // The rows of a block in global memory, seen through a raw buffer of `bytes` bytes at `base`: whatever
    // lies past the end reads as zero and is not written, so ragged blocks need no branch, and an address
    // is one per-lane constant (lane_offset) plus a wave-uniform offset per instruction.
    VA_DEV static __amdgpu_buffer_rsrc_t rows(const void* base, unsigned bytes) {
        // base and bytes are wave-uniform but come out of loaded work records: say so, or every access is
        // wrapped in a loop over the distinct values of the lanes
        const unsigned long long a = reinterpret_cast<unsigned long long>(base);
        const unsigned long long ua = ((unsigned long long)(unsigned)__builtin_amdgcn_readfirstlane((int)(a >> 32)) << 32) |
                                      (unsigned)__builtin_amdgcn_readfirstlane((int)(a & 0xffffffffu));
        return __builtin_amdgcn_make_buffer_rsrc(reinterpret_cast<void*>(ua), 0,
                                                 __builtin_amdgcn_readfirstlane((int)bytes), 0x00020000);
    }

    // soff(j) = byte offset of row j * RPI of the block (wave-uniform; added to the per-lane offset, not
    // passed as the scalar offset of the access: the range check only catches what the per-lane part
    // carries past the end).  After the call regs[j] holds chunk lane % CPR of row j * RPI + lane / CPR.
    // Exactly N load instructions.
    template <typename RowOffset>
    VA_DEV static void load(bf16x8 (&regs)[N], __amdgpu_buffer_rsrc_t rsrc, int lane_off, RowOffset soff) {
#pragma unroll
        for (int j = 0; j < N; ++j)
            regs[j] = __builtin_bit_cast(bf16x8, __builtin_amdgcn_raw_buffer_load_b128(rsrc, lane_off + soff(j), 0, 0));
    }
    // regs as left by load() -> regs[t] = fragment t of row lane % 32 (k-slots d = 16 t + 8 (lane / 32) + 0..7).
    // `slice` is the byte offset of 32 * D * 2 bytes of LDS that no other wave touches meanwhile.
    VA_DEV static void to_fragments(bf16x8 (&regs)[N], char* lds, int slice, const FragAddr<D>& fa, int lane) {
        // the write offsets are derived from the lane number on the spot (see lane_offset)
        asm volatile("" : "+v"(lane));
        const int c = lane % CPR;
#pragma unroll
        for (int j = 0; j < N; ++j)
            *reinterpret_cast<bf16x8*>(lds + slice + tile_off<D>(j * RPI + lane / CPR, c)) = regs[j];
#pragma unroll
        for (int t = 0; t < N; ++t) regs[t] = fa.rowmajor(lds, slice, 0, t);
    }
};

// ---------------------------------------------------------------- coalesced output rows
//
// A wave holds a 32 x D result transposed in its accumulators: lane % 32 is the row, and registers
// 4 q .. 4 q + 3 of block dt hold columns 32 dt + 8 q + 4 (lane / 32) + 0..3.  Stored directly, every
// lane would write 8-byte pieces 2 D bytes apart.  Instead the block goes through 32 * D * 2 bytes of
// LDS that belong to the wave and leaves as whole rows, 16 bytes per lane, 16-byte chunks of one row in
// consecutive lanes.  The 8-byte units of a row are XOR-permuted with a function of the row so that both
// the column-wise writes and the row-wise reads are free of bank conflicts.
template <int D>
__host__ __device__ constexpr int out_stage_perm(int row) { return D == 64 ? ((row >> 1) & 15) : (row & 31); }

// Per-lane LDS offsets of the staging pattern, in the closed form used by store_block_rows: the offset
// of a piece is one lane constant XOR a compile-time constant (plus a compile-time row step), so nothing
// but the two lane constants has to live in registers.
template <int D>
struct OutStage {
    static constexpr int RB = D * 2, CPR = D / 8, RPI = 64 / CPR, N = 32 / RPI;
    // write side: lane (row = lane % 32, hf = lane / 32) writes 8-byte unit 8 dt + 2 q + hf of its row
    static __host__ __device__ constexpr int wbase(int lane) {
        const int row = lane & 31, hf = lane >> 5;
        return row * RB + ((hf ^ out_stage_perm<D>(row)) << 3);
    }
    static __host__ __device__ constexpr int woff(int lane, int dt, int q) { return wbase(lane) ^ ((8 * dt + 2 * q) << 3); }
    // read side: instruction `it`, lane (x = lane / CPR, c = lane % CPR) reads 16-byte chunk c of row it * RPI + x
    static __host__ __device__ constexpr int rbase(int lane) {
        const int x = lane / CPR, c = lane % CPR;
        return x * RB + ((c ^ (out_stage_perm<D>(x) >> 1)) << 4);
    }
    static __host__ __device__ constexpr int roff(int lane, int it) {
        return (rbase(lane) ^ ((out_stage_perm<D>(it * RPI) >> 1) << 4)) + it * RPI * RB;
    }
    static __host__ __device__ constexpr bool rswap(int lane) { return out_stage_perm<D>(lane / CPR) & 1; }
    // the closed forms against the plain definition, every lane and piece
    static constexpr bool self_check() {
        for (int lane = 0; lane < 64; ++lane) {
            const int row = lane & 31, hf = lane >> 5;
            for (int dt = 0; dt < D / 32; ++dt)
                for (int q = 0; q < 4; ++q)
                    if (woff(lane, dt, q) != row * RB + (((8 * dt + 2 * q + hf) ^ out_stage_perm<D>(row)) << 3)) return false;
            for (int it = 0; it < N; ++it) {
                const int r = it * RPI + lane / CPR, c = lane % CPR, pr = out_stage_perm<D>(r);
                if (roff(lane, it) != r * RB + ((c ^ (pr >> 1)) << 4)) return false;
                if (rswap(lane) != bool(pr & 1)) return false;
            }
        }
        return true;
    }
    static_assert(self_check(), "staging offsets disagree with the staging layout");
};

// The rows go out through a raw buffer as in RowBlock (rsrc, lane_off, soff(j) = byte offset of row
// j * RPI): rows past the end of the buffer are dropped by the hardware.  Exactly RowBlock<D>::N store
// instructions, whatever the number of valid rows, so that a later wait can count them.
// NB = number of 32-column blocks the accumulator holds ((DR + 31) / 32 when the rows in memory are
// shorter than the geometry; the lanes of the columns past DR come with a lane_off past the buffer).
template <int D, int NB = D / 32, typename RowOffset>
VA_DEV void store_block_rows(char* stage, const f32x16 (&acc)[NB], float factor, int lane,
                             __amdgpu_buffer_rsrc_t rsrc, int lane_off, RowOffset soff) {
    using S = OutStage<D>;
    // This code runs with few registers free.  The lane constants are made opaque here so that they are
    // derived from the lane number on the spot instead of being kept (or spilled) across the kernel.
    int l = lane;
    asm volatile("" : "+v"(l));
    const int wb = S::wbase(l);
#pragma unroll
    for (int dt = 0; dt < NB; ++dt)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            f32x4 f = {acc[dt][4 * q] * factor, acc[dt][4 * q + 1] * factor, acc[dt][4 * q + 2] * factor,
                       acc[dt][4 * q + 3] * factor};
            *reinterpret_cast<bf16x4*>(stage + (wb ^ ((8 * dt + 2 * q) << 3))) = __builtin_convertvector(f, bf16x4);
            if (q == 3) __builtin_amdgcn_sched_barrier(0);  // bounded live ranges
        }
    // the wave reads back only what it wrote itself
    const int rb = S::rbase(l);
    const bool swap = S::rswap(l);
#pragma unroll
    for (int it = 0; it < S::N; ++it) {
        u32x4 v = *reinterpret_cast<const u32x4*>(
            stage + ((rb ^ ((out_stage_perm<D>(it * S::RPI) >> 1) << 4)) + it * S::RPI * S::RB));
        if (swap) v = u32x4{v[2], v[3], v[0], v[1]};
        __builtin_amdgcn_raw_buffer_store_b128(v, rsrc, lane_off + soff(it), 0, 0);
    }
}

// float pairs -> packed bf16 (round to nearest even)
VA_DEV bf16x8 to_bf16x8(float a0, float a1, float a2, float a3, float a4, float a5, float a6, float a7) {
    f32x8 f = {a0, a1, a2, a3, a4, a5, a6, a7};
    return __builtin_convertvector(f, bf16x8);
}

}  // namespace va
