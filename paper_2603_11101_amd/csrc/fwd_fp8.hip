// Forward kernel, FP8: Q, K, V are OCP E4M3 bytes with one float32 descale per
// head, or (template flag BLOCK) one per 128 tokens of a sample and head, handed
// over as one value per token row and head; both products run on v_mfma_f32_32x32x64_f8f6f4 (64 contraction slots
// per instruction, twice the bf16 rate); scores, softmax, row sums and LSE are
// float32; the probabilities are requantised to E4M3 for the second product.
//
// The paper's FP8 material (section 2.2.3) concerns weight quantisation and
// only supplies the scaling vocabulary; the per-head scale is its per-channel
// rule applied along the head axis, the block scale its block-wise rule applied
// to (tokens of one sample) x (one head).  Everything else here is this library's.
//
// Block scales in the kernel.  A lane owns one query row, so the Q scale is a
// per-lane constant.  A key tile (64 keys from a multiple of 64 in the sample)
// lies inside one 128-token block, so the K and V scales are one pair of
// numbers per tile, read from the tile's first row one tile ahead.  The K scale
// multiplies the score factor.  The V scale is folded into the exponent: the
// kernel runs its online softmax on score' = score + log2(v_descale), so that
// what it requantises to E4M3 and feeds to the second product is p * v_descale
// (up to the common reference), and sum(p * v_descale * V8) needs no rescaling
// of O when the block changes; the row sum takes psum / v_descale per tile,
// which removes the factor again.
//
// Head dimensions 64, 128 and 256 (one, two or four contraction steps of the first product; two, four or
// eight 32-row blocks of O^T; one workgroup per CU at 256, where the tiles and the output staging take
// 128 KiB of LDS).
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
#include <type_traits>

#include "kernels.h"
#include "mfma_util.h"
#include "work_fetch.h"

namespace va {

namespace {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kPShift = 8.0f;  // probabilities are stored as p * 2^8 in E4M3
// The softmax reference may trail a row's true maximum by this many powers of two before O is rescaled:
// the stored probabilities then reach 2^(8 + 0.75) = 431, still below the largest E4M3 value 448.
constexpr float kMaxLag = 0.75f;

typedef int i32x8 __attribute__((ext_vector_type(8)));
typedef int i32x2 __attribute__((ext_vector_type(2)));

// "This value is needed here": makes the compiler place its wait for an ordinary load at this point (see
// settle() in mfma_util.h).  Plain functions, not statements inside the kernel template: an operand whose
// type depends on a template parameter would have its constraint checked against the host target as well.
VA_DEV void settle8(const i32x8& f) { asm volatile("" ::"v"(f)); }
VA_DEV void settle_scalar(float f) { asm volatile("" ::"v"(f)); }

VA_DEV f32x16 mfma_f8(i32x8 a, i32x8 b, f32x16 c) {
    // formats 0 = E4M3 for both operands; block scales 127 = 2^0
    return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, c, 0, 0, 0, 127, 0, 127);
}

// LDS tile of 64 rows x D bytes (D = head dimension, one byte per value), 16-byte chunks, chunk c of row r
// stored at c ^ swz(r).  Conflict free for (1) 16 lanes reading one chunk of the rows
// {x, 32 + x : x in 0..7} (+ 16 b), and (2) 32 lanes reading 8 consecutive rows by 32 bytes with the
// transposing byte read.  A 256-byte line of the 64 banks holds 256 / D rows; the rows that share a line
// (and, for (2), the two chunks a lane pair reads) must land on different chunk positions:
//   D =  64: 4 rows per line; rows r, r + 4 (bit 2) and r + 32 (bit 5) share a line position -> bits 1, 0
//   D = 128: 2 rows per line; bits 1-2 of the row choose among 4 chunk pairs, bit 5 the chunk of the pair
//   D = 256: one row per line; bits 0-2 of the row choose among 8 chunk pairs, bit 5 the chunk of the pair
template <int D>
__host__ __device__ constexpr int swz8(int r) {
    constexpr int shift = D == 64 ? 2 : D == 128 ? 1 : 0, mask = D == 64 ? 1 : D == 128 ? 3 : 7;
    return (((r >> shift) & mask) << 1) | ((r >> 5) & 1);
}
template <int D>
__host__ __device__ constexpr int off8(int r, int c) { return r * D + ((c ^ swz8<D>(r)) << 4); }

template <int D>
constexpr int kTileBytesOf = kFwdKvTile * D;  // 64 rows of D bytes

// Both access patterns against the 64 banks of 4 bytes: every bank at most once per group of lanes that is
// served together (16 lanes of a 16-byte read, 32 lanes of an 8-byte transposing read).
template <int D>
constexpr bool swz8_conflict_free() {
    for (int b = 0; b < 2; ++b)
        for (int quarter = 0; quarter < 4; ++quarter)
            for (int c = 0; c < D / 16; ++c) {
                bool used[16] = {};
                for (int i = 0; i < 16; ++i) {
                    const int l32 = (quarter & 1) * 16 + i;
                    const int r = 32 * ((l32 >> 2) & 1) + 4 * (l32 >> 3) + (l32 & 3) + 16 * b;
                    const int slot = (off8<D>(r, c) % 256) / 16;
                    if (used[slot]) return false;
                    used[slot] = true;
                }
            }
    for (int r0 = 0; r0 < 64; r0 += 8)
        for (int dt = 0; dt < D / 32; ++dt) {
            bool used[32] = {};
            for (int i = 0; i < 32; ++i) {
                const int r = r0 + (i & 15) / 2, c = 2 * dt + (i >> 4);
                const int slot = ((off8<D>(r, c) + 8 * (i & 1)) % 256) / 8;
                if (used[slot]) return false;
                used[slot] = true;
            }
        }
    return true;
}
static_assert(swz8_conflict_free<64>() && swz8_conflict_free<128>() && swz8_conflict_free<256>(),
              "the tile swizzle leaves a bank conflict");

// Asynchronous copy of one 64 x D-byte tile by 4 waves (see AsyncTile in mfma_util.h): a wave instruction
// fills 1 KiB of the tile (1024 / D rows); the lane that fills chunk position pc of row r fetches chunk
// pc ^ swz(r) of that row, so the swizzle costs nothing.
template <int D>
struct AsyncTile8 {
    static constexpr int CPR = D / 16, RPI = 64 / CPR, INSTR = 64 / RPI, PER_WAVE = INSTR / 4;
    int voff[PER_WAVE];
    int first;
    VA_DEV void init(int wave, int lane, int row_bytes) {
        first = __builtin_amdgcn_readfirstlane(wave * PER_WAVE);
        const int pc = lane % CPR;
#pragma unroll
        for (int j = 0; j < PER_WAVE; ++j) {
            const int r = (wave * PER_WAVE + j) * RPI + lane / CPR;
            voff[j] = r * row_bytes + ((pc ^ swz8<D>(r)) << 4);
        }
    }
    VA_DEV void issue(i32x4 rsrc, unsigned tile_lds, int soffset) const {
#pragma unroll
        for (int j = 0; j < PER_WAVE; ++j) buffer_load_lds_16(tile_lds + (first + j) * 1024, voff[j], rsrc, soffset);
    }
};

// Per-lane LDS offsets of the two fragment patterns in closed form: one lane constant XOR a
// compile-time constant, plus a compile-time row step.
//
// K fragment (first operand of S^T): A-lane l32 of block b reads tile row a_row + 16 b with
// a_row = 32 (bit 2 of l32) + 4 (l32 / 8) + l32 % 4, contraction slots d = 64 t + 32 hf + 0..31, i.e. the
// chunks 4 t + 2 hf and 4 t + 2 hf + 1.
// V^T fragment (first operand of O^T): column d = 32 dt + l32, keys 32 hf + 0..31 through four
// transposing byte reads.  In a group of 16 lanes, lane i receives byte (i % 8) of the 8 bytes addressed
// by lane 2 e + i / 8 as element e (measured); lane s of the group therefore points at row s / 2,
// columns 8 (s % 2) .. + 7 of an 8 x 16 block.
template <int D>
struct FragAddr8 {
    static __host__ __device__ constexpr int a_row(int lane) {
        const int l32 = lane & 31;
        return 32 * ((l32 >> 2) & 1) + 4 * (l32 >> 3) + (l32 & 3);
    }
    static __host__ __device__ constexpr int k_base(int lane) {
        const int r = a_row(lane), hf = lane >> 5;
        return r * D + (((2 * hf) ^ swz8<D>(r)) << 4);
    }
    static __host__ __device__ constexpr int k_off(int lane, int b, int t, int e) {
        return (k_base(lane) ^ ((4 * t + e) << 4)) + b * 16 * D;
    }
    static __host__ __device__ constexpr int v_base(int lane) {
        const int hf = lane >> 5, s16 = lane & 15;
        const int r = 32 * hf + (s16 >> 1);
        const int chunk = (lane >> 4) & 1;  // chunk of the lane's 8 columns inside a 32-column block
        return r * D + ((chunk ^ swz8<D>(r)) << 4) + 8 * (s16 & 1);
    }
    static __host__ __device__ constexpr int v_off(int lane, int x, int dt) {
        return (v_base(lane) ^ ((2 * dt) << 4)) + x * 8 * D;
    }
    static constexpr bool self_check() {
        for (int lane = 0; lane < 64; ++lane) {
            const int hf = lane >> 5, s16 = lane & 15;
            for (int b = 0; b < 2; ++b)
                for (int t = 0; t < D / 64; ++t)
                    for (int e = 0; e < 2; ++e)
                        if (k_off(lane, b, t, e) != off8<D>(a_row(lane) + 16 * b, 4 * t + 2 * hf + e)) return false;
            for (int x = 0; x < 4; ++x)
                for (int dt = 0; dt < D / 32; ++dt) {
                    const int col = 32 * dt + 16 * ((lane >> 4) & 1) + 8 * (s16 & 1);
                    const int vr = 32 * hf + 8 * x + (s16 >> 1);
                    if (v_off(lane, x, dt) != off8<D>(vr, col >> 4) + (col & 8)) return false;
                }
        }
        return true;
    }
    static_assert(self_check(), "fragment address closed forms disagree with the tile layout");
    int kb, vb;
    VA_DEV explicit FragAddr8(int lane) : kb(k_base(lane)), vb(v_base(lane)) {}
    // `tile` is a multiple of the tile size and the lane constants lie below it, so the compile-time chunk bits
    // can be XOR-ed into the lane constant first: those values do not change from tile to tile, and what is left
    // per tile is one addition each.
    VA_DEV i32x8 k_frag(const char* lds, int tile, int b, int t) const {
        const int lo_at = (kb ^ ((4 * t) << 4)) + tile + b * 16 * D;
        const int hi_at = (kb ^ ((4 * t + 1) << 4)) + tile + b * 16 * D;
        const i32x4 lo = *reinterpret_cast<const i32x4*>(lds + lo_at);
        const i32x4 hi = *reinterpret_cast<const i32x4*>(lds + hi_at);
        return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    }
    VA_DEV i32x8 v_frag(const char* lds, int tile, int dt) const {
        typedef __attribute__((address_space(3))) i32x2* lds_i32x2;
        const int at = (vb ^ ((2 * dt) << 4)) + tile;
        i32x8 vf;
#pragma unroll
        for (int x = 0; x < 4; ++x) {
            const i32x2 two = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_i32x2)(lds_char*)(lds + at + x * 8 * D));
            vf[2 * x] = two[0];
            vf[2 * x + 1] = two[1];
        }
        return vf;
    }
};

// Persistent like the bf16 forward: workgroup b runs the works the host assigned to it; the first K/V tile
// and the Q fragments of the next work are fetched while the last key tile of the current one is processed.
// WINDOW: the sliding-window mask, as in the bf16 forward (the P word of a work holds the width W; key
// tiles below the window of the work's first row are not visited, those reaching below the window of its
// last row carry the mask).
template <int D, int HPB, bool BLOCK, bool WINDOW>
__global__ __launch_bounds__(256, D <= 128 ? 2 : 1) void fwd_fp8_kernel(AttnParams p) {
    constexpr int kTileBytes = kTileBytesOf<D>;
    constexpr int BMT = kFwdBlockRows / HPB;
    constexpr int BN = kFwdKvTile;
    constexpr int KSTEPS = D / 64;
    constexpr int DT = D / 32;
    // two stages of (K tile, V tile), then one 32 x D bf16 slice per wave for the output rows
    extern __shared__ __attribute__((aligned(16))) char smem[];
    constexpr int kStaging = 2 * 2 * kTileBytes;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int hf = lane >> 5, l32 = lane & 31;
    RowWorkStream<HPB> works{p, lane};
    RowWork cur;
    if (!works.start((int)blockIdx.x, &cur)) return;

    const int kv_row_bytes = p.Hkv * D;
    const int tile_step = __builtin_amdgcn_readfirstlane(BN * kv_row_bytes);
    const unsigned smem_lds = lds_addr(smem);
    AsyncTile8<D> loader;
    loader.init(wave, lane, kv_row_bytes);
    const FragAddr8<D> fa(lane);

    // first key tile a work visits: 0 unless the window has moved past it
    auto first_tile = [&](const RowWork& w) {
        return WINDOW ? max(0, w.q_row0 - w.seq_row0 + 1 - w.P) / BN : 0;
    };
    auto kv_rsrc = [&](const void* base, const RowWork& w) {
        return make_rsrc(static_cast<const char*>(base) + ((size_t)w.seq_row0 * p.Hkv + w.g) * D,
                         (unsigned)(w.L - 1) * kv_row_bytes + D);
    };
    // the stacked row this lane owns
    const int row = wave * 32 + l32;
    const int tok = row % BMT, head_in_block = row / BMT;
    const int q_tok_bytes = p.Hq * D;
    // Q fragments of that row, contraction slots d = 64 t + 32 hf + 0..31, through a raw buffer that ends
    // with the last valid token of the block: rows past it read as zero.  The score factor
    // scale * q_descale[h] * k_descale[g] * log2(e) of the row comes with them; with block scales it is
    // scale * q_descale[row, h] * log2(e), and the K and V scales of the work's first key tile come too.
    i32x8 qf[KSTEPS];
    float c_row;
    float kd_next = 1.0f, vd_next = 1.0f;  // BLOCK: scales of the key tile that is processed next
    const int kv_descale_step = __builtin_amdgcn_readfirstlane(BN * p.Hkv * 4);
    const __amdgpu_buffer_rsrc_t kd_all = RowBlock<D>::rows(p.k_descale, BLOCK ? (unsigned)p.T * p.Hkv * 4u : 0u);
    const __amdgpu_buffer_rsrc_t vd_all = RowBlock<D>::rows(p.v_descale, BLOCK ? (unsigned)p.T * p.Hkv * 4u : 0u);
    auto load_kv_descale = [&](const RowWork& w, int kt) {
        const int soff = __builtin_amdgcn_readfirstlane((w.seq_row0 * p.Hkv + w.g) * 4 + kt * kv_descale_step);
        kd_next = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(kd_all, 0, soff, 0));
        vd_next = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(vd_all, 0, soff, 0));
    };
    auto load_q = [&](const RowWork& w) {
        const __amdgpu_buffer_rsrc_t rows = RowBlock<D>::rows(
            static_cast<const char*>(p.q) + ((size_t)w.q_row0 * p.Hq + w.h0) * D,
            (unsigned)(w.q_rows - 1) * q_tok_bytes + HPB * D);
        const int off = tok * q_tok_bytes + head_in_block * D + 32 * hf;
#pragma unroll
        for (int t = 0; t < KSTEPS; ++t) {
            const u32x4 lo = __builtin_amdgcn_raw_buffer_load_b128(rows, off + 64 * t, 0, 0);
            const u32x4 hi = __builtin_amdgcn_raw_buffer_load_b128(rows, off + 64 * t + 16, 0, 0);
            qf[t] = __builtin_bit_cast(i32x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
        }
        if constexpr (BLOCK) {
            const __amdgpu_buffer_rsrc_t qd_rows = RowBlock<D>::rows(
                p.q_descale + (size_t)w.q_row0 * p.Hq + w.h0, (unsigned)((w.q_rows - 1) * p.Hq + HPB) * 4u);
            const float qd = __builtin_bit_cast(
                float, __builtin_amdgcn_raw_buffer_load_b32(qd_rows, (tok * p.Hq + head_in_block) * 4, 0, 0));
            // rows past the block read 0: give them a factor that keeps their (unused) arithmetic finite
            c_row = p.scale * kLog2e * (tok < w.q_rows ? qd : 1.0f);
            load_kv_descale(w, first_tile(w));
        } else {
            c_row = p.scale * p.q_descale[w.h0 + head_in_block] * p.k_descale[w.g] * kLog2e;
        }
    };
    // output rows and the LSE store that leave at the end of a work: vector memory operations younger than
    // the loads of the next work's first tile
    constexpr int kEpilogueStores = RowBlock<D>::N + 1;
    const int o_tok_bytes = p.Hq * D * 2;
    auto out_soff = [&](int j) {
        const int rr = __builtin_amdgcn_readfirstlane(wave * 32 + j * RowBlock<D>::RPI);
        return (rr % BMT) * o_tok_bytes + (rr / BMT) * (D * 2);
    };

    int stage = 0;
    loader.issue(kv_rsrc(p.k, cur), smem_lds, first_tile(cur) * tile_step);
    loader.issue(kv_rsrc(p.v, cur), smem_lds + kTileBytes, first_tile(cur) * tile_step);
    load_q(cur);
    // Every ordinary load is consumed before the loop head, here and at the end of a work, so that the
    // compiler has no wait of its own to place at the top of a work, where output rows are still leaving.
    auto settle_q = [&] {
#pragma unroll
        for (int t = 0; t < KSTEPS; ++t) settle8(qf[t]);
        settle_scalar(c_row);
        if constexpr (BLOCK) {
            settle_scalar(kd_next);
            settle_scalar(vd_next);
        }
    };
    settle_q();

    for (;;) {
        const bool has_next = works.has_next();
        const RowWork nxt = works.peek_next();
        const i32x4 k_rsrc = kv_rsrc(p.k, cur), v_rsrc = kv_rsrc(p.v, cur);
        const bool row_valid = tok < cur.q_rows;
        const int row_in_sample = cur.q_row0 - cur.seq_row0 + tok;
        const int vis = WINDOW ? row_in_sample + 1 : RowMask(cur.P, cur.P2, cur.L, p.mask_mode).vis(row_in_sample);
        const int lo = WINDOW ? max(0, row_in_sample + 1 - cur.P) : 0;
        const float c = c_row;
        const float v_descale = BLOCK ? 1.0f : p.v_descale[cur.g];

        f32x16 o[DT];
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int r = 0; r < 16; ++r) o[dt][r] = 0.0f;
        float m = -INFINITY;  // reference point of the exponentials, base 2
        float lsum = 0.0f;    // sum of p * 2^8, this lane's share

        wait_async_loads_except<kEpilogueStores>();  // the first tile has landed; the last work's output may still be leaving
        __syncthreads();

        auto tile = [&](const int kt, auto last_tag, auto masked_tag) {
            constexpr bool last = decltype(last_tag)::value;
            constexpr bool masked = decltype(masked_tag)::value;
            const int j0 = kt * BN;
            const int k_tile = stage * 2 * kTileBytes;
            const int v_tile = k_tile + kTileBytes;
            // Block scales of this tile: score factor, log2 of the V scale, its reciprocal.  They were loaded a
            // tile ago and are consumed here, before anything new is issued, so that no wait for them can
            // land behind the loads of the next tile.
            float ct = c, lv = 0.0f, rvd = 1.0f;
            if constexpr (BLOCK) {
                ct = c * kd_next;
                lv = __builtin_amdgcn_logf(vd_next);  // base 2
                rvd = __builtin_amdgcn_rcpf(vd_next);
                asm volatile("" : "+v"(ct), "+v"(lv), "+v"(rvd));
                if constexpr (!last) load_kv_descale(cur, kt + 1);
            }
            {
                const unsigned nk = smem_lds + (stage ^ 1) * 2 * kTileBytes;
                if constexpr (!last) {
                    loader.issue(k_rsrc, nk, (kt + 1) * tile_step);
                    loader.issue(v_rsrc, nk + kTileBytes, (kt + 1) * tile_step);
                } else if (has_next) {
                    loader.issue(kv_rsrc(p.k, nxt), nk, first_tile(nxt) * tile_step);
                    loader.issue(kv_rsrc(p.v, nxt), nk + kTileBytes, first_tile(nxt) * tile_step);
                }
            }
            // S^T: two blocks of 32 keys x 32 query rows, alternating so that no MFMA waits for the last one.
            // Register r of half hf of block b holds key 32 hf + 16 b + r of the tile (see the top of the file).
            f32x16 s[2];
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int r = 0; r < 16; ++r) s[b][r] = 0.0f;
#pragma unroll
            for (int t = 0; t < KSTEPS; ++t)
#pragma unroll
                for (int b = 0; b < 2; ++b) s[b] = mfma_f8(fa.k_frag(smem, k_tile, b, t), qf[t], s[b]);
            // the Q fragments are free now: those of the next work can start loading
            if constexpr (last) {
                if (has_next) load_q(nxt);
            }
            if constexpr (masked) {
#pragma unroll
                for (int b = 0; b < 2; ++b)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        if (j0 + 32 * hf + 16 * b + r >= vis || (WINDOW && j0 + 32 * hf + 16 * b + r < lo)) s[b][r] = -INFINITY;
            }
            // V^T fragments on their way while the softmax runs
            i32x8 vf[DT];
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) vf[dt] = fa.v_frag(smem, v_tile, dt);

            float mx = s[0][0];
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[b][r]);
            mx = pair_max(mx) * ct;
            if constexpr (BLOCK) mx += lv;
            if (__builtin_amdgcn_ballot_w64(mx > m + kMaxLag) != 0) {  // wave-uniform: some row needs a new reference
                asm volatile("");  // keep this a branch: folded into a select, its multiplications would run on every tile
                const float m_new = fmaxf(m, mx);
                // a row that has seen no key yet keeps m = -inf and takes the reference 0 for this tile
                const float alpha = __builtin_amdgcn_exp2f(m - (m_new == -INFINITY ? 0.0f : m_new));
                m = m_new;
                lsum *= alpha;
#pragma unroll
                for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                    for (int r = 0; r < 16; ++r) o[dt][r] *= alpha;
            }
            const float shift = (BLOCK ? kPShift + lv : kPShift) - (m == -INFINITY ? 0.0f : m);
            float psum = 0.0f;
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float pv = __builtin_amdgcn_exp2f(__builtin_fmaf(s[b][r], ct, shift));
                    s[b][r] = pv;
                    psum += pv;
                }
            lsum += BLOCK ? psum * rvd : psum;

            // P^T operand: byte e of the lane = register e % 16 of block e / 16 = key 32 hf + e
            i32x8 pf;
#pragma unroll
            for (int w = 0; w < 8; ++w) {
                const int b = w >> 2, r = (w & 3) * 4;
                // The low half first; the half it leaves alone is overwritten next, so whatever the destination
                // register holds serves as the old value: the empty statement declares it defined, at no cost (a zero,
                // or a copy of a live value, would have to be moved there first: one more instruction per word).
                int word;
                asm volatile("" : "=v"(word));
                word = __builtin_amdgcn_cvt_pk_fp8_f32(s[b][r], s[b][r + 1], word, false);
                word = __builtin_amdgcn_cvt_pk_fp8_f32(s[b][r + 2], s[b][r + 3], word, true);
                pf[w] = word;
            }
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) o[dt] = mfma_f8(vf[dt], pf, o[dt]);

            stage ^= 1;
            if constexpr (!last) {
                wait_async_loads();
                __syncthreads();
            }
        };
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
        // O = v_descale * (V8^T P8) / sum(p * 2^8): the 2^8 of the stored probabilities cancels.  The rows
        // leave through this wave's own staging slice, so no other wave has to be waited for.
        store_block_rows<D>(smem + kStaging + wave * (32 * D * 2), o, v_descale / lsum, lane,
                            RowBlock<D>::rows(static_cast<__bf16*>(p.out) + ((size_t)cur.q_row0 * p.Hq + cur.h0) * D,
                                              (unsigned)(cur.q_rows - 1) * o_tok_bytes + HPB * D * 2),
                            RowBlock<D>::lane_offset(lane, o_tok_bytes), out_soff);
        {
            const __amdgpu_buffer_rsrc_t lse_rows =
                RowBlock<D>::rows(p.lse + (size_t)cur.h0 * p.T + cur.q_row0, (unsigned)((HPB - 1) * p.T + cur.q_rows) * 4u);
            const int off = (row_valid && hf == 0) ? (head_in_block * p.T + tok) * 4 : 0x7ffffff0;
            __builtin_amdgcn_raw_buffer_store_b32(
                __builtin_bit_cast(unsigned, (m + __builtin_amdgcn_logf(lsum) - kPShift) * kLn2), lse_rows, off, 0, 0);
        }
        if (!has_next) break;
        settle_q();
        works.advance();
        cur = nxt;
    }
}

template <int D, int HPB, bool BLOCK, bool WINDOW>
hipError_t launch_w(const AttnParams& p, hipStream_t stream) {
    // two stages of (K tile, V tile), then one 32 x D bf16 staging slice per wave
    constexpr size_t smem = 2 * 2 * kTileBytesOf<D> + 4 * 32 * D * 2;
    const hipError_t attr = VA_ALLOW_DYNAMIC_LDS((&fwd_fp8_kernel<D, HPB, BLOCK, WINDOW>), smem);
    if (attr != hipSuccess) return attr;
    hipLaunchKernelGGL((fwd_fp8_kernel<D, HPB, BLOCK, WINDOW>), dim3((unsigned)p.num_workgroups), dim3(256), smem, stream, p);
    return hipGetLastError();
}

template <int D, int HPB, bool BLOCK>
hipError_t launch_h(const AttnParams& p, hipStream_t stream) {
    if (p.mask_mode == VA_MASK_SLIDING_WINDOW) return launch_w<D, HPB, BLOCK, true>(p, stream);
    return launch_w<D, HPB, BLOCK, false>(p, stream);
}

template <int D, bool BLOCK>
hipError_t launch_b(const AttnParams& p, hipStream_t stream) {
    switch (heads_per_block(p.Hq, p.Hkv)) {
        case 1: return launch_h<D, 1, BLOCK>(p, stream);
        case 2: return launch_h<D, 2, BLOCK>(p, stream);
        case 4: return launch_h<D, 4, BLOCK>(p, stream);
        default: return launch_h<D, 8, BLOCK>(p, stream);
    }
}

template <int D>
hipError_t launch_d(const AttnParams& p, bool blockwise, hipStream_t stream) {
    return blockwise ? launch_b<D, true>(p, stream) : launch_b<D, false>(p, stream);
}

}  // namespace

hipError_t launch_fwd_fp8(const AttnParams& p, bool blockwise, hipStream_t stream) {
    if (p.num_items == 0) return hipSuccess;
    switch (p.D) {
        case 64: return launch_d<64>(p, blockwise, stream);
        case 128: return launch_d<128>(p, blockwise, stream);
        case 256: return launch_d<256>(p, blockwise, stream);
        default: return hipErrorNotSupported;
    }
}

}  // namespace va
