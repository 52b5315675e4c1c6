/*
 * varlen_attn.h - C ABI of the packed variable-length attention library for
 * AMD MI355X (gfx950).
 *
 * The operation is the one behind the paper's "Data Packing" + "Variable-Length
 * Flash-Attention" recipe (section 2.2.1, paragraphs (1) and (2); measured in
 * section 3.2): several samples are concatenated end to end into one token
 * stream, and softmax attention is computed on the valid tokens only, each
 * sample attending to itself alone.  Inside a sample the mask is causal
 * (autoregressive decoder, section 2.2.1 (1)) or prefix-LM (the pi-0.5 case of
 * section 2.2.2: a bidirectional prefix, and a suffix that attends the prefix
 * and the whole suffix), with two variants of the latter listed under "Mask"
 * below.
 *
 * Conventions that hold for every entry point
 *   - Plain C types only.  "host" pointers are ordinary memory; "device"
 *     pointers are HIP device memory owned by the caller, which must stay alive
 *     until the stream has passed the call.
 *   - The library never allocates or frees device memory and never
 *     synchronises; device entry points only enqueue kernels on `stream`
 *     (a hipStream_t passed as void*; NULL = the default stream).
 *   - Return value: VA_OK (0) or a negative VA_E* code; va_last_error() then
 *     holds a message (thread-local, valid until the next failing call on the
 *     same thread).  On error nothing has been enqueued and no output touched.
 *   - Layouts (row-major, innermost last): Q, O, dO, dQ are [T, Hq, D];
 *     K, V, dK, dV are [T, Hkv, D]; LSE is [Hq, T] float32.  T is the number of
 *     packed tokens, cu_seqlens[num_seqs].  Rows >= T of any buffer are never
 *     read or written.  Query head h uses KV head h / (Hq / Hkv).
 *   - Sample s owns rows [cu_seqlens[s], cu_seqlens[s+1]).  Zero-length
 *     samples are legal and produce nothing.
 *   - Mask: local query row i of a sample of length L sees keys j < vis(i):
 *       VA_MASK_CAUSAL                vis(i) = i + 1
 *       VA_MASK_PREFIX_LM             vis(i) = P if i < P else L
 *       VA_MASK_PREFIX_LM_CAUSAL      vis(i) = P if i < P else i + 1
 *       VA_MASK_THREE_BLOCK           vis(i) = P if i < P, P2 if i < P2, else L
 *     with P = prefix_lens[s], 0 <= P <= L.  Under VA_MASK_THREE_BLOCK a sample
 *     is three blocks [0, P), [P, P2), [P2, L), each seeing itself and the
 *     blocks before it (the prefix / state / action layout of flow-matching
 *     action experts, the family section 2.2.2 adapts), and prefix_lens holds
 *     2 * num_seqs entries: P = prefix_lens[2 s], P2 = prefix_lens[2 s + 1],
 *     0 <= P <= P2 <= L.
 *       VA_MASK_SLIDING_WINDOW        vis(i) = i + 1, and the keys start at
 *                                     lo(i) = max(0, i + 1 - W) instead of 0
 *     (causal, at most the W most recent keys, the row's own included), with
 *     W = prefix_lens[s] >= 1 per sample; a W of L or more is the causal mask.
 *   - LSE[h, r] = ln sum_j exp(scale * q_r . k_j) over the visible keys
 *     (natural logarithm, scale included).
 */
#ifndef VARLEN_ATTN_H
#define VARLEN_ATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define VA_OK 0
#define VA_EINVAL (-1)       /* null pointer, negative size, inconsistent arguments */
#define VA_EUNSUPPORTED (-2) /* head_dim not in {48,64,80,96,128,160,192,256}, Hq % Hkv != 0, unknown mask/pass */
#define VA_EALIGN (-3)       /* a tensor pointer is not 16-byte aligned */
#define VA_ESIZE (-4)        /* output/workspace buffer too small, sample longer than budget or max_seqlen */
#define VA_EHIP (-5)         /* the HIP runtime refused a launch */

#define VA_MASK_CAUSAL 0
#define VA_MASK_PREFIX_LM 1
#define VA_MASK_PREFIX_LM_CAUSAL 2
#define VA_MASK_THREE_BLOCK 3
#define VA_MASK_SLIDING_WINDOW 4

#define VA_PASS_FWD 0
#define VA_PASS_BWD_DKDV 1
#define VA_PASS_BWD_DQ 2

/* Shapes shared by the device calls. */
typedef struct {
    int32_t total_tokens; /* T = cu_seqlens[num_seqs] */
    int32_t num_seqs;     /* n */
    int32_t num_q_heads;  /* Hq */
    int32_t num_kv_heads; /* Hkv, Hq % Hkv == 0 */
    int32_t head_dim;     /* D in {48, 64, 80, 96, 128, 160, 192, 256}; the FP8 forward takes 64, 128 and 256 */
    int32_t max_seqlen;   /* >= every sample length; validation only, never changes results */
    int32_t mask_mode;    /* VA_MASK_* ; VA_MASK_CAUSAL ignores prefix_lens */
} va_shape;

/* Message of the last failing call on this thread (static storage).  This library's own; no passage of the
 * paper. */
const char* va_last_error(void);

/* ------------------------------------------------------------------ host, integers only */

/*
 * Online first-fit packing (section 2.2.1 (2): samples are concatenated into
 * sequences close to the maximum context length; the bin rule is this build's
 * reading).  Samples are taken in index order; each goes to the lowest-numbered
 * bin with at least lens[i] free tokens, a new bin being opened when none has.
 *   lens[N]           host in   sample lengths, 0 <= lens[i] <= budget
 *   bin_of_sample[N]  host out  bin index of each sample
 *   pos_in_bin[N]     host out  placement order of the sample inside its bin
 *   num_bins          host out
 * VA_ESIZE if a sample is longer than the budget (outputs untouched).
 */
int va_pack_first_fit(const int32_t* lens, int32_t N, int32_t budget,
                      int32_t* bin_of_sample, int32_t* pos_in_bin, int32_t* num_bins);

/*
 * Layout of one bin (section 2.2.1 (2): the samples of a bin are concatenated
 * end to end, and the variable-length interface of 2.2.1 (1) is told where each
 * one starts): exclusive prefix sums of its samples' lengths.
 *   lens[n], prefix[n] (prefix may be NULL)  host in, in placement order
 *   cu_seqlens[n+1]   host out, cu_seqlens[0] = 0
 *   prefix_lens[n]    host out (may be NULL when prefix is NULL); VA_EINVAL unless 0 <= P <= L
 * (one boundary per sample; the two boundaries of VA_MASK_THREE_BLOCK go through it one at a
 * time, or are handed to va_build_worklist directly)
 *   max_seqlen        host out
 */
int va_bin_layout(const int32_t* lens, const int32_t* prefix, int32_t n,
                  int32_t* cu_seqlens, int32_t* prefix_lens, int32_t* max_seqlen);

/*
 * (This library's own; the paper names no tiling.)
 * Tile shape the kernels of `pass` use for these head counts: *rows is the
 * number of token rows of a work item (query rows for VA_PASS_FWD and
 * VA_PASS_BWD_DQ, key rows for VA_PASS_BWD_DKDV) and *cols the number of token
 * rows of the tiles it loops over.
 */
int va_tile_shape(int32_t pass, int32_t head_dim, int32_t num_q_heads, int32_t num_kv_heads,
                  int32_t* rows, int32_t* cols);

/*
 * Work list of one pass over one packed stream, in records of 8 int32 words:
 *   record 0   {magic "VAW4", pass, rows, cols, head_dim, mask_mode, num_items, total_tokens}
 *   record 1   {num_workgroups, num_works, works_per_item, flags, first table record,
 *               first work-id record, total records, number of merge records}
 *   items      num_items records from record 2 on, heaviest first (ties by sample, then tile)
 *   table      two records per persistent workgroup: the item of its first work, then
 *              {id of that work, id of its second work, first schedule position,
 *              number of works, 0, 0, 0, 0}
 *   work ids   num_works words, 8 per record: item * works_per_item + head chunk,
 *              grouped by workgroup in the order the workgroup runs them
 *   merges     (dK/dV lists) one record per split key tile, see below
 * Only tiles holding at least one visible (query, key) pair are listed and no
 * tile spans two samples (the varlen rule of section 2.2.1 (1): compute on
 * valid tokens only).
 *   forward / dQ item: {q_row0, q_rows, seq_row0, P2 or -1, n_full, n_tiles, P or -1, L}
 *   dK/dV item:        {kv_row0, kv_rows | (slot + 1) << 8, seq_row0, qt_first, qt_count, P2 or -1, P or -1, L}
 * (n_tiles key tiles hold a key some row of the item sees, the first n_full of them
 * no hidden pair; P and P2 are the sample's block ends, -1 where the mask has none)
 * Under VA_MASK_SLIDING_WINDOW the P word holds the window W, n_full and n_tiles
 * are those of the causal mask, and the lower edge follows from W: of the tiles
 * of cols keys below n_tiles an item visits those from lo(first row) / cols on,
 * and its mask-free tiles are those from ceil(lo(last row) / cols) up to n_full;
 * qt_count of a dK/dV item ends with the last query tile holding a row that
 * still sees a key of the item; an item's weight in the order of the list and in
 * the schedule is the number of tiles it visits.
 * A work is one item for one head chunk: the query heads one workgroup stacks
 * (forward, dQ) or one KV head (dK/dV), so works_per_item depends on the head
 * counts the list was built for.  The forward and dQ kernels run num_workgroups
 * persistent workgroups; the table assigns the works to them longest-processing-
 * time first, with a work's cost taken as its inner-loop steps plus a fixed part.
 * Within that, works that read the same rows (the K and V rows of one sample
 * and KV head) go to workgroups of one XCD, at about the same position of their
 * queues, so that the XCD's L2 fetches the rows once.
 * The dK/dV kernel runs one work per workgroup and ignores the table.  Workgroup
 * b of its launch runs work b (item order), or, when flags has bit 0 set, the
 * work at position b of the id array: an order that puts the key tiles of one
 * (sample, KV head) next to each other on one XCD, chosen by the builder where
 * the list holds at least four works per workgroup slot and a replay of the
 * hardware's dispatch says it ends within 3 % of item order.
 * Split key tiles: where few heavy dK/dV works per workgroup slot would leave
 * most of the chip idle in the last round (257 equal works on 256 slots), the
 * builder cuts the query tiles of the work that ends last into pieces.  Each
 * piece is an item of its own (qt_first, qt_count: its part of the tile's query
 * tiles; slot >= 0: the partial-sum slot of the workspace its workgroups write
 * float32 dK and dV sums to; slot + 1 = 0 marks an item that writes dK and dV
 * itself), and a merge record {kv_row0, kv_rows, first slot, pieces, qt_first,
 * qt_count of the whole tile, 0, 0} tells the merge kernel to add the pieces, in
 * slot order, into dK and dV.  The pieces of a tile hold consecutive slots.
 * va_worklist_size gives the buffer size (an upper bound: it does not know the
 * mask); va_build_worklist fills a host buffer of at least that size.  The
 * caller copies the buffer to the device unchanged and hands both copies to the
 * device calls, which validate the host copy (records, bounds, that every item
 * lies inside one sample of cu_seqlens and carries the block ends of
 * prefix_lens, that the table partitions the works and repeats each
 * workgroup's first work faithfully, that the pieces of a split tile cover its
 * query tiles once) and return VA_EINVAL on a mismatch.  The device copy must
 * be a byte copy of the validated host copy: the kernels read it unchecked.
 */
int va_worklist_size(const int32_t* cu_seqlens, int32_t num_seqs, int32_t pass, int32_t head_dim,
                      int32_t num_q_heads, int32_t num_kv_heads, size_t* bytes);
int va_build_worklist(const int32_t* cu_seqlens, const int32_t* prefix_lens, int32_t num_seqs,
                      int32_t mask_mode, int32_t pass, int32_t head_dim,
                      int32_t num_q_heads, int32_t num_kv_heads,
                      void* host_out, size_t bytes, int32_t* num_items);

/*
 * The validation the device calls apply to the host copy of a work list, on its
 * own (this library's own; host only, nothing is launched): VA_OK when the list
 * is one the kernels of `pass` may follow for this stream (shape, cu_seqlens
 * and prefix_lens as in the device calls), else the error the device call
 * would return.  For callers that build or cache lists away from the call that
 * uses them, and for testing the builder.
 */
int va_check_worklist(const void* worklist_host, int32_t pass, const int32_t* cu_seqlens,
                      const int32_t* prefix_lens, const va_shape* shape);

/*
 * Per-head OCP E4M3 quantisation on the host (per-channel scaling of section
 * 2.2.3 applied along the head axis): descale[h] = amax_h / 448 (1 when the
 * head is all zero), code = round-to-nearest-even e4m3 of x / descale[h],
 * saturating at +-448.  x is bfloat16 bits, host, [T, H, D].
 */
int va_quantize_e4m3_per_head(const uint16_t* x_bf16, int32_t T, int32_t H, int32_t D,
                              uint8_t* codes, float* descale);

/* ------------------------------------------------------------------ device */

/*
 * Bytes of device scratch varlen_attn_bwd needs for these shapes (this library's
 * own): delta and LSE * log2(e), float32 [Hq, T] each, then the partial-sum
 * slots of split key tiles (see va_build_worklist; reserved whether a list
 * splits a tile or not, 16 MiB at most head counts).  0 for a null or
 * unsupported shape.
 */
size_t varlen_attn_bwd_workspace_bytes(const va_shape* shape);

/*
 * Forward (section 2.2.1 (1): attention on the valid tokens of the packed
 * stream of 2.2.1 (2), sample by sample; masks of 2.2.1 (1) and 2.2.2):
 * O = softmax(scale * Q K^T + mask) V per sample, and LSE.
 *   q, k, v        device in   bfloat16
 *   cu_seqlens     host  in    [num_seqs + 1] (validated here: monotone, [0] = 0, last = T)
 *   prefix_lens    host  in    [num_seqs] ([2 num_seqs] under VA_MASK_THREE_BLOCK), NULL allowed for
 *                              VA_MASK_CAUSAL (validated: 0 <= P <= L, and P <= P2 <= L);
 *                              the kernels take each sample's P from the work list built from it
 *   scale          positive and finite
 *   worklist       device in   copy of va_build_worklist(VA_PASS_FWD)
 *   worklist_host  host  in    the same bytes (header and bounds are validated here)
 *   out            device out  bfloat16 [T, Hq, D]
 *   lse            device out  float32 [Hq, T]
 */
int varlen_attn_fwd(const void* q, const void* k, const void* v,
                    const int32_t* cu_seqlens, const int32_t* prefix_lens,
                    const void* worklist, const void* worklist_host,
                    const va_shape* shape, float scale,
                    void* out, float* lse, void* stream);

/*
 * Backward of the same operation (the training step of section 2.2.1 needs the
 * gradients of what the forward computes; the paper prints no formula, the
 * schedule is this library's own): dQ, dK, dV from dO, recomputing the
 * probabilities from the saved LSE.  delta = rowsum(dO * O) per row; dK/dV per key tile; dQ per query tile.
 * At head_dim <= 128 the dQ kernel computes delta for its own rows (every row
 * belongs to exactly one of its works), runs first, and the dK/dV kernel reads
 * what it wrote: two kernels.  At head_dim 256 a separate pass over O and dO
 * comes first: three kernels.  No atomics; results do not depend on scheduling.
 *   out, lse            device in   what varlen_attn_fwd wrote
 *   dout                device in   bfloat16 [T, Hq, D]
 *   worklist_dkdv/_dq   device in   va_build_worklist(VA_PASS_BWD_DKDV / VA_PASS_BWD_DQ)
 *   *_host              host  in    the same bytes
 *   dq, dk, dv          device out  bfloat16
 *   workspace           device      at least varlen_attn_bwd_workspace_bytes(shape), 256-byte aligned
 */
int varlen_attn_bwd(const void* q, const void* k, const void* v, const void* out, const float* lse,
                    const void* dout, const int32_t* cu_seqlens, const int32_t* prefix_lens,
                    const void* worklist_dkdv, const void* worklist_dkdv_host,
                    const void* worklist_dq, const void* worklist_dq_host,
                    const va_shape* shape, float scale,
                    void* dq, void* dk, void* dv,
                    void* workspace, size_t workspace_bytes, void* stream);

/*
 * The same quantisation on the device (the on-device step the per-head
 * scaling of section 2.2.3 needs before the FP8 forward), bit-identical to
 * va_quantize_e4m3_per_head (non-finite inputs included: in both a NaN
 * becomes the NaN code 0x7F at its own place and stays out of the maximum, and
 * an infinity makes the descale of its head infinite):
 *   x        device in   bfloat16 [T, H, D], 16-byte aligned, D a multiple of 8
 *   codes    device out  uint8 [T, H, D], 8-byte aligned
 *   descale  device out  float32 [H]; holds the per-head maxima while the call runs
 * Four small kernels on `stream`; nothing is allocated, nothing waits.
 * VA_EINVAL for null pointers or bad sizes, VA_EALIGN, VA_EHIP.
 */
int va_quantize_e4m3_per_head_device(const void* x_bf16, int32_t T, int32_t H, int32_t D,
                                     void* codes, float* descale, void* stream);

/*
 * (This library's own, for harnesses that account for the backward kernel by kernel.)
 * Whether varlen_attn_bwd at this head_dim launches the separate delta pass
 * (1) or its dQ kernel computes delta (0); see varlen_attn_bwd.  Host only,
 * no error cases: any other head_dim answers 1.
 */
int va_bwd_has_delta_kernel(int32_t head_dim);

/*
 * The backward restricted to some of its kernels (this library's own; the
 * paper names no such call).  `stages` is a non-empty combination of
 *   VA_BWD_STAGE_DELTA  delta = rowsum(dO * O) (kept negated) and LSE * log2(e) into the workspace
 *   VA_BWD_STAGE_DKDV   dK and dV; reads both arrays from the workspace
 *   VA_BWD_STAGE_DQ     dQ; at head_dim <= 128 its kernel also writes both arrays
 *                       (VA_BWD_STAGE_DELTA is then implied and costs nothing extra)
 * in the order varlen_attn_bwd runs them; VA_BWD_STAGE_ALL is varlen_attn_bwd.
 * For callers that need one side only (frozen keys and values: dQ alone) and
 * for timing one kernel at a time with the caller's own events.  A call with
 * VA_BWD_STAGE_DKDV but without the stage that fills the workspace reads what
 * an earlier call with the same q, k, v, out, lse, dout and workspace left
 * there.  Outputs of stages not selected are not touched (their pointers must
 * still be valid device pointers).  Same arguments and errors as
 * varlen_attn_bwd; VA_EINVAL for an empty or unknown stage set.
 */
#define VA_BWD_STAGE_DELTA 1u
#define VA_BWD_STAGE_DKDV 2u
#define VA_BWD_STAGE_DQ 4u
#define VA_BWD_STAGE_ALL 7u
int varlen_attn_bwd_stages(const void* q, const void* k, const void* v, const void* out, const float* lse,
                           const void* dout, const int32_t* cu_seqlens, const int32_t* prefix_lens,
                           const void* worklist_dkdv, const void* worklist_dkdv_host,
                           const void* worklist_dq, const void* worklist_dq_host,
                           const va_shape* shape, float scale,
                           void* dq, void* dk, void* dv,
                           void* workspace, size_t workspace_bytes, void* stream, uint32_t stages);

/*
 * varlen_attn_bwd without a workspace argument, for callers that cannot
 * allocate device memory where they call it (code under HIP graph capture,
 * serving loops and harnesses that forbid hipMalloc): the scratch the backward
 * needs lives in a device array inside the library, VA_STATIC_WORKSPACE_BYTES
 * per GPU the library is used on, held until the process ends.  The call
 * allocates and frees nothing.  Shapes whose
 * varlen_attn_bwd_workspace_bytes exceeds that size are refused with
 * VA_ESIZE (use varlen_attn_bwd then).  All calls on one GPU share the one
 * array: calls that may overlap there (two streams, two threads) race; calls
 * on one stream are ordered like any other work.  Nothing in the array needs
 * a defined value on entry (every word a kernel reads was written earlier in
 * the same call).  The first call on a device looks the array's address up
 * (hipGetSymbolAddress); make that call outside a stream capture.
 * Otherwise arguments, results (bit for bit) and errors are those of
 * varlen_attn_bwd; VA_EHIP if the address cannot be obtained.
 */
#define VA_STATIC_WORKSPACE_BYTES ((size_t)32 << 20)
int varlen_attn_bwd_static(const void* q, const void* k, const void* v, const void* out, const float* lse,
                           const void* dout, const int32_t* cu_seqlens, const int32_t* prefix_lens,
                           const void* worklist_dkdv, const void* worklist_dkdv_host,
                           const void* worklist_dq, const void* worklist_dq_host,
                           const va_shape* shape, float scale,
                           void* dq, void* dk, void* dv, void* stream);

/*
 * FP8 forward: Q, K, V are OCP E4M3 bytes with one float32 descale per head
 * (device arrays q_descale[Hq], k_descale[Hkv], v_descale[Hkv]).  Scores are
 * (scale * q_descale[h] * k_descale[g]) * (Q8 . K8) in float32; the softmax and
 * LSE are float32; the probabilities are requantised to E4M3 (times 256) for
 * the second product; the row sum uses the unquantised probabilities.
 * Output bfloat16 O and float32 LSE as in varlen_attn_fwd.  head_dim 64, 128 or 256
 * (VA_EUNSUPPORTED otherwise).
 * (Scaling vocabulary of section 2.2.3; applying FP8 to the attention operands
 * is this library's extension: the paper quantises weights.)
 * Accuracy of the LSE: the matrix unit sums E4M3 products with about 17
 * significant bits, so the LSE carries a relative error of about 1.4e-5: within
 * 1e-3 absolute up to |LSE| of about 70, beyond that in proportion (the bfloat16
 * forward holds 1e-5 there).  Scores that large come from peaked softmaxes with
 * scale * |q| * |k| far above the 1 / sqrt(head_dim) the workloads use.
 */
int varlen_attn_fwd_fp8(const void* q8, const void* k8, const void* v8,
                        const float* q_descale, const float* k_descale, const float* v_descale,
                        const int32_t* cu_seqlens, const int32_t* prefix_lens,
                    const void* worklist, const void* worklist_host,
                        const va_shape* shape, float scale,
                        void* out, float* lse, void* stream);

/*
 * Block-wise scaling (the finest granularity section 2.2.3 names, applied to
 * the attention operands): one scale for every block of VA_FP8_BLOCK_TOKENS
 * consecutive tokens of ONE sample and one head (all head_dim values of those
 * tokens).  Blocks start at the sample's first token, the last one of a sample
 * may be short, and no block spans two samples.  descale = amax of the block /
 * 448 (1 when the block is all zero), code = round-to-nearest-even e4m3 of
 * x / descale, saturating at +-448.  The scales are returned one per token row,
 * descale_tok[t, h] = the descale of the block that holds token t, so that a
 * reader needs no block arithmetic; the rows of one block hold equal values.
 *   x            bfloat16 bits [T, H, D], T = cu_seqlens[num_seqs]
 *   cu_seqlens   host in  [num_seqs + 1], validated (starts at 0, monotone)
 *   codes        out      uint8 [T, H, D]
 *   descale_tok  out      float32 [T, H]
 * The host routine takes host buffers.  The device routine takes device
 * buffers (x 16-byte, codes 8-byte, descale_tok 4-byte aligned, D a multiple
 * of 8) and a second, device-resident copy of cu_seqlens with
 * the same contents, launches one kernel on `stream`, allocates nothing, does
 * not wait, and is bit-identical to the host routine (NaN and infinity treated
 * as in the per-head pair).  A
 * device copy that disagrees with the host copy gives wrong scales but no
 * access outside [0, T).
 * VA_EINVAL for null pointers, bad sizes or a bad cu_seqlens, VA_EALIGN, VA_EHIP.
 */
#define VA_FP8_BLOCK_TOKENS 128
int va_quantize_e4m3_blockwise(const uint16_t* x_bf16, const int32_t* cu_seqlens, int32_t num_seqs,
                               int32_t H, int32_t D, uint8_t* codes, float* descale_tok);
int va_quantize_e4m3_blockwise_device(const void* x_bf16, const int32_t* cu_seqlens,
                                      const int32_t* cu_seqlens_device, int32_t num_seqs,
                                      int32_t H, int32_t D, void* codes, float* descale_tok, void* stream);

/*
 * FP8 forward with block-wise scales: as varlen_attn_fwd_fp8, but the descale
 * arrays are per token row and head, in the layout va_quantize_e4m3_blockwise
 * writes: q_descale_tok[T, Hq], k_descale_tok[T, Hkv], v_descale_tok[T, Hkv],
 * device, float32, positive and finite.  A key tile of the kernel (64 keys
 * from a multiple of 64 inside the sample) lies inside one block, so the kernel
 * reads the K and V scale of a tile's first row; the arrays must therefore be
 * constant over each block, as the quantiser writes them.  The V scale enters
 * the exponent of the probabilities (p * v_descale is what is requantised to
 * E4M3), the row sum divides it out again: the V maxima of the blocks of one
 * sample and head should lie within a factor 2^64 of each other, or keys of the
 * smaller blocks can lose their weight in the row sum.
 * Same shapes, work list, outputs and errors as varlen_attn_fwd_fp8;
 * additionally VA_ESIZE when T * Hq * 4 bytes does not fit 31 bits.
 */
int varlen_attn_fwd_fp8_blockwise(const void* q8, const void* k8, const void* v8,
                                  const float* q_descale_tok, const float* k_descale_tok,
                                  const float* v_descale_tok,
                                  const int32_t* cu_seqlens, const int32_t* prefix_lens,
                                  const void* worklist, const void* worklist_host,
                                  const va_shape* shape, float scale,
                                  void* out, float* lse, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* VARLEN_ATTN_H */
