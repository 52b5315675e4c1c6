/*
 * fp64 CPU oracle for packed variable-length attention, forward and backward.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing in the product path may call this file:
 * it exists so the tests, the smoke check and the benchmark's CPU-baseline leg
 * have a slow, obviously correct answer to compare the GPU kernels with.  It
 * shares no code, header, table or helper with the HIP library.
 *
 * What it computes.  The paper (section 2.2.1, paragraphs (1) "Variable-Length
 * Flash-Attention" and (2) "Data Packing"; results section 3.2) packs several
 * samples end to end into one token stream and runs softmax attention on the
 * valid tokens only.  The method is exact: it reaches the same result as
 * running every sample alone, so the oracle is the plain textbook definition,
 * one sample at a time, one query row at a time, with no tiling, no running
 * softmax and no saved-statistics trick.  The paper prints no formula; the
 * readings taken (mask shapes, head grouping, natural-log LSE) are this build's
 * and are listed in the design notes.
 *
 * For sample s occupying rows [c, c+L) of the stream, query head h, KV head
 * g = h / (Hq/Hkv), local query row i:
 *     A(i)  = the keys j of the sample that row i may attend, by mask mode:
 *             causal: j <= i.  Prefix-LM with prefix length P: tokens [0, P) form one block, the rest a
 *             second one, and a row sees its own block and the block before it (a bidirectional prefix, a
 *             suffix that sees everything).  Mode 2: the same with a causal suffix (a suffix row sees the
 *             prefix and the suffix keys up to its own).  Mode 3: three blocks [0, P), [P, P2), [P2, L), each
 *             seeing itself and the blocks before it; prefix_lens then holds the pair (P, P2),
 *             0 <= P <= P2 <= L, for every sample.  Mode 4: sliding window of W = prefix_lens[s] >= 1
 *             keys: j <= i and i - j < W.
 *     s_ij  = scale * sum_d Q[c+i,h,d] K[c+j,g,d]        for j in A(i)
 *     m_i   = max_j s_ij,  Z_i = sum_j exp(s_ij - m_i)
 *     LSE[h,c+i] = m_i + ln Z_i
 *     p_ij  = exp(s_ij - m_i) / Z_i
 *     O[c+i,h,:] = sum_j p_ij V[c+j,g,:]
 * Backward for a given dO (LSE carries no gradient):
 *     delta_i = sum_d dO_id O_id,  dP_ij = sum_d dO_id V_jd
 *     dS_ij = p_ij (dP_ij - delta_i)
 *     dQ_i = scale sum_j dS_ij K_j
 *     dK_j = scale sum_{h in group} sum_i dS_ij Q_i
 *     dV_j =       sum_{h in group} sum_i p_ij dO_i
 *
 * Inputs are float32 arrays holding values that are already rounded to the
 * storage type of the GPU path (bf16, or dequantised e4m3); they are promoted
 * to double and every operation is done in double.  Outputs are double.
 * Layouts: Q, O, dO, dQ are [T, Hq, D]; K, V, dK, dV are [T, Hkv, D];
 * LSE is [Hq, T].  `sel` lists the sample indices to process (NULL = all);
 * rows of other samples are left untouched.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_MASK_CAUSAL 0
#define ORACLE_MASK_PREFIX_BIDIR_SUFFIX 1
#define ORACLE_MASK_PREFIX_CAUSAL_SUFFIX 2
#define ORACLE_MASK_THREE_BLOCK 3
#define ORACLE_MASK_SLIDING_WINDOW 4 /* causal, and at most the W most recent keys: j > i - W */

/*
 * The mask as a predicate on one (query row i, key j) pair of a sample, stated through the block each token
 * lies in: block 0 = [0, P), block 1 = [P, P2) (three-block mask only), last block = the rest.
 *   causal            j <= i
 *   sliding window    j <= i and i - j < W               (W = prefix_lens[s])
 *   prefix-LM         block(j) <= block(i)               (two blocks: prefix, suffix; each bidirectional)
 *   ... causal suffix block(j) < block(i), or both in the prefix, or both in the suffix and j <= i
 *   three blocks      block(j) <= block(i)
 */
typedef struct {
    int mode;
    int L;
    int P;  /* end of block 0; the window W under the sliding-window mask */
    int P2; /* end of block 1 (three-block mask), else unused */
} sample_mask;

static sample_mask mask_of_sample(const int32_t *prefix_lens, int mode, int s, int L)
{
    sample_mask m = {mode, L, 0, 0};
    if (mode == ORACLE_MASK_THREE_BLOCK) {
        m.P = prefix_lens[2 * s];
        m.P2 = prefix_lens[2 * s + 1];
    } else if (mode != ORACLE_MASK_CAUSAL) {
        m.P = prefix_lens[s];
        m.P2 = m.P; /* two blocks: block 1 is empty */
    }
    return m;
}

static int block_of(const sample_mask *m, int x) { return x < m->P ? 0 : x < m->P2 ? 1 : 2; }

static int allowed(const sample_mask *m, int i, int j)
{
    switch (m->mode) {
    case ORACLE_MASK_CAUSAL: return j <= i;
    case ORACLE_MASK_SLIDING_WINDOW: return j <= i && i - j < m->P;
    case ORACLE_MASK_PREFIX_BIDIR_SUFFIX:
    case ORACLE_MASK_THREE_BLOCK: return block_of(m, j) <= block_of(m, i);
    case ORACLE_MASK_PREFIX_CAUSAL_SUFFIX: {
        const int bi = block_of(m, i), bj = block_of(m, j);
        if (bj != bi) return bj < bi;
        return bi == 0 ? 1 : j <= i;
    }
    default: return 0;
    }
}

/* a[j] = 1 where query row i may attend key j, for all keys of the sample */
static void row_mask(const sample_mask *m, int i, unsigned char *a)
{
    for (int j = 0; j < m->L; ++j) a[j] = (unsigned char)allowed(m, i, j);
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* softmax probabilities of one query row over the keys j < L with a[j] set; returns LSE. p[j] filled where a[j]. */
static double row_softmax(const float *q_row, const float *k_base, size_t k_stride,
                          const unsigned char *a, int L, int D, double scale, double *p)
{
    double m = -INFINITY;
    for (int j = 0; j < L; ++j) {
        if (!a[j]) continue;
        const float *k_row = k_base + (size_t)j * k_stride;
        double s = 0.0;
        for (int d = 0; d < D; ++d) s += (double)q_row[d] * (double)k_row[d];
        s *= scale;
        p[j] = s;
        if (s > m) m = s;
    }
    double Z = 0.0;
    for (int j = 0; j < L; ++j) {
        if (!a[j]) continue;
        p[j] = exp(p[j] - m);
        Z += p[j];
    }
    for (int j = 0; j < L; ++j)
        if (a[j]) p[j] /= Z;
    return m + log(Z);
}

int oracle_attn_fwd(const float *q, const float *k, const float *v,
                    const int32_t *cu_seqlens, const int32_t *prefix_lens, int mask_mode,
                    int num_seqs, int Hq, int Hkv, int D, double scale,
                    const int32_t *sel, int nsel,
                    double *out, double *lse, int nthreads)
{
    if (Hkv <= 0 || Hq % Hkv != 0 || D <= 0) return -1;
    if (mask_mode != ORACLE_MASK_CAUSAL && prefix_lens == NULL) return -1;
    const int G = Hq / Hkv;
    const int T = cu_seqlens[num_seqs];
    const int nwork = (sel ? nsel : num_seqs) * Hq;
    int maxL = 0;
    for (int s = 0; s < num_seqs; ++s) {
        int L = cu_seqlens[s + 1] - cu_seqlens[s];
        if (L < 0) return -2;
        if (L > maxL) maxL = L;
    }
#ifdef _OPENMP
    if (nthreads > 0) omp_set_num_threads(nthreads);
#endif
    (void)nthreads;
#pragma omp parallel
    {
        double *p = (double *)malloc(sizeof(double) * (size_t)(maxL > 0 ? maxL : 1));
        unsigned char *a = (unsigned char *)malloc((size_t)(maxL > 0 ? maxL : 1));
#pragma omp for schedule(dynamic, 1)
        for (int w = 0; w < nwork; ++w) {
            const int s = sel ? sel[w / Hq] : w / Hq;
            const int h = w % Hq;
            const int g = h / G;
            const int c = cu_seqlens[s];
            const int L = cu_seqlens[s + 1] - c;
            const sample_mask mask = mask_of_sample(prefix_lens, mask_mode, s, L);
            for (int i = 0; i < L; ++i) {
                row_mask(&mask, i, a);
                const float *q_row = q + ((size_t)(c + i) * Hq + h) * D;
                const float *k_base = k + ((size_t)c * Hkv + g) * D;
                const float *v_base = v + ((size_t)c * Hkv + g) * D;
                const size_t kv_stride = (size_t)Hkv * D;
                double l = row_softmax(q_row, k_base, kv_stride, a, L, D, scale, p);
                lse[(size_t)h * T + (c + i)] = l;
                double *o_row = out + ((size_t)(c + i) * Hq + h) * D;
                for (int d = 0; d < D; ++d) o_row[d] = 0.0;
                for (int j = 0; j < L; ++j) {
                    if (!a[j]) continue;
                    const float *v_row = v_base + (size_t)j * kv_stride;
                    for (int d = 0; d < D; ++d) o_row[d] += p[j] * (double)v_row[d];
                }
            }
        }
        free(p);
        free(a);
    }
    return 0;
}

int oracle_attn_bwd(const float *q, const float *k, const float *v, const float *dout,
                    const int32_t *cu_seqlens, const int32_t *prefix_lens, int mask_mode,
                    int num_seqs, int Hq, int Hkv, int D, double scale,
                    const int32_t *sel, int nsel,
                    double *dq, double *dk, double *dv, int nthreads)
{
    if (Hkv <= 0 || Hq % Hkv != 0 || D <= 0) return -1;
    if (mask_mode != ORACLE_MASK_CAUSAL && prefix_lens == NULL) return -1;
    const int G = Hq / Hkv;
    const int nwork = (sel ? nsel : num_seqs) * Hkv;
    int maxL = 0;
    for (int s = 0; s < num_seqs; ++s) {
        int L = cu_seqlens[s + 1] - cu_seqlens[s];
        if (L < 0) return -2;
        if (L > maxL) maxL = L;
    }
#ifdef _OPENMP
    if (nthreads > 0) omp_set_num_threads(nthreads);
#endif
    (void)nthreads;
#pragma omp parallel
    {
        double *p = (double *)malloc(sizeof(double) * (size_t)(maxL > 0 ? maxL : 1));
        double *o = (double *)malloc(sizeof(double) * (size_t)D);
        unsigned char *a = (unsigned char *)malloc((size_t)(maxL > 0 ? maxL : 1));
#pragma omp for schedule(dynamic, 1)
        for (int w = 0; w < nwork; ++w) {
            /* one (sample, KV head) owns its dK, dV rows: no two threads share them */
            const int s = sel ? sel[w / Hkv] : w / Hkv;
            const int g = w % Hkv;
            const int c = cu_seqlens[s];
            const int L = cu_seqlens[s + 1] - c;
            const sample_mask mask = mask_of_sample(prefix_lens, mask_mode, s, L);
            const size_t kv_stride = (size_t)Hkv * D;
            const float *k_base = k + ((size_t)c * Hkv + g) * D;
            const float *v_base = v + ((size_t)c * Hkv + g) * D;
            double *dk_base = dk + ((size_t)c * Hkv + g) * D;
            double *dv_base = dv + ((size_t)c * Hkv + g) * D;
            for (int j = 0; j < L; ++j)
                for (int d = 0; d < D; ++d) {
                    dk_base[(size_t)j * kv_stride + d] = 0.0;
                    dv_base[(size_t)j * kv_stride + d] = 0.0;
                }
            for (int h = g * G; h < (g + 1) * G; ++h) {
                for (int i = 0; i < L; ++i) {
                    row_mask(&mask, i, a);
                    const float *q_row = q + ((size_t)(c + i) * Hq + h) * D;
                    const float *do_row = dout + ((size_t)(c + i) * Hq + h) * D;
                    double *dq_row = dq + ((size_t)(c + i) * Hq + h) * D;
                    row_softmax(q_row, k_base, kv_stride, a, L, D, scale, p);
                    /* this row's own fp64 output, then delta */
                    for (int d = 0; d < D; ++d) o[d] = 0.0;
                    for (int j = 0; j < L; ++j) {
                        if (!a[j]) continue;
                        const float *v_row = v_base + (size_t)j * kv_stride;
                        for (int d = 0; d < D; ++d) o[d] += p[j] * (double)v_row[d];
                    }
                    double delta = 0.0;
                    for (int d = 0; d < D; ++d) delta += (double)do_row[d] * o[d];
                    for (int d = 0; d < D; ++d) dq_row[d] = 0.0;
                    for (int j = 0; j < L; ++j) {
                        if (!a[j]) continue;
                        const float *k_row = k_base + (size_t)j * kv_stride;
                        const float *v_row = v_base + (size_t)j * kv_stride;
                        double dP = 0.0;
                        for (int d = 0; d < D; ++d) dP += (double)do_row[d] * (double)v_row[d];
                        const double dS = p[j] * (dP - delta);
                        double *dk_row = dk_base + (size_t)j * kv_stride;
                        double *dv_row = dv_base + (size_t)j * kv_stride;
                        for (int d = 0; d < D; ++d) {
                            dq_row[d] += scale * dS * (double)k_row[d];
                            dk_row[d] += scale * dS * (double)q_row[d];
                            dv_row[d] += p[j] * (double)do_row[d];
                        }
                    }
                }
            }
        }
        free(p);
        free(o);
        free(a);
    }
    return 0;
}

/*
 * Probabilities and score gradients of one (sample, head), written out densely
 * as [L, L] row-major (zero outside the mask).  Used only by the invariant
 * tests (rows of p sum to one, rows of dS sum to zero).
 */
int oracle_attn_probs(const float *q, const float *k, const float *v, const float *dout,
                      const int32_t *cu_seqlens, const int32_t *prefix_lens, int mask_mode,
                      int Hq, int Hkv, int D, double scale, int s, int h,
                      double *p_out, double *ds_out)
{
    const int G = Hq / Hkv;
    const int g = h / G;
    const int c = cu_seqlens[s];
    const int L = cu_seqlens[s + 1] - c;
    const sample_mask mask = mask_of_sample(prefix_lens, mask_mode, s, L);
    unsigned char *a = (unsigned char *)malloc((size_t)(L > 0 ? L : 1));
    const size_t kv_stride = (size_t)Hkv * D;
    const float *k_base = k + ((size_t)c * Hkv + g) * D;
    const float *v_base = v + ((size_t)c * Hkv + g) * D;
    double *p = (double *)malloc(sizeof(double) * (size_t)(L > 0 ? L : 1));
    double *o = (double *)malloc(sizeof(double) * (size_t)D);
    for (int i = 0; i < L; ++i) {
        row_mask(&mask, i, a);
        const float *q_row = q + ((size_t)(c + i) * Hq + h) * D;
        row_softmax(q_row, k_base, kv_stride, a, L, D, scale, p);
        for (int j = 0; j < L; ++j) p_out[(size_t)i * L + j] = a[j] ? p[j] : 0.0;
        if (ds_out) {
            const float *do_row = dout + ((size_t)(c + i) * Hq + h) * D;
            for (int d = 0; d < D; ++d) o[d] = 0.0;
            for (int j = 0; j < L; ++j)
                if (a[j])
                    for (int d = 0; d < D; ++d) o[d] += p[j] * (double)v_base[(size_t)j * kv_stride + d];
            double delta = 0.0;
            for (int d = 0; d < D; ++d) delta += (double)do_row[d] * o[d];
            for (int j = 0; j < L; ++j) {
                double dS = 0.0;
                if (a[j]) {
                    double dP = 0.0;
                    for (int d = 0; d < D; ++d) dP += (double)do_row[d] * (double)v_base[(size_t)j * kv_stride + d];
                    dS = p[j] * (dP - delta);
                }
                ds_out[(size_t)i * L + j] = dS;
            }
        }
    }
    free(p);
    free(o);
    free(a);
    return 0;
}
