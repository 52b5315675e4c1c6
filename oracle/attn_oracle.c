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
 *     vis(i) = i + 1                      causal
 *            = P  if i < P, else L        prefix-LM with prefix length P
 *            = i + 1 if i >= P (mode 2)   prefix-LM, causal suffix
 *            = P if i < P, P2 if i < P2, else L   (mode 3) three blocks, each seeing
 *              itself and the blocks before it; prefix_lens then holds the pair
 *              (P, P2), 0 <= P <= P2 <= L, for every sample
 *     (mode 4) sliding window of W = prefix_lens[s] >= 1 keys: vis(i) = i + 1 and the
 *              keys start at lo(i) = max(0, i + 1 - W) instead of 0 (lo = 0 in every other mode)
 *     s_ij  = scale * sum_d Q[c+i,h,d] K[c+j,g,d]        for lo(i) <= j < vis(i)
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

/* number of keys query row i of a sample (length L, block ends P and P2) may attend to */
static int visible(int i, int L, int P, int P2, int mode)
{
    if (mode == ORACLE_MASK_CAUSAL || mode == ORACLE_MASK_SLIDING_WINDOW) return i + 1;
    if (i < P) return P;
    if (mode == ORACLE_MASK_PREFIX_BIDIR_SUFFIX) return L;
    if (mode == ORACLE_MASK_THREE_BLOCK) return i < P2 ? P2 : L;
    return i + 1;
}

/* first key query row i may attend to: 0, except under the sliding window of W keys (W travels in P) */
static int first_visible(int i, int P, int mode)
{
    if (mode == ORACLE_MASK_SLIDING_WINDOW && i + 1 - P > 0) return i + 1 - P;
    return 0;
}

/* block ends of sample s: prefix_lens holds one entry per sample, or the pair (P, P2) in mode 3 */
static void block_ends(const int32_t *prefix_lens, int mode, int s, int *P, int *P2)
{
    *P = 0;
    *P2 = 0;
    if (mode == ORACLE_MASK_THREE_BLOCK) {
        *P = prefix_lens[2 * s];
        *P2 = prefix_lens[2 * s + 1];
    } else if (mode != ORACLE_MASK_CAUSAL) {
        *P = prefix_lens[s];
    }
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* softmax probabilities of one query row over the keys lo .. nvis - 1; returns LSE. p[lo..nvis) filled. */
static double row_softmax(const float *q_row, const float *k_base, size_t k_stride,
                          int lo, int nvis, int D, double scale, double *p)
{
    double m = -INFINITY;
    for (int j = lo; j < nvis; ++j) {
        const float *k_row = k_base + (size_t)j * k_stride;
        double s = 0.0;
        for (int d = 0; d < D; ++d) s += (double)q_row[d] * (double)k_row[d];
        s *= scale;
        p[j] = s;
        if (s > m) m = s;
    }
    double Z = 0.0;
    for (int j = lo; j < nvis; ++j) {
        p[j] = exp(p[j] - m);
        Z += p[j];
    }
    for (int j = lo; j < nvis; ++j) p[j] /= Z;
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
#pragma omp for schedule(dynamic, 1)
        for (int w = 0; w < nwork; ++w) {
            const int s = sel ? sel[w / Hq] : w / Hq;
            const int h = w % Hq;
            const int g = h / G;
            const int c = cu_seqlens[s];
            const int L = cu_seqlens[s + 1] - c;
            int P, P2;
            block_ends(prefix_lens, mask_mode, s, &P, &P2);
            for (int i = 0; i < L; ++i) {
                const int nvis = visible(i, L, P, P2, mask_mode);
                const int lo = first_visible(i, P, mask_mode);
                const float *q_row = q + ((size_t)(c + i) * Hq + h) * D;
                const float *k_base = k + ((size_t)c * Hkv + g) * D;
                const float *v_base = v + ((size_t)c * Hkv + g) * D;
                const size_t kv_stride = (size_t)Hkv * D;
                double l = row_softmax(q_row, k_base, kv_stride, lo, nvis, D, scale, p);
                lse[(size_t)h * T + (c + i)] = l;
                double *o_row = out + ((size_t)(c + i) * Hq + h) * D;
                for (int d = 0; d < D; ++d) o_row[d] = 0.0;
                for (int j = lo; j < nvis; ++j) {
                    const float *v_row = v_base + (size_t)j * kv_stride;
                    for (int d = 0; d < D; ++d) o_row[d] += p[j] * (double)v_row[d];
                }
            }
        }
        free(p);
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
#pragma omp for schedule(dynamic, 1)
        for (int w = 0; w < nwork; ++w) {
            /* one (sample, KV head) owns its dK, dV rows: no two threads share them */
            const int s = sel ? sel[w / Hkv] : w / Hkv;
            const int g = w % Hkv;
            const int c = cu_seqlens[s];
            const int L = cu_seqlens[s + 1] - c;
            int P, P2;
            block_ends(prefix_lens, mask_mode, s, &P, &P2);
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
                    const int nvis = visible(i, L, P, P2, mask_mode);
                    const int lo = first_visible(i, P, mask_mode);
                    const float *q_row = q + ((size_t)(c + i) * Hq + h) * D;
                    const float *do_row = dout + ((size_t)(c + i) * Hq + h) * D;
                    double *dq_row = dq + ((size_t)(c + i) * Hq + h) * D;
                    row_softmax(q_row, k_base, kv_stride, lo, nvis, D, scale, p);
                    /* this row's own fp64 output, then delta */
                    for (int d = 0; d < D; ++d) o[d] = 0.0;
                    for (int j = lo; j < nvis; ++j) {
                        const float *v_row = v_base + (size_t)j * kv_stride;
                        for (int d = 0; d < D; ++d) o[d] += p[j] * (double)v_row[d];
                    }
                    double delta = 0.0;
                    for (int d = 0; d < D; ++d) delta += (double)do_row[d] * o[d];
                    for (int d = 0; d < D; ++d) dq_row[d] = 0.0;
                    for (int j = lo; j < nvis; ++j) {
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
    int P, P2;
    block_ends(prefix_lens, mask_mode, s, &P, &P2);
    const size_t kv_stride = (size_t)Hkv * D;
    const float *k_base = k + ((size_t)c * Hkv + g) * D;
    const float *v_base = v + ((size_t)c * Hkv + g) * D;
    double *p = (double *)malloc(sizeof(double) * (size_t)(L > 0 ? L : 1));
    double *o = (double *)malloc(sizeof(double) * (size_t)D);
    for (int i = 0; i < L; ++i) {
        const int nvis = visible(i, L, P, P2, mask_mode);
        const int lo = first_visible(i, P, mask_mode);
        const float *q_row = q + ((size_t)(c + i) * Hq + h) * D;
        row_softmax(q_row, k_base, kv_stride, lo, nvis, D, scale, p);
        for (int j = 0; j < L; ++j) p_out[(size_t)i * L + j] = j >= lo && j < nvis ? p[j] : 0.0;
        if (ds_out) {
            const float *do_row = dout + ((size_t)(c + i) * Hq + h) * D;
            for (int d = 0; d < D; ++d) o[d] = 0.0;
            for (int j = lo; j < nvis; ++j)
                for (int d = 0; d < D; ++d) o[d] += p[j] * (double)v_base[(size_t)j * kv_stride + d];
            double delta = 0.0;
            for (int d = 0; d < D; ++d) delta += (double)do_row[d] * o[d];
            for (int j = 0; j < L; ++j) {
                double dS = 0.0;
                if (j >= lo && j < nvis) {
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
    return 0;
}
