/* float64 CPU oracle of causal GQA attention over a paged KV cache, plain C + OpenMP.
 *
 * TEST INFRASTRUCTURE ONLY: this file is never linked into the product library and shares
 * no code with it.  It is the same definition as oracle/ref_numpy.py, written out with
 * scalar loops so that it can be timed on the host cores and used on larger samples:
 *
 *   for sequence i, query row t (pos = ctx_len_i + t), query head h, kappa = h / (Hq/Hkv):
 *       s_j = scale * <q[qsl_i+t, h, :], K_j>,  j = 0..pos      (causal, own key included)
 *       p_j = exp(s_j - max s) / sum exp(s_j - max s)
 *       out[qsl_i+t, h, :] = sum_j p_j V_j
 *
 * (fused softmax(QK^T)V operator: paper Section 3.3.1; paged KV pool: Section 2.1; decode
 * vs prefill rows: Section 2.3; GQA: Table 1.)  Inputs are bf16 bit patterns widened exactly
 * to double; every sum is a plain left-to-right double sum.
 *
 * Cache layout (include/ooco.h):
 *   K element (block b, kv head kh, dim d, slot s) at (((b*Hkv+kh)*(hd/8) + d/8)*BS + s)*8 + d%8
 *   V element                                       at  ((b*Hkv+kh)*hd + d)*BS + s
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static double widen(uint16_t bits)
{
    uint32_t u = ((uint32_t)bits) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/* Returns the number of threads used (>0), or <0 on bad arguments / allocation failure. */
int ooco_oracle_attn_mixed(const uint16_t *q, const uint16_t *k_cache, const uint16_t *v_cache,
                           const int32_t *block_tables, const int32_t *seq_lens,
                           const int32_t *query_start_loc, const int32_t *ctx_lens, double *out,
                           int num_seqs, int Hq, int Hkv, int hd, int BS, int max_blocks_per_seq,
                           double scale, int num_threads)
{
    if (Hq <= 0 || Hkv <= 0 || Hq % Hkv || hd % 8 || BS <= 0) return -1;
    const int g = Hq / Hkv;
    int max_len = 0;
    for (int i = 0; i < num_seqs; ++i) {
        int c = query_start_loc[i + 1] - query_start_loc[i];
        if (c < 0 || ctx_lens[i] + c != seq_lens[i]) return -2;
        if ((seq_lens[i] + BS - 1) / BS > max_blocks_per_seq) return -3;
        if (seq_lens[i] > max_len) max_len = seq_lens[i];
    }
    const int total_rows = num_seqs ? query_start_loc[num_seqs] : 0;
    /* row -> sequence map so the parallel loop can run over (row, head) pairs */
    int32_t *row_seq = (int32_t *)malloc(sizeof(int32_t) * (size_t)(total_rows > 0 ? total_rows : 1));
    if (!row_seq) return -4;
    for (int i = 0; i < num_seqs; ++i)
        for (int r = query_start_loc[i]; r < query_start_loc[i + 1]; ++r) row_seq[r] = i;

    int used = 1, failed = 0;
#ifdef _OPENMP
    if (num_threads > 0) omp_set_num_threads(num_threads);
#endif
#pragma omp parallel
    {
#ifdef _OPENMP
#pragma omp single
        used = omp_get_num_threads();
#endif
        double *s = (double *)malloc(sizeof(double) * (size_t)(max_len > 0 ? max_len : 1));
        double *qv = (double *)malloc(sizeof(double) * (size_t)hd);
        double *acc = (double *)malloc(sizeof(double) * (size_t)hd);
        if (!s || !qv || !acc) {
#pragma omp atomic write
            failed = 1;
        } else {
#pragma omp for schedule(dynamic, 1)
            for (long item = 0; item < (long)total_rows * Hq; ++item) {
                const int r = (int)(item / Hq), h = (int)(item % Hq);
                const int i = row_seq[r];
                const int t = r - query_start_loc[i];
                const int pos = ctx_lens[i] + t;
                const int kh = h / g;
                const int32_t *table = block_tables + (size_t)i * max_blocks_per_seq;
                for (int d = 0; d < hd; ++d) qv[d] = widen(q[((size_t)r * Hq + h) * hd + d]);
                double mx = -INFINITY;
                for (int j = 0; j <= pos; ++j) {
                    const size_t b = (size_t)table[j / BS];
                    const int sl = j % BS;
                    double dot = 0.0;
                    for (int d = 0; d < hd; ++d)
                        dot += qv[d] * widen(k_cache[(((b * Hkv + kh) * (hd / 8) + d / 8) * BS + sl) * 8 + d % 8]);
                    s[j] = scale * dot;
                    if (s[j] > mx) mx = s[j];
                }
                double den = 0.0;
                for (int j = 0; j <= pos; ++j) {
                    s[j] = exp(s[j] - mx);
                    den += s[j];
                }
                for (int d = 0; d < hd; ++d) acc[d] = 0.0;
                for (int j = 0; j <= pos; ++j) {
                    const size_t b = (size_t)table[j / BS];
                    const int sl = j % BS;
                    const double p = s[j] / den;
                    for (int d = 0; d < hd; ++d)
                        acc[d] += p * widen(v_cache[((b * Hkv + kh) * hd + d) * BS + sl]);
                }
                for (int d = 0; d < hd; ++d) out[((size_t)r * Hq + h) * hd + d] = acc[d];
            }
        }
        free(s);
        free(qv);
        free(acc);
    }
    free(row_seq);
    return failed ? -4 : used;
}

/* dst_pool[dst_ids[p]] <- src_pool[src_ids[p]], whole blocks of K and of V. */
void ooco_oracle_block_copy(const uint16_t *k_src, const uint16_t *v_src, uint16_t *k_dst, uint16_t *v_dst,
                            const int64_t *src_ids, const int64_t *dst_ids, int64_t num_pairs,
                            int Hkv, int hd, int BS)
{
    const size_t blk = (size_t)Hkv * hd * BS;
    for (int64_t p = 0; p < num_pairs; ++p) {
        memcpy(k_dst + (size_t)dst_ids[p] * blk, k_src + (size_t)src_ids[p] * blk, blk * sizeof(uint16_t));
        memcpy(v_dst + (size_t)dst_ids[p] * blk, v_src + (size_t)src_ids[p] * blk, blk * sizeof(uint16_t));
    }
}
