/*
 * attn_oracle.c -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, fp64 CPU evaluation of scaled-dot-product attention, used only
 * by the tests, the smoke check and the benchmark's cpu_baseline leg.  It shares
 * no code, header, table or helper with the HIP library and must never be called
 * from the product path.
 *
 * What it computes.  The paper studies the fused ("flash") attention kernel of
 * LLM inference at Llama3-8B shapes with variable-length batches and a causal
 * mask (section "Method and Investigated Kernels"; Fig. 2 caption), and names the
 * 29-line PyTorch-native formulation as the plain baseline (Table I; Introduction).
 * Flash attention is exact attention, so the oracle is that plain definition
 * written out: for every sequence s, query head h and new-token index i,
 *
 *     kvh   = h / (Hq / Hkv)                     grouped-query head mapping
 *     off   = seq_lens[s] - n_q(s)               cached-prefix length
 *     limit = causal ? off + i + 1 : seq_lens[s] keys visible to query i
 *     x_j   = scale * sum_d q[i,h,d] * k[j,kvh,d]            j in [0, limit)
 *     m     = max_j x_j;  p_j = exp(x_j - m);  l = sum_j p_j
 *     out[i,h,:] = (sum_j p_j * v[j,kvh,:]) / l
 *
 * all in fp64, two-pass softmax, no tiling, no online rescaling.  Key j of
 * sequence s lives at row kv_start_loc[s] + j of a packed [total_kv, Hkv, D]
 * array (contiguous mode), or at slot j % block_size of physical block
 * block_table[s][j / block_size] of a [num_blocks, block_size, Hkv, D] pool
 * (paged mode; the paper only cites PagedAttention, the layout is this build's
 * reading).  Inputs are the already-rounded fp32 or bf16 values, widened exactly.
 *
 * Pins (tests/test_oracle_pins.py): a hand-computed 2x2 case, uniform-softmax and
 * one-hot closed forms, a dense-mask brute force, torch's fp64 softmax(QK^T)V,
 * and the structural equivalences paged==contiguous, GQA==repeated MHA,
 * chunked==slice of full prefill, decode==last prefill row.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1 };

typedef struct {
    int dtype;
    int num_seqs, num_q_heads, num_kv_heads, head_dim;
    const void *q;
    int64_t q_stride_tok, q_stride_head;
    const void *k, *v;
    int64_t kv_stride_block, kv_stride_tok, kv_stride_head;
    const int32_t *block_table; /* NULL -> contiguous */
    int block_table_stride, block_size;
    const int32_t *query_start_loc; /* [num_seqs+1] */
    const int32_t *kv_start_loc;    /* [num_seqs+1], contiguous only */
    const int32_t *seq_lens;        /* [num_seqs] */
    float scale;
    int causal;
} oracle_problem;

/* Exact widening of one stored element to double. */
static double load_elem(const void *base, int64_t idx, int dtype)
{
    if (dtype == ORACLE_F32)
        return (double)((const float *)base)[idx];
    uint32_t bits = (uint32_t)((const uint16_t *)base)[idx] << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

/* Element offset of key/value row j of sequence s, head kvh, channel 0. */
static int64_t kv_row_offset(const oracle_problem *p, int s, int j, int kvh)
{
    if (p->block_table == NULL)
        return ((int64_t)p->kv_start_loc[s] + j) * p->kv_stride_tok + (int64_t)kvh * p->kv_stride_head;
    int logical = j / p->block_size;
    int slot = j % p->block_size;
    int64_t phys = p->block_table[(int64_t)s * p->block_table_stride + logical];
    return phys * p->kv_stride_block + (int64_t)slot * p->kv_stride_tok + (int64_t)kvh * p->kv_stride_head;
}

/* One output row: sequence s, new-token index i, query head h -> out[0..D). */
static int attend_row(const oracle_problem *p, int s, int i, int h, double *out)
{
    const int D = p->head_dim;
    const int group = p->num_q_heads / p->num_kv_heads;
    const int kvh = h / group;
    const int n_q = p->query_start_loc[s + 1] - p->query_start_loc[s];
    const int n_kv = p->seq_lens[s];
    const int off = n_kv - n_q;
    int limit = p->causal ? off + i + 1 : n_kv;
    if (limit > n_kv)
        limit = n_kv;
    for (int d = 0; d < D; ++d)
        out[d] = 0.0;
    if (limit <= 0)
        return 0; /* no visible key: defined as zeros */

    double *x = (double *)malloc((size_t)limit * sizeof(double));
    double *qrow = (double *)malloc((size_t)D * sizeof(double));
    if (!x || !qrow) {
        free(x);
        free(qrow);
        return -1;
    }
    const int64_t qoff = ((int64_t)p->query_start_loc[s] + i) * p->q_stride_tok + (int64_t)h * p->q_stride_head;
    for (int d = 0; d < D; ++d)
        qrow[d] = load_elem(p->q, qoff + d, p->dtype);

    const double scale = (double)p->scale;
    double m = -INFINITY;
    for (int j = 0; j < limit; ++j) {
        const int64_t ko = kv_row_offset(p, s, j, kvh);
        double dot = 0.0;
        for (int d = 0; d < D; ++d)
            dot += qrow[d] * load_elem(p->k, ko + d, p->dtype);
        x[j] = scale * dot;
        if (x[j] > m)
            m = x[j];
    }
    double l = 0.0;
    for (int j = 0; j < limit; ++j) {
        x[j] = exp(x[j] - m);
        l += x[j];
    }
    for (int j = 0; j < limit; ++j) {
        const int64_t vo = kv_row_offset(p, s, j, kvh);
        const double pj = x[j];
        for (int d = 0; d < D; ++d)
            out[d] += pj * load_elem(p->v, vo + d, p->dtype);
    }
    for (int d = 0; d < D; ++d)
        out[d] /= l;
    free(x);
    free(qrow);
    return 0;
}

/*
 * Full output: out is fp64 [total_q, Hq, D], densely packed.
 * Returns 0, or -1 on allocation failure.
 */
int oracle_attention(const oracle_problem *p, double *out)
{
    int rc = 0;
    const int Hq = p->num_q_heads, D = p->head_dim;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int s = 0; s < p->num_seqs; ++s) {
        for (int h = 0; h < Hq; ++h) {
            const int q0 = p->query_start_loc[s];
            const int n_q = p->query_start_loc[s + 1] - q0;
            for (int i = 0; i < n_q; ++i) {
                double *o = out + (((int64_t)q0 + i) * Hq + h) * D;
                if (attend_row(p, s, i, h, o) != 0) {
#pragma omp atomic write
                    rc = -1;
                }
            }
        }
    }
    return rc;
}

/*
 * Sampled output: row r is (sel_seq[r], sel_tok[r] = new-token index inside the
 * sequence, sel_head[r]) -> out[r*D .. r*D+D).  Used at sizes where the full
 * result would take minutes.
 */
int oracle_attention_rows(const oracle_problem *p, int n_sel, const int32_t *sel_seq, const int32_t *sel_tok,
                          const int32_t *sel_head, double *out)
{
    int rc = 0;
    const int D = p->head_dim;
#pragma omp parallel for schedule(dynamic, 1)
    for (int r = 0; r < n_sel; ++r) {
        if (attend_row(p, sel_seq[r], sel_tok[r], sel_head[r], out + (int64_t)r * D) != 0) {
#pragma omp atomic write
            rc = -1;
        }
    }
    return rc;
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
