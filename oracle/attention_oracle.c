/*
 * TEST INFRASTRUCTURE — the correctness oracle, not part of the product.
 *
 * Plain, slow, fp64 causal attention over the concatenated [system ; context]
 * key/value sequence, exactly the definition the paper starts from (Sec. 3.3,
 * Eq. 4):
 *
 *     o_t = sum_{j=1..l} exp(q_t . k_j) / sigma_t^{1->l} * v_j ,
 *     sigma_t^{b->e} = sum_{j=b..e} exp(q_t . k_j),
 *
 * with the log-sum-exp beta = log(sigma) of App. A (Eq. 12) returned beside it.
 * The softmax scale, which the paper folds into q, is an explicit factor on
 * every logit here.  Nothing in this file uses the split / relay form
 * (Eq. 5-7, 11): the relay result must *equal* this one, so this file is the
 * thing it is compared against.
 *
 * There is no tiling, no fusion and no reordering: one row at a time, logits
 * for every visible position, max-shifted exponentials, one weighted sum.
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may call
 * into this file; it shares no code with the HIP library.
 *
 * Layouts (row-major, innermost index last):
 *   q            [n_tokens][Hq][d]                    float32
 *   k_sys,v_sys  [s][Hkv][d]                          float32
 *   k_cache,v_cache [num_blocks][Hkv][block_size][d]  float32
 *   block_tables [n_requests][max_blocks_per_seq]     int32
 * Inputs hold values that are exactly representable in bfloat16 (the caller
 * rounds once); every product and sum below is done in double.
 *
 * A "row" is one (token, query head) pair.  Token t belongs to request
 * token_request[t] and sees all s system positions (they precede every request
 * token, Sec. 3.3) followed by the first token_visible[t] positions of that
 * request's own context, gathered through its block table.  Decoding has one
 * token per request that sees the whole context (Alg. 1: the new key/value is
 * appended before attending); a prompt-phase token j of m new ones sees
 * c - m + j + 1 context positions (causal mask, new tokens last).
 * Query head h reads key/value head h / (Hq / Hkv).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum {
    ORACLE_OK = 0,
    ORACLE_BAD_ARGUMENT = -1,
    ORACLE_BAD_BLOCK_INDEX = -2,
    ORACLE_OUT_OF_MEMORY = -3
};

static double dot_fp64(const float *a, const float *b, int d)
{
    double acc = 0.0;
    for (int e = 0; e < d; ++e)
        acc += (double)a[e] * (double)b[e];
    return acc;
}

/* One (token, head) row of Eq. 4 over [system ; first `visible` context tokens]. */
static int attend_one_row(int Hkv, int d, int s, double scale,
                          const float *q_row, int kv_head, int visible,
                          const float *k_sys, const float *v_sys,
                          const float *k_cache, const float *v_cache,
                          int num_blocks, int block_size,
                          const int32_t *block_table_row, int max_blocks_per_seq,
                          double *out_row, double *lse_row)
{
    const int n = s + visible;
    for (int e = 0; e < d; ++e)
        out_row[e] = 0.0;
    if (n == 0) {              /* nothing to attend to: defined as zero output */
        *lse_row = -INFINITY;
        return ORACLE_OK;
    }
    if ((visible + block_size - 1) / block_size > max_blocks_per_seq)
        return ORACLE_BAD_ARGUMENT;

    double *z = (double *)malloc(sizeof(double) * (size_t)n);
    const float **vptr = (const float **)malloc(sizeof(const float *) * (size_t)n);
    if (!z || !vptr) {
        free(z);
        free(vptr);
        return ORACLE_OUT_OF_MEMORY;
    }

    /* logits z_j = scale * q . k_j for positions 1..l in sequence order */
    for (int j = 0; j < s; ++j) {
        const size_t off = ((size_t)j * Hkv + kv_head) * d;
        z[j] = scale * dot_fp64(q_row, k_sys + off, d);
        vptr[j] = v_sys + off;
    }
    for (int j = 0; j < visible; ++j) {
        const int32_t blk = block_table_row[j / block_size];
        if (blk < 0 || blk >= num_blocks) {
            free(z);
            free(vptr);
            return ORACLE_BAD_BLOCK_INDEX;
        }
        const size_t off =
            (((size_t)blk * Hkv + kv_head) * block_size + (size_t)(j % block_size)) * d;
        z[s + j] = scale * dot_fp64(q_row, k_cache + off, d);
        vptr[s + j] = v_cache + off;
    }

    double zmax = z[0];
    for (int j = 1; j < n; ++j)
        if (z[j] > zmax)
            zmax = z[j];

    double sigma = 0.0;                     /* sigma^{1->l} * exp(-zmax) */
    for (int j = 0; j < n; ++j) {
        const double w = exp(z[j] - zmax);
        sigma += w;
        const float *v = vptr[j];
        for (int e = 0; e < d; ++e)
            out_row[e] += w * (double)v[e];
    }
    for (int e = 0; e < d; ++e)
        out_row[e] /= sigma;
    *lse_row = zmax + log(sigma);           /* beta^{1->l}, natural log */

    free(z);
    free(vptr);
    return ORACLE_OK;
}

/*
 * Computes n_rows rows.  Row r is (token row_token[r], query head row_head[r]);
 * out is [n_rows][d] and lse is [n_rows], both double.  Returns ORACLE_OK or a
 * negative error; *threads_used (nullable) receives the thread count that ran.
 */
int oracle_attention_rows(int n_tokens, int n_requests, int Hq, int Hkv, int d, int s,
                          double scale,
                          const float *q,
                          const int32_t *token_request, const int32_t *token_visible,
                          const float *k_sys, const float *v_sys,
                          const float *k_cache, const float *v_cache,
                          int num_blocks, int block_size,
                          const int32_t *block_tables, int max_blocks_per_seq,
                          int n_rows, const int32_t *row_token, const int32_t *row_head,
                          double *out, double *lse,
                          int n_threads, int *threads_used)
{
    if (n_tokens < 0 || n_requests < 0 || Hq <= 0 || Hkv <= 0 || d <= 0 || s < 0 ||
        block_size <= 0 || max_blocks_per_seq < 0 || n_rows < 0 || Hq % Hkv != 0)
        return ORACLE_BAD_ARGUMENT;
    const int group = Hq / Hkv;
    for (int r = 0; r < n_rows; ++r) {
        const int t = row_token[r], h = row_head[r];
        if (t < 0 || t >= n_tokens || h < 0 || h >= Hq)
            return ORACLE_BAD_ARGUMENT;
        if (token_request[t] < 0 || token_request[t] >= n_requests || token_visible[t] < 0)
            return ORACLE_BAD_ARGUMENT;
    }

    int status = ORACLE_OK;
    int used = 1;
#ifdef _OPENMP
    if (n_threads > 0)
        omp_set_num_threads(n_threads);
#pragma omp parallel
    {
#pragma omp single
        used = omp_get_num_threads();
#pragma omp for schedule(dynamic, 1)
        for (int r = 0; r < n_rows; ++r) {
            const int t = row_token[r], h = row_head[r];
            const int req = token_request[t];
            const int rc = attend_one_row(
                Hkv, d, s, scale, q + ((size_t)t * Hq + h) * d, h / group, token_visible[t],
                k_sys, v_sys, k_cache, v_cache, num_blocks, block_size,
                block_tables + (size_t)req * max_blocks_per_seq, max_blocks_per_seq,
                out + (size_t)r * d, lse + r);
            if (rc != ORACLE_OK) {
#pragma omp critical
                status = rc;
            }
        }
    }
#else
    (void)n_threads;
    for (int r = 0; r < n_rows; ++r) {
        const int t = row_token[r], h = row_head[r];
        const int req = token_request[t];
        const int rc = attend_one_row(
            Hkv, d, s, scale, q + ((size_t)t * Hq + h) * d, h / group, token_visible[t],
            k_sys, v_sys, k_cache, v_cache, num_blocks, block_size,
            block_tables + (size_t)req * max_blocks_per_seq, max_blocks_per_seq,
            out + (size_t)r * d, lse + r);
        if (rc != ORACLE_OK)
            status = rc;
    }
#endif
    if (threads_used)
        *threads_used = used;
    return status;
}
