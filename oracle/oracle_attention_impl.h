/*
 * Body of the reference attention, compiled once per precision by oracle.c
 * with REAL = double (suffix _f64) and REAL = float (suffix _f32).
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing outside tests, the smoke check and the
 * benchmark's CPU-baseline leg may call this.
 *
 * What is computed (the definition of single-query softmax attention over a
 * paged KV cache; rollout in the paper's inference-engine layer, System
 * Overview, is batched decoding whose per-token step is this operation):
 *
 *   for sequence b with L = context_lens[b] tokens, query head h, g = h / G:
 *     K_t = k_pages[ block_table[b][t/16] ][g][t%16][0..d)      t = 0..L-1
 *     V_t = v_pages[ same indices ]
 *     s_t = scale * sum_i q[b][h][i] * K_t[i]                   i ascending
 *     m   = max_t s_t
 *     p_t = exp(s_t - m),  l = sum_t p_t                        t ascending
 *     out[i] = ( sum_t p_t * V_t[i] ) / l                       t ascending
 *
 * Two passes over the tokens (max first, then sums): no running rescale, no
 * splitting, no blocking.  L == 0 gives a zero row.
 */

/* one element of a pool, decoded to REAL: bf16 is exact; fp8 is code * scale */
static REAL NAME(kv_elem)(const void *pages, const float *scales, int kv_dtype,
                          int64_t page, int Hkv, int g, int slot, int d, int i)
{
    int64_t idx = (((int64_t)page * Hkv + g) * ORACLE_PAGE + slot) * d + i;
    if (kv_dtype == ORACLE_KV_BF16)
        return (REAL)oracle_bf16_to_float(((const uint16_t *)pages)[idx]);
    return (REAL)oracle_e4m3fn_to_float(((const uint8_t *)pages)[idx]) *
           (REAL)scales[(int64_t)page * Hkv + g];
}

/* scores s_t for t in [t0, t1) of row (b, h) */
static void NAME(scores)(int Hq, int Hkv, int d, int max_blocks, int kv_dtype,
                         const uint16_t *qrow, const void *k_pages, const float *k_scales,
                         const int32_t *block_table, REAL scale, int b, int h,
                         int t0, int t1, REAL *s)
{
    int G = Hq / Hkv, g = h / G;
    for (int t = t0; t < t1; ++t) {
        int64_t page = block_table[(int64_t)b * max_blocks + t / ORACLE_PAGE];
        REAL dot = 0;
        for (int i = 0; i < d; ++i)
            dot += (REAL)oracle_bf16_to_float(qrow[i]) *
                   NAME(kv_elem)(k_pages, k_scales, kv_dtype, page, Hkv, g, t % ORACLE_PAGE, d, i);
        s[t - t0] = scale * dot;
    }
}

/*
 * Unnormalised attention of row (b, h) over tokens [t0, t1):
 *   m = max s_t, l = sum exp(s_t - m), acc[i] = sum exp(s_t - m) V_t[i].
 * The full result is acc / l with [t0, t1) = [0, L).  Exposed so that the
 * split-and-merge identity can be tested on the CPU.
 */
static int NAME(partial_row)(int Hq, int Hkv, int d, int max_blocks, int kv_dtype,
                             const uint16_t *qrow, const void *k_pages, const void *v_pages,
                             const float *k_scales, const float *v_scales,
                             const int32_t *block_table, float scale_f, int b, int h,
                             int t0, int t1, REAL *m_out, REAL *l_out, REAL *acc);

int NAME(oracle_partial)(int Hq, int Hkv, int d, int max_blocks, int kv_dtype,
                         const uint16_t *q, const void *k_pages, const void *v_pages,
                         const float *k_scales, const float *v_scales,
                         const int32_t *block_table, float scale_f, int b, int h,
                         int t0, int t1, REAL *m_out, REAL *l_out, REAL *acc)
{
    /* decode: the query row of (b, h) in q [B][Hq][d] */
    return NAME(partial_row)(Hq, Hkv, d, max_blocks, kv_dtype, q + ((int64_t)b * Hq + h) * d, k_pages, v_pages,
                             k_scales, v_scales, block_table, scale_f, b, h, t0, t1, m_out, l_out, acc);
}

/* the same for an explicit query row (bf16 [d]) of head h attending sequence b */
static int NAME(partial_row)(int Hq, int Hkv, int d, int max_blocks, int kv_dtype,
                             const uint16_t *q, const void *k_pages, const void *v_pages,
                             const float *k_scales, const float *v_scales,
                             const int32_t *block_table, float scale_f, int b, int h,
                             int t0, int t1, REAL *m_out, REAL *l_out, REAL *acc)
{
    int G = Hq / Hkv, g = h / G, n = t1 - t0;
    for (int i = 0; i < d; ++i) acc[i] = 0;
    *l_out = 0;
    *m_out = -(REAL)INFINITY;
    if (n <= 0) return 0;
    REAL *s = (REAL *)malloc(sizeof(REAL) * (size_t)n);
    if (!s) return -1;
    NAME(scores)(Hq, Hkv, d, max_blocks, kv_dtype, q, k_pages, k_scales, block_table,
                 (REAL)scale_f, b, h, t0, t1, s);
    REAL m = s[0];
    for (int t = 1; t < n; ++t) if (s[t] > m) m = s[t];
    REAL l = 0;
    for (int t = 0; t < n; ++t) {
        REAL p = REAL_EXP(s[t] - m);
        int64_t page = block_table[(int64_t)b * max_blocks + (t0 + t) / ORACLE_PAGE];
        l += p;
        for (int i = 0; i < d; ++i)
            acc[i] += p * NAME(kv_elem)(v_pages, v_scales, kv_dtype, page, Hkv, g,
                                        (t0 + t) % ORACLE_PAGE, d, i);
    }
    free(s);
    *m_out = m;
    *l_out = l;
    return 0;
}

/*
 * Merge of n partial results of one row (the identity split-K relies on):
 *   M = max_s m_s;  out = sum_s e^{m_s-M} acc_s / sum_s e^{m_s-M} l_s.
 * Parts with l_s == 0 (no tokens) are skipped.  All parts empty -> zero row.
 */
void NAME(oracle_combine)(int n, int d, const REAL *m, const REAL *l, const REAL *acc, REAL *out)
{
    REAL M = -(REAL)INFINITY, den = 0;
    for (int i = 0; i < d; ++i) out[i] = 0;
    for (int s = 0; s < n; ++s) if (l[s] > 0 && m[s] > M) M = m[s];
    for (int s = 0; s < n; ++s) {
        if (!(l[s] > 0)) continue;
        REAL w = REAL_EXP(m[s] - M);
        den += w * l[s];
        for (int i = 0; i < d; ++i) out[i] += w * acc[(int64_t)s * d + i];
    }
    if (den > 0)
        for (int i = 0; i < d; ++i) out[i] /= den;
}

/*
 * out[r][0..d) for the listed rows r -> (b, h) = (rows_bh[2r], rows_bh[2r+1]).
 * Threads split the rows only, so results do not depend on the thread count.
 */
int NAME(oracle_attend_rows)(int Hq, int Hkv, int d, int max_blocks, int kv_dtype,
                             const uint16_t *q, const void *k_pages, const void *v_pages,
                             const float *k_scales, const float *v_scales,
                             const int32_t *block_table, const int32_t *context_lens,
                             float scale, const int32_t *rows_bh, int n_rows, REAL *out)
{
    int err = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int r = 0; r < n_rows; ++r) {
        int b = rows_bh[2 * r], h = rows_bh[2 * r + 1];
        REAL m, l, *o = out + (int64_t)r * d;
        int rc = NAME(oracle_partial)(Hq, Hkv, d, max_blocks, kv_dtype, q, k_pages, v_pages,
                                      k_scales, v_scales, block_table, scale, b, h,
                                      0, context_lens[b], &m, &l, o);
        if (rc) {
#pragma omp atomic write
            err = rc;
        }
        if (l > 0)
            for (int i = 0; i < d; ++i) o[i] /= l;
    }
    return err;
}

/* every (b, h): out is [B][Hq][d] */
int NAME(oracle_paged_decode_attention)(int B, int Hq, int Hkv, int d, int max_blocks, int kv_dtype,
                                        const uint16_t *q, const void *k_pages, const void *v_pages,
                                        const float *k_scales, const float *v_scales,
                                        const int32_t *block_table, const int32_t *context_lens,
                                        float scale, REAL *out)
{
    int n = B * Hq;
    int32_t *rows = (int32_t *)malloc(sizeof(int32_t) * 2 * (size_t)(n > 0 ? n : 1));
    if (!rows) return -1;
    for (int b = 0; b < B; ++b)
        for (int h = 0; h < Hq; ++h) {
            rows[2 * (b * Hq + h)] = b;
            rows[2 * (b * Hq + h) + 1] = h;
        }
    int rc = NAME(oracle_attend_rows)(Hq, Hkv, d, max_blocks, kv_dtype, q, k_pages, v_pages,
                                      k_scales, v_scales, block_table, context_lens, scale,
                                      rows, n, out);
    free(rows);
    return rc;
}

/*
 * Several query tokens per sequence over the paged cache, causal (a resumed
 * trajectory re-computes attention for a stretch of its stored tokens at once).
 * Sequence b owns the query rows q_start[b] .. q_start[b+1]-1 of q
 * [rows][Hq][d]; they are its LAST n_b positions: row i sits at position
 * pos = context_lens[b] - n_b + i and attends the tokens 0 .. pos, i.e. it is
 * the single-query problem with context length pos + 1.  Rows with pos < 0
 * (more queries than tokens) give zero rows.  out is [rows][Hq][d].
 */
int NAME(oracle_paged_prefill_attention)(int B, int Hq, int Hkv, int d, int max_blocks, int kv_dtype,
                                         const uint16_t *q, const int32_t *q_start,
                                         const void *k_pages, const void *v_pages,
                                         const float *k_scales, const float *v_scales,
                                         const int32_t *block_table, const int32_t *context_lens,
                                         float scale, REAL *out)
{
    int err = 0;
    for (int b = 0; b < B; ++b) {
        int n = q_start[b + 1] - q_start[b];
#pragma omp parallel for schedule(dynamic, 1) collapse(2)
        for (int i = 0; i < n; ++i)
            for (int h = 0; h < Hq; ++h) {
                int64_t r = (int64_t)q_start[b] + i;
                int pos = context_lens[b] - n + i;
                REAL m, l, *o = out + (r * Hq + h) * d;
                int rc = NAME(partial_row)(Hq, Hkv, d, max_blocks, kv_dtype, q + (r * Hq + h) * d, k_pages,
                                           v_pages, k_scales, v_scales, block_table, scale, b, h, 0, pos + 1,
                                           &m, &l, o);
                if (rc) {
#pragma omp atomic write
                    err = rc;
                }
                if (l > 0)
                    for (int j = 0; j < d; ++j) o[j] /= l;
            }
    }
    return err;
}
