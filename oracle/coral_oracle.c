/*
 * TEST INFRASTRUCTURE -- not part of the product.
 *
 * Plain, slow fp64 CPU definition of the weight-grouped LM head of a
 * speculative-decoding draft model (paper section 3.3 "LM Head Router" and
 * the appendix "Discussion on LM Head Router").  Only tests, the smoke check
 * and the benchmark's cpu_baseline leg may call it.  It shares no code with
 * the HIP library and includes none of its headers.
 *
 * What is computed, in the paper's order:
 *   gate      s[m,n] = sum_j W2[n,j] * u[m,j] (+ bias[n])        (Eq. 7: the
 *             W2 projection of the router; softmax is monotone, so the
 *             selection below is taken on s itself)
 *   top-n     the g groups with the largest s[m,.]                (section
 *             4.2.3: the top-n of the N groups are activated)
 *   logits    z[m,r] = sum_j W[r,j] * h[m,j] for the rows r of token m's own
 *             selected groups only (section 3.3: only a subset of the LM-head
 *             parameters is activated; Eq. 8 gives zero mass outside them)
 *   top-k     the k largest z[m,.] among those rows (appendix, tree
 *             decoding: ten candidates per draft token)
 *   dense     the same with every vocabulary row a candidate (the "N/A" row
 *             of Table 4)
 *   lse / log p_router  per-group log-sum-exp and the router's log-softmax,
 *             the two terms of Eq. 8's log p(x) = log p_router(n) + z - lse_n
 *
 * Every sum is a left-to-right fp64 accumulation over j = 0..H-1; inputs
 * (fp32 or bf16 bit patterns) widen to fp64 exactly.  Orders are total:
 * larger value first, then smaller index, so results are unique.
 *
 * Pins (tests/test_oracle_pins.py): brute force in numpy on tiny inputs,
 * float64 matmul + argsort, one-hot closed forms, g = G equals dense,
 * partition and nesting invariants, planted-mistake checks.  The paper prints
 * no worked numbers for this path, so agreement with the paper's own
 * implementation is "parity unpinned"; only shapes and byte counts are pinned
 * to its Table 1 and appendix.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1, ORACLE_F16 = 2 };

enum {
    ORACLE_OK = 0,
    ORACLE_ERR_ARG = -1,
    ORACLE_ERR_PARTITION = -2,
    ORACLE_ERR_NOMEM = -3
};

static inline double widen(const void *base, size_t idx, int dtype)
{
    if (dtype == ORACLE_F32)
        return (double)((const float *)base)[idx];
    const uint16_t h = ((const uint16_t *)base)[idx];
    if (dtype == ORACLE_F16) {      /* IEEE binary16: 1 sign, 5 exponent (bias 15), 10 fraction bits */
        const int sign = h >> 15, ex = (h >> 10) & 31, fr = h & 1023;
        double v;
        if (ex == 0)
            v = ldexp((double)fr, -24);                    /* zero and subnormals */
        else if (ex == 31)
            v = fr ? NAN : INFINITY;
        else
            v = ldexp((double)(1024 + fr), ex - 25);
        return sign ? -v : v;
    }
    uint32_t u = ((uint32_t)h) << 16;                      /* bf16: the upper half of a float */
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

int coral_oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void coral_oracle_set_threads(int n)
{
#ifdef _OPENMP
    if (n > 0)
        omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* The vocabulary partition must hold every id exactly once (section 3.3:
 * the head is divided into N groups). */
int coral_oracle_check_partition(const int32_t *offsets, const int32_t *rows,
                                 int G, int V)
{
    if (!offsets || !rows || G < 1 || V < 1)
        return ORACLE_ERR_ARG;
    if (offsets[0] != 0 || offsets[G] != V)
        return ORACLE_ERR_PARTITION;
    for (int n = 0; n < G; ++n)
        if (offsets[n + 1] < offsets[n])
            return ORACLE_ERR_PARTITION;
    unsigned char *seen = calloc((size_t)V, 1);
    if (!seen)
        return ORACLE_ERR_NOMEM;
    int rc = ORACLE_OK;
    for (int i = 0; i < V; ++i) {
        int32_t r = rows[i];
        if (r < 0 || r >= V || seen[r]) {
            rc = ORACLE_ERR_PARTITION;
            break;
        }
        seen[r] = 1;
    }
    free(seen);
    return rc;
}

/* Eq. 7, W2 projection: s[m,n] = sum_j gate_W[n,j] * hidden[m,j] + bias[n]. */
int coral_oracle_gate(const void *hidden, const void *gate_W,
                      const float *gate_bias, int M, int H, int G, int dtype,
                      double *s)
{
    if (!hidden || !gate_W || !s || M < 1 || H < 1 || G < 1)
        return ORACLE_ERR_ARG;
    for (int m = 0; m < M; ++m)
        for (int n = 0; n < G; ++n) {
            double acc = 0.0;
            for (int j = 0; j < H; ++j)
                acc += widen(gate_W, (size_t)n * H + j, dtype) *
                       widen(hidden, (size_t)m * H + j, dtype);
            if (gate_bias)
                acc += (double)gate_bias[n];
            s[(size_t)m * G + n] = acc;
        }
    return ORACLE_OK;
}

struct scored {
    double val;
    int32_t id;
};

static int by_value_then_id(const void *a, const void *b)
{
    const struct scored *x = a, *y = b;
    if (x->val > y->val)
        return -1;
    if (x->val < y->val)
        return 1;
    if (x->id < y->id)
        return -1;
    if (x->id > y->id)
        return 1;
    return 0;
}

/* Full order of the groups per token: larger score first, then lower group
 * id.  order[m, 0..g) is the selection. */
int coral_oracle_rank_groups(const double *s, int M, int G, int32_t *order)
{
    if (!s || !order || M < 1 || G < 1)
        return ORACLE_ERR_ARG;
    struct scored *buf = malloc((size_t)G * sizeof *buf);
    if (!buf)
        return ORACLE_ERR_NOMEM;
    for (int m = 0; m < M; ++m) {
        for (int n = 0; n < G; ++n) {
            buf[n].val = s[(size_t)m * G + n];
            buf[n].id = n;
        }
        qsort(buf, (size_t)G, sizeof *buf, by_value_then_id);
        for (int n = 0; n < G; ++n)
            order[(size_t)m * G + n] = buf[n].id;
    }
    free(buf);
    return ORACLE_OK;
}

/* z[i] = sum_j lm_W[rows[i], j] * hidden_row[j] for one token. */
int coral_oracle_logits_rows(const void *hidden_row, const void *lm_W, int H,
                             int V, const int32_t *rows, int64_t n_rows,
                             int dtype, double *z)
{
    if (!hidden_row || !lm_W || !rows || !z || H < 1 || V < 1 || n_rows < 0)
        return ORACLE_ERR_ARG;
    for (int64_t i = 0; i < n_rows; ++i)
        if (rows[i] < 0 || rows[i] >= V)
            return ORACLE_ERR_ARG;
    double *h = malloc((size_t)H * sizeof *h);
    if (!h)
        return ORACLE_ERR_NOMEM;
    for (int j = 0; j < H; ++j)
        h[j] = widen(hidden_row, (size_t)j, dtype);
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n_rows; ++i) {
        size_t base = (size_t)rows[i] * H;
        double acc = 0.0;
        for (int j = 0; j < H; ++j)
            acc += widen(lm_W, base + j, dtype) * h[j];
        z[i] = acc;
    }
    free(h);
    return ORACLE_OK;
}

/* Full sort of n candidates by (value descending, id ascending); emits the
 * first k and the value ranked k+1 (-inf if there is none). */
int coral_oracle_top_k(const double *z, const int32_t *ids, int64_t n, int k,
                       int32_t *out_ids, double *out_z, double *next_z)
{
    if (!z || !ids || !out_ids || !out_z || k < 1 || (int64_t)k > n)
        return ORACLE_ERR_ARG;
    struct scored *buf = malloc((size_t)n * sizeof *buf);
    if (!buf)
        return ORACLE_ERR_NOMEM;
    for (int64_t i = 0; i < n; ++i) {
        buf[i].val = z[i];
        buf[i].id = ids[i];
    }
    qsort(buf, (size_t)n, sizeof *buf, by_value_then_id);
    for (int i = 0; i < k; ++i) {
        out_ids[i] = buf[i].id;
        out_z[i] = buf[i].val;
    }
    if (next_z)
        *next_z = ((int64_t)k < n) ? buf[k].val : -INFINITY;
    free(buf);
    return ORACLE_OK;
}

static double logsumexp(const double *x, int64_t n)
{
    double mx = -INFINITY;
    for (int64_t i = 0; i < n; ++i)
        if (x[i] > mx)
            mx = x[i];
    double acc = 0.0;
    for (int64_t i = 0; i < n; ++i)
        acc += exp(x[i] - mx);
    return mx + log(acc);
}

/*
 * The grouped head for M tokens.
 *   forced_sel  NULL: select by the gate (top-g of s).  Otherwise [M,g] group
 *               ids to use instead (s and log p_router are still computed).
 * Outputs (any of the optional ones may be NULL):
 *   s[M,G] gate scores, sel[M,g] selected groups in rank order,
 *   topk_ids[M,k], topk_z[M,k], next_z[M] (value ranked k+1, or -inf),
 *   lse[M,g] log-sum-exp of the logits of each selected group (Eq. 8's
 *   per-group softmax normaliser), logp_router[M,G] = log softmax of s over
 *   all G groups (Eq. 7).
 */
int coral_oracle_grouped(const void *hidden, const void *gate_W,
                         const float *gate_bias, const void *lm_W,
                         const int32_t *offsets, const int32_t *rows, int M,
                         int H, int V, int G, int g, int k, int dtype,
                         const int32_t *forced_sel, double *s, int32_t *sel,
                         int32_t *topk_ids, double *topk_z, double *next_z,
                         double *lse, double *logp_router)
{
    if (!hidden || !gate_W || !lm_W || !offsets || !rows || !s || !sel ||
        !topk_ids || !topk_z)
        return ORACLE_ERR_ARG;
    if (M < 1 || H < 1 || V < 1 || G < 1 || g < 1 || g > G || k < 1)
        return ORACLE_ERR_ARG;
    int rc = coral_oracle_check_partition(offsets, rows, G, V);
    if (rc)
        return rc;
    rc = coral_oracle_gate(hidden, gate_W, gate_bias, M, H, G, dtype, s);
    if (rc)
        return rc;
    int32_t *order = malloc((size_t)M * G * sizeof *order);
    if (!order)
        return ORACLE_ERR_NOMEM;
    rc = coral_oracle_rank_groups(s, M, G, order);
    if (rc) {
        free(order);
        return rc;
    }
    for (int m = 0; m < M; ++m)
        for (int i = 0; i < g; ++i) {
            int32_t n = forced_sel ? forced_sel[(size_t)m * g + i]
                                   : order[(size_t)m * G + i];
            if (n < 0 || n >= G) {
                free(order);
                return ORACLE_ERR_ARG;
            }
            for (int i2 = 0; i2 < i; ++i2)
                if (sel[(size_t)m * g + i2] == n) {
                    free(order);
                    return ORACLE_ERR_ARG;
                }
            sel[(size_t)m * g + i] = n;
        }
    free(order);

    if (logp_router)
        for (int m = 0; m < M; ++m) {
            double l = logsumexp(s + (size_t)m * G, G);
            for (int n = 0; n < G; ++n)
                logp_router[(size_t)m * G + n] = s[(size_t)m * G + n] - l;
        }

    for (int m = 0; m < M; ++m) {
        int64_t n_cand = 0;
        for (int i = 0; i < g; ++i) {
            int32_t n = sel[(size_t)m * g + i];
            n_cand += offsets[n + 1] - offsets[n];
        }
        if ((int64_t)k > n_cand)
            return ORACLE_ERR_ARG;
        int32_t *cand = malloc((size_t)n_cand * sizeof *cand);
        double *z = malloc((size_t)n_cand * sizeof *z);
        if (!cand || !z) {
            free(cand);
            free(z);
            return ORACLE_ERR_NOMEM;
        }
        int64_t pos = 0;
        for (int i = 0; i < g; ++i) {
            int32_t n = sel[(size_t)m * g + i];
            for (int32_t t = offsets[n]; t < offsets[n + 1]; ++t)
                cand[pos++] = rows[t];
        }
        const void *hrow = (dtype == ORACLE_F32)
                               ? (const void *)((const float *)hidden + (size_t)m * H)
                               : (const void *)((const uint16_t *)hidden + (size_t)m * H);
        rc = coral_oracle_logits_rows(hrow, lm_W, H, V, cand, n_cand, dtype, z);
        if (!rc && lse) {
            pos = 0;
            for (int i = 0; i < g; ++i) {
                int32_t n = sel[(size_t)m * g + i];
                int64_t len = offsets[n + 1] - offsets[n];
                lse[(size_t)m * g + i] = logsumexp(z + pos, len);
                pos += len;
            }
        }
        if (!rc)
            rc = coral_oracle_top_k(z, cand, n_cand, k, topk_ids + (size_t)m * k,
                                    topk_z + (size_t)m * k,
                                    next_z ? next_z + m : NULL);
        free(cand);
        free(z);
        if (rc)
            return rc;
    }
    return ORACLE_OK;
}

/* The dense head: every vocabulary row is a candidate for every token. */
int coral_oracle_dense(const void *hidden, const void *lm_W, int M, int H,
                       int V, int k, int dtype, int32_t *topk_ids,
                       double *topk_z, double *next_z)
{
    if (!hidden || !lm_W || !topk_ids || !topk_z)
        return ORACLE_ERR_ARG;
    if (M < 1 || H < 1 || V < 1 || k < 1 || k > V)
        return ORACLE_ERR_ARG;
    int32_t *cand = malloc((size_t)V * sizeof *cand);
    double *z = malloc((size_t)V * sizeof *z);
    if (!cand || !z) {
        free(cand);
        free(z);
        return ORACLE_ERR_NOMEM;
    }
    for (int32_t r = 0; r < V; ++r)
        cand[r] = r;
    int rc = ORACLE_OK;
    for (int m = 0; m < M && !rc; ++m) {
        const void *hrow = (dtype == ORACLE_F32)
                               ? (const void *)((const float *)hidden + (size_t)m * H)
                               : (const void *)((const uint16_t *)hidden + (size_t)m * H);
        rc = coral_oracle_logits_rows(hrow, lm_W, H, V, cand, V, dtype, z);
        if (!rc)
            rc = coral_oracle_top_k(z, cand, V, k, topk_ids + (size_t)m * k,
                                    topk_z + (size_t)m * k,
                                    next_z ? next_z + m : NULL);
    }
    free(cand);
    free(z);
    return rc;
}
