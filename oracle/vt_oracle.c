/*
 * CPU oracle for the trimmed-LM-head path of VocabTrim.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition of what
 * the GPU library computes.  Only the tests, the smoke check and the
 * benchmark's cpu_baseline leg may build, load or call it; the product path
 * never does.  It shares no code, header, table or helper with the HIP
 * sources.
 *
 * Every real-valued quantity is fp64.  Inputs stored as bf16 or fp32 are
 * widened exactly.  No blocking, fusion or reordering: each function is the
 * definition written out, in the paper's order and notation.
 *
 * Pins (see tests/test_oracle_*.py): library bincount / lexsort / fp64 matmul /
 * logsumexp, brute force on tiny inputs, closed forms (h = 0 gives -ln k,
 * two-level logits), invariants (counts sum to the token count, probabilities
 * sum to 1, k = V reproduces the full head).  The paper prints no worked value
 * of a count, a logit or a log-probability, so none of these pins is a value
 * from the paper; its printed head sizes pin only the shapes.
 */
#define _GNU_SOURCE
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ------------------------------------------------------------------ */
/* threads (only the projection loop is parallel: rows are independent) */
/* ------------------------------------------------------------------ */
static int g_threads = 0; /* 0 = OpenMP default */

void vt_oracle_set_threads(int t) { g_threads = t; }

int vt_oracle_get_threads(void) {
#ifdef _OPENMP
    return g_threads > 0 ? g_threads : omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------ */
/* Algorithm 1 (Count Token Frequencies): c[t_i] <- c[t_i] + 1          */
/* The counter vector is accumulated into, so a corpus may be fed in    */
/* chunks; the caller zeroes it before the first chunk ("initialize     */
/* with zeros").  Ids outside [0, V) cannot occur in the paper (same    */
/* tokenizer on both sides); here they are skipped and tallied.         */
/* ------------------------------------------------------------------ */
void vt_oracle_count(const void *ids, int ids_are_int64, int64_t n_ids, int32_t V,
                     int64_t *c, int64_t *n_invalid) {
    for (int64_t i = 0; i < n_ids; ++i) {
        int64_t t = ids_are_int64 ? ((const int64_t *)ids)[i] : (int64_t)((const int32_t *)ids)[i];
        if (t >= 0 && t < (int64_t)V) {
            c[t] = c[t] + 1;
        } else if (n_invalid) {
            *n_invalid += 1;
        }
    }
}

/* ------------------------------------------------------------------ */
/* Eq. 1, first line: V_trim = V[Top-K(c, k)].                          */
/* Top-K = the k ids with the largest counts; equal counts -> the lower */
/* id first.  Done as a full sort of all (count, id) pairs.  The k      */
/* survivors are then listed by ascending id (the canonical row order   */
/* of the trimmed head), which is the token index mapper T_{d->t}.      */
/* ------------------------------------------------------------------ */
typedef struct {
    int64_t count;
    int32_t id;
} vt_pair;

static int cmp_count_desc_id_asc(const void *a, const void *b) {
    const vt_pair *x = (const vt_pair *)a, *y = (const vt_pair *)b;
    if (x->count != y->count) return x->count > y->count ? -1 : 1;
    if (x->id != y->id) return x->id < y->id ? -1 : 1;
    return 0;
}

static int cmp_i32_asc(const void *a, const void *b) {
    int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

/* rank_order (nullable, [k]) receives the same ids in (count desc, id asc) order. */
void vt_oracle_select(const int64_t *c, int32_t V, int32_t k, int32_t *map, int32_t *rank_order) {
    vt_pair *p = (vt_pair *)malloc((size_t)V * sizeof(vt_pair));
    for (int32_t id = 0; id < V; ++id) {
        p[id].count = c[id];
        p[id].id = id;
    }
    qsort(p, (size_t)V, sizeof(vt_pair), cmp_count_desc_id_asc);
    for (int32_t j = 0; j < k; ++j) {
        map[j] = p[j].id;
        if (rank_order) rank_order[j] = p[j].id;
    }
    qsort(map, (size_t)k, sizeof(int32_t), cmp_i32_asc);
    free(p);
}

/* ------------------------------------------------------------------ */
/* Eq. 1, second line: W_trim = W[Top-K(c, k), :]  (row copy, bit-exact) */
/* W is [V, d] row-major, one row per token.                             */
/* ------------------------------------------------------------------ */
void vt_oracle_gather(const void *W, int64_t elem_bytes, int32_t d, const int32_t *map, int32_t k,
                      void *W_trim) {
    const size_t row = (size_t)d * (size_t)elem_bytes;
    for (int32_t j = 0; j < k; ++j) {
        memcpy((char *)W_trim + (size_t)j * row, (const char *)W + (size_t)map[j] * row, row);
    }
}

/* ------------------------------------------------------------------ */
/* exact widening of the stored element types                          */
/* ------------------------------------------------------------------ */
static double widen_bf16(uint16_t bits) {
    uint32_t u = (uint32_t)bits << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

static double load_elem(const void *p, int is_bf16, size_t idx) {
    return is_bf16 ? widen_bf16(((const uint16_t *)p)[idx]) : (double)((const float *)p)[idx];
}

/* ------------------------------------------------------------------ */
/* LM-head projection with the trimmed head (Alg. 2, the drafter's      */
/* output over the trimmed vocabulary):                                  */
/*   z[i, j] = sum_{t=0}^{d-1} h[i, t] * W_trim[j, t]                    */
/* fp64, summed left to right.                                           */
/* ------------------------------------------------------------------ */
void vt_oracle_logits(const void *h, const void *W_trim, int is_bf16, int32_t n, int32_t k,
                      int32_t d, double *z) {
    double *hd = (double *)malloc((size_t)n * (size_t)d * sizeof(double));
    for (size_t q = 0; q < (size_t)n * (size_t)d; ++q) hd[q] = load_elem(h, is_bf16, q);
#ifdef _OPENMP
    int nt = vt_oracle_get_threads();
#pragma omp parallel for schedule(static) num_threads(nt)
#endif
    for (int32_t j = 0; j < k; ++j) {
        for (int32_t i = 0; i < n; ++i) {
            double s = 0.0;
            for (int32_t t = 0; t < d; ++t) {
                s += hd[(size_t)i * d + t] * load_elem(W_trim, is_bf16, (size_t)j * d + t);
            }
            z[(size_t)i * k + j] = s;
        }
    }
    free(hd);
}

/* ------------------------------------------------------------------ */
/* log-softmax over the k trimmed logits of each row:                   */
/*   M_i = max_j z[i,j];  S_i = sum_j exp(z[i,j] - M_i);                 */
/*   lse_i = M_i + log S_i;  logp[i,j] = z[i,j] - lse_i                  */
/* ------------------------------------------------------------------ */
void vt_oracle_log_softmax(const double *z, int32_t n, int32_t k, double *lse, double *logp) {
    for (int32_t i = 0; i < n; ++i) {
        const double *zi = z + (size_t)i * k;
        double M = zi[0];
        for (int32_t j = 1; j < k; ++j)
            if (zi[j] > M) M = zi[j];
        double S = 0.0;
        for (int32_t j = 0; j < k; ++j) S += exp(zi[j] - M);
        lse[i] = M + log(S);
        if (logp)
            for (int32_t j = 0; j < k; ++j) logp[(size_t)i * k + j] = zi[j] - lse[i];
    }
}

/* ------------------------------------------------------------------ */
/* Draft-token selection (EAGLE-2 style: the m most probable tokens per */
/* node, greedy when m = 1) followed by the mapper of Alg. 2:            */
/*   y_hat = T_{d->t}(z_hat) = map[z_hat].                               */
/* Full sort of the k trimmed indices by (logit desc, target id asc).    */
/* ------------------------------------------------------------------ */
typedef struct {
    const double *z;
    const int32_t *map;
} vt_sort_ctx;

static int cmp_logit_desc_id_asc(const void *a, const void *b, void *ctx) {
    const vt_sort_ctx *c = (const vt_sort_ctx *)ctx;
    int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    if (c->z[x] != c->z[y]) return c->z[x] > c->z[y] ? -1 : 1;
    if (c->map[x] != c->map[y]) return c->map[x] < c->map[y] ? -1 : 1;
    return 0;
}

void vt_oracle_top_m(const double *z, const double *lse, int32_t n, int32_t k, const int32_t *map,
                     int32_t m, int32_t *out_ids, double *out_logp, int32_t *out_trim_idx) {
    int32_t *order = (int32_t *)malloc((size_t)k * sizeof(int32_t));
    for (int32_t i = 0; i < n; ++i) {
        vt_sort_ctx ctx = {z + (size_t)i * k, map};
        for (int32_t j = 0; j < k; ++j) order[j] = j;
        qsort_r(order, (size_t)k, sizeof(int32_t), cmp_logit_desc_id_asc, &ctx);
        for (int32_t r = 0; r < m; ++r) {
            int32_t j = order[r];
            out_ids[(size_t)i * m + r] = map[j];
            out_logp[(size_t)i * m + r] = ctx.z[j] - lse[i];
            if (out_trim_idx) out_trim_idx[(size_t)i * m + r] = j;
        }
    }
    free(order);
}
