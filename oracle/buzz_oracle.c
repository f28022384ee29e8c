/*
 * buzz_oracle.c -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, obviously-correct CPU implementation of the BUZZ sparse
 * KV-cache decode path (arxiv 2410.23079), written from the paper:
 *
 *   - cache append before attention            (Sec. 3.1, eq. 2)
 *   - softmax attention over the retained rows  (Sec. 3.1, eq. 3 and eq. 5)
 *   - accumulated attention score per row       (Alg. 2 input "A"; Sec. 4.1
 *                                                "accumulated attention scores")
 *   - the eviction policy                       (Sec. 3.3, Alg. 1, Alg. 2,
 *                                                Remark 1, Remark 2)
 *
 * Everything is computed in double precision, row by row, in the order the
 * paper states it.  No blocking, no fusion, no split softmax.  The only
 * parallelism is an OpenMP loop over independent (batch, kv-head) units,
 * which the paper treats as separate caches ("we only consider one head").
 *
 * Only tests, the smoke check and the CPU-baseline leg of the benchmark may
 * call this file.  It shares no code, header, table or helper with the HIP
 * library, and neither includes the other.
 *
 * Readings of the paper where it is silent or ambiguous (each one is also
 * listed in the design notes of this repository):
 *   - the score that is accumulated is the post-softmax probability, summed
 *     over decode steps and over the query heads that share a kv head;
 *   - a decode step attends to its own freshly appended token, and that token
 *     receives score in the same step (eq. 2 updates K before eq. 3);
 *   - the threshold T counts the tokens that have left the window and are not
 *     yet sampled ("new" tokens); eviction fires when that count reaches T;
 *   - segments are anchored at the first new token, the last one may be
 *     ragged and still yields min(keep, len) survivors (Alg. 2 loop bound);
 *   - arg-max ties go to the lowest index; NaN scores rank below everything;
 *   - keep > 1 per segment takes the top-`keep` under (score desc, index asc)
 *     and emits them in index order;
 *   - interval sampling of old tokens keeps offsets 0, s^, 2 s^, ... ;
 *     s^ = floor((s+1)/2) unless the caller overrides it (s^ = 1 keeps all);
 *   - in prefill the eviction runs once when the count compared with T is
 *     >= T, and again while the rows do not fit their container (Remark 2):
 *     T + k + w rows when T bounds old + new tokens together, or an explicit
 *     capacity less the T rows buffered before the next eviction;
 *   - optional variants: log-n scaled attention (Sec. 3.5) multiplies the
 *     softmax scale by log(n)/log(512), n = number of tokens the query sees,
 *     itself included; and the threshold may instead bound old + new tokens
 *     together, which is how the proof of the Parameter Estimation theorem
 *     reads T; the ablation of Sec. 4.3 that drops the local-max function
 *     keeps the first rows of every segment instead of the highest-scoring;
 *     the H2O-style baseline the paper compares with (Sec. 4.1) keeps the
 *     `keep` highest accumulated scores among all rows between sink and
 *     window, with no segments and no old / new distinction.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    int32_t batch, n_q_heads, n_kv_heads, head_dim;
    int32_t sink;        /* k  */
    int32_t window;      /* w  */
    int32_t segment;     /* s  */
    int32_t keep;        /* survivors per segment; the paper uses 1 */
    int32_t evict_every; /* T  */
    int32_t old_stride;  /* s^ ; 0 => floor((s+1)/2) */
    int32_t auto_evict;  /* decode_step evicts by itself when the count reaches T */
    int32_t variant;     /* bit 0: log-n scaled attention (Sec. 3.5): scale *= log(n)/log(512), n = tokens so far
                            bit 1: T bounds old + new tokens together (the reading used by the theorem's proof)
                            bit 2: ablation "no local max" (Sec. 4.3): new tokens are interval-sampled too, i.e.
                                   the first `keep` rows of every segment survive whatever their scores
                            bit 3: H2O-style baseline (Sec. 4.1, "greedy accumulated attention scores"): every row
                                   between sink and window, old or new, competes in one segment; the `keep`
                                   highest-scoring survive */
    int64_t capacity;    /* logical row bound used by Remark 2; 0 => none */
    double  softmax_scale; /* 0 => 1/sqrt(head_dim) */
} oracle_config;

typedef struct {
    double  *K, *V;  /* [n][D] */
    double  *A;      /* [n]  accumulated score */
    int32_t *pos;    /* [n]  original token index */
    int64_t  n, n_old, alloc;
} unit_t;

typedef struct {
    oracle_config cfg;
    int64_t  n_units;
    int64_t  tokens_seen;
    unit_t  *u;
} oracle_t;

enum { ORACLE_OK = 0, ORACLE_EINVAL = -1, ORACLE_ECAPACITY = -2, ORACLE_ENOMEM = -3 };

static int64_t old_stride_of(const oracle_config *c)
{
    return c->old_stride > 0 ? c->old_stride : (c->segment + 1) / 2; /* Sec. 3.3, BeeHive */
}

/* softmax scale for a query that sees n_ctx tokens (itself included) */
static double scale_of(const oracle_config *c, int64_t n_ctx)
{
    double s = c->softmax_scale != 0.0 ? c->softmax_scale : 1.0 / sqrt((double)c->head_dim); /* eq. 3 */
    if (c->variant & 1) s *= log((double)n_ctx) / log(512.0);   /* Sec. 3.5: log_512(n) / sqrt(d) */
    return s;
}

static int unit_reserve(unit_t *x, int64_t rows, int64_t D)
{
    if (rows <= x->alloc) return 0;
    int64_t na = x->alloc ? x->alloc : 64;
    while (na < rows) na *= 2;
    double *K = realloc(x->K, sizeof(double) * na * D);
    if (!K) return -1;
    x->K = K;
    double *V = realloc(x->V, sizeof(double) * na * D);
    if (!V) return -1;
    x->V = V;
    double *A = realloc(x->A, sizeof(double) * na);
    if (!A) return -1;
    x->A = A;
    int32_t *p = realloc(x->pos, sizeof(int32_t) * na);
    if (!p) return -1;
    x->pos = p;
    x->alloc = na;
    return 0;
}

int oracle_create(const oracle_config *cfg, oracle_t **out)
{
    if (!cfg || !out) return ORACLE_EINVAL;
    if (cfg->batch < 1 || cfg->n_kv_heads < 1 || cfg->n_q_heads < 1 || cfg->head_dim < 1) return ORACLE_EINVAL;
    if (cfg->n_q_heads % cfg->n_kv_heads) return ORACLE_EINVAL;
    if (cfg->sink < 0 || cfg->window < 0 || cfg->segment < 1 || cfg->keep < 0 || cfg->evict_every < 1) return ORACLE_EINVAL;
    if (cfg->old_stride < 0) return ORACLE_EINVAL;
    oracle_t *o = calloc(1, sizeof(*o));
    if (!o) return ORACLE_ENOMEM;
    o->cfg = *cfg;
    o->n_units = (int64_t)cfg->batch * cfg->n_kv_heads;
    o->u = calloc((size_t)o->n_units, sizeof(unit_t));
    if (!o->u) { free(o); return ORACLE_ENOMEM; }
    *out = o;
    return ORACLE_OK;
}

void oracle_destroy(oracle_t *o)
{
    if (!o) return;
    for (int64_t i = 0; i < o->n_units; ++i) {
        free(o->u[i].K); free(o->u[i].V); free(o->u[i].A); free(o->u[i].pos);
    }
    free(o->u);
    free(o);
}

/* a ranks strictly before b in the selection order: larger score first,
 * NaN treated as -infinity, equal scores -> smaller index first. */
static int ranks_before(double sa, int64_t ia, double sb, int64_t ib)
{
    if (isnan(sa)) sa = -INFINITY;
    if (isnan(sb)) sb = -INFINITY;
    if (sa > sb) return 1;
    if (sa < sb) return 0;
    return ia < ib;
}

/* The eviction branch of Alg. 1 (split, sample both parts, concatenate) plus Alg. 2, on one unit. */
static int unit_evict(const oracle_config *c, unit_t *x)
{
    const int64_t k = c->sink, w = c->window, D = c->head_dim;
    const int64_t sh = old_stride_of(c);
    if (x->n <= k + w) return 0;                     /* Remark 1: fill sink and window first */
    const int global = c->variant & 8;               /* H2O-style baseline: no old / new split, no segments */
    const int64_t lo = global ? k : k + x->n_old;    /* K_new = K[k + n_old : -w]  (Alg. 1) */
    const int64_t hi = x->n - w;
    if (lo > hi) return ORACLE_EINVAL;
    const int64_t s = global ? (hi > lo ? hi - lo : 1) : c->segment;   /* ... = one segment over the whole middle */

    int64_t *keep_idx = malloc(sizeof(int64_t) * (size_t)(x->n + 1));
    if (!keep_idx) return ORACLE_ENOMEM;
    int64_t m = 0;
    for (int64_t j = 0; j < k; ++j) keep_idx[m++] = j;            /* K[:k] */
    int64_t cnt_old = 0;
    for (int64_t j = k; j < lo; j += sh) { keep_idx[m++] = j; ++cnt_old; }   /* interval_sample(s^, K_old) */
    int64_t cnt_new = 0;
    for (int64_t idx = lo; idx < hi; idx += s) {                  /* local_max_sample(s, K_new), Alg. 2 */
        const int64_t end = idx + s < hi ? idx + s : hi;
        const int64_t len = end - idx;
        const int64_t take = c->keep < len ? c->keep : len;
        /* a row survives iff fewer than `take` rows of its segment rank before it */
        for (int64_t j = idx; j < end; ++j) {
            int64_t before = 0;
            for (int64_t i = idx; i < end; ++i) {
                if (i == j) continue;
                if (c->variant & 4) before += i < j;                       /* ablation: interval sampling, scores unused */
                else if (ranks_before(x->A[i], i, x->A[j], j)) ++before;
            }
            if (before < take) { keep_idx[m++] = j; ++cnt_new; }
        }
    }
    for (int64_t j = hi; j < x->n; ++j) keep_idx[m++] = j;        /* K[-w:] */

    /* concatenate [sink, old', new', window]; keep_idx is increasing so a
     * forward in-order copy never overwrites an unread row */
    for (int64_t r = 0; r < m; ++r) {
        const int64_t j = keep_idx[r];
        if (j == r) continue;
        memmove(x->K + r * D, x->K + j * D, sizeof(double) * D);
        memmove(x->V + r * D, x->V + j * D, sizeof(double) * D);
        x->A[r] = x->A[j];
        x->pos[r] = x->pos[j];
    }
    x->n = m;
    x->n_old = cnt_old + cnt_new;
    free(keep_idx);
    return 0;
}

int oracle_evict(oracle_t *o)
{
    if (!o) return ORACLE_EINVAL;
    int rc = 0;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < o->n_units; ++i) {
        int r = unit_evict(&o->cfg, &o->u[i]);
        if (r) {
#pragma omp critical
            rc = r;
        }
    }
    return rc;
}

static int64_t new_count_of(const oracle_config *c, const unit_t *x)
{
    int64_t v = x->n - c->sink - x->n_old - c->window;
    return v > 0 ? v : 0;
}

/* the quantity compared with T: buffered new tokens (Alg. 1), or old + new (proof of the theorem) */
static int64_t trigger_count_of(const oracle_config *c, const unit_t *x)
{
    const int64_t nc = new_count_of(c, x);
    return (c->variant & 2) ? x->n_old + nc : nc;
}

/* softmax(scale * q . K_j) over rows j < n of one unit; p has n entries */
static void softmax_row(const double *q, const double *K, int64_t n, int64_t D, double scale, double *p)
{
    double mx = -INFINITY;
    for (int64_t j = 0; j < n; ++j) {
        double dot = 0.0;
        for (int64_t d = 0; d < D; ++d) dot += q[d] * K[j * D + d];
        p[j] = scale * dot;
        if (p[j] > mx) mx = p[j];
    }
    double sum = 0.0;
    for (int64_t j = 0; j < n; ++j) { p[j] = exp(p[j] - mx); sum += p[j]; }
    for (int64_t j = 0; j < n; ++j) p[j] /= sum;
}

/*
 * Prefill (eq. 1 gives K, V; Remark 2 gives the sampling).
 *   K, V     [batch][n_kv_heads][N][D]
 *   q_obs    [batch][n_q_heads][n_obs][D] -- queries of the last n_obs prompt
 *            positions; query t sits at position N - n_obs + t and attends
 *            causally to keys 0..that position.  May be NULL when n_obs == 0.
 *   init     [batch][n_kv_heads][N] starting scores, or NULL for zeros.
 */
int oracle_prefill(oracle_t *o, const double *K, const double *V, int64_t N,
                   const double *q_obs, int64_t n_obs, const double *init)
{
    if (!o || !K || !V || N < 0 || n_obs < 0 || n_obs > N || (n_obs > 0 && !q_obs)) return ORACLE_EINVAL;
    const oracle_config *c = &o->cfg;
    const int64_t D = c->head_dim, G = c->n_q_heads / c->n_kv_heads, Hkv = c->n_kv_heads, Hq = c->n_q_heads;
    int rc = 0;
#pragma omp parallel for schedule(dynamic)
    for (int64_t ui = 0; ui < o->n_units; ++ui) {
        unit_t *x = &o->u[ui];
        const int64_t b = ui / Hkv, h = ui % Hkv;
        if (unit_reserve(x, N + 1, D)) {
#pragma omp critical
            rc = ORACLE_ENOMEM;
            continue;
        }
        memcpy(x->K, K + ui * N * D, sizeof(double) * N * D);
        memcpy(x->V, V + ui * N * D, sizeof(double) * N * D);
        for (int64_t j = 0; j < N; ++j) { x->A[j] = init ? init[ui * N + j] : 0.0; x->pos[j] = (int32_t)j; }
        x->n = N; x->n_old = 0;
        double *p = malloc(sizeof(double) * (size_t)(N + 1));
        if (!p) {
#pragma omp critical
            rc = ORACLE_ENOMEM;
            continue;
        }
        for (int64_t t = 0; t < n_obs; ++t) {
            const int64_t i = N - n_obs + t;               /* position of this query */
            for (int64_t g = 0; g < G; ++g) {
                const double *q = q_obs + (((b * Hq) + h * G + g) * n_obs + t) * D;
                softmax_row(q, x->K, i + 1, D, scale_of(c, i + 1), p);  /* causal: keys 0..i */
                for (int64_t j = 0; j <= i; ++j) x->A[j] += p[j];
            }
        }
        free(p);
        /* Remark 2 */
        if (trigger_count_of(c, x) >= c->evict_every) {
            int r = unit_evict(c, x);
            if (r) {
#pragma omp critical
                rc = r;
            }
        }
        /* Remark 2: keep sampling until the selected tokens fit their container.  Without an explicit
         * capacity the container has T + k + w rows when T bounds old + new tokens together (the
         * remark's own figure); when T counts new tokens only, one sampling is all there is.  An
         * explicit capacity must also leave room for the T tokens buffered before the next eviction. */
        const int64_t container = c->capacity > 0 ? c->capacity - c->evict_every
                                  : (c->variant & 2) ? c->evict_every + c->sink + c->window : 0;
        while (container > 0 && x->n > container && x->n > c->sink + c->window) {
            const int64_t before = x->n;
            int r = unit_evict(c, x);
            if (r || x->n >= before) {             /* nothing left to thin (s^ = 1): it cannot fit */
#pragma omp critical
                rc = r ? r : ORACLE_ECAPACITY;
                break;
            }
        }
    }
    o->tokens_seen = N;
    return rc;
}

/*
 * One decode step (eq. 2, eq. 3 / eq. 5, score accumulation, Alg. 1 trigger).
 *   q [batch][n_q_heads][D], k_new/v_new [batch][n_kv_heads][D],
 *   out [batch][n_q_heads][D].
 */
int oracle_decode_step(oracle_t *o, const double *q, const double *k_new, const double *v_new, double *out)
{
    if (!o || !q || !k_new || !v_new || !out) return ORACLE_EINVAL;
    const oracle_config *c = &o->cfg;
    const int64_t D = c->head_dim, G = c->n_q_heads / c->n_kv_heads, Hkv = c->n_kv_heads, Hq = c->n_q_heads;
    const double scale = scale_of(c, o->tokens_seen + 1);   /* the new token counts */
    int rc = 0;
#pragma omp parallel for schedule(static)
    for (int64_t ui = 0; ui < o->n_units; ++ui) {
        unit_t *x = &o->u[ui];
        const int64_t b = ui / Hkv, h = ui % Hkv;
        if (unit_reserve(x, x->n + 1, D)) {
#pragma omp critical
            rc = ORACLE_ENOMEM;
            continue;
        }
        /* eq. 2: K <- [K, K_t], V <- [V, V_t] */
        memcpy(x->K + x->n * D, k_new + ui * D, sizeof(double) * D);
        memcpy(x->V + x->n * D, v_new + ui * D, sizeof(double) * D);
        x->A[x->n] = 0.0;
        x->pos[x->n] = (int32_t)o->tokens_seen;
        x->n += 1;
        double *p = malloc(sizeof(double) * (size_t)x->n);
        if (!p) {
#pragma omp critical
            rc = ORACLE_ENOMEM;
            continue;
        }
        for (int64_t g = 0; g < G; ++g) {
            const double *qg = q + ((b * Hq) + h * G + g) * D;
            double *og = out + ((b * Hq) + h * G + g) * D;
            softmax_row(qg, x->K, x->n, D, scale, p);            /* eq. 3: A_t */
            for (int64_t d = 0; d < D; ++d) og[d] = 0.0;
            for (int64_t j = 0; j < x->n; ++j)                    /* O_t = A_t V */
                for (int64_t d = 0; d < D; ++d) og[d] += p[j] * x->V[j * D + d];
            for (int64_t j = 0; j < x->n; ++j) x->A[j] += p[j];   /* accumulated score */
        }
        free(p);
        if (c->auto_evict && trigger_count_of(c, x) >= c->evict_every) {  /* Alg. 1: buffer T, then sample */
            int r = unit_evict(c, x);
            if (r) {
#pragma omp critical
                rc = r;
            }
        }
    }
    o->tokens_seen += 1;
    return rc;
}

int oracle_len(const oracle_t *o, int64_t *n, int64_t *n_old, int64_t *new_count)
{
    if (!o) return ORACLE_EINVAL;
    const unit_t *x = &o->u[0];
    if (n) *n = x->n;
    if (n_old) *n_old = x->n_old;
    if (new_count) *new_count = new_count_of(&o->cfg, x);
    return ORACLE_OK;
}

/* copy out the retained rows in cache order: K,V [units][n][D], A [units][n], pos [units][n]; any may be NULL */
int oracle_export(const oracle_t *o, double *K, double *V, double *A, int32_t *pos)
{
    if (!o) return ORACLE_EINVAL;
    const int64_t D = o->cfg.head_dim;
    for (int64_t ui = 0; ui < o->n_units; ++ui) {
        const unit_t *x = &o->u[ui];
        const int64_t n = x->n;
        if (K) memcpy(K + ui * n * D, x->K, sizeof(double) * n * D);
        if (V) memcpy(V + ui * n * D, x->V, sizeof(double) * n * D);
        if (A) memcpy(A + ui * n, x->A, sizeof(double) * n);
        if (pos) memcpy(pos + ui * n, x->pos, sizeof(int32_t) * n);
    }
    return ORACLE_OK;
}

/* overwrite the accumulated scores (lock-step comparison: the selection is
 * then run on exactly the array the other implementation holds) */
int oracle_set_scores(oracle_t *o, const double *A)
{
    if (!o || !A) return ORACLE_EINVAL;
    for (int64_t ui = 0; ui < o->n_units; ++ui) {
        unit_t *x = &o->u[ui];
        memcpy(x->A, A + ui * x->n, sizeof(double) * x->n);
    }
    return ORACLE_OK;
}
