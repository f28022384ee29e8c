/*
 * Host sanitizer driver for the CPU oracle (test infrastructure): includes the oracle's source and drives every
 * entry point -- prefill with observed queries, decode steps with automatic evictions, Remark 2's repeated
 * sampling, manual eviction, score override, export -- under AddressSanitizer and UBSan.
 * Built and run by tests/test_host_sanitizers.py; exits 0 when everything ran and the sizes are the expected ones.
 */
#include "../oracle/buzz_oracle.c"
#include <stdio.h>

static double rnd(uint64_t *s)
{
    *s = *s * 6364136223846793005ull + 1442695040888963407ull;
    return (double)((*s >> 33) & 0xffffff) / (double)0x1000000 - 0.5;
}

static int run(int variant, int old_stride, int64_t capacity, int keep, int64_t N, int steps)
{
    oracle_config c = {.batch = 2, .n_q_heads = 4, .n_kv_heads = 2, .head_dim = 8, .sink = 3, .window = 9, .segment = 5,
                       .keep = keep, .evict_every = 7, .old_stride = old_stride, .auto_evict = 1, .variant = variant,
                       .capacity = capacity, .softmax_scale = 0.0};
    oracle_t *o = NULL;
    if (oracle_create(&c, &o)) return 1;
    const int64_t units = 4, D = 8, n_obs = N < 6 ? N : 6;
    uint64_t seed = 12345 + (uint64_t)variant * 77 + (uint64_t)N;
    double *K = malloc(sizeof(double) * (size_t)(units * N * D + 1)), *V = malloc(sizeof(double) * (size_t)(units * N * D + 1));
    double *q = malloc(sizeof(double) * (size_t)(2 * 4 * n_obs * D + 1)), *init = malloc(sizeof(double) * (size_t)(units * N + 1));
    for (int64_t i = 0; i < units * N * D; ++i) { K[i] = rnd(&seed); V[i] = rnd(&seed); }
    for (int64_t i = 0; i < 2 * 4 * n_obs * D; ++i) q[i] = rnd(&seed);
    for (int64_t i = 0; i < units * N; ++i) init[i] = (i % 11 == 0) ? NAN : (double)(i % 3);
    int rc = oracle_prefill(o, K, V, N, n_obs ? q : NULL, n_obs, init);
    if (rc) { fprintf(stderr, "prefill rc %d\n", rc); return 2; }
    double qs[4 * 2 * 8], ks[2 * 2 * 8], vs[2 * 2 * 8], out[4 * 2 * 8];
    for (int t = 0; t < steps; ++t) {
        for (int i = 0; i < 64; ++i) qs[i] = rnd(&seed);
        for (int i = 0; i < 32; ++i) { ks[i] = rnd(&seed); vs[i] = rnd(&seed); }
        if (oracle_decode_step(o, qs, ks, vs, out)) return 3;
        for (int i = 0; i < 64; ++i) if (!(out[i] > -1.0 && out[i] < 1.0)) return 4;   /* convex combination of V */
    }
    if (oracle_evict(o)) return 5;
    int64_t n, n_old, nc;
    oracle_len(o, &n, &n_old, &nc);
    double *Ko = malloc(sizeof(double) * (size_t)(units * n * D + 1)), *Vo = malloc(sizeof(double) * (size_t)(units * n * D + 1));
    double *A = malloc(sizeof(double) * (size_t)(units * n + 1));
    int32_t *pos = malloc(sizeof(int32_t) * (size_t)(units * n + 1));
    if (oracle_export(o, Ko, Vo, A, pos)) return 6;
    for (int64_t u = 0; u < units; ++u)
        for (int64_t j = 1; j < n; ++j) if (pos[u * n + j] <= pos[u * n + j - 1]) return 7;   /* positional order */
    for (int64_t i = 0; i < units * n; ++i) A[i] = (double)(i % 5);
    if (oracle_set_scores(o, A)) return 8;
    if (oracle_evict(o)) return 9;
    printf("variant %d stride %d capacity %lld keep %d N %lld: n %lld n_old %lld\n", variant, old_stride,
           (long long)capacity, keep, (long long)N, (long long)n, (long long)n_old);
    free(K); free(V); free(q); free(init); free(Ko); free(Vo); free(A); free(pos);
    oracle_destroy(o);
    return 0;
}

int main(void)
{
    int rc = 0;
    rc |= run(0, 1, 0, 1, 200, 40);      /* persistent survivors */
    rc |= run(0, 0, 0, 2, 150, 30);      /* the paper's old stride */
    rc |= run(0, 0, 3 + 9 + 7 + 4, 1, 300, 25);   /* Remark 2 with an explicit capacity */
    rc |= run(2, 0, 0, 1, 300, 25);      /* T bounds old + new */
    rc |= run(1 | 4, 1, 0, 1, 64, 20);   /* log-n scale, interval sampling of new tokens */
    rc |= run(0, 1, 0, 0, 50, 20);       /* keep 0 */
    rc |= run(0, 1, 0, 3, 0, 30);        /* empty prompt */
    rc |= run(0, 1, 0, 9, 5, 30);        /* prompt shorter than sink + window, keep above the segment */
    return rc;
}
