// Host sanitizer driver for the C ABI (test infrastructure): drives the library's host code -- validation, layout,
// the integer bookkeeping of Alg. 1 -- through dry-run caches (no kernel is launched, no GPU is needed), with
// buzz_api.cpp compiled under AddressSanitizer and UBSan.  Built and run by tests/test_host_sanitizers.py.
#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include "buzz.h"

static int fail(const char* what, long a, long b)
{
    fprintf(stderr, "sanitize_abi: %s (%ld vs %ld)\n", what, a, b);
    return 1;
}

static buzz_config_t config(int sink, int window, int segment, int keep, int T, int old_stride, uint32_t flags,
                            int64_t max_context, int64_t capacity)
{
    buzz_config_t c;
    memset(&c, 0, sizeof(c));
    c.batch = 2; c.n_q_heads = 8; c.n_kv_heads = 2; c.head_dim = 128; c.kv_dtype = BUZZ_BF16;
    c.sink = sink; c.window = window; c.segment = segment; c.keep = keep; c.evict_every = T; c.old_stride = old_stride;
    c.flags = flags | BUZZ_FLAG_DRY_RUN; c.max_context = max_context; c.capacity = capacity;
    return c;
}

// sizes by the closed form of Alg. 1 (every segment yields min(keep, len) rows)
static void closed_form_step(int64_t& n, int64_t& n_old, int k, int w, int s, int c, int T, int sh, bool append)
{
    if (append) n += 1;
    const int64_t newc = n - k - n_old - w;
    if (newc < T || n <= k + w) return;
    const int64_t old2 = (n_old + sh - 1) / sh;
    const int64_t cc = c < s ? c : s;
    const int64_t new2 = cc * (newc / s) + (newc % s < cc ? newc % s : cc);
    n_old = old2 + new2;
    n = k + n_old + w;
}

static int drive(int k, int w, int s, int c, int T, int old_stride, int64_t N, int steps)
{
    buzz_config_t cfg = config(k, w, s, c, T, old_stride, BUZZ_FLAG_AUTO_EVICT, N + steps, 0);
    size_t bytes = 0;
    if (buzz_workspace_bytes(&cfg, &bytes) != BUZZ_OK || bytes == 0) return fail("workspace_bytes", 0, 0);
    buzz_cache_t* h = nullptr;
    if (buzz_cache_create(&cfg, nullptr, 0, &h) != BUZZ_OK) return fail("create", 0, 0);
    if (buzz_decode_step(h, nullptr, nullptr, nullptr, nullptr, nullptr) != BUZZ_ESTATE) return fail("decode before prefill", 0, 0);
    if (buzz_prefill(h, nullptr, nullptr, N, nullptr, 0, nullptr, nullptr) != BUZZ_OK) return fail("prefill", 0, 0);
    const int sh = old_stride ? old_stride : (s + 1) / 2;
    int64_t n = N, n_old = 0;
    closed_form_step(n, n_old, k, w, s, c, T, sh, false);
    for (int t = 0; t <= steps; ++t) {
        int64_t gn, go, gnew;
        if (buzz_cache_len(h, &gn, &go, &gnew) != BUZZ_OK) return fail("len", 0, 0);
        if (gn != n || go != n_old) return fail("sizes differ from the closed form", (long)gn, (long)n);
        if (t == steps) break;
        if (buzz_decode_step(h, nullptr, nullptr, nullptr, nullptr, nullptr) != BUZZ_OK) return fail("decode", t, 0);
        closed_form_step(n, n_old, k, w, s, c, T, sh, true);
    }
    if (buzz_decode_step(h, nullptr, nullptr, nullptr, nullptr, nullptr) != BUZZ_ECAPACITY) return fail("max_context", 0, 0);
    if (buzz_evict(h, nullptr) != BUZZ_OK) return fail("evict", 0, 0);
    if (buzz_cache_export(h, nullptr, nullptr, nullptr, nullptr, nullptr) != BUZZ_OK) return fail("export (dry)", 0, 0);
    if (buzz_cache_set_splits(h, 1 << 20) != BUZZ_EINVAL) return fail("set_splits", 0, 0);
    if (buzz_cache_destroy(h) != BUZZ_OK) return fail("destroy", 0, 0);
    return 0;
}

int main()
{
    int rc = 0;
    rc |= drive(4, 64, 16, 1, 16, 1, 512, 300);
    rc |= drive(4, 64, 16, 2, 16, 0, 512, 300);
    rc |= drive(0, 0, 5, 1, 5, 1, 150, 80);
    rc |= drive(2, 20, 3, 9, 1, 1, 100, 60);
    rc |= drive(4, 32, 8, 0, 8, 1, 2, 120);
    rc |= drive(4, 8192, 128, 16, 128, 1, 131072, 300);
    // validation paths
    size_t bytes;
    buzz_config_t bad = config(4, 64, 16, 1, 16, 1, 0, 1000, 0);
    bad.n_q_heads = 7;
    if (buzz_workspace_bytes(&bad, &bytes) != BUZZ_EINVAL) rc |= fail("bad heads accepted", 0, 0);
    bad = config(4, 64, 16, 1, 16, 1, 0, 1000, 0);
    bad.head_dim = 96;
    if (buzz_workspace_bytes(&bad, &bytes) != BUZZ_EUNSUPPORTED) rc |= fail("head_dim without a kernel accepted", 0, 0);
    rc |= drive(4, 64, 5000, 3, 6000, 1, 12000, 40);           // a segment beyond one wave's reach, ragged
    // an eviction that cannot fit an explicit capacity is refused before the step changes anything
    buzz_config_t tight = config(2, 10, 4, 1, 4, 1, BUZZ_FLAG_AUTO_EVICT, 1000, 2 + 10 + 4 + 6);
    buzz_cache_t* h = nullptr;
    if (buzz_cache_create(&tight, nullptr, 0, &h) != BUZZ_OK) return fail("create tight", 0, 0);
    buzz_prefill(h, nullptr, nullptr, 12, nullptr, 0, nullptr, nullptr);
    int status = BUZZ_OK, steps = 0;
    while ((status = buzz_decode_step(h, nullptr, nullptr, nullptr, nullptr, nullptr)) == BUZZ_OK && steps < 100) ++steps;
    int64_t n, n_old, nc;
    buzz_cache_len(h, &n, &n_old, &nc);
    if (status != BUZZ_ECAPACITY || steps != 27 || n != 21 || n_old != 6 || nc != 3) rc |= fail("tight capacity", steps, (long)n);
    buzz_cache_destroy(h);
    if (buzz_suggest_threshold(5, 1024) != 4437) rc |= fail("suggest_threshold", (long)buzz_suggest_threshold(5, 1024), 4437);
    if (!rc) printf("sanitize_abi ok\n");
    return rc;
}
