"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every declared symbol,
validates arguments before touching anything, and its integer bookkeeping (Alg. 1 sizes) matches the
oracle's, using the dry-run flag that skips all kernel launches."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle.buzz_oracle import OracleCache, OracleConfig
from paper_2410_23079_amd import (FLAG_AUTO_EVICT, FLAG_DRY_RUN, BuzzCache, BuzzConfig, BuzzError, library_path,
                                  load_library, workspace_bytes)
from paper_2410_23079_amd.binding import EXPORTS

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
DRY = FLAG_AUTO_EVICT | FLAG_DRY_RUN


def cfg(**kw):
    base = dict(batch=2, n_q_heads=8, n_kv_heads=2, head_dim=128, kv_dtype="bf16", sink=4, window=64, segment=16,
                keep=2, evict_every=16, max_context=4096, old_stride=1, flags=DRY)
    base.update(kw)
    return BuzzConfig(**base)


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "buzz.h")).read()
    declared = set(re.findall(r"\b(buzz_[a-z_]+)\s*\(", header))
    assert declared == set(EXPORTS)
    lib = ctypes.CDLL(library_path())
    for name in declared:
        assert getattr(lib, name) is not None


def test_strerror_covers_all_codes():
    lib = load_library()
    texts = {lib.buzz_strerror(c).decode() for c in range(0, -6, -1)}
    assert len(texts) == 6 and "unknown status" not in texts
    assert lib.buzz_strerror(-99).decode() == "unknown status"


@pytest.mark.parametrize("bad", [
    dict(batch=0), dict(n_q_heads=7), dict(kv_dtype_code=5), dict(sink=-1), dict(window=-1), dict(segment=0),
    dict(keep=-1), dict(evict_every=0), dict(old_stride=-1), dict(max_context=0), dict(capacity=10),
    dict(flags=1024), dict(flags=512 | 32), dict(flags=512 | 128), dict(softmax_scale=float("nan")), dict(softmax_scale=-1.0),
])
def test_invalid_configurations_are_rejected(bad):
    c = cfg()
    raw = c.to_c()
    for k, v in bad.items():
        setattr(raw, "kv_dtype" if k == "kv_dtype_code" else k, v)
    out = ctypes.c_size_t()
    assert load_library().buzz_workspace_bytes(ctypes.byref(raw), ctypes.byref(out)) == -1


@pytest.mark.parametrize("bad", [dict(head_dim=96), dict(n_q_heads=18), dict(segment=(1 << 28) + 1)])
def test_unsupported_shapes_say_so(bad):
    with pytest.raises(BuzzError) as e:
        workspace_bytes(cfg(**bad))
    assert e.value.code == -5


def test_null_pointers_and_small_workspace():
    lib = load_library()
    raw = cfg(flags=FLAG_AUTO_EVICT).to_c()
    h = ctypes.c_void_p()
    assert lib.buzz_workspace_bytes(None, None) == -1
    assert lib.buzz_cache_create(ctypes.byref(raw), None, 1 << 40, ctypes.byref(h)) == -1        # no workspace
    assert lib.buzz_cache_create(ctypes.byref(raw), 0x1001, 1 << 40, ctypes.byref(h)) == -1      # misaligned
    assert lib.buzz_cache_create(ctypes.byref(raw), 0x1000, 1024, ctypes.byref(h)) == -2         # too small
    assert lib.buzz_bench_copy(None, None, 16, None) == -1
    assert lib.buzz_cache_len(None, None, None, None) == -1
    assert lib.buzz_decode_step(None, None, None, None, None, None) == -1
    assert lib.buzz_cache_destroy(None) == 0


def test_state_errors_and_argument_checks_come_before_any_launch():
    lib = load_library()
    raw = cfg(flags=FLAG_AUTO_EVICT).to_c()       # a real (non-dry) handle over a fake workspace: nothing may touch it
    h = ctypes.c_void_p()
    need = workspace_bytes(cfg(flags=FLAG_AUTO_EVICT))
    assert lib.buzz_cache_create(ctypes.byref(raw), 0x10000, need, ctypes.byref(h)) == 0
    assert lib.buzz_decode_step(h, 1, 1, 1, 1, None) == -3          # no prefill yet
    assert lib.buzz_evict(h, None) == -3
    assert lib.buzz_cache_export(h, None, None, None, None, None) == -3
    assert lib.buzz_prefill(h, None, None, 10, None, 0, None, None) == -1        # null K, V
    assert lib.buzz_prefill(h, 1, 1, 10, None, 3, None, None) == -1              # n_obs without q_obs
    assert lib.buzz_prefill(h, 1, 1, 10, 1, 11, None, None) == -1                # n_obs > n_prompt
    assert lib.buzz_prefill(h, 1, 1, 5000, None, 0, None, None) == -2            # beyond max_context
    assert lib.buzz_cache_set_splits(h, -1) == -1
    assert lib.buzz_cache_set_splits(h, 100000) == -1
    assert lib.buzz_cache_destroy(h) == 0


def test_workspace_grows_with_context_and_covers_kv():
    small, big = workspace_bytes(cfg(max_context=2048)), workspace_bytes(cfg(max_context=65536))
    assert big > small
    c = cfg(max_context=65536)
    kv_min = 2 * c.batch * c.n_kv_heads * (c.sink + c.window + c.evict_every) * c.head_dim * 2
    assert big > kv_min


@pytest.mark.parametrize("dtype,elem", [("fp32", 4), ("fp16", 2), ("bf16", 2)])
def test_workspace_size_follows_the_rows_the_cache_must_hold(dtype, elem):
    """The workspace holds K and V for every row the cache can ever retain (found by driving a dry-run cache
    to max_context), and not a multiple of that."""
    B, H, D, w, T, ctx = 2, 4, 128, 4096, 64, 12288
    c = cfg(batch=B, n_q_heads=H, n_kv_heads=H, head_dim=D, kv_dtype=dtype, window=w, evict_every=T, segment=64,
            keep=8, old_stride=1, max_context=ctx)
    g = BuzzCache(c)
    g.prefill(None, None, n_prompt=8192)
    rows = g.lengths()[0]
    for _ in range(ctx - 8192):
        g.decode_step(None, None, None, None)
        rows = max(rows, g.lengths()[0])
    per_row = 2 * D * elem + 8                               # K, V, score, position
    need = B * H * rows * per_row
    got = workspace_bytes(c)
    assert got >= need
    # side arrays (logit buffers, prompt scores, selection lists, statistics) are small next to K and V here
    assert got <= 1.3 * need + B * H * ctx * 4 + (8 << 20)


def test_a_long_cache_with_wide_groups_has_room_for_its_splits():
    """Eight query heads per kv head and 16k rows need 16 key-range splits per unit for the LDS staging of the
    logits; the workspace must have partial-result slots for them although 512 units alone would get 8."""
    c = cfg(batch=32, n_q_heads=128, n_kv_heads=16, head_dim=64, kv_dtype="bf16", sink=4, window=16000, segment=64,
            keep=8, evict_every=64, old_stride=1, max_context=16400)
    g = BuzzCache(c)
    g.prefill(None, None, n_prompt=16100)
    for _ in range(200):
        g.decode_step(None, None, None, None)               # would say BUZZ_ECAPACITY if the splits did not fit
    assert g.lengths()[0] >= 16004


def closed_form(N, steps, k, w, s, c, T, sh):
    def evict(n, n_old):
        if n <= k + w:
            return n, n_old
        new = n - k - n_old - w
        o2 = -(-n_old // sh)
        n2 = min(c, s) * (new // s) + min(c, new % s)
        return k + o2 + n2 + w, o2 + n2
    n, n_old = N, 0
    if n - k - w >= T:
        n, n_old = evict(n, n_old)
    sizes = [(n, n_old)]
    for _ in range(steps):
        n += 1
        if n - k - n_old - w >= T:
            n, n_old = evict(n, n_old)
        sizes.append((n, n_old))
    return sizes


@pytest.mark.parametrize("seed", range(10))
def test_dry_run_sizes_match_closed_form_and_oracle(seed):
    r = np.random.default_rng(seed)
    k, w = int(r.integers(0, 6)), int(r.integers(0, 50))
    s, keep = int(r.integers(1, 20)), int(r.integers(0, 5))
    T = int(r.integers(1, 40))
    old_stride = int(r.choice([0, 1, 2, 3]))
    sh = old_stride or (s + 1) // 2
    N, steps = int(r.integers(0, 400)), 150
    g = BuzzCache(cfg(sink=k, window=w, segment=s, keep=keep, evict_every=T, old_stride=old_stride,
                      max_context=N + steps))
    g.prefill(None, None, n_prompt=N)
    o = OracleCache(OracleConfig(1, 1, 1, 2, sink=k, window=w, segment=s, keep=keep, evict_every=T,
                                 old_stride=old_stride))
    o.prefill(np.zeros((1, 1, N, 2)), np.zeros((1, 1, N, 2)))
    expect = closed_form(N, steps, k, w, s, keep, T, sh)
    assert g.lengths()[:2] == expect[0] == o.lengths()[:2]
    z = np.zeros((1, 1, 2))
    for t in range(steps):
        g.decode_step(None, None, None, None)
        o.decode_step(z, z, z)
        assert g.lengths() == o.lengths()
        assert g.lengths()[:2] == expect[t + 1]
    with pytest.raises(BuzzError) as e:                       # max_context reached
        g.decode_step(None, None, None, None)
    assert e.value.code == -2


def test_dry_run_benchmark_configs_match_the_sizes_in_the_scope_table():
    from workloads import WORKLOADS
    expect = {"tiny": (96, 112), "llama7b_layer": (1412, 1476), "llama7b_full": (3844, 3876),
              "gqa8b_layer": (7684, 7716), "long131k": (23556, 23572),
              # paper parameters: 3836 prompt tokens -> ceil(3836/5) = 768 old; evictions at steps 341 (768 -> 256
              # old, 341 -> 69 new) and 1125 (325 -> 109, 784 -> 157); 411 tokens buffered at the end
              "llama7b_layer_paper": (4 + 768 + 256, 4 + 266 + 411 + 256)}
    from paper_2410_23079_amd import FLAG_THRESHOLD_TOTAL
    for name, wl in WORKLOADS.items():
        g = BuzzCache(BuzzConfig(wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.dtype, wl.sink, wl.window,
                                 wl.segment, wl.keep, wl.evict_every, wl.max_context, old_stride=wl.old_stride,
                                 flags=DRY | (FLAG_THRESHOLD_TOTAL if wl.threshold_total else 0)))
        g.prefill(None, None, n_prompt=wl.prompt)
        a = g.lengths()[0]
        for _ in range(wl.decode_steps):
            g.decode_step(None, None, None, None)
        assert (a, g.lengths()[0]) == expect[name], name


def test_explicit_capacity_and_remark2_resampling():
    # paper stride: prefill keeps halving the survivors until they fit the old capacity
    g = BuzzCache(cfg(sink=4, window=64, segment=16, keep=1, evict_every=16, old_stride=0, capacity=4 + 64 + 16 + 6,
                      max_context=2000))
    g.prefill(None, None, n_prompt=512)
    o = OracleCache(OracleConfig(1, 1, 1, 2, sink=4, window=64, segment=16, keep=1, evict_every=16, old_stride=0,
                                 capacity=4 + 64 + 16 + 6))
    o.prefill(np.zeros((1, 1, 512, 2)), np.zeros((1, 1, 512, 2)))
    assert g.lengths() == o.lengths() and g.lengths()[1] <= 6
    # persistent survivors cannot be resampled: the prefill must refuse
    g2 = BuzzCache(cfg(sink=4, window=64, segment=16, keep=1, evict_every=16, old_stride=1, capacity=4 + 64 + 16 + 6,
                       max_context=2000))
    with pytest.raises(BuzzError) as e:
        g2.prefill(None, None, n_prompt=512)
    assert e.value.code == -2


def test_boundaries_of_the_prefill_bookkeeping():
    """Literal sizes at the edges: exactly T tokens between sink and window (Alg. 1: the eviction fires when the
    count reaches T), survivors that exactly fill the capacity (Remark 2 samples again only while they do not
    fit), a prompt that exactly fills the sink, and a prompt of exactly max_context tokens."""
    k, w, s, T = 4, 10, 5, 20
    for between, want in ((T - 1, (k + w + T - 1, 0)), (T, (k + 4 + w, 4)), (T + 1, (k + 5 + w, 5))):
        g = BuzzCache(cfg(sink=k, window=w, segment=s, keep=1, evict_every=T, old_stride=1, max_context=200))
        g.prefill(None, None, n_prompt=k + w + between)
        assert g.lengths()[:2] == want, between
    # 100 tokens between sink and window, one survivor per 5 = 20 survivors
    for room, want_old in ((20, 20), (19, 10), (10, 10), (9, 5)):     # s^ = 2: 20 -> 10 -> 5
        g = BuzzCache(cfg(sink=k, window=w, segment=s, keep=1, evict_every=T, old_stride=2,
                          capacity=k + w + T + room, max_context=400))
        g.prefill(None, None, n_prompt=k + w + 100)
        assert g.lengths()[1] == want_old, room
    # every token survives (keep >= segment): the survivors are all 100 tokens and must be accepted
    g = BuzzCache(cfg(sink=k, window=w, segment=s, keep=s, evict_every=T, old_stride=1, max_context=k + w + 100))
    g.prefill(None, None, n_prompt=k + w + 100)
    assert g.lengths()[:2] == (k + w + 100, 100)
    with pytest.raises(BuzzError) as e:                        # ... and the context is full
        g.decode_step(None, None, None, None)
    assert e.value.code == -2
    # a prompt that exactly fills the sink: the next token goes to the ring, not to a fifth sink row
    g = BuzzCache(cfg(sink=k, window=w, segment=s, keep=1, evict_every=T, old_stride=1, max_context=200))
    g.prefill(None, None, n_prompt=k)
    for i in range(w + T + 3):
        g.decode_step(None, None, None, None)
    assert g.lengths()[0] == k + 4 + w + 3                     # one eviction of T = 20 tokens left 4


def test_explicit_capacity_at_its_smallest():
    """`capacity` counts sink, old rows, window and the T buffered rows: with no room for old rows it is still a
    valid cache (nothing survives an eviction), one row less is not; the H2O-style variant needs room for its
    `keep` survivors."""
    from paper_2410_23079_amd import FLAG_GLOBAL_TOPK
    k, w, T = 4, 10, 20
    g = BuzzCache(cfg(sink=k, window=w, segment=5, keep=0, evict_every=T, old_stride=1, capacity=k + w + T, max_context=300))
    g.prefill(None, None, n_prompt=100)
    assert g.lengths()[:2] == (k + w, 0)
    with pytest.raises(BuzzError) as e:
        BuzzCache(cfg(sink=k, window=w, segment=5, keep=0, evict_every=T, old_stride=1, capacity=k + w + T - 1, max_context=300))
    assert e.value.code == -1
    BuzzCache(cfg(sink=k, window=w, segment=5, keep=7, evict_every=T, capacity=k + 7 + w + T, max_context=300,
                  flags=DRY | FLAG_GLOBAL_TOPK))
    with pytest.raises(BuzzError) as e:
        BuzzCache(cfg(sink=k, window=w, segment=5, keep=7, evict_every=T, capacity=k + 7 + w + T - 1, max_context=300,
                      flags=DRY | FLAG_GLOBAL_TOPK))
    assert e.value.code == -1


def test_the_entry_point_without_allocation_keeps_the_same_books():
    a, b = BuzzCache(cfg(flags=DRY | FLAG_AUTO_EVICT)), BuzzCache(cfg(flags=DRY | FLAG_AUTO_EVICT))
    a.prefill(None, None, n_prompt=300)
    b.prefill(None, None, n_prompt=300)
    for _ in range(100):
        a.decode_step(None, None, None, None)
        b.decode_step_static(None, None, None, None)
        assert a.lengths() == b.lengths()


def test_theorem_threshold_helper():
    from paper_2410_23079_amd import suggest_threshold
    assert suggest_threshold(5, 1024) == round(1024 * 26 / 6)      # (s^2+1)/(s+1) = 4.33 for s = 5
    assert suggest_threshold(4, 1024) == 3 * 1024                  # s - 1 for even s
    assert suggest_threshold(1, 10) == 10 and suggest_threshold(0, 10) == 0 and suggest_threshold(3, 0) == 1


@pytest.mark.parametrize("seed", range(6))
def test_total_threshold_sizes_match_oracle(seed):
    from paper_2410_23079_amd import FLAG_THRESHOLD_TOTAL
    r = np.random.default_rng(50 + seed)
    k, w = int(r.integers(0, 5)), int(r.integers(1, 30))
    s, keep = int(r.integers(2, 9)), int(r.integers(1, 3))
    T = int(r.integers(20, 120))
    N, steps = int(r.integers(0, 600)), 300
    g = BuzzCache(cfg(sink=k, window=w, segment=s, keep=keep, evict_every=T, old_stride=0, max_context=N + steps,
                      flags=DRY | FLAG_THRESHOLD_TOTAL))
    o = OracleCache(OracleConfig(1, 1, 1, 2, sink=k, window=w, segment=s, keep=keep, evict_every=T, old_stride=0,
                                 threshold_total=True))
    g.prefill(None, None, n_prompt=N)
    o.prefill(np.zeros((1, 1, N, 2)), np.zeros((1, 1, N, 2)))
    assert g.lengths() == o.lengths()
    z = np.zeros((1, 1, 2))
    for _ in range(steps):
        g.decode_step(None, None, None, None)
        o.decode_step(z, z, z)
        assert g.lengths() == o.lengths()
        assert g.lengths()[1] <= T


def test_decode_step_that_cannot_evict_fails_before_it_changes_anything():
    """Alg. 1's eviction branch inside a decode step: when its survivors would not fit an explicit capacity the
    step is refused as a whole -- no token appended, sizes unchanged, and a retry fails the same way."""
    k, w, s, T = 2, 10, 4, 4
    g = BuzzCache(cfg(sink=k, window=w, segment=s, keep=1, evict_every=T, old_stride=1, capacity=k + w + T + 6,
                      max_context=1000))
    g.prefill(None, None, n_prompt=k + w)
    for _ in range(6 * T):                                     # six evictions fill the six old rows
        g.decode_step(None, None, None, None)
    assert g.lengths() == (k + 6 + w, 6, 0)
    for _ in range(T - 1):
        g.decode_step(None, None, None, None)
    before = g.lengths()
    assert before == (k + 6 + w + T - 1, 6, T - 1)
    for _ in range(2):                                         # the step that would trigger the seventh eviction
        with pytest.raises(BuzzError) as e:
            g.decode_step(None, None, None, None)
        assert e.value.code == -2
        assert g.lengths() == before


@pytest.mark.parametrize("seed", range(6))
def test_global_topk_sizes_match_oracle(seed):
    """H2O-style baseline: after every eviction the cache holds sink + min(keep, middle) + window rows."""
    from paper_2410_23079_amd import FLAG_GLOBAL_TOPK
    r = np.random.default_rng(70 + seed)
    k, w = int(r.integers(0, 5)), int(r.integers(0, 30))
    B, T = int(r.integers(1, 40)), int(r.integers(1, 25))
    N, steps = int(r.integers(0, 300)), 120
    g = BuzzCache(cfg(sink=k, window=w, segment=7, keep=B, evict_every=T, old_stride=0, max_context=N + steps,
                      flags=DRY | FLAG_GLOBAL_TOPK))
    o = OracleCache(OracleConfig(1, 1, 1, 2, sink=k, window=w, segment=7, keep=B, evict_every=T, old_stride=0,
                                 global_topk=True))
    g.prefill(None, None, n_prompt=N)
    o.prefill(np.zeros((1, 1, N, 2)), np.zeros((1, 1, N, 2)))
    assert g.lengths() == o.lengths()
    z = np.zeros((1, 1, 2))
    for _ in range(steps):
        g.decode_step(None, None, None, None)
        o.decode_step(z, z, z)
        assert g.lengths() == o.lengths()
        assert g.lengths()[1] <= B and g.lengths()[0] <= k + B + w + T


def test_segments_longer_than_a_wave_can_rank_are_accepted():
    assert workspace_bytes(cfg(segment=5000, max_context=20000)) > 0
    assert workspace_bytes(cfg(n_q_heads=2, segment=200000, keep=64, evict_every=200000, max_context=500000)) > 0


def test_import_restores_the_bookkeeping():
    """Checkpoint / resume: a cache loaded with another cache's sizes continues with the same sizes (Alg. 1)."""
    a = BuzzCache(cfg(max_context=3000))
    a.prefill(None, None, n_prompt=700)
    for _ in range(45):
        a.decode_step(None, None, None, None)
    n, n_old, new = a.lengths()
    b = BuzzCache(cfg(max_context=3000))
    b.import_rows(None, None, None, None, n_old=n_old, tokens_seen=745, n=n)
    assert b.lengths() == a.lengths()
    for _ in range(200):
        a.decode_step(None, None, None, None)
        b.decode_step(None, None, None, None)
        assert a.lengths() == b.lengths()
    lib = load_library()
    h = b._h
    assert lib.buzz_cache_import(h, None, None, None, None, 10, 11, 20, None) == -1      # n_old > n
    assert lib.buzz_cache_import(h, None, None, None, None, 10, 0, 5, None) == -1        # fewer tokens seen than rows
    assert lib.buzz_cache_import(h, None, None, None, None, 6, 3, 6, None) == -1         # old rows without a full sink
    assert lib.buzz_cache_import(h, None, None, None, None, 10, 0, 5000, None) == -2     # beyond max_context
    assert lib.buzz_cache_import(h, None, None, None, None, 2500, 0, 2500, None) == -2   # more buffered rows than the ring holds
    # the edges themselves are inside: as many tokens as max_context, a ring exactly full (window 64 + T 16 rows)
    assert lib.buzz_cache_import(h, None, None, None, None, 10, 0, 3000, None) == 0
    assert lib.buzz_cache_import(h, None, None, None, None, 4 + 80, 0, 100, None) == 0
    assert b.lengths() == (84, 0, 16)
    assert lib.buzz_cache_import(h, None, None, None, None, 4 + 81, 0, 100, None) == -2
    assert b.lengths() == (84, 0, 16)                                                    # the failed call changed nothing


def test_a_prompt_shorter_than_the_sink_fills_the_sink_first():
    """Remark 1: the first tokens go to the sink; the counts grow by one per token either way."""
    g = BuzzCache(cfg(sink=4, window=10, segment=5, keep=1, evict_every=20, old_stride=1, max_context=100))
    g.prefill(None, None, n_prompt=2)
    seen = []
    for _ in range(40):
        g.decode_step(None, None, None, None)
        seen.append(g.lengths())
    assert seen[0] == (3, 0, 0) and seen[1] == (4, 0, 0) and seen[11] == (14, 0, 0) and seen[12] == (15, 0, 1)
    assert seen[31] == (4 + 4 + 10, 4, 0)                   # 34 tokens: 20 between sink and window -> 4 survivors
