"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle in lock-step.

Bars (written out in tests/lockstep.py): retained positions, K rows and V rows bit-exact; attention
outputs within 2e-3 max relative error per head vector (and within 1e-4, what fp32 accumulation gives);
accumulated scores within 1e-4.
"""
import numpy as np
import pytest
import torch

from workloads import decode_inputs, get_workload, prompt_inputs

pytestmark = pytest.mark.gpu


def lockstep():
    from tests import lockstep as ls
    return ls


def small(name="tiny", **kw):
    return get_workload(name).scaled(**kw)


def run(wl, device="cuda", **kw):
    p = prompt_inputs(wl, device=device)
    d = decode_inputs(wl, device=device)
    print(f"[parity] {wl.name} B{wl.batch} Hq{wl.n_q_heads} Hkv{wl.n_kv_heads} D{wl.head_dim} {wl.dtype} "
          f"N{wl.prompt} steps{wl.decode_steps} k{wl.sink} w{wl.window} s{wl.segment} c{wl.keep} "
          f"T{wl.evict_every} sh{wl.old_stride} {kw}", flush=True)
    st = lockstep().run_lockstep(wl, p, d, **kw)
    print(f"[parity]   worst out {st['out']:.2e} score {st['score']:.2e} prefill-score {st['prefill_score']:.2e} "
          f"evictions {st['evictions']}", flush=True)
    return st


# ------------------------------------------------------------------ config 1 in full
def test_tiny_full():
    st = run(get_workload("tiny"))
    assert st["evictions"] == 256 // 16


def test_tiny_full_default_mode():
    """Without FLAG_DETERMINISTIC the waves claim tiles dynamically: same bars against the oracle."""
    st = run(get_workload("tiny"), deterministic=False)
    assert st["evictions"] == 256 // 16


def test_tiny_paper_old_stride():
    """The paper's default s^ = floor((s+1)/2): old survivors are interval-sampled at every eviction."""
    st = run(small(old_stride=0))
    assert st["evictions"] == 16


def test_tiny_paper_old_stride_with_capacity():
    """Remark 2: with an explicit capacity the prefill keeps sampling until the rows fit."""
    wl = small(old_stride=0, prompt=512, decode_steps=40)
    run(wl, capacity=wl.sink + wl.window + wl.evict_every + 6)


# ------------------------------------------------------------------ shapes, dtypes, group sizes, ragged everything
@pytest.mark.parametrize("dtype", ["fp32", "fp16", "bf16"])
@pytest.mark.parametrize("D", [64, 128, 256])
@pytest.mark.parametrize("G", [1, 2, 3, 4, 5, 6, 7, 8])
def test_shapes(dtype, D, G):
    wl = small(batch=2, n_kv_heads=2, n_q_heads=2 * G, head_dim=D, dtype=dtype, prompt=300, decode_steps=45,
               sink=3, window=40, segment=7, keep=2, evict_every=10, n_obs=9)
    run(wl)


@pytest.mark.parametrize("deterministic", [True, False])
@pytest.mark.parametrize("G", [2, 8])
def test_group_sizes(G, deterministic):
    wl = small(batch=1, n_kv_heads=3, n_q_heads=3 * G, head_dim=128, dtype="bf16", prompt=700, decode_steps=40,
               sink=4, window=64, segment=16, keep=3, evict_every=16, n_obs=40)
    run(wl, deterministic=deterministic)


@pytest.mark.parametrize("dtype", ["fp32", "fp16"])
def test_single_block_units_default_mode(dtype):
    """One split per unit, many tiles per wave, tiles claimed dynamically."""
    wl = small(batch=1, n_kv_heads=4, n_q_heads=4, head_dim=128, dtype=dtype, prompt=3000, decode_steps=24,
               sink=4, window=1500, segment=16, keep=4, evict_every=8, n_obs=16)
    run(wl, splits=1, deterministic=False)


@pytest.mark.parametrize("kv_loads", ["streaming", "cached"])
@pytest.mark.parametrize("G,dtype", [(1, "fp16"), (4, "bf16"), (2, "fp32")])
def test_forced_kv_load_flavour(G, dtype, kv_loads):
    """Both load flavours of every kernel family, whatever the working-set size would have chosen."""
    wl = small(batch=1, n_kv_heads=3, n_q_heads=3 * G, head_dim=128, dtype=dtype, prompt=1300, decode_steps=24,
               sink=4, window=128, segment=16, keep=2, evict_every=16, n_obs=12)
    run(wl, kv_loads=kv_loads)


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_widest_rows_and_groups(dtype):
    """head_dim 256 with 8 query heads per kv head: the largest per-block footprint the kernels support."""
    wl = small(batch=1, n_kv_heads=2, n_q_heads=16, head_dim=256, dtype=dtype, prompt=900, decode_steps=36,
               sink=4, window=128, segment=16, keep=2, evict_every=16, n_obs=12)
    run(wl)


@pytest.mark.parametrize("splits", [1, 2, 5, 16])
def test_split_counts(splits):
    wl = small(batch=1, n_kv_heads=2, n_q_heads=2, head_dim=128, dtype="fp16", prompt=2000, decode_steps=20,
               sink=4, window=900, segment=16, keep=4, evict_every=8, n_obs=16)
    run(wl, splits=splits, check_auto=False)


@pytest.mark.parametrize("device_merge", [False, True])
@pytest.mark.parametrize("G,dtype,heads", [(1, "fp16", 8), (4, "bf16", 8), (2, "fp32", 16), (8, "bf16", 8)])
def test_split_merge_through_one_die_or_device_memory(G, dtype, heads, device_merge):
    """Units that divide evenly over the 8 dies with several splits each: by default a unit's blocks share a
    die and merge through its L2 (eq. 3 / eq. 5 split softmax); with the flag they merge through device memory."""
    wl = small(batch=1, n_kv_heads=heads, n_q_heads=heads * G, head_dim=128, dtype=dtype, prompt=2600, decode_steps=36,
               sink=4, window=1100, segment=16, keep=3, evict_every=16, n_obs=24)
    run(wl, device_merge=device_merge, deterministic=False)


@pytest.mark.parametrize("G,dtype,old_stride", [(1, "fp32", 1), (4, "bf16", 1), (1, "fp16", 0)])
def test_export_then_import_resumes_the_cache(G, dtype, old_stride):
    """Checkpoint / resume: rows exported from a running cache and imported into a fresh one give the same
    attention outputs (same rows, other places in the ring: sums within rounding), the same evictions and the
    same final rows."""
    from paper_2410_23079_amd import FLAG_AUTO_EVICT, FLAG_DETERMINISTIC, BuzzCache
    ls = lockstep()
    wl = small(batch=2, n_kv_heads=2, n_q_heads=2 * G, head_dim=128, dtype=dtype, prompt=900, decode_steps=90,
               sink=4, window=100, segment=16, keep=2, evict_every=16, old_stride=old_stride, n_obs=24)
    p, d = prompt_inputs(wl, device="cuda"), decode_inputs(wl, device="cuda")
    a, b = (BuzzCache(ls.buzz_config(wl, flags=FLAG_AUTO_EVICT | FLAG_DETERMINISTIC)) for _ in range(2))
    a.prefill(p["K"], p["V"], q_obs=p["q_obs"])
    out_a, out_b = (torch.empty(wl.batch, wl.n_q_heads, wl.head_dim, dtype=torch.float32, device="cuda") for _ in range(2))
    first = 37                                                  # mid-cycle: buffered rows, ring head moved twice
    for t in range(first):
        a.decode_step(d["q"][t], d["k"][t], d["v"][t], out_a)
    K, V, S, P = a.export()
    n, n_old, _ = a.lengths()
    b.import_rows(K, V, S, P, n_old=n_old, tokens_seen=wl.prompt + first)
    assert a.lengths() == b.lengths()
    for t in range(first, wl.decode_steps):
        a.decode_step(d["q"][t], d["k"][t], d["v"][t], out_a)
        b.decode_step(d["q"][t], d["k"][t], d["v"][t], out_b)
        e = ls.rel_err(out_b.double().cpu().numpy(), out_a.double().cpu().numpy())
        assert e <= ls.REPRO_TOL, f"step {t}: resumed cache differs by {e}"
        assert a.lengths() == b.lengths()
    for i, (x, y) in enumerate(zip(a.export(), b.export())):
        if i == 2:
            assert torch.allclose(x, y, rtol=ls.REPRO_TOL, atol=ls.REPRO_TOL)
        else:
            assert torch.equal(x, y)


def test_die_local_merge_refuses_blocks_on_an_unexpected_die():
    """The guard of the die-local merge, forced from the host: with a wrong record of which die serves which
    launch-order number every block reports a mismatch and the outputs of the step are NaN, not numbers; the
    kernels run to their end, and with the probe's record restored the cache goes on as if nothing had happened
    (the stored rows and scores never depended on the merge)."""
    from paper_2410_23079_amd import FLAG_AUTO_EVICT, FLAG_DETERMINISTIC, BuzzCache
    ls = lockstep()
    wl = small(batch=1, n_kv_heads=8, n_q_heads=32, head_dim=128, dtype="bf16", prompt=2600, decode_steps=12,
               sink=4, window=1100, segment=16, keep=3, evict_every=16, n_obs=24)
    p, d = prompt_inputs(wl, device="cuda"), decode_inputs(wl, device="cuda")
    a, b = (BuzzCache(ls.buzz_config(wl, flags=FLAG_AUTO_EVICT | FLAG_DETERMINISTIC)) for _ in range(2))
    for c in (a, b):
        c.prefill(p["K"], p["V"], q_obs=p["q_obs"])
    out_a, out_b = (torch.empty(wl.batch, wl.n_q_heads, wl.head_dim, dtype=torch.float32, device="cuda") for _ in range(2))
    for t in range(wl.decode_steps):
        wrong = t in (3, 4)
        b.override_die_map(0x88888888 if wrong else -1)          # die 8 does not exist: no block can match
        a.decode_step(d["q"][t], d["k"][t], d["v"][t], out_a)
        b.decode_step(d["q"][t], d["k"][t], d["v"][t], out_b)
        if wrong:
            assert torch.isnan(out_b).all() and torch.isfinite(out_a).all()
        else:
            assert torch.equal(out_a, out_b)
    for x, y in zip(a.export(), b.export()):
        assert torch.equal(x, y)


@pytest.mark.parametrize("deterministic", [True, False])
@pytest.mark.parametrize("G,dtype", [(1, "bf16"), (4, "fp16"), (2, "fp32")])
def test_more_units_than_compute_units(deterministic, G, dtype):
    """360 units on 256 compute units: one 4-wave block per unit, several blocks per compute unit."""
    wl = small(batch=45, n_kv_heads=8, n_q_heads=8 * G, head_dim=64, dtype=dtype, prompt=300, decode_steps=40,
               sink=2, window=150, segment=8, keep=2, evict_every=8, n_obs=4)
    st = run(wl, units=[(0, 0), (17, 3), (31, 7), (44, 5), (44, 7)], deterministic=deterministic)
    assert st["evictions"] == 5


@pytest.mark.parametrize("dtype,G", [("bf16", 1), ("fp16", 2)])
def test_prefill_scores_from_every_prompt_query(dtype, G):
    """n_obs = N (H2O-style prompt scores) beyond one scoring pass of 4096 queries, ragged tiles everywhere."""
    wl = small(batch=1, n_kv_heads=2, n_q_heads=2 * G, head_dim=64, dtype=dtype, prompt=4500, decode_steps=8,
               sink=4, window=700, segment=32, keep=3, evict_every=8, n_obs=4500)
    run(wl, units=[(0, 1)])


@pytest.mark.parametrize("dtype", ["fp16", "bf16"])
def test_prefill_scores_from_every_prompt_query_wide_rows(dtype):
    """head_dim 256 takes the matrix-core scoring with 32-row chunks; several chunks, blocks and a ragged end."""
    wl = small(batch=1, n_kv_heads=2, n_q_heads=4, head_dim=256, dtype=dtype, prompt=1130, decode_steps=4,
               sink=4, window=200, segment=16, keep=2, evict_every=8, n_obs=1130)
    run(wl, units=[(0, 1)])


@pytest.mark.parametrize("G", [1, 2])
def test_prefill_scores_when_logits_jump(G):
    """Key rows of growing norm late in the prompt: the scaled logits of one query jump by ~20, then by far more
    than 2^7 in log2 units, so a softmax sum taken against an earlier reference overflows single precision and
    the matrix-core scoring has to move its reference (both when the sum grows large and when it is infinite)."""
    wl = small(batch=1, n_kv_heads=2, n_q_heads=2 * G, head_dim=128, dtype="fp16", prompt=900, decode_steps=6,
               sink=4, window=64, segment=16, keep=2, evict_every=8, n_obs=900)
    p = prompt_inputs(wl, device="cuda")
    d = decode_inputs(wl, device="cuda")
    K = p["K"].float()
    K[:, :, 300:304] *= 20.0
    K[:, :, 520:523] *= 60.0
    K[:, 1, 700:702] *= 200.0
    p["K"] = K.to(p["K"].dtype)
    st = lockstep().run_lockstep(wl, p, d)
    print(f"[parity]   jumping logits G{G}: prefill-score {st['prefill_score']:.2e} out {st['out']:.2e}", flush=True)


@pytest.mark.parametrize("seed", range(48))
def test_random_configurations(seed):
    """Seeded random shapes, cache parameters and variants through the whole lock-step protocol."""
    r = np.random.default_rng(9000 + seed)
    dtype = ["fp32", "fp16", "bf16"][seed % 3]
    D = int(r.choice([64, 128, 256]))
    G = int(r.choice([1, 1, 2, 3, 4, 8]))
    Hkv = int(r.choice([1, 2, 3, 8]))
    B = int(r.choice([1, 2]))
    k, w = int(r.integers(0, 6)), int(r.integers(0, 200))
    s = int(r.integers(1, 40))
    c = int(r.integers(0, 5))
    T = int(r.integers(1, 40))
    old_stride = int(r.choice([1, 1, 0, 2, 3]))
    N = int(r.integers(0, 1500))
    steps = int(r.integers(T + 1, 3 * T + 30))
    variant = seed % 4
    kw = {}
    if variant == 1:
        kw["log_n"] = True
    elif variant == 2 and c > 0:
        kw["global_topk"] = True
        c = int(r.integers(1, 60))
    elif variant == 3:
        kw["interval_new"] = True
    wl = small(batch=B, n_kv_heads=Hkv, n_q_heads=Hkv * G, head_dim=D, dtype=dtype, prompt=N, decode_steps=steps,
               sink=k, window=w, segment=s, keep=c, evict_every=T, old_stride=old_stride, n_obs=min(N, int(r.integers(0, 40))))
    run(wl, deterministic=bool(seed % 2), device_merge=bool((seed // 2) % 2), **kw)


@pytest.mark.parametrize("seed", range(10))
def test_random_long_configurations(seed):
    """The same with long prompts, windows and segments and large keep (several blocks per unit, long segments)."""
    r = np.random.default_rng(770000 + seed)
    dtype = ["fp32", "fp16", "bf16"][seed % 3]
    D = int(r.choice([64, 128, 128, 256]))
    G = int(r.choice([1, 1, 2, 4, 5, 8]))
    Hkv = int(r.choice([1, 2, 4, 8]))
    B = int(r.choice([1, 2, 4]))
    k, w = int(r.integers(0, 9)), int(r.integers(0, 5000))
    s = int(r.integers(1, 300))
    c = int(r.integers(0, 40))
    T = int(r.integers(1, 300))
    old_stride = int(r.choice([1, 1, 1, 0, 2, 5]))
    N = int(r.integers(0, 24000))
    steps = int(min(400, r.integers(T + 1, 2 * T + 40)))
    variant = seed % 5
    kw = {}
    if variant == 1:
        kw["log_n"] = True
    elif variant == 2 and c > 0:
        kw["global_topk"] = True
        c = int(r.integers(1, 600))
    elif variant == 3:
        kw["interval_new"] = True
    wl = small(batch=B, n_kv_heads=Hkv, n_q_heads=Hkv * G, head_dim=D, dtype=dtype, prompt=N, decode_steps=steps,
               sink=k, window=w, segment=s, keep=c, evict_every=T, old_stride=old_stride, n_obs=min(N, int(r.integers(0, 48))))
    run(wl, deterministic=bool(seed % 2), device_merge=bool((seed // 2) % 2), **kw)


@pytest.mark.parametrize("seed", range(10))
def test_random_prompt_scoring(seed):
    """Prompt scores from all or a random number of prompt queries, both scoring paths, random shapes."""
    r = np.random.default_rng(880000 + seed)
    dtype = ["fp16", "bf16", "fp16", "bf16", "fp32"][seed % 5]
    D = int(r.choice([64, 128, 128, 256]))
    G = int(r.choice([1, 2, 4, 8]))
    Hkv = int(r.choice([1, 2, 3]))
    B = int(r.choice([1, 2]))
    N = int(r.integers(1, 1200 if dtype == "fp32" else 5200))
    n_obs = N if seed % 2 == 0 else int(r.integers(0, N + 1))
    k, w = int(r.integers(0, 6)), int(r.integers(0, 600))
    s, c, T = int(r.integers(1, 80)), int(r.integers(0, 6)), int(r.integers(1, 100))
    kw = {"log_n": True} if seed % 3 == 0 else {}
    wl = small(batch=B, n_kv_heads=Hkv, n_q_heads=Hkv * G, head_dim=D, dtype=dtype, prompt=N, decode_steps=3,
               sink=k, window=w, segment=s, keep=c, evict_every=T, old_stride=1, n_obs=n_obs)
    run(wl, **kw)


# ------------------------------------------------------------------ degenerate cases of the method
def test_keep_zero_streaming():
    run(small(prompt=200, decode_steps=40, keep=0, n_obs=8))


def test_keep_covers_segment():
    run(small(prompt=200, decode_steps=40, segment=4, keep=4, evict_every=8, n_obs=8))


def test_no_sink_no_window():
    run(small(prompt=150, decode_steps=30, sink=0, window=0, segment=5, keep=1, evict_every=5, n_obs=8))


def test_prompt_shorter_than_sink_and_window_fill():
    """Remark 1: sink and window fill first; the first eviction happens only after T tokens left the window."""
    run(small(prompt=2, decode_steps=120, sink=4, window=32, segment=8, keep=1, evict_every=8, n_obs=2))


def test_empty_prompt():
    run(small(prompt=0, decode_steps=60, sink=2, window=16, segment=4, keep=1, evict_every=4, n_obs=0))


@pytest.mark.parametrize("keep", [5, 150])
def test_segment_longer_than_wave(keep):
    run(small(prompt=1500, decode_steps=10, sink=4, window=64, segment=200, keep=keep, evict_every=300, n_obs=16))


def test_longest_segment_one_wave_ranks():
    """segment = 4096 (the most one wave ranks): two full segments and a ragged one at prefill, ties broken by index."""
    run(small(prompt=9000, decode_steps=6, sink=4, window=64, segment=4096, keep=9, evict_every=5000, n_obs=16))


def test_keep_larger_than_segment_keeps_everything():
    """A segment cannot yield more rows than it has: keep = 9 on segments of 4 behaves like keep = 4."""
    st = run(small(prompt=200, decode_steps=40, segment=4, keep=9, evict_every=8, n_obs=8))
    assert st["evictions"] == 5


@pytest.mark.parametrize("between", [15, 16, 17])
def test_prompt_with_exactly_T_tokens_between_sink_and_window(between):
    """Alg. 1's first loops: a prompt is sampled as soon as T (= 16) tokens lie between sink and window, not one
    earlier, and a 17th starts a ragged second segment."""
    wl = small(prompt=4 + between + 64, decode_steps=20, n_obs=8)            # k 4, w 64, s 16, T 16
    from paper_2410_23079_amd import BuzzCache
    g = BuzzCache(lockstep().buzz_config(wl, flags=2))                       # dry run: sizes only
    g.prefill(None, None, n_prompt=wl.prompt)
    assert g.lengths() == {15: (83, 0, 15), 16: (69, 1, 0), 17: (70, 2, 0)}[between]
    run(wl)


def plant_odd_scores(ps):
    """NaN, +inf and -inf among the starting scores, several per segment, on every unit."""
    N = ps.shape[-1]
    for j in range(5, N, 7):
        ps[..., j] = float("nan")
    for j in range(9, N, 23):
        ps[..., j] = float("inf")
    for j in range(12, N, 11):
        ps[..., j] = float("-inf")
    ps[..., 40:56] = float("nan")                            # one whole segment of NaN: the lowest indices win


@pytest.mark.parametrize("keep,old_stride", [(1, 1), (3, 1), (2, 0)])
def test_nan_and_infinite_scores_rank_as_stated(keep, old_stride):
    """Alg. 2's argmax on scores that are not numbers: NaN ranks below everything (ties with -inf), +inf above,
    ties go to the lowest index -- at the prefill (separate selection kernel) and in decode evictions (one-launch
    eviction for persistent survivors, selection + gather where old rows are re-sampled)."""
    wl = small(prompt=600, decode_steps=50, sink=4, window=64, segment=16, keep=keep, evict_every=16,
               old_stride=old_stride, n_obs=12)
    st = run(wl, plant=plant_odd_scores)
    assert st["evictions"] == 3


@pytest.mark.parametrize("segment,keep", [(5000, 7), (9000, 300)])
def test_segments_longer_than_one_wave_can_rank(segment, keep):
    """Segments beyond 4096 rows take the block-wide selection (radix select + prefix sum): two full segments and a
    ragged one at prefill, ties everywhere (prompt scores of a short observation window are mostly equal)."""
    run(small(prompt=2 * segment + 1500, decode_steps=4, sink=4, window=64, segment=segment, keep=keep,
              evict_every=segment + 1000, n_obs=16))


def test_long_segments_with_nan_and_infinite_scores():
    st = run(small(prompt=11000, decode_steps=4, sink=4, window=64, segment=5000, keep=40, evict_every=6000, n_obs=12),
             plant=plant_odd_scores)
    assert st["evictions"] == 0                                  # everything happens in the prefill's selection


@pytest.mark.parametrize("prompt,keep,G,dtype", [(700, 40, 1, "fp32"), (9000, 500, 1, "fp16"), (9000, 5000, 4, "bf16")])
def test_global_topk_h2o_style(prompt, keep, G, dtype):
    """Sec. 4.1's H2O baseline as a variant: the top `keep` accumulated scores among all rows between sink and
    window survive every eviction (short middle: one wave ranks it; long middle: the block-wide selection)."""
    wl = small(batch=1, n_kv_heads=2, n_q_heads=2 * G, head_dim=64, dtype=dtype, prompt=prompt, decode_steps=40,
               sink=4, window=64, segment=16, keep=keep, evict_every=16, n_obs=24)
    st = run(wl, global_topk=True)
    assert st["evictions"] == 2


def test_global_topk_with_odd_scores():
    wl = small(prompt=600, decode_steps=40, sink=4, window=64, segment=16, keep=30, evict_every=16, n_obs=12)
    run(wl, global_topk=True, plant=plant_odd_scores)


def test_unbuffered_eviction_every_step():
    run(small(prompt=100, decode_steps=50, sink=2, window=20, segment=3, keep=1, evict_every=1, n_obs=4))


def test_capacity_error_when_eviction_is_skipped():
    from paper_2410_23079_amd import BuzzCache, BuzzError
    ls = lockstep()
    wl = small(prompt=100, decode_steps=64, sink=2, window=20, segment=4, keep=1, evict_every=4)
    p, d = prompt_inputs(wl, device="cuda"), decode_inputs(wl, device="cuda")
    c = BuzzCache(ls.buzz_config(wl, flags=0))
    c.prefill(p["K"], p["V"])
    out = torch.empty(wl.batch, wl.n_q_heads, wl.head_dim, dtype=torch.float32, device="cuda")
    for t in range(4):
        c.decode_step(d["q"][t], d["k"][t], d["v"][t], out)
    before = c.lengths()
    with pytest.raises(BuzzError) as e:
        c.decode_step(d["q"][4], d["k"][4], d["v"][4], out)
    assert e.value.code == -2 and c.lengths() == before        # failed call left the cache unchanged
    c.evict()
    c.decode_step(d["q"][4], d["k"][4], d["v"][4], out)
    torch.cuda.synchronize()


def test_log_n_scale_argument():
    """Sec. 3.5: the log-n variant only changes the softmax scale, which is a configuration argument."""
    import math
    ls = lockstep()
    wl = small(prompt=300, decode_steps=20, n_obs=8)
    p, d = prompt_inputs(wl, device="cuda"), decode_inputs(wl, device="cuda")
    scale = math.log(812) / math.log(512) / math.sqrt(wl.head_dim)
    from oracle.buzz_oracle import OracleCache
    from paper_2410_23079_amd import BuzzCache
    units = [(0, h) for h in range(wl.n_kv_heads)]
    g = BuzzCache(ls.buzz_config(wl, softmax_scale=scale))
    o = OracleCache(ls.oracle_config(wl, len(units), softmax_scale=scale, auto_evict=True))
    g.prefill(p["K"], p["V"])
    o.prefill(ls.unit_slices(p["K"], units, 1), ls.unit_slices(p["V"], units, 1))
    out = torch.empty(wl.batch, wl.n_q_heads, wl.head_dim, dtype=torch.float32, device="cuda")
    for t in range(3):                                           # no eviction yet: scores cannot reorder anything
        g.decode_step(d["q"][t], d["k"][t], d["v"][t], out)
        ref = o.decode_step(ls.unit_slices(d["q"][t], units, 1), ls.unit_slices(d["k"][t], units, 1),
                            ls.unit_slices(d["v"][t], units, 1))
        assert ls.rel_err(ls.unit_slices(out, units, 1), ref) <= ls.OUT_EXPECT


# ------------------------------------------------------------------ variants named by the paper
def test_log_n_scaled_attention_tracks_context_length():
    """Sec. 3.5: scale = log_512(n)/sqrt(d) with n = tokens the query sees, prompt scoring included."""
    run(small(prompt=480, decode_steps=64, n_obs=24), log_n=True)          # crosses n = 512


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_log_n_prompt_scores_from_the_first_query_on(dtype):
    """Sec. 3.5 at n = 1: log_512(1) = 0, the first prompt query attends uniformly (to its one visible key)."""
    run(small(batch=1, n_kv_heads=2, n_q_heads=4, head_dim=128, dtype=dtype, prompt=330, decode_steps=12,
              sink=4, window=64, segment=16, keep=2, evict_every=8, n_obs=330), log_n=True)


@pytest.mark.parametrize("G,dtype", [(1, "fp32"), (4, "bf16")])
def test_log_n_from_an_empty_cache(G, dtype):
    """Sec. 3.5 during decode at n = 1, 2, ...: the scale starts at 0 and grows with the tracked length."""
    run(small(batch=1, n_kv_heads=2, n_q_heads=2 * G, head_dim=128, dtype=dtype, prompt=0, decode_steps=70,
              sink=2, window=16, segment=4, keep=1, evict_every=4, n_obs=0), log_n=True)


def test_log_n_with_grouped_queries():
    run(small(batch=1, n_kv_heads=2, n_q_heads=8, head_dim=128, dtype="bf16", prompt=600, decode_steps=40,
              sink=4, window=64, segment=16, keep=2, evict_every=16, n_obs=20), log_n=True)


def test_threshold_bounds_old_plus_new_with_theorem_parameters():
    """The proof's reading of T, with T from the Parameter Estimation theorem (s = 5: T/w = 4.33)."""
    from paper_2410_23079_amd import suggest_threshold
    w, s = 24, 5
    T = suggest_threshold(s, w)
    assert T == round(w * 26 / 6)
    wl = small(prompt=400, decode_steps=260, sink=2, window=w, segment=s, keep=1, evict_every=T, old_stride=0, n_obs=16)
    st = run(wl, threshold_total=True, capacity=wl.sink + w + 2 * T)
    assert st["evictions"] >= 3
    st = run(wl, threshold_total=True)                   # Remark 2's own container: T + k + w rows, no capacity given
    assert st["evictions"] >= 3


def test_interval_sampling_of_new_tokens():
    """Ablation of Sec. 4.3 without the local-max function."""
    run(small(prompt=300, decode_steps=48, keep=2), interval_new=True)


def objective_table(wl, tag):
    """Mean |O^ - O| / |O| over the decode steps (the eviction objective of Sec. 3.1, O = full attention written
    out with torch in float64) for BUZZ, the two ablations of Sec. 4.3 and the baselines of Sec. 4.1 as variants of
    this library: H2O-style (global top-k of accumulated scores) and sink + window, the last two also with the
    budget BUZZ ends up with (H2O-style: keep = BUZZ's final survivor count; sink + window: the window widened by
    it).  Returns {variant: (deviation, retained rows at the end)}."""
    import math
    from paper_2410_23079_amd import FLAG_AUTO_EVICT, FLAG_GLOBAL_TOPK, FLAG_INTERVAL_NEW, BuzzCache
    ls = lockstep()
    p, d = prompt_inputs(wl, device="cuda"), decode_inputs(wl, device="cuda")
    steps, N, G = wl.decode_steps, wl.prompt, wl.group
    Kall = torch.cat([p["K"], d["k"].permute(1, 2, 0, 3)], dim=2).double().repeat_interleave(G, dim=1)   # [B,Hq,N+steps,D]
    Vall = torch.cat([p["V"], d["v"].permute(1, 2, 0, 3)], dim=2).double().repeat_interleave(G, dim=1)
    full = []
    for t in range(steps):
        n = N + t + 1
        lg = torch.einsum("bhd,bhnd->bhn", d["q"][t].double(), Kall[:, :, :n]) / math.sqrt(wl.head_dim)
        full.append(torch.einsum("bhn,bhnd->bhd", torch.softmax(lg, dim=-1), Vall[:, :, :n]))

    def deviation(flags=0, **over):
        cfg = ls.buzz_config(wl, flags=FLAG_AUTO_EVICT | flags, **over)
        c = BuzzCache(cfg)
        c.prefill(p["K"], p["V"], q_obs=p["q_obs"])
        out = torch.empty(wl.batch, wl.n_q_heads, wl.head_dim, dtype=torch.float32, device="cuda")
        dev = 0.0
        for t in range(steps):
            c.decode_step(d["q"][t], d["k"][t], d["v"][t], out)
            dev += float(((out.double() - full[t]).norm(dim=-1) / full[t].norm(dim=-1)).mean())
        rows = c.lengths()[0]
        c.close()
        return dev / steps, rows

    res = {"BUZZ": deviation()}
    budget = res["BUZZ"][1] - wl.sink - wl.window             # survivors (and buffered rows) BUZZ ends with
    res["no local max"] = deviation(FLAG_INTERVAL_NEW)
    res["swapped strides"] = deviation(segment=(wl.segment + 1) // 2, old_stride=wl.segment)
    res["H2O-style, same budget"] = deviation(FLAG_GLOBAL_TOPK, keep=budget)
    res["sink + window, same budget"] = deviation(keep=0, window=wl.window + budget)
    res["sink + window"] = deviation(keep=0)
    print(f"[objective, {tag}] mean |O^ - O| / |O| (retained rows): "
          + "; ".join(f"{k} {v[0]:.4f} ({v[1]})" for k, v in res.items()), flush=True)
    return res


def test_objective_on_clustered_keys():
    """The objective on config 5's recipe (keys and queries around 50 topic means per head), scaled down.  Heavy
    hitters are query-dependent there, so only the weakest claims are asserted: segment winners beat keeping
    nothing but sink and window, at the small budget and at BUZZ's own."""
    wl = small("long131k", batch=1, n_kv_heads=4, n_q_heads=4, head_dim=128, dtype="bf16", prompt=4096, decode_steps=64,
               sink=4, window=256, segment=32, keep=4, evict_every=32, n_obs=256)
    res = objective_table(wl, "clustered keys")
    assert res["BUZZ"][0] < res["sink + window"][0]
    assert res["BUZZ"][1] == res["no local max"][1]
    assert abs(res["H2O-style, same budget"][1] - res["BUZZ"][1]) <= wl.evict_every
    assert abs(res["sink + window, same budget"][1] - res["BUZZ"][1]) <= wl.evict_every


def test_local_max_beats_the_ablations_on_the_papers_objective():
    """Sec. 3.1 states the goal as keeping the evicted cache's attention output close to the full one.
    On synthetic keys with planted heavy hitters, at one cache budget, BUZZ's output must be closer to full
    attention than the no-local-max ablation and than sink + window (Sec. 4.3 reports the same ordering in ROUGE,
    which needs the trained model and is not reproduced here).  The H2O-style baseline is reported at the same
    budget; no order between it and BUZZ is asserted (planted keys are heavy for every query, which is the case
    greedy global selection is made for; the paper's case against it rests on the structure of natural text)."""
    wl = small(batch=2, n_kv_heads=4, n_q_heads=4, head_dim=64, dtype="fp32", prompt=2048, decode_steps=128,
               sink=4, window=128, segment=16, keep=1, evict_every=16, n_obs=256, planted_frac=0.04)
    res = objective_table(wl, "planted heavy keys")
    assert res["BUZZ"][1] == res["no local max"][1]
    assert res["BUZZ"][0] < res["no local max"][0] < res["sink + window"][0]
    assert res["BUZZ"][0] < res["sink + window, same budget"][0]
    assert abs(res["H2O-style, same budget"][1] - res["BUZZ"][1]) <= wl.evict_every


@pytest.mark.parametrize("name,kw", [("tiny", {}), ("llama7b_layer", dict(batch=1, n_kv_heads=4, n_q_heads=4, decode_steps=256))])
def test_free_run_parts_only_at_near_ties(name, kw):
    """GPU (fp32 scores) and oracle (fp64 scores) evicting on their own scores keep the same rows, or part at a
    near-tie (relative score gap below 1e-5)."""
    wl = small(name, **kw)
    p, d = prompt_inputs(wl, device="cuda"), decode_inputs(wl, device="cuda")
    res = lockstep().run_free(wl, p, d)
    print(f"[free run] {wl.name}: {res['agreed']} evictions agreed, parted at step {res['parted_at']}, "
          f"largest gap {res['gap']:.2e}", flush=True)
    # either every eviction of the run agreed (16 for config 1, 8 for the slice of config 2; what these seeds
    # give), or the runs parted at a near-tie, which run_free has verified row by row
    if res["parted_at"] is None:
        assert res["agreed"] == wl.decode_steps // wl.evict_every
    else:
        assert res["gap"] <= 1e-5


def test_default_and_deterministic_modes_agree_over_many_steps():
    """Config 4's shape (eight blocks per unit merge through device memory in every launch), 10 240 steps with
    evictions: a cache in the default mode and one in the deterministic mode stay within rounding of each other.
    (A merge that ran ahead of a partial showed up about once in 10^5 launches before the publishing waves
    waited for their own stores.)"""
    from paper_2410_23079_amd import FLAG_AUTO_EVICT, FLAG_DETERMINISTIC, FLAG_DEVICE_MERGE, BuzzCache
    ls = lockstep()
    wl = get_workload("gqa8b_layer")
    p, d = prompt_inputs(wl, device="cuda"), decode_inputs(wl, device="cuda")
    steps = wl.decode_steps
    # the first cache merges a unit's splits through one die's L2, the second through device memory
    caches = [BuzzCache(ls.buzz_config(wl, flags=FLAG_AUTO_EVICT | f, max_context=wl.prompt + steps + 1))
              for f in (0, FLAG_DETERMINISTIC | FLAG_DEVICE_MERGE)]
    outs = [torch.empty(wl.batch, wl.n_q_heads, wl.head_dim, dtype=torch.float32, device="cuda") for _ in caches]
    worst = torch.zeros((), device="cuda")
    for _ in range(10240 // steps):
        for c in caches:
            c.prefill(p["K"], p["V"], q_obs=p["q_obs"])
        for t in range(steps):
            for c, o in zip(caches, outs):
                c.decode_step(d["q"][t], d["k"][t], d["v"][t], o)
            worst = torch.maximum(worst, (outs[0] - outs[1]).abs().amax() / outs[1].abs().amax())
        assert caches[0].lengths() == caches[1].lengths()
    print(f"[parity]   default vs deterministic over 10240 steps: worst relative difference {float(worst):.2e}", flush=True)
    assert float(worst) < 1e-4


# ------------------------------------------------------------------ full-size configs, sampled units
def sampled_units(wl, count, seed):
    r = np.random.default_rng(seed)
    flat = r.choice(wl.batch * wl.n_kv_heads, size=min(count, wl.batch * wl.n_kv_heads), replace=False)
    return sorted((int(u) // wl.n_kv_heads, int(u) % wl.n_kv_heads) for u in flat)


def test_llama7b_layer_full_size():
    wl = get_workload("llama7b_layer")
    st = run(wl, units=sampled_units(wl, 6, 2), deterministic=False)
    assert st["evictions"] == 512 // 32


@pytest.mark.parametrize("device_merge", [False, True])
def test_gqa8b_layer_full_size(device_merge):
    """Config 4 at full size against the oracle: eight blocks per unit merge in every launch, through one die's
    L2 (default) or through device memory."""
    wl = get_workload("gqa8b_layer").scaled(decode_steps=130)
    st = run(wl, units=sampled_units(wl, 3, 4), check_auto=False, deterministic=False, device_merge=device_merge)
    assert st["evictions"] == 2


def test_long131k_full_size():
    wl = get_workload("long131k").scaled(decode_steps=130)
    st = run(wl, units=sampled_units(wl, 2, 5), check_auto=False, deterministic=False)
    assert st["evictions"] == 1


def test_llama7b_full_one_layer_full_size():
    wl = get_workload("llama7b_full").scaled(decode_steps=66)
    st = run(wl, units=sampled_units(wl, 3, 3), check_auto=False, deterministic=False)
    assert st["evictions"] == 1


def test_paper_parameters_full_size():
    """Config 2's shape with the paper's parameterisation (s = 5, s^ = 3, T from the theorem, bounding old + new)."""
    wl = get_workload("llama7b_layer_paper").scaled(decode_steps=360)
    st = run(wl, units=sampled_units(wl, 4, 6), check_auto=False, deterministic=False)
    assert st["evictions"] == 1
