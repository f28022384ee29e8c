"""Pins for the CPU oracle: each test checks it against something other than itself --
a library routine, a closed form, a value the paper prints, an invariant, or brute force.

Citations are to the paper (arxiv 2410.23079): Sec. 3.1 eq. 2/3/5, Sec. 3.3 (Alg. 1, Alg. 2,
Remarks 1-2), Sec. 3.4 (Parameter Estimation theorem, printed value for s = 5), Sec. 4.1 baselines.
"""
import math
import os

import numpy as np
import pytest
import torch

from oracle.buzz_oracle import OracleCache, OracleConfig

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rng(seed):
    return np.random.default_rng(seed)


def sdpa64(q, K, V, scale=None):
    """Library attention in float64: q [H,D], K,V [H,n,D] -> [H,D]."""
    qt = torch.from_numpy(np.ascontiguousarray(q))[:, None, :]
    out = torch.nn.functional.scaled_dot_product_attention(
        qt, torch.from_numpy(np.ascontiguousarray(K)), torch.from_numpy(np.ascontiguousarray(V)), scale=scale)
    return out[:, 0, :].numpy()


def make(B, Hq, Hkv, D, N, steps, seed):
    r = rng(seed)
    return dict(
        K=r.standard_normal((B, Hkv, N, D)), V=r.standard_normal((B, Hkv, N, D)),
        q_obs=r.standard_normal((B, Hq, N, D)),
        q=r.standard_normal((steps, B, Hq, D)), k=r.standard_normal((steps, B, Hkv, D)),
        v=r.standard_normal((steps, B, Hkv, D)))


# ---------------------------------------------------------------- P1: full attention (Remark 1; eq. 3)
@pytest.mark.parametrize("G", [1, 4])
def test_full_attention_when_nothing_is_evicted(G):
    B, Hkv, D, N, steps = 2, 2, 16, 24, 10
    Hq = Hkv * G
    x = make(B, Hq, Hkv, D, N, steps, 1)
    for cfg in (
        OracleConfig(B, Hq, Hkv, D, sink=4, window=N + steps, segment=4, keep=1, evict_every=2),      # sink+window >= all
        OracleConfig(B, Hq, Hkv, D, sink=2, window=3, segment=4, keep=4, evict_every=4, old_stride=1),  # keep >= segment
    ):
        o = OracleCache(cfg)
        o.prefill(x["K"], x["V"])
        Kall, Vall = x["K"].copy(), x["V"].copy()
        for t in range(steps):
            out = o.decode_step(x["q"][t], x["k"][t], x["v"][t])
            Kall = np.concatenate([Kall, x["k"][t][:, :, None, :]], axis=2)
            Vall = np.concatenate([Vall, x["v"][t][:, :, None, :]], axis=2)
            for b in range(B):
                ref = sdpa64(x["q"][t][b], np.repeat(Kall[b], G, axis=0), np.repeat(Vall[b], G, axis=0))
                np.testing.assert_allclose(out[b], ref, rtol=1e-12, atol=1e-13)
        assert o.lengths()[0] == N + steps
        _, _, _, pos = o.export()
        assert (pos == np.arange(N + steps)).all()


def test_softmax_scale_argument_and_default():
    B, Hq, Hkv, D, N = 1, 2, 2, 8, 12
    x = make(B, Hq, Hkv, D, N, 1, 2)
    for scale in (0.0, 0.37):
        o = OracleCache(OracleConfig(B, Hq, Hkv, D, sink=4, window=64, segment=4, softmax_scale=scale))
        o.prefill(x["K"], x["V"])
        out = o.decode_step(x["q"][0], x["k"][0], x["v"][0])
        Kall = np.concatenate([x["K"], x["k"][0][:, :, None, :]], axis=2)
        Vall = np.concatenate([x["V"], x["v"][0][:, :, None, :]], axis=2)
        ref = sdpa64(x["q"][0][0], Kall[0], Vall[0], scale=(scale or 1 / math.sqrt(D)))
        np.testing.assert_allclose(out[0], ref, rtol=1e-12, atol=1e-13)


# ---------------------------------------------------------------- accumulated score = column sums of the causal matrix
@pytest.mark.parametrize("G,n_obs,B", [(1, 20, 1), (2, 7, 1), (2, 0, 1), (2, 9, 3)])
def test_prefill_and_decode_scores_are_causal_column_sums(G, n_obs, B):
    Hkv, D, N, steps = 2, 8, 20, 6
    Hq = Hkv * G
    x = make(B, Hq, Hkv, D, N, steps, 3)
    init = rng(4).random((B, Hkv, N))
    o = OracleCache(OracleConfig(B, Hq, Hkv, D, sink=2, window=1000, segment=4))
    o.prefill(x["K"], x["V"], q_obs=x["q_obs"][:, :, N - n_obs:, :] if n_obs else None, init_score=init)
    for t in range(steps):
        o.decode_step(x["q"][t], x["k"][t], x["v"][t])
    _, _, A, _ = o.export()
    # library route: full [queries x keys] causal softmax with torch, then sum the columns
    Kall = np.concatenate([x["K"], np.moveaxis(x["k"], 0, 2)], axis=2)      # [B,Hkv,N+steps,D]
    qs = np.concatenate([x["q_obs"][:, :, N - n_obs:, :], np.moveaxis(x["q"], 0, 2)], axis=2)  # [B,Hq,n_obs+steps,D]
    qpos = np.concatenate([np.arange(N - n_obs, N), np.arange(N, N + steps)])
    expect = np.concatenate([init, np.zeros((B, Hkv, steps))], axis=2)
    for b in range(B):
        for h in range(Hq):
            logits = torch.from_numpy(qs[b, h] @ Kall[b, h // G].T / math.sqrt(D))
            mask = torch.from_numpy(np.arange(N + steps)[None, :] > qpos[:, None])
            P = torch.softmax(logits.masked_fill(mask, -math.inf), dim=-1).numpy()
            expect[b, h // G] += P.sum(axis=0)
    np.testing.assert_allclose(A, expect, rtol=1e-11, atol=1e-13)


def test_exported_rows_are_the_input_rows_at_the_exported_positions():
    """Every (batch, kv-head) unit's exported K / V rows are the caller's rows at the exported token
    positions (the cache stores keys and values as given, eq. 2), also after evictions."""
    B, Hq, Hkv, D, N, steps = 2, 6, 3, 8, 70, 25
    x = make(B, Hq, Hkv, D, N, steps, 91)
    o = OracleCache(OracleConfig(B, Hq, Hkv, D, sink=3, window=7, segment=5, keep=2, evict_every=6, old_stride=2))
    o.prefill(x["K"], x["V"], q_obs=x["q_obs"][:, :, -4:, :])
    Kall = np.concatenate([x["K"], np.moveaxis(x["k"], 0, 2)], axis=2)
    Vall = np.concatenate([x["V"], np.moveaxis(x["v"], 0, 2)], axis=2)
    for t in range(steps):
        o.decode_step(x["q"][t], x["k"][t], x["v"][t])
        K, V, _, pos = o.export()
        for b in range(B):
            for h in range(Hkv):
                assert (K[b, h] == Kall[b, h][pos[b, h]]).all() and (V[b, h] == Vall[b, h][pos[b, h]]).all()


def test_set_scores_reaches_every_unit():
    """Scores written with set_scores come back from export unit by unit, and the next eviction ranks by them."""
    B, Hq, Hkv, D, N = 2, 2, 2, 4, 30
    x = make(B, Hq, Hkv, D, N, 1, 92)
    o = OracleCache(OracleConfig(B, Hq, Hkv, D, sink=2, window=4, segment=6, keep=1, evict_every=1000, old_stride=1,
                                 auto_evict=False))
    o.prefill(x["K"], x["V"])
    n = o.lengths()[0]
    A = rng(93).random((B, Hkv, n))
    o.set_scores(A)
    assert (o.export()[2] == A).all()
    o.evict()
    pos = o.export()[3]
    for b in range(B):
        for h in range(Hkv):
            want = [2 + i + int(np.argmax(A[b, h, 2 + i:min(2 + i + 6, n - 4)])) for i in range(0, n - 6, 6)]
            assert list(pos[b, h, 2:-4]) == want


def test_softmax_is_taken_relative_to_the_largest_logit():
    """Logits far outside exp's range still give the library's probabilities (eq. 3 evaluated stably)."""
    B, Hq, Hkv, D = 1, 1, 1, 2
    K = np.array([[[[0.0, 0.0], [400.0, 0.0], [401.0, 0.0]]]])
    V = np.array([[[[1.0, 0.0], [0.0, 1.0], [0.0, 3.0]]]])
    o = OracleCache(OracleConfig(B, Hq, Hkv, D, sink=1, window=100, segment=4, softmax_scale=1.0))
    o.prefill(K, V)
    q = np.array([[[2.0, 0.0]]]); k = np.array([[[-400.0, 0.0]]]); v = np.array([[[5.0, 5.0]]])
    out = o.decode_step(q, k, v)
    p = torch.softmax(torch.tensor([0.0, 800.0, 802.0, -800.0], dtype=torch.float64), 0).numpy()
    np.testing.assert_allclose(out[0, 0], p @ np.array([[1.0, 0.0], [0.0, 1.0], [0.0, 3.0], [5.0, 5.0]]), rtol=1e-13)
    np.testing.assert_allclose(o.export()[2][0, 0], p, rtol=1e-13, atol=0)


# ---------------------------------------------------------------- P8: probability mass
def test_each_decode_step_adds_group_size_to_total_score():
    B, Hkv, G, D, N = 1, 2, 4, 8, 40
    Hq = Hkv * G
    x = make(B, Hq, Hkv, D, N, 5, 5)
    o = OracleCache(OracleConfig(B, Hq, Hkv, D, sink=2, window=8, segment=4, keep=1, evict_every=4,
                                 old_stride=1, auto_evict=False))
    o.prefill(x["K"], x["V"], q_obs=x["q_obs"][:, :, -3:, :])
    # prefill evicts (30 new >= 4), so mass is no longer 3*G; track increments instead
    prev = o.export()[2].sum(axis=2)
    for t in range(5):
        o.decode_step(x["q"][t], x["k"][t], x["v"][t])
        cur = o.export()[2].sum(axis=2)
        np.testing.assert_allclose(cur - prev, G, rtol=1e-12)
        prev = cur
    o2 = OracleCache(OracleConfig(B, Hq, Hkv, D, sink=2, window=100, segment=4))
    o2.prefill(x["K"], x["V"], q_obs=x["q_obs"][:, :, -3:, :])
    np.testing.assert_allclose(o2.export()[2].sum(axis=2), 3 * G, rtol=1e-12)


# ---------------------------------------------------------------- P2: StreamingLLM special case (Sec. 4.1 baselines)
def test_keep_zero_is_sink_plus_window():
    B, Hq, Hkv, D, N, steps = 1, 2, 2, 8, 50, 13
    k, w, T = 3, 10, 4
    x = make(B, Hq, Hkv, D, N, steps, 6)
    o = OracleCache(OracleConfig(B, Hq, Hkv, D, sink=k, window=w, segment=5, keep=0, evict_every=T, old_stride=1))
    o.prefill(x["K"], x["V"])
    Kall, Vall = x["K"].copy(), x["V"].copy()
    buffered = 0
    for t in range(steps):
        out = o.decode_step(x["q"][t], x["k"][t], x["v"][t])
        Kall = np.concatenate([Kall, x["k"][t][:, :, None, :]], axis=2)
        Vall = np.concatenate([Vall, x["v"][t][:, :, None, :]], axis=2)
        tot = N + t + 1
        buffered += 1
        keep_pos = np.concatenate([np.arange(k), np.arange(tot - w - buffered, tot)])
        ref = sdpa64(x["q"][t][0], Kall[0][:, keep_pos], Vall[0][:, keep_pos])
        np.testing.assert_allclose(out[0], ref, rtol=1e-12, atol=1e-13)
        if buffered == T:
            buffered = 0
        pos = o.export()[3]
        expect = np.concatenate([np.arange(k), np.arange(tot - w - buffered, tot)])
        assert (pos[0, 0] == expect).all()


# ---------------------------------------------------------------- P3: constant scores -> interval sampling (ties -> lowest index)
@pytest.mark.parametrize("keep", [1, 2])
def test_constant_scores_reduce_to_interval_sampling(keep):
    B, Hq, Hkv, D, N = 1, 1, 1, 4, 61
    k, w, s = 3, 7, 6
    x = make(B, Hq, Hkv, D, N, 0, 7)
    o = OracleCache(OracleConfig(B, Hq, Hkv, D, sink=k, window=w, segment=s, keep=keep, evict_every=1, old_stride=1))
    o.prefill(x["K"], x["V"])                      # no observed queries: every score is 0
    pos = o.export()[3][0, 0]
    lo, hi = k, N - w
    mid = [j for j in range(lo, hi) if (j - lo) % s < keep]
    assert list(pos) == list(range(k)) + mid + list(range(hi, N))
    assert o.lengths()[1] == len(mid)


# ---------------------------------------------------------------- P4: brute force of Alg. 1 + Alg. 2 with python slices
def brute_force_evict(pos, score, k, w, s, keep, n_old, old_stride):
    n = len(pos)
    if n <= k + w:
        return list(pos), n_old
    idx = list(range(n))
    old = idx[k:k + n_old][::old_stride]
    new = idx[k + n_old:n - w]
    picked = []
    for a in range(0, len(new), s):
        seg = new[a:a + s]
        def key(j):
            v = score[j]
            return (-(v if not math.isnan(v) else -math.inf), j)
        picked += sorted(sorted(seg, key=key)[:keep])
    res = idx[:k] + old + picked + idx[n - w:]
    return [pos[j] for j in res], len(old) + len(picked)


@pytest.mark.parametrize("seed", range(12))
def test_eviction_matches_brute_force_on_tiny_inputs(seed):
    r = rng(100 + seed)
    D = 2
    k, w = int(r.integers(0, 4)), int(r.integers(0, 6))
    s = int(r.integers(1, 9))
    keep = int(r.integers(0, 4))
    old_stride = int(r.choice([0, 1, 2, 3]))
    eff_stride = old_stride or (s + 1) // 2
    N = int(r.integers(1, 64))
    K = np.zeros((1, 1, N, D))
    K[0, 0, :, 0] = np.arange(N)                       # column 0 carries the token index, so rows can be traced
    # few distinct values -> many ties; an occasional NaN
    init = r.integers(0, 4, size=(1, 1, N)).astype(np.float64)
    if seed % 3 == 0 and N > 3:
        init[0, 0, r.integers(0, N)] = np.nan
    o = OracleCache(OracleConfig(1, 1, 1, D, sink=k, window=w, segment=s, keep=keep, evict_every=10 ** 6,
                                 old_stride=old_stride, auto_evict=False))
    o.prefill(K, -K, init_score=init)
    pos, n_old = list(range(N)), 0
    score = list(init[0, 0])
    tok = N
    for rnd in range(4):
        o.evict()
        pos, n_old = brute_force_evict(pos, score, k, w, s, keep, n_old, eff_stride)
        Ko, Vo, _, got_pos = o.export()
        assert list(got_pos[0, 0]) == pos
        assert o.lengths()[:2] == (len(pos), n_old)
        np.testing.assert_array_equal(Ko[0, 0, :, 0], pos)
        np.testing.assert_array_equal(Vo[0, 0, :, 0], -np.asarray(pos, dtype=np.float64))
        # append a few more rows, then plant fresh random scores on every retained row
        for _ in range(int(r.integers(1, 12))):
            row = np.zeros((1, 1, D))
            row[0, 0, 0] = tok
            o.decode_step(np.zeros((1, 1, D)), row, -row)
            pos.append(tok)
            tok += 1
        A = r.integers(0, 4, size=(1, 1, len(pos))).astype(np.float64)
        o.set_scores(A)
        score = list(A[0, 0])


def test_rows_move_with_their_positions():
    """K, V and score of a survivor travel together (the cache stays aligned after compaction)."""
    D, N = 3, 40
    r = rng(9)
    K = np.arange(N, dtype=np.float64)[None, None, :, None] + np.zeros((1, 1, N, D))
    V = -K
    init = r.random((1, 1, N))
    o = OracleCache(OracleConfig(1, 1, 1, D, sink=2, window=5, segment=4, keep=1, evict_every=1, old_stride=1))
    o.prefill(K, V, init_score=init)
    Ko, Vo, A, pos = o.export()
    np.testing.assert_array_equal(Ko[0, 0, :, 0], pos[0, 0])
    np.testing.assert_array_equal(Vo[0, 0, :, 1], -pos[0, 0])
    np.testing.assert_array_equal(A[0, 0], init[0, 0, pos[0, 0]])


# ---------------------------------------------------------------- P6: shrink ratio (Sec. 3.3 buffering strategy)
@pytest.mark.parametrize("L,s,c", [(100, 5, 1), (103, 5, 1), (64, 16, 4), (70, 16, 4), (7, 16, 4)])
def test_one_eviction_shrinks_middle_as_stated(L, s, c):
    k, w = 4, 6
    N = k + L + w
    K = rng(0).standard_normal((1, 1, N, 2))
    o = OracleCache(OracleConfig(1, 1, 1, 2, sink=k, window=w, segment=s, keep=c, evict_every=1, old_stride=1))
    o.prefill(K, K, init_score=rng(1).random((1, 1, N)))
    n, n_old, new = o.lengths()
    assert n_old == c * (L // s) + min(c, L % s)
    assert n == k + n_old + w and new == 0
    if c == 1 and L % s == 0:
        assert L - n_old == L * (s - 1) // s      # "reduces ... by approximately (s-1)/s"


# ---------------------------------------------------------------- P5: size recurrence and the printed 4.33 (Sec. 3.4, App. C.1)
def read_golden():
    vals = {}
    with open(os.path.join(GOLDEN, "parameter_estimation.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                a, b = line.split()
                vals[a] = float(b)
    return vals


def drive_capacity_threshold(s, T_total, rounds, keep=1):
    """Evict whenever old+new reaches T_total (the reading used by the theorem's proof); returns sizes after each."""
    k, w, D = 2, 3, 1
    o = OracleCache(OracleConfig(1, 1, 1, D, sink=k, window=w, segment=s, keep=keep, evict_every=10 ** 6,
                                 old_stride=0, auto_evict=False))
    o.prefill(np.zeros((1, 1, k + w, D)), np.zeros((1, 1, k + w, D)))
    sizes = []
    z = np.zeros((1, 1, D))
    for _ in range(rounds):
        while True:
            n, n_old, new = o.lengths()
            if n_old + new >= T_total:
                break
            o.decode_step(z, z, z)
        o.evict()
        sizes.append(o.lengths()[1])
    return sizes


@pytest.mark.parametrize("s", [3, 4, 5, 6, 7, 8, 16])
def test_size_recurrence_and_fixed_point(s):
    T_total = 2000
    sh = (s + 1) // 2
    sizes = drive_capacity_threshold(s, T_total, rounds=40)
    a = 0
    for got in sizes:
        a = -(-a // sh) + -(-(T_total - a) // s)          # ceil version of the proof's recurrence
        assert got == a
    limit = sizes[-1]
    predicted = (s * s + 1) / (s + 1) if s % 2 else (s - 1)
    assert abs(T_total / limit - predicted) / predicted < 0.01
    # the floor version printed in the proof stays within its own +-2 bracket of ours
    fl = 0
    for got in sizes:
        fl = fl // sh + (T_total - fl) // s
    assert abs(fl - limit) <= 4


def test_printed_ratio_for_stride_five():
    g = read_golden()
    s = int(g["stride"])
    sizes = drive_capacity_threshold(s, 2600, rounds=40)
    assert round(2600 / sizes[-1], 2) == pytest.approx(g["predicted_T_over_w"], abs=0.011)
    assert round((s * s + 1) / (s + 1), 2) == g["predicted_T_over_w"]


# ---------------------------------------------------------------- P7 + P10: size bound and data-independent closed form
def closed_form_sizes(N, steps, k, w, s, c, T, sh):
    """Integer-only replay of Alg. 1 sizes: returns list of (n, n_old) after prefill and after each step."""
    def evict(n, n_old):
        if n <= k + w:
            return n, n_old
        new = n - k - n_old - w
        old2 = -(-n_old // sh)
        new2 = min(c, s) * (new // s) + min(c, new % s)
        return k + old2 + new2 + w, old2 + new2
    n, n_old = N, 0
    if n - k - w >= T:
        n, n_old = evict(n, n_old)
    out = [(n, n_old)]
    for _ in range(steps):
        n += 1
        if n - k - n_old - w >= T:
            n, n_old = evict(n, n_old)
        out.append((n, n_old))
    return out


@pytest.mark.parametrize("seed", range(8))
def test_sizes_are_data_independent_and_bounded(seed):
    r = rng(200 + seed)
    k, w = int(r.integers(0, 5)), int(r.integers(1, 20))
    s, c = int(r.integers(1, 10)), int(r.integers(0, 4))
    T = int(r.integers(1, 15))
    old_stride = int(r.choice([0, 1, 2]))
    sh = old_stride or (s + 1) // 2
    N, steps, D = int(r.integers(1, 120)), 60, 4
    x = make(1, 2, 1, D, N, steps, 300 + seed)
    o = OracleCache(OracleConfig(1, 2, 1, D, sink=k, window=w, segment=s, keep=c, evict_every=T,
                                 old_stride=old_stride))
    o.prefill(x["K"], x["V"], q_obs=x["q_obs"][:, :, -min(N, 5):, :])
    expect = closed_form_sizes(N, steps, k, w, s, c, T, sh)
    assert o.lengths()[:2] == expect[0]
    segs_kept = expect[0][1]
    for t in range(steps):
        o.decode_step(x["q"][t], x["k"][t], x["v"][t])
        n, n_old, new = o.lengths()
        assert (n, n_old) == expect[t + 1]
        assert new < T
        # cache never exceeds sink + window + buffered + (segments x keep) when survivors persist
        if sh == 1:
            total_new = max(0, N + t + 1 - k - w)
            assert n_old <= c * (-(-total_new // s) + (t + 1) // T + 1)
            assert n <= k + w + T + n_old
        assert n <= N + t + 1
    pos = o.export()[3][0, 0]
    assert (np.diff(pos) > 0).all()                      # positional order is preserved
    assert list(pos[:min(k, len(pos))]) == list(range(min(k, len(pos))))
    assert list(pos[-min(w, len(pos)):]) == list(range(N + steps - min(w, len(pos)), N + steps))


# ---------------------------------------------------------------- P9: convexity and permutation invariance (eq. 3)
def test_output_is_convex_combination_and_permutation_invariant():
    B, Hq, Hkv, D, N = 1, 2, 1, 6, 30
    x = make(B, Hq, Hkv, D, N, 1, 11)
    cfg = OracleConfig(B, Hq, Hkv, D, sink=2, window=100, segment=4)
    o = OracleCache(cfg)
    o.prefill(x["K"], x["V"])
    out = o.decode_step(x["q"][0], x["k"][0], x["v"][0])
    Vall = np.concatenate([x["V"], x["v"][0][:, :, None, :]], axis=2)[0, 0]
    assert (out[0] <= Vall.max(axis=0) + 1e-12).all() and (out[0] >= Vall.min(axis=0) - 1e-12).all()
    perm = rng(12).permutation(N)
    o2 = OracleCache(cfg)
    o2.prefill(x["K"][:, :, perm], x["V"][:, :, perm])
    out2 = o2.decode_step(x["q"][0], x["k"][0], x["v"][0])
    np.testing.assert_allclose(out, out2, rtol=1e-12, atol=1e-14)


# ---------------------------------------------------------------- old-token interval sampling with the paper's stride
def test_old_tokens_are_interval_sampled_with_half_stride():
    D, k, w, s, T = 2, 2, 4, 5, 10
    N = k + w
    z = np.zeros((1, 1, D))
    o = OracleCache(OracleConfig(1, 1, 1, D, sink=k, window=w, segment=s, keep=1, evict_every=T))   # s^ = 3
    o.prefill(np.zeros((1, 1, N, D)), np.zeros((1, 1, N, D)))
    for _ in range(T):
        o.decode_step(z, z, z)
    # scores are uniform-ish but not tied; read the survivors rather than predicting them
    pos1 = list(o.export()[3][0, 0])
    old1 = pos1[k:-w]
    assert len(old1) == T // s
    for _ in range(T):
        o.decode_step(z, z, z)
    pos2 = list(o.export()[3][0, 0])
    old2 = pos2[k:-w]
    assert old2[:len(old1[::3])] == old1[::3]            # floor((5+1)/2) = 3
    assert len(old2) == len(old1[::3]) + T // s


# ---------------------------------------------------------------- planted heavy keys win their segments (sanity of the whole path)
def test_planted_heavy_keys_survive():
    from workloads import get_workload, prompt_inputs, decode_inputs
    wl = get_workload("tiny").scaled(prompt=256, decode_steps=32)
    p = prompt_inputs(wl)
    d = decode_inputs(wl)
    o = OracleCache(OracleConfig(wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.sink, wl.window, wl.segment,
                                 wl.keep, wl.evict_every, wl.old_stride))
    o.prefill(p["K"].double().numpy(), p["V"].double().numpy(), q_obs=p["q_obs"].double().numpy())
    for t in range(wl.decode_steps):
        o.decode_step(d["q"][t].double().numpy(), d["k"][t].double().numpy(), d["v"][t].double().numpy())
    n, n_old, _ = o.lengths()
    assert n <= wl.sink + wl.window + wl.evict_every + n_old
    assert n_old == -(-(256 - 4 - 64) // 16) + 32 // 16


# ---------------------------------------------------------------- variants: log-n scaling (Sec. 3.5) and the proof's threshold
def test_log_n_scale_follows_context_length_and_is_plain_attention_at_512():
    B, Hq, Hkv, D, N, steps = 1, 2, 1, 8, 508, 8
    x = make(B, Hq, Hkv, D, N, steps, 21)
    o = OracleCache(OracleConfig(B, Hq, Hkv, D, sink=4, window=10 ** 6, segment=4, log_n=True))
    plain = OracleCache(OracleConfig(B, Hq, Hkv, D, sink=4, window=10 ** 6, segment=4))
    o.prefill(x["K"], x["V"])
    plain.prefill(x["K"], x["V"])
    Kall, Vall = x["K"].copy(), x["V"].copy()
    for t in range(steps):
        out = o.decode_step(x["q"][t], x["k"][t], x["v"][t])
        ref_plain = plain.decode_step(x["q"][t], x["k"][t], x["v"][t])
        Kall = np.concatenate([Kall, x["k"][t][:, :, None, :]], axis=2)
        Vall = np.concatenate([Vall, x["v"][t][:, :, None, :]], axis=2)
        n = N + t + 1
        ref = sdpa64(x["q"][t][0], np.repeat(Kall[0], 2, axis=0), np.repeat(Vall[0], 2, axis=0),
                     scale=math.log(n) / math.log(512) / math.sqrt(D))
        np.testing.assert_allclose(out[0], ref, rtol=1e-12, atol=1e-13)
        if n == 512:                                     # "degrades to the traditional attention formula"
            np.testing.assert_allclose(out, ref_plain, rtol=1e-12, atol=1e-13)
        else:
            assert np.abs(out - ref_plain).max() > 1e-9


def test_log_n_prefill_scores_use_each_query_position():
    B, Hq, Hkv, D, N, n_obs = 1, 1, 1, 8, 30, 6
    x = make(B, Hq, Hkv, D, N, 0, 22)
    o = OracleCache(OracleConfig(B, Hq, Hkv, D, sink=2, window=1000, segment=4, log_n=True))
    o.prefill(x["K"], x["V"], q_obs=x["q_obs"][:, :, N - n_obs:, :])
    A = o.export()[2][0, 0]
    expect = np.zeros(N)
    for t in range(n_obs):
        i = N - n_obs + t
        logits = torch.from_numpy(x["q_obs"][0, 0, i] @ x["K"][0, 0, :i + 1].T) * (math.log(i + 1) / math.log(512) / math.sqrt(D))
        expect[:i + 1] += torch.softmax(logits, dim=-1).numpy()
    np.testing.assert_allclose(A, expect, rtol=1e-11, atol=1e-13)


@pytest.mark.parametrize("s", [3, 5, 6])
def test_total_threshold_runs_the_proofs_recurrence_by_itself(s):
    """With T bounding old + new, automatic eviction reproduces a' = ceil(a/s^) + ceil((T-a)/s)."""
    k, w, D, T = 2, 3, 1, 600
    sh = (s + 1) // 2
    o = OracleCache(OracleConfig(1, 1, 1, D, sink=k, window=w, segment=s, keep=1, evict_every=T, old_stride=0,
                                 threshold_total=True))
    o.prefill(np.zeros((1, 1, k + w, D)), np.zeros((1, 1, k + w, D)))
    z = np.zeros((1, 1, D))
    a, seen = 0, []
    for _ in range(12 * T):
        before = o.lengths()
        o.decode_step(z, z, z)
        after = o.lengths()
        if after[2] == 0 and before[2] > 0:              # the buffered tokens were just consumed
            a = -(-a // sh) + -(-(T - a) // s)
            assert after[1] == a
            seen.append(a)
    assert len(seen) >= 8
    predicted = (s * s + 1) / (s + 1) if s % 2 else (s - 1)
    assert abs(T / seen[-1] - predicted) / predicted < 0.03


def test_interval_sampling_of_new_tokens_ignores_scores():
    """Ablation without the local-max function (Sec. 4.3): survivors are fixed positions, whatever the scores."""
    k, w, s, c, T, D = 2, 5, 4, 1, 11, 2
    r = np.random.default_rng(31)
    N = k + w + 2 * T + 3
    K = r.standard_normal((1, 1, N, D)); V = r.standard_normal((1, 1, N, D))
    o = OracleCache(OracleConfig(1, 1, 1, D, sink=k, window=w, segment=s, keep=c, evict_every=T, old_stride=1,
                                 interval_new=True))
    o.prefill(K, V, init_score=r.standard_normal((1, 1, N)))
    pos = o.export()[3][0, 0]
    mid = np.arange(k, N - w)
    expect = np.concatenate([np.arange(k), mid[::s], np.arange(N - w, N)])          # plain strided slices
    np.testing.assert_array_equal(pos, expect)
    o2 = OracleCache(OracleConfig(1, 1, 1, D, sink=k, window=w, segment=s, keep=2, evict_every=T, old_stride=1,
                                  interval_new=True))
    o2.prefill(K, V, init_score=r.standard_normal((1, 1, N)))
    expect2 = np.concatenate([np.arange(k), np.sort(np.concatenate([mid[::s], mid[1::s]])), np.arange(N - w, N)])
    np.testing.assert_array_equal(o2.export()[3][0, 0], expect2)


# ---------------------------------------------------------------- Remark 2: a prefill samples until the rows fit their container
def replay_prefill(N, k, w, s, sh, T, c, score, capacity=0, total=False):
    """Alg. 1's sampling applied to a prompt with Python slices and `sorted`, repeated as Remark 2 says.
    Returns the retained token indices.  (Under either reading of T the count compared with T at a prefill
    is the number of prompt tokens between sink and window: there are no old tokens yet.)"""
    idx = list(range(N))
    if N - k - w < T:                                    # fewer than T tokens between sink and window: keep all
        return idx
    mid = idx[k:N - w]
    old = []
    for a in range(0, len(mid), s):                      # Alg. 2 on the new tokens
        seg = mid[a:a + s]
        old += sorted(sorted(seg, key=lambda j: (-score[j], j))[:c])
    if capacity:
        fits = lambda rows: k + rows + w + T <= capacity     # room for the next T buffered tokens remains
    elif total:
        fits = lambda rows: k + rows + w <= T + k + w        # the remark's container of length T + k + w
    else:
        fits = lambda rows: True
    while not fits(len(old)):
        assert len(old[::sh]) < len(old), "cannot fit"
        old = old[::sh]                                  # interval sampling of what are now old tokens
    return idx[:k] + old + idx[N - w:]


@pytest.mark.parametrize("seed", range(12))
def test_prefill_samples_until_it_fits_the_container(seed):
    r = rng(400 + seed)
    k, w = int(r.integers(0, 5)), int(r.integers(0, 12))
    s, c = int(r.integers(2, 9)), int(r.integers(1, 3))
    sh = int(r.choice([0, 2, 3, 4]))
    eff = sh or (s + 1) // 2
    if eff < 2:
        sh = eff = 2
    T = int(r.integers(4, 30))
    N = int(r.integers(k + w + T, 700))
    total = bool(seed % 2)
    capacity = 0 if seed % 3 == 0 else k + w + T + int(r.integers(1, 12))
    D = 2
    K = np.zeros((1, 1, N, D))
    K[0, 0, :, 0] = np.arange(N)
    init = r.integers(0, 5, size=(1, 1, N)).astype(np.float64)       # ties everywhere
    o = OracleCache(OracleConfig(1, 1, 1, D, sink=k, window=w, segment=s, keep=c, evict_every=T, old_stride=sh,
                                 capacity=capacity, threshold_total=total))
    o.prefill(K, -K, init_score=init)
    expect = replay_prefill(N, k, w, s, eff, T, c, init[0, 0], capacity, total)
    Ko, Vo, A, pos = o.export()
    assert list(pos[0, 0]) == expect
    assert o.lengths() == (len(expect), len(expect) - k - w, 0)
    np.testing.assert_array_equal(Ko[0, 0, :, 0], expect)
    np.testing.assert_array_equal(A[0, 0], init[0, 0, expect])
    if capacity:
        assert len(expect) + T <= capacity
    elif total:
        assert len(expect) <= T + k + w


def test_prefill_container_literal_cases():
    """N = 100, k = 2, w = 8, s = 5, s^ = 3, T = 10, all scores 0 (ties go to the lowest index): Alg. 2 keeps
    tokens 2, 7, ..., 87 (18 of them).  Remark 2's container of T + k + w = 20 rows has room for 10, so one more
    interval sampling leaves tokens 2, 17, ..., 77 (6).  A capacity of 25 rows leaves, after the T rows kept free
    for buffering, room for 5: two more samplings, tokens 2 and 47.  Counting new tokens only and no capacity:
    one sampling, 18 rows."""
    N, k, w, s, T, D = 100, 2, 8, 5, 10, 1
    z = np.zeros((1, 1, N, D))
    window = list(range(92, 100))

    def retained(**kw):
        o = OracleCache(OracleConfig(1, 1, 1, D, sink=k, window=w, segment=s, keep=1, evict_every=T, old_stride=0, **kw))
        o.prefill(z, z)
        return list(o.export()[3][0, 0]), o.lengths()

    pos, lens = retained(threshold_total=True)
    assert pos == [0, 1, 2, 17, 32, 47, 62, 77] + window and lens == (16, 6, 0)
    pos, lens = retained(capacity=25)
    assert pos == [0, 1, 2, 47] + window and lens == (12, 2, 0)
    pos, lens = retained(capacity=25, threshold_total=True)
    assert pos == [0, 1, 2, 47] + window and lens == (12, 2, 0)
    pos, lens = retained()
    assert pos == [0, 1] + list(range(2, 92, 5)) + window and lens == (28, 18, 0)


def test_prefill_that_cannot_fit_says_so():
    """Survivors that persist (s^ = 1) cannot be thinned: a container they do not fit is an error, not a loop."""
    from oracle.buzz_oracle import OracleError
    z = np.zeros((1, 1, 100, 1))
    o = OracleCache(OracleConfig(1, 1, 1, 1, sink=2, window=8, segment=5, keep=1, evict_every=10, old_stride=1,
                                 capacity=25))
    with pytest.raises(OracleError):
        o.prefill(z, z)


# ---------------------------------------------------------------- Alg. 1's first loops: when a prompt is sampled at all
@pytest.mark.parametrize("total", [False, True])
def test_prefill_trigger_boundary_literals(total):
    """k = 2, w = 3, s = 4, keep 1, T = 8.  With T - 1 = 7 tokens between sink and window nothing is sampled
    (12 rows stay); with exactly T = 8 the threshold is reached: two segments, 2 survivors, 7 rows; with 9 a
    ragged third segment adds one: 8 rows."""
    k, w, s, T, D = 2, 3, 4, 8, 1
    for M, expect in ((7, (12, 0, 7)), (8, (7, 2, 0)), (9, (8, 3, 0))):
        N = k + M + w
        z = np.zeros((1, 1, N, D))
        o = OracleCache(OracleConfig(1, 1, 1, D, sink=k, window=w, segment=s, keep=1, evict_every=T, old_stride=1,
                                     threshold_total=total))
        o.prefill(z, z)
        assert o.lengths() == expect, (M, o.lengths())
    # the same boundary during decoding: the eviction falls on the step that buffers the T-th token, not the next
    o = OracleCache(OracleConfig(1, 1, 1, D, sink=k, window=w, segment=s, keep=1, evict_every=T, old_stride=1,
                                 threshold_total=total))
    o.prefill(np.zeros((1, 1, k + w, D)), np.zeros((1, 1, k + w, D)))
    z = np.zeros((1, 1, D))
    sizes = []
    for _ in range(9):
        o.decode_step(z, z, z)
        sizes.append(o.lengths())
    assert sizes[6] == (12, 0, 7) and sizes[7] == (7, 2, 0) and sizes[8] == (8, 2, 1)


# ---------------------------------------------------------------- H2O-style baseline (Sec. 4.1): global top-k by accumulated score
@pytest.mark.parametrize("seed", range(8))
def test_global_topk_matches_a_library_sort(seed):
    """One segment over everything between sink and window: the survivors are the first `keep` entries of a
    stable library sort by descending score (numpy.lexsort: ties keep index order), whatever was old or new."""
    r = rng(600 + seed)
    k, w, B, T, D = int(r.integers(0, 4)), int(r.integers(0, 7)), int(r.integers(1, 12)), int(r.integers(1, 9)), 2
    N = int(r.integers(k + w + T, 90))
    K = np.zeros((1, 1, N, D)); K[0, 0, :, 0] = np.arange(N)
    score = r.integers(0, 6, size=N).astype(np.float64)
    o = OracleCache(OracleConfig(1, 1, 1, D, sink=k, window=w, segment=3, keep=B, evict_every=T, old_stride=0,
                                 auto_evict=False, global_topk=True))
    o.prefill(K, -K, init_score=score[None, None])
    pos = list(range(N))
    if N - k - w >= T:
        mid = np.arange(k, N - w)
        order = np.lexsort((mid, -score[mid]))               # primary key: score descending; secondary: index
        pos = list(range(k)) + sorted(mid[order[:B]].tolist()) + list(range(N - w, N))
    assert list(o.export()[3][0, 0]) == pos
    tok = N
    for rnd in range(3):                                     # a few rounds: old survivors compete again with new rows
        for _ in range(T):
            row = np.zeros((1, 1, D)); row[0, 0, 0] = tok
            o.decode_step(np.zeros((1, 1, D)), row, -row)
            pos.append(tok); tok += 1
        A = r.integers(0, 6, size=len(pos)).astype(np.float64)
        o.set_scores(A[None, None])
        o.evict()
        n = len(pos)
        mid = np.arange(k, n - w)
        order = np.lexsort((mid, -A[mid]))
        keep_idx = sorted(mid[order[:B]].tolist())
        kept_scores, dropped = A[keep_idx], np.delete(A[mid], [i - k for i in keep_idx])
        assert dropped.size == 0 or kept_scores.min() >= dropped.max()      # greedy: nothing evicted outranks a survivor
        pos = [pos[j] for j in list(range(k)) + keep_idx + list(range(n - w, n))]
        assert list(o.export()[3][0, 0]) == pos
        assert o.lengths() == (len(pos), min(B, n - k - w), 0)


def test_global_topk_literal_and_contrast_with_segments():
    """Scores 0 1 2 ... 19 between a sink of 1 and a window of 2 (23 tokens): the H2O-style top 4 are the last four
    middle tokens (17..20), where segments of 5 with one survivor each keep one token per hive (5, 10, 15, 20)."""
    N, k, w = 23, 1, 2
    z = np.zeros((1, 1, N, 1))
    score = np.zeros((1, 1, N)); score[0, 0, 1:21] = np.arange(20)
    h2o = OracleCache(OracleConfig(1, 1, 1, 1, sink=k, window=w, segment=5, keep=4, evict_every=1, global_topk=True))
    h2o.prefill(z, z, init_score=score)
    assert list(h2o.export()[3][0, 0]) == [0, 17, 18, 19, 20, 21, 22]
    buzz = OracleCache(OracleConfig(1, 1, 1, 1, sink=k, window=w, segment=5, keep=1, evict_every=1, old_stride=1))
    buzz.prefill(z, z, init_score=score)
    assert list(buzz.export()[3][0, 0]) == [0, 5, 10, 15, 20, 21, 22]
