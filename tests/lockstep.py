"""Lock-step comparison of the HIP library with the CPU oracle on one workload (test helper).

Protocol.  Both sides receive the same tensors.  Attention outputs and accumulated scores are compared
numerically at every step.  The retained index sets must be bit-exact, and because a selection decided
by fp32 scores can legitimately differ from one decided by fp64 scores at a near-tie, the selection on
both sides runs on the same fp32 score array: before every eviction the oracle adopts the scores the
GPU exported (after they have been checked against its own), then both evict, then the retained
positions, K rows and V rows are compared exactly.  The prompt scores are handled the same way: they
are computed once by the library's prefill scoring (a cache configured so that nothing is evicted),
checked against the oracle's, and handed to both sides as starting scores.
"""
from __future__ import annotations

import numpy as np
import torch

from oracle.buzz_oracle import OracleCache, OracleConfig
from paper_2410_23079_amd import (FLAG_AUTO_EVICT, FLAG_CACHED, FLAG_DETERMINISTIC, FLAG_DEVICE_MERGE, FLAG_GLOBAL_TOPK, FLAG_INTERVAL_NEW, FLAG_LOG_N,
                                 FLAG_STREAMING, FLAG_THRESHOLD_TOTAL, BuzzCache, BuzzConfig)
from workloads import Workload

OUT_TOL = 2e-3      # contract: max |o - o_ref| / max |o_ref| per (batch, head) vector
OUT_EXPECT = 1e-4   # what fp32 accumulation over exactly widened inputs should reach (regression guard)
SCORE_TOL = 1e-4    # relative to max(1, |score|)
REPRO_TOL = 1e-5    # two runs without FLAG_DETERMINISTIC: same rows summed in another order


def buzz_config(wl: Workload, flags=0, max_context=None, **over) -> BuzzConfig:
    kw = dict(batch=wl.batch, n_q_heads=wl.n_q_heads, n_kv_heads=wl.n_kv_heads, head_dim=wl.head_dim,
              kv_dtype=wl.dtype, sink=wl.sink, window=wl.window, segment=wl.segment, keep=wl.keep,
              evict_every=wl.evict_every, old_stride=wl.old_stride, flags=flags,
              max_context=max_context or wl.max_context)
    kw.update(over)
    return BuzzConfig(**kw)


def oracle_config(wl: Workload, n_units: int, **over) -> OracleConfig:
    kw = dict(batch=n_units, n_q_heads=wl.group, n_kv_heads=1, head_dim=wl.head_dim, sink=wl.sink,
              window=wl.window, segment=wl.segment, keep=wl.keep, evict_every=wl.evict_every,
              old_stride=wl.old_stride, auto_evict=False)
    kw.update(over)
    return OracleConfig(**kw)


def unit_slices(t: torch.Tensor, units, heads_per_unit: int):
    """[B,H,...] -> float64 numpy [len(units), heads_per_unit, ...] for the chosen (batch, kv-head) units."""
    rows = [t[b, h * heads_per_unit:(h + 1) * heads_per_unit] for b, h in units]
    return torch.stack(rows).double().cpu().numpy()


def rel_err(got: np.ndarray, ref: np.ndarray) -> float:
    """max over vectors (last axis) of max|got-ref| / max|ref|."""
    num = np.abs(got - ref).max(axis=-1)
    den = np.maximum(np.abs(ref).max(axis=-1), 1e-30)
    return float((num / den).max())


def score_err(got: np.ndarray, ref: np.ndarray) -> float:
    """max |got-ref| / max(1, |ref|) over the finite entries; 0 for empty arrays.  Where the reference is NaN or
    infinite (planted starting scores stay that way: NaN + p = NaN, inf + p = inf) the other side must hold the
    same, else the error is infinite."""
    if got.size == 0:
        return 0.0
    fin = np.isfinite(ref)
    odd_same = np.array_equal(np.isnan(got), np.isnan(ref)) and np.array_equal(got[~fin & ~np.isnan(ref)],
                                                                                ref[~fin & ~np.isnan(ref)])
    if not odd_same:
        return float("inf")
    if not fin.any():
        return 0.0
    return float((np.abs(got[fin] - ref[fin]) / np.maximum(1.0, np.abs(ref[fin]))).max())


def gpu_prompt_scores(wl: Workload, prompt, n_obs: int, flags: int = 0):
    """Prompt scores from the library's own prefill scoring, with a window so large nothing is evicted."""
    N = prompt["K"].shape[2]
    cfg = buzz_config(wl, flags=flags, max_context=N + 1, sink=0, window=N + 1, keep=1, old_stride=1)
    c = BuzzCache(cfg)
    q_obs = prompt["q_obs"][:, :, prompt["q_obs"].shape[2] - n_obs:, :].contiguous() if n_obs else None
    c.prefill(prompt["K"], prompt["V"], q_obs=q_obs)
    _, _, score, pos = c.export()
    assert (pos.cpu().numpy() == np.arange(N)).all()
    c.close()
    return score


def run_lockstep(wl: Workload, prompt, decode, units=None, steps=None, n_obs=None, splits=0,
                 check_auto=True, capacity=0, log_n=False, threshold_total=None, deterministic=True,
                 interval_new=False, kv_loads=None, device_merge=False, plant=None, global_topk=False):
    """Returns a dict of the worst errors seen; raises AssertionError on any parity failure.
    kv_loads: None (the library decides), "streaming" or "cached" (forces the K/V load flavour).
    device_merge: split partials always travel through device memory (else through one die's L2 where possible).
    plant: callable that edits the fp32 prompt scores [B,Hkv,N] in place before both sides start from them."""
    G, D = wl.group, wl.head_dim
    N = prompt["K"].shape[2]
    steps = decode["q"].shape[0] if steps is None else steps
    n_obs = min(wl.n_obs, N) if n_obs is None else n_obs
    if units is None:
        units = [(b, h) for b in range(wl.batch) for h in range(wl.n_kv_heads)]
    U = len(units)
    uidx_b = torch.tensor([b for b, _ in units])
    uidx_h = torch.tensor([h for _, h in units])
    stats = dict(out=0.0, score=0.0, prefill_score=0.0, evictions=0)
    if threshold_total is None:
        threshold_total = wl.threshold_total
    vflags = ((FLAG_LOG_N if log_n else 0) | (FLAG_THRESHOLD_TOTAL if threshold_total else 0)
              | (FLAG_DETERMINISTIC if deterministic else 0) | (FLAG_INTERVAL_NEW if interval_new else 0)
              | {None: 0, "streaming": FLAG_STREAMING, "cached": FLAG_CACHED}[kv_loads]
              | (FLAG_DEVICE_MERGE if device_merge else 0) | (FLAG_GLOBAL_TOPK if global_topk else 0))
    okw = dict(log_n=log_n, threshold_total=threshold_total, interval_new=interval_new, global_topk=global_topk)

    # ---- prompt scores: library vs oracle, then shared
    Kp, Vp = unit_slices(prompt["K"], units, 1), unit_slices(prompt["V"], units, 1)
    o_probe = OracleCache(oracle_config(wl, U, sink=0, window=N + 1, old_stride=1, log_n=log_n))
    q_obs_u = unit_slices(prompt["q_obs"][:, :, prompt["q_obs"].shape[2] - n_obs:, :], units, G) if n_obs else None
    o_probe.prefill(Kp, Vp, q_obs=q_obs_u)
    ref_ps = o_probe.export()[2][:, 0]                                   # [U,N]
    ps = gpu_prompt_scores(wl, prompt, n_obs, FLAG_LOG_N if log_n else 0)   # [B,Hkv,N] fp32 on GPU
    got_ps = ps[uidx_b, uidx_h].double().cpu().numpy()
    err = score_err(got_ps, ref_ps)
    stats["prefill_score"] = err
    assert err <= SCORE_TOL, f"prefill scores off by {err}"
    if plant is not None:
        plant(ps)
        got_ps = ps[uidx_b, uidx_h].double().cpu().numpy()

    # ---- both sides start from the same fp32 prompt scores
    gpu = BuzzCache(buzz_config(wl, flags=vflags, max_context=N + steps, capacity=capacity))
    if splits:
        gpu.set_splits(splits)
    gpu.prefill(prompt["K"], prompt["V"], init_score=ps)
    ora = OracleCache(oracle_config(wl, U, capacity=capacity, **okw))
    ora.prefill(Kp, Vp, init_score=got_ps[:, None, :])
    auto = None
    if check_auto and plant is None:                          # (the automatic cache scores its own prompt)
        auto = BuzzCache(buzz_config(wl, flags=FLAG_AUTO_EVICT | vflags, max_context=N + steps, capacity=capacity))
        if splits:
            auto.set_splits(splits)
        q_obs = prompt["q_obs"][:, :, prompt["q_obs"].shape[2] - n_obs:, :].contiguous() if n_obs else None
        auto.prefill(prompt["K"], prompt["V"], q_obs=q_obs)                # scoring + sampling in one call

    def compare_state(tag):
        Kg, Vg, Sg, Pg = gpu.export()
        Ko, Vo, So, Po = ora.export()
        assert gpu.lengths() == ora.lengths(), f"{tag}: sizes {gpu.lengths()} vs {ora.lengths()}"
        pg = Pg[uidx_b, uidx_h].cpu().numpy()
        assert (pg == Po[:, 0]).all(), f"{tag}: retained positions differ"
        assert (Kg[uidx_b, uidx_h].double().cpu().numpy() == Ko[:, 0]).all(), f"{tag}: K rows differ"
        assert (Vg[uidx_b, uidx_h].double().cpu().numpy() == Vo[:, 0]).all(), f"{tag}: V rows differ"
        sg = Sg[uidx_b, uidx_h].double().cpu().numpy()
        e = score_err(sg, So[:, 0])
        stats["score"] = max(stats["score"], e)
        assert e <= SCORE_TOL, f"{tag}: scores off by {e}"
        return sg

    compare_state("after prefill")
    out = torch.empty(wl.batch, wl.n_q_heads, D, dtype=torch.float32, device=prompt["K"].device)
    out_auto = torch.empty_like(out)
    T = wl.evict_every
    for t in range(steps):
        q, k, v = decode["q"][t], decode["k"][t], decode["v"][t]
        gpu.decode_step(q, k, v, out)
        ref = ora.decode_step(unit_slices(q, units, G), unit_slices(k, units, 1), unit_slices(v, units, 1))
        got = unit_slices(out, units, G)
        e = rel_err(got, ref)
        stats["out"] = max(stats["out"], e)
        assert e <= OUT_TOL, f"step {t}: output error {e} > {OUT_TOL}"
        assert e <= OUT_EXPECT, f"step {t}: output error {e} above what fp32 accumulation should give"
        if auto is not None:
            auto.decode_step(q, k, v, out_auto)
            if deterministic:
                assert torch.equal(out, out_auto), f"step {t}: auto-evict cache diverged from the manual one"
            else:                                          # same rows, summed in a timing-dependent order
                e2 = rel_err(unit_slices(out_auto, units, G), got.astype(np.float64))
                assert e2 <= REPRO_TOL, f"step {t}: two runs of the default mode differ by {e2}"
        _, n_old_now, new_now = gpu.lengths()
        if (n_old_now + new_now if threshold_total else new_now) >= T:
            sg = compare_state(f"step {t} before eviction")
            ora.set_scores(sg[:, None, :])                                 # selection runs on the GPU's fp32 scores
            gpu.evict()
            ora.evict()
            compare_state(f"step {t} after eviction")
            stats["evictions"] += 1
    compare_state("end")
    if auto is not None:
        a, b = gpu.export(), auto.export()
        assert gpu.lengths() == auto.lengths()
        for i, (x, y) in enumerate(zip(a, b)):               # K, V, score, pos
            if i == 2 and not deterministic:
                assert torch.allclose(x, y, rtol=REPRO_TOL, atol=REPRO_TOL), "scores of two default-mode runs differ"
            else:
                assert torch.equal(x, y), "auto-evict cache differs from the manually evicted one"
        auto.close()
    gpu.close()
    return stats


def run_free(wl: Workload, prompt, decode, units=None, steps=None):
    """Free run: GPU (fp32 scores) and oracle (fp64 scores) each evict on their OWN accumulated scores.

    Both start from the same prompt scores.  At every eviction the retained position sets are compared; the
    first difference must be a near-tie: every row one side kept and the other did not has, in the oracle's
    scores, a counterpart on the other side within a relative gap of 1e-5.  Returns a dict with the number of
    evictions that agreed and, if the runs parted, the largest gap found at the parting eviction."""
    G, D = wl.group, wl.head_dim
    N = prompt["K"].shape[2]
    steps = wl.decode_steps if steps is None else steps
    if units is None:
        units = [(b, h) for b in range(wl.batch) for h in range(wl.n_kv_heads)]
    U = len(units)
    uidx_b = torch.tensor([b for b, _ in units]); uidx_h = torch.tensor([h for _, h in units])
    n_obs = min(wl.n_obs, N)
    ps = gpu_prompt_scores(wl, prompt, n_obs)
    gpu = BuzzCache(buzz_config(wl, flags=FLAG_THRESHOLD_TOTAL if wl.threshold_total else 0, max_context=N + steps))
    gpu.prefill(prompt["K"], prompt["V"], init_score=ps)
    ora = OracleCache(oracle_config(wl, U, threshold_total=wl.threshold_total))
    ora.prefill(unit_slices(prompt["K"], units, 1)[:, 0][:, None], unit_slices(prompt["V"], units, 1)[:, 0][:, None],
                init_score=ps[uidx_b, uidx_h].double().cpu().numpy()[:, None, :])
    out = torch.empty(wl.batch, wl.n_q_heads, D, dtype=torch.float32, device=prompt["K"].device)
    res = dict(agreed=0, parted_at=None, gap=0.0)
    for t in range(steps):
        q, k, v = decode["q"][t], decode["k"][t], decode["v"][t]
        gpu.decode_step(q, k, v, out)
        ora.decode_step(unit_slices(q, units, G), unit_slices(k, units, 1), unit_slices(v, units, 1))
        _, n_old_now, new_now = gpu.lengths()
        if (n_old_now + new_now if wl.threshold_total else new_now) < wl.evict_every:
            continue
        _, _, A_before, P_before = ora.export()
        gpu.evict()
        ora.evict()
        Pg = gpu.export()[3][uidx_b, uidx_h].cpu().numpy()
        Po = ora.export()[3][:, 0]
        if (Pg == Po).all():
            res["agreed"] += 1
            continue
        res["parted_at"] = t
        for u in range(U):                                   # every one-sided row needs a near-tied counterpart
            score_of = dict(zip(P_before[u, 0].tolist(), A_before[u, 0].tolist()))
            g_only = sorted(set(Pg[u].tolist()) - set(Po[u].tolist()))
            o_only = sorted(set(Po[u].tolist()) - set(Pg[u].tolist()))
            assert len(g_only) == len(o_only), "the two runs kept different numbers of rows"
            for a_pos, b_pos in zip(g_only, o_only):         # same segment, in order
                sa, sb = score_of[a_pos], score_of[b_pos]
                gap = abs(sa - sb) / max(abs(sa), abs(sb), 1e-30)
                res["gap"] = max(res["gap"], gap)
                assert gap <= 1e-5, f"step {t}: rows {a_pos} / {b_pos} differ by {gap:.2e}, not a near-tie"
        break
    gpu.close()
    return res
