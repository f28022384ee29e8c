"""Benchmark of the BUZZ decode hot path on one MI355X.

One "step" = one decode step of every layer: append, split decode attention over the retained cache,
score accumulation, and the beehive eviction whenever T tokens have been buffered.  Inputs are seeded,
synthetic and resident in HBM before the timed region starts.  Prints ONE JSON line.

The headline workload is the largest single-GPU one (`llama7b_full`: 32 layers, 33 GB of cache traffic per
step, HBM-bound).  Whatever --steps / --warmup are, the caches are first rolled forward (untimed) to the
point of the eviction cycle at which the timed steps contain ceil(steps / T) evictions, so the eviction cost
is always inside the number.  Without --workload the line also carries compact sub-records of the other
benchmark workloads (`others`), measured the same way.
"""
from __future__ import annotations

import argparse
import gc
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
DEFAULT_WORKLOAD = "llama7b_full"
# (workload, force streaming K/V loads): the sub-records of a default run
OTHERS = [("llama7b_layer", False), ("llama7b_layer", True), ("gqa8b_layer", False), ("long131k", False)]
MAX_INPUT_STEPS = 512          # distinct decode inputs per stream; longer runs cycle through them (i.i.d. draws)


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", default=None, help=f"default {DEFAULT_WORKLOAD}, plus sub-records of the others")
    ap.add_argument("--layers", type=int, default=None, help="override the workload's layer count")
    ap.add_argument("--splits", type=int, default=0, help="key-range splits per unit (0 = automatic)")
    ap.add_argument("--streaming", action="store_true",
                    help="force streaming (non-temporal) K/V loads, as a cache that is one of many layers would use")
    ap.add_argument("--device-merge", action="store_true",
                    help="merge a unit's splits through device memory even where its blocks can share a die")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-profile-pass", action="store_true")
    ap.add_argument("--no-others", action="store_true", help="no sub-records of the other workloads")
    ap.add_argument("--copy-calibration-mib", type=int, default=0,
                    help="also run the library's plain copy kernel once on this many MiB (for rocprofv3 --pmc runs: "
                         "its known size gives the scale of the byte counters)")
    ap.add_argument("--prefill-obs", type=int, default=0,
                    help="also time the prefill of one layer with this many observed prompt queries (prefill scoring; "
                         "off the decode metric) and report it as `prefill_scoring`")
    return ap.parse_args()


def make_caches(wl, layers, max_context, splits, flags):
    from paper_2410_23079_amd import FLAG_THRESHOLD_TOTAL, BuzzCache, BuzzConfig
    caches = []
    for _ in range(layers):
        c = BuzzCache(BuzzConfig(wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.dtype, wl.sink, wl.window,
                                 wl.segment, wl.keep, wl.evict_every, max_context, old_stride=wl.old_stride,
                                 flags=flags | (FLAG_THRESHOLD_TOTAL if wl.threshold_total else 0)))
        if splits:
            c.set_splits(splits)
        caches.append(c)
    return caches


def prefill_all(wl, caches, device):
    """Prefill every layer's cache from its seeded prompt; returns the median time of one layer's buzz_prefill
    (prompt scoring with the workload's n_obs, sampling, compaction; not part of the decode metric)."""
    import torch
    from workloads import prompt_inputs
    times = []
    for layer, c in enumerate(caches):
        p = prompt_inputs(wl, layer=layer, device=device)
        n_obs = min(wl.n_obs, wl.prompt)
        q_obs = p["q_obs"][:, :, p["q_obs"].shape[2] - n_obs:, :].contiguous() if n_obs else None
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        c.prefill(p["K"], p["V"], q_obs=q_obs)
        torch.cuda.synchronize()
        times.append(time.perf_counter() - t0)
        del p
    times.sort()
    return times[len(times) // 2] * 1e3


def step_views(dec):
    """Per decode-input stream, the (q, k, v) tensors of every step: slicing them inside the timed loop would
    charge ~8 us of host time per step, more than the smallest workload's whole kernel."""
    return [[(d["q"][t], d["k"][t], d["v"][t]) for t in range(d["q"].shape[0])] for d in dec]


class Runner:
    """Drives the caches of one workload step by step and knows where in the eviction cycle they are."""

    def __init__(self, wl, caches, views, out, stream):
        self.wl, self.caches, self.views, self.out, self.stream = wl, caches, views, out, stream
        self.done = 0                                   # decode steps since the prefill

    def run(self, count):
        n_in = len(self.views[0])
        for t in range(self.done, self.done + count):
            for layer, c in enumerate(self.caches):
                q, k, v = self.views[layer % len(self.views)][t % n_in]
                c.decode_step(q, k, v, self.out, self.stream)
        self.done += count

    def until_next_eviction(self):
        """Decode steps left until the automatic eviction fires (it fires at the end of that step)."""
        _, n_old, new = self.caches[0].lengths()
        have = n_old + new if self.wl.threshold_total else new
        return max(1, self.wl.evict_every - have)

    def roll_for(self, steps):
        """Untimed steps that bring the caches to the point of the eviction cycle from which the next `steps`
        steps contain ceil(steps / T) evictions, the odd one in the middle of its share of the steps: the
        eviction has to fire on step (r + 1) // 2 from here, r = steps mod T.  Returns (steps rolled, evictions
        the next `steps` steps will contain)."""
        T = self.wl.evict_every
        r = steps % T
        m = (r + 1) // 2 if r else self.until_next_eviction()   # r = 0: any alignment gives steps / T evictions
        rolled = 0
        while self.until_next_eviction() != m and rolled < 3 * T:   # (bounded: under the total-threshold reading
            self.run(1)                                             # a cycle can be shorter than m)
            rolled += 1
        u = self.until_next_eviction()
        period = T if not self.wl.threshold_total else None
        expected = (0 if u > steps else (steps - u) // period + 1) if period else None
        return rolled, expected


def measure(wl, layers, steps, warmup, splits, streaming, device, profile, copy_mib=0, device_merge=False):
    """One workload: prefill, roll, warm up, K timed steps, then (optionally) K more steps with per-kernel
    events.  Returns the measurements; frees the caches."""
    import torch
    from paper_2410_23079_amd import FLAG_AUTO_EVICT, FLAG_DEVICE_MERGE, FLAG_STREAMING
    from workloads import decode_inputs

    T = wl.evict_every
    budget = warmup + 2 * steps + 6 * T + 2            # decode steps both passes can take, rolls included
    n_streams = min(layers, 4)                         # decode inputs: a few distinct seeded streams, reused over layers
    dec = step_views([decode_inputs(wl, layer=i, device=device, steps=min(budget, MAX_INPUT_STEPS))
                      for i in range(n_streams)])
    stream = torch.cuda.current_stream().cuda_stream
    out = torch.empty(wl.batch, wl.n_q_heads, wl.head_dim, dtype=torch.float32, device=device)
    flags = FLAG_AUTO_EVICT | (FLAG_STREAMING if streaming else 0) | (FLAG_DEVICE_MERGE if device_merge else 0)
    caches = make_caches(wl, layers, wl.prompt + budget, splits, flags)
    prefill_ms = prefill_all(wl, caches, device)
    if copy_mib:
        from paper_2410_23079_amd import bench_copy
        src = torch.full((copy_mib << 20,), 7, dtype=torch.uint8, device=device)
        dst = torch.empty_like(src)
        bench_copy(dst, src)
        torch.cuda.synchronize()
        del src, dst
    run = Runner(wl, caches, dec, out, stream)

    run.run(warmup)
    rolled, timed_evictions = run.roll_for(steps)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run.run(steps)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    n_end = caches[0].lengths()[0]
    res = {"steps_per_s": steps / elapsed, "ms_per_step": elapsed / steps * 1e3, "rolled_steps": rolled,
           "prefill_ms_per_layer": prefill_ms,
           "evictions_in_timed_steps": timed_evictions, "retained_rows_end": n_end}

    # second pass: the next K steps, aligned the same way, with HIP events around every kernel (on the launch stream)
    if profile:
        run.roll_for(steps)
        for c in caches:
            c.profile(True)
        run.run(steps)
        torch.cuda.synchronize()
        prof = [c.profile_read() for c in caches]
        for c in caches:
            c.profile(False)
        launches = sum(p["attn_launches"] for p in prof)
        attn_ms = sum(p["attn_ms"] for p in prof)
        ev_ms = sum(p["evict_ms"] for p in prof) + sum(p["epilogue_ms"] for p in prof)
        evictions = sum(p["evictions"] for p in prof)
        kv_bytes = sum(p["attn_row_bytes"] for p in prof)            # sum over launches of units * n * 2 * D * e
        units = wl.batch * wl.n_kv_heads
        elem = 4 if wl.dtype == "fp32" else 2
        rows = kv_bytes / (units * 2 * wl.head_dim * elem)           # sum over launches of n
        # algorithmic bytes of the attention + score pass: K and V rows plus the fp32 score read and write
        algo_bytes = kv_bytes + units * rows * 8.0
        achieved = algo_bytes / (attn_ms * 1e-3) / 1e9 if attn_ms else 0.0
        attn_us = attn_ms * 1e3 / max(launches, 1)
        evict_us_per_step = ev_ms * 1e3 / steps / layers             # amortised, per layer
        res.update({
            "kernel": "attn_split_mfma_kernel" if (wl.group > 1 and wl.dtype != "fp32") else "attn_split_kernel",
            "achieved_gbs": achieved, "frac": achieved / HBM_PEAK_GBS, "avg_launch_us": attn_us, "launches": launches,
            "bytes_per_launch": algo_bytes / max(launches, 1),
            "evictions": evictions // layers, "evict_avg_us": ev_ms * 1e3 / max(evictions, 1),
            "evict_us_per_step": evict_us_per_step,
            "evict_share_of_step": evict_us_per_step / (attn_us + evict_us_per_step) if attn_us else 0.0,
            # what one layer's step costs beyond its kernels: launch latency and host time not hidden by the GPU
            "launch_gap_us": elapsed / steps / layers * 1e6 - attn_us - evict_us_per_step,
        })
    res["_caches"] = caches                                         # the caller may still want one (prefill scoring)
    return res


def prefill_scoring(wl, cache, n_obs, device, reps=3):
    """Time of one layer's prefill with and without scoring by the last n_obs prompt queries.  The difference is
    the two scoring kernels.  The method's own contraction is q.k for every causal (query, key) pair: 2 D flops
    per pair and query head; the kernels form every logit twice (row statistics, then probabilities), so the
    matrix cores do twice that."""
    import torch
    from workloads import prompt_inputs
    p = prompt_inputs(wl.scaled(n_obs=n_obs), device=device)
    q_obs = p["q_obs"][:, :, p["q_obs"].shape[2] - n_obs:, :].contiguous()

    def timed(q):
        cache.prefill(p["K"], p["V"], q_obs=q)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            cache.prefill(p["K"], p["V"], q_obs=q)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / reps

    with_scoring, without = timed(q_obs), timed(None)
    N = wl.prompt
    pairs = n_obs * (N - n_obs) + n_obs * (n_obs + 1) / 2             # causal (query, key) pairs per head
    flops = 2.0 * wl.head_dim * pairs * wl.batch * wl.n_q_heads       # the method's contraction, once
    dt = max(with_scoring - without, 1e-9)
    mfma = wl.dtype != "fp32"
    peak = 2500.0 if mfma else 157.3
    return {"n_obs": n_obs, "prefill_ms": with_scoring * 1e3, "prefill_without_scoring_ms": without * 1e3,
            "scoring_ms": dt * 1e3, "flops": flops, "achieved": flops / dt / 1e12, "unit": "TFLOP/s",
            "bound": "mfma" if mfma else "alu", "peak": peak, "frac": flops / dt / 1e12 / peak,
            "frac_counting_both_passes": 2.0 * flops / dt / 1e12 / peak}


def cpu_baseline(wl, budget_s=12.0):
    """The oracle as it stands, on the host cores, on a bounded sample: one layer, a subset of the (batch,
    kv-head) units, prompt scores left at zero (prefill is not part of the metric), decode steps for about
    `budget_s` seconds and at least one eviction period."""
    from oracle.buzz_oracle import OracleCache, OracleConfig
    from workloads import decode_inputs, prompt_inputs
    B = wl.batch                                       # bound host memory (fp64 copies of the prompt) to ~2 GB:
    while B > 1 and B * wl.n_kv_heads * wl.prompt * wl.head_dim * 16 > (2 << 30):
        B //= 2                                        # units are independent and identical in cost
    sub = wl.scaled(batch=B)
    p = prompt_inputs(sub, device="cpu")
    n_in = min(sub.decode_steps, MAX_INPUT_STEPS)
    d = decode_inputs(sub, device="cpu", steps=n_in)
    o = OracleCache(OracleConfig(sub.batch, sub.n_q_heads, sub.n_kv_heads, sub.head_dim, sub.sink, sub.window,
                                 sub.segment, sub.keep, sub.evict_every, sub.old_stride,
                                 threshold_total=sub.threshold_total))
    Kp, Vp = p["K"].double().numpy(), p["V"].double().numpy()
    del p
    q, k, v = (d[x].double().numpy() for x in ("q", "k", "v"))
    done, dt, t_start = 0, 0.0, time.perf_counter()
    while time.perf_counter() - t_start < budget_s or done < sub.evict_every:
        o.prefill(Kp, Vp)                               # (untimed) back to the prompt: the workload's own context lengths
        t0 = time.perf_counter()
        for t in range(sub.decode_steps):
            o.decode_step(q[t % n_in], k[t % n_in], v[t % n_in])
            done += 1
            if time.perf_counter() - t_start >= budget_s and done >= sub.evict_every:
                break
        dt += time.perf_counter() - t0
    frac = (sub.batch * sub.n_kv_heads) / (wl.batch * wl.n_kv_heads)
    steps_per_s = done / dt * frac / wl.layers          # scaled to the full batch and layer stack
    cores = int(os.environ.get("OMP_NUM_THREADS", "0")) or os.cpu_count()
    return {"value": steps_per_s, "unit": "steps/s", "cores": cores, "kind": "oracle",
            "sample": f"1 layer, {sub.batch * sub.n_kv_heads} of {wl.batch * wl.n_kv_heads} (batch, kv-head) units, "
                      f"{done} decode steps (runs of up to {sub.decode_steps} from the prompt) incl. their evictions, {dt:.1f} s; "
                      f"scaled by units and {wl.layers} layer(s)"}


def release(res):
    import torch
    for c in res.pop("_caches", []):
        c.close()
    gc.collect()
    torch.cuda.empty_cache()


def default_counts(wl, steps, warmup):
    w = warmup if warmup is not None else min(64, wl.decode_steps // 8)
    s = steps if steps is not None else wl.decode_steps - w
    return s, w


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (the path shards without communication over layers, "
              "batch and kv heads); run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    from workloads import get_workload

    wl = get_workload(args.workload or DEFAULT_WORKLOAD)
    layers = args.layers or wl.layers
    steps, warmup = default_counts(wl, args.steps, args.warmup)
    device = "cuda:0"
    torch.cuda.set_device(0)

    res = measure(wl, layers, steps, warmup, args.splits, args.streaming, device, not args.no_profile_pass,
                  copy_mib=args.copy_calibration_mib, device_merge=args.device_merge)
    roofline = None
    extra = {}
    if not args.no_profile_pass:
        traffic = traffic_parts = None                             # HBM bytes per launch from rocprofv3 --pmc runs
        tpath = os.path.join(ROOT, "profiles", "hbm_traffic.json")
        if os.path.exists(tpath):
            t = json.load(open(tpath)).get(wl.name)
            if t and layers == wl.layers and not args.splits:
                traffic = t["fetch_bytes_per_launch"] + t["write_bytes_per_launch"]
                traffic_parts = {"fetch_bytes": t["fetch_bytes_per_launch"], "write_bytes": t["write_bytes_per_launch"],
                                 "source": t["source"]}
        roofline = {"bound": "hbm", "kernel": res["kernel"], "achieved": res["achieved_gbs"], "peak": HBM_PEAK_GBS,
                    "unit": "GB/s", "frac": res["frac"], "avg_launch_us": res["avg_launch_us"],
                    "launches": res["launches"], "bytes_per_launch": res["bytes_per_launch"], "traffic": traffic,
                    "traffic_parts": traffic_parts}
        extra = {k: res[k] for k in ("evictions", "evict_avg_us", "evict_us_per_step", "evict_share_of_step",
                                     "launch_gap_us")}
        extra["step_bytes_over_peak_over_step_time"] = (res["bytes_per_launch"] * layers / HBM_PEAK_GBS / 1e9) \
            / (res["ms_per_step"] * 1e-3)
    extra["evictions_in_timed_steps"] = res["evictions_in_timed_steps"]
    extra["rolled_steps"] = res["rolled_steps"]
    extra["prefill_ms_per_layer"] = res["prefill_ms_per_layer"]
    if args.prefill_obs:
        extra["prefill_scoring"] = prefill_scoring(wl, res["_caches"][0], min(args.prefill_obs, wl.prompt), device)
    n_end = res["retained_rows_end"]
    release(res)

    others = None
    if args.workload is None and not args.no_others:
        others = []
        for name, streaming in OTHERS:
            owl = get_workload(name)
            osteps, owarm = default_counts(owl, None, None)
            r = measure(owl, owl.layers, osteps, owarm, 0, streaming, device, True)
            release(r)
            others.append({"workload": name, "kv_loads": "streaming" if streaming else "auto", "steps": osteps,
                           "warmup": owarm, **{k: (round(v, 4) if isinstance(v, float) else v) for k, v in r.items()}})

    base = None if args.no_cpu_baseline else cpu_baseline(wl)
    line = {
        "metric": "decode_steps_per_sec_incl_eviction", "value": res["steps_per_s"], "unit": "steps/s", "n_gpus": 1,
        "steps": steps, "warmup": warmup, "ms_per_step": res["ms_per_step"], "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "kv_dtype": wl.dtype, "data": "synthetic",
        "tokens_per_s": res["steps_per_s"] * wl.batch,
        "config": {"workload": wl.name, "layers": layers, "batch": wl.batch, "n_q_heads": wl.n_q_heads,
                   "n_kv_heads": wl.n_kv_heads, "head_dim": wl.head_dim, "prompt": wl.prompt, "sink": wl.sink,
                   "window": wl.window, "segment": wl.segment, "keep": wl.keep, "evict_every": wl.evict_every,
                   "old_stride": wl.old_stride, "threshold_total": wl.threshold_total, "retained_rows_end": n_end,
                   "splits": args.splits or "auto", "kv_loads": "streaming" if args.streaming else "auto",
                   "split_merge": "device" if args.device_merge else "auto"},
        "roofline": roofline, "cpu_baseline": base,
    }
    line.update(extra)
    if others is not None:
        line["others"] = others
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
