"""Benchmark of the BUZZ decode hot path on one MI355X.

One "step" = one decode step of every layer: append, split decode attention over the retained cache,
score accumulation, and the beehive eviction whenever T tokens have been buffered.  Inputs are seeded,
synthetic and resident in HBM before the timed region starts.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", default="llama7b_layer")
    ap.add_argument("--layers", type=int, default=None, help="override the workload's layer count")
    ap.add_argument("--splits", type=int, default=0, help="key-range splits per unit (0 = automatic)")
    ap.add_argument("--streaming", action="store_true",
                    help="force streaming (non-temporal) K/V loads, as a cache that is one of many layers would use")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-profile-pass", action="store_true")
    ap.add_argument("--copy-calibration-mib", type=int, default=0,
                    help="also run the library's plain copy kernel once on this many MiB (for rocprofv3 --pmc runs: "
                         "its known size gives the scale of the byte counters)")
    ap.add_argument("--pipe-probe", action="store_true",
                    help="instead of a workload: time the matrix / vector instruction mix of the prompt-scoring "
                         "kernels alone and print how far the two pipes overlap")
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
    import torch
    from workloads import prompt_inputs
    for layer, c in enumerate(caches):
        p = prompt_inputs(wl, layer=layer, device=device)
        n_obs = min(wl.n_obs, wl.prompt)
        q_obs = p["q_obs"][:, :, p["q_obs"].shape[2] - n_obs:, :].contiguous() if n_obs else None
        c.prefill(p["K"], p["V"], q_obs=q_obs)
        torch.cuda.synchronize()
        del p


def step_views(dec):
    """Per decode-input stream, the (q, k, v) tensors of every step: slicing them inside the timed loop would
    charge ~8 us of host time per step, more than config 1's whole kernel."""
    return [[(d["q"][t], d["k"][t], d["v"][t]) for t in range(d["q"].shape[0])] for d in dec]


def run_steps(caches, views, out, first, count, stream):
    for t in range(first, first + count):
        for layer, c in enumerate(caches):
            q, k, v = views[layer % len(views)][t]
            c.decode_step(q, k, v, out, stream)


def prefill_scoring(wl, cache, n_obs, device, reps=3):
    """Time of one layer's prefill with and without scoring by the last n_obs prompt queries.  The difference is
    the two scoring kernels; their work is 2 x 2 D flops per (query, visible key) pair and query head."""
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
    flops = 4.0 * wl.head_dim * pairs * wl.batch * wl.n_q_heads
    dt = max(with_scoring - without, 1e-9)
    mfma = wl.dtype != "fp32"
    peak = 2500.0 if mfma else 157.3
    return {"n_obs": n_obs, "prefill_ms": with_scoring * 1e3, "prefill_without_scoring_ms": without * 1e3,
            "scoring_ms": dt * 1e3, "flops": flops, "achieved": flops / dt / 1e12, "unit": "TFLOP/s",
            "bound": "mfma" if mfma else "alu", "peak": peak, "frac": flops / dt / 1e12 / peak}


def cpu_baseline(wl, budget_s=20.0):
    """The oracle as it stands, on the host cores, on a bounded sample: one layer, every (batch, kv-head) unit,
    prompt scores left at zero (prefill is not part of the metric), decode steps until the time budget is used."""
    import numpy as np
    from oracle.buzz_oracle import OracleCache, OracleConfig, _load
    from workloads import decode_inputs, prompt_inputs
    B = wl.batch                                       # bound host memory (fp64 copies of the prompt) to ~4 GB:
    while B > 1 and B * wl.n_kv_heads * wl.prompt * wl.head_dim * 16 > (4 << 30):
        B //= 2                                        # units are independent and identical in cost
    sub = wl.scaled(batch=B)
    p = prompt_inputs(sub, device="cpu")
    steps = sub.decode_steps
    d = decode_inputs(sub, device="cpu", steps=steps)
    o = OracleCache(OracleConfig(sub.batch, sub.n_q_heads, sub.n_kv_heads, sub.head_dim, sub.sink, sub.window,
                                 sub.segment, sub.keep, sub.evict_every, sub.old_stride,
                                 threshold_total=sub.threshold_total))
    o.prefill(p["K"].double().numpy(), p["V"].double().numpy())
    del p
    q, k, v = (d[x].double().numpy() for x in ("q", "k", "v"))
    done, t0 = 0, time.perf_counter()
    while done < steps and (time.perf_counter() - t0 < budget_s or done < sub.evict_every):
        o.decode_step(q[done], k[done], v[done])
        done += 1
    dt = time.perf_counter() - t0
    frac = (sub.batch * sub.n_kv_heads) / (wl.batch * wl.n_kv_heads)
    steps_per_s = done / dt * frac / wl.layers          # scaled to the full batch and layer stack
    cores = int(os.environ.get("OMP_NUM_THREADS", "0")) or os.cpu_count()
    return {"value": steps_per_s, "unit": "steps/s", "cores": cores, "kind": "oracle",
            "sample": f"1 layer, {sub.batch * sub.n_kv_heads} of {wl.batch * wl.n_kv_heads} (batch, kv-head) units, "
                      f"{done} decode steps incl. {done // sub.evict_every} evictions, {dt:.1f} s; "
                      f"scaled by units and {wl.layers} layer(s)"}


def pipe_probe(iters=20000, clock_ghz=2.4):
    """Cycles (at the nominal clock) a SIMD needs per 16 x 64 tile of the prompt-scoring instruction mix: its 16
    MFMAs alone, its 48 vector instructions alone, both; 1, 2 and 3 waves per SIMD (256, 512, 768 blocks)."""
    import torch
    from paper_2410_23079_amd import bench_pipes
    torch.cuda.set_device(0)
    out = torch.empty(768 * 256, dtype=torch.float32, device="cuda:0")
    res = {}
    for blocks in (256, 512, 768):
        waves = blocks * 4 / 1024
        for name, work in (("mfma", 1), ("vector", 2), ("both", 3)):
            bench_pipes(work, blocks, 100, out)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            bench_pipes(work, blocks, iters, out)
            e1.record()
            e1.synchronize()
            res[f"{name}_cycles_per_tile_{int(waves)}_waves_per_simd"] = round(
                e0.elapsed_time(e1) * 1e-3 * clock_ghz * 1e9 / (iters * waves), 1)
    return res


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (the path shards without communication over layers, "
              "batch and kv heads); run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2410_23079_amd import FLAG_AUTO_EVICT, FLAG_STREAMING
    from workloads import decode_inputs, get_workload

    if args.pipe_probe:
        print(json.dumps({"pipe_probe": pipe_probe()}), flush=True)
        return
    wl = get_workload(args.workload)
    layers = args.layers or wl.layers
    warmup = args.warmup if args.warmup is not None else min(64, wl.decode_steps // 8)
    steps = args.steps if args.steps is not None else wl.decode_steps - warmup
    total = warmup + steps
    device = "cuda:0"
    torch.cuda.set_device(0)

    n_streams = min(layers, 4)                          # decode inputs: a few distinct seeded streams, reused over layers
    dec = step_views([decode_inputs(wl, layer=i, device=device, steps=total) for i in range(n_streams)])
    stream = torch.cuda.current_stream().cuda_stream
    out = torch.empty(wl.batch, wl.n_q_heads, wl.head_dim, dtype=torch.float32, device=device)
    flags = FLAG_AUTO_EVICT | (FLAG_STREAMING if args.streaming else 0)
    caches = make_caches(wl, layers, wl.prompt + total, args.splits, flags)
    prefill_all(wl, caches, device)

    if args.copy_calibration_mib:
        from paper_2410_23079_amd import bench_copy
        src = torch.full((args.copy_calibration_mib << 20,), 7, dtype=torch.uint8, device=device)
        dst = torch.empty_like(src)
        bench_copy(dst, src)
        torch.cuda.synchronize()
        del src, dst
    run_steps(caches, dec, out, 0, warmup, stream)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run_steps(caches, dec, out, warmup, steps, stream)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    n_end = caches[0].lengths()[0]

    # second pass, same steps, with HIP events around every kernel (on the launch stream)
    roofline = None
    extra = {}
    if not args.no_profile_pass:
        prefill_all(wl, caches, device)
        run_steps(caches, dec, out, 0, warmup, stream)
        for c in caches:
            c.profile(True)
        run_steps(caches, dec, out, warmup, steps, stream)
        torch.cuda.synchronize()
        prof = [c.profile_read() for c in caches]
        for c in caches:
            c.profile(False)
        launches = sum(p["attn_launches"] for p in prof)
        attn_ms = sum(p["attn_ms"] for p in prof)
        flush_ms = sum(p["epilogue_ms"] for p in prof)
        ev_ms = sum(p["evict_ms"] for p in prof)
        evictions = sum(p["evictions"] for p in prof)
        kv_bytes = sum(p["attn_row_bytes"] for p in prof)            # sum over launches of units * n * 2 * D * e
        units = wl.batch * wl.n_kv_heads
        elem = 4 if wl.dtype == "fp32" else 2
        rows = kv_bytes / (units * 2 * wl.head_dim * elem)           # sum over launches of n
        # algorithmic bytes of the attention + score pass: K and V rows plus the fp32 score read and write
        algo_bytes = kv_bytes + units * rows * 8.0
        achieved = algo_bytes / (attn_ms * 1e-3) / 1e9 if attn_ms else 0.0
        traffic = None                                             # HBM bytes per launch from rocprofv3 --pmc runs
        tpath = os.path.join(ROOT, "profiles", "hbm_traffic.json")
        if os.path.exists(tpath):
            t = json.load(open(tpath)).get(wl.name)
            if t and layers == wl.layers and not args.splits:
                traffic = {"fetch_bytes": t["fetch_bytes_per_launch"], "write_bytes": t["write_bytes_per_launch"],
                           "source": t["source"]}
        kname = "attn_split_mfma_kernel" if (wl.group > 1 and wl.dtype != "fp32") else "attn_split_kernel"
        roofline = {"bound": "hbm", "kernel": kname, "achieved": achieved, "peak": HBM_PEAK_GBS,
                    "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                    "avg_launch_us": attn_ms * 1e3 / max(launches, 1), "launches": launches,
                    "bytes_per_launch": algo_bytes / max(launches, 1), "traffic": traffic}
        extra = {"evictions": evictions,
                 "evict_avg_us": (ev_ms + flush_ms) * 1e3 / max(evictions, 1),
                 "evict_time_over_attn_time": (ev_ms + flush_ms) / attn_ms if attn_ms else 0.0,
                 "step_bytes_over_peak_over_step_time": (algo_bytes / max(launches, 1) * layers / HBM_PEAK_GBS / 1e9)
                                                        / (elapsed / steps)}

    if args.prefill_obs:
        extra["prefill_scoring"] = prefill_scoring(wl, caches[0], min(args.prefill_obs, wl.prompt), device)

    base = None if args.no_cpu_baseline else cpu_baseline(wl)
    line = {
        "metric": "decode_steps_per_sec_incl_eviction", "value": steps / elapsed, "unit": "steps/s", "n_gpus": 1,
        "steps": steps, "warmup": warmup, "ms_per_step": elapsed / steps * 1e3, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": f"{wl.dtype} storage, f32 accumulate", "data": "synthetic",
        "tokens_per_s": steps / elapsed * wl.batch,
        "config": {"workload": wl.name, "layers": layers, "batch": wl.batch, "n_q_heads": wl.n_q_heads,
                   "n_kv_heads": wl.n_kv_heads, "head_dim": wl.head_dim, "prompt": wl.prompt, "sink": wl.sink,
                   "window": wl.window, "segment": wl.segment, "keep": wl.keep, "evict_every": wl.evict_every,
                   "old_stride": wl.old_stride, "threshold_total": wl.threshold_total, "retained_rows_end": n_end, "splits": args.splits or "auto",
                   "kv_loads": "streaming" if args.streaming else "auto"},
        "roofline": roofline, "cpu_baseline": base,
    }
    line.update(extra)
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
