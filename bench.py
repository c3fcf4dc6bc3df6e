#!/usr/bin/env python3
"""Benchmark of the embedding-cache step on one MI355X.

A "step" is one pass of the whole path over one synthetic minibatch: het_lookup (dedup, probe,
stale refresh, miss fill, gather) followed by het_update (dedup, gradient coalescing, optimizer
apply with clock increment, policy trim with write-back).  The workload is configuration 2
(1M ids, dim 64, 4096 x 26 lookups per batch, Zipf 1.05, LFU cache of 100k rows, s = 100,
Adagrad, backing table in HBM).  Inputs are resident in HBM before the timed region.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 2] [--no-cpu-baseline]

Prints one JSON line: lookups+updates per second, plus the roofline position of the dominant
kernel (timed with HIP events inside this script) and the CPU oracle timed on a bounded sample.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0       # MI355X published HBM3E bandwidth

TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic.json")


def measured_traffic(kernel, config, build_id):
    """HBM bytes per launch (fetch + write) of `kernel` on workload `config`, from the rocprofv3
    FETCH_SIZE / WRITE_SIZE counter runs recorded in profiles/hbm_traffic.json (scaled there by a
    256 MiB device copy of the same run).  The record names the build it was measured on; for any
    other build of the library, or a workload that was not measured, the answer is None."""
    try:
        with open(TRAFFIC_FILE) as fh:
            rec = json.load(fh)
    except (OSError, ValueError):
        return None
    entry = rec.get(f"config{config}", {})
    if entry.get("build_id") != build_id:
        return None
    return entry.get("bytes_per_launch", {}).get(kernel)


def cpu_model():
    try:
        with open("/proc/cpuinfo") as fh:
            for line in fh:
                if line.startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown CPU"


def algorithmic_bytes(w, c):
    """HBM bytes one step must move, from device counters `c` (per-step averages):
    ids read twice, out written, cached rows read for the gather, grads read, apply read+write
    of value (+accumulator), both ends of every fill / refresh / write-back, keys-clocks-policy
    metadata and the victim scan."""
    R = 4 * w.dim
    Q = 2 if w.optimizer else 1
    n, U = w.n, c["unique_lookup"]
    rows_io = w.n_grad_rows * R
    moved = c["miss"] + c["stale_dirty"] + c["evicted_dirty"]
    P = w.capacity + w.n
    return (16 * n + rows_io + U * R + rows_io + 2 * U * Q * R + 2 * moved * Q * R + 32 * U + 8 * P)


def kernel_bytes(w, c, name):
    """Algorithmic bytes of one launch of the kernels the roofline line may name."""
    R = 4 * w.dim
    Q = 2 if w.optimizer else 1
    U = c["unique_lookup"]
    if name == "apply_kernel":      # grads read, value (+accumulator) read and written, index arrays
        return w.n_grad_rows * R + 2 * U * Q * R + 4 * w.n + 12 * U
    if name == "fill_gather_kernel":
        # cached rows read once per key, out written, refreshed rows read and written with their
        # optimizer state (and the fetched ones where the table is behind the host link: with the
        # table in HBM the update reads a missed key's row from the table itself), index arrays
        moved = c["stale"] + (c["miss"] if w.backing == "host" else 0)
        return U * R + w.n_grad_rows * R + 2 * moved * Q * R + 8 * w.n + 4 * U
    return None


def policy_study(args, w, dev):
    """Miss rate against cache size and policy (Section 5.2, Figure 8) on the synthetic stream of
    config `w`: one JSON line with a row per (size, policy)."""
    import torch
    from paper_2112_07221_amd import hetcache as hc
    from paper_2112_07221_amd import workloads as wl
    W, K = args.warmup, args.steps
    ids = torch.from_numpy(wl.IdStream(w).batches(W + K)).to(dev)
    grads = torch.from_numpy(wl.grad_pool(w)).to(dev)
    out = torch.empty(w.n_grad_rows, w.dim, device=dev)
    offsets = torch.from_numpy(wl.bag_offsets(w)).to(dev) if w.pooled else None
    table = wl.table_init(w)
    rows = []
    for frac in (0.03, 0.05, 0.10, 0.15):
        for policy, pname in ((wl.LRU, "LRU"), (wl.LFU, "LFU"), (wl.LFU_LIGHT, "LFU-light (cap 16)")):
            Wt = torch.from_numpy(table).to(dev)
            At = torch.zeros_like(Wt) if w.optimizer else None
            Cg = torch.zeros(w.vocab, dtype=torch.int32, device=dev)
            cache = hc.HetCache(int(w.vocab * frac), w.dim, w.s, policy, w.n, w.optimizer, w.eps)
            cache.attach_backing(Wt, At, Cg, hc.BACKING_HBM)

            def step(t):
                if t == 0 and W + K > 1:
                    cache.prefetch(ids[1])
                if t + 2 < W + K:
                    cache.prefetch(ids[t + 2])
                if w.pooled:
                    cache.lookup_pooled(ids[t], offsets, out)
                    cache.update_pooled(ids[t], offsets, grads[t % w.grad_pool], w.lr)
                else:
                    cache.lookup(ids[t], out)
                    cache.update(ids[t], grads[t % w.grad_pool], w.lr)
            for t in range(W):
                step(t)
            before = cache.stats()["total"]
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for t in range(W, W + K):
                step(t)
            torch.cuda.synchronize()
            ms = (time.perf_counter() - t0) * 1e3 / K
            tot = cache.stats()["total"]
            miss = tot["miss"] - before["miss"]
            uniq = (tot["unique"] - before["unique"]) / 2.0
            rows.append({"cache_frac": frac, "policy": pname, "miss_rate_per_unique": miss / uniq,
                         "miss_rate_per_lookup": miss / (K * w.n), "ms_per_step": ms})
            cache.close()
            del Wt, At, Cg
    print(json.dumps({"study": "miss rate against cache size and policy", "config": w.index, "steps": K, "warmup": W,
                      "rows": rows}))


def pattern_study(args, w, dev):
    """What plain kernels with the access patterns of the path's heavy steps reach on this GPU at
    this config's sizes (het_profile_rows): a streaming copy, a gather of the batch's rows, and the
    optimizer step's read-modify-write of the batch's distinct rows with and without their
    gradients.  One JSON line."""
    import torch
    from paper_2112_07221_amd import hetcache as hc
    from paper_2112_07221_amd import workloads as wl
    rng = np.random.default_rng(20211207)
    batch = wl.IdStream(w).batches(3)[2]
    n, D, R = int(w.n), int(w.dim), 4 * int(w.dim)
    U = int(np.unique(batch).size)
    P = int(w.capacity + w.n)
    V = int(min(w.vocab, 4_000_000))            # (a table of this many rows stands for the global one: far beyond the caches)
    Q = 2 if w.optimizer else 1
    src = torch.randn(V, D, device=dev)
    outb = torch.empty(n, D, device=dev)
    x = torch.randn(P, D, device=dev)
    a = torch.rand(P, D, device=dev) if w.optimizer else None
    grads = torch.randn(n, D, device=dev)
    as_dev = lambda v: torch.from_numpy(np.ascontiguousarray(v, dtype=np.int32)).to(dev)
    ids_zipf = as_dev(np.sort(batch % V))                         # the batch's ids in sorted order, as the gather reads them
    ids_scattered = as_dev(rng.choice(V, size=n, replace=False))  # as many distinct rows, anywhere
    slots = as_dev(np.sort(rng.choice(P, size=U, replace=False))) # the batch's distinct keys sit in U of the P slots
    rows = []

    def add(name, nbytes, ms):
        rows.append({"pattern": name, "bytes": nbytes, "us": ms * 1e3, "GBps": nbytes / (ms * 1e-3) / 1e9,
                     "frac_of_8TBps": nbytes / (ms * 1e-3) / 8e12})

    big = torch.empty(1 << 20, 64, device=dev)                    # 256 MiB
    add("streaming copy, 256 MiB", 2 * big.numel() * 4, hc.profile_rows(hc.PATTERN_COPY, torch.empty_like(big), src=big, n=big.shape[0]))
    del big
    add(f"streaming copy of n = {n} rows", 2 * n * R, hc.profile_rows(hc.PATTERN_COPY, outb, src=src, n=n))
    add("gather of n distinct rows from anywhere in the table", 2 * n * R,
        hc.profile_rows(hc.PATTERN_GATHER, outb, src=src, idx=ids_scattered))
    add(f"gather of the batch's n rows in sorted order ({U} distinct; bytes counted as the path does: U read, n written)", (U + n) * R,
        hc.profile_rows(hc.PATTERN_GATHER, outb, src=src, idx=ids_zipf))
    add(f"update of U = {U} distinct cached rows ({'row and accumulator' if Q == 2 else 'row'} read and written)", 2 * U * Q * R,
        hc.profile_rows(hc.PATTERN_UPDATE, x, a=a, idx=slots))
    for per in (2, 3):
        gidx = as_dev(rng.permutation(n)[: U * per] if U * per <= n else rng.integers(0, n, U * per))
        add(f"update of U rows, each with {per} gradient rows from anywhere in the batch", (2 * U * Q + U * per) * R,
            hc.profile_rows(hc.PATTERN_UPDATE, x, a=a, src=grads, idx=slots, gidx=gidx, per=per))
    shuffled = as_dev(rng.permutation(slots.cpu().numpy()))   # the path's order: by key, which says nothing about the slot
    add("update of U distinct cached rows, taken in random order of slot", 2 * U * Q * R,
        hc.profile_rows(hc.PATTERN_UPDATE, x, a=a, idx=shuffled))
    gidx = as_dev(rng.permutation(n)[: U * 2] if U * 2 <= n else rng.integers(0, n, U * 2))
    add("update of U rows in random order of slot, each with 2 gradient rows from anywhere in the batch", (2 * U * Q + U * 2) * R,
        hc.profile_rows(hc.PATTERN_UPDATE, x, a=a, src=grads, idx=shuffled, gidx=gidx, per=2))
    print(json.dumps({"study": "plain kernels with the path's access patterns", "config": w.index, "n": n, "unique": U,
                      "dim": D, "slots": P, "build_id": hc.build_id(), "rows": rows}))


def trace_kernels(args, w, dev):
    """Where the two heavy kernels' time goes: per-workgroup time stamps (het_profile_trace) of one
    lookup and one update after `--warmup` steps, summarised per role and per phase.  One JSON line."""
    import torch
    from paper_2112_07221_amd import hetcache as hc
    from paper_2112_07221_amd import workloads as wl
    T = args.warmup + 8
    table = wl.table_init(w)
    ids = torch.from_numpy(wl.IdStream(w).batches(T)).to(dev)
    grads = torch.from_numpy(wl.grad_pool(w)).to(dev)
    Wt = torch.from_numpy(table).to(dev)
    At = torch.zeros_like(Wt) if w.optimizer else None
    Cg = torch.zeros(w.vocab, dtype=torch.int32, device=dev)
    offsets = torch.from_numpy(wl.bag_offsets(w)).to(dev) if w.pooled else None
    out = torch.empty(w.n_grad_rows, w.dim, device=dev)
    cache = hc.HetCache(w.capacity, w.dim, w.s, w.policy, w.n, w.optimizer, w.eps)
    cache.attach_backing(Wt, At, Cg, hc.BACKING_HBM)
    cap = 1 << 15
    kernels = {"apply_kernel": {1: "carried sort stage", 2: "select stage", 3: "id check", 4: "update tile"},
               "fill_gather_kernel": {1: "carried sort stage", 2: "fetch", 3: "bookkeeping of the fetched keys", 4: "select stage",
                                      5: "gather", 6: "host link"}}
    rec = {k: torch.zeros(cap, hc.TRACE_WORDS, dtype=torch.int64, device=dev) for k in kernels}

    def step(t):
        if t == 0:
            cache.prefetch(ids[1])
        if t + 2 < T:
            cache.prefetch(ids[t + 2])
        if w.pooled:
            cache.lookup_pooled(ids[t], offsets, out)
            cache.update_pooled(ids[t], offsets, grads[t % w.grad_pool], w.lr)
        else:
            cache.lookup(ids[t], out)
            cache.update(ids[t], grads[t % w.grad_pool], w.lr)

    for t in range(args.warmup):
        step(t)
    q = lambda v, p: float(np.percentile(v, p))
    reps = []
    for r in range(3):
        torch.cuda.synchronize()
        for k in kernels:
            rec[k].zero_()
            cache.profile_trace(rec[k], k)
        step(args.warmup + r)
        torch.cuda.synchronize()
        one = {}
        for k, roles in kernels.items():
            cache.profile_trace(None, k)
            a = rec[k].cpu().numpy()
            used = a[:, 6] > 0
            k0 = a[used, 0].min()
            us = lambda x: (x - k0) / 100.0                   # 100 MHz counter
            d = {"kernel_span_us": float(us(a[used, 5].max())), "workgroups": int(used.sum()), "roles": {}}
            for role, name in roles.items():
                m = a[:, 6] == role
                if not m.any():
                    continue
                st, en = us(a[m, 0]), us(a[m, 5])
                d["roles"][name] = {"workgroups": int(m.sum()), "start_us_p50_max": [q(st, 50), float(st.max())],
                                    "end_us_p50_p90_max": [q(en, 50), q(en, 90), float(en.max())],
                                    "duration_us_p50_p90_max": [q(en - st, 50), q(en - st, 90), float((en - st).max())],
                                    "sum_of_durations_us": float((en - st).sum())}
            if k == "apply_kernel":
                d["tile_phases_us"] = {}
                wk = a[a[:, 6] == 4]
                for i, name in ((1, "tile loaded, segments listed"), (2, "short segments"), (3, "long segments"),
                                (4, "barrier before the border runs"), (5, "border runs finished")):
                    ok = (wk[:, i] > 0) & (wk[:, i - 1] > 0)
                    if ok.any():
                        dd = (wk[ok, i] - wk[ok, i - 1]) / 100.0
                        d["tile_phases_us"][name] = {"workgroups": int(ok.sum()), "p50": q(dd, 50), "p90": q(dd, 90), "max": float(dd.max())}
            one[k] = d
        reps.append(one)
    cache.close()
    print(json.dumps({"study": "time stamps inside the lookup's second kernel and the update's kernel", "config": w.index,
                      "build_id": hc.build_id(), "warmup": args.warmup, "steps": reps}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=900)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--config", type=int, default=2)
    ap.add_argument("--profile-steps", type=int, default=50)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-prefetch", action="store_true", help="do not announce the next batch's ids")
    ap.add_argument("--prefetch-order", choices=("before", "between", "after"), default="before",
                    help="announce the next ids before the lookup, between lookup and update, or after the update")
    ap.add_argument("--no-cache", action="store_true",
                    help="context figure: the same step without the cache (reads and writes go to the global table)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 256 MiB device copy five times (a known-size reference for HBM counters)")
    ap.add_argument("--cpu-iters", type=int, default=0, help="oracle iterations to time (0 = auto)")
    ap.add_argument("--policy-study", action="store_true",
                    help="instead of the benchmark: miss rate and step time of the chosen config for cache sizes of "
                         "3, 5, 10 and 15 %% of the vocabulary under LRU, LFU and light-weight LFU (the experiment of the paper's "
                         "Figure 8, and the claim of its Section 4.3)")
    ap.add_argument("--trace-kernels", action="store_true",
                    help="instead of the benchmark: per-workgroup time stamps inside fill_gather_kernel and apply_kernel "
                         "(table in HBM), summarised per role and phase")
    ap.add_argument("--pattern-study", action="store_true",
                    help="instead of the benchmark: what plain copy, gather and read-modify-write kernels reach at the "
                         "chosen config's sizes (reference points beside the streaming peak)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding, no collectives); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2112_07221_amd import hetcache as hc
    from paper_2112_07221_amd import workloads as wl

    w = wl.WORKLOADS[args.config]
    dev = torch.device("cuda:0")
    if args.policy_study:
        policy_study(args, w, dev)
        return
    if args.pattern_study:
        pattern_study(args, w, dev)
        return
    if args.trace_kernels:
        trace_kernels(args, w, dev)
        return
    K, W = args.steps, args.warmup
    total = W + K + args.profile_steps

    # ---- inputs, staged on the device before anything is timed
    table = wl.table_init(w)
    ids_np = wl.IdStream(w).batches(total)
    grads_np = wl.grad_pool(w)
    ids = torch.from_numpy(ids_np).to(dev)
    grads = torch.from_numpy(grads_np).to(dev)
    host = w.backing == "host"
    if host:
        Wt = torch.from_numpy(table).pin_memory()
        At = torch.zeros_like(Wt).pin_memory() if w.optimizer else None
        Cg = torch.zeros(w.vocab, dtype=torch.int32).pin_memory()
    else:
        Wt = torch.from_numpy(table).to(dev)
        At = torch.zeros_like(Wt) if w.optimizer else None
        Cg = torch.zeros(w.vocab, dtype=torch.int32, device=dev)
    offsets = torch.from_numpy(wl.bag_offsets(w)).to(dev) if w.pooled else None
    out = torch.empty(w.n_grad_rows, w.dim, device=dev)

    cache = hc.HetCache(w.capacity, w.dim, w.s, hc.POLICY_NONE if args.no_cache else w.policy, w.n, w.optimizer, w.eps)
    cache.attach_backing(Wt, At, Cg, hc.BACKING_PINNED_HOST if host else hc.BACKING_HBM)

    def step(t):
        # the ids of batch t+2 are announced (the kernels of this step and the next carry their
        # sort); lookup t; update t
        pf = not args.no_prefetch and t + 1 < total
        if pf and args.prefetch_order == "before":
            # two ahead: a sort has more stages than one step has kernels to carry them
            if t == 0:
                cache.prefetch(ids[1])
            if t + 2 < total:
                cache.prefetch(ids[t + 2])
        if w.pooled:
            cache.lookup_pooled(ids[t], offsets, out)
        else:
            cache.lookup(ids[t], out)
        if pf and args.prefetch_order == "between":
            cache.prefetch(ids[t + 1])
        if w.pooled:
            cache.update_pooled(ids[t], offsets, grads[t % w.grad_pool], w.lr)
        else:
            cache.update(ids[t], grads[t % w.grad_pool], w.lr)
        if pf and args.prefetch_order == "after":
            cache.prefetch(ids[t + 1])

    if args.calibrate_copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---- warm-up (cold cache), then the timed region
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for t in range(W):
        step(t)
    torch.cuda.synchronize()
    warm_ms = (time.perf_counter() - t0) * 1e3 / max(W, 1)
    before = cache.stats()["total"]

    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    wall0 = time.perf_counter()
    e0.record()
    enqueue_ms = 0.0
    K_host = max(1, min(K, 100))                 # host cost of a step: over the first steps, before the launch queue fills and the host waits for the GPU
    for t in range(W, W + K):
        step(t)
        if t + 1 == W + K_host:
            enqueue_ms = (time.perf_counter() - wall0) * 1e3
    e1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - wall0) * 1e3
    gpu_ms = e0.elapsed_time(e1)
    ms_per_step = max(gpu_ms, wall_ms) / K
    after = cache.stats()
    assert after["error_bits"] == 0, "device error bits set during the run"
    tot = after["total"]
    per_step = {k: (tot[k] - before[k]) / K for k in tot}
    per_step["unique_lookup"] = per_step["unique"] / 2.0      # counted by lookup and by update

    # ---- per-kernel durations, HIP events around every launch (outside the timed region)
    roofline, per_step_us, kern = None, {}, {}
    if args.profile_steps > 0:
        cache.profile_begin()
        for t in range(W + K, total):
            step(t)
        prof = cache.profile_end()
        kern = {k: {"avg_us": ms * 1e3 / cnt, "launches_per_step": cnt / args.profile_steps}
                for k, (ms, cnt) in prof.items()}
        per_step_us = {k: v["avg_us"] * v["launches_per_step"] for k, v in kern.items()}
        candidates = [k for k in per_step_us if kernel_bytes(w, per_step, k) is not None]
        dominant = max(candidates, key=lambda k: per_step_us[k])
        dom_bytes = kernel_bytes(w, per_step, dominant)
        achieved = dom_bytes / (kern[dominant]["avg_us"] * 1e-6) / 1e9
        roofline = {"bound": "hbm", "kernel": dominant, "achieved": achieved, "peak": HBM_PEAK_GBPS,
                    "unit": "GB/s", "frac": achieved / HBM_PEAK_GBPS,
                    "traffic": measured_traffic(dominant, w.index, hc.build_id()),
                    "bytes_per_launch": dom_bytes, "avg_us": kern[dominant]["avg_us"]}
    step_bytes = algorithmic_bytes(w, per_step)

    result = {
        "metric": "embedding lookups+updates/sec and achieved HBM GB/s (% peak), 1 MI355X",
        "value": 2.0 * w.n / (ms_per_step * 1e-3),
        "unit": "lookups+updates/s",
        "n_gpus": 1, "steps": K, "warmup": W, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"config {w.index} ({w.name}): vocab {w.vocab}, dim {w.dim}, "
                               f"{w.batch}x{w.width} ids/batch, Zipf {w.alpha}, cache {w.capacity} "
                               f"{'LFU' if w.policy else 'LRU'}, s={w.s}, "
                               f"{'Adagrad' if w.optimizer else 'SGD'}, backing {w.backing}"
                               + (" -- WITHOUT the cache (context figure)" if args.no_cache else ""),
                   "ids_per_step": w.n, "unique_per_step": per_step["unique_lookup"],
                   "miss_per_step": per_step["miss"], "stale_per_step": per_step["stale"],
                   "evicted_dirty_per_step": per_step["evicted_dirty"],
                   "warmup_ms_per_step": warm_ms, "host_enqueue_ms_per_step": enqueue_ms / K_host},
        "step_hbm": {"algorithmic_bytes": step_bytes,
                     "achieved_GBps": step_bytes / (ms_per_step * 1e-3) / 1e9,
                     "frac_of_peak": step_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBPS},
        "roofline": roofline,
        "build_id": hc.build_id(),
        "kernel_launches_per_step": round(sum(v["launches_per_step"] for v in kern.values()), 2) if per_step_us else None,
        "kernels_us_per_step": {k: round(v, 2) for k, v in sorted(per_step_us.items(), key=lambda x: -x[1])},
    }
    if host:
        link = (per_step["miss"] + per_step["stale_dirty"] + per_step["evicted_dirty"]) * 4 * w.dim \
            * (2 if w.optimizer else 1)
        if args.no_cache:       # every row of the gather and both ways of every updated row cross the link
            link = (w.n_grad_rows * (w.width if w.pooled else 1) + 2 * per_step["unique_lookup"] * (2 if w.optimizer else 1)) * 4 * w.dim
        result["host_link"] = {"bytes_per_step": link, "achieved_GBps": link / (ms_per_step * 1e-3) / 1e9}

    # ---- CPU oracle on a bounded sample of the same stream (reported baseline, not a target)
    if not args.no_cpu_baseline:
        from oracle.het_oracle import Oracle
        o = Oracle(w.capacity, w.dim, w.s, w.policy, w.n, w.optimizer, w.eps, table)
        offs = wl.bag_offsets(w) if w.pooled else None
        n_cpu = args.cpu_iters or min(total, 200)
        budget_s = 20.0
        done = 0
        c0 = time.perf_counter()
        for t in range(n_cpu):
            if w.pooled:
                o.lookup_pooled(ids_np[t], offs)
                o.update_pooled(ids_np[t], offs, grads_np[t % w.grad_pool], w.lr)
            else:
                o.lookup(ids_np[t])
                o.update(ids_np[t], grads_np[t % w.grad_pool], w.lr)
            done += 1
            if time.perf_counter() - c0 > budget_s:
                break
        cpu_s = time.perf_counter() - c0
        result["cpu_baseline"] = {
            "value": 2.0 * w.n * done / cpu_s, "unit": "lookups+updates/s", "cores": 1,
            "kind": "oracle",
            "sample": f"first {done} iterations of the same stream from a cold cache, fp64 oracle, "
                      f"{cpu_s:.1f} s on one host core (of {os.cpu_count()} visible; {cpu_model()})"}
    cache.close()
    print(json.dumps(result))


if __name__ == "__main__":
    main()
