#!/usr/bin/env python3
"""Benchmark of the GPU-resident hot path: hot-embedding lookups/s for forward +
backward + sparse SGD on hot-only mini-batches, and achieved HBM GB/s against the
MI355X roofline, next to the CPU oracle timed on the host.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 1..5]

One GPU only.  Prints ONE JSON line.  Setup (profile -> cutoff -> hot tables ->
partition into hot mini-batches) runs through the same library and is reported as
per-stage throughput; the timed region is K steps of fae_embbag_fwd +
fae_embbag_bwd_sgd cycling over distinct hot mini-batches resident in HBM.
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

HBM_PEAK_GBPS = 8000.0  # MI355X HBM3E, published


def log(*a):
    print("[bench]", *a, file=sys.stderr, flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--config", type=int, default=3, help="workload 1..5 (default 3: 26 tables, dim 64, batch 16384)")
    ap.add_argument("--also", type=str, default="5",
                    help="comma list of further workloads reported under other_workloads (default 5; '' = none)")
    ap.add_argument("--batches", type=int, default=0, help="distinct hot mini-batches to cycle over (0 = per workload)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--cpu-seconds", type=float, default=10.0)
    ap.add_argument("--set", action="append", default=[], help="library option name=value (ablation)")
    ap.add_argument("--graph", action="store_true",
                    help="capture each step into a HIP graph and time the replays (same kernels, fewer launches)")
    ap.add_argument("--presort", choices=["auto", "fused", "side", "none", "ahead"], default="auto",
                    help="where the backward's sort runs: in the forward's launch (fused; needs one-hot tables "
                         "and at most 16384 samples), on the side stream, inside fae_embbag_bwd_sgd, or one step "
                         "ahead on the side stream (the next batch's sort beside this batch's forward and "
                         "backward).  auto: fused where the shape allows, else ahead for steps of up to 4 M lookups")
    args = ap.parse_args()
    if args.graph and args.presort == "ahead":
        print("bench.py: --graph captures one stream; --presort ahead uses two", file=sys.stderr)
        sys.exit(2)
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    line = run_workload(args, args.config, args.steps, args.warmup, with_cpu=not args.no_cpu)
    others = []
    for c in [int(x) for x in args.also.split(",") if x.strip()]:
        if c == args.config:
            continue
        # fewer steps for the long-step workloads: keep the whole run within a couple of minutes
        k = args.steps if c != 5 else max(10, args.steps // 10)
        o = run_workload(args, c, k, max(3, args.warmup // 5), with_cpu=False)
        others.append({key: o[key] for key in ("value", "unit", "steps", "ms_per_step", "config", "roofline")})
    line["other_workloads"] = others
    print(json.dumps(line), flush=True)


def run_workload(args, cfg_id, n_steps, n_warmup, with_cpu):
    import torch
    from paper_2103_00686_amd import binding as B
    from paper_2103_00686_amd import synth as S
    from paper_2103_00686_amd.hotpath import HotBatch, HotPath

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda", 0)
    if args.graph and torch.cuda.current_stream() == torch.cuda.default_stream():
        torch.cuda.set_stream(torch.cuda.Stream())     # capture needs a stream of its own
    w = S.workload(cfg_id, "full")
    nt, D = w.n_tables, w.dim
    n_batches = args.batches or {1: 32, 2: 32, 3: 32, 4: 16, 5: 4}[cfg_id]
    hp = HotPath(w.rows, D, 0)
    for kv in args.set:
        k, v = kv.split("=")
        B.fae_set_option(hp.ctx, k, int(v))
    stages = {}

    def timed(fn):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        r = fn()
        torch.cuda.synchronize()
        return r, time.perf_counter() - t0

    # ---- a1: profile the sampled stream, chunk by chunk ---------------------------
    chunk = min(w.profile_samples, 1 << 18)
    # counters and code objects exist before the clock starts: one untimed call on a few samples, then zeroed counters
    ch = S.make_chunk(w, 0, 0, min(1024, w.profile_samples), device=dev)
    hp.profile(B.Batch(ch.n_samples, ch.indices, ch.offsets, ch.n_lookups))
    hp.sync()
    hp.alloc_counts()
    del ch
    t_prof, n_prof_lookups = 0.0, 0
    for first in range(0, w.profile_samples, chunk):
        n = min(chunk, w.profile_samples - first)
        ch = S.make_chunk(w, 0, first, n, device=dev)
        b = B.Batch(n, ch.indices, ch.offsets, ch.n_lookups)
        _, dt = timed(lambda: hp.profile(b))
        t_prof += dt
        n_prof_lookups += sum(ch.n_lookups)
        del ch, b
    hp.sync()
    stages["profile_lookups_per_s"] = n_prof_lookups / t_prof
    stages["profile_lookups"] = n_prof_lookups
    log(f"{w.name}: profiled {n_prof_lookups} lookups in {t_prof*1e3:.2f} ms")

    # ---- a2: cutoff ----------------------------------------------------------------
    if w.hot_rule == "cutoff":
        H = [w.cutoff] * nt
        n_hot, dt = timed(lambda: hp.count_hot(H))
        c = None
    else:
        (c, H, n_hot), dt = timed(lambda: hp.choose_cutoff(w.budget_bytes, w.small_table_bytes))
    stages["cutoff_rows_per_s"] = sum(w.rows) / dt
    log(f"cutoff c={c} hot rows={sum(n_hot)} ({sum(n_hot)*D*4/2**30:.3f} GiB) in {dt*1e3:.2f} ms")

    # ---- a3 + a4: classify, remap, hot tables (procedural weights) -------------------
    _, dt = timed(lambda: hp.build(H, n_hot, seed=w.seed))
    stages["build_rows_per_s"] = sum(w.rows) / dt
    log(f"built hot tables in {dt*1e3:.2f} ms")

    # ---- a5: hot mini-batches --------------------------------------------------------
    batches = []
    t_part, n_part_lookups = 0.0, 0
    if w.conditional_hot:
        for i in range(n_batches):
            ch = S.make_chunk(w, 100 + i, 0, w.batch, device=dev, hot_remap=hp.remap)
            b = B.Batch(w.batch, ch.indices, ch.offsets, ch.n_lookups)
            (hs, cs, hb), dt = timed(lambda: hp.partition(b))
            t_part += dt
            n_part_lookups += sum(ch.n_lookups)
            assert hb.n_samples == w.batch
            batches.append(hb)
    elif cfg_id == 1:
        for i in range(n_batches):   # each step works on the hot subset of one 1024-sample batch
            ch = S.make_chunk(w, 100 + i, 0, w.batch, device=dev)
            b = B.Batch(w.batch, ch.indices, ch.offsets, ch.n_lookups)
            (hs, cs, hb), dt = timed(lambda: hp.partition(b))
            t_part += dt
            n_part_lookups += sum(ch.n_lookups)
            batches.append(hb)
    else:
        first, span = 0, 1 << 19
        while len(batches) < n_batches and first < (1 << 26):
            ch = S.make_chunk(w, 100, first, span, device=dev)
            b = B.Batch(span, ch.indices, ch.offsets, ch.n_lookups)
            (hs, cs, hb), dt = timed(lambda: hp.partition(b))
            t_part += dt
            n_part_lookups += sum(ch.n_lookups)
            for k in range(hb.n_samples // w.batch):
                if len(batches) < n_batches:
                    sl = hb.slice(k * w.batch, w.batch)
                    batches.append(HotBatch(sl.n_samples, [s.clone() for s in sl.slots], sl.offsets, sl.n_lookups))
            log(f"partitioned samples [{first},{first+span}): {hb.n_samples} hot; {len(batches)} hot batches so far")
            first += span
            del ch, b, hb
    stages["partition_lookups_per_s"] = n_part_lookups / max(t_part, 1e-9)
    assert batches, "no hot batch could be formed"

    # ---- step inputs resident in HBM ---------------------------------------------------
    gouts = [S.upstream_grads(w, 200 + i, hb.n_samples, device=dev) for i, hb in enumerate(batches)]
    outs = [torch.empty((hb.n_samples, nt, D), dtype=torch.float32, device=dev) for hb in batches]
    ws_need = max(B.fae_bwd_workspace_bytes(hp.hot_tables, hb.n_samples, hb.n_lookups) for hb in batches)
    hp._workspace("bwd", ws_need)
    steps_fn, presort = hp.prepare_steps(batches, gouts, outs, w.lr, presort=args.presort, single_stream=args.graph)

    # accounting per batch: lookups, bags, distinct rows
    acct = []
    for hb in batches:
        NL = sum(hb.n_lookups)
        NB = 0
        n_csr = 0
        U = 0
        for s, o in zip(hb.slots, hb.offsets):
            U += int(torch.unique(s).numel())
            if o is None:
                NB += hb.n_samples
            else:
                NB += int((o[1:] > o[:-1]).sum())
                n_csr += 1
        acct.append(dict(NL=NL, NB=NB, U=U, S=hb.n_samples, n_csr=n_csr))
    mean = lambda k: sum(a[k] for a in acct) / len(acct)
    NL, NB, U, Sm = mean("NL"), mean("NB"), mean("U"), mean("S")
    n_csr = acct[0]["n_csr"]
    off_bytes = 4 * (Sm + 1) * n_csr
    bytes_fwd = 4 * NL + off_bytes + 4 * D * U + 4 * D * Sm * nt
    bytes_bwd = 4 * NL + off_bytes + 4 * D * NB + 8 * D * U
    per_lookup_bytes = (4 * NL + off_bytes + 4 * D * NL + 4 * D * Sm * nt) + (4 * NL + off_bytes + 4 * D * NL + 8 * D * U)
    log(f"{len(batches)} hot batches: {NL:.0f} lookups, {NB:.0f} bags, {U:.0f} distinct rows per step")

    # ---- timed region ----------------------------------------------------------------
    nb = len(steps_fn)
    eager_fn = steps_fn
    if args.graph:
        for fn in steps_fn:
            fn()
        torch.cuda.synchronize()
        # one graph holds the whole cycle of hot batches; step i of the timed loop replays it when
        # i is the first batch of a cycle, so K steps need K rounded up to whole cycles of launches
        cycle = torch.cuda.CUDAGraph()
        with torch.cuda.graph(cycle, stream=torch.cuda.current_stream()):
            for fn in steps_fn:
                fn()
        if n_steps % nb or n_warmup % nb:
            n_steps, n_warmup = max(nb, n_steps // nb * nb), n_warmup // nb * nb
            log(f"graph mode: whole cycles of {nb} batches only -> {n_steps} steps, {n_warmup} warm-up")
        steps_fn = [cycle.replay] + [lambda: None] * (nb - 1)
    for i in range(n_warmup):
        steps_fn[i % nb]()
    torch.cuda.synchronize()
    hp.sync()
    t0 = time.perf_counter()
    for i in range(n_steps):
        steps_fn[i % nb]()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    hp.sync()
    lookups_done = sum(acct[i % nb]["NL"] for i in range(n_steps))
    value = lookups_done / elapsed
    ms_per_step = elapsed / n_steps * 1e3
    log(f"{n_steps} steps in {elapsed*1e3:.1f} ms: {ms_per_step*1e3:.1f} us/step, {value/1e9:.3f} G lookups/s")

    # ---- per-kernel pass (HIP events on the library's stream, same steps) -------------
    B.fae_timing_enable(hp.ctx, True)
    B.fae_timing_reset(hp.ctx)
    k_steps = min(n_steps, 200)
    for i in range(k_steps):
        eager_fn[i % nb]()
    torch.cuda.synchronize()
    kern = {}
    for k in range(B.FAE_K_COUNT):
        ms, n = B.fae_timing_read(hp.ctx, k)
        if n:
            kern[B.fae_kernel_name(k)] = dict(avg_us=ms / n * 1e3, launches_per_step=n / k_steps, us_per_step=ms / k_steps * 1e3)
    B.fae_timing_enable(hp.ctx, False)
    alg = {  # algorithmic bytes per launch
        "fwd": bytes_fwd,
        "bwd_reduce": 8 * NL + 4 * D * NB + 8 * D * U,
        "fwd_sort": bytes_fwd + 12 * NL,
        "sort_scatter": 16 * NL,
        "sort_hist": 4 * NL,
        "bwd_keys": 12 * NL + off_bytes,
        "lds_sort": 12 * NL,
    }
    cand = {k: v for k, v in kern.items() if k in alg}
    dom = max(cand, key=lambda k: cand[k]["us_per_step"])
    dom_gbps = alg[dom] / (kern[dom]["avg_us"] * 1e-6) / 1e9
    roofline = {"bound": "hbm", "kernel": dom, "achieved": round(dom_gbps, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": round(dom_gbps / HBM_PEAK_GBPS, 4), "traffic": None,
                "avg_launch_us": round(kern[dom]["avg_us"], 2), "alg_bytes_per_launch": int(alg[dom]),
                "measured": f"HIP events around every launch, separate pass of {k_steps} steps of the same loop",
                "step_compulsory_bytes": int(bytes_fwd + bytes_bwd),
                "step_frac": round((bytes_fwd + bytes_bwd) / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                "per_lookup_GBps": round(per_lookup_bytes / (ms_per_step * 1e-3) / 1e9, 1),
                "kernels_us_per_step": {k: round(v["us_per_step"], 2) for k, v in kern.items()}}

    # ---- what a plain streaming copy reaches on this device (1 GiB read + 1 GiB write) ------
    src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
    dst = torch.empty_like(src)
    for _ in range(3):
        B.fae_copy_probe(hp.ctx, dst, src)
    B.fae_timing_enable(hp.ctx, True)
    B.fae_timing_reset(hp.ctx)
    for _ in range(10):
        B.fae_copy_probe(hp.ctx, dst, src)
    ms, n = B.fae_timing_read(hp.ctx, 13)
    B.fae_timing_enable(hp.ctx, False)
    copy_gbps = 2 * src.numel() * 4 / (ms / n * 1e-3) / 1e9
    roofline["copy_ceiling_GBps"] = round(copy_gbps, 1)
    sink = torch.zeros(4, dtype=torch.float32, device=dev)
    for _ in range(3):
        B.fae_read_probe(hp.ctx, src, sink)
    B.fae_timing_enable(hp.ctx, True)
    B.fae_timing_reset(hp.ctx)
    for _ in range(10):
        B.fae_read_probe(hp.ctx, src, sink)
    ms, n = B.fae_timing_read(hp.ctx, 17)
    B.fae_timing_enable(hp.ctx, False)
    roofline["read_ceiling_GBps"] = round(src.numel() * 4 / (ms / n * 1e-3) / 1e9, 1)
    roofline["frac_of_copy_ceiling"] = round(dom_gbps / copy_gbps, 4)
    roofline["step_frac_of_copy_ceiling"] = round((bytes_fwd + bytes_bwd) / (ms_per_step * 1e-3) / 1e9 / copy_gbps, 4)
    del src, dst

    # ---- steps around the path: sampled hot-size estimate, embedding synchronisation -------
    chunks = [S.sample_chunks(w, z, 1024, 35) for z in range(nt)]
    hp.estimate_hot(H, chunks, 1024, 0.999)
    (est, _), dt = timed(lambda: hp.estimate_hot(H, chunks, 1024, 0.999))
    stages["estimate_call_us"] = dt * 1e6
    stages["estimate_rel_err"] = (sum(e["rows"] for e in est) - sum(n_hot)) / max(sum(n_hot), 1)
    stages["estimate_ci_rel_halfwidth"] = sum(e["half_rows"] for e in est) / max(sum(n_hot), 1)
    if w.hot_rule != "cutoff":
        (c_s, H_s, _), dt = timed(lambda: hp.choose_cutoff_sampled(w.budget_bytes, chunks, 1024, 0.999, w.small_table_bytes))
        stages["cutoff_sampled_ms"] = dt * 1e3
        stages["cutoff_sampled_c"] = c_s
    if sum(w.rows) * D * 4 <= (64 << 30):    # full tables that fit beside the hot set (contents do not matter here)
        full = [torch.empty((r, D), dtype=torch.float32, device=dev) for r in w.rows]
        sync_bytes = sum(n_hot) * (2 * D * 4 + 4)
        for name, fn in (("sync_to_full_GBps", hp.sync_to_full), ("sync_from_full_GBps", hp.sync_from_full)):
            fn(full)
            B.fae_timing_enable(hp.ctx, True)
            B.fae_timing_reset(hp.ctx)
            for _ in range(5):
                fn(full)
            ms, n = B.fae_timing_read(hp.ctx, 15)
            B.fae_timing_enable(hp.ctx, False)
            stages[name] = sync_bytes / (ms / n * 1e-3) / 1e9
        stages["sync_bytes"] = sync_bytes
        del full

    # ---- the oracle on the host, bounded sample ----------------------------------------
    cpu = None
    if with_cpu:
        cpu = cpu_baseline(hp, batches[0], gouts[0], w, args.cpu_seconds)

    line = {
        "metric": "hot-embedding lookups/sec (fwd+bwd+SGD)", "value": value, "unit": "lookups/s",
        "n_gpus": 1, "steps": n_steps, "warmup": n_warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": w.name, "config_index": cfg_id, "tables": nt, "dim": D, "batch": w.batch,
                   "zipf_s": w.zipf_s, "hot_rows": int(sum(hp.n_hot)), "hot_bytes": int(sum(hp.n_hot)) * D * 4,
                   "cutoff_c": c, "lookups_per_step": NL, "distinct_rows_per_step": U, "hot_batches": nb, "launch": "hip graph replay" if args.graph else "eager", "presort": presort,
                   "profile_samples": w.profile_samples},
        "roofline": roofline, "cpu_baseline": cpu, "stages": {k: float(f"{v:.4g}") for k, v in stages.items()},
    }
    # measured HBM traffic of the dominant kernel, if a counter summary for it is committed
    roofline["traffic"] = committed_traffic(cfg_id, dom)
    # measured HBM traffic of the whole step: committed per-launch figures of every kernel the step
    # launches, times launches per step, over the step time measured here (null if a kernel has none)
    per = {k: committed_traffic(cfg_id, k) for k in kern if k not in ("fill",)}
    if per and all(v is not None for v in per.values()):
        tb = sum(per[k] * kern[k]["launches_per_step"] for k in per)
        roofline["step_traffic_bytes"] = int(tb)
        roofline["step_traffic_frac"] = round(tb / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4)
    else:
        roofline["step_traffic_bytes"] = roofline["step_traffic_frac"] = None
    del steps_fn, batches, gouts, outs, hp
    torch.cuda.empty_cache()
    return line


def committed_traffic(cfg_id, kernel):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 --pmc summary (FETCH_SIZE and
    WRITE_SIZE runs, each scaled by what the same counter reads for the 1 GiB copy probe)."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    try:
        with open(path) as f:
            t = json.load(f)
        return t[f"cfg{cfg_id}"][kernel]["hbm_bytes_per_launch"]
    except (OSError, KeyError, ValueError):
        return None


def cpu_baseline(hp, hb, gout, w, budget_s):
    """The oracle as it stands (single thread) on the first samples of hot batch 0; the
    tables are compacted to the rows the sample touches (same arithmetic, smaller arrays)."""
    import numpy as np
    import torch
    from oracle import fae_oracle as O

    cap_lookups = 2_000_000
    n = hb.n_samples
    while n > 1 and sum(hb.n_lookups) * n / hb.n_samples > cap_lookups:
        n //= 2
    sub = hb.slice(0, n)
    slots, offs, Ws = [], [], []
    for z, (s, o) in enumerate(zip(sub.slots, sub.offsets)):
        s_cpu = s.cpu().numpy()
        uniq, inv = np.unique(s_cpu, return_inverse=True)
        Ws.append(hp.hotW[z][torch.from_numpy(uniq.astype(np.int64)).to(hp.dev)].cpu().numpy().copy()
                  if uniq.size else np.zeros((1, w.dim), dtype=np.float32))
        slots.append(inv.astype(np.int32))
        offs.append(None if o is None else o.cpu().numpy())
    g = gout[:n].cpu().numpy().copy()
    lookups = sum(sub.n_lookups)
    reps, t0 = 0, time.perf_counter()
    while True:
        O.embbag_fwd(Ws, n, slots, offs)
        O.embbag_bwd_sgd(Ws, n, slots, offs, g, w.lr)
        reps += 1
        dt = time.perf_counter() - t0
        if dt >= budget_s or reps >= 1000:
            break
    return {"value": lookups * reps / dt, "unit": "lookups/s", "cores": 1, "kind": "oracle",
            "sample": f"first {n} samples of hot batch 0 ({lookups} lookups), {reps} fwd+bwd+SGD steps in {dt:.1f} s",
            "host_cores_available": os.cpu_count()}


if __name__ == "__main__":
    main()
