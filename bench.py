#!/usr/bin/env python3
"""Benchmark of the GPU-resident hot path: hot-embedding lookups/s for forward +
backward + sparse SGD on hot-only mini-batches, and achieved HBM GB/s against the
MI355X roofline, next to the CPU oracle timed on the host.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 1..5] [--also 1,2,4,5]

One GPU only.  Prints ONE JSON line.  Setup (profile -> cutoff -> hot tables ->
partition into hot mini-batches) runs through the same library and is reported per
stage (throughput, algorithmic bytes, fraction of the HBM peak); the timed region is K
steps of forward + backward/SGD cycling over distinct hot mini-batches resident in HBM,
repeated for five windows (the line carries the median window and the spread).  Steps 1
and 3 of every workload are compared with the oracle on sampled bags and rows before the
clock starts.

    python bench.py --ceiling        streaming-probe sweep (copy / read / fill launch shapes)
    python bench.py --profile-sweep  histogram variants per table size
    python bench.py --traffic-from DIR   turn rocprofv3 --pmc CSVs into profiles/hbm_traffic.json
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0  # MI355X HBM3E, published
WINDOWS = 5             # timed windows of K steps each; the median is the line's value


def log(*a):
    print("[bench]", *a, file=sys.stderr, flush=True)


def csrc_hash() -> str:
    """Hash of the kernel sources: HBM-traffic figures measured on other sources are not quoted."""
    h = hashlib.sha256()
    d = os.path.join(ROOT, "paper_2103_00686_amd", "csrc")
    for name in sorted(os.listdir(d)):
        if name.endswith((".hip", ".h")):
            h.update(name.encode())
            with open(os.path.join(d, name), "rb") as f:
                h.update(f.read())
    return h.hexdigest()[:16]


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--config", type=int, default=3, help="workload 1..5 (default 3: 26 tables, dim 64, batch 16384)")
    ap.add_argument("--also", type=str, default="1,2,4,5",
                    help="comma list of further workloads reported under other_workloads ('' = none)")
    ap.add_argument("--batches", type=int, default=0, help="distinct hot mini-batches to cycle over (0 = per workload)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline legs")
    ap.add_argument("--no-parity", action="store_true", help="skip the oracle check of steps 1 and 3")
    ap.add_argument("--no-extras", action="store_true", help="skip the probes and the steps around the path (profiling runs)")
    ap.add_argument("--cpu-seconds", type=float, default=3.0, help="budget of each cpu_baseline leg")
    ap.add_argument("--set", action="append", default=[], help="library option name=value (ablation)")
    ap.add_argument("--graph", action="store_true",
                    help="capture each step into a HIP graph and time the replays (same kernels, fewer launches)")
    ap.add_argument("--presort", choices=["auto", "fused", "side", "none", "ahead"], default="auto",
                    help="where the backward's sort runs: in the forward's launch (fused; needs one-hot tables "
                         "and at most 16384 samples), on the side stream, inside fae_embbag_bwd_sgd, or one step "
                         "ahead on the side stream (the next batch's sort beside this batch's forward and "
                         "backward).  auto: fused where the shape allows, else ahead for steps of up to 4 M lookups")
    ap.add_argument("--ceiling", action="store_true", help="sweep the streaming probes' launch shapes and exit")
    ap.add_argument("--profile-sweep", action="store_true", help="time the histogram variants per table size and exit")
    ap.add_argument("--traffic-from", type=str, default="", help="directory with rocprofv3 --pmc counter CSVs")
    args = ap.parse_args()
    if args.traffic_from:
        write_traffic(args.traffic_from)
        return
    if args.graph and args.presort == "ahead":
        print("bench.py: --graph captures one stream; --presort ahead uses two", file=sys.stderr)
        sys.exit(2)
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    if args.ceiling:
        ceiling_sweep()
        return
    if args.profile_sweep:
        profile_sweep()
        return
    line = run_workload(args, args.config, headline=True)
    others = []
    for c in [int(x) for x in args.also.split(",") if x.strip()]:
        if c == args.config:
            continue
        o = run_workload(args, c, headline=False)
        others.append({key: o[key] for key in ("value", "unit", "steps", "warmup", "ms_per_step", "ms_per_step_min",
                                                "ms_per_step_max", "windows", "launch_bound", "parity_checked", "config",
                                                "roofline", "cpu_baseline", "stages")})
    line["other_workloads"] = others
    print(json.dumps(line), flush=True)


# =====================================================================================
# one workload
# =====================================================================================
def run_workload(args, cfg_id, headline):
    import torch
    from paper_2103_00686_amd import binding as B
    from paper_2103_00686_amd import synth as S
    from paper_2103_00686_amd.hotpath import HotBatch, HotPath

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda", 0)
    if args.graph and torch.cuda.current_stream() == torch.cuda.default_stream():
        torch.cuda.set_stream(torch.cuda.Stream())     # capture needs a stream of its own
    n_steps, n_warmup = args.steps, args.warmup
    w = S.workload(cfg_id, "full")
    nt, D = w.n_tables, w.dim
    n_batches = args.batches or {1: 32, 2: 32, 3: 32, 4: 16, 5: 4}[cfg_id]
    hp = HotPath(w.rows, D, 0)
    for kv in args.set:
        k, v = kv.split("=")
        B.fae_set_option(hp.ctx, k, int(v))
    stages = {}

    def timed(fn):
        """(result, wall seconds, kernel seconds by HIP events on the library's stream)."""
        B.fae_timing_enable(hp.ctx, True)
        B.fae_timing_reset(hp.ctx)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        r = fn()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        kms = sum(B.fae_timing_read(hp.ctx, k)[0] for k in range(B.FAE_K_COUNT))
        B.fae_timing_enable(hp.ctx, False)
        return r, dt, kms * 1e-3

    def stage(name, units, unit_name, alg_bytes, wall_s, kern_s, note=None):
        gbps = alg_bytes / max(kern_s, 1e-12) / 1e9
        stages[name] = {unit_name + "_per_s": units / max(wall_s, 1e-12), unit_name: units, "alg_bytes": int(alg_bytes),
                        "wall_ms": wall_s * 1e3, "kernel_ms": kern_s * 1e3, "kernel_GBps": gbps,
                        "frac_of_peak": gbps / HBM_PEAK_GBPS}
        if note:
            stages[name]["note"] = note

    # ---- a1: profile the sampled stream, chunk by chunk ---------------------------
    chunk = min(w.profile_samples, 1 << 18)
    # counters and code objects exist before the clock starts: one untimed call on a few samples, then zeroed counters
    ch = S.make_chunk(w, 0, 0, min(1024, w.profile_samples), device=dev)
    hp.profile(B.Batch(ch.n_samples, ch.indices, ch.offsets, ch.n_lookups))
    hp.sync()
    hp.alloc_counts()
    del ch
    t_prof, k_prof, n_prof_lookups = 0.0, 0.0, 0
    cpu_prof_sample = None
    for first in range(0, w.profile_samples, chunk):
        n = min(chunk, w.profile_samples - first)
        ch = S.make_chunk(w, 0, first, n, device=dev)
        b = B.Batch(n, ch.indices, ch.offsets, ch.n_lookups)
        _, dt, kt = timed(lambda: hp.profile(b))
        t_prof += dt
        k_prof += kt
        n_prof_lookups += sum(ch.n_lookups)
        if cpu_prof_sample is None and not args.no_cpu:   # a bounded piece of the same stream for the oracle's leg
            cap = max(1, min(n, (4 << 20) * n // max(sum(ch.n_lookups), 1)))
            cpu_prof_sample = [(i[:cap] if o is None else i[:int(o[cap])]).cpu().numpy() for i, o in zip(ch.indices, ch.offsets)]
        del ch, b
    hp.sync()
    stage("profile", n_prof_lookups, "lookups", 4 * n_prof_lookups, t_prof, k_prof,
          "algorithmic bytes = the index stream; counter updates are scattered 4-byte atomics (sector traffic on top)")
    log(f"{w.name}: profiled {n_prof_lookups} lookups in {t_prof*1e3:.2f} ms")

    # ---- a2: cutoff ----------------------------------------------------------------
    hp.count_hot([1] * nt)            # untimed: the kernel's code object is loaded by its first launch
    if w.hot_rule == "cutoff":
        H = [w.cutoff] * nt
        n_hot, dt, kt = timed(lambda: hp.count_hot(H))
        c = None
    else:
        (c, H, n_hot), dt, kt = timed(lambda: hp.choose_cutoff(w.budget_bytes, w.small_table_bytes))
    stage("cutoff", sum(w.rows), "rows", 4 * sum(w.rows), dt, kt, "bytes of one pass over the counters")
    log(f"cutoff c={c} hot rows={sum(n_hot)} ({sum(n_hot)*D*4/2**30:.3f} GiB) in {dt*1e3:.2f} ms")

    # ---- a3 + a4: classify, remap, hot tables (procedural weights) -------------------
    _, dt, kt = timed(lambda: hp.build(H, n_hot, seed=w.seed))
    stage("build", sum(w.rows), "rows", 2 * 4 * sum(w.rows) + 4 * sum(w.rows) + 4 * sum(n_hot) + 4 * D * sum(n_hot), dt, kt,
          "counters read by the count and the scatter pass, remap and hot ids written, hot rows written (procedural "
          "weights: nothing read, one 64-bit hash per element)")
    log(f"built hot tables in {dt*1e3:.2f} ms")

    # ---- a5: hot mini-batches --------------------------------------------------------
    batches = []
    t_part, k_part, n_part_lookups, n_part_hot, n_part_samples = 0.0, 0.0, 0, 0, 0
    cpu_part_sample = None

    def keep_part_sample(ch, n):
        cap = max(1, min(n, (2 << 20) * n // max(sum(ch.n_lookups), 1)))
        return (cap, [(i[:cap] if o is None else i[:int(o[cap])]).cpu().numpy() for i, o in zip(ch.indices, ch.offsets)],
                [None if o is None else o[:cap + 1].cpu().numpy() for o in ch.offsets])

    if w.conditional_hot or cfg_id == 1:
        for i in range(n_batches):   # workload 1: each step works on the hot subset of one 1024-sample batch
            ch = S.make_chunk(w, 100 + i, 0, w.batch, device=dev, hot_remap=hp.remap if w.conditional_hot else None)
            b = B.Batch(w.batch, ch.indices, ch.offsets, ch.n_lookups)
            (hs, cs, hb), dt, kt = timed(lambda: hp.partition(b))
            t_part += dt
            k_part += kt
            n_part_lookups += sum(ch.n_lookups)
            n_part_hot += sum(hb.n_lookups)
            n_part_samples += w.batch
            assert hb.n_samples == w.batch or not w.conditional_hot
            batches.append(hb)
            if cpu_part_sample is None and not args.no_cpu:
                cpu_part_sample = keep_part_sample(ch, w.batch)
    else:
        first, span = 0, 1 << 19
        while len(batches) < n_batches and first < (1 << 26):
            ch = S.make_chunk(w, 100, first, span, device=dev)
            b = B.Batch(span, ch.indices, ch.offsets, ch.n_lookups)
            (hs, cs, hb), dt, kt = timed(lambda: hp.partition(b))
            t_part += dt
            k_part += kt
            n_part_lookups += sum(ch.n_lookups)
            n_part_hot += sum(hb.n_lookups)
            n_part_samples += span
            for k in range(hb.n_samples // w.batch):
                if len(batches) < n_batches:
                    sl = hb.slice(k * w.batch, w.batch)
                    batches.append(HotBatch(sl.n_samples, [s.clone() for s in sl.slots], sl.offsets, sl.n_lookups))
            log(f"partitioned samples [{first},{first+span}): {hb.n_samples} hot; {len(batches)} hot batches so far")
            if cpu_part_sample is None and not args.no_cpu:
                cpu_part_sample = keep_part_sample(ch, span)
            first += span
            del ch, b, hb
    stage("partition", n_part_lookups, "lookups", 8 * n_part_lookups + 4 * n_part_hot + 8 * n_part_samples, t_part, k_part,
          "index stream + one 4-byte remap entry per lookup + slots of the hot samples + flags and offsets; the remap "
          "gathers move a 32-byte sector per entry")
    assert batches, "no hot batch could be formed"

    # ---- step inputs resident in HBM ---------------------------------------------------
    gouts = [S.upstream_grads(w, 200 + i, hb.n_samples, device=dev) for i, hb in enumerate(batches)]
    outs = [torch.empty((hb.n_samples, nt, D), dtype=torch.float32, device=dev) for hb in batches]
    ws_need = max(B.fae_bwd_workspace_bytes(hp.hot_tables, hb.n_samples, hb.n_lookups) for hb in batches)
    hp._workspace("bwd", ws_need)
    steps_fn, presort = hp.prepare_steps(batches, gouts, outs, w.lr, presort=args.presort, single_stream=args.graph)
    nb = len(steps_fn)

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

    # ---- steps 1 to 3 against the oracle (sampled bags and rows), before any clock starts ----------
    it = 0          # steps taken so far: the callables of a cycle are called in cyclic order throughout
    parity = False
    if not args.no_parity:
        n_chk = min(3, nb)
        parity = parity_check(hp, w, batches, gouts, outs, steps_fn, n_chk)
        it = n_chk

    # ---- timed region ----------------------------------------------------------------
    eager_fn = steps_fn
    if args.graph:
        while it % nb:               # finish the cycle: a graph holds whole cycles
            steps_fn[it % nb]()
            it += 1
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
    for _ in range(n_warmup):
        steps_fn[it % nb]()
        it += 1
    windows = []
    for _ in range(WINDOWS):
        torch.cuda.synchronize()
        hp.sync()
        first_it = it
        t0 = time.perf_counter()
        for _ in range(n_steps):
            steps_fn[it % nb]()
            it += 1
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
        hp.sync()            # also raises if a step was flagged invalid on the device
        lookups_done = sum(acct[i % nb]["NL"] for i in range(first_it, it))
        windows.append((elapsed / n_steps, lookups_done / elapsed))
    windows.sort()
    s_per_step, value = windows[len(windows) // 2]
    ms_per_step = s_per_step * 1e3
    log(f"{WINDOWS} windows of {n_steps} steps: median {ms_per_step*1e3:.1f} us/step (min {windows[0][0]*1e6:.1f}, "
        f"max {windows[-1][0]*1e6:.1f}), {value/1e9:.3f} G lookups/s")

    # ---- per-kernel pass (HIP events on the library's stream, same steps) -------------
    B.fae_timing_enable(hp.ctx, True)
    B.fae_timing_reset(hp.ctx)
    k_steps = min(n_steps, 200)
    if args.graph:
        it = 0
    for _ in range(k_steps):
        eager_fn[it % nb]()
        it += 1
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
    step_bytes = bytes_fwd + bytes_bwd
    roofline = {"bound": "hbm", "kernel": dom, "achieved": round(dom_gbps, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": round(dom_gbps / HBM_PEAK_GBPS, 4), "traffic": None,
                "avg_launch_us": round(kern[dom]["avg_us"], 2), "alg_bytes_per_launch": int(alg[dom]),
                "measured": f"HIP events around every launch, separate pass of {k_steps} steps of the same loop",
                "step_compulsory_bytes": int(step_bytes),
                "step_frac": round(step_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                "per_lookup_GBps": round(per_lookup_bytes / (ms_per_step * 1e-3) / 1e9, 1),
                "kernels_us_per_step": {k: round(v["us_per_step"], 2) for k, v in kern.items()}}

    if not args.no_extras:
        # ---- what plain streaming kernels reach on this device (1 GiB each way) ----------------------
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        sink = torch.zeros(4, dtype=torch.float32, device=dev)

        def probe(fn, klass, nbytes):
            for _ in range(3):
                fn()
            B.fae_timing_enable(hp.ctx, True)
            B.fae_timing_reset(hp.ctx)
            for _ in range(10):
                fn()
            ms, n = B.fae_timing_read(hp.ctx, klass)
            B.fae_timing_enable(hp.ctx, False)
            return nbytes / (ms / n * 1e-3) / 1e9
        gib = src.numel() * 4
        copy_gbps = probe(lambda: B.fae_copy_probe(hp.ctx, dst, src), 13, 2 * gib)
        roofline["copy_ceiling_GBps"] = round(copy_gbps, 1)
        roofline["read_ceiling_GBps"] = round(probe(lambda: B.fae_read_probe(hp.ctx, src, sink), 17, gib), 1)
        roofline["fill_ceiling_GBps"] = round(probe(lambda: B.fae_fill_probe(hp.ctx, dst, 0.0), 18, gib), 1)
        roofline["frac_of_copy_ceiling"] = round(dom_gbps / copy_gbps, 4)
        roofline["step_frac_of_copy_ceiling"] = round(step_bytes / (ms_per_step * 1e-3) / 1e9 / copy_gbps, 4)
        del src, dst

        # ---- steps around the path: sampled hot-size estimate, embedding synchronisation -------
        chunks = [S.sample_chunks(w, z, 1024, 35) for z in range(nt)]
        hp.estimate_hot(H, chunks, 1024, 0.999)
        (est, _), dt, _ = timed(lambda: hp.estimate_hot(H, chunks, 1024, 0.999))
        around = {"estimate_call_us": dt * 1e6,
                  "estimate_rel_err": (sum(e["rows"] for e in est) - sum(n_hot)) / max(sum(n_hot), 1),
                  "estimate_ci_rel_halfwidth": sum(e["half_rows"] for e in est) / max(sum(n_hot), 1)}
        if w.hot_rule != "cutoff":
            (c_s, H_s, _), dt, _ = timed(lambda: hp.choose_cutoff_sampled(w.budget_bytes, chunks, 1024, 0.999, w.small_table_bytes))
            around["cutoff_sampled_ms"] = dt * 1e3
            around["cutoff_sampled_c"] = c_s
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
                around[name] = sync_bytes / (ms / n * 1e-3) / 1e9
            around["sync_bytes"] = sync_bytes
            del full
        stages["around_the_path"] = around

    # ---- the oracle on the host, bounded samples ----------------------------------------
    cpu = None
    if not args.no_cpu:
        cpu = cpu_baseline(hp, batches[0], gouts[0], w, args.cpu_seconds, cpu_prof_sample, cpu_part_sample)

    def rnd(v):
        if isinstance(v, dict):
            return {k: rnd(x) for k, x in v.items()}
        if isinstance(v, float):
            return float(f"{v:.4g}")
        return v

    line = {
        "metric": "hot-embedding lookups/sec (fwd+bwd+SGD)", "value": value, "unit": "lookups/s",
        "n_gpus": 1, "steps": n_steps, "warmup": n_warmup, "ms_per_step": ms_per_step,
        "ms_per_step_min": windows[0][0] * 1e3, "ms_per_step_max": windows[-1][0] * 1e3, "windows": WINDOWS,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        # a step this short is paced by launches and latencies, not by bandwidth: reported, but it does not decide the target
        "launch_bound": bool(step_bytes / (HBM_PEAK_GBPS * 1e9) < 10e-6),
        "parity_checked": parity,
        "config": {"workload": w.name, "config_index": cfg_id, "tables": nt, "dim": D, "batch": w.batch,
                   "zipf_s": w.zipf_s, "hot_rows": int(sum(hp.n_hot)), "hot_bytes": int(sum(hp.n_hot)) * D * 4,
                   "cutoff_c": c, "lookups_per_step": NL, "distinct_rows_per_step": U, "hot_batches": nb,
                   "launch": "hip graph replay" if args.graph else "eager", "presort": presort,
                   "profile_samples": w.profile_samples},
        "roofline": roofline, "cpu_baseline": rnd(cpu) if cpu else None, "stages": rnd(stages),
    }
    # measured HBM traffic of the dominant kernel, if a counter summary for these kernel sources is committed
    roofline["traffic"] = committed_traffic(cfg_id, dom)
    roofline["traffic_csrc_sha"] = committed_traffic_sha()
    # measured HBM traffic of the whole step: committed per-launch figures of every kernel the step
    # launches, times launches per step, over the step time measured here (null if a kernel has none)
    per = {k: committed_traffic(cfg_id, k) for k in kern if k not in ("fill",)}
    if per and all(v is not None for v in per.values()):
        tb = sum(per[k] * kern[k]["launches_per_step"] for k in per)
        roofline["step_traffic_bytes"] = int(tb)
        roofline["step_traffic_frac"] = round(tb / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4)
    else:
        roofline["step_traffic_bytes"] = roofline["step_traffic_frac"] = None
    del steps_fn, eager_fn, batches, gouts, outs, hp
    torch.cuda.empty_cache()
    return line


# =====================================================================================
# HBM traffic measured with rocprofv3 --pmc (committed summary)
# =====================================================================================
_TRAFFIC = None


def _traffic():
    global _TRAFFIC
    if _TRAFFIC is None:
        try:
            with open(os.path.join(ROOT, "profiles", "hbm_traffic.json")) as f:
                _TRAFFIC = json.load(f)
        except (OSError, ValueError):
            _TRAFFIC = {}
        if _TRAFFIC.get("csrc_sha") != csrc_hash():
            _TRAFFIC = {"stale": True}     # measured on other kernel sources: not quoted
    return _TRAFFIC


def committed_traffic_sha():
    t = _traffic()
    return None if t.get("stale") or not t else t.get("csrc_sha")


def committed_traffic(cfg_id, kernel):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 --pmc summary (FETCH_SIZE and
    WRITE_SIZE runs, each scaled by what the same counter reads for the 1 GiB copy probe); None
    when there is no figure, or when it was measured on kernel sources other than the present ones."""
    try:
        return _traffic()[f"cfg{cfg_id}"][kernel]["hbm_bytes_per_launch"]
    except (KeyError, TypeError):
        return None


KERNEL_CLASS = {"fwd_onehot_kernel": "fwd", "fwd_wave_kernel": "fwd", "fwd_group_kernel": "fwd",
                "bwd_reduce_kernel": "bwd_reduce", "bwd_reduce_walk_kernel": "bwd_reduce", "bwd_fixup_kernel": "bwd_fixup",
                "lds_sort_kernel": "lds_sort", "sort_scatter_kernel": "sort_scatter", "sort_hist_kernel": "sort_hist",
                "sort_colscan_kernel": "sort_colscan", "bwd_keys_kernel": "bwd_keys", "fae_copy_probe_kernel": "copy_probe",
                "fwd_sort_kernel": "fwd_sort"}


def write_traffic(directory):
    """DIR/cfg<N>_fetch/*counter_collection.csv and DIR/cfg<N>_write/*counter_collection.csv (rocprofv3
    --pmc FETCH_SIZE / WRITE_SIZE --kernel-trace --output-format csv of `bench.py --config N --also ''`)
    -> profiles/hbm_traffic.json: per workload and kernel class the HBM bytes per launch, each counter
    scaled by what it reads for the copy probe's 1 GiB, averaged over the later half of the launches."""
    import collections
    import csv
    import glob
    out = {"csrc_sha": csrc_hash()}
    for cfg in range(1, 6):
        per = {}
        for tag in ("fetch", "write"):
            files = glob.glob(os.path.join(directory, f"cfg{cfg}_{tag}", "**", "*counter_collection.csv"), recursive=True)
            if not files:
                continue
            acc = collections.defaultdict(list)
            for path in files:
                with open(path) as f:
                    for row in csv.DictReader(f):
                        base = row["Kernel_Name"].split("(")[0].replace("void ", "").split("<")[0].strip()
                        if base in KERNEL_CLASS:
                            acc[KERNEL_CLASS[base]].append((float(row["Counter_Value"]),
                                                            int(row["End_Timestamp"]) - int(row["Start_Timestamp"])))
            for k, v in acc.items():
                v = v[len(v) // 2:] if len(v) > 3 else v
                per.setdefault(k, {})[tag] = (sum(x[0] for x in v) / len(v), sum(x[1] for x in v) / len(v) / 1e3, len(v))
        if "copy_probe" not in per or len(per["copy_probe"]) < 2:
            continue
        f_scale = (1 << 20) / per["copy_probe"]["fetch"][0]      # counter reading for 1 GiB read -> KiB
        w_scale = (1 << 20) / per["copy_probe"]["write"][0]
        out[f"cfg{cfg}"] = {}
        for k, v in per.items():
            if "fetch" not in v or "write" not in v:
                continue
            hbm = (v["fetch"][0] * f_scale + v["write"][0] * w_scale) * 1024
            out[f"cfg{cfg}"][k] = {"hbm_bytes_per_launch": int(hbm), "fetch_KiB_raw": round(v["fetch"][0], 1),
                                   "write_KiB_raw": round(v["write"][0], 1), "fetch_scale": round(f_scale, 4),
                                   "write_scale": round(w_scale, 4),
                                   "avg_us_under_pmc": round(0.5 * (v["fetch"][1] + v["write"][1]), 1),
                                   "launches_averaged": v["fetch"][2]}
    with open(os.path.join(ROOT, "profiles", "hbm_traffic.json"), "w") as f:
        json.dump(out, f, indent=1)
    print(json.dumps(out, indent=1))


# =====================================================================================
# steps 1..3 against the oracle (outside the timed region)
# =====================================================================================
def parity_check(hp, w, batches, gouts, outs, steps_fn, n_chk):
    """Takes the first n_chk steps of the cycle one by one through the very callables the timed
    loop uses and compares steps 1 and n_chk with the oracle on sampled bags and sampled rows.
    The oracle follows a fixed set of rows R per table through all the steps: the rows of the
    sampled bags of the checked steps, sampled rows of the first batch and its most popular rows.
    The update of a row depends only on the lookups that hit it, so the oracle's update of R on
    the batch reduced to the lookups into R is its update of R on the whole batch; bags made only
    of rows in R have their true pooled output in the reduced batch.  Tolerance as in the parity
    tests: |gpu - ref| <= 1e-5 * sum|terms| (+ the bound inherited from earlier steps)."""
    import numpy as np
    import torch
    from oracle import fae_oracle as O
    rtol = 1e-5
    rng = np.random.default_rng(20210300686 % (1 << 32))
    nt, D = w.n_tables, w.dim
    checked = sorted({0, n_chk - 1})
    hbs = [batches[k] for k in range(n_chk)]
    slots = [[s.cpu().numpy() for s in hb.slots] for hb in hbs]
    offs = [[None if o is None else o.cpu().numpy() for o in hb.offsets] for hb in hbs]
    bags, R = {}, []
    for z in range(nt):
        rows = []
        for k in checked:
            S_k = hbs[k].n_samples
            pick = np.unique(rng.integers(0, max(S_k, 1), 64)) if S_k else np.zeros(0, np.int64)
            bags[(k, z)] = pick
            if offs[k][z] is None:
                rows.append(slots[k][z][pick])
            else:
                o = offs[k][z]
                rows.extend(slots[k][z][o[p]:o[p + 1]] for p in pick)
        s0 = slots[0][z]
        if s0.size:
            u, cnt = np.unique(s0, return_counts=True)
            rows.append(u[np.argsort(cnt)[-8:]])                       # the longest runs
            rows.append(u[rng.integers(0, u.size, 256)])
        R.append(np.unique(np.concatenate(rows)) if rows else np.zeros(0, np.int32))
    Wc = [hp.hotW[z][torch.from_numpy(R[z].astype(np.int64)).to(hp.dev)].cpu().numpy().copy() if R[z].size
          else np.zeros((1, D), np.float32) for z in range(nt)]
    # ^ before the first step the library's rows are the initial weights, which the parity tests
    #   compare bit for bit with the oracle's generator; from here on the oracle updates its own copy
    tol = [np.zeros_like(x) for x in Wc]
    for k in range(n_chk):
        outs[k].fill_(float("nan"))
        steps_fn[k]()
        hp.sync()
        S_k = hbs[k].n_samples
        if S_k == 0:
            continue
        g = gouts[k].cpu().numpy()
        out = outs[k].cpu().numpy() if k in checked else None
        for z in range(nt):
            if R[z].size == 0:
                continue
            sl = slots[k][z]
            hit = np.isin(sl, R[z])
            o = offs[k][z]
            bag = np.arange(S_k) if o is None else np.repeat(np.arange(S_k), np.diff(o))
            sub_off = np.zeros(S_k + 1, dtype=np.int32)
            np.cumsum(np.bincount(bag[hit], minlength=S_k), out=sub_off[1:])
            sub_sl = np.searchsorted(R[z], sl[hit]).astype(np.int32)
            if k in checked:
                ref, mag = O.embbag_fwd([Wc[z]], S_k, [sub_sl], [sub_off], want_mag=True)
                inh = O.embbag_fwd([tol[z]], S_k, [sub_sl], [sub_off]).astype(np.float64) * 1.001
                p = bags[(k, z)]
                err = np.abs(out[p, z, :].astype(np.float64) - ref[p, 0, :])
                bound = rtol * mag[p, 0, :] + inh[p, 0, :] + 1e-30
                if (err > bound).any():
                    raise AssertionError(f"{w.name}: step {k + 1}, table {z}: pooled output outside the oracle's bound")
            gz = np.ascontiguousarray(g[:, z:z + 1, :])
            uniq, runlen, mg = O.embbag_bwd_sgd([Wc[z]], S_k, [sub_sl], [sub_off], gz, w.lr, want_mag=True)
            t_new = tol[z][uniq[0]].astype(np.float64)
            if k in checked:
                got = hp.hotW[z][torch.from_numpy(R[z][uniq[0]].astype(np.int64)).to(hp.dev)].cpu().numpy()
                err = np.abs(got.astype(np.float64) - Wc[z][uniq[0]])
                if (err > rtol * mg[0] + t_new + 1e-30).any():
                    raise AssertionError(f"{w.name}: step {k + 1}, table {z}: updated rows outside the oracle's bound")
            tol[z][uniq[0]] = ((t_new + rtol * mg[0]) * 1.001).astype(np.float32)
    log(f"steps {[k + 1 for k in checked]} agree with the oracle on {sum(len(b) for b in bags.values())} sampled bags "
        f"and {sum(r.size for r in R)} followed rows")
    return True


# =====================================================================================
# the oracle timed on the host
# =====================================================================================
def cpu_baseline(hp, hb, gout, w, budget_s, prof_sample, part_sample):
    """The oracle as it stands, on bounded samples of this workload's inputs: one thread as
    written, and a plain parallel-for over the tables on the host's cores (threads that each
    call the oracle for their tables; the C code is single-threaded and releases the interpreter
    lock).  `value` is the faster of the two step legs, `cores` the threads that leg used.  For
    the step the tables are compacted to the rows the sample touches (same arithmetic, smaller
    arrays)."""
    from concurrent.futures import ThreadPoolExecutor
    import numpy as np
    import torch
    from oracle import fae_oracle as O

    host_cores = os.cpu_count() or 1
    nt = w.n_tables
    n_thr = max(1, min(nt, host_cores, 16))
    pool = ThreadPoolExecutor(max_workers=n_thr)

    def rate(work_units, fn_one, fn_par):
        """units/s single-threaded and over the tables in parallel, each leg bounded by budget_s."""
        res = {}
        for name, fn in (("single_thread", fn_one), ("parallel_tables", fn_par)):
            reps, t0 = 0, time.perf_counter()
            while True:
                fn()
                reps += 1
                dt = time.perf_counter() - t0
                if dt >= budget_s or reps >= 200:
                    break
            res[name] = {"value": work_units * reps / dt, "cores": 1 if name == "single_thread" else n_thr,
                         "reps": reps, "seconds": round(dt, 2)}
        return res

    # ---- the step: forward + backward/SGD ------------------------------------------------
    cap_lookups = 1_000_000
    n = hb.n_samples
    while n > 1 and sum(hb.n_lookups) * n / max(hb.n_samples, 1) > cap_lookups:
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
    gz = [np.ascontiguousarray(g[:, z:z + 1, :]) for z in range(nt)]
    lookups = sum(sub.n_lookups)

    def step_one():
        O.embbag_fwd(Ws, n, slots, offs)
        O.embbag_bwd_sgd(Ws, n, slots, offs, g, w.lr)

    def step_table(z):
        O.embbag_fwd([Ws[z]], n, [slots[z]], [offs[z]])
        O.embbag_bwd_sgd([Ws[z]], n, [slots[z]], [offs[z]], gz[z], w.lr)

    step = rate(lookups, step_one, lambda: list(pool.map(step_table, range(nt))))
    best = max(step.values(), key=lambda r: r["value"])
    out = {"value": best["value"], "unit": "lookups/s", "cores": best["cores"], "kind": "oracle",
           "sample": f"first {n} samples of hot batch 0 ({lookups} lookups), forward + backward + SGD; each leg up to "
                     f"{budget_s:.0f} s; single thread as written, and a parallel-for over the {nt} tables on {n_thr} threads",
           "host_cores_available": host_cores, "step": step}

    # ---- the pre-processing stages ----------------------------------------------------------
    stage = {}
    if prof_sample is not None:
        idx = [np.ascontiguousarray(i, dtype=np.int32) for i in prof_sample]
        cnts = [np.zeros(r, dtype=np.uint32) for r in w.rows]
        stage["profile_lookups_per_s"] = rate(sum(i.size for i in idx),
                                              lambda: [O.histogram(w.rows[z], idx[z], cnts[z]) for z in range(nt)],
                                              lambda: list(pool.map(lambda z: O.histogram(w.rows[z], idx[z], cnts[z]), range(nt))))
        stage["profile_sample_lookups"] = sum(i.size for i in idx)
        # classify + remap + hot ids on the counters of that sample (every row of every table)
        stage["build_rows_per_s"] = rate(sum(w.rows), lambda: [O.classify(cnts[z], 1) for z in range(nt)],
                                         lambda: list(pool.map(lambda z: O.classify(cnts[z], 1), range(nt))))
        del cnts
    if part_sample is not None:
        n_s, idx, off = part_sample
        idx = [np.ascontiguousarray(i, dtype=np.int32) for i in idx]
        remap = [r[:w.rows[z]].cpu().numpy() for z, r in enumerate(hp.remap)]
        nl = sum(i.size for i in idx)
        # the input classifier is one pass over the samples (a sample is hot iff all its tables agree): single leg
        reps, t0 = 0, time.perf_counter()
        while True:
            O.partition(w.rows, n_s, idx, off, remap)
            reps += 1
            dt = time.perf_counter() - t0
            if dt >= budget_s or reps >= 200:
                break
        stage["partition_lookups_per_s"] = {"single_thread": {"value": nl * reps / dt, "cores": 1, "reps": reps,
                                                              "seconds": round(dt, 2)}}
        stage["partition_sample_lookups"] = nl
        del remap
    out["stages"] = stage
    pool.shutdown()
    return out


# =====================================================================================
# sweeps (their output is what profiles/ and the design notes quote)
# =====================================================================================
def ceiling_sweep():
    """Streaming probes over launch shapes: 16-byte accesses in flight per lane, one workgroup per
    chunk or a fixed number per compute unit, plain or non-temporal accesses; 1 GiB and 109 MB."""
    import torch
    from paper_2103_00686_amd import binding as B
    from paper_2103_00686_amd.hotpath import HotPath
    dev = torch.device("cuda", 0)
    hp = HotPath([16], 4, 0)
    rows = []
    for nbytes in (1 << 30, 109051904):
        src = torch.empty(nbytes // 4, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        sink = torch.zeros(4, dtype=torch.float32, device=dev)
        kinds = (("copy", 13, 2 * nbytes, lambda: B.fae_copy_probe(hp.ctx, dst, src)),
                 ("read", 17, nbytes, lambda: B.fae_read_probe(hp.ctx, src, sink)),
                 ("fill", 18, nbytes, lambda: B.fae_fill_probe(hp.ctx, dst, 1.0)))
        for unroll in (1, 2, 4, 8):
            for nt_ in (0, 1):
                for wpc in (0, 1, 2, 4, 8, 16, 32):
                    B.fae_set_option(hp.ctx, "probe_unroll", unroll)
                    B.fae_set_option(hp.ctx, "probe_nt", nt_)
                    B.fae_set_option(hp.ctx, "probe_wgs_per_cu", wpc)
                    for name, klass, moved, fn in kinds:
                        for _ in range(2):
                            fn()
                        B.fae_timing_enable(hp.ctx, True)
                        B.fae_timing_reset(hp.ctx)
                        for _ in range(7):
                            fn()
                        ms, n = B.fae_timing_read(hp.ctx, klass)
                        B.fae_timing_enable(hp.ctx, False)
                        rows.append({"kind": name, "bytes": nbytes, "unroll": unroll, "nt": nt_, "wgs_per_cu": wpc,
                                     "us": round(ms / n * 1e3, 1), "GBps": round(moved / (ms / n * 1e-3) / 1e9, 1)})
        del src, dst
    for r in rows:
        print(json.dumps(r))
    for nbytes in (1 << 30, 109051904):
        for kind in ("copy", "read", "fill"):
            best = max((r for r in rows if r["kind"] == kind and r["bytes"] == nbytes), key=lambda r: r["GBps"])
            print("best", json.dumps(best))


def profile_sweep():
    """Histogram variants (global atomics / LDS-privatised) per table size: one table of R rows,
    2^24 lookups, Zipf(1.1) over a seeded row permutation."""
    import torch
    from paper_2103_00686_amd import binding as B
    from paper_2103_00686_amd import synth as S
    from paper_2103_00686_amd.hotpath import HotPath
    dev = torch.device("cuda", 0)
    n = 1 << 24
    for R in (10 ** 3, 10 ** 4, 16384, 10 ** 5, 10 ** 6, 10 ** 7, 10 ** 8):
        w = S.Workload(f"sweep-1x{R}-d16", 9, (R,), 16, ("one",), 1.1, n, n, "cutoff", cutoff=1)
        ch = S.make_chunk(w, 0, 0, n, device=dev)
        b = B.Batch(n, ch.indices, ch.offsets, ch.n_lookups)
        res = {"rows": R, "lookups": n}
        for variant, name in ((1, "global_atomics"), (2, "lds_privatised")):
            hp = HotPath([R], 16, 0)
            B.fae_set_option(hp.ctx, "profile_variant", variant)
            hp.profile(b)
            hp.sync()
            B.fae_timing_enable(hp.ctx, True)
            B.fae_timing_reset(hp.ctx)
            for _ in range(5):
                hp.profile(b)
            ms, k = B.fae_timing_read(hp.ctx, 9)
            B.fae_timing_enable(hp.ctx, False)
            res[name + "_us"] = round(ms / k * 1e3, 1)
            res[name + "_index_GBps"] = round(4 * n / (ms / k * 1e-3) / 1e9, 1)
            del hp
        print(json.dumps(res), flush=True)


if __name__ == "__main__":
    main()
