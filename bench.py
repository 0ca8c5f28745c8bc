"""Benchmark of the Conf-KV decode step on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic input:
L x conf_kv_attend, conf_kv_step, conf_kv_evict_compact, all through the C ABI.
Workload: the Llama-3-8B-shape single-step microbenchmark (32 layers, 32/8 heads,
D = 128, V = 128256, batch 8, 4096-token cache per unit with the newest 128 tokens FP16
and the rest INT8; budgets 1024/2048; protected window 128; logits N(0, 3)).

The step shrinks every cache (4097 -> 2048 or 1024 slots), so the cache is re-loaded from
the resident FP16 prompt tensors between timed steps; the re-load (layer by layer, followed by
a read of 512 MiB of unrelated memory that writes the re-load's dirty cache lines back) is
outside the timed region.  Each step is bracketed by HIP events on the launch stream with a device
synchronisation on both sides; `ms_per_step` is the mean event time of the K steps.

Prints ONE JSON line.  `roofline` describes the attention + mass-EMA kernel (the dominant
kernel): algorithmic bytes per launch / its mean launch duration, against 8 TB/s.
`cpu_baseline` is the float64 numpy oracle timed on this machine's host cores on a bounded
sample of the same workload's units, extrapolated to the whole step.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
DTYPE = "int8+fp16 storage, fp16 mfma, fp32 accumulate"
# HBM bytes per conf_kv_attend launch on the default workload come from the tracked counter
# summary (two rocprofv3 --pmc runs, FETCH_SIZE and WRITE_SIZE in KiB per dispatch, each scaled by
# what the same counter reads for a plain 1 GiB device copy): parsed at run time, so the figure
# cannot outlive the file it came from.
COUNTER_FILE = {1: os.path.join(ROOT, "profiles", "bench_llama3_8b_b8_t4096_hbm_counters.txt")}


def counter_traffic(workload_index, kernel="attend_mfma_kernel"):
    """(bytes per launch, file name) from the tracked FETCH_SIZE / WRITE_SIZE summary, or (None, None)."""
    path = COUNTER_FILE.get(workload_index)
    if not path or not os.path.exists(path):
        return None, None
    mean = {}
    for line in open(path):
        if line.startswith("#") or "mean=" not in line:
            continue
        for ctr in ("FETCH_SIZE", "WRITE_SIZE"):
            if f" {ctr} " in line:
                who = "copy" if "copyBuffer" in line else kernel if kernel in line else None
                if who:
                    mean[(who, ctr)] = float(line.split("mean=")[1])
    try:
        copy_kib = float(1 << 20)                       # the calibration copy reads and writes 1 GiB
        scale_f = copy_kib / mean[("copy", "FETCH_SIZE")]
        scale_w = copy_kib / mean[("copy", "WRITE_SIZE")]
        kib = mean[(kernel, "FETCH_SIZE")] * scale_f + mean[(kernel, "WRITE_SIZE")] * scale_w
    except (KeyError, ZeroDivisionError):
        return None, None
    return int(kib * 1024), os.path.relpath(path, ROOT)


def attend_bytes_per_launch(wl, n8, n16):
    """Algorithmic HBM bytes of one conf_kv_attend launch (one layer), n16 counting the new token.

    Per unit: INT8 slots (2D codes + 2 fp16 scales), FP16 slots (4D), EMA read + write
    (8 B per slot), q and out (4 G D), the new K/V read and written (8 D + 8 D... the write
    is counted once: 4D) and its position.
    """
    D, G = wl.head_dim, wl.group
    n = n8 + n16
    chan = getattr(wl, "scale_mode", "token") == "channel"     # then 2 x D fp16 scales per unit instead
    tq = max(1, getattr(wl, "max_chunk", 0))                    # tokens per call here: q, out and new rows scale with it
    per_unit = (n8 * (2 * D + (0 if chan else 4)) + (4 * D if chan else 0) + n16 * 4 * D + 8 * n
                + tq * (4 * G * D + 8 * D + 4))
    return per_unit * wl.batch * wl.n_kv_heads


def step_bytes(wl, n8, n16, moved_bytes):
    """Algorithmic bytes of the whole step: attention, logits, ranking, compaction moves (the
    rows the order-preserving compaction has to move on its cheaper side, read + written, as
    counted by the library), demotion."""
    D = wl.head_dim
    att = attend_bytes_per_launch(wl, n8, n16) * wl.n_layers
    logits = 4 * wl.vocab * wl.batch
    n = n8 + n16
    rank = 8 * max(0, n - wl.protected) * wl.units
    demote = wl.units * (4 * D + 2 * D + (0 if getattr(wl, "scale_mode", "token") == "channel" else 4))
    return att + logits + rank + int(moved_bytes) + demote, att


def read_probe(torch, pkg, launch_bytes):
    """What a plain read-only pass reaches on this machine (context for the roofline fraction, which
    is quoted against the published 8 TB/s): the library's probe kernel (16-byte loads, 8 in
    flight per thread, 4096 workgroups) over 2 GiB in one launch, and over different regions of
    `launch_bytes` each, one launch per region -- the shape of a decode step, where every layer's
    cache is read once and nothing is reused between launches.  torch's sum is timed the same way
    as a cross-check."""
    x = torch.empty(1 << 29, dtype=torch.float32, device="cuda").normal_()
    per = max(4, launch_bytes // 16 * 4)                 # floats per region, a multiple of 16 bytes
    regions = [x[i * per:(i + 1) * per] for i in range(min(28, x.numel() // per))]
    wgs = 4096                                           # best of a sweep from 256 to 16384
    out = torch.zeros(wgs, dtype=torch.int32, device="cuda")

    def timed(fn, reps):
        for _ in range(2):
            fn()
        torch.cuda.synchronize()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        ev[0].record()
        for _ in range(reps):
            fn()
        ev[1].record()
        torch.cuda.synchronize()
        return ev[0].elapsed_time(ev[1]) / reps

    big = timed(lambda: pkg.probe_read(x, out, wgs), 5)
    reg = timed(lambda: [pkg.probe_read(r, out, wgs) for r in regions], 3) / len(regions)
    big_t = timed(lambda: x.sum(), 5)
    reg_t = timed(lambda: [r.sum() for r in regions], 3) / len(regions)
    gb = lambda nbytes, ms: nbytes / ms / 1e6
    return {"kind": "conf_kv_probe_read (torch.sum as cross-check)",
            "stream_2GiB_GBps": gb(x.numel() * 4, big), "per_launch_GBps": gb(per * 4, reg),
            "per_launch_bytes": per * 4, "per_launch_us": reg * 1e3,
            "torch_sum_stream_GBps": gb(x.numel() * 4, big_t), "torch_sum_per_launch_GBps": gb(per * 4, reg_t)}


def _cpu_worker(job):
    """One oracle worker: the units `count` (ids) of the workload, timing attend + evict/compact/demote."""
    wl, seed, worker, count, tight = job
    from threadpoolctl import threadpool_limits
    from oracle import confkv_oracle as O
    from synth import generate as gen
    sys.path.insert(0, os.path.join(ROOT, "tests"))
    from harness import policy_of
    pol = policy_of(wl)
    G = wl.group
    times = []
    with threadpool_limits(limits=1):
        for uid in count:                      # unit ids (layer * B + b) * Hkv + kv-head
            l, b, g = uid // (wl.batch * wl.n_kv_heads), uid // wl.n_kv_heads % wl.batch, uid % wl.n_kv_heads
            K, V = gen.prefill_unit(wl, seed, l, b, g)
            u = O.load_prefill(K, V, wl.fp16_window, scale_mode=getattr(wl, "scale_mode", "token"))
            q, kn, vn = gen.step_inputs(wl, seed, l, 0)
            t0 = time.perf_counter()
            O.attend_unit(u, q[b, g * G:(g + 1) * G], kn[b, g], vn[b, g], wl.prefill, pol.sm_scale, pol.ema_decay)
            N = pol.n_tight[l] if tight else pol.n_loose[l]
            O.evict_compact_unit(u, N, pol.protected, pol.alpha, pol.fp16_window)
            times.append(time.perf_counter() - t0)
    return times


def cpu_baseline(wl, seed, units_per_core=128):
    """The oracle, as it stands, on a bounded sample of units of the same workload, one process
    per host core this process may run on (at most 16, the machine's CPU share).  Must run before the
    GPU is initialised: the workers are forked."""
    import multiprocessing as mp
    from oracle import confkv_oracle as O
    from synth import generate as gen
    sys.path.insert(0, os.path.join(ROOT, "tests"))
    from harness import policy_of
    pol = policy_of(wl)
    cores = max(1, min(16, len(os.sched_getaffinity(0))))
    logits = gen.step_logits(wl, seed, 0)
    t0 = time.perf_counter()
    c = O.confidence(logits[0], pol.weights)
    t_conf = time.perf_counter() - t0
    tight = bool(c >= pol.tau)
    t0 = time.perf_counter()
    with mp.get_context("fork").Pool(cores) as pool:
        # every units-th unit of the workload, at most units_per_core per worker (all of them when they fit)
        take = min(wl.units, cores * units_per_core)
        ids = [int(i) for i in np.linspace(0, wl.units - 1, take).round()] if take < wl.units else list(range(wl.units))
        per = pool.map(_cpu_worker, [(wl, seed, w, ids[w::cores], tight) for w in range(cores)])
    wall = time.perf_counter() - t0
    times = np.concatenate([np.asarray(p) for p in per])
    per_unit = float(times.mean())                      # with all cores busy at once
    step_s = (per_unit * wl.units + t_conf * wl.batch) / cores
    return {"value": 1.0 / step_s, "unit": "steps/s", "cores": cores, "kind": "oracle",
            "sample": f"{'all ' if times.size == wl.units else ''}{times.size} of {wl.units} units of workload {wl.name} (attend + evict/compact/demote, "
                      f"{per_unit * 1e3:.2f} ms per unit with {cores} processes busy) plus 1 of {wl.batch} confidence "
                      f"rows ({t_conf * 1e3:.2f} ms); extrapolated to all units spread over the {cores} cores "
                      f"(os.cpu_count() = {os.cpu_count()}, affinity = {len(os.sched_getaffinity(0))}; "
                      f"sample took {wall:.1f} s)"}


def steady_state(args, wl, kv, torch, gen, reload, qs, ks, vs, out, conf, sel):
    """K consecutive decode steps after W warm-up steps on one loaded prompt (the cache sawtooths
    between the budgets as the logits alternate between confident and uncertain runs)."""
    L = wl.n_layers
    logits_by_std = {}
    def logits_for(t):
        std = gen.logit_std(wl, t)
        if std not in logits_by_std:
            logits_by_std[std] = torch.from_numpy(gen.step_logits(wl, args.seed, t)).cuda()
        return logits_by_std[std]
    reload(); torch.cuda.synchronize()
    rows = []
    moved0 = 0
    graph = None
    if args.static_plan:
        kv.static_plan(True)
    if args.graph:
        # the timed steps are replays of one recorded step: launch shapes from the budgets, the
        # step's logits copied into the recorded tensor before each replay (outside the interval)
        kv.static_plan(True)
        glogits = torch.empty_like(logits_for(0))
        assert args.warmup >= 1, "--graph records after at least one step outside the graph"
    for t in range(args.warmup + args.steps):
        if t == args.warmup:
            moved0 = kv.counters().compact_bytes
            if args.graph:
                graph = torch.cuda.CUDAGraph()
                with torch.cuda.graph(graph):
                    for l in range(L):
                        kv.attend(l, qs[l], ks[l], vs[l], out)
                    kv.step(glogits, conf, sel)
                    kv.evict_compact()
        lg = logits_for(t)
        ln, n16 = kv.lengths()
        n = ln.astype(np.int64) + 1
        n16u = n16.astype(np.int64) + 1                                  # [L][B][Hkv], with the append
        D, G = wl.head_dim, wl.group
        att_bytes = int(((n[:, :, None] - n16u) * (2 * D + 4) + n16u * 4 * D + 8 * n[:, :, None]).sum()
                        + wl.units * (4 * G * D + 8 * D + 4))
        other_bytes = int(4 * wl.vocab * wl.batch + 8 * np.maximum(0, n - wl.protected).sum() * wl.n_kv_heads
                          + wl.units * (6 * D + 4))                      # logits, ranking inputs, demotion
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
        if graph is not None:
            glogits.copy_(lg)
            ev[0].record()
            graph.replay()
            for e in ev[1:]:
                e.record()
            torch.cuda.synchronize()
            rows.append((ev[0].elapsed_time(ev[3]), float("nan"), float("nan"), float("nan"), att_bytes,
                         float(n.mean()), other_bytes))
            continue
        ev[0].record()
        for l in range(L):
            kv.attend(l, qs[l], ks[l], vs[l], out)
        ev[1].record()
        kv.step(lg, conf, sel)
        ev[2].record()
        kv.evict_compact()
        ev[3].record()
        torch.cuda.synchronize()
        if t >= args.warmup:
            rows.append((ev[0].elapsed_time(ev[3]), ev[0].elapsed_time(ev[1]), ev[1].elapsed_time(ev[2]),
                         ev[2].elapsed_time(ev[3]), att_bytes, float(n.mean()), other_bytes))
    r = np.array(rows)
    st = kv.counters()
    ms_step = float(r[:, 0].mean())
    moved = (st.compact_bytes - moved0) / args.steps
    total_bytes = float(r[:, 4].mean() + r[:, 6].mean() + moved)
    att_gbps = float((r[:, 4] / (r[:, 1] * 1e-3)).mean() / 1e9)
    if graph is not None:
        # no events inside a replay: the attention share of the step is not measured in this mode
        print(json.dumps({
            "metric": "decode_steps_per_s", "value": 1000.0 / ms_step, "unit": "steps/s", "n_gpus": 1,
            "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_step, "higher_is_better": True,
            "scaling": "weak", "vs_baseline": None, "dtype": DTYPE, "data": "synthetic",
            "config": {"workload": wl.name, "mode": "steady-state, every timed step a replay of one recorded HIP graph",
                       "layers": L, "batch": wl.batch, "layout": args.layout, "evict_page": args.evict_page,
                       "mean_cache_len": float(r[:, 5].mean()), "attend_splits": kv.attend_splits(0)},
            "step_hbm": {"algorithmic_bytes": total_bytes, "compaction_bytes": moved,
                         "achieved_GBps": total_bytes / (ms_step * 1e-3) / 1e9,
                         "frac_of_peak": total_bytes / (ms_step * 1e-3) / 1e9 / HBM_PEAK_GBS},
            "counters": {"evicted": int(st.evicted), "demoted": int(st.demoted), "tight": int(st.tight_steps),
                         "loose": int(st.loose_steps)},
        }))
        return
    print(json.dumps({
        "metric": "decode_steps_per_s", "value": 1000.0 / ms_step, "unit": "steps/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": DTYPE, "data": "synthetic",
        "config": {"workload": wl.name, "mode": "steady-state", "layers": L, "batch": wl.batch, "layout": args.layout,
                   "evict_page": args.evict_page,
                   "mean_cache_len": float(r[:, 5].mean()), "attend_splits": kv.attend_splits(0)},
        "roofline": {"bound": "hbm", "kernel": "attend", "achieved": att_gbps, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": att_gbps / HBM_PEAK_GBS, "traffic": None,
                     "bytes_per_launch": float(r[:, 4].mean()) / L, "launch_ms": float(r[:, 1].mean()) / L},
        "step_breakdown_ms": {"attend_x_layers": float(r[:, 1].mean()), "confidence": float(r[:, 2].mean()),
                              "evict_compact": float(r[:, 3].mean())},
        "step_hbm": {"algorithmic_bytes": total_bytes, "compaction_bytes": moved,
                     "achieved_GBps": total_bytes / (ms_step * 1e-3) / 1e9,
                     "frac_of_peak": total_bytes / (ms_step * 1e-3) / 1e9 / HBM_PEAK_GBS},
        "counters": {"evicted": int(st.evicted), "demoted": int(st.demoted), "tight": int(st.tight_steps),
                     "loose": int(st.loose_steps)},
    }))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", type=int, default=1)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--steady", action="store_true",
                    help="multi-step workloads: load the prompt once and time K consecutive decode steps")
    ap.add_argument("--graph", action="store_true",
                    help="with --steady: record one decode step into a HIP graph after the warm-up and time replays of it")
    ap.add_argument("--static-plan", action="store_true",
                    help="with --steady: launch shapes from the budgets (what --graph uses), without the graph")
    ap.add_argument("--layers", type=int, default=0, help="keep only the first N layers (0 = all)")
    ap.add_argument("--scales", choices=["token", "channel"], default="token",
                    help="granularity of the INT8 scales (channel: the paper's literal per-(head, channel) reading)")
    ap.add_argument("--chunk", type=int, default=1,
                    help="tokens per attention call (conf_kv_attend_chunk when above 1; at most 128 / group size)")
    ap.add_argument("--evict-page", type=int, default=0,
                    help="coarsened eviction: whole pages of this many original positions go (0 = token level)")
    ap.add_argument("--layout", choices=["contiguous", "paged"], default="contiguous",
                    help="paged: INT8 slots in pages of --evict-page slots behind a block table (no row moves)")
    ap.add_argument("--rank-scope", choices=["kv_head", "layer"], default="kv_head",
                    help="layer: one kept set per (layer, sequence) from the importance summed over its kv-heads")
    ap.add_argument("--copy-probe", action="store_true",
                    help="run a plain 1 GiB device-to-device copy a few times and exit (counter calibration)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    cpu = None
    if not (args.no_cpu_baseline or args.copy_probe or args.steady):
        # (before anything touches the GPU: the oracle's workers are forked)
        from synth.workloads import workload as _workload
        cpu = cpu_baseline(_workload(args.workload), args.seed)
    import torch
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.copy_probe:
        # known traffic for scaling the FETCH_SIZE / WRITE_SIZE counters: each copy reads 1 GiB
        # and writes 1 GiB
        x = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").random_(0, 255)
        y = torch.empty_like(x)
        for _ in range(5):
            y.copy_(x)
        torch.cuda.synchronize()
        print(json.dumps({"copy_probe_bytes_read": 1 << 30, "copy_probe_bytes_written": 1 << 30, "copies": 5}))
        return
    import paper_2605_24786_amd as pkg
    from synth import generate as gen
    from synth.workloads import workload

    wl = workload(args.workload)
    if args.scales != "token":
        wl = wl.scaled(name=wl.name + "_" + args.scales + "_scales", scale_mode=args.scales)
    if args.chunk > 1:
        wl = wl.scaled(name=wl.name + f"_chunk{args.chunk}", max_chunk=args.chunk)
    if args.evict_page > 1:
        wl = wl.scaled(name=wl.name + f"_page{args.evict_page}", evict_page=args.evict_page)
    if args.layout != "contiguous":
        wl = wl.scaled(name=wl.name + "_" + args.layout, layout=args.layout)
    if args.rank_scope != "kv_head":
        wl = wl.scaled(name=wl.name + "_layer_scope", rank_scope=args.rank_scope)
    if args.layers and args.layers < wl.n_layers:
        wl = wl.scaled(n_layers=args.layers, n_tight=wl.n_tight[:args.layers], n_loose=wl.n_loose[:args.layers])
    L = wl.n_layers
    t_setup = time.time()
    kv = pkg.from_workload(wl)
    prompts = []
    for l in range(L):
        K, V = gen.prefill_layer(wl, args.seed, l, threads=16)
        prompts.append((torch.from_numpy(K).cuda(), torch.from_numpy(V).cuda()))
    qs, ks, vs = [], [], []
    tq = args.chunk
    for l in range(L):
        if tq == 1:
            q, k, v = gen.step_inputs(wl, args.seed, l, 0)
        else:    # [B][tq][heads][D]: the inputs of tq consecutive steps
            parts = [gen.step_inputs(wl, args.seed, l, t) for t in range(tq)]
            q, k, v = (np.ascontiguousarray(np.stack([p[j] for p in parts], axis=1)) for j in range(3))
        qs.append(torch.from_numpy(q).cuda()); ks.append(torch.from_numpy(k).cuda()); vs.append(torch.from_numpy(v).cuda())
    logits = torch.from_numpy(gen.step_logits(wl, args.seed, tq - 1)).cuda()
    out = torch.empty(tuple(qs[0].shape), dtype=torch.float16, device="cuda")
    conf = torch.empty(wl.batch, dtype=torch.float32, device="cuda")
    sel = torch.empty(wl.batch, dtype=torch.uint8, device="cuda")
    print(f"# setup {time.time() - t_setup:.1f}s: {wl.name}, state {kv.state.numel() / 2**30:.2f} GiB", file=sys.stderr, flush=True)

    # Between timed steps (outside the timed region) the caches are loaded again, one layer at a
    # time with a synchronisation after each, and then 512 MiB of unrelated memory are read once.
    # The re-load writes gigabytes at several TB/s: issued back to back it leaves the power
    # management throttling and some 290 MB of dirty lines in L2 and the Infinity Cache, which the
    # first launches of the timed step then pay for (measured: 21.6 instead of 20.4 us per
    # attention launch).  A decode step in a serving loop follows other work, not a bulk write of
    # its own cache, so the timed step starts from clean caches and a settled clock.
    scrub = torch.empty(1 << 27, dtype=torch.float32, device="cuda").normal_() if not args.steady else None
    scrub_out = torch.zeros(4096, dtype=torch.int32, device="cuda")

    def reload():
        for l in range(L):
            kv.load_prefill(l, prompts[l][0], prompts[l][1])
            torch.cuda.synchronize()
        if scrub is not None:
            pkg.probe_read(scrub, scrub_out, 4096)

    def one_step(ev=None):
        # returns per-phase events when ev is given: [start, after attends, after step, end]
        if ev: ev[0].record()
        for l in range(L):
            if tq == 1:
                kv.attend(l, qs[l], ks[l], vs[l], out)
            else:
                kv.attend_chunk(l, qs[l], ks[l], vs[l], out)
        if ev: ev[1].record()
        kv.step(logits, conf, sel)
        if ev: ev[2].record()
        kv.evict_compact()
        if ev: ev[3].record()

    if args.steady:
        assert tq == 1, "--steady times single-token steps"
        steady_state(args, wl, kv, torch, gen, reload, qs, ks, vs, out, conf, sel)
        return
    for _ in range(args.warmup):
        reload(); torch.cuda.synchronize()
        one_step(); torch.cuda.synchronize()

    len_before = wl.prefill + tq
    n8_b = max(0, wl.prefill - wl.fp16_window) if wl.fp16_window >= 0 else 0
    n16_b = len_before - n8_b
    t_step, t_att, t_conf, t_evict = [], [], [], []
    moved0 = kv.counters().compact_bytes
    for _ in range(args.steps):
        reload(); torch.cuda.synchronize()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
        one_step(ev)
        torch.cuda.synchronize()
        t_step.append(ev[0].elapsed_time(ev[3]))
        t_att.append(ev[0].elapsed_time(ev[1]))
        t_conf.append(ev[1].elapsed_time(ev[2]))
        t_evict.append(ev[2].elapsed_time(ev[3]))
    ln, n16 = kv.lengths()
    st = kv.counters()

    ms_step = float(np.mean(t_step))
    # the dominant kernel: the L attention launches of a step run back to back between two
    # HIP events of the timed region, so their mean duration is that interval / L
    att_launch_ms = float(np.mean(t_att)) / L
    att_bytes = attend_bytes_per_launch(wl, n8_b, n16_b)
    n_after = int(ln.mean())
    moved = (st.compact_bytes - moved0) / args.steps
    total_bytes, att_total = step_bytes(wl, n8_b, n16_b, moved)
    achieved = att_bytes / (att_launch_ms * 1e-3) / 1e9
    plain = (args.scales == "token" and tq == 1 and not args.layers and args.evict_page <= 1
             and args.rank_scope == "kv_head" and args.layout == "contiguous")
    traffic, traffic_file = counter_traffic(args.workload) if plain else (None, None)
    result = {
        "metric": "decode_steps_per_s", "value": 1000.0 / ms_step, "unit": "steps/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": DTYPE, "data": "synthetic",
        "config": {"workload": wl.name, "layers": L, "batch": wl.batch, "q_heads": wl.n_q_heads,
                   "kv_heads": wl.n_kv_heads, "head_dim": wl.head_dim, "vocab": wl.vocab,
                   "cache_len": wl.prefill, "fp16_window": wl.fp16_window, "budgets": [wl.n_tight[0], wl.n_loose[0]],
                   "protected": wl.protected, "kv_storage": "int8+fp16", "int8_scales": "per " + args.scales, "tokens_per_call": tq, "evict_page": args.evict_page, "layout": args.layout, "rank_scope": args.rank_scope, "attend_splits": kv.attend_splits(0),
                   "len_after": n_after, "tight_sequences": int(st.tight_steps > 0),
                   "between_steps": "cache re-loaded layer by layer, then 512 MiB of unrelated memory read (untimed)"},
        "roofline": {"bound": "hbm", "kernel": ("attend_wide_kernel" if tq * wl.group > 16 else "attend_mfma_kernel<16>" if tq > 1 else f"attend_mfma_kernel<{wl.group}>") if (tq > 1 or wl.group > 1) and wl.fp16_window >= 0 and wl.head_dim == 128 else "attend_kernel", "achieved": achieved,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": traffic, "traffic_source": traffic_file, "bytes_per_launch": att_bytes,
                     "launch_ms": att_launch_ms},
        "step_breakdown_ms": {"attend_x_layers": float(np.mean(t_att)), "confidence": float(np.mean(t_conf)),
                              "evict_compact": float(np.mean(t_evict))},
        "step_hbm": {"algorithmic_bytes": total_bytes, "compaction_bytes": moved, "achieved_GBps": total_bytes / (ms_step * 1e-3) / 1e9,
                     "frac_of_peak": total_bytes / (ms_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
                     "attend_GBps": att_total / (float(np.mean(t_att)) * 1e-3) / 1e9},
    }
    if cpu is not None:
        result["cpu_baseline"] = cpu
    kv.close()
    del kv, prompts
    torch.cuda.empty_cache()
    result["roofline"]["read_probe"] = read_probe(torch, pkg, att_bytes)
    result["roofline"]["frac_of_read_probe"] = achieved / result["roofline"]["read_probe"]["stream_2GiB_GBps"]
    prop = torch.cuda.get_device_properties(0)
    result["device"] = {"name": prop.name, "arch": prop.gcnArchName, "compute_units": prop.multi_processor_count,
                        "wavefront": prop.warp_size, "lds_bytes_per_workgroup": prop.shared_memory_per_block,
                        "l2_bytes": prop.L2_cache_size, "hbm_bytes": prop.total_memory}
    print(json.dumps(result))


if __name__ == "__main__":
    main()
