"""Whole-length runs of the workloads against the oracle: record on the GPU, replay on the CPU.

A run of thousands of decode steps cannot wait for a float64 oracle between steps, so the
lock-step comparison is split in two:

  record   the HIP library runs every unit for the full number of steps on inputs drawn on the
           device (``synth.device_gen``).  For a seeded sample of units the harness keeps what
           those units consumed (prompt, per-step q / k / v slices, the sequence's tight / loose
           choice) and what the library produced for them (attention outputs, the kept position
           set after every step, the full cache state every ``full_every`` steps and at the end).
           The confidence of every sequence at every step is checked on the fly by a thread pool
           (Eq. 1 in float64 on the logits row copied back), and properties that hold for ALL
           units are checked every step from the library's own read-outs: length within budget,
           FP16 window respected, positions increasing, protected window intact.
  replay   one child process per group of units (the oracle never touches the GPU) walks the
           recorded steps with ``oracle.confkv_oracle``: attention output within tolerance, kept
           sets equal (a difference is measured against the cut-off in the oracle's float64
           scores: within 1e-6 relative it is a counted tie and the oracle adopts the GPU's set,
           beyond it the run fails), payload bits / codes / scales / tags equal and the EMA within
           tolerance at every full-state check point.

Nothing the oracle consumes comes from the HIP path except the kept set it adopts after a counted
tie, exactly as in the lock-step harness.
"""
from __future__ import annotations

import dataclasses
import json
import os
import subprocess
import sys
import tempfile
import time
from collections import deque
from concurrent.futures import ThreadPoolExecutor

import numpy as np

from synth import generate as gen
from synth.device_gen import DeviceInputs

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
sys.path.insert(0, HERE)
from harness import CONF_ATOL, TIE_REL, f32, pick_units  # noqa: E402

PLANES = ("pos", "ema", "is16", "k16", "v16", "k8", "v8", "ks", "vs")


def _conf_rows(rows, weights, tau, c_gpu, sel_gpu):
    """Eq. 1 in float64 on logit rows; returns (max |c - c_ref|, ties, flips)."""
    from oracle import confkv_oracle as O
    err, ties, flips = 0.0, 0, []
    for x, cg, sg in zip(rows, c_gpu, sel_gpu):
        c = O.confidence(x, weights)
        err = max(err, abs(float(cg) - c))
        if bool(sg) != (c >= tau):
            rel = abs(c - tau) / tau
            if rel <= TIE_REL:
                ties += 1
            else:
                flips.append(rel)
    return err, ties, flips


def record_and_replay(pkg, wl, seed: int, follow, steps: int, full_every: int, workers: int = 16,
                      needle_report: bool = False, log=print):
    """Runs `steps` decode steps of workload `wl` on the GPU and replays the followed units with
    the oracle.  Returns a summary dict; raises AssertionError on any parity failure."""
    import torch
    t_begin = time.time()
    L, B, Hkv, G, D, T0 = wl.n_layers, wl.batch, wl.n_kv_heads, wl.group, wl.head_dim, wl.prefill
    units = pick_units(wl, follow, seed)
    n = len(units)
    li = torch.tensor([u[0] for u in units], device="cuda")
    bi = torch.tensor([u[1] for u in units], device="cuda")
    gi = torch.tensor([u[2] for u in units], device="cuda")
    dg = DeviceInputs(wl, seed)
    kv = pkg.from_workload(wl)
    prompts = {}
    for l in range(L):
        K, V = dg.prefill_layer(l)
        kv.load_prefill(l, K, V)
        for i, (ul, b, g) in enumerate(units):
            if ul == l:
                prompts[i] = (K[b, g].cpu().numpy(), V[b, g].cpu().numpy())
        del K, V
    torch.cuda.synchronize()
    log(f"  prompt loaded in {time.time() - t_begin:.1f}s: {wl.units} units of {T0} slots, {n} followed, "
        f"attend splits {kv.attend_splits(0)}")

    rec_q = torch.empty((steps, n, G, D), dtype=torch.float16, device="cuda")
    rec_k = torch.empty((steps, n, D), dtype=torch.float16, device="cuda")
    rec_v = torch.empty((steps, n, D), dtype=torch.float16, device="cuda")
    rec_o = torch.empty((steps, n, G, D), dtype=torch.float16, device="cuda")
    rec_sel = np.zeros((steps, B), dtype=np.uint8)
    out_all = torch.empty((L, B, wl.n_q_heads, D), dtype=torch.float16, device="cuda")
    conf = torch.empty(B, dtype=torch.float32, device="cuda")
    sel = torch.empty(B, dtype=torch.uint8, device="cuda")
    pos_after = [[] for _ in range(n)]
    fulls = {}                                    # step -> list over units of export dicts
    weights = (f32(wl.w_entropy), f32(wl.w_margin), f32(wl.w_top))
    tau = f32(wl.tau)
    pool = ThreadPoolExecutor(max_workers=workers)
    pending = deque()
    conf_err, budget_ties, budget_flips = 0.0, 0, []
    n_tight = np.array(wl.n_tight)[:, None]
    n_loose = np.array(wl.n_loose)[:, None]
    lengths_trace, tight_steps = [], 0
    needles = gen.needle_slots(wl, seed)
    needle_rows = []
    rng = np.random.default_rng(seed + 99)

    def drain(keep: int):
        nonlocal conf_err, budget_ties, budget_flips
        while len(pending) > keep:
            e, ties, flips = pending.popleft().result()
            conf_err = max(conf_err, e)
            budget_ties += ties
            budget_flips += flips

    def needle_table(when):
        held = np.zeros(len(needles), dtype=np.int64)
        for l in range(L):
            for b in range(B):
                for g in range(Hkv):
                    held += np.isin(needles, kv.export(l, b, g, planes=("pos",))["pos"])
        needle_rows.append((when, (held / wl.units).tolist()))

    t_loop = time.time()
    for t in range(steps):
        q, k, v = dg.step_inputs(t)
        for l in range(L):
            kv.attend(l, q[l], k[l], v[l], out_all[l])
        logits = dg.step_logits(t)
        kv.step(logits, conf, sel)
        kv.evict_compact()
        rec_q[t] = q.view(L, B, Hkv, G, D)[li, bi, gi]
        rec_k[t] = k[li, bi, gi]
        rec_v[t] = v[li, bi, gi]
        rec_o[t] = out_all.view(L, B, Hkv, G, D)[li, bi, gi]
        conf_h, sel_h = conf.cpu().numpy(), sel.cpu().numpy()           # (synchronises)
        rec_sel[t] = sel_h
        tight_steps += int(sel_h.sum())
        pending.append(pool.submit(_conf_rows, logits.cpu().numpy(), weights, tau, conf_h, sel_h))
        drain(48)
        # ---- every unit, from the library's read-outs ----
        ln, n16 = kv.lengths()
        N = np.where(sel_h[None, :].astype(bool), n_tight, n_loose)
        assert np.all(ln <= np.maximum(N, wl.protected)), f"step {t}: a cache is over its budget"
        if wl.fp16_window >= 0:
            assert n16.max() <= wl.fp16_window, f"step {t}: FP16 window exceeded"
        lengths_trace.append(int(ln[0, 0]))
        newest = T0 + t
        for _ in range(2):
            l, b, g = int(rng.integers(L)), int(rng.integers(B)), int(rng.integers(Hkv))
            pos = kv.export(l, b, g, planes=("pos",))["pos"]
            P = min(wl.protected, pos.size)
            assert np.all(np.diff(pos) > 0), f"step {t} unit {(l, b, g)}: positions not increasing"
            assert np.array_equal(pos[-P:], np.arange(newest - P + 1, newest + 1)), \
                f"step {t} unit {(l, b, g)}: protected window broken"
        # ---- followed units: kept sets every step, full state at the check points ----
        for i, key in enumerate(units):
            pos_after[i].append(kv.export(*key, planes=("pos",))["pos"].copy())
        if (t + 1) % full_every == 0 or t == steps - 1:
            fulls[t] = [kv.export(*key) for key in units]
        if needle_report and needles.size and (gen.is_probe_step(wl, t) or t == steps - 1):
            needle_table(t)
        if (t + 1) % max(1, steps // 8) == 0:
            log(f"  step {t + 1}/{steps}: len={lengths_trace[-1]} tight so far {tight_steps} "
                f"({time.time() - t_loop:.1f}s)")
    drain(0)
    pool.shutdown()
    st = kv.counters()
    gpu_s = time.time() - t_loop
    assert st.device_errors == 0
    assert conf_err <= CONF_ATOL, f"confidence off by {conf_err:.3g}"
    assert not budget_flips, f"budget choices differ beyond a tie: {budget_flips[:5]}"

    # ---- hand the records to the replay processes ----
    q_h, k_h, v_h, o_h = (x.cpu().numpy() for x in (rec_q, rec_k, rec_v, rec_o))
    tmp = tempfile.mkdtemp(prefix="confkv_replay_")
    meta = dict(workload=dataclasses.asdict(wl), steps=steps, full_steps=sorted(fulls), units=[list(u) for u in units])
    groups = [list(range(i, n, min(workers, n))) for i in range(min(workers, n))]
    procs = []
    env = dict(os.environ, OMP_NUM_THREADS="1", OPENBLAS_NUM_THREADS="1", MKL_NUM_THREADS="1",
               PYTHONPATH=ROOT + os.pathsep + os.environ.get("PYTHONPATH", ""))
    for gidx, members in enumerate(groups):
        arrays = {}
        for i in members:
            b = units[i][1]
            arrays[f"K0_{i}"], arrays[f"V0_{i}"] = prompts[i]
            arrays[f"q_{i}"], arrays[f"k_{i}"], arrays[f"v_{i}"], arrays[f"o_{i}"] = q_h[:, i], k_h[:, i], v_h[:, i], o_h[:, i]
            arrays[f"sel_{i}"] = rec_sel[:, b]
            arrays[f"pos_{i}"] = np.concatenate(pos_after[i]) if steps else np.zeros(0, np.int32)
            arrays[f"posoff_{i}"] = np.concatenate([[0], np.cumsum([p.size for p in pos_after[i]])]).astype(np.int64)
            for s, exports in fulls.items():
                for name in PLANES:
                    arrays[f"full_{s}_{i}_{name}"] = exports[i][name]
        path = os.path.join(tmp, f"group{gidx}.npz")
        np.savez(path, **arrays)
        with open(path + ".json", "w") as f:
            json.dump(dict(meta, members=members), f)
        procs.append((path, subprocess.Popen([sys.executable, os.path.join(HERE, "replay_unit.py"), path],
                                             env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    t_rep = time.time()
    reports, failures = [], []
    for path, p in procs:
        out, _ = p.communicate()
        if p.returncode != 0:
            failures.append(out[-2000:])
            continue
        with open(path + ".out.json") as f:
            reports.append(json.load(f))
    for name in os.listdir(tmp):
        os.remove(os.path.join(tmp, name))
    os.rmdir(tmp)
    assert not failures, "replay failed:\n" + "\n----\n".join(failures)
    summary = dict(
        workload=wl.name, steps=steps, units_total=wl.units, units_followed=n,
        unit_steps=sum(r["unit_steps"] for r in reports),
        max_out_err_x_tol=max(r["max_out_err"] for r in reports),
        max_conf_err=conf_err, max_ema_rel=max(r["max_ema_rel"] for r in reports),
        evictions_followed=sum(r["evictions"] for r in reports),
        evict_ties=sum(r["evict_ties"] for r in reports), evict_flips=sum((r["evict_flips"] for r in reports), []),
        budget_ties=budget_ties, tight_sequence_steps=tight_steps, full_state_checks=len(fulls) * n,
        evicted_all_units=int(st.evicted), demoted_all_units=int(st.demoted),
        length_min=min(lengths_trace), length_max=max(lengths_trace),
        sawtooth_drops=int(np.sum(np.diff(lengths_trace) < -1)),
        gpu_loop_s=gpu_s, replay_s=time.time() - t_rep, needles=needle_rows)
    kv.close()
    assert not summary["evict_flips"], f"kept sets differ beyond a tie: {summary['evict_flips'][:5]}"
    assert summary["max_out_err_x_tol"] <= 1.0
    return summary
