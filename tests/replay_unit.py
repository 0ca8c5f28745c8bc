"""Replay of recorded units with the CPU oracle (child process of tests/longrun.py; no GPU).

usage: python tests/replay_unit.py <group.npz>      (reads <group.npz>.json, writes <group.npz>.out.json)

For every recorded unit: load the prompt, then per decode step feed the recorded q / k / v slice to
``oracle.attend_unit``, compare the attention output, apply the recorded tight / loose choice,
evict and demote with the oracle and compare the kept positions with the recorded ones; at the
check points compare the whole cache state.  Exits non-zero with the message of the first failed
comparison.
"""
from __future__ import annotations

import json
import os
import sys

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(HERE))
sys.path.insert(0, HERE)

from oracle import confkv_oracle as O  # noqa: E402
from synth.workloads import Workload  # noqa: E402
from harness import OUT_ATOL, OUT_RTOL, Report, adopt_gpu_choice, compare_unit_state, policy_of  # noqa: E402

PLANES = ("pos", "ema", "is16", "k16", "v16", "k8", "v8", "ks", "vs")


def main(path: str) -> None:
    meta = json.load(open(path + ".json"))
    w = meta["workload"]
    for key in ("n_tight", "n_loose", "logit_std"):
        w[key] = tuple(w[key])
    wl = Workload(**w)
    pol = policy_of(wl)
    data = np.load(path)
    steps, T0 = meta["steps"], wl.prefill
    full_steps = set(meta["full_steps"])
    rep = Report()
    lengths = []
    for i in meta["members"]:
        l, b, g = meta["units"][i]
        key = (l, b, g)
        u = O.load_prefill(data[f"K0_{i}"], data[f"V0_{i}"], wl.fp16_window, scale_mode=wl.scale_mode)
        q, k, v, o, sel = (data[f"{n}_{i}"] for n in ("q", "k", "v", "o", "sel"))
        pos_all, off = data[f"pos_{i}"], data[f"posoff_{i}"]
        for t in range(steps):
            ref, _ = O.attend_unit(u, q[t], k[t], v[t], T0 + t, pol.sm_scale, pol.ema_decay, pol.mass_gain)
            err = float(np.max(np.abs(o[t].astype(np.float64) - ref) / (OUT_ATOL + OUT_RTOL * np.abs(ref))))
            rep.max_out_err = max(rep.max_out_err, err)
            assert err <= 1.0, f"step {t} unit {key}: attention output off by {err:.3g} x tolerance"
            tight = bool(sel[t])
            N = pol.n_tight[l] if tight else pol.n_loose[l]
            gpu_pos = pos_all[off[t]:off[t + 1]].astype(np.int64)
            keep, evict = O.select_evictions(u, N, pol.protected, pol.alpha, ranker=pol.ranker, seed=pol.ranker_seed,
                                             unit_key=(l * pol.batch + b) * pol.n_kv_heads + g, page=pol.evict_page)
            rep.evictions += int(evict.size)
            if np.array_equal(u.pos[keep], gpu_pos):
                if evict.size:
                    u.take(keep)
                O.demote(u, pol.fp16_window)
            else:
                u = adopt_gpu_choice(pol, l, key, u, gpu_pos, tight, rep)
            if t in full_steps:
                ex = {name: data[f"full_{t}_{i}_{name}"] for name in PLANES}
                ex["n"] = int(ex["pos"].shape[0])
                compare_unit_state(ex, u, f"after step {t} unit {key}", rep)
            if i == meta["members"][0]:
                lengths.append(u.n)
            rep.unit_steps += 1
    out = dict(unit_steps=rep.unit_steps, max_out_err=rep.max_out_err, max_ema_rel=rep.max_ema_rel,
               evictions=rep.evictions, evict_ties=rep.evict_ties, evict_flips=rep.evict_flips, lengths=lengths)
    with open(path + ".out.json", "w") as f:
        json.dump(out, f)


if __name__ == "__main__":
    try:
        main(sys.argv[1])
    except AssertionError as e:
        print(f"PARITY FAILURE: {e}")
        sys.exit(3)
