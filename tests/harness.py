"""Lock-step parity harness: the HIP library against the CPU oracle on the same seeded inputs.

Units (layer, batch, kv-head) evolve independently given their inputs and their sequence's
budget, so the oracle follows a chosen subset of units while the GPU runs all of them.
Per step the harness compares, for every followed unit: the attention output (2e-3 rel /
1e-3 abs), the confidence (1e-5 abs), the tight/loose choice, and after eviction the kept
position set, the precision tags, the FP16 payload bits, the INT8 codes and scales
(all bit-exact) and the EMA (diagnostic tolerance).  A discrete mismatch is classified by
its distance to the decision threshold measured in the ORACLE's float64 values; the
oracle then adopts the GPU's choice so later steps stay comparable.
"""
from __future__ import annotations

import copy
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

from oracle import confkv_oracle as O
from synth import generate as gen

OUT_RTOL, OUT_ATOL = 2e-3, 1e-3
CONF_ATOL = 1e-5
TIE_REL = 1e-6
EMA_RTOL, EMA_ATOL = 1e-5, 1e-8


def f32(x) -> float:
    return float(np.float32(x))


def policy_of(wl) -> O.Policy:
    return O.Policy(wl.n_layers, list(wl.n_tight), list(wl.n_loose), wl.protected, wl.fp16_window,
                    tau=f32(wl.tau), alpha=f32(wl.alpha), ema_decay=f32(wl.ema_decay),
                    sm_scale=f32(1.0 / np.sqrt(wl.head_dim)),
                    weights=(f32(wl.w_entropy), f32(wl.w_margin), f32(wl.w_top)),
                    mass_gain=None if getattr(wl, "mass_gain", None) is None else f32(wl.mass_gain),
                    ranker=getattr(wl, "ranker", "composite"), rank_scope=getattr(wl, "rank_scope", "kv_head"),
                    ranker_seed=getattr(wl, "ranker_seed", 0), evict_page=getattr(wl, "evict_page", 0),
                    batch=wl.batch, n_kv_heads=wl.n_kv_heads)


@dataclass
class Report:
    steps: int = 0
    unit_steps: int = 0
    max_out_err: float = 0.0          # max over elements of |gpu - ref| / (atol + rtol |ref|)
    max_conf_err: float = 0.0
    max_ema_rel: float = 0.0
    budget_ties: int = 0              # tight/loose flips with |c - tau| <= 1e-6 tau
    budget_flips: List[float] = field(default_factory=list)   # relative distances of the others
    evict_ties: int = 0               # kept-set flips within 1e-6 relative of the cut-off
    evict_flips: List[float] = field(default_factory=list)
    evictions: int = 0
    tight_steps: int = 0
    lengths: List[int] = field(default_factory=list)          # length of the first followed unit

    def ok(self) -> bool:
        return (self.max_out_err <= 1.0 and self.max_conf_err <= CONF_ATOL
                and not self.budget_flips and not self.evict_flips)


def pick_units(wl, count: Optional[int], seed: int = 0) -> List[Tuple[int, int, int]]:
    allu = [(l, b, g) for l in range(wl.n_layers) for b in range(wl.batch) for g in range(wl.n_kv_heads)]
    if count is None or count >= len(allu):
        return allu
    rng = np.random.default_rng(1000 + seed)
    idx = sorted(rng.choice(len(allu), size=count, replace=False))
    return [allu[i] for i in idx]


def compare_unit_state(ex: dict, u: O.UnitCache, tag: str, rep: Report) -> None:
    """One exported unit (the dict ConfKV.export returns) against the oracle's unit: length, kept
    positions, precision tags, FP16 payload bits, INT8 codes and scales bit for bit; the EMA
    within EMA_RTOL / EMA_ATOL."""
    assert ex["n"] == u.n, f"{tag}: length gpu {ex['n']} oracle {u.n}"
    assert np.array_equal(ex["pos"], u.pos.astype(np.int32)), f"{tag}: kept positions differ"
    assert np.array_equal(ex["is16"], u.is16), f"{tag}: precision tags differ"
    m16, m8 = u.is16, ~u.is16
    for name in ("k16", "v16"):
        assert np.array_equal(ex[name][m16].view(np.uint16), getattr(u, name)[m16].view(np.uint16)), \
            f"{tag}: {name} payload bits differ"
    for name in ("k8", "v8"):
        assert np.array_equal(ex[name][m8], getattr(u, name)[m8]), f"{tag}: {name} codes differ"
    if u.kcs is not None:
        assert np.array_equal(ex["ks"].view(np.uint16), u.kcs.view(np.uint16)), f"{tag}: K channel scales differ"
        assert np.array_equal(ex["vs"].view(np.uint16), u.vcs.view(np.uint16)), f"{tag}: V channel scales differ"
    else:
        for name in ("ks", "vs"):
            assert np.array_equal(ex[name][m8].view(np.uint16), getattr(u, name)[m8].view(np.uint16)), \
                f"{tag}: {name} scales differ"
    ref = u.ema.astype(np.float64)
    err = np.abs(ex["ema"].astype(np.float64) - ref)
    bound = EMA_ATOL + EMA_RTOL * np.abs(ref)
    assert np.all(err <= bound), f"{tag}: EMA off by {np.max(err / bound):.3g} x tolerance"
    nz = ref > 1e-12
    if nz.any():
        rep.max_ema_rel = max(rep.max_ema_rel, float(np.max(err[nz] / ref[nz])))


def adopt_gpu_choice(p: O.Policy, layer: int, key, pre: O.UnitCache, gpu_pos: np.ndarray, tight: bool,
                     rep: Report) -> O.UnitCache:
    """Kept sets differ: measure, in the oracle's float64 scores, how close the disputed slots were
    to the cut-off (within TIE_REL: a counted tie, else a flip that fails the run), then replay the
    oracle's compaction with the GPU's kept set so later steps stay comparable."""
    N = p.n_tight[layer] if tight else p.n_loose[layer]
    n = pre.n
    if p.evict_page > 1 or p.ranker != "composite" or p.rank_scope != "kv_head":
        # no near-tie analysis for the variants: any difference counts as a flip
        rep.evict_flips.append(1.0)
        u = pre.copy()
        u.take(np.flatnonzero(np.isin(pre.pos, gpu_pos)))
        O.demote(u, p.fp16_window)
        return u
    p_eff = min(p.protected, n)
    ncand = n - p_eff
    s = O.rank_scores(pre.ema[:ncand], pre.pos[:ncand], p.alpha)
    keep_o, evict_o = O.select_evictions(pre, N, p.protected, p.alpha)
    keep_g = np.flatnonzero(np.isin(pre.pos, gpu_pos))
    assert keep_g.size == gpu_pos.size == keep_o.size, f"unit {key}: kept-set sizes differ"
    disputed = np.setxor1d(keep_o, keep_g)
    assert np.all(disputed < ncand), f"unit {key}: a protected slot is disputed"
    cut = np.max(s[evict_o])                       # highest evicted score = the cut-off
    rel = float(np.max(np.abs(s[disputed] - cut)) / max(abs(cut), 1e-300))
    if rel <= TIE_REL:
        rep.evict_ties += 1
    else:
        rep.evict_flips.append(rel)
    u = pre.copy()
    u.take(keep_g)
    O.demote(u, p.fp16_window)
    return u


class Lockstep:
    def __init__(self, pkg, wl, seed: int = 0, units: Optional[int] = None, threads: int = 8,
                 ema0: bool = False, **override):
        import torch
        self.torch = torch
        self.wl, self.seed = wl, seed
        self.kv = pkg.from_workload(wl, **override)
        self.units = pick_units(wl, units, seed)
        self.report = Report()
        followed_layers = {l for (l, _, _) in self.units}
        ounits: Dict[Tuple[int, int, int], O.UnitCache] = {}
        for l in range(wl.n_layers):
            K, V = gen.prefill_layer(wl, seed, l, threads=threads)
            e0 = None
            if ema0:
                e0 = np.random.default_rng(77 + l).random((wl.batch, wl.n_kv_heads, wl.prefill)).astype(np.float32)
            self.kv.load_prefill(l, torch.from_numpy(K).cuda(), torch.from_numpy(V).cuda(),
                                 None if e0 is None else torch.from_numpy(e0).cuda())
            if l in followed_layers:
                for (ul, b, g) in self.units:
                    if ul == l:
                        ounits[(l, b, g)] = O.load_prefill(K[b, g], V[b, g], wl.fp16_window,
                                                           None if e0 is None else e0[b, g],
                                                           scale_mode=getattr(wl, "scale_mode", "token"))
        torch.cuda.synchronize()
        self.run = O.OracleRun(policy_of(wl), ounits, wl.prefill)
        self.t = 0
        B, Hq, D = wl.batch, wl.n_q_heads, wl.head_dim
        self.out = torch.empty((B, Hq, D), dtype=torch.float16, device="cuda")
        self.conf = torch.empty(B, dtype=torch.float32, device="cuda")
        self.sel = torch.empty(B, dtype=torch.uint8, device="cuda")

    # ---- comparisons ----
    def compare_state(self, when: str):
        for key, u in self.run.units.items():
            compare_unit_state(self.kv.export(*key), u, f"{when} step {self.t} unit {key}", self.report)

    # ---- the prompt's own attention, before the decode loop ----
    def observe(self, first: int, tq: int, want_out: bool = True):
        """One conf_kv_observe call per layer over the cached slots first .. first + tq - 1 with
        seeded queries (drawn like decode queries, from a step index of their own); outputs and
        state of the followed units are compared with the oracle's."""
        torch, wl, kv, rep = self.torch, self.wl, self.kv, self.report
        G = wl.group
        for l in range(wl.n_layers):
            parts = [gen.step_inputs(wl, self.seed + 7919, l, first + i)[0] for i in range(tq)]
            q = np.ascontiguousarray(np.stack(parts, axis=1))                      # [B][tq][Hq][D]
            out = torch.empty((wl.batch, tq, wl.n_q_heads, wl.head_dim), dtype=torch.float16,
                              device="cuda") if want_out else None
            kv.observe(l, first, torch.from_numpy(q).cuda(), out)
            ref = self.run.observe(l, q, first, G)
            if ref and want_out:
                got = out.cpu().numpy().astype(np.float64)
                for (ul, b, g), r in ref.items():
                    o = got[b, :, g * G:(g + 1) * G]
                    err = np.max(np.abs(o - r) / (OUT_ATOL + OUT_RTOL * np.abs(r)))
                    rep.max_out_err = max(rep.max_out_err, float(err))
                    assert err <= 1.0, f"observe {first}+{tq} unit {(ul, b, g)}: out off by {err:.3g} x tolerance"
        self.compare_state(f"after observe {first}+{tq}")

    # ---- a decode step recorded once into a HIP graph and replayed ----
    def record_step(self, tq: int = 1):
        """Record the calls of one decode step (one conf_kv_attend -- or, with tq > 1, one
        conf_kv_attend_chunk of tq tokens -- per layer, conf_kv_step, conf_kv_evict_compact) into
        a graph over fixed input / output tensors.  Nothing runs while recording; every later
        ``step`` fills the tensors and replays the graph."""
        torch, wl, kv = self.torch, self.wl, self.kv
        L, B, Hq, Hkv, D = wl.n_layers, wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim
        tok = () if tq == 1 else (tq,)
        self.gq = torch.zeros((L, B) + tok + (Hq, D), dtype=torch.float16, device="cuda")
        self.gk = torch.zeros((L, B) + tok + (Hkv, D), dtype=torch.float16, device="cuda")
        self.gv = torch.zeros((L, B) + tok + (Hkv, D), dtype=torch.float16, device="cuda")
        self.gout = torch.zeros((L, B) + tok + (Hq, D), dtype=torch.float16, device="cuda")
        self.glogits = torch.zeros((B, wl.vocab), dtype=torch.float32, device="cuda")
        self.graph = torch.cuda.CUDAGraph()
        self.graph_tq = tq
        with torch.cuda.graph(self.graph):
            for l in range(L):
                if tq == 1:
                    kv.attend(l, self.gq[l], self.gk[l], self.gv[l], self.gout[l])
                else:
                    kv.attend_chunk(l, self.gq[l], self.gk[l], self.gv[l], self.gout[l])
            kv.step(self.glogits, self.conf, self.sel)
            kv.evict_compact()
        self.replays = 0

    def _replay(self):
        """Fill the recorded tensors with this step's inputs and replay; returns the per-layer
        (q, k, v) the oracle gets and the outputs ([L][B][Hq][D], or [L][B][tq][Hq][D])."""
        torch, wl, tq = self.torch, self.wl, self.graph_tq
        if tq == 1:
            ins = [gen.step_inputs(wl, self.seed, l, self.t) for l in range(wl.n_layers)]
        else:
            ins = []
            for l in range(wl.n_layers):
                parts = [gen.step_inputs(wl, self.seed, l, self.t + i) for i in range(tq)]
                ins.append(tuple(np.ascontiguousarray(np.stack([p[j] for p in parts], axis=1)) for j in range(3)))
        for j, dst in enumerate((self.gq, self.gk, self.gv)):
            dst.copy_(torch.from_numpy(np.stack([x[j] for x in ins])))
        self.glogits.copy_(torch.from_numpy(gen.step_logits(wl, self.seed, self.t + tq - 1)))
        self.gout.zero_()
        self.graph.replay()
        self.replays += 1
        return ins, self.gout.cpu().numpy().astype(np.float64)

    # ---- one decode step ----
    def step(self, check_state: bool = True, tq: int = 1):
        """One decode step; tq > 1 feeds tq tokens through one conf_kv_attend_chunk call per
        layer (the inputs of steps t .. t + tq - 1, the logits of the last one).  After
        ``record_step`` the GPU side of the step is a replay of the recorded graph."""
        torch, wl, kv, rep = self.torch, self.wl, self.kv, self.report
        G = wl.group
        replayed = None
        if getattr(self, "graph", None) is not None:
            assert tq == self.graph_tq, "a recorded step is replayed with the token count it was recorded with"
            replayed = self._replay()
        for l in range(wl.n_layers):
            if replayed is not None and tq == 1:
                q, k, v = replayed[0][l]
                ref = self.run.attend(l, q, k, v, G)
                got = replayed[1][l]
            elif replayed is not None:
                q, k, v = replayed[0][l]
                ref = self.run.attend_chunk(l, q, k, v, G)
                got = replayed[1][l].transpose(0, 2, 1, 3)                       # [B][Hq][tq][D]
                ref = {key: r.transpose(1, 0, 2) for key, r in ref.items()}      # [G][tq][D]
            elif tq == 1:
                q, k, v = gen.step_inputs(wl, self.seed, l, self.t)
                kv.attend(l, torch.from_numpy(q).cuda(), torch.from_numpy(k).cuda(),
                          torch.from_numpy(v).cuda(), self.out)
                ref = self.run.attend(l, q, k, v, G)
                got = self.out.cpu().numpy().astype(np.float64) if ref else None
            else:
                parts = [gen.step_inputs(wl, self.seed, l, self.t + i) for i in range(tq)]
                q, k, v = (np.ascontiguousarray(np.stack([p[j] for p in parts], axis=1)) for j in range(3))
                out = torch.empty((wl.batch, tq, wl.n_q_heads, wl.head_dim), dtype=torch.float16, device="cuda")
                kv.attend_chunk(l, torch.from_numpy(q).cuda(), torch.from_numpy(k).cuda(),
                                torch.from_numpy(v).cuda(), out)
                ref = self.run.attend_chunk(l, q, k, v, G)
                # [B][tq][Hq][D] -> per unit [tq][G][D], compared like the single-token case
                got = out.cpu().numpy().astype(np.float64).transpose(0, 2, 1, 3) if ref else None
                ref = {key: r.transpose(1, 0, 2) for key, r in ref.items()}      # [G][tq][D]
            if ref:
                for (ul, b, g), r in ref.items():
                    o = got[b, g * G:(g + 1) * G]
                    err = np.max(np.abs(o - r) / (OUT_ATOL + OUT_RTOL * np.abs(r)))
                    rep.max_out_err = max(rep.max_out_err, float(err))
                    assert err <= 1.0, f"step {self.t} unit {(ul, b, g)}: attention output off by {err:.3g} x tolerance"
        logits = gen.step_logits(wl, self.seed, self.t + tq - 1)
        if replayed is None:
            kv.step(torch.from_numpy(logits).cuda(), self.conf, self.sel)
        c_ref, tight_ref = self.run.step(logits)
        c_gpu = self.conf.cpu().numpy().astype(np.float64)
        sel_gpu = self.sel.cpu().numpy().astype(bool)
        cerr = float(np.max(np.abs(c_gpu - c_ref)))
        rep.max_conf_err = max(rep.max_conf_err, cerr)
        assert cerr <= CONF_ATOL, f"step {self.t}: confidence off by {cerr:.3g}"
        tau = self.run.policy.tau
        for b in range(wl.batch):
            if sel_gpu[b] != tight_ref[b]:
                rel = abs(c_ref[b] - tau) / tau
                if rel <= TIE_REL:
                    rep.budget_ties += 1
                else:
                    rep.budget_flips.append(rel)
        rep.tight_steps += int(sel_gpu.sum())
        # eviction: keep pre-evict copies so the oracle can adopt a GPU tie-break
        before = {key: u.copy() for key, u in self.run.units.items()}
        if replayed is None:
            kv.evict_compact()
        gone = self.run.evict_compact(sel_gpu)      # the oracle follows the GPU's budget choice
        self.last_before, self.last_gone = before, gone
        for key, u in self.run.units.items():
            ex_pos = self.kv.export(*key)["pos"].astype(np.int64)
            rep.evictions += int(gone[key].size)
            if np.array_equal(ex_pos, u.pos):
                continue
            self._adopt(key, before[key], ex_pos, sel_gpu[key[1]])
        if check_state:
            self.compare_state("after evict")
        self.t += tq
        rep.steps += 1
        rep.unit_steps += len(self.run.units)
        first = next(iter(self.run.units.values()))
        rep.lengths.append(first.n)

    def _adopt(self, key, pre: O.UnitCache, gpu_pos: np.ndarray, tight: bool):
        self.run.units[key] = adopt_gpu_choice(self.run.policy, key[0], key, pre, gpu_pos, tight, self.report)

    def close(self):
        self.kv.close()
