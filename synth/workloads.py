"""Shapes and policy parameters of the five seeded synthetic workloads.

Data only: this module (and the rest of ``synth``) holds no arithmetic of the
cache-management method.  Both the CPU oracle's tests and the HIP path's tests
take their shapes, hyper-parameters and input tensors from here.

Defaults not fixed by a workload follow the paper's hyper-parameter table
(Appendix "Reproducibility details", Table "Hyperparameter settings"):
tau = 0.7, alpha = 0.65 (0.70 for the retrieval workload), EMA decay 0.9,
confidence weights (0.4, 0.3, 0.3) from Eq. 1.
"""
from __future__ import annotations

import dataclasses
from dataclasses import dataclass, field
from typing import List, Optional, Tuple


@dataclass(frozen=True)
class Workload:
    name: str
    n_layers: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    vocab: int
    batch: int
    prefill: int                  # T0: tokens in every unit's cache before the first decode step
    steps: int                    # decode steps of the full run
    n_tight: Tuple[int, ...]      # per-layer N_high (budget on confident steps)
    n_loose: Tuple[int, ...]      # per-layer N_low  (budget on uncertain steps)
    protected: int                # P
    fp16_window: int              # W; < 0 means an FP16-only cache
    tau: float = 0.7
    alpha: float = 0.65
    ema_decay: float = 0.9
    w_entropy: float = 0.4
    w_margin: float = 0.3
    w_top: float = 0.3
    # ranker variants (configuration only; both implementations read them)
    mass_gain: Optional[float] = None    # None: 1 - ema_decay
    ranker: str = "composite"            # or "random"
    rank_scope: str = "kv_head"          # or "layer"
    ranker_seed: int = 0
    scale_mode: str = "token"            # or "channel": INT8 scales per (kv-head, channel)
    max_chunk: int = 0                   # most tokens per multi-token attend call (0: single-token only)
    evict_page: int = 0                  # > 1: whole pages of that many original positions are evicted
    layout: str = "contiguous"           # or "paged": INT8 slots in pages of evict_page reached through a block table
    # input recipe
    heavy_hitter_prob: float = 0.02      # fraction of key positions shifted by +3 u
    heavy_hitter_gain: float = 3.0
    query_mean_gain: Optional[float] = None   # None -> sqrt(head_dim); queries are z + gain * u
    logit_std: Tuple[float, ...] = (0.5, 6.0)  # alternates in runs of ``logit_run`` steps
    logit_run: int = 32
    # retrieval stress (workload 3) only
    n_needles: int = 0
    needle_gain: float = 6.0
    probe_every: int = 0                 # probe steps are t % probe_every == 0
    probe_logit_std: float = 0.5
    offprobe_logit_std: float = 6.0

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def units(self) -> int:
        return self.n_layers * self.batch * self.n_kv_heads

    @property
    def capacity(self) -> int:
        """Slots a unit needs: the longest cache it can ever hold, plus the append."""
        slack = self.evict_page - 1 if self.evict_page > 1 else 0     # a page reaching into the window stays
        longest = max(self.prefill, max(self.n_loose), self.protected + slack) + max(1, self.max_chunk)
        if self.layout == "paged":           # the FP16 slots' metadata rows and a partly filled page come on top
            longest += self.fp16_window + 16 + self.evict_page
        return ((longest + 63) // 64) * 64

    def scaled(self, **kw) -> "Workload":
        """A smaller copy (same recipe) for tests the oracle finishes in seconds."""
        return dataclasses.replace(self, **kw)


def linear_budgets(first: int, last: int, n_layers: int) -> Tuple[int, ...]:
    """Integer budgets falling linearly from ``first`` (layer 0) to ``last`` (last layer)."""
    if n_layers == 1:
        return (first,)
    span = first - last
    den = n_layers - 1
    return tuple(first - (span * l + den // 2) // den for l in range(n_layers))


def _uniform(n: int, n_layers: int) -> Tuple[int, ...]:
    return tuple([n] * n_layers)


def workload(index: int) -> Workload:
    """The five configurations the build is measured and checked on."""
    if index == 0:   # GPT-2-small shape, FP16-only cache
        return Workload("gpt2s_fp16_b1", 12, 12, 12, 64, 50257, 1, 512, 256,
                        _uniform(256, 12), _uniform(512, 12), 64, -1)
    if index == 1:   # Llama-3-8B shape, single-step microbenchmark
        return Workload("llama3_8b_b8_t4096_step", 32, 32, 8, 128, 128256, 8, 4096, 1,
                        _uniform(1024, 32), _uniform(2048, 32), 128, 128,
                        logit_std=(3.0,), logit_run=1)
    if index == 2:   # Qwen-32B shape, long generation
        return Workload("qwen32b_b1_long", 64, 40, 8, 128, 152064, 1, 4096, 4096,
                        _uniform(512, 64), _uniform(2048, 64), 128, 64)
    if index == 3:   # long-context retrieval stress
        return Workload("llama3_8b_b1_needle32k", 32, 32, 8, 128, 128256, 1, 32768, 512,
                        _uniform(512, 32), _uniform(4096, 32), 128, 128, alpha=0.70,
                        heavy_hitter_prob=0.0, n_needles=16, probe_every=32)
    if index == 4:   # pyramidal per-layer budgets at batch
        tight = linear_budgets(1024, 128, 32)
        return Workload("llama3_8b_b32_pyramid", 32, 32, 8, 128, 128256, 32, 2048, 2048,
                        tight, tuple(2 * n for n in tight), 64, 64)
    raise ValueError(f"no workload {index}")


def small(index: int) -> Workload:
    """Reduced copies that keep the recipe and span several tiles plus a ragged tail."""
    w = workload(index)
    if index == 0:
        return w.scaled(n_layers=2, n_q_heads=3, n_kv_heads=3, vocab=5003, prefill=200, steps=48,
                        n_tight=_uniform(96, 2), n_loose=_uniform(224, 2), protected=24,
                        logit_run=8)
    if index == 1:
        return w.scaled(n_layers=2, batch=2, n_q_heads=8, n_kv_heads=2, vocab=12007, prefill=777,
                        n_tight=_uniform(200, 2), n_loose=_uniform(400, 2), protected=40,
                        fp16_window=40, logit_std=(3.0, 6.0), logit_run=1)
    if index == 2:
        return w.scaled(n_layers=2, n_q_heads=10, n_kv_heads=2, vocab=9001, prefill=600, steps=40,
                        n_tight=_uniform(150, 2), n_loose=_uniform(610, 2), protected=48,
                        fp16_window=24, logit_run=6)
    if index == 3:
        return w.scaled(n_layers=2, n_q_heads=8, n_kv_heads=2, vocab=8009, prefill=3000, steps=20,
                        n_tight=_uniform(128, 2), n_loose=_uniform(700, 2), protected=32,
                        fp16_window=32, n_needles=6, probe_every=5)
    if index == 4:
        tight = linear_budgets(160, 40, 3)
        return w.scaled(n_layers=3, batch=3, n_q_heads=8, n_kv_heads=2, vocab=7001, prefill=300,
                        steps=40, n_tight=tight, n_loose=tuple(2 * n for n in tight),
                        protected=16, fp16_window=16, logit_run=5)
    raise ValueError(f"no workload {index}")
