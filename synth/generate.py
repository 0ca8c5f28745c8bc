"""Seeded synthetic input tensors for the workloads in ``synth.workloads``.

Every tensor is a pure function of (seed, workload recipe, tensor id, indices):
the stream is numpy's counter-based Philox generator keyed by a SeedSequence of
those integers, so any single unit (layer, batch, kv-head) or step can be
regenerated on its own, in any order, on any machine.  Values are drawn as
float32 normals and stored as fp16 (Q, K, V) or fp32 (logits); the *stored*
arrays are what both the CPU oracle and the HIP path consume.

Recipe (stand-in for the paper's real activations, which need trained weights):
  * keys/values ~ N(0, 1) i.i.d.;
  * every (layer, kv-head) has a fixed unit vector u; a key position is a heavy
    hitter with probability ``heavy_hitter_prob`` and then gets + gain * u;
  * queries are z + sqrt(D) * u with z ~ N(0, I), so heavy hitters score about
    +gain above the rest after the 1/sqrt(D) softmax scale;
  * logits ~ N(0, s_t) with the standard deviation s_t alternating in runs;
  * retrieval workload: needle keys gain * sqrt(D)... see ``prefill_unit``.
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from typing import Tuple

import numpy as np

from .workloads import Workload

# tensor ids (first key word after the seed)
_T_DIR, _T_PREFILL, _T_STEP_Q, _T_STEP_KV, _T_LOGITS, _T_NEEDLE, _T_HH = range(1, 8)


def _rng(seed: int, *ids: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(np.random.SeedSequence([seed, *ids])))


def unit_direction(wl: Workload, seed: int, layer: int, kv_head: int) -> np.ndarray:
    """The fixed unit vector u of one (layer, kv-head), float64 [D]."""
    g = _rng(seed, _T_DIR, layer, kv_head)
    v = g.standard_normal(wl.head_dim)
    return v / np.sqrt(np.sum(v * v))


def needle_slots(wl: Workload, seed: int) -> np.ndarray:
    """Prefill positions of the planted needles (shared by all units), sorted, distinct."""
    if wl.n_needles == 0:
        return np.zeros(0, dtype=np.int64)
    g = _rng(seed, _T_NEEDLE)
    slots = set()
    while len(slots) < wl.n_needles:
        slots.add(int(g.random() * wl.prefill))
    return np.array(sorted(slots), dtype=np.int64)


def prefill_unit(wl: Workload, seed: int, layer: int, b: int, kv_head: int
                 ) -> Tuple[np.ndarray, np.ndarray]:
    """Prefill K and V of one unit: fp16 [T0, D] each, position-ordered."""
    g = _rng(seed, _T_PREFILL, layer, b, kv_head)
    T, D = wl.prefill, wl.head_dim
    k = g.standard_normal((T, D), dtype=np.float32)
    v = g.standard_normal((T, D), dtype=np.float32)
    u = unit_direction(wl, seed, layer, kv_head).astype(np.float32)
    if wl.heavy_hitter_prob > 0.0:
        hh = g.random(T) < wl.heavy_hitter_prob
        k[hh] += np.float32(wl.heavy_hitter_gain) * u
    if wl.n_needles:
        # a needle key is the unit probe direction times the gain, in score units:
        # probe query sqrt(D) u  .  needle gain*u  / sqrt(D)  = gain
        k[needle_slots(wl, seed)] = np.float32(wl.needle_gain) * u
    return k.astype(np.float16), v.astype(np.float16)


def prefill_heavy_hitters(wl: Workload, seed: int, layer: int, b: int, kv_head: int) -> np.ndarray:
    """Prompt positions of one unit whose keys got the heavy-hitter offset (same draws as
    ``prefill_unit``), sorted."""
    if wl.heavy_hitter_prob <= 0.0:
        return np.zeros(0, dtype=np.int64)
    g = _rng(seed, _T_PREFILL, layer, b, kv_head)
    T, D = wl.prefill, wl.head_dim
    g.standard_normal((T, D), dtype=np.float32)
    g.standard_normal((T, D), dtype=np.float32)
    return np.flatnonzero(g.random(T) < wl.heavy_hitter_prob).astype(np.int64)


def prefill_layer(wl: Workload, seed: int, layer: int, threads: int = 8
                  ) -> Tuple[np.ndarray, np.ndarray]:
    """Prefill K and V of one layer: fp16 [B, Hkv, T0, D] each."""
    B, H, T, D = wl.batch, wl.n_kv_heads, wl.prefill, wl.head_dim
    K = np.empty((B, H, T, D), dtype=np.float16)
    V = np.empty((B, H, T, D), dtype=np.float16)

    def fill(bh):
        b, h = divmod(bh, H)
        K[b, h], V[b, h] = prefill_unit(wl, seed, layer, b, h)

    if threads > 1 and B * H > 1:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(fill, range(B * H)))
    else:
        for bh in range(B * H):
            fill(bh)
    return K, V


def is_probe_step(wl: Workload, t: int) -> bool:
    return wl.probe_every > 0 and t % wl.probe_every == 0


def step_inputs(wl: Workload, seed: int, layer: int, t: int
                ) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Decode-step tensors of one layer: q fp16 [B, Hq, D], k_new and v_new fp16 [B, Hkv, D]."""
    B, Hq, Hkv, D, G = wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.group
    gq = _rng(seed, _T_STEP_Q, layer, t)
    gk = _rng(seed, _T_STEP_KV, layer, t)
    U = np.stack([unit_direction(wl, seed, layer, h) for h in range(Hkv)]).astype(np.float32)
    gain = np.float32(np.sqrt(D) if wl.query_mean_gain is None else wl.query_mean_gain)
    z = gq.standard_normal((B, Hq, D), dtype=np.float32)
    mean = np.repeat(U, G, axis=0)[None, :, :] * gain          # head h belongs to kv-head h // G
    if wl.probe_every > 0:
        q = mean + np.float32(0.0) * z if is_probe_step(wl, t) else z
    else:
        q = z + mean
    k = gk.standard_normal((B, Hkv, D), dtype=np.float32)
    v = gk.standard_normal((B, Hkv, D), dtype=np.float32)
    if wl.heavy_hitter_prob > 0.0:
        hh = gk.random((B, Hkv)) < wl.heavy_hitter_prob
        k += hh[:, :, None] * (np.float32(wl.heavy_hitter_gain) * U)[None, :, :]
    return q.astype(np.float16), k.astype(np.float16), v.astype(np.float16)


def logit_std(wl: Workload, t: int) -> float:
    if wl.probe_every > 0:
        return wl.probe_logit_std if is_probe_step(wl, t) else wl.offprobe_logit_std
    return wl.logit_std[(t // wl.logit_run) % len(wl.logit_std)]


def step_logits(wl: Workload, seed: int, t: int) -> np.ndarray:
    """Next-token logits of one decode step: fp32 [B, V]."""
    g = _rng(seed, _T_LOGITS, t)
    x = g.standard_normal((wl.batch, wl.vocab), dtype=np.float32)
    return x * np.float32(logit_std(wl, t))
