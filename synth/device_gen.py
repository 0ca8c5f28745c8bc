"""The recipe of ``synth.generate`` drawn on the GPU, for runs of thousands of decode steps.

Same structure (i.i.d. N(0,1) keys / values, heavy-hitter keys shifted along the unit's fixed
direction, queries with a persistent mean along it, probe steps and needles of the retrieval
workload, logits whose standard deviation alternates in runs), but the normals come from
torch's seeded device generator instead of numpy's Philox, so a whole step's tensors for all
layers cost three launches instead of seconds of host time.  Every tensor is a pure function
of (seed, tensor id, layer or step): the generator is re-seeded from those integers before
each draw.  The values are stored as fp16 (Q, K, V) / fp32 (logits) on the device; the HIP
path reads them there and the CPU oracle gets copies of the stored slices it follows, so both
sides consume the same stored arrays.  Data only: no arithmetic of the method lives here.
"""
from __future__ import annotations

import numpy as np

from . import generate as gen
from .workloads import Workload

_T_PREFILL, _T_STEP, _T_LOGITS = 11, 12, 13


def _mix(seed: int, *ids: int) -> int:
    """A 63-bit seed from the integers (an ordinary multiplicative hash; any injective-enough map does)."""
    x = (seed + 0x9E3779B97F4A7C15) & 0xFFFFFFFFFFFFFFFF
    for i in ids:
        x = ((x ^ (i + 0x632BE59BD9B4E019)) * 0xD1342543DE82EF95) & 0xFFFFFFFFFFFFFFFF
        x ^= x >> 32
    return x & 0x7FFFFFFFFFFFFFFF


class DeviceInputs:
    def __init__(self, wl: Workload, seed: int, device: str = "cuda"):
        import torch
        self.torch, self.wl, self.seed, self.device = torch, wl, seed, device
        self.g = torch.Generator(device=device)
        dirs = np.stack([[gen.unit_direction(wl, seed, l, h) for h in range(wl.n_kv_heads)]
                         for l in range(wl.n_layers)]).astype(np.float32)          # [L][Hkv][D]
        self.U = torch.from_numpy(dirs).to(device)
        self.needles = torch.from_numpy(gen.needle_slots(wl, seed)).to(device)
        gain = np.sqrt(wl.head_dim) if wl.query_mean_gain is None else wl.query_mean_gain
        self.q_mean = (self.U.repeat_interleave(wl.group, dim=1) * float(gain))[:, None]   # [L][1][Hq][D]

    def _randn(self, shape, *ids):
        self.g.manual_seed(_mix(self.seed, *ids))
        return self.torch.randn(shape, generator=self.g, device=self.device, dtype=self.torch.float32)

    def _rand(self, shape, *ids):
        self.g.manual_seed(_mix(self.seed, *ids))
        return self.torch.rand(shape, generator=self.g, device=self.device, dtype=self.torch.float32)

    def prefill_layer(self, layer: int):
        """Prompt K and V of one layer: fp16 [B][Hkv][T0][D] each, on the device."""
        wl, torch = self.wl, self.torch
        shape = (wl.batch, wl.n_kv_heads, wl.prefill, wl.head_dim)
        k = self._randn(shape, _T_PREFILL, layer, 0)
        v = self._randn(shape, _T_PREFILL, layer, 1)
        u = self.U[layer][None, :, None, :]                                          # [1][Hkv][1][D]
        if wl.heavy_hitter_prob > 0.0:
            hh = self._rand(shape[:3], _T_PREFILL, layer, 2) < wl.heavy_hitter_prob
            k += hh[..., None] * (float(wl.heavy_hitter_gain) * u)
        if wl.n_needles:
            k[:, :, self.needles] = (float(wl.needle_gain) * u).expand(wl.batch, -1, self.needles.numel(), -1)
        return k.to(torch.float16), v.to(torch.float16)

    def step_inputs(self, t: int):
        """Decode-step tensors of ALL layers: q fp16 [L][B][Hq][D], k_new / v_new fp16 [L][B][Hkv][D]."""
        wl, torch = self.wl, self.torch
        L, B, Hq, Hkv, D = wl.n_layers, wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim
        z = self._randn((L, B, Hq, D), _T_STEP, t, 0)
        if wl.probe_every > 0:
            q = self.q_mean.expand(L, B, Hq, D) if gen.is_probe_step(wl, t) else z
        else:
            q = z + self.q_mean
        k = self._randn((L, B, Hkv, D), _T_STEP, t, 1)
        v = self._randn((L, B, Hkv, D), _T_STEP, t, 2)
        if wl.heavy_hitter_prob > 0.0:
            hh = self._rand((L, B, Hkv), _T_STEP, t, 3) < wl.heavy_hitter_prob
            k += hh[..., None] * (float(wl.heavy_hitter_gain) * self.U[:, None])
        return q.to(torch.float16).contiguous(), k.to(torch.float16), v.to(torch.float16)

    def step_logits(self, t: int):
        """Next-token logits of one decode step: fp32 [B][V] on the device."""
        wl = self.wl
        x = self._randn((wl.batch, wl.vocab), _T_LOGITS, t)
        return x * float(gen.logit_std(wl, t))
