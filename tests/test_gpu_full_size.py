"""Variants and edge shapes at full size (the five workloads themselves, at their full step
counts, are in test_gpu_configs.py).

The GPU runs every unit; the float64 oracle follows a seeded sample of units (units evolve
independently given their inputs and their sequence's budget) for a few decode steps; the
first step is always the heaviest one (full prompt length, largest eviction).  Properties that
hold at any size are checked on ALL units from the GPU state: lengths within budget, FP16
window respected, positions strictly increasing with the protected window intact.
"""
import os
import sys

import numpy as np
import pytest

from synth import generate as gen
from synth.workloads import workload

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
from harness import Lockstep  # noqa: E402

pytestmark = pytest.mark.gpu

def _invariants_all_units(ls, wl, step):
    kv = ls.kv
    ln, n16 = kv.lengths()
    sel = ls.sel.cpu().numpy().astype(bool)
    for l in range(wl.n_layers):
        for b in range(wl.batch):
            N = wl.n_tight[l] if sel[b] else wl.n_loose[l]
            assert ln[l, b] <= max(N, wl.protected), (l, b, ln[l, b], N)      # budget never exceeded
    if wl.fp16_window >= 0:
        assert n16.max() <= wl.fp16_window
    rng = np.random.default_rng(step)
    for _ in range(6):                                                          # spot-check exports
        l, b, g = int(rng.integers(wl.n_layers)), int(rng.integers(wl.batch)), int(rng.integers(wl.n_kv_heads))
        ex = kv.export(l, b, g)
        pos = ex["pos"]
        assert np.all(np.diff(pos) > 0)
        P = min(wl.protected, ex["n"])
        newest = wl.prefill + step
        assert np.array_equal(pos[-P:], np.arange(newest - P + 1, newest + 1))  # protected window kept
        assert not ex["is16"][:ex["n"] - n16[l, b, g]].any() and ex["is16"][ex["n"] - n16[l, b, g]:].all()


def test_full_size_channel_scales(lib):
    """The roofline workload's shape with INT8 scales per (kv-head, channel): 4 of its layers,
    the prompt calibration over 4096 tokens, the first step's large eviction and demotion."""
    wl = workload(1).scaled(name="llama3_8b_b8_t4096_channel_scales", n_layers=4, n_tight=(1024,) * 4,
                            n_loose=(2048,) * 4, steps=3, scale_mode="channel", logit_std=(0.5, 6.0), logit_run=1)
    print(f"channel scales at full size: {wl.units} units of {wl.prefill} slots", flush=True)
    ls = Lockstep(lib, wl, seed=0, units=6, threads=16)
    for t in range(wl.steps):
        ls.step()
        _invariants_all_units(ls, wl, t)
        print(f"  step {t}: len={ls.report.lengths[-1]} out_err={ls.report.max_out_err:.3f}xtol", flush=True)
    rep = ls.report
    print(f"  ema_rel={rep.max_ema_rel:.2e} evictions={rep.evictions} flips={rep.evict_flips}/{rep.budget_flips}", flush=True)
    assert rep.ok(), (rep.evict_flips, rep.budget_flips)
    assert ls.kv.counters().device_errors == 0
    ls.close()


def test_full_size_chunks(lib):
    """Four tokens per attention call at the roofline workload's shape (4 of its layers): the
    16-row score stash only just fits next to the tile buffers, the chunk straddles the splits'
    FP16 shares, and the first step's eviction takes 2052 tokens per unit."""
    wl = workload(1).scaled(name="llama3_8b_b8_t4096_chunk4", n_layers=4, n_tight=(1024,) * 4,
                            n_loose=(2048,) * 4, steps=3, max_chunk=4, logit_std=(0.5, 6.0), logit_run=1)
    print(f"chunks at full size: {wl.units} units of {wl.prefill} slots", flush=True)
    ls = Lockstep(lib, wl, seed=0, units=6, threads=16)
    for t, tq in enumerate((4, 3, 4)):
        ls.step(tq=tq)
        _invariants_all_units(ls, wl, ls.t - 1)
        print(f"  step {t} (tq={tq}): len={ls.report.lengths[-1]} out_err={ls.report.max_out_err:.3f}xtol", flush=True)
    rep = ls.report
    print(f"  ema_rel={rep.max_ema_rel:.2e} evictions={rep.evictions} flips={rep.evict_flips}/{rep.budget_flips}", flush=True)
    assert rep.ok(), (rep.evict_flips, rep.budget_flips)
    assert ls.kv.counters().device_errors == 0
    ls.close()


def test_full_size_many_row_chunks(lib):
    """Sixteen tokens per attention call at the roofline workload's shape (4 of its layers): 64
    query rows per kv-head on the many-rows kernel (four row blocks per K/V tile, four splits per
    unit exchanging 64 rows of partials, importance from the second pass over the keys), then an
    eviction of more than two thousand tokens per unit."""
    wl = workload(1).scaled(name="llama3_8b_b8_t4096_chunk16", n_layers=4, n_tight=(1024,) * 4,
                            n_loose=(2048,) * 4, steps=3, max_chunk=16, logit_std=(0.5, 6.0), logit_run=1)
    print(f"many-row chunks at full size: {wl.units} units of {wl.prefill} slots", flush=True)
    ls = Lockstep(lib, wl, seed=0, units=6, threads=16)
    for t, tq in enumerate((16, 11, 16)):
        ls.step(tq=tq)
        _invariants_all_units(ls, wl, ls.t - 1)
        print(f"  step {t} (tq={tq}): len={ls.report.lengths[-1]} out_err={ls.report.max_out_err:.3f}xtol", flush=True)
    rep = ls.report
    print(f"  ema_rel={rep.max_ema_rel:.2e} evictions={rep.evictions} flips={rep.evict_flips}/{rep.budget_flips}", flush=True)
    assert rep.ok(), (rep.evict_flips, rep.budget_flips)
    assert ls.kv.counters().device_errors == 0
    ls.close()


def test_full_size_replayed_steps(lib):
    """A recorded decode step replayed at the roofline workload's shape (4 of its layers, four
    splits per unit, the launch configuration the benchmark times): the first step runs outside
    the graph (4097 -> 2048 or 1024 slots per unit), the following ones are replays whose
    caches shrink and grow with the budget choices; outputs, kept sets and state of the
    followed units against the oracle, invariants on all units."""
    wl = workload(1).scaled(name="llama3_8b_b8_t4096_replay", n_layers=4, n_tight=(1024,) * 4, n_loose=(2048,) * 4,
                            steps=10, logit_std=(0.5, 6.0), logit_run=2)
    print(f"replayed steps at full size: {wl.units} units of {wl.prefill} slots", flush=True)
    ls = Lockstep(lib, wl, seed=2, units=6, threads=16)
    ls.kv.static_plan(True)
    ls.step()
    ls.record_step()
    for t in range(1, wl.steps):
        ls.step(check_state=(t % 3 == 0 or t == wl.steps - 1))
        _invariants_all_units(ls, wl, t)
        print(f"  replay {t}: len={ls.report.lengths[-1]} out_err={ls.report.max_out_err:.3f}xtol", flush=True)
    rep = ls.report
    assert ls.replays == wl.steps - 1 and rep.ok(), (rep.evict_flips, rep.budget_flips)
    assert ls.kv.counters().device_errors == 0 and rep.evictions > 0 and 0 < rep.tight_steps < rep.steps * wl.batch
    ls.close()


def test_full_size_grouped_heads_of_64_channels(lib):
    """Eight query heads of 64 channels per kv-head (the shape of the 20B mixture-of-experts model
    the paper evaluates) at the roofline workload's batch and length, 4 layers: the matrix-core
    body with the head padded to its 128-channel tiles."""
    wl = workload(1).scaled(name="b8_t4096_hq64_hkv8_d64", n_layers=4, n_q_heads=64, n_kv_heads=8, head_dim=64,
                            n_tight=(1024,) * 4, n_loose=(2048,) * 4, steps=3, logit_std=(0.5, 6.0), logit_run=1)
    print(f"64-channel grouped heads at full size: {wl.units} units of {wl.prefill} slots", flush=True)
    ls = Lockstep(lib, wl, seed=1, units=6, threads=16)
    for t in range(wl.steps):
        ls.step()
        _invariants_all_units(ls, wl, t)
        print(f"  step {t}: len={ls.report.lengths[-1]} out_err={ls.report.max_out_err:.3f}xtol", flush=True)
    rep = ls.report
    assert rep.ok(), (rep.evict_flips, rep.budget_flips)
    assert ls.kv.counters().device_errors == 0 and rep.evictions > 0
    ls.close()


def test_full_size_observation_window(lib):
    """Importance from the prompt's own attention at the roofline workload's shape (4 of its
    layers): the last 32 prompt tokens observe the prompt in windows of 4 (the window ends inside
    the FP16 tail and starts in INT8 slots when the tail is shorter than 32), then decode steps
    evict by what the observation left."""
    wl = workload(1).scaled(name="llama3_8b_b8_t4096_observe", n_layers=4, n_tight=(1024,) * 4,
                            n_loose=(2048,) * 4, steps=3, max_chunk=4, fp16_window=24,
                            logit_std=(0.5, 6.0), logit_run=1)
    print(f"observation window at full size: {wl.units} units of {wl.prefill} slots", flush=True)
    ls = Lockstep(lib, wl, seed=2, units=6, threads=16)
    for k, first in enumerate(range(wl.prefill - 32, wl.prefill, 4)):
        ls.observe(first, 4, want_out=k % 2 == 0)
    print(f"  observed: out_err={ls.report.max_out_err:.3f}xtol ema_rel={ls.report.max_ema_rel:.2e}", flush=True)
    # the observation gave every followed unit a non-trivial importance profile
    for u in ls.run.units.values():
        assert np.count_nonzero(u.ema) > 0.99 * u.n
    for t in range(3):
        ls.step()
        _invariants_all_units(ls, wl, t)
        print(f"  step {t}: len={ls.report.lengths[-1]} out_err={ls.report.max_out_err:.3f}xtol", flush=True)
    rep = ls.report
    print(f"  ema_rel={rep.max_ema_rel:.2e} evictions={rep.evictions} flips={rep.evict_flips}/{rep.budget_flips}", flush=True)
    assert rep.ok(), (rep.evict_flips, rep.budget_flips)
    assert ls.kv.counters().device_errors == 0 and rep.evictions > 0
    ls.close()


def test_chunks_on_long_units_take_the_two_launch_form(lib):
    """Four tokens per call on 64 units of 9000 slots: sixteen rows of scores for a slice of such
    a unit do not fit on chip next to the tile buffers at any resident split count, so the call
    goes through scratch in two launches."""
    wl = workload(1).scaled(name="llama3_8b_b8_t9000_chunk4", n_layers=2, prefill=9000, steps=2,
                            n_tight=(4096,) * 2, n_loose=(8192,) * 2, max_chunk=4)
    print(f"long units, chunks: {wl.units} units of {wl.prefill} slots", flush=True)
    ls = Lockstep(lib, wl, seed=4, units=3, threads=16)
    for t, tq in enumerate((4, 2)):
        ls.step(tq=tq)
        _invariants_all_units(ls, wl, ls.t - 1)
        print(f"  step {t} (tq={tq}): len={ls.report.lengths[-1]} out_err={ls.report.max_out_err:.3f}xtol", flush=True)
    rep = ls.report
    assert rep.ok(), (rep.evict_flips, rep.budget_flips)
    st = ls.kv.counters()
    assert st.device_errors == 0 and rep.evictions > 0
    ls.close()


@pytest.mark.parametrize("evict_page", [0, 16])
def test_page_fragmentation_of_token_level_eviction(lib, evict_page):
    """With evict_page = 16 the same run under coarsened eviction: no page of 16 is partially dead
    (the newest one aside).  With 0: what token-level eviction would cost a paged layout ("Compatibility with serving systems",
    "Limitations": partially dead blocks): after a steady-state run at workload 4's shape (4 of
    its layers), group the ORIGINAL positions into pages of 16 and 32 tokens and count, per unit,
    the pages that still hold a live token against the pages the live tokens would fill if packed.
    No kernel is involved beyond the ordinary decode path; the numbers are printed for the
    design notes and only sanity-checked here."""
    import torch
    wl = workload(4).scaled(n_layers=4, n_tight=workload(4).n_tight[:4], n_loose=workload(4).n_loose[:4],
                            steps=120, logit_run=3, evict_page=evict_page)
    kv = lib.from_workload(wl)
    for l in range(wl.n_layers):
        K, V = gen.prefill_layer(wl, 0, l, threads=16)
        kv.load_prefill(l, torch.from_numpy(K).cuda(), torch.from_numpy(V).cuda())
    out = torch.empty((wl.batch, wl.n_q_heads, wl.head_dim), dtype=torch.float16, device="cuda")
    for t in range(wl.steps):
        for l in range(wl.n_layers):
            q, k, v = gen.step_inputs(wl, 0, l, t)
            kv.attend(l, torch.from_numpy(q).cuda(), torch.from_numpy(k).cuda(), torch.from_numpy(v).cuda(), out)
        kv.step(torch.from_numpy(gen.step_logits(wl, 0, t)).cuda())
        kv.evict_compact()
    rng = np.random.default_rng(0)
    for page in (16, 32):
        live_pages = packed_pages = partial = 0
        for _ in range(48):
            l, b, g = int(rng.integers(wl.n_layers)), int(rng.integers(wl.batch)), int(rng.integers(wl.n_kv_heads))
            pos = kv.export(l, b, g)["pos"]
            ids, counts = np.unique(pos // page, return_counts=True)
            live_pages += ids.size
            packed_pages += -(-pos.size // page)
            partial += int((counts < page).sum())
            if evict_page == page:                      # only the newest page may be short
                assert not (counts[:-1] < page).any()
        print(f"evict_page {evict_page}, page size {page}: live pages {live_pages}, packed {packed_pages} "
              f"(overhead {live_pages / packed_pages:.2f}x), partially dead {partial / live_pages:.0%}", flush=True)
        assert live_pages >= packed_pages
    assert kv.counters().device_errors == 0 and kv.counters().evicted > 0
    kv.close()


def test_needle_retention_full_size(lib):
    """Retrieval stress at full cache length (one layer): every planted needle survives the
    32769 -> 4096 eviction after the first probe step, on every unit of the layer."""
    wl = workload(3).scaled(n_layers=1, n_tight=(512,), n_loose=(4096,))
    ls = Lockstep(lib, wl, seed=0, units=1, threads=16)
    ls.step()
    slots = gen.needle_slots(wl, 0)
    kept = 0
    for g in range(wl.n_kv_heads):
        ex = ls.kv.export(0, 0, g)
        assert ex["n"] == 4096
        kept += int(np.isin(slots, ex["pos"]).sum())
    print(f"needles retained: {kept}/{len(slots) * wl.n_kv_heads}", flush=True)
    assert kept == len(slots) * wl.n_kv_heads
    ls.close()


def test_many_long_units_take_the_two_launch_form(lib):
    """A batch of long contexts: 320 units of 11 000 slots in one layer.  No single-kernel plan
    exists (a unit's scores do not fit on chip in one split, and two splits of 320 units cannot
    all be resident), so attention runs as two launches through the scratch buffer; results
    follow the oracle like everywhere else."""
    wl = workload(1).scaled(name="llama3_8b_b40_t11000", n_layers=1, batch=40, prefill=11000, steps=2,
                            n_tight=(4096,), n_loose=(8192,))
    print(f"long batch: {wl.units} units of {wl.prefill} slots", flush=True)
    ls = Lockstep(lib, wl, seed=3, units=3, threads=16)
    splits = ls.kv.attend_splits(0)
    print(f"  attend splits: {splits}", flush=True)
    assert splits >= 1000
    for t in range(wl.steps):
        ls.step()
        _invariants_all_units(ls, wl, t)
        print(f"  step {t}: len={ls.report.lengths[-1]} out_err={ls.report.max_out_err:.3f}xtol", flush=True)
    rep = ls.report
    assert rep.ok(), (rep.evict_flips, rep.budget_flips)
    assert ls.kv.counters().device_errors == 0
    ls.close()
