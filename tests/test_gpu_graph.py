"""A decode step recorded once into a HIP graph and replayed, against the oracle in lock-step.

What changes from step to step (lengths, ring heads, budgets, the positions appended tokens get,
the tags the in-kernel waits compare) lives on the device, so the recorded launches hold nothing
of one particular step: every replay must give what the eager calls give, i.e. match the oracle
at every step -- attention output, confidence, kept positions and the whole cache state.  Between
replays the test does ordinary eager work (copies into the graph's input tensors, synchronising
exports), as a serving loop would.
"""
import os
import sys

import numpy as np
import pytest

from synth.workloads import small

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
from harness import Lockstep  # noqa: E402

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)


CASES = {
    # cache still growing when the step is recorded (lengths 40 -> budget), FP16 only, D = 64
    "growing_fp16": dict(idx=0, kw=dict(prefill=40, steps=96, n_tight=(60, 50), n_loose=(100, 90), protected=12,
                                        logit_std=(0.5, 6.0), logit_run=6), eager=2),
    # mixed INT8 / FP16 cache over several splits, prompt longer than the loose budget at recording time
    "mixed_long_prompt": dict(idx=1, kw=dict(steps=80, logit_std=(0.5, 6.0), logit_run=7), eager=1),
    # recorded in the steady state; groups of 12 query heads (16-row kernel), per-layer budgets
    "pyramid_wide_groups": dict(idx=4, kw=dict(n_q_heads=24, steps=72, logit_std=(0.5, 6.0), logit_run=5), eager=6),
    # paged layout: the block table edits are replayed too
    "paged": dict(idx=1, kw=dict(n_layers=2, batch=2, n_q_heads=8, n_kv_heads=2, vocab=2003, prefill=300, steps=80,
                                 n_tight=(150, 120), n_loose=(260, 230), protected=16, fp16_window=16, alpha=0.5,
                                 logit_std=(0.5, 6.0), logit_run=5, evict_page=16, layout="paged"), eager=3),
}


@pytest.mark.parametrize("case", sorted(CASES))
def test_replayed_steps_match_the_oracle(lib, case):
    c = CASES[case]
    wl = small(c["idx"]).scaled(**c["kw"])
    say(f"graph replay {case}: {wl.n_layers} layers, batch {wl.batch}, prefill {wl.prefill}, {wl.steps} steps")
    ls = Lockstep(lib, wl, seed=41)
    ls.kv.static_plan(True)
    for _ in range(c["eager"]):                   # outside the graph: first launches set kernel attributes
        ls.step()
    ls.record_step()
    for t in range(c["eager"], wl.steps):
        ls.step(check_state=(t % 8 == 0 or t == wl.steps - 1))
    rep = ls.report
    say(f"  {ls.replays} replays: evictions {rep.evictions}, tight steps {rep.tight_steps}, lengths "
        f"{min(rep.lengths)}..{max(rep.lengths)}, max out err {rep.max_out_err:.3g} x tol")
    assert ls.replays >= 64
    assert rep.ok() and rep.evictions > 0 and 0 < rep.tight_steps < rep.steps * wl.batch
    assert ls.kv.counters().device_errors == 0
    ls.close()


@pytest.mark.parametrize("G,tq,mc", [(4, 4, 4), (4, 16, 16)])
def test_replayed_multi_token_steps(lib, G, tq, mc):
    """Steps of tq tokens per call (the 16-row kernel, and the many-rows kernel at 64 rows per
    kv-head) recorded once and replayed: positions move on by tq per replay, the telescoped
    importance update and the eviction behind it match the oracle at every step."""
    wl = small(1).scaled(n_layers=2, batch=2, n_q_heads=2 * G, n_kv_heads=2, head_dim=128, vocab=3001, prefill=300,
                         steps=40, n_tight=(180, 150), n_loose=(330, 300), protected=40, fp16_window=24, alpha=0.5,
                         logit_std=(0.5, 6.0), logit_run=3, max_chunk=mc)
    say(f"graph replay of {tq}-token steps: G={G}")
    ls = Lockstep(lib, wl, seed=47)
    ls.kv.static_plan(True)
    ls.step(tq=tq)
    ls.record_step(tq)
    for t in range(1, wl.steps):
        ls.step(check_state=(t % 8 == 0 or t == wl.steps - 1), tq=tq)
    rep = ls.report
    say(f"  {ls.replays} replays: evictions {rep.evictions}, lengths {min(rep.lengths)}..{max(rep.lengths)}")
    assert ls.replays == wl.steps - 1 and rep.ok() and rep.evictions > 0
    assert ls.kv.counters().device_errors == 0
    ls.close()


def test_static_plan_changes_no_result(lib):
    """The same eager run of a growing cache with and without conf_kv_static_plan (more splits
    from the first step on): same kept sets, outputs and EMA equal up to the summation order."""
    wl = small(1).scaled(prefill=40, steps=12, n_tight=(800, 800), n_loose=(1600, 1600), logit_std=(0.5, 6.0),
                         logit_run=3)
    runs = []
    for on in (False, True):
        ls = Lockstep(lib, wl, seed=5, units=2)
        ls.kv.static_plan(on)
        outs = []
        for _ in range(wl.steps):
            ls.step(check_state=False)
            outs.append(ls.out.cpu().numpy().copy())
        state = {key: ls.kv.export(*key) for key in ls.run.units}
        runs.append((outs, state, ls.kv.attend_splits(0)))
        ls.close()
    (o0, s0, p0), (o1, s1, p1) = runs
    say(f"static plan: splits {p0} -> {p1}")
    assert p1 > p0
    for key in s0:
        assert np.array_equal(s0[key]["pos"], s1[key]["pos"])
        np.testing.assert_allclose(s0[key]["ema"], s1[key]["ema"], rtol=5e-6, atol=1e-8)
    for a, b in zip(o0, o1):
        np.testing.assert_allclose(a.astype(np.float32), b.astype(np.float32), rtol=2e-3, atol=2e-3)


def test_tag_restart_under_replay(lib, monkeypatch):
    """The device-side tag bases start just below their restart threshold (test hook): within
    three replayed steps the commit asks for the clearing, the next commit's compaction kernel
    clears the exchange words and both bases start over -- with the oracle matched at every
    step on the way, so no launch met a stale or missing word."""
    T = 0xFF000000
    monkeypatch.setenv("CONF_KV_TEST_TAG_BASE", str(T - 3))
    wl = small(1).scaled(steps=10, logit_std=(0.5, 6.0), logit_run=3)
    assert wl.n_layers == 2
    ls = Lockstep(lib, wl, seed=43)
    monkeypatch.delenv("CONF_KV_TEST_TAG_BASE")
    ls.kv.static_plan(True)
    assert ls.kv.tag_state() == (T - 3, T - 3, 0)
    seen = []
    ls.step()
    seen.append(ls.kv.tag_state())
    ls.record_step()
    for t in range(1, wl.steps):
        ls.step()
        seen.append(ls.kv.tag_state())
    say(f"tag states: {seen[:5]}")
    assert seen[:5] == [(T - 1, T - 2, 0), (T + 1, T - 1, 1), (0, 0, 0), (2, 1, 0), (4, 2, 0)]
    assert ls.report.ok() and ls.kv.counters().device_errors == 0
    ls.close()
