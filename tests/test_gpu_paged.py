"""The paged layout (block table over pages of `evict_page` INT8 slots; "Compatibility with serving
systems", "Limitations") against the oracle and against the contiguous layout.

The oracle knows nothing of layouts: it keeps a position-sorted cache and evicts whole pages of
original positions (``select_page_evictions``).  conf_kv_export must return that same view from the
paged storage, bit for bit, at every step; and the same run under the contiguous layout must give
bit-identical outputs and state (the attention kernel adds in the same order, only the row
addresses differ), while the paged run moves no payload row.
"""
import os
import sys

import numpy as np
import pytest

from synth import generate as gen
from synth.workloads import small, workload

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
from harness import Lockstep  # noqa: E402
from longrun import record_and_replay  # noqa: E402

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)


@pytest.mark.parametrize("G,W,P,page,batch", [(4, 16, 16, 16, 2), (5, 24, 48, 8, 1), (2, 0, 8, 32, 3), (8, 32, 40, 16, 1)])
def test_lockstep_paged_layout(lib, G, W, P, page, batch):
    """Decode loops in the paged layout: whole state bit-identical to the oracle's at every step
    (kept positions, tags, payload bits, codes, scales; EMA within tolerance), through many page
    evictions, page allocations by demotion and budget switches."""
    wl = small(1).scaled(n_layers=2, batch=batch, n_q_heads=2 * G, n_kv_heads=2, head_dim=128, vocab=2003,
                         prefill=300, steps=60, n_tight=(150, 120), n_loose=(260, 230), protected=P, fp16_window=W,
                         alpha=0.5, logit_std=(0.5, 6.0), logit_run=5, evict_page=page, layout="paged")
    say(f"lockstep paged G={G} W={W} P={P} page={page} batch={batch} capacity={wl.capacity}")
    ls = Lockstep(lib, wl, seed=21)
    for t in range(wl.steps):
        ls.step()
        for key, u in ls.run.units.items():               # no page is partially dead but the newest
            live = np.bincount((u.pos // page).astype(np.int64))
            newest = int(u.pos[-1]) // page
            assert not [k for k, c in enumerate(live) if c not in (0, page) and k != newest], (t, key)
    rep, st = ls.report, ls.kv.counters()
    say(f"  out_err={rep.max_out_err:.3f}xtol ema_rel={rep.max_ema_rel:.2e} evictions={rep.evictions} "
        f"tight={rep.tight_steps} demoted={st.demoted} table bytes={st.compact_bytes}")
    assert rep.ok(), rep.evict_flips
    assert rep.evictions > 0 and rep.tight_steps > 0 and st.demoted > 0 and st.device_errors == 0
    # the only "moves" are block-table entries: 8 bytes per live page and eviction event, never a row
    assert st.compact_bytes <= 8 * (wl.capacity // page) * wl.units * wl.steps
    ls.close()


def test_paged_equals_contiguous_bit_for_bit(lib):
    """The same seeded run under both layouts: attention outputs, confidence, and every exported
    plane agree bit for bit after every step; the contiguous run moves rows, the paged one none."""
    import torch
    base = small(4).scaled(n_layers=2, batch=2, n_q_heads=8, n_kv_heads=2, vocab=3001, prefill=500, steps=50,
                           n_tight=(160, 96), n_loose=(320, 192), protected=32, fp16_window=16, evict_page=16,
                           logit_run=4)
    kvs = {name: lib.from_workload(base.scaled(layout=name)) for name in ("contiguous", "paged")}
    for l in range(base.n_layers):
        K, V = gen.prefill_layer(base, 5, l)
        for kv in kvs.values():
            kv.load_prefill(l, torch.from_numpy(K).cuda(), torch.from_numpy(V).cuda())
    outs = {name: torch.empty((base.batch, base.n_q_heads, base.head_dim), dtype=torch.float16, device="cuda") for name in kvs}
    conf = {name: torch.empty(base.batch, dtype=torch.float32, device="cuda") for name in kvs}
    for t in range(base.steps):
        for l in range(base.n_layers):
            q, k, v = (torch.from_numpy(x).cuda() for x in gen.step_inputs(base, 5, l, t))
            for name, kv in kvs.items():
                kv.attend(l, q, k, v, outs[name])
            assert torch.equal(outs["contiguous"], outs["paged"]), (t, l)
        lg = torch.from_numpy(gen.step_logits(base, 5, t)).cuda()
        for name, kv in kvs.items():
            kv.step(lg, conf[name])
            kv.evict_compact()
        assert torch.equal(conf["contiguous"], conf["paged"])
        for l in range(base.n_layers):
            for b in range(base.batch):
                for g in range(base.n_kv_heads):
                    a, p = kvs["contiguous"].export(l, b, g), kvs["paged"].export(l, b, g)
                    assert a["n"] == p["n"], (t, l, b, g)
                    for name in ("pos", "ema", "is16", "k16", "v16", "k8", "v8", "ks", "vs"):
                        assert np.array_equal(a[name].view(np.uint8), p[name].view(np.uint8)), (t, l, b, g, name)
    sc, sp = kvs["contiguous"].counters(), kvs["paged"].counters()
    say(f"evicted {sc.evicted} = {sp.evicted}; bytes moved: contiguous {sc.compact_bytes}, paged (table entries) {sp.compact_bytes}")
    assert sc.evicted == sp.evicted > 0 and sc.demoted == sp.demoted > 0
    # what the paged run counts are block-table entries (8 bytes per live page and eviction event)
    assert 0 < sp.compact_bytes <= 8 * (base.capacity // 16) * base.units * base.steps
    for kv in kvs.values():
        kv.close()


def test_paged_layout_rules(lib):
    """What the layout needs is checked when the handle is made; conf_kv_import is refused."""
    ok = dict(n_layers=1, batch=1, n_q_heads=8, n_kv_heads=2, head_dim=128, vocab=1000, capacity=512, fp16_window=16,
              protected_window=16, n_tight=[64], n_loose=[128], evict_page=16, layout="paged")
    lib.ConfKV(**ok).close()
    for bad in (dict(evict_page=0), dict(evict_page=24), dict(fp16_window=32), dict(fp16_window=-1),
                dict(scale_mode="channel"), dict(rank_scope="layer"), dict(max_chunk=2), dict(n_q_heads=2),
                dict(capacity=144)):
        with pytest.raises(lib.ConfKVError) as e:
            lib.ConfKV(**dict(ok, **bad))
        assert e.value.status == lib.binding.ERR_BAD_SHAPE, bad
    kv = lib.ConfKV(**ok)
    view = dict(n=0, pos=np.zeros(0, np.int32), ema=np.zeros(0, np.float32), is16=np.zeros(0, np.uint8))
    with pytest.raises(lib.ConfKVError) as e:
        kv.import_unit(0, 0, 0, view)
    assert e.value.status == lib.binding.ERR_BAD_STATE
    kv.close()


def test_paged_layout_at_full_size(lib):
    """Workload 4's shape (batch 32, 8192 units, pyramidal budgets) in the paged layout with pages
    of 16, 256 decode steps: recorded on the GPU, followed units replayed by the oracle."""
    wl = workload(4).scaled(name="llama3_8b_b32_pyramid_paged16", steps=256, evict_page=16, layout="paged", logit_run=8)
    s = record_and_replay(lib, wl, seed=0, follow=16, steps=wl.steps, full_every=32, log=say)
    s.pop("needles")
    say("  " + str(s))
    assert s["evictions_followed"] > 0 and s["tight_sequence_steps"] > 0
