"""The seeded input generators: deterministic, keyed per unit/step, right shapes and recipe."""
import numpy as np

from synth import generate as gen
from synth.workloads import linear_budgets, small, workload


def test_workload_shapes_follow_the_configs():
    w = [workload(i) for i in range(5)]
    assert (w[0].n_layers, w[0].n_q_heads, w[0].n_kv_heads, w[0].head_dim, w[0].vocab) == (12, 12, 12, 64, 50257)
    assert w[0].fp16_window < 0 and w[0].units == 144 and w[0].group == 1
    assert (w[1].batch, w[1].prefill, w[1].units, w[1].group) == (8, 4096, 2048, 4)
    assert (w[2].n_layers, w[2].group, w[2].vocab, w[2].fp16_window, w[2].protected) == (64, 5, 152064, 64, 128)
    assert (w[3].prefill, w[3].n_needles, w[3].alpha) == (32768, 16, 0.70)
    assert w[4].n_tight[0] == 1024 and w[4].n_tight[-1] == 128 and sum(w[4].n_tight) == 18432
    assert all(b == 2 * a for a, b in zip(w[4].n_tight, w[4].n_loose))
    assert all(x >= y for x, y in zip(w[4].n_tight, w[4].n_tight[1:]))
    for x in w:
        assert x.capacity % 64 == 0 and x.capacity > max(x.prefill, max(x.n_loose))
        assert all(a <= b for a, b in zip(x.n_tight, x.n_loose))
    assert linear_budgets(10, 10, 1) == (10,)


def test_generators_are_deterministic_and_keyed():
    wl = small(1)
    k1, v1 = gen.prefill_unit(wl, 0, 1, 1, 0)
    k2, v2 = gen.prefill_unit(wl, 0, 1, 1, 0)
    assert k1.dtype == np.float16 and k1.shape == (wl.prefill, wl.head_dim)
    assert np.array_equal(k1, k2) and np.array_equal(v1, v2)
    assert not np.array_equal(k1, gen.prefill_unit(wl, 0, 1, 0, 0)[0])
    assert not np.array_equal(k1, gen.prefill_unit(wl, 1, 1, 1, 0)[0])
    K, V = gen.prefill_layer(wl, 0, 1, threads=4)
    assert K.shape == (wl.batch, wl.n_kv_heads, wl.prefill, wl.head_dim)
    assert np.array_equal(K[1, 0], k1) and np.array_equal(V[1, 0], v1)
    q, k, v = gen.step_inputs(wl, 0, 0, 3)
    assert q.shape == (wl.batch, wl.n_q_heads, wl.head_dim) and k.shape == (wl.batch, wl.n_kv_heads, wl.head_dim)
    assert np.array_equal(q, gen.step_inputs(wl, 0, 0, 3)[0])
    lg = gen.step_logits(wl, 0, 0)
    assert lg.dtype == np.float32 and lg.shape == (wl.batch, wl.vocab)


def test_recipe_statistics():
    wl = workload(0)
    u = gen.unit_direction(wl, 0, 2, 5)
    assert abs(np.sum(u * u) - 1) < 1e-12
    k, v = gen.prefill_unit(wl.scaled(prefill=20000), 0, 2, 0, 5)
    proj = k.astype(np.float64) @ u
    frac = np.mean(proj > 1.5)                       # heavy hitters sit near +3 along u
    assert 0.05 < frac < 0.11                        # 2% planted + the N(0,1) tail above 1.5 (6.7%)
    assert abs(np.mean(proj > 2.5) - (0.02 * 0.69 + 0.0062)) < 0.006
    assert abs(v.astype(np.float64).std() - 1) < 0.01
    q, _, _ = gen.step_inputs(wl, 0, 2, 0)
    assert abs(float(q[0, 5].astype(np.float64) @ u) - np.sqrt(wl.head_dim)) < 4.0
    assert gen.logit_std(wl, 0) == 0.5 and gen.logit_std(wl, 31) == 0.5 and gen.logit_std(wl, 32) == 6.0
    assert abs(gen.step_logits(wl, 0, 40).std() - 6.0) < 0.1


def test_needle_workload():
    wl = small(3)
    slots = gen.needle_slots(wl, 0)
    assert len(slots) == wl.n_needles and len(set(slots)) == wl.n_needles and slots.max() < wl.prefill
    k, _ = gen.prefill_unit(wl, 0, 0, 0, 1)
    u = gen.unit_direction(wl, 0, 0, 1)
    assert np.allclose(k[slots].astype(np.float64), (6.0 * u)[None].repeat(len(slots), 0), atol=5e-3)
    q_probe, _, _ = gen.step_inputs(wl, 0, 0, 0)
    q_off, _, _ = gen.step_inputs(wl, 0, 0, 1)
    s = q_probe[0, 5].astype(np.float64) @ k[slots[0]].astype(np.float64) / np.sqrt(wl.head_dim)
    assert abs(s - 6.0) < 0.05                        # probe query scores the needle at the gain
    assert abs(float(q_off[0, 5].astype(np.float64) @ u)) < 5.0
    assert gen.logit_std(wl, 0) == 0.5 and gen.logit_std(wl, 1) == 6.0
