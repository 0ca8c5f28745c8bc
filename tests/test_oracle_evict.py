"""Pins for the oracle's ranker, eviction, compaction, quantiser and whole step.

Ranking is a plain top-k of a stated score ("Budget and ranker"): pinned by a
pure-Python full sort, by exhaustive subset enumeration on tiny caches, by its
reductions to textbook policies (alpha = 0: sliding window; alpha = 1: heavy
hitters plus a recent window) and by the invariants the method states
(protected window always kept, budget never exceeded, no-op below the budget).
"""
import itertools
import math

import numpy as np
import pytest

from oracle import confkv_oracle as O


def _unit(rng, n, D=8, W=-1, ema=None, pos=None):
    u = O.load_prefill(rng.standard_normal((n, D)).astype(np.float16),
                       rng.standard_normal((n, D)).astype(np.float16), W,
                       ema0=ema)
    if pos is not None:
        u.pos = np.asarray(pos, dtype=np.int64)
    return u


def _py_scores(ema, pos, alpha):
    a_lo, a_hi, p_lo, p_hi = min(ema), max(ema), min(pos), max(pos)
    out = []
    for a, p in zip(ema, pos):
        ah = 0.0 if a_hi == a_lo else (a - a_lo) / (a_hi - a_lo)
        rh = 0.0 if p_hi == p_lo else (p - p_lo) / (p_hi - p_lo)
        out.append(alpha * ah + (1 - alpha) * rh)
    return out


def test_full_sort_brute_force():
    rng = np.random.default_rng(0)
    for trial in range(20):
        n = int(rng.integers(12, 60))
        P = int(rng.integers(1, 10))
        N = int(rng.integers(P, n))
        ema = rng.random(n).astype(np.float32)
        pos = np.cumsum(rng.integers(1, 4, n))
        u = _unit(rng, n, ema=ema, pos=pos)
        keep, evict = O.select_evictions(u, N, P, 0.65)
        nc = n - P
        s = _py_scores([float(x) for x in ema[:nc]], [int(x) for x in pos[:nc]], 0.65)
        order = sorted(range(nc), key=lambda i: (s[i], pos[i]))
        want_evict = sorted(order[:n - N])
        assert list(evict) == want_evict
        assert list(keep) == [i for i in range(n) if i not in set(want_evict)]


@pytest.mark.parametrize("seed", range(6))
def test_exhaustive_subsets_tiny(seed):
    # among all ways to drop e candidates, the chosen one maximises the sorted kept scores
    rng = np.random.default_rng(100 + seed)
    n, P, N = 9, 2, 5
    ema = rng.random(n).astype(np.float32)
    u = _unit(rng, n, ema=ema)
    keep, evict = O.select_evictions(u, N, P, 0.65)
    nc, e = n - P, n - N
    s = O.rank_scores(ema[:nc], u.pos[:nc], 0.65)
    best = max(itertools.combinations(range(nc), e),
               key=lambda drop: sorted(s[i] for i in range(nc) if i not in drop))
    assert sorted(best) == list(evict)
    assert min(s[i] for i in keep if i < nc) >= max(s[i] for i in evict)


def test_alpha_zero_is_sliding_window():
    rng = np.random.default_rng(1)
    n, N, P = 100, 40, 8
    u = _unit(rng, n, ema=rng.random(n).astype(np.float32))
    keep, evict = O.select_evictions(u, N, P, 0.0)
    assert list(keep) == list(range(n - N, n)) and list(evict) == list(range(n - N))


def test_alpha_one_keeps_heavy_hitters_plus_recent_window():
    rng = np.random.default_rng(2)
    n, N, P = 80, 30, 10
    ema = rng.random(n).astype(np.float32)
    u = _unit(rng, n, ema=ema)
    keep, _ = O.select_evictions(u, N, P, 1.0)
    top = np.argsort(-ema[:n - P].astype(np.float64), kind="stable")[:N - P]
    assert set(keep) == set(top) | set(range(n - P, n))


def test_invariants_and_noop():
    rng = np.random.default_rng(3)
    for trial in range(30):
        n = int(rng.integers(5, 70))
        P = int(rng.integers(0, 20))
        N = int(rng.integers(1, 80))
        u = _unit(rng, n, ema=rng.random(n).astype(np.float32))
        before = u.copy()
        gone = O.evict_compact_unit(u, N, P, 0.65, -1)
        if n <= N:                                             # no-op below the budget
            assert u.n == n and gone.size == 0
            continue
        p_eff = min(P, n)
        assert u.n == max(N, p_eff)                            # budget met unless the window is larger
        assert np.array_equal(u.pos[-p_eff:] if p_eff else u.pos[:0],
                              before.pos[n - p_eff:])          # protected window survives
        assert np.all(np.diff(u.pos) > 0)                      # order kept
        # compaction is a pure gather of the surviving rows
        idx = np.searchsorted(before.pos, u.pos)
        assert np.array_equal(before.k16[idx], u.k16) and np.array_equal(before.ema[idx], u.ema)
        assert set(gone) == set(before.pos) - set(u.pos)


def test_window_larger_than_budget_wins():
    rng = np.random.default_rng(4)
    u = _unit(rng, 20, ema=rng.random(20).astype(np.float32))
    O.evict_compact_unit(u, 4, 10, 0.65, -1)
    assert u.n == 10 and list(u.pos) == list(range(10, 20))


def test_ties_evict_oldest_first_and_degenerate_minmax():
    rng = np.random.default_rng(5)
    n = 12
    u = _unit(rng, n, ema=np.full(n, 0.25, dtype=np.float32))
    # equal mass: alpha = 1 gives all-zero scores, so the oldest go first
    _, evict = O.select_evictions(u, 8, 2, 1.0)
    assert list(evict) == [0, 1, 2, 3]
    # a single candidate: both normalisations are 0/0 -> defined as 0
    assert O.rank_scores(np.array([0.3], np.float32), np.array([7]), 0.65)[0] == 0.0


def test_quantiser_properties():
    rng = np.random.default_rng(6)
    for mag in (1e-3, 0.05, 1.0, 30.0, 2000.0):
        x = (rng.standard_normal((200, 128)) * mag).astype(np.float16)
        for row in x:
            codes, scale = O.quantize_vector(row)
            assert codes.dtype == np.int8 and codes.min() >= -127 and codes.max() <= 127
            amax = np.max(np.abs(row)).astype(np.float64)
            s = float(scale)
            normal = s >= 2.0 ** -14                                    # fp16 scale not sub-normal
            assert abs(s - amax / 127) <= max(amax / 127 * 2.0 ** -11, 2.0 ** -25) * (1 + 1e-6)
            err = np.abs(row.astype(np.float64) - codes.astype(np.float64) * s)
            unclamped = np.abs(row.astype(np.float64) / s) <= 127.5
            assert np.all(err[unclamped] <= s / 2 * (1 + 1e-12))
            if normal:
                assert abs(int(codes[np.argmax(np.abs(row))])) == 127   # absmax maps to +-127


def test_quantiser_rounds_half_to_even_and_handles_zero():
    codes, scale = O.quantize_vector(np.zeros(16, dtype=np.float16))
    assert scale == 0 and not codes.any()
    # amax = 127 -> scale exactly 1: values k + 0.5 sit exactly on a tie
    x = np.array([127, 0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 3.25], dtype=np.float16)
    codes, scale = O.quantize_vector(x)
    assert float(scale) == 1.0 and list(codes) == [127, 0, 2, 2, 0, -2, -2, 3]
    # a vector too small for an fp16 scale drops to zero codes
    codes, scale = O.quantize_vector(np.full(8, 6e-8, dtype=np.float16))
    assert scale == 0 and not codes.any()


def test_fp32_evaluation_of_quantiser_matches_float64():
    # the kernel's arithmetic (fp32 IEEE divide + rint) takes the same decisions
    rng = np.random.default_rng(7)
    x = (rng.standard_normal((4000, 128)) * rng.choice([0.01, 1, 50], (4000, 1))).astype(np.float16)
    amax = np.max(np.abs(x), axis=1)
    scale = (amax.astype(np.float32) / np.float32(127)).astype(np.float16)
    c32 = np.clip(np.rint(x.astype(np.float32) / scale.astype(np.float32)[:, None]), -127, 127)
    for i in range(0, 4000, 37):
        codes, s = O.quantize_vector(x[i])
        assert s == scale[i] and np.array_equal(codes, c32[i].astype(np.int8))


def test_demotion_order_and_window():
    rng = np.random.default_rng(8)
    D = 16
    u = _unit(rng, 30, D=D, W=6)
    assert u.n16 == 6 and list(np.flatnonzero(u.is16)) == list(range(24, 30))
    snap = u.copy()
    O.append_token(u, rng.standard_normal(D).astype(np.float16), rng.standard_normal(D).astype(np.float16), 30)
    k24 = u.k16[24].copy()
    assert O.demote(u, 6) == 1
    assert not u.is16[24] and u.is16[25:].all() and u.n16 == 6
    codes, scale = O.quantize_vector(k24)
    assert np.array_equal(u.k8[24], codes) and u.ks[24] == scale
    assert np.array_equal(u.k8[:24], snap.k8[:24])               # earlier INT8 tokens untouched
    # FP16-only cache never demotes
    u2 = _unit(rng, 30, D=D, W=-1)
    assert u2.n16 == 30 and O.demote(u2, -1) == 0


def test_whole_step_sawtooth_and_postconditions():
    # loose steps grow the cache by one token; the first tight step drops it to N_tight
    rng = np.random.default_rng(9)
    D, G, T0, P, W = 16, 2, 40, 8, 12
    pol = O.Policy(1, [24], [64], P, W, sm_scale=1 / math.sqrt(D))
    u = _unit(rng, T0, D=D, W=W)
    run = O.OracleRun(pol, {(0, 0, 0): u}, T0)
    V = 501
    lens = []
    for t in range(30):
        q = rng.standard_normal((1, G, D)).astype(np.float16)
        kn = rng.standard_normal((1, 1, D)).astype(np.float16)
        vn = rng.standard_normal((1, 1, D)).astype(np.float16)
        run.attend(0, q, kn, vn, G)
        logits = np.zeros((1, V), dtype=np.float32)
        if t == 20:
            logits[0, 3] = 40.0                                 # a confident step
        c, tight = run.step(logits)
        assert tight[0] == (t == 20)
        run.evict_compact(tight)
        lens.append(u.n)
        assert u.n <= (24 if tight[0] else 64) and u.n16 <= W
        assert np.all(np.diff(u.pos) > 0) and u.pos[-1] == T0 + t
        assert not u.is16[:u.n - u.n16].any() and u.is16[u.n - u.n16:].all()
        assert list(u.pos[-P:]) == list(range(T0 + t - P + 1, T0 + t + 1))
    assert lens[:20] == list(range(41, 61)) and lens[20] == 24 and lens[21:] == list(range(25, 34))
