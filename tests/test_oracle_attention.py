"""Pins for the oracle's attention, attention-mass and EMA arithmetic.

Attention reaches a result with a plain definition (softmax attention over the
stored values), so it is pinned against a pure-Python evaluation, against
torch's float64 scaled-dot-product attention, against its own blockwise and
split-merged forms ("Tiled attention and mixed precision": running max and
normaliser), and on special cases with known answers.
"""
import math

import numpy as np
import pytest
import torch

from oracle import confkv_oracle as O


def _rand(rng, *shape):
    return rng.standard_normal(shape)


def test_naive_matches_pure_python_loops():
    rng = np.random.default_rng(0)
    G, n, D = 2, 5, 3
    q, k, v = _rand(rng, G, D), _rand(rng, n, D), _rand(rng, n, D)
    scale = 0.37
    out, p = O.attention_naive(q, k, v, scale)
    for h in range(G):
        s = [scale * sum(q[h][d] * k[i][d] for d in range(D)) for i in range(n)]
        mx = max(s)
        e = [math.exp(x - mx) for x in s]
        Z = sum(e)
        for i in range(n):
            assert abs(p[h, i] - e[i] / Z) < 1e-14
        for d in range(D):
            assert abs(out[h, d] - sum(e[i] / Z * v[i][d] for i in range(n))) < 1e-13


def test_naive_matches_torch_sdpa_float64():
    rng = np.random.default_rng(1)
    G, n, D = 5, 333, 128
    q, k, v = _rand(rng, G, D), _rand(rng, n, D), _rand(rng, n, D)
    out, _ = O.attention_naive(q, k, v, 1 / math.sqrt(D))
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q)[None], torch.from_numpy(k)[None], torch.from_numpy(v)[None])[0].numpy()
    assert np.max(np.abs(out - ref)) < 1e-12


@pytest.mark.parametrize("block", [1, 7, 128, 301])
def test_blockwise_equals_naive(block):
    rng = np.random.default_rng(2)
    G, n, D = 4, 301, 64
    q, k, v = 3 * _rand(rng, G, D), _rand(rng, n, D), _rand(rng, n, D)
    scale = 1 / math.sqrt(D)
    out, p = O.attention_naive(q, k, v, scale)
    outb, m, l = O.attention_blockwise(q, k, v, scale, block)
    assert np.max(np.abs(out - outb)) < 1e-12
    s = scale * (q @ k.T)
    assert np.max(np.abs(np.exp(s - m[:, None]) / l[:, None] - p)) < 1e-12
    assert np.allclose(m, np.max(s, axis=1), rtol=0, atol=1e-12)


def test_split_merge_equals_naive():
    rng = np.random.default_rng(3)
    G, n, D = 4, 517, 32
    q, k, v = 2 * _rand(rng, G, D), _rand(rng, n, D), _rand(rng, n, D)
    scale = 0.2
    out, p = O.attention_naive(q, k, v, scale)
    for cuts in ([0, 517], [0, 1, 517], [0, 100, 101, 400, 517], list(range(0, 517, 37)) + [517]):
        ms, ls, os_ = [], [], []
        for lo, hi in zip(cuts[:-1], cuts[1:]):
            o, m, l = O.attention_blockwise(q, k[lo:hi], v[lo:hi], scale, 64)
            ms.append(m); ls.append(l); os_.append(o * l[:, None])
        outm, M, L = O.merge_partials(np.array(ms), np.array(ls), np.array(os_))
        assert np.max(np.abs(outm - out)) < 1e-12
        s = scale * (q @ k.T)
        assert np.max(np.abs(np.exp(s - M[:, None]) / L[:, None] - p)) < 1e-12


def test_special_cases():
    rng = np.random.default_rng(4)
    D = 16
    q = _rand(rng, 3, D)
    # one token: p = 1, out = v
    k, v = _rand(rng, 1, D), _rand(rng, 1, D)
    out, p = O.attention_naive(q, k, v, 0.25)
    assert np.all(p == 1.0) and np.allclose(out, np.repeat(v, 3, 0), atol=1e-15)
    # all-equal scores (identical keys): p = 1/n, out = mean(v)
    n = 9
    k = np.repeat(_rand(rng, 1, D), n, 0)
    v = _rand(rng, n, D)
    out, p = O.attention_naive(q, k, v, 0.25)
    assert np.allclose(p, 1 / n, atol=1e-15) and np.allclose(out, v.mean(0)[None], atol=1e-14)
    # a dominant key takes all the mass and the output is its value (not its key)
    k = _rand(rng, n, D)
    k[4] = 50 * q[0]
    out, p = O.attention_naive(q[:1], k, v, 1.0)
    assert p[0, 4] > 1 - 1e-12 and np.allclose(out[0], v[4], atol=1e-9)


def test_int8_path_is_fp16_path_on_dequantised_values():
    rng = np.random.default_rng(5)
    n, D, G = 40, 64, 2
    k16 = _rand(rng, n, D).astype(np.float16)
    v16 = _rand(rng, n, D).astype(np.float16)
    u = O.load_prefill(k16, v16, fp16_window=8)
    assert u.n16 == 8 and not u.is16[:32].any() and u.is16[32:].all()
    kd, vd = u.stored_k(), u.stored_v()
    # INT8 slots read code*scale, FP16 slots the fp16 value
    assert np.array_equal(kd[32:], k16[32:].astype(np.float64))
    assert np.array_equal(kd[:32], u.k8[:32].astype(np.float64) * u.ks[:32].astype(np.float64)[:, None])
    q = _rand(rng, G, D).astype(np.float16)
    knew, vnew = _rand(rng, D).astype(np.float16), _rand(rng, D).astype(np.float16)
    out, A = O.attend_unit(u, q, knew, vnew, n, 0.125, 0.9)
    kfull = np.vstack([kd, knew.astype(np.float64)[None]])
    vfull = np.vstack([vd, vnew.astype(np.float64)[None]])
    ref, p = O.attention_naive(q.astype(np.float64), kfull, vfull, 0.125)
    assert np.array_equal(out, ref) and np.array_equal(A, p.sum(0))


def _fresh_unit(rng, n, D, W=-1):
    return O.load_prefill(_rand(rng, n, D).astype(np.float16), _rand(rng, n, D).astype(np.float16), W)


def test_mass_sums_to_group_size_and_ema_closed_form():
    rng = np.random.default_rng(6)
    D, G, lam = 32, 4, 0.9
    u = _fresh_unit(rng, 50, D, W=10)
    for t in range(12):
        q = (2 * _rand(rng, G, D)).astype(np.float16)
        _, A = O.attend_unit(u, q, _rand(rng, D).astype(np.float16), _rand(rng, D).astype(np.float16),
                             50 + t, 1 / math.sqrt(D), lam)
        assert abs(A.sum() - G) < 1e-12                     # mass sums to the query-head count
        # no eviction: sum_i a_i = G (1 - lambda^(t+1)), up to fp32 storage rounding
        assert abs(float(u.ema.astype(np.float64).sum()) - G * (1 - lam ** (t + 1))) < 2e-6
    assert u.n == 62 and u.ema.dtype == np.float32


def test_ema_decay_extremes():
    rng = np.random.default_rng(7)
    D, G = 16, 2
    for lam in (0.0, 1.0):
        u = _fresh_unit(rng, 20, D)
        A = None
        for t in range(3):
            _, A = O.attend_unit(u, _rand(rng, G, D).astype(np.float16), _rand(rng, D).astype(np.float16),
                                 _rand(rng, D).astype(np.float16), 20 + t, 0.25, lam)
        if lam == 0.0:
            assert np.array_equal(u.ema, A.astype(np.float32))   # last step's mass only
        else:
            assert not u.ema.any()                                # never moves off 0


def test_new_token_is_attended_and_gets_mass():
    rng = np.random.default_rng(8)
    D = 16
    u = _fresh_unit(rng, 10, D)
    q = _rand(rng, 1, D).astype(np.float16)
    knew = (40 * q[0].astype(np.float32)).astype(np.float16)      # the new key dominates
    vnew = _rand(rng, D).astype(np.float16)
    out, A = O.attend_unit(u, q, knew, vnew, 10, 1.0, 0.5)
    assert A[-1] > 0.999999 and np.allclose(out[0], vnew.astype(np.float64), atol=1e-5)
    assert u.pos[-1] == 10 and u.is16[-1] and abs(float(u.ema[-1]) - 0.5 * A[-1]) < 1e-7
