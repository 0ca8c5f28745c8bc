"""Pins for the oracle's per-(kv-head, channel) INT8 scale variant ("Tiled attention and mixed
precision": symmetric INT8 per head and channel, s = max|x| / 127; "Precision and layer
allocation" names the same granularity).  The scales are fixed on the prompt tokens.
"""
import numpy as np
import pytest

from oracle import confkv_oracle as O


def test_channel_scales_closed_form_and_axis():
    # column d holds values of magnitude up to d + 1, row t is scaled by (t + 1) / T <= 1:
    # the per-channel maximum is d + 1, the per-token maximum would be D (t + 1) / T
    T, D = 7, 5
    x = (np.outer((np.arange(T) + 1) / T, np.arange(D) + 1) * np.where(np.arange(T) % 2, -1, 1)[:, None])
    x = x.astype(np.float16)
    s = O.channel_scales(x)
    want = (np.arange(1, D + 1, dtype=np.float32) / np.float32(127)).astype(np.float16)
    assert s.dtype == np.float16 and np.array_equal(s, want)


def test_channel_mode_is_the_per_token_quantiser_on_the_transposed_matrix():
    # per-channel scales over a token set are per-vector scales of the columns: the pinned
    # per-token quantiser applied to column d must give the same scale and the same codes
    rng = np.random.default_rng(5)
    x = (rng.standard_normal((33, 12)) * rng.uniform(0.01, 30, size=12)).astype(np.float16)
    s = O.channel_scales(x)
    codes = np.stack([O.quantize_channels(x[t], s) for t in range(x.shape[0])])
    for d in range(x.shape[1]):
        c_col, s_col = O.quantize_vector(x[:, d])
        assert s_col == s[d]
        assert np.array_equal(c_col, codes[:, d])


def test_round_trip_error_bound_and_saturation():
    rng = np.random.default_rng(6)
    x = rng.standard_normal((200, 16)).astype(np.float16)
    s = O.channel_scales(x)
    codes = np.stack([O.quantize_channels(r, s) for r in x])
    back = O.dequantize_channels(codes, s)
    # inside the calibrated range the error is at most half a step (plus the fp16 rounding of
    # the scale, which can leave the largest value up to half a step outside 127 steps)
    assert np.all(np.abs(back - x.astype(np.float64)) <= 0.5 * s.astype(np.float64)[None, :] * (1 + 1e-12)
                  + np.abs(x.astype(np.float64)) * 2.0 ** -11)
    # the largest value of every channel takes the last code
    top = np.argmax(np.abs(x), axis=0)
    assert np.all(np.abs(codes[top, np.arange(16)]) == 127)
    # a later token outside the range saturates, sign kept
    big = (10 * np.max(np.abs(x), axis=0) * np.where(np.arange(16) % 2, -1, 1)).astype(np.float16)
    c = O.quantize_channels(big, s)
    assert np.array_equal(c, np.where(np.arange(16) % 2, -127, 127).astype(np.int8))


def test_zero_channel_and_half_way_rounding():
    x = np.zeros((4, 3), np.float16)
    x[:, 1] = [127, 0.5, 1.5, 2.5]            # scale exactly 1: halves round to even
    x[:, 2] = [-254, 3, -3, 1]                # scale exactly 2: 3/2 -> 2, -3/2 -> -2, 1/2 -> 0
    s = O.channel_scales(x)
    assert list(s) == [0, 1, 2]
    codes = np.stack([O.quantize_channels(r, s) for r in x])
    assert np.array_equal(codes[:, 0], [0, 0, 0, 0])
    assert np.array_equal(codes[:, 1], [127, 0, 2, 2])
    assert np.array_equal(codes[:, 2], [-127, 2, -2, 0])


def test_prefill_calibrates_on_every_prompt_token_and_demotion_reuses_the_scales():
    rng = np.random.default_rng(7)
    T, D, W = 40, 8, 6
    k = rng.standard_normal((T, D)).astype(np.float16)
    v = rng.standard_normal((T, D)).astype(np.float16)
    k[T - 1, 3] = 50.0                         # the largest value sits in the FP16 window
    u = O.load_prefill(k, v, W, scale_mode="channel")
    assert u.n16 == W and np.array_equal(u.kcs, O.channel_scales(k)) and np.array_equal(u.vcs, O.channel_scales(v))
    assert u.kcs[3] == np.float16(np.float32(50.0) / np.float32(127))
    # INT8 slots hold the codes of their own row against the fixed scales
    for i in range(T - W):
        assert np.array_equal(u.k8[i], O.quantize_channels(k[i], u.kcs))
        assert np.array_equal(u.v8[i], O.quantize_channels(v[i], u.vcs))
    # a decode step appends, demotes the oldest FP16 slot against the same scales
    kn, vn = (100 * rng.standard_normal(D)).astype(np.float16), rng.standard_normal(D).astype(np.float16)
    kcs = u.kcs.copy()
    O.append_token(u, kn, vn, T)
    old = u.k16[T - W].copy()
    O.demote(u, W)
    assert np.array_equal(u.kcs, kcs)
    assert np.array_equal(u.k8[T - W], O.quantize_channels(old, kcs)) and not u.is16[T - W]


def test_attention_folds_the_channel_scales_into_query_and_output():
    # with per-channel scales the score is (q * s_k) . codes and the INT8 part of the output
    # is s_v * (p @ codes): written out with explicit loops, independent of stored_k / stored_v
    rng = np.random.default_rng(8)
    T, D, G, W = 24, 8, 3, 4
    k = rng.standard_normal((T, D)).astype(np.float16)
    v = rng.standard_normal((T, D)).astype(np.float16)
    u = O.load_prefill(k, v, W, scale_mode="channel")
    q = rng.standard_normal((G, D)).astype(np.float16)
    kn, vn = rng.standard_normal(D).astype(np.float16), rng.standard_normal(D).astype(np.float16)
    ref = u.copy()
    out, A = O.attend_unit(u, q, kn, vn, T, 0.3, 0.9)
    n8 = T - W
    ks, vs = ref.kcs.astype(np.float64), ref.vcs.astype(np.float64)
    want = np.zeros((G, D))
    mass = np.zeros(T + 1)
    for h in range(G):
        s = np.zeros(T + 1)
        for i in range(T + 1):
            if i < n8:
                s[i] = 0.3 * sum(float(q[h, d]) * ks[d] * int(ref.k8[i, d]) for d in range(D))
            else:
                row = kn if i == T else k[i]
                s[i] = 0.3 * sum(float(q[h, d]) * float(row[d]) for d in range(D))
        p = np.exp(s - s.max())
        p /= p.sum()
        mass += p
        for d in range(D):
            acc8 = sum(p[i] * int(ref.v8[i, d]) for i in range(n8))
            acc16 = sum(p[i] * float((vn if i == T else v[i])[d]) for i in range(n8, T + 1))
            want[h, d] = vs[d] * acc8 + acc16
    assert np.allclose(out, want, rtol=1e-12, atol=1e-13)
    assert np.allclose(A, mass, rtol=1e-12, atol=1e-13)


def test_token_mode_is_unchanged_by_the_variant():
    rng = np.random.default_rng(9)
    k = rng.standard_normal((20, 8)).astype(np.float16)
    v = rng.standard_normal((20, 8)).astype(np.float16)
    u = O.load_prefill(k, v, 5)
    assert u.kcs is None and u.vcs is None
    for i in range(15):
        c, s = O.quantize_vector(k[i])
        assert np.array_equal(u.k8[i], c) and u.ks[i] == s
    with pytest.raises(ValueError):
        O.load_prefill(k, v, 5, scale_mode="row")
