"""GPU parity: every C-ABI entry point of the HIP library against the CPU oracle.

All tests here need an MI355X and call through the C ABI (ctypes -> libconfkv.so).
Tolerances: attention output 2e-3 relative / 1e-3 absolute; confidence 1e-5 absolute;
budget choices, kept-token sets and cache contents bit-exact except ties within 1e-6
relative of the threshold or cut-off, which the harness counts.
"""
import math
import os
import sys

import numpy as np
import pytest

from oracle import confkv_oracle as O
from synth import generate as gen
from synth.workloads import small, workload

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
from harness import CONF_ATOL, Lockstep, f32, policy_of  # noqa: E402

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return torch


def _mk(lib, **kw):
    base = dict(n_layers=1, batch=1, n_q_heads=4, n_kv_heads=1, head_dim=128, vocab=1000, capacity=256,
                fp16_window=16, protected_window=8, n_tight=[64], n_loose=[128])
    base.update(kw)
    return lib.ConfKV(**base)


# ------------------------------------------------------------------ confidence / budget

@pytest.mark.parametrize("V,B", [(2, 1), (4096, 2), (4097, 3), (50257, 1), (128256, 8), (152064, 1)])
def test_confidence_matches_oracle(lib, torch_cuda, V, B):
    torch = torch_cuda
    say(f"confidence V={V} B={B}")
    kv = _mk(lib, vocab=V, batch=B)
    rng = np.random.default_rng(V + B)
    conf = torch.zeros(B, dtype=torch.float32, device="cuda")
    sel = torch.zeros(B, dtype=torch.uint8, device="cuda")
    w = (f32(0.4), f32(0.3), f32(0.3))
    for std in (0.5, 3.0, 6.0, 12.0):
        x = (rng.standard_normal((B, V)) * std).astype(np.float32) + np.float32(rng.normal() * 30)
        kv.step(torch.from_numpy(x).cuda(), conf, sel)
        c = conf.cpu().numpy()
        ref = np.array([O.confidence(r, w) for r in x])
        assert np.max(np.abs(c - ref)) <= CONF_ATOL, (std, c, ref)
        far = np.abs(ref - f32(0.7)) > 1e-5
        assert np.array_equal(sel.cpu().numpy().astype(bool)[far], (ref >= f32(0.7))[far])
    kv.close()


def test_confidence_closed_forms_and_budgets(lib, torch_cuda):
    torch = torch_cuda
    V, B, L = 50257, 4, 3
    kv = _mk(lib, vocab=V, batch=B, n_layers=L, n_tight=[64, 48, 32], n_loose=[128, 96, 64])
    x = np.zeros((B, V), dtype=np.float32)
    x[1] = 5.0                                   # uniform at another level
    x[2] = -1.0e4; x[2, 123] = 0.0               # one-hot -> c = 1
    x[3] = -np.inf; x[3, :3] = 1.5               # three equal maxima, rest -inf
    conf = torch.zeros(B, dtype=torch.float32, device="cuda")
    sel = torch.zeros(B, dtype=torch.uint8, device="cuda")
    kv.step(torch.from_numpy(x).cuda(), conf, sel)
    c = conf.cpu().numpy().astype(np.float64)
    assert abs(c[0] - (0.15 + 0.3 / V)) < CONF_ATOL and abs(c[1] - c[0]) < 1e-7
    assert abs(c[2] - 1.0) < CONF_ATOL
    assert abs(c[3] - (0.4 * (1 - math.log(3) / math.log(V)) + 0.15 + 0.1)) < CONF_ATOL
    assert list(sel.cpu().numpy()) == [0, 0, 1, 0]
    st = kv.counters()
    assert (st.tight_steps, st.loose_steps) == (1, 3)
    # the chosen budgets act in the next eviction: fill every layer past both budgets
    D = 128
    rng = np.random.default_rng(0)
    for l in range(L):
        K = torch.from_numpy(rng.standard_normal((B, 1, 200, D)).astype(np.float16)).cuda()
        kv.load_prefill(l, K, K)
    kv.evict_compact()
    ln, _ = kv.lengths()
    assert ln.tolist() == [[128, 128, 64, 128], [96, 96, 48, 96], [64, 64, 32, 64]]
    kv.close()


# ------------------------------------------------------------------ prompt load / export

@pytest.mark.parametrize("D,W,T0", [(128, 16, 100), (64, 8, 37), (128, -1, 50), (64, 0, 20), (128, 300, 40)])
def test_prefill_quantiser_bit_exact(lib, torch_cuda, D, W, T0):
    torch = torch_cuda
    say(f"prefill D={D} W={W} T0={T0}")
    B, H = 2, 2
    kv = _mk(lib, batch=B, n_q_heads=2 * H, n_kv_heads=H, head_dim=D, fp16_window=W, capacity=320 if W < 300 else 512,
             n_tight=[200], n_loose=[300])
    rng = np.random.default_rng(D + T0)
    mag = rng.choice([1e-3, 0.05, 1.0, 40.0], size=(B, H, T0, 1))
    K = (rng.standard_normal((B, H, T0, D)) * mag).astype(np.float16)
    V = (rng.standard_normal((B, H, T0, D)) * mag).astype(np.float16)
    K[0, 0, 3] = 0                                         # a zero vector
    K[1, 1, 5] = np.float16(6e-8)                          # scale underflows to zero
    K[0, 1, 7, :8] = np.array([127, 0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 3.25], np.float16)  # exact ties
    e0 = rng.random((B, H, T0)).astype(np.float32)
    kv.load_prefill(0, torch.from_numpy(K).cuda(), torch.from_numpy(V).cuda(), torch.from_numpy(e0).cuda())
    for b in range(B):
        for g in range(H):
            u = O.load_prefill(K[b, g], V[b, g], W, e0[b, g])
            ex = kv.export(0, b, g)
            assert ex["n"] == T0 and np.array_equal(ex["pos"], np.arange(T0))
            assert np.array_equal(ex["is16"], u.is16) and np.array_equal(ex["ema"], e0[b, g])
            m8 = ~u.is16
            assert np.array_equal(ex["k8"][m8], u.k8[m8]) and np.array_equal(ex["v8"][m8], u.v8[m8])
            assert np.array_equal(ex["ks"][m8].view(np.uint16), u.ks[m8].view(np.uint16))
            assert np.array_equal(ex["vs"][m8].view(np.uint16), u.vs[m8].view(np.uint16))
            assert np.array_equal(ex["k16"][u.is16].view(np.uint16), K[b, g][u.is16].view(np.uint16))
            assert np.array_equal(ex["v16"][u.is16].view(np.uint16), V[b, g][u.is16].view(np.uint16))
    kv.close()


# ------------------------------------------------------------------ attention + mass EMA

def _attend_case(lib, torch, D, G, H, B, T0, W, splits, seed, scale_q=1.0, two_launch=False,
                 scale_mode="token", late_gain=1.0):
    say(f"attend D={D} G={G} Hkv={H} B={B} T0={T0} W={W} splits={splits} two_launch={two_launch} "
        f"scales={scale_mode}")
    if splits:
        os.environ["CONF_KV_SPLITS"] = str(splits)
    else:
        os.environ.pop("CONF_KV_SPLITS", None)
    if two_launch:
        os.environ["CONF_KV_TWO_LAUNCH"] = "1"
    try:
        cap = ((T0 + 8 + 63) // 64) * 64
        kv = _mk(lib, batch=B, n_q_heads=G * H, n_kv_heads=H, head_dim=D, fp16_window=W, capacity=cap,
                 protected_window=4, n_tight=[cap - 2], n_loose=[cap - 1], scale_mode=scale_mode)
    finally:
        os.environ.pop("CONF_KV_SPLITS", None)
        os.environ.pop("CONF_KV_TWO_LAUNCH", None)
    assert (kv.attend_splits(0) >= 1000) == two_launch
    rng = np.random.default_rng(seed)
    K = rng.standard_normal((B, H, T0, D)).astype(np.float16)
    V = rng.standard_normal((B, H, T0, D)).astype(np.float16)
    if scale_mode == "channel":
        # channels of very different ranges (what per-channel scales are for), one dead channel
        K = (K * rng.choice([0.05, 0.3, 1.0, 4.0], size=(B, H, 1, D))).astype(np.float16)
        V = (V * rng.choice([0.05, 0.3, 1.0, 4.0], size=(B, H, 1, D))).astype(np.float16)
        K[..., 5] = 0
        V[..., 17] = 0
    e0 = rng.random((B, H, T0)).astype(np.float32)
    kv.load_prefill(0, torch.from_numpy(K).cuda(), torch.from_numpy(V).cuda(), torch.from_numpy(e0).cuda())
    units = {(b, g): O.load_prefill(K[b, g], V[b, g], W, e0[b, g], scale_mode=scale_mode)
             for b in range(B) for g in range(H)}
    out = torch.zeros((B, G * H, D), dtype=torch.float16, device="cuda")
    sm, lam = f32(1 / math.sqrt(D)), f32(0.9)
    for t in range(3):
        q = (rng.standard_normal((B, G * H, D)) * scale_q).astype(np.float16)
        kn = (rng.standard_normal((B, H, D)) * late_gain).astype(np.float16)   # late_gain > 1: codes saturate
        vn = (rng.standard_normal((B, H, D)) * late_gain).astype(np.float16)
        kv.attend(0, torch.from_numpy(q).cuda(), torch.from_numpy(kn).cuda(), torch.from_numpy(vn).cuda(), out)
        got = out.cpu().numpy().astype(np.float64)
        for (b, g), u in units.items():
            ref, A = O.attend_unit(u, q[b, g * G:(g + 1) * G], kn[b, g], vn[b, g], T0 + t, sm, lam)
            err = np.max(np.abs(got[b, g * G:(g + 1) * G] - ref) / (1e-3 + 2e-3 * np.abs(ref)))
            assert err <= 1.0, f"step {t} unit {(b, g)}: out off by {err:.3g} x tol"
            ex = kv.export(0, b, g)
            assert ex["n"] == u.n and ex["pos"][-1] == T0 + t and ex["is16"][-1]
            assert np.array_equal(ex["k16"][-1].view(np.uint16), kn[b, g].view(np.uint16))
            assert np.array_equal(ex["v16"][-1].view(np.uint16), vn[b, g].view(np.uint16))
            e_ref = u.ema.astype(np.float64)
            e_err = np.abs(ex["ema"].astype(np.float64) - e_ref)
            assert np.all(e_err <= 1e-8 + 5e-6 * e_ref), f"step {t} unit {(b, g)}: EMA off, max rel {np.max(e_err / (e_ref + 1e-30)):.3g}"
        kv.evict_compact()                          # budgets above the length: commit + demotion only
        for (b, g), u in units.items():
            O.demote(u, W)
            if scale_mode == "channel":
                ex = kv.export(0, b, g)
                m8 = ~u.is16
                assert np.array_equal(ex["k8"][m8], u.k8[m8]) and np.array_equal(ex["v8"][m8], u.v8[m8])
                assert np.array_equal(ex["ks"].view(np.uint16), u.kcs.view(np.uint16))
                assert np.array_equal(ex["vs"].view(np.uint16), u.vcs.view(np.uint16))
    assert kv.counters().evicted == 0
    kv.close()



@pytest.mark.parametrize("D,G,H,B,T0,W,splits", [
    (64, 1, 3, 1, 200, -1, 0),        # GPT-2-like: MHA, FP16-only
    (64, 1, 2, 2, 700, -1, 5),
    (128, 4, 2, 2, 777, 40, 0),       # Llama-like GQA, mixed INT8 / FP16
    (128, 4, 2, 1, 777, 40, 1),       # one workgroup per unit
    (128, 4, 1, 1, 1500, 128, 7),     # ragged splits across the INT8 / FP16 boundary
    (128, 5, 2, 1, 600, 24, 3),       # Qwen-like group of five
    (128, 2, 1, 1, 300, 0, 2),        # W = 0: only the new token is FP16
    (128, 8, 1, 1, 260, 16, 2),
    (128, 3, 2, 1, 333, 20, 3),       # odd group sizes
    (128, 7, 1, 2, 411, 48, 2),
    (128, 6, 1, 1, 190, 8, 0),
    (64, 3, 1, 1, 150, 10, 2),
    (64, 7, 1, 1, 97, -1, 0),
    (64, 4, 2, 1, 130, 100, 4),
    (64, 8, 2, 2, 900, 48, 3),        # 64-channel heads in groups of eight (mixed INT8 / FP16), ragged splits
    (64, 8, 1, 1, 2100, 128, 0),      # the same at the default plan of a longer unit
    (64, 4, 2, 1, 777, -1, 5),        # 64-channel grouped heads, FP16-only
    (64, 2, 1, 1, 300, 0, 2),
    (64, 5, 1, 2, 411, 33, 1),
    (128, 16, 1, 2, 900, 64, 3),      # sixteen query heads per kv-head: the 16-row kernel with one token
    (128, 12, 2, 1, 500, 32, 0),      # twelve: four padding rows
    (128, 9, 1, 1, 300, -1, 2),
    (128, 4, 1, 1, 36000, -1, 0),     # longer than any register-resident path assumes
    (128, 4, 1, 1, 5, 2, 0),          # a tiny cache
    (128, 1, 1, 1, 0, 4, 0),          # empty cache: the query sees only itself
])
def test_attend_matches_oracle(lib, torch_cuda, D, G, H, B, T0, W, splits):
    _attend_case(lib, torch_cuda, D, G, H, B, T0, W, splits, seed=D + G + T0)


@pytest.mark.parametrize("D,G,H,B,T0,W,splits", [
    (128, 4, 2, 2, 700, 32, 3), (128, 4, 1, 1, 300, 16, 1), (64, 1, 3, 1, 333, -1, 4),
    (128, 5, 2, 1, 1000, 64, 7), (64, 2, 2, 2, 150, 0, 2), (128, 8, 1, 1, 520, 200, 5),
    (64, 8, 2, 1, 800, 40, 4), (64, 4, 1, 2, 500, -1, 3), (128, 12, 1, 1, 700, 48, 3)])
def test_attend_two_launch_form(lib, torch_cuda, D, G, H, B, T0, W, splits):
    """The form used when the splits of a unit cannot all be resident: scores and partials go
    through scratch and a second kernel finishes.  Forced here on small shapes."""
    _attend_case(lib, torch_cuda, D, G, H, B, T0, W, splits, seed=T0 + G, two_launch=True)


@pytest.mark.parametrize("G,H,B,T0,W,splits,two_launch", [
    (4, 2, 2, 777, 40, 0, False),      # matrix-core body, default plan
    (4, 1, 1, 1500, 128, 7, False),    # ragged splits across the INT8 / FP16 boundary
    (5, 2, 1, 600, 24, 3, False), (8, 1, 1, 260, 16, 2, False), (2, 1, 1, 300, 0, 2, False),
    (3, 2, 1, 333, 20, 1, False), (7, 1, 2, 411, 48, 2, False), (6, 1, 1, 190, 8, 0, False),
    (1, 2, 1, 500, 16, 3, False),      # G = 1: vector-ALU body
    (4, 2, 2, 700, 32, 3, True), (1, 1, 1, 300, 8, 2, True), (5, 1, 1, 900, 64, 5, True),
    (4, 1, 1, 5, 2, 0, False),         # a tiny cache
])
def test_attend_channel_scales(lib, torch_cuda, G, H, B, T0, W, splits, two_launch):
    """INT8 scales per (kv-head, channel), fixed on the prompt and folded into the query and the
    output ("Tiled attention and mixed precision"); late tokens three times the prompt's range
    saturate when they are demoted."""
    _attend_case(lib, torch_cuda, 128, G, H, B, T0, W, splits, seed=7 * G + T0, two_launch=two_launch,
                 scale_mode="channel", late_gain=3.0)


def test_attend_channel_scales_sharp_softmax(lib, torch_cuda):
    _attend_case(lib, torch_cuda, 128, 4, 1, 1, 900, 32, 6, seed=5, scale_q=6.0, scale_mode="channel")


def _chunk_case(lib, torch, G, H, B, T0, W, splits, tqs, seed, scale_mode="token", two_launch=False):
    say(f"chunks G={G} Hkv={H} B={B} T0={T0} W={W} splits={splits} tq={tqs} scales={scale_mode} two_launch={two_launch}")
    D = 128
    if splits:
        os.environ["CONF_KV_SPLITS"] = str(splits)
    if two_launch:
        os.environ["CONF_KV_TWO_LAUNCH"] = "1"
    try:
        room = max(16, max(tqs))                    # the budgets stay above every length the case reaches
        cap = ((T0 + sum(tqs) + room + 8 + 63) // 64) * 64
        kv = _mk(lib, batch=B, n_q_heads=G * H, n_kv_heads=H, head_dim=D, fp16_window=W, capacity=cap,
                 protected_window=4, n_tight=[cap - room - 1], n_loose=[cap - room], scale_mode=scale_mode,
                 max_chunk=max(tqs))
    finally:
        os.environ.pop("CONF_KV_SPLITS", None)
        os.environ.pop("CONF_KV_TWO_LAUNCH", None)
    rng = np.random.default_rng(seed)
    K = rng.standard_normal((B, H, T0, D)).astype(np.float16)
    V = rng.standard_normal((B, H, T0, D)).astype(np.float16)
    e0 = rng.random((B, H, T0)).astype(np.float32)
    kv.load_prefill(0, torch.from_numpy(K).cuda(), torch.from_numpy(V).cuda(), torch.from_numpy(e0).cuda())
    units = {(b, g): O.load_prefill(K[b, g], V[b, g], W, e0[b, g], scale_mode=scale_mode)
             for b in range(B) for g in range(H)}
    sm, lam = f32(1 / math.sqrt(D)), f32(0.9)
    pos = T0
    for tq in tqs:
        q = rng.standard_normal((B, tq, G * H, D)).astype(np.float16)
        kn = rng.standard_normal((B, tq, H, D)).astype(np.float16)
        vn = rng.standard_normal((B, tq, H, D)).astype(np.float16)
        # keys of the chunk that attract the chunk's own later queries: the causal part matters
        kn[:, 0] = (kn[:, 0].astype(np.float32) + 0.5 * q[:, -1, ::G][:, :H].astype(np.float32)).astype(np.float16)
        out = torch.zeros((B, tq, G * H, D), dtype=torch.float16, device="cuda")
        if tq == 1:
            kv.attend(0, torch.from_numpy(q[:, 0].copy()).cuda(), torch.from_numpy(kn[:, 0].copy()).cuda(),
                      torch.from_numpy(vn[:, 0].copy()).cuda(), out[:, 0])
        else:
            kv.attend_chunk(0, torch.from_numpy(q).cuda(), torch.from_numpy(kn).cuda(), torch.from_numpy(vn).cuda(), out)
        got = out.cpu().numpy().astype(np.float64)
        for (b, g), u in units.items():
            ref, _ = O.attend_chunk_unit(u, q[b, :, g * G:(g + 1) * G], kn[b, :, g], vn[b, :, g], pos, sm, lam)
            o = got[b, :, g * G:(g + 1) * G]
            err = np.max(np.abs(o - ref) / (1e-3 + 2e-3 * np.abs(ref)))
            assert err <= 1.0, f"tq {tq} unit {(b, g)}: out off by {err:.3g} x tol"
            ex = kv.export(0, b, g)
            assert ex["n"] == u.n and np.array_equal(ex["pos"], u.pos.astype(np.int32)) and ex["is16"][-tq:].all()
            assert np.array_equal(ex["k16"][-tq:].view(np.uint16), kn[b, :, g].view(np.uint16))
            assert np.array_equal(ex["v16"][-tq:].view(np.uint16), vn[b, :, g].view(np.uint16))
            e_ref = u.ema.astype(np.float64)
            e_err = np.abs(ex["ema"].astype(np.float64) - e_ref)
            assert np.all(e_err <= 1e-8 + 5e-6 * e_ref), f"tq {tq} unit {(b, g)}: EMA off, max rel {np.max(e_err / (e_ref + 1e-30)):.3g}"
        pos += tq
        kv.evict_compact()                          # budgets above the length: commit + demotion only
        for u in units.values():
            O.demote(u, W)
    for (b, g), u in units.items():
        ex = kv.export(0, b, g)
        assert np.array_equal(ex["is16"], u.is16)
        m8 = ~u.is16
        assert np.array_equal(ex["k8"][m8], u.k8[m8]) and np.array_equal(ex["v8"][m8], u.v8[m8])
    assert kv.counters().evicted == 0
    kv.close()


def _observe_case(lib, torch, G, H, B, T0, W, splits, windows, seed, scale_mode="token", two_launch=False,
                  decode_after=3):
    """The prompt's own attention over an observation window: conf_kv_observe against the oracle's
    observe_unit on the same cache, window by window, then decode steps with evictions ranked by
    the importance it left."""
    say(f"observe G={G} Hkv={H} B={B} T0={T0} W={W} splits={splits} windows={windows} scales={scale_mode} "
        f"two_launch={two_launch}")
    D = 128
    if splits:
        os.environ["CONF_KV_SPLITS"] = str(splits)
    if two_launch:
        os.environ["CONF_KV_TWO_LAUNCH"] = "1"
    try:
        cap = ((T0 + 8 + 63) // 64) * 64
        kv = _mk(lib, batch=B, n_q_heads=G * H, n_kv_heads=H, head_dim=D, fp16_window=W, capacity=cap,
                 protected_window=4, n_tight=[T0 - 20], n_loose=[T0 - 20], scale_mode=scale_mode,
                 max_chunk=max(2, max(tq for _, tq in windows)))
    finally:
        os.environ.pop("CONF_KV_SPLITS", None)
        os.environ.pop("CONF_KV_TWO_LAUNCH", None)
    rng = np.random.default_rng(seed)
    K = rng.standard_normal((B, H, T0, D)).astype(np.float16)
    V = rng.standard_normal((B, H, T0, D)).astype(np.float16)
    e0 = rng.random((B, H, T0)).astype(np.float32)
    kv.load_prefill(0, torch.from_numpy(K).cuda(), torch.from_numpy(V).cuda(), torch.from_numpy(e0).cuda())
    units = {(b, g): O.load_prefill(K[b, g], V[b, g], W, e0[b, g], scale_mode=scale_mode)
             for b in range(B) for g in range(H)}
    sm, lam = f32(1 / math.sqrt(D)), f32(0.9)
    for k, (first, tq) in enumerate(windows):
        q = rng.standard_normal((B, tq, G * H, D)).astype(np.float16)
        # sharpen: each query leans on a few keys it may see and on one it may not (ahead of it)
        for b in range(B):
            for g in range(H):
                near = K[b, g, rng.integers(0, first + 1)].astype(np.float32)
                ahead = K[b, g, min(T0 - 1, first + tq)].astype(np.float32)
                q[b, :, g * G:(g + 1) * G] = (q[b, :, g * G:(g + 1) * G].astype(np.float32) + 0.4 * near
                                              + 0.4 * ahead).astype(np.float16)
        want_out = k % 2 == 0                        # the output is optional
        out = torch.zeros((B, tq, G * H, D), dtype=torch.float16, device="cuda") if want_out else None
        kv.observe(0, first, torch.from_numpy(q).cuda(), out)
        got = out.cpu().numpy().astype(np.float64) if want_out else None
        for (b, g), u in units.items():
            before = u.ema.copy()
            ref, _ = O.observe_unit(u, q[b, :, g * G:(g + 1) * G], first, sm, lam)
            if want_out:
                o = got[b, :, g * G:(g + 1) * G]
                err = np.max(np.abs(o - ref) / (1e-3 + 2e-3 * np.abs(ref)))
                assert err <= 1.0, f"window {(first, tq)} unit {(b, g)}: out off by {err:.3g} x tol"
            ex = kv.export(0, b, g)
            assert ex["n"] == u.n == T0 and np.array_equal(ex["is16"], u.is16)
            e_ref = u.ema.astype(np.float64)
            e_err = np.abs(ex["ema"].astype(np.float64) - e_ref)
            assert np.all(e_err <= 1e-8 + 5e-6 * e_ref), \
                f"window {(first, tq)} unit {(b, g)}: EMA off, max rel {np.max(e_err / (e_ref + 1e-30)):.3g}"
            # slots past the window keep their bits
            assert np.array_equal(ex["ema"][first + tq:].view(np.uint32), before[first + tq:].view(np.uint32))
    # decode: the ranking now runs on what the observation left
    pos = T0
    for step in range(decode_after):
        q = rng.standard_normal((B, G * H, D)).astype(np.float16)
        kn = rng.standard_normal((B, H, D)).astype(np.float16)
        vn = rng.standard_normal((B, H, D)).astype(np.float16)
        out = torch.zeros((B, G * H, D), dtype=torch.float16, device="cuda")
        kv.attend(0, torch.from_numpy(q).cuda(), torch.from_numpy(kn).cuda(), torch.from_numpy(vn).cuda(), out)
        got = out.cpu().numpy().astype(np.float64)
        kv.evict_compact()
        for (b, g), u in units.items():
            ref, _ = O.attend_unit(u, q[b, g * G:(g + 1) * G], kn[b, g], vn[b, g], pos, sm, lam)
            err = np.max(np.abs(got[b, g * G:(g + 1) * G] - ref) / (1e-3 + 2e-3 * np.abs(ref)))
            assert err <= 1.0, f"decode {step} unit {(b, g)}: out off by {err:.3g} x tol"
            O.evict_compact_unit(u, T0 - 20, 4, f32(0.65), W)
            ex = kv.export(0, b, g)
            assert ex["n"] == u.n
            # (seeded inputs: no score pair at the cut is closer than the EMA tolerance)
            assert np.array_equal(ex["pos"], u.pos.astype(np.int32)), f"decode {step} unit {(b, g)}: kept set differs"
        pos += 1
    kv.close()


@pytest.mark.parametrize("G,H,B,T0,W,splits,windows,scales", [
    (4, 2, 2, 600, 64, 0, ((568, 4), (572, 4), (576, 4), (596, 4)), "token"),   # windows inside the FP16 tail
    (4, 1, 1, 900, 32, 3, ((100, 4), (104, 3), (860, 4), (864, 4), (896, 4)), "token"),  # INT8 slots as window
    (1, 2, 1, 400, 16, 2, ((368, 16), (384, 16)), "token"),                     # MHA, window crosses INT8 -> FP16
    (2, 1, 1, 300, 0, 2, ((292, 8),), "token"),                                 # W = 0: the whole cache is INT8
    (3, 1, 2, 260, -1, 2, ((0, 5), (5, 5), (255, 5)), "token"),                 # FP16-only cache, from slot 0
    (4, 1, 1, 700, 48, 3, ((690, 2), (692, 4), (696, 4)), "channel"),           # per-channel scales
    (8, 1, 1, 3000, 128, 0, ((2996, 2), (2998, 2)), "token"),                   # default plan of a long unit
    (4, 1, 1, 500, 40, 1, ((499, 1),), "token"),                                # a single query
])
def test_observe_matches_oracle(lib, torch_cuda, G, H, B, T0, W, splits, windows, scales):
    _observe_case(lib, torch_cuda, G, H, B, T0, W, splits, windows, seed=G * 100 + T0, scale_mode=scales)


@pytest.mark.parametrize("G,H,B,T0,W,splits,windows", [
    (4, 2, 1, 1200, 64, 0, ((1100, 16), (1116, 16), (1132, 12), (1190, 10))),   # 64-row windows, INT8 then FP16 slots
    (5, 1, 2, 700, 32, 2, ((0, 12), (12, 12), (600, 16))),                       # from slot 0; 80 rows
    (8, 1, 1, 640, 16, 4, ((500, 16), (624, 16))),                               # 128 rows, the last window ends the prompt
    (2, 1, 1, 300, -1, 0, ((100, 20), (120, 16))),                               # FP16-only cache
])
def test_observe_many_rows(lib, torch_cuda, G, H, B, T0, W, splits, windows):
    """Observation windows of more than 16 query rows per kv-head."""
    _observe_case(lib, torch_cuda, G, H, B, T0, W, splits, windows, seed=G * 10 + T0)


@pytest.mark.parametrize("G,T0,W,mc", [(4, 300, 32, 16), (5, 150, 16, 12), (1, 200, 8, 3)])
def test_observe_prompt_covers_every_query(lib, torch_cuda, G, T0, W, mc):
    """conf_kv_observe_prompt: every prompt query observes the prompt, in one call; equal to the
    oracle's observe_unit over the same consecutive windows, i.e. to T0 single-token decode steps
    over the stored prompt."""
    torch = torch_cuda
    H, B, D = 2, 2, 128
    say(f"observe_prompt G={G} T0={T0} W={W} max_chunk={mc}")
    kv = _mk(lib, batch=B, n_q_heads=G * H, n_kv_heads=H, head_dim=D, fp16_window=W, capacity=((T0 + 71) // 64) * 64,
             protected_window=4, n_tight=[T0 - 20], n_loose=[T0 - 20], max_chunk=mc)
    rng = np.random.default_rng(T0 + G)
    K = rng.standard_normal((B, H, T0, D)).astype(np.float16)
    V = rng.standard_normal((B, H, T0, D)).astype(np.float16)
    q = (rng.standard_normal((B, T0, G * H, D)) * 1.5).astype(np.float16)
    kv.load_prefill(0, torch.from_numpy(K).cuda(), torch.from_numpy(V).cuda())
    kv.observe_prompt(0, torch.from_numpy(q).cuda())
    sm, lam = f32(1 / math.sqrt(D)), f32(0.9)
    for b in range(B):
        for g in range(H):
            u = O.load_prefill(K[b, g], V[b, g], W)
            for first in range(0, T0, mc):
                O.observe_unit(u, q[b, first:first + mc, g * G:(g + 1) * G], first, sm, lam)
            ex = kv.export(0, b, g)
            e_ref = u.ema.astype(np.float64)
            e_err = np.abs(ex["ema"].astype(np.float64) - e_ref)
            assert np.all(e_err <= 1e-8 + 1e-5 * e_ref), f"unit {(b, g)}: EMA off, max rel {np.max(e_err / (e_ref + 1e-30)):.3g}"
            assert abs(float(e_ref.sum()) - G * (1 - lam ** T0) ) < 1e-3 * G     # all the mass of T0 steps is there
    assert kv.counters().device_errors == 0
    kv.close()


def test_observe_two_launch_form(lib, torch_cuda):
    _observe_case(lib, torch_cuda, 4, 2, 1, 1200, 64, 4, ((1190, 4), (1194, 4)), seed=5, two_launch=True)


def test_observe_call_errors(lib, torch_cuda):
    torch = torch_cuda

    def _raises(status, call):
        with pytest.raises(lib.ConfKVError) as ei:
            call()
        assert ei.value.status == status
    B, H, G, D, T0 = 1, 1, 4, 128, 100
    K = torch.zeros((B, H, T0, D), dtype=torch.float16, device="cuda")
    q = torch.zeros((B, 4, G * H, D), dtype=torch.float16, device="cuda")
    # needs the 16-row kernel: max_chunk >= 2
    kv = _mk(lib, batch=B, n_q_heads=G * H, n_kv_heads=H, head_dim=D, fp16_window=16, capacity=128,
             protected_window=4, n_tight=[80], n_loose=[90])
    kv.load_prefill(0, K, K, None)
    _raises(lib.binding.ERR_INVALID_ARG, lambda: kv.observe(0, 90, q[:, :1]))
    kv.close()
    kv = _mk(lib, batch=B, n_q_heads=G * H, n_kv_heads=H, head_dim=D, fp16_window=16, capacity=128,
             protected_window=4, n_tight=[80], n_loose=[90], max_chunk=4)
    _raises(lib.binding.ERR_BAD_STATE, lambda: kv.observe(0, 0, q))        # nothing loaded yet
    kv.load_prefill(0, K, K, None)
    _raises(lib.binding.ERR_INVALID_ARG, lambda: kv.observe(0, 97, q))      # window past the prompt
    _raises(lib.binding.ERR_INVALID_ARG, lambda: kv.observe(0, -1, q))
    kv.observe(0, 96, q)
    out = torch.zeros((B, G * H, D), dtype=torch.float16, device="cuda")
    kv.attend(0, q[:, 0].contiguous(), K[:, :, 0].contiguous(), K[:, :, 0].contiguous(), out)
    _raises(lib.binding.ERR_BAD_STATE, lambda: kv.observe(0, 96, q))        # the decode loop has begun
    kv.evict_compact()
    _raises(lib.binding.ERR_BAD_STATE, lambda: kv.observe(0, 96, q))
    kv.close()


@pytest.mark.parametrize("G,H,B,T0,W,splits,tqs,scales", [
    (4, 2, 2, 777, 40, 0, (4, 1, 3, 4), "token"),        # Llama-like group: up to 4 tokens a call
    (4, 1, 1, 1500, 128, 7, (4, 4), "token"),            # ragged splits, the chunk crosses tile borders
    (1, 2, 1, 300, 16, 2, (16, 5, 16), "token"),         # MHA: 16 tokens a call
    (2, 1, 1, 300, 0, 2, (8, 8), "token"),               # W = 0: everything but the chunk is INT8
    (5, 2, 1, 600, 24, 3, (3, 2, 3), "token"),           # 15 of 16 rows in use
    (8, 1, 1, 260, 16, 2, (2, 2), "token"),
    (3, 1, 2, 200, -1, 2, (5, 5, 1, 5), "token"),        # FP16-only cache at D = 128
    (4, 1, 1, 0, 6, 0, (4, 4, 4), "token"),              # from an empty cache: the chunk sees only itself
    (4, 2, 1, 700, 32, 3, (4, 2, 4), "channel"),         # per-channel scales
    (1, 1, 1, 500, 20, 1, (16, 16), "channel"),
    (4, 1, 1, 3000, 64, 0, (4, 4), "token"),             # default plan of a long unit (several splits)
])
def test_attend_chunk_matches_oracle(lib, torch_cuda, G, H, B, T0, W, splits, tqs, scales):
    """Several tokens per call: one read of the cache serves all their queries; outputs, the
    telescoped importance update, the appended rows and the later demotions follow the oracle."""
    _chunk_case(lib, torch_cuda, G, H, B, T0, W, splits, tqs, seed=11 * G + T0, scale_mode=scales)


@pytest.mark.parametrize("G,H,B,T0,W,splits,tqs", [
    (4, 2, 1, 777, 40, 0, (16, 8, 12)),          # 64, 32 and 48 query rows per kv-head
    (5, 1, 2, 600, 24, 2, (12, 16)),             # 60 rows (4 blocks), 80 rows (8 blocks, 3 of padding)
    (8, 1, 1, 500, 16, 0, (16,)),                # 128 rows: every block real
    (4, 1, 1, 3000, 64, 0, (16, 16)),            # default plan of a long unit (several splits)
    (4, 1, 1, 3000, 64, 8, (16, 5)),             # eight splits, the chunk straddles their FP16 shares
    (2, 1, 1, 300, 0, 2, (32,)),                 # W = 0: everything but the chunk is INT8
    (3, 1, 2, 200, -1, 2, (20, 7)),              # FP16-only cache
    (4, 1, 1, 0, 6, 0, (16, 16)),                # from an empty cache
    (1, 2, 1, 400, 16, 0, (64, 100)),            # MHA: 64 and 100 tokens a call
])
def test_attend_chunk_many_rows(lib, torch_cuda, G, H, B, T0, W, splits, tqs):
    """Calls with more query rows per kv-head than one matrix-core tile (up to 128): several row
    blocks per K/V tile, no score stash, the importance from a second pass over the keys."""
    _chunk_case(lib, torch_cuda, G, H, B, T0, W, splits, tqs, seed=17 * G + T0)


@pytest.mark.parametrize("G,H,B,T0,W,splits,tqs,scales", [
    (4, 2, 2, 700, 32, 3, (4, 3), "token"), (1, 1, 1, 500, 16, 5, (16, 7), "token"),
    (5, 1, 1, 900, 64, 7, (3, 3), "channel"), (2, 1, 1, 300, -1, 2, (8, 8), "token")])
def test_attend_chunk_two_launch_form(lib, torch_cuda, G, H, B, T0, W, splits, tqs, scales):
    """Multi-token calls on caches too long for a single launch go through scratch like the
    single-token ones; forced here on small shapes."""
    _chunk_case(lib, torch_cuda, G, H, B, T0, W, splits, tqs, seed=13 * G + T0, scale_mode=scales, two_launch=True)


@pytest.mark.parametrize("G,W,scales", [(4, 8, "token"), (1, 8, "token"), (2, -1, "token"), (4, 30, "channel")])
def test_lockstep_chunks_with_eviction(lib, torch_cuda, G, W, scales):
    """Whole steps whose attention appends 1 .. 16/G tokens at a time, with the budget rule
    evicting in between (several tokens leave per step) on wrapping rings."""
    mc = 16 // G
    wl = small(1).scaled(n_layers=2, batch=2, n_q_heads=2 * G, n_kv_heads=2, head_dim=128, vocab=3001,
                         prefill=100, steps=150, n_tight=(90, 70), n_loose=(100, 96), protected=max(8, mc),
                         fp16_window=W, logit_std=(0.5, 6.0), logit_run=5, alpha=0.5, scale_mode=scales,
                         max_chunk=mc)
    say(f"chunk lockstep: G={G} W={W} scales={scales} max_chunk={mc}")
    ls = Lockstep(lib, wl, seed=29)
    rng = np.random.default_rng(4)
    for t in range(wl.steps):
        ls.step(tq=int(rng.integers(1, mc + 1)))
    rep = ls.report
    st = ls.kv.counters()
    say(f"  out_err={rep.max_out_err:.3f}xtol ema_rel={rep.max_ema_rel:.2e} evictions={rep.evictions} "
        f"ties={rep.evict_ties} flips={rep.evict_flips}/{rep.budget_flips} demoted={st.demoted}")
    assert rep.ok(), (rep.evict_flips, rep.budget_flips)
    assert rep.evictions > wl.steps and st.device_errors == 0
    ls.close()


@pytest.mark.parametrize("G,W,mc", [(4, 8, 16), (5, 24, 12), (1, 8, 40)])
def test_lockstep_many_row_chunks_with_eviction(lib, torch_cuda, G, W, mc):
    """Whole steps whose attention appends up to `mc` tokens at a time (up to 64 query rows per
    kv-head), with the budget rule evicting in between."""
    wl = small(1).scaled(n_layers=2, batch=2, n_q_heads=2 * G, n_kv_heads=2, head_dim=128, vocab=3001,
                         prefill=300, steps=60, n_tight=(220, 180), n_loose=(330, 300), protected=max(8, mc),
                         fp16_window=W, logit_std=(0.5, 6.0), logit_run=5, alpha=0.5, max_chunk=mc)
    say(f"many-row chunk lockstep: G={G} W={W} max_chunk={mc}")
    ls = Lockstep(lib, wl, seed=31)
    rng = np.random.default_rng(6)
    for t in range(wl.steps):
        ls.step(tq=int(rng.integers(1, mc + 1)))
    rep = ls.report
    st = ls.kv.counters()
    say(f"  out_err={rep.max_out_err:.3f}xtol ema_rel={rep.max_ema_rel:.2e} evictions={rep.evictions} "
        f"ties={rep.evict_ties} flips={rep.evict_flips}/{rep.budget_flips} demoted={st.demoted}")
    assert rep.ok(), (rep.evict_flips, rep.budget_flips)
    assert rep.evictions > wl.steps and st.device_errors == 0
    ls.close()


def test_chunk_call_errors(lib, torch_cuda):
    torch = torch_cuda
    kv = _mk(lib, max_chunk=3, capacity=64, n_tight=[40], n_loose=[50])
    D = 128
    z = lambda *shape: torch.zeros(shape, dtype=torch.float16, device="cuda")
    with pytest.raises(lib.ConfKVError) as ei:
        kv.attend_chunk(0, z(1, 4, 4, D), z(1, 4, 1, D), z(1, 4, 1, D), z(1, 4, 4, D))     # tq > max_chunk
    assert ei.value.status == lib.binding.ERR_INVALID_ARG
    kv.attend_chunk(0, z(1, 3, 4, D), z(1, 3, 1, D), z(1, 3, 1, D), z(1, 3, 4, D))
    with pytest.raises(lib.ConfKVError) as ei:
        kv.attend(0, z(1, 4, D), z(1, 1, D), z(1, 1, D), z(1, 4, D))                       # second append before the commit
    assert ei.value.status == lib.binding.ERR_BAD_STATE
    assert kv.lengths()[0][0, 0] == 3
    kv.evict_compact()
    assert kv.lengths()[0][0, 0] == 3 and np.array_equal(kv.export(0, 0, 0)["pos"], [0, 1, 2])
    kv.close()
    plain = _mk(lib)                                                                        # max_chunk = 0
    with pytest.raises(lib.ConfKVError):
        plain.attend_chunk(0, z(1, 2, 4, D), z(1, 2, 1, D), z(1, 2, 1, D), z(1, 2, 4, D))
    plain.close()


def test_attend_sharp_softmax(lib, torch_cuda):
    # large-magnitude queries: a few slots take nearly all the mass, the rest underflow
    _attend_case(lib, torch_cuda, 128, 4, 1, 1, 900, 32, 6, seed=5, scale_q=6.0)


def test_ema_mass_invariant_without_eviction(lib, torch_cuda):
    # no eviction: sum_i ema_i = G (1 - lambda^t) after t steps (EMA starts at 0)
    torch = torch_cuda
    D, G, H, T0, W = 128, 4, 2, 500, 32
    kv = _mk(lib, n_q_heads=G * H, n_kv_heads=H, fp16_window=W, capacity=640, n_tight=[600], n_loose=[620])
    rng = np.random.default_rng(3)
    K = torch.from_numpy(rng.standard_normal((1, H, T0, D)).astype(np.float16)).cuda()
    kv.load_prefill(0, K, K)
    out = torch.zeros((1, G * H, D), dtype=torch.float16, device="cuda")
    lam = float(f32(0.9))
    for t in range(10):
        q = torch.from_numpy(rng.standard_normal((1, G * H, D)).astype(np.float16)).cuda()
        kn = torch.from_numpy(rng.standard_normal((1, H, D)).astype(np.float16)).cuda()
        kv.attend(0, q, kn, kn, out)
        kv.evict_compact()
        for g in range(H):
            ex = kv.export(0, 0, g)
            assert abs(ex["ema"].astype(np.float64).sum() - G * (1 - lam ** (t + 1))) < 2e-5
    kv.close()


# ------------------------------------------------------------------ ranking / eviction / compaction

def _evict_case(lib, torch, n, N, P, W, alpha, ema, D=64, seed=0):
    rng = np.random.default_rng(seed)
    cap = ((max(n, N, P) + 1 + 63) // 64) * 64
    kv = _mk(lib, n_q_heads=1, n_kv_heads=1, head_dim=D, fp16_window=W, protected_window=P, capacity=cap,
             n_tight=[N], n_loose=[N], alpha=alpha)
    K = rng.standard_normal((1, 1, n, D)).astype(np.float16)
    V = rng.standard_normal((1, 1, n, D)).astype(np.float16)
    kv.load_prefill(0, torch.from_numpy(K).cuda(), torch.from_numpy(V).cuda(),
                    torch.from_numpy(ema.reshape(1, 1, n).astype(np.float32)).cuda())
    u = O.load_prefill(K[0, 0], V[0, 0], W, ema.astype(np.float32))
    kv.evict_compact()
    gone = O.evict_compact_unit(u, N, P, f32(alpha), W)
    ex = kv.export(0, 0, 0)
    assert ex["n"] == u.n, (ex["n"], u.n)
    assert np.array_equal(ex["pos"], u.pos.astype(np.int32))
    assert np.array_equal(ex["is16"], u.is16) and np.array_equal(ex["ema"], u.ema)
    m8 = ~u.is16
    assert np.array_equal(ex["k8"][m8], u.k8[m8]) and np.array_equal(ex["v8"][m8], u.v8[m8])
    assert np.array_equal(ex["ks"][m8].view(np.uint16), u.ks[m8].view(np.uint16))
    assert np.array_equal(ex["k16"][u.is16].view(np.uint16), u.k16[u.is16].view(np.uint16))
    assert np.array_equal(ex["v16"][u.is16].view(np.uint16), u.v16[u.is16].view(np.uint16))
    assert kv.counters().evicted == gone.size
    kv.close()
    return u


def _page_case(lib, torch, n, N, P, W, page, alpha, ema, thin=None, D=64, seed=0):
    """Coarsened eviction of one unit against the oracle; thin = keep every slot with that
    probability first (positions with gaps, brought in through conf_kv_import)."""
    rng = np.random.default_rng(seed)
    cap = ((max(n, N, P + page) + 1 + 63) // 64) * 64
    cfg = dict(n_q_heads=1, n_kv_heads=1, head_dim=D, fp16_window=W, protected_window=P, capacity=cap,
               n_tight=[N], n_loose=[N], alpha=alpha, evict_page=page)
    kv = _mk(lib, **cfg)
    K = rng.standard_normal((1, 1, n, D)).astype(np.float16)
    V = rng.standard_normal((1, 1, n, D)).astype(np.float16)
    kv.load_prefill(0, torch.from_numpy(K).cuda(), torch.from_numpy(V).cuda(),
                    torch.from_numpy(ema.reshape(1, 1, n).astype(np.float32)).cuda())
    u = O.load_prefill(K[0, 0], V[0, 0], W, ema.astype(np.float32))
    if thin is not None:
        idx = np.flatnonzero(rng.random(n) < thin)
        view = kv.export(0, 0, 0)
        view = {k: (int(idx.size) if k == "n" else np.ascontiguousarray(np.asarray(x)[idx])) for k, x in view.items()}
        kv.close()
        kv = _mk(lib, **cfg)
        kv.import_unit(0, 0, 0, view)
        u.take(idx)
    n0 = u.n
    kv.evict_compact()
    gone = O.evict_compact_unit(u, N, P, f32(alpha), W, page=page)
    ex = kv.export(0, 0, 0)
    assert ex["n"] == u.n, (ex["n"], u.n)
    assert np.array_equal(ex["pos"], u.pos.astype(np.int32))
    assert np.array_equal(ex["is16"], u.is16) and np.array_equal(ex["ema"], u.ema)
    m8 = ~u.is16
    assert np.array_equal(ex["k8"][m8], u.k8[m8]) and np.array_equal(ex["v8"][m8], u.v8[m8])
    assert np.array_equal(ex["k16"][u.is16].view(np.uint16), u.k16[u.is16].view(np.uint16))
    assert kv.counters().evicted == gone.size == n0 - u.n
    kv.close()
    return u, gone


@pytest.mark.parametrize("n,N,P,W,page,thin", [
    (300, 100, 20, 30, 16, None), (300, 100, 20, -1, 16, None), (1000, 999, 1, 16, 32, None),
    (515, 64, 64, 8, 16, None), (200, 50, 0, 0, 4, None), (4000, 512, 128, 64, 16, None),
    (260, 100, 10, 150, 8, None), (90, 200, 10, 16, 16, None), (700, 699, 16, 32, 16, None),
    (3000, 2998, 64, -1, 32, None), (2500, 1024, 128, 64, 16, 0.7), (900, 300, 16, 32, 32, 0.4),
    (1200, 600, 40, -1, 16, 0.5), (400, 399, 8, 16, 2, 0.9), (5000, 4000, 128, 128, 1024, None),
])
def test_evict_pages_random_ema(lib, torch_cuda, n, N, P, W, page, thin):
    say(f"evict pages n={n} N={N} P={P} W={W} page={page} thin={thin}")
    rng = np.random.default_rng(n + N + page)
    u, gone = _page_case(lib, torch_cuda, n, N, P, W, page, 0.65, rng.random(n), thin=thin, seed=n)
    # pages go whole
    left = set((u.pos // page).tolist())
    assert not left & set((gone // page).tolist())


def test_evict_pages_ties_and_degenerate(lib, torch_cuda):
    say("evict pages: ties, degenerate cases")
    # every score equal (alpha = 1, equal mass): the oldest pages go, the last one whole
    u, gone = _page_case(lib, torch_cuda, 300, 250, 10, 16, 16, 1.0, np.full(300, 0.25))
    assert gone.tolist() == list(range(64)) and u.n == 236
    # recency only: a sliding window in whole pages
    u, gone = _page_case(lib, torch_cuda, 300, 251, 10, 16, 16, 0.0, np.random.default_rng(0).random(300))
    assert gone.tolist() == list(range(64))
    # two values: pages of equal mean tie exactly, older first
    ema = np.where((np.arange(512) // 16) % 2 == 0, 0.125, 0.875)
    u, gone = _page_case(lib, torch_cuda, 512, 400, 16, 32, 16, 1.0, ema)
    assert sorted(set((gone // 16).tolist())) == [0, 2, 4, 6, 8, 10, 12]
    # nothing can go: every candidate shares its page with a protected slot
    u, gone = _page_case(lib, torch_cuda, 60, 10, 40, 8, 64, 0.65, np.random.default_rng(1).random(60))
    assert gone.size == 0 and u.n == 60
    # fewer evictable slots than asked for: all of them go
    u, gone = _page_case(lib, torch_cuda, 100, 10, 30, 8, 32, 0.65, np.random.default_rng(2).random(100))
    assert gone.tolist() == list(range(64)) and u.n == 36
    # page of one = the token rule
    rng = np.random.default_rng(3)
    ema = rng.random(400)
    a, _ = _page_case(lib, torch_cuda, 400, 200, 16, 32, 1, 0.65, ema, seed=3)
    b = _evict_case(lib, torch_cuda, 400, 200, 16, 32, 0.65, ema, seed=3)
    assert np.array_equal(a.pos, b.pos)


@pytest.mark.parametrize("paired", [0, 1])
@pytest.mark.parametrize("G,D,W,N", [(4, 128, 16, (150, 230)), (1, 64, -1, (150, 230)), (2, 128, 120, (60, 100)),
                                     (3, 64, 12, (150, 230))])
def test_lockstep_both_compaction_forms(lib, torch_cuda, paired, G, D, W, N):
    """The compaction kernel has a form with one workgroup per plane and one that pairs K with V
    (chosen by the unit count); both are forced here on the same runs, the third of which evicts
    FP16 slots (the FP16 window is wider than the budgets).  Each run has a first step that moves
    hundreds of rows per unit (the chunked walk) and steady steps that move a few (the one-pass
    path of the unit's first workgroup), at both head dimensions."""
    wl = small(1).scaled(n_layers=2, batch=2, n_q_heads=2 * G, n_kv_heads=2, head_dim=D, vocab=2003, prefill=260,
                         steps=24, n_tight=(N[0],) * 2, n_loose=(N[1],) * 2, protected=20, fp16_window=W,
                         alpha=0.5, logit_std=(0.5, 6.0), logit_run=4)
    say(f"lockstep compaction form paired={paired} G={G} D={D} W={W} N={N}")
    os.environ["CONF_KV_COMPACT_PAIRED"] = str(paired)
    try:
        ls = Lockstep(lib, wl, seed=21)
        for t in range(wl.steps):
            ls.step()
        rep = ls.report
        assert rep.ok(), rep.evict_flips
        assert rep.evictions > 0 and rep.tight_steps > 0 and ls.kv.counters().device_errors == 0
        ls.close()
    finally:
        os.environ.pop("CONF_KV_COMPACT_PAIRED", None)


@pytest.mark.parametrize("prefill,D,W", [(6000, 128, 64), (1200, 64, -1), (40000, 128, 32)])
def test_lockstep_layer_scope_on_every_ranking_kernel(lib, torch_cuda, prefill, D, W):
    """One kept set per (layer, sequence) from the importance summed over the kv-heads, at unit
    lengths that take each ranking kernel in turn: the first step evicts thousands of slots (the
    register-resident kernels up to 33 792 slots, the scratch one above), the following ones one
    or two (the one-wavefront kernel)."""
    wl = small(1).scaled(n_layers=1, batch=2, n_q_heads=4, n_kv_heads=2, head_dim=D, vocab=1009, prefill=prefill,
                         steps=4, n_tight=(prefill // 3,), n_loose=(prefill // 2,), protected=16, fp16_window=W,
                         rank_scope="layer", logit_std=(0.5, 6.0), logit_run=2)
    say(f"lockstep layer scope prefill={prefill} D={D} W={W} capacity={wl.capacity}")
    ls = Lockstep(lib, wl, seed=31)
    for t in range(wl.steps):
        ls.step()
    rep = ls.report
    assert rep.ok(), rep.evict_flips
    assert rep.evictions > prefill // 3 and ls.kv.counters().device_errors == 0
    ls.close()


def test_expired_waits_end_the_kernels_and_are_reported(lib, torch_cuda):
    """The bounded in-kernel waits (splits of a unit waiting for each other's statistics, the
    confidence merger waiting for the chunks of its row) expire deterministically: a test hook
    makes split 0 of every unit and chunk 0 of every logit row keep their words to themselves, and
    the bound is a few polls.  Every kernel still runs to its end, each expired wait is counted
    and conf_kv_counters reports CONF_KV_ERR_DEVICE; a handle without the hook is unaffected."""
    torch = torch_cuda
    say("expired waits")
    B, H, G, D, T0, V = 1, 2, 4, 128, 3000, 50000
    rng = np.random.default_rng(0)
    K = torch.from_numpy(rng.standard_normal((B, H, T0, D)).astype(np.float16)).cuda()
    q = torch.from_numpy(rng.standard_normal((B, G * H, D)).astype(np.float16)).cuda()
    kn = torch.from_numpy(rng.standard_normal((B, H, D)).astype(np.float16)).cuda()
    lg = torch.from_numpy(rng.standard_normal((B, V)).astype(np.float32)).cuda()
    out = torch.empty_like(q)
    cfg = dict(batch=B, n_q_heads=G * H, n_kv_heads=H, head_dim=D, vocab=V, fp16_window=32, capacity=3072,
               protected_window=8, n_tight=[2000], n_loose=[2500])
    os.environ["CONF_KV_SPIN_LIMIT"] = "200"
    os.environ["CONF_KV_TEST_WITHHOLD"] = "1"
    os.environ["CONF_KV_SPLITS"] = "8"
    try:
        bad = _mk(lib, **cfg)
    finally:
        os.environ.pop("CONF_KV_SPIN_LIMIT", None)
        os.environ.pop("CONF_KV_TEST_WITHHOLD", None)
        os.environ.pop("CONF_KV_SPLITS", None)
    bad.load_prefill(0, K, K)
    assert bad.attend_splits(0) == 8
    bad.attend(0, q, kn, kn, out)
    torch.cuda.synchronize()
    # no split of either unit ever sees split 0's words (every split gathers all eight sets)
    assert bad.counters(check=False).device_errors == H * 8
    bad.step(lg)
    torch.cuda.synchronize()
    assert bad.counters(check=False).device_errors == H * 8 + B         # the row's merger never sees chunk 0
    bad.evict_compact()
    for _ in range(3):
        bad.attend(0, q, kn, kn, out)
        bad.step(lg)
        bad.evict_compact()
    torch.cuda.synchronize()
    st = bad.counters(check=False)
    assert st.device_errors == 4 * (H * 8 + B)
    with pytest.raises(lib.ConfKVError) as ei:
        bad.counters()
    assert ei.value.status == lib.binding.ERR_DEVICE
    bad.close()
    good = _mk(lib, **cfg)
    good.load_prefill(0, K, K)
    good.attend(0, q, kn, kn, out)
    good.step(lg)
    good.evict_compact()
    assert good.counters().device_errors == 0
    good.close()


def test_lockstep_wide_groups(lib, torch_cuda):
    """Groups of twelve query heads per kv-head through decode steps with evictions and demotions,
    and an observation window first (one query per call at this group size)."""
    wl = small(1).scaled(n_layers=2, batch=2, n_q_heads=24, n_kv_heads=2, head_dim=128, vocab=2003, prefill=300,
                         steps=16, n_tight=(150, 120), n_loose=(230, 200), protected=20, fp16_window=24,
                         logit_std=(0.5, 6.0), logit_run=3)
    say(f"lockstep G=12 capacity={wl.capacity}")
    ls = Lockstep(lib, wl, seed=12)
    for first in range(296, 300):
        ls.observe(first, 1)
    for t in range(wl.steps):
        ls.step()
    rep = ls.report
    assert rep.ok(), rep.evict_flips
    assert rep.evictions > 0 and ls.kv.counters().device_errors == 0
    ls.close()


@pytest.mark.parametrize("G,D,W,page,scope,tq", [(4, 128, 16, 16, "kv_head", 1), (1, 64, -1, 8, "kv_head", 1),
                                                 (4, 128, 24, 32, "layer", 1), (2, 128, 16, 16, "kv_head", 4)])
def test_lockstep_page_eviction(lib, torch_cuda, G, D, W, page, scope, tq):
    """Decode loops with coarsened eviction: state bit-identical to the oracle's at every step, and
    no page of original positions is ever partially dead (the newest, still filling one aside)."""
    wl = small(1).scaled(n_layers=2, batch=2, n_q_heads=2 * G, n_kv_heads=2, head_dim=D, vocab=2003, prefill=260,
                         steps=40, n_tight=(150, 120), n_loose=(230, 200), protected=20, fp16_window=W,
                         alpha=0.5, logit_std=(0.5, 6.0), logit_run=5, evict_page=page, rank_scope=scope,
                         max_chunk=tq if tq > 1 else 0)
    say(f"lockstep pages G={G} D={D} W={W} page={page} scope={scope} tq={tq} capacity={wl.capacity}")
    ls = Lockstep(lib, wl, seed=11)
    t = 0
    while t < wl.steps:
        ls.step(tq=tq)
        t += tq
        for key, u in ls.run.units.items():
            live = np.bincount((u.pos // page).astype(np.int64))
            newest = int(u.pos[-1]) // page
            bad = [k for k, c in enumerate(live) if c not in (0, page) and k != newest]
            assert not bad, (t, key, bad)
    rep = ls.report
    assert rep.ok(), rep.evict_flips
    assert rep.evictions > 0 and rep.tight_steps > 0
    assert ls.kv.counters().device_errors == 0
    ls.close()


@pytest.mark.parametrize("n,N,P,W", [(300, 100, 20, 30), (300, 100, 20, -1), (1000, 999, 1, 16),
                                     (515, 64, 64, 8), (200, 50, 0, 0), (4000, 512, 128, 64),
                                     (260, 100, 10, 150), (90, 200, 10, 16),
                                     # one to five slots over the budget: the one-wavefront ranking kernel
                                     (700, 699, 16, 32), (700, 698, 16, 32), (1300, 1297, 8, 64),
                                     (2100, 2096, 128, 64), (640, 635, 16, 700), (3000, 2998, 64, -1),
                                     # above 33 792 slots the scores live in scratch, not in registers
                                     (36000, 20000, 128, -1), (34000, 33990, 64, -1)])
def test_evict_random_ema(lib, torch_cuda, n, N, P, W):
    say(f"evict n={n} N={N} P={P} W={W}")
    rng = np.random.default_rng(n + N)
    _evict_case(lib, torch_cuda, n, N, P, W, 0.65, rng.random(n), seed=n)


def test_evict_ties_and_degenerate(lib, torch_cuda):
    torch = torch_cuda
    n = 400
    # all-equal EMA and alpha = 1: every score ties, the oldest go first
    u = _evict_case(lib, torch, n, 100, 16, 32, 1.0, np.full(n, 0.25))
    assert list(u.pos) == list(range(300, 400))
    # few distinct EMA levels: many exact ties at the cut-off
    rng = np.random.default_rng(1)
    _evict_case(lib, torch, n, 150, 16, 32, 1.0, rng.integers(0, 4, n) / 4.0)
    # alpha = 0: pure recency (sliding window)
    u = _evict_case(lib, torch, n, 150, 16, 32, 0.0, rng.random(n))
    assert list(u.pos) == list(range(250, 400))
    # protected window larger than the budget: the window wins
    u = _evict_case(lib, torch, n, 8, 50, 16, 0.65, rng.random(n))
    assert list(u.pos) == list(range(350, 400))
    # a single candidate
    _evict_case(lib, torch, 20, 19, 19, 4, 0.65, rng.random(20))
    # a few slots over the budget with ties at the cut-off: oldest first among equal scores
    u = _evict_case(lib, torch, n, n - 3, 16, 32, 1.0, np.full(n, 0.5))
    assert list(u.pos) == list(range(3, 400))
    lv = rng.integers(0, 3, n) / 2.0
    for over in (1, 2, 3, 4):
        _evict_case(lib, torch, n, n - over, 16, 32, 1.0, lv)
        _evict_case(lib, torch, n, n - over, 16, 500, 0.65, lv)


# ------------------------------------------------------------------ whole decode steps

@pytest.mark.parametrize("idx", [0, 1, 2, 3, 4])
def test_lockstep_small_workloads(lib, torch_cuda, idx):
    wl = small(idx)
    say(f"lockstep workload {idx}: {wl.name} (reduced) steps={wl.steps}")
    ls = Lockstep(lib, wl, seed=idx)
    for t in range(wl.steps):
        ls.step()
    rep = ls.report
    st = ls.kv.counters()
    say(f"  out_err={rep.max_out_err:.3f}xtol conf_err={rep.max_conf_err:.2e} ema_rel={rep.max_ema_rel:.2e} "
        f"evictions={rep.evictions} tight={rep.tight_steps} ties(evict/budget)={rep.evict_ties}/{rep.budget_ties} "
        f"flips={rep.evict_flips}/{rep.budget_flips} demoted={st.demoted}")
    assert rep.ok(), (rep.evict_flips, rep.budget_flips)
    assert rep.evictions > 0 and st.device_errors == 0
    if wl.fp16_window >= 0:
        assert st.demoted > 0
    ls.close()


def _expected_moves(pre, gone_pos, D, fp16_only, scale_bytes=4):
    """What the compaction has to move for one unit: (right shift?, head advance, bytes read +
    written).  Holes close from the side with fewer rows; the head-side shift is open when all
    holes lie in one payload ring (all INT8 in a mixed cache, any in an FP16-only one)."""
    idx = np.searchsorted(pre.pos, gone_pos)                        # evicted slot numbers
    n8_old = int((~pre.is16).sum())
    idx8 = idx[idx < n8_old]
    e, e8 = idx.size, idx8.size
    n_new, n8_new, first = pre.n - e, n8_old - e8, int(idx.min())
    if fp16_only:
        span, last, adv, can = n_new, int(idx.max()), e, True
    else:
        span, last, adv, can = n8_new, (int(idx8.max()) if e8 else -1), e8, (e8 > 0 and e == e8)
    left_rows = span - min(first, span)
    right_rows = last + 1 - adv
    right = can and right_rows < left_rows
    meta = right_rows if right else n_new - first
    if fp16_only:
        rows8, rows16 = 0, (right_rows if right else left_rows)
    else:
        rows8 = right_rows if right else left_rows
        rows16 = n_new - max(first, n8_new) if e > e8 else 0
    return right, (adv if right else 0), 2 * (rows8 * (2 * D + scale_bytes) + rows16 * 4 * D + meta * 8)


@pytest.mark.parametrize("G,D,W,alpha", [(4, 128, 8, 0.1), (1, 64, 8, 0.65), (5, 128, 8, 0.9), (1, 128, 8, 0.9),
                                         (1, 64, -1, 0.9), (3, 128, -1, 0.3), (4, 128, 30, 0.9)])
def test_lockstep_long_run_wraps_the_rings(lib, torch_cuda, G, D, W, alpha):
    """Many more steady-state steps than the unit has slots: the compaction closes holes from
    whichever side moves fewer rows, so the ring heads travel round the allocation several
    times (a recency-heavy ranker evicts old slots, which makes the head-side shift the cheap
    one), and budget switches (several holes at once) are mixed in.  W = -1 is the FP16-only
    cache; W = 30 exceeds the protected window, so FP16 slots get evicted too."""
    wl = small(1).scaled(n_layers=1, batch=1, n_q_heads=2 * G, n_kv_heads=2, head_dim=D, vocab=3001,
                         prefill=100, steps=700, n_tight=(97,), n_loose=(104,), protected=8,
                         fp16_window=W, logit_std=(0.5, 6.0), logit_run=7, alpha=alpha)
    assert wl.capacity == 128
    say(f"ring wrap: G={G} D={D} W={W} alpha={alpha} capacity={wl.capacity} steps={wl.steps}")
    ls = Lockstep(lib, wl, seed=11)
    travel = {key: 0 for key in ls.run.units}       # rows the slot-anchored ring head should have advanced
    shifts = {"left": 0, "right": 0}
    moved_bytes = 0                                 # traffic of the moves the compaction has to make
    for t in range(wl.steps):
        ls.step(check_state=(t % 3 == 0 or t > wl.steps - 10))
        for key, gone_pos in ls.last_gone.items():
            if gone_pos.size == 0:
                continue
            right, adv, nbytes = _expected_moves(ls.last_before[key], gone_pos, D, W < 0)
            travel[key] += adv
            shifts["right" if right else "left"] += 1
            moved_bytes += nbytes
    say(f"  ring head travel per unit: {travel}, shifts {shifts}")
    if alpha < 0.8:
        assert min(travel.values()) > 2 * wl.capacity   # every unit's rings wrapped at least twice
    else:
        assert min(shifts.values()) > 50                # both directions, on rings that have wrapped
        assert min(travel.values()) > wl.capacity
    rep = ls.report
    st = ls.kv.counters()
    say(f"  out_err={rep.max_out_err:.3f}xtol ema_rel={rep.max_ema_rel:.2e} evictions={rep.evictions} "
        f"tight={rep.tight_steps} flips={rep.evict_flips}/{rep.budget_flips} demoted={st.demoted}")
    assert rep.ok(), (rep.evict_flips, rep.budget_flips)
    assert rep.tight_steps > 0 and rep.tight_steps < wl.steps
    assert st.device_errors == 0 and (W < 0 or st.demoted > 2 * wl.capacity)
    assert st.compact_bytes == moved_bytes, (st.compact_bytes, moved_bytes)
    ls.close()


@pytest.mark.parametrize("G,W,alpha,steps", [(4, 8, 0.1, 400), (1, 8, 0.9, 300), (5, 30, 0.65, 300)])
def test_lockstep_channel_scales(lib, torch_cuda, G, W, alpha, steps):
    """Whole decode steps with per-(kv-head, channel) INT8 scales: prompt calibration, eviction,
    ring compaction in both directions (the scales do not travel with the rows) and demotion
    against the fixed scales, bit-exact against the oracle."""
    wl = small(1).scaled(n_layers=2, batch=2, n_q_heads=2 * G, n_kv_heads=2, head_dim=128, vocab=3001,
                         prefill=100, steps=steps, n_tight=(97, 80), n_loose=(104, 100), protected=8,
                         fp16_window=W, logit_std=(0.5, 6.0), logit_run=7, alpha=alpha, scale_mode="channel")
    say(f"channel scales lockstep: G={G} W={W} alpha={alpha}")
    ls = Lockstep(lib, wl, seed=23)
    moved_bytes = 0
    for t in range(wl.steps):
        ls.step(check_state=(t % 3 == 0 or t > wl.steps - 10))
        for key, gone_pos in ls.last_gone.items():
            if gone_pos.size:
                moved_bytes += _expected_moves(ls.last_before[key], gone_pos, 128, False, scale_bytes=0)[2]
    rep = ls.report
    st = ls.kv.counters()
    say(f"  out_err={rep.max_out_err:.3f}xtol ema_rel={rep.max_ema_rel:.2e} evictions={rep.evictions} "
        f"flips={rep.evict_flips}/{rep.budget_flips} demoted={st.demoted}")
    assert rep.ok(), (rep.evict_flips, rep.budget_flips)
    assert rep.evictions > 0 and st.demoted > 0 and st.device_errors == 0
    assert st.compact_bytes == moved_bytes, (st.compact_bytes, moved_bytes)
    ls.close()


def test_channel_scales_need_calibration_and_round_trip(lib, torch_cuda):
    torch = torch_cuda
    D, G, H = 128, 4, 2
    kw = dict(n_q_heads=G * H, n_kv_heads=H, fp16_window=4, capacity=64, protected_window=4,
              n_tight=[40], n_loose=[50], scale_mode="channel")
    a = _mk(lib, **kw)
    rng = np.random.default_rng(9)
    out = torch.zeros((1, G * H, D), dtype=torch.float16, device="cuda")
    q = torch.from_numpy(rng.standard_normal((1, G * H, D)).astype(np.float16)).cuda()
    kn = torch.from_numpy(rng.standard_normal((1, H, D)).astype(np.float16)).cuda()
    a.attend(0, q, kn, kn, out)                     # an empty cache: the query sees only itself
    assert np.allclose(out.cpu().numpy()[0, :G].astype(np.float64), kn.cpu().numpy()[0, 0].astype(np.float64))
    with pytest.raises(lib.ConfKVError) as ei:      # no scales were ever given to this layer
        a.evict_compact()
    assert ei.value.status == lib.binding.ERR_BAD_STATE
    a.close()
    # hand a calibrated cache over to a second handle and keep decoding on both
    a = _mk(lib, **kw)
    b = _mk(lib, **kw)
    K = (rng.standard_normal((1, H, 30, D)) * rng.choice([0.1, 1.0, 5.0], size=(1, H, 1, D))).astype(np.float16)
    a.load_prefill(0, torch.from_numpy(K).cuda(), torch.from_numpy(K[:, :, ::-1].copy()).cuda())
    for g in range(H):
        view = a.export(0, 0, g)
        assert view["ks"].shape == (D,) and view["n"] == 30
        b.import_unit(0, 0, g, view)
        bad = dict(view)
        bad["ks"] = view["ks"].copy()
        bad["ks"][3] = np.float16(-1.0)
        with pytest.raises(lib.ConfKVError):
            b.import_unit(0, 0, g, bad)
    oa, ob = torch.zeros_like(out), torch.zeros_like(out)
    for t in range(12):
        q = torch.from_numpy(rng.standard_normal((1, G * H, D)).astype(np.float16)).cuda()
        kn = torch.from_numpy((2 * rng.standard_normal((1, H, D))).astype(np.float16)).cuda()
        a.attend(0, q, kn, kn, oa)
        b.attend(0, q, kn, kn, ob)
        assert torch.equal(oa, ob)
        a.evict_compact()
        b.evict_compact()
    for g in range(H):
        va, vb = a.export(0, 0, g), b.export(0, 0, g)
        for name in va:
            assert np.array_equal(np.asarray(va[name]).view(np.uint8) if hasattr(va[name], "view") else va[name],
                                  np.asarray(vb[name]).view(np.uint8) if hasattr(vb[name], "view") else vb[name]), name
    a.close()
    b.close()


@pytest.mark.parametrize("idx,variant", [
    (1, dict(ema_decay=1.0, mass_gain=1.0)),                       # cumulative mass (H2O-shaped importance)
    (4, dict(mass_gain=0.25)),
    (1, dict(ranker="random", ranker_seed=12345)),                  # matched-rate random eviction
    (0, dict(ranker="random", ranker_seed=(1 << 63) + 77)),
    (1, dict(rank_scope="layer")),                                  # one kept set per (layer, sequence)
    (4, dict(rank_scope="layer")),
    (2, dict(rank_scope="layer", ranker="random", ranker_seed=3)),
    (0, dict(rank_scope="layer", alpha=1.0)),
    # the variants together: the paper's literal reading (layer-shared kept set, per-channel
    # scales), and several tokens per call under the random and the cumulative-mass rankers
    (1, dict(rank_scope="layer", scale_mode="channel")),
    (4, dict(rank_scope="layer", scale_mode="channel", max_chunk=4, tq=3)),
    (1, dict(ranker="random", ranker_seed=9, max_chunk=4, tq=4)),
    (2, dict(ema_decay=1.0, mass_gain=1.0, max_chunk=3, tq=2)),
])
def test_lockstep_ranker_variants(lib, torch_cuda, idx, variant):
    """The ranking variants against the oracle's: cumulative mass instead of the EMA, random
    eviction at the budget rule's rate, and the paper's literal one-kept-set-per-layer reading."""
    variant = dict(variant)
    tq = variant.pop("tq", 1)
    wl = small(idx).scaled(**variant)
    if wl.steps < 12:
        wl = wl.scaled(steps=12)
    say(f"variant {variant} tq={tq} on workload {idx} (reduced), steps={wl.steps}")
    ls = Lockstep(lib, wl, seed=20 + idx)
    for t in range(wl.steps):
        ls.step(tq=tq)
        if variant.get("rank_scope") == "layer":
            for (l, b, g), u in ls.run.units.items():              # kv-heads of a sequence stay aligned
                assert np.array_equal(u.pos, ls.run.units[(l, b, 0)].pos)
    rep = ls.report
    say(f"  out_err={rep.max_out_err:.3f}xtol ema_rel={rep.max_ema_rel:.2e} evictions={rep.evictions} "
        f"ties={rep.evict_ties} flips={rep.evict_flips}/{rep.budget_flips}")
    assert rep.ok(), (rep.evict_flips, rep.budget_flips)
    assert rep.evictions > 0 and ls.kv.counters().device_errors == 0
    if variant.get("mass_gain") == 1.0:
        # the importance is the running sum: it adds up to G per step and unit, minus what left
        ex = ls.kv.export(0, 0, 0)
        assert ex["ema"].sum() <= wl.steps * tq * wl.group + 1e-3 and ex["ema"].max() > 1.0
    ls.close()


def test_lockstep_geometric_pyramid(lib, torch_cuda):
    """Per-layer budgets from the library's pyramidal schedule (beta = 0.5 as in the paper)."""
    L = 4
    tight = lib.pyramid_budgets(180, L, 0.5, 60)
    assert tight == O.pyramid_geometric(180, L, 0.5, 60) and tight[0] == 180 and tight[-1] < tight[0]
    wl = small(4).scaled(n_layers=L, n_tight=tuple(tight), n_loose=tuple(2 * n for n in tight), steps=24)
    say(f"pyramid budgets {tight}")
    ls = Lockstep(lib, wl, seed=8)
    for t in range(wl.steps):
        ls.step()
    ln, _ = ls.kv.lengths()
    sel = ls.sel.cpu().numpy().astype(bool)
    for l in range(L):
        for b in range(wl.batch):
            assert ln[l, b] <= max(wl.protected, tight[l] if sel[b] else 2 * tight[l])
    assert ls.report.ok() and ls.report.evictions > 0
    ls.close()


def test_import_round_trip_and_rejections(lib, torch_cuda):
    """conf_kv_import is the inverse of conf_kv_export: a handle rebuilt from the exported views of
    another (whose rings have moved) attends, evicts and demotes bit-identically; malformed views
    are refused and leave the unit as it was."""
    torch = torch_cuda
    wl = small(1).scaled(n_layers=1, batch=1, n_q_heads=8, n_kv_heads=2, vocab=3001, prefill=150, steps=30,
                         n_tight=(120,), n_loose=(140,), protected=8, fp16_window=12, alpha=0.3,
                         logit_std=(0.5, 6.0), logit_run=3)
    say(f"import: capacity={wl.capacity}")
    a = Lockstep(lib, wl, seed=5)
    for t in range(wl.steps):                      # moves both ring heads of handle a
        a.step(check_state=False)
    b = lib.from_workload(wl)
    views = {g: a.kv.export(0, 0, g) for g in range(2)}
    for g in range(2):
        b.import_unit(0, 0, g, views[g])
        back = b.export(0, 0, g)
        for name, x in views[g].items():
            y = back[name]
            same = (x == y) if name == "n" else np.array_equal(np.asarray(x).view(np.uint8), np.asarray(y).view(np.uint8))
            assert same, f"kv-head {g}: {name} differs after import"
    # the same steps on both handles
    B, Hq, D = wl.batch, wl.n_q_heads, wl.head_dim
    out_a = torch.empty((B, Hq, D), dtype=torch.float16, device="cuda")
    out_b = torch.empty_like(out_a)
    conf = torch.empty(B, dtype=torch.float32, device="cuda")
    sel = torch.empty(B, dtype=torch.uint8, device="cuda")
    for t in range(wl.steps, wl.steps + 12):
        q, k, v = (torch.from_numpy(x).cuda() for x in gen.step_inputs(wl, 5, 0, t))
        lg = torch.from_numpy(gen.step_logits(wl, 5, t)).cuda()
        for kv, out in ((a.kv, out_a), (b, out_b)):
            kv.attend(0, q, k, v, out)
            kv.step(lg, conf, sel)
            kv.evict_compact()
        assert torch.equal(out_a, out_b), f"step {t}: outputs differ after import"
    for g in range(2):
        xa, xb = a.kv.export(0, 0, g), b.export(0, 0, g)
        for name in xa:
            same = (xa[name] == xb[name]) if name == "n" else \
                np.array_equal(np.asarray(xa[name]).view(np.uint8), np.asarray(xb[name]).view(np.uint8))
            assert same, f"kv-head {g}: {name} differs {12} steps after import"
    # rejections
    good = b.export(0, 0, 0)
    def refused(**change):
        v = dict(good); v.update(change)
        with pytest.raises(lib.ConfKVError) as e:
            b.import_unit(0, 0, 0, v)
        return e.value.status
    pos_bad = good["pos"].copy(); pos_bad[3] = pos_bad[2]
    assert refused(pos=pos_bad) == -1                                   # positions not increasing
    tags = good["is16"].copy(); tags[0] = True
    assert refused(is16=tags) == -1                                     # INT8 behind FP16
    assert refused(is16=np.ones_like(good["is16"])) == -1               # more FP16 slots than the window
    assert refused(n=wl.capacity) == -4
    assert refused(k8=None) == -1
    after = b.export(0, 0, 0)
    assert all(np.array_equal(np.asarray(good[k]), np.asarray(after[k])) for k in good if k != "n")
    q, k, v = (torch.from_numpy(x).cuda() for x in gen.step_inputs(wl, 5, 0, 99))
    b.attend(0, q, k, v, out_b)
    with pytest.raises(lib.ConfKVError) as e:
        b.import_unit(0, 0, 0, good)
    assert e.value.status == -5                                         # an append awaits its commit
    b.close()
    a.close()


@pytest.mark.parametrize("G,D,W", [(4, 128, 6), (1, 64, -1), (2, 128, 0)])
def test_lockstep_from_empty_cache_to_full_capacity(lib, torch_cuda, G, D, W):
    """Degenerate ends of the size range: decoding starts on an empty cache (the first query
    sees only its own token), the FP16 window fills and the first demotions happen, and the
    loose budget is capacity - 1, so every slot of the allocation, the last included, is used."""
    wl = small(1).scaled(n_layers=1, batch=2, n_q_heads=2 * G, n_kv_heads=2, head_dim=D, vocab=2003,
                         prefill=0, steps=150, n_tight=(40,), n_loose=(63,), protected=5, fp16_window=W,
                         logit_std=(0.5, 6.0), logit_run=30)
    assert wl.capacity == 64
    say(f"empty -> full: G={G} D={D} W={W}")
    ls = Lockstep(lib, wl, seed=31)
    seen = set()
    for t in range(wl.steps):
        ls.step()
        seen.add(ls.report.lengths[-1])
    assert 1 in seen and 63 in seen and 40 in seen
    assert ls.report.ok() and ls.report.evictions > 0 and ls.kv.counters().device_errors == 0
    ls.close()


def test_call_order_and_capacity_errors(lib, torch_cuda):
    torch = torch_cuda
    kv = _mk(lib, capacity=64, n_tight=[32], n_loose=[60], protected_window=4)
    z = torch.zeros((1, 4, 128), dtype=torch.float16, device="cuda")
    kn = torch.zeros((1, 1, 128), dtype=torch.float16, device="cuda")
    with pytest.raises(lib.ConfKVError) as e:
        kv.load_prefill(0, torch.zeros((1, 1, 64, 128), dtype=torch.float16, device="cuda"), kn)
    assert e.value.status == -4
    flat = torch.zeros(8 * 128 + 8, dtype=torch.float16, device="cuda")
    ok_k, off_k = flat[:8 * 128].view(1, 1, 8, 128), flat[1:8 * 128 + 1].view(1, 1, 8, 128)
    with pytest.raises(lib.ConfKVError) as e:
        kv.load_prefill(0, off_k, ok_k)                 # prompt rows are read in 16-byte pieces
    assert e.value.status == -1
    kv.attend(0, z, kn, kn, z)
    with pytest.raises(lib.ConfKVError) as e:
        kv.attend(0, z, kn, kn, z)                      # second append before the commit
    assert e.value.status == -5
    with pytest.raises(lib.ConfKVError) as e:
        kv.attend(3, z, kn, kn, z)
    assert e.value.status == -3
    kv.evict_compact()
    ln, n16 = kv.lengths()
    assert ln.tolist() == [[1]] and n16.tolist() == [[[1]]]
    kv.close()


def test_probe_read_reads_every_byte_once(lib, torch_cuda):
    """The bandwidth probe of the benchmark: its fold is the XOR of every 32-bit word, so a
    skipped or doubly read range would show."""
    torch = torch_cuda
    rng = np.random.default_rng(12)
    for n16, wgs in ((1, 1), (1000, 7), (70001, 256), (1 << 20, 2048)):
        x = rng.integers(-2**31, 2**31 - 1, size=n16 * 4, dtype=np.int64).astype(np.int32)
        out = torch.zeros(wgs, dtype=torch.int32, device="cuda")
        lib.probe_read(torch.from_numpy(x).cuda(), out, wgs)
        got = np.bitwise_xor.reduce(out.cpu().numpy().view(np.uint32))
        assert got == np.bitwise_xor.reduce(x.view(np.uint32)), (n16, wgs)


def _random_config(seed):
    """A seeded draw from the space of supported configurations (shapes, windows, budgets,
    ranker and scale variants, tokens per call), small enough for the oracle."""
    rng = np.random.default_rng(1000 + seed)
    D = int(rng.choice([64, 128], p=[0.3, 0.7]))
    G = int(rng.choice([1, 2, 3, 4, 5, 8]))
    H = int(rng.choice([1, 2, 3]))
    B = int(rng.choice([1, 2, 3]))
    W = int(rng.choice([-1, 0, 3, 12, 40]))
    P = int(rng.choice([0, 1, 7, 20]))
    prefill = int(rng.choice([0, 5, 60, 130, 333]))
    loose = int(rng.integers(max(P, 8) + 4, max(prefill, 24) + 16))     # most runs have to evict
    tight = int(rng.integers(max(1, loose // 3), loose + 1))
    L = int(rng.choice([1, 2]))
    kw = dict(n_layers=L, batch=B, n_q_heads=G * H, n_kv_heads=H, head_dim=D, vocab=int(rng.choice([257, 1000, 5003])),
              prefill=prefill, steps=int(rng.integers(12, 30)), n_tight=(tight,) * L, n_loose=(loose,) * L,
              protected=P, fp16_window=W, logit_std=(0.5, 6.0), logit_run=int(rng.integers(1, 6)),
              alpha=float(rng.choice([0.0, 0.3, 0.65, 1.0])), ema_decay=float(rng.choice([0.5, 0.9, 1.0])))
    if rng.random() < 0.3:
        kw["mass_gain"] = float(rng.choice([0.25, 1.0]))
    if rng.random() < 0.25:
        kw.update(ranker="random", ranker_seed=int(rng.integers(0, 2**62)))
    if rng.random() < 0.3:
        kw["rank_scope"] = "layer"
    if D == 128 and W >= 0 and rng.random() < 0.4:
        kw["scale_mode"] = "channel"
    if rng.random() < 0.3:
        kw["evict_page"] = int(rng.choice([2, 4, 16]))
    tq_max = 1
    if D == 128 and rng.random() < 0.5:
        tq_max = int(rng.integers(2, 16 // G + 1)) if 16 // G >= 2 else 1
        if tq_max > 1:
            kw["max_chunk"] = tq_max
    return kw, tq_max


@pytest.mark.parametrize("seed", list(range(32)))
def test_lockstep_random_configurations(lib, torch_cuda, seed):
    """Seeded random configurations across the whole option space, a few dozen steps each, in
    lock-step with the oracle: combinations no hand-written case covers."""
    kw, tq_max = _random_config(seed)
    wl = small(1).scaled(name=f"random{seed}", **kw)
    say(f"random config {seed}: {kw} capacity={wl.capacity}")
    ls = Lockstep(lib, wl, seed=seed)
    rng = np.random.default_rng(seed)
    for t in range(wl.steps):
        ls.step(tq=int(rng.integers(1, tq_max + 1)))
    rep = ls.report
    say(f"  out_err={rep.max_out_err:.3f}xtol ema_rel={rep.max_ema_rel:.2e} evictions={rep.evictions} "
        f"ties={rep.evict_ties} flips={rep.evict_flips}/{rep.budget_flips}")
    assert rep.ok(), (rep.evict_flips, rep.budget_flips)
    assert ls.kv.counters().device_errors == 0
    ls.close()


def test_heavy_hitter_recall_by_ranker_mode(lib, torch_cuda):
    """The structure of the matched-rate isolation study on synthetic data: every ranker evicts the
    same number of tokens (the budget rule decides how many), and what differs is which heavy-hitter
    keys of the prompt survive.  Ranking by attention alone keeps nearly all of them; the composite
    score gives a third of its weight to recency and keeps fewer, still well above recency alone
    (which keeps those that happen to be recent: about the kept fraction) and random."""
    torch = torch_cuda
    base = small(1).scaled(n_layers=1, batch=2, n_q_heads=8, n_kv_heads=2, prefill=1500, steps=24,
                           n_tight=(300,), n_loose=(300,), protected=32, fp16_window=32, logit_run=4)
    modes = {"composite": dict(alpha=0.65), "attention only": dict(alpha=1.0), "recency only": dict(alpha=0.0),
             "cumulative mass": dict(alpha=0.65, ema_decay=1.0, mass_gain=1.0),
             "random": dict(ranker="random", ranker_seed=5),
             # coarsened eviction: a heavy hitter survives only with its whole page
             "attention only, pages of 4": dict(alpha=1.0, evict_page=4),
             "attention only, pages of 16": dict(alpha=1.0, evict_page=16)}
    recall, kept_n = {}, {}
    for name, variant in modes.items():
        wl = base.scaled(**variant)
        kv = lib.from_workload(wl)
        K, V = gen.prefill_layer(wl, 0, 0)
        kv.load_prefill(0, torch.from_numpy(K).cuda(), torch.from_numpy(V).cuda())
        out = torch.empty((wl.batch, wl.n_q_heads, wl.head_dim), dtype=torch.float16, device="cuda")
        for t in range(wl.steps):
            q, k, v = gen.step_inputs(wl, 0, 0, t)
            kv.attend(0, torch.from_numpy(q).cuda(), torch.from_numpy(k).cuda(), torch.from_numpy(v).cuda(), out)
            kv.step(torch.from_numpy(gen.step_logits(wl, 0, t)).cuda())
            kv.evict_compact()
        hit = tot = 0
        for b in range(wl.batch):
            for g in range(wl.n_kv_heads):
                pos = kv.export(0, b, g)["pos"]
                hh = gen.prefill_heavy_hitters(wl, 0, 0, b, g)
                hit += int(np.isin(hh, pos).sum())
                tot += hh.size
                kept_n[name] = pos.size
        recall[name] = hit / tot
        kv.close()
    say("heavy-hitter recall after 1500 -> 300 slots: " + ", ".join(f"{k} {v:.2f}" for k, v in recall.items()))
    token_level = [k for k in modes if "pages" not in k]
    assert len({kept_n[k] for k in token_level}) == 1          # matched rate
    assert all(kept_n["composite"] - 16 < kept_n[k] <= kept_n["composite"] for k in modes)
    # whole pages dilute a single important token: recall falls with the page size
    assert recall["attention only"] >= recall["attention only, pages of 4"] >= recall["attention only, pages of 16"]
    assert recall["attention only, pages of 16"] > recall["random"]
    assert recall["attention only"] > 0.8
    assert recall["composite"] > recall["recency only"] + 0.1 and recall["composite"] > recall["random"] + 0.15
    assert recall["cumulative mass"] > recall["recency only"] + 0.1
    assert 0.1 <= recall["recency only"] <= 0.3 and recall["random"] <= 0.3     # the kept fraction is 0.2
