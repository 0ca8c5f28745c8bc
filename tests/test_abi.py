"""The C-ABI library on a machine without a GPU: it loads, exports every symbol the header
declares, sizes buffers, and rejects bad arguments before touching the device."""
import ctypes as C
import os
import re

import pytest

import paper_2605_24786_amd as pkg

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def clib():
    return pkg.load_library()


def test_exports_every_declared_symbol(clib):
    header = open(os.path.join(ROOT, "include", "conf_kv.h")).read()
    body = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(conf_kv_[a-z0-9_]+)\s*\(", body))
    assert declared == set(pkg.SYMBOLS), declared ^ set(pkg.SYMBOLS)
    for name in declared:
        assert getattr(clib, name) is not None


def test_config_struct_matches_header():
    header = open(os.path.join(ROOT, "include", "conf_kv.h")).read()
    block = re.search(r"typedef struct conf_kv_config \{(.*?)\} conf_kv_config;", header, re.S).group(1)
    block = re.sub(r"/\*.*?\*/", "", block, flags=re.S)
    names = []
    for decl in block.split(";"):
        decl = decl.strip()
        if not decl:
            continue
        decl = re.sub(r"^(const\s+)?(int32_t|uint64_t|float)\s*\*?", "", decl)
        names += [n.strip().lstrip("*") for n in decl.split(",")]
    assert names == [f[0] for f in pkg.ConfKVConfig._fields_]


def _cfg(**kw):
    base = dict(n_layers=2, batch=1, n_q_heads=8, n_kv_heads=2, head_dim=128, vocab=1000, capacity=256,
                fp16_window=16, protected_window=8, n_tight=[64, 64], n_loose=[128, 128])
    base.update(kw)
    return pkg.make_config(**base)


def test_buffer_sizes(clib):
    cfg, *_ = _cfg()
    sb, kb = clib.conf_kv_state_bytes(C.byref(cfg)), clib.conf_kv_scratch_bytes(C.byref(cfg))
    U, cap, D = 4, 256, 128
    payload = U * (cap * (2 * D + 4 + 8) + 32 * 2 * D * 2)      # INT8 rows + scales + meta + FP16 ring
    assert payload <= sb <= payload + 64 * 1024 and sb % 256 == 0 and kb > 0
    cfgc, *_ = _cfg(scale_mode="channel")                        # per-channel scales: [U][D], not [U][cap]
    sbc = clib.conf_kv_state_bytes(C.byref(cfgc))
    assert 0 < sbc < sb and sb - sbc >= U * (cap - D) * 4 - 4 * 256
    cfg16, *_ = _cfg(fp16_window=-1)                             # FP16-only: no INT8 planes
    sb16 = clib.conf_kv_state_bytes(C.byref(cfg16))
    assert U * cap * (4 * D + 8) <= sb16 <= U * cap * (4 * D + 8) + 64 * 1024


@pytest.mark.parametrize("bad", [dict(head_dim=96), dict(n_q_heads=34, n_kv_heads=2), dict(n_q_heads=18, n_kv_heads=2, head_dim=64), dict(n_q_heads=7),
                                 dict(capacity=100), dict(capacity=128), dict(vocab=1), dict(alpha=1.5),
                                 dict(n_tight=[200, 64]), dict(protected_window=-1), dict(n_layers=0),
                                 dict(ema_decay=-0.1), dict(mass_gain=float("nan")), dict(_ranker=2),
                                 dict(_rank_scope=-1), dict(_scale_mode=2), dict(max_chunk=-1), dict(max_chunk=33),
                                 dict(max_chunk=5, scale_mode="channel"),
                                 dict(max_chunk=2, head_dim=64), dict(max_chunk=70, n_tight=[64, 64], n_loose=[200, 200]),
                                 dict(scale_mode="channel", head_dim=64), dict(evict_page=-1), dict(evict_page=1025),
                                 dict(evict_page=64, protected_window=200, capacity=256),
                                 dict(scale_mode="channel", fp16_window=-1),
                                 # the paged layout: pages a power of two, only whole INT8 pages evictable, ...
                                 dict(layout="paged"), dict(layout="paged", evict_page=24),
                                 dict(layout="paged", evict_page=16, fp16_window=32, protected_window=16),
                                 dict(layout="paged", evict_page=16, fp16_window=-1),
                                 dict(layout="paged", evict_page=16, protected_window=16, n_q_heads=2),
                                 dict(layout="paged", evict_page=16, protected_window=16, rank_scope="layer"),
                                 dict(layout="paged", evict_page=16, protected_window=16, capacity=144),
                                 dict(_layout=2)])
def test_bad_configs_are_rejected(clib, bad):
    kw = dict(bad)
    if "n_layers" in kw:
        kw.update(n_tight=[], n_loose=[])
    raw = {k[1:]: kw.pop(k) for k in list(kw) if k.startswith("_")}    # enum fields set past the binding's names
    cfg, *_ = _cfg(**kw)
    for k, v in raw.items():
        setattr(cfg, k, v)
    assert clib.conf_kv_state_bytes(C.byref(cfg)) == 0
    h = C.c_void_p()
    assert clib.conf_kv_create(C.byref(h), C.byref(cfg), 256, 512) == pkg.binding.ERR_BAD_SHAPE
    assert not h.value


def test_null_and_misaligned_arguments(clib):
    cfg, *_ = _cfg()
    h = C.c_void_p()
    E = pkg.binding.ERR_INVALID_ARG
    assert clib.conf_kv_create(None, C.byref(cfg), 256, 512) == E
    assert clib.conf_kv_create(C.byref(h), C.byref(cfg), None, 512) == E
    assert clib.conf_kv_create(C.byref(h), C.byref(cfg), 257, 512) == E
    assert clib.conf_kv_destroy(None) == E
    assert clib.conf_kv_attend(None, 0, 16, 16, 16, 16, None) == E
    assert clib.conf_kv_step(None, 16, None, None, None) == E
    assert clib.conf_kv_evict_compact(None, None) == E
    assert clib.conf_kv_lengths(None, None, None) == E
    assert clib.conf_kv_last_hip_error(None) == 0
    # the bandwidth probe validates its arguments before anything is launched
    bad = pkg.binding.ERR_INVALID_ARG
    assert clib.conf_kv_probe_read(None, 1024, 256, 4, None) == bad
    assert clib.conf_kv_probe_read(256, 1000, 256, 4, None) == bad       # not a multiple of 16
    assert clib.conf_kv_probe_read(264, 1024, 256, 4, None) == bad       # misaligned source
    assert clib.conf_kv_probe_read(256, 1024, 256, 0, None) == bad
    for s in range(-7, 1):
        assert pkg.strerror(s) and pkg.strerror(s) != "unknown status"
    assert pkg.strerror(-99) == "unknown status"


def test_no_cpu_fallback():
    import torch
    if torch.cuda.is_available():
        pytest.skip("GPU present")
    with pytest.raises(RuntimeError, match="needs a GPU"):
        pkg.ConfKV(n_layers=1, batch=1, n_q_heads=1, n_kv_heads=1, head_dim=64, vocab=10, capacity=64,
                   fp16_window=-1, protected_window=2, n_tight=[8], n_loose=[16])


def test_pyramid_budgets_match_the_oracle(clib):
    """Host arithmetic, no GPU: the library's pyramidal schedule against the oracle's formula."""
    from oracle import confkv_oracle as O
    for n0, L, beta, n_min in [(256, 12, 0.5, 96), (128, 12, 0.5, 96), (4096, 64, 0.5, 96),
                               (2048, 32, 0.5, 96), (1000, 7, 0.3, 10), (512, 1, 0.5, 96), (100, 4, 1.0, 96)]:
        assert pkg.pyramid_budgets(n0, L, beta, n_min) == O.pyramid_geometric(n0, L, beta, n_min)
    out = (C.c_int32 * 4)()
    for bad in [(0, 4, 0.5, 96), (64, 0, 0.5, 96), (64, 4, 0.0, 96), (64, 4, 1.5, 96), (64, 4, 0.5, 0)]:
        assert clib.conf_kv_pyramid_budgets(*bad, out) == pkg.binding.ERR_INVALID_ARG
    assert clib.conf_kv_pyramid_budgets(64, 4, 0.5, 96, None) == pkg.binding.ERR_INVALID_ARG
