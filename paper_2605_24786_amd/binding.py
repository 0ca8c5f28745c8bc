"""ctypes binding of libconfkv.so: argument marshalling only.

Every step of the decode path runs inside the HIP library; this module passes device
pointers of torch tensors and the current HIP stream through the C ABI declared in
include/conf_kv.h and owns the two device buffers the library asks the caller for.
There is no CPU fallback: importing works without a GPU (so the ABI can be inspected),
creating a ``ConfKV`` does not.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libconfkv.so")

OK = 0
ERR_INVALID_ARG, ERR_BAD_SHAPE, ERR_BAD_LAYER, ERR_CAPACITY, ERR_BAD_STATE, ERR_HIP, ERR_DEVICE = (
    -1, -2, -3, -4, -5, -6, -7)


class ConfKVConfig(C.Structure):
    _fields_ = [
        ("n_layers", C.c_int32), ("batch", C.c_int32), ("n_q_heads", C.c_int32),
        ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("vocab", C.c_int32),
        ("capacity", C.c_int32), ("fp16_window", C.c_int32), ("protected_window", C.c_int32),
        ("tau", C.c_float), ("alpha", C.c_float), ("ema_decay", C.c_float), ("sm_scale", C.c_float),
        ("w_entropy", C.c_float), ("w_margin", C.c_float), ("w_top", C.c_float),
        ("n_tight", C.POINTER(C.c_int32)), ("n_loose", C.POINTER(C.c_int32)),
        ("mass_gain", C.c_float), ("ranker", C.c_int32), ("rank_scope", C.c_int32),
        ("ranker_seed", C.c_uint64), ("scale_mode", C.c_int32), ("max_chunk", C.c_int32),
        ("evict_page", C.c_int32), ("layout", C.c_int32),
    ]


RANKERS = {"composite": 0, "random": 1}
RANK_SCOPES = {"kv_head": 0, "layer": 1}
SCALE_MODES = {"token": 0, "channel": 1}
LAYOUTS = {"contiguous": 0, "paged": 1}


class ConfKVStats(C.Structure):
    _fields_ = [("evicted", C.c_uint64), ("demoted", C.c_uint64), ("tight_steps", C.c_uint64),
                ("loose_steps", C.c_uint64), ("device_errors", C.c_uint64), ("compact_bytes", C.c_uint64)]


class ConfKVError(RuntimeError):
    def __init__(self, status: int, what: str):
        super().__init__(f"{what}: {strerror(status)} (status {status})")
        self.status = status


# every symbol include/conf_kv.h declares: name -> (restype, argtypes)
_P = C.c_void_p
SYMBOLS = {
    "conf_kv_state_bytes": (C.c_size_t, [C.POINTER(ConfKVConfig)]),
    "conf_kv_scratch_bytes": (C.c_size_t, [C.POINTER(ConfKVConfig)]),
    "conf_kv_create": (C.c_int, [C.POINTER(_P), C.POINTER(ConfKVConfig), _P, _P]),
    "conf_kv_destroy": (C.c_int, [_P]),
    "conf_kv_load_prefill": (C.c_int, [_P, C.c_int32, _P, _P, C.c_int32, _P, _P]),
    "conf_kv_attend": (C.c_int, [_P, C.c_int32, _P, _P, _P, _P, _P]),
    "conf_kv_attend_chunk": (C.c_int, [_P, C.c_int32, C.c_int32, _P, _P, _P, _P, _P]),
    "conf_kv_observe": (C.c_int, [_P, C.c_int32, C.c_int32, C.c_int32, _P, _P, _P]),
    "conf_kv_observe_prompt": (C.c_int, [_P, C.c_int32, _P, _P]),
    "conf_kv_step": (C.c_int, [_P, _P, _P, _P, _P]),
    "conf_kv_step_static": (C.c_int, [_P, _P, _P, _P, _P]),
    "conf_kv_evict_compact": (C.c_int, [_P, _P]),
    "conf_kv_static_plan": (C.c_int, [_P, C.c_int32]),
    "conf_kv_tag_state": (C.c_int, [_P, _P, _P, _P]),
    "conf_kv_lengths": (C.c_int, [_P, _P, _P]),
    "conf_kv_export": (C.c_int, [_P, C.c_int32, C.c_int32, C.c_int32] + [_P] * 10),
    "conf_kv_pyramid_budgets": (C.c_int, [C.c_int32, C.c_int32, C.c_double, C.c_int32, _P]),
    "conf_kv_import": (C.c_int, [_P, C.c_int32, C.c_int32, C.c_int32, C.c_int32] + [_P] * 9),
    "conf_kv_counters": (C.c_int, [_P, C.POINTER(ConfKVStats)]),
    "conf_kv_attend_splits": (C.c_int, [_P, C.c_int32]),
    "conf_kv_strerror": (C.c_char_p, [C.c_int]),
    "conf_kv_last_hip_error": (C.c_int, [_P]),
    "conf_kv_probe_read": (C.c_int, [_P, C.c_size_t, _P, C.c_int32, _P]),
}

_lib = None


def stale_sources() -> list:
    """Sources of the library that were modified after libconfkv.so was built (empty: up to date)."""
    if not os.path.exists(LIB_PATH):
        return []
    built = os.path.getmtime(LIB_PATH)
    dirs = [os.path.join(_HERE, "csrc"), os.path.join(os.path.dirname(_HERE), "include")]
    out = []
    for d in dirs:
        for name in sorted(os.listdir(d)) if os.path.isdir(d) else []:
            if name.endswith((".hip", ".h")) and os.path.getmtime(os.path.join(d, name)) > built:
                out.append(name)
    return out


def load_library() -> C.CDLL:
    """Loads libconfkv.so, building it first if it has never been built.  A library older than
    its sources is rebuilt when CONF_KV_REBUILD=1 and otherwise loaded with a loud warning (the
    GPU machines run what was built beforehand; they do not compile)."""
    global _lib
    if _lib is None:
        stale = stale_sources()
        if not os.path.exists(LIB_PATH) or (stale and os.environ.get("CONF_KV_REBUILD") == "1"):
            from . import build as _build
            _build.build()
        elif stale:
            import warnings
            warnings.warn(f"libconfkv.so is older than {', '.join(stale)}: the loaded library does not contain "
                          f"those edits (run `python -m paper_2605_24786_amd.build`, or set CONF_KV_REBUILD=1)",
                          RuntimeWarning, stacklevel=2)
        lib = C.CDLL(LIB_PATH)
        for name, (res, args) in SYMBOLS.items():
            fn = getattr(lib, name)
            fn.restype = res
            fn.argtypes = args
        _lib = lib
    return _lib


def strerror(status: int) -> str:
    return load_library().conf_kv_strerror(status).decode()


def make_config(n_layers, batch, n_q_heads, n_kv_heads, head_dim, vocab, capacity, fp16_window,
                protected_window, n_tight: Sequence[int], n_loose: Sequence[int], tau=0.7, alpha=0.65,
                ema_decay=0.9, sm_scale=None, w_entropy=0.4, w_margin=0.3, w_top=0.3, mass_gain=None,
                ranker="composite", rank_scope="kv_head", ranker_seed=0, scale_mode="token", max_chunk=0,
                evict_page=0, layout="contiguous"):
    """A ConfKVConfig plus the two int32 arrays it points to (keep the tuple alive)."""
    nt = (C.c_int32 * len(n_tight))(*[int(x) for x in n_tight])
    nl = (C.c_int32 * len(n_loose))(*[int(x) for x in n_loose])
    if sm_scale is None:
        sm_scale = 1.0 / float(np.sqrt(head_dim))
    cfg = ConfKVConfig(n_layers, batch, n_q_heads, n_kv_heads, head_dim, vocab, capacity,
                       fp16_window, protected_window, tau, alpha, ema_decay, sm_scale,
                       w_entropy, w_margin, w_top, nt, nl,
                       -1.0 if mass_gain is None else float(mass_gain), RANKERS[ranker],
                       RANK_SCOPES[rank_scope], int(ranker_seed), SCALE_MODES[scale_mode], int(max_chunk),
                       int(evict_page), LAYOUTS[layout])
    return cfg, nt, nl


def pyramid_budgets(n0: int, n_layers: int, beta: float = 0.5, n_min: int = 96):
    """Per-layer budgets of the pyramidal extension (host arithmetic in the library)."""
    out = (C.c_int32 * n_layers)()
    rc = load_library().conf_kv_pyramid_budgets(n0, n_layers, beta, n_min, out)
    if rc != OK:
        raise ConfKVError(rc, "conf_kv_pyramid_budgets")
    return list(out)


def probe_read(src, out, workgroups: int, stream=None) -> None:
    """One read-only pass over the torch tensor `src` (see conf_kv_probe_read); `out` is a zeroed
    uint32/int32 tensor of `workgroups` elements."""
    import torch
    st = torch.cuda.current_stream().cuda_stream if stream is None else stream
    rc = load_library().conf_kv_probe_read(src.data_ptr(), src.numel() * src.element_size(), out.data_ptr(),
                                           workgroups, st)
    if rc != OK:
        raise ConfKVError(rc, "conf_kv_probe_read")


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


class ConfKV:
    """One cache manager instance on the current CUDA/HIP device (torch owns the memory)."""

    def __init__(self, **kw):
        import torch
        if not torch.cuda.is_available():
            raise RuntimeError("ConfKV needs a GPU: the decode path has no CPU implementation")
        self._torch = torch
        self.lib = load_library()
        self.cfg, self._nt, self._nl = make_config(**kw)
        sb = self.lib.conf_kv_state_bytes(C.byref(self.cfg))
        kb = self.lib.conf_kv_scratch_bytes(C.byref(self.cfg))
        if sb == 0:
            raise ConfKVError(ERR_BAD_SHAPE, "conf_kv_state_bytes")
        self.state = torch.empty(sb, dtype=torch.uint8, device="cuda")
        self.scratch = torch.empty(kb, dtype=torch.uint8, device="cuda")
        h = _P()
        self._check(self.lib.conf_kv_create(C.byref(h), C.byref(self.cfg), self.state.data_ptr(),
                                            self.scratch.data_ptr()), "conf_kv_create")
        self.h = h

    # -- plumbing --
    def _check(self, status: int, what: str) -> int:
        if status < 0:
            raise ConfKVError(status, what)
        return status

    def _stream(self):
        return self._torch.cuda.current_stream().cuda_stream

    def close(self):
        if getattr(self, "h", None):
            self.lib.conf_kv_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- the C ABI, same names --
    def load_prefill(self, layer: int, k16, v16, ema0=None):
        T0 = int(k16.shape[2])
        return self._check(self.lib.conf_kv_load_prefill(self.h, layer, _ptr(k16), _ptr(v16), T0,
                                                         _ptr(ema0), self._stream()), "conf_kv_load_prefill")

    def attend(self, layer: int, q16, knew16, vnew16, out16):
        return self._check(self.lib.conf_kv_attend(self.h, layer, _ptr(q16), _ptr(knew16), _ptr(vnew16),
                                                   _ptr(out16), self._stream()), "conf_kv_attend")

    def attend_chunk(self, layer: int, q16, knew16, vnew16, out16):
        """q16 / out16 [B][tq][Hq][D], knew16 / vnew16 [B][tq][Hkv][D]; tq = q16.shape[1]."""
        tq = int(q16.shape[1])
        return self._check(self.lib.conf_kv_attend_chunk(self.h, layer, tq, _ptr(q16), _ptr(knew16), _ptr(vnew16),
                                                         _ptr(out16), self._stream()), "conf_kv_attend_chunk")

    def observe(self, layer: int, first: int, q16, out16=None):
        """q16 / out16 [B][tq][Hq][D]: queries of the cached slots first .. first + tq - 1; out16 optional."""
        tq = int(q16.shape[1])
        return self._check(self.lib.conf_kv_observe(self.h, layer, first, tq, _ptr(q16), _ptr(out16),
                                                    self._stream()), "conf_kv_observe")

    def observe_prompt(self, layer: int, q16):
        """q16 [B][T0][Hq][D]: the queries of every prompt token of the layer's freshly loaded cache."""
        return self._check(self.lib.conf_kv_observe_prompt(self.h, layer, _ptr(q16), self._stream()),
                           "conf_kv_observe_prompt")

    def step(self, logits, conf=None, sel=None):
        return self._check(self.lib.conf_kv_step(self.h, _ptr(logits), _ptr(conf), _ptr(sel),
                                                 self._stream()), "conf_kv_step")

    def static_plan(self, on: bool = True):
        """Launch shapes from the budgets instead of the lengths so far: call before recording a step into a graph."""
        return self._check(self.lib.conf_kv_static_plan(self.h, int(bool(on))), "conf_kv_static_plan")

    def tag_state(self):
        """(attention tag base, confidence tag base, clearing pending) from the device; synchronises."""
        a, c, p = C.c_uint32(0), C.c_uint32(0), C.c_int32(0)
        self._check(self.lib.conf_kv_tag_state(self.h, C.byref(a), C.byref(c), C.byref(p)), "conf_kv_tag_state")
        return a.value, c.value, p.value

    def step_static(self, logits, conf=None, sel=None):
        return self._check(self.lib.conf_kv_step_static(self.h, _ptr(logits), _ptr(conf), _ptr(sel),
                                                        self._stream()), "conf_kv_step_static")

    def evict_compact(self):
        return self._check(self.lib.conf_kv_evict_compact(self.h, self._stream()), "conf_kv_evict_compact")

    def lengths(self):
        c = self.cfg
        ln = np.zeros((c.n_layers, c.batch), dtype=np.int32)
        n16 = np.zeros((c.n_layers, c.batch, c.n_kv_heads), dtype=np.int32)
        self._check(self.lib.conf_kv_lengths(self.h, ln.ctypes.data, n16.ctypes.data), "conf_kv_lengths")
        return ln, n16

    def export(self, layer: int, b: int, kv_head: int, planes=None):
        """Position-sorted view of one unit.  `planes` limits the copy to some of "pos", "ema",
        "is16", "k16", "v16", "k8", "v8", "ks", "vs" (the others get NULL pointers and are absent
        from the result); None fetches everything."""
        c = self.cfg
        cap, D = c.capacity, c.head_dim
        chan = c.scale_mode == SCALE_MODES["channel"]       # then ks / vs are the channel scales [D]
        want = (lambda name: planes is None or name in planes)
        shapes = dict(pos=(cap, np.int32), ema=(cap, np.float32), is16=(cap, np.uint8), k16=((cap, D), np.uint16),
                      v16=((cap, D), np.uint16), k8=((cap, D), np.int8), v8=((cap, D), np.int8),
                      ks=(max(cap, D), np.uint16), vs=(max(cap, D), np.uint16))
        buf = {name: np.zeros(shape, dt) for name, (shape, dt) in shapes.items() if want(name)}
        ptr = lambda name: buf[name].ctypes.data if name in buf else None
        n = C.c_int32(0)
        self._check(self.lib.conf_kv_export(self.h, layer, b, kv_head, ptr("pos"), ptr("ema"), ptr("is16"),
                                            ptr("k16"), ptr("v16"), ptr("k8"), ptr("v8"), ptr("ks"), ptr("vs"),
                                            C.addressof(n)), "conf_kv_export")
        m = n.value
        out = dict(n=m)
        for name, x in buf.items():
            if name in ("ks", "vs"):
                out[name] = x[:D if chan else m].view(np.float16)
            elif name in ("k16", "v16"):
                out[name] = x[:m].view(np.float16)
            elif name == "is16":
                out[name] = x[:m].astype(bool)
            else:
                out[name] = x[:m]
        return out

    def import_unit(self, layer: int, b: int, kv_head: int, view: dict):
        """`view` is what export() returns (n, pos, ema, is16, k16, v16, k8, v8, ks, vs)."""
        n = int(view["n"])
        keep = [np.ascontiguousarray(view["pos"], np.int32), np.ascontiguousarray(view["ema"], np.float32),
                np.ascontiguousarray(view["is16"], np.uint8)]
        for name, dt in (("k16", np.uint16), ("v16", np.uint16), ("k8", np.int8), ("v8", np.int8),
                         ("ks", np.uint16), ("vs", np.uint16)):
            x = view.get(name)
            if x is None:
                keep.append(None)
            else:
                x = np.ascontiguousarray(x)
                keep.append(x.view(dt) if x.dtype != dt else x)
        ptrs = [None if x is None else x.ctypes.data for x in keep]
        self._check(self.lib.conf_kv_import(self.h, layer, b, kv_head, n, *ptrs), "conf_kv_import")

    def counters(self, check: bool = True) -> ConfKVStats:
        st = ConfKVStats()
        rc = self.lib.conf_kv_counters(self.h, C.byref(st))
        if check:
            self._check(rc, "conf_kv_counters")
        return st

    def attend_splits(self, layer: int) -> int:
        return self._check(self.lib.conf_kv_attend_splits(self.h, layer), "conf_kv_attend_splits")


def from_workload(wl, **override) -> ConfKV:
    """A ConfKV shaped like a ``synth.workloads.Workload`` (duck-typed; no import of synth)."""
    kw = dict(n_layers=wl.n_layers, batch=wl.batch, n_q_heads=wl.n_q_heads, n_kv_heads=wl.n_kv_heads,
              head_dim=wl.head_dim, vocab=wl.vocab, capacity=wl.capacity, fp16_window=wl.fp16_window,
              protected_window=wl.protected, n_tight=wl.n_tight, n_loose=wl.n_loose, tau=wl.tau,
              alpha=wl.alpha, ema_decay=wl.ema_decay, w_entropy=wl.w_entropy, w_margin=wl.w_margin,
              w_top=wl.w_top, mass_gain=getattr(wl, "mass_gain", None),
              ranker=getattr(wl, "ranker", "composite"), rank_scope=getattr(wl, "rank_scope", "kv_head"),
              ranker_seed=getattr(wl, "ranker_seed", 0), scale_mode=getattr(wl, "scale_mode", "token"),
              max_chunk=getattr(wl, "max_chunk", 0), evict_page=getattr(wl, "evict_page", 0),
              layout=getattr(wl, "layout", "contiguous"))
    kw.update(override)
    return ConfKV(**kw)
