"""Writes tests/golden/oracle_regression.json: what the CPU oracle computes on a few seeded
inputs, so that an unintended change to the oracle's arithmetic shows up as a diff of this file.
Calls nothing but oracle/ and numpy.  Run from the repository root:

    python tests/golden/make_oracle_regression.py
"""
import hashlib
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
from oracle import confkv_oracle as O  # noqa: E402


def digest(a: np.ndarray) -> str:
    return hashlib.sha256(np.ascontiguousarray(a).tobytes()).hexdigest()[:16]


def compute() -> dict:
    rng = np.random.default_rng(20260524)
    out = {}
    # Eq. 1 on seeded logits of three temperatures
    w = tuple(float(np.float32(x)) for x in (0.4, 0.3, 0.3))
    out["confidence"] = [repr(float(O.confidence((rng.standard_normal(5003) * s).astype(np.float32), w)))
                         for s in (0.5, 3.0, 9.0)]
    out["pyramid"] = O.pyramid_geometric(1024, 12, 0.5, 96)
    # one unit through three decode steps: attention, EMA, eviction, demotion
    T, D, G, W, P = 90, 16, 3, 10, 6
    K = rng.standard_normal((T, D)).astype(np.float16)
    V = rng.standard_normal((T, D)).astype(np.float16)
    for mode in ("token", "channel"):
        u = O.load_prefill(K, V, W, ema0=rng.random(T).astype(np.float32), scale_mode=mode)
        gone_all, outs = [], []
        for t in range(3):
            q = rng.standard_normal((G, D)).astype(np.float16)
            kn, vn = rng.standard_normal(D).astype(np.float16), rng.standard_normal(D).astype(np.float16)
            o, _ = O.attend_unit(u, q, kn, vn, T + t, 0.25, float(np.float32(0.9)))
            outs.append(np.round(o, 12))
            gone = O.evict_compact_unit(u, 80 - 7 * t, P, float(np.float32(0.65)), W)
            gone_all.append([int(x) for x in gone])
        out[mode] = {"evicted": gone_all, "out": digest(np.stack(outs)), "ema": digest(u.ema),
                     "k8": digest(u.k8[~u.is16]), "v8": digest(u.v8[~u.is16]),
                     "scales": digest(u.ks[~u.is16] if mode == "token" else u.kcs), "n": u.n, "n16": u.n16}
    # several tokens in one call
    u = O.load_prefill(K, V, W)
    q = rng.standard_normal((4, G, D)).astype(np.float16)
    kn, vn = rng.standard_normal((4, D)).astype(np.float16), rng.standard_normal((4, D)).astype(np.float16)
    o, Wm = O.attend_chunk_unit(u, q, kn, vn, T, 0.25, float(np.float32(0.9)))
    out["chunk"] = {"out": digest(np.round(o, 12)), "mass": digest(np.round(Wm, 12)), "ema": digest(u.ema)}
    # the random ranker's draws
    out["random_scores"] = [repr(float(x)) for x in O.random_scores(12345, 7, np.arange(4))]
    # importance from an observation window at the end of the prompt (nothing appended)
    u = O.load_prefill(K, V, W)
    q = rng.standard_normal((5, G, D)).astype(np.float16)
    o, Wm = O.observe_unit(u, q, T - 5, 0.25, float(np.float32(0.9)))
    out["observe"] = {"out": digest(np.round(o, 12)), "mass": digest(np.round(Wm, 12)), "ema": digest(u.ema)}
    # coarsened eviction: whole pages of 8 original positions, twice (the second on gapped positions)
    u = O.load_prefill(K, V, W, ema0=rng.random(T).astype(np.float32))
    gone = [[int(x) for x in O.evict_compact_unit(u, N, P, float(np.float32(0.65)), W, page=8)] for N in (70, 41)]
    out["pages"] = {"evicted": gone, "n": u.n, "ema": digest(u.ema)}
    return out


if __name__ == "__main__":
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "oracle_regression.json")
    with open(path, "w") as f:
        json.dump(compute(), f, indent=1, sort_keys=True)
        f.write("\n")
    print("wrote", path)
