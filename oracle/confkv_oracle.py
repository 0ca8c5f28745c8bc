"""CPU oracle for the Conf-KV per-decode-step path.  TEST INFRASTRUCTURE ONLY.

A plain, slow, float64 numpy statement of what one decode step of the
confidence-aware KV-cache manager computes, written from the paper's Method
section (Eq. 1, the budget and ranker paragraph, Algorithm 1, the tiled
attention / mixed-precision paragraph and the pyramidal-budget formula).
It shares no code, tables or helpers with the HIP library and imports nothing
from it.  Only tests, the smoke check and the benchmark's CPU-baseline leg may
import this module; the product path never does.

Precision: every floating-point step is float64 over the *stored* inputs
(fp16 K/V/Q values, int8 codes with fp16 scales, fp32 logits and fp32 EMA
metadata are all exactly representable in float64).  Two storage formats round:
the EMA metadata is kept as fp32 (computed in float64, rounded on store), and
the INT8 quantiser's scale is fl16(fl32(amax / 127)) -- both are state formats
of the cache, not arithmetic shortcuts.

Readings of the paper taken here (each is listed again where it is used):
  * one importance value and one kept set per (layer, kv-head); the attention
    mass of a token is the SUM over the query heads that share the kv-head
    (the literal per-layer reading is the ``rank_scope = "layer"`` variant);
  * INT8 scales are per token and per kv-head (absmax over the channels); the
    paper's literal "per head and channel" wording is the ``scale_mode =
    "channel"`` variant: one scale per (kv-head, channel), fixed from the prompt;
  * the new token is appended before its own attention and counts toward the
    cache length and the protected window;
  * the FP16 window holds the W newest *retained* tokens; nothing is promoted.

Every public function names the passage it follows.  Pinned by tests/test_oracle_*.py.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

F64 = np.float64


# --------------------------------------------------------------------------------------
# Confidence estimator and budget selector  (Method, Eq. 1; "Budget and ranker")
# --------------------------------------------------------------------------------------

def softmax64(x: np.ndarray) -> np.ndarray:
    """Plain max-subtracted softmax of a 1-D array, float64."""
    x = np.asarray(x, dtype=F64)
    e = np.exp(x - np.max(x))
    return e / np.sum(e)


def confidence_terms(logits: np.ndarray) -> Tuple[float, float, float]:
    """(normalised entropy, log-prob margin, top probability) of one logit row.

    Eq. 1's ingredients: H_hat = H(p) / log V with p = softmax(logits) and
    0 log 0 = 0; m = log p_(1) - log p_(2) with the two largest probabilities
    counted with multiplicity; p_(1).
    """
    p = softmax64(logits)
    V = p.shape[0]
    nz = p > 0.0
    H = -np.sum(p[nz] * np.log(p[nz]))
    H_hat = H / np.log(F64(V))
    top2 = np.sort(p)[-2:]            # ascending: [p_(2), p_(1)]
    p1, p2 = top2[1], top2[0]
    with np.errstate(divide="ignore"):
        m = np.log(p1) - np.log(p2)   # +inf when p_(2) underflows to 0
    return float(H_hat), float(m), float(p1)


def confidence(logits: np.ndarray, w: Sequence[float] = (0.4, 0.3, 0.3)) -> float:
    """Eq. 1: c = w_H (1 - H_hat) + w_m sigmoid(m) + w_p p_(1)."""
    H_hat, m, p1 = confidence_terms(logits)
    sig = 1.0 / (1.0 + np.exp(-F64(m)))
    return float(F64(w[0]) * (1.0 - H_hat) + F64(w[1]) * sig + F64(w[2]) * p1)


def select_budget(c: float, tau: float, n_tight: int, n_loose: int) -> Tuple[bool, int]:
    """Budget rule: N = N_high (tight) if c >= tau else N_low (loose); N_high <= N_low."""
    if n_tight > n_loose:
        raise ValueError("N_high must not exceed N_low")
    tight = bool(F64(c) >= F64(tau))
    return tight, (n_tight if tight else n_loose)


def pyramid_geometric(n0: int, n_layers: int, beta: float = 0.5, n_min: int = 96) -> List[int]:
    """Pyramidal layer budgets: N(l) = max(N_min, N(0) * beta**(l / L)), floored to an integer."""
    return [max(n_min, int(np.floor(F64(n0) * F64(beta) ** (F64(l) / F64(n_layers)))))
            for l in range(n_layers)]


# --------------------------------------------------------------------------------------
# INT8 quantiser  ("Tiled attention and mixed precision": symmetric, s = max|x| / 127)
# --------------------------------------------------------------------------------------

def quantize_vector(x16: np.ndarray) -> Tuple[np.ndarray, np.float16]:
    """Symmetric INT8 codes and fp16 scale of one fp16 vector (one token, one kv-head).

    scale = fl16(fl32(max|x| / 127)); code_d = clamp(round_half_even(x_d / scale), -127, 127)
    with the division taken with the rounded scale.  A zero vector, or one whose
    scale rounds to zero, gets scale 0 and all-zero codes.
    """
    x16 = np.asarray(x16, dtype=np.float16)
    amax = np.max(np.abs(x16)) if x16.size else np.float16(0)
    s32 = np.float32(amax) / np.float32(127.0)
    scale = np.float16(s32)
    if not np.isfinite(scale) or scale == 0:
        return np.zeros(x16.shape, dtype=np.int8), np.float16(0)
    r = np.rint(x16.astype(F64) / F64(scale))
    return np.clip(r, -127, 127).astype(np.int8), scale


def dequantize(codes: np.ndarray, scale) -> np.ndarray:
    """Stored value of INT8 tokens: code * scale, float64.  codes [.., D], scale [..]."""
    return codes.astype(F64) * np.asarray(scale, dtype=F64)[..., None]


def channel_scales(x16: np.ndarray) -> np.ndarray:
    """One fp16 scale per channel of a kv-head from a set of tokens x16 [T, D].

    The paper's literal granularity ("per head and channel", s = max|x| / 127) leaves open
    which tokens the maximum runs over; here it runs over the tokens given (the prompt) and
    the scales stay fixed afterwards.  scale_d = fl16(fl32(max_t |x_{t,d}| / 127)); a
    channel whose scale is zero or not finite gets scale 0 (its codes are all zero).
    """
    x16 = np.asarray(x16, dtype=np.float16)
    D = x16.shape[1]
    amax = np.max(np.abs(x16), axis=0) if x16.shape[0] else np.zeros(D, np.float16)
    s = (amax.astype(np.float32) / np.float32(127.0)).astype(np.float16)
    s[~np.isfinite(s)] = 0
    return s


def quantize_channels(x16: np.ndarray, scales: np.ndarray) -> np.ndarray:
    """INT8 codes of one fp16 vector against fixed per-channel scales.

    code_d = clamp(round_half_even(x_d / scale_d), -127, 127); a value beyond the range the
    scales were fixed on saturates.  Channels with scale 0 get code 0.
    """
    x = np.asarray(x16, dtype=np.float16).astype(F64)
    s = np.asarray(scales, dtype=np.float16).astype(F64)
    live = s > 0
    r = np.zeros(x.shape, dtype=F64)
    r[live] = np.rint(x[live] / s[live])
    return np.clip(r, -127, 127).astype(np.int8)


def dequantize_channels(codes: np.ndarray, scales: np.ndarray) -> np.ndarray:
    """Stored value under per-channel scales: code_{t,d} * scale_d, float64."""
    return codes.astype(F64) * np.asarray(scales, dtype=np.float16).astype(F64)[None, :]


# --------------------------------------------------------------------------------------
# Attention over a stored cache  ("Tiled attention and mixed precision")
# --------------------------------------------------------------------------------------

def attention_naive(q: np.ndarray, k: np.ndarray, v: np.ndarray, sm_scale: float
                    ) -> Tuple[np.ndarray, np.ndarray]:
    """Plain softmax attention of G query heads over n cached tokens.

    q [G, D], k [n, D], v [n, D] float64 -> (out [G, D], p [G, n]).  No mask: a
    decode query sees every retained slot and itself.
    """
    s = F64(sm_scale) * (q @ k.T)
    s = s - np.max(s, axis=1, keepdims=True)
    e = np.exp(s)
    p = e / np.sum(e, axis=1, keepdims=True)
    return p @ v, p


def attention_blockwise(q: np.ndarray, k: np.ndarray, v: np.ndarray, sm_scale: float,
                        block: int = 128) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """The same attention read in blocks with a running max and normaliser.

    Returns (out [G, D], m [G], l [G]) with out = o / l; m and l are the final
    running max and normaliser, from which the exact probabilities follow as
    exp(s - m) / l.
    """
    G, D = q.shape
    n = k.shape[0]
    m = np.full(G, -np.inf)
    l = np.zeros(G)
    o = np.zeros((G, D))
    for lo in range(0, n, block):
        kb, vb = k[lo:lo + block], v[lo:lo + block]
        s = F64(sm_scale) * (q @ kb.T)                        # [G, b]
        m_new = np.maximum(m, np.max(s, axis=1))
        corr = np.exp(m - m_new)
        e = np.exp(s - m_new[:, None])
        l = l * corr + np.sum(e, axis=1)
        o = o * corr[:, None] + e @ vb
        m = m_new
    return o / l[:, None], m, l


def merge_partials(ms: np.ndarray, ls: np.ndarray, os_: np.ndarray
                   ) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Combine split partials (m_j, l_j, o_j un-normalised) of disjoint token ranges.

    ms, ls [J, G]; os_ [J, G, D].  M = max_j m_j, L = sum_j l_j e^{m_j - M},
    out = sum_j o_j e^{m_j - M} / L.
    """
    M = np.max(ms, axis=0)
    wgt = np.exp(ms - M[None, :])
    L = np.sum(ls * wgt, axis=0)
    out = np.sum(os_ * wgt[:, :, None], axis=0) / L[:, None]
    return out, M, L


# --------------------------------------------------------------------------------------
# Per-unit cache state  ("Cache manager": K/V storage, valid length, position, EMA mass)
# --------------------------------------------------------------------------------------

@dataclass
class UnitCache:
    """The cache of one (layer, batch, kv-head), slots in increasing original position.

    A slot is either FP16 (k16/v16 rows valid) or INT8 (k8/v8 codes with ks/vs scales).
    INT8 slots always precede FP16 slots because demotion takes the oldest FP16 token.
    With per-channel scales (``kcs``/``vcs`` [D] set) the per-token ks/vs are unused.
    """
    head_dim: int
    pos: np.ndarray = field(default_factory=lambda: np.zeros(0, dtype=np.int64))
    ema: np.ndarray = field(default_factory=lambda: np.zeros(0, dtype=np.float32))
    is16: np.ndarray = field(default_factory=lambda: np.zeros(0, dtype=bool))
    k16: np.ndarray = None
    v16: np.ndarray = None
    k8: np.ndarray = None
    v8: np.ndarray = None
    ks: np.ndarray = field(default_factory=lambda: np.zeros(0, dtype=np.float16))
    vs: np.ndarray = field(default_factory=lambda: np.zeros(0, dtype=np.float16))
    kcs: Optional[np.ndarray] = None      # per-channel K scales [D] fp16, or None: per-token scales
    vcs: Optional[np.ndarray] = None

    def __post_init__(self):
        D = self.head_dim
        if self.k16 is None:
            self.k16 = np.zeros((0, D), dtype=np.float16)
            self.v16 = np.zeros((0, D), dtype=np.float16)
            self.k8 = np.zeros((0, D), dtype=np.int8)
            self.v8 = np.zeros((0, D), dtype=np.int8)

    @property
    def n(self) -> int:
        return int(self.pos.shape[0])

    @property
    def n16(self) -> int:
        return int(np.count_nonzero(self.is16))

    def stored_k(self) -> np.ndarray:
        """Stored key values, float64 [n, D]: the fp16 value, or code * scale."""
        k8 = dequantize(self.k8, self.ks) if self.kcs is None else dequantize_channels(self.k8, self.kcs)
        return np.where(self.is16[:, None], self.k16.astype(F64), k8)

    def stored_v(self) -> np.ndarray:
        v8 = dequantize(self.v8, self.vs) if self.vcs is None else dequantize_channels(self.v8, self.vcs)
        return np.where(self.is16[:, None], self.v16.astype(F64), v8)

    def take(self, keep: np.ndarray) -> None:
        """Gather the slots ``keep`` (increasing) into contiguous storage: the compaction."""
        for name in ("pos", "ema", "is16", "k16", "v16", "k8", "v8", "ks", "vs"):
            setattr(self, name, getattr(self, name)[keep])

    def copy(self) -> "UnitCache":
        c = UnitCache(self.head_dim)
        for name in ("pos", "ema", "is16", "k16", "v16", "k8", "v8", "ks", "vs"):
            setattr(c, name, getattr(self, name).copy())
        c.kcs = None if self.kcs is None else self.kcs.copy()
        c.vcs = None if self.vcs is None else self.vcs.copy()
        return c


def load_prefill(k16: np.ndarray, v16: np.ndarray, fp16_window: int,
                 ema0: Optional[np.ndarray] = None, scale_mode: str = "token") -> UnitCache:
    """A unit holding T0 prefill tokens at positions 0..T0-1, EMA = ema0 or 0, then demoted.

    ``scale_mode = "channel"`` fixes the unit's per-channel scales on all T0 prompt tokens
    (those that stay FP16 included) before the demotion.
    """
    T, D = k16.shape
    u = UnitCache(D)
    if scale_mode == "channel":
        u.kcs = channel_scales(k16)
        u.vcs = channel_scales(v16)
    elif scale_mode != "token":
        raise ValueError(scale_mode)
    u.pos = np.arange(T, dtype=np.int64)
    u.ema = np.zeros(T, dtype=np.float32) if ema0 is None else np.asarray(ema0, np.float32).copy()
    u.is16 = np.ones(T, dtype=bool)
    u.k16 = np.asarray(k16, np.float16).copy()
    u.v16 = np.asarray(v16, np.float16).copy()
    u.k8 = np.zeros((T, D), dtype=np.int8)
    u.v8 = np.zeros((T, D), dtype=np.int8)
    u.ks = np.zeros(T, dtype=np.float16)
    u.vs = np.zeros(T, dtype=np.float16)
    demote(u, fp16_window)
    return u


def append_token(u: UnitCache, k_new: np.ndarray, v_new: np.ndarray, pos_new: int) -> None:
    """Algorithm 1's append: the new token enters in FP16 with EMA 0 at the next slot."""
    D = u.head_dim
    if u.n and pos_new <= int(u.pos[-1]):
        raise ValueError("positions must increase")
    u.pos = np.append(u.pos, np.int64(pos_new))
    u.ema = np.append(u.ema, np.float32(0))
    u.is16 = np.append(u.is16, True)
    u.k16 = np.vstack([u.k16, np.asarray(k_new, np.float16).reshape(1, D)])
    u.v16 = np.vstack([u.v16, np.asarray(v_new, np.float16).reshape(1, D)])
    u.k8 = np.vstack([u.k8, np.zeros((1, D), np.int8)])
    u.v8 = np.vstack([u.v8, np.zeros((1, D), np.int8)])
    u.ks = np.append(u.ks, np.float16(0))
    u.vs = np.append(u.vs, np.float16(0))


def attend_unit(u: UnitCache, q: np.ndarray, k_new: np.ndarray, v_new: np.ndarray, pos_new: int,
                sm_scale: float, ema_decay: float, mass_gain: Optional[float] = None
                ) -> Tuple[np.ndarray, np.ndarray]:
    """One decode step's attention for one unit, with the EMA importance update.

    Appends the new token, attends the G query heads q [G, D] (fp16 values) over all
    stored slots, forms the per-token mass A_i = sum over the G heads of p_{h,i}
    (so sum_i A_i = G), and updates a_i <- lambda a_i + (1 - lambda) A_i for every
    slot including the new one ("Budget and ranker"; Algorithm 1, EMA line).
    ``mass_gain`` replaces the factor (1 - lambda); (lambda, gain) = (1, 1) is the plain
    running sum of the mass that the cumulative-attention baselines of the experimental
    setup rank by.
    Returns (out [G, D] float64, A [n] float64).
    """
    append_token(u, k_new, v_new, pos_new)
    out, p = attention_naive(np.asarray(q).astype(F64), u.stored_k(), u.stored_v(), sm_scale)
    A = np.sum(p, axis=0)
    lam = F64(ema_decay)
    gain = (1.0 - lam) if mass_gain is None else F64(mass_gain)
    u.ema = (lam * u.ema.astype(F64) + gain * A).astype(np.float32)
    return out, A


def attend_chunk_unit(u: UnitCache, q: np.ndarray, k_new: np.ndarray, v_new: np.ndarray, pos0: int,
                      sm_scale: float, ema_decay: float, mass_gain: Optional[float] = None
                      ) -> Tuple[np.ndarray, np.ndarray]:
    """Tq consecutive tokens of one sequence in one call (a chunk of a prompt, or several
    decode tokens that are all kept): q [Tq, G, D], k_new / v_new [Tq, D], positions
    pos0 .. pos0 + Tq - 1.  Defined as what Tq single-token steps without eviction in
    between compute: query t attends the cache and the chunk's tokens 0 .. t (causal), and
    the importance follows a <- lambda a + gain A_t once per query, which telescopes to

        a_i <- lambda^Tq a_i + gain * sum_t lambda^(Tq-1-t) A_{t,i}

    (a token of the chunk starts at 0 and receives no mass from the queries before it).
    The stored fp32 importance is written once, at the end of the call.
    Returns (out [Tq, G, D] float64, W [n] float64 = the weighted mass sum above).
    """
    q = np.asarray(q)
    Tq = q.shape[0]
    lam = F64(ema_decay)
    gain = (1.0 - lam) if mass_gain is None else F64(mass_gain)
    n_old = u.n
    a = np.concatenate([u.ema.astype(F64), np.zeros(Tq)])
    outs = []
    for t in range(Tq):
        append_token(u, k_new[t], v_new[t], pos0 + t)
        out, p = attention_naive(q[t].astype(F64), u.stored_k(), u.stored_v(), sm_scale)
        A = np.sum(p, axis=0)                       # over the n_old + t + 1 visible slots
        a[:n_old + t + 1] = lam * a[:n_old + t + 1] + gain * A
        a[n_old + t + 1:] = 0.0                     # tokens not yet appended hold nothing
        outs.append(out)
    W = a - (lam ** Tq) * np.concatenate([u.ema[:n_old].astype(F64), np.zeros(Tq)])
    u.ema = a.astype(np.float32)
    return np.stack(outs), W


def observe_unit(u: UnitCache, q: np.ndarray, first: int, sm_scale: float, ema_decay: float,
                 mass_gain: Optional[float] = None) -> Tuple[np.ndarray, np.ndarray]:
    """Importance from queries of tokens that are ALREADY in the cache (the prompt's own
    attention, taken over an observation window at its end): q [Tq, G, D] are the queries of
    the cached slots first .. first + Tq - 1.  Nothing is appended.  Defined like
    ``attend_chunk_unit`` on the stored values: query t sees slots 0 .. first + t, the
    importance of every slot below first + Tq follows a <- lambda a + gain A_t once per query
    (a window slot counts from 0 at its own query, whatever it held before), and slots at or
    above first + Tq are neither seen nor changed.  Calling it for consecutive windows
    first = s, s + Tq, .. is the same as one call over their union.
    Returns (out [Tq, G, D] float64, W [first + Tq] float64 = the weighted mass received).
    """
    q = np.asarray(q)
    Tq = q.shape[0]
    if first < 0 or first + Tq > u.n:
        raise ValueError("window outside the cache")
    lam = F64(ema_decay)
    gain = (1.0 - lam) if mass_gain is None else F64(mass_gain)
    K, V = u.stored_k(), u.stored_v()
    a = u.ema.astype(F64).copy()
    a[first:first + Tq] = 0.0
    base = a.copy()
    outs = []
    for t in range(Tq):
        vis = first + t + 1
        out, p = attention_naive(q[t].astype(F64), K[:vis], V[:vis], sm_scale)
        a[:vis] = lam * a[:vis] + gain * np.sum(p, axis=0)
        outs.append(out)
    n_eff = first + Tq
    W = a[:n_eff] - (lam ** Tq) * base[:n_eff]
    new = u.ema.astype(F64)
    new[:n_eff] = a[:n_eff]
    u.ema = new.astype(np.float32)
    return np.stack(outs), W


# --------------------------------------------------------------------------------------
# Ranking, eviction, compaction, demotion  ("Budget and ranker"; Algorithm 1)
# --------------------------------------------------------------------------------------

def _minmax(x: np.ndarray) -> np.ndarray:
    """Min-max normalisation to [0, 1]; all zeros when max == min."""
    lo, hi = np.min(x), np.max(x)
    if hi == lo:
        return np.zeros(x.shape, dtype=F64)
    return (x - lo) / (hi - lo)


def rank_scores(ema: np.ndarray, pos: np.ndarray, alpha: float) -> np.ndarray:
    """s_i = alpha * a_hat_i + (1 - alpha) * r_hat_i over the candidate set given."""
    a_hat = _minmax(np.asarray(ema).astype(F64))
    r_hat = _minmax(np.asarray(pos).astype(F64))
    al = F64(alpha)
    return al * a_hat + (1.0 - al) * r_hat


_M64 = (1 << 64) - 1


def splitmix64(x: int) -> int:
    """One output of the SplitMix64 generator (Steele, Lea, Flood 2014) for state x."""
    z = (x + 0x9E3779B97F4A7C15) & _M64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _M64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _M64
    return z ^ (z >> 31)


def random_scores(seed: int, unit_key: int, pos: np.ndarray) -> np.ndarray:
    """Scores of the random ranker (matched-rate isolation study: which token goes is drawn
    at random while how many go stays the budget rule's).  A counter-based draw, so both
    implementations get the same numbers: score = top 53 bits of
    splitmix64(seed + unit_key * 2^32 + position) scaled to [0, 1)."""
    out = np.empty(len(pos), dtype=F64)
    for i, p in enumerate(np.asarray(pos).tolist()):
        r = splitmix64((int(seed) + (int(unit_key) << 32) + int(p)) & _M64)
        out[i] = (r >> 11) * 2.0 ** -53
    return out


def shared_importance(units: Sequence["UnitCache"]) -> np.ndarray:
    """Layer-level importance of the paper's literal reading: the manager keeps one EMA of
    the head-averaged attention per layer.  With the mass kept per kv-head group this is
    the sum over the groups (the 1/heads factor drops out of the min-max normalisation),
    accumulated in kv-head order in float64."""
    acc = np.zeros(units[0].n, dtype=F64)
    for u in units:
        assert u.n == units[0].n and np.array_equal(u.pos, units[0].pos)
        acc = acc + u.ema.astype(F64)
    return acc


def select_evictions(u: UnitCache, budget: int, protected: int, alpha: float,
                     importance: Optional[np.ndarray] = None, ranker: str = "composite",
                     seed: int = 0, unit_key: int = 0, page: int = 0
                     ) -> Tuple[np.ndarray, np.ndarray]:
    """Slots to keep and to evict so that the length is at most the budget.

    ``page`` > 1 coarsens the eviction to whole pages (``select_page_evictions``).

    If n <= N nothing happens.  Otherwise the newest P_eff = min(P, n) slots are
    protected, the other n - P_eff are candidates ranked by ``rank_scores``, and the
    e = min(n - N, n - P_eff) lowest are evicted; equal scores go oldest first.
    ``importance`` [n] replaces the unit's own EMA (layer-shared ranking);
    ``ranker`` = "random" ranks by ``random_scores`` instead.
    Returns (keep slots increasing, evicted slots increasing).
    """
    n = u.n
    if n <= budget:
        return np.arange(n), np.zeros(0, dtype=np.int64)
    p_eff = min(protected, n)
    n_cand = n - p_eff
    e = min(n - budget, n_cand)
    if e <= 0:
        return np.arange(n), np.zeros(0, dtype=np.int64)
    if ranker == "random":
        s = random_scores(seed, unit_key, u.pos[:n_cand])
    else:
        a = u.ema if importance is None else importance
        s = rank_scores(a[:n_cand], u.pos[:n_cand], alpha)
    if page and page > 1:
        evict = select_page_evictions(s, u.pos[:n], n_cand, e, page)
    else:
        order = np.lexsort((u.pos[:n_cand], s))    # by score, then older first
        evict = np.sort(order[:e])
    keep = np.setdiff1d(np.arange(n), evict)
    return keep, evict


def select_page_evictions(s: np.ndarray, pos: np.ndarray, n_cand: int, e: int, page: int) -> np.ndarray:
    """Coarsened eviction ("Compatibility with serving systems" and "Limitations": token-level
    eviction leaves partially dead blocks in a paged layout unless eviction is coarsened).

    A page is the set of live slots whose original positions share floor(pos / page); slots
    are position-sorted, so a page is a run of consecutive slots.  ``s`` [n_cand] are the
    token scores of the candidates, exactly those the token-level rule ranks.  A page can go
    only when every live slot of it is a candidate (none lies in the protected window).  Its
    score is the mean of its slots' scores: their sum in slot order, in float64, divided by
    their number.  Pages go whole, lowest score first and older first among equal scores,
    until at least ``e`` slots are gone (so the length is at most the budget; it may fall
    short of it by up to page - 1 slots) or no page that can go is left.
    Returns the evicted slots, increasing.
    """
    pid = np.asarray(pos).astype(np.int64) // int(page)
    n = len(pid)
    pages = []                                      # (score, first slot, slot count)
    i0 = 0
    while i0 < n:
        i1 = i0
        while i1 < n and pid[i1] == pid[i0]:
            i1 += 1
        if i1 <= n_cand:
            tot = F64(0.0)
            for i in range(i0, i1):
                tot = F64(tot + F64(s[i]))
            pages.append((F64(tot / F64(i1 - i0)), i0, i1 - i0))
        i0 = i1
    pages.sort(key=lambda t: (t[0], t[1]))
    gone, out = 0, []
    for _, first, cnt in pages:
        if gone >= e:
            break
        out.extend(range(first, first + cnt))
        gone += cnt
    return np.array(sorted(out), dtype=np.int64)


def demote(u: UnitCache, fp16_window: int) -> int:
    """Quantise the oldest FP16 slots to INT8 until at most W stay FP16 (W < 0: never)."""
    if fp16_window < 0:
        return 0
    done = 0
    while u.n16 > fp16_window:
        i = int(np.argmax(u.is16))                 # oldest FP16 slot (INT8 slots come first)
        if u.kcs is None:
            u.k8[i], u.ks[i] = quantize_vector(u.k16[i])
            u.v8[i], u.vs[i] = quantize_vector(u.v16[i])
        else:
            u.k8[i] = quantize_channels(u.k16[i], u.kcs)
            u.v8[i] = quantize_channels(u.v16[i], u.vcs)
        u.k16[i] = 0
        u.v16[i] = 0
        u.is16[i] = False
        done += 1
    return done


def evict_compact_unit(u: UnitCache, budget: int, protected: int, alpha: float, fp16_window: int,
                       **ranking) -> np.ndarray:
    """Algorithm 1's per-layer tail for one unit: rank, evict, compact, then demote.

    ``ranking`` goes to ``select_evictions`` (importance, ranker, seed, unit_key, page).
    Returns the original positions that were evicted.
    """
    keep, evict = select_evictions(u, budget, protected, alpha, **ranking)
    gone = u.pos[evict].copy()
    if evict.size:
        u.take(keep)
    demote(u, fp16_window)
    return gone


# --------------------------------------------------------------------------------------
# Whole decode step over a set of units  (Algorithm 1)
# --------------------------------------------------------------------------------------

@dataclass
class Policy:
    n_layers: int
    n_tight: Sequence[int]
    n_loose: Sequence[int]
    protected: int
    fp16_window: int
    tau: float = float(np.float32(0.7))
    alpha: float = float(np.float32(0.65))
    ema_decay: float = float(np.float32(0.9))
    sm_scale: float = 1.0
    weights: Tuple[float, float, float] = (float(np.float32(0.4)), float(np.float32(0.3)),
                                           float(np.float32(0.3)))
    mass_gain: Optional[float] = None      # None: 1 - ema_decay
    ranker: str = "composite"              # or "random"
    rank_scope: str = "kv_head"            # or "layer": one kept set per (layer, sequence)
    ranker_seed: int = 0
    evict_page: int = 0                    # > 1: whole pages of that many positions are evicted
    batch: int = 1                         # needed for the random ranker's unit keys
    n_kv_heads: int = 1


class OracleRun:
    """Follows a chosen set of units (layer, b, kv_head) through decode steps.

    Units evolve independently given their inputs and their sequence's budget, so a
    run may hold any subset of them.
    """

    def __init__(self, policy: Policy, units: Dict[Tuple[int, int, int], UnitCache], next_pos: int):
        self.policy = policy
        self.units = units
        self.next_pos = next_pos
        self.pending = 1          # tokens appended per layer since the last evict_compact

    def attend(self, layer: int, q: np.ndarray, k_new: np.ndarray, v_new: np.ndarray, group: int
               ) -> Dict[Tuple[int, int, int], np.ndarray]:
        """q [B, Hq, D], k_new/v_new [B, Hkv, D] fp16 -> {unit: out [G, D]} for followed units."""
        outs = {}
        p = self.policy
        self.pending = 1
        for (l, b, g), u in self.units.items():
            if l != layer:
                continue
            out, _ = attend_unit(u, q[b, g * group:(g + 1) * group], k_new[b, g], v_new[b, g],
                                 self.next_pos, p.sm_scale, p.ema_decay, p.mass_gain)
            outs[(l, b, g)] = out
        return outs

    def attend_chunk(self, layer: int, q: np.ndarray, k_new: np.ndarray, v_new: np.ndarray, group: int
                     ) -> Dict[Tuple[int, int, int], np.ndarray]:
        """q [B, Tq, Hq, D], k_new/v_new [B, Tq, Hkv, D] fp16 -> {unit: out [Tq, G, D]}."""
        outs = {}
        p = self.policy
        self.pending = int(q.shape[1])
        for (l, b, g), u in self.units.items():
            if l != layer:
                continue
            out, _ = attend_chunk_unit(u, q[b, :, g * group:(g + 1) * group], k_new[b, :, g], v_new[b, :, g],
                                       self.next_pos, p.sm_scale, p.ema_decay, p.mass_gain)
            outs[(l, b, g)] = out
        return outs

    def observe(self, layer: int, q: np.ndarray, first: int, group: int
                ) -> Dict[Tuple[int, int, int], np.ndarray]:
        """q [B, Tq, Hq, D]: queries of the cached slots first .. first + Tq - 1 of every followed
        unit of the layer -> {unit: out [Tq, G, D]}; importance updated, nothing appended."""
        outs = {}
        p = self.policy
        for (l, b, g), u in self.units.items():
            if l != layer:
                continue
            out, _ = observe_unit(u, q[b, :, g * group:(g + 1) * group], first, p.sm_scale, p.ema_decay,
                                  p.mass_gain)
            outs[(l, b, g)] = out
        return outs

    def step(self, logits: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
        """logits [B, V] fp32 -> (c [B] float64, tight [B] bool)."""
        p = self.policy
        c = np.array([confidence(row, p.weights) for row in logits])
        tight = c >= F64(p.tau)
        return c, tight

    def evict_compact(self, tight: np.ndarray) -> Dict[Tuple[int, int, int], np.ndarray]:
        p = self.policy
        gone = {}
        if p.rank_scope == "layer":
            # one ranking per (layer, sequence) from the importance shared by its kv-heads;
            # every kv-head of a followed (layer, sequence) must be followed
            for (l, b) in sorted({(l, b) for (l, b, _) in self.units}):
                group = [self.units[(l, b, g)] for g in range(p.n_kv_heads)]
                N = p.n_tight[l] if tight[b] else p.n_loose[l]
                shared = shared_importance(group)
                key = (1 << 40) + l * p.batch + b
                for g, u in enumerate(group):
                    gone[(l, b, g)] = evict_compact_unit(u, N, p.protected, p.alpha, p.fp16_window,
                                                         importance=shared, ranker=p.ranker,
                                                         seed=p.ranker_seed, unit_key=key,
                                                         page=p.evict_page)
        else:
            for (l, b, g), u in self.units.items():
                N = p.n_tight[l] if tight[b] else p.n_loose[l]
                key = (l * p.batch + b) * p.n_kv_heads + g
                gone[(l, b, g)] = evict_compact_unit(u, N, p.protected, p.alpha, p.fp16_window,
                                                     ranker=p.ranker, seed=p.ranker_seed, unit_key=key,
                                                     page=p.evict_page)
        self.next_pos += self.pending
        self.pending = 1
        return gone
