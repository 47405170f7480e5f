"""CPU oracle for the per-iteration sampling epilogue (TEST INFRASTRUCTURE ONLY).

A plain, slow, dense implementation of what the decision-plane hot path
computes: logits row -> penalties -> temperature -> top-k / top-p / min-p
filter -> softmax over the survivors -> inverse-CDF categorical draw, plus
speculative hot-vocab sampling (SHVS).  It exists to check the HIP library
and to be timed as a CPU baseline.  Only tests, the smoke check and the
benchmark's CPU-baseline leg may import it; it shares no code with the HIP
path and must never be used to produce results for a caller.

Every function cites the passage of the paper it follows.  Where the paper is
silent the convention chosen is stated in the function's docstring.

Pins (tests marked "not gpu"): Philox against an independent library
implementation (the counter-based engine in PyTorch's ATen headers) and the
closed forms of its round constants; penalties against hand-computed rows; top-k against
pairwise order properties; softmax-on-subset against a library masked
softmax; the draw by exhaustive enumeration of all 2^24 uniforms; SHVS by
enumeration of the accept/draw grid and chi-square tests against the
filtered distribution.  No function here is "parity unpinned".

All floating point that decides *which* tokens survive is float32 with one
rounding per operation (penalties, division by temperature, the min-p
threshold); all probability mass is float64.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional, Sequence

import numpy as np

AMBIGUITY_WINDOW = 1e-6  # relative distance to a CDF / nucleus / acceptance boundary

# ----------------------------------------------------------------------------------------------
# Counter-based random numbers (section 5.1, deterministic random number generation)
# ----------------------------------------------------------------------------------------------
# The paper pre-generates random numbers so that the result does not depend on the number of
# samplers.  The same property is obtained here from a counter-based generator keyed by
# (seed, row, step): Philox4x32 with 10 rounds, as defined by Salmon, Moraes, Dror and Shaw,
# "Parallel random numbers: as easy as 1, 2, 3" (SC'11).  Constants are the published ones.
_PHILOX_M0 = np.uint64(0xD2511F53)
_PHILOX_M1 = np.uint64(0xCD9E8D57)
_PHILOX_W0 = 0x9E3779B9  # golden ratio
_PHILOX_W1 = 0xBB67AE85  # sqrt(3) - 1
_MASK32 = np.uint64(0xFFFFFFFF)


def philox4x32_10(counter: np.ndarray, key: np.ndarray) -> np.ndarray:
    """Philox4x32-10 block function.

    counter: [..., 4] uint32, key: [..., 2] uint32 (broadcastable).  Returns [..., 4] uint32.
    One round multiplies counter words 0 and 2 by the two round multipliers, swaps the high and
    low halves into the other lanes and xors in the key; the key is bumped by the two Weyl
    constants between rounds.
    """
    counter = np.asarray(counter, dtype=np.uint32)
    key = np.asarray(key, dtype=np.uint32)
    c0, c1, c2, c3 = (counter[..., i].astype(np.uint64) for i in range(4))
    k0 = key[..., 0].astype(np.uint64)
    k1 = key[..., 1].astype(np.uint64)
    for r in range(10):
        p0 = _PHILOX_M0 * c0  # 64-bit product, no overflow: both factors < 2^32
        p1 = _PHILOX_M1 * c2
        hi0, lo0 = p0 >> np.uint64(32), p0 & _MASK32
        hi1, lo1 = p1 >> np.uint64(32), p1 & _MASK32
        c0, c1, c2, c3 = (hi1 ^ c1 ^ k0) & _MASK32, lo1, (hi0 ^ c3 ^ k1) & _MASK32, lo0
        if r < 9:
            k0 = (k0 + np.uint64(_PHILOX_W0)) & _MASK32
            k1 = (k1 + np.uint64(_PHILOX_W1)) & _MASK32
    return np.stack([c0, c1, c2, c3], axis=-1).astype(np.uint32)


def row_uniforms(seed: int, rows: np.ndarray, step) -> tuple[np.ndarray, np.ndarray, np.ndarray]:
    """The three uniforms of a (row, step) pair: ``(u_draw, u_acc, u_tail)`` in [0, 1).

    Convention (the paper names no generator): one Philox block per (row, step) with
    key = (seed low 32 bits, seed high 32 bits) and counter = (row low, step low, step high,
    row high), so that global row indices that differ by 2^32 do not share their uniforms;
    word i is turned into ``(x >> 8) * 2^-24``, which is exact in float32 and float64.
    Word 0 drives the categorical draw, word 1 the SHVS acceptance test, word 2 the SHVS tail
    draw (three independent variates, as the exactness identity of section 5.3 assumes).
    ``step`` may be an array broadcastable against ``rows``.
    """
    rows = np.asarray(rows, dtype=np.uint64)
    step = np.asarray(step, dtype=np.uint64)
    rows, step = np.broadcast_arrays(rows, step)
    ctr = np.stack(
        [rows & _MASK32, step & _MASK32, step >> np.uint64(32), rows >> np.uint64(32)], axis=-1
    ).astype(np.uint32)
    key = np.array([seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF], dtype=np.uint32)
    x = philox4x32_10(ctr, key)
    u = (x >> np.uint32(8)).astype(np.float64) * (2.0 ** -24)
    return u[..., 0], u[..., 1], u[..., 2]


# ----------------------------------------------------------------------------------------------
# Step 1: logits adjustment (section 2.1 Eq. (1), section 2.2)
# ----------------------------------------------------------------------------------------------
def history_histograms(hist_row: np.ndarray, n_prompt: int, V: int) -> tuple[np.ndarray, np.ndarray]:
    """Dense histograms of section 2.2: returns ``(C_o, M_p or M_o)``.

    ``hist_row`` is the row's token history; its first ``n_prompt`` ids are the prompt ``Y_p``,
    the rest the generated tokens ``Y_<s``.  ``C_o = Hist(Y_<s)`` counts generated tokens only;
    the mask is ``(Hist(Y_p) > 0) or (C_o > 0)``.
    """
    hist_row = np.asarray(hist_row, dtype=np.int64)
    if hist_row.size and (hist_row.min() < 0 or hist_row.max() >= V):
        raise ValueError("history id outside [0, V)")
    n_prompt = int(min(max(n_prompt, 0), hist_row.size))
    c_p = np.bincount(hist_row[:n_prompt], minlength=V)
    c_o = np.bincount(hist_row[n_prompt:], minlength=V)
    return c_o, (c_p > 0) | (c_o > 0)


class IncrementalHistory:
    """The incremental penalty state of section 5.2 for a batch of B sequences.

    A row-append token buffer ``Y`` of shape ``[L_max, B]`` (the tokens generated at step s form
    row s) and the histograms carried from step to step instead of being rebuilt:
    ``C_o^{s+1} = C_o^s + Hist(Y_s)`` and ``M_o^{s+1} = (C_o^{s+1} > 0)``; the prompt histogram
    ``C_p`` (hence ``M_p``) is invariant over the steps of a sequence.  Dense ``[B, V]`` arrays, as
    the paper writes them.  A sequence may be restarted (its slot evicted and given a new prompt)
    at any step; its generated tokens then start again at row 0 of its column.
    """

    def __init__(self, B: int, V: int, L_max: int):
        self.B, self.V, self.L_max = B, V, L_max
        self.Y = np.full((L_max, B), -1, dtype=np.int64)
        self.n_out = np.zeros(B, dtype=np.int64)          # generated tokens per sequence
        self.C_o = np.zeros((B, V), dtype=np.int64)
        self.M_p = np.zeros((B, V), dtype=bool)

    def restart(self, b: int, prompt_ids) -> None:
        prompt_ids = np.asarray(prompt_ids, dtype=np.int64)
        if prompt_ids.size and (prompt_ids.min() < 0 or prompt_ids.max() >= self.V):
            raise ValueError("prompt id outside [0, V)")
        self.Y[:, b] = -1
        self.n_out[b] = 0
        self.C_o[b] = 0
        self.M_p[b] = np.bincount(prompt_ids, minlength=self.V) > 0

    def append(self, ids) -> None:
        """One step: ``ids[b]`` is the token generated for sequence b (negative: none this step)."""
        ids = np.asarray(ids, dtype=np.int64)
        for b in range(self.B):
            t = int(ids[b])
            if t < 0:
                continue
            if t >= self.V:
                raise ValueError("token id outside [0, V)")
            if self.n_out[b] >= self.L_max:
                raise ValueError("token buffer full")
            self.Y[self.n_out[b], b] = t
            self.n_out[b] += 1
            self.C_o[b, t] += 1                            # C_o += Hist(Y_s): a one-hot row per sequence

    def histograms(self, b: int) -> tuple[np.ndarray, np.ndarray]:
        """``(C_o, M_p or M_o)`` of sequence b, what ``history_histograms`` rebuilds from the token list."""
        return self.C_o[b], self.M_p[b] | (self.C_o[b] > 0)


def apply_penalties(z: np.ndarray, c_o: np.ndarray, mask: np.ndarray, rep: float, freq: float,
                    pres: float, literal_division: bool = False) -> np.ndarray:
    """``Z' = ApplyPenalty(Z, Y_<s)`` (Eq. (1)), float32, one rounding per operation.

    Repetition (section 2.2): factor ``f = 1 + (rep - 1) * mask``.  The paper prints
    ``Z' = Z / f``; dividing a negative logit by f > 1 would *raise* it, so the sign-aware form
    of the penalty it cites is used: ``z > 0 ? z / f : z * f``  (``literal_division=True`` keeps
    the printed form, for tests only).
    Frequency and presence ("follow analogously", section 2.2) use the generated-token
    histogram: ``z <- z - fl(freq * C_o)``, then ``z <- z - pres`` where ``C_o > 0``.
    Order: repetition, frequency, presence; all before temperature (Eq. (1) precedes Eq. (2)).
    Columns outside the history are returned bit-identical.
    """
    z = np.asarray(z, dtype=np.float32)
    f = np.where(mask, np.float32(rep), np.float32(1.0)).astype(np.float32)
    if literal_division:
        zr = (z / f).astype(np.float32)
    else:
        zr = np.where(z > 0, z / f, z * f).astype(np.float32)
    zr = np.where(mask, zr, z)
    t = (np.float32(freq) * c_o.astype(np.float32)).astype(np.float32)
    zf = ((zr - t).astype(np.float32) - np.float32(pres)).astype(np.float32)
    return np.where(c_o > 0, zf, zr).astype(np.float32)


def apply_constraints(z_row: np.ndarray, bias_ids=None, bias_vals=None, allow_ids=None) -> np.ndarray:
    """Logit bias and allow-list of one row, before the penalties (section 5.2 lists allow-lists among
    the constraints that compose on the survivor set, section 6 of the paper "optional biases").

    Convention (the paper gives none): an allow-list, if the row has one, masks every other column
    to -inf; a bias entry adds ``fl32(z + bias)`` to its column (entries naming the same column
    add up in list order); a bias on a column the allow-list masks leaves it masked.  Both are
    independent of the order of the survivors (a column's value changes, the filters of Eq. (2)
    then see the changed row), and both come before ``ApplyPenalty``, as a logits processor that
    runs ahead of the sampler would.  Returns float32.
    """
    z = np.array(z_row, dtype=np.float32, copy=True)
    V = z.size
    if allow_ids is not None:
        allow_ids = np.asarray(allow_ids, dtype=np.int64)
        if allow_ids.size and (allow_ids.min() < 0 or allow_ids.max() >= V):
            raise ValueError("allowed id outside [0, V)")
        keep = np.zeros(V, dtype=bool)
        keep[allow_ids] = True
        z[~keep] = -np.inf
    if bias_ids is not None:
        bias_ids = np.asarray(bias_ids, dtype=np.int64)
        bias_vals = np.asarray(bias_vals, dtype=np.float32)
        if bias_ids.size and (bias_ids.min() < 0 or bias_ids.max() >= V):
            raise ValueError("biased id outside [0, V)")
        for i, v in zip(bias_ids, bias_vals):
            z[i] = np.float32(z[i] + v)
    return z


# ----------------------------------------------------------------------------------------------
# Step 2: temperature, filter, stable softmax (Eq. (2); truncation-first filtering, section 5.2)
# ----------------------------------------------------------------------------------------------
@dataclass
class RowDist:
    """The filtered distribution of one row, i.e. the subset K_b with its index map (section 5.2)."""

    V: int
    error: bool = False
    greedy: bool = False
    greedy_id: int = -1
    ids: np.ndarray = field(default_factory=lambda: np.zeros(0, np.int64))  # K_b, ascending token id
    w: np.ndarray = field(default_factory=lambda: np.zeros(0, np.float64))  # exp(y - y_max) on K_b
    n: int = 0  # |K_b|
    n_k: int = 0
    n_m: int = 0
    n_p: int = 0
    S_k: float = 0.0  # mass of the top-k prefix (all of V when top-k is off)
    nucleus_margin: float = np.inf  # relative distance of top_p * S_k to the nearest prefix mass
    alt: list = field(default_factory=list)  # RowDist alternatives when the nucleus is ambiguous

    @property
    def S_K(self) -> float:
        return float(np.cumsum(self.w)[-1]) if self.n else 0.0

    def probs(self) -> np.ndarray:
        """Dense p-tilde over V (zero outside K_b)."""
        p = np.zeros(self.V, dtype=np.float64)
        if self.greedy:
            p[self.greedy_id] = 1.0
        elif self.n:
            p[self.ids] = self.w / self.S_K
        return p


def _survivors(order: np.ndarray, w_sorted: np.ndarray, n: int, V: int) -> tuple[np.ndarray, np.ndarray]:
    keep = order[:n]
    by_id = np.argsort(keep, kind="stable")
    return keep[by_id].astype(np.int64), w_sorted[:n][by_id]


def row_distribution(z_row: np.ndarray, par, hist_row: Optional[np.ndarray] = None,
                     literal_division: bool = False, histograms: Optional[tuple] = None) -> RowDist:
    """Steps (1) and (2) of section 2.1 for one row; returns K_b and the weights on it.

    Conventions where the paper is silent:
    * temperature 0 means greedy: argmax of the penalised logits, lowest id on ties;
    * ``y = z' / temperature`` is an IEEE float32 division;
    * the survivors are a prefix of the total order (y descending, token id ascending):
      top-k keeps exactly k; min-p keeps ``y >= fl32(y_max + fl32(ln(min_p)))`` (equivalent to
      p_v >= min_p * p_max); top-p keeps the shortest prefix of the top-k prefix whose mass is
      >= top_p times the top-k prefix mass; K_b is the shortest of the three, at least one token;
    * weights ``w = exp(y - y_max)`` and all sums are float64; truncating first and normalising
      on K_b is identical to a masked softmax over V (section 5.2).
    NaN or +inf logits, an all -inf row, a negative temperature or a non-positive repetition
    penalty give ``error`` (sampled id -1).
    """
    z = np.asarray(z_row, dtype=np.float32)
    V = z.size
    temperature = np.float32(par["temperature"])
    rep = np.float32(par["rep_penalty"])
    if not (temperature >= 0) or not (rep > 0):
        return RowDist(V=V, error=True)
    if histograms is not None:  # carried from step to step (section 5.2) instead of rebuilt from the token list
        c_o, mask = histograms
        z = apply_penalties(z, c_o, mask, rep, par["freq_penalty"], par["pres_penalty"], literal_division)
    elif hist_row is not None and len(hist_row):
        c_o, mask = history_histograms(hist_row, int(par["n_prompt"]), V)
        z = apply_penalties(z, c_o, mask, rep, par["freq_penalty"], par["pres_penalty"],
                            literal_division)
    if np.isnan(z).any() or np.isposinf(z).any() or np.isneginf(z).all():
        return RowDist(V=V, error=True)
    if temperature == 0:
        return RowDist(V=V, greedy=True, greedy_id=int(np.argmax(z)), n=1)
    with np.errstate(over="ignore"):
        y = (z / temperature).astype(np.float32)
    if np.isposinf(y).any():
        return RowDist(V=V, error=True)
    order = np.argsort(-y, kind="stable")  # y descending, ties by ascending id
    ys = y[order]
    y_max = ys[0]
    if np.isneginf(y_max):
        return RowDist(V=V, error=True)
    w_sorted = np.exp(ys.astype(np.float64) - np.float64(y_max))
    top_k = int(par["top_k"])
    n_k = top_k if 1 <= top_k < V else V
    min_p = np.float32(par["min_p"])
    if min_p > 0:
        thr = np.float32(y_max + np.float32(np.log(np.float64(min_p))))
        n_m = int(np.count_nonzero(ys >= thr))
    else:
        n_m = V
    cum = np.cumsum(w_sorted[:n_k])
    S_k = float(cum[-1])
    top_p = np.float64(np.float32(par["top_p"]))
    margin = np.inf
    n_p_alts: list[int] = []
    if top_p >= 1:
        n_p = n_k
    elif top_p <= 0:
        n_p = 1
    else:
        target = top_p * S_k
        n_p = min(int(np.searchsorted(cum, target, side="left")) + 1, n_k)
        margin = (cum[n_p - 1] - target) / S_k
        if margin < AMBIGUITY_WINDOW and n_p < n_k:
            n_p_alts.append(n_p + 1)
        if n_p >= 2:
            below = (target - cum[n_p - 2]) / S_k
            margin = min(margin, below)
            if below < AMBIGUITY_WINDOW:
                n_p_alts.append(n_p - 1)
    n = max(1, min(n_k, n_m, n_p))
    ids, w = _survivors(order, w_sorted, n, V)
    d = RowDist(V=V, ids=ids, w=w, n=n, n_k=n_k, n_m=n_m, n_p=n_p, S_k=S_k,
                nucleus_margin=float(margin))
    for n_p2 in n_p_alts:
        n2 = max(1, min(n_k, n_m, n_p2))
        if n2 != n:
            ids2, w2 = _survivors(order, w_sorted, n2, V)
            d.alt.append(RowDist(V=V, ids=ids2, w=w2, n=n2, n_k=n_k, n_m=n_m, n_p=n_p2, S_k=S_k))
    return d


# ----------------------------------------------------------------------------------------------
# Step 3: token selection (section 2.1 (3)) and SHVS (section 5.3)
# ----------------------------------------------------------------------------------------------
def inverse_cdf(ids: np.ndarray, w: np.ndarray, u) -> tuple[np.ndarray, np.ndarray]:
    """``y ~ Categorical(w / sum w)`` by inverse CDF over ``ids`` in the given order.

    Returns the first id whose running mass exceeds ``u * total`` (float64), and, per draw, the
    relative distance of ``u * total`` to the nearest of the two CDF steps bounding that id.
    If rounding leaves no such id, the last id of positive weight is returned.  ``u`` may be an
    array (one draw per element).
    """
    cum = np.cumsum(w)
    total = cum[-1]
    target = np.asarray(u, dtype=np.float64) * total
    if not total > 0:  # no positive weight: nothing can be drawn from this set
        return np.full(target.shape, -1, np.int64), np.full(target.shape, np.inf)
    j = np.searchsorted(cum, target, side="right")  # first index with cum > target
    last_pos = int(np.flatnonzero(w > 0)[-1])
    j = np.minimum(j, last_pos)
    lo = np.where(j > 0, cum[np.maximum(j - 1, 0)], -np.inf)
    margin = np.minimum(cum[j] - target, target - lo) / total
    return ids[j], margin


def shvs_masses(d: RowDist, hot_mask: np.ndarray) -> tuple[float, float, float]:
    """``(S_H, S_tail, alpha)`` of Eq. (7) with the weights restricted to K_b.

    The paper defines the masses on the un-filtered weights; so that SHVS reproduces the
    *filtered* full-vocabulary distribution the weights are ``w_v * 1[v in K_b]`` -- the
    exactness identity Eq. (9) holds for any non-negative weights.
    """
    hot = hot_mask[d.ids]
    S_H = float(np.cumsum(d.w[hot])[-1]) if hot.any() else 0.0
    S_T = float(np.cumsum(d.w[~hot])[-1]) if (~hot).any() else 0.0
    return S_H, S_T, S_H / d.S_K


def draw(d: RowDist, u_draw, u_acc=None, u_tail=None, hot_mask: Optional[np.ndarray] = None,
         biased_fallback: bool = False):
    """Token id(s) for the given uniform(s); returns ``(ids, margin, accepted)``.

    Without a hot set: inverse CDF over K_b in ascending token id with ``u_draw``.
    With a hot set (section 5.3, Eq. (8)): accept iff ``u_acc <= alpha_b`` (evaluated as
    ``u_acc * S_K <= S_H``, and never when ``S_H = 0``); on acceptance draw from the hot
    proposal q (K_b intersected with the hot set, ascending token id, ``u_draw``); on rejection
    draw from the tail proposal r (K_b minus the hot set, ascending token id, ``u_tail``).
    Greedy rows ignore the hot set.  ``margin`` is the relative distance to the nearest decision
    boundary (CDF step or acceptance threshold).  ``biased_fallback=True`` plants the classic
    mistake of re-running the full sampler on rejection (tests only).
    """
    u_draw = np.asarray(u_draw, dtype=np.float64)
    if d.error:
        return np.full(u_draw.shape, -1, np.int64), np.full(u_draw.shape, np.inf), None
    if d.greedy:
        return np.full(u_draw.shape, d.greedy_id, np.int64), np.full(u_draw.shape, np.inf), None
    if hot_mask is None:
        ids, margin = inverse_cdf(d.ids, d.w, u_draw)
        return ids, margin, None
    u_acc = np.asarray(u_acc, dtype=np.float64)
    u_tail = np.asarray(u_tail, dtype=np.float64)
    hot = hot_mask[d.ids]
    S_H, S_T, _ = shvs_masses(d, hot_mask)
    S_K = d.S_K
    accepted = (u_acc * S_K <= S_H) & (S_H > 0)
    out = np.empty(u_draw.shape, np.int64)
    margin = np.abs(u_acc * S_K - S_H) / S_K * np.ones(u_draw.shape)
    if hot.any():
        ih, mh = inverse_cdf(d.ids[hot], d.w[hot], u_draw)
    else:
        ih, mh = np.full(u_draw.shape, -1, np.int64), np.full(u_draw.shape, np.inf)
    if biased_fallback:
        it, mt = inverse_cdf(d.ids, d.w, u_tail)
    elif (~hot).any():
        it, mt = inverse_cdf(d.ids[~hot], d.w[~hot], u_tail)
    else:
        it, mt = np.full(u_draw.shape, -1, np.int64), np.full(u_draw.shape, np.inf)
    out = np.where(accepted, ih, it)
    margin = np.minimum(margin, np.where(accepted, mh, mt))
    return out, margin, accepted


# ----------------------------------------------------------------------------------------------
# Whole batch
# ----------------------------------------------------------------------------------------------
@dataclass
class RowResult:
    id: int
    alt_ids: set  # other ids that are acceptable because a decision lies within the ambiguity window
    ambiguous: bool
    n: int
    p_chosen: float  # p-tilde of the returned id
    alpha: float  # SHVS hot mass (nan without a hot set)
    accepted: Optional[bool]
    S_k: float
    dist: Optional[RowDist] = None
    alt_p: tuple = ()  # p-tilde of ``id`` under the neighbouring nucleus lengths, when the boundary is ambiguous
    S_k_used: bool = False  # the row's controls make S_k part of the method (0 < top_p < 1: it scales the nucleus target)


def _neighbours(d: RowDist, tok: int, hot_mask, accepted) -> set:
    """Ids adjacent to ``tok`` in the CDF walk that produced it."""
    ids = d.ids
    if hot_mask is not None:
        hot = hot_mask[d.ids]
        ids = d.ids[hot] if accepted else d.ids[~hot]
    j = int(np.searchsorted(ids, tok))
    return {int(ids[i]) for i in (j - 1, j + 1) if 0 <= i < ids.size}


def sample_row(z_row: np.ndarray, par, hist_row, hot_mask: Optional[np.ndarray], seed: int,
               row: int, step: int, keep_dist: bool = False, histograms: Optional[tuple] = None) -> RowResult:
    """One row of the sampling call: distribution, uniforms, draw, and the alternative ids that
    count as correct when a decision is within ``AMBIGUITY_WINDOW`` of a boundary."""
    d = row_distribution(z_row, par, hist_row, histograms=histograms)
    u_draw, u_acc, u_tail = (float(x) for x in row_uniforms(seed, np.array(row), step))
    tok, margin, acc = draw(d, u_draw, u_acc, u_tail, hot_mask)
    tok = int(tok)
    if d.error or d.greedy:
        return RowResult(tok, set(), False, d.n, 1.0 if d.greedy else 0.0, float("nan"), None, 0.0,
                         d if keep_dist else None)
    alt: set = set()
    ambiguous = False
    alpha = float("nan")
    accepted = None
    if hot_mask is not None:
        S_H, _, alpha = shvs_masses(d, hot_mask)
        accepted = bool(acc)
        if abs(u_acc * d.S_K - S_H) / d.S_K < AMBIGUITY_WINDOW:
            ambiguous = True
            hot = hot_mask[d.ids]
            if accepted and (~hot).any():
                alt.add(int(inverse_cdf(d.ids[~hot], d.w[~hot], u_tail)[0]))
            if (not accepted) and hot.any():
                alt.add(int(inverse_cdf(d.ids[hot], d.w[hot], u_draw)[0]))
    if float(margin) < AMBIGUITY_WINDOW:
        ambiguous = True
        alt |= _neighbours(d, tok, hot_mask, accepted)
    alt_p = []
    for d2 in d.alt:  # nucleus boundary within the window: the neighbouring prefix lengths
        ambiguous = True
        t2, _, a2 = draw(d2, u_draw, u_acc, u_tail, hot_mask)
        alt.add(int(t2))
        alt |= _neighbours(d2, int(t2), hot_mask, None if a2 is None else bool(a2))
        j2 = int(np.searchsorted(d2.ids, tok))
        if j2 < d2.ids.size and int(d2.ids[j2]) == tok:  # the same id, normalised over the other prefix
            alt_p.append(float(d2.w[j2] / d2.S_K))
    alt.discard(tok)
    p_chosen = float(d.w[np.searchsorted(d.ids, tok)] / d.S_K)
    return RowResult(tok, alt, ambiguous, d.n, p_chosen, alpha, accepted, d.S_k,
                     d if keep_dist else None, tuple(alt_p), bool(0.0 < float(par["top_p"]) < 1.0))


def sample_with_state(logits_f32: np.ndarray, params, state: IncrementalHistory, hot_ids, seed: int, step: int,
                      row_offset: int = 0) -> list[RowResult]:
    """The whole call with the penalties taken from the incremental state (row b is sequence b)."""
    B, V = logits_f32.shape
    hot_mask = hot_mask_from_ids(hot_ids, V)
    return [sample_row(logits_f32[b], params[b], None, hot_mask, seed, row_offset + b, step,
                       histograms=state.histograms(b)) for b in range(B)]


def hot_mask_from_ids(hot_ids: Optional[Sequence[int]], V: int) -> Optional[np.ndarray]:
    """Membership mask of the hot set H (section 5.3); ids must be distinct and inside [0, V)."""
    if hot_ids is None:
        return None
    hot_ids = np.asarray(hot_ids, dtype=np.int64)
    if hot_ids.size and (hot_ids.min() < 0 or hot_ids.max() >= V):
        raise ValueError("hot id outside [0, V)")
    m = np.zeros(V, dtype=bool)
    m[hot_ids] = True
    if int(m.sum()) != hot_ids.size:
        raise ValueError("duplicate hot id")
    return m


def sample(logits_f32: np.ndarray, params, hist_ptr: Optional[np.ndarray], hist_ids: Optional[np.ndarray],
           hot_ids: Optional[np.ndarray], seed: int, step: int, rows: Optional[Sequence[int]] = None,
           row_offset: int = 0, keep_dist: bool = False) -> list[RowResult]:
    """The whole call: ``logits[B, V]`` (float32 values) -> one RowResult per requested row.

    Rows are independent (section 5.1): each depends only on its own logits, history and
    parameters; the random numbers are keyed by ``row_offset + row`` so any partition of the
    batch gives the same ids.
    """
    B, V = logits_f32.shape
    hot_mask = hot_mask_from_ids(hot_ids, V)
    out = []
    for b in (range(B) if rows is None else rows):
        if hist_ptr is not None and hist_ids is not None:
            hr = hist_ids[int(hist_ptr[b]):int(hist_ptr[b + 1])]
        else:
            hr = None
        out.append(sample_row(logits_f32[b], params[b], hr, hot_mask, seed, row_offset + b, step,
                              keep_dist))
    return out
