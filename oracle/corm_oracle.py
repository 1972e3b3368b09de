"""CPU oracle for CORM's decode hot path.  TEST INFRASTRUCTURE ONLY.

This is a plain, slow, fp64 numpy statement of what one decode step computes:
exact softmax attention over the live keys of a per-head cache, the record of
which keys the query considers important, the long-term-minor eviction rule
over the recent-query window, and the order-preserving gather of the
survivors.  It exists to check the HIP library; it shares no code with it and
nothing in the product path may import it (only tests, the smoke check and
the benchmark's CPU-baseline leg do).

What each function follows in the paper (arXiv 2404.15949):

* ``attention_scores``      Eq. (2): normalized attention score of q_t for every cached key.
* ``attention_output``      Eq. (1): softmax(q K^T / sqrt(d_h)) V for one query.
* ``importance_threshold``  Def. 3.1: a key is important at step t iff its score >= 1/t.
* ``important``             Def. 3.1 applied to the scores as they are stored.
* ``corm_eviction``         Algorithm 1 (Section 4.2), extended to a query group (Section 5.3).
* ``keep_from_score_window``Def. 4.1 plus the recent-r protection of Section 4.2 "Approach".
* ``stable_compact``        the ``nonzero`` / gather of Algorithm 1.

Readings taken where the paper is silent or inconsistent (each is listed in
the design notes of this repository):

* Algorithm 1 concatenates the new message row along the *row* axis (the
  listing says dim=1, which cannot work for [m,l] and [1,l]; the row count test
  and the docstring shapes show rows are meant).
* After the gather the message columns are gathered with the same indices,
  otherwise the next call's shapes do not match.
* ``t`` is the 1-based position of the current query in its sequence (tokens
  seen so far), not the live cache length.
* The comparison is inclusive (>=), done in fp32 on the score as stored, against
  fp32(c) / fp32(t) with IEEE round-to-nearest division; c = 1 is the paper's rule.
* Keys that did not exist when a message row was recorded count as minor in it.
* Grouped-query attention: a key is discarded only if every query head of its
  group considered it minor in every recorded row of the window.
* ``r >= 1`` is required (``decision[-0:]`` would protect everything).

Parity status: every function here is pinned by tests/test_oracle_pins.py
(closed forms, library softmax, brute-force subset enumeration, independent
reformulations).  The paper's quality tables need its datasets and weights and
are not reproduced: those numbers are "parity unpinned".
"""
from __future__ import annotations

from typing import List, Optional, Sequence, Tuple

import numpy as np

# --------------------------------------------------------------------------
# storage formats


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bfloat16 (ties to even); returns fp32 holding bf16 values."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    bits = x.view(np.uint32).astype(np.uint64)
    lsb = (bits >> np.uint64(16)) & np.uint64(1)
    rounded = (bits + np.uint64(0x7FFF) + lsb) & np.uint64(0xFFFF0000)
    out = rounded.astype(np.uint32).view(np.float32).reshape(x.shape)
    nan = np.isnan(x)
    if nan.any():
        out = np.where(nan, x, out)
    return out


def round_to_storage(alpha: np.ndarray, dtype: str) -> np.ndarray:
    """Scores as the recent-message record stores them: fp64 -> fp32 (RNE), then bf16 (RNE) if asked."""
    s = np.asarray(alpha, dtype=np.float64).astype(np.float32)
    if dtype == "bf16":
        s = round_to_bf16(s)
    elif dtype != "f32":
        raise ValueError(f"unknown score dtype {dtype!r}")
    return s


# --------------------------------------------------------------------------
# Eq. (1), Eq. (2)


def attention_scores(q: np.ndarray, keys: np.ndarray, sm_scale: Optional[float] = None) -> np.ndarray:
    """Eq. (2): alpha_{t,i} = exp(q k_i^T / sqrt(d)) / sum_j exp(q k_j^T / sqrt(d)), over the cached keys."""
    q = np.asarray(q, dtype=np.float64)
    keys = np.asarray(keys, dtype=np.float64)
    d = q.shape[-1]
    scale = 1.0 / np.sqrt(float(d)) if sm_scale is None else float(sm_scale)
    logits = (keys @ q) * scale
    e = np.exp(logits - logits.max())
    return e / e.sum()


def attention_output(alpha: np.ndarray, values: np.ndarray) -> np.ndarray:
    """Eq. (1) for one query: the score-weighted sum of the cached values."""
    return np.asarray(alpha, dtype=np.float64) @ np.asarray(values, dtype=np.float64)


# --------------------------------------------------------------------------
# Def. 3.1


def importance_threshold(t: int, c: float = 1.0) -> np.float32:
    """Def. 3.1 threshold c/t in fp32 (c = 1 in the paper)."""
    return np.float32(np.float32(c) / np.float32(t))


def important(stored_scores: np.ndarray, t: int, c: float = 1.0) -> np.ndarray:
    """Def. 3.1: important iff stored score >= c/t (fp32 compare, NaN counts as minor)."""
    return np.asarray(stored_scores, dtype=np.float32) >= importance_threshold(t, c)


def important_fraction(stored_scores: np.ndarray, t: int, c: float = 1.0) -> float:
    """Share of the live keys a query finds important (Def. 3.1): the per-head quantity behind the
    sparsity figures of Section 3 (1 - this value is the share of minor keys).  Empty cache: 0."""
    imp = important(stored_scores, t, c)
    return float(imp.mean()) if imp.size else 0.0


# --------------------------------------------------------------------------
# Algorithm 1


def stable_compact(decision: np.ndarray) -> np.ndarray:
    """Ascending indices of the kept slots (``nonzero`` of Algorithm 1); always 1-D."""
    return np.flatnonzero(np.asarray(decision, dtype=bool))


def corm_eviction(keys, values, message, attn_score, w: int, r: int, t: int, c: float = 1.0):
    """One call of Algorithm 1 for one KV head and its group of G query heads.

    keys, values : [l, d]   cache including the current token
    message      : [m, G, l-1] bool, the recorded importance rows (m <= w)
    attn_score   : [G, l]   the current step's scores *as stored* (fp32 or bf16 values)
    Returns (keys', values', message', indices) where indices are the kept old slots.
    """
    if r < 1 or w < 1:
        raise ValueError("w and r must be >= 1")
    l = keys.shape[0]
    m, G = message.shape[0], message.shape[1]
    assert message.shape[2] == l - 1 and attn_score.shape == (G, l)

    # update attention message: the new key did not exist in older rows -> minor there
    message = np.concatenate([message, np.zeros((m, G, 1), dtype=bool)], axis=2)
    cur_message = important(attn_score, t, c)
    message = np.concatenate([message, cur_message[None]], axis=0)[-w:]

    if message.shape[0] < w:
        return keys, values, message, np.arange(l)

    # long-term minor keys: minor for every head of the group in every recorded row
    decision = message.any(axis=(0, 1))
    decision[-r:] = True          # always keep the r most recent slots
    indices = stable_compact(decision)
    return keys[indices], values[indices], message[:, :, indices], indices


def keep_from_score_window(scores: np.ndarray, row_steps: Sequence[int], w: int, r: int,
                           c: float = 1.0) -> np.ndarray:
    """Def. 4.1 + recent-r protection, from a window of stored scores.

    scores    : [m, G, l] stored scores of the last m <= w recorded queries for the
                l live keys (0 where the key did not exist yet)
    row_steps : [m] the step t_j of each row (its threshold is c / t_j)
    Returns keep [l] bool.  With fewer than w rows nothing is evicted.
    """
    scores = np.asarray(scores, dtype=np.float32)
    m, _, l = scores.shape
    if m < w:
        return np.ones(l, dtype=bool)
    scores = scores[-w:]
    row_steps = list(row_steps)[-w:]
    keep = np.zeros(l, dtype=bool)
    for j, tj in enumerate(row_steps):
        keep |= important(scores[j], tj, c).any(axis=0)
    keep[-r:] = True
    return keep


# --------------------------------------------------------------------------
# Stateful per-unit cache: one KV head of one sequence in one layer


class UnitCache:
    """The cache of one KV head (with its G query heads) of one sequence.

    Holds the paper's per-head state: keys, values, the boolean message, plus the
    absolute position of every live key (for index parity with the device path).
    """

    def __init__(self, d: int, G: int, w: int, r: int, c: float = 1.0, score_dtype: str = "f32",
                 sm_scale: Optional[float] = None):
        self.d, self.G, self.w, self.r, self.c = d, G, w, r, float(c)
        self.score_dtype = score_dtype
        self.sm_scale = 1.0 / np.sqrt(float(d)) if sm_scale is None else float(sm_scale)
        self.keys = np.zeros((0, d), dtype=np.float64)
        self.values = np.zeros((0, d), dtype=np.float64)
        self.positions = np.zeros((0,), dtype=np.int64)
        self.message = np.zeros((0, G, 0), dtype=bool)
        self.row_steps: List[int] = []

    # -- bulk load without recording (prompt keys before the window starts)
    def preload(self, keys: np.ndarray, values: np.ndarray, first_position: int = 0) -> None:
        n = keys.shape[0]
        self.keys = np.concatenate([self.keys, np.asarray(keys, dtype=np.float64)], axis=0)
        self.values = np.concatenate([self.values, np.asarray(values, dtype=np.float64)], axis=0)
        self.positions = np.concatenate([self.positions, first_position + np.arange(n, dtype=np.int64)])
        m = self.message.shape[0]
        self.message = np.concatenate([self.message, np.zeros((m, self.G, n), dtype=bool)], axis=2)

    @property
    def l(self) -> int:
        return self.keys.shape[0]

    def attend(self, q: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
        """Eq. (2) and Eq. (1) for the G queries of the group: (alpha [G,l], out [G,d])."""
        alpha = np.stack([attention_scores(q[g], self.keys, self.sm_scale) for g in range(self.G)])
        out = np.stack([attention_output(alpha[g], self.values) for g in range(self.G)])
        return alpha, out

    def step(self, q: np.ndarray, k_new: np.ndarray, v_new: np.ndarray, t: int,
             recorded: Optional[np.ndarray] = None, evict: bool = True):
        """One decode step at absolute step t (the query is token number t, position t-1).

        Order as in Algorithm 1: append, attend over all l keys, record, decide, gather.
        ``recorded`` ([G, l], stored values) replaces the oracle's own rounded scores as
        the input of the record/evict part (slaved-trajectory parity).
        Returns dict(out, alpha, stored, keep, indices).
        """
        self.keys = np.concatenate([self.keys, np.asarray(k_new, dtype=np.float64)[None]], axis=0)
        self.values = np.concatenate([self.values, np.asarray(v_new, dtype=np.float64)[None]], axis=0)
        self.positions = np.concatenate([self.positions, np.array([t - 1], dtype=np.int64)])
        return self._attend_record_evict(q, t, recorded, evict)

    def _attend_record_evict(self, q, t, recorded, evict):
        alpha, out = self.attend(np.asarray(q, dtype=np.float64))
        stored = round_to_storage(alpha, self.score_dtype) if recorded is None \
            else np.asarray(recorded, dtype=np.float32)
        l = self.l
        if evict:
            keys, values, message, indices = corm_eviction(
                self.keys, self.values, self.message, stored, self.w, self.r, t, self.c)
        else:  # record only: Algorithm 1 up to and including the row append
            m = self.message.shape[0]
            message = np.concatenate([self.message, np.zeros((m, self.G, 1), dtype=bool)], axis=2)
            message = np.concatenate([message, important(stored, t, self.c)[None]], axis=0)[-self.w:]
            keys, values, indices = self.keys, self.values, np.arange(l)
        keep = np.zeros(l, dtype=bool)
        keep[indices] = True
        self.keys, self.values, self.message = keys, values, message
        self.positions = self.positions[indices]
        self.row_steps = (self.row_steps + [t])[-self.w:]
        return {"out": out, "alpha": alpha, "stored": stored, "keep": keep, "indices": indices}


def seed_from_prompt(unit: UnitCache, K0: np.ndarray, V0: np.ndarray, Qtail: np.ndarray,
                     recorded_rows: Optional[Sequence[np.ndarray]] = None):
    """Feed a prompt of P tokens, recording only its last n = len(Qtail) queries.

    The paper does not say how the message is initialised from a prompt.  Reading
    taken: the prompt is processed token by token; positions before P-n contribute
    keys only (their queries are not recorded), positions P-n..P-1 are ordinary
    steps of Algorithm 1 (step number = position + 1), so the first eviction fires
    when the w-th row is recorded.  Returns the list of per-step results.
    """
    P = K0.shape[0]
    n = Qtail.shape[0]
    unit.preload(K0[:P - n], V0[:P - n], 0)
    results = []
    for j in range(n):
        p = P - n + j
        rec = None if recorded_rows is None else recorded_rows[j]
        results.append(unit.step(Qtail[j], K0[p], V0[p], p + 1, recorded=rec))
    return results
