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
* ``note_of_query``         Section 4.2 "Approach": per query, the keys it considers important.
* ``long_term_minor``       Def. 4.1, extended to a query group (Section 5.3).
* ``survivors``             the decision of Section 4.2 / Algorithm 1: window of w queries, r newest keys kept.
* ``UnitCache.step``        one step of Algorithm 1 around Eq. (1), (2): append, attend, note, decide, gather.
* ``keep_from_score_window``Def. 4.1 plus the recent-r protection, straight from a window of stored scores.
* ``stable_compact``        the ascending index list of Algorithm 1's gather.

Readings taken where the paper is silent or inconsistent (each is listed in
the design notes of this repository):

* Algorithm 1 concatenates the new message row along the *row* axis (the
  listing says dim=1, which cannot work for [m,l] and [1,l]; the row count test
  and the docstring shapes show rows are meant).
* The listing returns the message with its old column count although the cache
  has shrunk; the columns must follow the keys.  Here a note is addressed by the
  key's absolute position instead, so nothing has to follow anything.
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
reformulations, a hand-derived trace).  The paper's quality tables need its datasets and weights and
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
# Section 4.2: the recent message, Def. 4.1, the eviction decision


def stable_compact(keep: np.ndarray) -> np.ndarray:
    """Ascending slots of the kept keys (what Algorithm 1's index list holds); always 1-D."""
    return np.flatnonzero(np.asarray(keep, dtype=bool))


def note_of_query(stored_scores: np.ndarray, positions: np.ndarray, t: int, width: int,
                  c: float = 1.0) -> np.ndarray:
    """What Section 4.2 records for the query of step t: the keys it considers important.

    stored_scores [G, l] for the live keys, whose absolute positions are ``positions`` [l].
    Returns bool [G, width] over ABSOLUTE positions: True where head g found the key at that
    position important (Def. 3.1).  Every position the query did not see -- evicted earlier,
    or not yet in the sequence -- is False, i.e. minor.
    """
    found = np.zeros((stored_scores.shape[0], width), dtype=bool)
    found[:, positions] = important(stored_scores, t, c)
    return found


def long_term_minor(notes: np.ndarray, positions: np.ndarray) -> np.ndarray:
    """Def. 4.1 for every live key, extended to a query group (Section 5.3).

    notes [n, G, width]: the notes of the n most recent queries (see ``note_of_query``).
    A key is a long-term minor key iff no head of its group found it important in any of them.
    """
    found_by_someone = notes.any(axis=(0, 1))          # per absolute position: some head, in some note
    return ~found_by_someone[positions]


def survivors(notes: np.ndarray, positions: np.ndarray, w: int, r: int) -> np.ndarray:
    """The eviction decision of Section 4.2 for the live keys (ascending slots): bool [l], True = stays.

    Nothing goes before w queries have been observed.  After that a key goes as soon as it is a
    long-term minor key of the last w queries -- except the keys in the r newest slots, which stay
    whatever the notes say (too few observations of them yet).
    """
    if r < 1 or w < 1:
        raise ValueError("w and r must be >= 1")
    l = len(positions)
    if notes.shape[0] < w:
        return np.ones(l, dtype=bool)
    stays = ~long_term_minor(notes[notes.shape[0] - w:], positions)
    stays[max(l - r, 0):] = True
    return stays


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

    State: the live keys and values in slot order, the absolute position of each, and the recent
    message -- ``notes`` [n <= w, G, width], one note per observed query, oldest first, each a
    boolean table over absolute positions (``note_of_query``), with the step of each in
    ``note_steps``.  Because a note is addressed by position and not by slot, an eviction leaves
    the notes untouched: the columns of evicted keys are simply never looked at again.
    """

    def __init__(self, d: int, G: int, w: int, r: int, c: float = 1.0, score_dtype: str = "f32",
                 sm_scale: Optional[float] = None):
        self.d, self.G, self.w, self.r, self.c = d, G, w, r, float(c)
        self.score_dtype = score_dtype
        self.sm_scale = 1.0 / np.sqrt(float(d)) if sm_scale is None else float(sm_scale)
        self.keys = np.zeros((0, d), dtype=np.float64)
        self.values = np.zeros((0, d), dtype=np.float64)
        self.positions = np.zeros((0,), dtype=np.int64)
        self.notes = np.zeros((0, G, 0), dtype=bool)
        self.note_steps: List[int] = []

    @property
    def l(self) -> int:
        return self.keys.shape[0]

    def _widen_notes(self, width: int) -> None:
        """Make room for positions < width; positions no earlier query saw are minor for it."""
        n, G, have = self.notes.shape
        if width > have:
            grown = np.zeros((n, G, max(width, have + have // 4 + 64)), dtype=bool)
            grown[:, :, :have] = self.notes
            self.notes = grown

    def preload(self, keys: np.ndarray, values: np.ndarray, first_position: int = 0) -> None:
        """Bulk load of keys whose own queries are not observed (the prompt before the window)."""
        n = keys.shape[0]
        self.keys = np.concatenate([self.keys, np.asarray(keys, dtype=np.float64)], axis=0)
        self.values = np.concatenate([self.values, np.asarray(values, dtype=np.float64)], axis=0)
        self.positions = np.concatenate([self.positions, first_position + np.arange(n, dtype=np.int64)])

    def append(self, k_new: np.ndarray, v_new: np.ndarray, position: int) -> None:
        """The current token's key and value enter the cache in the next free slot."""
        self.keys = np.concatenate([self.keys, np.asarray(k_new, dtype=np.float64)[None]], axis=0)
        self.values = np.concatenate([self.values, np.asarray(v_new, dtype=np.float64)[None]], axis=0)
        self.positions = np.concatenate([self.positions, np.array([position], dtype=np.int64)])

    def attend(self, q: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
        """Eq. (2) and Eq. (1) for the G queries of the group: (alpha [G,l], out [G,d])."""
        alpha = np.stack([attention_scores(q[g], self.keys, self.sm_scale) for g in range(self.G)])
        out = np.stack([attention_output(alpha[g], self.values) for g in range(self.G)])
        return alpha, out

    def observe_and_evict(self, stored: np.ndarray, t: int) -> Tuple[np.ndarray, np.ndarray]:
        """The part of a step after attention (Algorithm 1): note what the query of step t found
        important, forget notes older than the last w, decide, and close the gaps in slot order.

        stored [G, l]: the query's scores as the record stores them.  Returns (keep [l], kept slots).
        """
        self._widen_notes(int(self.positions[-1]) + 1)
        note = note_of_query(stored, self.positions, t, self.notes.shape[2], self.c)
        self.notes = np.concatenate([self.notes, note[None]], axis=0)
        self.note_steps = self.note_steps + [t]
        if len(self.note_steps) > self.w:
            self.notes, self.note_steps = self.notes[1:], self.note_steps[1:]
        keep = survivors(self.notes, self.positions, self.w, self.r)
        slots = stable_compact(keep)
        self.keys, self.values, self.positions = self.keys[slots], self.values[slots], self.positions[slots]
        return keep, slots

    def step(self, q: np.ndarray, k_new: np.ndarray, v_new: np.ndarray, t: int,
             recorded: Optional[np.ndarray] = None):
        """One decode step at absolute step t (the query is token number t, position t-1).

        Order as in Algorithm 1: the new key is in the cache, the query attends over all l keys,
        its note is taken, the decision falls, the survivors close ranks.
        ``recorded`` ([G, l], stored values) replaces the oracle's own rounded scores as
        the input of the note / decision part (slaved-trajectory parity).
        Returns dict(out, alpha, stored, keep, indices).
        """
        self.append(k_new, v_new, t - 1)
        alpha, out = self.attend(np.asarray(q, dtype=np.float64))
        stored = round_to_storage(alpha, self.score_dtype) if recorded is None \
            else np.asarray(recorded, dtype=np.float32)
        keep, slots = self.observe_and_evict(stored, t)
        return {"out": out, "alpha": alpha, "stored": stored, "keep": keep, "indices": slots}

    def message(self) -> np.ndarray:
        """The recent message restricted to the live keys, [n, G, l] in slot order: the boolean
        matrix Algorithm 1 carries from call to call."""
        return self.notes[:, :, self.positions]


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
