"""Do the oracle's pins bite?  Each case plants ONE plausible mistake in the CPU oracle (a dropped
term, a wrong sign, index, axis, comparison or rounding), runs every pin of test_oracle_pins.py against
the broken oracle and demands that at least one of them fails.  A mutant that survives means the pins
leave that line of the oracle unchecked.  The mistakes are planted by rewriting one snippet of the
function's source text, so a mutant also fails loudly when the oracle's text changes under it.
CPU only; nothing here touches the device path."""
import inspect
import textwrap

import pytest

from oracle import corm_oracle as O
from oracle import snapshot as SNAP
from tests import test_oracle_pins as pins

PIN_PARAMS = {
    "test_keep_set_is_the_unique_subset_satisfying_the_definition": [{"G": 1}, {"G": 2}],
    "test_three_formulations_agree": [{"variant": "mha"}, {"variant": "gqa"}, {"variant": "bf16"}],
    "test_prompt_seeding_equals_the_causal_attention_matrix": [{"G": 1}, {"G": 2}],
    "test_unit_rebuilt_from_header_layout_arrays_is_the_unit_that_wrote_them":
        [{"ring_kind": "f32"}, {"ring_kind": "bf16"}, {"ring_kind": "bits"}],
}


def _pin_calls():
    calls = []
    for name, fn in sorted(vars(pins).items()):
        if not name.startswith("test_") or not callable(fn):
            continue
        if inspect.signature(fn).parameters:
            calls += [(name, fn, kw) for kw in PIN_PARAMS[name]]
        else:
            calls.append((name, fn, {}))
    return calls


def test_every_pin_is_reachable_from_here():
    names = {n for n, _, _ in _pin_calls()}
    assert len(names) >= 20 and set(PIN_PARAMS) <= names


# (where, old snippet, new snippet, what the mistake is); where = "function" or "Class.method"
MUTANTS = [
    ("attention_scores", "(keys @ q) * scale", "(keys @ q)", "Eq. 2 without the 1/sqrt(d) scale"),
    ("attention_scores", "e / e.sum()", "e / e.max()", "Eq. 2 normalised by the maximum, not the sum"),
    ("attention_scores", "np.exp(logits - logits.max())", "np.exp(logits)", "no maximum subtracted: overflow"),
    ("attention_scores", "(keys @ q) * scale", "(keys @ q[::-1]) * scale", "query components reversed"),
    ("attention_scores", "(keys @ q) * scale", "-(keys @ q) * scale", "sign of the logits"),
    ("attention_output", "np.asarray(alpha, dtype=np.float64) @", "np.asarray(alpha, dtype=np.float64)[::-1] @",
     "Eq. 1 pairs scores with the wrong values"),
    ("importance_threshold", "np.float32(c) / np.float32(t)", "np.float32(c) / np.float32(t + 1)",
     "threshold c/(t+1): 0-based step"),
    ("importance_threshold", "np.float32(np.float32(c) / np.float32(t))",
     "np.float32(np.float32(c) * np.float32(1.0 / t))", "reciprocal then multiply: doubly rounded"),
    ("important", ">= importance_threshold", "> importance_threshold", "strict compare in Def. 3.1"),
    ("important_fraction", "float(imp.mean())", "float(1.0 - imp.mean())", "share of minor, not important, keys"),
    ("stable_compact", "np.flatnonzero(np.asarray(keep, dtype=bool))",
     "np.flatnonzero(np.asarray(keep, dtype=bool))[::-1]", "kept indices in descending order"),
    ("note_of_query", "np.zeros((stored_scores.shape[0], width), dtype=bool)",
     "np.ones((stored_scores.shape[0], width), dtype=bool)",
     "a key counts as important to the queries that never saw it"),
    ("note_of_query", "important(stored_scores, t, c)", "important(stored_scores, len(positions), c)",
     "threshold from the live length instead of the step"),
    ("note_of_query", "found[:, positions] =", "found[:, np.arange(len(positions))] =",
     "note addressed by slot, not by position: wrong after the first eviction"),
    ("long_term_minor", "notes.any(axis=(0, 1))", "notes.any(axis=0).all(axis=0)", "group rule: AND over the heads instead of OR"),
    ("long_term_minor", "notes.any(axis=(0, 1))", "notes[-1:].any(axis=(0, 1))", "only the current query decides"),
    ("long_term_minor", "notes.any(axis=(0, 1))", "notes[:-1].any(axis=(0, 1))", "current query left out"),
    ("long_term_minor", "return ~found_by_someone[positions]", "return found_by_someone[positions]",
     "the important keys are evicted"),
    ("long_term_minor", "return ~found_by_someone[positions]", "return ~found_by_someone[:len(positions)]",
     "notes read by slot, not by position"),
    ("survivors", "notes.shape[0] < w", "notes.shape[0] <= w", "first eviction one step late"),
    ("survivors", "notes.shape[0] < w", "notes.shape[0] < w - 1", "first eviction one step early"),
    ("survivors", "notes[notes.shape[0] - w:]", "notes[notes.shape[0] - w + 1:]", "window of w-1 queries"),
    ("survivors", "stays[max(l - r, 0):] = True", "stays[max(l - r - 1, 0):] = True", "r+1 recent slots protected"),
    ("survivors", "stays[max(l - r, 0):] = True", "stays[max(l - r + 1, 0):] = True", "r-1 recent slots protected"),
    ("survivors", "stays[max(l - r, 0):] = True", "stays[:r] = True", "oldest, not newest, slots protected"),
    ("survivors", "stays[max(l - r, 0):] = True", "pass", "no recent protection"),
    ("UnitCache.observe_and_evict", "if len(self.note_steps) > self.w:", "if len(self.note_steps) > self.w + 1:",
     "window holds w+1 notes"),
    ("UnitCache.observe_and_evict", "self.notes[1:], self.note_steps[1:]", "self.notes[:-1], self.note_steps[:-1]",
     "the newest note is dropped instead of the oldest"),
    ("UnitCache.observe_and_evict", "self.keys[slots], self.values[slots], self.positions[slots]",
     "self.keys[slots], self.values, self.positions[slots]", "values not gathered"),
    ("UnitCache.observe_and_evict", "self.keys[slots], self.values[slots], self.positions[slots]",
     "self.keys[slots], self.values[slots], self.positions", "positions not gathered"),
    ("UnitCache._widen_notes", "grown[:, :, :have] = self.notes", "pass", "older notes lost when the table grows"),
    ("UnitCache.step", "self.append(k_new, v_new, t - 1)", "self.append(k_new, v_new, t)",
     "position of the new key off by one"),
    ("UnitCache.step", "if recorded is None", "if True", "fed scores ignored"),
    ("UnitCache.message", "self.notes[:, :, self.positions]", "self.notes[:, :, :self.l]",
     "message read by slot instead of by position"),
    ("keep_from_score_window", "important(scores[j], tj, c)", "important(scores[j], row_steps[-1], c)",
     "every row thresholded with the current step"),
    ("keep_from_score_window", "scores = scores[-w:]", "scores = scores[:w]", "oldest w rows instead of newest"),
    ("keep_from_score_window", "if m < w:", "if m <= w:", "window counted full one row late"),
    ("keep_from_score_window", "keep[-r:] = True", "keep[-(r + 1):] = True", "r+1 recent slots protected"),
    ("keep_from_score_window", ".any(axis=0)", ".all(axis=0)", "group rule: AND over the heads"),
    ("round_to_bf16", "(bits + np.uint64(0x7FFF) + lsb)", "(bits)", "truncation instead of round-to-nearest"),
    ("round_to_bf16", "(bits + np.uint64(0x7FFF) + lsb)", "(bits + np.uint64(0x8000))", "ties away from zero"),
    ("round_to_storage", "s = round_to_bf16(s)", "pass", "bf16 ring not rounded"),
    ("round_to_storage", "astype(np.float32)", "astype(np.float16).astype(np.float32)", "scores stored through fp16"),
    ("UnitCache.attend", "attention_scores(q[g], self.keys, self.sm_scale)",
     "attention_scores(q[0], self.keys, self.sm_scale)", "every head of the group uses the first head's query"),
    ("UnitCache.attend", "attention_output(alpha[g], self.values)", "attention_output(alpha[g], self.keys)",
     "output mixes keys instead of values"),
    ("UnitCache.preload", "first_position + np.arange(n, dtype=np.int64)",
     "first_position + 1 + np.arange(n, dtype=np.int64)", "prompt positions 1-based"),
    ("seed_from_prompt", "p + 1, recorded=rec", "p, recorded=rec", "prompt step numbers 0-based"),
    ("seed_from_prompt", "unit.preload(K0[:P - n], V0[:P - n], 0)", "unit.preload(K0[:P - n], V0[:P - n], 0)\n"
     "    n = n - 1", "last prompt query not recorded"),
    # rebuilding a unit from plain arrays (oracle/snapshot.py)
    ("snapshot:unit_from_device_arrays", "row = sc_all[:, (tau - 1) % w]", "row = sc_all[:, tau % w]",
     "ring slot of a step off by one"),
    ("snapshot:unit_from_device_arrays", "born = u.positions <= tau - 1", "born = u.positions < tau - 1",
     "a step's own key counts as not yet there"),
    ("snapshot:unit_from_device_arrays", "born = u.positions <= tau - 1", "born = u.positions <= tau",
     "the next step's key counts as already there"),
    ("snapshot:unit_from_device_arrays", "& born[None, :]", "", "junk in columns of keys not yet born is believed"),
    ("snapshot:unit_from_device_arrays", "pos_t >> 5", "pos_t >> 4", "wrong word of the bit ring"),
    ("snapshot:unit_from_device_arrays", "(pos_t & 31)", "(pos_t & 15)", "wrong bit of the word"),
    ("snapshot:unit_from_device_arrays", "max(t_first, t_prev - w + 1)", "max(t_first, t_prev - w)",
     "window of w+1 rows"),
    ("snapshot:unit_from_device_arrays", "max(t_first, t_prev - w + 1)", "max(1, t_prev - w + 1)",
     "rows from before the first recorded step"),
    ("snapshot:unit_from_device_arrays", "O.important(row, tau, thr_scale)", "O.important(row, t_prev, thr_scale)",
     "every row thresholded with the latest step"),
    ("snapshot:unit_from_device_arrays", "ring[b, h * G:(h + 1) * G].index_select(2, pos_t))",
     "ring[b, h:h + G].index_select(2, pos_t))", "query heads of the wrong group (score ring)"),
    ("snapshot:unit_from_device_arrays", "ring[b, h * G:(h + 1) * G].index_select(2, pos_t >> 5)",
     "ring[b, h:h + G].index_select(2, pos_t >> 5)", "query heads of the wrong group (bit ring)"),
    ("snapshot:unit_from_device_arrays", "u.keys = _f32(K[b, h, :l])", "u.keys = _f32(K[h, b, :l])",
     "sequence and head swapped"),
    ("snapshot:unit_from_device_arrays", "u.values = _f32(V[b, h, :l])", "u.values = _f32(K[b, h, :l])",
     "values read from the key array"),
]


def _mutated(where, old, new):
    """Returns (owner, attribute name, original, replacement) with one snippet of the source rewritten."""
    mod = O
    if ":" in where:
        mod, where = SNAP, where.split(":")[1]
    owner, name = (mod, where) if "." not in where else (getattr(mod, where.split(".")[0]), where.split(".")[1])
    orig = inspect.getattr_static(owner, name)
    src = textwrap.dedent(inspect.getsource(orig))
    assert src.count(old) == 1, f"{where}: snippet {old!r} occurs {src.count(old)} times: the oracle's text changed"
    ns = {}
    exec(compile(src.replace(old, new), f"<mutant of {where}>", "exec"), vars(mod), ns)   # module globals, own locals
    return owner, name, orig, ns[name]


@pytest.mark.filterwarnings("ignore::RuntimeWarning")
@pytest.mark.parametrize("where,old,new,what", MUTANTS, ids=[f"{m[0]}:{m[3]}" for m in MUTANTS])
def test_planted_mistake_is_caught_by_a_pin(where, old, new, what):
    owner, name, orig, repl = _mutated(where, old, new)
    caught = []
    setattr(owner, name, repl)
    try:
        for pin_name, fn, kw in _pin_calls():
            try:
                fn(**kw)
            except Exception:          # an assertion, or the broken oracle tripping over itself
                caught.append(pin_name)
    finally:
        setattr(owner, name, orig)
    assert caught, f"no pin notices: {what} ({where}: {old!r} -> {new!r})"
