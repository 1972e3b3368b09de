"""Parity harness: drives the HIP library through its C ABI and the CPU oracle side by side.

Slaved trajectory: the oracle replays the whole sequence itself, but the record / evict /
compact part of each step is fed the scores the device recorded in its ring, so both caches
stay identical and keep / indices / K' / V' / lens' are compared bit for bit at every step,
while `out` and the oracle's own fp64 scores are compared within tolerance.

Snapshot step: the oracle is rebuilt from a copy of the device state of a few units (cache
rows, positions and the ring window), computes one step, and is compared the same way.
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np
import torch

from oracle import corm_oracle as O
from oracle.snapshot import unit_from_device_arrays
from paper_2404_15949_amd import corm, inputs

OUT_TOL = {"f32": 1e-5, "bf16": 2e-3}          # max_c |delta| / max_c |ref| per output row
# recorded score vs the oracle's fp64 score: fp32 arithmetic error, plus bf16 storage rounding
SCORE_RTOL = {"f32": 2e-5, "bf16": 2.0 ** -8 + 5e-5}   # bf16 half-ulp is 2^-8 relative at worst
SCORE_ATOL_OF_MAX = {"f32": 2e-6, "bf16": 1e-5}


def out_rel_err(got: np.ndarray, ref: np.ndarray) -> float:
    return float(np.abs(got - ref).max() / max(np.abs(ref).max(), 1e-30))


def make_state(wl: inputs.Workload, device, Lcap=None, Tcap=None, thr_scale=1.0, want_masks=True,
               workspace=None, score_dtype=None) -> corm.LayerState:
    n_replay = min(wl.w, wl.P)
    Lcap = wl.P + wl.D if Lcap is None else Lcap
    Tcap = wl.P + wl.D if Tcap is None else Tcap
    return corm.LayerState(wl.B, wl.Hq, wl.Hkv, wl.d, Lcap, Tcap, wl.w, wl.r, wl.dtype, thr_scale=thr_scale,
                           device=device, workspace=workspace, want_masks=want_masks, score_dtype=score_dtype)


def ring_row(st: corm.LayerState, b: int, slot: int) -> np.ndarray:
    """Row `slot` of sequence b's ring as float32 [Hq, Tcap].  A bit ring (the boolean message) reads as
    1.0 / 0.0, which the oracle's threshold test maps back to the recorded boolean for any threshold in (0, 1]."""
    if st.ring_bits:
        words = st.ring[b, :, slot].cpu().numpy().view(np.uint32)
        bits = np.unpackbits(np.ascontiguousarray(words).view(np.uint8), axis=1, bitorder="little")
        return bits[:, :st.Tcap].astype(np.float32)
    return _f32(st.ring[b, :, slot])


def check_recorded(wl, st, recorded_g, alpha_g, t, thr_scale, where) -> float:
    """The row the device recorded for one head against the oracle's fp64 scores: within tolerance for a score
    ring; for a bit ring, equal to the oracle's own threshold test except within rounding of the threshold.
    Returns error / bound (score ring) or 0."""
    a = alpha_g
    if st.ring_bits:
        thr = float(O.importance_threshold(t, thr_scale))
        own = a >= thr
        differ = own != (recorded_g > 0.5)
        assert (np.abs(a[differ] - thr) <= 1e-4 * thr).all(), ("recorded bit", where)
        return 0.0
    err = np.abs(recorded_g.astype(np.float64) - a)
    bound = SCORE_RTOL[wl.dtype] * a + SCORE_ATOL_OF_MAX[wl.dtype] * a.max()
    assert (err <= bound).all(), ("recorded score", where, float((err / bound).max()))
    return float((err / bound).max())


def step_inputs(wl: inputs.Workload, x: Dict[str, torch.Tensor], j: int, n_replay: int):
    """q, k_new, v_new ([B,H,d], contiguous) and the absolute step t of trajectory step j."""
    P = wl.P
    if j < n_replay:
        p = P - n_replay + j
        k = x["K0"][:, :, p].contiguous()
        v = x["V0"][:, :, p].contiguous()
    else:
        p = P + (j - n_replay)
        k = x["Kn"][j - n_replay].contiguous()
        v = x["Vn"][j - n_replay].contiguous()
    return x["Q"][j].contiguous(), k, v, p + 1


def _f32(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy()


def live_slots(st: corm.LayerState, b: int, h: int) -> np.ndarray:
    """Slots of unit (b,h) below lens whose live bit is set (deferred compaction), ascending."""
    l = int(st.lens[b, h].item())
    words = st.live[b, h].cpu().numpy()
    bits = np.unpackbits(words.view(np.uint8), bitorder="little")[:l]
    return np.nonzero(bits)[0]


def check_unit_state(st: corm.LayerState, b: int, h: int, u: O.UnitCache, t: int, lazy: bool = False) -> None:
    """Device cache of unit (b,h) == the oracle's, bit for bit (rows, order, positions, lens).

    lazy: the device defers compaction; its live slots, read in slot order, must be the oracle's cache."""
    if lazy:
        sl = live_slots(st, b, h)
        assert len(sl) == u.l, (b, h, len(sl), u.l)
        assert int(st.nlive[b, h].item()) == u.l, (b, h, "nlive")
        sel = torch.from_numpy(sl).to(st.K.device)
        pos_d, K_d, V_d = st.pos[b, h].index_select(0, sel), st.K[b, h].index_select(0, sel), st.V[b, h].index_select(0, sel)
        lh_d = st.last_hit[b, h].index_select(0, sel)
        l = u.l
    else:
        l = int(st.lens[b, h].item())
        assert l == u.l, (b, h, l, u.l)
        pos_d, K_d, V_d, lh_d = st.pos[b, h, :l], st.K[b, h, :l], st.V[b, h, :l], st.last_hit[b, h, :l]
    assert np.array_equal(pos_d.cpu().numpy().astype(np.int64), u.positions), (b, h)
    Kd = _f32(K_d).astype(np.float64)
    Vd = _f32(V_d).astype(np.float64)
    assert np.array_equal(Kd, u.keys), (b, h, "K rows")
    assert np.array_equal(Vd, u.values), (b, h, "V rows")
    # last_hit summary vs the oracle's recent message
    lh = lh_d.cpu().numpy()
    msg = u.message()                                                       # [n, G, l]
    n = msg.shape[0]
    steps = np.asarray(u.note_steps, dtype=np.int64)
    assert len(steps) == n
    hit_any = msg.any(axis=1)                                               # [n, l]
    last = np.where(hit_any, steps[:, None], 0).max(axis=0) if n else np.zeros(l, dtype=np.int64)
    lo = t - st.w  # hits at steps <= t-w are outside the window
    assert np.array_equal(np.where(lh > lo, lh, 0), last), (b, h, "last_hit")


def run_slaved_trajectory(wl: inputs.Workload, device="cuda:0", layer=0, thr_scale=1.0, check_state_every=1,
                          units: Optional[Sequence[Tuple[int, int]]] = None, steps: Optional[int] = None,
                          use_split_calls=False, seq_offsets: Optional[Sequence[int]] = None,
                          Lcap: Optional[int] = None, Tcap: Optional[int] = None,
                          lazy: Optional[Tuple[int, int]] = None, seed_kernel: bool = False,
                          score_dtype: Optional[str] = None) -> Dict:
    """Run replay + decode on the device, slaving one oracle per checked unit.  Returns a report.

    seq_offsets[b]: sequence b behaves as if o_b tokens preceded its prompt (their keys already evicted):
    its positions and its step counter t are shifted by o_b, so sequences of one batch sit at different steps.

    lazy = (dead_num, dead_den): run corm_decode_step_lazy with that compaction policy; the oracle (which
    compacts at every step, as Algorithm 1 does) is compared with the device's live slots in slot order, and
    the policy itself (when a unit was compacted) is checked against its definition.

    seed_kernel: the prompt tail is not replayed step by step; the whole prompt is preloaded and one
    corm_prefill_seed call records its last min(w, P) queries.  The oracle still replays those positions as
    ordinary steps (fed the scores the device wrote into the ring), and must end in the same state."""
    x_cpu = inputs.make_layer(wl, layer, device="cpu")
    x = {k: v.to(device) for k, v in x_cpu.items() if k != "sinks"}
    n_replay = min(wl.w, wl.P)
    n_steps = n_replay + wl.D if steps is None else steps
    offs = np.zeros(wl.B, dtype=np.int64) if seq_offsets is None else np.asarray(seq_offsets, dtype=np.int64)
    offs_dev = torch.from_numpy(offs).to(device=device, dtype=torch.int32)
    st = make_state(wl, device, thr_scale=thr_scale, Lcap=Lcap,
                    Tcap=(wl.P + wl.D + int(offs.max())) if Tcap is None else Tcap, score_dtype=score_dtype)
    G = wl.G
    pre = wl.P - n_replay
    n_pre = wl.P if seed_kernel else pre
    st.preload(x["K0"][:, :, :n_pre], x["V0"][:, :, :n_pre])
    st.pos[:, :, :n_pre] += offs_dev.view(-1, 1, 1)
    units = [(b, h) for b in range(wl.B) for h in range(wl.Hkv)] if units is None else list(units)
    oracles = {}
    for (b, h) in units:
        u = O.UnitCache(wl.d, G, wl.w, wl.r, thr_scale, score_dtype=wl.dtype)
        u.preload(_f32(x_cpu["K0"][b, h, :pre]), _f32(x_cpu["V0"][b, h, :pre]), first_position=int(offs[b]))
        oracles[(b, h)] = u
    t_first = (torch.full((wl.B,), pre + 1, dtype=torch.int32, device=device) + offs_dev)
    slaves = Slaves(wl, st, oracles, units, offs, thr_scale, lazy,
                    slots_before={u: np.arange(pre) for u in units}, used_before={u: pre for u in units})
    j_first = 0
    if seed_kernel:
        assert not use_split_calls and n_steps >= n_replay
        j_first = n_replay
        slaves.worst_score = _seed_with_kernel(wl, st, x, x_cpu, oracles, units, offs, offs_dev, n_replay, t_first,
                                               thr_scale)
        slaves.evicted_total += sum(wl.P - oracles[u].l for u in units)
        for u in units:     # the seeding call leaves every unit compacted: slots 0 .. l-1 hold the live keys
            slaves.slots_before[u] = np.arange(oracles[u].l)
            slaves.used_before[u] = oracles[u].l
    for j in range(j_first, n_steps):
        q, k, v, t = step_inputs(wl, x, j, n_replay)
        t_dev = torch.full((wl.B,), t, dtype=torch.int32, device=device) + offs_dev
        if use_split_calls:
            corm.corm_append(st.desc, st.K, st.V, st.lens, st.pos, st.last_hit, k, v, t_dev, st.status)
            corm.corm_decode_attend(st.desc, q, st.K, st.V, st.lens, st.pos, t_dev, st.ring, st.last_hit, st.out,
                                    st.workspace, status=st.status)
            corm.corm_evict_mask(st.desc, st.ring, st.lens, st.pos, t_dev, t_first, st.keep)
            keep_lit = st.keep.clone()
            corm.corm_evict_mask_summary(st.desc, st.last_hit, st.lens, t_dev, t_first, st.keep)
            lens_before = st.lens.cpu().numpy()
            for (b, h) in units:
                lb = int(lens_before[b, h])
                assert torch.equal(keep_lit[b, h, :lb], st.keep[b, h, :lb]), ("literal vs summary mask", j, b, h)
            corm.corm_compact(st.desc, st.K, st.V, st.pos, st.last_hit, st.lens, st.keep, st.kept_idx, st.workspace)
        elif lazy is not None:
            st.step_lazy(q, k, v, t_dev, t_first, dead_num=lazy[0], dead_den=lazy[1])
        else:
            st.step(q, k, v, t_dev, t_first)
        slaves.after_step(j, q, k, v, t,
                          check_state=bool(check_state_every) and ((j + 1) % check_state_every == 0 or j == n_steps - 1))
    return slaves.report(n_steps)


class Slaves:
    """One oracle per checked unit, slaved to the device: after every device step each oracle takes the same
    step, fed the scores the device recorded, and is compared with what the device left (keep mask, kept
    indices, lens bit for bit; out and the recorded scores within tolerance; every importance decision that
    differs from the fp64 one within the score tolerance of c/t).  The oracles of different units are
    independent, so they step on a pool of host threads (numpy releases the interpreter lock)."""

    def __init__(self, wl, st, oracles, units, offs, thr_scale, lazy, slots_before, used_before, threads=None):
        self.wl, self.st, self.oracles, self.units, self.offs = wl, st, oracles, list(units), offs
        self.thr_scale, self.lazy = thr_scale, lazy
        self.slots_before, self.used_before = slots_before, used_before   # lazy mode: live slots / slots in use
        self.worst_out = self.worst_score = 0.0
        self.flips = self.evicted_total = self.compactions = 0
        n = min(16, os.cpu_count() or 1) if threads is None else threads
        self.pool = ThreadPoolExecutor(max_workers=n) if n > 1 and len(self.units) > 1 else None

    def after_step(self, j, q, k, v, t, check_state=True):
        wl, st, lazy, thr_scale, G = self.wl, self.st, self.lazy, self.thr_scale, self.wl.G
        torch.cuda.synchronize()
        assert int(st.status.item()) == 0, ("device status", int(st.status.item()), j)
        out = st.out.cpu().numpy()
        keep_d = st.keep.cpu().numpy()
        idx_d = st.kept_idx.cpu().numpy()
        lens_d = st.lens.cpu().numpy()
        live_d = st.live.cpu().numpy() if lazy is not None else None
        qc, kc, vc = _f32(q), _f32(k), _f32(v)
        ring_rows = {b: ring_row(st, b, (t + int(self.offs[b]) - 1) % wl.w) for b in sorted({u[0] for u in self.units})}
        tol = OUT_TOL[wl.dtype]
        cap = st.Lcap

        def one(unit):
            b, h = unit
            u = self.oracles[unit]
            tb = t + int(self.offs[b])
            live_pos = np.concatenate([u.positions, [tb - 1]])
            recorded = ring_rows[b][h * G:(h + 1) * G][:, live_pos]
            res = u.step(qc[b, h * G:(h + 1) * G], kc[b, h], vc[b, h], tb, recorded=recorded)
            l = len(live_pos)
            compacted = 0
            if lazy is None:
                assert np.array_equal(keep_d[b, h, :l].astype(bool), res["keep"]), ("keep", j, b, h)
                assert int(lens_d[b, h]) == u.l, ("lens", j, b, h, int(lens_d[b, h]), u.l)
                assert np.array_equal(idx_d[b, h, :u.l].astype(np.int64), res["indices"]), ("kept_idx", j, b, h)
            else:
                L = self.used_before[unit] + 1                                # slots in use after the append
                sl = np.concatenate([self.slots_before[unit], [L - 1]])        # slots of the oracle's keys
                kd = keep_d[b, h, :L].astype(bool)
                assert np.array_equal(kd[sl], res["keep"]), ("keep (live slots)", j, b, h)
                assert int(kd.sum()) == int(res["keep"].sum()), ("a dead slot was revived", j, b, h)
                T = u.l
                want_compact = T < L and ((L - T) * lazy[1] >= L * lazy[0] or L + 1 >= cap)
                assert int(lens_d[b, h]) == (T if want_compact else L), ("lens / policy", j, b, h, L, T)
                compacted = int(want_compact)
                bits = np.unpackbits(live_d[b, h].view(np.uint8), bitorder="little")[:int(lens_d[b, h])]
                now = np.nonzero(bits)[0]
                assert np.array_equal(now, np.arange(T) if want_compact else sl[res["keep"]]), ("live", j, b, h)
                self.slots_before[unit] = now
                self.used_before[unit] = int(lens_d[b, h])
            w_out = w_score = 0.0
            for g in range(G):
                e = out_rel_err(out[b, h * G + g].astype(np.float64), res["out"][g])
                w_out = max(w_out, e)
                assert e <= tol, ("out", j, b, h, g, e)
                w_score = max(w_score, check_recorded(wl, st, recorded[g], res["alpha"][g], tb, thr_scale, (j, b, h, g)))
            own = O.important(O.round_to_storage(res["alpha"], "f32" if st.ring_bits else wl.dtype), tb, thr_scale)
            flipped = own != O.important(recorded, tb, thr_scale)
            n_flip = 0
            if flipped.any():      # a decision may differ from the fp64 one only within the score tolerance of c/t
                a = res["alpha"]
                thr = float(O.importance_threshold(tb, thr_scale))
                bound = (np.full_like(a, 1e-4 * thr) if st.ring_bits else
                         SCORE_RTOL[wl.dtype] * a + SCORE_ATOL_OF_MAX[wl.dtype] * a.max(axis=1, keepdims=True))
                assert (np.abs(a - thr)[flipped] <= bound[flipped]).all(), ("importance flip far from c/t", j, b, h)
                n_flip = int(flipped.sum())
            return w_out, w_score, n_flip, l - u.l, compacted

        results = list(self.pool.map(one, self.units)) if self.pool else [one(u) for u in self.units]
        for w_out, w_score, n_flip, gone, compacted in results:
            self.worst_out, self.worst_score = max(self.worst_out, w_out), max(self.worst_score, w_score)
            self.flips += n_flip
            self.evicted_total += gone
            self.compactions += compacted
        if check_state:
            for (b, h) in self.units:
                check_unit_state(st, b, h, self.oracles[(b, h)], t + int(self.offs[b]), lazy=lazy is not None)

    def report(self, n_steps) -> Dict:
        if self.pool:
            self.pool.shutdown()
        return {"compactions": self.compactions, "steps": n_steps, "units": len(self.units),
                "worst_out_rel_err": self.worst_out, "worst_score_err_over_bound": self.worst_score,
                "importance_flips_vs_fp64": self.flips, "evicted_total": self.evicted_total,
                "final_lens": self.st.lens.cpu().numpy().tolist()}


def run_slaved_from_seeded_state(wl: inputs.Workload, device, layer: int, units: Sequence[Tuple[int, int]],
                                 n_decode: int, check_state_every: int = 0, lazy: Optional[Tuple[int, int]] = None,
                                 expect_path: Optional[int] = None, progress=None) -> Dict:
    """A whole decode trajectory at a workload's full size, as the benchmark runs it: inputs generated on the
    device, the whole prompt preloaded, the window seeded by one corm_prefill_seed call (checked by tests of
    its own), then n_decode fused steps on ALL units of the layer.  The oracles of the listed units are rebuilt
    from the device state after the prompt and slaved from there on, every step."""
    m = min(wl.w, wl.P)
    x = inputs.make_layer(wl, layer, device=device, n_decode=n_decode, n_replay=m)
    st = make_state(wl, device, Lcap=wl.P + n_decode, Tcap=wl.P + n_decode)
    if expect_path is not None:
        assert corm.corm_selected_path(st.desc) == expect_path
    st.preload(x["K0"], x["V0"])
    t = torch.full((wl.B,), wl.P, dtype=torch.int32, device=device)
    tf = torch.zeros_like(t)
    st.prefill_seed(x["Q"][:m].permute(1, 2, 0, 3).contiguous(), t, tf)
    torch.cuda.synchronize()
    assert int(st.status.item()) == 0
    t_first = wl.P - m + 1
    assert int(tf.min().item()) == int(tf.max().item()) == t_first
    oracles = {u: oracle_from_snapshot(st, u[0], u[1], wl.P, t_first, wl.dtype, 1.0) for u in units}
    slaves = Slaves(wl, st, oracles, units, np.zeros(wl.B, dtype=np.int64), 1.0, lazy,
                    slots_before={u: np.arange(oracles[u].l) for u in units},
                    used_before={u: oracles[u].l for u in units})
    seeded_evictions = sum(wl.P - oracles[u].l for u in units)
    for j in range(n_decode):
        q, k, v, tt = step_inputs(wl, x, m + j, m)
        t_dev = torch.full((wl.B,), tt, dtype=torch.int32, device=device)
        if lazy is not None:
            st.step_lazy(q, k, v, t_dev, tf, dead_num=lazy[0], dead_den=lazy[1])
        else:
            st.step(q, k, v, t_dev, tf)
        last = j == n_decode - 1
        slaves.after_step(j, q, k, v, tt, check_state=last or (bool(check_state_every) and (j + 1) % check_state_every == 0))
        if progress and ((j + 1) % 32 == 0 or last):
            progress(f"step {j + 1}/{n_decode}: evicted so far {slaves.evicted_total}, worst out err {slaves.worst_out:.2e}")
    rep = slaves.report(n_decode)
    rep["evicted_by_the_prompt"] = seeded_evictions
    lens = np.asarray(rep.pop("final_lens"))
    rep["final_lens_min_mean_max"] = (int(lens.min()), float(lens.mean()), int(lens.max()))
    return rep


def _seed_with_kernel(wl, st, x, x_cpu, oracles, units, offs, offs_dev, n_replay, t_first, thr_scale) -> float:
    """One corm_prefill_seed call against the oracle replaying the same prompt positions as steps."""
    dev = st.K.device
    G = wl.G
    q_tail = x["Q"][:n_replay].permute(1, 2, 0, 3).contiguous()                   # [B, Hq, m, d]
    t_dev = torch.full((wl.B,), wl.P, dtype=torch.int32, device=dev) + offs_dev
    tf_out = torch.zeros(wl.B, dtype=torch.int32, device=dev)
    st.prefill_seed(q_tail, t_dev, tf_out)
    torch.cuda.synchronize()
    assert int(st.status.item()) == 0, ("device status", int(st.status.item()))
    assert torch.equal(tf_out, t_first), "t_first"
    keep_d = st.keep.cpu().numpy()
    idx_d = st.kept_idx.cpu().numpy()
    lens_d = st.lens.cpu().numpy()
    ring_b = {b: np.stack([ring_row(st, b, sl) for sl in range(wl.w)], axis=1)            # [Hq, w, Tcap]
              for b in sorted({u[0] for u in units})}
    Qc = _f32(x_cpu["Q"][:n_replay])

    def one(unit):
        b, h = unit
        u = oracles[unit]
        worst = 0.0
        res = None
        for j in range(n_replay):
            p = wl.P - n_replay + j
            tb = p + 1 + int(offs[b])
            live_pos = np.concatenate([u.positions, [tb - 1]])
            recorded = ring_b[b][h * G:(h + 1) * G, (tb - 1) % wl.w][:, live_pos]
            res = u.step(Qc[j, b, h * G:(h + 1) * G], _f32(x_cpu["K0"][b, h, p]), _f32(x_cpu["V0"][b, h, p]), tb,
                         recorded=recorded)
            for g in range(G):
                worst = max(worst, check_recorded(wl, st, recorded[g], res["alpha"][g], tb, thr_scale,
                                                  ("seeded", j, b, h, g)))
        assert np.array_equal(keep_d[b, h, :wl.P].astype(bool), res["keep"]), ("keep after seeding", b, h)
        assert int(lens_d[b, h]) == u.l, ("lens after seeding", b, h)
        assert np.array_equal(idx_d[b, h, :u.l].astype(np.int64), res["indices"]), ("kept_idx after seeding", b, h)
        return worst

    n_threads = min(16, os.cpu_count() or 1)
    if n_threads > 1 and len(units) > 1:
        with ThreadPoolExecutor(max_workers=n_threads) as pool:
            worsts = list(pool.map(one, units))
    else:
        worsts = [one(u) for u in units]
    for (b, h) in units:
        check_unit_state(st, b, h, oracles[(b, h)], wl.P + int(offs[b]))
    return max(worsts) if worsts else 0.0


# ------------------------------------------------------------------ snapshot mode

def oracle_from_snapshot(st: corm.LayerState, b: int, h: int, t_prev: int, t_first: int, dtype: str,
                         thr_scale: float) -> O.UnitCache:
    """Rebuild the oracle state of unit (b,h) from device memory as it stands after step t_prev."""
    return unit_from_device_arrays(st.K, st.V, st.pos, st.lens, st.ring, b, h, st.Hq // st.Hkv, st.w, st.r,
                                   t_prev, t_first, dtype, thr_scale)


def snapshot_step_check(st: corm.LayerState, wl: inputs.Workload, q, k, v, t: int, t_first: int,
                        units: Sequence[Tuple[int, int]], thr_scale: float = 1.0) -> Dict:
    """One device step checked against oracles rebuilt from the device state just before it.

    q, k, v: this step's device inputs ([B,Hq,d], [B,Hkv,d]); the state `st` must have keep/kept_idx arrays.
    Compares, for every listed unit: keep mask, kept indices, lens', the compacted K/V/pos rows (bit for
    bit, the oracle being fed the scores the device recorded) and `out` / recorded scores within tolerance.
    """
    dev = st.K.device
    G = wl.G
    oracles = {u: oracle_from_snapshot(st, u[0], u[1], t - 1, t_first, wl.dtype, thr_scale) for u in units}
    t_dev = torch.full((wl.B,), t, dtype=torch.int32, device=dev)
    tf_dev = torch.full((wl.B,), t_first, dtype=torch.int32, device=dev)
    st.step(q, k, v, t_dev, tf_dev)
    torch.cuda.synchronize()
    assert int(st.status.item()) == 0
    slot = (t - 1) % wl.w
    tol = OUT_TOL[wl.dtype]
    worst = 0.0
    evicted = 0
    for (b, h) in units:
        u = oracles[(b, h)]
        live_pos = np.concatenate([u.positions, [t - 1]])
        pos_t = torch.from_numpy(live_pos).to(dev)
        recorded = _f32(st.ring[b, h * G:(h + 1) * G, slot].index_select(1, pos_t))
        res = u.step(_f32(q[b, h * G:(h + 1) * G]), _f32(k[b, h]), _f32(v[b, h]), t, recorded=recorded)
        l = len(live_pos)
        assert np.array_equal(st.keep[b, h, :l].cpu().numpy().astype(bool), res["keep"]), ("keep", t, b, h)
        assert int(st.lens[b, h].item()) == u.l, ("lens", t, b, h)
        assert np.array_equal(st.kept_idx[b, h, :u.l].cpu().numpy().astype(np.int64), res["indices"]), ("idx", t, b, h)
        evicted += l - u.l
        for g in range(G):
            e = out_rel_err(st.out[b, h * G + g].cpu().numpy().astype(np.float64), res["out"][g])
            worst = max(worst, e)
            assert e <= tol, ("out", t, b, h, g, e)
            a = res["alpha"][g]
            err = np.abs(recorded[g].astype(np.float64) - a)
            assert (err <= SCORE_RTOL[wl.dtype] * a + SCORE_ATOL_OF_MAX[wl.dtype] * a.max()).all(), ("score", t, b, h, g)
        check_unit_state(st, b, h, u, t)
    return {"worst_out_rel_err": worst, "evicted": evicted}
