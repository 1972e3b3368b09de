"""Parity harness: drives the HIP library through its C ABI and the CPU oracle side by side.

Slaved trajectory: the oracle replays the whole sequence itself, but the record / evict /
compact part of each step is fed the scores the device recorded in its ring, so both caches
stay identical and keep / indices / K' / V' / lens' are compared bit for bit at every step,
while `out` and the oracle's own fp64 scores are compared within tolerance.

Snapshot step: the oracle is rebuilt from a copy of the device state of a few units (cache
rows, positions and the ring window), computes one step, and is compared the same way.
"""
from __future__ import annotations

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
    tol = OUT_TOL[wl.dtype]
    worst_out = 0.0
    worst_score = 0.0
    flips = 0
    evicted_total = 0
    compactions = 0
    cap = st.Lcap
    slots_before = {u: np.arange(pre) for u in units}     # lazy mode: live slots and slots in use before a step
    used_before = {u: pre for u in units}
    j_first = 0
    if seed_kernel:
        assert not use_split_calls and n_steps >= n_replay
        j_first = n_replay
        worst_score = _seed_with_kernel(wl, st, x, x_cpu, oracles, units, offs, offs_dev, n_replay, t_first, thr_scale)
        evicted_total += sum(wl.P - oracles[u].l for u in units)
        for u in units:     # the seeding call leaves every unit compacted: slots 0 .. l-1 hold the live keys
            slots_before[u] = np.arange(oracles[u].l)
            used_before[u] = oracles[u].l
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
        torch.cuda.synchronize()
        assert int(st.status.item()) == 0, ("device status", int(st.status.item()), j)
        ring_all = st.ring
        out = st.out.cpu().numpy()
        keep_d = st.keep.cpu().numpy()
        idx_d = st.kept_idx.cpu().numpy()
        lens_d = st.lens.cpu().numpy()
        qc, kc, vc = _f32(q), _f32(k), _f32(v)
        ring_rows = {}
        for (b, h) in units:
            u = oracles[(b, h)]
            tb = t + int(offs[b])
            if b not in ring_rows:
                ring_rows[b] = ring_row(st, b, (tb - 1) % wl.w)              # [Hq, Tcap]
            live_pos = np.concatenate([u.positions, [tb - 1]])
            recorded = ring_rows[b][h * G:(h + 1) * G][:, live_pos]
            res = u.step(qc[b, h * G:(h + 1) * G], kc[b, h], vc[b, h], tb, recorded=recorded)
            l = len(live_pos)
            if lazy is None:
                assert np.array_equal(keep_d[b, h, :l].astype(bool), res["keep"]), ("keep", j, b, h)
                assert int(lens_d[b, h]) == u.l, ("lens", j, b, h, int(lens_d[b, h]), u.l)
                assert np.array_equal(idx_d[b, h, :u.l].astype(np.int64), res["indices"]), ("kept_idx", j, b, h)
            else:
                L = used_before[(b, h)] + 1                                   # slots in use after the append
                sl = np.concatenate([slots_before[(b, h)], [L - 1]])           # slots of the oracle's keys
                kd = keep_d[b, h, :L].astype(bool)
                assert np.array_equal(kd[sl], res["keep"]), ("keep (live slots)", j, b, h)
                assert int(kd.sum()) == int(res["keep"].sum()), ("a dead slot was revived", j, b, h)
                T = u.l
                want_compact = T < L and ((L - T) * lazy[1] >= L * lazy[0] or L + 1 >= cap)
                assert int(lens_d[b, h]) == (T if want_compact else L), ("lens / policy", j, b, h, L, T)
                compactions += int(want_compact)
                now = live_slots(st, b, h)
                assert np.array_equal(now, np.arange(T) if want_compact else sl[res["keep"]]), ("live", j, b, h)
                slots_before[(b, h)] = now
                used_before[(b, h)] = int(lens_d[b, h])
            evicted_total += l - u.l
            for g in range(G):
                e = out_rel_err(out[b, h * G + g].astype(np.float64), res["out"][g])
                worst_out = max(worst_out, e)
                assert e <= tol, ("out", j, b, h, g, e)
                worst_score = max(worst_score, check_recorded(wl, st, recorded[g], res["alpha"][g], tb, thr_scale,
                                                              (j, b, h, g)))
            own = O.important(O.round_to_storage(res["alpha"], "f32" if st.ring_bits else wl.dtype), tb, thr_scale)
            flipped = own != O.important(recorded, tb, thr_scale)
            if flipped.any():      # a decision may differ from the fp64 one only within the score tolerance of c/t
                a = res["alpha"]
                thr = float(O.importance_threshold(tb, thr_scale))
                bound = (np.full_like(a, 1e-4 * thr) if st.ring_bits else
                         SCORE_RTOL[wl.dtype] * a + SCORE_ATOL_OF_MAX[wl.dtype] * a.max(axis=1, keepdims=True))
                assert (np.abs(a - thr)[flipped] <= bound[flipped]).all(), ("importance flip far from c/t", j, b, h)
                flips += int(flipped.sum())
            if check_state_every and ((j + 1) % check_state_every == 0 or j == n_steps - 1):
                check_unit_state(st, b, h, u, tb, lazy=lazy is not None)
    return {"compactions": compactions, "steps": n_steps, "units": len(units), "worst_out_rel_err": worst_out,
            "worst_score_err_over_bound": worst_score, "importance_flips_vs_fp64": flips,
            "evicted_total": evicted_total, "final_lens": st.lens.cpu().numpy().tolist()}


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
    worst = 0.0
    keep_d = st.keep.cpu().numpy()
    idx_d = st.kept_idx.cpu().numpy()
    ring_b = {}
    for (b, h) in units:
        u = oracles[(b, h)]
        if b not in ring_b:
            ring_b[b] = np.stack([ring_row(st, b, sl) for sl in range(wl.w)], axis=1)   # [Hq, w, Tcap]
        res = None
        for j in range(n_replay):
            p = wl.P - n_replay + j
            tb = p + 1 + int(offs[b])
            live_pos = np.concatenate([u.positions, [tb - 1]])
            recorded = ring_b[b][h * G:(h + 1) * G, (tb - 1) % wl.w][:, live_pos]
            res = u.step(_f32(x_cpu["Q"][j, b, h * G:(h + 1) * G]), _f32(x_cpu["K0"][b, h, p]),
                         _f32(x_cpu["V0"][b, h, p]), tb, recorded=recorded)
            for g in range(G):
                worst = max(worst, check_recorded(wl, st, recorded[g], res["alpha"][g], tb, thr_scale,
                                                  ("seeded", j, b, h, g)))
        assert np.array_equal(keep_d[b, h, :wl.P].astype(bool), res["keep"]), ("keep after seeding", b, h)
        assert int(st.lens[b, h].item()) == u.l, ("lens after seeding", b, h)
        assert np.array_equal(idx_d[b, h, :u.l].astype(np.int64), res["indices"]), ("kept_idx after seeding", b, h)
        check_unit_state(st, b, h, u, wl.P + int(offs[b]))
    return worst


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
