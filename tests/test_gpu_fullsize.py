"""Parity at the benchmark definition's full per-layer sizes, in the launch configuration bench.py times:
the device runs every unit; a sample of units is checked against oracles rebuilt from the device state
(snapshot mode), step by step, bit for bit on masks / indices / cache rows and within tolerance on out."""
import sys

import numpy as np
import pytest
import torch

from paper_2404_15949_amd import corm, inputs
from tests import harness

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
W = inputs.WORKLOADS


def say(*a):
    print("[case]", *a, flush=True)
    sys.stdout.flush()


def _run(wl, layer, n_decode, check_steps, units, expect_path=None, expect_evictions=False, seed_kernel=False):
    say("full size", wl.name, "layer", layer, "B", wl.B, "Hq/Hkv", wl.Hq, wl.Hkv, "P", wl.P, "w", wl.w,
        "q_mean", bool(wl.q_mean_scales))
    n_replay = min(wl.w, wl.P)
    x = inputs.make_layer(wl, layer, device=DEV, n_decode=n_decode, n_replay=n_replay)
    st = harness.make_state(wl, DEV, Lcap=wl.P + n_decode, Tcap=wl.P + n_decode)
    if expect_path is not None:
        assert corm.corm_selected_path(st.desc) == expect_path
    pre = wl.P - n_replay
    tf = torch.full((wl.B,), pre + 1, dtype=torch.int32, device=DEV)
    if seed_kernel:
        # as bench.py sets up: the whole prompt preloaded, its last w queries recorded by one dense call
        st.preload(x["K0"], x["V0"])
        tf_out = torch.zeros_like(tf)
        st.prefill_seed(x["Q"][:n_replay].permute(1, 2, 0, 3).contiguous(),
                        torch.full((wl.B,), wl.P, dtype=torch.int32, device=DEV), tf_out)
        assert torch.equal(tf_out, tf)
        first = n_replay
    else:
        st.preload(x["K0"][:, :, :pre], x["V0"][:, :, :pre])
        # the prompt tail: all but its last position unchecked (the last one carries the bulk eviction)
        for j in range(n_replay - 1):
            q, k, v, t = harness.step_inputs(wl, x, j, n_replay)
            st.step(q, k, v, torch.full((wl.B,), t, dtype=torch.int32, device=DEV), tf)
        first = n_replay - 1
    torch.cuda.synchronize()
    assert int(st.status.item()) == 0
    total_evicted = 0
    worst = 0.0
    for j in range(first, n_replay + n_decode):
        q, k, v, t = harness.step_inputs(wl, x, j, n_replay)
        if j in check_steps or j == first:
            rep = harness.snapshot_step_check(st, wl, q, k, v, t, pre + 1, units)
            total_evicted += rep["evicted"]
            worst = max(worst, rep["worst_out_rel_err"])
            say("step", j, "t", t, rep)
        else:
            st.step(q, k, v, torch.full((wl.B,), t, dtype=torch.int32, device=DEV), tf)
    torch.cuda.synchronize()
    assert int(st.status.item()) == 0
    lens = st.lens.cpu().numpy()
    say("final live fraction", float(lens.mean()) / (wl.P + n_decode), "min", int(lens.min()), "max", int(lens.max()))
    if expect_evictions:
        assert total_evicted > 0 and lens.min() < wl.P
    return lens


def _sample_units(wl, n, seed=0):
    rng = np.random.default_rng(seed)
    return sorted({(int(rng.integers(wl.B)), int(rng.integers(wl.Hkv))) for _ in range(n)})


def test_config2_llama7b_one_layer():
    wl = W["llama7b_1layer"]
    n_replay = wl.w
    _run(wl, 0, 6, {n_replay, n_replay + 3, n_replay + 5}, _sample_units(wl, 10), expect_path=1)


@pytest.mark.parametrize("layer", [0, 2])
def test_config3_llama7b_batch16_layer(layer):
    """One dense (0) and one sparse (2) layer of the full stack; the launch is exactly the one bench.py times."""
    wl = W["llama7b_b16"]
    n_replay = wl.w
    _run(wl, layer, 5, {n_replay, n_replay + 4}, _sample_units(wl, 12, seed=layer), expect_path=2)


def test_config3_as_the_bench_runs_it():
    """Seeded by corm_prefill_seed (the bench's set-up), then exact decode steps on the fused unit kernel."""
    wl = W["llama7b_b16"]
    n_replay = wl.w
    _run(wl, 5, 4, {n_replay, n_replay + 3}, _sample_units(wl, 4, seed=12), expect_path=2, seed_kernel=True)
    _run(wl.replace(q_mean_scales=inputs.STRUCTURED_Q_MEAN), 3, 4, {n_replay, n_replay + 3},
         _sample_units(wl, 4, seed=13), expect_path=2, expect_evictions=True, seed_kernel=True)


def test_config3_structured_queries_evict_and_compact():
    """Same shape with per-head query means: heads diverge (live fraction ~0.3-0.97), every step evicts,
    the bulk eviction at the end of the prompt takes the serial compaction path, decode steps the parallel one."""
    wl = W["llama7b_b16"].replace(q_mean_scales=inputs.STRUCTURED_Q_MEAN)
    n_replay = wl.w
    lens = _run(wl, 2, 6, {n_replay, n_replay + 1, n_replay + 5}, _sample_units(wl, 12, seed=5), expect_path=2,
                expect_evictions=True)
    assert lens.max() - lens.min() > 1000


def test_config4_long_context():
    wl = W["long32k"]
    n_replay = wl.w
    _run(wl, 0, 3, {n_replay + 2}, [(0, 0), (3, 31)], expect_path=1)


def test_config5_gqa():
    wl = W["gqa_llama3"]
    n_replay = wl.w
    _run(wl, 0, 4, {n_replay, n_replay + 3}, _sample_units(wl, 6), expect_path=1)


def test_config5_gqa_structured_evicts():
    wl = W["gqa_llama3"].replace(q_mean_scales=(3.0, 5.0), key_scale=1.5)
    n_replay = wl.w
    _run(wl, 0, 4, {n_replay, n_replay + 3}, _sample_units(wl, 6, seed=2), expect_path=1, expect_evictions=True)


def _all_units(wl):
    return [(b, h) for b in range(wl.B) for h in range(wl.Hkv)]


def test_config3_every_unit_of_a_layer():
    """All 512 units of one layer of the eviction-heavy variant at three decode steps after the prompt
    (oracles rebuilt from the device state before each, one per unit): ragged
    lengths, evictions and compaction in every corner of the launch, not only in a sample."""
    wl = W["llama7b_b16"].replace(q_mean_scales=inputs.STRUCTURED_Q_MEAN)
    n_replay = wl.w
    _run(wl, 2, 3, {n_replay, n_replay + 1, n_replay + 2}, _all_units(wl), expect_path=2, expect_evictions=True,
         seed_kernel=True)


def test_config3_literal_generator_many_units():
    """The headline workload itself (literal generator, nothing evicted): 128 of the 512 units at two steps."""
    wl = W["llama7b_b16"]
    n_replay = wl.w
    _run(wl, 7, 2, {n_replay + 1}, _all_units(wl)[1::4], expect_path=2, seed_kernel=True)


def test_config5_gqa_every_unit():
    """All 128 units of the grouped-query workload (MFMA attend kernel), eviction-heavy variant, one step."""
    wl = W["gqa_llama3"].replace(q_mean_scales=(3.0, 5.0), key_scale=1.5)
    _run(wl, 0, 1, set(), _all_units(wl), expect_path=1, expect_evictions=True, seed_kernel=True)


def test_config4_long_context_more_units():
    """16 of the 128 units of the 32k-token workload, one step after the seeded prompt."""
    wl = W["long32k"]
    _run(wl, 0, 1, set(), _all_units(wl)[3::8], expect_path=1, seed_kernel=True)


# ------------------------------------------------------------------ whole trajectories at full size

def _report(name, rep):
    say(name, {k: v for k, v in rep.items() if k != "final_lens"})


@pytest.mark.parametrize("half", [0, 1])
def test_config2_whole_trajectory_every_unit(half):
    """llama7b_1layer exactly as defined; the window seeded from the 4096-token prompt by the dense call, the
    oracles replaying its last 1024 positions as steps of Algorithm 1 on the scores the call recorded; then
    all 256 decode steps on the split path, every unit slaved at every step (ring wrap-around from step w + 1
    on, lengths running towards Lcap).  The device runs all 32 units; the two cases slave heads 0-15 and
    16-31 (half the host work each), together every unit."""
    wl = W["llama7b_1layer"]
    st = harness.make_state(wl, DEV)
    assert corm.corm_selected_path(st.desc) == 1
    del st
    units = [(0, h) for h in range(16 * half, 16 * half + 16)]
    say("whole trajectory", wl, "units", units)
    rep = harness.run_slaved_trajectory(wl, DEV, check_state_every=64, seed_kernel=True, units=units)
    _report("config 2", rep)
    assert rep["steps"] == wl.w + wl.D and rep["units"] == 16


@pytest.mark.parametrize("variant", ["literal", "structured"])
def test_config3_whole_decode_trajectory_of_a_sparse_layer(variant):
    """One sparse layer of llama7b_b16 over all 512 decode steps, in the launch configuration the benchmark
    times (fused unit kernel, all 512 units on the device); 16 units, spread over sequences and the four
    head classes, are slaved at every step.  Literal generator (nothing evicted: lengths reach Lcap) and the
    eviction-heavy variant (heads diverge, compaction at every step)."""
    wl = W["llama7b_b16"]
    if variant == "structured":
        wl = wl.replace(q_mean_scales=inputs.STRUCTURED_Q_MEAN)
    units = [(b, (5 * b + 3) % wl.Hkv) for b in range(wl.B)]                  # every sequence, heads of all classes
    say("whole decode trajectory", variant, wl.name, "units", units)
    rep = harness.run_slaved_from_seeded_state(wl, DEV, 2, units, wl.D, check_state_every=128, expect_path=2,
                                               progress=say)
    _report("config 3 " + variant, rep)
    assert rep["steps"] == 512 and rep["units"] == 16
    if variant == "structured":
        assert rep["evicted_total"] > 1000 and rep["final_lens_min_mean_max"][0] < 2000


def test_config3_whole_decode_trajectory_deferred_compaction():
    """The same eviction-heavy layer with corm_decode_step_lazy (dead fraction 1/4) over all 512 steps."""
    wl = W["llama7b_b16"].replace(q_mean_scales=inputs.STRUCTURED_Q_MEAN)
    units = [(b, (7 * b + 1) % wl.Hkv) for b in range(wl.B)]
    say("whole decode trajectory, deferred compaction", wl.name, "units", units)
    rep = harness.run_slaved_from_seeded_state(wl, DEV, 3, units, wl.D, check_state_every=128, lazy=(1, 4),
                                               expect_path=2, progress=say)
    _report("config 3 structured, deferred", rep)
    assert rep["evicted_total"] > 1000 and rep["compactions"] > 0


def test_config4_long_context_both_head_classes():
    """long32k: 32 of the 128 units (every sequence; even heads and odd heads, whose keys are twice as long),
    three decode steps after the seeded 32768-token prompt."""
    wl = W["long32k"]
    units = [(b, h) for b in range(wl.B) for h in (0, 1, 6, 13, 18, 23, 28, 31)]
    assert len(units) == 32 and {h % 2 for _, h in units} == {0, 1}
    say("long32k", "units", units)
    rep = harness.run_slaved_from_seeded_state(wl, DEV, 0, units, 3, check_state_every=1, expect_path=1, progress=say)
    _report("config 4", rep)


@pytest.mark.parametrize("variant", ["literal", "structured"])
def test_config5_gqa_64_decode_steps(variant):
    """gqa_llama3: 16 of the 128 units over 64 decode steps after the seeded 8192-token prompt (MFMA attend
    kernel, four query heads per unit)."""
    wl = W["gqa_llama3"]
    if variant == "structured":
        wl = wl.replace(q_mean_scales=(3.0, 5.0), key_scale=1.5)
    units = [(b, (3 * b + 1) % wl.Hkv) for b in range(wl.B)]
    say("gqa_llama3", variant, "units", units)
    rep = harness.run_slaved_from_seeded_state(wl, DEV, 0, units, 64, check_state_every=32, expect_path=1, progress=say)
    _report("config 5 " + variant, rep)
    if variant == "structured":
        assert rep["evicted_total"] > 0


# ------------------------------------------------------------------ the largest shapes the interface accepts

def test_longest_unit_the_interface_accepts():
    """One unit of fp32 d = 128 rows at the slot limit (byte offsets inside a unit are 32-bit: Lcap * 512 B
    < 2^31, i.e. 4194303 slots, 2 GiB of K and of V): the last prompt position with its bulk eviction
    (more than half of four million keys leave in one compaction) and a decode step, against an oracle
    rebuilt from the device state."""
    wl = W["tiny_f32"].replace(name="longest_unit", B=1, Hq=1, Hkv=1, d=128, P=4194301, D=2, w=4, r=4)
    n_replay = wl.w
    lens = _run(wl, 0, 2, {n_replay + 1}, [(0, 0)], expect_path=1, expect_evictions=True)
    assert 4 <= int(lens[0, 0]) < wl.P // 2


def test_most_units_the_interface_accepts():
    """65520 units (the launch grid allows 65535), short caches: the fused unit kernel with one workgroup
    per unit, first and last units included in the sample."""
    wl = W["tiny_f32"].replace(name="most_units", B=4095, Hq=16, Hkv=16, d=64, P=40, D=6, w=8, r=4)
    n_replay = wl.w
    units = sorted(set(_sample_units(wl, 40, seed=21)) | {(0, 0), (wl.B - 1, wl.Hkv - 1)})
    _run(wl, 0, 6, {n_replay, n_replay + 5}, units, expect_path=2, expect_evictions=True)


# ------------------------------------------------------------------ prompt seeding at full size

def _seed_check(wl, layer, units, rows_per_unit=5, expect_evictions=False):
    """corm_prefill_seed on the full prompt of one layer, checked on sampled units: Def. 4.1 evaluated
    literally by the oracle on the rows the kernel recorded must give the kernel's keep mask, kept
    indices, compacted rows and lens bit for bit; sampled rows of recorded scores are compared with the
    oracle's causal attention rows within tolerance."""
    from oracle import corm_oracle as O
    say("seed full size", wl.name, "layer", layer, "B", wl.B, "Hq/Hkv", wl.Hq, wl.Hkv, "P", wl.P, "w", wl.w)
    m = min(wl.w, wl.P)
    x = inputs.make_layer(wl, layer, device=DEV, n_decode=1, n_replay=m)
    st = harness.make_state(wl, DEV, Lcap=wl.P + 8, Tcap=wl.P + 8)
    st.preload(x["K0"], x["V0"])
    q_tail = x["Q"][:m].permute(1, 2, 0, 3).contiguous()
    t = torch.full((wl.B,), wl.P, dtype=torch.int32, device=DEV)
    tf = torch.zeros_like(t)
    st.prefill_seed(q_tail, t, tf)
    torch.cuda.synchronize()
    assert int(st.status.item()) == 0
    assert int(tf.min().item()) == int(tf.max().item()) == wl.P - m + 1
    G, P = wl.G, wl.P
    rng = np.random.default_rng(11)
    steps = np.arange(P - m + 1, P + 1)                      # tau_j
    evicted = 0
    for (b, h) in units:
        ring = st.ring[b, h * G:(h + 1) * G, :, :P].float().cpu().numpy()      # [G, w, P], slot-major
        scores = np.stack([ring[:, (tau - 1) % wl.w] for tau in steps])        # [m, G, P]
        born = np.arange(P)[None, :] <= (steps - 1)[:, None]                   # key visible to query j
        scores = np.where(born[:, None, :], scores, 0.0)
        keep = O.keep_from_score_window(scores, steps.tolist(), wl.w, wl.r)
        idx = O.stable_compact(keep)
        assert np.array_equal(st.keep[b, h, :P].cpu().numpy().astype(bool), keep), ("keep", b, h)
        l = int(st.lens[b, h].item())
        assert l == len(idx), ("lens", b, h, l, len(idx))
        assert np.array_equal(st.kept_idx[b, h, :l].cpu().numpy().astype(np.int64), idx), ("kept_idx", b, h)
        assert np.array_equal(st.pos[b, h, :l].cpu().numpy().astype(np.int64), idx), ("pos", b, h)
        sel = torch.from_numpy(idx).to(DEV)
        assert torch.equal(st.K[b, h, :l], x["K0"][b, h].index_select(0, sel)), ("K rows", b, h)
        assert torch.equal(st.V[b, h, :l], x["V0"][b, h].index_select(0, sel)), ("V rows", b, h)
        hit = np.stack([O.important(scores[j], int(steps[j])) for j in range(m)]).any(axis=1) & born   # [m, P]
        last = np.where(hit, steps[:, None], 0).max(axis=0)[idx]
        lh = st.last_hit[b, h, :l].cpu().numpy()
        assert np.array_equal(np.where(lh > P - wl.w, lh, 0), last), ("last_hit", b, h)
        evicted += P - l
        K64 = x["K0"][b, h].float().cpu().numpy().astype(np.float64)
        for j in sorted({0, m - 1, *rng.integers(0, m, rows_per_unit).tolist()}):
            p = P - m + j
            for g in range(G):
                a = O.attention_scores(x["Q"][j, b, h * G + g].float().cpu().numpy(), K64[:p + 1])
                err = np.abs(scores[j, g, :p + 1].astype(np.float64) - a)
                bound = harness.SCORE_RTOL[wl.dtype] * a + harness.SCORE_ATOL_OF_MAX[wl.dtype] * a.max()
                assert (err <= bound).all(), ("seeded score", b, h, j, g, float((err / bound).max()))
    say("evicted in sampled units", evicted, "of", len(units) * P)
    if expect_evictions:
        assert evicted > 0


def test_config3_prompt_seeding():
    wl = W["llama7b_b16"]
    _seed_check(wl, 2, _sample_units(wl, 6, seed=3))
    _seed_check(wl.replace(q_mean_scales=inputs.STRUCTURED_Q_MEAN), 2, _sample_units(wl, 8, seed=4),
                expect_evictions=True)


def test_config3_prompt_seeding_every_unit():
    """The bulk eviction at the end of the prompt, all 512 units of a layer of the eviction-heavy variant."""
    wl = W["llama7b_b16"].replace(q_mean_scales=inputs.STRUCTURED_Q_MEAN)
    _seed_check(wl, 4, _all_units(wl), rows_per_unit=1, expect_evictions=True)


def test_config5_prompt_seeding_gqa():
    wl = W["gqa_llama3"].replace(q_mean_scales=(3.0, 5.0), key_scale=1.5)
    _seed_check(wl, 0, _all_units(wl)[::4], rows_per_unit=2, expect_evictions=True)


def test_config4_prompt_seeding_long_context():
    wl = W["long32k"]
    _seed_check(wl, 0, [(3, 31)], rows_per_unit=3)


# ------------------------------------------------------------------ deferred compaction at full size

def test_config3_structured_lazy_steps():
    """The eviction-heavy variant of config 3 in the launch configuration `bench.py --structured --lazy-frac 1/4`
    times: window seeded by corm_prefill_seed, then corm_decode_step_lazy.  All 512 units are followed by
    oracles rebuilt from the device state after the prompt and fed the recorded scores: at every step the
    keep decision on the live slots, and at the end the live rows in slot order, last_hit and the live
    counts, must be the oracle's; dead slots stay dead; out within tolerance."""
    from oracle import corm_oracle as O
    wl = W["llama7b_b16"].replace(q_mean_scales=inputs.STRUCTURED_Q_MEAN)
    n_decode, frac = 12, (1, 4)
    m = wl.w
    say("lazy full size", wl.name, "B", wl.B, "heads", wl.Hq, "P", wl.P, "w", wl.w, "frac", frac)
    x = inputs.make_layer(wl, 2, device=DEV, n_decode=n_decode, n_replay=m)
    st = harness.make_state(wl, DEV, Lcap=wl.P + n_decode, Tcap=wl.P + n_decode)
    assert corm.corm_selected_path(st.desc) == 2
    st.preload(x["K0"], x["V0"])
    t = torch.full((wl.B,), wl.P, dtype=torch.int32, device=DEV)
    tf = torch.zeros_like(t)
    st.prefill_seed(x["Q"][:m].permute(1, 2, 0, 3).contiguous(), t, tf)
    torch.cuda.synchronize()
    units = _all_units(wl)
    t_first = wl.P - m + 1
    oracles = {u: harness.oracle_from_snapshot(st, u[0], u[1], wl.P, t_first, wl.dtype, 1.0) for u in units}
    slots = {u: np.arange(oracles[u].l) for u in units}
    used = {u: oracles[u].l for u in units}
    G = wl.G
    evicted = compactions = 0
    for j in range(n_decode):
        q, k, v, tt = harness.step_inputs(wl, x, m + j, m)
        st.step_lazy(q, k, v, torch.full((wl.B,), tt, dtype=torch.int32, device=DEV), tf, dead_num=frac[0],
                     dead_den=frac[1])
        torch.cuda.synchronize()
        assert int(st.status.item()) == 0
        for (b, h) in units:
            u = oracles[(b, h)]
            live_pos = np.concatenate([u.positions, [tt - 1]])
            pos_t = torch.from_numpy(live_pos).to(DEV)
            recorded = st.ring[b, h * G:(h + 1) * G, (tt - 1) % wl.w].index_select(1, pos_t).float().cpu().numpy()
            res = u.step(q[b, h * G:(h + 1) * G].float().cpu().numpy(), k[b, h].float().cpu().numpy(),
                         v[b, h].float().cpu().numpy(), tt, recorded=recorded)
            L = used[(b, h)] + 1
            sl = np.concatenate([slots[(b, h)], [L - 1]])
            kd = st.keep[b, h, :L].cpu().numpy().astype(bool)
            assert np.array_equal(kd[sl], res["keep"]) and int(kd.sum()) == int(res["keep"].sum()), ("keep", j, b, h)
            T = u.l
            want = T < L and ((L - T) * frac[1] >= L * frac[0] or L + 1 >= st.Lcap)
            assert int(st.lens[b, h].item()) == (T if want else L), ("lens / policy", j, b, h)
            compactions += int(want)
            evicted += len(live_pos) - T
            slots[(b, h)] = harness.live_slots(st, b, h)
            used[(b, h)] = int(st.lens[b, h].item())
            for g in range(G):
                e = harness.out_rel_err(st.out[b, h * G + g].cpu().numpy().astype(np.float64), res["out"][g])
                assert e <= harness.OUT_TOL[wl.dtype], ("out", j, b, h, g, e)
    for (b, h) in units:
        harness.check_unit_state(st, b, h, oracles[(b, h)], wl.P + n_decode, lazy=True)
    say("evicted", evicted, "compactions", compactions, "slots in use", sum(used[u] for u in units),
        "live", sum(oracles[u].l for u in units))
    assert evicted > 0


# ------------------------------------------------------------------ grouped queries on the fused unit kernel

@pytest.mark.parametrize("G", [2, 4])
@pytest.mark.parametrize("lazy", [None, (1, 4)])
def test_grouped_queries_with_many_units(G, lazy):
    """At two or more units per compute unit the grouped-query unit kernel runs its small-stage instance
    (two workgroups per compute unit): 512 units, whole trajectories of a sample of them, exact and deferred."""
    wl = W["gqa_llama3"].replace(name=f"gqa_many_units_g{G}", B=64, Hq=8 * G, Hkv=8, P=640, D=16, w=24, r=24,
                                 key_scale=1.5, q_mean_scales=(0.0, 2.0, 3.0))
    st = harness.make_state(wl, DEV)
    assert corm.corm_selected_path(st.desc) == 2
    del st
    units = sorted(set(_sample_units(wl, 24, seed=30 + G)) | {(0, 0), (wl.B - 1, wl.Hkv - 1)})
    rep = harness.run_slaved_trajectory(wl, DEV, check_state_every=5, units=units, lazy=lazy)
    say("report", G, lazy, {k: v for k, v in rep.items() if k != "final_lens"})
    assert rep["evicted_total"] > 0


@pytest.mark.parametrize("B,Hkv", [(75, 4), (65, 8), (33, 8)])
def test_unit_kernel_pairs_units_of_partial_blocks(B, Hkv):
    """The unit kernel ranks blocks of 64 units by length and pairs long with short ones; unit counts that leave
    partial blocks (38, 65 and 33 units per XCD here) and diverging lengths: every unit must still be served
    exactly once -- a unit served twice or not at all shows in its cache, checked on a sample and, for lens, on
    all units."""
    wl = W["llama7b_1layer"].replace(name=f"partial_blocks_{B}x{Hkv}", B=B, Hq=Hkv, Hkv=Hkv, P=700, D=10, w=32, r=32,
                                     key_scale=1.5, q_mean_scales=(0.0, 2.0, 3.0, 5.0))
    n_replay = wl.w
    units = sorted(set(_sample_units(wl, 30, seed=B)) | {(0, 0), (B - 1, Hkv - 1)})
    lens = _run(wl, 0, 10, {n_replay + 3, n_replay + 9}, units, expect_path=2, expect_evictions=True)
    assert lens.max() - lens.min() > 100          # ragged: the ranked order is in use
    assert (lens >= wl.r).all() and (lens <= wl.P + 10).all()
    # every unit, every step: out is rewritten and exactly one key (the step's own) is appended
    x = inputs.make_layer(wl, 0, device=DEV, n_decode=6, n_replay=n_replay)
    st = harness.make_state(wl, DEV, Lcap=wl.P + 6, Tcap=wl.P + 6)
    st.preload(x["K0"], x["V0"])
    t = torch.full((B,), wl.P, dtype=torch.int32, device=DEV)
    tf = torch.zeros_like(t)
    st.prefill_seed(x["Q"][:n_replay].permute(1, 2, 0, 3).contiguous(), t, tf)
    for j in range(6):
        q, k, v, tt = harness.step_inputs(wl, x, n_replay + j, n_replay)
        before = st.lens.clone()
        st.out.fill_(float("nan"))
        st.step(q, k, v, torch.full((B,), tt, dtype=torch.int32, device=DEV), tf)
        torch.cuda.synchronize()
        assert torch.isfinite(st.out).all(), ("a unit was not served", j)
        after = st.lens
        assert (after <= before + 1).all() and (after >= wl.r).all(), ("lens", j)
        newest = st.pos.gather(2, (after.long() - 1).unsqueeze(-1)).squeeze(-1)
        assert (newest == tt - 1).all(), ("the step's key is not the newest of every unit", j)
        second = st.pos.gather(2, (after.long() - 2).unsqueeze(-1)).squeeze(-1)
        assert (second == tt - 2).all(), ("a unit appended twice or skipped a step", j)
    assert int(st.status.item()) == 0


def test_more_query_heads_than_grid_rows():
    """131072 query heads (4096 sequences x 32 heads, 8 KV heads): more than the 65535 rows a launch grid has in
    its second dimension; seeded by the dense call, then decoded, on a sample of units."""
    wl = W["gqa_llama3"].replace(name="many_heads", B=4096, Hq=32, Hkv=8, P=40, D=6, w=8, r=4, key_scale=2.0)
    units = sorted(set(_sample_units(wl, 30, seed=41)) | {(0, 0), (wl.B - 1, wl.Hkv - 1)})
    rep = harness.run_slaved_trajectory(wl, DEV, check_state_every=2, units=units, seed_kernel=True)
    say("report", {k: v for k, v in rep.items() if k != "final_lens"})
    assert rep["evicted_total"] > 0
