"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element."""
import sys

import numpy as np
import pytest
import torch

from oracle import corm_oracle as O
from paper_2404_15949_amd import corm, inputs
from tests import harness

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
W = inputs.WORKLOADS


@pytest.fixture(params=["split", "unit", "split_valu"], autouse=True)
def launch_path(request):
    """Every test runs with both ways of launching attend + record: split kernels (several workgroups
    per unit) and the fused one-workgroup-per-unit kernel."""
    corm.set_default_path({"split": 1, "unit": 2, "split_valu": 3}[request.param])
    yield request.param
    corm.set_default_path(0)


def say(*a):
    print("[case]", *a, flush=True)
    sys.stdout.flush()


# ------------------------------------------------------------------ whole trajectories, every unit, every step

TRAJ = {
    # the tiny fp32 workload exactly as defined (4 heads, d 64, P 512, D 64, w 32)
    "tiny_f32": (W["tiny_f32"], 1),
    # bf16 d128 MHA, L crosses one 512-key split boundary with a ragged tail
    "bf16_mha": (W["llama7b_1layer"].replace(B=2, Hq=4, Hkv=4, P=700, D=60, w=48, r=48), 6),
    # grouped queries on bf16: G = 4 and G = 2, G = 8
    "bf16_gqa4": (W["gqa_llama3"].replace(B=2, Hq=8, Hkv=2, P=600, D=40, w=40, r=40), 8),
    "bf16_gqa2": (W["gqa_llama3"].replace(B=1, Hq=4, Hkv=2, P=300, D=30, w=24, r=24), 8),
    "bf16_gqa8": (W["gqa_llama3"].replace(B=1, Hq=8, Hkv=1, P=530, D=20, w=4, r=4, key_scale=2.0), 8),
    # other row geometries: fp32 d128 (512-byte rows), bf16 d64 (128-byte rows)
    "f32_d128": (W["tiny_f32"].replace(d=128, Hq=2, Hkv=2, P=540, D=30, w=24, r=24), 6),
    "bf16_d64": (W["llama7b_1layer"].replace(B=1, Hq=2, Hkv=2, d=64, P=520, D=30, w=24, r=24), 6),
    "f32_gqa4": (W["tiny_f32"].replace(Hq=4, Hkv=1, P=200, D=30, w=16, r=16), 6),
    # r < w: keys may be evicted while younger than the window; r > w
    "r_lt_w": (W["tiny_f32"].replace(P=128, D=40, w=24, r=3), 1),
    "r_gt_w": (W["tiny_f32"].replace(P=128, D=40, w=8, r=40), 1),
    # key-norm mixes of the other workloads at reduced size
    "sparse_layer": (W["llama7b_b16"].replace(layers=3, B=2, Hq=2, Hkv=2, P=600, D=30, w=32, r=32), 6),
    "odd_head_x2": (W["long32k"].replace(B=1, Hq=4, Hkv=4, P=1100, D=30, w=64, r=64), 10),
    # structured queries: heads diverge in length
    "structured": (W["llama7b_1layer"].replace(B=1, Hq=4, Hkv=4, P=1200, D=40, w=96, r=96,
                                               q_mean_scales=inputs.STRUCTURED_Q_MEAN), 10),
}


@pytest.mark.parametrize("name", list(TRAJ))
def test_slaved_trajectory(name):
    wl, every = TRAJ[name]
    layer = 2 if name == "sparse_layer" else 0
    say("trajectory", name, wl)
    rep = harness.run_slaved_trajectory(wl, DEV, layer=layer, check_state_every=every)
    say("report", name, {k: v for k, v in rep.items() if k != "final_lens"})
    if name not in ("r_gt_w",):
        assert rep["evicted_total"] > 0, "nothing was evicted: compaction not exercised"


# deferred compaction: the same trajectories, the oracle still compacting at every step
LAZY = {
    "tiny_f32": (1, 4),          # compact at 25 % dead slots
    "bf16_mha": (1, 8),
    "bf16_gqa4": (1, 4),
    "bf16_gqa8": (1, 16),
    "f32_d128": (1, 2),
    "bf16_d64": (1, 4),
    "r_lt_w": (1, 3),
    "structured": (1, 4),
    "sparse_layer": (1, 1),      # never by fraction: dead slots pile up until the unit is all dead rows or full
}


@pytest.mark.parametrize("name", list(LAZY))
def test_lazy_trajectory(name):
    """corm_decode_step_lazy: live keys in slot order, out, recorded scores and last_hit equal the
    oracle's at every step, dead slots stay dead, and units are compacted exactly when the policy says."""
    wl, every = TRAJ[name]
    layer = 2 if name == "sparse_layer" else 0
    say("lazy trajectory", name, LAZY[name], wl)
    rep = harness.run_slaved_trajectory(wl, DEV, layer=layer, check_state_every=every, lazy=LAZY[name])
    say("report", name, {k: v for k, v in rep.items() if k != "final_lens"})
    assert rep["evicted_total"] > 0
    if name != "sparse_layer":
        assert rep["compactions"] > 0, "no unit was ever compacted: the policy branch is not exercised"


def test_lazy_with_zero_fraction_is_the_exact_step():
    """dead_num = 0 compacts at every eviction: slot for slot the state corm_decode_step leaves."""
    wl, _ = TRAJ["bf16_mha"]
    x = {k: v.to(DEV) for k, v in inputs.make_layer(wl, 0, device="cpu").items() if k != "sinks"}
    n_replay = min(wl.w, wl.P)
    pre = wl.P - n_replay
    sts = [harness.make_state(wl, DEV), harness.make_state(wl, DEV)]
    for st in sts:
        st.preload(x["K0"][:, :, :pre], x["V0"][:, :, :pre])
    tf = torch.full((wl.B,), pre + 1, dtype=torch.int32, device=DEV)
    for j in range(n_replay + wl.D):
        q, k, v, t = harness.step_inputs(wl, x, j, n_replay)
        td = torch.full((wl.B,), t, dtype=torch.int32, device=DEV)
        sts[0].step(q, k, v, td, tf)
        sts[1].step_lazy(q, k, v, td, tf, dead_num=0, dead_den=1)
        torch.cuda.synchronize()
        assert torch.equal(sts[0].lens, sts[1].lens), j
        assert torch.equal(sts[0].lens, sts[1].nlive), j
        assert torch.equal(sts[0].out, sts[1].out), j
        assert torch.equal(sts[0].keep, sts[1].keep), j
    for name in ("K", "V", "pos", "last_hit", "ring"):
        a, b = getattr(sts[0], name), getattr(sts[1], name)
        for bb in range(wl.B):
            for h in range(wl.Hkv):
                l = int(sts[0].lens[bb, h].item())
                if name == "ring":
                    continue
                assert torch.equal(a[bb, h, :l], b[bb, h, :l]), (name, bb, h)
    assert torch.equal(sts[0].ring, sts[1].ring)
    assert int(sts[1].status.item()) == 0


def test_lazy_unit_out_of_slots_compacts_or_flags():
    """A capacity far below the sequence length: deferred compaction must compact in time (slots about to
    run out), and the status flag is raised only when the live keys themselves no longer fit."""
    wl = W["tiny_f32"].replace(P=96, D=60, w=8, r=5)
    say("lazy, Lcap << Tcap")
    rep = harness.run_slaved_trajectory(wl, DEV, thr_scale=1e9, check_state_every=1, Lcap=100, Tcap=96 + 60,
                                        lazy=(1, 1))
    say("report", rep)
    # the fraction alone never triggers (dead < slots): every unit is compacted once, when its slots run out
    assert rep["compactions"] == wl.B * wl.Hkv and rep["evicted_total"] > 0


def test_lazy_bad_arguments():
    wl = W["tiny_f32"]
    st = harness.make_state(wl, DEV)
    q = torch.zeros(wl.B, wl.Hq, wl.d, device=DEV)
    k = torch.zeros(wl.B, wl.Hkv, wl.d, device=DEV)
    t = torch.ones(wl.B, dtype=torch.int32, device=DEV)
    args = (st.desc, q, k, k, st.K, st.V, st.lens)
    rest = (st.pos, st.last_hit, t, t, st.ring, st.out)
    kw = dict(workspace=st.workspace, status=st.status, check=False)
    assert corm.corm_decode_step_lazy(*args, None, *rest, **kw) == corm.CORM_EINVAL
    assert corm.corm_decode_step_lazy(*args, st.live.data_ptr() + 4, *rest, **kw) == corm.CORM_EINVAL
    assert corm.corm_decode_step_lazy(*args, st.live, *rest, dead_num=-1, **kw) == corm.CORM_EINVAL
    assert corm.corm_decode_step_lazy(*args, st.live, *rest, dead_num=3, dead_den=2, **kw) == corm.CORM_EINVAL
    assert corm.corm_decode_step_lazy(*args, st.live, *rest, dead_num=1, dead_den=0, **kw) == corm.CORM_EINVAL
    torch.cuda.synchronize()
    assert int(st.lens.sum().item()) == 0   # nothing ran


# prompt seeding by the dense kernel, then ordinary decode steps on the state it left
SEEDED = ["tiny_f32", "bf16_mha", "bf16_gqa4", "bf16_gqa8", "f32_d128", "bf16_d64", "f32_gqa4", "r_lt_w", "structured"]


@pytest.mark.parametrize("name", SEEDED)
def test_prefill_seed_then_decode(name):
    """corm_prefill_seed leaves the state the oracle reaches by taking the prompt's last w positions as
    ordinary steps of Algorithm 1 (fed the scores the kernel recorded): ring rows within tolerance, keep
    mask, kept indices, compacted rows, lens and last_hit bit for bit; the decode steps that follow agree
    as in the replayed trajectories."""
    wl, every = TRAJ[name]
    say("prefill seed", name, wl)
    rep = harness.run_slaved_trajectory(wl, DEV, check_state_every=every, seed_kernel=True)
    say("report", name, {k: v for k, v in rep.items() if k != "final_lens"})
    assert rep["evicted_total"] > 0


def test_prefill_seed_offsets_and_short_tail():
    """Sequences at different steps (positions shifted, so ring rows start at unaligned columns), and a
    prompt shorter than the window (m = P < w: rows recorded, nothing evicted yet)."""
    wl = W["tiny_f32"].replace(B=3, P=300, D=12, w=32, r=32)
    harness.run_slaved_trajectory(wl, DEV, check_state_every=4, seq_offsets=[0, 7, 1000], seed_kernel=True)
    wl = W["llama7b_1layer"].replace(B=1, Hq=2, Hkv=2, P=40, D=30, w=64, r=4, key_scale=3.0)
    rep = harness.run_slaved_trajectory(wl, DEV, check_state_every=1, seed_kernel=True)
    assert rep["evicted_total"] > 0   # the window fills during decode


def test_prefill_seed_on_a_cache_with_holes():
    """Positions need not be consecutive: keys are dropped from the part of the prompt before the tail (as an
    earlier eviction would have), then the tail is seeded.  A key is visible to a query by its position, ring
    entries go to the position's column, and the oracle replaying the tail over the same thinned cache must
    agree bit for bit on the decision and the compacted rows."""
    wl = W["llama7b_1layer"].replace(B=2, Hq=4, Hkv=2, P=900, D=4, w=64, r=16)
    x_cpu = inputs.make_layer(wl, 0, device="cpu")
    x = {k: v.to(DEV) for k, v in x_cpu.items() if k != "sinks"}
    m, G, P = wl.w, wl.G, wl.P
    pre = P - m
    st = harness.make_state(wl, DEV, Tcap=P + 8, Lcap=P + 8)
    st.preload(x["K0"], x["V0"])
    rng = np.random.default_rng(3)
    mask = np.ones((wl.B, wl.Hkv, st.Lcap), dtype=np.uint8)
    mask[:, :, :pre] = rng.random((wl.B, wl.Hkv, pre)) < 0.7
    corm.corm_compact(st.desc, st.K, st.V, st.pos, st.last_hit, st.lens, torch.from_numpy(mask).to(DEV), None,
                      st.workspace)
    torch.cuda.synchronize()
    t = torch.full((wl.B,), P, dtype=torch.int32, device=DEV)
    tf = torch.zeros_like(t)
    st.prefill_seed(x["Q"][:m].permute(1, 2, 0, 3).contiguous(), t, tf)
    torch.cuda.synchronize()
    assert int(st.status.item()) == 0
    evicted = 0
    for b in range(wl.B):
        ring = st.ring[b].float().cpu().numpy()
        for h in range(wl.Hkv):
            kept = np.nonzero(mask[b, h, :pre])[0]
            u = O.UnitCache(wl.d, G, wl.w, wl.r, score_dtype=wl.dtype)
            u.preload(x_cpu["K0"][b, h, kept].float().numpy(), x_cpu["V0"][b, h, kept].float().numpy())
            u.positions = kept.astype(np.int64)
            res = None
            for j in range(m):
                p = pre + j
                live_pos = np.concatenate([u.positions, [p]])
                recorded = ring[h * G:(h + 1) * G, p % wl.w][:, live_pos]
                res = u.step(x_cpu["Q"][j, b, h * G:(h + 1) * G].float().numpy(), x_cpu["K0"][b, h, p].float().numpy(),
                             x_cpu["V0"][b, h, p].float().numpy(), p + 1, recorded=recorded)
                for g in range(G):
                    a = res["alpha"][g]
                    err = np.abs(recorded[g].astype(np.float64) - a)
                    assert (err <= harness.SCORE_RTOL[wl.dtype] * a + harness.SCORE_ATOL_OF_MAX[wl.dtype] * a.max()).all()
            n_before = len(kept) + m
            assert np.array_equal(st.keep[b, h, :n_before].cpu().numpy().astype(bool), res["keep"]), (b, h)
            harness.check_unit_state(st, b, h, u, P)
            evicted += n_before - u.l
    assert evicted > 0


def test_prefill_seed_bad_arguments():
    wl = W["tiny_f32"]
    st = harness.make_state(wl, DEV)
    q = torch.zeros(wl.B, wl.Hq, wl.w, wl.d, device=DEV)
    t = torch.full((wl.B,), wl.P, dtype=torch.int32, device=DEV)
    tf = torch.zeros_like(t)
    kw = dict(workspace=st.workspace, status=st.status, check=False)
    args = (st.K, st.V, st.lens, st.pos, st.last_hit, t, tf, st.ring)
    assert corm.corm_prefill_seed(st.desc, q, 0, *args, **kw) == corm.CORM_EINVAL
    assert corm.corm_prefill_seed(st.desc, q, wl.w + 1, *args, **kw) == corm.CORM_EINVAL
    assert corm.corm_prefill_seed(st.desc, None, wl.w, *args, **kw) == corm.CORM_EINVAL
    assert corm.corm_prefill_seed(st.desc, q.data_ptr() + 4, wl.w, *args, **kw) == corm.CORM_EINVAL
    # a tail longer than the prompt so far: flagged on the device, nothing written
    st.lens.fill_(8)
    st.pos[:, :, :8] = torch.arange(8, dtype=torch.int32, device=DEV)
    t8 = torch.full((wl.B,), 8, dtype=torch.int32, device=DEV)
    assert corm.corm_prefill_seed(st.desc, q, wl.w, st.K, st.V, st.lens, st.pos, st.last_hit, t8, tf, st.ring,
                                  **kw) == corm.CORM_OK
    torch.cuda.synchronize()
    assert int(st.status.item()) & corm.CORM_DEV_BAD_STEP
    assert float(st.ring.abs().sum().item()) == 0.0


@pytest.mark.parametrize("mode", ["exact", "lazy"])
@pytest.mark.parametrize("name", ["bf16_mha", "f32_gqa4", "bf16_gqa4"])
def test_summary_only_state_equals_the_ring_state(name, mode):
    """score_ring == NULL: prompt seeding and every decode step leave the same bits (out, keep, lens, live
    masks, K, V, pos, last_hit) as the same calls with a ring, whose parity with the oracle the other tests
    establish."""
    wl, _ = TRAJ[name]
    x = {k: v.to(DEV) for k, v in inputs.make_layer(wl, 0, device="cpu").items() if k != "sinks"}
    m = min(wl.w, wl.P)
    a = corm.LayerState(wl.B, wl.Hq, wl.Hkv, wl.d, wl.P + wl.D, wl.P + wl.D, wl.w, wl.r, wl.dtype, device=DEV,
                        want_masks=True)
    b = corm.LayerState(wl.B, wl.Hq, wl.Hkv, wl.d, wl.P + wl.D, wl.P + wl.D, wl.w, wl.r, wl.dtype, device=DEV,
                        want_masks=True, want_ring=False)
    q_tail = x["Q"][:m].permute(1, 2, 0, 3).contiguous()
    t = torch.full((wl.B,), wl.P, dtype=torch.int32, device=DEV)
    tfs = []
    for st in (a, b):
        st.preload(x["K0"], x["V0"])
        tf = torch.zeros_like(t)
        st.prefill_seed(q_tail, t, tf)
        tfs.append(tf)

    def same(j):
        torch.cuda.synchronize()
        assert torch.equal(a.lens, b.lens) and torch.equal(a.keep, b.keep) and torch.equal(a.live, b.live), j
        for bb in range(wl.B):
            for h in range(wl.Hkv):
                l = int(a.lens[bb, h].item())
                for nm in ("K", "V", "pos", "last_hit"):
                    assert torch.equal(getattr(a, nm)[bb, h, :l], getattr(b, nm)[bb, h, :l]), (nm, j, bb, h)

    same("seed")
    assert int((a.lens < wl.P).sum().item()) > 0, "the bulk eviction removed nothing"
    for j in range(m, m + wl.D):
        q, k, v, tt = harness.step_inputs(wl, x, j, m)
        td = torch.full((wl.B,), tt, dtype=torch.int32, device=DEV)
        for st, tf in zip((a, b), tfs):
            if mode == "lazy":
                st.step_lazy(q, k, v, td, tf, dead_num=1, dead_den=8)
            else:
                st.step(q, k, v, td, tf)
        same(j)
        assert torch.equal(a.out, b.out), j
    assert int(a.status.item()) == 0 and int(b.status.item()) == 0


@pytest.mark.parametrize("mode", ["exact", "lazy"])
@pytest.mark.parametrize("name", ["bf16_mha", "bf16_gqa4", "structured", "sparse_layer"])
def test_step_without_mask_outputs_equals_the_step_with_them(name, mode):
    """The calls as the benchmark makes them -- keep = kept_idx = NULL, where the compaction launches may leave
    at once on their unit's word of the workspace -- against the same calls with the mask outputs, whose parity with
    the oracle the other tests establish: lens, the live masks and counts, out, K, V, pos, last_hit and the
    ring must be the same bits after every step; some steps evict in some units only, some in none.  Two
    layers share one workspace, as the layers of a stack do."""
    wl, _ = TRAJ[name]
    layers = (2, 0) if name == "sparse_layer" else (0, 1)
    xs = [{k: v.to(DEV) for k, v in inputs.make_layer(wl, l, device="cpu").items() if k != "sinks"} for l in layers]
    m = min(wl.w, wl.P)
    pre = wl.P - m
    ws = None
    pairs = []
    for x in xs:
        a = harness.make_state(wl, DEV, want_masks=True)
        ws = a.workspace if ws is None else ws
        b = harness.make_state(wl, DEV, want_masks=False, workspace=ws)      # every maskless layer on one workspace
        for st in (a, b):
            st.preload(x["K0"][:, :, :pre], x["V0"][:, :, :pre])
        pairs.append((a, b, x))
    tf = torch.full((wl.B,), pre + 1, dtype=torch.int32, device=DEV)
    evicting_steps = quiet_steps = 0
    for j in range(m + wl.D):
        for a, b, x in pairs:
            q, k, v, tt = harness.step_inputs(wl, x, j, m)
            td = torch.full((wl.B,), tt, dtype=torch.int32, device=DEV)
            before = (a.lens if mode == "exact" else (a.nlive if j else torch.full_like(a.nlive, pre))).clone()
            for st in (a, b):
                if mode == "lazy":
                    st.step_lazy(q, k, v, td, tf, dead_num=1, dead_den=8)
                else:
                    st.step(q, k, v, td, tf)
            torch.cuda.synchronize()
            assert torch.equal(a.lens, b.lens) and torch.equal(a.out, b.out), (j, "lens / out")
            if mode == "lazy":
                assert torch.equal(a.live, b.live) and torch.equal(a.nlive, b.nlive), (j, "live")
            after = a.lens if mode == "exact" else a.nlive
            lost = int((before + 1 - after).sum().item())       # keys evicted in this step, all units
            assert lost >= 0
            evicting_steps += int(lost > 0)
            quiet_steps += int(lost == 0)
            used = torch.arange(a.Lcap, device=DEV).view(1, 1, -1) < a.lens.unsqueeze(-1)
            for nm in ("pos", "last_hit"):
                assert torch.equal(getattr(a, nm) * used, getattr(b, nm) * used), (nm, j)
            for nm in ("K", "V"):
                assert torch.equal(getattr(a, nm) * used.unsqueeze(-1), getattr(b, nm) * used.unsqueeze(-1)), (nm, j)
    for a, b, _ in pairs:
        assert torch.equal(a.ring, b.ring)
        assert int(a.status.item()) == 0 and int(b.status.item()) == 0
    assert evicting_steps > 0 and quiet_steps > 0, (evicting_steps, quiet_steps)


# the boolean message (score_dtype "bit"): the ring holds what Algorithm 1 itself keeps
BITS = ["tiny_f32", "bf16_mha", "bf16_gqa4", "bf16_gqa8", "r_lt_w", "structured"]


@pytest.mark.parametrize("name", BITS)
def test_bit_ring_trajectory(name):
    """A bit per (recorded query, key position) instead of a score: the slaved oracle takes the recorded
    booleans as its message; every recorded bit must equal the oracle's own threshold test except within
    rounding of the threshold; decisions, indices and caches bit for bit as always."""
    wl, every = TRAJ[name]
    say("bit ring", name, wl)
    rep = harness.run_slaved_trajectory(wl, DEV, check_state_every=every, score_dtype="bit")
    say("report", name, {k: v for k, v in rep.items() if k != "final_lens"})
    assert rep["evicted_total"] > 0


@pytest.mark.parametrize("name", ["tiny_f32", "bf16_mha", "bf16_gqa4", "bf16_d64", "f32_d128"])
def test_bit_ring_prefill_seed(name):
    """corm_prefill_seed writing the boolean message: whole words by plain stores where a wave's 64 positions
    are two words of a row, single bits into cleared rows elsewhere (offset positions below)."""
    wl, every = TRAJ[name]
    rep = harness.run_slaved_trajectory(wl, DEV, check_state_every=every, seed_kernel=True, score_dtype="bit")
    assert rep["evicted_total"] > 0
    if name == "tiny_f32":
        wl2 = W["tiny_f32"].replace(B=3, P=300, D=12, w=32, r=32)
        harness.run_slaved_trajectory(wl2, DEV, check_state_every=4, seq_offsets=[0, 7, 1000], seed_kernel=True,
                                      score_dtype="bit")


@pytest.mark.parametrize("ring", [None, "bit"])
def test_row_density_matches_the_oracle(ring):
    """corm_row_density (the sparsity measurement of Section 3) on the row a step just recorded: per query head
    exactly the oracle's share of important keys among the recorded scores."""
    wl = W["gqa_llama3"].replace(B=2, Hq=8, Hkv=2, P=700, D=4, w=16, r=16)
    x = {k: v.to(DEV) for k, v in inputs.make_layer(wl, 0, device="cpu").items() if k != "sinks"}
    st = harness.make_state(wl, DEV, score_dtype=ring)
    n_replay = min(wl.w, wl.P)
    pre = wl.P - n_replay
    st.preload(x["K0"][:, :, :pre], x["V0"][:, :, :pre])
    dens = torch.zeros(wl.B, wl.Hq, dtype=torch.float32, device=DEV)
    G = wl.G
    for j in range(6):
        q, k, v, t = harness.step_inputs(wl, x, j, n_replay)
        td = torch.full((wl.B,), t, dtype=torch.int32, device=DEV)
        corm.corm_append(st.desc, st.K, st.V, st.lens, st.pos, st.last_hit, k, v, td, st.status)
        corm.corm_decode_attend(st.desc, q, st.K, st.V, st.lens, st.pos, td, st.ring, st.last_hit, st.out,
                                st.workspace, status=st.status)
        corm.corm_row_density(st.desc, st.ring, st.lens, st.pos, td, dens)
        torch.cuda.synchronize()
        got = dens.cpu().numpy()
        for b in range(wl.B):
            row = harness.ring_row(st, b, (t - 1) % wl.w)
            for hq in range(wl.Hq):
                h = hq // G
                l = int(st.lens[b, h].item())
                positions = st.pos[b, h, :l].cpu().numpy()
                want = np.float32(O.important(row[hq][positions], t).sum()) / np.float32(l)
                assert got[b, hq] == want, (j, b, hq, got[b, hq], want)
                assert abs(O.important_fraction(row[hq][positions], t) - float(want)) < 1e-6
    assert 0.0 < got.min() and got.max() < 1.0


def test_f32_ring_on_a_bf16_cache():
    """score_dtype is independent of kv_dtype: fp32 probabilities recorded for a bf16 cache (decode steps and
    prompt seeding)."""
    wl, every = TRAJ["bf16_gqa4"]
    harness.run_slaved_trajectory(wl, DEV, check_state_every=every, score_dtype="f32")
    rep = harness.run_slaved_trajectory(wl, DEV, check_state_every=every, score_dtype="f32", seed_kernel=True)
    assert rep["evicted_total"] > 0


def test_bit_ring_split_calls_and_lazy():
    """The literal mask (corm_evict_mask) reads the bits; deferred compaction and ragged steps work on a bit ring."""
    wl = W["tiny_f32"].replace(B=3, P=300, D=40, w=32, r=8)
    harness.run_slaved_trajectory(wl, DEV, check_state_every=2, use_split_calls=True, score_dtype="bit")
    harness.run_slaved_trajectory(wl, DEV, check_state_every=2, seq_offsets=[0, 7, 1000], score_dtype="bit")
    rep = harness.run_slaved_trajectory(TRAJ["bf16_mha"][0], DEV, check_state_every=6, lazy=(1, 8), score_dtype="bit")
    assert rep["compactions"] > 0


def test_split_calls_equal_the_fused_step():
    """append + decode_attend + evict_mask (literal, also == summary) + compact: the same bits
    as the fused step, checked against the same oracle."""
    wl = W["gqa_llama3"].replace(B=2, Hq=4, Hkv=2, P=560, D=30, w=24, r=24)
    say("split calls", wl)
    a = harness.run_slaved_trajectory(wl, DEV, check_state_every=5, use_split_calls=True)
    b = harness.run_slaved_trajectory(wl, DEV, check_state_every=5, use_split_calls=False)
    assert a["final_lens"] == b["final_lens"] and a["evicted_total"] == b["evicted_total"] > 0


@pytest.mark.parametrize("c,expect", [(0.0, "none"), (1e9, "window")])
def test_threshold_extremes(c, expect):
    wl = W["tiny_f32"].replace(P=96, D=30, w=8, r=5)
    say("threshold extreme", c)
    rep = harness.run_slaved_trajectory(wl, DEV, thr_scale=c, check_state_every=1)
    lens = np.array(rep["final_lens"])
    if expect == "none":
        assert (lens == wl.P + wl.D).all() and rep["evicted_total"] == 0
    else:
        assert (lens == wl.r).all()


def test_sequences_at_different_steps():
    """t is per sequence: one batch whose sequences sit at different absolute steps (different thresholds
    c/t, different ring slots in the same launch)."""
    wl = W["tiny_f32"].replace(B=3, Hq=2, Hkv=2, P=140, D=30, w=16, r=16)
    say("ragged t", wl)
    rep = harness.run_slaved_trajectory(wl, DEV, check_state_every=2, seq_offsets=[0, 7, 1000])
    assert rep["evicted_total"] > 0


def test_capacity_smaller_than_the_sequence():
    """Slots per unit (Lcap) far below the number of positions (Tcap): legal as long as eviction keeps the
    cache short; here c is huge, so every unit holds r (+1) keys once the window is full."""
    wl = W["tiny_f32"].replace(P=96, D=60, w=8, r=5)
    say("Lcap << Tcap")
    rep = harness.run_slaved_trajectory(wl, DEV, thr_scale=1e9, check_state_every=1, Lcap=96, Tcap=96 + 60)
    assert (np.array(rep["final_lens"]) == wl.r).all()


@pytest.mark.parametrize("G,P", [(4, 3040), (2, 6100), (1, 12250)])
def test_unit_kernel_at_its_lds_limit(G, P, launch_path):
    """The longest caches the fused unit kernel takes (48 KiB of logits in LDS beside its static arrays):
    forced onto that path, it must really be the one that runs, and stay exact."""
    wl = W["gqa_llama3"].replace(name=f"lds_limit_g{G}", B=1, Hq=G, Hkv=1, P=P, D=12, w=8, r=8, key_scale=1.5)
    st = harness.make_state(wl, DEV, Lcap=wl.P + wl.D, Tcap=wl.P + wl.D)
    if launch_path == "unit":
        assert corm.corm_selected_path(st.desc) == 2
    del st
    rep = harness.run_slaved_trajectory(wl, DEV, check_state_every=4)
    say("report", G, P, {k: v for k, v in rep.items() if k != "final_lens"})
    assert rep["evicted_total"] > 0


def _random_shapes(n, seed=2024):
    """Seeded draw of small workloads across the shapes the interface accepts: odd head counts, every group
    size, both row widths and dtypes, prompts shorter than the window, r on either side of w, thresholds off
    the default, every kind of ring, exact and deferred compaction, replayed and dense prompt seeding."""
    rng = np.random.default_rng(seed)
    out = []
    for i in range(n):
        G = int(rng.choice([1, 1, 2, 4, 8]))
        Hkv = int(rng.choice([1, 2, 3, 5]))
        dtype = str(rng.choice(["f32", "bf16"]))
        w = int(rng.choice([1, 2, 5, 16, 33, 64]))
        wl = W["tiny_f32"].replace(
            name=f"random{i}", B=int(rng.integers(1, 4)), Hq=G * Hkv, Hkv=Hkv, d=int(rng.choice([64, 128])),
            dtype=dtype, P=int(rng.choice([1, 3, 17, 64, 255, 513, 700, 1030])), D=int(rng.integers(6, 28)),
            w=w, r=int(rng.choice([1, 2, w, w, 2 * w + 1])), key_scale=float(rng.choice([0.5, 1.0, 2.0])),
            n_sinks=int(rng.choice([0, 4])), seed=int(rng.integers(1 << 20)))
        kw = dict(thr_scale=float(rng.choice([0.25, 1.0, 1.0, 3.0])),
                  lazy=(1, int(rng.choice([2, 4, 8]))) if rng.random() < 0.4 else None,
                  seed_kernel=bool(rng.random() < 0.5),
                  score_dtype=(None, None, "bit", "f32")[int(rng.integers(4))],
                  slack=int(rng.choice([0, 1, 7, 64])))
        out.append((wl, kw))
    return out


RANDOM_SHAPES = _random_shapes(48)


@pytest.mark.parametrize("case", range(len(RANDOM_SHAPES)))
def test_random_shapes(case):
    wl, kw = RANDOM_SHAPES[case]
    kw = dict(kw)
    slack = kw.pop("slack")
    say("random shape", case, wl, kw, "slack", slack)
    rep = harness.run_slaved_trajectory(wl, DEV, check_state_every=3, Lcap=wl.P + wl.D + slack,
                                        Tcap=wl.P + wl.D + slack, **kw)
    say("report", case, {k: v for k, v in rep.items() if k != "final_lens"})


def test_w1_r1():
    wl = W["tiny_f32"].replace(P=40, D=30, w=1, r=1)
    say("w=1 r=1")
    harness.run_slaved_trajectory(wl, DEV, check_state_every=1)


# ------------------------------------------------------------------ the threshold arithmetic

def test_device_threshold_is_the_ieee_quotient():
    ts = np.unique(np.concatenate([np.arange(1, 70000), np.random.default_rng(0).integers(1, 2 ** 24, 50000)]))
    t = torch.from_numpy(ts.astype(np.int32)).to(DEV)
    thr = torch.empty(len(ts), dtype=torch.float32, device=DEV)
    for c in (1.0, 0.5, 3.0, 0.0):
        corm.corm_threshold(c, t, len(ts), thr)
        want = np.float32(c) / ts.astype(np.float32)
        assert np.array_equal(thr.cpu().numpy().view(np.uint32), want.astype(np.float32).view(np.uint32)), c


# ------------------------------------------------------------------ standalone calls on arbitrary inputs

def _rand_state(B, Hq, Hkv, d, Lcap, Tcap, w, r, dtype, lens, seed=0):
    st = corm.LayerState(B, Hq, Hkv, d, Lcap, Tcap, w, r, dtype, device=DEV, want_masks=True)
    g = torch.Generator(device="cpu"); g.manual_seed(seed)
    st.K.copy_(torch.randn(B, Hkv, Lcap, d, generator=g).to(st.dtype))
    st.V.copy_(torch.randn(B, Hkv, Lcap, d, generator=g).to(st.dtype))
    st.lens.copy_(torch.tensor(lens, dtype=torch.int32).view(B, Hkv))
    return st, g


def test_compact_standalone_random_masks():
    """corm_compact on arbitrary keep masks == stable gather; edge lens 0, 1, tile and split boundaries."""
    lens = [0, 1, 255, 256, 257, 512, 513, 1000]
    B, Hkv, Lcap, d = 2, 4, 1000, 128
    st, g = _rand_state(B, Hkv, Hkv, d, Lcap, Lcap, 4, 4, "bf16", lens)
    pos = torch.stack([torch.sort(torch.randperm(5000, generator=g)[:Lcap]).values for _ in range(B * Hkv)])
    st.pos.copy_(pos.view(B, Hkv, Lcap).int())
    st.last_hit.copy_(torch.randint(0, 999, (B, Hkv, Lcap), generator=g).int())
    for trial, pkeep in enumerate([0.5, 0.97, 0.03, 1.0, 0.0]):
        say("compact trial", trial, pkeep)
        keep = (torch.rand(B, Hkv, Lcap, generator=g) < pkeep).to(torch.uint8)
        K0, V0 = st.K.clone(), st.V.clone()
        pos0, lh0, lens0 = st.pos.clone(), st.last_hit.clone(), st.lens.clone()
        st.keep.copy_(keep)
        corm.corm_compact(st.desc, st.K, st.V, st.pos, st.last_hit, st.lens, st.keep, st.kept_idx, st.workspace)
        torch.cuda.synchronize()
        for b in range(B):
            for h in range(Hkv):
                l = int(lens0[b, h])
                idx = O.stable_compact(keep[b, h, :l].numpy())
                n = len(idx)
                assert int(st.lens[b, h]) == n
                it = torch.from_numpy(idx).to(DEV)
                assert torch.equal(st.kept_idx[b, h, :n].long(), it)
                assert torch.equal(st.K[b, h, :n], K0[b, h][it]) and torch.equal(st.V[b, h, :n], V0[b, h][it])
                assert torch.equal(st.pos[b, h, :n], pos0[b, h][it]) and torch.equal(st.last_hit[b, h, :n], lh0[b, h][it])
        # idempotence: compacting again with an all-ones mask changes nothing
        K1, lens1 = st.K.clone(), st.lens.clone()
        st.keep.fill_(1)
        corm.corm_compact(st.desc, st.K, st.V, st.pos, st.last_hit, st.lens, st.keep, None, st.workspace)
        torch.cuda.synchronize()
        assert torch.equal(st.lens, lens1)
        for b in range(B):
            for h in range(Hkv):
                n = int(lens1[b, h])
                assert torch.equal(st.K[b, h, :n], K1[b, h, :n])
        # restore full units for the next trial
        st.K.copy_(K0); st.V.copy_(V0); st.pos.copy_(pos0); st.last_hit.copy_(lh0); st.lens.copy_(lens0)


def test_evict_mask_standalone_random_ring():
    """corm_evict_mask on an arbitrary ring == the oracle's windowed rule on the same stored scores."""
    B, Hq, Hkv, d, Lcap, Tcap, w, r = 2, 4, 2, 64, 300, 400, 6, 4
    lens = [0, 3, 300, 257]
    for dtype in ("f32", "bf16"):
        st, g = _rand_state(B, Hq, Hkv, d, Lcap, Tcap, w, r, dtype, lens, seed=3)
        G = Hq // Hkv
        pos = torch.stack([torch.sort(torch.randperm(340, generator=g)[:Lcap]).values for _ in range(B * Hkv)])
        st.pos.copy_(pos.view(B, Hkv, Lcap).int())
        ring = (torch.rand(B, Hq, w, Tcap, generator=g) ** 6 * 0.02).to(st.dtype)
        st.ring.copy_(ring)
        for (tcur, tfirst) in [(345, 1), (345, 341), (345, 340), (350, 300)]:
            say("evict_mask", dtype, tcur, tfirst)
            t = torch.full((B,), tcur, dtype=torch.int32, device=DEV)
            tf = torch.full((B,), tfirst, dtype=torch.int32, device=DEV)
            st.keep.fill_(7)
            corm.corm_evict_mask(st.desc, st.ring, st.lens, st.pos, t, tf, st.keep)
            torch.cuda.synchronize()
            rows = list(range(max(tfirst, tcur - w + 1), tcur + 1))
            for b in range(B):
                for h in range(Hkv):
                    l = lens[b * Hkv + h]
                    if l == 0:
                        continue
                    p = pos.view(B, Hkv, Lcap)[b, h, :l].numpy()
                    sc = np.zeros((len(rows), G, l), dtype=np.float32)
                    for a, tau in enumerate(rows):
                        row = ring[b, h * G:(h + 1) * G, (tau - 1) % w].float().numpy()[:, p]
                        sc[a] = np.where(p[None, :] <= tau - 1, row, 0.0)
                    want = O.keep_from_score_window(sc, rows, w, r)
                    got = st.keep[b, h, :l].cpu().numpy().astype(bool)
                    assert np.array_equal(got, want), (dtype, tcur, tfirst, b, h)
                    if len(rows) >= w and l > 50:
                        assert not want.all()


def test_attend_edge_lengths_and_status_flags():
    """decode_attend on lens 0 / 1 / split boundaries, and the device status bits (no faults)."""
    B, Hq, Hkv, d, Lcap, Tcap, w, r = 1, 6, 6, 128, 1100, 1100, 8, 8
    lens = [0, 1, 511, 512, 513, 1100]
    st, g = _rand_state(B, Hq, Hkv, d, Lcap, Tcap, w, r, "bf16", lens, seed=5)
    st.pos.copy_(torch.arange(Lcap, dtype=torch.int32).expand(B, Hkv, Lcap))
    q = torch.randn(B, Hq, d, generator=g).to(torch.bfloat16).to(DEV)
    t = torch.full((B,), Lcap, dtype=torch.int32, device=DEV)
    say("attend edge lengths")
    corm.corm_decode_attend(st.desc, q, st.K, st.V, st.lens, st.pos, t, st.ring, st.last_hit, st.out, st.workspace,
                            status=st.status)
    torch.cuda.synchronize()
    assert int(st.status.item()) == 0
    slot = (Lcap - 1) % w
    for h, l in enumerate(lens):
        if l == 0:
            assert torch.count_nonzero(st.out[0, h]) == 0
            continue
        K = st.K[0, h, :l].float().cpu().numpy(); V = st.V[0, h, :l].float().cpu().numpy()
        a = O.attention_scores(q[0, h].float().cpu().numpy(), K)
        ref = O.attention_output(a, V)
        assert harness.out_rel_err(st.out[0, h].cpu().numpy().astype(np.float64), ref) <= 2e-3
        rec = st.ring[0, h, slot, :l].float().cpu().numpy()
        assert (np.abs(rec - a) <= 2.0 ** -8 * a + 1e-5 * a.max()).all()
        lh = st.last_hit[0, h, :l].cpu().numpy()
        assert np.array_equal(lh == Lcap, O.important(rec, Lcap))
    assert torch.equal(st.lens.cpu().view(-1), torch.tensor(lens, dtype=torch.int32))   # attend leaves lens alone
    # a full unit cannot take an append; a step beyond the ring's columns is not recorded
    say("status: unit full")
    k = torch.randn(B, Hkv, d, generator=g).to(torch.bfloat16).to(DEV)
    K_before = st.K.clone()
    tf = t.clone()            # window not full: nothing is evicted
    st.step(q, k, k, t, tf)
    torch.cuda.synchronize()
    assert int(st.status.item()) & corm.CORM_DEV_UNIT_FULL
    assert torch.equal(st.K[0, 5], K_before[0, 5])
    st.status.zero_()
    rc = corm.corm_append(st.desc, st.K, st.V, st.lens, st.pos, st.last_hit, k, k, t, st.status)
    torch.cuda.synchronize()
    assert int(st.status.item()) & corm.CORM_DEV_UNIT_FULL
    say("status: step beyond Tcap")
    st.status.zero_()
    st.lens.fill_(4)
    ring_before = st.ring.clone()
    t_bad = torch.full((B,), Tcap + 1, dtype=torch.int32, device=DEV)
    corm.corm_decode_attend(st.desc, q, st.K, st.V, st.lens, st.pos, t_bad, st.ring, st.last_hit, st.out,
                            st.workspace, status=st.status)
    torch.cuda.synchronize()
    assert int(st.status.item()) & corm.CORM_DEV_BAD_STEP
    assert torch.equal(st.ring, ring_before)
    say("status: lens out of range is clamped")
    st.status.zero_()
    st.lens.fill_(Lcap + 5)
    corm.corm_decode_attend(st.desc, q, st.K, st.V, st.lens, st.pos, t, st.ring, st.last_hit, st.out,
                            st.workspace, status=st.status)
    torch.cuda.synchronize()
    assert int(st.status.item()) & corm.CORM_DEV_BAD_LENS


def test_repeat_run_is_bit_identical():
    """Same inputs twice -> identical state (no race in the split arrival or the in-place compaction)."""
    wl = W["llama7b_1layer"].replace(B=2, Hq=4, Hkv=4, P=1300, D=24, w=64, r=64,
                                     q_mean_scales=inputs.STRUCTURED_Q_MEAN)
    say("repeatability", wl)
    x = {k: v.to(DEV) for k, v in inputs.make_layer(wl, 0).items() if k != "sinks"}
    n_replay = wl.w
    snaps = []
    for rep in range(2):
        st = harness.make_state(wl, DEV)
        pre = wl.P - n_replay
        st.preload(x["K0"][:, :, :pre], x["V0"][:, :, :pre])
        tf = torch.full((wl.B,), pre + 1, dtype=torch.int32, device=DEV)
        outs = []
        for j in range(n_replay + wl.D):
            q, k, v, t = harness.step_inputs(wl, x, j, n_replay)
            st.step(q, k, v, torch.full((wl.B,), t, dtype=torch.int32, device=DEV), tf)
            outs.append(st.out.clone())
        torch.cuda.synchronize()
        lens = st.lens.cpu()
        live = torch.arange(st.Lcap).view(1, 1, -1) < lens.unsqueeze(-1)
        snaps.append((torch.stack(outs).cpu(), lens, (st.K.cpu() * live.unsqueeze(-1)), st.pos.cpu() * live,
                      st.ring.cpu()))
    for a, b in zip(*snaps):
        assert torch.equal(a, b)
    assert snaps[0][1].min() < wl.P


def test_compact_few_holes_takes_the_parallel_path():
    """Units that lose at most 16 keys are compacted chunk-parallel with staged boundary rows; holes at the
    first slot, around the 512-slot chunk boundaries, at the end, and runs that straddle a boundary."""
    B, Hkv, Lcap, d = 1, 8, 2100, 128
    lens = [2100, 2048, 1537, 1025, 1024, 513, 512, 40]
    st, g = _rand_state(B, Hkv, Hkv, d, Lcap, Lcap, 4, 4, "bf16", lens, seed=11)
    st.pos.copy_(torch.arange(Lcap, dtype=torch.int32).expand(B, Hkv, Lcap) * 3 + 1)
    st.last_hit.copy_(torch.randint(0, 999, (B, Hkv, Lcap), generator=g).int())
    hole_sets = [
        [0], [511], [512], [513], [1023, 1024], [510, 511, 512, 513], [0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15],
        [5, 700, 1400], list(range(505, 521)), [39], [0, 39], list(range(1016, 1032)), [1536], [2047], [2099],
        [100, 600, 1100, 1600, 2050], list(range(496, 512)), list(range(512, 528)),
    ]
    rng = np.random.default_rng(7)
    for _ in range(6):
        hole_sets.append(sorted(rng.choice(2100, size=int(rng.integers(1, 17)), replace=False).tolist()))
    K0, V0 = st.K.clone(), st.V.clone()
    pos0, lh0, lens0 = st.pos.clone(), st.last_hit.clone(), st.lens.clone()
    for trial, holes in enumerate(hole_sets):
        say("few holes", trial, holes[:6], "...")
        keep = torch.ones(B, Hkv, Lcap, dtype=torch.uint8)
        keep[:, :, holes] = 0
        st.keep.copy_(keep)
        st.kept_idx.fill_(-1)
        corm.corm_compact(st.desc, st.K, st.V, st.pos, st.last_hit, st.lens, st.keep, st.kept_idx, st.workspace)
        torch.cuda.synchronize()
        for h in range(Hkv):
            l = lens[h]
            idx = O.stable_compact(keep[0, h, :l].numpy())
            n = len(idx)
            assert int(st.lens[0, h]) == n, (trial, h)
            it = torch.from_numpy(idx).to(DEV)
            assert torch.equal(st.kept_idx[0, h, :n].long(), it), (trial, h)
            assert torch.equal(st.K[0, h, :n], K0[0, h][it]) and torch.equal(st.V[0, h, :n], V0[0, h][it]), (trial, h)
            assert torch.equal(st.pos[0, h, :n], pos0[0, h][it]), (trial, h)
            assert torch.equal(st.last_hit[0, h, :n], lh0[0, h][it]), (trial, h)
        st.K.copy_(K0); st.V.copy_(V0); st.pos.copy_(pos0); st.last_hit.copy_(lh0); st.lens.copy_(lens0)


def test_two_phase_calls_on_two_streams_equal_the_fused_step():
    """corm_step_attend on one stream and corm_step_evict on another, ordered by events and alternating
    two workspaces (the benchmark's pipeline), leave exactly the state the fused call leaves."""
    wl = W["llama7b_1layer"].replace(B=2, Hq=4, Hkv=4, P=1300, D=24, w=64, r=64,
                                     q_mean_scales=inputs.STRUCTURED_Q_MEAN)
    say("two-phase pipeline", wl)
    n_layers = 3
    xs = [{k: v.to(DEV) for k, v in inputs.make_layer(wl, l).items() if k != "sinks"} for l in range(n_layers)]
    n_replay = wl.w
    pre = wl.P - n_replay
    results = []
    for mode in ("fused", "pipelined"):
        sts = [harness.make_state(wl, DEV, want_masks=False) for _ in range(n_layers)]
        for st, x in zip(sts, xs):
            st.preload(x["K0"][:, :, :pre], x["V0"][:, :, :pre])
        tf = torch.full((wl.B,), pre + 1, dtype=torch.int32, device=DEV)
        wss = [sts[0].workspace, sts[1].workspace]
        main, side = torch.cuda.current_stream(), torch.cuda.Stream()
        ev_att = [torch.cuda.Event() for _ in range(n_layers)]
        ev_evi = [torch.cuda.Event() for _ in range(n_layers)]
        outs = []
        n = 0
        for j in range(n_replay + wl.D):
            td = torch.full((wl.B,), pre + 1 + j, dtype=torch.int32, device=DEV)
            for l, (st, x) in enumerate(zip(sts, xs)):
                q, k, v, t = harness.step_inputs(wl, x, j, n_replay)
                if mode == "fused":
                    st.step(q, k, v, td, tf)
                else:
                    if n >= 2:
                        main.wait_event(ev_evi[(n - 2) % n_layers])
                    st.step_attend(q, k, v, td, tf, stream=main, workspace=wss[n % 2])
                    ev_att[l].record(main)
                    side.wait_event(ev_att[l])
                    st.step_evict(stream=side, workspace=wss[n % 2])
                    ev_evi[l].record(side)
                    td.record_stream(side)
                n += 1
            if mode == "pipelined":
                main.wait_stream(side)
            outs.append(torch.stack([st.out.clone() for st in sts]))
        torch.cuda.synchronize()
        lens = torch.stack([st.lens for st in sts]).cpu()
        live = torch.arange(sts[0].Lcap).view(1, 1, 1, -1) < lens.unsqueeze(-1)
        Ks = torch.stack([st.K for st in sts]).cpu() * live.unsqueeze(-1)
        results.append((torch.stack(outs).cpu(), lens, Ks, torch.stack([st.pos for st in sts]).cpu() * live,
                        torch.stack([st.ring for st in sts]).cpu()))
        assert all(int(st.status.item()) == 0 for st in sts)
    for a, b in zip(*results):
        assert torch.equal(a, b)
    assert results[0][1].min() < wl.P


def test_decode_step_under_hip_graph_capture():
    """The library allocates nothing and records no memset, so a caller may capture a step in a HIP graph:
    every replay (inputs refreshed in place, eager work and synchronizations in between) must leave exactly
    the state an eager twin reaches."""
    wl, _ = TRAJ["bf16_mha"]
    x = {k: v.to(DEV) for k, v in inputs.make_layer(wl, 0, device="cpu").items() if k != "sinks"}
    n_replay = min(wl.w, wl.P)
    pre = wl.P - n_replay
    a, b = harness.make_state(wl, DEV), harness.make_state(wl, DEV)
    for st in (a, b):
        st.preload(x["K0"][:, :, :pre], x["V0"][:, :, :pre])
    tf = torch.full((wl.B,), pre + 1, dtype=torch.int32, device=DEV)
    q0, k0, v0, t0 = harness.step_inputs(wl, x, 0, n_replay)
    qs, ks, vs = q0.clone(), k0.clone(), v0.clone()
    ts = torch.full((wl.B,), t0, dtype=torch.int32, device=DEV)
    # first step eagerly on both (warm-up before capture), then capture the step of `a`
    a.step(qs, ks, vs, ts, tf)
    b.step(q0, k0, v0, ts.clone(), tf)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            a.step(qs, ks, vs, ts, tf)
    torch.cuda.synchronize()
    # capture does not execute: `a` is still one step behind what the next replay will compute
    evicted = 0
    for j in range(1, n_replay + wl.D):
        q, k, v, t = harness.step_inputs(wl, x, j, n_replay)
        qs.copy_(q); ks.copy_(k); vs.copy_(v); ts.fill_(t)
        graph.replay()
        b.step(q, k, v, torch.full((wl.B,), t, dtype=torch.int32, device=DEV), tf)
        torch.cuda.synchronize()
        assert torch.equal(a.lens, b.lens), j
        assert torch.equal(a.out, b.out), j
        assert torch.equal(a.keep, b.keep) and torch.equal(a.kept_idx, b.kept_idx), j
        evicted += int((a.keep == 0).sum().item())
        (a.out.sum() + a.lens.sum()).item()   # eager work between replays
    for nm in ("K", "V", "pos", "last_hit"):
        for bb in range(wl.B):
            for h in range(wl.Hkv):
                l = int(a.lens[bb, h].item())
                assert torch.equal(getattr(a, nm)[bb, h, :l], getattr(b, nm)[bb, h, :l]), (nm, bb, h)
    assert torch.equal(a.ring, b.ring)
    assert int(a.status.item()) == 0 and int(b.status.item()) == 0


def test_c_abi_client_without_python(launch_path):
    """The boundary from a plain C++ process (dlopen + HIP runtime, no torch): a few dozen decode steps
    checked there against closed forms (c = 0: full attention; c huge: a sliding window of r keys)."""
    import os
    import subprocess
    if launch_path != "split":
        pytest.skip("the client runs in its own process with the library's own path choice: once is enough")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    exe = os.path.join(root, "tests", "abi_client", "abi_client")
    if not os.path.exists(exe):
        pytest.skip("tests/abi_client/abi_client is not built (__graft_entry__.build() compiles it)")
    res = subprocess.run([exe, corm.LIB_PATH], capture_output=True, text=True, timeout=120)
    say("abi_client", res.returncode, res.stdout[-400:], res.stderr[-200:])
    assert res.returncode == 0 and "all checks passed" in res.stdout


@pytest.mark.parametrize("score_dtype", [None, "bit"])
def test_ring_needs_no_initialisation(score_dtype, monkeypatch):
    """No call reads a ring column it did not write for a query of the current window: a ring that starts
    out full of ones (every entry 'important') gives the same trajectory, the literal mask included."""
    wl = W["tiny_f32"].replace(B=2, Hq=4, Hkv=2, P=150, D=30, w=12, r=5)
    make = harness.make_state

    def dirty(*a, **kw):
        st = make(*a, **kw)
        st.ring.fill_(-1 if st.ring_bits else 1.0)
        return st

    monkeypatch.setattr(harness, "make_state", dirty)
    say("dirty ring", score_dtype)
    rep = harness.run_slaved_trajectory(wl, DEV, check_state_every=2, score_dtype=score_dtype, use_split_calls=True)
    rep2 = harness.run_slaved_trajectory(wl, DEV, check_state_every=2, score_dtype=score_dtype)
    rep3 = harness.run_slaved_trajectory(wl, DEV, check_state_every=2, score_dtype=score_dtype, seed_kernel=True)
    assert rep["evicted_total"] > 0 and rep["final_lens"] == rep2["final_lens"] == rep3["final_lens"]


@pytest.mark.parametrize("mode", ["exact", "lazy", "seeded"])
def test_slots_beyond_lens_are_never_read(mode, monkeypatch):
    """Slots at or above lens hold unspecified data: caches that start out full of NaN rows (and junk
    positions and hit records, and a workspace of junk bytes) give the same trajectory -- a NaN that reached a
    dot product, even with weight zero, would poison out."""
    wl = W["llama7b_1layer"].replace(B=2, Hq=4, Hkv=2, P=530, D=30, w=16, r=6, key_scale=1.5)
    make = harness.make_state

    def dirty(*a, **kw):
        st = make(*a, **kw)
        st.K.fill_(float("nan"))
        st.V.fill_(float("nan"))
        st.pos.fill_(-7)
        st.last_hit.fill_(12345)
        st.workspace.fill_(0xAB)      # the workspace too: only what corm_workspace_init sets is relied on
        corm.corm_workspace_init(st.desc, st.workspace)
        return st

    monkeypatch.setattr(harness, "make_state", dirty)
    say("dirty slots", mode)
    rep = harness.run_slaved_trajectory(wl, DEV, check_state_every=2, lazy=(1, 4) if mode == "lazy" else None,
                                        seed_kernel=mode == "seeded")
    assert rep["evicted_total"] > 0


@pytest.mark.parametrize("lazy", [False, True])
def test_layers_round_robin_on_three_streams(lazy):
    """The benchmark's launch configuration: independent layers dealt round-robin over three streams, one
    workspace per stream, joined after every step.  Every layer must end bit for bit where it ends when the
    layers run one after the other on one stream with one workspace."""
    wl = W["llama7b_b16"].replace(layers=5, B=2, Hq=4, Hkv=4, P=900, D=24, w=48, r=48,
                                  q_mean_scales=inputs.STRUCTURED_Q_MEAN)
    n_replay = wl.w
    xs = [{k: v.to(DEV) for k, v in inputs.make_layer(wl, l, device="cpu").items() if k != "sinks"}
          for l in range(wl.layers)]
    tf = torch.full((wl.B,), wl.P - n_replay + 1, dtype=torch.int32, device=DEV)
    results = []
    for n_streams in (1, 3):
        states = [harness.make_state(wl, DEV) for _ in range(wl.layers)]
        for st, x in zip(states, xs):
            st.preload(x["K0"][:, :, :wl.P - n_replay], x["V0"][:, :, :wl.P - n_replay])
        main = torch.cuda.current_stream()
        streams = [main] + [torch.cuda.Stream() for _ in range(n_streams - 1)]
        wss = [states[k].workspace for k in range(n_streams)]      # one workspace per stream
        outs = []
        torch.cuda.synchronize()
        for j in range(n_replay + wl.D):
            t = harness.step_inputs(wl, xs[0], j, n_replay)[3]
            t_dev = torch.full((wl.B,), t, dtype=torch.int32, device=DEV)   # (on the main stream, before the fork)
            for s in streams[1:]:
                s.wait_stream(main)
            for l, (st, x) in enumerate(zip(states, xs)):
                k_ = l % n_streams
                with torch.cuda.stream(streams[k_]):
                    q, k, v, _ = harness.step_inputs(wl, x, j, n_replay)      # (its copies run on this stream too)
                    if lazy:
                        st.step_lazy(q, k, v, t_dev, tf, dead_num=1, dead_den=4, stream=streams[k_], workspace=wss[k_])
                    else:
                        corm.corm_decode_step(st.desc, q, k, v, st.K, st.V, st.lens, st.pos, st.last_hit, t_dev, tf,
                                              st.ring, st.out, st.keep, st.kept_idx, wss[k_], status=st.status,
                                              stream=streams[k_])
                t_dev.record_stream(streams[k_])
            for s in streams[1:]:
                main.wait_stream(s)
            outs.append(torch.stack([st.out for st in states]).clone())
        torch.cuda.synchronize()
        assert all(int(st.status.item()) == 0 for st in states)
        snap = []
        for st in states:
            lens = st.lens.cpu()
            used = torch.arange(st.Lcap).view(1, 1, -1) < lens.unsqueeze(-1)
            snap.append((lens, st.K.cpu() * used.unsqueeze(-1), st.V.cpu() * used.unsqueeze(-1), st.pos.cpu() * used,
                         st.last_hit.cpu() * used, st.ring.cpu(), st.live.cpu() if lazy else lens))
        results.append((torch.stack(outs).cpu(), snap))
        del states
    assert torch.equal(results[0][0], results[1][0]), "out differs between one and three streams"
    for l, (a, b) in enumerate(zip(results[0][1], results[1][1])):
        for i, (u, v) in enumerate(zip(a, b)):
            assert torch.equal(u, v), ("layer", l, "field", i)
    assert min(int(s[0].min()) for s in results[0][1]) < wl.P


def test_bench_prints_one_json_line_with_the_required_fields(launch_path):
    """bench.py on the smallest workload with a short step count: the last line of stdout is one JSON object
    with the fields the driver reads, the roofline and the CPU-baseline objects included."""
    import json
    import os
    import subprocess
    if launch_path != "split":
        pytest.skip("a process of its own: once is enough")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    res = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--workload", "tiny_f32", "--steps", "3",
                          "--warmup", "1", "--cpu-units", "4"], capture_output=True, text=True, timeout=280)
    assert res.returncode == 0, res.stderr[-600:]
    lines = [ln for ln in res.stdout.splitlines() if ln.strip()]
    assert len(lines) == 1
    r = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in r, key
    assert r["n_gpus"] == 1 and r["steps"] == 3 and r["warmup"] == 1 and r["value"] > 0 and r["vs_baseline"] is None
    assert r["config"]["workload"] == "tiny_f32" and r["dtype"] == "f32" and r["data"] == "synthetic"
    for key in ("bound", "achieved", "peak", "unit", "frac", "traffic"):
        assert key in r["roofline"], key
    assert r["roofline"]["bound"] == "hbm" and r["roofline"]["peak"] == 8000.0
    assert abs(r["roofline"]["frac"] - r["roofline"]["achieved"] / r["roofline"]["peak"]) < 1e-9
    for key in ("value", "unit", "cores", "kind", "sample"):
        assert key in r["cpu_baseline"], key
    assert r["cpu_baseline"]["kind"] == "oracle" and r["cpu_baseline"]["value"] > 0
    assert r["cpu_baseline"]["cores"] == os.cpu_count() and 1 <= r["cpu_baseline"]["threads"] <= 16
    assert r["config"]["streams"] == 1 and "sequence" in r["value_is"] and "traffic_source" in r["roofline"]
    assert r["overlapped"] is None and r["eviction_heavy"] is None      # one layer: nothing to overlap
    # two layers of the headline shape: the eviction-heavy leg runs too, and really evicts
    res = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--layers", "2", "--steps", "3", "--warmup", "1",
                          "--cpu-units", "2", "--cpu-steps", "2"], capture_output=True, text=True, timeout=280)
    assert res.returncode == 0, res.stderr[-600:]
    r = json.loads([ln for ln in res.stdout.splitlines() if ln.strip()][-1])
    assert r["config"]["workload"] == "llama7b_b16" and r["roofline"]["kernel"] == "corm_unit_kernel"
    assert r["roofline"]["bytes_per_key"] == 2 * 128 * 2 + 2 + 8
    assert r["overlapped"]["streams"] == 3 and r["overlapped"]["steps_per_s"] > 0
    eh = r["eviction_heavy"]
    for mode in ("compaction_at_every_step", "deferred_compaction_1_4"):
        assert eh[mode]["steps_per_s"] > 0 and 0.2 < eh[mode]["live_fraction_end"] < 0.9, (mode, eh[mode])   # (the first two layers are the dense ones)
        assert eh[mode]["live_fraction_per_head"]["min"] < eh[mode]["live_fraction_per_head"]["max"]
    assert eh["compaction_at_every_step"]["keys_evicted"] > 0 and eh["compaction_at_every_step"]["moved_bytes_per_step"] > 0
