#!/usr/bin/env python3
"""Benchmark of the CORM decode hot path on one MI355X.

A "step" is one decode step of the whole stack: for every layer one fused launch that appends
the token's key/value, attends over every unit's live keys, records the scores, decides the
evictions and compacts the caches.  Default workload: the LLaMA-2-7B-shaped full stack
(32 layers x 32 heads, d 128, bf16, batch 16, prompt 4096, w = r = 1024) on seeded synthetic
inputs.  Inputs are resident in HBM before the timed region; the prompt is untimed set-up.

Prints ONE JSON line (the last line of stdout).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E peak


def log(*a):
    print("[bench]", *a, file=sys.stderr, flush=True)


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=256)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--workload", default="llama7b_b16")
    ap.add_argument("--layers", type=int, default=None, help="override the number of layers: a stack of layers of the workload's shape (the one-layer workloads as "
                    "a model with that many layers would run them), or fewer layers for short counter runs")
    ap.add_argument("--structured", action="store_true",
                    help="supplementary variant: per-head query means so that eviction happens at w >= 256")
    ap.add_argument("--w", type=int, default=None, help="override the window of recorded queries (the paper's w/r "
                    "sweep, Section 5; the ring holds w rows, so memory follows it)")
    ap.add_argument("--r", type=int, default=None, help="override the number of protected recent keys (default: = w)")
    ap.add_argument("--streams", type=int, default=3, choices=[1, 2, 3, 4],
                    help="layers are issued round-robin on this many streams (they are independent)")
    ap.add_argument("--path", type=int, default=0, choices=[0, 1, 2, 3],
                    help="corm_force_path: 0 by shape, 1 split kernels, 2 one workgroup per unit, 3 split without MFMA")
    ap.add_argument("--lazy-frac", default=None, metavar="NUM/DEN",
                    help="deferred compaction (corm_decode_step_lazy): a unit is compacted once NUM/DEN of its "
                         "slots are dead; default: compact at every step (corm_decode_step)")
    ap.add_argument("--seed", default="kernel", choices=["kernel", "replay"],
                    help="how the prompt fills the recent-query window before decoding (untimed set-up): one "
                         "corm_prefill_seed call per layer, or its last w tokens replayed through corm_decode_step")
    ap.add_argument("--ring", default="scores", choices=["scores", "bits"],
                    help="what the ring records: the queries' probabilities in the KV dtype (default), or the boolean "
                         "message of Algorithm 1, one bit per recorded query and key position")
    ap.add_argument("--no-ring", action="store_true",
                    help="summary-only state: no score ring is allocated or written (score_ring = NULL); decisions "
                         "come from last_hit alone and are bit-identical")
    ap.add_argument("--extra-steps", type=int, default=4, help="untimed single-stream steps after the timed region "
                    "(exclusive measurement of the dominant kernel)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (reference dispatch for rocprofv3 byte counters)")
    ap.add_argument("--cpu-units", type=int, default=128)
    ap.add_argument("--cpu-steps", type=int, default=16)
    return ap.parse_args()


def algorithmic_bytes(lens_before, wl, esz, ssz, part="step"):
    """Bytes a launch must move for units whose live lengths (before the append) are lens_before.
    part="attend": what the attend kernel streams -- every live K and V row once, plus per unit the G
    queries, k_new and v_new read and the appended row written.
    part="step": that plus the record kernel's share: ring row written, pos and last_hit read, out written.
    Rows moved by the compaction, the logits scratch and the split partials are NOT counted."""
    L = lens_before.double() + 1.0
    per_key = 2 * wl.d * esz
    per_unit = (wl.G + 4) * wl.d * esz
    if part == "step":
        per_key += wl.G * ssz + 8
        per_unit += wl.G * wl.d * 4
    return float((L * per_key).sum().item() + L.numel() * per_unit)


def measured_traffic(kernel, workload, bytes_per_launch):
    """HBM bytes per launch from the committed rocprofv3 counter summary (FETCH_SIZE + WRITE_SIZE, calibrated
    against a plain copy), scaled from that run's algorithmic bytes per launch to this run's; None if there is
    no summary for this kernel and workload."""
    path = os.path.join(ROOT, "profiles", "unit_kernel_llama7b_b16_hbm_traffic.txt")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch="):
                kv = dict(item.split("=") for item in line.split())
                if kv["kernel"] == kernel and kv["workload"] == workload:
                    return float(kv["traffic_bytes_per_launch"]) / float(kv["algorithmic_bytes_per_launch"]) \
                        * bytes_per_launch
    except OSError:
        pass
    return None


def main():
    args = parse()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU (units are independent; no collective exists in the path); "
              "--gpus N with N > 1 is not supported", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2404_15949_amd import corm, inputs

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    corm.lib()  # fail loudly now if the HIP library is missing
    corm.corm_force_path(args.path)

    wl = inputs.WORKLOADS[args.workload]
    if args.structured:
        wl = wl.replace(q_mean_scales=inputs.STRUCTURED_Q_MEAN)
    if args.w is not None or args.r is not None:
        w_new = wl.w if args.w is None else args.w
        wl = wl.replace(w=w_new, r=w_new if args.r is None else args.r)
        assert 1 <= wl.w and 1 <= wl.r, "w and r must be at least 1"
    layers = wl.layers if args.layers is None else args.layers
    K_steps, W_steps = args.steps, args.warmup
    n_dec = W_steps + K_steps + args.extra_steps
    n_replay = min(wl.w, wl.P)
    Lcap = Tcap = (wl.P + n_dec + 63) // 64 * 64   # ring rows start on 128-byte lines (seeding stores whole lines)
    esz = 2 if wl.dtype == "bf16" else 4
    B, Hq, Hkv, d = wl.B, wl.Hq, wl.Hkv, wl.d

    # the resident state must fit the device: say so before allocating anything
    ring_b = 0 if args.no_ring else layers * B * Hq * wl.w * (Tcap // 8 if args.ring == "bits" else Tcap * esz)
    kv_b = 2 * layers * B * Hkv * Lcap * (d * esz + 4)
    total_mem = torch.cuda.mem_get_info()[1]
    if ring_b + kv_b > 0.93 * total_mem:
        print(f"bench.py: the state of this run ({kv_b / 2**30:.0f} GiB of K, V and metadata + {ring_b / 2**30:.0f} GiB "
              f"of score ring) does not fit the device ({total_mem / 2**30:.0f} GiB); use --ring bits, --no-ring or a "
              f"smaller --w / --layers", file=sys.stderr)
        sys.exit(2)

    # ---------------- set-up (untimed): allocate, generate, feed the prompt
    t0 = time.time()
    score_dtype = "bit" if args.ring == "bits" else None
    desc = corm.make_desc(B, Hq, Hkv, d, Lcap, Tcap, wl.w, wl.r, wl.dtype, score_dtype=score_dtype)
    ws = torch.empty(corm.corm_workspace_bytes(desc), dtype=torch.uint8, device=dev)
    corm.corm_workspace_init(desc, ws)
    lens_all = torch.zeros(layers, B, Hkv, dtype=torch.int32, device=dev)
    lazy = tuple(int(v) for v in args.lazy_frac.split("/")) if args.lazy_frac else None
    nlive_all = torch.zeros(layers, B, Hkv, dtype=torch.int32, device=dev)   # lazy mode: live keys per unit
    states, Qs, Kns, Vns = [], [], [], []
    pre = wl.P - n_replay
    t_all = (torch.arange(n_replay + n_dec, dtype=torch.int32, device=dev) + (pre + 1)).view(-1, 1).repeat(1, B)
    t_first = torch.full((B,), pre + 1, dtype=torch.int32, device=dev)
    for l in range(layers):
        st = corm.LayerState(B, Hq, Hkv, d, Lcap, Tcap, wl.w, wl.r, wl.dtype, device=dev, workspace=ws,
                             want_ring=not args.no_ring, score_dtype=score_dtype)
        st.lens = lens_all[l]
        st.nlive = nlive_all[l]
        x = inputs.make_layer(wl, l, device=dev, n_decode=n_dec, n_replay=n_replay)
        if args.seed == "kernel":
            st.preload(x["K0"], x["V0"])          # the whole prompt; the seeding call comes below
            Kns.append(x["Kn"])
            Vns.append(x["Vn"])
        else:
            st.preload(x["K0"][:, :, :pre], x["V0"][:, :, :pre])
            # keys/values of the replayed prompt tail in step-major layout, then the decode tokens
            Kt = x["K0"][:, :, pre:].permute(2, 0, 1, 3).contiguous()
            Vt = x["V0"][:, :, pre:].permute(2, 0, 1, 3).contiguous()
            Kns.append(torch.cat([Kt, x["Kn"]], dim=0))
            Vns.append(torch.cat([Vt, x["Vn"]], dim=0))
            del Kt, Vt
        Qs.append(x["Q"])
        states.append(st)
        del x
    torch.cuda.synchronize()
    log(f"allocated + generated {layers} layers in {time.time() - t0:.1f}s; "
        f"{torch.cuda.memory_allocated() / 2**30:.1f} GiB resident")

    # Launch order of one step.  --streams 1: every layer's fused step call on one stream.  --streams N:
    # layers are dealt round-robin to N streams, each with its own workspace.  Layers are independent and a
    # layer always runs on the same stream, so no event is needed; the device overlaps the tail of one
    # layer's launch (its record / compaction work, which moves few bytes) with the head of the next.
    main = torch.cuda.current_stream()
    streams = [main] + [torch.cuda.Stream() for _ in range(args.streams - 1)]
    wss = [ws] + [torch.empty_like(ws) for _ in range(args.streams - 1)]
    for extra in streams[1:]:
        extra.wait_stream(main)

    kv_off = n_replay if args.seed == "kernel" else 0   # Kns / Vns start at the first decode token

    def layer_step(l, j, tj, wsk, stream):
        st = states[l]
        kn, vn = Kns[l][j - kv_off], Vns[l][j - kv_off]
        if lazy:
            corm.corm_decode_step_lazy(st.desc, Qs[l][j], kn, vn, st.K, st.V, st.lens, st.live, st.pos,
                                       st.last_hit, tj, t_first, st.ring, st.out, None, st.nlive, lazy[0], lazy[1],
                                       wsk, status=st.status, stream=stream)
        else:
            corm.corm_decode_step(st.desc, Qs[l][j], kn, vn, st.K, st.V, st.lens, st.pos, st.last_hit,
                                  tj, t_first, st.ring, st.out, None, None, wsk, status=st.status, stream=stream)

    def run_step(j, probe_layer=-1, probe_events=None):
        tj = t_all[j]
        for l in range(layers):
            if l == probe_layer:
                corm.corm_profile_attend(probe_events[0], probe_events[1])
            k = l % len(streams)
            layer_step(l, j, tj, wss[k], streams[k])

    def join():
        for extra in streams[1:]:
            main.wait_stream(extra)

    def fork():
        for extra in streams[1:]:
            extra.wait_stream(main)

    t0 = time.time()
    seeding = {"how": "replay of the last w prompt tokens through corm_decode_step"}
    if args.seed == "kernel":
        # one dense call per layer: ring rows and last_hit of the last w prompt queries, then the bulk eviction
        t_last = torch.full((B,), wl.P, dtype=torch.int32, device=dev)
        tf_out = torch.zeros_like(t_first)
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(layers + 1)]
        ev[0].record()
        for l in range(layers):
            q_tail = Qs[l][:n_replay].permute(1, 2, 0, 3).contiguous()
            st = states[l]
            corm.corm_prefill_seed(st.desc, q_tail, n_replay, st.K, st.V, st.lens, st.pos, st.last_hit, t_last, tf_out,
                                   st.ring, None, None, ws, status=st.status)
            ev[l + 1].record()
            del q_tail
        torch.cuda.synchronize()
        assert torch.equal(tf_out, t_first)
        ms = sorted(ev[l].elapsed_time(ev[l + 1]) for l in range(layers))
        pairs = n_replay * wl.P - n_replay * (n_replay - 1) // 2     # (query, visible key) pairs per head
        seeding = {"how": "corm_prefill_seed, one call per layer (layout copy of the queries included)",
                   "median_ms_per_layer": ms[len(ms) // 2],
                   "algorithmic_tflops": 2.0 * d * pairs * B * Hq / (ms[len(ms) // 2] * 1e-3) / 1e12,
                   "ring_gb_written_per_layer": 0.0 if args.no_ring else
                   pairs * B * Hq * (0.125 if args.ring == "bits" else esz) / 1e9}
    else:
        for j in range(n_replay):          # prompt tail: seeds the recent-query window; bulk eviction at its end
            run_step(j)
        join()
        torch.cuda.synchronize()
    # keys_all: the live keys per unit (what the next step attends to); lens_all also counts dead slots
    keys_all = nlive_all if lazy else lens_all
    log(f"prompt seeding ({args.seed}, last {n_replay} positions) {time.time() - t0:.1f}s; "
        f"live fraction after the prompt {keys_all.float().mean().item() / wl.P:.4f}")
    assert all(int(s.status.item()) == 0 for s in states)

    # ---------------- CPU baseline: the oracle, timed on a bounded sample of the same workload
    cpu_baseline = None
    # (the oracle is rebuilt from compacted device snapshots and from the recorded score window)
    if not args.no_cpu_baseline and not lazy and not args.no_ring:
        cpu_baseline = cpu_baseline_leg(args, wl, states, Qs, Kns, Vns, n_replay, pre, layers, kv_off)

    if args.calibrate_copy:
        src = torch.ones(2 ** 28, dtype=torch.float32, device=dev)   # 1 GiB read + 1 GiB written
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---------------- warm-up, then the timed region
    for j in range(n_replay, n_replay + W_steps):
        run_step(j)
    join()
    lens_hist = torch.empty(K_steps + 1, layers, B, Hkv, dtype=torch.int32, device=dev)
    lens_hist[0].copy_(keys_all)
    # HIP events around the attend kernel of ONE launch per step (layer k mod layers), recorded by the
    # library on the stream it launches on: the dominant kernel's duration, measured inside the timed region
    hip = HipEvents()
    pairs = [(hip.create(), hip.create()) for _ in range(K_steps)]
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ev0.record()
    fork()
    for k in range(K_steps):
        run_step(n_replay + W_steps + k, probe_layer=k % layers, probe_events=pairs[k])
        join()                             # the step ends when every stream has finished it
        lens_hist[k + 1].copy_(keys_all)   # one tiny copy per step: the live lengths the next step starts from
        fork()
    ev1.record()
    torch.cuda.synchronize()
    ms_total = ev0.elapsed_time(ev1)
    assert all(int(s.status.item()) == 0 for s in states)

    ms_per_step = ms_total / K_steps
    n_launch = K_steps * layers
    ssz = 0 if args.no_ring else (0.125 if args.ring == "bits" else esz)   # ring bytes per key and head
    # the whole step (every launch of every layer) against its algorithmic bytes
    total_bytes = sum(algorithmic_bytes(lens_hist[k], wl, esz, ssz) for k in range(K_steps))
    step_gbs = total_bytes / (ms_total * 1e-3) / 1e9
    # The dominant kernel (the launch that streams K and V).  With several streams its launches overlap, so
    # a per-launch event duration also counts the time a launch waits for compute units held by its
    # neighbour; an exclusive measurement follows the timed region: a few more steps on ONE stream with
    # events around every such launch.
    overlapped_ms = sum(hip.elapsed_ms(a, b_) for (a, b_) in pairs) / len(pairs)
    n_probe_steps = min(4, args.extra_steps)
    probe_pairs, probe_bytes = [], []
    for s in range(n_probe_steps):
        j = n_replay + W_steps + K_steps + s
        tj = t_all[j]
        lens_now = keys_all.clone()
        for l in range(layers):
            pr = (hip.create(), hip.create())
            corm.corm_profile_attend(pr[0], pr[1])
            layer_step(l, j, tj, wss[0], main)
            probe_pairs.append(pr)
            probe_bytes.append(algorithmic_bytes(lens_now[l], wl, esz, ssz, "attend"))
    torch.cuda.synchronize()
    probe_ms = [hip.elapsed_ms(a, b_) for (a, b_) in probe_pairs]
    avg_attend_ms = sum(probe_ms) / len(probe_ms)
    bytes_per_launch = sum(probe_bytes) / len(probe_bytes)
    achieved = bytes_per_launch / (avg_attend_ms * 1e-3) / 1e9
    live_end = lens_hist[-1].float().mean().item() / (wl.P + W_steps + K_steps)
    unit_path = corm.corm_selected_path(desc) == 2
    gqa_mfma = wl.dtype == "bf16" and d == 128 and wl.G > 1 and args.path != 3
    kernel_name = "corm_unit_kernel" if unit_path else ("corm_attend_gqa_kernel" if gqa_mfma else "corm_attend_kernel")
    evicted = int((lens_hist[:-1].long() + 1 - lens_hist[1:].long()).sum().item())

    result = {
        "metric": "decode steps/sec and achieved HBM GB/s (% of peak), attend+evict+compact",
        "value": 1000.0 / ms_per_step,
        "unit": "decode steps/s",
        "n_gpus": 1, "steps": K_steps, "warmup": W_steps, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": wl.dtype, "data": "synthetic",
        "device": f"{torch.cuda.get_device_name(0) or 'AMD GPU'} ({torch.cuda.get_device_properties(0).gcnArchName}, "
                  f"{torch.cuda.get_device_properties(0).multi_processor_count} CUs, {total_mem / 2**30:.0f} GiB)",
        "config": {"workload": wl.name + ("+structured_queries" if args.structured else ""),
                   "layers": layers, "batch": B, "q_heads": Hq, "kv_heads": Hkv, "head_dim": d,
                   "prompt": wl.P, "w": wl.w, "r": wl.r, "tokens_per_step": B, "streams": args.streams, "path": corm.corm_selected_path(desc),
                   "score_ring": "none (summary-only state)" if args.no_ring else
                   ("boolean message, 1 bit per entry" if args.ring == "bits" else f"{wl.dtype} probabilities"),
                   "compaction": f"deferred until {lazy[0]}/{lazy[1]} of a unit's slots are dead" if lazy
                   else "at every step",
                   "live_fraction_end": live_end, "keys_evicted_in_timed_region": evicted},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS,
                     "traffic": measured_traffic(kernel_name, wl.name, bytes_per_launch),
                     "kernel": kernel_name, "bytes_per_launch": bytes_per_launch,
                     "avg_launch_ms": avg_attend_ms, "launches_probed": len(probe_ms),
                     "how": "exclusive: one stream, HIP events around every launch of this kernel, "
                            f"{n_probe_steps} steps right after the timed region",
                     "avg_launch_ms_overlapped_in_timed_region": overlapped_ms},
        "whole_step": {"achieved": step_gbs, "unit": "GB/s", "frac": step_gbs / HBM_PEAK_GBS,
                       "avg_layer_step_ms": ms_total / n_launch, "layer_steps": n_launch,
                       "note": "algorithmic bytes of all launches / wall time of the timed region "
                               "(every kernel of the step, launch gaps included)"},
        "prompt_seeding_untimed": seeding,
        "cpu_baseline": cpu_baseline,
    }
    if cpu_baseline:
        result["gpu_over_cpu"] = result["value"] / cpu_baseline["value"]
    print(json.dumps(result), flush=True)


class HipEvents:
    """Raw hipEvent_t handles through the HIP runtime that torch already loaded (plumbing only)."""

    def __init__(self):
        import ctypes
        self.ct = ctypes
        self.hip = ctypes.CDLL("libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]

    def create(self) -> int:
        ev = self.ct.c_void_p()
        rc = self.hip.hipEventCreate(self.ct.byref(ev))
        assert rc == 0, f"hipEventCreate failed: {rc}"
        return ev.value

    def elapsed_ms(self, a: int, b: int) -> float:
        ms = self.ct.c_float()
        rc = self.hip.hipEventElapsedTime(self.ct.byref(ms), a, b)
        assert rc == 0, f"hipEventElapsedTime failed: {rc}"
        return ms.value


def cpu_baseline_leg(args, wl, states, Qs, Kns, Vns, n_replay, pre, layers, kv_off):
    """Time the oracle (as it stands) on a sample of units of the workload's first decode steps, starting
    from copies of the device state after the prompt.  The device state is not touched."""
    import numpy as np
    import torch
    from concurrent.futures import ThreadPoolExecutor
    from oracle.snapshot import unit_from_device_arrays

    rng = np.random.default_rng(0)
    # (no more oracle steps than decode inputs were generated: a short --steps / --warmup run has few)
    n_units, n_steps = args.cpu_units, max(1, min(args.cpu_steps, Kns[0].shape[0] - (n_replay - kv_off)))
    G = wl.G
    picks = [(int(rng.integers(layers)), int(rng.integers(wl.B)), int(rng.integers(wl.Hkv))) for _ in range(n_units)]
    t_prev = wl.P
    work = []
    for (l, b, h) in picks:
        st = states[l]
        u = unit_from_device_arrays(st.K, st.V, st.pos, st.lens, st.ring, b, h, G, wl.w, wl.r, t_prev, pre + 1,
                                    wl.dtype, 1.0)
        q = Qs[l][n_replay:n_replay + n_steps, b, h * G:(h + 1) * G].float().cpu().numpy()
        k = Kns[l][n_replay - kv_off:n_replay - kv_off + n_steps, b, h].float().cpu().numpy()
        v = Vns[l][n_replay - kv_off:n_replay - kv_off + n_steps, b, h].float().cpu().numpy()
        work.append((u, q, k, v))
    cores = min(os.cpu_count() or 1, 16)

    def run(item):
        u, q, k, v = item
        for s in range(n_steps):
            u.step(q[s], k[s], v[s], t_prev + 1 + s)
        return u.l

    t0 = time.perf_counter()
    with ThreadPoolExecutor(max_workers=cores) as ex:
        list(ex.map(run, work))
    dt = time.perf_counter() - t0
    unit_steps_per_s = n_units * n_steps / dt
    units_per_step = layers * wl.B * wl.Hkv
    log(f"cpu baseline: {n_units} units x {n_steps} steps in {dt:.1f}s on {cores} threads")
    return {"value": unit_steps_per_s / units_per_step, "unit": "decode steps/s", "cores": cores, "kind": "oracle",
            "sample": f"{n_units} random (layer, sequence, head) units x {n_steps} decode steps from the state after "
                      f"the prompt, {dt:.1f} s wall; extrapolated to the {units_per_step} units of a full step"}


if __name__ == "__main__":
    main()
