#!/usr/bin/env python3
"""Benchmark of the CORM decode hot path on one MI355X.

A "step" is one decode step of the whole stack: for every layer, in sequence on ONE stream (layers of a
model depend on each other), one fused call that appends the token's key/value, attends over every
unit's live keys, records the scores, decides the evictions and compacts the caches.  Default workload:
the LLaMA-2-7B-shaped full stack (32 layers x 32 heads, d 128, bf16, batch 16, prompt 4096,
w = r = 1024) on seeded synthetic inputs.  Inputs are resident in HBM before the timed region; the
prompt is untimed set-up.

`value` is that sequential number.  The same JSON line also carries, measured in the same run:
  overlapped      the same stack with independent layers dealt to three streams (what a model's other
                  kernels would hide: the record / compaction tail of one layer under the next),
  eviction_heavy  the labelled supplementary variant of the workload (per-head query means, live
                  fraction ~0.37: the regime the method is for), with compaction at every step and
                  deferred, sequential layers,
  roofline        the dominant kernel, HIP events around its launches inside the timed region,
  cpu_baseline    the CPU oracle on a bounded sample.

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
    ap.add_argument("--steps", type=int, default=128)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--workload", default="llama7b_b16")
    ap.add_argument("--layers", type=int, default=None, help="override the number of layers: a stack of layers of the workload's shape (the one-layer workloads as "
                    "a model with that many layers would run them), or fewer layers for short counter runs")
    ap.add_argument("--structured", action="store_true",
                    help="run the supplementary variant AS the main workload: per-head query means so that "
                         "eviction happens at w >= 256")
    ap.add_argument("--w", type=int, default=None, help="override the window of recorded queries (the paper's w/r "
                    "sweep, Section 5; the ring holds w rows, so memory follows it)")
    ap.add_argument("--r", type=int, default=None, help="override the number of protected recent keys (default: = w)")
    ap.add_argument("--streams", type=int, default=1, choices=[1, 2, 3, 4],
                    help="streams of the region that gives `value`: 1 = layers in sequence (default); N = independent "
                         "layers dealt round-robin to N streams")
    ap.add_argument("--overlap-streams", type=int, default=3, choices=[0, 2, 3, 4],
                    help="streams of the additional `overlapped` region (0 = skip it)")
    ap.add_argument("--path", type=int, default=0, choices=[0, 1, 2, 3],
                    help="corm_launch_opts.path: 0 by shape, 1 split kernels, 2 one workgroup per unit, 3 split without MFMA")
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
    ap.add_argument("--no-eviction-heavy", action="store_true",
                    help="skip the supplementary eviction-heavy leg (it runs by default on the headline workload)")
    ap.add_argument("--eviction-heavy-steps", type=int, default=None,
                    help="timed steps of each mode of the eviction-heavy leg (default: --steps, at most 64)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (reference dispatch for rocprofv3 byte counters)")
    ap.add_argument("--cpu-units", type=int, default=128)
    ap.add_argument("--cpu-steps", type=int, default=16)
    return ap.parse_args()


def algorithmic_bytes(lens_before, wl, esz, ssz, part="step"):
    """Bytes a launch must move for units whose live lengths (before the append) are lens_before.
    part="attend": what a split-path attend kernel streams -- every live K and V row once, plus per unit the G
    queries, k_new and v_new read and the appended row written.
    part="step": the whole layer-step, which is also what the fused unit kernel does in one launch: that plus
    the ring row written (G * score bytes per key), pos and last_hit read (8 B per key), out written.
    Rows moved by the compaction, the logits scratch and the split partials are NOT counted."""
    L = lens_before.double() + 1.0
    per_key = 2 * wl.d * esz
    per_unit = (wl.G + 4) * wl.d * esz
    if part == "step":
        per_key += wl.G * ssz + 8
        per_unit += wl.G * wl.d * 4
    return float((L * per_key).sum().item() + L.numel() * per_unit)


def committed_traffic(kernel, workload, bytes_per_launch):
    """HBM bytes per launch of the dominant kernel from the COMMITTED rocprofv3 counter summary (FETCH_SIZE +
    WRITE_SIZE, calibrated against a plain copy): the ratio traffic / algorithmic bytes measured there, applied
    to this run's algorithmic bytes per launch.  Not measured in this run (counters need the profiler).
    Returns (bytes or None, where the figure comes from)."""
    rel = "profiles/unit_kernel_llama7b_b16_hbm_traffic.txt"
    try:
        for line in open(os.path.join(ROOT, rel)):
            if line.startswith("traffic_bytes_per_launch="):
                kv = dict(item.split("=") for item in line.split())
                if kv["kernel"] == kernel and kv["workload"] == workload:
                    ratio = float(kv["traffic_bytes_per_launch"]) / float(kv["algorithmic_bytes_per_launch"])
                    return ratio * bytes_per_launch, f"{rel} (rocprofv3 FETCH_SIZE + WRITE_SIZE of a profiled run of " \
                                                     f"this kernel: traffic / algorithmic = {ratio:.3f}, applied to " \
                                                     "this run's bytes per launch; NOT measured in this run)"
    except OSError:
        pass
    return None, "no committed counter summary for this kernel and workload"


class HipEvents:
    """Raw hipEvent_t handles through the HIP runtime that torch already loaded (plumbing only)."""

    def __init__(self):
        import ctypes
        self.ct = ctypes
        self.hip = ctypes.CDLL("libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self.hip.hipEventDestroy.argtypes = [ctypes.c_void_p]

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

    def destroy(self, *evs) -> None:
        for e in evs:
            self.hip.hipEventDestroy(e)


class Stack:
    """Device state and inputs of `layers` layers of one workload, the prompt already fed (untimed set-up)."""

    def __init__(self, args, wl, layers, n_dec, dev):
        import torch
        from paper_2404_15949_amd import corm, inputs
        self.torch, self.corm = torch, corm
        self.args, self.wl, self.layers, self.dev = args, wl, layers, dev
        self.n_replay = n_replay = min(wl.w, wl.P)
        self.esz = esz = 2 if wl.dtype == "bf16" else 4
        B, Hq, Hkv, d = wl.B, wl.Hq, wl.Hkv, wl.d
        self.Lcap = Lcap = Tcap = (wl.P + n_dec + 63) // 64 * 64   # ring rows start on 128-byte lines (seeding stores whole lines)
        self.ssz = 0 if args.no_ring else (0.125 if args.ring == "bits" else esz)   # ring bytes per key and head

        # the resident state must fit the device: say so before allocating anything
        ring_b = 0 if args.no_ring else layers * B * Hq * wl.w * (Tcap // 8 if args.ring == "bits" else Tcap * esz)
        kv_b = 2 * layers * B * Hkv * Lcap * (d * esz + 4)
        free_mem, self.total_mem = torch.cuda.mem_get_info()
        if ring_b + kv_b > 0.93 * free_mem:
            print(f"bench.py: the state of this run ({kv_b / 2**30:.0f} GiB of K, V and metadata + {ring_b / 2**30:.0f} GiB "
                  f"of score ring) does not fit the device ({free_mem / 2**30:.0f} of {self.total_mem / 2**30:.0f} GiB free); "
                  f"use --ring bits, --no-ring or a smaller --w / --layers", file=sys.stderr)
            sys.exit(2)

        t0 = time.time()
        score_dtype = "bit" if args.ring == "bits" else None
        self.desc = corm.make_desc(B, Hq, Hkv, d, Lcap, Tcap, wl.w, wl.r, wl.dtype, score_dtype=score_dtype)
        self.ws = torch.empty(corm.corm_workspace_bytes(self.desc), dtype=torch.uint8, device=dev)
        corm.corm_workspace_init(self.desc, self.ws)
        self.wss = [self.ws]
        self.lens_all = torch.zeros(layers, B, Hkv, dtype=torch.int32, device=dev)
        self.nlive_all = torch.zeros(layers, B, Hkv, dtype=torch.int32, device=dev)   # deferred mode: live keys per unit
        self.states, self.Qs, self.Kns, self.Vns = [], [], [], []
        self.pre = pre = wl.P - n_replay
        self.t_all = (torch.arange(n_replay + n_dec, dtype=torch.int32, device=dev) + (pre + 1)).view(-1, 1).repeat(1, B)
        self.t_first = torch.full((B,), pre + 1, dtype=torch.int32, device=dev)
        for l in range(layers):
            st = corm.LayerState(B, Hq, Hkv, d, Lcap, Tcap, wl.w, wl.r, wl.dtype, device=dev, workspace=self.ws,
                                 want_ring=not args.no_ring, score_dtype=score_dtype)
            st.lens = self.lens_all[l]
            st.nlive = self.nlive_all[l]
            x = inputs.make_layer(wl, l, device=dev, n_decode=n_dec, n_replay=n_replay)
            if args.seed == "kernel":
                st.preload(x["K0"], x["V0"])          # the whole prompt; the seeding call comes below
                self.Kns.append(x["Kn"])
                self.Vns.append(x["Vn"])
            else:
                st.preload(x["K0"][:, :, :pre], x["V0"][:, :, :pre])
                # keys/values of the replayed prompt tail in step-major layout, then the decode tokens
                Kt = x["K0"][:, :, pre:].permute(2, 0, 1, 3).contiguous()
                Vt = x["V0"][:, :, pre:].permute(2, 0, 1, 3).contiguous()
                self.Kns.append(torch.cat([Kt, x["Kn"]], dim=0))
                self.Vns.append(torch.cat([Vt, x["Vn"]], dim=0))
                del Kt, Vt
            self.Qs.append(x["Q"])
            self.states.append(st)
            del x
        torch.cuda.synchronize()
        log(f"{wl.name}{'+structured_queries' if wl.q_mean_scales else ''}: allocated + generated {layers} layers in "
            f"{time.time() - t0:.1f}s; {torch.cuda.memory_allocated() / 2**30:.1f} GiB resident")
        self.kv_off = n_replay if args.seed == "kernel" else 0   # Kns / Vns start at the first decode token
        self.main = torch.cuda.current_stream()
        self.extra_streams = []
        self.next_j = n_replay          # trajectory step the next region starts from
        self.seeding = self._feed_prompt()

    def workspaces(self, n):
        while len(self.wss) < n:
            self.wss.append(self.torch.empty_like(self.ws))
        return self.wss[:n]

    def streams(self, n):
        while len(self.extra_streams) < n - 1:
            self.extra_streams.append(self.torch.cuda.Stream())
        return [self.main] + self.extra_streams[:n - 1]

    def layer_step(self, l, j, tj, wsk, stream, lazy=None, events=None):
        """One fused call.  events: (start, stop) hipEvent_t handles the library records around the launch that
        streams K and V."""
        corm, st = self.corm, self.states[l]
        kn, vn = self.Kns[l][j - self.kv_off], self.Vns[l][j - self.kv_off]
        opts = corm.make_opts(attend_events=events) if events else None
        if lazy:
            corm.corm_decode_step_lazy(st.desc, self.Qs[l][j], kn, vn, st.K, st.V, st.lens, st.live, st.pos,
                                       st.last_hit, tj, self.t_first, st.ring, st.out, None, st.nlive, lazy[0], lazy[1],
                                       wsk, status=st.status, stream=stream, opts=opts)
        else:
            corm.corm_decode_step(st.desc, self.Qs[l][j], kn, vn, st.K, st.V, st.lens, st.pos, st.last_hit,
                                  tj, self.t_first, st.ring, st.out, None, None, wsk, status=st.status, stream=stream,
                                  opts=opts)

    def _feed_prompt(self):
        torch, corm, wl, args = self.torch, self.corm, self.wl, self.args
        n_replay, layers, B = self.n_replay, self.layers, wl.B
        t0 = time.time()
        seeding = {"how": "replay of the last w prompt tokens through corm_decode_step"}
        if args.seed == "kernel":
            # one dense call per layer: ring rows and last_hit of the last w prompt queries, then the bulk eviction
            t_last = torch.full((B,), wl.P, dtype=torch.int32, device=self.dev)
            tf_out = torch.zeros_like(self.t_first)
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(layers + 1)]
            ev[0].record()
            for l in range(layers):
                q_tail = self.Qs[l][:n_replay].permute(1, 2, 0, 3).contiguous()
                st = self.states[l]
                corm.corm_prefill_seed(st.desc, q_tail, n_replay, st.K, st.V, st.lens, st.pos, st.last_hit, t_last,
                                       tf_out, st.ring, None, None, self.ws, status=st.status)
                ev[l + 1].record()
                del q_tail
            torch.cuda.synchronize()
            assert torch.equal(tf_out, self.t_first)
            ms = sorted(ev[l].elapsed_time(ev[l + 1]) for l in range(layers))
            pairs = n_replay * wl.P - n_replay * (n_replay - 1) // 2     # (query, visible key) pairs per head
            seeding = {"how": "corm_prefill_seed, one call per layer (layout copy of the queries included)",
                       "median_ms_per_layer": ms[len(ms) // 2],
                       "algorithmic_tflops": 2.0 * wl.d * pairs * B * wl.Hq / (ms[len(ms) // 2] * 1e-3) / 1e12,
                       "ring_gb_written_per_layer": 0.0 if args.no_ring else
                       pairs * B * wl.Hq * (0.125 if args.ring == "bits" else self.esz) / 1e9}
        else:
            for j in range(n_replay):          # prompt tail: seeds the recent-query window; bulk eviction at its end
                for l in range(layers):
                    self.layer_step(l, j, self.t_all[j], self.ws, self.main)
            torch.cuda.synchronize()
        self.nlive_all.copy_(self.lens_all)    # (every slot below lens is live after the prompt)
        log(f"prompt seeding ({args.seed}, last {n_replay} positions) {time.time() - t0:.1f}s; "
            f"live fraction after the prompt {self.lens_all.float().mean().item() / wl.P:.4f}")
        self.check_status()
        return seeding

    def check_status(self):
        assert all(int(s.status.item()) == 0 for s in self.states), "a kernel flagged a device-side condition"

    def region(self, n_steps, n_streams, lazy=None, hip=None, probe=False):
        """Runs n_steps decode steps of the whole stack from where the last region ended.  n_streams == 1: every
        layer's call on one stream, in layer order.  n_streams > 1: layers dealt round-robin to that many
        streams, each with a workspace of its own; a layer always runs on the same stream, so no event is
        needed between its steps, and all streams are joined at the end of every step.
        Returns wall ms, the live lengths every step started from and ended with [n_steps + 1, layers, B, Hkv],
        and (probe) the dominant-kernel launches that were bracketed by HIP events: one launch per step, layer
        k mod layers in step k, as (ms, live lengths before that launch)."""
        torch = self.torch
        layers = self.layers
        streams = self.streams(n_streams)
        wss = self.workspaces(n_streams)
        keys_all = self.nlive_all if lazy else self.lens_all
        hist = torch.empty(n_steps + 1, layers, self.wl.B, self.wl.Hkv, dtype=torch.int32, device=self.dev)
        hist[0].copy_(keys_all)
        pairs = [(hip.create(), hip.create()) for _ in range(n_steps)] if probe else None
        torch.cuda.synchronize()
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ev0.record()
        for extra in streams[1:]:
            extra.wait_stream(self.main)
        for k in range(n_steps):
            j = self.next_j + k
            tj = self.t_all[j]
            for l in range(layers):
                s = l % n_streams
                self.layer_step(l, j, tj, wss[s], streams[s], lazy, pairs[k] if probe and l == k % layers else None)
            for extra in streams[1:]:          # the step ends when every stream has finished it
                self.main.wait_stream(extra)
            hist[k + 1].copy_(keys_all)        # one tiny copy per step: the live lengths the next step starts from
            for extra in streams[1:]:
                extra.wait_stream(self.main)
        ev1.record()
        torch.cuda.synchronize()
        self.next_j += n_steps
        self.check_status()
        probes = None
        if probe:
            probes = [(hip.elapsed_ms(a, b_), hist[k, k % layers]) for k, (a, b_) in enumerate(pairs)]
            hip.destroy(*[e for pr in pairs for e in pr])
        return ev0.elapsed_time(ev1), hist, probes

    def summarize(self, ms_total, hist):
        """steps/s and the whole step against its algorithmic bytes (every launch of every layer, gaps included)."""
        n_steps = hist.shape[0] - 1
        total_bytes = sum(algorithmic_bytes(hist[k], self.wl, self.esz, self.ssz) for k in range(n_steps))
        gbs = total_bytes / (ms_total * 1e-3) / 1e9
        evicted = int((hist[:-1].long() + 1 - hist[1:].long()).sum().item())
        slots = self.wl.P + (self.next_j - self.n_replay)          # tokens every sequence has seen by now
        per_layer = hist[-1].float().mean(dim=(1, 2)) / slots
        return {"steps_per_s": 1000.0 * n_steps / ms_total, "ms_per_step": ms_total / n_steps,
                "avg_layer_step_ms": ms_total / (n_steps * self.layers),
                "whole_step_gbs": gbs, "whole_step_frac": gbs / HBM_PEAK_GBS,
                "live_fraction_end": float(hist[-1].float().mean().item()) / slots,
                "live_fraction_per_layer": {"min": float(per_layer.min().item()), "mean": float(per_layer.mean().item()),
                                            "max": float(per_layer.max().item())},
                "live_fraction_per_head": {"min": float(hist[-1].min().item()) / slots,
                                           "max": float(hist[-1].max().item()) / slots},
                "keys_evicted": evicted, "steps": n_steps}

    def moved_bytes_per_step(self, n_steps=2):
        """Rows the exact compaction moves, counted on a few untimed steps: a survivor whose slot changed is
        read and written once (2 * (2 * d * s + 8) bytes).  Uses the optional kept_idx output of the step call."""
        torch, corm = self.torch, self.corm
        wl = self.wl
        idx = torch.empty(wl.B, wl.Hkv, self.Lcap, dtype=torch.int32, device=self.dev)
        ar = torch.arange(self.Lcap, dtype=torch.int32, device=self.dev).view(1, 1, -1)
        moved = 0
        for k in range(n_steps):
            j = self.next_j + k
            for l in range(self.layers):
                st = self.states[l]
                kn, vn = self.Kns[l][j - self.kv_off], self.Vns[l][j - self.kv_off]
                corm.corm_decode_step(st.desc, self.Qs[l][j], kn, vn, st.K, st.V, st.lens, st.pos, st.last_hit,
                                      self.t_all[j], self.t_first, st.ring, st.out, None, idx, self.ws, status=st.status)
                live = ar < st.lens.view(wl.B, wl.Hkv, 1)
                moved += int(((idx != ar) & live).sum().item())
        self.next_j += n_steps
        self.nlive_all.copy_(self.lens_all)
        return moved / n_steps * 2 * (2 * wl.d * self.esz + 8)

    def free(self):
        self.states.clear(); self.Qs.clear(); self.Kns.clear(); self.Vns.clear(); self.wss.clear()
        self.ws = self.lens_all = self.nlive_all = None
        self.torch.cuda.empty_cache()


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
    corm.set_default_path(args.path)

    wl = inputs.WORKLOADS[args.workload]
    if args.structured:
        wl = wl.replace(q_mean_scales=inputs.STRUCTURED_Q_MEAN)
    if args.w is not None or args.r is not None:
        w_new = wl.w if args.w is None else args.w
        wl = wl.replace(w=w_new, r=w_new if args.r is None else args.r)
        assert 1 <= wl.w and 1 <= wl.r, "w and r must be at least 1"
    layers = wl.layers if args.layers is None else args.layers
    K_steps, W_steps = args.steps, args.warmup
    lazy = tuple(int(v) for v in args.lazy_frac.split("/")) if args.lazy_frac else None
    n_over = K_steps if args.overlap_streams and args.streams == 1 and layers > 1 else 0   # (one layer: nothing to overlap)
    hip = HipEvents()

    stack = Stack(args, wl, layers, W_steps + K_steps + n_over + 2, dev)

    # ---------------- CPU baseline: the oracle, timed on a bounded sample of the same workload
    cpu_baseline = None
    # (the oracle is rebuilt from compacted device snapshots and from the recorded score window)
    if not args.no_cpu_baseline and not args.no_ring:
        cpu_baseline = cpu_baseline_leg(args, stack)

    if args.calibrate_copy:
        src = torch.ones(2 ** 28, dtype=torch.float32, device=dev)   # 1 GiB read + 1 GiB written
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---------------- warm-up, then the timed region that gives `value`
    stack.region(W_steps, args.streams, lazy)
    ms_total, hist, probes = stack.region(K_steps, args.streams, lazy, hip=hip, probe=True)
    head = stack.summarize(ms_total, hist)

    # the dominant kernel (the launch that streams K and V): HIP events recorded by the library on the stream it
    # launches on, around one launch per step of the timed region
    unit_path = corm.corm_selected_path(stack.desc) == 2
    gqa_mfma = wl.dtype == "bf16" and wl.d == 128 and wl.G > 1 and args.path != 3
    kernel_name = "corm_unit_kernel" if unit_path else ("corm_attend_gqa_kernel" if gqa_mfma else "corm_attend_kernel")
    part = "step" if unit_path else "attend"
    probe_ms = [ms for ms, _ in probes]
    probe_bytes = [algorithmic_bytes(lens, wl, stack.esz, stack.ssz, part) for _, lens in probes]
    avg_ms = sum(probe_ms) / len(probe_ms)
    bytes_per_launch = sum(probe_bytes) / len(probe_bytes)
    achieved = bytes_per_launch / (avg_ms * 1e-3) / 1e9
    traffic, traffic_source = committed_traffic(kernel_name, wl.name, bytes_per_launch)
    per_key = 2 * wl.d * stack.esz + (wl.G * stack.ssz + 8 if part == "step" else 0)
    how = ("HIP events recorded by the library around one launch of this kernel per step of the timed region "
           f"(layer k mod {layers} in step k), on the stream it is launched on")
    if args.streams > 1:
        how += f"; {args.streams} streams: a launch's duration includes the time it shares the device with its neighbours"

    # ---------------- the same stack, independent layers overlapped on several streams
    overlapped = None
    if n_over:
        ms_o, hist_o, _ = stack.region(n_over, args.overlap_streams, lazy)
        o = stack.summarize(ms_o, hist_o)
        overlapped = {"streams": args.overlap_streams, "steps_per_s": o["steps_per_s"], "ms_per_step": o["ms_per_step"],
                      "avg_layer_step_ms": o["avg_layer_step_ms"], "whole_step_frac": o["whole_step_frac"],
                      "steps": o["steps"],
                      "note": "layers are independent here, so they can be dealt to streams: the record / compaction "
                              "tail of one layer hides under the next layer's stream, as it would under a model's "
                              "projections and MLP.  Not the headline: a model's layers run in sequence"}

    total_mem = stack.total_mem
    seeding = stack.seeding
    desc_path = corm.corm_selected_path(stack.desc)

    # ---------------- the eviction-heavy variant of the same workload (supplementary, labelled)
    eviction_heavy = None
    if not args.no_eviction_heavy and not args.structured and not lazy and args.workload == "llama7b_b16" \
            and args.w is None and args.seed == "kernel":
        stack.free()
        del stack
        torch.cuda.empty_cache()
        Ke = min(K_steps, 64) if args.eviction_heavy_steps is None else args.eviction_heavy_steps
        wl_e = wl.replace(q_mean_scales=inputs.STRUCTURED_Q_MEAN)
        st_e = Stack(args, wl_e, layers, 2 * (W_steps + Ke) + 4, dev)
        st_e.region(W_steps, 1, None)
        ms_x, hist_x, _ = st_e.region(Ke, 1, None)
        exact = st_e.summarize(ms_x, hist_x)
        moved = st_e.moved_bytes_per_step(2)
        st_e.region(W_steps, 1, (1, 4))
        ms_l, hist_l, _ = st_e.region(Ke, 1, (1, 4))
        lazy_r = st_e.summarize(ms_l, hist_l)
        alg_step = exact["whole_step_gbs"] * 1e9 * exact["ms_per_step"] * 1e-3
        keep = ("steps_per_s", "ms_per_step", "avg_layer_step_ms", "whole_step_frac", "live_fraction_end",
                "live_fraction_per_layer", "live_fraction_per_head", "keys_evicted", "steps")
        eviction_heavy = {
            "workload": wl_e.name + "+structured_queries",
            "what": "the same shapes with a fixed per-head query mean (scales 1, 2, 3, 5 cycling over heads): the "
                    "long-range query similarity real models show and AR(1) queries lack, so that keys are really "
                    "evicted (the paper's ~70 % reduction regime); layers in sequence on one stream",
            "compaction_at_every_step": {**{k: exact[k] for k in keep}, "call": "corm_decode_step",
                                         "moved_bytes_per_step": moved, "algorithmic_bytes_per_step": alg_step,
                                         "moved_over_algorithmic": moved / alg_step},
            "deferred_compaction_1_4": {**{k: lazy_r[k] for k in keep}, "call": "corm_decode_step_lazy, dead 1/4"},
        }
        st_e.free()

    result = {
        "metric": "decode steps/sec and achieved HBM GB/s (% of peak), attend+evict+compact",
        "value": head["steps_per_s"],
        "unit": "decode steps/s",
        "n_gpus": 1, "steps": K_steps, "warmup": W_steps, "ms_per_step": head["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": wl.dtype, "data": "synthetic",
        "value_is": ("layers in sequence on one stream" if args.streams == 1 else
                     f"independent layers dealt round-robin to {args.streams} streams"),
        "device": f"{torch.cuda.get_device_name(0) or 'AMD GPU'} ({torch.cuda.get_device_properties(0).gcnArchName}, "
                  f"{torch.cuda.get_device_properties(0).multi_processor_count} CUs, {total_mem / 2**30:.0f} GiB)",
        "config": {"workload": wl.name + ("+structured_queries" if args.structured else ""),
                   "layers": layers, "batch": wl.B, "q_heads": wl.Hq, "kv_heads": wl.Hkv, "head_dim": wl.d,
                   "prompt": wl.P, "w": wl.w, "r": wl.r, "tokens_per_step": wl.B, "streams": args.streams,
                   "path": desc_path,
                   "score_ring": "none (summary-only state)" if args.no_ring else
                   ("boolean message, 1 bit per entry" if args.ring == "bits" else f"{wl.dtype} probabilities"),
                   "compaction": f"deferred until {lazy[0]}/{lazy[1]} of a unit's slots are dead" if lazy
                   else "at every step",
                   "live_fraction_end": head["live_fraction_end"],
                   "live_fraction_per_layer": head["live_fraction_per_layer"],
                   "live_fraction_per_head": head["live_fraction_per_head"],
                   "keys_evicted_in_timed_region": head["keys_evicted"]},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS,
                     "traffic": traffic, "traffic_source": traffic_source,
                     "kernel": kernel_name, "bytes_per_launch": bytes_per_launch,
                     "bytes_per_key": per_key,
                     "bytes_are": ("K row + V row + ring entries + pos and last_hit per live key, plus per unit the "
                                   "queries, the new key / value, the appended row and out" if part == "step" else
                                   "K row + V row per live key, plus per unit the queries, the new key / value and the "
                                   "appended row (the record launch's bytes are not this kernel's)"),
                     "avg_launch_ms": avg_ms, "launches_probed": len(probe_ms), "how": how},
        "whole_step": {"achieved": head["whole_step_gbs"], "unit": "GB/s", "frac": head["whole_step_frac"],
                       "avg_layer_step_ms": head["avg_layer_step_ms"], "layer_steps": K_steps * layers,
                       "note": "algorithmic bytes of all launches / wall time of the timed region "
                               "(every kernel of the step, launch gaps included)"},
        "overlapped": overlapped,
        "eviction_heavy": eviction_heavy,
        "prompt_seeding_untimed": seeding,
        "cpu_baseline": cpu_baseline,
    }
    if cpu_baseline:
        result["gpu_over_cpu"] = result["value"] / cpu_baseline["value"]
    print(json.dumps(result), flush=True)


def cpu_baseline_leg(args, stack):
    """Time the oracle (as it stands) on a sample of units of the workload's first decode steps, starting
    from copies of the device state after the prompt.  The device state is not touched."""
    import numpy as np
    from concurrent.futures import ThreadPoolExecutor
    from oracle.snapshot import unit_from_device_arrays

    wl, layers, n_replay, kv_off = stack.wl, stack.layers, stack.n_replay, stack.kv_off
    rng = np.random.default_rng(0)
    # (no more oracle steps than decode inputs were generated: a short --steps / --warmup run has few)
    n_units, n_steps = args.cpu_units, max(1, min(args.cpu_steps, stack.Kns[0].shape[0] - (n_replay - kv_off)))
    G = wl.G
    picks = [(int(rng.integers(layers)), int(rng.integers(wl.B)), int(rng.integers(wl.Hkv))) for _ in range(n_units)]
    t_prev = wl.P
    work = []
    for (l, b, h) in picks:
        st = stack.states[l]
        u = unit_from_device_arrays(st.K, st.V, st.pos, st.lens, st.ring, b, h, G, wl.w, wl.r, t_prev, stack.pre + 1,
                                    wl.dtype, 1.0)
        q = stack.Qs[l][n_replay:n_replay + n_steps, b, h * G:(h + 1) * G].float().cpu().numpy()
        k = stack.Kns[l][n_replay - kv_off:n_replay - kv_off + n_steps, b, h].float().cpu().numpy()
        v = stack.Vns[l][n_replay - kv_off:n_replay - kv_off + n_steps, b, h].float().cpu().numpy()
        work.append((u, q, k, v))
    host_cores = os.cpu_count() or 1
    threads = min(host_cores, 16)      # the share of host cores that goes with one GPU

    def run(item):
        u, q, k, v = item
        for s in range(n_steps):
            u.step(q[s], k[s], v[s], t_prev + 1 + s)
        return u.l

    t0 = time.perf_counter()
    with ThreadPoolExecutor(max_workers=threads) as ex:
        list(ex.map(run, work))
    dt = time.perf_counter() - t0
    unit_steps_per_s = n_units * n_steps / dt
    units_per_step = layers * wl.B * wl.Hkv
    log(f"cpu baseline: {n_units} units x {n_steps} steps in {dt:.1f}s on {threads} threads ({host_cores} host cores)")
    return {"value": unit_steps_per_s / units_per_step, "unit": "decode steps/s", "cores": host_cores,
            "threads": threads, "kind": "oracle",
            "sample": f"{n_units} random (layer, sequence, head) units x {n_steps} decode steps from the state after "
                      f"the prompt, {dt:.1f} s wall on a pool of {threads} threads over units; extrapolated to the "
                      f"{units_per_step} units of a full step"}


if __name__ == "__main__":
    main()
