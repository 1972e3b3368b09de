"""Seeded synthetic workloads shaped like the paper's LLaMA-2-7B / LLaMA-3-8B runs.

This module only draws random tensors.  It holds none of the method's
arithmetic (no softmax, no threshold, no eviction) and is shared by the HIP
path's tests, the benchmark and the CPU oracle's tests, so that both sides
consume exactly the same stored bits.

The paper evaluates on PG-19 / LongBench text with real model weights
(Section 5, "Settings"); none of that is available here, so keys, values and
queries are synthetic:

* keys and values are i.i.d. N(0,1); keys are multiplied by a per-layer or
  per-head norm scale and a few "attention sink" keys are multiplied by 4;
* queries follow an AR(1) process q_t = rho q_{t-1} + sqrt(1-rho^2) n_t with
  rho = 0.9, which mimics the similarity of adjacent queries that the paper
  observes (Section 3.3), optionally plus a fixed per-head mean vector that
  mimics long-range query similarity;
* everything is rounded once to the workload's storage dtype.

Tensors are produced per layer so that the largest workload can be generated
directly in device memory one layer at a time.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Dict, Optional, Tuple

import torch

RHO = 0.9
SINK_GAIN = 4.0


@dataclasses.dataclass(frozen=True)
class Workload:
    """Shape and recipe of one synthetic workload."""

    name: str
    layers: int
    B: int            # sequences in the batch
    Hq: int           # query heads
    Hkv: int          # key/value heads
    d: int            # head dimension
    dtype: str        # "f32" or "bf16": storage type of q, K, V and of the score ring
    P: int            # prompt length
    D: int            # decode steps
    w: int            # recent-query window
    r: int            # protected recent keys
    key_scale: float = 1.0
    dense_layers: int = 0           # layers [0, dense_layers) use dense_key_scale and no extra sinks
    dense_key_scale: float = 1.0
    n_sinks: int = 4                # number of sink keys per unit
    random_sinks: bool = False      # False: positions 0..n_sinks-1; True: random positions in [0, P)
    odd_head_key_scale: float = 1.0  # extra factor on odd kv heads
    q_mean_scales: Tuple[float, ...] = ()  # per-head persistent query mean; head h uses scales[h % len]
    seed: int = 0

    @property
    def G(self) -> int:
        return self.Hq // self.Hkv

    @property
    def torch_dtype(self) -> torch.dtype:
        return torch.float32 if self.dtype == "f32" else torch.bfloat16

    def replace(self, **kw) -> "Workload":
        return dataclasses.replace(self, **kw)


#: The five workloads of the benchmark definition, in its order.
WORKLOADS: Dict[str, Workload] = {
    "tiny_f32": Workload("tiny_f32", layers=1, B=1, Hq=4, Hkv=4, d=64, dtype="f32",
                         P=512, D=64, w=32, r=32),
    "llama7b_1layer": Workload("llama7b_1layer", layers=1, B=1, Hq=32, Hkv=32, d=128, dtype="bf16",
                               P=4096, D=256, w=1024, r=1024),
    "llama7b_b16": Workload("llama7b_b16", layers=32, B=16, Hq=32, Hkv=32, d=128, dtype="bf16",
                            P=4096, D=512, w=1024, r=1024, key_scale=1.5, dense_layers=2,
                            dense_key_scale=0.5, n_sinks=32, random_sinks=True),
    "long32k": Workload("long32k", layers=1, B=4, Hq=32, Hkv=32, d=128, dtype="bf16",
                        P=32768, D=256, w=2048, r=2048, odd_head_key_scale=2.0),
    "gqa_llama3": Workload("gqa_llama3", layers=1, B=16, Hq=32, Hkv=8, d=128, dtype="bf16",
                           P=8192, D=512, w=1024, r=1024),
}

#: Query-mean scales of the supplementary variant that makes eviction actually
#: happen at w >= 256 (heads cycle through these).
STRUCTURED_Q_MEAN = (1.0, 2.0, 3.0, 5.0)


def _stream_seed(seed: int, name: str, layer: int, kind: str) -> int:
    """A 63-bit seed derived from (seed, workload, layer, tensor kind) by FNV-1a."""
    h = 0xCBF29CE484222325
    for byte in f"{seed}/{name}/{layer}/{kind}".encode():
        h ^= byte
        h = (h * 0x100000001B3) & 0xFFFFFFFFFFFFFFFF
    return h & 0x7FFFFFFFFFFFFFFF


def _generator(wl: Workload, layer: int, kind: str, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(_stream_seed(wl.seed, wl.name, layer, kind))
    return g


def _randn(shape, gen: torch.Generator, device) -> torch.Tensor:
    return torch.randn(shape, generator=gen, device=device, dtype=torch.float32)


def layer_key_scale(wl: Workload, layer: int) -> float:
    return wl.dense_key_scale if layer < wl.dense_layers else wl.key_scale


def make_layer(wl: Workload, layer: int, device="cpu", n_decode: Optional[int] = None,
               n_replay: Optional[int] = None) -> Dict[str, torch.Tensor]:
    """Draw the inputs of one layer.

    Returns a dict of tensors in the workload's storage dtype:

    ``K0, V0``  [B, Hkv, P, d]      prompt keys / values (positions 0..P-1)
    ``Kn, Vn``  [n_decode, B, Hkv, d] keys / values of the decode tokens (positions P..)
    ``Q``       [n_replay + n_decode, B, Hq, d] queries of positions P-n_replay .. P+n_decode-1
    ``sinks``   [B, Hkv, n_sinks] int64 positions of the sink keys (informational)

    ``n_replay`` defaults to min(w, P): the prompt tail whose attention rows
    seed the recent-query window.  ``n_decode`` defaults to ``wl.D``.
    """
    n_decode = wl.D if n_decode is None else n_decode
    n_replay = min(wl.w, wl.P) if n_replay is None else n_replay
    dt = wl.torch_dtype
    B, Hq, Hkv, d, P = wl.B, wl.Hq, wl.Hkv, wl.d, wl.P

    gk = _generator(wl, layer, "K", device)
    gv = _generator(wl, layer, "V", device)
    gq = _generator(wl, layer, "Q", device)
    gs = _generator(wl, layer, "sinks", "cpu")

    scale = layer_key_scale(wl, layer)
    head_scale = torch.full((Hkv,), scale, dtype=torch.float32)
    if wl.odd_head_key_scale != 1.0:
        head_scale[1::2] *= wl.odd_head_key_scale
    head_scale = head_scale.to(device)

    K0 = _randn((B, Hkv, P, d), gk, device) * head_scale.view(1, Hkv, 1, 1)
    Kn = _randn((n_decode, B, Hkv, d), gk, device) * head_scale.view(1, 1, Hkv, 1)
    V0 = _randn((B, Hkv, P, d), gv, device)
    Vn = _randn((n_decode, B, Hkv, d), gv, device)

    # attention sinks: a few prompt keys with a 4x larger norm
    dense = layer < wl.dense_layers
    if wl.random_sinks:
        n_s = 0 if dense else wl.n_sinks
        sinks = torch.stack([torch.randperm(P, generator=gs)[:n_s] for _ in range(B * Hkv)])
        sinks = sinks.view(B, Hkv, n_s).sort(dim=-1).values
    else:
        n_s = min(wl.n_sinks, P)
        sinks = torch.arange(n_s).expand(B, Hkv, n_s).contiguous()
    if n_s:
        idx = sinks.to(device).unsqueeze(-1).expand(B, Hkv, n_s, d)
        K0.scatter_(2, idx, K0.gather(2, idx) * SINK_GAIN)

    # AR(1) queries, stationary N(0,1) marginals, one stream per (b, query head)
    T = n_replay + n_decode
    noise = _randn((T, B, Hq, d), gq, device)
    Q = torch.empty_like(noise)
    c = math.sqrt(1.0 - RHO * RHO)
    Q[0] = noise[0]
    for i in range(1, T):
        torch.add(Q[i - 1] * RHO, noise[i], alpha=c, out=Q[i])
    if wl.q_mean_scales:
        gm = _generator(wl, layer, "Qmean", device)
        a = torch.tensor([wl.q_mean_scales[h % len(wl.q_mean_scales)] for h in range(Hq)],
                         dtype=torch.float32, device=device)
        mu = _randn((B, Hq, d), gm, device) * a.view(1, Hq, 1)
        Q += mu.unsqueeze(0)

    return {"K0": K0.to(dt), "V0": V0.to(dt), "Kn": Kn.to(dt), "Vn": Vn.to(dt),
            "Q": Q.to(dt), "sinks": sinks}


def small_variant(wl: Workload, **kw) -> Workload:
    """A reduced copy of a workload (same recipe, smaller shape) for tests."""
    return wl.replace(**kw)
