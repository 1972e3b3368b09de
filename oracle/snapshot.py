"""Rebuild an oracle unit from copies of plain state arrays.  TEST INFRASTRUCTURE ONLY.

Used for snapshot parity (the oracle resumes from a copy of the cache and of the recorded score
window and must reproduce the next step) and by the benchmark's CPU-baseline leg.  Takes torch
tensors in the layouts the C header documents and only reads them; imports nothing of the
device path.
"""
from __future__ import annotations

import numpy as np
import torch

from . import corm_oracle as O


def _f32(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy()


def unit_from_device_arrays(K, V, pos, lens, ring, b: int, h: int, G: int, w: int, r: int, t_prev: int,
                            t_first: int, dtype: str, thr_scale: float = 1.0) -> O.UnitCache:
    """State of unit (b, h) after step t_prev.

    K, V [B,Hkv,Lcap,d]; pos [B,Hkv,Lcap]; lens [B,Hkv]; ring [B,Hq,w,Tcap] with the row of step
    tau in slot (tau-1) mod w and columns indexed by absolute position (or, int32, the boolean message
    [B,Hq,w,ceil(Tcap/32)]: bit pos % 32 of word pos // 32).  The oracle's notes (which keys each
    recorded query found important) are rebuilt by thresholding each recorded row with its own c/tau
    (Def. 3.1); keys that did not exist at step tau count as minor in that row, whatever the array holds
    there.
    """
    d = K.shape[-1]
    u = O.UnitCache(d, G, w, r, thr_scale, score_dtype=dtype)
    l = int(lens[b, h].item())
    u.keys = _f32(K[b, h, :l]).astype(np.float64)
    u.values = _f32(V[b, h, :l]).astype(np.float64)
    u.positions = pos[b, h, :l].cpu().numpy().astype(np.int64)
    rows = list(range(max(t_first, t_prev - w + 1), t_prev + 1))
    pos_t = torch.from_numpy(u.positions).to(ring.device)
    bits = ring.dtype == torch.int32     # the ring holds the boolean message itself, 32 positions per word
    if bits:
        words = ring[b, h * G:(h + 1) * G].index_select(2, pos_t >> 5)     # [G, w, l]
        sc_all = ((words >> (pos_t & 31)) & 1).cpu().numpy().astype(bool)
    else:
        sc_all = _f32(ring[b, h * G:(h + 1) * G].index_select(2, pos_t))   # [G, w, l]
    width = int(u.positions[-1]) + 1 if l else 0
    notes = np.zeros((len(rows), G, width), dtype=bool)
    for a, tau in enumerate(rows):
        born = u.positions <= tau - 1
        row = sc_all[:, (tau - 1) % w]
        notes[a][:, u.positions] = (row if bits else O.important(row, tau, thr_scale)) & born[None, :]
    u.notes = notes
    u.note_steps = rows
    return u
