"""ctypes binding of libcorm.so: same names and argument order as include/corm.h.

Argument marshalling only -- every step of the path runs in the HIP kernels.
torch is used for device memory and streams: tensors are passed as their
``data_ptr()``.  There is no CPU fallback: if the library has not been built
(``python -c "import __graft_entry__ as g; g.build()"``) loading raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcorm.so")

CORM_F32, CORM_BF16, CORM_BIT = 0, 1, 2
CORM_OK, CORM_EINVAL, CORM_EUNSUPPORTED, CORM_ECAPACITY, CORM_EHIP = 0, -1, -2, -3, -4
CORM_DEV_UNIT_FULL, CORM_DEV_BAD_STEP, CORM_DEV_BAD_LENS = 1, 2, 4
CORM_STATIC_SCRATCH_BYTES = 40 << 20

EXPORTS = ("corm_version", "corm_strerror", "corm_workspace_bytes", "corm_workspace_init", "corm_append",
           "corm_decode_attend", "corm_decode_attend_static", "corm_evict_mask", "corm_evict_mask_summary", "corm_row_density", "corm_compact",
           "corm_decode_step", "corm_step_attend", "corm_step_evict", "corm_decode_step_lazy", "corm_prefill_seed",
           "corm_selected_path", "corm_threshold")


class corm_desc(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("Hq", ctypes.c_int32), ("Hkv", ctypes.c_int32), ("d", ctypes.c_int32),
                ("Lcap", ctypes.c_int32), ("Tcap", ctypes.c_int32), ("w", ctypes.c_int32), ("r", ctypes.c_int32),
                ("kv_dtype", ctypes.c_int32), ("score_dtype", ctypes.c_int32),
                ("thr_scale", ctypes.c_float), ("sm_scale", ctypes.c_float)]


class corm_launch_opts(ctypes.Structure):
    _fields_ = [("path", ctypes.c_int32), ("reserved", ctypes.c_int32),
                ("attend_start_event", ctypes.c_void_p), ("attend_stop_event", ctypes.c_void_p)]


class CormError(RuntimeError):
    def __init__(self, code: int, what: str):
        super().__init__(f"{what}: {strerror(code)} ({code})")
        self.code = code


_lib = None


def lib() -> ctypes.CDLL:
    """Load libcorm.so (once).  Raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it first (__graft_entry__.build()); "
                               "there is no fallback path")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32p, sz = ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t
        dp = ctypes.POINTER(corm_desc)
        op = ctypes.POINTER(corm_launch_opts)
        L.corm_version.restype = ctypes.c_int
        L.corm_version.argtypes = []
        L.corm_strerror.restype = ctypes.c_char_p
        L.corm_strerror.argtypes = [ctypes.c_int]
        L.corm_workspace_bytes.argtypes = [dp, ctypes.POINTER(ctypes.c_size_t)]
        L.corm_workspace_init.argtypes = [dp, vp, sz, vp]
        L.corm_append.argtypes = [dp, vp, vp, i32p, i32p, i32p, vp, vp, i32p, i32p, vp]
        L.corm_decode_attend.argtypes = [dp, vp, vp, vp, i32p, i32p, i32p, vp, i32p, vp, vp, sz, i32p, op, vp]
        L.corm_decode_attend_static.argtypes = [dp, vp, vp, vp, i32p, i32p, i32p, vp, i32p, vp, i32p, op, vp]
        L.corm_evict_mask.argtypes = [dp, vp, i32p, i32p, i32p, i32p, vp, vp]
        L.corm_evict_mask_summary.argtypes = [dp, i32p, i32p, i32p, i32p, vp, vp]
        L.corm_row_density.argtypes = [dp, vp, i32p, i32p, i32p, vp, vp]
        L.corm_compact.argtypes = [dp, vp, vp, i32p, i32p, i32p, vp, i32p, vp, sz, vp]
        L.corm_step_attend.argtypes = [dp, vp, vp, vp, vp, vp, i32p, i32p, i32p, i32p, i32p, vp, vp, vp, vp, sz,
                                       i32p, op, vp]
        L.corm_step_evict.argtypes = [dp, vp, vp, i32p, i32p, i32p, i32p, vp, sz, vp]
        L.corm_selected_path.argtypes = [dp, op]
        L.corm_decode_step.argtypes = [dp, vp, vp, vp, vp, vp, i32p, i32p, i32p, i32p, i32p, vp, vp, vp, i32p,
                                       vp, sz, i32p, op, vp]
        L.corm_decode_step_lazy.argtypes = [dp, vp, vp, vp, vp, vp, i32p, vp, i32p, i32p, i32p, i32p, vp, vp, vp,
                                            i32p, ctypes.c_int32, ctypes.c_int32, vp, sz, i32p, op, vp]
        L.corm_prefill_seed.argtypes = [dp, vp, ctypes.c_int32, vp, vp, i32p, i32p, i32p, i32p, i32p, vp, vp, i32p,
                                        vp, sz, i32p, vp]
        L.corm_threshold.argtypes = [ctypes.c_float, i32p, ctypes.c_int32, vp, vp]
        for name in EXPORTS:
            if name not in ("corm_version", "corm_strerror"):
                getattr(L, name).restype = ctypes.c_int
        _lib = L
    return _lib


def strerror(code: int) -> str:
    return lib().corm_strerror(code).decode()


def _ptr(x) -> Optional[int]:
    """Device (or raw integer) pointer of an argument; None stays NULL."""
    if x is None:
        return None
    if isinstance(x, torch.Tensor):
        return x.data_ptr()
    return int(x)


def _stream(stream) -> Optional[int]:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream if torch.cuda.is_available() else None
    if isinstance(stream, torch.cuda.Stream):
        return stream.cuda_stream
    return int(stream)


# Launch options of the attend / step wrappers below when a call passes none: a setting of this BINDING (the
# library itself keeps no such state), so that a test fixture or the benchmark can route every call of a
# run through one launch path.
_default_path = 0


def set_default_path(path: int) -> None:
    """0 = by shape, 1 = split kernels, 2 = one workgroup per unit, 3 = split kernels without MFMA."""
    global _default_path
    if path not in (0, 1, 2, 3):
        raise ValueError("path must be 0..3")
    _default_path = path


def make_opts(path: Optional[int] = None, attend_events=None) -> corm_launch_opts:
    """attend_events: (start, stop) raw hipEvent_t handles (ints), recorded around the launch that streams K and V."""
    ev = attend_events or (None, None)
    return corm_launch_opts(_default_path if path is None else path, 0, ev[0], ev[1])


def _opts(opts):
    """The pointer argument for a call: the caller's options, or the binding's defaults (NULL when there are none)."""
    if opts is None:
        if _default_path == 0:
            return None
        opts = make_opts()
    return ctypes.byref(opts)


def _check(code: int, what: str) -> int:
    if code != CORM_OK:
        raise CormError(code, what)
    return code


def make_desc(B, Hq, Hkv, d, Lcap, Tcap, w, r, kv_dtype, score_dtype=None, thr_scale=1.0, sm_scale=0.0) -> corm_desc:
    def code(x):
        if x in (CORM_F32, CORM_BF16, CORM_BIT):
            return x
        return {"f32": CORM_F32, "bf16": CORM_BF16, "bit": CORM_BIT, torch.float32: CORM_F32,
                torch.bfloat16: CORM_BF16}[x]
    kv = code(kv_dtype)
    sc = kv if score_dtype is None else code(score_dtype)
    return corm_desc(B, Hq, Hkv, d, Lcap, Tcap, w, r, kv, sc, thr_scale, sm_scale)


# ---- the C entry points, one wrapper each (raise=False returns the status code instead)

def corm_version() -> int:
    return lib().corm_version()


def corm_workspace_bytes(desc: corm_desc, check=True) -> int:
    n = ctypes.c_size_t(0)
    rc = lib().corm_workspace_bytes(ctypes.byref(desc), ctypes.byref(n))
    if check:
        _check(rc, "corm_workspace_bytes")
        return n.value
    return rc


def corm_workspace_init(desc, workspace, workspace_bytes=None, stream=None, check=True) -> int:
    nbytes = workspace.numel() * workspace.element_size() if workspace_bytes is None else workspace_bytes
    rc = lib().corm_workspace_init(ctypes.byref(desc), _ptr(workspace), nbytes, _stream(stream))
    return _check(rc, "corm_workspace_init") if check else rc


def corm_append(desc, K, V, lens, pos, last_hit, k_new, v_new, t, status=None, stream=None, check=True) -> int:
    rc = lib().corm_append(ctypes.byref(desc), _ptr(K), _ptr(V), _ptr(lens), _ptr(pos), _ptr(last_hit),
                           _ptr(k_new), _ptr(v_new), _ptr(t), _ptr(status), _stream(stream))
    return _check(rc, "corm_append") if check else rc


def corm_decode_attend(desc, q, K, V, lens, pos, t, score_ring, last_hit, out, workspace, workspace_bytes=None,
                       status=None, stream=None, check=True, opts=None) -> int:
    nbytes = workspace.numel() * workspace.element_size() if workspace_bytes is None else workspace_bytes
    rc = lib().corm_decode_attend(ctypes.byref(desc), _ptr(q), _ptr(K), _ptr(V), _ptr(lens), _ptr(pos), _ptr(t),
                                  _ptr(score_ring), _ptr(last_hit), _ptr(out), _ptr(workspace), nbytes,
                                  _ptr(status), _opts(opts), _stream(stream))
    return _check(rc, "corm_decode_attend") if check else rc


def corm_decode_attend_static(desc, q, K, V, lens, pos, t, score_ring, last_hit, out, status=None, stream=None,
                              check=True, opts=None) -> int:
    rc = lib().corm_decode_attend_static(ctypes.byref(desc), _ptr(q), _ptr(K), _ptr(V), _ptr(lens), _ptr(pos),
                                         _ptr(t), _ptr(score_ring), _ptr(last_hit), _ptr(out), _ptr(status),
                                         _opts(opts), _stream(stream))
    return _check(rc, "corm_decode_attend_static") if check else rc


def corm_evict_mask(desc, score_ring, lens, pos, t, t_first, keep, stream=None, check=True) -> int:
    rc = lib().corm_evict_mask(ctypes.byref(desc), _ptr(score_ring), _ptr(lens), _ptr(pos), _ptr(t), _ptr(t_first),
                               _ptr(keep), _stream(stream))
    return _check(rc, "corm_evict_mask") if check else rc


def corm_evict_mask_summary(desc, last_hit, lens, t, t_first, keep, stream=None, check=True) -> int:
    rc = lib().corm_evict_mask_summary(ctypes.byref(desc), _ptr(last_hit), _ptr(lens), _ptr(t), _ptr(t_first),
                                       _ptr(keep), _stream(stream))
    return _check(rc, "corm_evict_mask_summary") if check else rc


def _nbytes(workspace, workspace_bytes):
    if workspace_bytes is not None:
        return workspace_bytes
    return 0 if workspace is None or not isinstance(workspace, torch.Tensor) else workspace.numel() * workspace.element_size()


def corm_compact(desc, K, V, pos, last_hit, lens, keep, kept_idx=None, workspace=None, workspace_bytes=None,
                 stream=None, check=True) -> int:
    rc = lib().corm_compact(ctypes.byref(desc), _ptr(K), _ptr(V), _ptr(pos), _ptr(last_hit), _ptr(lens), _ptr(keep),
                            _ptr(kept_idx), _ptr(workspace), _nbytes(workspace, workspace_bytes), _stream(stream))
    return _check(rc, "corm_compact") if check else rc


def corm_step_attend(desc, q, k_new, v_new, K, V, lens, pos, last_hit, t, t_first, score_ring, out, keep=None,
                     workspace=None, workspace_bytes=None, status=None, stream=None, check=True, opts=None) -> int:
    rc = lib().corm_step_attend(ctypes.byref(desc), _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(K), _ptr(V), _ptr(lens),
                                _ptr(pos), _ptr(last_hit), _ptr(t), _ptr(t_first), _ptr(score_ring), _ptr(out),
                                _ptr(keep), _ptr(workspace), _nbytes(workspace, workspace_bytes), _ptr(status),
                                _opts(opts), _stream(stream))
    return _check(rc, "corm_step_attend") if check else rc


def corm_step_evict(desc, K, V, lens, pos, last_hit, kept_idx=None, workspace=None, workspace_bytes=None,
                    stream=None, check=True) -> int:
    rc = lib().corm_step_evict(ctypes.byref(desc), _ptr(K), _ptr(V), _ptr(lens), _ptr(pos), _ptr(last_hit),
                               _ptr(kept_idx), _ptr(workspace), _nbytes(workspace, workspace_bytes), _stream(stream))
    return _check(rc, "corm_step_evict") if check else rc


def corm_row_density(desc, score_ring, lens, pos, t, density, stream=None, check=True) -> int:
    rc = lib().corm_row_density(ctypes.byref(desc), _ptr(score_ring), _ptr(lens), _ptr(pos), _ptr(t), _ptr(density),
                                _stream(stream))
    return _check(rc, "corm_row_density") if check else rc


def corm_selected_path(desc, opts=None, check=True) -> int:
    rc = lib().corm_selected_path(ctypes.byref(desc), _opts(opts))
    if rc < 0 and check:
        raise CormError(rc, "corm_selected_path")
    return rc


def corm_decode_step(desc, q, k_new, v_new, K, V, lens, pos, last_hit, t, t_first, score_ring, out, keep=None,
                     kept_idx=None, workspace=None, workspace_bytes=None, status=None, stream=None, check=True,
                     opts=None) -> int:
    nbytes = workspace_bytes
    if nbytes is None:
        nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    rc = lib().corm_decode_step(ctypes.byref(desc), _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(K), _ptr(V), _ptr(lens),
                                _ptr(pos), _ptr(last_hit), _ptr(t), _ptr(t_first), _ptr(score_ring), _ptr(out),
                                _ptr(keep), _ptr(kept_idx), _ptr(workspace), nbytes, _ptr(status), _opts(opts),
                                _stream(stream))
    return _check(rc, "corm_decode_step") if check else rc


def corm_decode_step_lazy(desc, q, k_new, v_new, K, V, lens, live, pos, last_hit, t, t_first, score_ring, out,
                          keep=None, nlive=None, dead_num=1, dead_den=4, workspace=None, workspace_bytes=None,
                          status=None, stream=None, check=True, opts=None) -> int:
    nbytes = workspace_bytes
    if nbytes is None:
        nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    rc = lib().corm_decode_step_lazy(ctypes.byref(desc), _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(K), _ptr(V),
                                     _ptr(lens), _ptr(live), _ptr(pos), _ptr(last_hit), _ptr(t), _ptr(t_first),
                                     _ptr(score_ring), _ptr(out), _ptr(keep), _ptr(nlive), dead_num, dead_den,
                                     _ptr(workspace), nbytes, _ptr(status), _opts(opts), _stream(stream))
    return _check(rc, "corm_decode_step_lazy") if check else rc


def corm_prefill_seed(desc, q_tail, m, K, V, lens, pos, last_hit, t, t_first, score_ring, keep=None, kept_idx=None,
                      workspace=None, workspace_bytes=None, status=None, stream=None, check=True) -> int:
    nbytes = workspace_bytes
    if nbytes is None:
        nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    rc = lib().corm_prefill_seed(ctypes.byref(desc), _ptr(q_tail), m, _ptr(K), _ptr(V), _ptr(lens), _ptr(pos),
                                 _ptr(last_hit), _ptr(t), _ptr(t_first), _ptr(score_ring), _ptr(keep), _ptr(kept_idx),
                                 _ptr(workspace), nbytes, _ptr(status), _stream(stream))
    return _check(rc, "corm_prefill_seed") if check else rc


def corm_threshold(c: float, t, n: int, thr, stream=None, check=True) -> int:
    rc = lib().corm_threshold(c, _ptr(t), n, _ptr(thr), _stream(stream))
    return _check(rc, "corm_threshold") if check else rc


# ---- device-memory plumbing for one layer (allocation only; no arithmetic of the method)

class LayerState:
    """The device arrays of one layer, allocated with torch, in the layouts corm.h documents."""

    def __init__(self, B, Hq, Hkv, d, Lcap, Tcap, w, r, dtype, thr_scale=1.0, device="cuda",
                 workspace: Optional[torch.Tensor] = None, want_masks=False, want_ring=True, score_dtype=None):
        tdt = {"f32": torch.float32, "bf16": torch.bfloat16}[dtype]
        self.desc = make_desc(B, Hq, Hkv, d, Lcap, Tcap, w, r, dtype, score_dtype=score_dtype, thr_scale=thr_scale)
        self.ring_bits = self.desc.score_dtype == CORM_BIT
        self.B, self.Hq, self.Hkv, self.d, self.Lcap, self.Tcap, self.w, self.r = B, Hq, Hkv, d, Lcap, Tcap, w, r
        self.dtype = tdt
        self.K = torch.zeros(B, Hkv, Lcap, d, dtype=tdt, device=device)
        self.V = torch.zeros(B, Hkv, Lcap, d, dtype=tdt, device=device)
        self.lens = torch.zeros(B, Hkv, dtype=torch.int32, device=device)
        self.pos = torch.zeros(B, Hkv, Lcap, dtype=torch.int32, device=device)
        self.last_hit = torch.zeros(B, Hkv, Lcap, dtype=torch.int32, device=device)
        # want_ring=False: summary-only state (score_ring == NULL in every call)
        if not want_ring:
            self.ring = None
        elif self.ring_bits:   # the boolean message: bit pos % 32 of word pos // 32
            self.ring = torch.zeros(B, Hq, w, (Tcap + 31) // 32, dtype=torch.int32, device=device)
        else:
            sdt = tdt if score_dtype is None else {"f32": torch.float32, "bf16": torch.bfloat16}[score_dtype]
            self.ring = torch.zeros(B, Hq, w, Tcap, dtype=sdt, device=device)
        self.out = torch.zeros(B, Hq, d, dtype=torch.float32, device=device)
        self.status = torch.zeros(1, dtype=torch.int32, device=device)
        self.keep = torch.zeros(B, Hkv, Lcap, dtype=torch.uint8, device=device) if want_masks else None
        self.kept_idx = torch.zeros(B, Hkv, Lcap, dtype=torch.int32, device=device) if want_masks else None
        # deferred compaction (step_lazy): live masks, all ones = every slot below lens holds a live key
        self.live = torch.full((B, Hkv, (Lcap + 63) // 64), -1, dtype=torch.int64, device=device)
        self.nlive = torch.zeros(B, Hkv, dtype=torch.int32, device=device)
        if workspace is None:
            workspace = torch.empty(corm_workspace_bytes(self.desc), dtype=torch.uint8, device=device)
            corm_workspace_init(self.desc, workspace)
        self.workspace = workspace

    def preload(self, K0: torch.Tensor, V0: torch.Tensor) -> None:
        """Copy n prompt keys/values [B,Hkv,n,d] into slots 0..n-1 (positions 0..n-1, never important yet)."""
        n = K0.shape[2]
        self.K[:, :, :n].copy_(K0)
        self.V[:, :, :n].copy_(V0)
        self.pos[:, :, :n] = torch.arange(n, dtype=torch.int32, device=self.pos.device)
        self.last_hit[:, :, :n] = 0
        self.lens.fill_(n)

    def step_attend(self, q, k_new, v_new, t, t_first, stream=None, workspace=None, opts=None) -> None:
        corm_step_attend(self.desc, q, k_new, v_new, self.K, self.V, self.lens, self.pos, self.last_hit, t, t_first,
                         self.ring, self.out, self.keep, self.workspace if workspace is None else workspace,
                         status=self.status, stream=stream, opts=opts)

    def step_evict(self, stream=None, workspace=None) -> None:
        corm_step_evict(self.desc, self.K, self.V, self.lens, self.pos, self.last_hit, self.kept_idx,
                        self.workspace if workspace is None else workspace, stream=stream)

    def step(self, q, k_new, v_new, t, t_first, stream=None, opts=None) -> None:
        corm_decode_step(self.desc, q, k_new, v_new, self.K, self.V, self.lens, self.pos, self.last_hit, t, t_first,
                         self.ring, self.out, self.keep, self.kept_idx, self.workspace, status=self.status,
                         stream=stream, opts=opts)

    def step_lazy(self, q, k_new, v_new, t, t_first, dead_num=1, dead_den=4, stream=None, workspace=None,
                  opts=None) -> None:
        corm_decode_step_lazy(self.desc, q, k_new, v_new, self.K, self.V, self.lens, self.live, self.pos,
                              self.last_hit, t, t_first, self.ring, self.out, self.keep, self.nlive, dead_num,
                              dead_den, self.workspace if workspace is None else workspace, status=self.status,
                              stream=stream, opts=opts)

    def prefill_seed(self, q_tail, t, t_first, stream=None, workspace=None) -> None:
        """q_tail [B,Hq,m,d]; the cache must already hold the whole prompt (preload)."""
        corm_prefill_seed(self.desc, q_tail, q_tail.shape[2], self.K, self.V, self.lens, self.pos, self.last_hit, t,
                          t_first, self.ring, self.keep, self.kept_idx,
                          self.workspace if workspace is None else workspace, status=self.status, stream=stream)
