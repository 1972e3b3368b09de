"""CPU-only checks of the C ABI: the library loads, exports every symbol the header declares,
and rejects bad arguments on the host before anything is launched."""
import ctypes
import os
import re

import pytest

from paper_2404_15949_amd import corm

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "corm.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(corm_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = _declared()
    assert set(names) == set(corm.EXPORTS), (names, corm.EXPORTS)
    raw = ctypes.CDLL(corm.LIB_PATH)
    for n in names:
        assert hasattr(raw, n), n
    assert corm.corm_version() >= 100
    assert "invalid" in corm.strerror(corm.CORM_EINVAL)


def _desc(**kw):
    base = dict(B=2, Hq=8, Hkv=2, d=128, Lcap=1024, Tcap=1024, w=16, r=16, kv_dtype="bf16")
    base.update(kw)
    return corm.make_desc(**base)


def test_desc_layout_matches_header():
    assert ctypes.sizeof(corm.corm_desc) == 12 * 4
    assert [f[0] for f in corm.corm_desc._fields_] == ["B", "Hq", "Hkv", "d", "Lcap", "Tcap", "w", "r", "kv_dtype",
                                                       "score_dtype", "thr_scale", "sm_scale"]


def test_workspace_size_formula():
    d = _desc()
    n = corm.corm_workspace_bytes(d)
    nsplit = (1024 + 511) // 512
    units, heads = 2 * 2, 2 * 8
    stage_rows = units * nsplit * 512
    need = (units * nsplit * 4 + units * 4 + units * (1024 // 64) * 8 + heads * nsplit * 4 * 130 * 4 + heads * 1024 * 4
            + stage_rows * (8 + 2 * 256)
            + heads * (1024 // 256) * 16 * 8 + heads * 16 * 16)     # prompt seeding: partial and merged row statistics
    assert need <= n <= need + 10 * 256


@pytest.mark.parametrize("kw,code", [
    (dict(d=96), corm.CORM_EUNSUPPORTED),
    (dict(Hq=6, Hkv=2), corm.CORM_EUNSUPPORTED),      # group of 3
    (dict(Hq=8, Hkv=3), corm.CORM_EINVAL),            # not divisible
    (dict(w=0), corm.CORM_EINVAL),
    (dict(r=0), corm.CORM_EINVAL),
    (dict(thr_scale=-1.0), corm.CORM_EINVAL),
    (dict(thr_scale=float("nan")), corm.CORM_EINVAL),
    (dict(Lcap=0), corm.CORM_EINVAL),
    (dict(B=0), corm.CORM_EINVAL),
    (dict(kv_dtype=7), corm.CORM_EUNSUPPORTED),
])
def test_bad_descriptors_are_rejected(kw, code):
    kv = kw.pop("kv_dtype", "bf16")
    d = _desc(**kw)
    if kv == 7:
        d.kv_dtype = 7
    assert corm.corm_workspace_bytes(d, check=False) == code


def test_null_and_misaligned_pointers_are_rejected_on_the_host():
    d = _desc()
    a = 4096  # a plausible aligned address; never dereferenced because validation fails first
    args = dict(q=a, k_new=a, v_new=a, K=a, V=a, lens=a, pos=a, last_hit=a, t=a, t_first=a, score_ring=a, out=a)
    order = ["q", "k_new", "v_new", "K", "V", "lens", "pos", "last_hit", "t", "t_first", "score_ring", "out"]
    for missing in order:
        if missing == "score_ring":
            continue   # a null ring is legal (summary-only state): that call would pass validation and launch
        v = dict(args); v[missing] = None
        rc = corm.corm_decode_step(d, *[v[k] for k in order], workspace=a, workspace_bytes=1 << 30, check=False)
        assert rc == corm.CORM_EINVAL, missing
    v = dict(args); v["K"] = a + 8
    rc = corm.corm_decode_step(d, *[v[k] for k in order], workspace=a, workspace_bytes=1 << 30, check=False)
    assert rc == corm.CORM_EINVAL
    # workspace too small / missing
    rc = corm.corm_decode_step(d, *[args[k] for k in order], workspace=a, workspace_bytes=16, check=False)
    assert rc == corm.CORM_ECAPACITY
    rc = corm.corm_decode_step(d, *[args[k] for k in order], workspace=None, workspace_bytes=0, check=False)
    assert rc == corm.CORM_EINVAL
    assert corm.corm_compact(d, None, a, a, a, a, a, workspace=a, workspace_bytes=1 << 30, check=False) == corm.CORM_EINVAL
    assert corm.corm_compact(d, a, a, a, a, a, a, workspace=a, workspace_bytes=8, check=False) == corm.CORM_ECAPACITY
    assert corm.corm_step_attend(d, a, a, a, a, a, a, a, a, None, a, a, a, workspace=a, workspace_bytes=1 << 30,
                                 check=False) == corm.CORM_EINVAL
    assert corm.corm_step_evict(d, a, a, None, a, a, workspace=a, workspace_bytes=1 << 30, check=False) == corm.CORM_EINVAL
    # launch options: a path outside 0..3, or one event without the other
    bad = corm.corm_launch_opts(4, 0, None, None)
    assert corm.corm_decode_step(d, *[args[k] for k in order], workspace=a, workspace_bytes=1 << 30, check=False,
                                 opts=bad) == corm.CORM_EINVAL
    one = corm.corm_launch_opts(0, 0, a, None)
    assert corm.corm_decode_step(d, *[args[k] for k in order], workspace=a, workspace_bytes=1 << 30, check=False,
                                 opts=one) == corm.CORM_EINVAL
    assert corm.corm_selected_path(d, bad, check=False) == corm.CORM_EINVAL
    assert corm.corm_evict_mask(d, a, a, a, a, None, a, check=False) == corm.CORM_EINVAL
    assert corm.corm_append(d, a, a, a, a, a, a + 4, a, a, check=False) == corm.CORM_EINVAL
    assert corm.corm_threshold(-1.0, a, 4, a, check=False) == corm.CORM_EINVAL


def test_two_threads_with_different_options_do_not_see_each_other():
    """What a call does depends on its arguments alone: two host threads that ask, in a tight loop, for
    different launch paths, different shapes' workspace sizes and different argument errors each get their
    own answers every time (ctypes releases the interpreter lock during a call, so the calls do overlap)."""
    import threading
    small, large = _desc(), _desc(B=64, Hq=32, Hkv=32, Lcap=4096, Tcap=4096)
    n_small, n_large = corm.corm_workspace_bytes(small), corm.corm_workspace_bytes(large)
    assert n_small != n_large
    a = 4096
    failures = []

    def worker(path, desc, want_bytes, bad_opts):
        opts = corm.corm_launch_opts(path, 0, None, None)
        for _ in range(3000):
            got = corm.corm_selected_path(desc, opts)
            if got != path:
                failures.append(("path", path, got))
            if corm.corm_workspace_bytes(desc) != want_bytes:
                failures.append(("bytes", path))
            rc = corm.corm_decode_attend(desc, a, a, a, a, a, a, a, a, a, a, workspace_bytes=1 << 40, check=False,
                                         opts=bad_opts)
            if rc != corm.CORM_EINVAL:
                failures.append(("opts", path, rc))

    th = [threading.Thread(target=worker, args=(1, small, n_small, corm.corm_launch_opts(7, 0, None, None))),
          threading.Thread(target=worker, args=(2, large, n_large, corm.corm_launch_opts(2, 0, None, a)))]
    for t in th:
        t.start()
    for t in th:
        t.join()
    assert not failures, failures[:5]
    # by shape (path 0), with no device to ask: 256 compute units are assumed
    assert corm.corm_selected_path(small) == 1 and corm.corm_selected_path(large) == 2


def test_static_scratch_entry_checks_its_arguments_and_its_limit_on_the_host():
    """corm_decode_attend_static: bad pointers and shapes beyond the library's device array are refused
    before any device call (so this runs without a GPU)."""
    a = 4096
    ok = _desc()
    assert corm.corm_decode_attend_static(ok, a, a, a, a, a, a, a, None, a, check=False) == corm.CORM_EINVAL
    assert corm.corm_decode_attend_static(ok, a + 4, a, a, a, a, a, a, a, a, check=False) == corm.CORM_EINVAL
    assert corm.corm_decode_attend_static(_desc(d=96), a, a, a, a, a, a, a, a, a, check=False) == corm.CORM_EUNSUPPORTED
    # logits alone: B*Hq*Lcap*4 bytes
    big = _desc(B=16, Hq=32, Hkv=32, Lcap=32768, Tcap=32768)
    assert 16 * 32 * 32768 * 4 > corm.CORM_STATIC_SCRATCH_BYTES
    assert corm.corm_decode_attend_static(big, a, a, a, a, a, a, a, a, a, check=False) == corm.CORM_ECAPACITY
    text = open(os.path.join(ROOT, "include", "corm.h")).read()
    assert re.search(r"#define\s+CORM_STATIC_SCRATCH_BYTES\s+\(40u << 20\)", text)
    assert corm.CORM_STATIC_SCRATCH_BYTES == 40 << 20


def test_host_code_under_address_and_undefined_behaviour_sanitizers():
    """tests/host_checks: the library's host code (descriptor validation, workspace layout, pointer and option
    checks, path selection, the static-scratch limit) compiled with ASan + UBSan and driven at and beyond the
    interface limits (4194303 slots, 65520 units, products beyond 32 bits), from two threads; any report from
    a sanitizer ends the program with a non-zero status.  Built by build(); built here if it is missing."""
    import subprocess
    import sys
    exe = os.path.join(ROOT, "tests", "host_checks", "host_checks")
    if not os.path.exists(exe):
        sys.path.insert(0, ROOT)
        import __graft_entry__
        __graft_entry__.build_host_checks()
    r = subprocess.run([exe], capture_output=True, text=True, timeout=300,
                       env={**os.environ, "ASAN_OPTIONS": "detect_leaks=0:abort_on_error=0",
                            "UBSAN_OPTIONS": "print_stacktrace=1:halt_on_error=1"})
    assert r.returncode == 0 and "host checks ok" in r.stdout, (r.returncode, r.stdout[-600:], r.stderr[-1200:])
    assert "Sanitizer" not in r.stderr and "runtime error" not in r.stderr, r.stderr[-1200:]
    syms = subprocess.run(["nm", exe], capture_output=True, text=True).stdout
    assert "__asan_init" in syms and "__ubsan_handle" in syms, "the program is not instrumented"


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(corm, "_lib", None)
    monkeypatch.setattr(corm, "LIB_PATH", "/nonexistent/libcorm.so")
    with pytest.raises(RuntimeError, match="no fallback"):
        corm.lib()


def test_bench_refuses_more_than_one_gpu():
    """The benchmark measures one GPU: `--gpus 2` (or a multi-rank launch) ends with a message, before
    anything touches a device."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    for argv, env in ((["--gpus", "2"], {}), ([], {"WORLD_SIZE": "2"})):
        r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), *argv], capture_output=True, text=True,
                           env={**os.environ, **env}, timeout=120)
        assert r.returncode == 2, (argv, env, r.returncode, r.stderr[-300:])
        assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_product_code_never_touches_the_oracle():
    """The oracle is test infrastructure: nothing in the package imports it, and bench.py only inside its
    cpu_baseline leg."""
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    pkg = os.path.join(root, "paper_2404_15949_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith(".py"):
                for ln in open(os.path.join(dirpath, f)):
                    assert not re.match(r"\s*(from|import)\s+.*\boracle\b", ln), (os.path.join(dirpath, f), ln)
            elif f.endswith((".hip", ".hpp", ".h")):
                assert "oracle" not in open(os.path.join(dirpath, f)).read().lower(), os.path.join(dirpath, f)
    bench = open(os.path.join(root, "bench.py")).read()
    uses = [ln for ln in bench.splitlines() if "import" in ln and "oracle" in ln]
    assert uses, "bench.py times the oracle as its CPU baseline"
    body = bench[bench.index("def cpu_baseline_leg"):]
    nxt = re.search(r"^(def |class |if __name__)", body[1:], flags=re.M)     # the next top-level statement
    body = body[:nxt.start() + 1] if nxt else body
    assert all(ln.strip() in body for ln in uses), "the oracle is imported outside the cpu_baseline leg"
