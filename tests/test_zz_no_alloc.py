"""corm_decode_attend_static (the attend call that allocates nothing: its split partials and logits live in a
device array inside the library) against corm_decode_attend with a caller's workspace, through the C ABI:
out, the recorded ring row and last_hit must be identical, on two calls in a row, the second with a smaller
input (the array keeps the first call's contents); a shape beyond the array is refused on the host."""
import sys

import pytest
import torch

from paper_2404_15949_amd import corm, inputs
from tests import harness

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _attend_both_ways(wl, n_keys, t_step, seed):
    """Fills a cache with n_keys prompt keys of the seeded generator and runs one attend + record at step
    t_step, once per entry point, from identical copies of the state.  Returns the two states."""
    print("[case] no-alloc attend", wl.name, "B", wl.B, "Hq/Hkv", wl.Hq, wl.Hkv, "d", wl.d, "keys", n_keys,
          "t", t_step, flush=True)
    sys.stdout.flush()
    x = inputs.make_layer(wl.replace(seed=seed), 0, device=DEV, n_decode=1, n_replay=1)
    states = []
    for which in ("workspace", "static"):
        st = harness.make_state(wl, DEV, Lcap=wl.P + 8, Tcap=wl.P + 8, want_masks=False)
        st.preload(x["K0"][:, :, :n_keys], x["V0"][:, :, :n_keys])
        st.ring.fill_(-1.0)
        st.out.fill_(float("nan"))
        t = torch.full((wl.B,), t_step, dtype=torch.int32, device=DEV)
        q = x["Q"][0].contiguous()
        if which == "workspace":
            assert corm.corm_selected_path(st.desc) == 1            # the path whose kernels use scratch memory
            corm.corm_decode_attend(st.desc, q, st.K, st.V, st.lens, st.pos, t, st.ring, st.last_hit, st.out,
                                    st.workspace, status=st.status)
        else:
            corm.corm_decode_attend_static(st.desc, q, st.K, st.V, st.lens, st.pos, t, st.ring, st.last_hit, st.out,
                                           status=st.status)
        torch.cuda.synchronize()
        assert int(st.status.item()) == 0
        states.append(st)
    return states


def _same(a, b, n_keys):
    assert torch.isfinite(a.out).all() and torch.equal(a.out, b.out), "out"
    assert torch.equal(a.ring, b.ring), "ring row"
    assert torch.equal(a.last_hit, b.last_hit), "last_hit"
    assert int((a.last_hit[:, :, :n_keys] > 0).sum().item()) > 0, "no key was found important: vacuous"
    assert torch.equal(a.lens, b.lens) and torch.equal(a.K, b.K) and torch.equal(a.V, b.V)


def test_static_scratch_attend_equals_workspace_attend_twice():
    big = inputs.WORKLOADS["gqa_llama3"].replace(name="no_alloc_big", B=3, Hq=16, Hkv=4, P=2300, D=1, w=8, r=8)
    a, b = _attend_both_ways(big, 2219, 2219, seed=5)        # several 512-key chunks and a ragged tail
    _same(a, b, 2219)
    small = inputs.WORKLOADS["tiny_f32"].replace(name="no_alloc_small", B=1, Hq=4, Hkv=4, d=64, P=700, D=1, w=8, r=8)
    a, b = _attend_both_ways(small, 601, 640, seed=6)       # smaller, another dtype and head size
    _same(a, b, 601)
    a, b = _attend_both_ways(big, 1000, 1000, seed=7)        # and the larger shape once more
    _same(a, b, 1000)


def test_static_scratch_refuses_shapes_beyond_the_array():
    d = corm.make_desc(4, 32, 32, 128, 66000, 66000, 8, 8, "bf16")
    need = 4 * 32 * 66000 * 4 + 4 * 32 * ((66000 + 511) // 512) * 4 * (128 + 2) * 4      # logits + partials
    assert need > corm.CORM_STATIC_SCRATCH_BYTES
    z = torch.zeros(64, dtype=torch.int32, device=DEV)
    rc = corm.corm_decode_attend_static(d, z, z, z, z, z, z, z, z, z, check=False)
    assert rc == corm.CORM_ECAPACITY
