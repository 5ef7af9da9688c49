"""sirllm_decay_select_static -- the entry point that allocates nothing, its scratch a static device array
inside the library -- against sirllm_decay_select with a caller-supplied workspace, through the C ABI.
Kept lists and compacted scores must agree bit for bit (both are exact integer / copy work on the same
inputs), on two calls in a row, the second smaller than the first: the second call finds the first call's
leftovers in the scratch and must clear what it needs itself."""
import ctypes as C

import numpy as np
import pytest
import torch

from helpers import to_np

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def b():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2405_12528_amd import binding
    return binding


def both_ways(b, n_streams, n_held, n_new, pol_t, levels, seed):
    """The same selection through both entry points, raw ctypes calls on raw device pointers."""
    L = b.raw()
    n_cand = n_held + n_new
    n_keep = min(n_cand, pol_t[0] + pol_t[1] + pol_t[2])
    rng = np.random.default_rng(seed)
    if levels:
        E = (rng.integers(0, levels, (n_streams, n_cand)) / 8.0).astype(np.float32)
    else:
        E = rng.gamma(2.0, 2.0, (n_streams, n_cand)).astype(np.float32)
    Ed = torch.from_numpy(E).to(DEV)
    pol = b.sirllm_policy(*pol_t)
    stream = torch.cuda.current_stream().cuda_stream
    outs = []
    for static in (False, True):
        idx = torch.full((n_streams, n_keep + 3), -7, dtype=torch.int32, device=DEV)
        out = torch.full((n_streams, n_keep + 3), -7.0, device=DEV)
        if static:
            rc = L.sirllm_decay_select_static(Ed.data_ptr(), n_cand, n_streams, n_held, n_new, C.byref(pol),
                                              idx.data_ptr(), n_keep + 3, out.data_ptr(), n_keep + 3, stream)
        else:
            nbytes = b.sirllm_workspace_bytes(n_streams, n_cand, 0, 0)
            ws = torch.zeros(max(nbytes, 256), dtype=torch.uint8, device=DEV)
            rc = L.sirllm_decay_select(Ed.data_ptr(), n_cand, n_streams, n_held, n_new, C.byref(pol),
                                       idx.data_ptr(), n_keep + 3, out.data_ptr(), n_keep + 3,
                                       ws.data_ptr() if nbytes else None, nbytes, stream)
        assert rc == b.SIRLLM_OK, b.sirllm_status_string(rc)
        torch.cuda.synchronize()
        outs.append((to_np(idx), to_np(out)))
    (i0, o0), (i1, o1) = outs
    np.testing.assert_array_equal(i1, i0)
    np.testing.assert_array_equal(o1.view(np.uint32), o0.view(np.uint32))
    assert (i1[:, n_keep:] == -7).all() and (i1[:, :n_keep] >= 0).all()
    return E, i1[:, :n_keep], o1[:, :n_keep]


def test_static_scratch_matches_workspace_on_two_calls_in_a_row(b, ref):
    # first call: 3 streams x 200000 slots (25 tiles per stream in the scratch), heavy ties
    E, gi, go = both_ways(b, 3, 190000, 10000, (4, 120000, 4096, 0.9), 40, seed=1)
    ri, ro = ref.decay_select(E, 190000, 10000, ref.Policy(4, 120000, 4096, 0.9))
    np.testing.assert_array_equal(gi, ri)
    np.testing.assert_array_equal(go.view(np.uint32), ro.view(np.uint32))
    # second call, smaller in every way (2 streams x 40000 slots): finds the first call's histograms in the array
    E, gi, go = both_ways(b, 2, 39000, 1000, (4, 20000, 512, 0.85), 0, seed=2)
    ri, ro = ref.decay_select(E, 39000, 1000, ref.Policy(4, 20000, 512, 0.85))
    np.testing.assert_array_equal(gi, ri)
    np.testing.assert_array_equal(go.view(np.uint32), ro.view(np.uint32))
    # and once more at the first size: nothing of the smaller call is in the way
    both_ways(b, 3, 190000, 10000, (4, 120000, 4096, 0.9), 40, seed=3)


def test_static_entry_point_below_the_scratch_sizes(b):
    # up to 32768 slots per stream one workgroup selects and the scratch is not touched; under budget: keep all
    both_ways(b, 2, 7168, 1024, (4, 3068, 1024, 0.85), 0, seed=4)
    both_ways(b, 1, 30000, 2768, (4, 16000, 68, 0.9), 100, seed=5)
    both_ways(b, 2, 40000, 100, (4, 50000, 512, 0.9), 0, seed=6)


def test_static_entry_point_rejects_what_does_not_fit(b):
    # 300 streams x 40000 slots need 300 x 4352 bytes of scratch, more than the array holds: refused on the host,
    # nothing launched, outputs untouched; the workspace entry point takes the same sizes
    n_streams, n_held, n_new = 300, 39000, 1000
    n_cand, n_keep = n_held + n_new, 4 + 20000 + 512
    assert b.sirllm_workspace_bytes(n_streams, n_cand, 0, 0) > b.SIRLLM_STATIC_SCRATCH_BYTES
    E = torch.rand((n_streams, n_cand), device=DEV)
    idx = torch.full((n_streams, n_keep), -7, dtype=torch.int32, device=DEV)
    out = torch.full((n_streams, n_keep), -7.0, device=DEV)
    pol = b.sirllm_policy(4, 20000, 512, 0.9)
    rc = b.raw().sirllm_decay_select_static(E.data_ptr(), n_cand, n_streams, n_held, n_new, C.byref(pol), idx.data_ptr(),
                                            n_keep, out.data_ptr(), n_keep, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    assert rc == b.SIRLLM_ERR_UNSUPPORTED
    assert bool((idx == -7).all()) and bool((out == -7.0).all())
    with pytest.raises(b.SirllmError):
        b.sirllm_decay_select_static(E, n_held, n_new, b.Policy(4, 20000, 512, 0.9), idx, out)
    # 240 streams of 133120 slots are the most that fit
    assert b.sirllm_workspace_bytes(240, 133120, 0, 0) <= b.SIRLLM_STATIC_SCRATCH_BYTES
    assert b.sirllm_workspace_bytes(241, 133120, 0, 0) > b.SIRLLM_STATIC_SCRATCH_BYTES
