"""bct_decode_step_static: the decode step whose kernel scratch is a fixed array inside the library.

The entry point exists for callers that cannot allocate device memory (graph capture, tight serving
loops).  It runs the same launches as bct_decode_step, so on equal inputs both must give the same
bits: outputs, state and step counter.  Two calls in a row share the one array on the GPU, the second
on a smaller cache; a cache that needs more scratch than the array holds is turned away.
"""
import ctypes

import numpy as np
import pytest

import bct_synth as syn
from _util import to_dev, to_np, torch_dtype

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def P():
    import torch
    assert torch.cuda.is_available()
    import paper_2411_15785_amd as pkg
    pkg.lib()
    return pkg


def _pair(P, w):
    """Two GPU caches of shape w with the same keys: one stepped through its workspace, one through the static scratch."""
    mk = to_dev(syn.make_keys(w), w.dtype)
    caches = []
    for _ in range(2):
        c = P.BctCache(w.M, w.B, w.Hq, w.Hkv, w.d, torch_dtype(w.dtype), w.scale, w.scale, flags=P.BCT_STEP_STREAMING)
        c.set_keys(mk)
        caches.append(c)
    return caches


def _raw_static_step(P, cache, q, wq, wv, out):
    """The call through the C ABI with plain pointers, as a caller without the binding would make it."""
    import torch
    vp = ctypes.c_void_p
    st = P.lib().bct_decode_step_static(cache._h, vp(q.data_ptr()) if q is not None else None,
                                        vp(wq.data_ptr()) if wq is not None else None,
                                        vp(wv.data_ptr()) if wv is not None else None,
                                        vp(out.data_ptr()) if out is not None else None,
                                        vp(torch.cuda.current_stream().cuda_stream))
    assert st == P.BCT_OK, P.bct_last_error()


def _run_and_compare(P, w, steps):
    import torch
    plain, static = _pair(P, w)
    for t in range(steps):
        q, wq, wv = (to_dev(a, w.dtype) for a in syn.make_step(w, t))
        if t == 1:      # a write-only step and a read-only step in between
            plain.decode_step(None, wq, wv)
            _raw_static_step(P, static, None, wq, wv, None)
            continue
        if t == 2:
            wq = wv = None
        o_plain = plain.decode_step(q, wq, wv)
        o_static = torch.full_like(o_plain, float("nan"))
        _raw_static_step(P, static, q, wq, wv, o_static)
        assert np.array_equal(to_np(o_plain, w.dtype), to_np(o_static, w.dtype)), f"{w.name} step {t}: outputs differ"
    assert plain.steps == static.steps == steps
    assert np.array_equal(to_np(plain.values_view(), w.dtype), to_np(static.values_view(), w.dtype)), f"{w.name}: states differ"
    assert np.array_equal(to_np(plain.keys_view(), w.dtype), to_np(static.keys_view(), w.dtype))


def test_static_scratch_step_equals_workspace_step_twice_in_a_row(P):
    import torch
    assert P.lib().bct_static_scratch_bytes() == 8 << 20
    # first call: half of config 2's batch (2.1 MiB of scratch: scores, 32 statistics tiles per row, 16 split-M
    # partial outputs per memory); second, right after it on the same GPU array, a smaller fp32 cache with
    # several query heads per KV head; third, config 2 itself (one workgroup per memory, no partials)
    big = syn.Workload("static_big", 1, 4, 32, 32, 128, 1024, "bf16", 5)
    small = syn.Workload("static_small", 1, 3, 8, 4, 64, 320, "f32", 6)
    st, plan = P.bct_plan_query(P.make_desc(big.M, big.B, big.Hq, big.Hkv, big.d, P.BCT_BF16, big.scale, big.scale))
    assert st == P.BCT_OK and plan["mv_splits"] == 16
    _run_and_compare(P, big, 5)
    _run_and_compare(P, small, 6)
    _run_and_compare(P, syn.WORKLOADS["cfg2"], 3)
    torch.cuda.synchronize()


def test_static_scratch_turns_away_a_cache_that_does_not_fit(P):
    w = syn.Workload("static_too_big", 1, 16, 32, 32, 128, 4096, "bf16", 1)
    c = P.BctCache(w.M, w.B, w.Hq, w.Hkv, w.d, torch_dtype(w.dtype), w.scale, w.scale)
    c.set_keys(to_dev(syn.make_keys(w), w.dtype))
    q, wq, wv = (to_dev(a, w.dtype) for a in syn.make_step(w, 0))
    with pytest.raises(P.BctError) as e:
        c.decode_step_static(q, wq, wv, q.clone())
    assert e.value.status == P.BCT_ERR_BUFFER_TOO_SMALL and "static scratch" in str(e.value)
    assert c.steps == 0
