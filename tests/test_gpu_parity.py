"""GPU parity: libbct (through its C ABI) against the CPU oracle, element by
element on the same seeded inputs.  Tolerances: fp32 out <= 1e-5 (max over
vectors of max|diff| / max|ref|); bf16 out <= 2e-2 absolute; stored bf16 state
within 1 ulp of the oracle's after one step from a common state; MK, step
counters, sizes and hard-addressed slots bit-exact.
"""
import math

import numpy as np
import pytest

import bct_synth as syn
from _util import bf16_ulp, f64, make_pair, rel_normwise, sub, to_dev, to_np, torch_dtype

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def P():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_2411_15785_amd as pkg
    pkg.lib()  # fails loudly if libbct.so is missing
    return pkg


@pytest.fixture(scope="module")
def R():
    from oracle import bct_ref
    return bct_ref


def check_out(got, ref, dtype, what=""):
    g, r = f64(got, dtype), f64(ref, dtype)
    assert np.all(np.isfinite(g)), what
    if dtype == "f32":
        e = rel_normwise(g, r)
        assert e <= 1e-5, f"{what}: fp32 out rel err {e:.3e}"
    else:
        e = float(np.max(np.abs(g - r)))
        assert e <= 2e-2, f"{what}: bf16 out abs err {e:.3e}"
        # far tighter in practice: within two bf16 ulps of the vector's largest entry
        tight = np.max(np.abs(g - r), axis=-1) / bf16_ulp(np.max(np.abs(r), axis=-1))
        assert np.max(tight) <= 2.0, f"{what}: bf16 out {np.max(tight):.2f} ulp of the vector max"
    return e


def check_state_one_step(got, ref, dtype, what="", before=None, rel=4e-6):
    """State after ONE step from a common state: the two sides differ only where the
    fp32 write weight differs in its last bits (~1e-6 relative), i.e. rare flips of one
    rounding.  Where the increment nearly cancels the old value the result is tiny and
    the weight error, which scales with the increment (at most |new| + |old|), is no
    longer small against ITS ulp: `before` (the common old state) adds that allowance."""
    g, r = f64(got, dtype), f64(ref, dtype)
    if dtype == "f32":
        e = float(np.max(np.abs(g - r)) / max(np.max(np.abs(r)), 1e-30))
        assert e <= 1e-5, f"{what}: fp32 state rel err {e:.3e}"
        return
    d = np.abs(g - r)
    ulp = bf16_ulp(r)
    allow = ulp * 1.0001
    if before is not None:
        allow = allow + rel * (np.abs(r) + np.abs(f64(before, dtype)))
    assert np.all(d <= allow), f"{what}: bf16 state off by {np.max(d / allow):.2f} x the allowance"
    frac = float(np.mean(d > 0))
    assert frac <= 5e-3, f"{what}: {frac:.2e} of the state elements differ"


def step_np(w, t, layer=0):
    return syn.make_step(w, t, layer)


def run_lockstep(w, ref, gpu, bs, steps, t0=0, every_state=0, what=""):
    worst = 0.0
    for t in range(t0, t0 + steps):
        q, wq, wv = step_np(w, t)
        o_ref = ref.decode_step(sub(q, bs), sub(wq, bs), sub(wv, bs))
        o_gpu = gpu.decode_step(to_dev(q, w.dtype), to_dev(wq, w.dtype), to_dev(wv, w.dtype))
        worst = max(worst, check_out(to_np(o_gpu, w.dtype)[bs], o_ref, w.dtype, f"{what} step {t}"))
    return worst


# ------------------------------------------------------------------ config 1 (fp32, whole run)

def test_cfg1_fp32_all_256_steps(P, R):
    w = syn.WORKLOADS["cfg1"]
    ref, gpu, mk, _, bs = make_pair(w, R.RefCache, P.BctCache)
    assert gpu.cache_bytes >= ref.cache_bytes()
    run_lockstep(w, ref, gpu, bs, w.decode_steps, what="cfg1")
    mk_g, mv_g, st = gpu.export()
    assert st == w.decode_steps == ref.steps
    assert np.array_equal(to_np(mk_g, w.dtype), mk)          # MK bit-exact, never written
    mv_r = ref.values()
    e = np.max(np.abs(to_np(mv_g, w.dtype).astype(np.float64) - mv_r)) / np.max(np.abs(mv_r))
    assert e <= 1e-5, f"cfg1 state rel err {e:.3e}"


# ------------------------------------------------------------------ single step from a common state, all variants

SMALL = [
    # name, B, Hq, Hkv, d, M, dtype
    ("f32_d64", 2, 4, 4, 64, 128, "f32"),
    ("f32_d128_gqa2", 2, 4, 2, 128, 192, "f32"),
    ("bf16_d128", 3, 4, 4, 128, 256, "bf16"),
    ("bf16_d128_gqa4", 2, 8, 2, 128, 320, "bf16"),
    ("bf16_d64_gqa8", 1, 8, 1, 64, 128, "bf16"),
    ("bf16_d128_gqa3", 2, 6, 2, 128, 64, "bf16"),
    ("f32_d64_gqa5", 1, 5, 1, 64, 64, "f32"),
    ("bf16_d128_m2112", 2, 2, 2, 128, 2112, "bf16"),   # 33 chunks of 64: ragged split of the MV pass
    ("bf16_m65536", 1, 1, 1, 128, 65536, "bf16"),       # the largest capacity the library accepts
    ("f32_d128_m65536", 1, 1, 1, 128, 65536, "f32"),
    ("bf16_gqa8_m4160", 1, 8, 1, 128, 4160, "bf16"),    # 8 query heads per KV head, 65 chunks of 64
    ("bf16_gqa2_m8128", 1, 4, 2, 128, 8128, "bf16"),    # 127 chunks of 64: the MV pass merges two (max, sum) pairs per lane
    # 192 memories or more of 32 KB to 256 KB, one query head per KV head: one workgroup of the MV pass per memory
    ("bf16_whole_m512", 8, 32, 32, 128, 512, "bf16"),         # 128 KB per memory: 512 threads
    ("f32_d64_whole_m320", 6, 32, 32, 64, 320, "f32"),        # 80 KB: 512 threads, 192 of their 512 slots idle
    ("bf16_d64_whole_m2048", 8, 32, 32, 64, 2048, "bf16"),    # 256 KB: 1024 threads, the largest
    ("f32_d128_whole_m128", 7, 28, 28, 128, 128, "f32"),      # 64 KB: 256 threads; 196 memories
    ("bf16_m1024_units128", 4, 32, 32, 128, 1024, "bf16"),    # too few memories: 16 KB workgroups, 16 partials
    # Caches of at most 128 slots and 512 memories take the one-launch step, all others the four-launch
    # step (flags = 2 forces the latter): these are cases on both sides of the two limits
    ("f32_d64_units640", 40, 16, 16, 64, 128, "f32"),
    ("bf16_d128_gqa2_units576", 36, 32, 16, 128, 192, "bf16"),
    ("bf16_d64_units1024", 64, 16, 16, 64, 64, "bf16"),
    ("f32_d128_gqa4_units520", 130, 16, 4, 128, 64, "f32"),
    ("bf16_units4096", 512, 8, 8, 64, 64, "bf16"),            # many small memories
    ("bf16_gqa4_units2048", 256, 32, 8, 128, 64, "bf16"),     # the MFMA read with a single 64-slot tile per memory
    ("bf16_m128_units512", 16, 32, 32, 128, 128, "bf16"),     # the largest cache of the one-launch step
    ("f32_gqa8_m128", 1, 8, 1, 128, 128, "f32"),
    ("bf16_gqa4_m128_d64", 3, 8, 2, 64, 128, "bf16"),
]


# flags: 0 shared keys, 1 per-sequence keys, 2 always the four-launch step (a different path only for
# caches small enough for the one-launch step)
SMALL_FLAGS = [c + (f,) for c in SMALL for f in (0, 1, 2) if f < 2 or (c[5] <= 128 and c[1] * c[3] <= 512)]


@pytest.mark.parametrize("name,B,Hq,Hkv,d,M,dtype,flags", SMALL_FLAGS)
@pytest.mark.parametrize("mode", ["rw", "write_only", "read_only"])
def test_one_step_from_common_state(P, R, name, B, Hq, Hkv, d, M, dtype, mode, flags):
    w = syn.Workload(name, 1, B, Hq, Hkv, d, M, dtype, 4)
    ref, gpu, mk, mv0, bs = make_pair(w, R.RefCache, P.BctCache, flags=flags, mv0=True)
    for t in range(3):
        q, wq, wv = step_np(w, t)
        if mode == "write_only":
            q = None
        if mode == "read_only":
            wq = wv = None
        # resynchronise: both sides start the step from the oracle's state
        before = ref.values()
        gpu.set_values(to_dev(before, dtype))
        o_ref = ref.decode_step(q, wq, wv)
        o_gpu = gpu.decode_step(to_dev(q, dtype), to_dev(wq, dtype), to_dev(wv, dtype))
        if mode != "write_only":
            check_out(to_np(o_gpu, dtype), o_ref, dtype, f"{name}/{mode} step {t}")
        else:
            assert o_gpu is None and o_ref is None
        mk_g, mv_g, st = gpu.export()
        assert np.array_equal(to_np(mk_g, dtype), mk)
        if mode == "read_only":
            assert np.array_equal(to_np(mv_g, dtype), ref.values())   # untouched, bit for bit
        else:
            check_state_one_step(to_np(mv_g, dtype), ref.values(), dtype, f"{name}/{mode} step {t}", before=before)
        assert st == t + 1


@pytest.mark.parametrize("dtype,G", [("bf16", 1), ("f32", 2)])
def test_more_memories_than_one_grid_dimension_holds(P, R, dtype, G):
    """66000 memories (batch 1100 x 60 KV heads): launches indexed by memory spill from grid.y into grid.z.
    Two decode steps from MV_0 = 0 and a chunk of three tokens, every memory compared."""
    from test_gpu_prefill import check_prefill_out
    w = syn.Workload("many_units", 1, 1100, 60 * G, 60, 64, 64, dtype, 0)
    ref, gpu, mk, _, _ = make_pair(w, R.RefCache, P.BctCache, max_prefill_T=3)
    for t in range(2):
        q, wq, wv = step_np(w, t)
        before = ref.values()
        gpu.set_values(to_dev(before, dtype))
        o_ref = ref.decode_step(q, wq, wv)
        o_gpu = gpu.decode_step(to_dev(q, dtype), to_dev(wq, dtype), to_dev(wv, dtype))
        check_out(to_np(o_gpu, dtype), o_ref, dtype, f"many units step {t}")
        check_state_one_step(to_np(gpu.export()[1], dtype), ref.values(), dtype, f"many units step {t}", before=before)
    q, wq, wv = syn.make_step(w, 2, T=3)
    before = ref.values()
    gpu.set_values(to_dev(before, dtype))
    o_ref = ref.prefill(q, wq, wv, 3)
    o_gpu = gpu.prefill(to_dev(q, dtype), to_dev(wq, dtype), to_dev(wv, dtype), 3)
    check_prefill_out(to_np(o_gpu, dtype), o_ref, dtype, "many units chunk")
    g, r = f64(to_np(gpu.export()[1], dtype), dtype), f64(ref.values(), dtype)
    assert np.max(np.abs(g - r)) <= (1e-5 if dtype == "f32" else 2.0 ** -7) * np.max(np.abs(r))
    assert gpu.steps == 5 and np.array_equal(to_np(gpu.keys_view(), dtype), mk)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_write_scale_one_is_algorithm_1_as_printed(P, R, dtype):
    w = syn.Workload("ws1", 1, 2, 2, 2, 64, 128, dtype, 4)
    ref, gpu, _, _, bs = make_pair(w, R.RefCache, P.BctCache, write_scale=1.0, read_scale=0.2)
    for t in range(3):
        q, wq, wv = step_np(w, t)
        gpu.set_values(to_dev(ref.values(), dtype))
        o_ref = ref.decode_step(q, wq, wv)
        o_gpu = gpu.decode_step(to_dev(q, dtype), to_dev(wq, dtype), to_dev(wv, dtype))
        check_out(to_np(o_gpu, dtype), o_ref, dtype, f"ws1 step {t}")
        check_state_one_step(to_np(gpu.export()[1], dtype), ref.values(), dtype, f"ws1 step {t}")


# ------------------------------------------------------------------ hard addressing: slots and indexing bit-exact

@pytest.mark.parametrize("dtype,d", [("f32", 64), ("bf16", 128)])
def test_hard_addressing_writes_exactly_one_slot(P, R, dtype, d):
    M, B, Hq, Hkv = 64, 2, 4, 2
    w = syn.Workload("hard", 1, B, Hq, Hkv, d, M, dtype, M)
    ref, gpu, mk, _, bs = make_pair(w, R.RefCache, P.BctCache, write_scale=1.0)
    K = f64(mk, dtype)
    order = np.random.default_rng(3).permutation(M)
    for t in range(M):
        wq64 = np.empty((B, Hkv, d))
        for h in range(Hkv):
            s = K[h] @ K[h, order[t]]
            gap = s[order[t]] - np.max(np.delete(s, order[t]))
            assert gap > 1.0
            wq64[:, h] = K[h, order[t]] * (300.0 / gap)
        wq = syn.pack(wq64, dtype)
        for h in range(Hkv):   # still separated by > 200 after rounding the query
            s = K[h] @ f64(wq[0, h], dtype)
            assert s[order[t]] - np.max(np.delete(s, order[t])) > 200.0
        q, _, wv = step_np(w, t)
        before = to_np(gpu.export()[1], dtype)
        o_gpu = gpu.decode_step(to_dev(q, dtype), to_dev(wq, dtype), to_dev(wv, dtype))
        o_ref = ref.decode_step(q, wq, wv)
        after = to_np(gpu.export()[1], dtype)
        others = np.delete(np.arange(M), order[t])
        assert np.array_equal(after[:, :, order[t], :], wv)                   # the slot holds wv_t bit for bit
        assert np.array_equal(after[:, :, others, :], before[:, :, others, :])  # nothing else moved
        assert np.array_equal(after, ref.values())                            # whole state bit-exact
        check_out(to_np(o_gpu, dtype), o_ref, dtype, f"hard step {t}")


# ------------------------------------------------------------------ determinism, checkpoint, capacity

def test_determinism_and_checkpoint_roundtrip(P, R):
    import torch
    w = syn.Workload("det", 1, 4, 8, 4, 128, 1024, "bf16", 8)
    outs, states = [], []
    for rep in range(2):
        _, gpu, _, _, _ = make_pair(w, R.RefCache, P.BctCache, mv0=True)
        o = []
        for t in range(6):
            q, wq, wv = step_np(w, t)
            o.append(to_np(gpu.decode_step(to_dev(q, w.dtype), to_dev(wq, w.dtype), to_dev(wv, w.dtype)), w.dtype))
            if rep == 1 and t == 2:   # checkpoint after step 3, restore into a fresh cache, continue there
                mk_c, mv_c, st_c = gpu.export()
                gpu2 = P.BctCache(w.M, w.B, w.Hq, w.Hkv, w.d, torch_dtype(w.dtype), w.scale, w.scale)
                gpu2.import_(mk_c, mv_c, st_c)
                gpu = gpu2
        outs.append(np.stack(o))
        states.append(to_np(gpu.export()[1], w.dtype))
        assert gpu.steps == 6
    assert np.array_equal(outs[0], outs[1])
    assert np.array_equal(states[0], states[1])


def test_capacity_is_constant_and_errors_are_reported(P, R):
    import ctypes
    import torch
    w = syn.Workload("cap", 1, 2, 2, 2, 64, 64, "f32", 8)
    gpu = P.BctCache(w.M, w.B, w.Hq, w.Hkv, w.d, torch.float32)
    L = P.lib()
    q, wq, wv = (to_dev(a, "f32") for a in step_np(w, 0))
    out = torch.empty_like(q)
    s = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    p = lambda t: ctypes.c_void_p(t.data_ptr())
    assert L.bct_decode_step(gpu._h, p(q), p(wq), p(wv), p(out), s) == P.BCT_ERR_STATE   # keys not set
    gpu.set_keys(to_dev(syn.make_keys(w), "f32"))
    assert L.bct_decode_step(gpu._h, p(q), p(wq), None, p(out), s) == P.BCT_ERR_INVALID_ARG
    assert L.bct_decode_step(gpu._h, p(q), None, None, None, s) == P.BCT_ERR_INVALID_ARG
    assert L.bct_decode_step(gpu._h, None, None, None, None, s) == P.BCT_ERR_INVALID_ARG
    assert L.bct_decode_step(None, p(q), p(wq), p(wv), p(out), s) == P.BCT_ERR_INVALID_ARG
    mis = ctypes.c_void_p(q.data_ptr() + 4)
    assert L.bct_decode_step(gpu._h, mis, p(wq), p(wv), p(out), s) == P.BCT_ERR_MISALIGNED
    assert gpu.steps == 0                                   # failed calls do not count
    free0 = torch.cuda.memory_allocated()
    for t in range(3 * w.M):                                # far past the capacity
        gpu.decode_step(q, wq, wv, out)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == free0           # no growth, no allocation in the step
    assert gpu.steps == 3 * w.M
    assert torch.isfinite(out).all()


# ------------------------------------------------------------------ extreme inputs

def score_tolerance(q, wq, mk, w, base):
    """Output tolerance when scores are large.  A scaled score s (natural units) comes from an fp32 sum of
    d exact products and carries a rounding error of about |s| 2^-24 (one rounding of the result; the
    errors of the partial sums mostly cancel); the softmax weight exp(s - max) inherits it as a RELATIVE
    error, numerator and normaliser both, so the output can be off by 2 |s|max 2^-24 relative (measured:
    0.5 |s|max 2^-24).  For |s|max <= 80 that is inside the 1e-5 of unit-scale inputs (the workloads'
    scores are N(0,1): |s| < 6); beyond, the bound grows with |s|max.  Returns (tolerance, |s|max)."""
    k = f64(mk, w.dtype)                                           # [Hkv][M][d]
    smax = 0.0
    for x in (q, wq):
        if x is None:
            continue
        xf = f64(x, w.dtype).reshape(-1, w.Hkv, x.shape[-2] // w.Hkv, w.d)      # [..][Hkv][G or 1][d]
        smax = max(smax, float(np.max(np.abs(np.einsum("nhgd,hmd->nhgm", xf, k)))) * w.scale)
    return max(base, 2.0 * smax * 2.0 ** -24), smax


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("kind", ["zero_keys", "huge_queries", "tiny_queries", "zero_write_value"])
def test_extreme_inputs(P, R, dtype, kind):
    """Degenerate softmaxes: all-zero keys (uniform weights), queries scaled until the softmax is one-hot
    (scores of several hundred), queries scaled towards zero, and a write of zeros (state unchanged).
    Every case is held to the plain tolerances except the fp32 outputs and the state of huge_queries,
    whose bound follows the score magnitude (score_tolerance)."""
    from test_gpu_prefill import check_prefill_out
    w = syn.Workload(f"extreme_{kind}", 1, 2, 4, 2, 128, 256, dtype, 0)
    ref, gpu, mk, mv0, _ = make_pair(w, R.RefCache, P.BctCache, mv0=True, max_prefill_T=40)
    if kind == "zero_keys":
        z = np.zeros_like(mk)
        ref.set_keys(z)
        gpu.set_keys(to_dev(z, dtype))

    def shape_inputs(q, wq, wv):
        if kind == "huge_queries":
            q, wq = (syn.pack(f64(a, dtype) * 256.0, dtype) for a in (q, wq))
        if kind == "tiny_queries":
            q, wq = (syn.pack(f64(a, dtype) * 2.0 ** -20, dtype) for a in (q, wq))
        if kind == "zero_write_value":
            wv = np.zeros_like(wv)
        return q, wq, wv

    for t in range(2):
        q, wq, wv = shape_inputs(*step_np(w, t))
        before = ref.values()
        gpu.set_values(to_dev(before, dtype))
        o_ref = ref.decode_step(q, wq, wv)
        o_gpu = gpu.decode_step(to_dev(q, dtype), to_dev(wq, dtype), to_dev(wv, dtype))
        tol, smax = score_tolerance(q, wq, mk, w, 1e-5)
        if kind == "huge_queries" and dtype == "f32":
            g, r = f64(to_np(o_gpu, dtype), dtype), f64(o_ref, dtype)
            e = rel_normwise(g, r)
            print(f"huge_queries fp32 step {t}: |s|max {smax:.0f}, out rel err {e:.2e}, bound {tol:.2e}")
            assert np.all(np.isfinite(g)) and smax > 400 and e <= tol, f"{kind} step {t}: {e:.2e} > {tol:.2e}"
        else:
            check_out(to_np(o_gpu, dtype), o_ref, dtype, f"{kind} step {t}")   # bf16: the bound is rounding, not scores
        got = to_np(gpu.export()[1], dtype)
        if kind == "zero_write_value":
            assert np.array_equal(got, before)
        elif kind == "huge_queries" and dtype == "f32":
            r = ref.values().astype(np.float64)
            assert np.max(np.abs(got - r)) <= tol * np.max(np.abs(r)), f"{kind} step {t}"
        else:
            check_state_one_step(got, ref.values(), dtype, f"{kind} step {t}", before=before,
                                 rel=tol if kind == "huge_queries" else 4e-6)
    # the same through a chunk
    T = 40
    q, wq, wv = shape_inputs(*syn.make_step(w, 2, T=T))
    gpu.set_values(to_dev(ref.values(), dtype))
    o_ref = ref.prefill(q, wq, wv, T)
    o_gpu = gpu.prefill(to_dev(q, dtype), to_dev(wq, dtype), to_dev(wv, dtype), T)
    g, r = f64(to_np(o_gpu, dtype), dtype), f64(o_ref, dtype)
    assert np.all(np.isfinite(g))
    if dtype == "f32":
        tol, smax = score_tolerance(q.reshape(-1, w.Hq, w.d), wq.reshape(-1, w.Hkv, w.d), mk, w, 1e-5)
        e = rel_normwise(g, r)
        print(f"{kind} fp32 chunk: |s|max {smax:.0f}, out rel err {e:.2e}, bound {tol:.2e}")
        assert e <= (tol if kind == "huge_queries" else 1e-5), kind
    else:
        # huge_queries: a one-hot read returns a stored value of up to 4 in size, where one bf16 spacing is
        # 0.031: the bound there is the relative one (spacings of the vector's largest entry)
        e = check_prefill_out(to_np(o_gpu, dtype), o_ref, dtype, f"{kind} chunk",
                              abs_bound=None if kind == "huge_queries" else 2e-2)
        print(f"{kind} bf16 chunk: out within {e:.2f} ulp of the vector max")
