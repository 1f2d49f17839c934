"""Seeded random sweep of decode-step shapes against the oracle: capacity, batch, heads, query heads
per KV head, head_dim, dtype, key sharing, forced path, step mode and step sizes all drawn from a
counter-based generator, so the cases are the same on every run.  Each case steps twice from a
common state (the oracle's) and checks the outputs and the state to the usual tolerances."""
import numpy as np
import pytest

import bct_synth as syn
from _util import make_pair, to_dev, to_np
from test_gpu_parity import check_out, check_state_one_step

pytestmark = pytest.mark.gpu


def draw_case(i):
    r = syn.integers(20241125, 6, i, (12,), 1 << 30)
    dtype = ("f32", "bf16")[r[0] % 2]
    d = (64, 128)[r[1] % 2]
    M = 64 * (1 + r[2] % (32 if r[3] % 4 else 3))      # a quarter of the cases stay at M <= 192 (one-launch step)
    B = 1 + r[4] % 6
    Hkv = 1 + r[5] % 4
    G = (1, 1, 2, 3, 4, 5, 8)[r[6] % 7]
    flags = (0, 0, 1, 2, 3)[r[7] % 5]
    mode = ("rw", "rw", "write_only", "read_only")[r[8] % 4]
    gated = bool(r[9] % 2) and mode != "read_only"
    return dict(dtype=dtype, d=d, M=int(M), B=int(B), Hkv=int(Hkv), G=G, flags=flags, mode=mode, gated=gated)


CASES = [draw_case(i) for i in range(40)]


@pytest.fixture(scope="module")
def P():
    import paper_2411_15785_amd as pkg
    pkg.lib()
    return pkg


@pytest.fixture(scope="module")
def R():
    from oracle import bct_ref
    return bct_ref


@pytest.mark.parametrize("i", range(len(CASES)))
def test_random_case(P, R, i):
    import torch
    c = CASES[i]
    what = f"case {i}: {c}"
    w = syn.Workload(f"rand{i}", 1, c["B"], c["Hkv"] * c["G"], c["Hkv"], c["d"], c["M"], c["dtype"], 0)
    ref, gpu, mk, _, _ = make_pair(w, R.RefCache, P.BctCache, flags=c["flags"], mv0=True, layer=i)
    dt = c["dtype"]
    for t in range(2):
        q, wq, wv = syn.make_step(w, t, layer=i)
        if c["mode"] == "write_only":
            q = None
        if c["mode"] == "read_only":
            wq = wv = None
        gate = None
        if c["gated"]:
            gate = np.abs(syn.normal(i, 9, t, (w.B, w.Hkv))).astype(np.float32)
            gate.reshape(-1)[::3] = 0.0
        before = ref.values()
        gpu.set_values(to_dev(before, dt))
        o_ref = ref.decode_step(q, wq, wv, gate=gate)
        o_gpu = gpu.decode_step(to_dev(q, dt), to_dev(wq, dt), to_dev(wv, dt),
                                gate=None if gate is None else torch.from_numpy(gate).cuda())
        if q is not None:
            check_out(to_np(o_gpu, dt), o_ref, dt, what)
        mk_g, mv_g, st = gpu.export()
        assert np.array_equal(to_np(mk_g, dt), mk), what
        if c["mode"] == "read_only":
            assert np.array_equal(to_np(mv_g, dt), before), what
        else:
            check_state_one_step(to_np(mv_g, dt), ref.values(), dt, what, before=before)
        assert st == t + 1


# ---------------------------------------------------------------- chunks (bf16 MFMA prefill)

def draw_chunk(i):
    r = syn.integers(20241126, 6, i, (12,), 1 << 30)
    d = (64, 128)[r[0] % 2]
    M = 64 * (1 + r[1] % 12)
    B = 1 + r[2] % 3
    Hkv = 1 + r[3] % 2
    G = (1, 1, 2, 3, 4, 8)[r[4] % 6]
    T = int((1 + r[5] % 300, 128, 129, 256, 127)[r[6] % 5] if r[6] % 3 else 1 + r[5] % 300)
    flags = (0, 0, 1)[r[7] % 3]
    mode = ("rw", "rw", "rw", "write_only", "read_only")[r[8] % 5]
    gated = bool(r[9] % 2) and mode != "read_only"
    scales = ((None, None), (0.2, 0.05), (-0.07, 0.11), (0.09, -0.1))[r[10] % 4]
    return dict(d=d, M=int(M), B=int(B), Hkv=int(Hkv), G=G, T=T, flags=flags, mode=mode, gated=gated, scales=scales)


CHUNKS = [draw_chunk(i) for i in range(24)]


@pytest.mark.parametrize("i", range(len(CHUNKS)))
def test_random_chunk(P, R, i):
    """Seeded random sweep of prefill chunks (bf16): ragged lengths around the 128-token sub-chunk, all modes,
    step sizes, per-sequence keys, scales of either sign; one chunk from a common random state."""
    import torch
    from test_gpu_prefill import check_prefill_out, check_prefill_state
    c = CHUNKS[i]
    what = f"chunk {i}: {c}"
    w = syn.Workload(f"randpf{i}", 1, c["B"], c["Hkv"] * c["G"], c["Hkv"], c["d"], c["M"], "bf16", 0)
    kw = {}
    if c["scales"][0] is not None:
        kw = dict(read_scale=c["scales"][0], write_scale=c["scales"][1])
    T = c["T"]
    ref, gpu, mk, _, _ = make_pair(w, R.RefCache, P.BctCache, flags=c["flags"], mv0=True, layer=100 + i,
                                   max_prefill_T=T, **kw)
    q, wq, wv = syn.make_step(w, 0, layer=100 + i, T=T)
    if c["mode"] == "write_only":
        q = None
    if c["mode"] == "read_only":
        wq = wv = None
    gate = None
    if c["gated"]:
        gate = np.abs(syn.normal(i, 9, 77, (w.B, T, w.Hkv))).astype(np.float32)
        gate.reshape(-1)[::5] = 0.0
    before = ref.values()
    o_ref = ref.prefill(q, wq, wv, T, gate=gate)
    o_gpu = gpu.prefill(to_dev(q, "bf16"), to_dev(wq, "bf16"), to_dev(wv, "bf16"), T,
                        gate=None if gate is None else torch.from_numpy(gate).cuda())
    if q is not None:
        e = check_prefill_out(to_np(o_gpu, "bf16"), o_ref, "bf16", what)
        print(f"{what}: out {e:.2f} ulp of the vector max")
    mk_g, mv_g, st = gpu.export()
    assert np.array_equal(to_np(mk_g, "bf16"), mk), what
    if c["mode"] == "read_only":
        assert np.array_equal(to_np(mv_g, "bf16"), before), what
    elif gate is None:
        frac = check_prefill_state(R, ref, mk, wq, wv, to_np(mv_g, "bf16"), T, what)
        print(f"{what}: {frac:.3%} of state elements differ")
    else:
        # with step sizes the written mass is eta-weighted: bound it with wv scaled by the largest step size
        gmax = float(np.max(gate))
        scaled = syn.pack(syn.unpack(wv, "bf16") * max(gmax, 1.0), "bf16")
        check_prefill_state(R, ref, mk, wq, scaled, to_np(mv_g, "bf16"), T, what)
    assert st == T
