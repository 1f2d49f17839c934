"""GPU parity of the per-token step size (bct_decode_step_gated, bct_prefill_gated) against the
oracle: MV <- MV + eta * ww^T wv with one eta per memory and token (section 3.5, the learning-rate
adaptation item).  Same tolerances as the plain calls: the gate multiplies the fp32 write weight."""
import numpy as np
import pytest

import bct_synth as syn
from _util import bf16_ulp, f64, make_pair, to_dev, to_np
from test_gpu_parity import check_out, check_state_one_step
from test_gpu_prefill import PF_WEIGHT_REL, check_prefill_out

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def P():
    import paper_2411_15785_amd as pkg
    pkg.lib()
    return pkg


@pytest.fixture(scope="module")
def R():
    from oracle import bct_ref
    return bct_ref


def gates(seed, shape):
    """Step sizes in [0, ~2.5], with some exact zeros and ones."""
    g = np.abs(syn.normal(seed, 9, 77, shape)).astype(np.float32)
    flat = g.reshape(-1)
    flat[::7] = 0.0
    flat[3::11] = 1.0
    return g


def gdev(g):
    import torch
    return torch.from_numpy(g).cuda()


@pytest.mark.parametrize("name,B,Hq,Hkv,d,M,dtype", [
    ("f32", 2, 4, 2, 64, 128, "f32"), ("bf16", 3, 4, 4, 128, 512, "bf16"), ("bf16_gqa", 2, 8, 2, 128, 4096, "bf16"),
    ("bf16_d64", 1, 2, 2, 64, 192, "bf16")])
def test_gated_decode_steps(P, R, name, B, Hq, Hkv, d, M, dtype):
    w = syn.Workload(name, 1, B, Hq, Hkv, d, M, dtype, 0)
    ref, gpu, mk, _, _ = make_pair(w, R.RefCache, P.BctCache, mv0=True)
    for t in range(5):
        q, wq, wv = syn.make_step(w, t)
        if t == 3:
            q = None                                     # a gated write-only step
        g = gates(t, (B, Hkv))
        before = ref.values()
        gpu.set_values(to_dev(before, dtype))            # common state: one step's worth of difference
        o_ref = ref.decode_step(q, wq, wv, gate=g)
        o_gpu = gpu.decode_step(to_dev(q, dtype), to_dev(wq, dtype), to_dev(wv, dtype), gate=gdev(g))
        if q is not None:
            check_out(to_np(o_gpu, dtype), o_ref, dtype, f"{name} step {t}")
        check_state_one_step(to_np(gpu.export()[1], dtype), ref.values(), dtype, f"{name} step {t}", before=before)
        # memories whose step size is zero did not move at all
        zero = g == 0.0
        assert np.array_equal(to_np(gpu.export()[1], dtype)[zero], before[zero])


def test_gate_of_ones_is_bitwise_the_plain_call(P, R):
    w = syn.Workload("ones", 1, 2, 4, 2, 128, 256, "bf16", 0)
    _, a, _, _, _ = make_pair(w, R.RefCache, P.BctCache, mv0=True, max_prefill_T=70)
    _, b, _, _, _ = make_pair(w, R.RefCache, P.BctCache, mv0=True, max_prefill_T=70)
    import torch
    for t in range(3):
        q, wq, wv = (to_dev(x, "bf16") for x in syn.make_step(w, t))
        oa = a.decode_step(q, wq, wv)
        ob = b.decode_step(q, wq, wv, gate=torch.ones((w.B, w.Hkv), device="cuda"))
        assert torch.equal(oa, ob) and torch.equal(a.values_view(), b.values_view())
    q, wq, wv = (to_dev(x, "bf16") for x in syn.make_step(w, 3, T=70))
    oa = a.prefill(q, wq, wv, 70)
    ob = b.prefill(q, wq, wv, 70, gate=torch.ones((w.B, 70, w.Hkv), device="cuda"))
    assert torch.equal(oa, ob) and torch.equal(a.values_view(), b.values_view())


@pytest.mark.parametrize("name,B,Hq,Hkv,d,M,dtype,T", [
    ("f32_T5", 2, 4, 2, 64, 128, "f32", 5), ("bf16_T200", 2, 4, 2, 128, 256, "bf16", 200),
    ("bf16_T512", 1, 2, 2, 128, 1024, "bf16", 512), ("bf16_d64_T130", 1, 2, 1, 64, 128, "bf16", 130)])
def test_gated_prefill_chunk(P, R, name, B, Hq, Hkv, d, M, dtype, T):
    w = syn.Workload(name, 1, B, Hq, Hkv, d, M, dtype, 0)
    ref, gpu, mk, _, _ = make_pair(w, R.RefCache, P.BctCache, mv0=True, max_prefill_T=T)
    q, wq, wv = syn.make_step(w, 0, T=T)
    g = gates(5, (B, T, Hkv))
    before = ref.values()
    o_ref = ref.prefill(q, wq, wv, T, gate=g)
    o_gpu = gpu.prefill(to_dev(q, dtype), to_dev(wq, dtype), to_dev(wv, dtype), T, gate=gdev(g))
    check_prefill_out(to_np(o_gpu, dtype), o_ref, dtype, name)
    got = to_np(gpu.export()[1], dtype)
    if dtype == "f32":
        check_state_one_step(got, ref.values(), dtype, name)
        return
    # as in the plain prefill test: one rounding flip plus the weight error on the written mass,
    # mass[m] = sum_t eta_t ww_t[m] from the oracle (the same gated chunk with wv = 1 into a zero state)
    aux = R.RefCache(M, B, Hq, Hkv, d, dtype, ref.read_scale, ref.write_scale, 0)
    aux.set_keys(mk)
    aux.prefill(None, wq, syn.pack(np.ones(wv.shape), dtype), T, gate=g)
    mass = f64(aux.values(), dtype)[..., 0]
    wvmax = np.max(np.abs(f64(wv, dtype)), axis=1)
    bound = mass[..., :, None] * wvmax[..., None, :] * 1.01
    r = f64(ref.values(), dtype)
    allow = bf16_ulp(r) * 1.0001 + PF_WEIGHT_REL * bound
    dlt = np.abs(f64(got, dtype) - r)
    assert np.all(dlt <= allow), f"{name}: state off by {np.max(dlt / allow):.2f} x the allowance"
    assert not np.array_equal(got, before)


@pytest.mark.parametrize("name,B,Hq,Hkv,d,M,dtype,T", [
    ("f32", 2, 4, 2, 64, 128, "f32", 5), ("bf16_small", 2, 4, 4, 128, 128, "bf16", 40),
    ("bf16_T200", 2, 4, 2, 128, 256, "bf16", 200), ("bf16_gqa4", 1, 8, 2, 128, 2048, "bf16", 130)])
def test_negative_step_sizes_on_every_path(P, R, name, B, Hq, Hkv, d, M, dtype, T):
    """eta of either sign: the decode step (one launch or four, vector or MFMA read) and the chunk (token by
    token in fp32, the MFMA path in bf16, where |eta| goes into the token's shift and the sign into its row
    of WV^T) all agree with the oracle's eta * ww, to the tolerances of the plain calls."""
    w = syn.Workload(name, 1, B, Hq, Hkv, d, M, dtype, 0)
    ref, gpu, mk, _, _ = make_pair(w, R.RefCache, P.BctCache, mv0=True, max_prefill_T=T)

    def signed(seed, shape):
        g = gates(seed, shape)
        flat = g.reshape(-1)
        flat[1::2] *= -1.0
        flat[5::13] = -1.0
        return g

    for t in range(3):
        q, wq, wv = syn.make_step(w, t)
        g = signed(t, (B, Hkv))
        before = ref.values()
        gpu.set_values(to_dev(before, dtype))
        o_ref = ref.decode_step(q, wq, wv, gate=g)
        o_gpu = gpu.decode_step(to_dev(q, dtype), to_dev(wq, dtype), to_dev(wv, dtype), gate=gdev(g))
        check_out(to_np(o_gpu, dtype), o_ref, dtype, f"{name} step {t}")
        check_state_one_step(to_np(gpu.export()[1], dtype), ref.values(), dtype, f"{name} step {t}", before=before)
    q, wq, wv = syn.make_step(w, 3, T=T)
    g = signed(9, (B, T, Hkv))
    before = ref.values()
    gpu.set_values(to_dev(before, dtype))
    o_ref = ref.prefill(q, wq, wv, T, gate=g)
    o_gpu = gpu.prefill(to_dev(q, dtype), to_dev(wq, dtype), to_dev(wv, dtype), T, gate=gdev(g))
    check_prefill_out(to_np(o_gpu, dtype), o_ref, dtype, name)
    got = to_np(gpu.export()[1], dtype)
    assert np.all(np.isfinite(f64(got, dtype)))
    if dtype == "f32":
        check_state_one_step(got, ref.values(), dtype, name)
        return
    aux = R.RefCache(M, B, Hq, Hkv, d, dtype, ref.read_scale, ref.write_scale, 0)
    aux.set_keys(mk)
    aux.prefill(None, wq, syn.pack(np.ones(wv.shape), dtype), T, gate=np.abs(g))     # mass of |eta| ww
    mass = f64(aux.values(), dtype)[..., 0]
    bound = mass[..., :, None] * np.max(np.abs(f64(wv, dtype)), axis=1)[..., None, :] * 1.01
    r = f64(ref.values(), dtype)
    dlt = np.abs(f64(got, dtype) - r)
    allow = bf16_ulp(r) * 1.0001 + PF_WEIGHT_REL * bound
    assert np.all(dlt <= allow), f"{name}: state off by {np.max(dlt / allow):.2f} x the allowance"


def test_gate_argument_errors(P, R):
    import torch
    w = syn.Workload("err", 1, 2, 2, 2, 128, 64, "bf16", 0)
    _, gpu, _, _, _ = make_pair(w, R.RefCache, P.BctCache, max_prefill_T=8)
    q, wq, wv = (to_dev(x, "bf16") for x in syn.make_step(w, 0))
    g = torch.ones((w.B, w.Hkv), device="cuda")
    with pytest.raises(P.BctError) as e:
        gpu.decode_step(q, None, None, gate=g)           # a gate without a write
    assert e.value.status == P.BCT_ERR_INVALID_ARG
    with pytest.raises(ValueError):
        gpu.decode_step(q, wq, wv, gate=g.double())
    with pytest.raises(ValueError):
        gpu.decode_step(q, wq, wv, gate=torch.ones((w.B, w.Hkv + 1), device="cuda"))
    assert gpu.steps == 0
