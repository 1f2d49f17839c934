"""GPU parity of bct_decode_step_keyed against the oracle's keyed step: the write also moves the
per-sequence keys, MK_t = MK_(t-1) + kappa ww^T wk (this build's reading of keys "updated by the same soft
write"; the paper gives no equation, section 3.5), after the token's write to MV and its read.  Every
step starts from the oracle's state (keys and values), so the one-step criteria of the plain step apply
to out, to MV and, unchanged, to MK."""
import numpy as np
import pytest

import bct_synth as syn
from _util import make_pair, to_dev, to_np
from test_gpu_parity import check_out, check_state_one_step

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def P():
    import torch
    assert torch.cuda.is_available()
    import paper_2411_15785_amd as pkg
    pkg.lib()
    return pkg


@pytest.fixture(scope="module")
def R():
    from oracle import bct_ref
    return bct_ref


def key_vectors(w, t):
    return syn.pack(syn.normal(syn.layer_seed(0), 8, t, (w.B, w.Hkv, w.d)), w.dtype)


def step_sizes(seed, shape):
    g = syn.normal(seed, 9, 78, shape).astype(np.float32)     # either sign, some exact zeros and ones
    flat = g.reshape(-1)
    flat[::5] = 0.0
    flat[2::7] = 1.0
    return g


def gdev(g):
    import torch
    return None if g is None else torch.from_numpy(g).cuda()


CASES = [
    # name, B, Hq, Hkv, d, M, dtype
    ("f32_small", 2, 4, 4, 64, 128, "f32"),            # small enough for the one-launch step: the keyed step streams
    ("f32_gqa2", 2, 4, 2, 128, 320, "f32"),
    ("bf16_m512", 3, 4, 4, 128, 512, "bf16"),
    ("bf16_gqa4", 2, 8, 2, 128, 2112, "bf16"),         # MFMA read for the values, vector write-only pass for the keys
    ("bf16_d64_gqa8", 1, 8, 1, 64, 192, "bf16"),
    ("bf16_m8192", 1, 2, 2, 128, 8192, "bf16"),        # 128 statistics tiles per row: two per lane of the value and key passes
    ("bf16_m16384", 1, 2, 1, 128, 16384, "bf16"),      # more than that: the normaliser launch runs twice
]


@pytest.mark.parametrize("name,B,Hq,Hkv,d,M,dtype", CASES)
def test_keyed_steps_from_common_state(P, R, name, B, Hq, Hkv, d, M, dtype):
    w = syn.Workload(name, 1, B, Hq, Hkv, d, M, dtype, 0)
    ref, gpu, mk0, _, _ = make_pair(w, R.RefCache, P.BctCache, flags=1, mv0=True)
    for t in range(4):
        q, wq, wv = syn.make_step(w, t)
        wk = key_vectors(w, t)
        if t == 2:
            q = None                                            # a keyed write-only step
        eta = step_sizes(t, (B, Hkv)) if t % 2 else None
        kappa = step_sizes(10 + t, (B, Hkv)) if t else None     # first step: kappa = 1 everywhere
        k_before, v_before = ref.keys(), ref.values()
        gpu.set_keys(to_dev(k_before, dtype))
        gpu.set_values(to_dev(v_before, dtype))
        o_ref = ref.decode_step_keyed(q, wq, wv, wk, gate=eta, kgate=kappa)
        o_gpu = gpu.decode_step_keyed(to_dev(q, dtype), to_dev(wq, dtype), to_dev(wv, dtype), to_dev(wk, dtype),
                                      gate=gdev(eta), key_gate=gdev(kappa))
        what = f"{name} keyed step {t}"
        if q is not None:
            check_out(to_np(o_gpu, dtype), o_ref, dtype, what)
        check_state_one_step(to_np(gpu.values_view(), dtype), ref.values(), dtype, what + " (MV)", before=v_before)
        k_gpu = to_np(gpu.keys_view(), dtype)
        check_state_one_step(k_gpu, ref.keys(), dtype, what + " (MK)", before=k_before)
        still = np.zeros((B, Hkv), bool) if kappa is None else kappa == 0.0
        assert np.array_equal(k_gpu[still], k_before[still])   # memories with kappa = 0 keep their keys bit for bit
        assert all(not np.array_equal(k_gpu[b, h], k_before[b, h]) for b in range(B) for h in range(Hkv) if not still[b, h])
    assert gpu.steps == 4


def test_zero_key_step_is_the_gated_step_bit_for_bit(P, R):
    import torch
    w = syn.Workload("keyed_zero", 1, 2, 4, 2, 128, 256, "bf16", 0)
    _, a, mk, _, _ = make_pair(w, R.RefCache, P.BctCache, flags=1 | P.BCT_STEP_STREAMING, mv0=True)
    _, b, _, _, _ = make_pair(w, R.RefCache, P.BctCache, flags=1 | P.BCT_STEP_STREAMING, mv0=True)
    for t in range(3):
        q, wq, wv = (to_dev(x, "bf16") for x in syn.make_step(w, t))
        eta = gdev(step_sizes(t, (w.B, w.Hkv)))
        oa = a.decode_step(q, wq, wv, gate=eta)
        ob = b.decode_step_keyed(q, wq, wv, to_dev(key_vectors(w, t), "bf16"), gate=eta,
                                 key_gate=torch.zeros((w.B, w.Hkv), device="cuda"))
        assert torch.equal(oa, ob) and torch.equal(a.values_view(), b.values_view())
        assert np.array_equal(to_np(b.keys_view(), "bf16"), mk)


def test_keyed_trajectory_follows_the_moving_keys(P, R):
    """Eight keyed steps without resynchronisation: later tokens are addressed through keys that the earlier
    ones moved, on both sides; the outputs stay inside the plain bounds."""
    w = syn.Workload("keyed_run", 1, 2, 4, 4, 128, 1024, "bf16", 0)
    ref, gpu, mk0, _, _ = make_pair(w, R.RefCache, P.BctCache, flags=1)
    for t in range(8):
        q, wq, wv = syn.make_step(w, t)
        wk = key_vectors(w, t)
        o_ref = ref.decode_step_keyed(q, wq, wv, wk)
        o_gpu = gpu.decode_step_keyed(to_dev(q, "bf16"), to_dev(wq, "bf16"), to_dev(wv, "bf16"), to_dev(wk, "bf16"))
        check_out(to_np(o_gpu, "bf16"), o_ref, "bf16", f"keyed run step {t}")
    k = syn.unpack(to_np(gpu.keys_view(), "bf16"), "bf16")
    assert np.max(np.abs(k - syn.unpack(mk0, "bf16"))) > 1e-3           # the keys did move
    assert np.mean(to_np(gpu.keys_view(), "bf16") != ref.keys()) < 1e-2   # and agree but for rare rounding flips


def test_keyed_step_argument_errors(P, R):
    w = syn.Workload("keyed_err", 1, 2, 2, 2, 128, 64, "bf16", 0)
    _, shared, _, _, _ = make_pair(w, R.RefCache, P.BctCache)
    q, wq, wv = (to_dev(x, "bf16") for x in syn.make_step(w, 0))
    wk = to_dev(key_vectors(w, 0), "bf16")
    with pytest.raises(P.BctError) as e:
        shared.decode_step_keyed(q, wq, wv, wk)                  # keys shared by the batch cannot be written
    assert e.value.status == P.BCT_ERR_STATE
    _, per_seq, _, _, _ = make_pair(w, R.RefCache, P.BctCache, flags=1)
    with pytest.raises(P.BctError) as e:
        per_seq.decode_step_keyed(q, None, None, wk)             # a key write needs the token's write
    assert e.value.status == P.BCT_ERR_INVALID_ARG
    assert shared.steps == 0 and per_seq.steps == 0
