"""GPU parity of the state-management calls: random initial MV (section 3.1 allows zero or random initial contents),
bit for bit against the oracle's generator, and the per-sequence export / import that swaps a
session's fixed-size state (section 4.3: memory independent of the sequence length)."""
import numpy as np
import pytest

import bct_synth as syn
from _util import make_pair, to_dev, to_np

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


@pytest.mark.parametrize("dtype,B,H,d,M", [("f32", 2, 2, 64, 128), ("bf16", 3, 4, 128, 1024), ("bf16", 1, 1, 64, 64)])
@pytest.mark.parametrize("seed,amp", [(0, 1.0), (2 ** 63 + 12345, 0.02)])
def test_random_initial_values_are_bit_exact(P, R, dtype, B, H, d, M, seed, amp):
    w = syn.Workload("rnd", 1, B, H, H, d, M, dtype, 0)
    ref, gpu, _, _, _ = make_pair(w, R.RefCache, P.BctCache)
    ref.randomize_values(seed, amp)
    gpu.randomize_values(seed, amp)
    got = to_np(gpu.export()[1], dtype)
    assert np.array_equal(got, ref.values())
    assert gpu.steps == 0
    # and the step from that state is the usual step
    q, wq, wv = syn.make_step(w, 0)
    o_ref = ref.decode_step(q, wq, wv)
    o_gpu = gpu.decode_step(to_dev(q, dtype), to_dev(wq, dtype), to_dev(wv, dtype))
    err = np.max(np.abs(syn.unpack(to_np(o_gpu, dtype), dtype) - syn.unpack(o_ref, dtype)))
    assert err <= (1e-5 if dtype == "f32" else 2e-2)


def test_session_swap_is_exact_and_touches_one_sequence(P, R):
    w = syn.Workload("swap", 1, 3, 4, 2, 128, 256, "bf16", 0)
    ref, gpu, _, mv0, _ = make_pair(w, R.RefCache, P.BctCache, mv0=True)
    other, _, _, _, _ = make_pair(w, R.RefCache, P.BctCache, mv0=True)   # an oracle that is never swapped
    for t in range(2):
        q, wq, wv = syn.make_step(w, t)
        ref.decode_step(q, wq, wv), other.decode_step(q, wq, wv)
        gpu.decode_step(to_dev(q, "bf16"), to_dev(wq, "bf16"), to_dev(wv, "bf16"))
    # park sequence 1, let another session use its slot, bring it back
    parked = gpu.export_sequence(1)
    assert np.array_equal(to_np(parked, "bf16"), to_np(gpu.export()[1], "bf16")[1])
    intruder = syn.pack(syn.normal(9, 9, 9, parked.shape), "bf16")
    gpu.import_sequence(1, to_dev(intruder, "bf16"))
    ref.import_sequence(1, intruder)
    now = to_np(gpu.export()[1], "bf16")
    assert np.array_equal(now[1], intruder)
    q, wq, wv = syn.make_step(w, 2)
    ref.decode_step(q, wq, wv)
    gpu.decode_step(to_dev(q, "bf16"), to_dev(wq, "bf16"), to_dev(wv, "bf16"))
    # sequences 0 and 2 never noticed: same state as the oracle that was never swapped, to the usual bound
    other.decode_step(q, wq, wv)
    g = syn.unpack(to_np(gpu.export()[1], "bf16"), "bf16")
    o = syn.unpack(other.values(), "bf16")
    for b in (0, 2):
        assert np.max(np.abs(g[b] - o[b])) <= 2.0 ** -7 * np.max(np.abs(o[b]))
    # bring the parked session back: bit for bit what was parked
    gpu.import_sequence(1, parked)
    assert np.array_equal(to_np(gpu.export_sequence(1), "bf16"), to_np(parked, "bf16"))
    assert gpu.steps == 3


def test_per_sequence_keys_travel_with_the_session(P, R):
    w = syn.Workload("swapk", 1, 2, 2, 2, 64, 64, "f32", 0)
    _, gpu, mk, _, _ = make_pair(w, R.RefCache, P.BctCache, flags=P.BCT_MK_PER_SEQUENCE, mv0=True)
    k1, v1 = gpu.export_sequence(1, with_keys=True)
    assert np.array_equal(to_np(k1, "f32"), mk[1])
    gpu.import_sequence(0, v1, mk=k1)                       # sequence 0 becomes a copy of sequence 1
    mk_g, mv_g, _ = gpu.export()
    assert np.array_equal(to_np(mk_g, "f32")[0], mk[1]) and np.array_equal(to_np(mv_g, "f32")[0], to_np(v1, "f32"))
    q, wq, wv = syn.make_step(w, 0)
    for a in (q, wq, wv):
        a[0] = a[1]                                         # same inputs -> same outputs for both sequences
    o = to_np(gpu.decode_step(to_dev(q, "f32"), to_dev(wq, "f32"), to_dev(wv, "f32")), "f32")
    assert np.array_equal(o[0], o[1])


def test_session_call_errors(P, R):
    w = syn.Workload("err", 1, 2, 2, 2, 64, 64, "bf16", 0)
    _, gpu, _, _, _ = make_pair(w, R.RefCache, P.BctCache)
    with pytest.raises(P.BctError) as e:
        gpu.export_sequence(2)                              # beyond the batch
    assert e.value.status == P.BCT_ERR_INVALID_ARG
    with pytest.raises(P.BctError):
        gpu.export_sequence(0, with_keys=True)              # shared keys: no per-sequence MK
    with pytest.raises(P.BctError):
        gpu.randomize_values(1, float("inf"))


@pytest.mark.parametrize("n_vec", [1, 255, 1024, 1025, 3 * 1024 + 77, 8192 * 1024 + 513])
def test_stream_copy_copies_exactly_its_range(P, n_vec):
    """bct_stream_copy: every byte of the range arrives, the bytes after it stay as they were (sizes that
    end inside a lane group, inside a workgroup's visit, and beyond one visit of the whole grid)."""
    import ctypes

    import torch
    g = torch.Generator(device="cpu").manual_seed(n_vec)
    src = torch.randint(0, 256, (n_vec * 16,), dtype=torch.uint8, generator=g).to("cuda:0")
    dst = torch.full((n_vec * 16 + 4096,), 0xA5, dtype=torch.uint8, device="cuda:0")
    st = P.lib().bct_stream_copy(ctypes.c_void_p(dst.data_ptr()), ctypes.c_void_p(src.data_ptr()), n_vec * 16,
                                 ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert st == P.BCT_OK
    torch.cuda.synchronize()
    assert torch.equal(dst[:n_vec * 16], src)
    assert bool((dst[n_vec * 16:] == 0xA5).all())
