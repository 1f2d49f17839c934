"""CPU-only checks of the C ABI: libbct.so loads without a GPU, exports every symbol
include/bct.h declares, and validates its arguments before the first HIP call."""
import ctypes
import os
import re

import pytest

import paper_2411_15785_amd as P
from paper_2411_15785_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2411_15785_amd import build
        build.build()
    return P.lib()


def declared_functions(header="bct.h", prefix="bct_"):
    src = open(os.path.join(ROOT, "include", header)).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(" + prefix + r"[a-z_]+)\s*\(", src)))


def test_every_declared_symbol_is_exported_and_bound(L):
    names = declared_functions()
    assert {"bct_cache_init", "bct_decode_step", "bct_prefill"} <= set(names)
    aids = declared_functions("bct_measure.h")
    assert {"bct_profile_enable", "bct_profile_read", "bct_stream_copy"} == set(aids) and not set(aids) & set(names)
    names = sorted(names + aids)
    for n in names:
        assert hasattr(L, n), f"{n} is declared in include/ but not exported by libbct.so"
    assert sorted(binding.EXPORTS) == names      # the binding names exactly the header's functions


def test_every_declared_model_symbol_is_exported_and_bound(L):
    from paper_2411_15785_amd import model
    names = declared_functions("bct_model.h", "bctm_")
    assert {"bctm_linear", "bctm_swiglu", "bctm_rmsnorm", "bctm_embed", "bctm_argmax", "bctm_pack_weight", "bctm_pack_rows"} <= set(names)
    ML = model.mlib()
    for n in names:
        assert hasattr(ML, n), f"{n} is declared in include/bct_model.h but not exported by libbct.so"
    assert sorted(model.MODEL_EXPORTS) == names


def test_model_entry_points_check_arguments_before_touching_the_gpu(L):
    from paper_2411_15785_amd import model
    ML = model.mlib()
    p = ctypes.c_void_p
    a, b, c = p(0x10000), p(0x20000), p(0x30000)
    assert ML.bctm_linear(a, b, None, c, 4, 72, 32, 0, None) == P.BCT_ERR_UNSUPPORTED       # K % 32
    assert ML.bctm_linear(a, b, None, c, 4, 64, 40, 0, None) == P.BCT_ERR_UNSUPPORTED       # N % 16
    assert ML.bctm_pack_weight(a, b, 40, 64, None) == P.BCT_ERR_UNSUPPORTED
    assert ML.bctm_pack_weight(a, a, 32, 64, None) == P.BCT_ERR_INVALID_ARG              # in place
    assert ML.bctm_pack_weight(a, None, 32, 64, None) == P.BCT_ERR_INVALID_ARG
    assert ML.bctm_linear(a, None, None, c, 4, 64, 32, 0, None) == P.BCT_ERR_INVALID_ARG
    assert ML.bctm_linear(a, b, None, c, 0, 64, 32, 0, None) == P.BCT_ERR_INVALID_ARG
    assert ML.bctm_linear(p(0x10008), b, None, c, 4, 64, 32, 0, None) == P.BCT_ERR_MISALIGNED
    assert ML.bctm_linear(a, b, p(0x40004), c, 4, 64, 32, 0, None) == P.BCT_ERR_MISALIGNED
    assert ML.bctm_swiglu(a, b, None, c, 4, 64, 32, 0, None) == P.BCT_ERR_INVALID_ARG
    assert ML.bctm_rmsnorm(a, b, c, 4, 12, 1e-5, 0, None) == P.BCT_ERR_UNSUPPORTED          # dim % 8
    assert ML.bctm_rmsnorm(a, b, c, 4, 32768, 1e-5, 0, None) == P.BCT_ERR_UNSUPPORTED
    assert ML.bctm_rmsnorm(a, b, c, 4, 40, 1e-5, 2, None) == P.BCT_ERR_UNSUPPORTED           # tiled: dim % 32
    assert ML.bctm_rmsnorm(a, b, a, 4, 64, 1e-5, 2, None) == P.BCT_ERR_INVALID_ARG           # tiled in place
    assert ML.bctm_rmsnorm(a, b, c, 4, 64, 1e-5, 1, None) == P.BCT_ERR_INVALID_ARG           # not its flag
    assert ML.bctm_linear(a, b, None, c, 4, 64, 32, 2, None) == P.BCT_ERR_INVALID_ARG        # no tiled output
    assert ML.bctm_linear(a, b, None, a, 4, 64, 32, 0, None) == P.BCT_ERR_INVALID_ARG        # out is x
    assert ML.bctm_swiglu(a, b, b, c, 4, 64, 48, 2, None) == P.BCT_ERR_UNSUPPORTED           # tiled out: N % 32
    assert ML.bctm_swiglu(a, b, b, c, 4, 64, 32, 8, None) == P.BCT_ERR_INVALID_ARG
    d = p(0x50000)
    assert ML.bctm_linear_split(a, b, c, 32, d, 24, None, 0, 4, 64, 0, None) == P.BCT_ERR_UNSUPPORTED   # width % 16
    assert ML.bctm_linear_split(a, b, c, 32, None, 16, None, 0, 4, 64, 0, None) == P.BCT_ERR_INVALID_ARG
    assert ML.bctm_linear_split(a, b, c, 32, d, 16, None, 16, 4, 64, 0, None) == P.BCT_ERR_INVALID_ARG  # out2 missing
    assert ML.bctm_linear_split(a, b, c, 0, d, 16, None, 0, 4, 64, 0, None) == P.BCT_ERR_INVALID_ARG
    assert ML.bctm_pack_rows(a, b, 4, 40, None) == P.BCT_ERR_UNSUPPORTED
    assert ML.bctm_pack_rows(a, a, 4, 64, None) == P.BCT_ERR_INVALID_ARG
    assert ML.bctm_embed(None, b, c, 4, 10, 64, None) == P.BCT_ERR_INVALID_ARG
    assert ML.bctm_embed(a, b, c, 4, 10, 12, None) == P.BCT_ERR_UNSUPPORTED
    assert ML.bctm_argmax(a, None, 4, 10, None) == P.BCT_ERR_INVALID_ARG
    assert ML.bctm_last_error().decode() != ""


def test_projection_kernel_choice():
    """bctm_linear_plan: which kernel a projection shape runs in (host logic).  The 7B-shaped stack: a decode
    batch streams the weights; a prompt chunk takes the matrix-core kernel, 256 x 256 where the shape allows."""
    from paper_2411_15785_amd import model as Mo
    S, SW, T128, T256 = (Mo.BCTM_KERNEL_STREAMING, Mo.BCTM_KERNEL_STREAMING_WIDE, Mo.BCTM_KERNEL_TILE128,
                         Mo.BCTM_KERNEL_TILE256)
    plan = Mo.bctm_linear_plan
    # decode batch of 32
    assert plan(32, 4096, 12288) == Mo.BCTM_KERNEL_STREAMING_TRIPLE and plan(32, 4096, 4096) == S
    assert plan(32, 11008, 4096) == S and plan(32, 4096, 6144) == S and plan(32, 4096, 12304) == S
    assert plan(32, 4096, 32000) == SW and plan(32, 4096, 11008, swiglu=True) == S
    assert plan(127, 4096, 4096) == S
    # prompt chunk of 32 x 512 rows
    for N in (12288, 4096, 32000):
        assert plan(16384, 4096, N) == T256
    assert plan(16384, 4096, 11008, swiglu=True) == T256
    # in between, and feature counts the larger tiles do not divide
    assert plan(128, 4096, 4096) == T128 and plan(1023, 4096, 4096) == T128 and plan(1024, 4096, 4096) == T256
    assert plan(4096, 4096, 384) == T128 and plan(4096, 4096, 192, swiglu=True) == T128
    assert plan(4096, 4096, 48) == S and plan(4096, 4096, 96, swiglu=True) == S
    assert plan(4096, 4096, 16416) == SW
    ML = Mo.mlib()
    k = ctypes.c_uint32(0)
    assert ML.bctm_linear_plan(4, 72, 32, 0, ctypes.byref(k)) == P.BCT_ERR_UNSUPPORTED
    assert ML.bctm_linear_plan(4, 64, 32, 0, None) == P.BCT_ERR_INVALID_ARG
    assert ML.bctm_linear_plan(0, 64, 32, 0, ctypes.byref(k)) == P.BCT_ERR_INVALID_ARG


def desc(**kw):
    d = dict(capacity_M=4096, batch=32, n_q_heads=32, n_kv_heads=32, head_dim=128, dtype=P.BCT_BF16,
             read_scale=0.0884, write_scale=0.0884, flags=0)
    d.update(kw)
    return P.make_desc(**d)


def test_query_sizes_are_exact_and_constant(L):
    st, cb, wb = P.bct_cache_query(desc(), 0)
    assert st == P.BCT_OK
    assert cb == 32 * 4096 * 128 * 2 + 32 * 32 * 4096 * 128 * 2      # MK + MV, nothing else
    st, cb2, wb2 = P.bct_cache_query(desc(), 512)
    assert st == P.BCT_OK and cb2 == cb and wb2 > wb                # prefill only adds workspace
    st, cbp, _ = P.bct_cache_query(desc(flags=P.BCT_MK_PER_SEQUENCE), 0)
    assert st == P.BCT_OK and cbp == 2 * 32 * 32 * 4096 * 128 * 2
    st, cbf, _ = P.bct_cache_query(desc(dtype=P.BCT_F32, head_dim=64, capacity_M=64, batch=1, n_q_heads=4,
                                        n_kv_heads=4), 0)
    assert st == P.BCT_OK and cbf == 2 * 4 * 64 * 64 * 4


@pytest.mark.parametrize("kw,status", [
    (dict(capacity_M=0), P.BCT_ERR_INVALID_ARG),
    (dict(batch=0), P.BCT_ERR_INVALID_ARG),
    (dict(n_q_heads=30), P.BCT_ERR_INVALID_ARG),            # not a multiple of n_kv_heads
    (dict(read_scale=float("nan")), P.BCT_ERR_INVALID_ARG),
    (dict(capacity_M=100), P.BCT_ERR_UNSUPPORTED),          # not a multiple of 64
    (dict(capacity_M=131072), P.BCT_ERR_UNSUPPORTED),
    (dict(head_dim=96), P.BCT_ERR_UNSUPPORTED),
    (dict(dtype=7), P.BCT_ERR_UNSUPPORTED),
    (dict(flags=8), P.BCT_ERR_UNSUPPORTED),
    (dict(flags=4), P.BCT_ERR_UNSUPPORTED),
    (dict(n_q_heads=32, n_kv_heads=2), P.BCT_ERR_UNSUPPORTED),   # 16 query heads per KV head
])
def test_bad_descriptors_are_rejected(L, kw, status):
    st, _, _ = P.bct_cache_query(desc(**kw), 0)
    assert st == status
    assert P.bct_last_error() != ""
    st, h = P.bct_cache_init(desc(**kw), 0, ctypes.c_void_p(0x1000), 1 << 40, ctypes.c_void_p(0x2000), 1 << 40, None)
    assert st == status and not h.value


def test_init_checks_pointers_and_sizes_before_touching_the_gpu(L):
    d = desc()
    _, cb, wb = P.bct_cache_query(d, 0)
    ok_c, ok_w = ctypes.c_void_p(0x10000), ctypes.c_void_p(0x20000)
    assert L.bct_cache_query(None, 0, None, None) == P.BCT_ERR_INVALID_ARG
    assert P.bct_cache_init(d, 0, None, cb, ok_w, wb, None)[0] == P.BCT_ERR_INVALID_ARG
    assert P.bct_cache_init(d, 0, ok_c, cb, None, wb, None)[0] == P.BCT_ERR_INVALID_ARG
    assert P.bct_cache_init(d, 0, ctypes.c_void_p(0x10010), cb, ok_w, wb, None)[0] == P.BCT_ERR_MISALIGNED
    assert P.bct_cache_init(d, 0, ok_c, cb - 1, ok_w, wb, None)[0] == P.BCT_ERR_BUFFER_TOO_SMALL
    assert P.bct_cache_init(d, 0, ok_c, cb, ok_w, wb - 1, None)[0] == P.BCT_ERR_BUFFER_TOO_SMALL
    assert P.bct_cache_init(d, 512, ok_c, cb, ok_w, wb, None)[0] == P.BCT_ERR_BUFFER_TOO_SMALL  # prefill needs more


def test_null_handles_and_messages(L):
    vp = ctypes.c_void_p
    assert L.bct_decode_step(None, vp(16), vp(16), vp(16), vp(16), None) == P.BCT_ERR_INVALID_ARG
    assert L.bct_prefill(None, vp(16), vp(16), vp(16), 4, vp(16), None) == P.BCT_ERR_INVALID_ARG
    assert L.bct_cache_set_keys(None, vp(16), None) == P.BCT_ERR_INVALID_ARG
    assert L.bct_cache_steps(None, None) == P.BCT_ERR_INVALID_ARG
    assert L.bct_stream_copy(vp(16), vp(16), 24, None) == P.BCT_ERR_INVALID_ARG   # not a multiple of 16
    assert L.bct_stream_copy(vp(8), vp(16), 32, None) == P.BCT_ERR_MISALIGNED
    L.bct_cache_destroy(None)                                                     # harmless
    for st in range(7):
        assert P.bct_strerror(st) not in ("", "unknown status")
    assert P.bct_strerror(99) == "unknown status"


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "one GPU" in r.stderr


def test_launch_plans_of_the_five_workloads(L):
    """Host logic: which path a decode step takes, decided from the descriptor alone."""
    import bct_synth as syn

    def plan(name, flags=0):
        w = syn.WORKLOADS[name]
        dt = P.BCT_F32 if w.dtype == "f32" else P.BCT_BF16
        st, info = P.bct_plan_query(P.make_desc(w.M, w.B, w.Hq, w.Hkv, w.d, dt, w.scale, w.scale, flags))
        assert st == P.BCT_OK
        return info

    c1 = plan("cfg1")            # 4 memories of 64 slots: one launch
    assert c1["one_launch"] == 1 and c1["launches"] == 1
    c1s = plan("cfg1", P.BCT_STEP_STREAMING)
    assert c1s["one_launch"] == 0 and c1s["scores_mfma"] == 0 and c1s["launches"] == 2     # one split: no merge
    c2 = plan("cfg2")            # M = 1024: too large for the one-launch step; 256 memories of 256 KB: one MV-pass workgroup each
    assert c2["one_launch"] == 0 and c2["scores_mfma"] == 1
    assert c2["mv_workgroup"] == 1024 and c2["mv_loads_per_lane"] == 16 and c2["mv_splits"] == 1 and c2["launches"] == 2
    w2 = syn.WORKLOADS["cfg2"]
    for batch, splits in ((4, 16), (5, 16), (6, 1), (8, 1), (9, 16)):     # 128, 160: too few memories; 288 x 256 KB: too much in all
        st, pl = P.bct_plan_query(P.make_desc(w2.M, batch, w2.Hq, w2.Hkv, w2.d, P.BCT_BF16, w2.scale, w2.scale))
        assert st == P.BCT_OK and pl["mv_splits"] == splits, (batch, pl)
    c3 = plan("cfg3")            # the headline shape: scores, MV pass (merging the 32 partials per row itself), merge
    assert c3 == dict(launches=3, one_launch=0, scores_mfma=1, slots_per_stat=128, normaliser_launch=0,
                      mv_workgroup=256, mv_loads_per_lane=4, mv_splits=64)
    assert c3["mv_workgroup"] * c3["mv_loads_per_lane"] * 16 * c3["mv_splits"] == 4096 * 128 * 2   # one memory, one-shot
    c4 = plan("cfg4")            # 4 query heads per KV head: the MFMA read, 16 KB workgroups; 128 partials per row: own launch
    assert c4["mv_workgroup"] == 128 and c4["mv_loads_per_lane"] == 8 and c4["normaliser_launch"] == 1
    w4 = syn.WORKLOADS["cfg4"]
    st, f4 = P.bct_plan_query(P.make_desc(w4.M, w4.B, w4.Hq, w4.Hkv, w4.d, P.BCT_F32, w4.scale, w4.scale))
    assert st == P.BCT_OK and f4["mv_workgroup"] == 512          # fp32 storage keeps the vector-ALU read
    assert c4["launches"] == 4
    c5 = plan("cfg5")            # 128 partials per row, two per lane of the MV pass: no normaliser launch
    assert c5["slots_per_stat"] == 128 and c5["normaliser_launch"] == 0 and c5["launches"] == 3
    c5 = plan("cfg5")
    assert c5["mv_splits"] * c5["mv_workgroup"] * c5["mv_loads_per_lane"] * 16 == 16384 * 128 * 2
    assert plan("cfg3", P.BCT_MK_PER_SEQUENCE)["scores_mfma"] == 0      # per-sequence keys: no shared contraction
    st, _ = P.bct_plan_query(desc(capacity_M=100))
    assert st == P.BCT_ERR_UNSUPPORTED
    assert L.bct_plan_query(ctypes.byref(desc()), None) == P.BCT_ERR_INVALID_ARG
