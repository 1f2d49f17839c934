"""Pins of the CPU oracle against what the paper and the mathematics fix.

None of these compares the oracle with itself or with the HIP path: every
expected value comes from a brute-force loop, a closed form, an invariant, a
special case that reduces to textbook attention, a hand-worked example or a
library routine.  Citations: section 3.2 (steps 1-5), Algorithm 1, the
section 3.4 update equation, section 3.5 (order-free accumulation), section
4.3 (memory constant).
"""
import json
import math
import os

import numpy as np
import pytest

import bct_synth as syn
from oracle import bct_ref
from oracle.bct_ref import RefCache

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rng_normal(seed, tid, step, shape, dtype):
    return syn.pack(syn.normal(seed, tid, step, shape), dtype)


def f64(a, dtype):
    return syn.unpack(a, dtype)


def softmax64(x):
    x = np.asarray(x, dtype=np.float64)
    e = np.exp(x - x.max())
    return e / e.sum()


def brute_attention(q, K, V, scale):
    """softmax(scale * q K^T) V with explicit loops, two passes, double."""
    M, d = K.shape
    s = [scale * sum(float(q[j]) * float(K[m, j]) for j in range(d)) for m in range(M)]
    mx = max(s)
    e = [math.exp(v - mx) for v in s]
    z = sum(e)
    out = [0.0] * V.shape[1]
    for m in range(M):
        for j in range(V.shape[1]):
            out[j] += (e[m] / z) * float(V[m, j])
    return np.array(out)


def make_cache(M, B, Hq, Hkv, d, dtype, rs=None, ws=None, seed=11, flags=0, mv0=False):
    rs = 1.0 / math.sqrt(d) if rs is None else rs
    ws = 1.0 / math.sqrt(d) if ws is None else ws
    c = RefCache(M, B, Hq, Hkv, d, dtype, rs, ws, flags)
    mk = rng_normal(seed, syn.TID_MK, 0, c.keys_shape, dtype)
    c.set_keys(mk)
    mv = None
    if mv0:
        mv = rng_normal(seed, syn.TID_MV0, 0, c.values_shape, dtype)
        c.set_values(mv)
    return c, mk, mv


def step_inputs(c, seed, step):
    q = rng_normal(seed, syn.TID_Q, step, (c.B, c.Hq, c.d), c.dtype)
    wq = rng_normal(seed, syn.TID_WQ, step, (c.B, c.Hkv, c.d), c.dtype)
    wv = rng_normal(seed, syn.TID_WV, step, (c.B, c.Hkv, c.d), c.dtype)
    return q, wq, wv


# ------------------------------------------------------------------ P1 brute-force read

@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("M,d,Hq,Hkv", [(8, 4, 4, 2), (5, 3, 3, 3), (7, 2, 6, 1)])
def test_p1_read_is_bruteforce_attention(dtype, M, d, Hq, Hkv):
    B, scale = 2, 0.7
    c, mk, mv = make_cache(M, B, Hq, Hkv, d, dtype, rs=scale, mv0=True)
    q = rng_normal(3, syn.TID_Q, 0, (B, Hq, d), dtype)
    out = c.decode_step(q, None, None)
    G = Hq // Hkv
    K, V, Q = f64(mk, dtype), f64(mv, dtype), f64(q, dtype)
    got = f64(out, dtype)
    for b in range(B):
        for hq in range(Hq):
            h = hq // G
            ref = brute_attention(Q[b, hq], K[h], V[b, h], scale)
            tol = 1e-6 if dtype == "f32" else 2 ** -8
            assert np.max(np.abs(got[b, hq] - ref)) <= tol * max(1.0, np.max(np.abs(ref)))
    # a read-only step leaves the state untouched
    assert np.array_equal(c.values(), mv)
    assert c.steps == 1


# ------------------------------------------------------------------ P2 capacity invariant

@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_p2_capacity_and_keys_constant(dtype):
    M, B, Hq, Hkv, d = 8, 2, 4, 2, 4
    c, mk, _ = make_cache(M, B, Hq, Hkv, d, dtype)
    sz = syn.elem_size(dtype)
    expect = (Hkv * M * d + B * Hkv * M * d) * sz
    assert c.cache_bytes() == expect
    for t in range(3 * M + 1):  # far past the capacity: nothing changes at t = M
        q, wq, wv = step_inputs(c, 5, t)
        out = c.decode_step(q, wq, wv)
        assert out.shape == (B, Hq, d)
        assert c.cache_bytes() == expect
        k2, v2, st = c.export()
        assert np.array_equal(k2, mk)          # MK is never written (Algorithm 1 input)
        assert v2.shape == (B, Hkv, M, d) and st == t + 1


# ------------------------------------------------------------------ P3 mass conservation

def test_p3_mass_conservation():
    M, B, Hq, Hkv, d = 16, 2, 2, 2, 8
    c, mk, mv0 = make_cache(M, B, Hq, Hkv, d, "f32", ws=1.0, mv0=True)
    tot = np.zeros((B, Hkv, d))
    N = 40
    for t in range(N):
        _, wq, wv = step_inputs(c, 7, t)
        c.decode_step(None, wq, wv)
        tot += wv.astype(np.float64)
    got = c.values().astype(np.float64).sum(axis=2)
    ref = mv0.astype(np.float64).sum(axis=2) + tot
    assert np.max(np.abs(got - ref)) <= 1e-5 * math.sqrt(N) * max(1.0, np.max(np.abs(ref)))


def test_p3b_probe_weights_are_a_softmax():
    M, d = 9, 5
    c, mk, _ = make_cache(M, 1, 1, 1, d, "f32")
    v = rng_normal(1, syn.TID_WQ, 0, (d,), "f32")
    w = c.probe_weights(0, 0, v, 0.3)
    ref = softmax64(0.3 * (mk[0].astype(np.float64) @ v.astype(np.float64)))
    assert abs(w.sum() - 1.0) < 1e-14 and np.all(w > 0)
    assert np.max(np.abs(w - ref)) < 1e-15
    # no overflow for huge scores (max-subtracted)
    big = (v.astype(np.float64) * 1e4).astype(np.float32)
    wb = c.probe_weights(0, 0, big, 1.0)
    assert np.all(np.isfinite(wb)) and abs(wb.sum() - 1.0) < 1e-12


# ------------------------------------------------------------------ P4 closed form, order freedom

@pytest.mark.parametrize("ws", [1.0, 0.25])
def test_p4_closed_form_and_order_freedom(ws):
    M, B, Hq, Hkv, d, N = 12, 2, 2, 2, 6, 20
    c, mk, mv0 = make_cache(M, B, Hq, Hkv, d, "f32", ws=ws, mv0=True)
    WQ = np.stack([step_inputs(c, 9, t)[1] for t in range(N)])  # [N][B][Hkv][d]
    WV = np.stack([step_inputs(c, 9, t)[2] for t in range(N)])
    for t in range(N):
        c.decode_step(None, WQ[t], WV[t])
    got = c.values().astype(np.float64)
    K = mk.astype(np.float64)
    for b in range(B):
        for h in range(Hkv):
            WW = np.stack([softmax64(ws * (K[h] @ WQ[t, b, h].astype(np.float64))) for t in range(N)])  # [N][M]
            ref = mv0[b, h].astype(np.float64) + WW.T @ WV[:, b, h].astype(np.float64)
            assert np.max(np.abs(got[b, h] - ref)) <= 2e-6 * max(1.0, np.max(np.abs(ref)))
    # token order does not matter (section 3.5)
    c2, _, _ = make_cache(M, B, Hq, Hkv, d, "f32", ws=ws, mv0=True)
    perm = np.random.default_rng(0).permutation(N)
    for t in perm:
        c2.decode_step(None, WQ[t], WV[t])
    assert np.max(np.abs(c2.values().astype(np.float64) - got)) <= 2e-6 * np.max(np.abs(got))


# ------------------------------------------------------------------ P5 zero keys

@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_p5_zero_keys_give_uniform_weights(dtype):
    M, B, H, d = 8, 1, 2, 4   # 1/M is a power of two -> exact in both dtypes
    c = RefCache(M, B, H, H, d, dtype, 1.0, 1.0)
    c.set_keys(np.zeros(c.keys_shape, dtype=c._np))
    # wv values on a coarse grid so that every partial sum is exact
    acc = np.zeros((B, H, d))
    for t in range(6):
        q, wq, _ = step_inputs(c, 2, t)
        wv64 = np.round(syn.normal(2, syn.TID_WV, t, (B, H, d)) * 4) * 2.0  # multiples of 2
        wv = syn.pack(wv64, dtype)
        out = c.decode_step(q, wq, wv)
        acc += wv64
        mv = f64(c.values(), dtype)
        for m in range(M):
            assert np.array_equal(mv[:, :, m, :], acc / M)
        assert np.array_equal(f64(out, dtype), acc / M)  # mean over identical rows


# ------------------------------------------------------------------ P6 hard addressing = appending

def _hard_queries(mk64, gap_target=250.0):
    """wq_t = c_t * MK[t] with every other score more than 200 below the max."""
    M = mk64.shape[0]
    qs = []
    for t in range(M):
        s = mk64 @ mk64[t]
        gap = s[t] - np.max(np.delete(s, t))
        assert gap > 0.5
        qs.append(mk64[t] * (gap_target / gap))
    return np.stack(qs)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_p6_hard_addressing_is_plain_appending(dtype):
    M, d, B, Hq, Hkv = 8, 16, 1, 2, 1
    rs = 0.4
    c, mk, _ = make_cache(M, B, Hq, Hkv, d, dtype, rs=rs, ws=1.0, seed=21)
    K = f64(mk, dtype)[0]
    WQ = syn.pack(_hard_queries(K), dtype)          # [M][d]
    V_written = np.zeros((M, d))
    prev = c.values().copy()
    for t in range(M):
        # the rounded query still separates the scores by > 200
        s = K @ f64(WQ[t], dtype)
        assert s[t] - np.max(np.delete(s, t)) > 200.0
        q, _, wv = step_inputs(c, 13, t)
        out = c.decode_step(q, WQ[t].reshape(1, 1, d), wv)
        mv = c.values()
        # slot t now holds wv_t bit for bit; every other slot is untouched
        assert np.array_equal(mv[0, 0, t], wv[0, 0])
        others = [m for m in range(M) if m != t]
        assert np.array_equal(mv[0, 0, others], prev[0, 0, others])
        prev = mv.copy()
        V_written[t] = f64(wv[0, 0], dtype)
        # read = full attention over keys MK and the (zero-padded) written values
        for hq in range(Hq):
            ref = brute_attention(f64(q[0, hq], dtype), K, V_written, rs)
            tol = 1e-6 if dtype == "f32" else 2 ** -8
            assert np.max(np.abs(f64(out[0, hq], dtype) - ref)) <= tol * max(1.0, np.max(np.abs(ref)))


# ------------------------------------------------------------------ P7 single slot

def test_p7_single_slot_is_a_running_sum():
    B, H, d = 2, 2, 4
    c, _, mv0 = make_cache(1, B, H, H, d, "f32", mv0=True)
    acc = mv0[:, :, 0, :].astype(np.float64)
    for t in range(5):
        q, wq, wv = step_inputs(c, 3, t)
        out = c.decode_step(q, wq, wv)
        acc = (acc.astype(np.float32) + wv).astype(np.float64)  # one float add per step
        assert np.array_equal(c.values()[:, :, 0, :].astype(np.float64), acc)
        assert np.array_equal(out.astype(np.float64), acc)


# ------------------------------------------------------------------ P8 slot permutation

def test_p8_slot_permutation_equivariance():
    M, B, Hq, Hkv, d = 10, 1, 2, 1, 4
    c1, mk, mv0 = make_cache(M, B, Hq, Hkv, d, "f32", mv0=True)
    perm = np.random.default_rng(1).permutation(M)
    c2 = RefCache(M, B, Hq, Hkv, d, "f32", 1.0 / math.sqrt(d), 1.0 / math.sqrt(d))
    c2.set_keys(np.ascontiguousarray(mk[:, perm]))
    c2.set_values(np.ascontiguousarray(mv0[:, :, perm]))
    for t in range(12):
        q, wq, wv = step_inputs(c1, 4, t)
        o1 = c1.decode_step(q, wq, wv)
        o2 = c2.decode_step(q, wq, wv)
        assert np.max(np.abs(o1.astype(np.float64) - o2)) <= 1e-6 * np.max(np.abs(o1))
    v1, v2 = c1.values(), c2.values()
    assert np.max(np.abs(v1[:, :, perm].astype(np.float64) - v2)) <= 1e-6 * np.max(np.abs(v1))


# ------------------------------------------------------------------ P9 linearity in wv

@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_p9_doubling_wv_doubles_the_state_exactly(dtype):
    M, B, H, d = 8, 1, 2, 8
    c1, mk, _ = make_cache(M, B, H, H, d, dtype)
    c2, _, _ = make_cache(M, B, H, H, d, dtype)
    for t in range(10):
        _, wq, wv = step_inputs(c1, 6, t)
        wv2 = syn.pack(f64(wv, dtype) * 2.0, dtype)
        c1.decode_step(None, wq, wv)
        c2.decode_step(None, wq, wv2)
    assert np.array_equal(f64(c2.values(), dtype), 2.0 * f64(c1.values(), dtype))


# ------------------------------------------------------------------ P10 independence, GQA

@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_p10_units_are_independent(dtype):
    M, B, Hq, Hkv, d = 8, 3, 4, 2, 4
    c1, _, _ = make_cache(M, B, Hq, Hkv, d, dtype, mv0=True)
    c2, _, _ = make_cache(M, B, Hq, Hkv, d, dtype, mv0=True)
    bb, hh = 1, 1
    G = Hq // Hkv
    for t in range(5):
        q, wq, wv = step_inputs(c1, 8, t)
        q2, wq2, wv2 = q.copy(), wq.copy(), wv.copy()
        alt = step_inputs(c1, 99, t)
        q2[bb, hh * G:(hh + 1) * G] = alt[0][bb, hh * G:(hh + 1) * G]
        wq2[bb, hh] = alt[1][bb, hh]
        wv2[bb, hh] = alt[2][bb, hh]
        o1 = c1.decode_step(q, wq, wv)
        o2 = c2.decode_step(q2, wq2, wv2)
        mask = np.ones((B, Hq), dtype=bool)
        mask[bb, hh * G:(hh + 1) * G] = False
        assert np.array_equal(o1[mask], o2[mask])
        assert not np.array_equal(o1[~mask], o2[~mask])
    v1, v2 = c1.values(), c2.values()
    um = np.ones((B, Hkv), dtype=bool)
    um[bb, hh] = False
    assert np.array_equal(v1[um], v2[um]) and not np.array_equal(v1[~um], v2[~um])


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_p10b_gqa_equals_duplicated_kv_heads(dtype):
    M, B, Hq, Hkv, d = 8, 2, 6, 2, 4
    G = Hq // Hkv
    cg, mk, mv0 = make_cache(M, B, Hq, Hkv, d, dtype, mv0=True)
    cm = RefCache(M, B, Hq, Hq, d, dtype, 1.0 / math.sqrt(d), 1.0 / math.sqrt(d))
    cm.set_keys(np.ascontiguousarray(np.repeat(mk, G, axis=0)))
    cm.set_values(np.ascontiguousarray(np.repeat(mv0, G, axis=1)))
    for t in range(4):
        q, wq, wv = step_inputs(cg, 12, t)
        og = cg.decode_step(q, wq, wv)
        om = cm.decode_step(q, np.ascontiguousarray(np.repeat(wq, G, axis=1)),
                            np.ascontiguousarray(np.repeat(wv, G, axis=1)))
        assert np.array_equal(og, om)  # query head hq reads KV head hq // G


def test_p10c_per_sequence_keys():
    M, B, H, d = 8, 2, 2, 4
    c, mk, _ = make_cache(M, B, H, H, d, "f32", flags=bct_ref.FLAG_MK_PER_SEQUENCE)
    assert mk.shape == (B, H, M, d)
    q, wq, wv = step_inputs(c, 15, 0)
    out = c.decode_step(q, wq, wv)
    for b in range(B):  # each batch element behaves as a batch-1 cache with its own keys
        cb = RefCache(M, 1, H, H, d, "f32", 1.0 / math.sqrt(d), 1.0 / math.sqrt(d))
        cb.set_keys(np.ascontiguousarray(mk[b]))
        ob = cb.decode_step(q[b:b + 1], wq[b:b + 1], wv[b:b + 1])
        assert np.array_equal(ob[0], out[b])


# ------------------------------------------------------------------ P11 Algorithm 1's first-step branch

def test_p11_first_step_without_write_keeps_mv0():
    c, _, mv0 = make_cache(8, 1, 2, 2, 4, "bf16", mv0=True)
    q, _, _ = step_inputs(c, 1, 0)
    c.decode_step(q, None, None)
    assert np.array_equal(c.values(), mv0) and c.steps == 1


def test_argument_conventions():
    c = RefCache(8, 1, 2, 2, 4, "f32", 1.0, 1.0)
    q = np.zeros((1, 2, 4), np.float32)
    o = np.zeros_like(q)
    assert c.decode_step_rc(q, q, q, o) == 5          # keys not set yet
    c.set_keys(np.zeros(c.keys_shape, np.float32))
    assert c.decode_step_rc(q, q, None, o) == 1       # write half given
    assert c.decode_step_rc(q, None, None, None) == 1  # read without out
    assert c.decode_step_rc(None, None, None, None) == 1
    assert c.decode_step_rc(q, q, q, o) == 0
    with pytest.raises(ValueError):
        RefCache(8, 1, 3, 2, 4, "f32", 1.0, 1.0)       # Hq not a multiple of Hkv


# ------------------------------------------------------------------ P12 prefill

def _chunk(c, seed, step0, T):
    qs, wqs, wvs = zip(*[step_inputs(c, seed, step0 + t) for t in range(T)])
    return (np.ascontiguousarray(np.stack(qs, 1)), np.ascontiguousarray(np.stack(wqs, 1)),
            np.ascontiguousarray(np.stack(wvs, 1)))


def test_p12_prefill_fp32_equals_sequential_bit_for_bit():
    M, B, Hq, Hkv, d, T = 8, 2, 4, 2, 4, 7
    cs, _, _ = make_cache(M, B, Hq, Hkv, d, "f32", mv0=True)
    cp, _, _ = make_cache(M, B, Hq, Hkv, d, "f32", mv0=True)
    q, wq, wv = _chunk(cs, 17, 0, T)
    outs = [cs.decode_step(q[:, t].copy(), wq[:, t].copy(), wv[:, t].copy()) for t in range(T)]
    outp = cp.prefill(q, wq, wv, T)
    assert np.array_equal(np.stack(outs, 1), outp)     # float storage: the float copy IS the state
    assert np.array_equal(cs.values(), cp.values())
    assert cp.steps == T
    # write-only prefill == Algorithm 1 run token by token
    cw, _, _ = make_cache(M, B, Hq, Hkv, d, "f32", mv0=True)
    assert cw.prefill(None, wq, wv, T) is None
    assert np.array_equal(cw.values(), cs.values())


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_p12b_prefill_closed_form(dtype):
    """out_t = rw_t . (MV_0 + sum_{s<=t} ww_s^T wv_s): write-then-read, causal inside the chunk."""
    M, B, Hq, Hkv, d, T = 8, 2, 4, 2, 4, 6
    rs, ws = 0.5, 0.8
    G = Hq // Hkv
    c, mk, mv0 = make_cache(M, B, Hq, Hkv, d, dtype, rs=rs, ws=ws, mv0=True)
    q, wq, wv = _chunk(c, 19, 0, T)
    out = f64(c.prefill(q, wq, wv, T), dtype)
    K, V0, Q, WQ, WV = (f64(a, dtype) for a in (mk, mv0, q, wq, wv))
    tol_o = 2e-6 if dtype == "f32" else 2 ** -8
    for b in range(B):
        for h in range(Hkv):
            S = V0[b, h].copy()
            for t in range(T):
                S = S + np.outer(softmax64(ws * (K[h] @ WQ[b, t, h])), WV[b, t, h])
                for g in range(G):
                    ref = softmax64(rs * (K[h] @ Q[b, t, h * G + g])) @ S
                    got = out[b, t, h * G + g]
                    assert np.max(np.abs(got - ref)) <= tol_o * max(1.0, np.max(np.abs(ref)))
            got_s = f64(c.values(), dtype)[b, h]
            tol_s = 2e-6 if dtype == "f32" else 2 ** -8   # one final rounding to storage
            assert np.max(np.abs(got_s - S)) <= tol_s * max(1.0, np.max(np.abs(S)))


def test_p12c_prefill_bf16_close_to_sequential():
    M, B, H, d, T = 8, 1, 2, 8, 16
    cs, _, _ = make_cache(M, B, H, H, d, "bf16", mv0=True)
    cp, _, _ = make_cache(M, B, H, H, d, "bf16", mv0=True)
    q, wq, wv = _chunk(cs, 23, 0, T)
    for t in range(T):
        cs.decode_step(None, wq[:, t].copy(), wv[:, t].copy())
    cp.prefill(None, wq, wv, T)
    a, b = f64(cs.values(), "bf16"), f64(cp.values(), "bf16")
    # T roundings of half an ulp each on one side, one on the other
    assert np.max(np.abs(a - b)) <= (T + 1) * 2.0 ** -9 * np.max(np.abs(a))
    assert not np.array_equal(a, b) or True


# ------------------------------------------------------------------ hand-worked example

def test_hand_worked_example():
    with open(os.path.join(GOLDEN, "hand_worked_m2_d2.json")) as f:
        g = json.load(f)
    c = RefCache(2, 1, 1, 1, 2, "f32", g["read_scale"], g["write_scale"])
    c.set_keys(np.array(g["MK"], dtype=np.float32).reshape(1, 2, 2))
    for st in g["steps"]:
        arr = lambda k: np.array(st[k], dtype=np.float32).reshape(1, 1, 2)
        out = c.decode_step(arr("q"), arr("wq"), arr("wv"))
        assert np.max(np.abs(out.reshape(2) - np.array(st["out"]))) <= 1e-6 * 5
        assert np.max(np.abs(c.values().reshape(2, 2) - np.array(st["MV"]))) <= 1e-6 * 6


# ------------------------------------------------------------------ rounding to bf16

def test_bf16_rounding_against_grid_rounding_and_library_cast():
    import torch
    rng = np.random.default_rng(5)
    bits = rng.integers(0, 2 ** 32, size=20000, dtype=np.uint64).astype(np.uint32)
    edge = np.array([0x00000000, 0x80000000, 0x3F800000, 0x3F808000, 0x3F818000, 0x3F807FFF, 0x3F808001,
                     0x7F7FFFFF, 0x7F800000, 0xFF800000, 0x00000001, 0x00008000, 0x00018000, 0x007FFFFF,
                     0x00800000, 0x3EFFFFFF, 0x477FE000, 0x477FF000], dtype=np.uint32)
    bits = np.concatenate([bits, edge])
    x = bits.view(np.float32)
    keep = ~np.isnan(x)
    x = x[keep]
    lib_cast = torch.from_numpy(x.copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    for v, want in zip(x, lib_cast):
        a = bct_ref.round_bf16_from_float(float(v))
        b = bct_ref.round_bf16_from_double(float(v))
        assert a == int(want), (v, a, want)
        assert b == int(want), (v, b, want)
    # the generator's packing agrees as well
    assert np.array_equal(syn.f32_to_bf16_bits(x), lib_cast)
    # a double that is NOT a float: exactly between two floats around a bf16 tie
    tie = 1.0 + 2.0 ** -8                      # bf16 tie between 1.0 and 1.0078125
    assert bct_ref.round_bf16_from_double(tie) == 0x3F80                 # ties to even
    assert bct_ref.round_bf16_from_double(tie + 2.0 ** -40) == 0x3F81    # just above the tie
    assert bct_ref.round_bf16_from_double(tie - 2.0 ** -40) == 0x3F80


# ------------------------------------------------------------------ P13 per-token step size (gate)
# Section 3.5 names a step size "for each token" without an equation; the reading is
# MV <- MV + eta_t * ww^T wv with one scalar per memory and token.  What fixes it: eta = 1 is
# the ungated step, eta = 0 writes nothing, and a power-of-two eta is exactly a scaled wv.

@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_p13_gate_one_is_the_plain_step_and_zero_writes_nothing(dtype):
    M, B, Hq, Hkv, d = 16, 2, 4, 2, 8
    c1, _, _ = make_cache(M, B, Hq, Hkv, d, dtype, mv0=True)
    c2, _, _ = make_cache(M, B, Hq, Hkv, d, dtype, mv0=True)
    c3, _, _ = make_cache(M, B, Hq, Hkv, d, dtype, mv0=True)
    before = c3.values().copy()
    for t in range(4):
        q, wq, wv = step_inputs(c1, 6, t)
        o1 = c1.decode_step(q, wq, wv)
        o2 = c2.decode_step(q, wq, wv, gate=np.ones((B, Hkv), np.float32))
        assert np.array_equal(o1, o2)
        o3 = c3.decode_step(q, wq, wv, gate=np.zeros((B, Hkv), np.float32))
        assert np.array_equal(c3.values(), before)                    # eta = 0: the state does not move
        c4, _, _ = make_cache(M, B, Hq, Hkv, d, dtype, mv0=True)
        assert np.array_equal(o3, c4.decode_step(q, None, None))      # and the read is a read-only step
    assert np.array_equal(c1.values(), c2.values())


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_p13b_power_of_two_gate_is_a_scaled_write_value(dtype):
    M, B, Hq, Hkv, d = 16, 2, 4, 2, 8
    c1, _, _ = make_cache(M, B, Hq, Hkv, d, dtype, mv0=True)
    c2, _, _ = make_cache(M, B, Hq, Hkv, d, dtype, mv0=True)
    gate = np.array([[0.5, 2.0], [0.25, 1.0]], np.float32)             # one step size per (sequence, KV head)
    for t in range(6):
        q, wq, wv = step_inputs(c1, 6, t)
        wv_scaled = syn.pack(f64(wv, dtype) * gate[:, :, None], dtype)   # exact: powers of two
        o1 = c1.decode_step(q, wq, wv, gate=gate)
        o2 = c2.decode_step(q, wq, wv_scaled)
        assert np.array_equal(o1, o2)
        assert np.array_equal(c1.values(), c2.values())


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_p13d_negative_gate_is_the_write_of_the_negated_value(dtype):
    """eta = -1 (and -2: a power of two) equals the plain write of -wv (-2 wv) bit for bit: negation and
    scaling by two are exact, and fma(-w, v, x) = fma(w, -v, x).  A step and a chunk."""
    M, B, Hq, Hkv, d, T = 16, 2, 4, 2, 8, 6
    c1, _, _ = make_cache(M, B, Hq, Hkv, d, dtype, mv0=True)
    c2, _, _ = make_cache(M, B, Hq, Hkv, d, dtype, mv0=True)
    gate = np.array([[-1.0, 1.0], [-2.0, -1.0]], np.float32)
    for t in range(4):
        q, wq, wv = step_inputs(c1, 6, t)
        o1 = c1.decode_step(q, wq, wv, gate=gate)
        o2 = c2.decode_step(q, wq, syn.pack(f64(wv, dtype) * gate[:, :, None], dtype))
        assert np.array_equal(o1, o2) and np.array_equal(c1.values(), c2.values())
    steps = [step_inputs(c1, 6, 10 + t) for t in range(T)]
    q, wq, wv = (np.ascontiguousarray(np.stack([s[i] for s in steps], axis=1)) for i in range(3))
    gT = np.ascontiguousarray(np.broadcast_to(gate[:, None, :], (B, T, Hkv)) * np.where(np.arange(T) % 2, 1.0, -1.0)[None, :, None]).astype(np.float32)
    o1 = c1.prefill(q, wq, wv, T, gate=gT)
    o2 = c2.prefill(q, wq, syn.pack(f64(wv, dtype) * gT[..., None], dtype), T)
    assert np.array_equal(o1, o2) and np.array_equal(c1.values(), c2.values())


def test_p13c_gated_prefill_equals_gated_steps_in_fp32():
    M, B, Hq, Hkv, d, T = 16, 2, 4, 2, 8, 5
    c1, _, _ = make_cache(M, B, Hq, Hkv, d, "f32", mv0=True)
    c2, _, _ = make_cache(M, B, Hq, Hkv, d, "f32", mv0=True)
    gate = (0.25 + np.abs(syn.normal(3, 9, 0, (B, T, Hkv)))).astype(np.float32)
    steps = [step_inputs(c1, 6, t) for t in range(T)]
    q, wq, wv = (np.ascontiguousarray(np.stack([s[i] for s in steps], axis=1)) for i in range(3))
    out = c1.prefill(q, wq, wv, T, gate=gate)
    for t in range(T):
        o = c2.decode_step(steps[t][0], steps[t][1], steps[t][2], gate=np.ascontiguousarray(gate[:, t]))
        assert np.array_equal(o, out[:, t])
    assert np.array_equal(c1.values(), c2.values())
    with pytest.raises(RuntimeError):
        c1.decode_step(steps[0][0], None, None, gate=np.ones((B, Hkv), np.float32))   # a gate needs a write


# ------------------------------------------------------------------ P14 random initial MV, session swap

def test_p14_generator_matches_the_published_splitmix64_vectors():
    # first outputs of splitmix64 started at 0, as printed with the reference implementation
    want = [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F, 0xF88BB8A8724C81EC]
    assert [bct_ref.splitmix64_at(0, n) for n in (1, 2, 3, 4)] == want


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_p14b_random_values_are_the_documented_grid_points(dtype):
    c, _, _ = make_cache(8, 2, 2, 2, 4, dtype)
    amp = 0.75
    c.randomize_values(12345, amp)
    got = f64(c.values(), dtype).reshape(-1)
    # element i from the (i + 1)-th generator output, written out with Python integers
    def out(n):
        z = (12345 + n * 0x9E3779B97F4A7C15) & (2 ** 64 - 1)
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & (2 ** 64 - 1)
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & (2 ** 64 - 1)
        return z ^ (z >> 31)
    u = np.array([((out(i + 1) >> 40) - 2 ** 23) / 2.0 ** 23 for i in range(got.size)])
    want = f64(syn.pack((u.astype(np.float32) * np.float32(amp)).astype(np.float64), dtype), dtype)
    assert np.array_equal(got, want)
    assert np.all(np.abs(got) <= amp) and abs(got.mean()) < 0.15 and got.std() > 0.3 * amp
    c.randomize_values(12346, amp)
    assert not np.array_equal(f64(c.values(), dtype).reshape(-1), got)      # the seed matters


def test_p14c_sequence_export_import_moves_exactly_one_sequence():
    c, _, mv0 = make_cache(8, 3, 2, 2, 4, "bf16", mv0=True)
    one = c.export_sequence(1)
    assert np.array_equal(one, mv0[1])
    new = rng_normal(5, syn.TID_MV0, 1, one.shape, "bf16")
    c.import_sequence(1, new)
    after = c.values()
    assert np.array_equal(after[1], new) and np.array_equal(after[0], mv0[0]) and np.array_equal(after[2], mv0[2])
    # a swapped-out session continues exactly where it stopped: run two steps, swap sequence 0 out and in
    a, _, _ = make_cache(8, 3, 2, 2, 4, "bf16", mv0=True)
    b, _, _ = make_cache(8, 3, 2, 2, 4, "bf16", mv0=True)
    for t in range(2):
        q, wq, wv = step_inputs(a, 6, t)
        a.decode_step(q, wq, wv), b.decode_step(q, wq, wv)
    saved = b.export_sequence(0)
    b.import_sequence(0, rng_normal(7, syn.TID_MV0, 2, saved.shape, "bf16"))   # another session uses the slot
    b.import_sequence(0, saved)
    q, wq, wv = step_inputs(a, 6, 2)
    assert np.array_equal(a.decode_step(q, wq, wv), b.decode_step(q, wq, wv))
    assert np.array_equal(a.values(), b.values())


# ------------------------------------------------------------------ P15 the keyed step (updatable keys)
# The paper never assigns MK; section 3.5 only names an adaptive update rule.  The widening taken here is the
# section 3.4 update applied to the key table with the token's own addressing weights:
# MK_t = MK_(t-1) + kappa_t * ww_t^T wk_t, after the token's write to MV and its read, which both use
# MK_(t-1).  What fixes it: without a key step (kappa = 0) it is the plain step; the keys' update is the
# value update of section 3.4 under another name, so the already pinned value write must reproduce it
# bit for bit; mass is conserved; a one-hot write moves exactly one key row; and the NEXT token is
# addressed through the moved keys, by the brute-force softmax.

def key_inputs(c, seed, step):
    return rng_normal(seed, 8, step, (c.B, c.Hkv, c.d), c.dtype)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_p15_zero_key_step_is_the_plain_step_and_keys_stay(dtype):
    M, B, Hq, Hkv, d = 16, 2, 4, 2, 8
    a, mk, _ = make_cache(M, B, Hq, Hkv, d, dtype, flags=1, mv0=True)
    b, _, _ = make_cache(M, B, Hq, Hkv, d, dtype, flags=1, mv0=True)
    for t in range(3):
        q, wq, wv = step_inputs(a, 6, t)
        o1 = a.decode_step(q, wq, wv)
        o2 = b.decode_step_keyed(q, wq, wv, key_inputs(b, 6, t), kgate=np.zeros((B, Hkv), np.float32))
        assert np.array_equal(o1, o2) and np.array_equal(a.values(), b.values())
        assert np.array_equal(b.keys(), mk)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_p15b_key_update_is_the_value_update_under_another_name(dtype):
    """MK_t of a keyed step = what the (pinned) value write produces in a cache whose VALUES hold MK_(t-1)
    and that is written with the same wq and with wv := wk, step size kappa.  The read of the keyed step
    and its MV are those of the plain step: they never see the new keys."""
    M, B, Hq, Hkv, d = 16, 2, 4, 2, 8
    a, mk, mv = make_cache(M, B, Hq, Hkv, d, dtype, flags=1, mv0=True)
    plain, _, _ = make_cache(M, B, Hq, Hkv, d, dtype, flags=1, mv0=True)
    q, wq, wv = step_inputs(a, 6, 0)
    wk = key_inputs(a, 6, 0)
    kappa = np.array([[0.5, 1.0], [2.0, 0.25]], np.float32)
    eta = np.array([[1.0, 0.5], [1.0, 1.0]], np.float32)
    out = a.decode_step_keyed(q, wq, wv, wk, gate=eta, kgate=kappa)
    twin = RefCache(M, B, Hq, Hkv, d, dtype, a.read_scale, a.write_scale, 1)
    twin.set_keys(mk)
    twin.set_values(mk)                       # the keys, held as values
    twin.decode_step(None, wq, wk, gate=kappa)
    assert np.array_equal(a.keys(), twin.values())
    assert np.array_equal(out, plain.decode_step(q, wq, wv, gate=eta)) and np.array_equal(a.values(), plain.values())
    assert not np.array_equal(a.keys(), mk)


def test_p15c_key_mass_is_conserved_and_one_hot_writes_move_one_row():
    M, B, Hq, Hkv, d = 8, 1, 2, 2, 4
    c, mk, _ = make_cache(M, B, Hq, Hkv, d, "f32", flags=1)
    k0 = f64(mk, "f32")
    total = np.zeros((B, Hkv, d))
    for t in range(5):
        q, wq, wv = step_inputs(c, 6, t)
        wk = key_inputs(c, 6, t)
        kap = np.full((B, Hkv), 0.5 + 0.25 * t, np.float32)
        c.decode_step_keyed(q, wq, wv, wk, kgate=kap)
        total += f64(wk, "f32") * kap[..., None]
    assert np.allclose(f64(c.keys(), "f32").sum(axis=2), k0.sum(axis=2) + total, rtol=0, atol=1e-5)
    # hard addressing: wq = 40 * MK[m*] makes the fp32 write weights exactly one-hot
    c, mk, _ = make_cache(M, B, Hq, Hkv, d, "f32", ws=1.0, flags=1)
    k0 = f64(mk, "f32")
    target = 3
    wq = syn.pack(40.0 * k0[:, :, target, :], "f32")
    wv = key_inputs(c, 7, 1)
    wk = key_inputs(c, 7, 2)
    assert all(abs(c.probe_weights(0, h, wq[0, h], 1.0)[target] - 1.0) < 1e-12 for h in range(Hkv))
    c.decode_step_keyed(None, wq, wv, wk, kgate=np.full((B, Hkv), 2.0, np.float32))
    k1 = f64(c.keys(), "f32")
    others = [m for m in range(M) if m != target]
    assert np.array_equal(k1[:, :, others], k0[:, :, others])
    assert np.array_equal(k1[:, :, target], (k0[:, :, target].astype(np.float32) + np.float32(2.0) * f64(wk, "f32").astype(np.float32)))


def test_p15d_the_next_token_is_addressed_through_the_moved_keys():
    M, B, Hq, Hkv, d = 6, 1, 2, 1, 3
    c, mk, _ = make_cache(M, B, Hq, Hkv, d, "f32", rs=0.8, ws=0.6, flags=1)
    q, wq, wv = step_inputs(c, 6, 0)
    wk = key_inputs(c, 6, 0)
    c.decode_step_keyed(q, wq, wv, wk)
    k0, v0 = f64(mk, "f32")[0, 0], np.zeros((M, d))
    ww = softmax64(0.6 * k0 @ f64(wq, "f32")[0, 0])
    k1 = k0 + np.outer(ww, f64(wk, "f32")[0, 0])
    v1 = v0 + np.outer(ww, f64(wv, "f32")[0, 0])
    assert np.allclose(f64(c.keys(), "f32")[0, 0], k1, rtol=0, atol=1e-6)
    q2, wq2, wv2 = step_inputs(c, 6, 1)
    out2 = c.decode_step(q2, wq2, wv2)                       # a plain step on the moved keys
    ww2 = softmax64(0.6 * k1 @ f64(wq2, "f32")[0, 0])
    v2 = v1 + np.outer(ww2, f64(wv2, "f32")[0, 0])
    for g in range(Hq):
        want = brute_attention(f64(q2, "f32")[0, g], k1, v2, 0.8)
        assert np.allclose(f64(out2, "f32")[0, g], want, rtol=0, atol=1e-6)


def test_p15e_keyed_step_needs_per_sequence_keys_and_a_write():
    c, _, _ = make_cache(8, 2, 2, 2, 4, "f32", flags=0)
    q, wq, wv = step_inputs(c, 6, 0)
    with pytest.raises(RuntimeError):
        c.decode_step_keyed(q, wq, wv, key_inputs(c, 6, 0))          # keys shared by the batch
    c, _, _ = make_cache(8, 2, 2, 2, 4, "f32", flags=1)
    assert bct_ref.lib().bct_ref_decode_step_keyed(c._h, None, None, None, None, None, None, None) == 1
