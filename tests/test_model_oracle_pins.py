"""Pins of oracle/model_ref (the glue of the decoder stack) to things other than itself:
closed forms, brute force, invariants, and torch's own bf16 conversion."""
import math
from types import SimpleNamespace

import numpy as np
import pytest
import torch

import bct_synth as syn
from oracle import model_ref as R


def bits(x):
    """float values that bf16 holds exactly -> uint16 bits (checked)."""
    x = np.asarray(x, dtype=np.float32)
    b = (x.view(np.uint32) >> 16).astype(np.uint16)
    assert np.all((x.view(np.uint32) & 0xFFFF) == 0), "test value is not a bf16 number"
    return b


# ---------------------------------------------------------------- rounding

def test_rounding_matches_torch_on_fp32_inputs():
    rng = np.random.default_rng(5)
    x = np.concatenate([rng.standard_normal(20000).astype(np.float32) * 10.0 ** rng.integers(-30, 30, 20000),
                        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895314e38, 3.4e38, 1e-40, 9.2e-41, -1e-45],
                                 dtype=np.float32)]).astype(np.float32)
    want = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(R.f64_to_bf16(x.astype(np.float64)), want)


def test_rounding_is_direct_not_via_fp32():
    # 1 + 2^-8 + 2^-30 lies above the midpoint of 1 and 1 + 2^-7: rounds up.  Through fp32 it would first
    # become the midpoint itself and then fall to the even neighbour 1.0.
    x = np.array([1.0 + 2.0 ** -8 + 2.0 ** -30, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8])
    got = R.bf16_to_f64(R.f64_to_bf16(x))
    assert got.tolist() == [1.0 + 2.0 ** -7, 1.0, 1.0 + 2.0 ** -6]


# ---------------------------------------------------------------- elementary operations

def test_embed_rows_and_out_of_range():
    table = bits(np.arange(12, dtype=np.float32).reshape(4, 3))
    out = R.embed(np.array([2, 0, 7, -1, 3]), table)
    assert R.bf16_to_f64(out).tolist() == [[6, 7, 8], [0, 1, 2], [0, 0, 0], [0, 0, 0], [9, 10, 11]]


def test_rmsnorm_closed_forms():
    # a 3-4-0-0 row has mean square 25/4; with eps = 0 the result is x / 2.5 * gain
    x = bits([[3.0, 4.0, 0.0, 0.0], [-8.0, -8.0, -8.0, -8.0]])
    g = bits([1.0, 0.5, 2.0, 1.0])
    out = R.bf16_to_f64(R.rmsnorm(x, g, 0.0))
    want0 = R.bf16_to_f64(R.f64_to_bf16(np.array([1.2, 0.8, 0.0, 0.0])))
    assert out[0].tolist() == want0.tolist()
    assert out[1].tolist() == [-1.0, -0.5, -2.0, -1.0]      # constant row: sign(c) * gain
    # eps enters under the root: constant row c -> gain / sqrt(1 + eps / c^2)
    out = R.bf16_to_f64(R.rmsnorm(bits([[0.5] * 8]), bits([1.0] * 8), 0.75))
    assert out[0].tolist() == [0.5] * 8                     # 0.5 / sqrt(0.25 + 0.75)


def test_rmsnorm_scale_invariance_and_unit_rms():
    x = syn.pack(syn.normal(3, 9, 0, (7, 256)), "bf16")
    g = bits([1.0] * 256)
    a = R.rmsnorm(x, g, 0.0)
    x4 = syn.pack(4.0 * syn.unpack(x, "bf16"), "bf16")      # exact scaling by a power of two
    assert np.array_equal(a, R.rmsnorm(x4, g, 0.0))
    rms = np.sqrt(np.mean(R.bf16_to_f64(a) ** 2, axis=1))
    assert np.all(np.abs(rms - 1.0) < 2e-3)


def test_linear_brute_force_and_orientation():
    rows, K, N = 3, 5, 4
    x = syn.pack(syn.normal(1, 9, 1, (rows, K)), "bf16")
    w = syn.pack(syn.normal(1, 9, 2, (N, K)), "bf16")
    res = syn.pack(syn.normal(1, 9, 3, (rows, N)), "bf16")
    xf, wf, rf = (syn.unpack(a, "bf16") for a in (x, w, res))
    want = np.zeros((rows, N))
    for r in range(rows):
        for n in range(N):
            want[r, n] = math.fsum(xf[r, k] * wf[n, k] for k in range(K)) + rf[r, n]
    got = R.bf16_to_f64(R.linear(x, w, res))
    assert np.all(np.abs(got - want) <= 2.0 ** -8 * np.abs(want) + 1e-30)
    # row n of w selects input feature sel[n]: a transposed weight would fail (w is not square)
    sel = [4, 0, 2]
    w1 = np.zeros((3, K), dtype=np.float32)
    w1[np.arange(3), sel] = 1.0
    assert np.array_equal(R.linear(x, bits(w1)), x[:, sel])
    # no residual means zero, and an identity weight plus residual is x + residual, rounded once
    eye = bits(np.eye(K, dtype=np.float32))
    r5 = syn.pack(syn.normal(1, 9, 4, (rows, K)), "bf16")
    assert np.array_equal(R.linear(x, eye, r5), R.f64_to_bf16(xf + syn.unpack(r5, "bf16")))


def test_swiglu_known_values():
    # one input feature x = 1: gate pre-activation = w_gate, up = w_up
    x = bits([[1.0]])
    for g, u, want in [(0.0, 3.0, 0.0), (1.0, 1.0, 0.7310585786300049), (-1.0, 2.0, -2 * 0.2689414213699951),
                       (40.0, 0.5, 20.0), (-40.0, 1.0, -40.0 * math.exp(-40.0))]:
        out = R.bf16_to_f64(R.swiglu(x, bits([[g]]), bits([[u]])))[0, 0]
        assert out == R.bf16_to_f64(R.f64_to_bf16(np.array([want])))[0], (g, u)
    # gate and up are not interchangeable
    a = R.swiglu(x, bits([[2.0]]), bits([[-1.0]]))
    b = R.swiglu(x, bits([[-1.0]]), bits([[2.0]]))
    assert not np.array_equal(a, b)


def test_argmax_lowest_index_on_ties():
    lg = bits([[1.0, 5.0, 5.0, -2.0], [-3.0, -1.0, -1.0, -7.0], [0.0, -0.0, 0.0, 0.0], [-4.0, -4.0, -4.0, 2.0]])
    assert R.argmax(lg).tolist() == [1, 1, 0, 3]


# ---------------------------------------------------------------- the stack

def small_shape(**kw):
    d = dict(n_layers=2, dim=64, n_q_heads=4, n_kv_heads=2, head_dim=32, ffn=96, vocab=40, capacity_M=64,
             batch=2, eps=1e-5)
    d.update(kw)
    s = SimpleNamespace(**d)
    s.q_width, s.kv_width = s.n_q_heads * s.head_dim, s.n_kv_heads * s.head_dim
    s.weight_shapes = lambda: {"attn_norm": (s.dim,), "w_q": (s.q_width, s.dim), "w_wq": (s.kv_width, s.dim),
                               "w_wv": (s.kv_width, s.dim), "w_o": (s.dim, s.q_width), "mlp_norm": (s.dim,),
                               "w_gate": (s.ffn, s.dim), "w_up": (s.ffn, s.dim), "w_down": (s.dim, s.ffn)}
    return s


def test_stack_with_silent_branches_is_embedding_through_the_head():
    # zero W_o and W_down: both branches add nothing, so the logits are head(rmsnorm(embedding))
    s = small_shape()
    w = syn.make_stack_weights(s, seed=1)
    for lw in w["layers"]:
        lw["w_o"][:] = 0
        lw["w_down"][:] = 0
    ids = syn.make_token_ids(1, 0, s.batch, s.vocab)
    nxt, logits = R.RefStack(s, w).forward(ids)
    e = syn.unpack(w["embed"], "bf16")[ids]
    h = e / np.sqrt(np.mean(e * e, axis=1, keepdims=True) + float(np.float32(s.eps))) * syn.unpack(w["final_norm"], "bf16")
    h = syn.unpack(syn.pack(h, "bf16"), "bf16")
    want = h @ syn.unpack(w["head"], "bf16").T
    got = syn.unpack(logits, "bf16")
    assert np.all(np.abs(got - want) <= 2.0 ** -8 * np.abs(want) + 1e-6)
    assert nxt.tolist() == np.argmax(got, axis=1).tolist()


def test_stack_attention_branch_reaches_the_residual_stream():
    # with W_down = 0 only attention moves the stream; the first token reads a memory that holds
    # only its own write, MV = ww (outer) wv, so out_h = (sum_m rw_m ww_m) * wv: a multiple of wv per head
    s = small_shape(n_layers=1, n_q_heads=2, n_kv_heads=2)
    w = syn.make_stack_weights(s, seed=2)
    w["layers"][0]["w_down"][:] = 0
    w["layers"][0]["w_o"] = bits(16.0 * np.eye(s.dim, dtype=np.float32))    # dim = q_width: stream += 16 * out
    ids = syn.make_token_ids(2, 0, s.batch, s.vocab)
    trace = []
    st = R.RefStack(s, w)
    st.forward(ids, trace=trace)
    lw = w["layers"][0]
    x0 = R.embed(ids, w["embed"])
    h = R.rmsnorm(x0, lw["attn_norm"], s.eps)
    wv = syn.unpack(R.linear(h, lw["w_wv"]), "bf16").reshape(s.batch, s.n_kv_heads, s.head_dim)
    delta = syn.unpack(trace[0], "bf16") - syn.unpack(x0, "bf16")
    a = (delta / 16.0).reshape(s.batch, s.n_q_heads, s.head_dim)
    for b in range(s.batch):
        for hh in range(s.n_q_heads):
            c = np.dot(a[b, hh], wv[b, hh]) / np.dot(wv[b, hh], wv[b, hh])
            assert 0.0 < c <= 1.0 + 1e-2                      # sum_m rw_m ww_m lies in (0, 1]
            assert np.linalg.norm(a[b, hh] - c * wv[b, hh]) <= 0.08 * np.linalg.norm(a[b, hh])


def test_stack_chunk_equals_token_by_token():
    # a chunk of T tokens per sequence gives the logits of T decode steps (row b*T + t <-> step t, sequence b)
    s = small_shape()
    w = syn.make_stack_weights(s, seed=3)
    T = 3
    ids = syn.make_token_ids(3, 0, s.batch * T, s.vocab).reshape(s.batch, T)
    one = R.RefStack(s, w)
    steps = [one.forward(np.ascontiguousarray(ids[:, t]))[1] for t in range(T)]
    chunk = R.RefStack(s, w).forward(np.ascontiguousarray(ids.reshape(-1)), T=T)[1].reshape(s.batch, T, -1)
    for t in range(T):
        a, b = syn.unpack(chunk[:, t], "bf16"), syn.unpack(steps[t], "bf16")
        assert np.max(np.abs(a - b)) <= 0.02 * np.max(np.abs(b))
