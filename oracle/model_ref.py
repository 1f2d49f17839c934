"""CPU oracle of the Llama-shaped glue around the bounded-cache layer: embedding,
RMS normalisation, dense projections, SwiGLU, greedy arg-max, and the stack that
chains them with oracle/bct_ref's cache (section 3.2 step 1 and Algorithm 1 give
the write projections wq = W_wq x, wv = W_wv x; the rest is the standard
pre-norm decoder block the paper's models are built from).

Test infrastructure only: imported by tests/, by the smoke check and by the
cpu_baseline leg of bench.py.  Every operation is its definition in fp64 with
one round-to-nearest-even to bf16 at the end, because the tensors between the
operations are stored as bf16.  bf16 tensors travel as uint16 bit patterns.
"""
from __future__ import annotations

import numpy as np

from . import bct_ref


def bf16_to_f64(bits: np.ndarray) -> np.ndarray:
    return (np.asarray(bits, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def f64_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even from fp64 straight to bf16 (8 significant bits, exponent range of fp32,
    gradual underflow); no intermediate fp32 rounding."""
    x = np.asarray(x, dtype=np.float64)
    a = np.abs(x)
    with np.errstate(divide="ignore"):
        e = np.floor(np.log2(np.where(a > 0, a, 1.0)))
    # log2 can be off by one at powers of two: correct with exact comparisons
    e = np.where(np.ldexp(1.0, e.astype(np.int64)) > a, e - 1, e)
    e = np.where(np.ldexp(1.0, (e + 1).astype(np.int64)) <= a, e + 1, e)
    e = np.maximum(e, -126.0)                        # subnormals share the smallest normal's spacing
    ulp = np.ldexp(1.0, (e - 7).astype(np.int64))
    r = np.rint(a / ulp) * ulp                       # rint rounds halves to even; a / ulp is exact
    r = np.where(r >= np.ldexp(1.0, 128), np.inf, r)
    r = np.copysign(r, x)
    return (r.astype(np.float32).view(np.uint32) >> 16).astype(np.uint16)


def embed(ids, table):
    """out[r] = table[ids[r]]; ids outside the table give a zero row."""
    ids = np.asarray(ids, dtype=np.int64)
    table = np.asarray(table, dtype=np.uint16)
    out = np.zeros((ids.size, table.shape[1]), dtype=np.uint16)
    ok = (ids >= 0) & (ids < table.shape[0])
    out[ok] = table[ids[ok]]
    return out


def rmsnorm(x, gain, eps):
    """out = x / sqrt(mean(x^2) + eps) * gain, row by row."""
    xf, g = bf16_to_f64(x), bf16_to_f64(gain)
    ms = np.mean(xf * xf, axis=1, keepdims=True)
    return f64_to_bf16(xf / np.sqrt(ms + float(np.float32(eps))) * g[None, :])


def linear_f64(x, w):
    return bf16_to_f64(x) @ bf16_to_f64(w).T


def linear(x, w, residual=None):
    """out[r][n] = sum_k x[r][k] w[n][k] (+ residual[r][n])."""
    y = linear_f64(x, w)
    if residual is not None:
        y = y + bf16_to_f64(residual)
    return f64_to_bf16(y)


def swiglu(x, w_gate, w_up):
    """out = silu(x W_gate^T) * (x W_up^T), silu(a) = a / (1 + exp(-a))."""
    g, u = linear_f64(x, w_gate), linear_f64(x, w_up)
    with np.errstate(over="ignore"):
        return f64_to_bf16(g / (1.0 + np.exp(-g)) * u)


def argmax(logits):
    """Index of the largest entry of each row, the lowest index among equal maxima."""
    return np.argmax(bf16_to_f64(logits), axis=1).astype(np.int32)


class RefStack:
    """The decoder stack on the CPU.  shape: an object with n_layers, dim, n_q_heads, n_kv_heads, head_dim,
    ffn, vocab, capacity_M, batch, eps; weights: the same dictionary layout as the GPU driver, as uint16 arrays."""

    def __init__(self, shape, weights):
        self.s, self.w = shape, weights
        s = shape
        scale = 1.0 / np.sqrt(s.head_dim)
        self.caches = []
        for l in range(s.n_layers):
            c = bct_ref.RefCache(s.capacity_M, s.batch, s.n_q_heads, s.n_kv_heads, s.head_dim, "bf16", scale, scale)
            c.set_keys(weights["keys"][l])
            c.set_values(None)
            self.caches.append(c)

    def forward(self, ids, T=1, trace=None):
        """ids [B*T] -> (next ids, logits bits).  trace, if a list, receives the residual stream after each layer."""
        s = self.s
        x = embed(ids, self.w["embed"])
        for l, lw in enumerate(self.w["layers"]):
            h = rmsnorm(x, lw["attn_norm"], s.eps)
            q, wq, wv = linear(h, lw["w_q"]), linear(h, lw["w_wq"]), linear(h, lw["w_wv"])
            c = self.caches[l]
            if T == 1:
                a = c.decode_step(q.reshape(s.batch, s.n_q_heads, s.head_dim),
                                  wq.reshape(s.batch, s.n_kv_heads, s.head_dim),
                                  wv.reshape(s.batch, s.n_kv_heads, s.head_dim))
            else:
                a = c.prefill(q.reshape(s.batch, T, s.n_q_heads, s.head_dim),
                              wq.reshape(s.batch, T, s.n_kv_heads, s.head_dim),
                              wv.reshape(s.batch, T, s.n_kv_heads, s.head_dim), T)
            x = linear(a.reshape(s.batch * T, -1), lw["w_o"], x)
            h = rmsnorm(x, lw["mlp_norm"], s.eps)
            x = linear(swiglu(h, lw["w_gate"], lw["w_up"]), lw["w_down"], x)
            if trace is not None:
                trace.append(x.copy())
        h = rmsnorm(x, self.w["final_norm"], s.eps)
        logits = linear(h, self.w["head"])
        return argmax(logits), logits
