"""Seeded synthetic inputs for the Bounded-Cache Transformer decode path.

This module serves BOTH the CPU oracle and the HIP path with the same bytes.
It holds none of the method's arithmetic: only a counter-based random number
generator, a normal transform, storage-dtype packing and the five workload
shapes.  It depends on numpy only and imports neither side.

Generator: value(seed, tensor_id, step, index) is a pure function of its four
integer arguments (splitmix64 finaliser over a mixed counter), so any slice of
any tensor at any step can be produced on its own, in any order.

Tensor ids: MK=1, q=2, wq=3, wv=4, weights=5, tokens=6, MV0=7.
"""
from __future__ import annotations

import dataclasses
import math

import numpy as np

BASE_SEED = 0x241115785

TID_MK = 1
TID_Q = 2
TID_WQ = 3
TID_WV = 4
TID_WEIGHTS = 5
TID_TOKENS = 6
TID_MV0 = 7

_M64 = np.uint64(0xFFFFFFFFFFFFFFFF)


def _splitmix64(x: np.ndarray) -> np.ndarray:
    """splitmix64 output function on an array of uint64 counters."""
    with np.errstate(over="ignore"):
        z = (x + np.uint64(0x9E3779B97F4A7C15)) & _M64
        z = ((z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)) & _M64
        z = ((z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)) & _M64
        return z ^ (z >> np.uint64(31))


def _stream_key(seed: int, tensor_id: int, step: int) -> np.uint64:
    k = np.array([seed & 0xFFFFFFFFFFFFFFFF], dtype=np.uint64)
    k = _splitmix64(k ^ np.uint64((tensor_id * 0xD1342543DE82EF95) & 0xFFFFFFFFFFFFFFFF))
    k = _splitmix64(k ^ np.uint64((step * 0xA0761D6478BD642F) & 0xFFFFFFFFFFFFFFFF))
    return k[0]


def raw_bits(seed: int, tensor_id: int, step: int, start: int, count: int) -> np.ndarray:
    """uint64 random bits for counters [start, start+count)."""
    key = _stream_key(seed, tensor_id, step)
    ctr = np.arange(start, start + count, dtype=np.uint64)
    return _splitmix64(ctr ^ key)


def _normal_block(key_args, start: int, n: int) -> np.ndarray:
    """Normals for flat indices [start, start+n).  Index i takes counter i // 2:
    the counter's 64 bits give two 32-bit uniforms, Box-Muller turns them into
    two normals, the even index takes the cosine branch and the odd the sine."""
    p0, p1 = start // 2, (start + n + 1) // 2
    bits = raw_bits(*key_args, p0, p1 - p0)
    u1 = ((bits >> np.uint64(32)).astype(np.float64) + 1.0) * (1.0 / 4294967296.0)
    u2 = (bits & np.uint64(0xFFFFFFFF)).astype(np.float64) * (1.0 / 4294967296.0)
    r = np.sqrt(-2.0 * np.log(u1))
    ang = (2.0 * math.pi) * u2
    z = np.empty((p1 - p0, 2), dtype=np.float64)
    np.multiply(r, np.cos(ang), out=z[:, 0])
    np.multiply(r, np.sin(ang), out=z[:, 1])
    off = start - 2 * p0
    return z.reshape(-1)[off:off + n]


def normal(seed: int, tensor_id: int, step: int, shape, start: int = 0) -> np.ndarray:
    """Standard normal samples (float64) of the given shape; element i of the
    flattened result depends only on (seed, tensor_id, step, start + i)."""
    count = int(np.prod(shape)) if len(shape) else 1
    out = np.empty(count, dtype=np.float64)
    blk = 1 << 20
    key_args = (seed, tensor_id, step)
    spans = [(s, min(blk, count - s)) for s in range(0, count, blk)]

    def work(span):
        s, n = span
        out[s:s + n] = _normal_block(key_args, start + s, n)

    if len(spans) <= 1:
        for sp in spans:
            work(sp)
    else:  # numpy releases the GIL inside its loops; blocks are independent
        import concurrent.futures
        import os
        with concurrent.futures.ThreadPoolExecutor(max_workers=min(16, os.cpu_count() or 1)) as ex:
            list(ex.map(work, spans))
    return out.reshape(shape)


def integers(seed: int, tensor_id: int, step: int, shape, high: int) -> np.ndarray:
    """Uniform integer ids in [0, high) (int64)."""
    count = int(np.prod(shape))
    b = raw_bits(seed, tensor_id, step, 0, count)
    return (b % np.uint64(high)).astype(np.int64).reshape(shape)


# ---------------------------------------------------------------- dtype packing

def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 values to bfloat16 storage (round-to-nearest-even),
    returned as uint16 bit patterns.  Input packing only."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bit patterns (uint16) to float32 exactly."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def pack(x: np.ndarray, dtype: str) -> np.ndarray:
    """float64 samples -> storage array: 'f32' -> float32, 'bf16' -> uint16 bits."""
    if dtype == "f32":
        return np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "bf16":
        return f32_to_bf16_bits(x.astype(np.float32))
    raise ValueError(f"unknown dtype {dtype!r}")


def unpack(a: np.ndarray, dtype: str) -> np.ndarray:
    """storage array -> float64 values (exact)."""
    if dtype == "f32":
        return np.asarray(a, dtype=np.float32).astype(np.float64)
    if dtype == "bf16":
        return bf16_bits_to_f32(a).astype(np.float64)
    raise ValueError(f"unknown dtype {dtype!r}")


def elem_size(dtype: str) -> int:
    return {"f32": 4, "bf16": 2}[dtype]


# ---------------------------------------------------------------- workloads

@dataclasses.dataclass(frozen=True)
class Workload:
    """Shape of one attention layer's bounded cache plus its step counts."""
    name: str
    layers: int
    B: int
    Hq: int
    Hkv: int
    d: int
    M: int
    dtype: str
    decode_steps: int
    prompt: int = 0          # tokens fed through prefill before decoding
    prefill_chunk: int = 0   # chunk length T of each prefill call

    @property
    def G(self) -> int:
        return self.Hq // self.Hkv

    @property
    def scale(self) -> float:
        return 1.0 / math.sqrt(self.d)

    def algorithmic_bytes_per_layer_step(self, shared_mk: bool = True) -> int:
        """Bytes the update rule and the read must move for one decode step of
        one layer: MV read + MV write (every slot is rewritten), MK once
        (shared over the batch) or B times, plus q/out/wq/wv."""
        sz = elem_size(self.dtype)
        mv = self.B * self.Hkv * self.M * self.d * sz
        mk = self.Hkv * self.M * self.d * sz * (1 if shared_mk else self.B)
        io = self.B * (2 * self.Hq + 2 * self.Hkv) * self.d * sz
        return 2 * mv + mk + io


WORKLOADS = {
    "cfg1": Workload("cfg1", 1, 1, 4, 4, 64, 64, "f32", 256),
    "cfg2": Workload("cfg2", 1, 8, 32, 32, 128, 1024, "bf16", 2048),
    "cfg3": Workload("cfg3", 32, 32, 32, 32, 128, 4096, "bf16", 8192, prompt=1024, prefill_chunk=512),
    "cfg4": Workload("cfg4", 1, 64, 32, 8, 128, 8192, "bf16", 16384),
    "cfg5": Workload("cfg5", 1, 16, 64, 64, 128, 16384, "bf16", 65536, prompt=2048, prefill_chunk=512),
}


def layer_seed(layer: int) -> int:
    return BASE_SEED + 1000003 * layer


def make_keys(w: Workload, layer: int = 0, per_sequence: bool = False) -> np.ndarray:
    """MK ~ N(0,1): [Hkv][M][d] (or [B][Hkv][M][d]) in storage dtype."""
    shape = (w.Hkv, w.M, w.d) if not per_sequence else (w.B, w.Hkv, w.M, w.d)
    return pack(normal(layer_seed(layer), TID_MK, 0, shape), w.dtype)


def make_values0(w: Workload, layer: int = 0) -> np.ndarray:
    """A random initial MV ~ N(0,1): [B][Hkv][M][d] in storage dtype."""
    return pack(normal(layer_seed(layer), TID_MV0, 0, (w.B, w.Hkv, w.M, w.d)), w.dtype)


def make_step(w: Workload, step: int, layer: int = 0, T: int = 0):
    """(q, wq, wv) ~ N(0,1) for one decode step (T == 0: [B][H][d]) or one
    prefill chunk of T tokens ([B][T][H][d]; token t of the chunk is global
    step `step + t`, each token drawn exactly as its decode step would be)."""
    s = layer_seed(layer)
    if T == 0:
        q = pack(normal(s, TID_Q, step, (w.B, w.Hq, w.d)), w.dtype)
        wq = pack(normal(s, TID_WQ, step, (w.B, w.Hkv, w.d)), w.dtype)
        wv = pack(normal(s, TID_WV, step, (w.B, w.Hkv, w.d)), w.dtype)
        return q, wq, wv
    qs, wqs, wvs = [], [], []
    for t in range(T):
        q, wq, wv = make_step(w, step + t, layer)
        qs.append(q)
        wqs.append(wq)
        wvs.append(wv)
    return (np.ascontiguousarray(np.stack(qs, axis=1)),
            np.ascontiguousarray(np.stack(wqs, axis=1)),
            np.ascontiguousarray(np.stack(wvs, axis=1)))


# ---------------------------------------------------------------- decoder-stack weights

STACK_WEIGHT_ORDER = ("attn_norm", "w_q", "w_wq", "w_wv", "w_o", "mlp_norm", "w_gate", "w_up", "w_down")


def make_stack_weights(shape, seed: int = 0):
    """Random-init weights of a Llama-shaped stack as bf16 bit patterns.

    shape: an object with n_layers, dim, n_q_heads, n_kv_heads, head_dim, ffn, vocab, capacity_M and a
    weight_shapes() dictionary.  Matrices ~ N(0, 1/fan_in) (the usual variance-preserving init), except that
    the three attention projections are scaled so that their outputs have unit variance like the q / wq / wv
    of the attention-only workloads; norm gains ~ 1 + 0.1 N(0,1); embedding ~ N(0,1); keys MK ~ N(0,1).
    """
    base = layer_seed(0) + 7919 * (seed + 1)
    tid = [0]

    def draw(shp, std, mean=0.0):
        tid[0] += 1
        return pack(mean + std * normal(base, TID_WEIGHTS, tid[0], shp), "bf16")

    layers = []
    for _ in range(shape.n_layers):
        lw = {}
        for name, shp in shape.weight_shapes().items():
            if len(shp) == 1:
                lw[name] = draw(shp, 0.1, 1.0)
            else:
                lw[name] = draw(shp, 1.0 / np.sqrt(shp[1]))
        layers.append(lw)
    keys = [draw((shape.n_kv_heads, shape.capacity_M, shape.head_dim), 1.0) for _ in range(shape.n_layers)]
    return {"embed": draw((shape.vocab, shape.dim), 1.0), "final_norm": draw((shape.dim,), 0.1, 1.0),
            "head": draw((shape.vocab, shape.dim), 1.0 / np.sqrt(shape.dim)), "layers": layers, "keys": keys}


def make_token_ids(seed: int, step: int, count: int, vocab: int) -> np.ndarray:
    return integers(layer_seed(0) + seed, TID_TOKENS, step, (count,), vocab).astype(np.int32)
