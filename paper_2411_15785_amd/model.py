"""ctypes binding of the bctm_ entry points (include/bct_model.h) and a driver that
chains them with the bounded-cache attention into a Llama-shaped decoder.

The driver holds weights and activations as torch tensors (device memory) and
calls the library once per operation on torch's current stream; it does no
arithmetic of its own.  There is no CPU fallback.
"""
from __future__ import annotations

import ctypes
import math
from dataclasses import dataclass

from . import binding
from .binding import BCT_OK, BctCache, BctError, _dptr, _stream_ptr, _torch

MODEL_EXPORTS = ["bctm_embed", "bctm_rmsnorm", "bctm_pack_weight", "bctm_pack_rows", "bctm_linear", "bctm_linear_split",
                 "bctm_swiglu", "bctm_linear_plan",
                 "bctm_argmax", "bctm_last_error"]

BCTM_KERNEL_STREAMING, BCTM_KERNEL_STREAMING_WIDE, BCTM_KERNEL_TILE128, BCTM_KERNEL_TILE256 = 0, 1, 2, 3
BCTM_KERNEL_STREAMING_TRIPLE = 4

BCTM_X_TILED = 1
BCTM_OUT_TILED = 2

_ready = False


def mlib() -> ctypes.CDLL:
    """libbct.so with the bctm_ prototypes set."""
    global _ready
    L = binding.lib()
    if _ready:
        return L
    vp, u32 = ctypes.c_void_p, ctypes.c_uint32
    L.bctm_embed.argtypes = [vp, vp, vp, u32, u32, u32, vp]
    L.bctm_rmsnorm.argtypes = [vp, vp, vp, u32, u32, ctypes.c_float, u32, vp]
    L.bctm_pack_weight.argtypes = [vp, vp, u32, u32, vp]
    L.bctm_pack_rows.argtypes = [vp, vp, u32, u32, vp]
    L.bctm_linear.argtypes = [vp, vp, vp, vp, u32, u32, u32, u32, vp]
    L.bctm_linear_split.argtypes = [vp, vp, vp, u32, vp, u32, vp, u32, u32, u32, u32, vp]
    L.bctm_swiglu.argtypes = [vp, vp, vp, vp, u32, u32, u32, u32, vp]
    L.bctm_linear_plan.argtypes = [u32, u32, u32, u32, ctypes.POINTER(u32)]
    L.bctm_argmax.argtypes = [vp, vp, u32, u32, vp]
    for n in MODEL_EXPORTS[:-1]:
        getattr(L, n).restype = ctypes.c_int
    L.bctm_last_error.argtypes = []
    L.bctm_last_error.restype = ctypes.c_char_p
    _ready = True
    return L


class BctModelError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        L = mlib()
        super().__init__(f"{where}: {L.bct_strerror(status).decode()} ({status}): {L.bctm_last_error().decode()}")


def _ck(st, where):
    if st != BCT_OK:
        raise BctModelError(st, where)


def _bf16_2d(t, name, cols=None):
    torch = _torch()
    if t.dtype != torch.bfloat16 or t.dim() != 2 or not t.is_contiguous() or not t.is_cuda or \
            (cols is not None and t.shape[1] != cols):
        raise ValueError(f"{name}: expected a contiguous 2-D bf16 device tensor"
                         + (f" with {cols} columns" if cols is not None else "")
                         + f", got {t.dtype} {tuple(t.shape)} on {t.device}")


def bctm_embed(ids, table, out=None):
    torch = _torch()
    _bf16_2d(table, "table")
    if ids.dtype != torch.int32 or ids.dim() != 1 or not ids.is_contiguous() or ids.device != table.device:
        raise ValueError("ids: expected a contiguous 1-D int32 tensor on the table's device")
    if out is None:
        out = torch.empty((ids.numel(), table.shape[1]), dtype=torch.bfloat16, device=table.device)
    _bf16_2d(out, "out", table.shape[1])
    if out.shape[0] != ids.numel():
        raise ValueError("out: one row per id")
    with torch.cuda.device(table.device):
        _ck(mlib().bctm_embed(_dptr(ids), _dptr(table), _dptr(out), ids.numel(), table.shape[0], table.shape[1],
                              _stream_ptr()), "bctm_embed")
    return out


def bctm_linear_plan(rows, K, N, swiglu=False):
    """The kernel a projection of this shape runs in (one of the BCTM_KERNEL_ values); host logic, no GPU."""
    k = ctypes.c_uint32(0)
    _ck(mlib().bctm_linear_plan(rows, K, N, 1 if swiglu else 0, ctypes.byref(k)), "bctm_linear_plan")
    return k.value


class TiledRows:
    """A [rows][K] activation matrix in the tiled order the projections read (include/bct_model.h):
    data holds 32 * ceil(rows / 32) * K bf16."""

    def __init__(self, rows, K, device, data=None):
        torch = _torch()
        n = 32 * ((rows + 31) // 32) * K
        if data is None:
            # zeros, not empty: rows past the end are read (never stored) and should be finite
            data = torch.zeros(n, dtype=torch.bfloat16, device=device)
        if data.dtype != torch.bfloat16 or data.numel() != n or not data.is_contiguous():
            raise ValueError(f"tiled data: expected {n} contiguous bf16")
        self.data, self.rows, self.K = data, rows, K


def bctm_pack_rows(x, out=None):
    torch = _torch()
    _bf16_2d(x, "x")
    rows, K = x.shape
    if out is None:
        out = TiledRows(rows, K, x.device)
    if (out.rows, out.K) != (rows, K):
        raise ValueError("out: tiled buffer of x's shape")
    with torch.cuda.device(x.device):
        _ck(mlib().bctm_pack_rows(_dptr(x), _dptr(out.data), rows, K, _stream_ptr()), "bctm_pack_rows")
    return out


def bctm_rmsnorm(x, gain, eps, out=None, tiled=False):
    """out: a tensor of x's shape, or (tiled=True) a TiledRows."""
    torch = _torch()
    _bf16_2d(x, "x")
    if gain.dtype != torch.bfloat16 or tuple(gain.shape) != (x.shape[1],) or not gain.is_contiguous() \
            or gain.device != x.device:
        raise ValueError("gain: expected a contiguous bf16 vector of x's row length on x's device")
    if tiled:
        if out is None:
            out = TiledRows(x.shape[0], x.shape[1], x.device)
        if not isinstance(out, TiledRows) or (out.rows, out.K) != tuple(x.shape):
            raise ValueError("out: a TiledRows of x's shape")
        dst = out.data
    else:
        if out is None:
            out = torch.empty_like(x)
        _bf16_2d(out, "out", x.shape[1])
        if out.shape[0] != x.shape[0]:
            raise ValueError("out: x's shape")
        dst = out
    with torch.cuda.device(x.device):
        _ck(mlib().bctm_rmsnorm(_dptr(x), _dptr(gain), _dptr(dst), x.shape[0], x.shape[1], eps,
                                BCTM_OUT_TILED if tiled else 0, _stream_ptr()), "bctm_rmsnorm")
    return out


class PackedWeight:
    """A weight matrix [N][K] in the tiled layout bctm_linear / bctm_swiglu stream (bctm_pack_weight)."""

    def __init__(self, data, N, K):
        self.data, self.N, self.K = data, N, K


def bctm_pack_weight(*ws):
    """One or more matrices [N_i][K] -> one PackedWeight of sum N_i features, matrix after matrix."""
    torch = _torch()
    for w in ws:
        _bf16_2d(w, "w", ws[0].shape[1])
    K = ws[0].shape[1]
    N = sum(w.shape[0] for w in ws)
    data = torch.empty(N * K, dtype=torch.bfloat16, device=ws[0].device)
    off = 0
    with torch.cuda.device(ws[0].device):
        for w in ws:
            _ck(mlib().bctm_pack_weight(_dptr(w), _dptr(data[off:]), w.shape[0], K, _stream_ptr()),
                "bctm_pack_weight")
            off += w.shape[0] * K
    return PackedWeight(data, N, K)


def _packed(w, name, K):
    if not isinstance(w, PackedWeight):
        raise ValueError(f"{name}: expected a PackedWeight (bctm_pack_weight)")
    if w.K != K:
        raise ValueError(f"{name}: packed for {w.K} inputs, x has {K}")


def _x_arg(x):
    """-> (data tensor, rows, K, flag) of a row-major tensor or a TiledRows."""
    if isinstance(x, TiledRows):
        return x.data, x.rows, x.K, BCTM_X_TILED
    _bf16_2d(x, "x")
    return x, x.shape[0], x.shape[1], 0


def bctm_linear(x, w, residual=None, out=None):
    """x: a [rows][K] tensor or a TiledRows; out / residual row-major [rows][N]."""
    torch = _torch()
    xd, rows, K, xf = _x_arg(x)
    _packed(w, "w", K)
    N = w.N
    if out is None:
        out = torch.empty((rows, N), dtype=torch.bfloat16, device=xd.device)
    _bf16_2d(out, "out", N)
    if residual is not None:
        _bf16_2d(residual, "residual", N)
    if out.shape[0] != rows or (residual is not None and residual.shape[0] != rows):
        raise ValueError("out / residual: one row per row of x")
    with torch.cuda.device(xd.device):
        _ck(mlib().bctm_linear(_dptr(xd), _dptr(w.data), _dptr(residual), _dptr(out), rows, K, N, xf,
                               _stream_ptr()), "bctm_linear")
    return out


def bctm_linear_split(x, w, outs):
    """One projection into two or three row-major outputs whose widths add up to w.N."""
    xd, rows, K, xf = _x_arg(x)
    _packed(w, "w", K)
    if len(outs) not in (2, 3) or sum(o.shape[1] for o in outs) != w.N:
        raise ValueError("outs: two or three tensors whose widths add up to the weight's features")
    for o in outs:
        _bf16_2d(o, "out")
        if o.shape[0] != rows:
            raise ValueError("outs: one row per row of x")
    o2, n2 = (outs[2], outs[2].shape[1]) if len(outs) == 3 else (None, 0)
    torch = _torch()
    with torch.cuda.device(xd.device):
        _ck(mlib().bctm_linear_split(_dptr(xd), _dptr(w.data), _dptr(outs[0]), outs[0].shape[1], _dptr(outs[1]),
                                     outs[1].shape[1], _dptr(o2), n2, rows, K, xf, _stream_ptr()), "bctm_linear_split")
    return outs


def bctm_swiglu(x, w_gate, w_up, out=None, tiled=False):
    """x: a [rows][K] tensor or a TiledRows; out: a [rows][N] tensor, or (tiled=True) a TiledRows."""
    torch = _torch()
    xd, rows, K, xf = _x_arg(x)
    _packed(w_gate, "w_gate", K)
    _packed(w_up, "w_up", K)
    if w_gate.N != w_up.N:
        raise ValueError("w_gate and w_up: same shape")
    N = w_gate.N
    if tiled:
        if out is None:
            out = TiledRows(rows, N, xd.device)
        if not isinstance(out, TiledRows) or (out.rows, out.K) != (rows, N):
            raise ValueError("out: a TiledRows [rows][N]")
        dst = out.data
    else:
        if out is None:
            out = torch.empty((rows, N), dtype=torch.bfloat16, device=xd.device)
        _bf16_2d(out, "out", N)
        if out.shape[0] != rows:
            raise ValueError("out: one row per row of x")
        dst = out
    with torch.cuda.device(xd.device):
        _ck(mlib().bctm_swiglu(_dptr(xd), _dptr(w_gate.data), _dptr(w_up.data), _dptr(dst), rows, K, N,
                               xf | (BCTM_OUT_TILED if tiled else 0), _stream_ptr()), "bctm_swiglu")
    return out


def bctm_argmax(logits, out=None):
    torch = _torch()
    _bf16_2d(logits, "logits")
    if out is None:
        out = torch.empty(logits.shape[0], dtype=torch.int32, device=logits.device)
    if out.dtype != torch.int32 or tuple(out.shape) != (logits.shape[0],) or not out.is_contiguous():
        raise ValueError("out: a contiguous int32 vector, one entry per row")
    with torch.cuda.device(logits.device):
        _ck(mlib().bctm_argmax(_dptr(logits), _dptr(out), logits.shape[0], logits.shape[1], _stream_ptr()),
            "bctm_argmax")
    return out


# ------------------------------------------------------------------ the stack


@dataclass(frozen=True)
class StackShape:
    """A Llama-shaped decoder whose attention layers are bounded caches (section 3.2)."""
    n_layers: int
    dim: int            # model width
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn: int            # SwiGLU hidden width
    vocab: int
    capacity_M: int
    batch: int
    eps: float = 1e-5

    def __post_init__(self):
        if self.dim % 32 or (self.n_q_heads * self.head_dim) % 32 or self.ffn % 32 or self.vocab % 16 or \
                (self.n_kv_heads * self.head_dim) % 16:
            raise ValueError("dim, n_q_heads * head_dim and ffn must be multiples of 32; vocab and "
                             "n_kv_heads * head_dim multiples of 16")

    @property
    def q_width(self):
        return self.n_q_heads * self.head_dim

    @property
    def kv_width(self):
        return self.n_kv_heads * self.head_dim

    def weight_shapes(self):
        """name -> shape of every per-layer weight, in the order load_layer expects."""
        return {"attn_norm": (self.dim,), "w_q": (self.q_width, self.dim), "w_wq": (self.kv_width, self.dim),
                "w_wv": (self.kv_width, self.dim), "w_o": (self.dim, self.q_width), "mlp_norm": (self.dim,),
                "w_gate": (self.ffn, self.dim), "w_up": (self.ffn, self.dim), "w_down": (self.dim, self.ffn)}

    def weight_bytes(self):
        per_layer = sum(math.prod(s) for s in self.weight_shapes().values())
        return 2 * (self.n_layers * per_layer + 2 * self.vocab * self.dim + self.dim)


class BctStack:
    """Token ids in, greedy next ids out: embedding, n_layers x (RMSNorm, W_q / W_wq / W_wv,
    bounded-cache attention, W_o + residual, RMSNorm, SwiGLU MLP + residual), RMSNorm, output head, arg-max.

    weights: {"embed": [vocab][dim], "final_norm": [dim], "head": [vocab][dim],
              "layers": [ {name: tensor} per layer, names of StackShape.weight_shapes() ],
              "keys": [ MK per layer, [Hkv][M][d] ]}  -- all bf16 device tensors.
    """

    def __init__(self, shape: StackShape, weights, max_prefill_T=0, device="cuda:0"):
        torch = _torch()
        self.shape = shape
        self.device = torch.device(device)
        s = shape
        self.caches = []
        ws = None
        for l in range(s.n_layers):
            c = BctCache(s.capacity_M, s.batch, s.n_q_heads, s.n_kv_heads, s.head_dim, torch.bfloat16,
                         max_prefill_T=max_prefill_T, device=device, workspace=ws)
            ws = c._workspace          # one stream steps the layers in turn: they share the workspace
            c.set_keys(weights["keys"][l])
            c.set_values(None)
            self.caches.append(c)
        # matrices are repacked once into the streaming layout; the row-major copies are not kept
        self.layers = []
        for l, lw in enumerate(weights["layers"]):
            pl = {}
            for n, shp in s.weight_shapes().items():
                if tuple(lw[n].shape) != shp or lw[n].dtype != torch.bfloat16:
                    raise ValueError(f"layer {l} {n}: expected bf16 {shp}")
                if len(shp) == 1:
                    pl[n] = lw[n]
                elif n not in ("w_q", "w_wq", "w_wv"):
                    pl[n] = bctm_pack_weight(lw[n])
            # the three projections of the attention input run as one launch with three outputs
            pl["w_qkv"] = bctm_pack_weight(lw["w_q"], lw["w_wq"], lw["w_wv"])
            self.layers.append(pl)
        self.embed, self.final_norm = weights["embed"], weights["final_norm"]
        self.head = bctm_pack_weight(weights["head"])
        self._bufs = {}

    def _buf(self, name, rows, cols):
        torch = _torch()
        k = (name, rows, cols)
        if k not in self._bufs:
            self._bufs[k] = torch.empty((rows, cols), dtype=torch.bfloat16, device=self.device)
        return self._bufs[k]

    def _tiled(self, name, rows, cols):
        k = ("tiled", name, rows, cols)
        if k not in self._bufs:
            self._bufs[k] = TiledRows(rows, cols, self.device)
        return self._bufs[k]

    def forward(self, ids, T=1, next_ids=None, head="all"):
        """ids int32 [B*T] (sequence-major: row b*T + t) -> (next ids, logits).
        T = 1 is a decode step; T > 1 pushes a chunk of T tokens per sequence through bct_prefill.
        head = "all": logits [B*T][vocab] and greedy ids [B*T] for every row; head = "last": only for the last
        token of every sequence ([B][vocab], [B]) - what a prompt needs, without a [B*T][vocab] product.
        next_ids: where to write the greedy tokens (may be ids itself: it is read first, written last).
        After the first call of a given (B, T, head) no memory is allocated, so a call can be captured in a
        HIP graph."""
        s = self.shape
        rows = s.batch * T
        if ids.numel() != rows:
            raise ValueError(f"ids: expected {rows} entries")
        if head not in ("all", "last"):
            raise ValueError('head: "all" or "last"')
        x = bctm_embed(ids, self.embed, self._buf("x", rows, s.dim))
        # every input of a projection is kept tiled, so that the projections read it in whole kilobytes
        h, f = self._tiled("h", rows, s.dim), self._tiled("f", rows, s.ffn)
        q, wq, wv = self._buf("q", rows, s.q_width), self._buf("wq", rows, s.kv_width), self._buf("wv", rows, s.kv_width)
        a = self._buf("a", rows, s.q_width)
        # a chunk's attention output is re-tiled for W_o (the matrix-core kernel reads whole tiles); for the
        # few rows of a decode step re-tiling would cost more than it saves
        at = self._tiled("a", rows, s.q_width) if rows >= 128 else None
        for l, lw in enumerate(self.layers):
            bctm_rmsnorm(x, lw["attn_norm"], s.eps, h, tiled=True)
            bctm_linear_split(h, lw["w_qkv"], (q, wq, wv))
            c = self.caches[l]
            if T == 1:
                c.decode_step(q.view(s.batch, s.n_q_heads, s.head_dim), wq.view(s.batch, s.n_kv_heads, s.head_dim),
                              wv.view(s.batch, s.n_kv_heads, s.head_dim),
                              a.view(s.batch, s.n_q_heads, s.head_dim))
            else:
                c.prefill(q.view(s.batch, T, s.n_q_heads, s.head_dim), wq.view(s.batch, T, s.n_kv_heads, s.head_dim),
                          wv.view(s.batch, T, s.n_kv_heads, s.head_dim), T,
                          a.view(s.batch, T, s.n_q_heads, s.head_dim))
            bctm_linear(bctm_pack_rows(a, at) if at is not None else a, lw["w_o"], x, x)
            bctm_rmsnorm(x, lw["mlp_norm"], s.eps, h, tiled=True)
            bctm_swiglu(h, lw["w_gate"], lw["w_up"], f, tiled=True)
            bctm_linear(f, lw["w_down"], x, x)
        if head == "last" and T > 1:
            # rows b*T + T-1, gathered with the embedding kernel (a row lookup) from x as the table
            torch = _torch()
            k = ("last_rows", s.batch, T)
            if k not in self._bufs:
                self._bufs[k] = (torch.arange(s.batch, dtype=torch.int32, device=self.device) * T + (T - 1)).contiguous()
            x = bctm_embed(self._bufs[k], x, self._buf("x_last", s.batch, s.dim))
            rows = s.batch
            h = self._tiled("h_last", rows, s.dim)
        bctm_rmsnorm(x, self.final_norm, s.eps, h, tiled=True)
        logits = bctm_linear(h, self.head, None, self._buf("logits", rows, s.vocab))
        nxt = bctm_argmax(logits, next_ids)
        return nxt, logits
