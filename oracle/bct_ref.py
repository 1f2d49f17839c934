"""ctypes binding of the CPU oracle (oracle/libbct_ref.so).

Test infrastructure only: imported by tests/, by the smoke check and by the
cpu_baseline leg of bench.py.  Works on numpy arrays in host memory; bf16
tensors travel as uint16 bit patterns.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libbct_ref.so")

F32 = 0
BF16 = 1
FLAG_MK_PER_SEQUENCE = 1

_DT = {"f32": F32, "bf16": BF16}
_NP = {"f32": np.float32, "bf16": np.uint16}


class _Desc(ctypes.Structure):
    _fields_ = [("M", ctypes.c_uint32), ("B", ctypes.c_uint32), ("Hq", ctypes.c_uint32),
                ("Hkv", ctypes.c_uint32), ("d", ctypes.c_uint32), ("dtype", ctypes.c_int32),
                ("read_scale", ctypes.c_float), ("write_scale", ctypes.c_float),
                ("flags", ctypes.c_uint32)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            from . import build as _b
            _b.build()
        L = ctypes.CDLL(_LIB_PATH)
        vp = ctypes.c_void_p
        L.bct_ref_cache_create.argtypes = [ctypes.POINTER(_Desc), ctypes.POINTER(vp)]
        L.bct_ref_cache_destroy.argtypes = [vp]
        L.bct_ref_cache_destroy.restype = None
        for n in ("bct_ref_cache_bytes", "bct_ref_keys_bytes", "bct_ref_values_bytes"):
            getattr(L, n).argtypes = [vp]
            getattr(L, n).restype = ctypes.c_size_t
        L.bct_ref_cache_set_keys.argtypes = [vp, vp]
        L.bct_ref_cache_set_values.argtypes = [vp, vp]
        L.bct_ref_cache_export.argtypes = [vp, vp, vp, ctypes.POINTER(ctypes.c_uint64)]
        L.bct_ref_cache_import.argtypes = [vp, vp, vp, ctypes.c_uint64]
        L.bct_ref_cache_steps.argtypes = [vp, ctypes.POINTER(ctypes.c_uint64)]
        L.bct_ref_decode_step.argtypes = [vp, vp, vp, vp, vp]
        L.bct_ref_prefill.argtypes = [vp, vp, vp, vp, ctypes.c_uint32, vp]
        L.bct_ref_cache_randomize_values.argtypes = [vp, ctypes.c_uint64, ctypes.c_float]
        L.bct_ref_splitmix64_at.argtypes = [ctypes.c_uint64, ctypes.c_uint64]
        L.bct_ref_splitmix64_at.restype = ctypes.c_uint64
        L.bct_ref_cache_export_sequence.argtypes = [vp, ctypes.c_uint32, vp, vp]
        L.bct_ref_cache_import_sequence.argtypes = [vp, ctypes.c_uint32, vp, vp]
        L.bct_ref_decode_step_gated.argtypes = [vp, vp, vp, vp, vp, vp]
        L.bct_ref_prefill_gated.argtypes = [vp, vp, vp, vp, vp, ctypes.c_uint32, vp]
        L.bct_ref_decode_step_keyed.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp]
        L.bct_ref_probe_weights.argtypes = [vp, ctypes.c_uint32, ctypes.c_uint32, vp, ctypes.c_double, vp]
        L.bct_ref_round_bf16_from_float.argtypes = [ctypes.c_float]
        L.bct_ref_round_bf16_from_float.restype = ctypes.c_uint16
        L.bct_ref_round_bf16_from_double.argtypes = [ctypes.c_double]
        L.bct_ref_round_bf16_from_double.restype = ctypes.c_uint16
        _lib = L
    return _lib


def _ptr(a):
    if a is None:
        return None
    assert a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(ctypes.c_void_p)


class RefCache:
    """One layer's bounded cache on the host: MK (static) and MV (state)."""

    def __init__(self, M, B, Hq, Hkv, d, dtype, read_scale, write_scale, flags=0):
        self.M, self.B, self.Hq, self.Hkv, self.d = M, B, Hq, Hkv, d
        self.dtype = dtype
        self.flags = flags
        self.read_scale, self.write_scale = read_scale, write_scale
        self._np = _NP[dtype]
        ds = _Desc(M, B, Hq, Hkv, d, _DT[dtype] if isinstance(dtype, str) else dtype,
                   read_scale, write_scale, flags)
        h = ctypes.c_void_p()
        rc = lib().bct_ref_cache_create(ctypes.byref(ds), ctypes.byref(h))
        if rc != 0:
            raise ValueError(f"bct_ref_cache_create failed ({rc})")
        self._h = h

    def __del__(self):
        if getattr(self, "_h", None) and _lib is not None:
            _lib.bct_ref_cache_destroy(self._h)
            self._h = None

    # -- shapes
    @property
    def keys_shape(self):
        s = (self.Hkv, self.M, self.d)
        return (self.B,) + s if self.flags & FLAG_MK_PER_SEQUENCE else s

    @property
    def values_shape(self):
        return (self.B, self.Hkv, self.M, self.d)

    def cache_bytes(self):
        return lib().bct_ref_cache_bytes(self._h)

    def _chk(self, a, shape):
        a = np.ascontiguousarray(a)
        assert a.dtype == self._np, (a.dtype, self._np)
        assert tuple(a.shape) == tuple(shape), (a.shape, shape)
        return a

    def set_keys(self, mk):
        mk = self._chk(mk, self.keys_shape)
        assert lib().bct_ref_cache_set_keys(self._h, _ptr(mk)) == 0

    def set_values(self, mv0=None):
        if mv0 is not None:
            mv0 = self._chk(mv0, self.values_shape)
        assert lib().bct_ref_cache_set_values(self._h, _ptr(mv0)) == 0

    def randomize_values(self, seed, amplitude):
        assert lib().bct_ref_cache_randomize_values(self._h, seed, amplitude) == 0

    def export_sequence(self, b):
        """-> MV[b] as [Hkv][M][d]."""
        mv = np.empty(self.values_shape[1:], dtype=self._np)
        assert lib().bct_ref_cache_export_sequence(self._h, b, None, _ptr(mv)) == 0
        return mv

    def import_sequence(self, b, mv):
        mv = self._chk(mv, self.values_shape[1:])
        assert lib().bct_ref_cache_import_sequence(self._h, b, None, _ptr(mv)) == 0

    def export(self):
        mk = np.empty(self.keys_shape, dtype=self._np)
        mv = np.empty(self.values_shape, dtype=self._np)
        st = ctypes.c_uint64()
        assert lib().bct_ref_cache_export(self._h, _ptr(mk), _ptr(mv), ctypes.byref(st)) == 0
        return mk, mv, st.value

    def values(self):
        mv = np.empty(self.values_shape, dtype=self._np)
        assert lib().bct_ref_cache_export(self._h, None, _ptr(mv), None) == 0
        return mv

    def import_(self, mk, mv, steps):
        mk = None if mk is None else self._chk(mk, self.keys_shape)
        mv = None if mv is None else self._chk(mv, self.values_shape)
        assert lib().bct_ref_cache_import(self._h, _ptr(mk), _ptr(mv), steps) == 0

    @property
    def steps(self):
        st = ctypes.c_uint64()
        assert lib().bct_ref_cache_steps(self._h, ctypes.byref(st)) == 0
        return st.value

    def _gate(self, gate, shape):
        if gate is None:
            return None
        gate = np.ascontiguousarray(gate)
        assert gate.dtype == np.float32 and gate.shape == tuple(shape), (gate.dtype, gate.shape, shape)
        return gate

    def decode_step(self, q, wq, wv, gate=None):
        """Returns out [B][Hq][d] (or None for a write-only step).  gate: float32 [B][Hkv] step sizes."""
        out = None
        if q is not None:
            q = self._chk(q, (self.B, self.Hq, self.d))
            out = np.empty_like(q)
        if wq is not None:
            wq = self._chk(wq, (self.B, self.Hkv, self.d))
        if wv is not None:
            wv = self._chk(wv, (self.B, self.Hkv, self.d))
        gate = self._gate(gate, (self.B, self.Hkv))
        rc = lib().bct_ref_decode_step_gated(self._h, _ptr(q), _ptr(wq), _ptr(wv), _ptr(gate), _ptr(out))
        if rc != 0:
            raise RuntimeError(f"bct_ref_decode_step failed ({rc})")
        return out

    def decode_step_keyed(self, q, wq, wv, wk, gate=None, kgate=None):
        """The keyed step (per-sequence keys): the write also moves the keys, MK += kappa ww^T wk, after the
        token's read.  wk: [B][Hkv][d]; gate / kgate: float32 [B][Hkv] step sizes of the value / key write."""
        out = None
        if q is not None:
            q = self._chk(q, (self.B, self.Hq, self.d))
            out = np.empty_like(q)
        wq, wv, wk = (self._chk(a, (self.B, self.Hkv, self.d)) for a in (wq, wv, wk))
        gate, kgate = self._gate(gate, (self.B, self.Hkv)), self._gate(kgate, (self.B, self.Hkv))
        rc = lib().bct_ref_decode_step_keyed(self._h, _ptr(q), _ptr(wq), _ptr(wv), _ptr(wk), _ptr(gate), _ptr(kgate),
                                             _ptr(out))
        if rc != 0:
            raise RuntimeError(f"bct_ref_decode_step_keyed failed ({rc})")
        return out

    def keys(self):
        mk = np.empty(self.keys_shape, dtype=self._np)
        assert lib().bct_ref_cache_export(self._h, _ptr(mk), None, None) == 0
        return mk

    def decode_step_rc(self, q, wq, wv, out):
        return lib().bct_ref_decode_step(self._h, _ptr(q), _ptr(wq), _ptr(wv), _ptr(out))

    def prefill(self, q, wq, wv, T, gate=None):
        out = None
        if q is not None:
            q = self._chk(q, (self.B, T, self.Hq, self.d))
            out = np.empty_like(q)
        if wq is not None:
            wq = self._chk(wq, (self.B, T, self.Hkv, self.d))
        if wv is not None:
            wv = self._chk(wv, (self.B, T, self.Hkv, self.d))
        gate = self._gate(gate, (self.B, T, self.Hkv))
        rc = lib().bct_ref_prefill_gated(self._h, _ptr(q), _ptr(wq), _ptr(wv), _ptr(gate), T, _ptr(out))
        if rc != 0:
            raise RuntimeError(f"bct_ref_prefill failed ({rc})")
        return out

    def probe_weights(self, b, h, vec, scale):
        vec = np.ascontiguousarray(vec)
        assert vec.dtype == self._np and vec.shape == (self.d,)
        w = np.empty(self.M, dtype=np.float64)
        assert lib().bct_ref_probe_weights(self._h, b, h, _ptr(vec), scale, _ptr(w)) == 0
        return w


def splitmix64_at(seed: int, n: int) -> int:
    return lib().bct_ref_splitmix64_at(seed, n)


def num_threads() -> int:
    return lib().bct_ref_num_threads()


def round_bf16_from_float(f: float) -> int:
    return lib().bct_ref_round_bf16_from_float(f)


def round_bf16_from_double(x: float) -> int:
    return lib().bct_ref_round_bf16_from_double(x)
