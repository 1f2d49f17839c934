"""ctypes binding of libbct.so: the same names as include/bct.h, argument marshalling only.

Every step of the decode path runs in the HIP kernels of the library.  PyTorch
appears here only as the owner of device memory and streams.  There is no CPU
fallback: if the library is missing, loading fails loudly.
"""
from __future__ import annotations

import ctypes
import math
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libbct.so")

BCT_OK = 0
BCT_ERR_INVALID_ARG = 1
BCT_ERR_UNSUPPORTED = 2
BCT_ERR_BUFFER_TOO_SMALL = 3
BCT_ERR_MISALIGNED = 4
BCT_ERR_STATE = 5
BCT_ERR_HIP = 6

BCT_F32 = 0
BCT_BF16 = 1
BCT_MK_PER_SEQUENCE = 1
BCT_STEP_STREAMING = 2

EXPORTS = [
    "bct_cache_query", "bct_cache_init", "bct_cache_set_keys", "bct_cache_set_values",
    "bct_decode_step", "bct_prefill", "bct_decode_step_gated", "bct_prefill_gated", "bct_cache_export",
    "bct_cache_randomize_values", "bct_cache_export_sequence", "bct_cache_import_sequence", "bct_plan_query", "bct_cache_import", "bct_cache_steps",
    "bct_cache_regions", "bct_cache_destroy", "bct_strerror", "bct_last_error", "bct_stream_copy",
    "bct_profile_enable", "bct_profile_read", "bct_decode_step_static", "bct_static_scratch_bytes",
    "bct_decode_step_keyed",
]


class bct_cache_desc(ctypes.Structure):
    _fields_ = [("capacity_M", ctypes.c_uint32), ("batch", ctypes.c_uint32),
                ("n_q_heads", ctypes.c_uint32), ("n_kv_heads", ctypes.c_uint32),
                ("head_dim", ctypes.c_uint32), ("dtype", ctypes.c_int32),
                ("read_scale", ctypes.c_float), ("write_scale", ctypes.c_float),
                ("flags", ctypes.c_uint32)]


class bct_plan_info(ctypes.Structure):
    _fields_ = [(n, ctypes.c_uint32) for n in ("launches", "one_launch", "scores_mfma", "slots_per_stat",
                                               "normaliser_launch", "mv_workgroup", "mv_loads_per_lane",
                                               "mv_splits")]


class BctError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        L = lib()
        super().__init__(f"{where}: {L.bct_strerror(status).decode()} ({status}): {L.bct_last_error().decode()}")


_lib = None


def lib() -> ctypes.CDLL:
    """Loads libbct.so (built by paper_2411_15785_amd/build.py); raises if it is not there."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2411_15785_amd.build` "
            "(there is no fallback path)")
    # Device pointers and streams come from torch, so the library must run on the HIP runtime
    # torch has loaded: import torch first, and the loader resolves libamdhip64 to that copy.
    # Loaded the other way round, the process holds two runtimes and launches fail.
    _torch()
    L = ctypes.CDLL(LIB_PATH)
    vp, sz, u32, u64 = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_uint32, ctypes.c_uint64
    dp = ctypes.POINTER(bct_cache_desc)
    L.bct_cache_query.argtypes = [dp, u32, ctypes.POINTER(sz), ctypes.POINTER(sz)]
    L.bct_cache_init.argtypes = [dp, u32, vp, sz, vp, sz, vp, ctypes.POINTER(vp)]
    L.bct_cache_set_keys.argtypes = [vp, vp, vp]
    L.bct_cache_set_values.argtypes = [vp, vp, vp]
    L.bct_decode_step.argtypes = [vp, vp, vp, vp, vp, vp]
    L.bct_decode_step_static.argtypes = [vp, vp, vp, vp, vp, vp]
    L.bct_decode_step_keyed.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp]
    L.bct_static_scratch_bytes.argtypes = []
    L.bct_prefill.argtypes = [vp, vp, vp, vp, u32, vp, vp]
    L.bct_plan_query.argtypes = [dp, ctypes.POINTER(bct_plan_info)]
    L.bct_cache_randomize_values.argtypes = [vp, u64, ctypes.c_float, vp]
    L.bct_cache_export_sequence.argtypes = [vp, u32, vp, vp, vp]
    L.bct_cache_import_sequence.argtypes = [vp, u32, vp, vp, vp]
    L.bct_decode_step_gated.argtypes = [vp, vp, vp, vp, vp, vp, vp]
    L.bct_prefill_gated.argtypes = [vp, vp, vp, vp, vp, u32, vp, vp]
    L.bct_cache_export.argtypes = [vp, vp, vp, ctypes.POINTER(u64), vp]
    L.bct_cache_import.argtypes = [vp, vp, vp, u64, vp]
    L.bct_cache_steps.argtypes = [vp, ctypes.POINTER(u64)]
    L.bct_cache_regions.argtypes = [vp, ctypes.POINTER(vp), ctypes.POINTER(sz), ctypes.POINTER(vp),
                                    ctypes.POINTER(sz)]
    L.bct_cache_destroy.argtypes = [vp]
    L.bct_cache_destroy.restype = None
    L.bct_strerror.argtypes = [ctypes.c_int]
    L.bct_strerror.restype = ctypes.c_char_p
    L.bct_last_error.argtypes = []
    L.bct_last_error.restype = ctypes.c_char_p
    L.bct_stream_copy.argtypes = [vp, vp, sz, vp]
    L.bct_profile_enable.argtypes = [vp, u32]
    fp = ctypes.POINTER(ctypes.c_float)
    L.bct_profile_read.argtypes = [vp, ctypes.POINTER(u32), fp, fp, fp]
    for n in EXPORTS:
        if n not in ("bct_cache_destroy", "bct_strerror", "bct_last_error", "bct_static_scratch_bytes"):
            getattr(L, n).restype = ctypes.c_int
    L.bct_static_scratch_bytes.restype = sz
    _lib = L
    return L


# ------------------------------------------------------------------ thin function-level wrappers

def make_desc(capacity_M, batch, n_q_heads, n_kv_heads, head_dim, dtype, read_scale, write_scale, flags=0):
    return bct_cache_desc(capacity_M, batch, n_q_heads, n_kv_heads, head_dim, dtype, read_scale, write_scale, flags)


def bct_cache_query(desc, max_prefill_T=0):
    """-> (status, cache_bytes, workspace_bytes)"""
    cb, wb = ctypes.c_size_t(0), ctypes.c_size_t(0)
    st = lib().bct_cache_query(ctypes.byref(desc) if desc is not None else None, max_prefill_T,
                               ctypes.byref(cb), ctypes.byref(wb))
    return st, cb.value, wb.value


def bct_cache_init(desc, max_prefill_T, cache_ptr, cache_bytes, ws_ptr, ws_bytes, stream):
    """-> (status, handle)"""
    h = ctypes.c_void_p()
    st = lib().bct_cache_init(ctypes.byref(desc) if desc is not None else None, max_prefill_T, cache_ptr,
                              cache_bytes, ws_ptr, ws_bytes, stream, ctypes.byref(h))
    return st, h


def bct_plan_query(desc):
    """-> (status, {field: value}) : the launch plan of a decode step for this descriptor."""
    info = bct_plan_info()
    st = lib().bct_plan_query(ctypes.byref(desc) if desc is not None else None, ctypes.byref(info))
    return st, {n: getattr(info, n) for n, _ in bct_plan_info._fields_}


def bct_last_error() -> str:
    return lib().bct_last_error().decode()


def bct_strerror(st: int) -> str:
    return lib().bct_strerror(st).decode()


# ------------------------------------------------------------------ tensor-level convenience

def _torch():
    import torch
    return torch


def _stream_ptr():
    return ctypes.c_void_p(_torch().cuda.current_stream().cuda_stream)


def _dptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


class BctCache:
    """One layer's bounded cache on the GPU.

    Device memory (cache, workspace) lives in torch tensors owned by this
    object; every operation is a call into libbct on torch's current stream.
    dtype: torch.float32 or torch.bfloat16.
    """

    def __init__(self, capacity_M, batch, n_q_heads, n_kv_heads, head_dim, dtype, read_scale=None,
                 write_scale=None, flags=0, max_prefill_T=0, device="cuda:0", workspace=None):
        torch = _torch()
        self.torch_dtype = dtype
        code = {torch.float32: BCT_F32, torch.bfloat16: BCT_BF16}.get(dtype)
        if code is None:
            raise ValueError(f"dtype {dtype} (torch.float32 or torch.bfloat16)")
        rs = 1.0 / math.sqrt(head_dim) if read_scale is None else read_scale
        ws = 1.0 / math.sqrt(head_dim) if write_scale is None else write_scale
        self.desc = make_desc(capacity_M, batch, n_q_heads, n_kv_heads, head_dim, code, rs, ws, flags)
        self.M, self.B, self.Hq, self.Hkv, self.d = capacity_M, batch, n_q_heads, n_kv_heads, head_dim
        self.flags = flags
        self.max_prefill_T = max_prefill_T
        self._h = None
        st, cb, wb = bct_cache_query(self.desc, max_prefill_T)
        if st != BCT_OK:
            raise BctError(st, "bct_cache_query")
        self.cache_bytes, self.workspace_bytes = cb, wb
        self.device = torch.device(device)
        self._cache_mem = torch.empty(cb, dtype=torch.uint8, device=self.device)
        # the workspace holds nothing between calls, so caches stepped on one stream may share one
        if workspace is None:
            workspace = torch.empty(max(wb, 256), dtype=torch.uint8, device=self.device)
        if workspace.dtype != torch.uint8 or workspace.numel() < wb or workspace.device != self.device:
            raise ValueError(f"workspace: need {wb} bytes of torch.uint8 on {self.device}")
        self._workspace = workspace
        with torch.cuda.device(self.device):
            st, h = bct_cache_init(self.desc, max_prefill_T, _dptr(self._cache_mem), cb, _dptr(self._workspace),
                                   self._workspace.numel(), _stream_ptr())
        if st != BCT_OK:
            raise BctError(st, "bct_cache_init")
        self._h = h

    def __del__(self):
        if getattr(self, "_h", None) and _lib is not None:
            _lib.bct_cache_destroy(self._h)
            self._h = None

    # -- shapes
    @property
    def keys_shape(self):
        s = (self.Hkv, self.M, self.d)
        return (self.B,) + s if self.flags & BCT_MK_PER_SEQUENCE else s

    @property
    def values_shape(self):
        return (self.B, self.Hkv, self.M, self.d)

    def _check(self, t, shape, name):
        if t is None:
            return
        if t.dtype != self.torch_dtype or tuple(t.shape) != tuple(shape) or not t.is_contiguous() \
                or t.device != self.device:
            raise ValueError(f"{name}: expected contiguous {self.torch_dtype} {tuple(shape)} on {self.device}, "
                             f"got {t.dtype} {tuple(t.shape)} on {t.device}")

    def _call(self, name, *args):
        torch = _torch()
        with torch.cuda.device(self.device):
            st = getattr(lib(), name)(self._h, *args, _stream_ptr())
        if st != BCT_OK:
            raise BctError(st, name)

    def set_keys(self, mk):
        self._check(mk, self.keys_shape, "mk")
        self._call("bct_cache_set_keys", _dptr(mk))

    def set_values(self, mv0=None):
        self._check(mv0, self.values_shape, "mv0")
        self._call("bct_cache_set_values", _dptr(mv0))

    def randomize_values(self, seed, amplitude):
        self._call("bct_cache_randomize_values", ctypes.c_uint64(seed), ctypes.c_float(amplitude))

    def export_sequence(self, b, with_keys=False):
        """-> MV[b] [Hkv][M][d] (and MK[b] first if with_keys) as fresh tensors."""
        torch = _torch()
        mv = torch.empty(self.values_shape[1:], dtype=self.torch_dtype, device=self.device)
        mk = torch.empty(self.values_shape[1:], dtype=self.torch_dtype, device=self.device) if with_keys else None
        self._call("bct_cache_export_sequence", ctypes.c_uint32(b), _dptr(mk), _dptr(mv))
        return (mk, mv) if with_keys else mv

    def import_sequence(self, b, mv, mk=None):
        self._check(mv, self.values_shape[1:], "mv")
        self._check(mk, self.values_shape[1:], "mk")
        self._call("bct_cache_import_sequence", ctypes.c_uint32(b), _dptr(mk), _dptr(mv))

    def _check_gate(self, gate, shape):
        torch = _torch()
        if gate is not None and (gate.dtype != torch.float32 or tuple(gate.shape) != tuple(shape)
                                 or not gate.is_contiguous() or gate.device != self.device):
            raise ValueError(f"gate: expected contiguous float32 {tuple(shape)} on {self.device}")

    def decode_step(self, q, k_new, v_new, out=None, gate=None):
        """One token per sequence; returns out [B][Hq][d] (None for a write-only step).
        gate: float32 [B][Hkv] step sizes of the write, or None."""
        torch = _torch()
        self._check_gate(gate, (self.B, self.Hkv))
        self._check(q, (self.B, self.Hq, self.d), "q")
        self._check(k_new, (self.B, self.Hkv, self.d), "k_new")
        self._check(v_new, (self.B, self.Hkv, self.d), "v_new")
        if q is not None and out is None:
            out = torch.empty_like(q)
        self._check(out, (self.B, self.Hq, self.d), "out")
        if gate is None:
            self._call("bct_decode_step", _dptr(q), _dptr(k_new), _dptr(v_new), _dptr(out))
        else:
            self._call("bct_decode_step_gated", _dptr(q), _dptr(k_new), _dptr(v_new), _dptr(gate), _dptr(out))
        return out

    def decode_step_keyed(self, q, k_new, v_new, key_new, out=None, gate=None, key_gate=None):
        """bct_decode_step_keyed: the write also moves the (per-sequence) keys after the token's read.
        key_new: [B][Hkv][d]; gate / key_gate: float32 [B][Hkv] or None."""
        torch = _torch()
        self._check_gate(gate, (self.B, self.Hkv))
        self._check_gate(key_gate, (self.B, self.Hkv))
        self._check(q, (self.B, self.Hq, self.d), "q")
        for t, n in ((k_new, "k_new"), (v_new, "v_new"), (key_new, "key_new")):
            self._check(t, (self.B, self.Hkv, self.d), n)
        if q is not None and out is None:
            out = torch.empty_like(q)
        self._check(out, (self.B, self.Hq, self.d), "out")
        self._call("bct_decode_step_keyed", _dptr(q), _dptr(k_new), _dptr(v_new), _dptr(key_new), _dptr(gate),
                   _dptr(key_gate), _dptr(out))
        return out

    def decode_step_static(self, q, k_new, v_new, out):
        """bct_decode_step_static: the caller passes every buffer, out included (None for a write-only step)."""
        self._check(q, (self.B, self.Hq, self.d), "q")
        self._check(k_new, (self.B, self.Hkv, self.d), "k_new")
        self._check(v_new, (self.B, self.Hkv, self.d), "v_new")
        self._check(out, (self.B, self.Hq, self.d), "out")
        self._call("bct_decode_step_static", _dptr(q), _dptr(k_new), _dptr(v_new), _dptr(out))
        return out

    def prefill(self, q, k_new, v_new, T, out=None, gate=None):
        """A chunk of T tokens per sequence; tensors are [B][T][H][d]; gate float32 [B][T][Hkv] or None."""
        torch = _torch()
        self._check_gate(gate, (self.B, T, self.Hkv))
        self._check(q, (self.B, T, self.Hq, self.d), "q")
        self._check(k_new, (self.B, T, self.Hkv, self.d), "k_new")
        self._check(v_new, (self.B, T, self.Hkv, self.d), "v_new")
        if q is not None and out is None:
            out = torch.empty_like(q)
        self._check(out, (self.B, T, self.Hq, self.d), "out")
        torch = _torch()
        with torch.cuda.device(self.device):
            if gate is None:
                st = lib().bct_prefill(self._h, _dptr(q), _dptr(k_new), _dptr(v_new), T, _dptr(out), _stream_ptr())
            else:
                st = lib().bct_prefill_gated(self._h, _dptr(q), _dptr(k_new), _dptr(v_new), _dptr(gate), T,
                                             _dptr(out), _stream_ptr())
        if st != BCT_OK:
            raise BctError(st, "bct_prefill")
        return out

    def export(self):
        """-> (mk, mv, steps) as fresh tensors."""
        torch = _torch()
        mk = torch.empty(self.keys_shape, dtype=self.torch_dtype, device=self.device)
        mv = torch.empty(self.values_shape, dtype=self.torch_dtype, device=self.device)
        st = ctypes.c_uint64()
        with torch.cuda.device(self.device):
            rc = lib().bct_cache_export(self._h, _dptr(mk), _dptr(mv), ctypes.byref(st), _stream_ptr())
        if rc != BCT_OK:
            raise BctError(rc, "bct_cache_export")
        return mk, mv, st.value

    def import_(self, mk, mv, steps):
        self._check(mk, self.keys_shape, "mk")
        self._check(mv, self.values_shape, "mv")
        torch = _torch()
        with torch.cuda.device(self.device):
            rc = lib().bct_cache_import(self._h, _dptr(mk), _dptr(mv), steps, _stream_ptr())
        if rc != BCT_OK:
            raise BctError(rc, "bct_cache_import")

    @property
    def steps(self):
        st = ctypes.c_uint64()
        rc = lib().bct_cache_steps(self._h, ctypes.byref(st))
        if rc != BCT_OK:
            raise BctError(rc, "bct_cache_steps")
        return st.value

    def _region(self, which):
        torch = _torch()
        mk, mv = ctypes.c_void_p(), ctypes.c_void_p()
        mkb, mvb = ctypes.c_size_t(), ctypes.c_size_t()
        rc = lib().bct_cache_regions(self._h, ctypes.byref(mk), ctypes.byref(mkb), ctypes.byref(mv),
                                     ctypes.byref(mvb))
        if rc != BCT_OK:
            raise BctError(rc, "bct_cache_regions")
        base = self._cache_mem.data_ptr()
        ptr, nb, shape = (mk.value, mkb.value, self.keys_shape) if which == "mk" else \
            (mv.value, mvb.value, self.values_shape)
        off = ptr - base
        return self._cache_mem[off:off + nb].view(self.torch_dtype).view(shape)

    def profile_enable(self, n_steps):
        rc = lib().bct_profile_enable(self._h, n_steps)
        if rc != BCT_OK:
            raise BctError(rc, "bct_profile_enable")

    def profile_read(self):
        """-> (n_recorded, ms_scores, ms_mv_pass, ms_merge): mean per-launch durations."""
        n = ctypes.c_uint32()
        a, b, c = ctypes.c_float(), ctypes.c_float(), ctypes.c_float()
        rc = lib().bct_profile_read(self._h, ctypes.byref(n), ctypes.byref(a), ctypes.byref(b), ctypes.byref(c))
        if rc != BCT_OK:
            raise BctError(rc, "bct_profile_read")
        return n.value, a.value, b.value, c.value

    def keys_view(self):
        """Zero-copy view of MK inside the cache memory (read it, do not write it)."""
        return self._region("mk")

    def values_view(self):
        """Zero-copy view of MV inside the cache memory."""
        return self._region("mv")
