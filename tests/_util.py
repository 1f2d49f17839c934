"""Helpers shared by the GPU parity tests: host<->device transfer of storage
arrays (bf16 as uint16 bit patterns on the host) and error measures."""
import math

import numpy as np

import bct_synth as syn


def torch_dtype(dtype):
    import torch
    return {"f32": torch.float32, "bf16": torch.bfloat16}[dtype]


def to_dev(a, dtype, device="cuda:0"):
    """numpy storage array (float32, or uint16 bf16 bits) -> device tensor."""
    import torch
    if a is None:
        return None
    a = np.ascontiguousarray(a)
    if dtype == "f32":
        return torch.from_numpy(a).to(device)
    return torch.from_numpy(a.view(np.int16)).to(device).view(torch.bfloat16)


def to_np(t, dtype):
    """device tensor -> numpy storage array (float32, or uint16 bits)."""
    import torch
    if t is None:
        return None
    if dtype == "f32":
        return t.detach().cpu().numpy()
    return t.detach().view(torch.int16).cpu().numpy().view(np.uint16)


def f64(a, dtype):
    return syn.unpack(a, dtype)


def rel_normwise(got, ref):
    """max over leading vectors of max_j|g-r| / max_j|r| (last axis = vector)."""
    num = np.max(np.abs(got - ref), axis=-1)
    den = np.maximum(np.max(np.abs(ref), axis=-1), 1e-30)
    return float(np.max(num / den))


def bf16_ulp(ref):
    """Spacing of bf16 numbers at |ref| (8 significand bits), floored at the smallest normal."""
    a = np.maximum(np.abs(ref), 2.0 ** -126)
    return 2.0 ** (np.floor(np.log2(a)) - 7)


def make_pair(w, ref_cls, gpu_cls, *, flags=0, read_scale=None, write_scale=None, mv0=False, layer=0,
              max_prefill_T=0, batch_subset=None):
    """Builds an oracle cache and a GPU cache of workload shape `w` holding the same MK (and MV_0).
    batch_subset: list of batch indices the ORACLE holds (the GPU always holds the whole batch)."""
    rs = w.scale if read_scale is None else read_scale
    ws = w.scale if write_scale is None else write_scale
    per_seq = bool(flags & 1)
    mk = syn.make_keys(w, layer, per_sequence=per_seq)
    mv = syn.make_values0(w, layer) if mv0 else None
    g = gpu_cls(w.M, w.B, w.Hq, w.Hkv, w.d, torch_dtype(w.dtype), rs, ws, flags, max_prefill_T)
    g.set_keys(to_dev(mk, w.dtype))
    if mv0:
        g.set_values(to_dev(mv, w.dtype))
    bs = list(range(w.B)) if batch_subset is None else list(batch_subset)
    r = ref_cls(w.M, len(bs), w.Hq, w.Hkv, w.d, w.dtype, rs, ws, flags & 1)   # bit 1 is a GPU-side choice of path
    r.set_keys(np.ascontiguousarray(mk[bs]) if per_seq else mk)
    if mv0:
        r.set_values(np.ascontiguousarray(mv[bs]))
    return r, g, mk, mv, bs


def sub(a, bs):
    return None if a is None else np.ascontiguousarray(a[bs])
