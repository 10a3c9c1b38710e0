"""Device-side fills of the synthetic tensors (same values as the host generator)."""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

from . import (BF16, MoEConfig, scale_f32, stream_key, tensor_dtype, tensor_shape, tensor_sigma)

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "fill.hip")
_LIB = os.path.join(_HERE, "libmoe_inputs_fill.so")
_lib = None


def build(force: bool = False) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = [os.environ.get("HIPCC", "/opt/rocm/bin/hipcc"), "--offload-arch=gfx950", "-O3", "-fPIC", "-shared",
               "-ffp-contract=off", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
               "-Wno-unused-command-line-argument", _SRC, "-o", _LIB]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(r.stderr)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.moe_inputs_fill_normal.restype = ctypes.c_int
        _lib.moe_inputs_fill_normal.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_uint64, ctypes.c_uint64,
                                                ctypes.c_uint64, ctypes.c_float, ctypes.c_void_p]
    return _lib


def copy_bytes(dst, src):
    """Plain device-to-device copy kernel (the yardstick for HBM counters)."""
    import torch
    assert dst.is_cuda and src.is_cuda and dst.is_contiguous() and src.is_contiguous()
    nbytes = src.numel() * src.element_size()
    assert nbytes == dst.numel() * dst.element_size() and nbytes % 16 == 0
    lib = _load()
    lib.moe_inputs_copy.restype = ctypes.c_int
    lib.moe_inputs_copy.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_uint64, ctypes.c_void_p]
    if lib.moe_inputs_copy(dst.data_ptr(), src.data_ptr(), nbytes, torch.cuda.current_stream().cuda_stream) != 0:
        raise RuntimeError("copy kernel launch failed")


def stream_read(src, workgroups: int, row_bytes: int = 5760, panels: int = 64):
    """Read yardstick: `workgroups` workgroups each stream their own slice of the byte tensor `src` into LDS (rows
    of row_bytes, 16-byte buffer loads, 32 KB in flight per workgroup).  Returns the bytes read in total."""
    import torch
    assert src.is_cuda and src.is_contiguous() and src.dtype == torch.uint8
    region = (src.numel() // workgroups) & ~4095
    panels = min(panels, region // (4 * 32 * row_bytes))
    lib = _load()
    lib.moe_inputs_stream_read.restype = ctypes.c_int64
    lib.moe_inputs_stream_read.argtypes = [ctypes.c_void_p, ctypes.c_uint64, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                           ctypes.c_void_p]
    per = lib.moe_inputs_stream_read(src.data_ptr(), region, row_bytes, panels, workgroups,
                                     torch.cuda.current_stream().cuda_stream)
    if per <= 0:
        raise RuntimeError("stream_read: bad arguments or launch failure")
    return per * workgroups


def fill_normal(out, seed: int, stream: int, start: int, sigma: float):
    """Fills the contiguous device tensor `out` (bf16 or fp32) with flat elements
    [start, start + out.numel()) of the stream."""
    import torch
    assert out.is_cuda and out.is_contiguous()
    bf16 = 1 if out.dtype == torch.bfloat16 else 0
    assert bf16 or out.dtype == torch.float32
    rc = _load().moe_inputs_fill_normal(out.data_ptr(), bf16, int(stream_key(seed, stream)), start, out.numel(),
                                        float(scale_f32(sigma)), torch.cuda.current_stream().cuda_stream)
    if rc != 0:
        raise RuntimeError("fill kernel launch failed")
    return out


def device_tensor(cfg: MoEConfig, stream: int, first: int = 0, count: int | None = None, device="cuda:0"):
    """Slices [first, first+count) along the leading dimension, generated in HBM."""
    import torch
    shape = tensor_shape(cfg, stream)
    if count is None:
        count = shape[0] - first
    inner = int(np.prod(shape[1:], dtype=np.int64))
    dt = torch.bfloat16 if tensor_dtype(cfg, stream) == BF16 else torch.float32
    out = torch.empty((count,) + tuple(shape[1:]), dtype=dt, device=device)
    return fill_normal(out, cfg.seed, stream, first * inner, tensor_sigma(cfg, stream))


def to_device(a: np.ndarray, device="cuda:0"):
    """Host array from the host generator -> device tensor (uint16 = bf16 bit patterns)."""
    import torch
    t = torch.from_numpy(np.ascontiguousarray(a))
    if a.dtype == np.uint16:
        t = t.view(torch.bfloat16)
    return t.to(device)


def to_host(t) -> np.ndarray:
    """Device tensor -> host array (bf16 as uint16 bit patterns)."""
    import torch
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.uint16).numpy()
    return t.numpy()
