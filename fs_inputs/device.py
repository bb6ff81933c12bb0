"""ctypes driver of the device-side input generator (libfs_inputs.so).

Used by GPU tests and the benchmark to materialise source K/V rows directly in
HBM.  torch is used only to own device memory and to name the stream.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np
import torch  # noqa: F401  -- first, so that libfs_inputs.so binds to the HIP runtime torch has already loaded

from . import gen

_LIB = None
_TABLES = {}


def lib_path() -> str:
    return os.path.join(os.path.dirname(os.path.abspath(__file__)), "libfs_inputs.so")


def _lib():
    global _LIB
    if _LIB is None:
        path = lib_path()
        if not os.path.exists(path):
            raise RuntimeError(f"{path} is not built; run __graft_entry__.build() first")
        L = ctypes.CDLL(path)
        L.fsi_fill_rows.restype = ctypes.c_int
        L.fsi_fill_rows.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p, ctypes.c_uint64, ctypes.c_int,
                                    ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int,
                                    ctypes.c_int64, ctypes.c_void_p]
        _LIB = L
    return _LIB


def device_table(device="cuda:0"):
    """The inverse-normal table of gen.normal_table() resident on ``device``."""
    import torch

    key = str(device)
    if key not in _TABLES:
        _TABLES[key] = torch.from_numpy(np.array(gen.normal_table())).to(device)
    return _TABLES[key]


def fill_rows(out, seed: int, model: int, layer: int, which: int, seq_id, pos, n_heads: int, head_dim: int):
    """Fill ``out`` (torch fp16/fp32 [n_tokens][n_heads][head_dim], on the GPU) for tokens (seq_id[i], pos[i]).

    ``seq_id`` / ``pos`` are int32 device tensors of n_tokens entries.  Asynchronous on
    torch's current stream.
    """
    import torch

    n_tokens = int(seq_id.numel())
    assert out.is_cuda and seq_id.is_cuda and pos.is_cuda
    assert seq_id.dtype == torch.int32 and pos.dtype == torch.int32 and pos.numel() == n_tokens
    assert out.is_contiguous() and out.numel() == n_tokens * n_heads * head_dim
    assert out.dtype in (torch.float16, torch.float32)
    tab = device_table(out.device)
    rc = _lib().fsi_fill_rows(out.data_ptr(), int(out.dtype == torch.float32), tab.data_ptr(), seed, model, layer,
                              which, seq_id.data_ptr(), pos.data_ptr(), n_heads * head_dim, n_tokens,
                              torch.cuda.current_stream(out.device).cuda_stream)
    if rc != 0:
        raise RuntimeError(f"fsi_fill_rows failed with code {rc}")
    return out
