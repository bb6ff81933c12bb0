"""Python face of the CPU oracle (oracle/fs_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, ``__graft_entry__.smoke()``
and the ``cpu_baseline`` leg of ``bench.py``.  The product package never imports
this module, and this module never imports the product package.

The C file is compiled with gcc into ``oracle/libfs_oracle.so``; ``build()``
does that, ``load()`` builds only when the library is missing.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

FP16, FP8, INT8, INT4 = 0, 1, 2, 3
OK, ERR_INVALID, ERR_NOMEM, ERR_STATE = 0, -1, -2, -3
FREE, PARTIAL, FULL = 0, 1, 2

_DIR = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_DIR, "libfs_oracle.so")
_LIB = None


class Geom(ctypes.Structure):
    _fields_ = [("dtype", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("n_layers", ctypes.c_int32), ("tokens_per_block", ctypes.c_int32), ("param_bytes", ctypes.c_int32),
                ("block_budget", ctypes.c_uint64), ("row_bytes", ctypes.c_uint64), ("kv_tile", ctypes.c_uint64),
                ("par_tile", ctypes.c_uint64), ("head_chunk", ctypes.c_uint64), ("layer_bytes", ctypes.c_uint64),
                ("block_bytes", ctypes.c_uint64)]


def build() -> str:
    """Compile the oracle with gcc (always recompiles)."""
    src = os.path.join(_DIR, "fs_oracle.c")
    cmd = ["gcc", "-std=c11", "-O2", "-ffp-contract=off", "-fPIC", "-shared", "-pthread", "-Wall", "-Wextra",
           "-o", _SO, src, "-lm"]
    subprocess.run(cmd, check=True)
    global _LIB
    _LIB = None
    return _SO


def load():
    global _LIB
    if _LIB is not None:
        return _LIB
    if not os.path.exists(_SO):
        build()
    L = ctypes.CDLL(_SO)
    vp, i32, i64, u64, dbl = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_uint64, ctypes.c_double
    gp = ctypes.POINTER(Geom)
    L.fso_geometry.restype = i32
    L.fso_geometry.argtypes = [i32, i32, i32, i32, u64, gp]
    for name in ("fso_row_offset", "fso_param_offset"):
        f = getattr(L, name)
        f.restype = u64
        f.argtypes = [gp, ctypes.c_int32, i32, i32, i32, i32]
    L.fso_block_bytes.restype = u64
    L.fso_block_bytes.argtypes = [i32, i32, i32, i32, i32]
    L.fso_lcm_slab_bytes.restype = u64
    L.fso_lcm_slab_bytes.argtypes = [vp, i32, u64]
    L.fso_block_offset.restype = u64
    L.fso_block_offset.argtypes = [gp, ctypes.c_int32]
    L.fso_pool_new.restype = vp
    L.fso_pool_new.argtypes = [u64, u64]
    L.fso_pool_delete.restype = None
    L.fso_pool_delete.argtypes = [vp]
    L.fso_model_add.restype = i32
    L.fso_model_add.argtypes = [vp, i32, i32, i32, i32, u64]
    L.fso_model_add_tokens.restype = i32
    L.fso_model_add_tokens.argtypes = [vp, i32, i32, i32, i32, i32]
    L.fso_model_remove.restype = i32
    L.fso_model_remove.argtypes = [vp, i32]
    L.fso_model_geometry.restype = i32
    L.fso_model_geometry.argtypes = [vp, i32, gp]
    L.fso_block_alloc.restype = i32
    L.fso_block_alloc.argtypes = [vp, i32, ctypes.POINTER(ctypes.c_int32)]
    L.fso_block_free.restype = i32
    L.fso_block_free.argtypes = [vp, i32, ctypes.c_int32]
    for name in ("fso_pool_n_slabs", "fso_pool_n_free"):
        f = getattr(L, name)
        f.restype = i64
        f.argtypes = [vp]
    for name in ("fso_model_live_blocks", "fso_model_blocks_per_slab"):
        f = getattr(L, name)
        f.restype = i64
        f.argtypes = [vp, i32]
    L.fso_pool_dump.restype = None
    L.fso_pool_dump.argtypes = [vp, vp, vp, vp, vp]
    L.fso_model_dump_live.restype = None
    L.fso_model_dump_live.argtypes = [vp, i32, vp]
    L.fso_f16_to_f32.restype = ctypes.c_float
    L.fso_f16_to_f32.argtypes = [ctypes.c_uint16]
    L.fso_f32_to_f16.restype = ctypes.c_uint16
    L.fso_f32_to_f16.argtypes = [ctypes.c_float]
    L.fso_e4m3_decode.restype = ctypes.c_float
    L.fso_e4m3_decode.argtypes = [ctypes.c_uint8]
    L.fso_e4m3_encode.restype = ctypes.c_uint8
    L.fso_e4m3_encode.argtypes = [ctypes.c_float]
    L.fso_quant_row_int8.restype = None
    L.fso_quant_row_int8.argtypes = [vp, i32, vp, vp]
    L.fso_quant_row_int4.restype = None
    L.fso_quant_row_int4.argtypes = [vp, i32, vp, vp, vp]
    L.fso_kv_append.restype = i32
    L.fso_kv_append.argtypes = [vp, gp, i32, vp, vp, i32, vp, vp, vp, i32, i64, vp, vp]
    L.fso_dequant_sequence.restype = i32
    L.fso_dequant_sequence.argtypes = [vp, gp, i32, vp, i32, vp, vp, vp, vp]
    L.fso_prefill_attention.restype = i32
    L.fso_prefill_attention.argtypes = [vp, gp, i32, i32, dbl, vp, vp, vp, vp, i32, i32, vp, vp, vp, vp, i32]
    L.fso_decode_attention.restype = i32
    L.fso_decode_attention.argtypes = [vp, gp, i32, i32, dbl, vp, vp, vp, i32, i32, vp, vp, vp, vp, i32]
    _LIB = L
    return L


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


# --------------------------------------------------------------------------- geometry
def geometry(dtype, n_kv_heads, head_dim, n_layers, block_budget) -> Geom:
    g = Geom()
    rc = load().fso_geometry(dtype, n_kv_heads, head_dim, n_layers, block_budget, ctypes.byref(g))
    if rc != OK:
        raise ValueError(f"fso_geometry failed: {rc}")
    return g


def block_bytes(dtype, n_kv_heads, head_dim, n_layers, tokens_per_block) -> int:
    """Sec. 3.2, forward: bytes of the laid-out block holding tokens_per_block tokens (0: invalid)."""
    return load().fso_block_bytes(dtype, n_kv_heads, head_dim, n_layers, tokens_per_block)


def lcm_slab_bytes(block_sizes, min_slab=0) -> int:
    """Sec. 5.2: smallest multiple of the lcm of the block sizes that is >= min_slab (0: invalid or > 2^40)."""
    a = np.ascontiguousarray(block_sizes, dtype=np.uint64)
    return load().fso_lcm_slab_bytes(a.ctypes.data_as(ctypes.c_void_p), len(a), int(min_slab))


def row_offset(g, blk, layer, head, which, tok) -> int:
    return load().fso_row_offset(ctypes.byref(g), blk, layer, head, which, tok)


def param_offset(g, blk, layer, head, which, tok) -> int:
    return load().fso_param_offset(ctypes.byref(g), blk, layer, head, which, tok)


def block_offset(g, blk) -> int:
    return load().fso_block_offset(ctypes.byref(g), blk)


# --------------------------------------------------------------------------- allocator
class Pool:
    """Slab table of one shared KV tensor (bookkeeping only; memory is passed separately)."""

    def __init__(self, slab_bytes: int, pool_bytes: int):
        self._L = load()
        self._p = self._L.fso_pool_new(slab_bytes, pool_bytes)
        if not self._p:
            raise ValueError("fso_pool_new failed")
        self.slab_bytes, self.pool_bytes = slab_bytes, pool_bytes

    def __del__(self):
        if getattr(self, "_p", None):
            self._L.fso_pool_delete(self._p)
            self._p = None

    def model_add(self, dtype, n_kv_heads, head_dim, n_layers, block_budget=None) -> int:
        return self._L.fso_model_add(self._p, dtype, n_kv_heads, head_dim, n_layers,
                                     self.slab_bytes if block_budget is None else block_budget)

    def model_add_tokens(self, dtype, n_kv_heads, head_dim, n_layers, tokens_per_block) -> int:
        """The paper's direction (Sec. 3.2 / 5.2): exactly tokens_per_block tokens per block."""
        return self._L.fso_model_add_tokens(self._p, dtype, n_kv_heads, head_dim, n_layers, tokens_per_block)

    def model_remove(self, model) -> int:
        return self._L.fso_model_remove(self._p, model)

    def model_geometry(self, model) -> Geom:
        g = Geom()
        rc = self._L.fso_model_geometry(self._p, model, ctypes.byref(g))
        if rc != OK:
            raise ValueError(f"fso_model_geometry failed: {rc}")
        return g

    def alloc(self, model):
        """Returns (rc, blk_id)."""
        out = ctypes.c_int32(-1)
        rc = self._L.fso_block_alloc(self._p, model, ctypes.byref(out))
        return rc, out.value

    def free(self, model, blk) -> int:
        return self._L.fso_block_free(self._p, model, blk)

    @property
    def n_slabs(self):
        return self._L.fso_pool_n_slabs(self._p)

    @property
    def n_free(self):
        return self._L.fso_pool_n_free(self._p)

    def live_blocks(self, model):
        return self._L.fso_model_live_blocks(self._p, model)

    def blocks_per_slab(self, model):
        return self._L.fso_model_blocks_per_slab(self._p, model)

    def dump(self):
        n = self.n_slabs
        state = np.empty(n, np.int32)
        key = np.empty(n, np.int32)
        used = np.empty(n, np.int32)
        fs = np.empty(max(self.n_free, 1), np.int32)
        self._L.fso_pool_dump(self._p, _ptr(state), _ptr(key), _ptr(used), _ptr(fs))
        return state, key, used, fs[: self.n_free].copy()

    def dump_live(self, model):
        live = np.empty(self.n_slabs * self.blocks_per_slab(model), np.uint8)
        self._L.fso_model_dump_live(self._p, model, _ptr(live))
        return live


# --------------------------------------------------------------------------- formats
def f16_to_f32(h: int) -> float:
    return load().fso_f16_to_f32(h)


def f32_to_f16(x: float) -> int:
    return load().fso_f32_to_f16(x)


def e4m3_decode(b: int) -> float:
    return load().fso_e4m3_decode(b)


def e4m3_encode(y: float) -> int:
    return load().fso_e4m3_encode(y)


def quant_row_int8(x):
    x = _c(x, np.float32)
    q = np.empty(x.shape[0], np.int8)
    s = np.empty(1, np.uint16)
    load().fso_quant_row_int8(_ptr(x), x.shape[0], _ptr(q), _ptr(s))
    return q, int(s[0])


def quant_row_int4(x):
    x = _c(x, np.float32)
    q = np.empty(x.shape[0] // 2, np.uint8)
    s = np.empty(1, np.uint16)
    z = np.empty(1, np.uint16)
    load().fso_quant_row_int4(_ptr(x), x.shape[0], _ptr(q), _ptr(s), _ptr(z))
    return q, int(s[0]), int(z[0])


# --------------------------------------------------------------------------- append / attention
def kv_append(pool_mem, g, layer, k_new, v_new, seq_idx, pos, block_tables, k_scale=None, v_scale=None):
    """pool_mem: uint8 numpy mirror of the pool; k_new/v_new: [n][H][D] float16 or float32."""
    assert pool_mem.dtype == np.uint8 and pool_mem.flags.c_contiguous
    k_new = np.ascontiguousarray(k_new)
    v_new = np.ascontiguousarray(v_new)
    assert k_new.dtype == v_new.dtype and k_new.dtype in (np.float16, np.float32)
    seq_idx = _c(seq_idx, np.int32)
    pos = _c(pos, np.int32)
    block_tables = _c(block_tables, np.int32)
    assert block_tables.ndim == 2
    ks = None if k_scale is None else _c(k_scale, np.float32)
    vs = None if v_scale is None else _c(v_scale, np.float32)
    rc = load().fso_kv_append(_ptr(pool_mem), ctypes.byref(g), layer, _ptr(k_new), _ptr(v_new),
                              int(k_new.dtype == np.float32), _ptr(seq_idx), _ptr(pos), _ptr(block_tables),
                              block_tables.shape[1], len(pos), _ptr(ks), _ptr(vs))
    if rc != OK:
        raise ValueError(f"fso_kv_append failed: {rc}")


def dequant_sequence(pool_mem, g, layer, block_table, n_tokens, k_scale=None, v_scale=None):
    """Dense float64 K^, V^ [n_tokens][H][D] of one sequence."""
    block_table = _c(block_table, np.int32)
    k = np.empty((n_tokens, g.n_kv_heads, g.head_dim), np.float64)
    v = np.empty_like(k)
    ks = None if k_scale is None else _c(k_scale, np.float32)
    vs = None if v_scale is None else _c(v_scale, np.float32)
    load().fso_dequant_sequence(_ptr(pool_mem), ctypes.byref(g), layer, _ptr(block_table), n_tokens, _ptr(ks),
                                _ptr(vs), _ptr(k), _ptr(v))
    return k, v


def decode_attention(pool_mem, g, layer, n_q_heads, sm_scale, q, block_tables, seq_lens, k_scale=None,
                     v_scale=None, n_threads=1, want_lse=True):
    """Returns (out float64 [n_seq][n_q][D], lse float64 [n_seq][n_q] or None)."""
    q = np.ascontiguousarray(q)
    assert q.dtype == np.float16 and q.ndim == 3
    block_tables = _c(block_tables, np.int32)
    seq_lens = _c(seq_lens, np.int32)
    n_seq = len(seq_lens)
    out = np.empty((n_seq, n_q_heads, g.head_dim), np.float64)
    lse = np.empty((n_seq, n_q_heads), np.float64) if want_lse else None
    ks = None if k_scale is None else _c(k_scale, np.float32)
    vs = None if v_scale is None else _c(v_scale, np.float32)
    rc = load().fso_decode_attention(_ptr(pool_mem), ctypes.byref(g), layer, n_q_heads, float(sm_scale),
                                     _ptr(q.view(np.uint16)), _ptr(block_tables), _ptr(seq_lens), n_seq,
                                     block_tables.shape[1], _ptr(ks), _ptr(vs), _ptr(out), _ptr(lse), n_threads)
    if rc != OK:
        raise ValueError(f"fso_decode_attention failed: {rc}")
    return out, lse


def prefill_attention(pool_mem, g, layer, n_q_heads, sm_scale, q, block_tables, seq_lens, q_offsets, k_scale=None,
                      v_scale=None, n_threads=1, want_lse=True):
    """Chunked-prefill attention (Sec. 2.1): q [n_rows][n_q][D] fp16, the chunks of the sequences one after the
    other (q_offsets [n_seq + 1]); row r of sequence b stands at position seq_lens[b] - n_b + r.
    Returns (out float64 [n_rows][n_q][D], lse float64 [n_rows][n_q] or None)."""
    q = np.ascontiguousarray(q)
    assert q.dtype == np.float16 and q.ndim == 3
    block_tables = _c(block_tables, np.int32)
    seq_lens = _c(seq_lens, np.int32)
    q_offsets = _c(q_offsets, np.int32)
    n_seq = len(seq_lens)
    assert len(q_offsets) == n_seq + 1 and int(q_offsets[-1]) == q.shape[0]
    out = np.empty((q.shape[0], n_q_heads, g.head_dim), np.float64)
    lse = np.empty((q.shape[0], n_q_heads), np.float64) if want_lse else None
    ks = None if k_scale is None else _c(k_scale, np.float32)
    vs = None if v_scale is None else _c(v_scale, np.float32)
    rc = load().fso_prefill_attention(_ptr(pool_mem), ctypes.byref(g), layer, n_q_heads, float(sm_scale),
                                      _ptr(q.view(np.uint16)), _ptr(block_tables), _ptr(seq_lens), _ptr(q_offsets),
                                      n_seq, block_tables.shape[1], _ptr(ks), _ptr(vs), _ptr(out), _ptr(lse), n_threads)
    if rc != OK:
        raise ValueError(f"fso_prefill_attention failed: {rc}")
    return out, lse
