"""Thin ctypes binding of libfineserve.so: argument marshalling only.

Every function has the name and meaning of its C-ABI twin in include/fineserve.h.  Device
buffers are torch tensors (torch owns device memory and names the stream); nothing is computed
here.  Importing this module fails loudly when the HIP library has not been built -- there is no
CPU or PyTorch fallback.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np
import torch  # noqa: F401  -- first, so that libfineserve.so binds to the HIP runtime torch has already loaded

FS_KV_FP16, FS_KV_FP8_E4M3, FS_KV_INT8, FS_KV_INT4 = 0, 1, 2, 3
FS_SRC_FP16, FS_SRC_FP32 = 0, 1
FS_OK, FS_ERR_INVALID, FS_ERR_NOMEM, FS_ERR_STATE, FS_ERR_DEVICE = 0, -1, -2, -3, -4
FS_SLAB_FREE, FS_SLAB_PARTIAL, FS_SLAB_FULL = 0, 1, 2

_DIR = os.path.dirname(os.path.abspath(__file__))
# FINESERVE_LIBRARY: another build of the same library (bench_timeline.py sets it to the profiling twin)
LIB_PATH = os.environ.get("FINESERVE_LIBRARY") or os.path.join(_DIR, "libfineserve.so")

EXPORTS = ["fs_pool_create", "fs_pool_destroy", "fs_pool_base", "fs_model_register", "fs_model_register_ex",
           "fs_block_bytes", "fs_slab_bytes_for_blocks", "fs_model_register_tokens",
           "fs_model_set_fp8_scales", "fs_model_unregister", "fs_model_geometry", "fs_block_alloc", "fs_block_free",
           "fs_blocks_alloc", "fs_blocks_free",
           "fs_pool_stats", "fs_pool_dump", "fs_model_dump_live", "fs_kv_append", "fs_kv_append_multi", "fs_decode_step_multi",
           "fs_decode_workspace_bytes",
           "fs_decode_attention", "fs_decode_attention_multi", "fs_decode_attention_multi_static", "fs_decode_status", "fs_prefill_workspace_bytes",
           "fs_prefill_attention", "fs_sched_select_batch", "fs_sched_place_models", "fs_model_stats", "fs_pool_set_option",
           "fs_pool_get_option", "fs_pool_last_attention_kernel_ms", "fs_last_error"]

(FS_OPT_DECODE_KERNEL, FS_OPT_SPLIT_BYTES, FS_OPT_KERNEL_TIMING, FS_OPT_PREFILL_COLUMN_BLOCKS, FS_OPT_PREFILL_WAVES,
 FS_OPT_PREFILL_PIPELINED, FS_OPT_PREFILL_STAGED_DEQUANT, FS_OPT_LAST_PREFILL_KERNEL) = range(8)


class fs_geometry_t(ctypes.Structure):
    _fields_ = [("kv_dtype", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("n_layers", ctypes.c_int32), ("tokens_per_block", ctypes.c_int32), ("param_bytes", ctypes.c_int32),
                ("blocks_per_slab", ctypes.c_int32), ("reserved", ctypes.c_int32), ("block_budget", ctypes.c_uint64),
                ("row_bytes", ctypes.c_uint64), ("kv_tile", ctypes.c_uint64), ("par_tile", ctypes.c_uint64),
                ("head_chunk", ctypes.c_uint64), ("layer_bytes", ctypes.c_uint64), ("block_bytes", ctypes.c_uint64)]


class fs_pool_stats_t(ctypes.Structure):
    _fields_ = [("n_slabs", ctypes.c_int64), ("slabs_free", ctypes.c_int64), ("slabs_partial", ctypes.c_int64),
                ("slabs_full", ctypes.c_int64), ("live_blocks", ctypes.c_int64), ("n_models", ctypes.c_int64),
                ("stranded_bytes", ctypes.c_uint64)]


class fs_model_stats_t(ctypes.Structure):
    _fields_ = [("slabs_partial", ctypes.c_int64), ("slabs_full", ctypes.c_int64), ("live_blocks", ctypes.c_int64),
                ("free_blocks_in_partial_slabs", ctypes.c_int64), ("live_bytes", ctypes.c_uint64),
                ("stranded_bytes", ctypes.c_uint64)]


class fs_append_t(ctypes.Structure):
    _fields_ = [("model", ctypes.c_int32), ("layer", ctypes.c_int32), ("src_dtype", ctypes.c_int32),
                ("max_blocks", ctypes.c_int32), ("k_new", ctypes.c_void_p), ("v_new", ctypes.c_void_p),
                ("seq_idx", ctypes.c_void_p), ("pos", ctypes.c_void_p), ("block_tables", ctypes.c_void_p),
                ("n_tokens", ctypes.c_int64)]


class fs_batch_t(ctypes.Structure):
    _fields_ = [("model", ctypes.c_int32), ("layer", ctypes.c_int32), ("n_q_heads", ctypes.c_int32),
                ("sm_scale", ctypes.c_float), ("q", ctypes.c_void_p), ("block_tables", ctypes.c_void_p),
                ("seq_lens", ctypes.c_void_p), ("seq_lens_host", ctypes.c_void_p), ("n_seq", ctypes.c_int32),
                ("max_blocks", ctypes.c_int32), ("out", ctypes.c_void_p), ("lse", ctypes.c_void_p)]


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with __graft_entry__.build() "
                          "(python paper_2509_06261_amd/build.py); there is no fallback path")
    L = ctypes.CDLL(LIB_PATH)
    vp, i32, i64, u64, f32 = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_uint64, ctypes.c_float
    pi32 = ctypes.POINTER(ctypes.c_int32)
    sig = {
        "fs_pool_create": (i32, [u64, u64, vp, ctypes.POINTER(vp)]),
        "fs_pool_destroy": (i32, [vp]),
        "fs_pool_base": (vp, [vp]),
        "fs_model_register": (i32, [vp, i32, i32, i32, i32, pi32]),
        "fs_model_register_ex": (i32, [vp, i32, i32, i32, i32, u64, pi32]),
        "fs_block_bytes": (u64, [i32, i32, i32, i32, i32]),
        "fs_slab_bytes_for_blocks": (u64, [vp, i32, u64]),
        "fs_model_register_tokens": (i32, [vp, i32, i32, i32, i32, i32, pi32]),
        "fs_model_set_fp8_scales": (i32, [vp, i32, vp, vp]),
        "fs_model_unregister": (i32, [vp, i32]),
        "fs_model_geometry": (i32, [vp, i32, ctypes.POINTER(fs_geometry_t)]),
        "fs_block_alloc": (i32, [vp, i32, pi32]),
        "fs_block_free": (i32, [vp, i32, ctypes.c_int32]),
        "fs_blocks_alloc": (i32, [vp, i32, i32, vp]),
        "fs_blocks_free": (i32, [vp, i32, vp, i32]),
        "fs_pool_stats": (i32, [vp, ctypes.POINTER(fs_pool_stats_t)]),
        "fs_pool_dump": (i32, [vp, vp, vp, vp, vp, ctypes.POINTER(ctypes.c_int64)]),
        "fs_model_dump_live": (i32, [vp, i32, vp]),
        "fs_kv_append": (i32, [vp, i32, i32, vp, vp, i32, vp, vp, vp, i32, i64, vp]),
        "fs_kv_append_multi": (i32, [vp, ctypes.POINTER(fs_append_t), i32, vp]),
        "fs_decode_step_multi": (i32, [vp, ctypes.POINTER(fs_append_t), i32, ctypes.POINTER(fs_batch_t), i32, vp, u64, vp]),
        "fs_decode_workspace_bytes": (u64, [vp, ctypes.POINTER(fs_batch_t), i32]),
        "fs_decode_attention": (i32, [vp, i32, i32, i32, f32, vp, vp, vp, i32, i32, vp, vp, vp, u64, vp]),
        "fs_decode_attention_multi": (i32, [vp, ctypes.POINTER(fs_batch_t), i32, vp, u64, vp]),
        "fs_decode_attention_multi_static": (i32, [vp, ctypes.POINTER(fs_batch_t), i32, vp, vp]),
        "fs_decode_status": (i32, [vp, vp]),
        "fs_prefill_workspace_bytes": (u64, [i32]),
        "fs_prefill_attention": (i32, [vp, i32, i32, i32, ctypes.c_float, vp, vp, vp, vp, vp, i32, i32, vp, vp, vp, u64, vp]),
        "fs_sched_select_batch": (i32, [vp, i32, vp, ctypes.c_double, vp, vp, vp, vp]),
        "fs_sched_place_models": (i32, [vp, vp, i32, vp, i32, vp]),
        "fs_model_stats": (i32, [vp, i32, ctypes.POINTER(fs_model_stats_t)]),
        "fs_pool_set_option": (i32, [vp, i32, i64]),
        "fs_pool_get_option": (i32, [vp, i32, ctypes.POINTER(ctypes.c_int64)]),
        "fs_pool_last_attention_kernel_ms": (f32, [vp]),
        "fs_last_error": (ctypes.c_char_p, []),
    }
    for name, (res, args) in sig.items():
        f = getattr(L, name)
        f.restype = res
        f.argtypes = args
    return L


_L = _load()


class FsError(RuntimeError):
    def __init__(self, code, where):
        self.code = code
        msg = _L.fs_last_error()
        super().__init__(f"{where} failed with {code}: {msg.decode() if msg else ''}")


def _dp(t):
    """Device (or host) address of a torch tensor / numpy array / None."""
    if t is None:
        return None
    if isinstance(t, np.ndarray):
        return t.ctypes.data
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    return getattr(stream, "cuda_stream", stream)


def fs_last_error() -> str:
    m = _L.fs_last_error()
    return m.decode() if m else ""


# ------------------------------------------------------------------ pool / models / blocks
def fs_pool_create(slab_bytes: int, pool_bytes: int, device_base=None):
    """device_base: a torch uint8 CUDA tensor of pool_bytes bytes (kept alive by the caller), a raw
    address, or None to let the library allocate."""
    out = ctypes.c_void_p()
    base = device_base if isinstance(device_base, (int, type(None))) else _dp(device_base)
    rc = _L.fs_pool_create(slab_bytes, pool_bytes, base, ctypes.byref(out))
    if rc != FS_OK:
        raise FsError(rc, "fs_pool_create")
    return out


def fs_pool_destroy(pool):
    return _L.fs_pool_destroy(pool)


def fs_pool_base(pool) -> int:
    return _L.fs_pool_base(pool)


def fs_model_register(pool, kv_dtype, n_kv_heads, head_dim, n_layers, block_budget_bytes=None):
    """Returns (tokens_per_block, model); block_budget_bytes selects fs_model_register_ex."""
    m = ctypes.c_int32(-1)
    if block_budget_bytes is None:
        rc = _L.fs_model_register(pool, kv_dtype, n_kv_heads, head_dim, n_layers, ctypes.byref(m))
    else:
        rc = _L.fs_model_register_ex(pool, kv_dtype, n_kv_heads, head_dim, n_layers, block_budget_bytes,
                                     ctypes.byref(m))
    if rc < 0:
        raise FsError(rc, "fs_model_register")
    return rc, m.value


def fs_block_bytes(kv_dtype, n_kv_heads, head_dim, n_layers, tokens_per_block) -> int:
    return _L.fs_block_bytes(kv_dtype, n_kv_heads, head_dim, n_layers, tokens_per_block)


def fs_slab_bytes_for_blocks(block_bytes, min_slab_bytes=0) -> int:
    a = np.ascontiguousarray(block_bytes, dtype=np.uint64)
    return _L.fs_slab_bytes_for_blocks(a.ctypes.data, len(a), int(min_slab_bytes))


def fs_model_register_tokens(pool, kv_dtype, n_kv_heads, head_dim, n_layers, tokens_per_block):
    """Returns (tokens_per_block, model)."""
    m = ctypes.c_int32(-1)
    rc = _L.fs_model_register_tokens(pool, kv_dtype, n_kv_heads, head_dim, n_layers, tokens_per_block, ctypes.byref(m))
    if rc < 0:
        raise FsError(rc, "fs_model_register_tokens")
    return rc, m.value


def fs_model_set_fp8_scales(pool, model, k_scale, v_scale):
    k = np.ascontiguousarray(k_scale, dtype=np.float32)
    v = np.ascontiguousarray(v_scale, dtype=np.float32)
    rc = _L.fs_model_set_fp8_scales(pool, model, k.ctypes.data, v.ctypes.data)
    if rc != FS_OK:
        raise FsError(rc, "fs_model_set_fp8_scales")


def fs_model_unregister(pool, model) -> int:
    return _L.fs_model_unregister(pool, model)


def fs_model_geometry(pool, model) -> fs_geometry_t:
    g = fs_geometry_t()
    rc = _L.fs_model_geometry(pool, model, ctypes.byref(g))
    if rc != FS_OK:
        raise FsError(rc, "fs_model_geometry")
    return g


def fs_block_alloc(pool, model):
    """Returns (rc, blk_id)."""
    out = ctypes.c_int32(-1)
    rc = _L.fs_block_alloc(pool, model, ctypes.byref(out))
    return rc, out.value


def fs_block_free(pool, model, blk_id) -> int:
    return _L.fs_block_free(pool, model, blk_id)


def fs_blocks_alloc(pool, model, n: int):
    """Returns (rc, ids): ids is an int32 numpy array of n block ids (meaningless unless rc == FS_OK)."""
    ids = np.empty(max(int(n), 1), dtype=np.int32)
    rc = _L.fs_blocks_alloc(pool, model, int(n), ids.ctypes.data)
    return rc, ids[:max(int(n), 0)]


def fs_blocks_free(pool, model, ids) -> int:
    ids = np.ascontiguousarray(ids, dtype=np.int32)
    return _L.fs_blocks_free(pool, model, ids.ctypes.data, len(ids))


def fs_pool_stats(pool) -> fs_pool_stats_t:
    s = fs_pool_stats_t()
    rc = _L.fs_pool_stats(pool, ctypes.byref(s))
    if rc != FS_OK:
        raise FsError(rc, "fs_pool_stats")
    return s


def fs_pool_dump(pool):
    """Returns (state, key, used, free_stack) int32 arrays."""
    n = fs_pool_stats(pool).n_slabs
    state, key, used, fstack = (np.empty(n, np.int32) for _ in range(4))
    nf = ctypes.c_int64(0)
    rc = _L.fs_pool_dump(pool, state.ctypes.data, key.ctypes.data, used.ctypes.data, fstack.ctypes.data,
                         ctypes.byref(nf))
    if rc != FS_OK:
        raise FsError(rc, "fs_pool_dump")
    return state, key, used, fstack[: nf.value].copy()


def fs_model_dump_live(pool, model) -> np.ndarray:
    g = fs_model_geometry(pool, model)
    live = np.empty(fs_pool_stats(pool).n_slabs * g.blocks_per_slab, np.uint8)
    rc = _L.fs_model_dump_live(pool, model, live.ctypes.data)
    if rc != FS_OK:
        raise FsError(rc, "fs_model_dump_live")
    return live


# ------------------------------------------------------------------ device calls
def fs_kv_append(pool, model, layer, k_new, v_new, seq_idx, pos, block_tables, stream=None):
    """k_new/v_new: CUDA fp16 or fp32 [n_tokens][H][D]; seq_idx/pos: CUDA int32 [n_tokens];
    block_tables: CUDA int32 [n_seq][max_blocks]."""
    import torch
    assert k_new.dtype == v_new.dtype and k_new.dtype in (torch.float16, torch.float32)
    assert k_new.is_contiguous() and v_new.is_contiguous() and block_tables.is_contiguous()
    assert seq_idx.dtype == torch.int32 and pos.dtype == torch.int32 and block_tables.dtype == torch.int32
    rc = _L.fs_kv_append(pool, model, layer, _dp(k_new), _dp(v_new),
                         FS_SRC_FP32 if k_new.dtype == torch.float32 else FS_SRC_FP16, _dp(seq_idx), _dp(pos),
                         _dp(block_tables), block_tables.shape[1], seq_idx.numel(), _stream(stream))
    if rc != FS_OK:
        raise FsError(rc, "fs_kv_append")


def make_append(model, layer, k_new, v_new, seq_idx, pos, block_tables) -> fs_append_t:
    """Fill an fs_append_t from torch tensors (which the caller keeps alive); arguments as fs_kv_append."""
    import torch
    assert k_new.dtype == v_new.dtype and k_new.dtype in (torch.float16, torch.float32)
    assert k_new.is_contiguous() and v_new.is_contiguous() and block_tables.is_contiguous()
    assert seq_idx.dtype == torch.int32 and pos.dtype == torch.int32 and block_tables.dtype == torch.int32
    a = fs_append_t()
    a.model, a.layer = model, layer
    a.src_dtype = FS_SRC_FP32 if k_new.dtype == torch.float32 else FS_SRC_FP16
    a.max_blocks = block_tables.shape[1]
    a.k_new, a.v_new, a.seq_idx, a.pos, a.block_tables = _dp(k_new), _dp(v_new), _dp(seq_idx), _dp(pos), _dp(block_tables)
    a.n_tokens = seq_idx.numel()
    return a


def fs_kv_append_multi(pool, appends, stream=None):
    arr = (fs_append_t * len(appends))(*appends)
    rc = _L.fs_kv_append_multi(pool, arr, len(appends), _stream(stream))
    if rc != FS_OK:
        raise FsError(rc, "fs_kv_append_multi")


def fs_decode_step_multi(pool, appends, batches, workspace, stream=None):
    aarr = (fs_append_t * max(len(appends), 1))(*appends)
    barr = (fs_batch_t * len(batches))(*batches)
    rc = _L.fs_decode_step_multi(pool, aarr, len(appends), barr, len(batches), _dp(workspace),
                                 workspace.numel() * workspace.element_size(), _stream(stream))
    if rc != FS_OK:
        raise FsError(rc, "fs_decode_step_multi")


def make_batch(model, layer, n_q_heads, sm_scale, q, block_tables, seq_lens, out, lse=None,
               seq_lens_host=None) -> fs_batch_t:
    """Fill an fs_batch_t from torch tensors (which the caller keeps alive)."""
    import torch
    assert q.dtype == torch.float16 and out.dtype == torch.float16 and q.is_contiguous() and out.is_contiguous()
    assert block_tables.dtype == torch.int32 and seq_lens.dtype == torch.int32 and block_tables.is_contiguous()
    b = fs_batch_t()
    b.model, b.layer, b.n_q_heads, b.sm_scale = model, layer, n_q_heads, sm_scale
    b.q, b.block_tables, b.seq_lens = _dp(q), _dp(block_tables), _dp(seq_lens)
    if seq_lens_host is not None:
        assert isinstance(seq_lens_host, np.ndarray) and seq_lens_host.dtype == np.int32
        b.seq_lens_host = seq_lens_host.ctypes.data
    b.n_seq, b.max_blocks = seq_lens.numel(), block_tables.shape[1]
    b.out, b.lse = _dp(out), _dp(lse)
    return b


def fs_decode_workspace_bytes(pool, batches) -> int:
    arr = (fs_batch_t * len(batches))(*batches)
    return _L.fs_decode_workspace_bytes(pool, arr, len(batches))


def fs_decode_attention(pool, model, layer, n_q_heads, sm_scale, q, block_tables, seq_lens, out, lse, workspace,
                        stream=None):
    rc = _L.fs_decode_attention(pool, model, layer, n_q_heads, sm_scale, _dp(q), _dp(block_tables), _dp(seq_lens),
                                seq_lens.numel(), block_tables.shape[1], _dp(out), _dp(lse), _dp(workspace),
                                workspace.numel() * workspace.element_size(), _stream(stream))
    if rc != FS_OK:
        raise FsError(rc, "fs_decode_attention")


def fs_decode_attention_multi(pool, batches, workspace, stream=None):
    arr = (fs_batch_t * len(batches))(*batches)
    rc = _L.fs_decode_attention_multi(pool, arr, len(batches), _dp(workspace),
                                      workspace.numel() * workspace.element_size(), _stream(stream))
    if rc != FS_OK:
        raise FsError(rc, "fs_decode_attention_multi")


def fs_decode_attention_multi_static(pool, batches, status_out=None, stream=None):
    """status_out: optional CUDA int32/uint32 tensor of one element."""
    arr = (fs_batch_t * len(batches))(*batches)
    rc = _L.fs_decode_attention_multi_static(pool, arr, len(batches), _dp(status_out), _stream(stream))
    if rc != FS_OK:
        raise FsError(rc, "fs_decode_attention_multi_static")


def fs_decode_status(workspace, stream=None) -> int:
    return _L.fs_decode_status(_dp(workspace), _stream(stream))


def fs_prefill_workspace_bytes(n_seq: int) -> int:
    return _L.fs_prefill_workspace_bytes(n_seq)


def fs_prefill_attention(pool, model, layer, n_q_heads, sm_scale, q, block_tables, seq_lens, q_offsets, q_offsets_host,
                         out, lse, workspace, stream=None):
    """q, out: fp16 [n_rows][n_q][D] torch tensors; q_offsets: int32 device tensor [n_seq + 1]; q_offsets_host: the
    same values as a numpy int32 array."""
    assert isinstance(q_offsets_host, np.ndarray) and q_offsets_host.dtype == np.int32
    assert q_offsets_host.shape[0] == seq_lens.numel() + 1 and q_offsets.numel() == seq_lens.numel() + 1
    assert int(q_offsets_host[-1]) == q.shape[0] == out.shape[0] and q.is_contiguous() and out.is_contiguous()
    rc = _L.fs_prefill_attention(pool, model, layer, n_q_heads, sm_scale, _dp(q), _dp(block_tables), _dp(seq_lens),
                                 _dp(q_offsets), q_offsets_host.ctypes.data, seq_lens.numel(), block_tables.shape[1],
                                 _dp(out), _dp(lse), _dp(workspace), workspace.numel() * workspace.element_size(),
                                 _stream(stream))
    if rc != FS_OK:
        raise FsError(rc, "fs_prefill_attention")


class fs_request_t(ctypes.Structure):
    _fields_ = [("arrival_time", ctypes.c_double), ("prompt_tokens", ctypes.c_int32), ("reserved", ctypes.c_int32)]


class fs_sched_params_t(ctypes.Structure):
    _fields_ = [("slo", ctypes.c_double), ("c0", ctypes.c_double), ("c1", ctypes.c_double), ("c2", ctypes.c_double),
                ("n_max", ctypes.c_int32), ("t_max", ctypes.c_int32)]


REQUEST_DTYPE = np.dtype([("arrival_time", np.float64), ("prompt_tokens", np.int32), ("reserved", np.int32)])


def fs_sched_select_batch(arrival, tokens, slo, n_max, t_max, c0, c1, c2, now):
    """Returns (selected, dropped): index arrays into the waiting queue."""
    n = len(arrival)
    w = np.zeros(n, dtype=REQUEST_DTYPE)
    w["arrival_time"], w["prompt_tokens"] = arrival, tokens
    par = fs_sched_params_t(slo, c0, c1, c2, n_max, t_max)
    sel, drp = np.empty(max(n, 1), np.int32), np.empty(max(n, 1), np.int32)
    ns, nd = ctypes.c_int32(0), ctypes.c_int32(0)
    rc = _L.fs_sched_select_batch(w.ctypes.data, n, ctypes.byref(par), float(now), sel.ctypes.data, ctypes.byref(ns),
                                  drp.ctypes.data, ctypes.byref(nd))
    if rc != FS_OK:
        raise FsError(rc, "fs_sched_select_batch")
    return sel[:ns.value].copy(), drp[:nd.value].copy()


def fs_sched_place_models(footprint, mu, capacity):
    f = np.ascontiguousarray(footprint, np.float64)
    m = np.ascontiguousarray(mu, np.float64)
    c = np.ascontiguousarray(capacity, np.float64)
    out = np.empty(max(len(f), 1), np.int32)
    rc = _L.fs_sched_place_models(f.ctypes.data, m.ctypes.data, len(f), c.ctypes.data, len(c), out.ctypes.data)
    if rc != FS_OK:
        raise FsError(rc, "fs_sched_place_models")
    return out[:len(f)].copy()


def fs_model_stats(pool, model) -> fs_model_stats_t:
    st = fs_model_stats_t()
    rc = _L.fs_model_stats(pool, model, ctypes.byref(st))
    if rc != FS_OK:
        raise FsError(rc, "fs_model_stats")
    return st


def fs_pool_set_option(pool, option: int, value: int) -> int:
    """Returns the status code (FS_ERR_INVALID for an unknown option or a value out of range)."""
    return _L.fs_pool_set_option(pool, int(option), int(value))


def fs_pool_get_option(pool, option: int) -> int:
    v = ctypes.c_int64(0)
    rc = _L.fs_pool_get_option(pool, int(option), ctypes.byref(v))
    if rc != FS_OK:
        raise FsError(rc, "fs_pool_get_option")
    return v.value


def fs_pool_last_attention_kernel_ms(pool) -> float:
    return _L.fs_pool_last_attention_kernel_ms(pool)
