"""Workload recipes shared by the CPU-oracle tests and the GPU parity tests.

Only *inputs* are built here (lengths, block tables, token index lists); every
allocation goes through whichever allocator the caller passes in -- the oracle's
or the HIP library's -- via an object with ``alloc(model) -> (rc, blk)`` and
``free(model, blk) -> rc``.
"""
from __future__ import annotations

import numpy as np

from fs_inputs import gen


def blocks_needed(n_tokens: int, T: int) -> int:
    return (int(n_tokens) + T - 1) // T


def alloc_sequences(pool, model: int, lens, T: int):
    """Allocate ceil(len/T) blocks per sequence, sequence by sequence; returns list of id lists."""
    out = []
    for n in lens:
        ids = []
        for _ in range(blocks_needed(n, T)):
            rc, b = pool.alloc(model)
            assert rc == 0, f"alloc failed rc={rc}"
            ids.append(b)
        out.append(ids)
    return out


def make_tables(blocks_per_seq, max_blocks=None) -> np.ndarray:
    """int32 [n_seq][max_blocks] block tables, unused entries 0."""
    mb = max(1, max(len(b) for b in blocks_per_seq)) if max_blocks is None else max_blocks
    t = np.zeros((len(blocks_per_seq), mb), np.int32)
    for i, b in enumerate(blocks_per_seq):
        t[i, : len(b)] = b
    return t


def shuffle_free_slabs(pool, model: int, n_blocks: int, seed: int, tag: int = 99):
    """Allocate n_blocks blocks, then free them in a seeded random order.

    With a LIFO free list the following allocations come out in that shuffled order,
    i.e. scattered randomly over the pool."""
    ids = []
    for _ in range(n_blocks):
        rc, b = pool.alloc(model)
        assert rc == 0
        ids.append(b)
    for i in gen.permutation(seed, tag, n_blocks):
        assert pool.free(model, ids[int(i)]) == 0


def token_index(lens, seq_base: int = 0):
    """(seq_idx, pos) int32 arrays naming every token of every sequence, sequence-major."""
    lens = np.asarray(lens, dtype=np.int64)
    seq_idx = np.repeat(np.arange(len(lens), dtype=np.int32), lens)
    starts = np.concatenate([[0], np.cumsum(lens)[:-1]])
    pos = (np.arange(int(lens.sum()), dtype=np.int64) - np.repeat(starts, lens)).astype(np.int32)
    return seq_idx, pos


def source_rows(seed: int, model: int, layer: int, which: int, lens, n_heads: int, head_dim: int,
                seq_base: int = 0, dtype=np.float16) -> np.ndarray:
    """[sum(lens)][H][D] source K or V rows of all sequences (global sequence number = seq_base + i)."""
    parts = [gen.normal_rows(seed, model, layer, which, seq_base + i, np.arange(n), n_heads, head_dim)
             for i, n in enumerate(lens)]
    return np.concatenate(parts, axis=0).astype(dtype)


def fp8_scales(k_rows: np.ndarray, v_rows: np.ndarray):
    """Static per-KV-head scales amax/448 for one layer from its source rows -> (k[H], v[H]) float32."""
    ks = (np.abs(k_rows.astype(np.float32)).max(axis=(0, 2)) / np.float32(448.0)).astype(np.float32)
    vs = (np.abs(v_rows.astype(np.float32)).max(axis=(0, 2)) / np.float32(448.0)).astype(np.float32)
    return ks, vs
