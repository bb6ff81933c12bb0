"""The synthetic workloads: shapes, lengths, pool sizes and slab-placement recipes.

Pure input description -- which models share a pool, how long the sequences are, and in which
order blocks are requested from (and returned to) an allocator.  The allocator itself is passed
in by the caller (the CPU oracle's or the HIP library's) as an object with
``alloc(model) -> (rc, blk)`` and ``free(model, blk) -> rc``; nothing here knows how either works.

The five configurations mirror the benchmark definition (the benchmark spec ``configs``); values the
definition leaves open (layer counts, pool sizes for configs 3 and 4, sequences per model in
config 5) are fixed here and echoed in every benchmark line.  The lengths stand in for the
ShareGPT conversation lengths the paper serves; K/V/q values are N(0,1) table deviates.
"""
from __future__ import annotations

import dataclasses
from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np

from . import gen

FP16, FP8, INT8, INT4 = 0, 1, 2, 3
DTYPE_NAME = {FP16: "fp16", FP8: "fp8_e4m3", INT8: "int8", INT4: "int4"}
KiB, MiB, GiB = 1 << 10, 1 << 20, 1 << 30


@dataclass
class ModelSpec:
    name: str
    kv_dtype: int
    n_kv_heads: int
    head_dim: int
    n_layers: int
    n_q_heads: int
    lens: np.ndarray                      # int32 [n_seq]
    tag: int = 0                          # generator stream id of this model
    src_f32: bool = False                 # K/V source rows handed to append as fp32 (else fp16)
    full_layers: Optional[int] = None     # depth of the real model this one is shaped after
    block_budget: Optional[int] = None    # None: one block per slab
    tokens_per_block: Optional[int] = None  # the paper's direction: tokens fixed, block bytes derived (Sec. 3.2 / 5.2)

    @property
    def n_seq(self) -> int:
        return len(self.lens)


@dataclass
class Workload:
    name: str
    slab_bytes: int
    pool_bytes: int
    models: List[ModelSpec]
    placement: str                        # "identity" | "shuffle" | "interleave" | "churn"
    seed: int = gen.MASTER_SEED
    churn_steps: int = 0
    notes: dict = field(default_factory=dict)


# ----------------------------------------------------------------------------- helpers
def blocks_needed(n_tokens: int, T: int) -> int:
    return (int(n_tokens) + T - 1) // T


def alloc_sequences(pool, model: int, lens, T: int):
    """Allocate ceil(len/T) blocks per sequence, sequence by sequence; returns a list of id lists."""
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
    """Allocate n_blocks blocks, then free them in a seeded random order, so that a LIFO free list
    hands later allocations out in that shuffled order (random scatter over the pool)."""
    ids = []
    for _ in range(n_blocks):
        rc, b = pool.alloc(model)
        assert rc == 0
        ids.append(b)
    for i in gen.permutation(seed, tag, n_blocks):
        assert pool.free(model, ids[int(i)]) == 0


def token_index(lens):
    """(seq_idx, pos) int32 arrays naming every token of every sequence, sequence-major."""
    lens = np.asarray(lens, dtype=np.int64)
    seq_idx = np.repeat(np.arange(len(lens), dtype=np.int32), lens)
    starts = np.concatenate([[0], np.cumsum(lens)[:-1]])
    pos = (np.arange(int(lens.sum()), dtype=np.int64) - np.repeat(starts, lens)).astype(np.int32)
    return seq_idx, pos


def source_rows(seed: int, tag: int, layer: int, which: int, lens, n_heads: int, head_dim: int, seq_ids=None,
                dtype=np.float16) -> np.ndarray:
    """[sum(lens)][H][D] source K or V rows; sequence i draws from generator stream seq_ids[i] (default i)."""
    seq_ids = range(len(lens)) if seq_ids is None else seq_ids
    parts = [gen.normal_rows(seed, tag, layer, which, int(s), np.arange(n), n_heads, head_dim)
             for s, n in zip(seq_ids, lens)]
    return np.concatenate(parts, axis=0).astype(dtype)


def fp8_scales_from_rows(k_rows: np.ndarray, v_rows: np.ndarray):
    """Static per-KV-head scales amax/448 of one layer from its source rows -> (k[H], v[H]) float32."""
    ks = (np.abs(k_rows.astype(np.float32)).max(axis=(0, 2)) / np.float32(448.0)).astype(np.float32)
    vs = (np.abs(v_rows.astype(np.float32)).max(axis=(0, 2)) / np.float32(448.0)).astype(np.float32)
    return ks, vs


def fp8_scales_table(n_layers: int, n_heads: int):
    """Static scales for large runs: the generator's largest magnitude / 448 (the amax of any long
    stream), times a small per-(layer, head) factor >= 1 so that every head has its own value."""
    amax = np.float32(np.abs(gen.normal_table()).max())
    idx = np.arange(n_layers * n_heads, dtype=np.float32).reshape(n_layers, n_heads)
    k = (amax / np.float32(448.0)) * (np.float32(1.0) + np.float32(0.01) * (idx % 7))
    v = (amax / np.float32(448.0)) * (np.float32(1.0) + np.float32(0.01) * (idx % 5))
    return k.astype(np.float32), v.astype(np.float32)


# ----------------------------------------------------------------------------- placement
def place(pool, wl: Workload, model_ids, T_of):
    """Run the workload's allocation recipe on ``pool``; returns per-model lists of per-sequence block
    id lists (and, for churn, the final lengths, which replace ModelSpec.lens)."""
    seed = wl.seed
    specs = wl.models
    if wl.placement in ("identity", "shuffle"):
        if wl.placement == "shuffle":
            n_slabs = wl.pool_bytes // wl.slab_bytes
            m0 = model_ids[0]
            bps = wl.slab_bytes // (specs[0].block_budget or wl.slab_bytes)
            shuffle_free_slabs(pool, m0, n_slabs * bps, seed, tag=7)
        return [alloc_sequences(pool, m, s.lens, T_of[m]) for m, s in zip(model_ids, specs)], None
    if wl.placement == "interleave":
        # sequence i of every model is allocated together, one block of each model in turn
        out = [[] for _ in specs]
        n_seq = max(s.n_seq for s in specs)
        for i in range(n_seq):
            need = [blocks_needed(s.lens[i], T_of[m]) if i < s.n_seq else 0 for m, s in zip(model_ids, specs)]
            ids = [[] for _ in specs]
            for j in range(max(need)):
                for k, m in enumerate(model_ids):
                    if j < need[k]:
                        rc, b = pool.alloc(m)
                        assert rc == 0
                        ids[k].append(b)
            for k, s in enumerate(specs):
                if i < s.n_seq:
                    out[k].append(ids[k])
        return out, None
    if wl.placement == "churn":
        return _churn(pool, wl, model_ids, T_of)
    raise ValueError(wl.placement)


def _churn(pool, wl: Workload, model_ids, T_of):
    """Allocate every sequence, then ``churn_steps`` times: pick a live sequence uniformly, free all its
    blocks, and allocate a fresh sequence of the same model with a new length (halved until it fits)."""
    specs = wl.models
    blocks = [alloc_sequences(pool, m, s.lens, T_of[m]) for m, s in zip(model_ids, specs)]
    lens = [np.array(s.lens, dtype=np.int32) for s in specs]
    owner = [(k, i) for k, s in enumerate(specs) for i in range(s.n_seq)]
    n_total = len(owner)
    picks = gen.uniform_ints(wl.seed, 41, wl.churn_steps, n_total)
    med, sig, cap = wl.notes["lognormal"]
    new_lens = gen.lognormal_lengths(wl.seed, 42, wl.churn_steps, med, sig, cap)
    for step in range(wl.churn_steps):
        k, i = owner[int(picks[step])]
        m, T = model_ids[k], T_of[model_ids[k]]
        for b in blocks[k][i]:
            assert pool.free(m, b) == 0
        n = int(new_lens[step])
        while True:
            ids = []
            ok = True
            for _ in range(blocks_needed(n, T)):
                rc, b = pool.alloc(m)
                if rc != 0:
                    ok = False
                    break
                ids.append(b)
            if ok:
                break
            for b in ids:
                assert pool.free(m, b) == 0
            n = max(1, n // 2)
        blocks[k][i] = ids
        lens[k][i] = n
    return blocks, lens


# ----------------------------------------------------------------------------- the five configurations
def config(n: int, seed: int = gen.MASTER_SEED) -> Workload:
    if n == 1:
        lens = gen.uniform_lengths(seed, 101, 8, 1, 256)
        return Workload("cfg1-tiny-fp16", 64 * KiB, 16 * MiB,
                        [ModelSpec("tiny-fp16", FP16, 4, 64, 1, 4, lens, tag=1, full_layers=1)], "shuffle", seed)
    if n == 2:
        lens = gen.uniform_lengths(seed, 102, 64, 512, 4096)
        return Workload("cfg2-llama8b-fp16", 2 * MiB, 32 * GiB,
                        [ModelSpec("8b-fp16", FP16, 8, 128, 32, 32, lens, tag=2, full_layers=32)], "shuffle", seed)
    if n == 3:
        la = gen.uniform_lengths(seed, 103, 128, 1024, 8192)
        lb = gen.uniform_lengths(seed, 104, 128, 1024, 8192)
        return Workload("cfg3-fp16+fp8", 2 * MiB, 128 * GiB,
                        [ModelSpec("8b-fp16", FP16, 8, 128, 32, 32, la, tag=3, full_layers=32),
                         ModelSpec("8b-fp8", FP8, 8, 128, 32, 32, lb, tag=4, full_layers=32)], "interleave", seed)
    if n == 4:
        lens = gen.uniform_lengths(seed, 105, 256, 1024, 8192)
        return Workload("cfg4-int4", 2 * MiB, 64 * GiB,
                        [ModelSpec("8b-int4", INT4, 8, 128, 32, 32, lens, tag=5, src_f32=True, full_layers=32)],
                        "shuffle", seed)
    if n == 5:
        ln = (2048.0, 1.0, 32768)
        mk = lambda t: gen.lognormal_lengths(seed, t, 256, *ln)  # noqa: E731
        models = [ModelSpec("8b-fp16", FP16, 8, 128, 8, 32, mk(106), tag=6, full_layers=32),
                  ModelSpec("8b-fp8", FP8, 8, 128, 8, 32, mk(107), tag=7, full_layers=32),
                  ModelSpec("8b-int8", INT8, 8, 128, 8, 32, mk(108), tag=8, full_layers=32),
                  ModelSpec("13b-int4-mha", INT4, 40, 128, 10, 40, mk(109), tag=9, src_f32=True, full_layers=40)]
        return Workload("cfg5-mixed-4-models", 2 * MiB, 160 * GiB, models, "churn", seed, churn_steps=100_000,
                        notes={"lognormal": ln})
    raise ValueError(f"no config {n}")


def with_head_dim(wl: Workload, head_dim: int) -> Workload:
    """A copy of a workload whose models have another head_dim (same heads, layers, lengths, placement; the pool grows
    with the rows): what the decode kernels are timed on beside head_dim 128."""
    models = [dataclasses.replace(s, head_dim=head_dim) for s in wl.models]
    grow = max(1, -(-head_dim // max(s.head_dim for s in wl.models)))
    return dataclasses.replace(wl, name=f"{wl.name}-d{head_dim}", pool_bytes=wl.pool_bytes * grow, models=models,
                               notes=dict(wl.notes))


def scaled_down(wl: Workload, n_seq: int, max_len: int, pool_bytes: int, churn_steps: int = 2000) -> Workload:
    """A small copy of a workload (fewer, shorter sequences, smaller pool) that keeps its models, slab size
    and placement recipe -- the size the CPU oracle checks in full."""
    models = []
    for s in wl.models:
        lens = np.minimum(s.lens[:n_seq], max_len).astype(np.int32)
        models.append(ModelSpec(s.name, s.kv_dtype, s.n_kv_heads, s.head_dim, s.n_layers, s.n_q_heads, lens, s.tag,
                                s.src_f32, s.full_layers, s.block_budget))
    notes = dict(wl.notes)
    if "lognormal" in notes:
        med, sig, _ = notes["lognormal"]
        notes["lognormal"] = (min(med, max_len / 4), sig, max_len)
    return Workload(wl.name + "-small", wl.slab_bytes, pool_bytes, models, wl.placement, wl.seed,
                    min(wl.churn_steps, churn_steps), notes)


def kv_bytes_per_token_layer(s: ModelSpec) -> int:
    """Algorithmic KV bytes of one token in one layer: K and V rows plus per-token parameters, all KV heads."""
    bits = {FP16: 16, FP8: 8, INT8: 8, INT4: 4}[s.kv_dtype]
    par = {FP16: 0, FP8: 0, INT8: 2, INT4: 4}[s.kv_dtype]
    return 2 * s.n_kv_heads * (s.head_dim * bits // 8 + par)
