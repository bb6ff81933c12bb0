"""Seeded synthetic-input generator (host side, numpy).

This module produces the *inputs* of the decode-attention path -- activations
q, new K/V rows and sequence lengths -- and nothing else.  It contains none of
the method's arithmetic (no quantizer, no layout, no attention).  The CPU
oracle's tests and the HIP path's tests both draw their inputs from here, so
that both sides see bit-identical source values.  ``gen.hip`` next to this file
implements exactly the same counter-based generator on the device, so that tens
of GiB of KV can be produced in HBM without crossing PCIe.

Generator definition (all integer arithmetic modulo 2**64):

    mix64(z): z ^= z >> 30; z *= 0xBF58476D1CE4E5B9; z ^= z >> 27;
              z *= 0x94D049BB133111EB; z ^= z >> 31          (splitmix64 finalizer)
    key  = mix64(mix64(seed ^ GOLD*(model+1)) + (layer << 34) + (which << 32) + seq)
    word(w) = mix64(key + GOLD*(w+1))
    element e = (pos*H + head)*D + dim  takes 16 bits of word(e >> 2):
    u = (word >> 16*(e & 3)) & 0xFFFF ;  x = TABLE[u]

TABLE[i] = float32(Phi^-1((i + 0.5) / 65536)), a 65536-entry inverse-normal
table, so the elements are N(0,1) deviates truncated to about +-4.17.  The table
is built once on the host (scipy) and the very same array is uploaded for the
device generator, so no transcendental function is evaluated twice.

``which``: 0 = K rows, 1 = V rows, 2 = q.
"""
from __future__ import annotations

import functools
import os

import numpy as np

GOLD = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
# every workload derives from this seed; FS_INPUT_SEED replays the tests and benchmarks on other draws
MASTER_SEED = int(os.environ.get("FS_INPUT_SEED", "20250906"))

WHICH_K, WHICH_V, WHICH_Q = 0, 1, 2


def mix64(z):
    """splitmix64 output function on uint64 scalars or arrays."""
    with np.errstate(over="ignore"):
        z = np.array(z, dtype=np.uint64)  # a private copy: the steps below work in place
        z ^= z >> np.uint64(30)
        z *= _M1
        z ^= z >> np.uint64(27)
        z *= _M2
        z ^= z >> np.uint64(31)
    return z if z.ndim else z[()]


@functools.lru_cache(maxsize=1)
def normal_table() -> np.ndarray:
    """The 65536-entry float32 inverse-normal table shared by host and device."""
    from scipy.special import ndtri

    i = np.arange(65536, dtype=np.float64)
    t = ndtri((i + 0.5) / 65536.0).astype(np.float32)
    t.setflags(write=False)
    return t


def stream_key(seed: int, model: int, layer: int, which: int, seq) -> np.ndarray:
    """Key of one (model, layer, K|V|q, sequence) stream; ``seq`` may be an array."""
    with np.errstate(over="ignore"):
        a = mix64(np.uint64(seed) ^ (GOLD * np.uint64(model + 1)))
        seq = np.asarray(seq, dtype=np.uint64)
        b = a + (np.uint64(layer) << np.uint64(34)) + (np.uint64(which) << np.uint64(32)) + seq
    return mix64(b)


def _u16(key, e):
    """16-bit draw for element counters ``e`` (uint64 array) under ``key``."""
    with np.errstate(over="ignore"):
        w = mix64(key + GOLD * ((e >> np.uint64(2)) + np.uint64(1)))
        sh = (e & np.uint64(3)) * np.uint64(16)
    return ((w >> sh) & np.uint64(0xFFFF)).astype(np.int64)


def normal_rows(seed: int, model: int, layer: int, which: int, seq: int, pos, n_heads: int,
                head_dim: int) -> np.ndarray:
    """float32 [len(pos)][n_heads][head_dim] source rows of one sequence.

    Row ``i`` is the K (which=0) or V (which=1) vector of token position
    ``pos[i]`` of global sequence number ``seq``.
    """
    pos = np.asarray(pos, dtype=np.uint64).reshape(-1)
    key = stream_key(seed, model, layer, which, seq)
    hd = n_heads * head_dim
    if hd % 4 == 0 and np.little_endian:
        # a row is hd / 4 whole words: draw each word once and read its four 16-bit fields in place
        # (field e & 3 of a word is bits 16 (e & 3) .. 16 (e & 3) + 15: the little-endian uint16 view);
        # rows go through in slices that reuse two work buffers
        wq = hd // 4
        out = np.empty((len(pos), hd), dtype=np.float32)
        table = normal_table()
        step = max(1, (1 << 18) // wq)
        col = np.arange(wq, dtype=np.uint64)[None, :]
        z = np.empty((step, wq), dtype=np.uint64)
        t = np.empty((step, wq), dtype=np.uint64)
        with np.errstate(over="ignore"):
            for r0 in range(0, len(pos), step):
                n = min(step, len(pos) - r0)
                zz, tt = z[:n], t[:n]
                np.multiply(pos[r0:r0 + n, None], np.uint64(wq), out=zz)
                zz += col
                zz += np.uint64(1)
                zz *= GOLD
                zz += key
                for sh, mul in ((30, _M1), (27, _M2), (31, None)):  # mix64, in place
                    np.right_shift(zz, np.uint64(sh), out=tt)
                    zz ^= tt
                    if mul is not None:
                        zz *= mul
                out[r0:r0 + n] = table[zz.view(np.uint16)]
        return out.reshape(len(pos), n_heads, head_dim)
    e = pos[:, None] * np.uint64(hd) + np.arange(hd, dtype=np.uint64)[None, :]
    x = normal_table()[_u16(key, e)]
    return x.reshape(len(pos), n_heads, head_dim)


def normal_q(seed: int, model: int, layer: int, seq_ids, n_q_heads: int, head_dim: int) -> np.ndarray:
    """float16 [n_seq][n_q_heads][head_dim] query activations (N(0,1) rounded to fp16)."""
    seq_ids = np.asarray(seq_ids, dtype=np.int64).reshape(-1)
    out = np.empty((len(seq_ids), n_q_heads, head_dim), dtype=np.float16)
    for i, s in enumerate(seq_ids):
        out[i] = normal_rows(seed, model, layer, WHICH_Q, int(s), [0], n_q_heads, head_dim)[0].astype(np.float16)
    return out


def normal_q_chunks(seed: int, model: int, layer: int, seq_ids, first_pos, n_new, n_q_heads: int,
                    head_dim: int) -> np.ndarray:
    """float16 [sum(n_new)][n_q_heads][head_dim] query rows of prefill chunks: for sequence seq_ids[i] the rows of
    positions first_pos[i] .. first_pos[i] + n_new[i] - 1, chunks one after the other."""
    parts = [normal_rows(seed, model, layer, WHICH_Q, int(s), np.arange(int(p), int(p) + int(n)), n_q_heads,
                         head_dim).astype(np.float16) for s, p, n in zip(seq_ids, first_pos, n_new)]
    if not parts:
        return np.empty((0, n_q_heads, head_dim), np.float16)
    return np.concatenate(parts, axis=0)


def _draw64(seed: int, tag: int, n: int) -> np.ndarray:
    key = stream_key(seed, 0xFFFF, 0, 3, tag)
    with np.errstate(over="ignore"):
        return mix64(key + GOLD * (np.arange(n, dtype=np.uint64) + np.uint64(1)))


def uniform_lengths(seed: int, tag: int, n: int, lo: int, hi: int) -> np.ndarray:
    """n integer lengths uniform in [lo, hi] (inclusive)."""
    w = _draw64(seed, tag, n)
    return (lo + (w % np.uint64(hi - lo + 1)).astype(np.int64)).astype(np.int32)


def lognormal_lengths(seed: int, tag: int, n: int, median: float, sigma: float, cap: int) -> np.ndarray:
    """n lengths round(median*exp(sigma*z)), z ~ N(0,1) from the table, clamped to [1, cap]."""
    w = _draw64(seed, tag, n)
    z = normal_table()[(w & np.uint64(0xFFFF)).astype(np.int64)].astype(np.float64)
    ln = np.rint(median * np.exp(sigma * z))
    return np.clip(ln, 1, cap).astype(np.int32)


def uniform_ints(seed: int, tag: int, n: int, hi: int) -> np.ndarray:
    """n integers uniform in [0, hi) -- used for churn traces and shuffles."""
    w = _draw64(seed, tag, n)
    return (w % np.uint64(hi)).astype(np.int64)


def permutation(seed: int, tag: int, n: int) -> np.ndarray:
    """A seeded permutation of range(n) (argsort of n 64-bit draws)."""
    return np.argsort(_draw64(seed, tag, n), kind="stable").astype(np.int64)
