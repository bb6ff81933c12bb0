"""Pins for the oracle's prefill (chunked prefill) attention (CPU only).

Nothing here re-types the oracle's loop: the references are (i) the oracle's *decode* attention -- itself pinned
to dense numpy in test_oracle_attention -- on sequences cut off after each query's position, (ii) a dense numpy
softmax with an explicit lower-triangular mask on contiguous arrays, (iii) properties: a query's output does not
depend on later tokens, and how the new tokens are cut into chunks does not matter.
"""
import numpy as np
import pytest

import oracle
from fs_inputs import gen
from test_oracle_attention import SEED, KiB, build


def chunk_inputs(sc, n_new):
    lens = sc["lens"]
    n_new = np.asarray(n_new, np.int32)
    q_off = np.concatenate([[0], np.cumsum(n_new)]).astype(np.int32)
    q = gen.normal_q_chunks(SEED, 0, sc["layer"], np.arange(len(lens)), lens - n_new, n_new, sc["n_q"], sc["g"].head_dim)
    return q, q_off


def run_prefill(sc, q, q_off, lens=None, n_threads=1):
    g = sc["g"]
    lens = sc["lens"] if lens is None else lens
    return oracle.prefill_attention(sc["mem"], g, sc["layer"], sc["n_q"], 1.0 / np.sqrt(g.head_dim), q, sc["tables"],
                                    lens, q_off, sc["ks"], sc["vs"], n_threads=n_threads)


@pytest.mark.parametrize("dtype", [oracle.FP16, oracle.FP8, oracle.INT8, oracle.INT4])
def test_each_row_equals_decode_attention_of_the_truncated_sequence(dtype):
    """Row at position p == decode attention of the same sequence cut to p + 1 tokens with that row as query."""
    lens = np.array([1, 7, 40, 90], np.int32)
    sc = build(dtype, 2, 32, 2, 8, lens, slab=16 * KiB, n_slabs=64, layer=1,
               src_dtype=np.float32 if dtype == oracle.INT4 else np.float16)
    n_new = np.array([1, 7, 13, 33], np.int32)  # whole prompts and trailing chunks
    q, q_off = chunk_inputs(sc, n_new)
    out, lse = run_prefill(sc, q, q_off)
    for b in range(len(lens)):
        for r in range(n_new[b]):
            row = q_off[b] + r
            cut = lens.copy()
            cut[b] = lens[b] - n_new[b] + r + 1
            qd = np.zeros((len(lens), sc["n_q"], 32), np.float16)
            qd[b] = q[row]
            ref, ref_lse = oracle.decode_attention(sc["mem"], sc["g"], 1, sc["n_q"], 1 / np.sqrt(32), qd, sc["tables"], cut,
                                                   sc["ks"], sc["vs"])
            assert np.array_equal(out[row], ref[b]) and np.array_equal(lse[row], ref_lse[b])


def test_fp16_whole_prompt_matches_dense_masked_softmax():
    """Whole-prompt prefill against softmax(mask(Q K^T)) V on contiguous fp64 arrays."""
    lens = np.array([5, 37, 64, 65], np.int32)
    H, D, n_q = 2, 64, 4
    sc = build(oracle.FP16, H, D, 1, n_q, lens, slab=32 * KiB, n_slabs=32)
    q, q_off = chunk_inputs(sc, lens)
    out, lse = run_prefill(sc, q, q_off, n_threads=3)
    off = 0
    for b, n in enumerate(lens):
        K = sc["k"][off:off + n].astype(np.float64)
        V = sc["v"][off:off + n].astype(np.float64)
        Q = q[q_off[b]:q_off[b + 1]].astype(np.float64)            # [n][n_q][D]
        mask = np.tril(np.ones((n, n), bool))                      # query i sees keys j <= i
        for h in range(n_q):
            S = (Q[:, h, :] @ K[:, h // (n_q // H), :].T) / np.sqrt(D)
            S = np.where(mask, S, -np.inf)
            m = S.max(axis=1, keepdims=True)
            P = np.exp(S - m)
            ref = (P @ V[:, h // (n_q // H), :]) / P.sum(axis=1, keepdims=True)
            assert np.max(np.abs(out[q_off[b]:q_off[b + 1], h] - ref)) < 1e-12
            assert np.max(np.abs(lse[q_off[b]:q_off[b + 1], h] - (m[:, 0] + np.log(P.sum(axis=1))))) < 1e-12
        off += n
    # first row of every prompt attends to one token: its output is that token's V exactly
    off = 0
    for b, n in enumerate(lens):
        for h in range(n_q):
            assert np.array_equal(out[q_off[b], h], sc["v"][off, h // (n_q // H)].astype(np.float64))
        off += n


def test_causality_later_tokens_do_not_matter():
    """Overwriting the stored bytes of the tokens after position p leaves every row at positions <= p unchanged,
    and changes the rows after p."""
    lens = np.array([50], np.int32)
    sc = build(oracle.INT8, 2, 32, 1, 4, lens, slab=16 * KiB, n_slabs=32)
    q, q_off = chunk_inputs(sc, lens)
    out, _ = run_prefill(sc, q, q_off)
    g, T = sc["g"], sc["T"]
    p = 20
    mem = sc["mem"].copy()
    for t in range(p + 1, 50):
        blk = int(sc["tables"][0, t // T])
        for h in range(2):
            for which in (0, 1):
                o = oracle.row_offset(g, blk, 0, h, which, t % T)
                mem[o:o + g.row_bytes] ^= 0x55
    sc2 = dict(sc, mem=mem)
    out2, _ = run_prefill(sc2, q, q_off)
    assert np.array_equal(out[:p + 1], out2[:p + 1])
    assert not np.array_equal(out[p + 1:], out2[p + 1:])


def test_chunking_does_not_matter_and_zero_length_chunks():
    """One call with the whole tail == two calls with the tail cut in two (each against the lengths it has seen);
    a sequence with no new tokens contributes no rows."""
    lens = np.array([30, 12, 77], np.int32)
    sc = build(oracle.INT4, 2, 32, 1, 8, lens, slab=16 * KiB, n_slabs=64, src_dtype=np.float32)
    n_new = np.array([20, 0, 40], np.int32)
    q, q_off = chunk_inputs(sc, n_new)
    out, lse = run_prefill(sc, q, q_off, n_threads=2)
    assert out.shape[0] == 60
    first = np.array([8, 0, 25], np.int32)
    second = n_new - first
    # first part: the sequences as they were before the second part was appended
    lens1 = lens - second
    q1 = np.concatenate([q[q_off[b]:q_off[b] + first[b]] for b in range(3)])
    o1, l1 = run_prefill(sc, q1, np.concatenate([[0], np.cumsum(first)]).astype(np.int32), lens=lens1)
    q2 = np.concatenate([q[q_off[b] + first[b]:q_off[b + 1]] for b in range(3)])
    o2, l2 = run_prefill(sc, q2, np.concatenate([[0], np.cumsum(second)]).astype(np.int32))
    joined = np.concatenate([o1[:8], o2[:12], o1[8:], o2[12:]])
    assert np.array_equal(out, joined)


def test_invalid_arguments_are_rejected():
    lens = np.array([10], np.int32)
    sc = build(oracle.FP16, 2, 32, 1, 2, lens, slab=16 * KiB, n_slabs=16)
    q = np.zeros((11, 2, 32), np.float16)
    with pytest.raises(ValueError):
        run_prefill(sc, q, np.array([0, 11], np.int32))  # more new tokens than the sequence holds
