"""Pins for the oracle's KV append and paged decode attention (CPU only).

The reference here is never the oracle itself: dense fp64 softmax(q K^T) V written with numpy
on contiguous arrays, closed-form special cases, and invariants the problem fixes (placement
independence, weights summing to one).
"""
import numpy as np
import pytest

import oracle
from fs_inputs import workloads as scenario
from fs_inputs import gen

SEED = gen.MASTER_SEED
KiB = 1 << 10


def dense_attention(q, K, V, sm_scale, n_kv):
    """Textbook attention on contiguous fp64 arrays. q [n_q][D]; K, V [n][H][D]."""
    n_q = q.shape[0]
    G = n_q // n_kv
    out = np.empty((n_q, K.shape[2]))
    lse = np.empty(n_q)
    for h in range(n_q):
        s = sm_scale * (K[:, h // G, :] @ q[h].astype(np.float64))
        m = s.max()
        p = np.exp(s - m)
        out[h] = (p[:, None] * V[:, h // G, :]).sum(axis=0) / p.sum()
        lse[h] = m + np.log(p.sum())
    return out, lse


def build(dtype, H, D, L, n_q, lens, slab=64 * KiB, n_slabs=64, budget=None, shuffle=True, layer=0, model_id=0,
          src_dtype=np.float16):
    pool = oracle.Pool(slab, n_slabs * slab)
    m = pool.model_add(dtype, H, D, L, budget)
    g = pool.model_geometry(m)
    T = g.tokens_per_block
    if shuffle:
        scenario.shuffle_free_slabs(pool, m, n_slabs * pool.blocks_per_slab(m), SEED, tag=7)
    tables = scenario.make_tables(scenario.alloc_sequences(pool, m, lens, T))
    mem = np.zeros(n_slabs * slab, np.uint8)
    k = scenario.source_rows(SEED, model_id, layer, gen.WHICH_K, lens, H, D, dtype=src_dtype)
    v = scenario.source_rows(SEED, model_id, layer, gen.WHICH_V, lens, H, D, dtype=src_dtype)
    ks = vs = None
    if dtype == oracle.FP8:
        ks1, vs1 = scenario.fp8_scales_from_rows(k, v)
        ks = np.ones((L, H), np.float32)
        vs = np.ones((L, H), np.float32)
        ks[layer], vs[layer] = ks1, vs1
    seq_idx, pos = scenario.token_index(lens)
    oracle.kv_append(mem, g, layer, k, v, seq_idx, pos, tables, ks, vs)
    q = gen.normal_q(SEED, model_id, layer, np.arange(len(lens)), n_q, D)
    return dict(pool=pool, m=m, g=g, T=T, tables=tables, mem=mem, k=k, v=v, ks=ks, vs=vs, q=q, lens=np.asarray(lens),
                layer=layer, n_q=n_q)


def run(sc, n_threads=1):
    g = sc["g"]
    return oracle.decode_attention(sc["mem"], g, sc["layer"], sc["n_q"], 1.0 / np.sqrt(g.head_dim), sc["q"],
                                   sc["tables"], sc["lens"], sc["ks"], sc["vs"], n_threads=n_threads)


def test_fp16_matches_dense_numpy_config1_shape():
    """Tiny config: 4 q heads = 4 KV heads, head_dim 64, 8 sequences, lengths in [1, 256], shuffled slabs."""
    lens = gen.uniform_lengths(SEED, 1, 8, 1, 256)
    sc = build(oracle.FP16, 4, 64, 1, 4, lens, n_slabs=256)
    out, lse = run(sc)
    off = 0
    for b, n in enumerate(lens):
        K = sc["k"][off:off + n].astype(np.float64)
        V = sc["v"][off:off + n].astype(np.float64)
        ref, ref_lse = dense_attention(sc["q"][b], K, V, 1 / 8.0, 4)
        assert np.max(np.abs(out[b] - ref)) < 1e-12
        assert np.max(np.abs(lse[b] - ref_lse)) < 1e-12
        off += n


@pytest.mark.parametrize("dtype", [oracle.FP16, oracle.FP8, oracle.INT8, oracle.INT4])
def test_gqa_quantized_equals_dense_attention_over_dequantized_values(dtype):
    """Attention over stored (quantized) KV equals dense attention over the dequantized values, where the
    dequantized values are rebuilt here from the stored bytes with numpy, not with the oracle."""
    lens = [1, 5, 33, 70]
    H, D, L, n_q = 2, 32, 2, 8
    sc = build(dtype, H, D, L, n_q, lens, slab=16 * KiB, n_slabs=64, layer=1,
               src_dtype=np.float32 if dtype == oracle.INT4 else np.float16)
    out, lse = run(sc)
    g, T, mem = sc["g"], sc["T"], sc["mem"]
    bits = {0: 16, 1: 8, 2: 8, 3: 4}[dtype]
    e4m3 = np.array([oracle.e4m3_decode(b) for b in range(256)], dtype=np.float64)  # pinned in test_oracle_formats
    for b, n in enumerate(lens):
        K = np.empty((n, H, D))
        V = np.empty((n, H, D))
        for t in range(n):
            blk = int(sc["tables"][b, t // T])
            for h in range(H):
                for which, dst in ((0, K), (1, V)):
                    base = blk * g.block_budget + 1 * g.layer_bytes + h * g.head_chunk
                    row = mem[base + which * g.kv_tile + (t % T) * g.row_bytes:][: g.row_bytes]
                    par = mem[base + 2 * g.kv_tile + which * g.par_tile + (t % T) * g.param_bytes:][: g.param_bytes]
                    if bits == 16:
                        x = row.view(np.float16).astype(np.float64)
                    elif dtype == oracle.FP8:
                        x = e4m3[row] * float((sc["vs"] if which else sc["ks"])[1, h])
                    elif dtype == oracle.INT8:
                        x = row.view(np.int8).astype(np.float64) * float(par.view(np.float16)[0])
                    else:
                        codes = np.stack([row & 15, row >> 4], axis=1).reshape(-1).astype(np.float64)
                        s, z = par.view(np.float16).astype(np.float64)
                        x = (codes - z) * s
                    dst[t, h] = x
        ref, ref_lse = dense_attention(sc["q"][b], K, V, 1 / np.sqrt(D), H)
        assert np.max(np.abs(out[b] - ref)) < 1e-12
        assert np.max(np.abs(lse[b] - ref_lse)) < 1e-12
        # and the dequantized values are close to the source (the quantizers did something sensible)
        off = int(np.sum(lens[:b]))
        tol = {0: 1e-3, 1: 0.3, 2: 0.05, 3: 0.45}[dtype]
        assert np.max(np.abs(K - sc["k"][off:off + n].astype(np.float64))) < tol
        Kd, Vd = oracle.dequant_sequence(mem, g, 1, sc["tables"][b], n, sc["ks"], sc["vs"])
        assert np.array_equal(Kd, K) and np.array_equal(Vd, V)


@pytest.mark.parametrize("dtype", [oracle.FP16, oracle.INT4])
def test_placement_invariance(dtype):
    """Same logical KV under contiguous vs shuffled block placement: identical outputs to the last bit."""
    lens = gen.uniform_lengths(SEED, 2, 6, 1, 200)
    a = build(dtype, 2, 64, 1, 4, lens, slab=16 * KiB, n_slabs=128, shuffle=False)
    b = build(dtype, 2, 64, 1, 4, lens, slab=16 * KiB, n_slabs=128, shuffle=True)
    assert not np.array_equal(a["tables"], b["tables"])
    assert np.array_equal(np.sort(a["tables"][0][:1]), a["tables"][0][:1])
    oa, la = run(a)
    ob, lb = run(b)
    assert np.array_equal(oa, ob) and np.array_equal(la, lb)
    ot, _ = run(b, n_threads=4)
    assert np.array_equal(ob, ot)  # the thread count does not change any bit


def test_weights_sum_to_one_and_single_token():
    lens = [1, 2, 63, 64, 65, 128, 129]  # block edges for T = 64 ... depends on geometry below
    sc = build(oracle.FP16, 2, 64, 1, 2, lens, slab=32 * KiB, n_slabs=32)
    T = sc["T"]
    assert T == 64
    # V == 1 everywhere -> out == 1 (softmax weights sum to one)
    g = sc["g"]
    ones = np.ones_like(sc["v"])
    seq_idx, pos = scenario.token_index(lens)
    oracle.kv_append(sc["mem"], g, 0, sc["k"], ones, seq_idx, pos, sc["tables"])
    out, lse = run(sc)
    assert np.max(np.abs(out - 1.0)) < 1e-12
    # restore V; a one-token sequence returns exactly that token's V row
    oracle.kv_append(sc["mem"], g, 0, sc["k"], sc["v"], seq_idx, pos, sc["tables"])
    out, lse = run(sc)
    assert np.array_equal(out[0], sc["v"][0].astype(np.float64))
    s0 = (sc["k"][0].astype(np.float64) * sc["q"][0].astype(np.float64)).sum(axis=1) / 8.0
    assert np.max(np.abs(lse[0] - s0)) < 1e-12


def test_zero_query_gives_mean_of_values_and_dominant_key_wins():
    lens = [37, 90]
    sc = build(oracle.FP16, 2, 32, 1, 4, lens, slab=8 * KiB, n_slabs=64)
    q0 = sc["q"].copy()
    sc["q"] = np.zeros_like(q0)
    out, lse = run(sc)
    off = 0
    for b, n in enumerate(lens):
        mean = sc["v"][off:off + n].astype(np.float64).mean(axis=0)  # [H][D]
        for h in range(4):
            assert np.max(np.abs(out[b, h] - mean[h // 2])) < 1e-12
            assert abs(lse[b, h] - np.log(n)) < 1e-12
        off += n
    # two query heads of one group with the same q give the same row
    sc["q"] = q0.copy()
    sc["q"][:, 1] = sc["q"][:, 0]
    out, _ = run(sc)
    assert np.array_equal(out[:, 0], out[:, 1])
    # plant one key aligned with q so that its logit is far above the rest: output ~ its V row
    g = sc["g"]
    k = sc["k"].copy()
    tgt = 20  # token 20 of sequence 0
    k[tgt, 0] = (sc["q"][0, 0].astype(np.float32) * 40).astype(np.float16)
    seq_idx, pos = scenario.token_index(lens)
    oracle.kv_append(sc["mem"], g, 0, k, sc["v"], seq_idx, pos, sc["tables"])
    out, _ = run(sc)
    assert np.max(np.abs(out[0, 0] - sc["v"][tgt, 0].astype(np.float64))) < 1e-6


def test_append_touches_only_defined_bytes_and_is_order_independent():
    lens = [50, 3]
    for dtype in range(4):
        sc = build(dtype, 2, 32, 2, 2, lens, slab=8 * KiB, n_slabs=32, layer=1,
                   src_dtype=np.float32 if dtype == oracle.INT4 else np.float16)
        g, T = sc["g"], sc["T"]
        # layer 0 was never appended: still zero
        touched = np.flatnonzero(sc["mem"])
        offs_in_block = touched % g.block_budget
        assert np.all(offs_in_block >= g.layer_bytes) and np.all(offs_in_block < 2 * g.layer_bytes)
        # appending token by token in reverse order gives the same bytes
        mem2 = np.zeros_like(sc["mem"])
        seq_idx, pos = scenario.token_index(lens)
        for i in reversed(range(len(pos))):
            oracle.kv_append(mem2, g, 1, sc["k"][i:i + 1], sc["v"][i:i + 1], seq_idx[i:i + 1], pos[i:i + 1],
                             sc["tables"], sc["ks"], sc["vs"])
        assert np.array_equal(mem2, sc["mem"])
