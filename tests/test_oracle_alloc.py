"""Pins for the oracle's geometry and slab allocator (CPU only)."""
import os

import numpy as np
import pytest

import oracle
from fs_inputs import gen

MiB = 1 << 20


def _a(x, n):
    return (x + n - 1) // n * n


# ---------------------------------------------------------------- geometry
@pytest.mark.parametrize("dtype,H,D,L,budget,T,chunk", [
    (oracle.FP16, 4, 64, 1, 64 << 10, 64, 16 << 10),
    (oracle.FP16, 8, 128, 32, 2 * MiB, 16, 8 << 10),
    (oracle.FP8, 8, 128, 32, 2 * MiB, 32, 8 << 10),
    (oracle.INT8, 8, 128, 32, 2 * MiB, 31, 8064),
    (oracle.INT4, 8, 128, 32, 2 * MiB, 60, 8160),
    (oracle.INT4, 40, 128, 40, 2 * MiB, 9, 1248),
    (oracle.FP16, 8, 128, 8, 2 * MiB, 64, 32 << 10),
    (oracle.FP8, 8, 128, 8, 2 * MiB, 128, 32 << 10),
    (oracle.INT8, 8, 128, 8, 2 * MiB, 126, 32 << 10),
    (oracle.INT4, 40, 128, 10, 2 * MiB, 38, 5184),
])
def test_tokens_per_block_table(dtype, H, D, L, budget, T, chunk):
    """Token counts and per-head chunk sizes worked out by hand from the block-size and
    token-size equations of Sec. 3.2 plus the 16/256-byte alignment of the layout."""
    g = oracle.geometry(dtype, H, D, L, budget)
    assert g.tokens_per_block == T
    assert g.head_chunk == chunk


def test_geometry_closed_form_random():
    """Independent recomputation: block_bytes(T) fits, block_bytes(T+1) does not; token-size equation."""
    rng = np.random.default_rng(5)
    bits = {oracle.FP16: 16, oracle.FP8: 8, oracle.INT8: 8, oracle.INT4: 4}
    par = {oracle.FP16: 0, oracle.FP8: 0, oracle.INT8: 2, oracle.INT4: 4}

    def block_bytes(dt, H, D, L, T):
        kv = _a(T * D * bits[dt] // 8, 16)
        p = _a(T * par[dt], 16) if par[dt] else 0
        return L * _a(H * (2 * kv + 2 * p), 256)

    for _ in range(400):
        dt = int(rng.integers(0, 4))
        H, D, L = int(rng.integers(1, 41)), int(rng.choice([32, 64, 96, 128, 256])), int(rng.integers(1, 41))
        budget = int(rng.choice([64 << 10, 256 << 10, 1 * MiB, 2 * MiB, 3 * MiB]))
        if block_bytes(dt, H, D, L, 1) > budget:
            with pytest.raises(ValueError):
                oracle.geometry(dt, H, D, L, budget)
            continue
        g = oracle.geometry(dt, H, D, L, budget)
        T = g.tokens_per_block
        assert block_bytes(dt, H, D, L, T) <= budget < block_bytes(dt, H, D, L, T + 1)
        assert g.block_bytes == block_bytes(dt, H, D, L, T)
        # TokenSize = #Heads x HeadDim x 2 x bytes(precision): the payload never exceeds the budget
        token_size = H * D * 2 * bits[dt] / 8
        assert T * L * token_size <= budget
        assert g.row_bytes == D * bits[dt] // 8 and g.param_bytes == par[dt]


def test_fp8_holds_twice_the_tokens_of_fp16():
    """Sec. 3.2 C2: an FP8 token is half an FP16 token, so equal bytes hold twice the tokens."""
    for L in (1, 8, 32):
        a = oracle.geometry(oracle.FP16, 8, 128, L, 2 * MiB).tokens_per_block
        b = oracle.geometry(oracle.FP8, 8, 128, L, 2 * MiB).tokens_per_block
        assert b == 2 * a


def test_offsets_are_disjoint_and_inside_the_block():
    for dt in range(4):
        g = oracle.geometry(dt, 3, 32, 2, 16 << 10)
        T = g.tokens_per_block
        spans = []
        for layer in range(2):
            for h in range(3):
                for which in range(2):
                    for t in range(T):
                        o = oracle.row_offset(g, 5, layer, h, which, t)
                        spans.append((o, o + g.row_bytes))
                        if g.param_bytes:
                            p = oracle.param_offset(g, 5, layer, h, which, t)
                            spans.append((p, p + g.param_bytes))
        spans.sort()
        base = oracle.block_offset(g, 5)
        assert base == 5 * (16 << 10)
        assert spans[0][0] >= base and spans[-1][1] <= base + g.block_bytes <= base + (16 << 10)
        for (a0, a1), (b0, b1) in zip(spans[:-1], spans[1:]):
            assert a1 <= b0
        assert oracle.row_offset(g, 5, 0, 0, 0, 0) % 16 == 0


# ---------------------------------------------------------------- the paper's worked example
def test_block_id_worked_example(golden_dir):
    rows = [list(map(int, ln.split())) for ln in open(os.path.join(golden_dir, "kv_slab_fig_example.txt"))
            if ln.strip() and not ln.startswith("#")]
    slab = 64 << 10
    pool = oracle.Pool(slab, 4 * slab)
    ids = {}
    for model_no, bps, slab_id, local, engine_id in rows:
        m = pool.model_add(oracle.FP16 if bps == 2 else oracle.FP8, 2, 64, 1, slab // bps)
        assert pool.blocks_per_slab(m) == bps
        ids[model_no] = (m, bps, slab_id, local, engine_id)
    m1, m2 = ids[1][0], ids[2][0]
    # Drive the allocator into the figure's state: Model 2 owns slab 0 and reaches local block 3,
    # Model 1 owns slab 1 and takes local block 0.
    got2 = [pool.alloc(m2)[1] for _ in range(4)]
    got1 = pool.alloc(m1)[1]
    assert got2[3] == ids[2][4] == ids[2][2] * ids[2][1] + ids[2][3]
    assert got1 == ids[1][4] == ids[1][2] * ids[1][1] + ids[1][3]
    g1, g2 = pool.model_geometry(m1), pool.model_geometry(m2)
    # view mapping: the two ids resolve to disjoint byte ranges at slab*slab_bytes + local*block_bytes
    assert oracle.block_offset(g1, got1) == 1 * slab + 0
    assert oracle.block_offset(g2, got2[3]) == 0 * slab + 3 * (slab // 4)
    state, key, used, _ = pool.dump()
    assert state[0] == oracle.FULL and state[1] == oracle.PARTIAL and key[0] == m2 and key[1] == m1


# ---------------------------------------------------------------- allocator behaviour
def test_initial_order_lifo_reuse_and_errors():
    slab = 64 << 10
    pool = oracle.Pool(slab, 8 * slab)
    m = pool.model_add(oracle.FP16, 4, 64, 1)
    assert [pool.alloc(m)[1] for _ in range(8)] == list(range(8))
    assert pool.alloc(m)[0] == oracle.ERR_NOMEM
    assert pool.free(m, 3) == 0 and pool.free(m, 6) == 0
    assert pool.free(m, 3) == oracle.ERR_STATE  # double free
    assert pool.free(m, 99) == oracle.ERR_INVALID
    assert pool.alloc(m)[1] == 6 and pool.alloc(m)[1] == 3  # most recently emptied slab first
    other = pool.model_add(oracle.FP8, 4, 64, 1)
    assert pool.free(other, 2) == oracle.ERR_STATE  # block of another model
    assert pool.model_remove(m) == oracle.ERR_STATE  # still holds blocks
    for b in range(8):
        assert pool.free(m, b) == 0
    assert pool.model_remove(m) == 0
    assert pool.n_free == 8


def test_partial_slab_lowest_id_lowest_local():
    slab = 64 << 10
    pool = oracle.Pool(slab, 4 * slab)
    m = pool.model_add(oracle.FP16, 2, 64, 1, slab // 4)  # 4 blocks per slab
    ids = [pool.alloc(m)[1] for _ in range(8)]
    assert ids == list(range(8))
    for b in (1, 2, 6):
        assert pool.free(m, b) == 0
    # partial slabs 0 (locals 1, 2 free) and 1 (local 2 free): lowest slab, lowest local first
    assert [pool.alloc(m)[1] for _ in range(4)] == [1, 2, 6, 8]


def _check_invariants(pool, models, live):
    state, key, used, free_stack = pool.dump()
    n = pool.n_slabs
    assert sorted(free_stack.tolist()) == np.flatnonzero(state == oracle.FREE).tolist()
    assert np.all(key[state == oracle.FREE] == -1) and np.all(used[state == oracle.FREE] == 0)
    total = 0
    spans = []
    for m in models:
        bps = pool.blocks_per_slab(m)
        lv = pool.dump_live(m).reshape(n, bps)
        assert set(np.flatnonzero(lv.reshape(-1)).tolist()) == live[m]
        per_slab = lv.sum(axis=1)
        assert np.all(per_slab[key != m] == 0)  # a slab holds blocks of exactly one key
        own = key == m
        assert np.array_equal(per_slab[own], used[own])
        assert np.all(state[own & (used == bps)] == oracle.FULL)
        assert np.all(state[own & (used < bps)] == oracle.PARTIAL)
        assert np.all(used[own] > 0)
        if bps == 1:
            assert not np.any(state[own] == oracle.PARTIAL)
        total += int(per_slab.sum())
        g = pool.model_geometry(m)
        for b in live[m]:
            o = oracle.block_offset(g, b)
            spans.append((o, o + g.block_budget))
    assert total == sum(len(v) for v in live.values())
    spans.sort()
    assert all(a[1] <= b[0] for a, b in zip(spans[:-1], spans[1:]))  # no two live blocks overlap
    assert not spans or spans[-1][1] <= pool.pool_bytes


def test_random_trace_invariants():
    slab = 64 << 10
    pool = oracle.Pool(slab, 48 * slab)
    models = [pool.model_add(oracle.FP16, 4, 64, 1), pool.model_add(oracle.FP8, 4, 64, 1, slab // 2),
              pool.model_add(oracle.INT4, 2, 64, 2, slab // 8), pool.model_add(oracle.INT8, 4, 64, 1)]
    live = {m: set() for m in models}
    ops = gen.uniform_ints(1234, 1, 6000, 1 << 30)
    for step, r in enumerate(ops):
        m = models[int(r) % 4]
        do_free = (int(r) >> 8) % 5 < 2 and live[m]
        if do_free:
            b = sorted(live[m])[(int(r) >> 12) % len(live[m])]
            assert pool.free(m, b) == 0
            live[m].discard(b)
        else:
            n_free_before = pool.n_free
            rc, b = pool.alloc(m)
            if rc == oracle.ERR_NOMEM:
                # no external fragmentation: NOMEM only when no slab is free and no slab of this key has room
                state, key, used, _ = pool.dump()
                assert n_free_before == 0 and not np.any((key == m) & (state == oracle.PARTIAL))
            else:
                assert rc == 0 and b not in live[m]
                live[m].add(b)
        if step % 97 == 0:
            _check_invariants(pool, models, live)
    _check_invariants(pool, models, live)
    for m in models:
        for b in sorted(live[m]):
            assert pool.free(m, b) == 0
    state, key, used, free_stack = pool.dump()
    assert np.all(state == oracle.FREE) and len(free_stack) == 48  # everything returns to the shared tensor


def test_any_free_slab_serves_any_model():
    slab = 64 << 10
    pool = oracle.Pool(slab, 6 * slab)
    a = pool.model_add(oracle.FP16, 4, 64, 1)
    b = pool.model_add(oracle.INT4, 4, 64, 1)
    ida = [pool.alloc(a)[1] for _ in range(6)]
    assert pool.alloc(b)[0] == oracle.ERR_NOMEM
    assert pool.free(a, ida[4]) == 0
    rc, blk = pool.alloc(b)  # the slab freed by model a is immediately usable by model b
    assert rc == 0 and blk == 4


# --------------------------------------------------------------------------- Sec. 3.2 forward / Sec. 5.2 slab size
def test_block_bytes_forward_is_the_block_size_equation():
    """block size = TokensPerBlock x TokenSize + Quant.Params (Sec. 3.2), recomputed independently; where the layout
    pads nothing it is exactly T x L x 2 x H x (D x bytes + param bytes); and it inverts fso_geometry."""
    import math

    bits = {oracle.FP16: 16, oracle.FP8: 8, oracle.INT8: 8, oracle.INT4: 4}
    par = {oracle.FP16: 0, oracle.FP8: 0, oracle.INT8: 2, oracle.INT4: 4}
    rng = np.random.default_rng(9)
    for _ in range(300):
        dt = int(rng.integers(0, 4))
        H, D, L, T = int(rng.integers(1, 41)), int(rng.choice([32, 64, 128, 256])), int(rng.integers(1, 41)), int(rng.integers(1, 200))
        kv = _a(T * D * bits[dt] // 8, 16)
        p = _a(T * par[dt], 16) if par[dt] else 0
        want = L * _a(H * (2 * kv + 2 * p), 256)
        got = oracle.block_bytes(dt, H, D, L, T)
        assert got == want
        g = oracle.geometry(dt, H, D, L, got)  # budget = the block's own size: T tokens fit (alignment may admit more)
        assert g.tokens_per_block >= T and g.block_bytes == got
        if T > 1:
            assert oracle.geometry(dt, H, D, L, got - 256).tokens_per_block < T
    # no padding anywhere: T multiple of 8, H x chunk multiple of 256
    assert oracle.block_bytes(oracle.FP16, 8, 128, 32, 16) == 16 * 32 * (2 * 8 * 128 * 2)
    assert oracle.block_bytes(oracle.INT8, 8, 128, 32, 16) == 16 * 32 * (2 * 8 * (128 + 2))
    assert oracle.block_bytes(oracle.INT4, 8, 128, 32, 16) == 16 * 32 * (2 * 8 * (64 + 4))
    assert oracle.block_bytes(oracle.FP16, 8, 128, 32, 0) == 0 and oracle.block_bytes(7, 8, 128, 32, 16) == 0
    # a token count the padding would let grow stays as imposed
    pool = oracle.Pool(oracle.block_bytes(oracle.INT8, 3, 64, 1, 5) * 4, oracle.block_bytes(oracle.INT8, 3, 64, 1, 5) * 64)
    m = pool.model_add_tokens(oracle.INT8, 3, 64, 1, 5)
    assert pool.model_geometry(m).tokens_per_block == 5 and pool.blocks_per_slab(m) == 4


def test_token_size_divides_by_the_tensor_parallel_degree():
    """TokenSize = #Heads / TP x HeadDim x 2 x bytes(precision) (Sec. 3.2): a GPU of a TP group registers its own
    share of the KV heads.  Where nothing is padded the block shrinks by exactly TP, and a fixed slab holds TP times
    the tokens; the quantized formats keep their per-token parameters per head, so they scale the same way."""
    bytes_x2 = {oracle.FP16: 4, oracle.FP8: 2, oracle.INT8: 2, oracle.INT4: 1}  # 2 x bytes(precision)
    par = {oracle.FP16: 0, oracle.FP8: 0, oracle.INT8: 2, oracle.INT4: 4}
    for heads, layers in ((8, 32), (40, 40), (32, 32)):  # 8B GQA, 13B MHA, 7B MHA shapes, head_dim 128
        for dt in (oracle.FP16, oracle.FP8, oracle.INT8, oracle.INT4):
            full = oracle.block_bytes(dt, heads, 128, layers, 16)
            for tp in (1, 2, 4, 8):
                if heads % tp:
                    continue
                h = heads // tp
                token_size = h * 128 * bytes_x2[dt]            # the equation, per layer
                want = 16 * layers * (token_size + 2 * h * par[dt])
                if (h * 16 * (128 * bytes_x2[dt] // 2 + par[dt]) * 2) % 256 == 0:  # the layer's heads end on a 256-byte boundary
                    assert oracle.block_bytes(dt, h, 128, layers, 16) == want == full // tp
                else:
                    assert want <= oracle.block_bytes(dt, h, 128, layers, 16) < want + 256 * layers
    # a 2 MiB slab of the FP16 8B shape: 16 tokens on one GPU, 32 / 64 / 128 on a TP group of 2 / 4 / 8
    assert [oracle.geometry(oracle.FP16, 8 // tp, 128, 32, 2 * MiB).tokens_per_block for tp in (1, 2, 4, 8)] == [16, 32, 64, 128]


def test_lcm_slab_size_against_math_lcm_and_the_figure():
    """Sec. 5.2: slab = multiple of the lcm of the co-located block sizes.  Checked against Python's math.lcm;
    the pair FP16 / FP8 at 16 tokens per block gives the picture of the slab figure: one slab seen as 1 block by
    one model and as 2 blocks by the other; with per-token parameters the lcm explodes (INT8, INT4)."""
    import math

    rng = np.random.default_rng(10)
    for _ in range(200):
        n = int(rng.integers(1, 5))
        sizes = [int(rng.integers(1, 64)) * 256 * int(rng.choice([1, 2, 3, 5, 8])) for _ in range(n)]
        lo = int(rng.integers(0, 1 << 24))
        l = math.lcm(*sizes)
        want = l * max(1, -(-lo // l))
        assert oracle.lcm_slab_bytes(sizes, lo) == want
    b16, b8 = (oracle.block_bytes(d, 8, 128, 32, 16) for d in (oracle.FP16, oracle.FP8))
    assert (b16, b8) == (2 * MiB, 1 * MiB) and oracle.lcm_slab_bytes([b16, b8]) == 2 * MiB
    pool = oracle.Pool(2 * MiB, 64 * MiB)
    a, b = pool.model_add_tokens(oracle.FP16, 8, 128, 32, 16), pool.model_add_tokens(oracle.FP8, 8, 128, 32, 16)
    assert pool.blocks_per_slab(a) == 1 and pool.blocks_per_slab(b) == 2
    assert pool.model_geometry(a).tokens_per_block == pool.model_geometry(b).tokens_per_block == 16
    all4 = [oracle.block_bytes(d, 8, 128, 32, 16) for d in (oracle.FP16, oracle.FP8, oracle.INT8, oracle.INT4)]
    assert oracle.lcm_slab_bytes(all4) == math.lcm(*all4) == 2 * MiB * 5 * 13 * 17  # 2.2 GiB: no usable slab
    assert oracle.lcm_slab_bytes([0, 256]) == 0 and oracle.lcm_slab_bytes([(1 << 39) + 256, (1 << 39) + 512]) == 0
