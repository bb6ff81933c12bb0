"""CPU-only tests of the HIP library's host side: it loads, exports every declared symbol,
and its geometry and slab allocator agree bit for bit with the oracle's.  No kernel is launched:
the pool is created over a caller-supplied (never dereferenced) base address."""
import os
import re

import numpy as np
import pytest

import oracle
import paper_2509_06261_amd as fs
from fs_inputs import gen

FAKE_BASE = 0x10000000
KiB, MiB = 1 << 10, 1 << 20


class FsPoolAdapter:
    """alloc/free facade over the C ABI with the oracle Pool's interface."""

    def __init__(self, slab, pool_bytes):
        self.pool = fs.fs_pool_create(slab, pool_bytes, FAKE_BASE)

    def model_add(self, dtype, H, D, L, budget=None):
        return fs.fs_model_register(self.pool, dtype, H, D, L, budget)[1]

    def model_add_tokens(self, dtype, H, D, L, T):
        return fs.fs_model_register_tokens(self.pool, dtype, H, D, L, T)[1]

    def alloc(self, m):
        return fs.fs_block_alloc(self.pool, m)

    def free(self, m, b):
        return fs.fs_block_free(self.pool, m, b)

    def close(self):
        fs.fs_pool_destroy(self.pool)


def test_every_declared_symbol_is_exported():
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    text = open(os.path.join(root, "include", "fineserve.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(fs_[a-z0-9_]+)\s*\(", text))
    assert declared, "no declarations found"
    assert declared == set(fs.binding.EXPORTS)
    for name in declared:
        assert hasattr(fs.binding._L, name), name


@pytest.mark.parametrize("dtype", [0, 1, 2, 3])
def test_geometry_matches_oracle(dtype):
    p = fs.fs_pool_create(2 * MiB, 64 * MiB, FAKE_BASE)
    rng = np.random.default_rng(dtype)
    shapes = [(8, 128, 32, None), (8, 128, 8, None), (40, 128, 40, None), (40, 128, 10, None), (4, 64, 1, 64 * KiB)]
    shapes += [(int(rng.integers(1, 41)), int(rng.choice([8, 16, 32, 64, 128, 256, 512])), int(rng.integers(1, 48)),
                int(rng.choice([64 * KiB, 512 * KiB, 2 * MiB]))) for _ in range(40)]
    for H, D, L, budget in shapes:
        try:
            og = oracle.geometry(dtype, H, D, L, budget or 2 * MiB)
        except ValueError:
            with pytest.raises(fs.binding.FsError):
                fs.fs_model_register(p, dtype, H, D, L, budget)
            continue
        T, m = fs.fs_model_register(p, dtype, H, D, L, budget)
        g = fs.fs_model_geometry(p, m)
        assert T == og.tokens_per_block == g.tokens_per_block
        for f in ("row_bytes", "kv_tile", "par_tile", "head_chunk", "layer_bytes", "block_bytes", "block_budget",
                  "param_bytes"):
            assert getattr(g, f) == getattr(og, f), f
        assert g.blocks_per_slab == 2 * MiB // (budget or 2 * MiB)
        assert fs.fs_model_unregister(p, m) == 0
    fs.fs_pool_destroy(p)


def test_worked_block_id_example_through_the_abi(golden_dir):
    rows = [list(map(int, ln.split())) for ln in open(os.path.join(golden_dir, "kv_slab_fig_example.txt"))
            if ln.strip() and not ln.startswith("#")]
    slab = 64 * KiB
    a = FsPoolAdapter(slab, 4 * slab)
    spec = {r[0]: r for r in rows}
    m2 = a.model_add(fs.FS_KV_FP8_E4M3, 2, 64, 1, slab // spec[2][1])
    m1 = a.model_add(fs.FS_KV_FP16, 2, 64, 1, slab // spec[1][1])
    got2 = [a.alloc(m2)[1] for _ in range(4)]
    got1 = a.alloc(m1)[1]
    assert got2[3] == spec[2][4] and got1 == spec[1][4]
    a.close()


def _run_trace(slab, n_slabs, model_specs, n_ops, seed):
    o = oracle.Pool(slab, n_slabs * slab)
    a = FsPoolAdapter(slab, n_slabs * slab)
    add = lambda pool, s: pool.model_add_tokens(*s[1:]) if s[0] == "tokens" else pool.model_add(*s)
    om = [add(o, s) for s in model_specs]
    am = [add(a, s) for s in model_specs]
    assert om == am
    live = [[] for _ in model_specs]
    r = gen.uniform_ints(seed, 5, n_ops, 1 << 40)
    for step in range(n_ops):
        x = int(r[step])
        k = x % len(model_specs)
        if (x >> 8) % 100 < 45 and live[k]:
            idx = (x >> 16) % len(live[k])
            b = live[k][idx]
            live[k][idx] = live[k][-1]
            live[k].pop()
            assert o.free(om[k], b) == a.free(am[k], b) == 0
        else:
            (rc1, b1), (rc2, b2) = o.alloc(om[k]), a.alloc(am[k])
            assert rc1 == rc2
            if rc1 == 0:
                assert b1 == b2
                live[k].append(b1)
        if (x >> 30) % 1000 == 0:  # occasional invalid operations must fail identically
            bogus = (x >> 12) % (n_slabs * 4)
            kk = (k + 1) % len(model_specs)
            if bogus not in live[kk]:
                assert o.free(om[kk], bogus) == a.free(am[kk], bogus) < 0
    ost, ok, ou, ofs = o.dump()
    ast, ak, au, afs = fs.fs_pool_dump(a.pool)
    assert np.array_equal(ost, ast) and np.array_equal(ok, ak) and np.array_equal(ou, au) and np.array_equal(ofs, afs)
    for x, y in zip(om, am):
        assert np.array_equal(o.dump_live(x), fs.fs_model_dump_live(a.pool, y))
    st = fs.fs_pool_stats(a.pool)
    assert st.live_blocks == sum(len(v) for v in live) and st.slabs_free == len(afs)
    assert st.slabs_free + st.slabs_partial + st.slabs_full == n_slabs
    a.close()


def test_allocator_matches_oracle_one_block_per_slab():
    specs = [(0, 8, 128, 8, None), (1, 8, 128, 8, None), (2, 8, 128, 8, None), (3, 40, 128, 10, None)]
    _run_trace(2 * MiB, 512, specs, 300_000, seed=11)


def test_allocator_matches_oracle_many_blocks_per_slab():
    slab = 256 * KiB
    specs = [(0, 4, 64, 1, slab // 2), (1, 4, 64, 1, slab // 4), (3, 2, 64, 2, slab // 16), (2, 4, 64, 1, slab)]
    _run_trace(slab, 96, specs, 300_000, seed=12)


def test_batched_alloc_and_free_equal_successive_single_calls():
    """fs_blocks_alloc / fs_blocks_free against the oracle's allocator called once per block: the same ids in the same
    order, the same slab table afterwards; a request the pool cannot serve whole takes nothing."""
    slab = 256 * KiB
    specs = [(0, 4, 64, 1, slab // 4), (2, 4, 64, 1, slab), (3, 2, 64, 2, slab // 16)]
    n_slabs = 64
    o = oracle.Pool(slab, n_slabs * slab)
    a = FsPoolAdapter(slab, n_slabs * slab)
    om = [o.model_add(*sp) for sp in specs]
    am = [a.model_add(*sp) for sp in specs]
    held = [[] for _ in specs]
    r = gen.uniform_ints(21, 6, 4000, 1 << 40)
    refused = 0
    for step in range(4000):
        x = int(r[step])
        k = x % len(specs)
        if (x >> 8) % 100 < 45 and held[k]:
            ids = held[k].pop((x >> 16) % len(held[k]))
            for b in ids:
                assert o.free(om[k], int(b)) == 0
            assert fs.fs_blocks_free(a.pool, am[k], ids) == 0
        else:
            n = (x >> 20) % 40
            rc, ids = fs.fs_blocks_alloc(a.pool, am[k], n)
            want, rco = [], 0
            before = o.dump()
            for _ in range(n):
                rco, b = o.alloc(om[k])
                if rco != 0:
                    break
                want.append(b)
            if rco != 0:  # the oracle ran out part-way: the batched call must have refused and taken nothing
                for b in reversed(want):
                    assert o.free(om[k], b) == 0
                assert all(np.array_equal(u, v) for u, v in zip(before, o.dump()))  # (freeing in reverse restores it)
                assert rc == fs.FS_ERR_NOMEM
                refused += 1
            else:
                assert rc == 0 and list(ids) == want
                if n:
                    held[k].append(np.array(want, np.int32))
        if step % 500 == 499 or step == 3999:
            for u, v in zip(o.dump(), fs.fs_pool_dump(a.pool)):
                assert np.array_equal(u, v)
            for u, v in zip(om, am):
                assert np.array_equal(o.dump_live(u), fs.fs_model_dump_live(a.pool, v))
    assert refused > 0
    bad = np.array([held[0][0][0], 10 ** 6], np.int32) if held[0] else np.array([10 ** 6], np.int32)
    assert fs.fs_blocks_free(a.pool, am[0], bad) < 0
    assert fs.fs_blocks_alloc(a.pool, am[0], -1)[0] == fs.FS_ERR_INVALID
    a.close()


def test_paper_direction_sizing_matches_oracle():
    """fs_block_bytes / fs_slab_bytes_for_blocks / fs_model_register_tokens (Sec. 3.2 forward, Sec. 5.2 lcm slab)."""
    rng = np.random.default_rng(21)
    for _ in range(300):
        dt = int(rng.integers(0, 4))
        H, D, L, T = int(rng.integers(1, 41)), int(rng.choice([32, 64, 128, 256])), int(rng.integers(1, 41)), int(rng.integers(1, 300))
        assert fs.fs_block_bytes(dt, H, D, L, T) == oracle.block_bytes(dt, H, D, L, T)
    for _ in range(200):
        sizes = [int(rng.integers(1, 64)) * 256 * int(rng.choice([1, 2, 3, 5, 8])) for _ in range(int(rng.integers(1, 5)))]
        lo = int(rng.integers(0, 1 << 24))
        assert fs.fs_slab_bytes_for_blocks(sizes, lo) == oracle.lcm_slab_bytes(sizes, lo)
    assert fs.fs_block_bytes(0, 8, 128, 32, 0) == 0 and fs.fs_slab_bytes_for_blocks([0, 256]) == 0
    assert fs.fs_slab_bytes_for_blocks([(1 << 39) + 256, (1 << 39) + 512]) == 0
    # token-fixed registration in an lcm-sized slab pool; allocator traces identical to the oracle's
    shapes = [(0, 4, 64, 2, 16), (1, 4, 64, 2, 16), (2, 3, 64, 1, 5)]
    blocks = [fs.fs_block_bytes(*s) for s in shapes]
    slab = fs.fs_slab_bytes_for_blocks(blocks, 100 * KiB)
    assert slab == oracle.lcm_slab_bytes(blocks, 100 * KiB) and all(slab % b == 0 for b in blocks)
    pool = fs.fs_pool_create(slab, 64 * slab, FAKE_BASE)
    for s, b in zip(shapes, blocks):
        T, m = fs.fs_model_register_tokens(pool, *s)
        g = fs.fs_model_geometry(pool, m)
        assert T == s[4] == g.tokens_per_block and g.block_budget == g.block_bytes == b and g.blocks_per_slab == slab // b
    with pytest.raises(fs.FsError):
        fs.fs_model_register_tokens(pool, 0, 4, 64, 2, 17)  # its block size does not divide the slab
    fs.fs_pool_destroy(pool)
    _run_trace(slab, 64, [("tokens",) + s for s in shapes], 100_000, seed=13)


def test_error_codes_without_device():
    p = fs.fs_pool_create(64 * KiB, 1 * MiB, FAKE_BASE)
    with pytest.raises(fs.binding.FsError):
        fs.fs_pool_create(100, 1000, FAKE_BASE)  # slab not a multiple of 256
    with pytest.raises(fs.binding.FsError):
        fs.fs_model_register(p, 0, 1024, 512, 64)  # one token does not fit a 64 KiB block
    with pytest.raises(fs.binding.FsError):
        fs.fs_model_register(p, 7, 4, 64, 1)  # unknown dtype
    T, m = fs.fs_model_register(p, fs.FS_KV_FP16, 4, 64, 1)
    assert T == 64
    rc, b = fs.fs_block_alloc(p, m)
    assert (rc, b) == (0, 0)
    assert fs.fs_model_unregister(p, m) == fs.FS_ERR_STATE
    assert fs.fs_block_free(p, m, 1) == fs.FS_ERR_STATE
    assert fs.fs_block_free(p, m, -1) == fs.FS_ERR_INVALID
    assert fs.fs_block_free(p, m + 1, 0) == fs.FS_ERR_INVALID
    assert fs.fs_block_free(p, m, 0) == 0
    assert fs.fs_model_unregister(p, m) == 0
    fs.fs_pool_destroy(p)


def test_pool_options_are_per_pool_and_range_checked():
    a = fs.fs_pool_create(64 * KiB, 1 * MiB, FAKE_BASE)
    b = fs.fs_pool_create(64 * KiB, 1 * MiB, FAKE_BASE)
    try:
        defaults = {fs.FS_OPT_DECODE_KERNEL: 0, fs.FS_OPT_SPLIT_BYTES: 0, fs.FS_OPT_KERNEL_TIMING: 0,
                    fs.FS_OPT_PREFILL_COLUMN_BLOCKS: 0, fs.FS_OPT_PREFILL_WAVES: 0, fs.FS_OPT_PREFILL_PIPELINED: 0,
                    fs.FS_OPT_PREFILL_STAGED_DEQUANT: 1, fs.FS_OPT_LAST_PREFILL_KERNEL: 0}
        for opt, v in defaults.items():
            assert fs.fs_pool_get_option(a, opt) == v
        assert fs.fs_pool_set_option(a, fs.FS_OPT_DECODE_KERNEL, 2) == fs.FS_OK
        assert fs.fs_pool_set_option(a, fs.FS_OPT_SPLIT_BYTES, 64 * KiB) == fs.FS_OK
        assert fs.fs_pool_set_option(a, fs.FS_OPT_PREFILL_COLUMN_BLOCKS, 16) == fs.FS_OK
        assert fs.fs_pool_set_option(a, fs.FS_OPT_PREFILL_WAVES, 4) == fs.FS_OK
        assert fs.fs_pool_set_option(a, fs.FS_OPT_PREFILL_STAGED_DEQUANT, 0) == fs.FS_OK
        assert fs.fs_pool_get_option(a, fs.FS_OPT_DECODE_KERNEL) == 2
        assert fs.fs_pool_get_option(a, fs.FS_OPT_SPLIT_BYTES) == 64 * KiB
        assert fs.fs_pool_get_option(a, fs.FS_OPT_PREFILL_STAGED_DEQUANT) == 0
        for opt, v in defaults.items():  # the other pool is untouched
            assert fs.fs_pool_get_option(b, opt) == v
        for opt, bad in ((fs.FS_OPT_DECODE_KERNEL, 3), (fs.FS_OPT_DECODE_KERNEL, -1), (fs.FS_OPT_SPLIT_BYTES, 100),
                         (fs.FS_OPT_SPLIT_BYTES, 1 << 31), (fs.FS_OPT_PREFILL_COLUMN_BLOCKS, 8),
                         (fs.FS_OPT_PREFILL_COLUMN_BLOCKS, 3), (fs.FS_OPT_PREFILL_WAVES, 2),
                         (fs.FS_OPT_LAST_PREFILL_KERNEL, 1), (99, 0)):
            assert fs.fs_pool_set_option(a, opt, bad) == fs.FS_ERR_INVALID, (opt, bad)
        with pytest.raises(fs.FsError):
            fs.fs_pool_get_option(a, 99)
        assert fs.fs_pool_last_attention_kernel_ms(a) < 0  # nothing timed
    finally:
        fs.fs_pool_destroy(a)
        fs.fs_pool_destroy(b)


def test_model_stats_count_slabs_per_key():
    slab = 64 * KiB
    p = fs.fs_pool_create(slab, 64 * slab, FAKE_BASE)
    try:
        _, m1 = fs.fs_model_register(p, fs.FS_KV_FP16, 2, 64, 1, slab // 4)   # four blocks per slab
        _, m2 = fs.fs_model_register(p, fs.FS_KV_INT4, 2, 64, 1)              # one block per slab
        g1, g2 = fs.fs_model_geometry(p, m1), fs.fs_model_geometry(p, m2)
        ids1 = [fs.fs_block_alloc(p, m1)[1] for _ in range(10)]   # 2 full slabs + 1 partial holding 2 of 4
        ids2 = [fs.fs_block_alloc(p, m2)[1] for _ in range(3)]
        s1, s2 = fs.fs_model_stats(p, m1), fs.fs_model_stats(p, m2)
        assert (s1.slabs_full, s1.slabs_partial, s1.live_blocks, s1.free_blocks_in_partial_slabs) == (2, 1, 10, 2)
        assert (s2.slabs_full, s2.slabs_partial, s2.live_blocks, s2.free_blocks_in_partial_slabs) == (3, 0, 3, 0)
        assert s1.live_bytes == 10 * g1.block_budget and s2.live_bytes == 3 * slab
        assert s1.stranded_bytes == 10 * (g1.block_budget - g1.block_bytes)
        assert s2.stranded_bytes == 3 * (g2.block_budget - g2.block_bytes)
        tot = fs.fs_pool_stats(p)
        assert tot.slabs_full == s1.slabs_full + s2.slabs_full and tot.slabs_partial == s1.slabs_partial + s2.slabs_partial
        assert tot.live_blocks == 13 and tot.stranded_bytes == s1.stranded_bytes + s2.stranded_bytes
        assert fs.fs_block_free(p, m1, ids1[0]) == 0     # a full slab of key 1 becomes partial
        s1 = fs.fs_model_stats(p, m1)
        assert (s1.slabs_full, s1.slabs_partial, s1.live_blocks, s1.free_blocks_in_partial_slabs) == (1, 2, 9, 3)
        for b in ids2:
            assert fs.fs_block_free(p, m2, b) == 0
        s2 = fs.fs_model_stats(p, m2)
        assert (s2.slabs_full, s2.slabs_partial, s2.live_blocks, s2.live_bytes) == (0, 0, 0, 0)
        with pytest.raises(fs.FsError):
            fs.fs_model_stats(p, 7)
    finally:
        fs.fs_pool_destroy(p)


def test_timeline_readings_are_in_the_profiling_twin_only():
    """The product library carries no timeline code (no fs_timeline_bytes); the twin that bench_timeline.py loads does,
    and exports everything the header declares as well."""
    import ctypes
    import os

    import paper_2509_06261_amd as fs
    from paper_2509_06261_amd import binding

    assert not hasattr(binding._L, "fs_timeline_bytes")
    twin = os.path.join(os.path.dirname(binding.LIB_PATH), "libfineserve_timeline.so")
    if not os.path.exists(twin):
        pytest.skip("the profiling twin is not built (python paper_2509_06261_amd/build.py --timeline)")
    T = ctypes.CDLL(twin)
    T.fs_timeline_bytes.restype = ctypes.c_uint64
    assert T.fs_timeline_bytes(None, None) > 0
    for name in fs.binding.EXPORTS:
        assert hasattr(T, name), name
