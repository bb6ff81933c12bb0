"""CPU-only parity of the library's scheduler calls (fs_sched_select_batch, fs_sched_place_models) with the oracle:
identical index lists on the worked examples and on thousands of random queues and clusters (ties included), and
the argument checks.  No device is touched."""
import numpy as np
import pytest

import paper_2509_06261_amd as fs
from oracle import sched
from test_oracle_sched import _examples, _random_queue


def test_select_batch_worked_examples_through_the_abi(golden_dir):
    for name, arr, tok, slo, n_max, t_max, c0, c1, c2, now, sel, drp in _examples(golden_dir):
        S, D = fs.fs_sched_select_batch(arr, tok, slo, n_max, t_max, c0, c1, c2, now)
        assert (S.tolist(), D.tolist()) == (sel, drp), name


def test_select_batch_matches_oracle_on_random_queues():
    rng = np.random.default_rng(41)
    for case in range(3000):
        n = int(rng.integers(0, 120)) if case % 50 else int(rng.integers(500, 1500))
        arr, tok, slo, n_max, t_max, c0, c1, c2, now = _random_queue(rng, n)
        n_max, t_max = min(n_max, 2**31 - 1), min(t_max, 2**31 - 1)
        S, D = fs.fs_sched_select_batch(arr, tok, slo, n_max, t_max, c0, c1, c2, now)
        So, Do = sched.select_batch(arr, tok, slo, n_max, t_max, c0, c1, c2, now)
        assert S.tolist() == So and D.tolist() == Do, case


def test_place_models_matches_oracle():
    rng = np.random.default_rng(42)
    for case in range(2000):
        nm, ng = int(rng.integers(0, 24)), int(rng.integers(0, 9))
        F = rng.choice([4.0, 8.0, 8.0, 16.0, 35.5, 70.25], nm) * float(rng.choice([1.0, 1 << 30]))
        mu = rng.choice([1.0 / 65536, 1.0 / 131072, 1.0 / 327680, 3.0], nm)
        cap = rng.choice([80.0, 80.0, 141.0, 288.0], ng) * (float(1 << 30) if F.size and F.max() > 1e6 else 1.0)
        got = fs.fs_sched_place_models(F, mu, cap)
        assert got.tolist() == sched.place_models(F.tolist(), mu.tolist(), cap.tolist()), case


def test_scheduler_argument_checks():
    with pytest.raises(fs.FsError):
        fs.fs_sched_select_batch([0.0], [-5], 1.0, 8, 100, 0.0, 1e-4, 0.0, 0.0)
    with pytest.raises(fs.FsError):
        fs.fs_sched_select_batch([float("nan")], [5], 1.0, 8, 100, 0.0, 1e-4, 0.0, 0.0)
    with pytest.raises(fs.FsError):
        fs.fs_sched_select_batch([0.0], [5], 1.0, -1, 100, 0.0, 1e-4, 0.0, 0.0)
    S, D = fs.fs_sched_select_batch([], [], 1.0, 8, 100, 0.0, 1e-4, 0.0, 0.0)
    assert len(S) == 0 and len(D) == 0
    assert fs.fs_sched_place_models([], [], [80.0]).tolist() == []
    assert fs.fs_sched_place_models([10.0], [1.0], []).tolist() == [-1]
