"""Pins of the scheduler oracle (oracle/sched.py): hand-worked examples of Algorithm 2, its invariants on random
queues, the common-deadline special case against the textbook result, a from-scratch rescan over the number of
removals, and Algorithm 1 against the paper's placement table, its score formula and its stated properties."""
import itertools
import os

import numpy as np
import pytest

from oracle import sched


def _examples(golden_dir):
    out = []
    for line in open(os.path.join(golden_dir, "sched_alg2_worked_examples.txt")):
        if line.startswith("#") or not line.strip():
            continue
        name, par, reqs, sel, drp = [x.strip() for x in line.split("|")]
        slo, now, c0, c1, c2, n_max, t_max = par.split()
        arr = [float(r.split(":")[0]) for r in reqs.split()]
        tok = [int(r.split(":")[1]) for r in reqs.split()]
        out.append((name, arr, tok, float(slo), int(n_max), int(t_max), float(c0), float(c1), float(c2), float(now),
                    [int(x) for x in sel.split()], [int(x) for x in drp.split()]))
    return out


def test_alg2_worked_examples(golden_dir):
    ex = _examples(golden_dir)
    assert len(ex) == 5
    for name, arr, tok, slo, n_max, t_max, c0, c1, c2, now, sel, drp in ex:
        S, D = sched.select_batch(arr, tok, slo, n_max, t_max, c0, c1, c2, now)
        assert (S, D) == (sel, drp), name


def _random_queue(rng, n):
    arr = np.round(rng.uniform(0, 2.0, n) * 16) / 16          # quantised: equal deadlines occur
    tok = rng.choice([16, 64, 100, 512, 512, 1000, 2048, 4096, 8000], n)
    slo = float(rng.choice([0.25, 0.5, 1.0, 2.0]))
    c0, c1, c2 = float(rng.choice([0.0, 0.01])), float(rng.choice([0.0, 5e-5, 2e-4])), float(rng.choice([0.0, 1e-9, 2e-8]))
    now = float(rng.uniform(0, 2.5))
    n_max, t_max = int(rng.choice([1, 4, 64, 10**6])), int(rng.choice([512, 8192, 10**9]))
    return arr.tolist(), [int(x) for x in tok], slo, n_max, t_max, c0, c1, c2, now


def test_alg2_invariants_and_rescan():
    rng = np.random.default_rng(31)
    for case in range(400):
        n = int(rng.integers(0, 40))
        arr, tok, slo, n_max, t_max, c0, c1, c2, now = _random_queue(rng, n)
        S, D = sched.select_batch(arr, tok, slo, n_max, t_max, c0, c1, c2, now)
        d = [a + slo for a in arr]
        alone_ok = [now + sched.ttft([tok[r]], c0, c1, c2) < d[r] for r in range(n)]
        assert D == [r for r in range(n) if not alone_ok[r]]                      # dropped: exactly the hopeless ones
        assert not set(S) & set(D) and len(set(S)) == len(S)
        assert all(d[a] <= d[b] for a, b in zip(S, S[1:]))                        # deadline order
        assert len(S) <= n_max and sum(tok[r] for r in S) <= t_max                # caps
        if S:
            assert now + sched.ttft([tok[r] for r in S], c0, c1, c2) < min(d[r] for r in S)   # the SLO of the batch's front
        # from scratch: the untrimmed batch is the deadline-ordered feasible set minus its k longest requests (the
        # latest first among equals), for the smallest k that lets the front make its deadline
        feas = sorted([r for r in range(n) if alone_ok[r]], key=lambda r: d[r])
        by_len = sorted(range(len(feas)), key=lambda k: (tok[feas[k]], k), reverse=True)
        for k in range(len(feas) + 1):
            rest = [feas[i] for i in sorted(set(range(len(feas))) - set(by_len[:k]))]
            if not rest or now + sched.ttft([tok[r] for r in rest], c0, c1, c2) < d[rest[0]]:
                break
        S_big, _ = sched.select_batch(arr, tok, slo, 10**9, 10**18, c0, c1, c2, now)
        assert S_big == rest
        assert S == S_big[:len(S)]                                                # trim keeps a prefix


def test_alg2_common_deadline_is_the_textbook_maximum():
    """All requests share one deadline and the latency is additive (c0 = c2 = 0): the most requests that can finish
    in time is what shortest-first packing gives (the Moore-Hodgson optimum for a common due date); removing the
    longest until the rest fits must reach the same count."""
    rng = np.random.default_rng(32)
    for _ in range(300):
        n = int(rng.integers(1, 30))
        tok = [int(x) for x in rng.integers(1, 5000, n)]
        c1, slo, now = 1e-4, 1.0, float(rng.uniform(0, 0.9))
        S, D = sched.select_batch([0.0] * n, tok, slo, 10**9, 10**18, 0.0, c1, 0.0, now)
        feasible = sorted(t for t in tok if now + c1 * t < slo)
        best = 0
        while best < len(feasible) and now + c1 * float(sum(feasible[:best + 1])) < slo:
            best += 1
        assert len(S) == best and len(D) == n - len(feasible)


def test_alg2_tiny_cases_against_exhaustive_search():
    """n <= 6: among all subsets that contain no hopeless request and whose front makes its deadline, the algorithm's
    batch is one of them, and with additive latency and a common deadline none is larger."""
    rng = np.random.default_rng(33)
    for _ in range(200):
        n = int(rng.integers(1, 7))
        tok = [int(x) for x in rng.choice([256, 512, 1024, 2048, 4096], n)]
        now, slo, c1 = float(rng.uniform(0, 0.5)), 0.75, 1e-4
        S, _ = sched.select_batch([0.0] * n, tok, slo, 10**9, 10**18, 0.0, c1, 0.0, now)
        best = 0
        for k in range(n + 1):
            for sub in itertools.combinations(range(n), k):
                if now + c1 * float(sum(tok[r] for r in sub)) < slo:
                    best = max(best, k)
        assert len(S) == best


def test_alg1_reproduces_the_papers_placement_table():
    """Table 'Placement Results': 70B AWQ (C) is placed first and alone on GPU 0; 8B FP16 (A) second on GPU 1; 8B FP8
    (B) third, next to A.  Footprints are weight bytes (proxy), mu = 1 / KV bytes per token (tokens per byte)."""
    GiB = float(1 << 30)
    F = [16.0 * GiB, 8.0 * GiB, 35.0 * GiB]                    # A: 8B fp16, B: 8B fp8, C: 70B 4-bit
    mu = [1.0 / (32 * 8 * 128 * 2 * 2), 1.0 / (32 * 8 * 128 * 2 * 1), 1.0 / (80 * 8 * 128 * 2 * 2)]
    assert sched.place_models(F, mu, [80.0 * GiB, 80.0 * GiB]) == [1, 1, 0]


def test_alg1_score_formula_properties_and_capacity():
    rng = np.random.default_rng(34)
    for _ in range(300):
        nm, ng = int(rng.integers(1, 9)), int(rng.integers(1, 5))
        F = [float(x) for x in rng.integers(1, 60, nm)]
        mu = [float(x) for x in rng.integers(1, 20, nm)]
        cap = [float(x) for x in rng.integers(20, 120, ng)]
        P = sched.place_models(F, mu, cap)
        # replay: at its turn every model sits on the arg-max GPU of the directly written score, and fits
        order = sorted(range(nm), key=lambda i: -F[i])
        res = [[] for _ in cap]
        for M in order:
            scores = []
            for G in range(ng):
                grp = res[G] + [M]
                k_rem = cap[G] - sum(F[m] for m in grp)
                scores.append(None if k_rem < 0 else (sum(mu[m] for m in grp) / len(grp)) * k_rem)
            cands = [s for s in scores if s is not None]
            if not cands:
                assert P[M] == -1
                continue
            assert scores[P[M]] == max(cands) and P[M] == scores.index(max(cands))
            res[P[M]].append(M)
        for G in range(ng):
            assert sum(F[m] for m in res[G]) <= cap[G]
    # property (ii) of Sec. 6.2: for equal remaining memory and resident mu, the smaller group is favoured
    assert sched.place_models([20.0, 10.0, 10.0, 5.0], [1.0, 1.0, 1.0, 5.0], [100.0, 100.0])[3] == 0
    # a model that fits nowhere is left unplaced, the others are not disturbed
    assert sched.place_models([90.0, 50.0, 50.0], [1.0, 1.0, 1.0], [60.0, 60.0]) == [-1, 0, 1]
