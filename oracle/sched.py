"""CPU oracle of FineServe's two-level scheduler (test infrastructure: only tests/, smoke() and the benchmarks'
cpu_baseline leg may import it).  Plain Python, the algorithms' steps in the paper's order and notation.

* select_batch   -- Algorithm 2 (Sec. 6.3), SLO-aware adaptive batching of one model's waiting queue.
* place_models   -- Algorithm 1 (Sec. 6.2), model-to-GPU placement with the score's averaged-mu proxy.

Readings where the paper is silent (also listed in the design notes):
  TTFT(R): the chunked-prefill latency of a request set is an input of Algorithm 2, obtained by profiling.  Here it
    is the three-coefficient model  c0 + c1 * sum(tokens) + c2 * sum(tokens^2)  (launch cost, linear layers,
    attention); the two sums are exact integers, and the expression is evaluated in this order in fp64.
  ties: requests of equal deadline keep their order in W; among equally long requests the one latest in deadline
    order is removed first.
  trim(S, Nmax, Tmax): the longest prefix of S in deadline order whose request count is <= Nmax and whose prompt
    tokens sum to <= Tmax.
  Algorithm 1: a GPU that cannot hold a model's base footprint is no candidate; equal scores go to the lowest
    GPU index; equal footprints keep their input order.
"""
from __future__ import annotations


def ttft(tokens, c0, c1, c2) -> float:
    """Predicted chunked-prefill latency of a set of requests (their prompt lengths)."""
    s1 = sum(int(n) for n in tokens)
    s2 = sum(int(n) * int(n) for n in tokens)
    return c0 + c1 * float(s1) + c2 * float(s2)


def select_batch(arrival, tokens, slo, n_max, t_max, c0, c1, c2, now):
    """Algorithm 2.  arrival[i], tokens[i]: the waiting requests W (index = identity).
    Returns (S, D): the requests to serve, in deadline order, and the dropped ones, in W order."""
    W = list(range(len(arrival)))
    S, D = [], []
    d = {}
    for r in W:                                        # lines 3-8
        d[r] = arrival[r] + slo
        if now + ttft([tokens[r]], c0, c1, c2) < d[r]:
            S.append(r)
        else:
            D.append(r)
    S.sort(key=lambda r: d[r])                         # line 10 (stable: W order among equal deadlines)
    while S:                                           # lines 11-16
        r0 = S[0]
        if now + ttft([tokens[r] for r in S], c0, c1, c2) < d[r0]:
            break
        longest = max(tokens[r] for r in S)
        r1 = [r for r in S if tokens[r] == longest][-1]
        S.remove(r1)
    kept, total = [], 0                                # line 17: trim
    for r in S:
        if len(kept) + 1 > n_max or total + tokens[r] > t_max:
            break
        kept.append(r)
        total += tokens[r]
    return kept, D


def place_models(footprint, mu, capacity):
    """Algorithm 1 with score(G | M) ~ (1 / |G'|) * sum_{m in G'} mu_m * K_rem(G').
    footprint[i] = F_M, mu[i] = marginal memory efficiency of model i; capacity[g] = T_G.
    Returns placement[i] = GPU of model i, or -1 where no GPU can hold the model."""
    order = sorted(range(len(footprint)), key=lambda i: -footprint[i])   # line 1 (stable)
    resident = [[] for _ in capacity]
    placement = [-1] * len(footprint)
    for M in order:
        best, best_score = -1, None
        for G in range(len(capacity)):
            members = resident[G] + [M]
            k_rem = capacity[G] - sum(footprint[m] for m in members)
            if k_rem < 0:
                continue
            score = (sum(mu[m] for m in members) / len(members)) * k_rem
            if best_score is None or score > best_score:
                best, best_score = G, score
        if best >= 0:
            resident[best].append(M)
            placement[M] = best
    return placement
