"""CPU oracle of FineServe's two-level scheduler (test infrastructure: only tests/, smoke() and the benchmarks'
cpu_baseline leg may import it).  Plain Python, written from the prose of Sec. 6.2 and Sec. 6.3; every set is
rescanned where it is needed (no running sums, no heaps).

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
    """Algorithm 2 (Sec. 6.3), restated from its prose.  arrival[i], tokens[i] describe waiting request i.

    A request's deadline is its arrival time plus the model's TTFT SLO.
    1. Requests that could not meet their deadline even if prefilled alone right now are given up (dropped).
    2. The rest are considered earliest deadline first.
    3. As long as prefilling all of them together would end after the most urgent one's deadline, the longest
       prompt is taken out again (it stays queued for a later round).
    4. What remains is cut to the model's caps on concurrent requests and batched prompt tokens.
    Returns (chosen, dropped): chosen in deadline order, dropped in queue order."""
    deadline = [a + slo for a in arrival]

    def finishes_in_time(batch, request):
        return now + ttft([tokens[i] for i in batch], c0, c1, c2) < deadline[request]

    # 1. hopeless requests
    dropped = [i for i in range(len(arrival)) if not finishes_in_time([i], i)]
    candidates = [i for i in range(len(arrival)) if finishes_in_time([i], i)]
    # 2. most urgent first; sorted() is stable, so equal deadlines keep their queue order
    candidates = sorted(candidates, key=lambda i: deadline[i])
    # 3. shed the longest prompts until the most urgent request is safe
    while candidates and not finishes_in_time(candidates, candidates[0]):
        longest = max(tokens[i] for i in candidates)
        victim = max(pos for pos, i in enumerate(candidates) if tokens[i] == longest)  # the latest such in deadline order
        del candidates[victim]
    # 4. the caps: the longest deadline-order prefix within n_max requests and t_max prompt tokens
    n_fit = 0
    while (n_fit < len(candidates) and n_fit + 1 <= n_max
           and sum(tokens[i] for i in candidates[:n_fit + 1]) <= t_max):
        n_fit += 1
    return candidates[:n_fit], dropped


def place_models(footprint, mu, capacity):
    """Algorithm 1 (Sec. 6.2), restated from its prose, with the score's averaged-mu proxy.
    footprint[i]: base memory footprint of model i; mu[i]: its marginal memory efficiency; capacity[g]: memory of
    GPU g.  Models are placed one at a time, the largest base footprint first; each goes to the GPU where
    (mean mu of the GPU's residents including the newcomer) x (memory left once all of them are loaded) is
    largest.  Returns placement[i] = GPU of model i, or -1 where no GPU can hold the model."""
    by_size = sorted(range(len(footprint)), key=lambda i: footprint[i], reverse=True)  # stable: input order among equals
    gpu_of = [-1] * len(footprint)

    def score(gpu, newcomer):
        group = [i for i in range(len(footprint)) if gpu_of[i] == gpu] + [newcomer]
        left = capacity[gpu] - sum(footprint[i] for i in group)
        if left < 0:
            return None  # does not fit
        return (sum(mu[i] for i in group) / len(group)) * left

    for model in by_size:
        scores = [score(gpu, model) for gpu in range(len(capacity))]
        fitting = [sc for sc in scores if sc is not None]
        if fitting:
            gpu_of[model] = scores.index(max(fitting))  # the lowest GPU index among equal scores
    return gpu_of
