"""Serving-loop measurement of the local scheduler (FineServe Sec. 6.3, Algorithm 2) over the slab-pool prefill path.

One 8B-shaped FP16-KV model on one GPU.  Synthetic requests (Poisson arrivals, log-normal prompt lengths) queue up;
at every scheduling point the waiting queue goes through fs_sched_select_batch (Algorithm 2) or through a plain
first-come-first-served batcher (the baseline of the paper's local-scheduler ablation); the chosen batch is then
REALLY prefilled: blocks from the slab allocator, fs_kv_append and fs_prefill_attention for every layer, timed with
HIP events, and the simulated clock advances by the measured time.  TTFT of a request = end of its batch's prefill
minus its arrival.  The latency model the scheduler uses (c0 + c1 * sum tokens + c2 * sum tokens^2) is fitted from
timed prefill batches of this run.  As in the paper's ablation the SLO is a multiple of the P90 TTFT that FCFS
reaches.  Prints one JSON line; `cpu_baseline` times the oracle's Algorithm 2 on the same queues.
The model's linear layers are not part of this library: "TTFT" here is the attention path's share of it.
"""
from __future__ import annotations

import argparse
import json
import sys
import time

import numpy as np


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--requests", type=int, default=600)
    ap.add_argument("--layers", type=int, default=8)
    ap.add_argument("--load", type=float, default=1.5, help="arrival rate as a multiple of the fitted token capacity")
    ap.add_argument("--slo-scale", type=float, default=1.0, help="SLO = scale x P90 TTFT of the FCFS run")
    ap.add_argument("--seed", type=int, default=20250906)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench_sched.py: this build runs on one GPU (--gpus 1).", file=sys.stderr)
        sys.exit(2)
    import torch

    if not torch.cuda.is_available():
        print("bench_sched.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    import paper_2509_06261_amd as fs

    dev = torch.device("cuda:0")
    H, D, NQ, L = 8, 128, 32, args.layers
    slab, pool_bytes = 2 << 20, 24 << 30
    pool_mem = torch.empty(pool_bytes, dtype=torch.uint8, device=dev)
    pool = fs.fs_pool_create(slab, pool_bytes, pool_mem)
    T, model = fs.fs_model_register(pool, fs.FS_KV_FP16, H, D, L)
    rng = np.random.default_rng(args.seed)
    torch.manual_seed(args.seed)
    n_max, t_max = 64, 32768
    max_rows = t_max
    k_src = torch.randn((max_rows, H, D), device=dev).to(torch.float16)
    v_src = torch.randn((max_rows, H, D), device=dev).to(torch.float16)
    q_src = torch.randn((max_rows, NQ, D), device=dev).to(torch.float16)
    out = torch.empty_like(q_src)
    sm = float(1.0 / np.sqrt(D))
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def prefill(lens):
        """Whole-prompt prefill of a batch through the slab pool; returns the measured GPU seconds."""
        lens = np.asarray(lens, np.int32)
        nblk = (lens + T - 1) // T
        table = np.zeros((len(lens), int(nblk.max())), np.int32)
        held = []
        for i, nb in enumerate(nblk):
            for j in range(int(nb)):
                rc, b = fs.fs_block_alloc(pool, model)
                assert rc == 0, "pool exhausted"
                table[i, j] = b
                held.append(b)
        q_off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
        n = int(q_off[-1])
        seq_idx = torch.from_numpy(np.repeat(np.arange(len(lens), dtype=np.int32), lens)).to(dev)
        pos = torch.from_numpy(np.concatenate([np.arange(l, dtype=np.int32) for l in lens])).to(dev)
        tab_d, len_d, off_d = torch.from_numpy(table).to(dev), torch.from_numpy(lens).to(dev), torch.from_numpy(q_off).to(dev)
        ws = torch.empty(fs.fs_prefill_workspace_bytes(len(lens)), dtype=torch.uint8, device=dev)
        ev0.record()
        for layer in range(L):
            fs.fs_kv_append(pool, model, layer, k_src[:n], v_src[:n], seq_idx, pos, tab_d)
            fs.fs_prefill_attention(pool, model, layer, NQ, sm, q_src[:n], tab_d, len_d, off_d, q_off, out[:n], None, ws)
        ev1.record()
        ev1.synchronize()
        for b in held:
            assert fs.fs_block_free(pool, model, b) == 0
        return ev0.elapsed_time(ev1) * 1e-3

    # ---- latency model: least squares over timed batches of this run ----
    shapes = [[256] * 4, [1024] * 4, [4096] * 2, [512] * 32, [2048] * 8, [8192], [64] * 16, [3000, 500, 1200], [1024] * 16]
    prefill(shapes[0])
    A, y = [], []
    for s in shapes:
        t = min(prefill(s) for _ in range(2))
        A.append([1.0, float(sum(s)), float(sum(x * x for x in s))])
        y.append(t)
    # (rows scaled by 1 / measured time: the fit minimises relative, not absolute, error)
    Aw = np.array(A) / np.array(y)[:, None]
    c0, c1, c2 = [max(float(v), 0.0) for v in np.linalg.lstsq(Aw, np.ones(len(y)), rcond=None)[0]]
    fit_err = float(np.max(np.abs(np.array(A) @ np.array([c0, c1, c2]) - np.array(y)) / np.array(y)))

    # ---- synthetic requests ----
    n_req = args.requests
    lens = np.clip(np.rint(rng.lognormal(np.log(1024.0), 0.8, n_req)), 16, 8192).astype(np.int32)
    mean_cost = c1 * float(lens.mean()) + c2 * float((lens.astype(np.float64) ** 2).mean())
    rate = args.load / mean_cost                         # requests per second
    arrival = np.cumsum(rng.exponential(1.0 / rate, n_req))

    def serve(policy, slo):
        """Runs the queue to the end; returns (ttft per request or inf when dropped, busy seconds, decision seconds)."""
        ttft = np.full(n_req, np.inf)
        waiting, nxt, t, busy, t_dec, n_dec = [], 0, 0.0, 0.0, 0.0, 0
        queues = []
        while nxt < n_req or waiting:
            while nxt < n_req and arrival[nxt] <= t:
                waiting.append(nxt)
                nxt += 1
            if not waiting:
                t = float(arrival[nxt])
                continue
            w = np.array(waiting)
            if policy == "alg2":
                h0 = time.perf_counter()
                sel, drp = fs.fs_sched_select_batch(arrival[w], lens[w], slo, n_max, t_max, c0, c1, c2, t)
                t_dec += time.perf_counter() - h0
                n_dec += 1
                queues.append((arrival[w].copy(), lens[w].copy(), t))
            else:  # first come first served, same caps, nothing dropped
                sel, tot = [], 0
                for k in range(len(w)):
                    if len(sel) + 1 > n_max or tot + int(lens[w[k]]) > t_max:
                        break
                    sel.append(k)
                    tot += int(lens[w[k]])
                sel, drp = np.array(sel, np.int32), np.zeros(0, np.int32)
            gone = set(int(x) for x in sel) | set(int(x) for x in drp)
            if len(sel):
                dt = prefill(lens[w[sel]])
                t += dt
                busy += dt
                ttft[w[sel]] = t - arrival[w[sel]]
            elif not len(drp):
                # nothing can be served now and nothing was dropped (cannot happen: a lone feasible request is served)
                t = float(arrival[nxt]) if nxt < n_req else t + 1e-3
            waiting = [r for k, r in enumerate(waiting) if k not in gone]
        return ttft, busy, t_dec, n_dec, queues, t

    ttft_fcfs, busy_f, _, _, _, end_f = serve("fcfs", 0.0)
    slo = args.slo_scale * float(np.percentile(ttft_fcfs, 90))
    ttft_alg2, busy_a, t_dec, n_dec, queues, end_a = serve("alg2", slo)
    att_f = float(np.mean(ttft_fcfs <= slo))
    att_a = float(np.mean(ttft_alg2 <= slo))

    result = {
        "metric": "TTFT-SLO attainment of the attention-path prefill, Algorithm 2 vs FCFS batching",
        "value": round(att_a, 4),
        "unit": "fraction of requests within the SLO",
        "n_gpus": 1,
        "higher_is_better": True,
        "vs_baseline": None,
        "data": "synthetic (Poisson arrivals, log-normal prompt lengths, N(0,1) fp16 q/K/V)",
        "config": {"workload": "one 8B-shaped FP16-KV model, whole-prompt prefill over the slab pool",
                   "requests": n_req, "layers": L, "load": args.load, "slo_scale": args.slo_scale,
                   "slo_s": round(slo, 5), "n_max": n_max, "t_max": t_max, "rate_req_per_s": round(rate, 2),
                   "mean_prompt_tokens": round(float(lens.mean()), 1)},
        "fcfs": {"attainment": round(att_f, 4), "p50_ttft_s": round(float(np.median(ttft_fcfs)), 5),
                 "p90_ttft_s": round(float(np.percentile(ttft_fcfs, 90)), 5), "makespan_s": round(end_f, 4)},
        "alg2": {"attainment": round(att_a, 4), "dropped": int(np.sum(~np.isfinite(ttft_alg2))),
                 "p50_ttft_s_served": round(float(np.median(ttft_alg2[np.isfinite(ttft_alg2)])), 5),
                 "makespan_s": round(end_a, 4), "decisions": n_dec,
                 "decision_us_mean": round(t_dec / max(n_dec, 1) * 1e6, 2)},
        "latency_model": {"c0_s": c0, "c1_s_per_token": c1, "c2_s_per_token2": c2, "max_rel_fit_error": round(fit_err, 3)},
    }
    # decision cost on a long queue (the serving loop's queues are short: there the call overhead dominates)
    nq = 4096
    qa, ql = np.sort(rng.uniform(0, 1.0, nq)), np.clip(np.rint(rng.lognormal(np.log(1024.0), 0.8, nq)), 16, 8192).astype(np.int32)
    h0 = time.perf_counter()
    for _ in range(20):
        big_sel, big_drp = fs.fs_sched_select_batch(qa, ql, 2.0, 1 << 30, 1 << 30, c0, c1, c2, 0.9)
    result["alg2"]["decision_us_queue_of_4096"] = round((time.perf_counter() - h0) / 20 * 1e6, 1)
    if not args.no_cpu_baseline:
        from oracle import sched as osched

        h0 = time.perf_counter()
        o_sel, o_drp = osched.select_batch(qa.tolist(), [int(x) for x in ql], 2.0, 1 << 30, 1 << 30, c0, c1, c2, 0.9)
        t_big = time.perf_counter() - h0
        assert o_sel == big_sel.tolist() and o_drp == big_drp.tolist(), "library and oracle disagree"

        h0 = time.perf_counter()
        for a, l, now in queues:
            osched.select_batch(a.tolist(), [int(x) for x in l], slo, n_max, t_max, c0, c1, c2, now)
        t_or = time.perf_counter() - h0
        result["cpu_baseline"] = {"value": round(t_or / max(len(queues), 1) * 1e6, 2), "unit": "us per decision",
                                  "cores": 1, "kind": "oracle", "sample": f"the {len(queues)} queues of this run",
                                  "us_queue_of_4096": round(t_big * 1e6, 1)}
    fs.fs_pool_destroy(pool)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
