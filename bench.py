#!/usr/bin/env python3
"""Benchmark of the KV-slab decode hot path on one MI355X.

A *step* is one decode step of one layer over the whole batch, one ``fs_decode_step_multi`` call: the
append of every sequence's newest token (quantize + scatter into its slab block; all models in the
launch that also prepares the work list), split-K paged attention over all co-located models, split
combine.  Slab allocation is host bookkeeping done while the workload
is set up (its rate is reported under ``extra``).  KV, block tables, queries and lengths are
resident in HBM before the timed region starts; the layer index rotates between steps so that no
step re-reads what the previous one left in cache.

Prints ONE JSON line: metric/value = algorithmic KV GB/s of the whole step on the four-model mixed
pool (config 5), plus ``roofline`` for the attention kernel (HIP-event time of that kernel alone)
and ``cpu_baseline`` (the CPU oracle timed on a bounded sample of the same workload).  The default
run adds under ``extra``:
  mixed_pool_loss  the control the benchmark definition asks for -- each model of the mixed pool alone in a
                   pool of its own precision with contiguous (identity) block tables and the SAME final
                   lengths: loss = 1 - BW_multi / (sum bytes_m / sum t_m);
  per_config       the same step timed on configs 2, 3 and 4, and on copies of config 2 with head_dim 64 and 256
                   (value, kernel time, fraction of peak).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
for _p in (ROOT, os.path.join(ROOT, "tests")):  # tests/: gpu_workload, the plumbing that stands a workload up
    if _p not in sys.path:
        sys.path.insert(0, _p)

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E bandwidth


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def cpu_baseline(gw, wl, layers, n_random, n_threads):
    """Time the CPU oracle (append of the newest token + decode attention) on a seeded sample of sequences of
    every model of the workload -- n_random seeded ones plus the shortest and the longest; returns
    (GB/s, tokens/s, description, threads used).  Only the two oracle calls are timed; drawing the sample's
    source rows and filling its host mirror of the cache (oracle append, one thread per sequence) are set-up."""
    from concurrent.futures import ThreadPoolExecutor

    import numpy as np

    import oracle
    from fs_inputs import gen, workloads

    total_bytes = 0
    total_time = 0.0
    total_seqs = 0
    used_threads = 1
    for k, s in enumerate(wl.models):
        lens_all = gw.lens[k]
        pick = set(gen.permutation(wl.seed, 77 + k, len(lens_all))[:n_random].tolist())
        pick.add(int(np.argmin(lens_all)))
        pick.add(int(np.argmax(lens_all)))
        seqs = np.array(sorted(pick), dtype=np.int64)
        lens = lens_all[seqs]
        g = oracle.geometry(s.kv_dtype, s.n_kv_heads, s.head_dim, s.n_layers, s.block_budget or wl.slab_bytes)
        T = g.tokens_per_block
        nblk = [workloads.blocks_needed(n, T) for n in lens]
        tab = np.zeros((len(seqs), max(nblk)), np.int32)
        nxt = 0
        for r, nb in enumerate(nblk):  # compact host mirror: only the sampled sequences' blocks
            tab[r, :nb] = np.arange(nxt, nxt + nb)
            nxt += nb
        mem = np.zeros(nxt * g.block_budget, np.uint8)
        layer = layers[k]
        dt = np.float32 if s.src_f32 else np.float16
        ks = vs = None
        if s.kv_dtype == workloads.FP8:
            ks, vs = workloads.fp8_scales_table(s.n_layers, s.n_kv_heads)
        k_last = np.empty((len(seqs), s.n_kv_heads, s.head_dim), dt)
        v_last = np.empty_like(k_last)

        def fill(r):  # cache fill of one sampled sequence (its blocks are its own): not timed
            n = int(lens[r])
            kr = workloads.source_rows(wl.seed, s.tag, layer, gen.WHICH_K, [n], s.n_kv_heads, s.head_dim, [seqs[r]], dt)
            vr = workloads.source_rows(wl.seed, s.tag, layer, gen.WHICH_V, [n], s.n_kv_heads, s.head_dim, [seqs[r]], dt)
            oracle.kv_append(mem, g, layer, kr, vr, np.zeros(n, np.int32), np.arange(n, dtype=np.int32), tab[r:r + 1], ks, vs)
            k_last[r], v_last[r] = kr[-1], vr[-1]

        with ThreadPoolExecutor(max_workers=n_threads) as ex:
            list(ex.map(fill, range(len(seqs))))
        q = gen.normal_q(wl.seed, s.tag, layer, seqs, s.n_q_heads, s.head_dim)
        t0 = time.perf_counter()
        oracle.kv_append(mem, g, layer, k_last, v_last, np.arange(len(seqs), dtype=np.int32),
                         (lens - 1).astype(np.int32), tab, ks, vs)
        oracle.decode_attention(mem, g, layer, s.n_q_heads, 1.0 / np.sqrt(s.head_dim), q, tab, lens, ks, vs,
                                n_threads=n_threads, want_lse=False)
        total_time += time.perf_counter() - t0
        total_bytes += int(lens.astype(np.int64).sum()) * workloads.kv_bytes_per_token_layer(s)
        total_seqs += len(seqs)
        used_threads = max(used_threads, min(n_threads, len(seqs)))
        del mem
    desc = (f"{n_random} seeded sequences per model plus its shortest and longest ({total_seqs} of "
            f"{sum(m.n_seq for m in wl.models)}), one layer each, append of the newest token + decode attention, "
            f"{total_bytes / 1e6:.1f} MB of KV")
    return total_bytes / total_time / 1e9, total_seqs / total_time, desc, used_threads


class Timed:
    """One workload stood up on the GPU and the step timed on it."""

    def __init__(self, wl, layers_cap=0, options=None):
        import torch

        import gpu_workload as harness
        import paper_2509_06261_amd as fs

        self.fs, self.wl, self.torch = fs, wl, torch
        log(f"[bench] workload {wl.name}: pool {wl.pool_bytes / 2**30:.1f} GiB, slabs {wl.slab_bytes // 1024} KiB, "
            f"placement {wl.placement}")
        self.gw = gw = harness.GpuWorkload(wl, options=options)

        class CountingAdapter(harness.AllocAdapter):
            calls = 0

            def alloc(self, model):
                CountingAdapter.calls += 1
                return super().alloc(model)

            def free(self, model, blk):
                CountingAdapter.calls += 1
                return super().free(model, blk)

        t0 = time.perf_counter()
        gw.place(CountingAdapter(gw.pool))
        self.t_place = time.perf_counter() - t0
        self.n_alloc_ops = CountingAdapter.calls
        self.stats = fs.fs_pool_stats(gw.pool)
        log(f"[bench] placed: {self.stats.live_blocks} live blocks of {self.stats.n_slabs} slabs in {self.t_place:.1f} s")
        self.n_layers_of = [s.n_layers if layers_cap <= 0 else min(layers_cap, s.n_layers) for s in wl.models]
        t0 = time.perf_counter()
        gw.populate([list(range(n)) for n in self.n_layers_of])
        torch.cuda.synchronize()
        log(f"[bench] KV populated for layers {self.n_layers_of} in {time.perf_counter() - t0:.1f} s")

    def close(self):
        self.gw.close()

    def algorithmic_bytes(self):
        """KV rows and parameters of every cached token (once per KV head), block-table entries and lengths read,
        queries read and outputs written: what one decode launch of one layer has to move."""
        import numpy as np

        gw, wl = self.gw, self.wl
        kv = gw.kv_bytes_per_layer_launch()
        table = sum(int(np.sum((gw.lens[k] + gw.T[m] - 1) // gw.T[m])) * 4 + 4 * s.n_seq
                    for k, (s, m) in enumerate(zip(wl.models, gw.model_ids)))
        qo = sum(2 * s.n_seq * s.n_q_heads * s.head_dim * 2 for s in wl.models)
        return kv + table + qo, kv

    def run(self, steps, warmup):
        """Times `steps` whole steps (after `warmup`), then the attention kernel alone over as many steps (HIP
        events on the launch stream).  Returns a dict of the measurements."""
        import numpy as np

        fs, gw, wl, torch = self.fs, self.gw, self.wl, self.torch
        n_layers_of = self.n_layers_of
        # per-layer batches (queries differ per layer), prepared before timing
        n_rot = max(n_layers_of)
        per_layer, keepalive = [], []
        for r in range(n_rot):
            layers = [r % n for n in n_layers_of]
            batches, keep = gw.make_batches(layers, with_lse=False)
            per_layer.append((layers, batches))
            keepalive.append(keep)
        self.first_layers = per_layer[0][0]
        ws = gw.workspace_for(per_layer[0][1])
        # newest-token rows for the per-step append (position n_b - 1 of every sequence), per model and layer
        step_appends, keep_rows = [], []
        for r in range(n_rot):
            appends, keep = gw.newest_token_appends(per_layer[r][0])
            step_appends.append(appends)
            keep_rows.append(keep)
        torch.cuda.synchronize()
        stream = torch.cuda.current_stream()

        def step(i):
            fs.fs_decode_step_multi(gw.pool, step_appends[i % n_rot], per_layer[i % n_rot][1], ws, stream)

        for i in range(warmup):
            step(i)
        torch.cuda.synchronize()
        status = fs.fs_decode_status(ws)
        assert status == 0, f"decode status {status}"
        t0 = time.perf_counter()
        for i in range(steps):
            step(warmup + i)
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
        # attention kernel alone, HIP events on the launch stream
        gw.set_option(fs.FS_OPT_KERNEL_TIMING, 1)
        kms = []
        for i in range(steps):
            step(warmup + steps + i)
            kms.append(fs.fs_pool_last_attention_kernel_ms(gw.pool))
        gw.set_option(fs.FS_OPT_KERNEL_TIMING, 0)
        kms = np.array(kms)
        algo, kv = self.algorithmic_bytes()
        del keepalive, keep_rows
        return {"ms_per_step": elapsed / steps * 1e3, "kernel_ms": kms, "algo_bytes": algo, "kv_bytes": kv,
                "timed_s": elapsed}

    def model_names(self):
        return [f"{s.name}:{s.n_q_heads}q/{s.n_kv_heads}kv/d{s.head_dim}/L{self.n_layers_of[k]}of{s.n_layers}"
                f"/T{self.gw.T[self.gw.model_ids[k]]}/{s.n_seq}seq" for k, s in enumerate(self.wl.models)]


def batched_allocator_rate(slab_bytes, n_slabs=65536, seq_blocks=64, rounds=40):
    """Blocks allocated + freed per second through fs_blocks_alloc / fs_blocks_free, a sequence's blocks per call
    (host bookkeeping only: the pool is created over an address that is never touched)."""
    from paper_2509_06261_amd import binding as fs

    pool = fs.fs_pool_create(slab_bytes, n_slabs * slab_bytes, 0x10000000)
    try:
        _, m = fs.fs_model_register(pool, 0, 8, 128, 8, None)
        n_seq = n_slabs // seq_blocks
        t0 = time.perf_counter()
        for _ in range(rounds):
            held = [fs.fs_blocks_alloc(pool, m, seq_blocks)[1] for _ in range(n_seq)]
            for ids in held[::2] + held[1::2]:
                fs.fs_blocks_free(pool, m, ids)
        dt = time.perf_counter() - t0
        return 2.0 * rounds * n_seq * seq_blocks / dt
    finally:
        fs.fs_pool_destroy(pool)


def summary(r):
    """value / kernel numbers of one Timed.run result, for the `extra` entries."""
    import numpy as np

    kms = r["kernel_ms"]
    k_mean = float(kms.mean())
    return {"bytes_per_launch": int(r["algo_bytes"]), "ms_per_step": round(r["ms_per_step"], 4),
            "value_GBps": round(r["algo_bytes"] / (r["ms_per_step"] * 1e-3) / 1e9, 1),
            "kernel_ms_mean": round(k_mean, 4),
            "kernel_ms_p10_p50_p90": [round(float(x), 4) for x in np.percentile(kms, [10, 50, 90])],
            "kernel_GBps": round(r["algo_bytes"] / (k_mean * 1e-3) / 1e9, 1),
            "kernel_frac_of_peak": round(r["algo_bytes"] / (k_mean * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
            "step_frac_of_peak": round(r["algo_bytes"] / (r["ms_per_step"] * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=40)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=5, help="workload: 2..5 (BASELINE.json configs, 1-based)")
    ap.add_argument("--head-dim", type=int, default=0, help="a copy of the workload with this head_dim (0 = as configured)")
    ap.add_argument("--kernel-mode", type=int, default=0, help="0 auto, 1 generic kernel, 2 MFMA kernel")
    ap.add_argument("--split-bytes", type=int, default=0)
    ap.add_argument("--layers", type=int, default=0, help="populate only the first N layers (0 = all)")
    ap.add_argument("--identity", action="store_true", help="control run: contiguous (identity) block placement")
    ap.add_argument("--only-model", type=int, default=-1, help="control run: only model k of the workload")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the mixed-pool-loss control and the configs 2-4 runs of the default invocation")
    ap.add_argument("--cpu-sample", type=int, default=32,
                    help="seeded sequences per model for the CPU oracle timing (the shortest and longest are added)")
    ap.add_argument("--copy-calibration-gib", type=float, default=0.0,
                    help="after the timed region also run a plain device copy of this size (counter calibration "
                         "for rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs)")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build targets one GPU (every box has one); --gpus must be 1. "
            "The path shards by sequence or by KV head with no exchange step (see DESIGN.md).")
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2509_06261_amd as fs
    from fs_inputs import workloads

    t_setup = time.perf_counter()
    wl = workloads.config(args.config)
    if args.head_dim:
        wl = workloads.with_head_dim(wl, args.head_dim)
    if args.identity:
        wl.placement = "identity"
    if args.only_model >= 0:
        wl.models = [wl.models[args.only_model]]
    plain = not (args.identity or args.only_model >= 0 or args.kernel_mode == 1 or args.layers or args.split_bytes or
                 args.head_dim)
    options = {}
    if args.kernel_mode:
        options[fs.FS_OPT_DECODE_KERNEL] = args.kernel_mode
    if args.split_bytes:
        options[fs.FS_OPT_SPLIT_BYTES] = args.split_bytes
    tw = Timed(wl, args.layers, options)
    gw = tw.gw
    r = tw.run(args.steps, args.warmup)
    ms_per_step, kms, algo_bytes, kv_bytes = r["ms_per_step"], r["kernel_ms"], r["algo_bytes"], r["kv_bytes"]
    kernel_ms = float(kms.mean())

    if args.copy_calibration_gib > 0:
        n = int(args.copy_calibration_gib * 2**30)
        src = torch.empty(n, dtype=torch.uint8, device=gw.device)
        src.fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        log(f"[bench] calibration: 3 device copies of {n} bytes each (reads {n}, writes {n})")
        del src, dst

    n_seq_total = sum(s.n_seq for s in wl.models)
    value = algo_bytes / (ms_per_step * 1e-3) / 1e9
    achieved = algo_bytes / (kernel_ms * 1e-3) / 1e9
    full_depth_tok_s = n_seq_total / (ms_per_step * 1e-3) / np.mean([s.full_layers or s.n_layers for s in wl.models])

    result = {
        "metric": "decode-attention KV GB/s, mixed-precision slab pool",
        "value": round(value, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "fp16/fp8_e4m3/int8/int4 KV, fp16 q, fp32 accumulate",
        "data": "synthetic (seeded N(0,1) table deviates; lengths per config)",
        "config": {
            "workload": wl.name + ("-identity" if args.identity else ""),
            "baseline_config_index": args.config,
            "models": tw.model_names(),
            "pool_GiB": wl.pool_bytes / 2**30,
            "slab_KiB": wl.slab_bytes // 1024,
            "placement": wl.placement,
            "churn_steps": wl.churn_steps if wl.placement == "churn" else 0,
            "live_slabs": int(tw.stats.live_blocks),
            "step": "fs_decode_step_multi: append of the newest token of every sequence + multi-model decode attention, one layer",
            "kernel_mode": args.kernel_mode,
        },
        "roofline": {
            "bound": "hbm",
            "kernel": "split-K paged decode attention",
            "achieved": round(achieved, 1),
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": round(achieved / HBM_PEAK_GBS, 4),
            "traffic": None,
            "kernel_ms_mean": round(kernel_ms, 4),
            "kernel_ms_p10_p50_p90": [round(float(x), 4) for x in np.percentile(kms, [10, 50, 90])],
            "algorithmic_bytes_per_launch": int(algo_bytes),
        },
        "extra": {
            "tokens_per_s_layer": round(n_seq_total / (ms_per_step * 1e-3), 1),
            "tokens_per_s_full_depth_equiv": round(float(full_depth_tok_s), 1),
            "kv_bytes_per_launch": int(kv_bytes),
            "alloc_free_calls": tw.n_alloc_ops,
            "alloc_free_calls_per_s_host": round(tw.n_alloc_ops / max(tw.t_place, 1e-9), 1),
            "alloc_free_blocks_per_s_batched": round(batched_allocator_rate(wl.slab_bytes), 1),
        },
    }
    # HBM traffic per launch measured with rocprofv3 --pmc (FETCH_SIZE / WRITE_SIZE, calibrated against a plain
    # copy) is recorded under profiles/ for the default workload and kernel; quote it when it applies.
    tpath = os.path.join(ROOT, "profiles", f"attention_traffic_cfg{args.config}.json")
    if os.path.exists(tpath) and plain:
        with open(tpath) as f:
            tr = json.load(f)
        result["roofline"]["traffic"] = tr.get("hbm_bytes_per_launch")
        result["roofline"]["traffic_source"] = tr.get("source")
    if not args.no_cpu_baseline:
        n_threads = min(os.cpu_count() or 1, 16)
        t0 = time.perf_counter()
        gbs, toks, desc, used = cpu_baseline(gw, wl, tw.first_layers, args.cpu_sample, n_threads)
        log(f"[bench] cpu oracle baseline took {time.perf_counter() - t0:.1f} s")
        result["cpu_baseline"] = {"value": round(gbs, 4), "unit": "GB/s", "cores": used, "kind": "oracle",
                                  "sample": desc, "tokens_per_s_layer": round(toks, 2)}
    final_lens = [np.array(l, dtype=np.int32) for l in gw.lens]
    tw.close()

    if plain and args.config == 5 and not args.no_extras:
        # ---- mixed-pool loss: every model alone, a pool of its own precision, identity tables, the same lengths ----
        ctl = []
        for k, s in enumerate(wl.models):
            spec = workloads.ModelSpec(s.name, s.kv_dtype, s.n_kv_heads, s.head_dim, s.n_layers, s.n_q_heads,
                                       final_lens[k], s.tag, s.src_f32, s.full_layers, s.block_budget)
            n_blocks = int(sum(workloads.blocks_needed(int(n), gw.T[gw.model_ids[k]]) for n in final_lens[k]))
            cw = workloads.Workload(f"control-{s.name}", wl.slab_bytes, (n_blocks + 8) * wl.slab_bytes, [spec],
                                    "identity", wl.seed)
            ct = Timed(cw)
            cr = ct.run(max(10, args.steps // 2), 3)
            ct.close()
            e = summary(cr)
            e["model"] = s.name
            ctl.append(e)
        sum_bytes = sum(e["bytes_per_launch"] for e in ctl)
        sum_kernel = sum(e["kernel_ms_mean"] for e in ctl)
        sum_step = sum(e["ms_per_step"] for e in ctl)
        bw_ctl_kernel = sum_bytes / (sum_kernel * 1e-3) / 1e9
        bw_ctl_step = sum_bytes / (sum_step * 1e-3) / 1e9
        result["extra"]["mixed_pool_loss"] = {
            "definition": "1 - BW_multi / (sum bytes_m / sum t_m); control = each model alone, single-precision pool, "
                          "identity (contiguous) block tables, the mixed pool's final (churned) lengths",
            "loss_kernel": round(1.0 - achieved / bw_ctl_kernel, 4),
            "loss_step": round(1.0 - value / bw_ctl_step, 4),
            "mixed_kernel_GBps": round(achieved, 1), "control_kernel_GBps": round(bw_ctl_kernel, 1),
            "mixed_step_GBps": round(value, 1), "control_step_GBps": round(bw_ctl_step, 1),
            "mixed_bytes": int(algo_bytes), "control_bytes": int(sum_bytes),
            "control": ctl,
        }
        # ---- the other configs ----
        per_config = {}
        # (and config 2 with head_dim 64 and 256: the MFMA kernel's other two instantiations)
        for cfg, head_dim in ((2, 128), (3, 128), (4, 128), (2, 64), (2, 256)):
            cw = workloads.config(cfg)
            if head_dim != 128:
                cw = workloads.with_head_dim(cw, head_dim)
            ct = Timed(cw)
            cr = ct.run(args.steps, args.warmup)
            e = summary(cr)
            e["workload"] = cw.name
            e["models"] = ct.model_names()
            ct.close()
            per_config[f"config{cfg}" + (f"_d{head_dim}" if head_dim != 128 else "")] = e
        result["extra"]["per_config"] = per_config
    result["extra"]["setup_s"] = round(time.perf_counter() - t_setup, 1)
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
