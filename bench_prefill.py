#!/usr/bin/env python3
"""Benchmark of prefill (chunked prefill) attention over the KV slab pool on one MI355X.

Not the headline benchmark (that is bench.py: decode): the prefill phase is the other user of the pool
(FineServe Sec. 2.1, 4.2).  A *step* prefills, for every model of the chosen BASELINE config, the last
``--chunk`` tokens (default: the whole prompt) of every sequence at one layer: ``fs_kv_append`` of the chunk's
keys and values, then ``fs_prefill_attention``.  The layer rotates between steps.  Queries are seeded N(0,1)
values drawn on the device (values do not change the work).

Prints ONE JSON line: value = attention TFLOP/s of the whole step (4 * head_dim flops per query head and
attended token), ``roofline`` for the prefill kernel (HIP-event time of the attention call alone, MFMA-bound:
fp16 dense peak 2.5 PFLOP/s) and ``cpu_baseline`` (the CPU oracle timed on a small sample of rows).
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

MFMA_F16_PEAK_TFLOPS = 2500.0  # MI355X published dense fp16 matrix rate


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=8)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", type=int, default=2, help="workload: 2..5 (BASELINE.json configs, 1-based)")
    ap.add_argument("--head-dim", type=int, default=0, help="a copy of the workload with this head_dim (0 = as configured)")
    ap.add_argument("--chunk", type=int, default=0, help="tokens prefilled per sequence (0 = the whole prompt)")
    ap.add_argument("--layers", type=int, default=2, help="layers populated and rotated over")
    ap.add_argument("--only-model", type=int, default=-1, help="only model k of the workload")
    ap.add_argument("--kernel", default="0,0", help="column blocks,waves: FS_OPT_PREFILL_COLUMN_BLOCKS / _WAVES (0,0 = automatic)")
    ap.add_argument("--cache-resident", action="store_true",
                    help="diagnosis: the attention reads every block table entry as the sequence's first block (K/V "
                         "stay in cache; results meaningless, timing = the kernel without its memory traffic)")
    ap.add_argument("--staged-dequant", type=int, default=1, help="FS_OPT_PREFILL_STAGED_DEQUANT (INT8 / INT4 models)")
    ap.add_argument("--pipelined", action="store_true", help="FS_OPT_PREFILL_PIPELINED (with --kernel 16,4)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration-gib", type=float, default=0.0,
                    help="after the timed region also run a plain device copy of this size (counter calibration "
                         "for rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs)")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench_prefill.py: this build targets one GPU; --gpus must be 1.")
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2509_06261_amd as fs
    from fs_inputs import gen, workloads
    from fs_inputs import device as gen_device
    import gpu_workload as harness

    ker_blocks, ker_waves = (int(x) for x in args.kernel.split(","))
    if ker_blocks not in (0, 1, 2, 4, 16) or ker_waves not in (0, 4, 8):
        raise SystemExit("bench_prefill.py: --kernel must be blocks in {0,1,2,4,16} and waves in {0,4,8}")
    options = {fs.FS_OPT_PREFILL_COLUMN_BLOCKS: ker_blocks, fs.FS_OPT_PREFILL_WAVES: ker_waves,
               fs.FS_OPT_PREFILL_PIPELINED: int(args.pipelined), fs.FS_OPT_PREFILL_STAGED_DEQUANT: int(args.staged_dequant)}
    wl = workloads.config(args.config)
    if args.head_dim:
        wl = workloads.with_head_dim(wl, args.head_dim)
    if args.only_model >= 0:
        wl.models = [wl.models[args.only_model]]
    gw = harness.GpuWorkload(wl, options=options)
    gw.place()
    n_layers_of = [min(args.layers, s.n_layers) for s in wl.models]
    gw.populate([list(range(n)) for n in n_layers_of])
    dev = gw.device

    per_model = []
    flops = 0.0
    kv_bytes = 0
    rows_total = 0
    for k, (s, m) in enumerate(zip(wl.models, gw.model_ids)):
        lens = gw.lens[k].astype(np.int64)
        n_new = lens if args.chunk <= 0 else np.minimum(lens, args.chunk)
        q_off = np.concatenate([[0], np.cumsum(n_new)]).astype(np.int32)
        n_rows = int(q_off[-1])
        # attended tokens: row r of a chunk sees len - n_new + r + 1 tokens
        attended = float(np.sum(n_new * (lens - n_new) + n_new * (n_new + 1) // 2))
        flops += 4.0 * s.head_dim * s.n_q_heads * attended
        kv_bytes += int(lens.sum()) * workloads.kv_bytes_per_token_layer(s)
        rows_total += n_rows
        # the chunk's tokens as (sequence, position) for the append, and its query rows (seeded, drawn on the device)
        seq_idx = np.repeat(np.arange(len(lens), dtype=np.int32), n_new)
        pos = np.concatenate([np.arange(l - n, l, dtype=np.int32) for l, n in zip(lens, n_new)])
        si, po = torch.from_numpy(seq_idx).to(dev), torch.from_numpy(pos).to(dev)
        dt = torch.float32 if s.src_f32 else torch.float16
        layers = []
        for layer in range(n_layers_of[k]):
            kb = torch.empty((n_rows, s.n_kv_heads, s.head_dim), dtype=dt, device=dev)
            vb = torch.empty_like(kb)
            gen_device.fill_rows(kb, wl.seed, s.tag, layer, gen.WHICH_K, si, po, s.n_kv_heads, s.head_dim)
            gen_device.fill_rows(vb, wl.seed, s.tag, layer, gen.WHICH_V, si, po, s.n_kv_heads, s.head_dim)
            q = torch.empty((n_rows, s.n_q_heads, s.head_dim), dtype=torch.float16, device=dev)
            gen_device.fill_rows(q, wl.seed, s.tag, layer, gen.WHICH_Q, si, po, s.n_q_heads, s.head_dim)
            layers.append((kb, vb, q))
        out = torch.empty((n_rows, s.n_q_heads, s.head_dim), dtype=torch.float16, device=dev)
        ws = torch.empty(fs.fs_prefill_workspace_bytes(len(lens)), dtype=torch.uint8, device=dev)
        one_block = gw.tables[k][:, :1].expand(-1, gw.tables[k].shape[1]).contiguous()
        per_model.append(dict(k=k, s=s, m=m, q_off=q_off, q_off_d=torch.from_numpy(q_off).to(dev), si=si, po=po,
                              layers=layers, out=out, ws=ws, sm=float(1.0 / np.sqrt(s.head_dim)), one_block=one_block))
    torch.cuda.synchronize()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    attn_ms = []

    def step(i, timed=False):
        for pm in per_model:
            layer = i % len(pm["layers"])
            kb, vb, q = pm["layers"][layer]
            fs.fs_kv_append(gw.pool, pm["m"], layer, kb, vb, pm["si"], pm["po"], gw.tables[pm["k"]])
            if timed:
                ev[0].record()
            tab = pm["one_block"] if args.cache_resident else gw.tables[pm["k"]]
            fs.fs_prefill_attention(gw.pool, pm["m"], layer, pm["s"].n_q_heads, pm["sm"], q, tab,
                                    gw.seq_lens[pm["k"]], pm["q_off_d"], pm["q_off"], pm["out"], None, pm["ws"])
            if timed:
                ev[1].record()
                ev[1].synchronize()
                attn_ms.append(ev[0].elapsed_time(ev[1]))

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    for pm in per_model:
        assert fs.fs_decode_status(pm["ws"]) == 0
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(args.warmup + i)
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) / args.steps * 1e3
    for i in range(args.steps):
        step(args.warmup + args.steps + i, timed=True)
    attn_ms_per_step = float(np.sum(attn_ms)) / args.steps
    if args.copy_calibration_gib > 0:
        n = int(args.copy_calibration_gib * 2**30)
        src = torch.empty(n, dtype=torch.uint8, device=dev)
        src.fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # measured HBM-side bytes per launch (counter runs summarised under profiles/), for the workload they were taken on
    traffic = None
    tpath = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles", "prefill_traffic_cfg2.json")
    if os.path.exists(tpath) and args.config == 2 and args.chunk <= 0 and args.only_model < 0 and (ker_blocks, ker_waves) == (0, 0):
        traffic = json.load(open(tpath))["hbm_bytes_per_launch"]
    result = {
        "metric": "prefill-attention TFLOP/s over the KV slab pool",
        "value": round(flops / (ms_per_step * 1e-3) / 1e12, 1),
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 3),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "fp16 MFMA over fp16/fp8_e4m3/int8/int4 KV, fp32 accumulate",
        "data": "synthetic (seeded N(0,1) table deviates; lengths per config)",
        "config": {
            "workload": wl.name + ("-whole-prompts" if args.chunk <= 0 else f"-last-{args.chunk}-tokens"),
            "baseline_config_index": args.config,
            "models": [f"{s.name}:{s.n_q_heads}q/{s.n_kv_heads}kv/d{s.head_dim}/T{gw.T[gw.model_ids[k]]}/{s.n_seq}seq"
                       for k, s in enumerate(wl.models)],
            "query_rows": rows_total,
            "step": "fs_kv_append(chunk) + fs_prefill_attention per model, one layer",
        },
        "roofline": {
            "bound": "mfma",
            "kernel": "paged prefill attention, workgroup kernel (8 waves x 32 logit columns share each K/V tile through LDS)" if (ker_blocks, ker_waves) == (0, 0) else f"paged prefill attention, variant {args.kernel}",
            "achieved": round(flops / (attn_ms_per_step * 1e-3) / 1e12, 1),
            "peak": MFMA_F16_PEAK_TFLOPS,
            "unit": "TFLOP/s",
            "frac": round(flops / (attn_ms_per_step * 1e-3) / 1e12 / MFMA_F16_PEAK_TFLOPS, 4),
            "traffic": traffic,
            "attention_ms_per_step": round(attn_ms_per_step, 3),
            "flops_per_step": flops,
            "kv_bytes_in_pool_per_layer": kv_bytes,
        },
    }
    if not args.no_cpu_baseline:
        # the oracle on a few rows of the first model's first sequence (fp64, one layer), bounded to seconds
        import oracle

        s = wl.models[0]
        g = oracle.geometry(s.kv_dtype, s.n_kv_heads, s.head_dim, s.n_layers, s.block_budget or wl.slab_bytes)
        n = int(min(gw.lens[0][0], 512))
        lens1 = np.array([n], np.int32)
        nb = workloads.blocks_needed(n, g.tokens_per_block)
        tab = np.arange(nb, dtype=np.int32)[None, :]
        mem = np.zeros(nb * g.block_budget, np.uint8)
        dtn = np.float32 if s.src_f32 else np.float16
        kr = workloads.source_rows(wl.seed, s.tag, 0, gen.WHICH_K, lens1, s.n_kv_heads, s.head_dim, [0], dtn)
        vr = workloads.source_rows(wl.seed, s.tag, 0, gen.WHICH_V, lens1, s.n_kv_heads, s.head_dim, [0], dtn)
        ks = vs = None
        if s.kv_dtype == workloads.FP8:
            ks, vs = workloads.fp8_scales_table(s.n_layers, s.n_kv_heads)
        si1, po1 = workloads.token_index(lens1)
        oracle.kv_append(mem, g, 0, kr, vr, si1, po1, tab, ks, vs)
        qh = gen.normal_q_chunks(wl.seed, s.tag, 0, [0], [0], [n], s.n_q_heads, s.head_dim)
        threads = min(8, os.cpu_count() or 1)
        t0 = time.perf_counter()
        oracle.prefill_attention(mem, g, 0, s.n_q_heads, 1.0 / np.sqrt(s.head_dim), qh, tab, lens1,
                                 np.array([0, n], np.int32), ks, vs, n_threads=threads, want_lse=False)
        dt_cpu = time.perf_counter() - t0
        f_cpu = 4.0 * s.head_dim * s.n_q_heads * n * (n + 1) / 2
        result["cpu_baseline"] = {"value": round(f_cpu / dt_cpu / 1e12, 6), "unit": "TFLOP/s", "cores": threads,
                                  "kind": "oracle", "sample": f"whole-prompt prefill of one {n}-token sequence of model 0, one layer"}
    print(json.dumps(result), flush=True)
    gw.close()


if __name__ == "__main__":
    main()
