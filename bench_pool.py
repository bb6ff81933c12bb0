"""Static partition vs one shared slab pool for two co-located models (FineServe Sec. 3.2, the experiment of the
static/dynamic figure; Sec. 5: the KV slab is the dynamic variant), driven through this library on one GPU.

Model A (FP16 KV) and model B (FP8 KV), both 8B-shaped, serve synthetic requests (Poisson arrivals, log-normal prompt
and output lengths).  Phase T1: both receive requests; phase T2: A is idle and B's rate doubles.  A request is
admitted (first come first served per model) when the slab allocator can give it the blocks of its prompt and its
output; it is then REALLY prefilled (fs_kv_append + fs_prefill_attention, all layers) and decoded one token per step
(fs_kv_append + decode attention, all layers) until its output is complete, and its blocks are freed.  The clock is
the measured GPU time (HIP events).  Two variants on the same memory and the same request trace:
  static : the memory is split in two halves, one pool per model (two fs_pool objects, one decode call per pool);
  shared : one pool, both models' blocks in the same slabs' pool, one fs_decode_attention_multi call per layer.
Reported per variant and phase: generated tokens per second, mean queue length, mean admission delay, mean slabs in
use per model.  Prints one JSON line.  No CPU oracle leg: the allocator's parity is covered by the tests; this is
a measurement of what the shared pool buys.
"""
from __future__ import annotations

import argparse
import json
import sys

import numpy as np


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--pool-gib", type=float, default=6.0)
    ap.add_argument("--layers", type=int, default=8)
    ap.add_argument("--phase-s", type=float, default=0.4, help="length of each phase on the measured-GPU-time clock")
    ap.add_argument("--rate-a", type=float, default=250.0, help="requests per second of model A in T1")
    ap.add_argument("--rate-b", type=float, default=250.0, help="requests per second of model B in T1 (doubles in T2)")
    ap.add_argument("--seed", type=int, default=20250906)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench_pool.py: this build runs on one GPU (--gpus 1).", file=sys.stderr)
        sys.exit(2)
    import torch

    if not torch.cuda.is_available():
        print("bench_pool.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    import paper_2509_06261_amd as fs

    dev = torch.device("cuda:0")
    H, D, NQ, L = 8, 128, 32, args.layers
    slab = 2 << 20
    n_slabs = int(args.pool_gib * (1 << 30)) // slab // 2 * 2
    pool_mem = torch.empty(n_slabs * slab, dtype=torch.uint8, device=dev)
    sm = float(1.0 / np.sqrt(D))
    MAXSEQ, MAXLEN = 1024, 8192
    rng = np.random.default_rng(args.seed)
    torch.manual_seed(args.seed)

    # ---- the request trace (shared by both variants) ----
    def arrivals(rate, t0, t1):
        out, t = [], t0
        while rate > 0:
            t += rng.exponential(1.0 / rate)
            if t >= t1:
                break
            out.append(t)
        return out

    P = args.phase_s
    trace = []  # (arrival, model, prompt, output)
    for model, spans in ((0, [(args.rate_a, 0.0, P)]), (1, [(args.rate_b, 0.0, P), (2 * args.rate_b, P, 2 * P)])):
        for rate, t0, t1 in spans:
            for t in arrivals(rate, t0, t1):
                prompt = int(np.clip(np.rint(rng.lognormal(np.log(1024.0), 0.7)), 16, 6000))
                output = int(np.clip(np.rint(rng.lognormal(np.log(192.0), 0.6)), 8, 1024))
                trace.append((t, model, prompt, output))
    trace.sort()

    k_src = torch.randn((MAXLEN, H, D), device=dev).to(torch.float16)
    q_src = torch.randn((MAXLEN, NQ, D), device=dev).to(torch.float16)
    out_buf = torch.empty_like(q_src)
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    class Engine:
        def __init__(self, pool, dtype):
            self.pool = pool
            self.T, self.m = fs.fs_model_register(pool, dtype, H, D, L)
            if dtype == fs.FS_KV_FP8_E4M3:
                sc = np.full((L, H), 4.0 / 448.0, np.float32)
                fs.fs_model_set_fp8_scales(pool, self.m, sc, sc)
            self.max_blocks = (MAXLEN + self.T - 1) // self.T
            self.table = np.zeros((MAXSEQ, self.max_blocks), np.int32)
            self.lens = np.zeros(MAXSEQ, np.int32)
            self.left = np.zeros(MAXSEQ, np.int32)
            self.blocks = [None] * MAXSEQ
            self.free_slots = list(range(MAXSEQ - 1, -1, -1))
            self.queue = []          # (arrival, prompt, output)
            self.done_tokens = 0
            self.delays = []

        def try_admit(self, now):
            """Admits from the queue head while blocks last; returns the admitted slots."""
            new = []
            while self.queue and self.free_slots:
                arrival, prompt, output = self.queue[0]
                need = (prompt + output + self.T - 1) // self.T
                got = []
                for _ in range(need):
                    rc, b = fs.fs_block_alloc(self.pool, self.m)
                    if rc != 0:
                        break
                    got.append(b)
                if len(got) < need:
                    for b in got:
                        fs.fs_block_free(self.pool, self.m, b)
                    break
                self.queue.pop(0)
                s = self.free_slots.pop()
                self.table[s, :need] = got
                self.lens[s], self.left[s], self.blocks[s] = prompt, output, got
                self.delays.append(now - arrival)
                new.append(s)
            return new

        def active(self):
            return np.nonzero(self.lens > 0)[0]

        def finish(self, slots):
            for s in slots:
                for b in self.blocks[s]:
                    assert fs.fs_block_free(self.pool, self.m, b) == 0
                self.lens[s], self.left[s], self.blocks[s] = 0, 0, None
                self.free_slots.append(int(s))

    def run(shared):
        if shared:
            pools = [fs.fs_pool_create(slab, n_slabs * slab, pool_mem)]
            eng = [Engine(pools[0], fs.FS_KV_FP16), Engine(pools[0], fs.FS_KV_FP8_E4M3)]
        else:
            half = n_slabs // 2 * slab
            pools = [fs.fs_pool_create(slab, half, pool_mem[:half]), fs.fs_pool_create(slab, half, pool_mem[half:])]
            eng = [Engine(pools[0], fs.FS_KV_FP16), Engine(pools[1], fs.FS_KV_FP8_E4M3)]
        ws = torch.empty(256 << 20, dtype=torch.uint8, device=dev)
        pws = torch.empty(fs.fs_prefill_workspace_bytes(MAXSEQ), dtype=torch.uint8, device=dev)
        now, nxt, steps = 0.0, 0, 0
        stats = {ph: {"tokens": [0, 0], "queue": [0.0, 0.0], "slabs": [0.0, 0.0], "time": 0.0} for ph in ("T1", "T2", "drain")}
        while nxt < len(trace) or any(e.queue for e in eng) or any(len(e.active()) for e in eng):
            while nxt < len(trace) and trace[nxt][0] <= now:
                t, m, prompt, output = trace[nxt]
                eng[m].queue.append((t, prompt, output))
                nxt += 1
            newly = [e.try_admit(now) for e in eng]
            if not any(len(e.active()) for e in eng):
                now = max(now, trace[nxt][0]) if nxt < len(trace) else now
                if nxt >= len(trace) and not any(e.queue for e in eng):
                    break
                continue
            ev0.record()
            # prefill of the newly admitted requests
            for e, new in zip(eng, newly):
                if not new:
                    continue
                lens = e.lens[new]
                q_off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
                n = int(q_off[-1])
                for c0 in range(0, len(new), 16):   # chunks of requests that fit the source buffers
                    part = new[c0:c0 + 16]
                    pl = e.lens[part]
                    while int(pl.sum()) > MAXLEN:
                        part, pl = part[:-1], pl[:-1]
                    # (requests cut off here are picked up by the next chunk only if the chunk loop revisits them;
                    #  prompts are capped at 6000 tokens, so a single request always fits)
                    off = np.concatenate([[0], np.cumsum(pl)]).astype(np.int32)
                    rows = int(off[-1])
                    si = torch.from_numpy(np.repeat(np.arange(len(part), dtype=np.int32), pl)).to(dev)
                    po = torch.from_numpy(np.concatenate([np.arange(x, dtype=np.int32) for x in pl])).to(dev)
                    tab = torch.from_numpy(e.table[part]).to(dev)
                    ld, od = torch.from_numpy(pl.astype(np.int32)).to(dev), torch.from_numpy(off).to(dev)
                    for layer in range(L):
                        fs.fs_kv_append(e.pool, e.m, layer, k_src[:rows], k_src[:rows], si, po, tab)
                        fs.fs_prefill_attention(e.pool, e.m, layer, NQ, sm, q_src[:rows], tab, ld, od, off, out_buf[:rows],
                                                None, pws)
                    rest = [s for s in new[c0:c0 + 16] if s not in set(part)]
                    assert not rest or len(part) >= 1
                    for s in rest:   # prefill the cut-off ones alone
                        x = int(e.lens[s])
                        si1 = torch.zeros(x, dtype=torch.int32, device=dev)
                        po1 = torch.arange(x, dtype=torch.int32, device=dev)
                        tab1 = torch.from_numpy(e.table[[s]]).to(dev)
                        l1 = torch.tensor([x], dtype=torch.int32, device=dev)
                        o1h = np.array([0, x], np.int32)
                        o1 = torch.from_numpy(o1h).to(dev)
                        for layer in range(L):
                            fs.fs_kv_append(e.pool, e.m, layer, k_src[:x], k_src[:x], si1, po1, tab1)
                            fs.fs_prefill_attention(e.pool, e.m, layer, NQ, sm, q_src[:x], tab1, l1, o1, o1h, out_buf[:x],
                                                    None, pws)
            # one decode step: every running sequence appends a token and attends
            acts = [e.active() for e in eng]
            dev_state = []
            for e, a in zip(eng, acts):
                if not len(a):
                    dev_state.append(None)
                    continue
                e.lens[a] += 1
                tab = torch.from_numpy(e.table[a]).to(dev)
                ld = torch.from_numpy(e.lens[a]).to(dev)
                si = torch.arange(len(a), dtype=torch.int32, device=dev)
                dev_state.append((tab, ld, si, ld - 1))
            for layer in range(L):
                batches = []
                for e, a, st in zip(eng, acts, dev_state):
                    if st is None:
                        continue
                    tab, ld, si, po = st
                    n = len(a)
                    fs.fs_kv_append(e.pool, e.m, layer, k_src[:n], k_src[:n], si, po, tab)
                    b = fs.make_batch(e.m, layer, NQ, sm, q_src[:n], tab, ld, out_buf[:n], None, e.lens[a])
                    if shared:
                        batches.append(b)
                    else:
                        fs.fs_decode_attention_multi(e.pool, [b], ws)
                if shared and batches:
                    fs.fs_decode_attention_multi(eng[0].pool, batches, ws)
            ev1.record()
            ev1.synchronize()
            dt = ev0.elapsed_time(ev1) * 1e-3
            ph = "T1" if now < P else ("T2" if now < 2 * P else "drain")
            st = stats[ph]
            st["time"] += dt
            for k, (e, a) in enumerate(zip(eng, acts)):
                st["tokens"][k] += len(a)
                st["queue"][k] += len(e.queue) * dt
                st["slabs"][k] += sum(len(e.blocks[s]) for s in a) * dt
                e.left[a] -= 1
                e.finish([s for s in a if e.left[s] <= 0])
            now += dt
            steps += 1
        res = {"steps": steps, "end_s": round(now, 4)}
        for ph, st in stats.items():
            t = max(st["time"], 1e-12)
            res[ph] = {"tokens_per_s": [round(x / t, 1) for x in st["tokens"]], "mean_queue": [round(x / t, 2) for x in st["queue"]],
                       "mean_slabs_in_use": [round(x / t, 1) for x in st["slabs"]], "seconds": round(st["time"], 4)}
        res["mean_admission_delay_s"] = [round(float(np.mean(e.delays)) if e.delays else 0.0, 5) for e in eng]
        res["generated_tokens"] = int(sum(sum(st["tokens"]) for st in stats.values()))
        for p in pools:
            fs.fs_pool_destroy(p)
        return res

    static = run(False)
    shared = run(True)
    result = {
        "metric": "generated tokens/s of two co-located models, shared slab pool vs static partition",
        "value": round(shared["generated_tokens"] / shared["end_s"], 1),
        "unit": "tokens/s (attention path, measured GPU time)",
        "n_gpus": 1,
        "higher_is_better": True,
        "vs_baseline": None,
        "data": "synthetic (Poisson arrivals, log-normal prompt and output lengths, N(0,1) fp16 q/K/V)",
        "config": {"workload": "8B-shaped FP16-KV model A + FP8-KV model B; T1 both active, T2 A idle and B at twice the rate",
                   "pool_GiB": round(n_slabs * slab / 2**30, 2), "slab_KiB": slab >> 10, "layers": L, "phase_s": P,
                   "rate_a": args.rate_a, "rate_b": args.rate_b, "requests": len(trace)},
        "static": static,
        "shared": shared,
        "speedup_end_to_end": round(static["end_s"] / shared["end_s"], 3),
    }
    print(json.dumps(result))


if __name__ == "__main__":
    main()
