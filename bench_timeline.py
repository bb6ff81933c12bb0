"""Timeline of the MFMA decode-attention kernel: where the waves' time goes inside a launch.

Loads the library's profiling twin (``libfineserve_timeline.so``: the same sources with ``-DFS_TIMELINE``, built by
``python paper_2509_06261_amd/build.py --timeline``), in which every wave of the decode kernel leaves clock readings
(the 100 MHz constant clock) at the end of the launch's workspace: per wave its start and end, per work item the moment
its ticket is resolved, its address table is ready, the tile loop is left and its output is written (clock readings
are ordered against memory operations only: arithmetic of the last tiles may land behind the third one).  One launch of a
config's decode attention (one layer) is read back and summarised: how the launch's wave time divides into look-ups,
streaming, output, pauses between items and idling at the end, how long items of each size tier take, and when the
tiers start.  The product library is never touched; the readings cost the kernel about 1 %.

    python bench_timeline.py [config ...]        (default: 5 2 4)
    python bench_timeline.py --prefill [config ...]   the prefill workgroup kernel instead (default: 2 4): per workgroup
        its start and end and the summed phases of its items, per item its begin and end; whole-prompt prefill as
        bench_prefill.py launches it, the last launch read back
"""
import os
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
TWIN = os.path.join(ROOT, "paper_2509_06261_amd", "libfineserve_timeline.so")
os.environ["FINESERVE_LIBRARY"] = TWIN  # before the package is imported
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))


def prefill(configs):
    import ctypes

    import numpy as np
    import torch  # noqa: F401

    import bench_prefill
    import paper_2509_06261_amd as fs
    from paper_2509_06261_amd import binding

    group_rows, item_rows = ctypes.c_uint64(0), ctypes.c_uint64(0)
    binding._L.fs_prefill_timeline_bytes.restype = ctypes.c_uint64
    tl_bytes = int(binding._L.fs_prefill_timeline_bytes(ctypes.byref(group_rows), ctypes.byref(item_rows)))
    group_rows = int(group_rows.value)
    seen = {}
    plain = fs.fs_prefill_attention

    def watched(*a, **k):  # the workspace is the call's last argument: clear its readings, remember it
        ws = a[-1]
        ws[ws.numel() - tl_bytes:].zero_()
        seen["ws"] = ws
        return plain(*a, **k)

    fs.fs_prefill_attention = binding.fs_prefill_attention = watched
    pct = lambda x, p: np.percentile(x, p).round(1)
    for cfg in configs:
        sys.argv = ["bench_prefill.py", "--config", str(cfg), "--no-cpu-baseline", "--steps", "2", "--warmup", "1"]
        try:
            bench_prefill.main()
        except SystemExit:
            pass
        ws = seen["ws"]
        rows = ws[ws.numel() - tl_bytes:].cpu().numpy().view(np.uint64).reshape(-1, 8)
        groups, items = rows[:group_rows], rows[group_rows:]
        groups, items = groups[groups[:, 0] != 0], items[items[:, 0] != 0]
        t0 = int(groups[:, 0].min())
        us = lambda x: (x.astype(np.int64) - t0) / 100.0
        g_end = us(groups[:, 1])
        span = float(g_end.max())
        begin, end = us(items[:, 0]), us(items[:, 1])
        qt = (items[:, 2] & 0xfffff).astype(np.int64)
        seq = (items[:, 2] >> 32).astype(np.int64)
        draw = (items[:, 3] >> 32).astype(np.float64) / 100.0
        dur = end - begin
        total = len(groups) * span
        ph = groups[:, 4:8].astype(np.float64).sum(axis=0) / 100.0
        n = len(items)
        fit, *_ = np.linalg.lstsq(np.vstack([np.ones(n), qt + 1]).T, dur, rcond=None)
        print(f"prefill, config {cfg}: {len(groups)} workgroups, {n} work items (sequence, KV head, query tile), launch {span:.1f} us")
        print(f"  workgroups end p0/p10/p50/p90/p100 {pct(g_end, [0, 10, 50, 90, 100])}; idle at the end {100 * float(np.sum(span - g_end)) / total:.1f} % "
              f"of the workgroups' time, inside items {100 * float(dur.sum()) / total:.1f} %, draw and its barriers {100 * float(draw.sum()) / total:.1f} % "
              f"({pct(draw, 50)} us per item)")
        print(f"  an item takes {pct(dur, 50)} ({pct(dur, 10)}-{pct(dur, 90)}) us; least squares: {fit[0]:.2f} us + {fit[1]:.3f} us x (query tile index + 1); "
              f"the fixed part is {100 * fit[0] * n / total:.1f} % of the workgroups' time")
        names = ["entry -> address table in LDS", "-> first sub-tiles staged", "-> last step done", "-> output written"]
        print("  phases per item (summed by the workgroups' first threads): " + ", ".join(f"{names[k]} {ph[k] / n:.2f} us" for k in range(4)))
        late = np.argsort(-end)[:3]
        print("  last items to end: " + "; ".join(f"sequence {seq[i]} tile {qt[i]}: {begin[i]:.0f} -> {end[i]:.0f} us" for i in late))


def main():
    import ctypes

    import numpy as np

    if not os.path.exists(TWIN):  # (build.py by path: importing the package would already load the library)
        import importlib.util

        spec = importlib.util.spec_from_file_location("fs_build", os.path.join(ROOT, "paper_2509_06261_amd", "build.py"))
        fs_build = importlib.util.module_from_spec(spec)
        spec.loader.exec_module(fs_build)
        fs_build.build(timeline=True)
    if "--prefill" in sys.argv[1:]:
        return prefill([int(a) for a in sys.argv[1:] if a != "--prefill"] or [2, 4])
    import torch

    import bench
    import paper_2509_06261_amd as fs
    from fs_inputs import workloads
    from paper_2509_06261_amd import binding

    wave_rows, item_rows = ctypes.c_uint64(0), ctypes.c_uint64(0)
    binding._L.fs_timeline_bytes.restype = ctypes.c_uint64
    tl_bytes = int(binding._L.fs_timeline_bytes(ctypes.byref(wave_rows), ctypes.byref(item_rows)))
    wave_rows = int(wave_rows.value)
    pct = lambda x, p: np.percentile(x, p).round(1)
    for cfg in [int(a) for a in sys.argv[1:]] or [5, 2, 4]:
        wl = workloads.config(cfg)
        t = bench.Timed(wl, layers_cap=2)
        gw = t.gw
        batches, keep = gw.make_batches([0] * len(wl.models), with_lse=False)
        need = fs.fs_decode_workspace_bytes(gw.pool, batches)
        ws = torch.zeros(need, dtype=torch.uint8, device="cuda:0")
        for _ in range(4):  # the last launch is the one read back
            ws[need - tl_bytes:].zero_()
            fs.fs_decode_attention_multi(gw.pool, batches, ws)
            torch.cuda.synchronize()
        assert fs.fs_decode_status(ws) == 0
        rows = ws[need - tl_bytes:].cpu().numpy().view(np.uint64).reshape(-1, 8)
        waves, items = rows[:wave_rows], rows[wave_rows:]
        waves, items = waves[waves[:, 0] != 0], items[items[:, 0] != 0]
        t0 = int(waves[:, 0].min())
        us = lambda x: (x.astype(np.int64) - t0) / 100.0
        w_start, w_end = us(waves[:, 0]), us(waves[:, 1])
        span = float(w_end.max())
        begin, table, tiles, end = us(items[:, 0]), us(items[:, 1]), us(items[:, 2]), us(items[:, 3])
        wave = (items[:, 4] & 0xffffffff).astype(np.int64)
        batch = ((items[:, 4] >> 32) & 0xff).astype(np.int64)
        tier = ((items[:, 4] >> 40) & 0xff).astype(np.int64)
        runs = (items[:, 5] & 0xffffffff).astype(np.int64)
        order = np.lexsort((begin, wave))
        same = wave[order][1:] == wave[order][:-1]
        gap = (begin[order][1:] - end[order][:-1])[same]
        total = len(waves) * span
        share = lambda x: 100.0 * float(np.sum(x)) / total
        print(f"config {cfg} ({wl.name}): {len(waves)} waves, {len(items)} work items, launch {span:.1f} us "
              f"(first wave's start to last wave's end)")
        print(f"  share of the waves' time: look-ups (ticket resolved -> address table ready) {share(table - begin):.1f} %, "
              f"streaming (-> clock reading behind the tile loop) {share(tiles - table):.1f} %, rest of the item (output; with a refill-free "
              f"last turn also what of that turn the compiler placed behind the reading) {share(end - tiles):.1f} %, "
              f"between items {share(gap):.1f} %, idle at the end of the launch {share(span - w_end):.1f} %")
        print(f"  per item, median (p10-p90): look-ups {pct(table - begin, 50)} ({pct(table - begin, 10)}-{pct(table - begin, 90)}) us, "
              f"rest of the item {pct(end - tiles, 50)} ({pct(end - tiles, 10)}-{pct(end - tiles, 90)}) us, "
              f"between items {pct(gap, 50)} us; items per wave {pct(waves[:, 2].astype(np.int64), 10)}-{pct(waves[:, 2].astype(np.int64), 90)}")
        print(f"  waves: first request {pct(np.array([table[wave == w].min() for w in np.unique(wave)]) , 50)} us after the launch's start (median); "
              f"end p0/p10/p50/p90/p100 {pct(w_end, [0, 10, 50, 90, 100])}; mean idle at the end {float(np.mean(span - w_end)):.1f} us")
        for b in sorted(set(batch.tolist())):
            s = wl.models[b]
            for tr in sorted(set(tier[batch == b].tolist())):
                m = (batch == b) & (tier == tr)
                full = m & (runs == runs[m].max())
                d = (end - begin)[full]
                print(f"  {s.name:14s} tier {tr}: {int(m.sum()):6d} items, {int(runs[m].max()):4d} runs at most; a full-sized item takes "
                      f"{pct(d, 50)} ({pct(d, 10)}-{pct(d, 90)}) us; started between {begin[m].min():.0f} and {begin[m].max():.0f} us")
        t.close()


if __name__ == "__main__":
    main()
