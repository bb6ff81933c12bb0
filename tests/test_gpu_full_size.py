"""GPU parity at the benchmark's full sizes (configs 2-5), in the launch configuration bench.py times:
the whole workload is placed and decoded in one multi-model launch; the allocator is compared with
the oracle operation by operation over the complete trace; appended bytes and attention outputs are
compared on a seeded sample of sequences per model (always including the shortest and the longest)
that the CPU oracle recomputes one by one; every other sequence is cross-checked between the two
independently written GPU kernels (MFMA vs generic).  Whole-prompt prefill over the same full-size pools, as
bench_prefill.py launches it (default kernel choice), is compared with the oracle on windows of query rows of
sampled sequences."""
import numpy as np
import pytest

from fs_inputs import workloads

pytestmark = pytest.mark.gpu


def _full_size(cfg, layers, n_random, prefill_random=None, many_items=False):
    import torch
    import gpu_harness

    wl = workloads.config(cfg)
    print(f"[full-size] config {cfg}: placing", flush=True)
    par = gpu_harness.Parity(wl, zero_pool=False)
    try:
        print(f"[full-size] config {cfg}: {par.n_alloc_ops} allocator calls identical; decoding", flush=True)
        errs = par.run_and_check(layers, n_random=n_random)
        print(f"[full-size] config {cfg}: sampled max abs err {errs}", flush=True)
        # all sequences: the MFMA kernel against the generic kernel on the same pool contents
        gw, fs = par.gw, par.fs
        outs = {}
        for mode in (0, 1):
            fs.fs_set_kernel_mode(mode)
            try:
                batches, keep = gw.make_batches(layers, with_lse=False)
                ws = gw.decode(batches)
                torch.cuda.synchronize()
                assert fs.fs_decode_status(ws) == 0
                outs[mode] = [o.float().cpu().numpy() for o in keep["out"]]
            finally:
                fs.fs_set_kernel_mode(0)
        for k, s in enumerate(wl.models):
            tol = 2 * (gpu_harness.TOL_FP16 if s.kv_dtype == workloads.FP16 else gpu_harness.TOL_QUANT)
            d = float(np.max(np.abs(outs[0][k] - outs[1][k])))
            assert np.all(np.isfinite(outs[0][k])) and d <= tol, f"model {k}: kernels differ by {d:.3e}"
        if many_items:
            # 16 KiB of KV per work item: more than 65535 items per batch (their products in the queue's interleaving
            # of the batches pass 32 bits), some 140 splits per sequence for the combine
            n_items = [sum(-(-int(l) // 32) for l in s.lens) * s.n_kv_heads for s in wl.models]
            assert max(n_items) > 65535, n_items
            fs.fs_set_split_bytes(16 * 1024)
            try:
                batches, keep = gw.make_batches(layers, with_lse=False)
                ws = gw.decode(batches)
                torch.cuda.synchronize()
                assert fs.fs_decode_status(ws) == 0
                fine = [o.float().cpu().numpy() for o in keep["out"]]
            finally:
                fs.fs_set_split_bytes(0)
            for k, s in enumerate(wl.models):
                tol = 2 * (gpu_harness.TOL_FP16 if s.kv_dtype == workloads.FP16 else gpu_harness.TOL_QUANT)
                d = float(np.max(np.abs(outs[0][k] - fine[k])))
                print(f"[full-size] config {cfg}: model {k}, {n_items[k]} items at 16 KiB: differs by {d:.2e}", flush=True)
                assert np.all(np.isfinite(fine[k])) and d <= tol, f"model {k}: split sizes differ by {d:.3e}"
        if prefill_random is not None:
            for k in range(len(wl.models)):
                print(f"[full-size] config {cfg}: whole-prompt prefill of model {k}", flush=True)
                perr = par.prefill_whole_prompts_and_check_windows(k, layers[k], prefill_random)
                print(f"[full-size] config {cfg}: prefill model {k}: max abs err {perr[0]:.2e} on {perr[1]} rows", flush=True)
        return errs
    finally:
        par.close()


def test_config2_llama8b_fp16_full():
    _full_size(2, [17], n_random=6, prefill_random=3)


def test_config3_fp16_fp8_interleaved_full():
    _full_size(3, [3, 29], n_random=3, prefill_random=1, many_items=True)


def test_config4_int4_full():
    _full_size(4, [11], n_random=4, prefill_random=1)


def test_config5_four_model_churned_pool_full():
    _full_size(5, [7, 0, 3, 9], n_random=2, prefill_random=1)
