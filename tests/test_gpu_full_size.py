"""GPU parity at the benchmark's full sizes (configs 2-5), in the launch configuration bench.py times:
the whole workload is placed and decoded in one multi-model launch; the allocator is compared with
the oracle operation by operation over the complete trace; appended bytes and attention outputs are
compared with the CPU oracle on every sequence of config 2 and, for configs 3-5, on 32 seeded sequences per
model plus the shortest and the longest; on top of that all sequences are cross-checked between the
two independently written GPU kernels (MFMA vs generic).  Whole-prompt prefill over the same full-size pools, as
bench_prefill.py launches it (default kernel choice), is compared with the oracle on windows of query rows of
sampled sequences.

One workload is stood up once per config (module-scoped fixture: placement in lock-step with the oracle's
allocator, one layer of KV per model, one multi-model decode launch); the comparisons are separate tests per
model so that each one stays short."""
import numpy as np
import pytest

from fs_inputs import workloads

pytestmark = pytest.mark.gpu

# config -> (layer per model, oracle sample per model (None = every sequence), prefill sample per model)
# "2-d64" / "2-d256": config 2 with head_dim 64 / 256, the launches bench.py times on the MFMA decode kernel's other two
# instantiations (whole-prompt prefill there runs the 16-column MFMA kernel)
CONFIGS = {"2": ([17], None, 3), "3": ([3, 29], 32, 1), "4": ([11], 32, 1), "5": ([7, 0, 3, 9], 32, 1),
           "2-d64": ([17], None, 1), "2-d256": ([17], None, 1)}


def combination_applies(test, params):
    """Collected: the per-model tests for the models a config has, the small-item test on the two-model config."""
    cfg = params.get("stood_up")
    if "k" in params and params["k"] >= len(CONFIGS[cfg][0]):
        return False
    return test != "test_many_small_items" or cfg == "3"


@pytest.fixture(scope="module", params=sorted(CONFIGS), ids=lambda c: f"config{c}")
def stood_up(request):
    import gpu_harness

    cfg = request.param
    layers, n_random, prefill_random = CONFIGS[cfg]
    wl = workloads.config(int(cfg.split("-")[0]))
    if "-d" in cfg:
        wl = workloads.with_head_dim(wl, int(cfg.split("-d")[1]))
    print(f"[full-size] config {cfg}: placing", flush=True)
    par = gpu_harness.Parity(wl, zero_pool=False)  # asserts every allocator call and the final slab table identical
    try:
        print(f"[full-size] config {cfg}: {par.n_alloc_ops} allocator calls identical; decoding", flush=True)
        keep = par.populate_and_decode(layers)
        yield dict(cfg=cfg, par=par, wl=wl, layers=layers, keep=keep, n_random=n_random, prefill_random=prefill_random)
    finally:
        par.close()


def test_allocator_trace_identical_and_decode_ran(stood_up):
    par, wl = stood_up["par"], stood_up["wl"]
    assert par.n_alloc_ops >= sum(s.n_seq for s in wl.models)
    par.check_allocator_state()


@pytest.mark.parametrize("k", range(4))
def test_bytes_and_outputs_against_the_oracle(stood_up, k):
    """Model k of the config: appended bytes bit-identical, decode outputs and lse within the tolerance, on every
    sequence (config 2) or on 32 seeded sequences plus the shortest and the longest (configs 3-5)."""
    par, wl = stood_up["par"], stood_up["wl"]
    err, n = par.check_model(k, stood_up["layers"], stood_up["keep"], stood_up["n_random"])
    want = wl.models[k].n_seq if stood_up["n_random"] is None else min(wl.models[k].n_seq, 32)
    assert n >= want
    print(f"[full-size] config {stood_up['cfg']} model {k} ({wl.models[k].name}): {n} sequences, max abs err {err:.2e}")


def _decode_all(par, layers):
    import torch

    batches, keep = par.gw.make_batches(layers, with_lse=False)
    ws = par.gw.decode(batches)
    torch.cuda.synchronize()
    assert par.fs.fs_decode_status(ws) == 0
    return [o.float().cpu().numpy() for o in keep["out"]]


def test_every_sequence_mfma_against_generic_kernel(stood_up):
    par, wl, layers = stood_up["par"], stood_up["wl"], stood_up["layers"]
    import gpu_harness

    outs = {}
    for mode in (0, 1):
        par.gw.set_option(par.fs.FS_OPT_DECODE_KERNEL, mode)
        try:
            outs[mode] = _decode_all(par, layers)
        finally:
            par.gw.set_option(par.fs.FS_OPT_DECODE_KERNEL, 0)
    for k, s in enumerate(wl.models):
        tol = 2 * (gpu_harness.TOL_FP16 if s.kv_dtype == workloads.FP16 else gpu_harness.TOL_QUANT)
        d = float(np.max(np.abs(outs[0][k] - outs[1][k])))
        assert np.all(np.isfinite(outs[0][k])) and d <= tol, f"model {k}: kernels differ by {d:.3e}"
        # and the launch the oracle tests looked at is this same deterministic launch
        assert np.array_equal(outs[0][k], stood_up["keep"]["out"][k].float().cpu().numpy())


def test_many_small_items(stood_up):
    """16 KiB of KV per work item: more than 65535 items per batch (their products in the queue's interleaving of
    the batches pass 32 bits), some 140 splits per sequence for the combine."""
    assert stood_up["cfg"] == "3"  # (collected for the two-model config only)
    par, wl, layers = stood_up["par"], stood_up["wl"], stood_up["layers"]
    import gpu_harness

    n_items = [sum(-(-int(l) // 32) for l in s.lens) * s.n_kv_heads for s in wl.models]
    assert max(n_items) > 65535, n_items
    base = [o.float().cpu().numpy() for o in stood_up["keep"]["out"]]
    par.gw.set_option(par.fs.FS_OPT_SPLIT_BYTES, 16 * 1024)
    try:
        fine = _decode_all(par, layers)
    finally:
        par.gw.set_option(par.fs.FS_OPT_SPLIT_BYTES, 0)
    for k, s in enumerate(wl.models):
        tol = 2 * (gpu_harness.TOL_FP16 if s.kv_dtype == workloads.FP16 else gpu_harness.TOL_QUANT)
        d = float(np.max(np.abs(base[k] - fine[k])))
        print(f"[full-size] config 3: model {k}, {n_items[k]} items at 16 KiB: differs by {d:.2e}", flush=True)
        assert np.all(np.isfinite(fine[k])) and d <= tol, f"model {k}: split sizes differ by {d:.3e}"


@pytest.mark.parametrize("k", range(4))
def test_whole_prompt_prefill_windows_against_the_oracle(stood_up, k):
    par, wl = stood_up["par"], stood_up["wl"]
    perr = par.prefill_whole_prompts_and_check_windows(k, stood_up["layers"][k], stood_up["prefill_random"])
    print(f"[full-size] config {stood_up['cfg']}: prefill model {k}: max abs err {perr[0]:.2e} on {perr[1]} rows", flush=True)
