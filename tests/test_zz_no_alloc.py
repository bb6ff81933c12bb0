"""fs_decode_attention_multi_static (the entry point for callers that cannot allocate: its workspace is an array
the library holds in device memory) against fs_decode_attention_multi (caller workspace) and the CPU oracle,
through the C ABI: two calls in a row on one stream, the second on a smaller input, so that the second call
meets the first one's leftovers in the shared array."""
import numpy as np
import pytest

from fs_inputs.workloads import FP16, INT4, KiB, MiB, ModelSpec, Workload

pytestmark = pytest.mark.gpu


def _decode_both_ways(par, gw, layers, models, n_keep=None):
    """Decodes the given models' batches (the first n_keep sequences of each, default all) through both entry
    points; returns (outputs, lse) of the workspace call and of the static call, and the static call's status."""
    import torch

    fs = par.fs
    results = []
    status = torch.full((1,), 77, dtype=torch.int32, device=gw.device)
    for static in (False, True):
        batches, keep = gw.make_batches(layers, models=models)
        if n_keep is not None:
            for b in batches:
                b.n_seq = n_keep
        # poison the outputs: a row that a call leaves unwritten must not pass
        for o, l in zip(keep["out"], keep["lse"]):
            o.fill_(float("nan"))
            l.fill_(float("nan"))
        if static:
            fs.fs_decode_attention_multi_static(gw.pool, batches, status)
        else:
            ws = gw.decode(batches)
            torch.cuda.synchronize()
            assert fs.fs_decode_status(ws) == 0
        torch.cuda.synchronize()
        results.append(([o.cpu().numpy() for o in keep["out"]], [l.cpu().numpy() for l in keep["lse"]]))
    return results[0], results[1], int(status.item())


def test_static_scratch_entry_matches_workspace_entry_twice():
    import gpu_harness

    la = np.array([1, 40, 333, 1500, 2600, 64, 4100], np.int32)
    lb = np.array([7, 900, 61, 2300, 120, 3000, 59], np.int32)
    wl = Workload("noalloc", 256 * KiB, 128 * MiB,
                  [ModelSpec("a", FP16, 8, 128, 2, 32, la, tag=41), ModelSpec("b", INT4, 8, 128, 2, 32, lb, tag=42, src_f32=True)],
                  "interleave")
    par = gpu_harness.Parity(wl, zero_pool=True)
    try:
        gw, fs = par.gw, par.fs
        layers = [1, 0]
        gw.populate([[1], [0]])
        gw.set_option(fs.FS_OPT_SPLIT_BYTES, 64 * KiB)  # several splits per long sequence: partial records go through the scratch
        try:
            # call 1: both models, all sequences; call 2: one model, its first three sequences
            for models, n_keep in (([0, 1], None), ([1], 3)):
                (o_ws, l_ws), (o_st, l_st), status = _decode_both_ways(par, gw, layers, models, n_keep)
                assert status == 0
                for i, k in enumerate(models):
                    n = len(gw.lens[k]) if n_keep is None else n_keep
                    seqs = np.arange(n)
                    ref = par.oracle_sequences(k, layers[k], seqs)
                    err = par.check_attention(k, seqs, ref, o_st[i], l_st[i])
                    # the same kernels over the same splits: the two entry points agree to the last bit
                    assert np.array_equal(o_st[i][:n].view(np.uint16), o_ws[i][:n].view(np.uint16))
                    assert np.array_equal(l_st[i][:n], l_ws[i][:n])
                    print(f"models {models} keep {n_keep}: model {k} max abs err vs oracle {err:.2e}, identical to the "
                          "workspace entry point")
        finally:
            gw.set_option(fs.FS_OPT_SPLIT_BYTES, 0)
        # a batch whose upper bound exceeds the array is refused on the host, before any launch
        batches, keep = gw.make_batches(layers, models=[0], host_lens=False)
        batches[0].max_blocks = 1 << 22  # no host lengths: sized for max_blocks * tokens_per_block per sequence
        with pytest.raises(fs.FsError) as ei:
            fs.fs_decode_attention_multi_static(gw.pool, batches)
        assert ei.value.code == fs.FS_ERR_NOMEM and "static scratch" in str(ei.value)
    finally:
        par.close()
