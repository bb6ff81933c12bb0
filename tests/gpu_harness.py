"""Parity machinery for the GPU tests: drives the HIP library and the CPU oracle on the same
seeded workload and compares them (allocator state, appended bytes, attention outputs).

The oracle never sees a value produced by the GPU: its KV bytes come from its own quantizer
applied to source rows regenerated on the host by fs_inputs.gen, placed by its own allocator.
"""
from __future__ import annotations

import numpy as np

import oracle
from fs_inputs import gen, workloads

TOL_FP16 = 2e-3   # max-abs, FP16 KV (benchmark definition)
TOL_QUANT = 4e-3  # max-abs, FP8 / INT8 / INT4 KV
TOL_LSE = 1e-3


def prefill_lse_tolerance(sm_scale, head_dim, staged_dequant):
    """lse = log sum exp(logits) moves by at most the largest logit error.  FP16 and FP8 keys reach the matrix cores
    exactly, and so do INT8 / INT4 codes on the exact-code path: the decode bound TOL_LSE holds.  With staged
    dequantization the INT8 / INT4 keys are rounded to fp16 (relative 2^-12 per element): a logit moves by at most
    |scale| 2^-12 sum_d |q_d k_d|, about |scale| 2^-12 * 0.64 * head_dim for unit-normal q and k, i.e. 1.8e-3 at
    scale 1/sqrt(128) if every element's error had the same sign (observed: up to 9.3e-4).  Hence 2e-3 at the usual
    scale, growing with |scale| sqrt(head_dim) beyond it -- for that path only."""
    if staged_dequant:  # (FS_OPT_LAST_PREFILL_KERNEL bit 16: the launch really took that path)
        return 2e-3 * max(1.0, abs(float(sm_scale)) * float(np.sqrt(head_dim)))
    return TOL_LSE


class LockstepAdapter:
    """Feeds every allocator call to the HIP library and to the oracle and insists on identical answers."""

    def __init__(self, fs_adapter, opool, fs_ids, o_ids):
        self.a, self.o = fs_adapter, opool
        self.map = dict(zip(fs_ids, o_ids))
        self.n_ops = 0

    def alloc(self, m):
        rc, b = self.a.alloc(m)
        orc, ob = self.o.alloc(self.map[m])
        assert (rc, b if rc == 0 else -1) == (orc, ob if orc == 0 else -1), f"alloc mismatch at op {self.n_ops}"
        self.n_ops += 1
        return rc, b

    def free(self, m, blk):
        rc = self.a.free(m, blk)
        assert rc == self.o.free(self.map[m], blk), f"free mismatch at op {self.n_ops}"
        self.n_ops += 1
        return rc


class Parity:
    def __init__(self, wl: workloads.Workload, zero_pool=False):
        import paper_2509_06261_amd as fs
        import gpu_workload as harness

        self.fs = fs
        self.wl = wl
        self.gw = harness.GpuWorkload(wl, zero_pool=zero_pool)
        self.opool = oracle.Pool(wl.slab_bytes, wl.pool_bytes)
        self.o_ids = [self.opool.model_add_tokens(s.kv_dtype, s.n_kv_heads, s.head_dim, s.n_layers, s.tokens_per_block)
                      if s.tokens_per_block else
                      self.opool.model_add(s.kv_dtype, s.n_kv_heads, s.head_dim, s.n_layers, s.block_budget)
                      for s in wl.models]
        self.ogeom = [self.opool.model_geometry(m) for m in self.o_ids]
        for m, og in zip(self.gw.model_ids, self.ogeom):
            assert self.gw.T[m] == og.tokens_per_block
        adapter = LockstepAdapter(harness.AllocAdapter(self.gw.pool), self.opool, self.gw.model_ids, self.o_ids)
        self.gw.place(adapter)
        self.n_alloc_ops = adapter.n_ops
        self.check_allocator_state()

    def close(self):
        self.gw.close()

    def last_prefill_staged(self):
        """Whether the pool's latest prefill launch dequantized INT8 / INT4 operands while staging them."""
        return bool(self.fs.fs_pool_get_option(self.gw.pool, self.fs.FS_OPT_LAST_PREFILL_KERNEL) >> 16 & 1)

    def check_allocator_state(self):
        ost, ok, ou, ofs = self.opool.dump()
        st, key, used, fstack = self.fs.fs_pool_dump(self.gw.pool)
        key_map = np.full(65, -1, np.int32)
        for a, o in zip(self.gw.model_ids, self.o_ids):
            key_map[a] = o
        assert np.array_equal(st, ost) and np.array_equal(used, ou) and np.array_equal(fstack, ofs)
        assert np.array_equal(np.where(key >= 0, key_map[np.maximum(key, 0)], -1), ok)

    # ------------------------------------------------------------------ oracle side
    def oracle_sequences(self, k, layer, seqs, sm_scale=None, want_mask=True):
        """Oracle KV bytes and attention for sequences ``seqs`` of model k at ``layer`` in a compact host mirror.
        Returns dict with mirror bytes per block, written mask, out, lse."""
        s, g = self.wl.models[k], self.ogeom[k]
        T = g.tokens_per_block
        lens = self.gw.lens[k][seqs]
        tab = self.gw.tables_host[k]
        real_blocks = []
        for i, n in zip(seqs, lens):
            real_blocks.extend(tab[i, : workloads.blocks_needed(n, T)].tolist())
        assert len(set(real_blocks)) == len(real_blocks), "a block is owned by two sequences"
        remap = {b: j for j, b in enumerate(real_blocks)}
        ctab = np.zeros((len(seqs), tab.shape[1]), np.int32)
        for r, (i, n) in enumerate(zip(seqs, lens)):
            nb = workloads.blocks_needed(n, T)
            ctab[r, :nb] = [remap[b] for b in tab[i, :nb]]
        dt = np.float32 if s.src_f32 else np.float16
        krows = workloads.source_rows(self.wl.seed, s.tag, layer, gen.WHICH_K, lens, s.n_kv_heads, s.head_dim, seqs, dt)
        vrows = workloads.source_rows(self.wl.seed, s.tag, layer, gen.WHICH_V, lens, s.n_kv_heads, s.head_dim, seqs, dt)
        ks = vs = None
        if s.kv_dtype == workloads.FP8:
            ks, vs = self.gw.scales[self.gw.model_ids[k]]
        seq_idx, pos = workloads.token_index(lens)
        mem0 = np.zeros(len(real_blocks) * g.block_budget, np.uint8)
        oracle.kv_append(mem0, g, layer, krows, vrows, seq_idx, pos, ctab, ks, vs)
        written = None
        if want_mask:
            # bytes the append defines are those that come out identical whatever was there before; the append
            # writes one layer, so that layer's slice of every block is compared (that the oracle's append leaves
            # every other byte alone is pinned by its own CPU tests)
            mem1 = np.full(len(real_blocks) * g.block_budget, 0xFF, np.uint8)
            oracle.kv_append(mem1, g, layer, krows, vrows, seq_idx, pos, ctab, ks, vs)
            lo, hi = layer * g.layer_bytes, (layer + 1) * g.layer_bytes
            written = mem0.reshape(-1, g.block_budget)[:, lo:hi] == mem1.reshape(-1, g.block_budget)[:, lo:hi]
            del mem1
        q = gen.normal_q(self.wl.seed, s.tag, layer, seqs, s.n_q_heads, s.head_dim)
        scale = 1.0 / np.sqrt(s.head_dim) if sm_scale is None else sm_scale
        out, lse = oracle.decode_attention(mem0, g, layer, s.n_q_heads, scale, q, ctab, lens, ks, vs, n_threads=8)
        return dict(real_blocks=real_blocks, mem=mem0, written=written, out=out, lse=lse, q=q, ctab=ctab, lens=lens, ks=ks,
                    vs=vs, layer=layer)

    # ------------------------------------------------------------------ prefill
    def prefill_and_check(self, k, layer, n_new, seqs=None, sm_scale=None):
        """fs_prefill_attention for model k (KV of ``layer`` already appended): the last n_new[i] tokens of every
        sequence are the chunk being prefilled.  All query rows of the sequences ``seqs`` (default: all) are compared
        with the oracle.  Returns (max abs error, rows compared)."""
        import torch

        gw, s = self.gw, self.wl.models[k]
        m = gw.model_ids[k]
        lens = gw.lens[k]
        n_new = np.asarray(n_new, np.int32)
        assert len(n_new) == len(lens) and np.all(n_new <= lens) and np.all(n_new >= 0)
        q_off = np.concatenate([[0], np.cumsum(n_new)]).astype(np.int32)
        q = gen.normal_q_chunks(self.wl.seed, s.tag, layer, np.arange(len(lens)), lens - n_new, n_new, s.n_q_heads,
                                s.head_dim)
        dev = gw.device
        q_d = torch.from_numpy(q).to(dev)
        out_d = torch.full_like(q_d, float("nan"))
        lse_d = torch.full((q.shape[0], s.n_q_heads), float("nan"), dtype=torch.float32, device=dev)
        q_off_d = torch.from_numpy(q_off).to(dev)
        ws = torch.empty(self.fs.fs_prefill_workspace_bytes(len(lens)), dtype=torch.uint8, device=dev)
        scale = float(1.0 / np.sqrt(s.head_dim)) if sm_scale is None else float(sm_scale)
        self.fs.fs_prefill_attention(gw.pool, m, layer, s.n_q_heads, scale, q_d, gw.tables[k],
                                     gw.seq_lens[k], q_off_d, q_off, out_d, lse_d, ws)
        torch.cuda.synchronize()
        assert self.fs.fs_decode_status(ws) == 0
        out, lse = out_d.cpu().numpy(), lse_d.cpu().numpy()
        assert np.all(np.isfinite(out.astype(np.float32))) and np.all(np.isfinite(lse)), "a query row was left unwritten"
        seqs = np.arange(len(lens)) if seqs is None else np.asarray(seqs)
        ref = self.oracle_sequences(k, layer, seqs, want_mask=False)
        rows = np.concatenate([np.arange(q_off[i], q_off[i + 1]) for i in seqs]) if len(seqs) else np.zeros(0, np.int64)
        sub_off = np.concatenate([[0], np.cumsum(n_new[seqs])]).astype(np.int32)
        o_out, o_lse = oracle.prefill_attention(ref["mem"], self.ogeom[k], layer, s.n_q_heads, scale,
                                                q[rows], ref["ctab"], ref["lens"], sub_off, ref["ks"], ref["vs"],
                                                n_threads=8)
        tol = TOL_FP16 if s.kv_dtype == workloads.FP16 else TOL_QUANT
        # Rows early in a prompt average few values: outputs reach |4| where rounding the result to fp16 alone costs
        # up to |ref| * 2^-11 (decode outputs, averages over hundreds of tokens, stay below 1).  That share is
        # allowed on top of the decode tolerance, element by element.
        diff = np.abs(out[rows].astype(np.float64) - o_out) if len(rows) else np.zeros(1)
        allowed = tol + np.abs(o_out) * 2.0 ** -11 if len(rows) else np.ones(1)
        err = float(np.max(diff))
        lerr = float(np.max(np.abs(lse[rows].astype(np.float64) - o_lse))) if len(rows) else 0.0
        assert np.all(diff <= allowed), f"prefill model {k} ({s.name}): max abs error {err:.3e}, tolerance {tol} + |ref| 2^-11"
        tol_lse = prefill_lse_tolerance(scale, s.head_dim, self.last_prefill_staged())
        assert lerr <= tol_lse, f"prefill model {k} ({s.name}): lse error {lerr:.3e} > {tol_lse:.1e}"
        print(f"prefill model {k} ({s.name}) scale {scale:.4f}: max abs err {err:.2e}, lse err {lerr:.2e}")
        return err, len(rows)

    def prefill_whole_prompts_and_check_windows(self, k, layer, n_random, window=40):
        """Whole-prompt fs_prefill_attention over ALL sequences of model k (KV of ``layer`` already appended), as the
        prefill benchmark launches it.  For a seeded sample of sequences (with the shortest and the longest) the
        query rows come from the seeded host generator; every other row is filler drawn on the device.  The oracle
        recomputes three windows of ``window`` rows per sampled sequence (the first rows, rows around the middle, the
        last rows; a row of a whole prompt at position r sees tokens 0..r, so a window [a, b) is the chunk of the
        last b - a tokens of the sequence cut at b) and, for the shortest sequence, every row.
        Returns (max abs error, rows compared)."""
        import torch

        gw, s = self.gw, self.wl.models[k]
        m = gw.model_ids[k]
        lens = gw.lens[k].astype(np.int64)
        q_off = np.concatenate([[0], np.cumsum(lens)])
        assert q_off[-1] < 2 ** 31
        dev = gw.device
        gen_t = torch.Generator(device=dev)
        gen_t.manual_seed(int(self.wl.seed) + 977 * s.tag + layer)
        q_d = torch.empty((int(q_off[-1]), s.n_q_heads, s.head_dim), dtype=torch.float16, device=dev)
        q_d.normal_(generator=gen_t)
        seqs = self.sample(k, n_random, tag=77)
        q_host = {}
        for i in seqs:
            qi = gen.normal_q_chunks(self.wl.seed, s.tag, layer, [i], [0], [lens[i]], s.n_q_heads, s.head_dim)
            q_host[int(i)] = qi
            q_d[q_off[i]: q_off[i + 1]] = torch.from_numpy(qi).to(dev)
        out_d = torch.full_like(q_d, float("nan"))
        lse_d = torch.full((q_d.shape[0], s.n_q_heads), float("nan"), dtype=torch.float32, device=dev)
        q_off32 = q_off.astype(np.int32)
        q_off_d = torch.from_numpy(q_off32).to(dev)
        ws = torch.empty(self.fs.fs_prefill_workspace_bytes(len(lens)), dtype=torch.uint8, device=dev)
        scale = 1.0 / np.sqrt(s.head_dim)
        self.fs.fs_prefill_attention(gw.pool, m, layer, s.n_q_heads, float(scale), q_d, gw.tables[k], gw.seq_lens[k],
                                     q_off_d, q_off32, out_d, lse_d, ws)
        torch.cuda.synchronize()
        assert self.fs.fs_decode_status(ws) == 0
        assert bool(torch.isfinite(out_d).all()) and bool(torch.isfinite(lse_d).all()), "a query row was left unwritten"
        ref = self.oracle_sequences(k, layer, seqs, want_mask=False)
        shortest = int(seqs[np.argmin(lens[seqs])])
        ctab, o_lens, n_new, q_rows, where = [], [], [], [], []
        for r, i in enumerate(seqs):
            n = int(lens[i])
            if int(i) == shortest and n <= 1200:
                wins = [(0, n)]
            else:
                w = min(window, n)
                mid = max(w, min(n, n // 2 + w // 2))
                wins = sorted({(0, w), (mid - w, mid), (n - w, n)})
            for a, b in wins:
                ctab.append(ref["ctab"][r])
                o_lens.append(b)
                n_new.append(b - a)
                q_rows.append(q_host[int(i)][a:b])
                where.append(np.arange(q_off[i] + a, q_off[i] + b))
        sub_off = np.concatenate([[0], np.cumsum(n_new)]).astype(np.int32)
        o_out, o_lse = oracle.prefill_attention(ref["mem"], self.ogeom[k], layer, s.n_q_heads, scale,
                                                np.concatenate(q_rows), np.stack(ctab), np.asarray(o_lens, np.int32),
                                                sub_off, ref["ks"], ref["vs"], n_threads=8)
        rows = torch.from_numpy(np.concatenate(where)).to(dev)
        out = out_d[rows].cpu().numpy().astype(np.float64)
        lse = lse_d[rows].cpu().numpy().astype(np.float64)
        tol = TOL_FP16 if s.kv_dtype == workloads.FP16 else TOL_QUANT
        diff = np.abs(out - o_out)
        err = float(np.max(diff))
        assert np.all(diff <= tol + np.abs(o_out) * 2.0 ** -11), \
            f"prefill model {k} ({s.name}): max abs error {err:.3e}, tolerance {tol} + |ref| 2^-11"
        lerr = float(np.max(np.abs(lse - o_lse)))
        tol_lse = prefill_lse_tolerance(scale, s.head_dim, self.last_prefill_staged())
        assert lerr <= tol_lse, f"prefill model {k} ({s.name}): lse error {lerr:.3e} > {tol_lse:.1e}"
        return err, len(rows)

    # ------------------------------------------------------------------ comparisons
    def check_bytes(self, k, ref):
        """Every byte the oracle's append defines must be identical in the GPU's slab blocks.  The append wrote one
        layer: that layer's slice of every block is fetched from the GPU in one gather."""
        import torch

        g = self.ogeom[k]
        m = self.gw.model_ids[k]
        gg = self.gw.geom[m]
        blocks = np.asarray(ref["real_blocks"], np.int64)
        if len(blocks) == 0:
            return
        for b in blocks[:: max(1, len(blocks) // 16)]:
            assert oracle.block_offset(g, int(b)) == int(b) * gg.block_budget
        lo, hi = ref["layer"] * g.layer_bytes, (ref["layer"] + 1) * g.layer_bytes
        view = self.gw.pool_mem[: (self.wl.pool_bytes // gg.block_budget) * gg.block_budget].view(-1, gg.block_budget)
        gpu = view[:, lo:hi][torch.from_numpy(blocks).to(self.gw.device)].cpu().numpy()
        want = ref["mem"].reshape(len(blocks), g.block_budget)[:, lo:hi]
        mask = ref["written"]
        assert mask.any()
        n_bad = int(np.count_nonzero((gpu != want) & mask))
        assert n_bad == 0, f"model {k}: {n_bad} appended bytes differ from the oracle"

    def check_attention(self, k, seqs, ref, out_gpu, lse_gpu=None):
        s = self.wl.models[k]
        tol = TOL_FP16 if s.kv_dtype == workloads.FP16 else TOL_QUANT
        got = out_gpu[seqs].astype(np.float64)
        assert np.all(np.isfinite(got))
        err = float(np.max(np.abs(got - ref["out"])))
        assert err <= tol, f"model {k} ({s.name}): max abs error {err:.3e} > {tol}"
        if lse_gpu is not None:
            lerr = float(np.max(np.abs(lse_gpu[seqs].astype(np.float64) - ref["lse"])))
            assert lerr <= TOL_LSE, f"model {k} ({s.name}): lse error {lerr:.3e}"
        return err

    def sample(self, k, n_random, tag=55):
        """Seeded sample of sequences of model k: n_random random ones plus the shortest and the longest."""
        lens = self.gw.lens[k]
        pick = set(gen.permutation(self.wl.seed, tag + k, len(lens))[:n_random].tolist())
        pick.add(int(np.argmin(lens)))
        pick.add(int(np.argmax(lens)))
        return np.array(sorted(pick), dtype=np.int64)

    def populate_and_decode(self, layers, kernel_mode=0, sm_scale=None):
        """Populate ``layers[k]`` of every model and decode all models in one multi launch; returns the keep-alive
        dict of make_batches (outputs under "out" and "lse")."""
        import torch

        gw = self.gw
        gw.set_option(self.fs.FS_OPT_DECODE_KERNEL, kernel_mode)
        try:
            gw.populate([[l] for l in layers])
            batches, keep = gw.make_batches(layers, sm_scale=sm_scale)
            ws = gw.decode(batches)
            torch.cuda.synchronize()
            status = self.fs.fs_decode_status(ws)
            assert status == 0, f"decode status {status}"
        finally:
            gw.set_option(self.fs.FS_OPT_DECODE_KERNEL, 0)
        return keep

    def check_model(self, k, layers, keep, n_random=None, with_bytes=True, sm_scale=None):
        """Compare model k's sampled (default: all) sequences with the oracle: appended bytes and attention outputs.
        Returns (max abs error, sequences compared)."""
        seqs = np.arange(len(self.gw.lens[k])) if n_random is None else self.sample(k, n_random)
        out_gpu, lse_gpu = keep["out"][k].cpu().numpy(), keep["lse"][k].cpu().numpy()
        err = 0.0
        for part in self.mirror_sized_parts(k, seqs):
            ref = self.oracle_sequences(k, layers[k], part, sm_scale=sm_scale, want_mask=with_bytes)
            if with_bytes:
                self.check_bytes(k, ref)
            err = max(err, self.check_attention(k, part, ref, out_gpu, lse_gpu))
        return err, len(seqs)

    def run_and_check(self, layers, n_random=None, with_bytes=True, kernel_mode=0, sm_scale=None):
        """Populate ``layers[k]`` of every model, decode all models in one multi launch, and compare the sampled
        (default: all) sequences with the oracle.  Returns max errors per model."""
        keep = self.populate_and_decode(layers, kernel_mode=kernel_mode, sm_scale=sm_scale)
        return [self.check_model(k, layers, keep, n_random, with_bytes, sm_scale)[0] for k in range(len(self.wl.models))]

    def mirror_sized_parts(self, k, seqs, max_bytes=3 << 30):
        """Cuts a list of sequences into parts whose blocks fit a host mirror of about max_bytes (the oracle's mirror
        holds whole blocks, all layers of them)."""
        T, budget = self.ogeom[k].tokens_per_block, self.ogeom[k].block_budget
        parts, cur, cur_bytes = [], [], 0
        for i in seqs:
            b = workloads.blocks_needed(int(self.gw.lens[k][i]), T) * budget
            if cur and cur_bytes + b > max_bytes:
                parts.append(np.array(cur, dtype=np.int64))
                cur, cur_bytes = [], 0
            cur.append(int(i))
            cur_bytes += b
        if cur:
            parts.append(np.array(cur, dtype=np.int64))
        return parts


def smoke():
    """Tiny end-to-end check used by __graft_entry__.smoke()."""
    wl = workloads.config(1)
    par = Parity(wl, zero_pool=True)
    try:
        errs = par.run_and_check([0])
        print(f"config 1 on cuda:0: allocator ops {par.n_alloc_ops} identical, appended bytes identical, "
              f"attention max abs err {errs[0]:.2e}")
    finally:
        par.close()
    # a small two-model mixed-precision pool through the multi-model launch
    wl = workloads.scaled_down(workloads.config(3), n_seq=4, max_len=300, pool_bytes=256 * workloads.MiB)
    par = Parity(wl, zero_pool=True)
    try:
        errs = par.run_and_check([1, 2])
        print(f"mixed fp16+fp8 pool: attention max abs err {errs}")
        perr = [par.prefill_and_check(k, layer, par.gw.lens[k])[0] for k, layer in ((0, 1), (1, 2))]
        print(f"whole-prompt prefill over the same pool: max abs err {perr}")
    finally:
        par.close()
