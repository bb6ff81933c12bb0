"""Driver that stands a synthetic workload up on the GPU through the C ABI (test and benchmark plumbing, no part
of the library).

Used by the GPU tests, ``__graft_entry__.smoke()`` and the ``bench*.py`` programs: it creates the pool,
registers the models, replays the workload's allocation recipe against ``fs_block_alloc`` /
``fs_block_free``, fills the KV cache with ``fs_kv_append`` from the device-side input generator,
and issues ``fs_decode_attention_multi``.  Argument plumbing only -- every step of the path runs in
libfineserve.so; torch owns device memory and the stream.
"""
from __future__ import annotations

import numpy as np
import torch

from fs_inputs import device as gen_device
from fs_inputs import gen, workloads

from paper_2509_06261_amd import binding as fs

# Pool options (fs_pool_set_option) applied to every workload stood up from here on: {option: value}.  The prefill
# tests select their kernel variant this way before the pool exists.
DEFAULT_OPTIONS = {}


class AllocAdapter:
    """alloc/free facade over the C ABI, in the shape fs_inputs.workloads.place expects."""

    def __init__(self, pool):
        self.pool = pool

    def alloc(self, model):
        return fs.fs_block_alloc(self.pool, model)

    def free(self, model, blk):
        return fs.fs_block_free(self.pool, model, blk)


class GpuWorkload:
    def __init__(self, wl: workloads.Workload, device="cuda:0", zero_pool=False, options=None):
        self.wl = wl
        self.device = torch.device(device)
        torch.cuda.set_device(self.device)
        alloc = torch.zeros if zero_pool else torch.empty
        self.pool_mem = alloc(wl.pool_bytes, dtype=torch.uint8, device=self.device)
        self.pool = fs.fs_pool_create(wl.slab_bytes, wl.pool_bytes, self.pool_mem)
        for opt, value in {**DEFAULT_OPTIONS, **(options or {})}.items():
            self.set_option(opt, value)
        self.model_ids, self.T, self.geom, self.scales = [], {}, {}, {}
        for s in wl.models:
            if s.tokens_per_block:
                T, m = fs.fs_model_register_tokens(self.pool, s.kv_dtype, s.n_kv_heads, s.head_dim, s.n_layers,
                                                   s.tokens_per_block)
            else:
                T, m = fs.fs_model_register(self.pool, s.kv_dtype, s.n_kv_heads, s.head_dim, s.n_layers, s.block_budget)
            self.model_ids.append(m)
            self.T[m] = T
            self.geom[m] = fs.fs_model_geometry(self.pool, m)
            if s.kv_dtype == workloads.FP8:
                ks, vs = workloads.fp8_scales_table(s.n_layers, s.n_kv_heads)
                fs.fs_model_set_fp8_scales(self.pool, m, ks, vs)
                self.scales[m] = (ks, vs)
        self.blocks = None
        self.lens = [np.array(s.lens, dtype=np.int32) for s in wl.models]
        self.tables_host, self.tables, self.seq_lens = [], [], []
        self._ws = None

    def set_option(self, option, value):
        rc = fs.fs_pool_set_option(self.pool, option, value)
        if rc != fs.FS_OK:
            raise fs.FsError(rc, f"fs_pool_set_option({option}, {value})")

    def close(self):
        if self.pool is not None:
            torch.cuda.synchronize(self.device)
            fs.fs_pool_destroy(self.pool)
            self.pool = None
            self.pool_mem = None
            self._ws = None
            self.tables, self.seq_lens = [], []
            torch.cuda.empty_cache()  # hand the (possibly >100 GiB) pool back before the next workload

    # ------------------------------------------------------------------ allocation
    def place(self, adapter=None):
        """Replay the allocation recipe; ``adapter`` lets a test drive a second allocator in lock-step."""
        adapter = adapter or AllocAdapter(self.pool)
        blocks, lens = workloads.place(adapter, self.wl, self.model_ids, self.T)
        self.blocks = blocks
        if lens is not None:
            self.lens = lens
        self.tables_host = [workloads.make_tables(b) for b in blocks]
        self.tables = [torch.from_numpy(t).to(self.device) for t in self.tables_host]
        self.seq_lens = [torch.from_numpy(np.ascontiguousarray(l)).to(self.device) for l in self.lens]
        return blocks

    # ------------------------------------------------------------------ KV fill
    def populate(self, layers_of_model=None, chunk_tokens=1 << 17, seq_subset=None, hold_back_newest=False):
        """Append every token of every sequence (or of ``seq_subset[k]``) for the given layers
        (default: all layers) from the device-side generator; with hold_back_newest all but each sequence's last."""
        for k, (s, m) in enumerate(zip(self.wl.models, self.model_ids)):
            layers = range(s.n_layers) if layers_of_model is None else layers_of_model[k]
            lens = self.lens[k]
            if seq_subset is not None:
                keep = np.zeros(len(lens), bool)
                keep[np.asarray(seq_subset[k], dtype=np.int64)] = True
                lens = np.where(keep, lens, 0)
            seq_idx, pos = workloads.token_index(lens)
            if hold_back_newest:
                older = pos < (np.asarray(self.lens[k])[seq_idx] - 1)
                seq_idx, pos = seq_idx[older], pos[older]
            n = len(pos)
            dt = torch.float32 if s.src_f32 else torch.float16
            for c0 in range(0, n, chunk_tokens):
                c1 = min(n, c0 + chunk_tokens)
                si = torch.from_numpy(seq_idx[c0:c1]).to(self.device)
                po = torch.from_numpy(pos[c0:c1]).to(self.device)
                kb = torch.empty((c1 - c0, s.n_kv_heads, s.head_dim), dtype=dt, device=self.device)
                vb = torch.empty_like(kb)
                for layer in layers:
                    gen_device.fill_rows(kb, self.wl.seed, s.tag, layer, gen.WHICH_K, si, po, s.n_kv_heads, s.head_dim)
                    gen_device.fill_rows(vb, self.wl.seed, s.tag, layer, gen.WHICH_V, si, po, s.n_kv_heads, s.head_dim)
                    fs.fs_kv_append(self.pool, m, layer, kb, vb, si, po, self.tables[k])
            torch.cuda.synchronize(self.device)

    def newest_token_appends(self, layers, models=None):
        """One fs_append_t per model: the newest token (position n_b - 1) of every sequence at ``layers[k]``, its rows
        drawn from the device-side generator.  Returns (appends, keepalive list)."""
        appends, keep = [], []
        for k, (s, m) in enumerate(zip(self.wl.models, self.model_ids)):
            if models is not None and k not in models:
                continue
            si = torch.arange(s.n_seq, dtype=torch.int32, device=self.device)
            po = (self.seq_lens[k] - 1).to(torch.int32)
            dt = torch.float32 if s.src_f32 else torch.float16
            kb = torch.empty((s.n_seq, s.n_kv_heads, s.head_dim), dtype=dt, device=self.device)
            vb = torch.empty_like(kb)
            gen_device.fill_rows(kb, self.wl.seed, s.tag, layers[k], gen.WHICH_K, si, po, s.n_kv_heads, s.head_dim)
            gen_device.fill_rows(vb, self.wl.seed, s.tag, layers[k], gen.WHICH_V, si, po, s.n_kv_heads, s.head_dim)
            appends.append(fs.make_append(m, layers[k], kb, vb, si, po, self.tables[k]))
            keep.append((si, po, kb, vb))
        return appends, keep

    # ------------------------------------------------------------------ decode
    def make_q(self, k, layer):
        s = self.wl.models[k]
        q = gen.normal_q(self.wl.seed, s.tag, layer, np.arange(s.n_seq), s.n_q_heads, s.head_dim)
        return q

    def make_batches(self, layers, with_lse=True, host_lens=True, models=None, sm_scale=None):
        """One fs_batch_t per model (``layers[k]`` = layer index; softmax scale 1/sqrt(head_dim) unless given).
        Returns (batches, keepalive dict)."""
        batches, keep = [], {"q": [], "out": [], "lse": [], "q_host": []}
        for k, (s, m) in enumerate(zip(self.wl.models, self.model_ids)):
            if models is not None and k not in models:
                continue
            qh = self.make_q(k, layers[k])
            q = torch.from_numpy(qh).to(self.device)
            out = torch.zeros((s.n_seq, s.n_q_heads, s.head_dim), dtype=torch.float16, device=self.device)
            lse = torch.zeros((s.n_seq, s.n_q_heads), dtype=torch.float32, device=self.device) if with_lse else None
            scale = float(1.0 / np.sqrt(s.head_dim)) if sm_scale is None else float(sm_scale)
            b = fs.make_batch(m, layers[k], s.n_q_heads, scale, q, self.tables[k],
                              self.seq_lens[k], out, lse, self.lens[k] if host_lens else None)
            batches.append(b)
            keep["q"].append(q)
            keep["out"].append(out)
            keep["lse"].append(lse)
            keep["q_host"].append(qh)
        return batches, keep

    def workspace_for(self, batches):
        need = fs.fs_decode_workspace_bytes(self.pool, batches)
        assert need > 0, fs.fs_last_error()
        if self._ws is None or self._ws.numel() < need:
            self._ws = torch.empty(need, dtype=torch.uint8, device=self.device)
        return self._ws

    def decode(self, batches, stream=None):
        ws = self.workspace_for(batches)
        fs.fs_decode_attention_multi(self.pool, batches, ws, stream)
        return ws

    # ------------------------------------------------------------------ inspection
    def read_block(self, m, blk) -> np.ndarray:
        """The defined-size prefix (block_bytes) of block ``blk`` of model ``m`` as host bytes."""
        g = self.geom[m]
        off = blk * g.block_budget
        return self.pool_mem[off: off + g.block_bytes].cpu().numpy()

    def kv_bytes_per_layer_launch(self, models=None) -> int:
        """Algorithmic KV bytes one decode launch reads: sum over sequences of len x token bytes."""
        total = 0
        for k, s in enumerate(self.wl.models):
            if models is not None and k not in models:
                continue
            total += int(self.lens[k].astype(np.int64).sum()) * workloads.kv_bytes_per_token_layer(s)
        return total
