"""Harness plumbing shared by bench.py and the full-size GPU tests: puts a
synthetic workload into HBM (pool memory, window queries, block tables built
through the library's own alloc/free calls).  No arithmetic of the stage."""

import numpy as np

from . import fastcache as fc
from . import synth


class DeviceWorkload:
    def __init__(self, wl, device="cuda:0", verbose=False):
        import torch
        self.torch, self.wl = torch, wl
        self.dev = torch.device(device)
        if verbose:
            print("[setup] %s: pool %.1f GiB, %d requests, %d tokens" % (
                wl.name, wl.pool_bytes() / 2**30, wl.n_req, wl.total_tokens), flush=True)
        self.lse = None
        self.parts = 1      # > 1: compress() issues the batch as that many calls
        self.kv = torch.empty(wl.pool_shape(), dtype=torch.float16, device=self.dev)
        synth.fill_pool_device(wl, self.kv)
        self.q = synth.fill_q_window_device(wl, self.dev)
        self.pool = fc.fc_pool_create(self.kv, wl.n_blocks, wl.n_layers, wl.n_heads, wl.head_dim)
        rows = synth.build_block_tables(
            wl, lambda n: fc.fc_pool_alloc(self.pool, n),
            lambda ids: fc.fc_pool_free(self.pool, ids),
            lambda ids, ix: ids[torch.from_numpy(ix).to(self.dev)].contiguous())
        self.bt = torch.full((wl.n_req, wl.max_blocks), -1, dtype=torch.int32, device=self.dev)
        for r in range(wl.n_req):
            self.bt[r, :rows[r].shape[0]] = rows[r]
        self.lens = wl.seq_lens.copy()
        torch.cuda.synchronize()
        # snapshot of the metadata so a benchmark can rewind between repetitions
        # (data blocks need no rewind: compaction writes only into free blocks)
        self.bt0 = self.bt.clone()
        self.stack0, self.top0 = fc.fc_pool_export_state(self.pool)
        self.stack0_dev = torch.from_numpy(self.stack0).to(self.dev)
        if verbose:
            print("[setup] done", flush=True)

    def rewind(self):
        fc.fc_pool_import_state(self.pool, self.stack0, self.top0)
        self.bt.copy_(self.bt0)
        self.lens[:] = self.wl.seq_lens

    def rewind_async(self):
        """Rewind without a host wait (device-to-device copies on the stream)."""
        fc.fc_pool_import_state_dev(self.pool, self.stack0_dev, self.top0)
        self.bt.copy_(self.bt0)
        self.lens[:] = self.wl.seq_lens

    def compress_in_parts(self, n_parts):
        """The batch as n_parts calls of consecutive requests (the others pass
        through as FC_METHOD_NONE), for pools too full for one call."""
        wl = self.wl
        edges = np.linspace(0, wl.n_req, n_parts + 1).astype(int)
        for a, b in zip(edges[:-1], edges[1:]):
            m = np.zeros(wl.n_req, dtype=np.int32)
            m[a:b] = wl.methods[a:b]
            fc.fc_compress_batch(self.pool, self.bt, self.lens, self.q, wl.window, m,
                                 wl.budgets, wl.pool_kernel, 0.0, None, None)

    def compress(self, scores_out=None, kept_out=None):
        wl = self.wl
        if self.parts > 1:
            return self.compress_in_parts(self.parts)
        if self.lse is not None:
            fc.fc_compress_batch_lse(self.pool, self.bt, self.lens, self.q, self.lse, wl.window,
                                     wl.methods, wl.budgets, wl.pool_kernel, 0.0, scores_out,
                                     kept_out)
            return
        fc.fc_compress_batch(self.pool, self.bt, self.lens, self.q, wl.window, wl.methods,
                             wl.budgets, wl.pool_kernel, 0.0, scores_out, kept_out)

    def compute_lse(self):
        """The window rows' log-sum-exp (what a prefill attention kernel would
        hand over), computed by the library; compress() then takes it as input."""
        wl = self.wl
        lse = self.torch.zeros((wl.n_req, wl.n_layers, wl.n_heads, wl.window),
                               dtype=self.torch.float32, device=self.dev)
        fc.fc_window_lse(self.pool, self.bt, self.lens, self.q, wl.window, wl.methods, lse)
        self.torch.cuda.synchronize()
        self.lse = lse

    def close(self):
        fc.fc_pool_destroy(self.pool)
        self.kv = None

    # ---- accounting (algorithmic bytes, stated per token per (layer, head)) ----

    def algorithmic_bytes(self):
        """Whole path: read K once to score (2*d bytes per token-head; nothing
        for streaming requests, which are not scored), re-read and write the
        kept K and V rows (2 * 2 * 2*d bytes per kept token-head)."""
        wl = self.wl
        n_lh = wl.n_layers * wl.n_heads
        row = 2 * wl.head_dim
        comp = wl.methods != synth.METHOD_NONE
        scored = comp & (wl.methods != synth.METHOD_STREAMING)
        tokens = int(wl.seq_lens[scored].astype(np.int64).sum())
        kept = int(wl.budgets[comp].astype(np.int64).sum())
        return n_lh * (tokens * row + kept * 4 * row)

    def kernel_algorithmic_bytes(self, score_mode="auto", fused_max_len=8192):
        """Algorithmic bytes per launch of each kernel that moves bulk data,
        following the library's scheduling: with auto, heads of at most
        `fused_max_len` tokens run in the fused kernel (score + gather bytes);
        the rest in the separate kernels."""
        wl = self.wl
        n_lh = wl.n_layers * wl.n_heads
        row = 2 * wl.head_dim
        L = wl.seq_lens.astype(np.int64)
        B = wl.budgets.astype(np.int64)
        snap = wl.methods == synth.METHOD_SNAPKV
        kn = wl.methods == synth.METHOD_KNORM
        stream = wl.methods == synth.METHOD_STREAMING
        fused = (snap | kn) & (L <= fused_max_len) & (score_mode == "auto")
        sep = (snap | kn) & ~fused
        return {
            "fused_unit": n_lh * int((L[fused] * row + B[fused] * 4 * row).sum()
                                     + (B[stream] * 4 * row).sum()),
            "snapkv_score": n_lh * int(L[snap & sep].sum()) * row,
            "knorm_score": n_lh * int(L[kn & sep].sum()) * row,
            "gather": n_lh * int(B[sep].sum()) * 4 * row,
        }
