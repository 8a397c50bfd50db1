"""Seeded synthetic workloads for the batched KV-cache compression stage.

This module only makes INPUTS: request lengths, methods, budgets, the order
in which pool blocks are handed out, and random fp16 K/V/Q bytes.  It holds
none of the stage's arithmetic (no scoring, no selection, no copying) so that
the HIP path and the CPU oracle can both be fed from it without sharing code.

The workloads stand in for the paper's evaluation inputs (single-image
GQA-like prompts and multi-image MileBench-like prompts served by
LLaVA-1.5-7B, "Evaluation Setup" section): same tensor shapes (32 layers x 32
heads x head_dim 128, 576 image tokens per image), synthetic values.
"""

from dataclasses import dataclass, field
import numpy as np

METHOD_NONE = 0
METHOD_SNAPKV = 1
METHOD_KNORM = 2
METHOD_STREAMING = 3

BLOCK_SIZE = 16


@dataclass
class Workload:
    name: str
    n_layers: int
    n_heads: int
    head_dim: int
    n_blocks: int
    window: int
    pool_kernel: int
    seq_lens: np.ndarray          # int32 [n_req]
    methods: np.ndarray           # int32 [n_req]
    budgets: np.ndarray           # int32 [n_req]
    seed: int
    outlier_channels: bool        # 4 key channels per (layer, head) scaled x8
    permuted: bool                # block tables permuted by alloc/free churn
    block_size: int = BLOCK_SIZE
    notes: str = ""
    extra: dict = field(default_factory=dict)

    @property
    def n_req(self):
        return int(self.seq_lens.shape[0])

    @property
    def max_blocks(self):
        return int(max(blocks_for(int(l), self.block_size) for l in self.seq_lens))

    @property
    def total_tokens(self):
        return int(self.seq_lens.sum())

    def pool_shape(self):
        return (self.n_layers, self.n_blocks, 2, self.n_heads, self.block_size,
                self.head_dim)

    def pool_bytes(self):
        n = 2
        for s in self.pool_shape():
            n *= s
        return n


def blocks_for(n_tokens, block_size=BLOCK_SIZE):
    return (n_tokens + block_size - 1) // block_size


def budget_from_pct(seq_len, pct, method, window):
    """Tokens kept per head for a percentage budget (integer division), never
    below the observation window for SnapKV and never below 1."""
    b = (int(seq_len) * int(pct)) // 100
    floor = window if method == METHOD_SNAPKV else 1
    return max(b, floor)


def _n_blocks_for_occupancy(seq_lens, budgets, occupancy, bs=BLOCK_SIZE):
    """Pool size such that (old + new blocks) / n_blocks == occupancy at the
    peak of one compression call (new blocks are taken before old ones are
    returned)."""
    old = sum(blocks_for(int(l), bs) for l in seq_lens)
    new = sum(blocks_for(int(b), bs) for b in budgets)
    return int(np.ceil((old + new) / occupancy))


def precall_occupancy_variant(wl, occupancy):
    """The same batch in a pool whose occupancy BEFORE the call is `occupancy`
    (the resident requests' blocks / n_blocks).  With a large kept fraction
    the batch then no longer fits one call (new blocks are taken before old
    ones come back) and has to be compressed in parts."""
    old = sum(blocks_for(int(l), wl.block_size) for l in wl.seq_lens)
    wl.n_blocks = int(np.ceil(old / occupancy))
    wl.name += "_precall%d" % round(occupancy * 100)
    wl.notes = "%d%% occupancy before the call" % round(occupancy * 100)
    return wl


def make_workload(config, n_layers=None, n_heads=None, n_req=None, seed=None,
                  max_len=None):
    """The five benchmark configurations (1-based), optionally shrunk in the
    number of layers / heads / requests for CPU-sized parity runs.  Shrinking
    never changes the per-(layer, head) problem: head_dim, lengths, window,
    budgets and block size stay as configured."""
    if config == 1:
        s = 0 if seed is None else seed
        lens = np.array([256], dtype=np.int32)
        return Workload("config1_tiny_snapkv", n_layers or 1, n_heads or 4, 64, 64,
                        16, 7, lens, np.array([METHOD_SNAPKV], np.int32),
                        np.array([64], np.int32), s, False, False)
    if config == 2:
        s = 2 if seed is None else seed
        lens = np.array([640], dtype=np.int32)
        return Workload("config2_llava_single", n_layers or 32, n_heads or 32, 128,
                        64, 32, 7, lens, np.array([METHOD_SNAPKV], np.int32),
                        np.array([budget_from_pct(640, 25, METHOD_SNAPKV, 32)],
                                 np.int32), s, True, False)
    if config == 3:
        s = 3 if seed is None else seed
        R = n_req or 32
        rng = np.random.Generator(np.random.PCG64(s))
        lens = rng.integers(600, 1201, size=R).astype(np.int32)
        methods = np.array([METHOD_SNAPKV if r % 2 == 0 else METHOD_KNORM
                            for r in range(R)], np.int32)
        budgets = np.array([budget_from_pct(lens[r], 50, methods[r], 32)
                            for r in range(R)], np.int32)
        nb = _n_blocks_for_occupancy(lens, budgets, 0.70)
        return Workload("config3_batched_mixed", n_layers or 32, n_heads or 32, 128,
                        nb, 32, 7, lens, methods, budgets, s, True, True,
                        notes="70% occupancy at the peak of the call")
    if config == 4:
        s = 4 if seed is None else seed
        R = n_req or 64
        rng = np.random.Generator(np.random.PCG64(s))
        k = rng.integers(2, 13, size=R)
        lens = (576 * k + 128).astype(np.int32)
        methods = np.full(R, METHOD_SNAPKV, np.int32)
        budgets = np.array([budget_from_pct(lens[r], 20, METHOD_SNAPKV, 64)
                            for r in range(R)], np.int32)
        nb = _n_blocks_for_occupancy(lens, budgets, 0.85)
        return Workload("config4_multi_image", n_layers or 32, n_heads or 32, 128,
                        nb, 64, 7, lens, methods, budgets, s, True, True,
                        notes="85% occupancy at the peak of the call")
    if config == 5:
        s = 5 if seed is None else seed
        R = n_req or 256
        rng = np.random.Generator(np.random.PCG64(s))
        hi = 16384 if max_len is None else max_len
        lens = rng.integers(512, hi + 1, size=R).astype(np.int32)
        pct = rng.integers(10, 51, size=R)
        methods = np.array([METHOD_SNAPKV if r % 2 == 0 else METHOD_KNORM
                            for r in range(R)], np.int32)
        budgets = np.array([budget_from_pct(lens[r], pct[r], methods[r], 32)
                            for r in range(R)], np.int32)
        live = sum(blocks_for(int(l)) for l in lens)
        nb = int(np.ceil(live / 0.90))
        return Workload("config5_high_concurrency", n_layers or 2, n_heads or 32, 128,
                        nb, 32, 7, lens, methods, budgets, s, True, True,
                        notes="pool sized for 90% occupancy by the resident requests; "
                              "layer count reduced so the pool fits one GPU",
                        extra={"pct": pct})
    raise ValueError("config must be 1..5")


# --------------------------------------------------------------------------
# block hand-out order
# --------------------------------------------------------------------------

def churn_permutation(wl):
    """Order in which a harness frees the blocks of a fully allocated fresh
    pool so that later allocations come back permuted.  Pure index data."""
    rng = np.random.Generator(np.random.PCG64(wl.seed + 1000))
    return rng.permutation(wl.n_blocks).astype(np.int64)


def round_robin_positions(wl):
    """Requests take their blocks one at a time in round-robin order from one
    run of pops.  Returns (total, pos) with pos[r][i] = index into that run
    of the i-th block of request r."""
    n_old = [blocks_for(int(l), wl.block_size) for l in wl.seq_lens]
    pos = [np.empty(n, dtype=np.int64) for n in n_old]
    k = 0
    for i in range(max(n_old)):
        for r in range(wl.n_req):
            if i < n_old[r]:
                pos[r][i] = k
                k += 1
    return k, pos


def build_block_tables(wl, alloc, free, take):
    """Drives any pool (oracle or device) through its public calls to produce
    the request block tables.

    alloc(n) -> ids, free(ids), take(ids, index_array) -> ids[index_array].
    Returns a list of per-request id arrays (in the pool's own array type).
    """
    if wl.permuted:
        ids_all = alloc(wl.n_blocks)
        free(take(ids_all, churn_permutation(wl)))
    total, pos = round_robin_positions(wl)
    ids = alloc(total)
    return [take(ids, pos[r]) for r in range(wl.n_req)]


# --------------------------------------------------------------------------
# values
# --------------------------------------------------------------------------

def outlier_channel_ids(wl):
    """int64 [n_layers][n_heads][4]: distinct key channels scaled x8."""
    rng = np.random.Generator(np.random.PCG64(wl.seed + 2000))
    out = np.empty((wl.n_layers, wl.n_heads, 4), dtype=np.int64)
    for l in range(wl.n_layers):
        for h in range(wl.n_heads):
            out[l, h] = rng.choice(wl.head_dim, size=4, replace=False)
    return out


def key_channel_gain(wl):
    """float32 [n_layers][n_heads][head_dim]: 8 on outlier channels, else 1."""
    g = np.ones((wl.n_layers, wl.n_heads, wl.head_dim), dtype=np.float32)
    if wl.outlier_channels:
        ids = outlier_channel_ids(wl)
        for l in range(wl.n_layers):
            for h in range(wl.n_heads):
                g[l, h, ids[l, h]] = 8.0
    return g


def fill_pool_host(wl):
    """The whole pool (every block, free ones included) as a float16 numpy
    array of wl.pool_shape(): N(0,1) rounded to fp16, key channels scaled by
    key_channel_gain.  For CPU-sized workloads."""
    rng = np.random.Generator(np.random.Philox(key=wl.seed + 3000))
    kv = rng.standard_normal(size=wl.pool_shape(), dtype=np.float32)
    gain = key_channel_gain(wl)                       # [l][h][d]
    kv[:, :, 0] *= gain[:, None, :, None, :]
    return kv.astype(np.float16)


def fill_q_window_host(wl):
    """float16 [n_req][n_layers][n_heads][window][head_dim], N(0,1)."""
    rng = np.random.Generator(np.random.Philox(key=wl.seed + 4000))
    q = rng.standard_normal(
        size=(wl.n_req, wl.n_layers, wl.n_heads, wl.window, wl.head_dim),
        dtype=np.float32)
    return q.astype(np.float16)


def fill_pool_device(wl, kv):
    """Same recipe written straight into a device tensor `kv` (torch, fp16,
    shape wl.pool_shape()), one layer slab at a time, for pools too large to
    stage on the host.  Consumers that need the bytes on the CPU download
    them from `kv`."""
    import torch
    gen = torch.Generator(device=kv.device)
    gen.manual_seed(wl.seed + 3000)
    gain = torch.from_numpy(key_channel_gain(wl)).to(kv.device)
    for l in range(wl.n_layers):
        slab = kv[l]                                   # [blocks][2][h][slot][d]
        n_chunk = max(1, slab.shape[0] // 8)
        for b0 in range(0, slab.shape[0], n_chunk):
            part = slab[b0:b0 + n_chunk]
            part.normal_(0.0, 1.0, generator=gen)
            part[:, 0].mul_(gain[l][None, :, None, :].to(part.dtype))
    return kv


def fill_q_window_device(wl, device):
    import torch
    gen = torch.Generator(device=device)
    gen.manual_seed(wl.seed + 4000)
    q = torch.empty((wl.n_req, wl.n_layers, wl.n_heads, wl.window, wl.head_dim),
                    dtype=torch.float16, device=device)
    q.normal_(0.0, 1.0, generator=gen)
    return q
