"""The pruned second pass of the SnapKV-style score (fc_set_score_pruning): a
call that does not ask for the scores keeps exactly the tokens the two-pass
path keeps.  Kept lists against the oracle (identical outside the threshold
band), gathered bytes, block tables and free list bit-exact: on the reduced
benchmark configurations, on the shapes that stress the bounds (first blocks
without a reference, every pooling width, ties, clustered scores, logits that
outrun the reference), and next to everything else a batch can hold."""

import numpy as np
import pytest

from oracle import fastcache_oracle as fo
from paper_2503_08461_amd import synth
from test_gpu_parity import _custom, _mixed_window_batch

pytestmark = pytest.mark.gpu


def _pruned(wl, **kw):
    from paper_2503_08461_amd import fastcache as fc
    from parity_util import SideBySide
    s = SideBySide(wl, **kw)
    fc.fc_set_score_pruning(s.pool, True)
    return s


def _run_pruned(wl, repeats=1, sbs_kw=None, **kw):
    s = _pruned(wl, **(sbs_kw or {}))
    try:
        out = [s.compress_and_compare(scores=False, **kw) for _ in range(repeats)]
    finally:
        s.close()
    print(wl.name, out, flush=True)
    return out


@pytest.mark.parametrize("L,W,d,pct", [(640, 32, 128, 25), (2048, 64, 128, 20), (4556, 64, 128, 20),
                                       (7040, 64, 128, 20), (8192, 48, 64, 10), (3000, 16, 128, 50),
                                       (2049, 33, 64, 35), (2500, 1, 128, 5), (5000, 17, 64, 3),
                                       (2111, 64, 128, 45), (4097, 64, 64, 99), (512, 32, 128, 50),
                                       (511, 64, 64, 30), (700, 64, 128, 80), (1200, 48, 64, 60),
                                       (1031, 16, 128, 10)])
def test_pruned_pass_keeps_what_two_passes_keep(L, W, d, pct):
    """Heads on both sides of the length limit of the pruned path (the second
    request of a case has half the length of the first), small and large
    budgets, every number of query tiles, ragged last blocks."""
    B = max(W, L * pct // 100)
    _run_pruned(_custom([L, L // 2 + 9], [B, max(W, (L // 2 + 9) * pct // 100)],
                        [fo.METHOD_SNAPKV] * 2, W=W, d=d, n_heads=4))


def test_reduced_benchmark_configurations():
    _run_pruned(synth.make_workload(2, n_layers=2, n_heads=3))
    _run_pruned(synth.make_workload(3, n_layers=1, n_heads=2, n_req=6))
    _run_pruned(synth.make_workload(4, n_layers=1, n_heads=2, n_req=4))
    _run_pruned(synth.make_workload(4, n_layers=2, n_heads=3, n_req=2))


@pytest.mark.parametrize("pool_kernel", [1, 3, 7, 15, 63])
def test_pooling_widths(pool_kernel):
    _run_pruned(_custom([3000, 2600], [500, 700], [fo.METHOD_SNAPKV] * 2, W=32, d=128, n_heads=3),
                pool_kernel=pool_kernel)


def test_budget_edges():
    # window only, window + 1, everything, everything but one
    wl = _custom([2100, 2100, 2100, 2100], [64, 65, 2100, 2099], [fo.METHOD_SNAPKV] * 4, W=64, d=128)
    _run_pruned(wl)


def test_mixed_methods_and_pass_through_in_one_batch():
    wl = _custom([3000, 1000, 2500, 4000, 2200, 90], [600, 200, 300, 900, 800, 60],
                 [fo.METHOD_SNAPKV, fo.METHOD_KNORM, fo.METHOD_STREAMING, fo.METHOD_SNAPKV,
                  fo.METHOD_NONE, fo.METHOD_SNAPKV], W=48, d=128, n_heads=3)
    _run_pruned(wl)


def test_all_scores_tie():
    """All-zero queries: every prefix token has the same score, and the kept
    prefix must be the lowest indices."""
    wl = _custom([2600, 2100], [600, 300], [fo.METHOD_SNAPKV] * 2, W=16, d=64)
    q = np.zeros((2, 1, 2, 16, 64), dtype=np.float16)
    out = _run_pruned(wl, sbs_kw={"q_host": q})
    assert out[0]["units_kept_identical"] == out[0]["units"]


def test_scores_clustered_around_the_threshold():
    """Keys that are all nearly alike: every column sum lies within a fraction
    of a per cent of the others, so the bounds decide nothing and the exact
    re-scoring carries the selection."""
    wl = _custom([3000], [600], [fo.METHOD_SNAPKV], W=32, d=64, n_heads=2)
    kv = synth.fill_pool_host(wl)
    rng = np.random.default_rng(3)
    kv[:, :, 0] = (0.25 + rng.integers(0, 3, size=kv[:, :, 0].shape) / 1024.0).astype(np.float16)
    _run_pruned(wl, sbs_kw={"kv_host": kv})


def test_logits_that_outrun_the_reference_fall_back_to_two_passes():
    """A few late keys a thousand times larger than the rest: their logits
    exceed everything seen before by more than the exponent range of fp32, the
    numerators against the running reference overflow, and the head must come
    out exactly as from the two-pass code (which subtracts the true maximum)."""
    from paper_2503_08461_amd import fastcache as fc
    from parity_util import SideBySide
    wl = _custom([3000, 2500], [600, 500], [fo.METHOD_SNAPKV] * 2, W=32, d=128, n_heads=2)
    kv = synth.fill_pool_host(wl)
    s0 = SideBySide(wl)     # only to learn where the tokens live
    try:
        bt = s0.bt_host.copy()
    finally:
        s0.close()
    for r, tok in ((0, 2000), (0, 2500), (1, 1700)):
        blk, slot = bt[r, tok // 16], tok % 16
        kv[:, blk, 0, :, slot, :] = np.float16(1200.0)
    q = np.abs(synth.fill_q_window_host(wl)) + np.float16(1.0)   # every query leans the same way
    _run_pruned(wl, sbs_kw={"kv_host": kv, "q_host": q})


def _keys_by_token(wl, make_key):
    """The synthetic pool with the K row of every (request, token) replaced by
    make_key(r, tok) -> fp16 [head_dim] (same for all layers and heads)."""
    from parity_util import SideBySide
    kv = synth.fill_pool_host(wl)
    s0 = SideBySide(wl)     # only to learn where the tokens live
    try:
        bt = s0.bt_host.copy()
    finally:
        s0.close()
    for r in range(wl.n_req):
        for tok in range(int(wl.seq_lens[r])):
            kv[:, bt[r, tok // 16], 0, :, tok % 16, :] = make_key(r, tok)
    return kv


@pytest.mark.parametrize("shape", ["ramp", "sinks", "late_and_uneven", "giant_sinks", "late_giants"])
def test_structured_attention_patterns(shape):
    """Inputs on which the factor between a row's running sum and its final sum
    behaves in the three extreme ways: it keeps shrinking along the whole head
    (logits that rise with the position), it is one from the start (a few
    dominant first tokens), and it differs wildly between the rows
    (half of the queries see their mass only at the end).  And two on which the
    scores span more octaves than the fine threshold buckets cover, so that the
    selection is decided 60 nats below the largest score: a few first tokens
    that take all the mass, and a few late ones (every reference before them is
    overtaken by 2^86: the squares of the numerators leave the fp32 range)."""
    d, W = 64, 32
    wl = _custom([3200, 2300], [640, 300], [fo.METHOD_SNAPKV] * 2, W=W, d=d, n_heads=2)
    rng = np.random.default_rng(17)
    u = np.zeros(d, np.float32)
    u[:8] = 1.0
    noise = lambda: 0.3 * rng.standard_normal(d).astype(np.float32)
    q = synth.fill_q_window_host(wl).astype(np.float32) * 0.3
    if shape == "ramp":
        key = lambda r, tok: (noise() + u * (6.0 * tok / 3200.0)).astype(np.float16)
        q[..., :8] += 2.0
    elif shape == "sinks":
        key = lambda r, tok: (noise() + (u * 8.0 if tok < 4 else 0.0)).astype(np.float16)
        q[..., :8] += 2.0
    elif shape == "late_and_uneven":
        key = lambda r, tok: (noise() + (u * 5.0 if tok >= int(wl.seq_lens[r]) - 200 else 0.0)).astype(np.float16)
        q[:, :, :, ::2, :8] += 2.5          # every other query row leans on the late keys
    elif shape == "giant_sinks":
        key = lambda r, tok: (noise() + (u * 30.0 if tok < 4 else 0.0)).astype(np.float16)
        q[..., :8] += 2.0
    else:
        late = lambda r, tok: int(wl.seq_lens[r]) - tok in (100, 150, 200)
        key = lambda r, tok: (noise() + (u * 30.0 if late(r, tok) else 0.0)).astype(np.float16)
        q[..., :8] += 2.0
    kv = _keys_by_token(wl, key)
    _run_pruned(wl, sbs_kw={"kv_host": kv, "q_host": q.astype(np.float16)})


def test_heads_beyond_the_fused_limit_share_a_call_with_pruned_ones():
    """A request too long for the fused kernel goes through the separate score,
    select and gather kernels; the other heads of the call are pruned."""
    wl = _custom([9000, 3000, 8200], [1500, 600, 4000], [fo.METHOD_SNAPKV] * 3, W=32, d=64, n_heads=2)
    _run_pruned(wl)


def test_repeated_calls_and_in_place_compaction():
    wl = _custom([5000, 3000], [2500, 1200], [fo.METHOD_SNAPKV] * 2, W=64, d=128, n_heads=2)
    s = _pruned(wl)
    try:
        s.compress_and_compare(scores=False)
        s.compress_and_compare(scores=False, budgets=np.array([600, 400], np.int32))
    finally:
        s.close()
    s = _pruned(wl, in_place=True)
    try:
        s.compress_and_compare(scores=False)
        s.compress_and_compare(scores=False, budgets=np.array([2100, 300], np.int32))
    finally:
        s.close()


def test_per_request_windows_and_pooling_widths():
    lens = [2700, 130, 3333, 2250, 4200, 96, 2064, 2513, 90, 8000]
    wl, methods, budgets, windows, pools, q_list = _mixed_window_batch(78, lens, d=128)
    budgets = np.minimum(budgets, np.maximum(windows, np.array(lens) // 4)).astype(np.int32)
    s = _pruned(wl)
    try:
        stats = s.compress_and_compare(methods, budgets, windows, pools, q_list=q_list, scores=False)
    finally:
        s.close()
    assert stats["units"] == len(lens) * wl.n_layers * wl.n_heads


def test_asking_for_the_scores_takes_the_two_pass_path():
    """With pruning switched on, a call that wants the scores still gets them,
    exact and complete."""
    wl = _custom([3000, 2200], [600, 300], [fo.METHOD_SNAPKV] * 2, W=64, d=128, n_heads=2)
    s = _pruned(wl)
    try:
        stats = s.compress_and_compare(scores=True)
        assert stats["max_rel_err"] < 2e-3 and stats["max_rel_err"] > 0.0
    finally:
        s.close()


@pytest.mark.parametrize("seed", range(8))
def test_random_long_batches(seed):
    rng = np.random.Generator(np.random.PCG64(9100 + seed))
    n_req = int(rng.integers(1, 4))
    W = int(rng.integers(1, 65))
    d = int(rng.choice([64, 128]))
    lens, methods, budgets = [], [], []
    for _ in range(n_req):
        m = int(rng.choice([fo.METHOD_SNAPKV, fo.METHOD_KNORM], p=[0.8, 0.2]))
        L = int(rng.integers(400, 8193))
        B = int(rng.integers(max(W, 1), L))
        lens.append(L); methods.append(m); budgets.append(B)
    wl = _custom(lens, budgets, methods, W=W, d=d, n_heads=int(rng.integers(1, 3)), seed=300 + seed)
    print("seed", seed, lens, budgets, methods, W, d, flush=True)
    _run_pruned(wl, pool_kernel=int(rng.choice([1, 5, 7, 9])))
