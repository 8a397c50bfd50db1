"""GPU parity of the stage when the window rows' log-sum-exp is handed in
(fc_compress_batch_lse) and of the call that computes it (fc_window_lse),
against the CPU oracle on the same seeded inputs."""

import numpy as np
import pytest

from oracle import fastcache_oracle as fo
from paper_2503_08461_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(params=[0, 1], ids=["auto_fused", "two_pass"])
def score_mode(request):
    """The fused kernel and the separate kernels both skip the first pass."""
    return request.param


def _run(wl, score_mode, lse, **kw):
    from parity_util import SideBySide
    s = SideBySide(wl, score_mode=score_mode)
    try:
        stats = s.compress_and_compare(lse=lse, **kw)
    finally:
        s.close()
    print(wl.name, lse, stats, flush=True)
    assert stats["max_rel_err"] < 2e-3
    return stats


def _custom(L, B, method, W=16, d=64, n_heads=2, n_layers=1, seed=11):
    lens = np.array(L, dtype=np.int32)
    nb = int(sum(synth.blocks_for(int(x)) for x in lens) * 2 + 8)
    return synth.Workload("custom", n_layers, n_heads, d, nb, W, 7, lens,
                          np.array(method, dtype=np.int32), np.array(B, dtype=np.int32),
                          seed, False, True)


@pytest.mark.parametrize("lse", ["oracle", "library"])
def test_config1_tiny(score_mode, lse):
    _run(synth.make_workload(1), score_mode, lse)


@pytest.mark.parametrize("lse", ["oracle", "library"])
def test_config2_shape_reduced_heads(score_mode, lse):
    _run(synth.make_workload(2, n_layers=2, n_heads=3), score_mode, lse)


@pytest.mark.parametrize("lse", ["oracle", "library"])
def test_config3_mixed_methods_permuted_tables(score_mode, lse):
    # key-norm requests ride along: their rows of the input are never read
    _run(synth.make_workload(3, n_layers=1, n_heads=2, n_req=6), score_mode, lse)


@pytest.mark.parametrize("lse", ["oracle", "library"])
def test_config4_window64_long(score_mode, lse):
    _run(synth.make_workload(4, n_layers=1, n_heads=2, n_req=3), score_mode, lse)


@pytest.mark.parametrize("W", [1, 5, 16, 17, 33, 48, 64])
def test_window_sizes_and_ragged_tails(W, score_mode):
    wl = _custom([200, 131, W], [max(W, 40), max(W, 70), W], [fo.METHOD_SNAPKV] * 3, W=W, d=128)
    _run(wl, score_mode, "oracle")
    _run(wl, score_mode, "library", scale=0.21, pool_kernel=3)


def test_none_and_streaming_requests_pass_by(score_mode):
    wl = _custom([100, 64, 50, 90], [30, 1, 20, 40],
                 [fo.METHOD_SNAPKV, fo.METHOD_NONE, fo.METHOD_STREAMING, fo.METHOD_SNAPKV])
    _run(wl, score_mode, "library")


def test_a_shifted_row_scales_that_rows_contribution():
    """What the header says about an input that is off: the scores are those of
    the oracle given the same input, not those of the exact soft-max."""
    import torch
    from paper_2503_08461_amd import fastcache as fc
    from parity_util import SideBySide, check_scores
    wl = _custom([300], [80], [fo.METHOD_SNAPKV], W=4, d=64, n_heads=1)
    s = SideBySide(wl)
    try:
        lse = fo.window_lse_batch(s.kv_host, s.bt_host, wl.seq_lens, s.q_host, 4, wl.methods)
        lse = (lse + np.array([0.5, -0.25, 0.0, 1.0])).astype(np.float32)
        scores = torch.zeros(300, dtype=torch.float32, device=s.dev)
        fc.fc_compress_batch_lse(s.pool, s.bt_dev, s.lens_g, s.q_dev,
                                 torch.from_numpy(lse).to(s.dev), 4, wl.methods, wl.budgets, 7,
                                 0.0, scores, None)
        keys = fo.fetch_rows(s.kv_host, 0, s.bt_host[0], 0, 0, 300)
        want = fo.snapkv_scores_given_lse(keys, s.q_host[0, 0, 0].astype(np.float64), 0.125, 7,
                                          lse[0, 0, 0])
        check_scores(scores.cpu().numpy(), want)
        exact = fo.snapkv_scores(keys, s.q_host[0, 0, 0].astype(np.float64), 0.125, 7)
        assert np.abs(want[:296] / exact[:296] - 1).max() > 0.05
    finally:
        s.close()


def test_errors_and_untouched_state():
    import torch
    from paper_2503_08461_amd import fastcache as fc
    from parity_util import SideBySide
    wl = _custom([100, 40], [30, 20], [fo.METHOD_SNAPKV, fo.METHOD_KNORM])
    s = SideBySide(wl)
    try:
        lse = torch.zeros((2, 1, 2, 16), dtype=torch.float32, device=s.dev)
        before = (s.bt_dev.clone(), s.kv_dev.clone(), fc.fc_pool_num_free(s.pool))

        def untouched():
            assert (s.bt_dev == before[0]).all() and (s.kv_dev == before[1]).all()
            assert fc.fc_pool_num_free(s.pool) == before[2]
            assert (s.lens_g == wl.seq_lens).all()

        # a SnapKV request without the input
        with pytest.raises(fc.FastCacheError) as e:
            fc.fc_compress_batch_lse(s.pool, s.bt_dev, s.lens_g, s.q_dev, None, 16, wl.methods,
                                     wl.budgets)
        assert e.value.code == fc.FC_EINVAL
        untouched()
        # fc_window_lse: window out of range, request shorter than the window
        for w in (0, 65):
            with pytest.raises(fc.FastCacheError) as e:
                fc.fc_window_lse(s.pool, s.bt_dev, s.lens_g, None, w, wl.methods, None)
            assert e.value.code == fc.FC_EINVAL
        q = torch.zeros((2, 1, 2, 48, 64), dtype=torch.float16, device=s.dev)
        out = torch.zeros((2, 1, 2, 48), dtype=torch.float32, device=s.dev)
        with pytest.raises(fc.FastCacheError) as e:
            fc.fc_window_lse(s.pool, s.bt_dev, s.lens_g, q, 48, None, out)   # request 1: L = 40
        assert e.value.code == fc.FC_EINVAL
        untouched()
        # without a method array every request is computed; nothing else changes
        q16 = s.q_dev
        out16 = torch.full((2, 1, 2, 16), float("nan"), dtype=torch.float32, device=s.dev)
        fc.fc_window_lse(s.pool, s.bt_dev, s.lens_g, q16, 16, None, out16)
        torch.cuda.synchronize()
        want = fo.window_lse_batch(s.kv_host, s.bt_host, wl.seq_lens, s.q_host, 16,
                                   np.array([fo.METHOD_SNAPKV] * 2))
        assert np.abs(out16.cpu().numpy() - want).max() <= 2e-3
        untouched()
        # only a key-norm request: no input needed
        m = np.array([fo.METHOD_NONE, fo.METHOD_KNORM], dtype=np.int32)
        fc.fc_compress_batch_lse(s.pool, s.bt_dev, s.lens_g, None, None, 16, m, wl.budgets)
        assert s.lens_g.tolist() == [100, 20]
    finally:
        s.close()


@pytest.mark.parametrize("seed", range(8))
def test_random_workloads(seed):
    rng = np.random.Generator(np.random.PCG64(7000 + seed))
    n_req = int(rng.integers(1, 6))
    W = int(rng.integers(1, 65))
    d = int(rng.choice([64, 128]))
    lens, methods, budgets = [], [], []
    for _ in range(n_req):
        m = int(rng.choice([fo.METHOD_SNAPKV, fo.METHOD_KNORM, fo.METHOD_NONE], p=[0.7, 0.2, 0.1]))
        lo = W if m == fo.METHOD_SNAPKV else 1
        L = int(rng.integers(lo, 3001)) if rng.random() < 0.7 else int(rng.integers(lo, lo + 40))
        B = int(rng.integers(lo, L + 1))
        lens.append(L); methods.append(m); budgets.append(B)
    wl = _custom(lens, budgets, methods, W=W, d=d, n_heads=int(rng.integers(1, 4)),
                 n_layers=int(rng.integers(1, 3)), seed=300 + seed)
    mode = int(rng.integers(0, 2))
    lse = ["oracle", "library"][int(rng.integers(0, 2))]
    kernel = int(rng.choice([1, 3, 5, 7, 9, 15]))
    print("seed", seed, "lens", lens, "budgets", budgets, "methods", methods, "W", W, "d", d,
          "mode", mode, "lse", lse, "pool", kernel, flush=True)
    _run(wl, mode, lse, pool_kernel=kernel)
