"""The entry point that allocates nothing (fc_compress_batch_noalloc, for callers
that cannot call hipMalloc) against fc_compress_batch on identical pools: two
calls in a row, the second on a smaller input; everything the stage produces
must be bit-identical, because the same kernels run."""

import numpy as np
import pytest

from oracle import fastcache_oracle as fo
from paper_2503_08461_amd import synth

pytestmark = pytest.mark.gpu


def _state(s):
    import torch
    from paper_2503_08461_amd import fastcache as fc
    torch.cuda.synchronize()
    stack, top = fc.fc_pool_export_state(s.pool)
    return (s.kv_dev.cpu().numpy().view(np.uint16).copy(), s.bt_dev.cpu().numpy().copy(),
            s.lens_g.copy(), stack[:top].copy(), top)


def _same(a, b, valid_blocks_only=True):
    kv_a, bt_a, lens_a, st_a, top_a = a
    kv_b, bt_b, lens_b, st_b, top_b = b
    assert top_a == top_b and (st_a == st_b).all()
    assert (lens_a == lens_b).all()
    assert (bt_a == bt_b).all()
    # every byte of the pool, free blocks included: the two calls run the same kernels
    assert (kv_a == kv_b).all()


def test_two_calls_in_a_row_match_the_allocating_entry_point():
    import torch
    from paper_2503_08461_amd import fastcache as fc
    from parity_util import SideBySide
    lens = [700, 333, 1200, 96, 8192, 250, 64, 513]
    methods = np.array([fo.METHOD_SNAPKV, fo.METHOD_KNORM, fo.METHOD_SNAPKV, fo.METHOD_STREAMING,
                        fo.METHOD_SNAPKV, fo.METHOD_NONE, fo.METHOD_SNAPKV, fo.METHOD_KNORM],
                       dtype=np.int32)
    budgets = np.array([300, 100, 400, 40, 2000, 1, 32, 200], dtype=np.int32)
    nb = int(sum(synth.blocks_for(x) for x in lens) * 2 + 8)
    wl = synth.Workload("noalloc", 2, 3, 128, nb, 32, 7, np.array(lens, np.int32), methods,
                        budgets, 23, False, True)
    a, b = SideBySide(wl), SideBySide(wl)     # identical pools, tables and queries
    try:
        n_lh = wl.n_layers * wl.n_heads
        comp = methods != fo.METHOD_NONE
        n_scores = int(np.array(lens)[comp].sum()) * n_lh
        n_kept = int(budgets[comp].sum()) * n_lh
        sc_a = torch.full((n_scores,), float("nan"), device=a.dev)
        sc_b = torch.full((n_scores,), float("nan"), device=a.dev)
        kp_a = torch.full((n_kept,), -7, dtype=torch.int32, device=a.dev)
        # first call: the library's kept scratch on both sides (no kept_out for the new
        # entry point, so that its fixed array is what the gather reads)
        fc.fc_compress_batch(a.pool, a.bt_dev, a.lens_g, a.q_dev, wl.window, methods, budgets,
                             wl.pool_kernel, 0.0, sc_a, kp_a)
        # pool b has never been through a call, so the library holds no scratch for it yet:
        # an allocation inside the call would show as less free device memory
        torch.cuda.synchronize()
        free_before = torch.cuda.mem_get_info()[0]
        fc.fc_compress_batch_noalloc(b.pool, b.bt_dev, b.lens_g, b.q_dev, wl.window, methods,
                                     budgets, wl.pool_kernel, 0.0, sc_b, None)
        torch.cuda.synchronize()
        assert torch.cuda.mem_get_info()[0] >= free_before
        _same(_state(a), _state(b))
        assert (sc_a.cpu().numpy().view(np.uint32) == sc_b.cpu().numpy().view(np.uint32)).all()
        assert (b.lens_g[comp] == budgets[comp]).all()

        # second call, smaller: three of the compressed requests again, lower budgets,
        # this time with the kept lists handed out by both
        m2 = np.zeros_like(methods)
        b2 = budgets.copy()
        for r, (m, bud) in {0: (fo.METHOD_KNORM, 120), 2: (fo.METHOD_SNAPKV, 64),
                            4: (fo.METHOD_SNAPKV, 700)}.items():
            m2[r], b2[r] = m, bud
        n_kept2 = int(b2[m2 != 0].sum()) * n_lh
        k2_a = torch.full((n_kept2,), -7, dtype=torch.int32, device=a.dev)
        k2_b = torch.full((n_kept2,), -7, dtype=torch.int32, device=a.dev)
        fc.fc_compress_batch(a.pool, a.bt_dev, a.lens_g, a.q_dev, wl.window, m2, b2,
                             wl.pool_kernel, 0.0, None, k2_a)
        fc.fc_compress_batch_noalloc(b.pool, b.bt_dev, b.lens_g, b.q_dev, wl.window, m2, b2,
                                     wl.pool_kernel, 0.0, None, k2_b)
        _same(_state(a), _state(b))
        assert (k2_a == k2_b).all() and int(k2_a.min()) >= 0
        assert a.lens_g[0] == 120 and b.lens_g[4] == 700
    finally:
        a.close()
        b.close()


def test_limits_are_refused_with_nothing_touched():
    from paper_2503_08461_amd import fastcache as fc
    from parity_util import SideBySide
    # a head longer than the fused kernel takes
    wl = synth.Workload("noalloc_long", 1, 1, 64, 1200, 16, 7, np.array([8200, 300], np.int32),
                        np.array([fo.METHOD_SNAPKV] * 2, np.int32), np.array([900, 100], np.int32),
                        5, False, True)
    s = SideBySide(wl)
    try:
        before = _state(s)
        with pytest.raises(fc.FastCacheError) as e:
            fc.fc_compress_batch_noalloc(s.pool, s.bt_dev, s.lens_g, s.q_dev, wl.window,
                                         wl.methods, wl.budgets)
        assert e.value.code == fc.FC_EINVAL
        fc.fc_set_score_mode(s.pool, fc.FC_SCORE_TWO_PASS)     # needs score scratch
        m = np.array([fo.METHOD_NONE, fo.METHOD_SNAPKV], np.int32)
        with pytest.raises(fc.FastCacheError) as e:
            fc.fc_compress_batch_noalloc(s.pool, s.bt_dev, s.lens_g, s.q_dev, wl.window, m,
                                         wl.budgets)
        assert e.value.code == fc.FC_EINVAL
        _same(before, _state(s))
        fc.fc_set_score_mode(s.pool, fc.FC_SCORE_AUTO)
        fc.fc_compress_batch_noalloc(s.pool, s.bt_dev, s.lens_g, s.q_dev, wl.window, m, wl.budgets)
        assert s.lens_g.tolist() == [8200, 100]
    finally:
        s.close()
    # more requests than the fixed descriptor space takes
    n = 65
    wl = synth.Workload("noalloc_many", 1, 1, 64, 400, 16, 7, np.full(n, 40, np.int32),
                        np.full(n, fo.METHOD_KNORM, np.int32), np.full(n, 10, np.int32), 6, False,
                        True)
    s = SideBySide(wl)
    try:
        before = _state(s)
        with pytest.raises(fc.FastCacheError) as e:
            fc.fc_compress_batch_noalloc(s.pool, s.bt_dev, s.lens_g, s.q_dev, wl.window,
                                         wl.methods, wl.budgets)
        assert e.value.code == fc.FC_EINVAL
        _same(before, _state(s))
        m = wl.methods.copy()
        m[0] = fo.METHOD_NONE                                  # 64 fit
        fc.fc_compress_batch_noalloc(s.pool, s.bt_dev, s.lens_g, s.q_dev, wl.window, m, wl.budgets)
        assert s.lens_g[0] == 40 and (s.lens_g[1:] == 10).all()
    finally:
        s.close()
