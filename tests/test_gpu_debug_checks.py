"""Ownership checks (fc_set_debug_checks): a double free, a foreign id, a
duplicate id and a corrupt block table are refused with FC_EINVAL and leave
the pool as it was; correct use behaves as without the checks (parity with the
oracle, pool invariants) and raises nothing."""

import numpy as np
import pytest

from oracle import fastcache_oracle as fo
from paper_2503_08461_amd import synth

pytestmark = pytest.mark.gpu


def _small_pool(n_blocks=32):
    import torch
    from paper_2503_08461_amd import fastcache as fc
    kv = torch.zeros((1, n_blocks, 2, 1, 16, 64), dtype=torch.float16, device="cuda:0")
    pool = fc.fc_pool_create(kv, n_blocks, 1, 1, 64)
    fc.fc_set_debug_checks(pool, True)
    return fc, torch, pool, kv


def _refused(fc, call):
    with pytest.raises(fc.FastCacheError) as e:
        call()
    assert e.value.code == fc.FC_EINVAL
    return str(e.value)


def test_double_free_foreign_and_duplicate_ids_are_refused():
    fc, torch, pool, kv = _small_pool()
    try:
        ids = fc.fc_pool_alloc(pool, 6)
        assert ids.cpu().tolist() == [0, 1, 2, 3, 4, 5]
        fc.fc_pool_free(pool, ids[:2].contiguous())
        snap = fc.fc_pool_export_state(pool)
        # double free
        msg = _refused(fc, lambda: fc.fc_pool_free(pool, ids[:2].contiguous()))
        assert "not handed out" in msg
        # one of the ids is fine, the other already free: nothing is pushed at all
        _refused(fc, lambda: fc.fc_pool_free(pool, ids[1:3].contiguous()))
        # ids outside the pool, and an id that was never handed out
        for bad in ([32], [-1], [2, 1 << 20], [31]):
            t = torch.tensor(bad, dtype=torch.int32, device="cuda:0")
            _refused(fc, lambda: fc.fc_pool_free(pool, t))
        # the same id twice in one call
        dup = torch.tensor([2, 3, 2], dtype=torch.int32, device="cuda:0")
        assert "twice" in _refused(fc, lambda: fc.fc_pool_free(pool, dup))
        after = fc.fc_pool_export_state(pool)
        assert after[1] == snap[1] and (after[0] == snap[0]).all()
        assert fc.fc_pool_num_free(pool) == 32 - 4
        # the refused ids are still the caller's and can be released properly
        fc.fc_pool_free(pool, ids[2:].contiguous())
        stack, top = fc.fc_pool_export_state(pool)
        assert top == 32 and sorted(stack.tolist()) == list(range(32))
        # and handed out again
        again = fc.fc_pool_alloc(pool, 32)
        assert sorted(again.cpu().tolist()) == list(range(32))
        _refused(fc, lambda: fc.fc_pool_free(pool, torch.cat([again, again[:1]])))
        fc.fc_pool_free(pool, again)
        # without the checks the same misuse goes unnoticed (ids are only clamped)
        fc.fc_set_debug_checks(pool, False)
        one = fc.fc_pool_alloc(pool, 1)
        fc.fc_pool_free(pool, one)
        assert fc.fc_pool_num_free(pool) == 32
    finally:
        fc.fc_pool_destroy(pool)


def test_import_state_redefines_what_is_free():
    fc, torch, pool, kv = _small_pool(16)
    try:
        ids = fc.fc_pool_alloc(pool, 8)
        stack, top = fc.fc_pool_export_state(pool)
        fc.fc_pool_free(pool, ids)
        fc.fc_pool_import_state(pool, stack, top)            # back to "8 handed out"
        fc.fc_pool_free(pool, ids[:4].contiguous())          # accepted again
        _refused(fc, lambda: fc.fc_pool_free(pool, ids[:4].contiguous()))
        dev_stack = torch.from_numpy(stack).cuda()
        fc.fc_pool_import_state_dev(pool, dev_stack, top)
        fc.fc_pool_free(pool, ids)
        assert fc.fc_pool_num_free(pool) == 16
    finally:
        fc.fc_pool_destroy(pool)


def test_pop_of_a_block_that_is_not_free_is_reported_once():
    fc, torch, pool, kv = _small_pool(16)
    try:
        # a corrupt free list from outside: block 5 is on the stack twice
        stack = np.arange(15, -1, -1, dtype=np.int32)
        stack[14] = 5                                         # pops return 0, 5, 2, ...
        fc.fc_pool_import_state(pool, stack, 16)
        ids = fc.fc_pool_alloc(pool, 6)                       # 0, 5, 2, 3, 4, 5: the second 5 is not free
        assert ids.cpu().tolist() == [0, 5, 2, 3, 4, 5]
        with pytest.raises(fc.FastCacheError) as e:
            fc.fc_pool_export_state(pool)
        assert e.value.code == fc.FC_EDEVICE and "not free" in str(e.value)
        # reported once; the pool itself keeps working
        out, top = fc.fc_pool_export_state(pool)
        assert top == 10 and (out == stack).all()
    finally:
        fc.fc_pool_destroy(pool)


def _custom(L, B, method, W=16, d=64, n_heads=2, n_layers=1, seed=11):
    lens = np.array(L, dtype=np.int32)
    nb = int(sum(synth.blocks_for(int(x)) for x in lens) * 2 + 8)
    return synth.Workload("custom", n_layers, n_heads, d, nb, W, 7, lens,
                          np.array(method, dtype=np.int32), np.array(B, dtype=np.int32),
                          seed, False, True)


def test_corrupt_block_tables_are_refused_and_correct_use_is_unchanged():
    import torch
    from paper_2503_08461_amd import fastcache as fc
    from parity_util import SideBySide
    wl = _custom([300, 77, 1200, 520], [100, 30, 400, 64],
                 [fo.METHOD_SNAPKV, fo.METHOD_KNORM, fo.METHOD_SNAPKV, fo.METHOD_STREAMING])
    s = SideBySide(wl)
    try:
        fc.fc_set_debug_checks(s.pool, True)
        good = s.bt_dev.clone()
        torch.cuda.synchronize()
        before = (s.kv_dev.clone(), fc.fc_pool_export_state(s.pool))

        def attempt():
            fc.fc_compress_batch(s.pool, s.bt_dev, s.lens_g, s.q_dev, wl.window, wl.methods,
                                 wl.budgets)
        free_id = int(fc.fc_pool_export_state(s.pool)[0][0])
        for (r, i, v) in ((0, 1, int(good[0, 0])),          # the same block twice in a row
                          (2, 5, int(good[1, 0])),          # a block of another request
                          (1, 0, free_id),                  # a block that is free
                          (3, 2, wl.n_blocks + 7),          # outside the pool
                          (3, 0, -1)):
            s.bt_dev.copy_(good)
            s.bt_dev[r, i] = v
            _refused(fc, attempt)
            s.bt_dev.copy_(good)
            torch.cuda.synchronize()
            now = fc.fc_pool_export_state(s.pool)
            assert now[1] == before[1][1] and (now[0] == before[1][0]).all()
            assert (s.lens_g == wl.seq_lens).all()
            assert torch.equal(s.kv_dev, before[0])
        # correct use: full parity with the oracle, twice in a row, then release everything
        stats = s.compress_and_compare()
        assert stats["max_rel_err"] < 2e-3
        s.compress_and_compare(budgets=np.array([50, 10, 100, 20], np.int32))
        for r in range(wl.n_req):
            n = fo.blocks_for(int(s.lens_g[r]), 16)
            fc.fc_pool_free(s.pool, s.bt_dev[r, :n].contiguous())
        stack, top = fc.fc_pool_export_state(s.pool)       # also: no flag was raised
        assert top == wl.n_blocks and sorted(stack.tolist()) == list(range(wl.n_blocks))
    finally:
        s.close()


def test_in_place_compaction_and_append_keep_the_books():
    import torch
    from paper_2503_08461_amd import fastcache as fc
    from parity_util import SideBySide
    wl = _custom([333, 160], [100, 48], [fo.METHOD_KNORM, fo.METHOD_KNORM], d=64, n_heads=1)
    s = SideBySide(wl, in_place=True)
    try:
        fc.fc_set_debug_checks(s.pool, True)
        s.compress_and_compare()                              # in place: 7 and 3 blocks kept
        # decode appends: request 1 is on a block boundary (48 tokens) and pops a block
        new_kv = torch.zeros((2, 1, 2, 1, 64), dtype=torch.float16, device=s.dev)
        lens = s.lens_g.copy()
        fc.fc_append_batch(s.pool, s.bt_dev, lens, new_kv)
        assert lens.tolist() == [101, 49]
        # everything the requests hold can be released exactly once
        for r in range(2):
            n = fo.blocks_for(int(lens[r]), 16)
            fc.fc_pool_free(s.pool, s.bt_dev[r, :n].contiguous())
            _refused(fc, lambda: fc.fc_pool_free(s.pool, s.bt_dev[r, :1].contiguous()))
        stack, top = fc.fc_pool_export_state(s.pool)
        assert top == wl.n_blocks and sorted(stack.tolist()) == list(range(wl.n_blocks))
    finally:
        s.close()
