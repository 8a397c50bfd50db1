"""GPU parity of the decode-side entry points (fc_append_batch,
fc_decode_attention) with oracle/decode_oracle.py, through the C ABI."""

import numpy as np
import pytest

from oracle import fastcache_oracle as fo
from oracle import decode_oracle as do
from paper_2503_08461_amd import synth

pytestmark = pytest.mark.gpu

RTOL, ATOL = 1e-3, 1e-4   # fp32 accumulation and hardware exp2 against the fp64 oracle


def _setup(lens, d=128, n_heads=3, n_layers=2, seed=5, spare=6, table_slack=2):
    from parity_util import SideBySide
    lens = np.array(lens, dtype=np.int32)
    nb = int(sum(synth.blocks_for(int(x)) for x in lens) + spare)
    wl = synth.Workload("decode", n_layers, n_heads, d, nb, 16, 7, np.maximum(lens, 0),
                        np.full(len(lens), fo.METHOD_NONE, np.int32), np.maximum(lens, 1), seed,
                        False, True)
    wl.extra["table_slack"] = table_slack
    return SideBySide(wl), wl


@pytest.mark.parametrize("d", [64, 128])
def test_decode_attention_matches_the_oracle(d):
    """Ragged lengths over several blocks and waves, a single token, an empty
    request, lengths that end inside and on a block boundary."""
    import torch
    from paper_2503_08461_amd import fastcache as fc
    lens = [1, 0, 15, 16, 17, 63, 64, 65, 700, 2049, 333]
    sbs, wl = _setup(lens, d=d)
    try:
        rng = np.random.default_rng(8)
        q = rng.standard_normal((len(lens), wl.n_layers, wl.n_heads, d)).astype(np.float16)
        out = fc.fc_decode_attention(sbs.pool, sbs.bt_dev, sbs.lens_g,
                                     torch.from_numpy(q).to(sbs.dev))
        torch.cuda.synchronize()
        got = out.cpu().numpy().astype(np.float64)
        want = do.decode_attention(sbs.kv_host, sbs.bt_host, sbs.lens_o, q)
        assert (got[1] == 0).all()
        err = np.abs(got - want)
        assert (err <= RTOL * np.abs(want) + ATOL).all(), float(err.max())
        # another scale
        out2 = fc.fc_decode_attention(sbs.pool, sbs.bt_dev, sbs.lens_g,
                                      torch.from_numpy(q).to(sbs.dev), scale=0.31)
        torch.cuda.synchronize()
        want2 = do.decode_attention(sbs.kv_host, sbs.bt_host, sbs.lens_o, q, scale=0.31)
        err2 = np.abs(out2.cpu().numpy() - want2)
        assert (err2 <= RTOL * np.abs(want2) + ATOL).all(), float(err2.max())
        sbs.compare_state()          # a read-only call
    finally:
        sbs.close()


def test_append_then_attend_then_compress_round_trip():
    """A few decode steps (append on both sides, block boundaries crossed, one
    request switched off), attention after each step, then a compression of the
    grown caches: state stays identical to the oracle's throughout."""
    import torch
    from paper_2503_08461_amd import fastcache as fc
    lens = [30, 16, 0, 47, 5]
    sbs, wl = _setup(lens, d=128, n_heads=2, n_layers=2, spare=20)
    try:
        rng = np.random.default_rng(9)
        enable = np.array([1, 1, 1, 1, 0], dtype=np.int32)
        for step in range(20):
            new = rng.standard_normal((len(lens), wl.n_layers, 2, wl.n_heads, 128)).astype(np.float16)
            fc.fc_append_batch(sbs.pool, sbs.bt_dev, sbs.lens_g, torch.from_numpy(new).to(sbs.dev),
                               enable)
            assert do.append_batch(sbs.kv_host, sbs.stack, sbs.bt_host, sbs.lens_o, new,
                                   enable) is None
            torch.cuda.synchronize()
            sbs.compare_state()
            q = rng.standard_normal((len(lens), wl.n_layers, wl.n_heads, 128)).astype(np.float16)
            got = fc.fc_decode_attention(sbs.pool, sbs.bt_dev, sbs.lens_g,
                                         torch.from_numpy(q).to(sbs.dev)).cpu().numpy()
            want = do.decode_attention(sbs.kv_host, sbs.bt_host, sbs.lens_o, q)
            assert (np.abs(got - want) <= RTOL * np.abs(want) + ATOL).all()
        assert sbs.lens_g.tolist() == [50, 36, 20, 67, 5]
        methods = np.array([fo.METHOD_KNORM, fo.METHOD_SNAPKV, fo.METHOD_STREAMING,
                            fo.METHOD_SNAPKV, fo.METHOD_NONE], np.int32)
        budgets = np.array([20, 16, 7, 30, 1], np.int32)
        sbs.compress_and_compare(methods, budgets)
    finally:
        sbs.close()


def test_append_errors_leave_everything_untouched():
    import torch
    from paper_2503_08461_amd import fastcache as fc
    lens = [32, 16, 7]
    sbs, wl = _setup(lens, d=64, n_heads=1, n_layers=1, spare=1)
    try:
        new = torch.zeros((3, 1, 2, 1, 64), dtype=torch.float16, device=sbs.dev)
        free = fc.fc_pool_num_free(sbs.pool)
        assert free == 1
        # two requests sit on a block boundary, one block is free
        with pytest.raises(fc.FastCacheError) as e:
            fc.fc_append_batch(sbs.pool, sbs.bt_dev, sbs.lens_g, new)
        assert e.value.code == fc.FC_ENOMEM
        # table row full: 32 tokens in a row of 2 entries
        narrow = sbs.bt_dev[:, :2].contiguous()
        with pytest.raises(fc.FastCacheError) as e:
            fc.fc_append_batch(sbs.pool, narrow, sbs.lens_g, new)
        assert e.value.code == fc.FC_EINVAL
        assert fc.fc_pool_num_free(sbs.pool) == free and sbs.lens_g.tolist() == lens
        sbs.compare_state()
        # with the first request switched off it goes through
        en = np.array([0, 1, 1], dtype=np.int32)
        fc.fc_append_batch(sbs.pool, sbs.bt_dev, sbs.lens_g, new, en)
        assert do.append_batch(sbs.kv_host, sbs.stack, sbs.bt_host, sbs.lens_o,
                               new.cpu().numpy(), en) is None
        torch.cuda.synchronize()
        sbs.compare_state()
    finally:
        sbs.close()


@pytest.mark.parametrize("d", [64, 128])
def test_attention_over_kept_lists_of_an_uncompacted_cache(d):
    """fc_decode_attention_kept on the uncompressed pool with the kept lists
    that a compression of a COPY of the batch produced: equal (to tolerance) to
    the oracle over those lists, and to the plain attention on the compacted copy."""
    import torch
    from paper_2503_08461_amd import fastcache as fc
    lens = [700, 64, 129, 2050, 16, 333]
    sbs, wl = _setup(lens, d=d, n_heads=2, n_layers=2, spare=240)
    try:
        rng = np.random.default_rng(10)
        n_lh = wl.n_layers * wl.n_heads
        methods = np.array([fo.METHOD_SNAPKV, fo.METHOD_KNORM, fo.METHOD_STREAMING,
                            fo.METHOD_SNAPKV, fo.METHOD_KNORM, fo.METHOD_SNAPKV], np.int32)
        budgets = np.array([140, 64, 17, 410, 1, 100], np.int32)
        q = rng.standard_normal((len(lens), wl.n_layers, wl.n_heads, d)).astype(np.float16)
        q_dev = torch.from_numpy(q).to(sbs.dev)
        bt_before, lens_before = sbs.bt_dev.clone(), sbs.lens_g.copy()
        kv_before = sbs.kv_host.copy()
        bt_host_before = sbs.bt_host.copy()
        kept_dev = torch.empty(int(budgets.sum()) * n_lh, dtype=torch.int32, device=sbs.dev)
        fc.fc_compress_batch(sbs.pool, sbs.bt_dev, sbs.lens_g, sbs.q_dev, wl.window, methods,
                             budgets, 7, 0.0, None, kept_dev)
        torch.cuda.synchronize()
        # the old blocks still hold the uncompressed caches (compaction writes only free blocks)
        got = fc.fc_decode_attention_kept(sbs.pool, bt_before, lens_before, budgets, kept_dev,
                                          q_dev).cpu().numpy().astype(np.float64)
        after = fc.fc_decode_attention(sbs.pool, sbs.bt_dev, sbs.lens_g,
                                       q_dev).cpu().numpy().astype(np.float64)
        kept_host = kept_dev.cpu().numpy()
        kept, off = [], 0
        for r in range(len(lens)):
            B = int(budgets[r])
            kept.append(kept_host[off:off + n_lh * B].reshape(wl.n_layers, wl.n_heads, B))
            off += n_lh * B
        want = do.decode_attention_kept(kv_before, bt_host_before, lens_before, kept, q)
        assert (np.abs(got - want) <= RTOL * np.abs(want) + ATOL).all()
        assert (np.abs(after - want) <= RTOL * np.abs(want) + ATOL).all()
    finally:
        sbs.close()
