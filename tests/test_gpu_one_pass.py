"""The opt-in one-pass scheduling (FC_SCORE_ONE_PASS: the token-split score
kernel, teams of workgroups that hold a head's keys in registers and exchange
row statistics) against the CPU oracle, through the C ABI, to the same bar as
the default scheduling.  Kept in a file of its own: it is not on the default
path, and it is the only kernel whose workgroups wait for each other."""

import numpy as np
import pytest

from oracle import fastcache_oracle as fo
from paper_2503_08461_amd import synth
from test_gpu_parity import _custom, _run, _sbs, _mixed_window_batch

pytestmark = pytest.mark.gpu

ONE_PASS = 2


@pytest.mark.parametrize("config,kw", [(1, {}), (2, dict(n_layers=2, n_heads=3)),
                                       (3, dict(n_layers=1, n_heads=2, n_req=6)),
                                       (4, dict(n_layers=1, n_heads=2, n_req=3))])
def test_reduced_configs(config, kw):
    _run(synth.make_workload(config, **kw), ONE_PASS)


@pytest.mark.parametrize("W", [1, 5, 16, 17, 33, 48, 64])
def test_window_sizes(W):
    _run(_custom([200, 131], [max(W, 40), max(W, 70)], [fo.METHOD_SNAPKV] * 2, W=W, d=128), ONE_PASS)


def test_degenerate_budgets_mixed_methods_and_custom_scale():
    # B == L (identity), B == W (window only), L == W == B, single token; pass-through rows
    _run(_custom([97, 80, 16, 1, 33, 50], [97, 16, 16, 1, 33, 10],
                 [fo.METHOD_KNORM, fo.METHOD_SNAPKV, fo.METHOD_SNAPKV, fo.METHOD_KNORM,
                  fo.METHOD_SNAPKV, fo.METHOD_NONE]), ONE_PASS)
    _run(_custom([300, 150], [100, 60], [fo.METHOD_SNAPKV, fo.METHOD_STREAMING], d=128), ONE_PASS,
         scale=0.05, pool_kernel=15)


def test_repeated_compression_and_in_place_compaction():
    from parity_util import SideBySide
    wl = _custom([400, 300], [200, 150], [fo.METHOD_SNAPKV] * 2, W=16, d=128)
    for in_place in (False, True):
        s = SideBySide(wl, score_mode=ONE_PASS, in_place=in_place)
        try:
            s.compress_and_compare()
            s.compress_and_compare(budgets=np.array([64, 20], np.int32))
        finally:
            s.close()


@pytest.mark.parametrize("L,W,d", [(513, 64, 128), (2049, 64, 128), (1500, 33, 64), (3000, 16, 128),
                                   (5000, 48, 128), (7040, 64, 128), (15000, 64, 64),
                                   (15360, 17, 128)])
def test_one_pass_teams_of_several_workgroups(L, W, d):
    """The token-split score kernel with teams of 1..64 workgroups per head (a
    workgroup holds 15 blocks): ragged block split, members with few or no
    blocks, teams that poll in several batches, the longest head it takes."""
    _run(_custom([L, L // 2 + 7], [max(W, L // 5), max(W, L // 4)], [fo.METHOD_SNAPKV] * 2,
                 W=W, d=d, n_heads=3), 2)


def test_one_pass_many_units_per_team_and_many_team_sizes():
    """More units than teams (every team walks several heads, with the blocks
    of the next head requested during the exchange of this one), and more
    distinct team sizes than launches (sizes rounded up along the ladder)."""
    lens = [300 + 241 * i for i in range(16)]                      # 19 .. 245 blocks
    wl = _custom(lens, [max(64, L // 4) for L in lens], [fo.METHOD_SNAPKV] * 16, W=64, d=64,
                 n_heads=8, n_layers=4)
    s = _sbs(wl, score_mode=2)
    try:
        stats = s.compress_and_compare()
    finally:
        s.close()
    assert stats["max_rel_err"] < 2e-3


def test_one_pass_refuses_heads_beyond_its_capacity():
    from paper_2503_08461_amd import fastcache as fc
    wl = _custom([15361, 200], [4000, 100], [fo.METHOD_SNAPKV] * 2, W=32, d=64, n_heads=1)
    s = _sbs(wl, score_mode=2)
    try:
        top = fc.fc_pool_num_free(s.pool)
        with pytest.raises(fc.FastCacheError) as e:
            fc.fc_compress_batch(s.pool, s.bt_dev, s.lens_g, s.q_dev, 32, wl.methods, wl.budgets)
        assert e.value.code == fc.FC_EINVAL
        assert fc.fc_pool_num_free(s.pool) == top and (s.lens_g == wl.seq_lens).all()
        s.compare_state()
    finally:
        s.close()


@pytest.mark.parametrize("threshold", [1, 1000, 4000])
def test_auto_mode_mixes_split_fused_and_separate_units(threshold):
    """One batch whose SnapKV requests fall on both sides of the split
    threshold, with key-norm and streaming requests, and one head that is too
    long for the fused kernel and for a team."""
    lens = [5000, 900, 2500, 1200, 300, 16000, 3100]
    methods = [fo.METHOD_SNAPKV, fo.METHOD_SNAPKV, fo.METHOD_KNORM, fo.METHOD_SNAPKV,
               fo.METHOD_STREAMING, fo.METHOD_SNAPKV, fo.METHOD_SNAPKV]
    wl = _custom(lens, [max(64, L // 3) for L in lens], methods, W=48, d=128, n_heads=2)
    s = _sbs(wl, score_mode=0, split_threshold=threshold)
    try:
        stats = s.compress_and_compare()
    finally:
        s.close()
    assert stats["max_rel_err"] < 2e-3




@pytest.mark.parametrize("d", [64, 128])
def test_per_request_window_and_pool_kernel_in_one_batch(d):
    lens = [700, 130, 333, 250, 1200, 96, 64, 513, 90, 8300]
    wl, methods, budgets, windows, pools, q_list = _mixed_window_batch(77, lens, d=d)
    sbs = _sbs(wl, score_mode=ONE_PASS)
    try:
        stats = sbs.compress_and_compare(methods, budgets, windows, pools, q_list=q_list)
    finally:
        sbs.close()
    assert stats["units"] == len(lens) * wl.n_layers * wl.n_heads
    assert stats["max_rel_err"] < 2e-3
