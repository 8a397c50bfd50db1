"""Host-side checks of the synthetic workload generator (no GPU)."""

import numpy as np

from paper_2503_08461_amd import synth
from oracle import fastcache_oracle as fo


def test_config_shapes_and_budgets():
    w1 = synth.make_workload(1)
    assert (w1.n_layers, w1.n_heads, w1.head_dim, w1.n_blocks) == (1, 4, 64, 64)
    assert w1.seq_lens.tolist() == [256] and w1.budgets.tolist() == [64] and w1.window == 16
    w2 = synth.make_workload(2)
    assert w2.budgets.tolist() == [160] and w2.seq_lens.tolist() == [640]
    w3 = synth.make_workload(3)
    assert w3.n_req == 32 and w3.seq_lens.min() >= 600 and w3.seq_lens.max() <= 1200
    assert (w3.methods[0::2] == synth.METHOD_SNAPKV).all()
    assert (w3.methods[1::2] == synth.METHOD_KNORM).all()
    assert (w3.budgets == w3.seq_lens // 2).all()
    w4 = synth.make_workload(4)
    assert w4.n_req == 64 and ((w4.seq_lens - 128) % 576 == 0).all()
    assert w4.seq_lens.min() >= 1280 and w4.seq_lens.max() <= 7040
    w5 = synth.make_workload(5)
    assert w5.n_req == 256 and w5.n_layers == 2
    # occupancy at the peak of the call
    for w, occ in ((w3, 0.70), (w4, 0.85)):
        old = sum(synth.blocks_for(int(l)) for l in w.seq_lens)
        new = sum(synth.blocks_for(int(b)) for b in w.budgets)
        assert abs((old + new) / w.n_blocks - occ) < 1e-3
    # config 4 must fit one MI355X
    assert w4.pool_bytes() < 215 * 2**30


def test_block_tables_are_disjoint_and_permuted():
    wl = synth.make_workload(3, n_layers=1, n_heads=1)
    st = fo.FreeStack(wl.n_blocks)
    rows = synth.build_block_tables(wl, st.alloc, st.free, lambda ids, ix: ids[ix])
    flat = np.concatenate(rows)
    assert len(set(flat.tolist())) == len(flat)
    assert st.top + len(flat) == wl.n_blocks
    assert not (np.diff(rows[0]) == 1).all()          # not contiguous
    # same seed, same tables
    st2 = fo.FreeStack(wl.n_blocks)
    rows2 = synth.build_block_tables(wl, st2.alloc, st2.free, lambda ids, ix: ids[ix])
    assert all((a == b).all() for a, b in zip(rows, rows2))


def test_fill_is_seeded_and_has_outlier_channels():
    wl = synth.make_workload(2, n_layers=1, n_heads=2)
    a = synth.fill_pool_host(wl)
    b = synth.fill_pool_host(wl)
    assert a.dtype == np.float16 and a.shape == wl.pool_shape() and (a == b).all()
    ids = synth.outlier_channel_ids(wl)
    k = a[0, :, 0, 0].astype(np.float64).reshape(-1, wl.head_dim)
    std = k.std(axis=0)
    assert (std[ids[0, 0]] > 6).all()
    rest = np.setdiff1d(np.arange(wl.head_dim), ids[0, 0])
    assert (std[rest] < 1.3).all()
    q = synth.fill_q_window_host(wl)
    assert q.shape == (1, 1, 2, 32, 128)
