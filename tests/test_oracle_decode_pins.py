"""Pins of the decode-side oracle (oracle/decode_oracle.py)."""

import numpy as np
import pytest

from oracle import fastcache_oracle as fo
from oracle import decode_oracle as do


def _pool(rng, n_layers, nb, n_heads, bs, d):
    return rng.standard_normal((n_layers, nb, 2, n_heads, bs, d)).astype(np.float16)


def test_append_positions_block_allocation_and_errors():
    rng = np.random.default_rng(3)
    n_layers, n_heads, bs, d, nb = 2, 3, 4, 8, 12
    kv = _pool(rng, n_layers, nb, n_heads, bs, d)
    st = fo.FreeStack(nb)
    lens = np.array([5, 8, 0, 3], dtype=np.int32)     # request 1 and 2 sit on a block boundary
    bt = np.full((4, 3), -1, dtype=np.int32)
    for r in range(4):
        n = fo.blocks_for(int(lens[r]), bs)
        bt[r, :n] = st.alloc(n)
    assert bt[:, 0].tolist() == [0, 2, -1, 4] and bt[1, 1] == 3
    new = rng.standard_normal((4, n_layers, 2, n_heads, d)).astype(np.float16)
    kv0, bt0 = kv.copy(), bt.copy()
    assert do.append_batch(kv, st, bt, lens, new, enable=[1, 1, 1, 0]) is None
    assert lens.tolist() == [6, 9, 1, 3]
    # new blocks popped in batch order: request 1 gets id 5, request 2 gets id 6
    assert bt[1, 2] == 5 and bt[2, 0] == 6 and (bt[3] == bt0[3]).all() and (bt[0] == bt0[0]).all()
    for r, (blk, slot) in {0: (bt[0, 1], 1), 1: (5, 0), 2: (6, 0)}.items():
        for l in range(n_layers):
            for c in (0, 1):
                assert (kv[l, blk, c, :, slot, :] == new[r, l, c]).all()
    # nothing else changed
    mask = np.ones(kv.shape, dtype=bool)
    for blk, slot in ((bt[0, 1], 1), (5, 0), (6, 0)):
        mask[:, blk, :, :, slot, :] = False
    assert (kv[mask] == kv0[mask]).all()
    # a full table row is an error, too few free blocks is ENOMEM; both change nothing
    lens2 = np.array([12], dtype=np.int32)
    assert do.append_batch(kv, st, bt[:1].copy(), lens2, new[:1]) == "EINVAL" and lens2[0] == 12
    st.alloc(st.num_free())
    lens3 = np.array([8], dtype=np.int32)
    top = st.top
    assert do.append_batch(kv, st, bt[1:2].copy(), lens3, new[:1]) == "ENOMEM"
    assert st.top == top and lens3[0] == 8


def test_decode_attention_closed_forms():
    rng = np.random.default_rng(4)
    n_layers, n_heads, bs, d, nb = 1, 2, 4, 8, 8
    kv = _pool(rng, n_layers, nb, n_heads, bs, d)
    st = fo.FreeStack(nb)
    st.free(st.alloc(nb)[rng.permutation(nb)])
    lens = np.array([9, 1, 0], dtype=np.int32)
    bt = np.full((3, 3), -1, dtype=np.int32)
    for r in range(3):
        n = fo.blocks_for(int(lens[r]), bs)
        bt[r, :n] = st.alloc(n)
    # q = 0: uniform weights, the output is the mean of the value rows
    q0 = np.zeros((3, n_layers, n_heads, d), dtype=np.float16)
    out = do.decode_attention(kv, bt, lens, q0)
    for h in range(n_heads):
        vals = fo.fetch_rows(kv, 0, bt[0], 1, h, 9)
        assert np.allclose(out[0, 0, h], vals.mean(axis=0), rtol=1e-13, atol=0)
        # one token: its value row whatever the query
        assert (out[1, 0, h] == fo.fetch_rows(kv, 0, bt[1], 1, h, 1)[0]).all()
    assert (out[2] == 0).all()
    # a huge scale picks the value row of the best-matching key (argmax)
    q = rng.standard_normal((3, n_layers, n_heads, d)).astype(np.float16)
    big = do.decode_attention(kv, bt, lens, q, scale=1e4)
    for h in range(n_heads):
        keys = fo.fetch_rows(kv, 0, bt[0], 0, h, 9)
        vals = fo.fetch_rows(kv, 0, bt[0], 1, h, 9)
        best = int(np.argmax(keys @ q[0, 0, h].astype(np.float64)))
        assert np.allclose(big[0, 0, h], vals[best], rtol=1e-9, atol=1e-12)
    # brute force with scalar loops on one head
    sc = 1.0 / np.sqrt(d)
    h = 1
    keys = fo.fetch_rows(kv, 0, bt[0], 0, h, 9)
    vals = fo.fetch_rows(kv, 0, bt[0], 1, h, 9)
    z = [sum(float(keys[t, c]) * float(q[0, 0, h, c]) for c in range(d)) * sc for t in range(9)]
    w = [np.exp(v - max(z)) for v in z]
    ref = [sum(w[t] * float(vals[t, c]) for t in range(9)) / sum(w) for c in range(d)]
    assert np.allclose(do.decode_attention(kv, bt, lens, q)[0, 0, h], ref, rtol=1e-12, atol=1e-15)
    # permuting the tokens of a request (rows of K and V together) does not change the output
    L = 9
    perm = rng.permutation(L)
    kv2 = kv.copy()
    for c in (0, 1):
        for hh in range(n_heads):
            rows = fo.fetch_rows(kv, 0, bt[0], c, hh, L)[perm]
            for t in range(L):
                kv2[0, bt[0, t // bs], c, hh, t % bs] = rows[t]
    assert np.allclose(do.decode_attention(kv2, bt, lens, q)[0], do.decode_attention(kv, bt, lens, q)[0],
                       rtol=1e-12, atol=1e-14)


def test_attention_over_kept_lists_equals_attention_after_compaction():
    """Pruning without compaction must attend to exactly what the compacted
    cache holds: compress a batch with the pruning oracle, then compare the
    attention over its kept lists on the ORIGINAL pool with the plain attention
    on the compacted pool; and with every token kept it is the plain attention."""
    rng = np.random.default_rng(6)
    n_layers, n_heads, bs, d, nb = 2, 2, 4, 8, 40
    kv = _pool(rng, n_layers, nb, n_heads, bs, d)
    st = fo.FreeStack(nb)
    lens0 = np.array([21, 9, 14], dtype=np.int32)
    bt = np.full((3, 6), -1, dtype=np.int32)
    for r in range(3):
        n = fo.blocks_for(int(lens0[r]), bs)
        bt[r, :n] = st.alloc(n)
    kv0, bt0 = kv.copy(), bt.copy()
    method = np.array([fo.METHOD_SNAPKV, fo.METHOD_KNORM, fo.METHOD_STREAMING])
    budget = np.array([9, 4, 6])
    qw = rng.standard_normal((3, n_layers, n_heads, 4, d)).astype(np.float16)
    lens = lens0.copy()
    status, _, kept = fo.compress_batch(kv, st, bt, lens, qw, 4, method, budget, 3)
    assert status is None
    q = rng.standard_normal((3, n_layers, n_heads, d)).astype(np.float16)
    a = do.decode_attention_kept(kv0, bt0, lens0, kept, q)
    b = do.decode_attention(kv, bt, lens, q)
    assert np.allclose(a, b, rtol=1e-13, atol=1e-15)
    everything = [np.tile(np.arange(L), (n_layers, n_heads, 1)) for L in lens0]
    assert np.allclose(do.decode_attention_kept(kv0, bt0, lens0, everything, q),
                       do.decode_attention(kv0, bt0, lens0, q), rtol=1e-13, atol=1e-15)
