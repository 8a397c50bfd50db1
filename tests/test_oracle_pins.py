"""Pins for the CPU oracle: hand-worked examples, closed forms, brute force on
tiny inputs, invariants.  None of these calls the HIP path."""

import math

import numpy as np
import pytest

from conftest import read_golden
from oracle import fastcache_oracle as fo


# ---------------------------------------------------------------- hand examples

def test_snapkv_hand_example():
    g = read_golden("snapkv_hand_example.txt")
    K = np.array(g["K"], dtype=np.float64)
    Q = np.array(g["Q"], dtype=np.float64)
    colsum = fo.snapkv_scores(K, Q, scale=1.0, pool_kernel=1)
    np.testing.assert_allclose(colsum[:6], g["COLSUM"][0], atol=2e-6)
    assert np.isinf(colsum[6:]).all() and (colsum[6:] > 0).all()
    pooled = fo.snapkv_scores(K, Q, scale=1.0, pool_kernel=3)
    np.testing.assert_allclose(pooled[:6], g["POOLED"][0], atol=2e-6)
    kept = fo.select_topk(pooled, 4)
    assert kept.tolist() == [int(x) for x in g["KEPT"][0]]
    # the normalisers of the two rows, recovered from the un-pooled column sums
    # of a key that only one row scores above the floor: a_4 = e^2/Z0 + 1/Z1
    Z0, Z1 = g["Z"][0]
    assert abs(colsum[4] - (math.e ** 2 / Z0 + 1.0 / Z1)) < 2e-6


def test_knorm_hand_example():
    g = read_golden("knorm_hand_example.txt")
    K = np.array(g["K"], dtype=np.float64)
    s = fo.knorm_scores(K)
    np.testing.assert_allclose(-s, g["NORMS"][0], atol=1e-6)
    for b in (4, 3, 2):
        assert fo.select_topk(s, b).tolist() == [int(x) for x in g["KEPT%d" % b][0]]


def test_pool_hand_example():
    g = read_golden("pool_hand_example.txt")
    ints = lambda tag: [int(x) for x in g[tag][0]]
    st = fo.FreeStack(8)
    assert st.stack.tolist() == ints("FRESH") and st.top == 8
    ids = st.alloc(2)
    assert ids.tolist() == ints("ALLOC2") and st.top == 6
    # 1 layer, 1 head, 4-token blocks, head_dim 2; keys from the key-norm example
    kn = read_golden("knorm_hand_example.txt")
    kv = np.zeros((1, 8, 2, 1, 4, 2), dtype=np.float16)
    keys = np.array(kn["K"], dtype=np.float16)
    vals = np.arange(16, dtype=np.float16).reshape(8, 2) + 100
    for j in range(8):
        kv[0, ids[j // 4], 0, 0, j % 4] = keys[j]
        kv[0, ids[j // 4], 1, 0, j % 4] = vals[j]
    bt = np.full((1, 2), -1, dtype=np.int32)
    bt[0, :2] = ids
    lens = np.array([8], dtype=np.int32)
    status, scores, kept = fo.compress_batch(
        kv, st, bt, lens, None, 0, np.array([fo.METHOD_KNORM]), np.array([4]))
    assert status is None
    assert st.stack[:st.top].tolist() == ints("AFTER_COMPRESS_STACK") and st.top == 7
    assert bt[0, :1].tolist() == ints("AFTER_COMPRESS_TABLE")
    assert int(lens[0]) == ints("AFTER_COMPRESS_LEN")[0]
    assert kept[0][0, 0].tolist() == [int(x) for x in kn["KEPT4"][0]]
    for t, idx in enumerate(kept[0][0, 0]):
        assert (kv[0, 2, 0, 0, t] == keys[idx]).all()
        assert (kv[0, 2, 1, 0, t] == vals[idx]).all()
    assert st.alloc(2).tolist() == ints("NEXT_ALLOC2")


# ---------------------------------------------------------------- closed forms

@pytest.mark.parametrize("L,W,d", [(8, 2, 2), (40, 5, 8), (33, 32, 4), (7, 7, 3)])
def test_uniform_attention_closed_form(L, W, d):
    """All-zero queries: every visible key gets 1/(position+1), so every prefix
    key scores sum_i 1/(L-W+i+1) before and after pooling."""
    rng = np.random.default_rng(1)
    K = rng.standard_normal((L, d))
    Q = np.zeros((W, d))
    s = fo.snapkv_scores(K, Q, 1.0 / math.sqrt(d), 7)
    expect = sum(1.0 / (L - W + i + 1) for i in range(W))
    np.testing.assert_allclose(s[:L - W], expect, rtol=1e-13)
    assert np.isposinf(s[L - W:]).all()
    if (L, W) == (8, 2):
        assert abs(expect - 15.0 / 56.0) < 1e-15
        assert fo.select_topk(s, 4).tolist() == [0, 1, 6, 7]


def test_single_query_is_plain_softmax():
    """Window of one query at the last position: no mask bites, the score of
    the prefix (kernel 1) is the plain softmax of scale*K q over all L keys."""
    rng = np.random.default_rng(2)
    L, d = 50, 16
    K = rng.standard_normal((L, d))
    q = rng.standard_normal((1, d))
    s = fo.snapkv_scores(K, q, 0.25, 1)
    z = 0.25 * (K @ q[0])
    ref = np.exp(z - z.max())
    ref /= ref.sum()
    np.testing.assert_allclose(s[:L - 1], ref[:L - 1], rtol=1e-12)


def test_softmax_mass_conservation():
    """Column sums over ALL keys (prefix and window) add up to W because each
    row is a probability distribution; the prefix part equals W minus the mass
    that rows put on window keys.  Checked through a brute-force of the corner."""
    rng = np.random.default_rng(3)
    L, W, d = 37, 6, 8
    K = rng.standard_normal((L, d))
    Q = rng.standard_normal((W, d))
    s = fo.snapkv_scores(K, Q, 0.3, 1)
    corner = 0.0
    for i in range(W):
        pos = L - W + i
        z = [0.3 * float(Q[i] @ K[j]) for j in range(pos + 1)]
        m = max(z)
        e = [math.exp(v - m) for v in z]
        corner += sum(e[L - W:]) / sum(e)
    assert abs(s[:L - W].sum() + corner - W) < 1e-12


# ---------------------------------------------------------------- brute force

def brute_snapkv(K, Q, scale, kernel):
    """Independent statement: materialise the full W x L matrix entry by entry
    with scalar arithmetic, mask, normalise, slice, pool."""
    L, W = len(K), len(Q)
    P = [[0.0] * L for _ in range(W)]
    for i in range(W):
        pos = L - W + i
        z = []
        for j in range(L):
            if j <= pos:
                z.append(scale * sum(float(Q[i][c]) * float(K[j][c]) for c in range(len(K[j]))))
            else:
                z.append(None)
        m = max(v for v in z if v is not None)
        den = sum(math.exp(v - m) for v in z if v is not None)
        for j in range(L):
            P[i][j] = 0.0 if z[j] is None else math.exp(z[j] - m) / den
    a = [sum(P[i][j] for i in range(W)) for j in range(L - W)]
    h = kernel // 2
    pooled = [max(a[max(0, j - h):min(len(a), j + h + 1)]) for j in range(len(a))]
    return pooled


@pytest.mark.parametrize("L,W,d,kernel,seed", [
    (24, 4, 8, 7, 0), (31, 16, 4, 3, 1), (19, 3, 5, 5, 2), (16, 16, 8, 7, 3), (40, 8, 16, 1, 4)])
def test_snapkv_against_brute_force(L, W, d, kernel, seed):
    rng = np.random.default_rng(seed)
    K = rng.standard_normal((L, d)).astype(np.float16).astype(np.float64)
    Q = rng.standard_normal((W, d)).astype(np.float16).astype(np.float64)
    scale = 1.0 / math.sqrt(d)
    s = fo.snapkv_scores(K, Q, scale, kernel)
    ref = brute_snapkv(K.tolist(), Q.tolist(), scale, kernel)
    np.testing.assert_allclose(s[:L - W], ref, rtol=1e-12, atol=0)
    assert np.isposinf(s[L - W:]).all()


def brute_select(scores, budget):
    order = sorted(range(len(scores)), key=lambda j: (-scores[j], j))
    return sorted(order[:budget])


@pytest.mark.parametrize("seed", range(8))
def test_select_against_brute_force_and_invariants(seed):
    rng = np.random.default_rng(seed)
    L = int(rng.integers(5, 80))
    B = int(rng.integers(1, L + 1))
    # few distinct values => many ties
    s = rng.integers(0, 5, size=L).astype(np.float64) / 4.0
    w = int(rng.integers(0, min(B, 4) + 1))
    if w:
        s[L - w:] = np.inf
    kept = fo.select_topk(s, B)
    assert kept.tolist() == brute_select(s.tolist(), B)
    assert len(kept) == B and (np.diff(kept) > 0).all()
    assert kept.min() >= 0 and kept.max() < L
    assert set(range(L - w, L)) <= set(kept.tolist())
    dropped = np.setdiff1d(np.arange(L), kept)
    if len(dropped):
        thr = s[kept].min()
        assert thr >= s[dropped].max()
        eq_kept = [j for j in kept if s[j] == thr]
        eq_drop = [j for j in dropped if s[j] == thr]
        if eq_kept and eq_drop:
            assert max(eq_kept) < min(eq_drop)


# ---------------------------------------------------------------- invariances

def test_maxpool_properties():
    rng = np.random.default_rng(5)
    a = rng.standard_normal(50)
    assert (fo.maxpool_same(a, 1) == a).all()
    assert (fo.maxpool_same(a, 7) >= a).all()
    c = np.full(20, 3.5)
    assert (fo.maxpool_same(c, 7) == c).all()
    np.testing.assert_array_equal(fo.maxpool_same(fo.maxpool_same(a, 3), 3),
                                  fo.maxpool_same(a, 5))
    # explicit edge handling on a ramp: out[j] = a[min(n-1, j+3)]
    r = np.arange(10.0)
    np.testing.assert_array_equal(fo.maxpool_same(r, 7), np.minimum(r + 3, 9))
    # a single spike spreads over exactly kernel positions
    z = np.zeros(21); z[10] = 1
    assert fo.maxpool_same(z, 7).nonzero()[0].tolist() == list(range(7, 14))


def test_knorm_is_library_norm_and_channel_permutation_invariant():
    rng = np.random.default_rng(6)
    K = rng.standard_normal((30, 16))
    s = fo.knorm_scores(K)
    np.testing.assert_allclose(-s, np.linalg.norm(K, axis=1), rtol=1e-14)
    perm = rng.permutation(16)
    np.testing.assert_allclose(fo.knorm_scores(K[:, perm]), s, rtol=1e-13)
    assert (s <= 0).all()


def test_snapkv_invariances():
    rng = np.random.default_rng(7)
    L, W, d = 45, 8, 16
    K = rng.standard_normal((L, d))
    Q = rng.standard_normal((W, d))
    s = fo.snapkv_scores(K, Q, 0.25, 7)
    # a constant vector added to every key shifts each row's logits uniformly
    c = rng.standard_normal(d)
    np.testing.assert_allclose(fo.snapkv_scores(K + c, Q, 0.25, 7)[:L - W], s[:L - W], rtol=1e-11)
    # permuting channels of Q and K together changes nothing
    perm = rng.permutation(d)
    np.testing.assert_allclose(fo.snapkv_scores(K[:, perm], Q[:, perm], 0.25, 7)[:L - W],
                               s[:L - W], rtol=1e-12)
    # scale matters (guards a dropped scale): doubling scale == doubling Q
    np.testing.assert_allclose(fo.snapkv_scores(K, Q, 0.5, 7)[:L - W],
                               fo.snapkv_scores(K, 2 * Q, 0.25, 7)[:L - W], rtol=1e-12)
    assert not np.allclose(fo.snapkv_scores(K, Q, 0.5, 7)[:L - W], s[:L - W])


def test_causal_corner_matters_and_is_lower_triangular():
    """Changing a window key j only affects rows i with position >= j."""
    rng = np.random.default_rng(8)
    L, W, d = 20, 4, 8
    K = rng.standard_normal((L, d))
    Q = np.zeros((W, d)); Q[0] = rng.standard_normal(d)   # only row 0 is non-uniform
    s0 = fo.snapkv_scores(K, Q, 1.0, 1)
    K2 = K.copy(); K2[L - W + 1] *= 5.0                   # key at the position of row 1
    s1 = fo.snapkv_scores(K2, Q, 1.0, 1)
    # row 0 cannot see that key; rows 1..3 are uniform whatever the keys are
    np.testing.assert_allclose(s0[:L - W], s1[:L - W], rtol=1e-13)
    K3 = K.copy(); K3[L - W] *= 5.0                       # key at row 0's own position: visible
    s2 = fo.snapkv_scores(K3, Q, 1.0, 1)
    assert not np.allclose(s0[:L - W], s2[:L - W])


# ---------------------------------------------------------------- pool + compaction

def _random_pool(rng, n_layers, n_blocks, n_heads, bs, d):
    return rng.standard_normal((n_layers, n_blocks, 2, n_heads, bs, d)).astype(np.float16)


def _live_ids(bt, lens, bs):
    out = []
    for r in range(len(lens)):
        out += bt[r, :fo.blocks_for(int(lens[r]), bs)].tolist()
    return out


def test_alloc_free_round_trip_restores_stack():
    st = fo.FreeStack(16)
    before = st.export()
    ids = st.alloc(5)
    assert ids.tolist() == [0, 1, 2, 3, 4]
    st.free(ids[::-1])
    after = st.export()
    assert (before[0] == after[0]).all() and before[1] == after[1]
    with pytest.raises(MemoryError):
        st.alloc(17)


def test_compress_batch_conservation_round_trip_and_identity():
    rng = np.random.default_rng(9)
    n_layers, n_heads, bs, d, nb = 2, 3, 4, 8, 64
    kv = _random_pool(rng, n_layers, nb, n_heads, bs, d)
    st = fo.FreeStack(nb)
    lens = np.array([21, 9, 16, 30], dtype=np.int32)
    W = 4
    method = np.array([fo.METHOD_SNAPKV, fo.METHOD_KNORM, fo.METHOD_NONE, fo.METHOD_SNAPKV])
    budget = np.array([10, 9, 0, 4])        # request 1: B == L (identity), request 3: B == W
    maxb = 8
    bt = np.full((4, maxb), -1, dtype=np.int32)
    for r in range(4):
        n = fo.blocks_for(int(lens[r]), bs)
        bt[r, :n] = st.alloc(n)
    q = rng.standard_normal((4, n_layers, n_heads, W, d)).astype(np.float16)
    kv0, bt0, lens0 = kv.copy(), bt.copy(), lens.copy()
    status, scores, kept = fo.compress_batch(kv, st, bt, lens, q, W, method, budget, 3)
    assert status is None
    assert lens.tolist() == [10, 9, 16, 4]
    # conservation: free + live == all ids exactly once
    live = _live_ids(bt, lens, bs)
    allids = sorted(st.stack[:st.top].tolist() + live)
    assert allids == list(range(nb))
    assert st.top + len(live) == nb
    # untouched request
    assert (bt[2] == bt0[2]).all() and scores[2] is None
    # round trip: new rows are the old rows at kept[t]
    for r in (0, 1, 3):
        for l in range(n_layers):
            for h in range(n_heads):
                k = kept[r][l, h]
                assert len(k) == budget[r] and (np.diff(k) > 0).all()
                for t, idx in enumerate(k):
                    for c in (0, 1):
                        new = kv[l, bt[r, t // bs], c, h, t % bs]
                        old = kv0[l, bt0[r, idx // bs], c, h, idx % bs]
                        assert (new == old).all()
    # B == L: identity
    assert (kept[1] == np.arange(9)).all()
    # B == W: exactly the window
    assert (kept[3] == np.arange(26, 30)).all()
    # old blocks are untouched by the copy (they are only released)
    for r in (0, 1, 3):
        for b in bt0[r, :fo.blocks_for(int(lens0[r]), bs)]:
            assert (kv[:, b] == kv0[:, b]).all()
    # push order: old blocks of request 0, then 1, then 3, in table order
    pushed = st.stack[st.top - (6 + 3 + 8):st.top].tolist()
    assert pushed == bt0[0, :6].tolist() + bt0[1, :3].tolist() + bt0[3, :8].tolist()


def test_errors_leave_state_untouched():
    rng = np.random.default_rng(10)
    kv = _random_pool(rng, 1, 8, 1, 4, 4)
    st = fo.FreeStack(8)
    bt = np.full((1, 7), -1, dtype=np.int32)
    bt[0, :7] = st.alloc(7)
    lens = np.array([28], dtype=np.int32)
    q = rng.standard_normal((1, 1, 1, 2, 4)).astype(np.float16)
    snap = (kv.copy(), bt.copy(), lens.copy(), st.export())

    def unchanged():
        return ((kv == snap[0]).all() and (bt == snap[1]).all() and (lens == snap[2]).all()
                and (st.stack == snap[3][0]).all() and st.top == snap[3][1])

    # needs 2 new blocks, 1 free
    assert fo.compress_batch(kv, st, bt, lens, q, 2, [fo.METHOD_SNAPKV], [8], 7)[0] == "ENOMEM"
    assert unchanged()
    for bad in ([fo.METHOD_SNAPKV], [0]), ([fo.METHOD_SNAPKV], [29]), ([fo.METHOD_SNAPKV], [1]), ([7], [4]):
        assert fo.compress_batch(kv, st, bt, lens, q, 2, bad[0], bad[1], 7)[0] == "EINVAL"
        assert unchanged()
    assert fo.compress_batch(kv, st, bt, lens, q, 2, [fo.METHOD_SNAPKV], [4], 4)[0] == "EINVAL"
    assert unchanged()
    assert fo.compress_batch(kv, st, bt, lens, q, 2, [fo.METHOD_SNAPKV], [4], 7)[0] is None


# ---------------------------------------------------------------- streaming (sinks + recent)

@pytest.mark.parametrize("L,B,n_sink", [(10, 5, 2), (10, 10, 4), (10, 1, 4), (10, 4, 4), (10, 3, 0),
                                         (37, 9, 4), (16, 16, 0)])
def test_streaming_keeps_sinks_and_most_recent(L, B, n_sink):
    s = fo.streaming_scores(L, B, n_sink)
    kept = fo.select_topk(s, B).tolist()
    sinks = min(n_sink, B)
    assert kept == list(range(sinks)) + list(range(L - (B - sinks), L))
    assert np.isposinf(s[kept]).all() and (np.delete(s, kept) == 0).all()


def test_streaming_through_compress_batch_reads_no_scores():
    rng = np.random.default_rng(11)
    kv = _random_pool(rng, 1, 16, 2, 4, 4)
    kv[:, :, 0] = np.nan            # keys are never looked at
    st = fo.FreeStack(16)
    bt = np.full((1, 5), -1, dtype=np.int32)
    bt[0, :5] = st.alloc(5)
    lens = np.array([18], dtype=np.int32)
    kv0, bt0 = kv.copy(), bt.copy()
    status, scores, kept = fo.compress_batch(kv, st, bt, lens, None, 0, [fo.METHOD_STREAMING], [7],
                                             n_sink=3)
    assert status is None and int(lens[0]) == 7
    want = [0, 1, 2, 14, 15, 16, 17]
    for h in range(2):
        assert kept[0][0, h].tolist() == want
        for t, idx in enumerate(want):
            new = kv[0, bt[0, t // 4], 1, h, t % 4]
            old = kv0[0, bt0[0, idx // 4], 1, h, idx % 4]
            assert (new == old).all()


# ---------------------------------------------------------------- in-place compaction

def test_in_place_compaction_matches_fresh_blocks_logically():
    """Compacting inside the request's own blocks must leave the same logical
    K/V sequence as compacting into fresh blocks, allocate nothing, keep the
    first ceil(B/bs) table entries and release the tail in table order."""
    rng = np.random.default_rng(12)
    n_layers, n_heads, bs, d, nb = 2, 2, 4, 8, 40
    kv_a = _random_pool(rng, n_layers, nb, n_heads, bs, d)
    kv_b = kv_a.copy()
    lens0 = np.array([23, 8, 17], dtype=np.int32)
    method = np.array([fo.METHOD_SNAPKV, fo.METHOD_KNORM, fo.METHOD_STREAMING])
    budget = np.array([9, 8, 5])
    q = rng.standard_normal((3, n_layers, n_heads, 4, d)).astype(np.float16)

    def setup():
        st = fo.FreeStack(nb)
        st.free(st.alloc(nb)[rng2.permutation(nb)])      # permuted ids
        bt = np.full((3, 6), -1, dtype=np.int32)
        for r in range(3):
            n = fo.blocks_for(int(lens0[r]), bs)
            bt[r, :n] = st.alloc(n)
        return st, bt

    rng2 = np.random.default_rng(13)
    st_a, bt_a = setup()
    rng2 = np.random.default_rng(13)
    st_b, bt_b = setup()
    assert (bt_a == bt_b).all()
    bt0 = bt_a.copy()
    la, lb = lens0.copy(), lens0.copy()
    sa = fo.compress_batch(kv_a, st_a, bt_a, la, q, 4, method, budget, 3)
    free_before = st_b.top
    sb = fo.compress_batch(kv_b, st_b, bt_b, lb, q, 4, method, budget, 3, in_place=True)
    assert sa[0] is None and sb[0] is None and (la == lb).all()
    for r in range(3):
        assert all((sa[2][r] == sb[2][r]).ravel())          # same kept lists
        B = int(budget[r])
        n_new, n_old = fo.blocks_for(B, bs), fo.blocks_for(int(lens0[r]), bs)
        assert (bt_b[r, :n_new] == bt0[r, :n_new]).all() and (bt_b[r, n_new:] == -1).all()
        for l in range(n_layers):
            for h in range(n_heads):
                for c in (0, 1):
                    a = np.stack([kv_a[l, bt_a[r, t // bs], c, h, t % bs] for t in range(B)])
                    b = np.stack([kv_b[l, bt_b[r, t // bs], c, h, t % bs] for t in range(B)])
                    assert (a == b).all()
    # nothing allocated, tails released in batch order then table order
    released = sum(fo.blocks_for(int(lens0[r]), bs) - fo.blocks_for(int(budget[r]), bs)
                   for r in range(3))
    assert st_b.top == free_before + released
    want = []
    for r in range(3):
        want += bt0[r, fo.blocks_for(int(budget[r]), bs):fo.blocks_for(int(lens0[r]), bs)].tolist()
    assert st_b.stack[free_before:st_b.top].tolist() == want
    # in place never runs out of blocks
    st_c = fo.FreeStack(6)
    bt_c = st_c.alloc(6)[None, :].copy()
    kv_c = _random_pool(rng, 1, 6, 1, bs, d)
    assert fo.compress_batch(kv_c, st_c, bt_c, np.array([24], np.int32), None, 0,
                             [fo.METHOD_KNORM], [20])[0] == "ENOMEM"
    assert fo.compress_batch(kv_c, st_c, bt_c, np.array([24], np.int32), None, 0,
                             [fo.METHOD_KNORM], [20], in_place=True)[0] is None


# ---------------------------------------------------------------- per-request window / pool kernel

def test_per_request_window_and_pool_kernel_equal_separate_uniform_calls():
    """A batch whose requests have their own observation window and pooling
    width must score and keep exactly what each request gets when it is
    compressed alone with its own sizes (units are independent; only the pool
    bookkeeping couples requests, and that depends on budgets alone), and a
    window of 1 with pooling width 1 must reduce to the plain softmax of the
    last query."""
    rng = np.random.default_rng(21)
    n_layers, n_heads, bs, d, nb = 2, 2, 4, 8, 96
    kv = _random_pool(rng, n_layers, nb, n_heads, bs, d)
    lens0 = np.array([37, 18, 25, 30], dtype=np.int32)
    windows = [6, 1, 4, 9]
    pools = [5, 1, 3, 7]
    method = np.array([fo.METHOD_SNAPKV, fo.METHOD_SNAPKV, fo.METHOD_KNORM, fo.METHOD_SNAPKV])
    budget = np.array([12, 5, 7, 9])
    q = [rng.standard_normal((n_layers, n_heads, w, d)).astype(np.float16) for w in windows]
    q[2] = None

    def tables(st):
        bt = np.full((4, 10), -1, dtype=np.int32)
        for r in range(4):
            n = fo.blocks_for(int(lens0[r]), bs)
            bt[r, :n] = st.alloc(n)
        return bt

    st = fo.FreeStack(nb)
    bt = tables(st)
    kv_m, lens = kv.copy(), lens0.copy()
    status, scores, kept = fo.compress_batch(kv_m, st, bt, lens, q, windows, method, budget, pools)
    assert status is None and lens.tolist() == budget.tolist()
    for r in range(4):
        st1 = fo.FreeStack(nb)
        bt1 = tables(st1)
        only = np.where(np.arange(4) == r, method, fo.METHOD_NONE)
        q1 = np.zeros((4, n_layers, n_heads, windows[r], d), dtype=np.float16)
        if q[r] is not None:
            q1[r] = q[r]
        s1, sc1, k1 = fo.compress_batch(kv.copy(), st1, bt1, lens0.copy(), q1, windows[r], only,
                                        budget, pools[r])
        assert s1 is None
        assert (sc1[r] == scores[r]).all() and (k1[r] == kept[r]).all()
    # window 1, pooling 1: scores of the prefix are the softmax row of the last token's query
    r = 1
    L = int(lens0[r])
    st2 = fo.FreeStack(nb)
    bt2 = tables(st2)
    for l in range(n_layers):
        for h in range(n_heads):
            keys = fo.fetch_rows(kv, l, bt2[r], 0, h, L)
            z = keys @ q[r][l, h, 0].astype(np.float64) / np.sqrt(d)
            pr = np.exp(z - z.max())
            pr /= pr.sum()
            assert np.allclose(scores[r][l, h][:L - 1], pr[:L - 1], rtol=1e-12, atol=0)
            assert np.isinf(scores[r][l, h][L - 1])
    # sizes are checked per SnapKV request only
    bad = list(pools)
    bad[2] = 4                                    # key-norm request: not looked at
    st3 = fo.FreeStack(nb)
    assert fo.compress_batch(kv.copy(), st3, tables(st3), lens0.copy(), q, windows, method,
                             budget, bad)[0] is None
    bad[0] = 4                                    # SnapKV request: even width is an error
    st4 = fo.FreeStack(nb)
    bt4 = tables(st4)
    top4 = st4.top
    assert fo.compress_batch(kv.copy(), st4, bt4, lens0.copy(), q, windows, method, budget,
                             bad)[0] == "EINVAL" and st4.top == top4
    wbad = list(windows)
    wbad[3] = 10                                  # window above the budget
    assert fo.compress_batch(kv.copy(), st4, bt4, lens0.copy(), q, wbad, method, budget,
                             pools)[0] == "EINVAL" and st4.top == top4


# ---------------------------------------------------------------- row log-sum-exp handed in

def test_window_lse_hand_example_and_closed_forms():
    """The normalisers of the hand-worked example (Z in the fixture) and the
    uniform closed form: all-zero queries give lse_i = log(number of visible keys)."""
    g = read_golden("snapkv_hand_example.txt")
    K = np.array(g["K"], dtype=np.float64)
    Q = np.array(g["Q"], dtype=np.float64)
    lse = fo.window_lse(K, Q, 1.0)
    np.testing.assert_allclose(np.exp(lse), g["Z"][0], rtol=1e-7)
    np.testing.assert_allclose(lse, [math.log(math.e + math.e ** 2 + 5), math.log(math.e + 7)],
                               rtol=1e-14)
    rng = np.random.default_rng(11)
    for L, W, d in [(8, 2, 2), (40, 5, 8), (33, 32, 4), (7, 7, 3)]:
        lse0 = fo.window_lse(rng.standard_normal((L, d)), np.zeros((W, d)), 0.3)
        np.testing.assert_allclose(lse0, [math.log(L - W + i + 1) for i in range(W)], rtol=1e-14)


def test_window_lse_is_library_logsumexp_of_the_visible_logits():
    from scipy.special import logsumexp
    rng = np.random.default_rng(12)
    L, W, d, scale = 37, 6, 8, 0.41
    K, Q = rng.standard_normal((L, d)) * 3, rng.standard_normal((W, d)) * 3
    lse = fo.window_lse(K, Q, scale)
    for i in range(W):
        vis = L - W + i + 1                      # keys 0 .. position of query i
        assert abs(lse[i] - logsumexp(scale * (K[:vis] @ Q[i]))) < 1e-12


@pytest.mark.parametrize("L,W,d,kernel,seed", [(24, 4, 4, 1, 0), (50, 7, 8, 7, 1), (19, 19, 4, 3, 2),
                                               (64, 16, 16, 5, 3)])
def test_scores_given_exact_lse_equal_the_plain_definition(L, W, d, kernel, seed):
    rng = np.random.default_rng(seed)
    K, Q = rng.standard_normal((L, d)) * 2, rng.standard_normal((W, d)) * 2
    scale = 1.0 / math.sqrt(d)
    a = fo.snapkv_scores(K, Q, scale, kernel)
    b = fo.snapkv_scores_given_lse(K, Q, scale, kernel, fo.window_lse(K, Q, scale))
    np.testing.assert_allclose(b[:L - W], a[:L - W], rtol=1e-12)
    assert np.isposinf(b[L - W:]).all()


def test_scores_given_lse_scale_with_exp_of_minus_the_shift():
    """A row whose log-sum-exp is handed in too large by t contributes exp(-t)
    times its soft-max row: with one window query the whole score scales, with
    two the columns are the weighted sum of the two soft-max rows."""
    rng = np.random.default_rng(13)
    L, d = 30, 8
    K, Q = rng.standard_normal((L, d)), rng.standard_normal((2, d))
    lse1 = fo.window_lse(K, Q[1:], 0.5)
    base = fo.snapkv_scores(K, Q[1:], 0.5, 1)
    got = fo.snapkv_scores_given_lse(K, Q[1:], 0.5, 1, lse1 + 0.75)
    np.testing.assert_allclose(got[:L - 1], math.exp(-0.75) * base[:L - 1], rtol=1e-12)
    # two rows, written out densely a second way
    lse = fo.window_lse(K, Q, 0.5)
    got2 = fo.snapkv_scores_given_lse(K, Q, 0.5, 1, lse + np.array([0.2, -0.4]))
    rows = []
    for i in range(2):
        vis = L - 2 + i + 1
        z = 0.5 * (K[:vis] @ Q[i])
        p = np.exp(z - z.max())
        p /= p.sum()
        rows.append(np.concatenate([p, np.zeros(L - vis)]))
    expect = math.exp(-0.2) * rows[0] + math.exp(0.4) * rows[1]
    np.testing.assert_allclose(got2[:L - 2], expect[:L - 2], rtol=1e-12)


def test_compress_batch_with_lse_equals_without_and_lse_batch_layout():
    rng = np.random.default_rng(14)
    n_layers, n_heads, bs, d, n_blocks = 2, 2, 4, 8, 40
    kv = rng.standard_normal((n_layers, n_blocks, 2, n_heads, bs, d)).astype(np.float16)
    lens = np.array([21, 9, 14])
    methods = np.array([fo.METHOD_SNAPKV, fo.METHOD_KNORM, fo.METHOD_SNAPKV])
    budgets = np.array([8, 4, 6])
    W = 3
    q = rng.standard_normal((3, n_layers, n_heads, W, d)).astype(np.float16)

    def fresh():
        st = fo.FreeStack(n_blocks)
        bt = np.full((3, 8), -1, dtype=np.int32)
        for r in range(3):
            nb = fo.blocks_for(int(lens[r]), bs)
            bt[r, :nb] = st.alloc(nb)
        return kv.copy(), st, bt, lens.copy()

    kv_a, st_a, bt_a, lens_a = fresh()
    lse = fo.window_lse_batch(kv_a, bt_a, lens_a, q, W, methods)
    assert lse.shape == (3, n_layers, n_heads, W) and (lse[1] == 0).all()
    keys = fo.fetch_rows(kv_a, 1, bt_a[2], 0, 0, 14)
    np.testing.assert_allclose(lse[2, 1, 0],
                               fo.window_lse(keys, q[2, 1, 0].astype(np.float64), 1 / math.sqrt(d)))
    status, s_a, k_a = fo.compress_batch(kv_a, st_a, bt_a, lens_a, q, W, methods, budgets, 3)
    kv_b, st_b, bt_b, lens_b = fresh()
    status_b, s_b, k_b = fo.compress_batch(kv_b, st_b, bt_b, lens_b, q, W, methods, budgets, 3,
                                           lse_window=lse)
    assert status is None and status_b is None
    for r in range(3):
        np.testing.assert_allclose(s_b[r], s_a[r], rtol=1e-12)
        assert (k_b[r] == k_a[r]).all()
    assert (kv_a == kv_b).all() and (bt_a == bt_b).all() and st_a.top == st_b.top
