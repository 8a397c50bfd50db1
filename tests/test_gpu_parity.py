"""GPU parity tests: HIP library (through the C ABI) vs the CPU oracle on the
same seeded inputs.  Run with `-m gpu` on an MI355X."""

import numpy as np
import pytest

from oracle import fastcache_oracle as fo
from paper_2503_08461_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(params=[0, 1], ids=["auto_fused", "two_pass"])
def score_mode(request):
    """Both schedulings of the hot path must meet the same bar (FC_SCORE_AUTO =
    0: fused score/select/gather kernel; FC_SCORE_TWO_PASS = 1: separate
    kernels)."""
    return request.param


def _sbs(wl, **kw):
    from parity_util import SideBySide
    return SideBySide(wl, **kw)


def _run(wl, score_mode=None, **kw):
    s = _sbs(wl, score_mode=score_mode)
    try:
        stats = s.compress_and_compare(**kw)
    finally:
        s.close()
    print(wl.name, stats, flush=True)
    assert stats["max_rel_err"] < 2e-3
    return stats


def test_config1_tiny_snapkv(score_mode):
    stats = _run(synth.make_workload(1), score_mode)
    assert stats["units"] == 4


def test_config2_shape_reduced_heads(score_mode):
    # LLaVA-1.5-7B per-head shape, 640 tokens = 40 full blocks, window 32
    _run(synth.make_workload(2, n_layers=2, n_heads=3), score_mode)


def test_config3_mixed_methods_permuted_tables(score_mode):
    # ragged lengths in [600, 1200], SnapKV and key-norm in one batch
    _run(synth.make_workload(3, n_layers=1, n_heads=2, n_req=6), score_mode)


def test_config4_window64_long(score_mode):
    # several thousand tokens per head, window 64
    _run(synth.make_workload(4, n_layers=1, n_heads=2, n_req=3), score_mode)


def test_config5_lengths_reduced(score_mode):
    """Pool at 90% occupancy: the batch is trimmed to what fits (new blocks are
    taken before old ones come back), the rest rides along as METHOD_NONE and
    is compressed by the following calls."""
    from paper_2503_08461_amd import fastcache as fc
    wl = synth.make_workload(5, n_layers=1, n_heads=2, n_req=6, max_len=5000)
    s = _sbs(wl, score_mode=score_mode)
    try:
        todo = list(range(wl.n_req))
        calls = 0
        while todo:
            free = fc.fc_pool_num_free(s.pool)
            methods = np.zeros(wl.n_req, dtype=np.int32)
            picked = []
            for r in todo:
                need = synth.blocks_for(int(wl.budgets[r]))
                if need <= free:
                    free -= need
                    methods[r] = wl.methods[r]
                    picked.append(r)
            assert picked, "nothing fits"
            stats = s.compress_and_compare(methods=methods)
            print("config5 sub-batch", picked, stats, flush=True)
            todo = [r for r in todo if r not in picked]
            calls += 1
        assert calls >= 2
    finally:
        s.close()


def _custom(L, B, method, W=16, d=64, n_heads=2, n_layers=1, seed=11, n_blocks=None):
    lens = np.array(L, dtype=np.int32)
    nb = n_blocks or int(sum(synth.blocks_for(int(x)) for x in lens) * 2 + 8)
    return synth.Workload("custom", n_layers, n_heads, d, nb, W, 7, lens,
                          np.array(method, dtype=np.int32), np.array(B, dtype=np.int32),
                          seed, False, True)


@pytest.mark.parametrize("W", [1, 5, 16, 17, 33, 48, 64])
def test_window_sizes(W, score_mode):
    _run(_custom([200, 131], [max(W, 40), max(W, 70)], [fo.METHOD_SNAPKV] * 2, W=W, d=128), score_mode)


@pytest.mark.parametrize("pool_kernel", [1, 3, 15])
def test_pool_kernels(pool_kernel, score_mode):
    _run(_custom([150], [60], [fo.METHOD_SNAPKV]), score_mode, pool_kernel=pool_kernel)


def test_degenerate_budgets(score_mode):
    # B == L (identity), B == W (window only), L == W == B, single token
    wl = _custom([97, 80, 16, 1, 33], [97, 16, 16, 1, 33],
                 [fo.METHOD_KNORM, fo.METHOD_SNAPKV, fo.METHOD_SNAPKV, fo.METHOD_KNORM,
                  fo.METHOD_SNAPKV])
    _run(wl, score_mode)


def test_none_requests_pass_through(score_mode):
    wl = _custom([100, 64, 50], [30, 1, 20], [fo.METHOD_SNAPKV, fo.METHOD_NONE, fo.METHOD_KNORM])
    _run(wl, score_mode)


def test_custom_scale(score_mode):
    _run(_custom([300], [100], [fo.METHOD_SNAPKV], d=128), score_mode, scale=0.05)


def test_all_ties_go_to_lower_index(score_mode):
    """All-zero queries: every prefix token has the same score, so the kept
    prefix must be the lowest indices (no tolerance band can hide this: the
    self-consistency check compares against the GPU's own scores)."""
    import torch  # noqa: F401
    from parity_util import SideBySide
    wl = _custom([256, 77], [64, 40], [fo.METHOD_SNAPKV] * 2, W=16)
    q = np.zeros((2, 1, 2, 16, 64), dtype=np.float16)
    s = SideBySide(wl, q_host=q, score_mode=score_mode)
    try:
        s.compress_and_compare()
        kept_prefix0 = 64 - 16
        # request 0: prefix kept == 0..47 means the first 48 rows are unchanged
        kv = s.kv_dev.cpu().numpy()
        b0 = s.bt_host[0, 0]
        assert (kv[:, b0].view(np.uint16) == s.kv_host[:, b0].view(np.uint16)).all()
        assert kept_prefix0 == 48
    finally:
        s.close()


def test_zero_keys_knorm_ties():
    """Identical (zero) keys: -0.0 scores everywhere, lowest indices win."""
    from parity_util import SideBySide
    wl = _custom([100], [37], [fo.METHOD_KNORM])
    kv = synth.fill_pool_host(wl)
    kv[:, :, 0] = 0
    s = SideBySide(wl, kv_host=kv)
    try:
        s.compress_and_compare()
    finally:
        s.close()


def test_errors_leave_everything_untouched():
    import torch
    from paper_2503_08461_amd import fastcache as fc
    from parity_util import SideBySide
    wl = _custom([200], [100], [fo.METHOD_SNAPKV], n_blocks=16)   # 13 live, 3 free, needs 7
    s = SideBySide(wl)
    try:
        before_kv = s.kv_dev.clone()
        before_bt = s.bt_dev.clone()
        stack0, top0 = fc.fc_pool_export_state(s.pool)

        def expect(code, **kw):
            args = dict(methods=wl.methods, budgets=wl.budgets, window=wl.window, pool_kernel=7)
            args.update(kw)
            lens = s.lens_g.copy()
            q = s.q_dev
            if args["window"] != wl.window:
                q = torch.zeros((1, 1, 2, args["window"], 64), dtype=torch.float16, device=s.dev)
            with pytest.raises(fc.FastCacheError) as ei:
                fc.fc_compress_batch(s.pool, s.bt_dev, lens, q, args["window"],
                                     args["methods"], args["budgets"], args["pool_kernel"])
            assert ei.value.code == code
            torch.cuda.synchronize()
            assert (lens == s.lens_g).all()
            assert torch.equal(before_kv, s.kv_dev) and torch.equal(before_bt, s.bt_dev)
            st, top = fc.fc_pool_export_state(s.pool)
            assert top == top0 and (st == stack0).all()

        expect(fc.FC_ENOMEM)
        expect(fc.FC_EINVAL, budgets=np.array([0], np.int32))
        expect(fc.FC_EINVAL, budgets=np.array([201], np.int32))
        expect(fc.FC_EINVAL, budgets=np.array([8], np.int32))            # below the window
        expect(fc.FC_EINVAL, methods=np.array([9], np.int32))
        expect(fc.FC_EINVAL, pool_kernel=4)
        expect(fc.FC_EINVAL, window=65)
        with pytest.raises(fc.FastCacheError) as ei:
            fc.fc_pool_alloc(s.pool, 4)
        assert ei.value.code == fc.FC_ENOMEM
        with pytest.raises(fc.FastCacheError) as ei:
            fc.fc_pool_free(s.pool, torch.zeros(14, dtype=torch.int32, device=s.dev))
        assert ei.value.code == fc.FC_EINVAL
        # and a request that fits still works afterwards
        s.compress_and_compare(budgets=np.array([40], np.int32))
    finally:
        s.close()


def test_alloc_free_are_lifo_and_match_the_oracle():
    import torch
    from paper_2503_08461_amd import fastcache as fc
    kv = torch.zeros((1, 32, 2, 1, 16, 64), dtype=torch.float16, device="cuda:0")
    pool = fc.fc_pool_create(kv, 32, 1, 1, 64)
    st = fo.FreeStack(32)
    try:
        a = fc.fc_pool_alloc(pool, 5)
        assert a.cpu().tolist() == st.alloc(5).tolist() == [0, 1, 2, 3, 4]
        b = fc.fc_pool_alloc(pool, 3)
        assert b.cpu().tolist() == st.alloc(3).tolist()
        fc.fc_pool_free(pool, a)
        st.free(np.arange(5, dtype=np.int32))
        c = fc.fc_pool_alloc(pool, 7)
        assert c.cpu().tolist() == st.alloc(7).tolist()
        sg, tg = fc.fc_pool_export_state(pool)
        assert tg == st.top and (sg[:tg] == st.stack[:tg]).all()
        # rewind
        fresh = fo.FreeStack(32)
        fc.fc_pool_import_state(pool, fresh.stack.copy(), fresh.top)
        assert fc.fc_pool_num_free(pool) == 32
        assert fc.fc_pool_alloc(pool, 2).cpu().tolist() == [0, 1]
    finally:
        fc.fc_pool_destroy(pool)


def test_repeated_compression_of_the_same_requests(score_mode):
    """Compress, then compress the compressed caches again (lengths shrink,
    tables are the library's own output)."""
    from parity_util import SideBySide
    wl = _custom([500, 333], [200, 150], [fo.METHOD_SNAPKV, fo.METHOD_KNORM], d=128)
    s = SideBySide(wl, score_mode=score_mode)
    try:
        s.compress_and_compare()
        s.compress_and_compare(budgets=np.array([64, 20], np.int32))
        s.compress_and_compare(budgets=np.array([16, 20], np.int32))
    finally:
        s.close()


def test_auto_mode_is_default_and_green():
    _run(synth.make_workload(4, n_layers=1, n_heads=4, n_req=2))


def test_select_with_massive_ties_and_clustered_scores():
    """Many identical keys (more than the candidate list holds) and scores that
    differ only in their lowest mantissa bits: the threshold search must fall
    back to refining over all keys and still break ties by index."""
    from parity_util import SideBySide
    wl = _custom([6000, 4097], [2500, 1], [fo.METHOD_KNORM] * 2, d=64, n_heads=2)
    kv = synth.fill_pool_host(wl)
    rng = np.random.default_rng(5)
    # keys take only 3 distinct norms, so thousands tie at the threshold
    vals = np.array([0.5, 1.0, 2.0], dtype=np.float16)
    kv[:, :, 0] = 0
    kv[:, :, 0, :, :, 0] = vals[rng.integers(0, 3, size=kv[:, :, 0, :, :, 0].shape)]
    s = SideBySide(wl, kv_host=kv)
    try:
        st = s.compress_and_compare()
        assert st["units_kept_identical"] == st["units"]
    finally:
        s.close()
    # clustered: norms equal up to one fp16 ulp in a single channel
    kv2 = synth.fill_pool_host(wl)
    kv2[:, :, 0] = 1.0
    kv2[:, :, 0, :, :, 0] = (1.0 + rng.integers(0, 2, size=kv2[:, :, 0, :, :, 0].shape) / 1024.0
                             ).astype(np.float16)
    s = SideBySide(wl, kv_host=kv2)
    try:
        s.compress_and_compare()
    finally:
        s.close()


@pytest.mark.parametrize("seed", range(16))
def test_random_workloads(seed):
    """Seeded random batches: ragged lengths (1..3000), any window 1..64, both
    head sizes, mixed methods and pass-through requests, random budgets and
    pool kernels, all three schedulings."""
    rng = np.random.Generator(np.random.PCG64(9000 + seed))
    n_req = int(rng.integers(1, 6))
    W = int(rng.integers(1, 65))
    d = int(rng.choice([64, 128]))
    lens, methods, budgets = [], [], []
    for _ in range(n_req):
        m = int(rng.choice([fo.METHOD_SNAPKV, fo.METHOD_KNORM, fo.METHOD_NONE], p=[0.5, 0.4, 0.1]))
        lo = W if m == fo.METHOD_SNAPKV else 1
        L = int(rng.integers(lo, 3001)) if rng.random() < 0.7 else int(rng.integers(lo, lo + 40))
        b_lo = W if m == fo.METHOD_SNAPKV else 1
        B = int(rng.integers(b_lo, L + 1))
        lens.append(L); methods.append(m); budgets.append(B)
    wl = _custom(lens, budgets, methods, W=W, d=d, n_heads=int(rng.integers(1, 4)),
                 n_layers=int(rng.integers(1, 3)), seed=100 + seed)
    mode = int(rng.integers(0, 3)) % 2
    kernel = int(rng.choice([1, 3, 5, 7, 9, 15]))
    print("seed", seed, "lens", lens, "budgets", budgets, "methods", methods, "W", W, "d", d,
          "mode", mode, "pool", kernel, flush=True)
    _run(wl, mode, pool_kernel=kernel)


@pytest.mark.parametrize("n_sink", [0, 4, 9])
def test_streaming_method_mixed_with_scored_methods(n_sink, score_mode):
    """StreamingLLM-style requests (sinks + most recent, nothing scored) in one
    batch with SnapKV, key-norm and pass-through requests, including a streaming
    request longer than the fused kernel's score capacity."""
    M = fo.METHOD_STREAMING
    wl = _custom([300, 9000, 77, 640, 50, 16], [60, 700, 77, 160, 3, 1],
                 [M, M, M, fo.METHOD_SNAPKV, fo.METHOD_KNORM, M], W=16, d=128, n_heads=2)
    s = _sbs(wl, score_mode=score_mode)
    try:
        st = s.compress_and_compare(n_sink=n_sink)
        assert st["units_kept_identical"] == st["units"]
    finally:
        s.close()


def test_streaming_request_of_maximum_length_next_to_scored_ones():
    """A streaming request needs no score buffer, whatever its length; key-norm
    and streaming units share the launch of the SnapKV units."""
    M = fo.METHOD_STREAMING
    wl = _custom([32768, 500, 400, 31000], [5000, 100, 90, 31000],
                 [M, fo.METHOD_SNAPKV, fo.METHOD_KNORM, M], W=33, d=64, n_heads=1)
    s = _sbs(wl)
    try:
        st = s.compress_and_compare(n_sink=4)
        assert st["units_kept_identical"] == st["units"]
    finally:
        s.close()


def test_pool_70_percent_full_before_the_call_takes_two_half_batches():
    """Config 3's lengths and budgets (keep 50 %) in a pool that is 70 % full
    before the call: one call would need 35 % of the pool in new blocks and
    only 30 % is free, so it is refused with nothing touched; the two halves
    of the batch, one after the other, fit (the first half's old blocks are
    back when the second asks) and match the oracle."""
    from paper_2503_08461_amd import fastcache as fc
    wl = synth.precall_occupancy_variant(synth.make_workload(3, n_layers=1, n_heads=2, n_req=8), 0.70)
    s = _sbs(wl)
    try:
        free0 = fc.fc_pool_num_free(s.pool)
        assert free0 < sum(synth.blocks_for(int(b)) for b in wl.budgets)
        bt0, lens0 = s.bt_dev.clone(), s.lens_g.copy()
        with pytest.raises(fc.FastCacheError) as e:
            fc.fc_compress_batch(s.pool, s.bt_dev, s.lens_g, s.q_dev, wl.window, wl.methods,
                                 wl.budgets, wl.pool_kernel)
        assert e.value.code == fc.FC_ENOMEM
        assert (s.bt_dev == bt0).all() and (s.lens_g == lens0).all()
        assert fc.fc_pool_num_free(s.pool) == free0
        for a, b in ((0, 4), (4, 8)):
            m = np.zeros(8, dtype=np.int32)
            m[a:b] = wl.methods[a:b]
            st = s.compress_and_compare(methods=m)
            assert st["max_rel_err"] < 2e-3
        assert (s.lens_g == wl.budgets).all()
    finally:
        s.close()


def test_in_place_compaction(score_mode):
    """FC_COMPACT_IN_PLACE: same kept lists, rows moved inside the request's own
    blocks (chunked so that no row is overwritten before it is read), tail
    blocks released, nothing allocated - here with a pool that has no free
    block at all, and with heads on both sides of the fused kernel's limit."""
    M = fo.METHOD_STREAMING
    lens = [700, 9000, 333, 64, 100, 2500]
    methods = [fo.METHOD_SNAPKV, fo.METHOD_KNORM, fo.METHOD_KNORM, fo.METHOD_SNAPKV, M,
               fo.METHOD_SNAPKV]
    budgets = [350, 8999, 333, 16, 37, 500]
    nb = int(sum(synth.blocks_for(x) for x in lens))           # pool exactly full
    wl = _custom(lens, budgets, methods, W=16, d=128, n_heads=2, n_blocks=nb)
    from parity_util import SideBySide
    from paper_2503_08461_amd import fastcache as fc
    s = SideBySide(wl, score_mode=score_mode, in_place=True)
    try:
        assert fc.fc_pool_num_free(s.pool) == 0
        st = s.compress_and_compare()
        assert st["units_kept_identical"] == st["units"]
        # compress the compressed caches again, still in place
        s.compress_and_compare(budgets=np.array([100, 4000, 50, 16, 5, 16], np.int32))
    finally:
        s.close()


def test_work_is_issued_on_the_callers_stream():
    """All device work of the pool calls goes to the stream that is passed in
    (a non-default stream here): results are complete after synchronising that
    stream alone, and match a run on the default stream bit for bit."""
    import torch
    from paper_2503_08461_amd import fastcache as fc
    wl = _custom([900, 450], [300, 200], [fo.METHOD_SNAPKV, fo.METHOD_KNORM], W=32, d=128, n_heads=4)
    kv_host = synth.fill_pool_host(wl)
    q_host = synth.fill_q_window_host(wl)
    outs = []
    for use_side_stream in (False, True):
        kv = torch.from_numpy(kv_host.copy()).cuda()
        q = torch.from_numpy(q_host.copy()).cuda()
        torch.cuda.synchronize()
        stream = torch.cuda.Stream() if use_side_stream else torch.cuda.current_stream()
        pool = fc.fc_pool_create(kv, wl.n_blocks, wl.n_layers, wl.n_heads, wl.head_dim)
        try:
            with torch.cuda.stream(stream):
                bt = torch.full((2, wl.max_blocks), -1, dtype=torch.int32, device="cuda")
                for r in range(2):
                    n = synth.blocks_for(int(wl.seq_lens[r]))
                    fc.fc_pool_alloc(pool, n, bt[r, :n], stream=stream)
                lens = wl.seq_lens.copy()
                kept = torch.empty(int(wl.budgets.sum()) * 4, dtype=torch.int32, device="cuda")
                fc.fc_compress_batch(pool, bt, lens, q, 32, wl.methods, wl.budgets, 7, 0.0, None,
                                     kept, stream=stream)
            stream.synchronize()
            outs.append((kv.cpu(), bt.cpu(), kept.cpu(), fc.fc_pool_export_state(pool)))
        finally:
            fc.fc_pool_destroy(pool)
    a, b = outs
    assert torch.equal(a[1], b[1]) and torch.equal(a[2], b[2])
    assert torch.equal(a[0].view(torch.int16), b[0].view(torch.int16))
    assert a[3][1] == b[3][1] and (a[3][0][:a[3][1]] == b[3][0][:b[3][1]]).all()


def _mixed_window_batch(seed, lens, n_layers=1, n_heads=2, d=64):
    rng = np.random.default_rng(seed)
    R = len(lens)
    methods = np.array([fo.METHOD_SNAPKV if r % 4 != 3 else fo.METHOD_KNORM for r in range(R)],
                       np.int32)
    windows = np.array([[64, 16, 33, 1, 48, 17, 5, 32][r % 8] for r in range(R)], np.int32)
    pools = np.array([[7, 1, 3, 15, 5, 63, 7, 9][r % 8] for r in range(R)], np.int32)
    budgets = np.array([max(int(windows[r]), int(lens[r]) // (2 + r % 3)) for r in range(R)],
                       np.int32)
    wl = _custom(lens, budgets, methods, W=16, d=d, n_heads=n_heads, n_layers=n_layers, seed=seed)
    q_list = [rng.standard_normal((n_layers, n_heads, int(windows[r]), d)).astype(np.float16)
              if methods[r] == fo.METHOD_SNAPKV else None for r in range(R)]
    return wl, methods, budgets, windows, pools, q_list


@pytest.mark.parametrize("d", [64, 128])
def test_per_request_window_and_pool_kernel_in_one_batch(d, score_mode):
    """Requests of one batch with their own observation window (1..64, every
    number of 16-row query tiles) and pooling width, key-norm requests mixed
    in, one head longer than the fused kernel's capacity."""
    lens = [700, 130, 333, 250, 1200, 96, 64, 513, 90, 8300]
    wl, methods, budgets, windows, pools, q_list = _mixed_window_batch(77, lens, d=d)
    sbs = _sbs(wl, score_mode=score_mode)
    try:
        stats = sbs.compress_and_compare(methods, budgets, windows, pools, q_list=q_list)
    finally:
        sbs.close()
    print(stats, flush=True)
    assert stats["units"] == len(lens) * wl.n_layers * wl.n_heads
    assert stats["max_rel_err"] < 2e-3


def test_per_request_sizes_errors():
    import torch
    from paper_2503_08461_amd import fastcache as fc
    lens = [200, 300, 150]
    wl, methods, budgets, windows, pools, q_list = _mixed_window_batch(78, lens)
    sbs = _sbs(wl)
    try:
        q_flat = torch.zeros((int(windows.sum()) + 65) * wl.n_layers * wl.n_heads * wl.head_dim,
                             dtype=torch.float16, device=sbs.dev)
        top = fc.fc_pool_num_free(sbs.pool)
        bad = pools.copy()
        bad[0] = 4
        with pytest.raises(fc.FastCacheError) as e:
            fc.fc_compress_batch_var(sbs.pool, sbs.bt_dev, sbs.lens_g, q_flat, windows, methods,
                                     budgets, bad)
        assert e.value.code == fc.FC_EINVAL
        bad_w = windows.copy()
        bad_w[1] = 65
        with pytest.raises(fc.FastCacheError) as e:
            fc.fc_compress_batch_var(sbs.pool, sbs.bt_dev, sbs.lens_g, q_flat, bad_w, methods,
                                     budgets, pools)
        assert e.value.code == fc.FC_EINVAL
        assert fc.fc_pool_num_free(sbs.pool) == top and (sbs.lens_g == np.array(lens)).all()
        sbs.compare_state()
    finally:
        sbs.close()


@pytest.mark.parametrize("seed", range(8))
def test_random_batches_with_per_request_sizes(seed):
    """Seeded random batches through fc_compress_batch_var: any window 1..64 and
    any odd pooling width per SnapKV request, all four methods and pass-through
    requests mixed, fresh-block and in-place compaction, fused and separate
    scheduling."""
    rng = np.random.Generator(np.random.PCG64(7000 + seed))
    R = int(rng.integers(2, 8))
    d = int(rng.choice([64, 128]))
    n_layers, n_heads = int(rng.integers(1, 3)), int(rng.integers(1, 4))
    lens, methods, budgets, windows, pools = [], [], [], [], []
    for _ in range(R):
        m = int(rng.choice([fo.METHOD_SNAPKV, fo.METHOD_KNORM, fo.METHOD_STREAMING, fo.METHOD_NONE],
                           p=[0.55, 0.2, 0.15, 0.1]))
        W = int(rng.integers(1, 65))
        lo = W if m == fo.METHOD_SNAPKV else 1
        L = int(rng.integers(lo, 2500)) if rng.random() < 0.7 else int(rng.integers(lo, lo + 30))
        B = int(rng.integers(lo, L + 1))
        lens.append(L); methods.append(m); budgets.append(B); windows.append(W)
        pools.append(int(rng.choice([1, 3, 5, 7, 9, 15, 31, 63])))
    methods, budgets = np.array(methods, np.int32), np.array(budgets, np.int32)
    windows, pools = np.array(windows, np.int32), np.array(pools, np.int32)
    wl = _custom(lens, budgets, methods, W=16, d=d, n_heads=n_heads, n_layers=n_layers,
                 seed=300 + seed)
    q_list = [rng.standard_normal((n_layers, n_heads, int(windows[r]), d)).astype(np.float16)
              if methods[r] == fo.METHOD_SNAPKV else None for r in range(R)]
    mode, in_place = int(rng.integers(0, 2)), bool(rng.integers(0, 2))
    print("seed", seed, "lens", lens, "methods", methods.tolist(), "budgets", budgets.tolist(),
          "windows", windows.tolist(), "pools", pools.tolist(), "d", d, "mode", mode,
          "in_place", in_place, flush=True)
    from parity_util import SideBySide
    sbs = SideBySide(wl, score_mode=mode, in_place=in_place)
    try:
        stats = sbs.compress_and_compare(methods, budgets, windows, pools, q_list=q_list,
                                         n_sink=int(rng.integers(0, 6)))
    finally:
        sbs.close()
    assert stats["max_rel_err"] < 2e-3
