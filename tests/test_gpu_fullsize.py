"""Parity at the benchmark's full sizes, in the launch configuration bench.py
times: the whole batch goes through one fc_compress_batch; pool state is
compared bit-exactly with the oracle (it depends on counts only), structural
properties are checked on every unit, and sampled units are checked element by
element against the oracle."""

import numpy as np
import pytest

from oracle import fastcache_oracle as fo
from paper_2503_08461_amd import synth
from parity_util import mlp_error_bound


pytestmark = pytest.mark.gpu


def _require_room(wl):
    """A configuration that does not run is a failure, not a skip: these sizes
    are what the benchmark reports."""
    import torch
    total = torch.cuda.get_device_properties(0).total_memory
    need = wl.pool_bytes() + (10 << 30)
    assert need <= total, "%s needs %.0f GiB of device memory, this device has %.0f GiB" % (
        wl.name, need / 2**30, total / 2**30)


def _oracle_pool_replay(wl):
    """The oracle's pool bookkeeping for the whole workload.  A pool array with
    zero layers makes compress_batch skip all scoring and copying and run
    only its allocation / reclaim steps, which depend on counts alone."""
    st = fo.FreeStack(wl.n_blocks)
    rows = synth.build_block_tables(wl, st.alloc, st.free, lambda ids, ix: ids[ix])
    bt = np.full((wl.n_req, wl.max_blocks), -1, dtype=np.int32)
    for r in range(wl.n_req):
        bt[r, :rows[r].shape[0]] = rows[r]
    bt0 = bt.copy()
    lens = wl.seq_lens.copy()
    skeleton = np.zeros((0, wl.n_blocks, 2, wl.n_heads, wl.block_size, wl.head_dim), np.float16)
    status, _, _ = fo.compress_batch(skeleton, st, bt, lens, None, wl.window, wl.methods,
                                     wl.budgets, wl.pool_kernel)
    assert status is None
    return st, bt0, bt, lens


@pytest.mark.parametrize("config,n_samples,lse,slab,want_scores", [
    (2, 48, False, True, True), (3, 40, False, True, True), (4, 24, False, True, True),
    (3, 16, True, False, True), (4, 16, True, False, True),
    (3, 24, False, False, False), (4, 24, False, True, False)])
def test_fullsize_batch(config, n_samples, lse, slab, want_scores):
    """lse: the window rows' log-sum-exp is produced by fc_window_lse and the
    batch goes through fc_compress_batch_lse (what bench.py's configN_lse
    workloads time); the result must still match the plain definition.
    slab: besides the sampled units, every (request, head) of one whole layer
    (seeded choice) is compared with the oracle element by element.
    want_scores False: the call does not ask for the scores, exactly as
    bench.py's timed call (long heads then take the pruned second pass of
    the score); kept lists and compacted bytes are held to the oracle's scores."""
    import torch
    from paper_2503_08461_amd import fastcache as fc
    from paper_2503_08461_amd.device_setup import DeviceWorkload
    from parity_util import check_unit_on_device
    wl = synth.make_workload(config)
    _require_room(wl)
    print("full-size", wl.name, "pool GiB %.1f" % (wl.pool_bytes() / 2**30), flush=True)
    dw = DeviceWorkload(wl)
    try:
        n_lh = wl.n_layers * wl.n_heads
        n_scores = int(wl.seq_lens.astype(np.int64).sum()) * n_lh
        n_kept = int(wl.budgets.astype(np.int64).sum()) * n_lh
        scores = torch.empty(n_scores, dtype=torch.float32, device=dw.dev) if want_scores else None
        kept = torch.empty(n_kept, dtype=torch.int32, device=dw.dev)
        if lse:
            dw.compute_lse()
        dw.compress(scores, kept)
        torch.cuda.synchronize()
        print("compressed", flush=True)

        # pool state: bit-exact with the oracle's bookkeeping
        st, bt0_o, bt_o, lens_o = _oracle_pool_replay(wl)
        assert (dw.bt0.cpu().numpy() == bt0_o).all()
        stack_g, top_g = fc.fc_pool_export_state(dw.pool)
        assert top_g == st.top and (stack_g[:top_g] == st.stack[:top_g]).all()
        assert (dw.lens == lens_o).all()
        bt_g = dw.bt.cpu().numpy()
        for r in range(wl.n_req):
            n = fo.blocks_for(int(lens_o[r]), wl.block_size)
            assert (bt_g[r, :n] == bt_o[r, :n]).all()

        # structure of every unit's kept list, checked on the device
        so = ko = 0
        offs = []
        for r in range(wl.n_req):
            L, B = int(wl.seq_lens[r]), int(wl.budgets[r])
            k = kept[ko:ko + n_lh * B].view(n_lh, B)
            assert bool((k[:, 1:] > k[:, :-1]).all()), "kept not ascending (request %d)" % r
            assert int(k.min()) >= 0 and int(k.max()) < L
            if wl.methods[r] == fo.METHOD_SNAPKV:
                W = wl.window
                want = torch.arange(L - W, L, device=dw.dev, dtype=torch.int32)
                assert bool((k[:, B - W:] == want).all()), "window not kept (request %d)" % r
                if want_scores:
                    s = scores[so:so + n_lh * L].view(n_lh, L)
                    assert bool(torch.isposinf(s[:, L - W:]).all())
                    assert bool(torch.isfinite(s[:, :L - W]).all())
            offs.append((so, ko))
            so += n_lh * L
            ko += n_lh * B

        # sampled units against the oracle, longest and shortest requests included
        rng = np.random.Generator(np.random.PCG64(100 + config))
        reqs = [int(np.argmax(wl.seq_lens)), int(np.argmin(wl.seq_lens))]
        worst, same_cnt = 0.0, 0
        for i in range(n_samples):
            r = reqs[i] if i < len(reqs) else int(rng.integers(wl.n_req))
            l, h = int(rng.integers(wl.n_layers)), int(rng.integers(wl.n_heads))
            L, B = int(wl.seq_lens[r]), int(wl.budgets[r])
            lh = l * wl.n_heads + h
            so, ko = offs[r]
            sg = scores[so + lh * L: so + (lh + 1) * L].cpu().numpy() if want_scores else None
            kg = kept[ko + lh * B: ko + (lh + 1) * B].cpu().numpy()
            q = dw.q[r, l, h].cpu().numpy() if wl.methods[r] == fo.METHOD_SNAPKV else None
            n_old, n_new = fo.blocks_for(L, 16), fo.blocks_for(B, 16)
            err, same = check_unit_on_device(
                dw.kv, q, bt0_o[r, :n_old], bt_o[r, :n_new], l, h, L, B, int(wl.methods[r]),
                wl.window, wl.pool_kernel, sg, kg, "(%s req %d layer %d head %d)" % (wl.name, r, l, h))
            worst = max(worst, err)
            same_cnt += int(same)
            if lse and q is not None:
                ids = torch.from_numpy(bt0_o[r, :n_old].astype(np.int64)).to(dw.dev)
                keys = dw.kv[l, ids, 0, h].cpu().numpy().reshape(-1, wl.head_dim)[:L]
                want = fo.window_lse(keys.astype(np.float64), q.astype(np.float64),
                                     1.0 / np.sqrt(wl.head_dim))
                got = dw.lse[r, l, h].cpu().numpy()
                assert np.abs(got - want).max() <= 2e-3, "log-sum-exp (req %d)" % r
        print("sampled units: %d, kept identical: %d, max rel score err %.2e" % (
            n_samples, same_cnt, worst), flush=True)
        assert worst < 2e-3

        # one whole layer slab, every request and head of it, element by element
        if slab:
            l = int(rng.integers(wl.n_layers))
            worst, same_cnt, units = 0.0, 0, 0
            for r in range(wl.n_req):
                L, B = int(wl.seq_lens[r]), int(wl.budgets[r])
                so, ko = offs[r]
                n_old, n_new = fo.blocks_for(L, 16), fo.blocks_for(B, 16)
                # the request's part of the layer in one transfer each
                sg_l = scores[so + l * wl.n_heads * L:
                              so + (l + 1) * wl.n_heads * L].cpu().numpy() if want_scores else None
                kg_l = kept[ko + l * wl.n_heads * B: ko + (l + 1) * wl.n_heads * B].cpu().numpy()
                q_l = dw.q[r, l].cpu().numpy() if wl.methods[r] == fo.METHOD_SNAPKV else None
                for h in range(wl.n_heads):
                    err, same = check_unit_on_device(
                        dw.kv, None if q_l is None else q_l[h], bt0_o[r, :n_old], bt_o[r, :n_new],
                        l, h, L, B, int(wl.methods[r]), wl.window, wl.pool_kernel,
                        None if sg_l is None else sg_l[h * L:(h + 1) * L], kg_l[h * B:(h + 1) * B],
                        "(%s req %d layer %d head %d)" % (wl.name, r, l, h))
                    worst = max(worst, err)
                    same_cnt += int(same)
                    units += 1
                if r % 8 == 7:
                    print("slab: layer %d, %d requests done" % (l, r + 1), flush=True)
            print("whole slab of layer %d: %d units, kept identical: %d, max rel score err %.2e" % (
                l, units, same_cnt, worst), flush=True)
            assert units == wl.n_req * wl.n_heads and worst < 2e-3
    finally:
        dw.close()


@pytest.mark.parametrize("MLP_ACTIVATION", ["gelu_erf", "gelu_tanh"])
def test_fullsize_chunk_mlp_config4(MLP_ACTIVATION):
    """The chunk-MLP compressor on the config-4 batch exactly as bench.py runs
    it (k = 5, hidden 256, image span = all but the first and last 64 tokens):
    pool state bit-exact with the oracle's bookkeeping, sampled (request, layer,
    head, K|V) units row by row against the oracle."""
    import torch
    from oracle import mlp_compressor_oracle as mo
    from paper_2503_08461_amd import fastcache as fc
    from paper_2503_08461_amd.device_setup import DeviceWorkload
    wl = synth.make_workload(4)
    _require_room(wl)
    k, hidden, d = 5, 256, wl.head_dim
    dw = DeviceWorkload(wl)
    try:
        gen = torch.Generator(device=dw.dev)
        gen.manual_seed(wl.seed + 5000)
        w1 = [(torch.randn((hidden, k * d), generator=gen, device=dw.dev) / (k * d) ** 0.5).half()
              for _ in range(2)]
        w2 = [(torch.randn((d, hidden), generator=gen, device=dw.dev) / hidden ** 0.5).half()
              for _ in range(2)]
        b1 = [0.1 * torch.randn(hidden, generator=gen, device=dw.dev) for _ in range(2)]
        b2 = [0.1 * torch.randn(d, generator=gen, device=dw.dev) for _ in range(2)]
        fc.fc_mlp_set_weights(dw.pool, k, w1, b1, w2, b2,
                              {"gelu_erf": fc.FC_ACT_GELU_ERF,
                               "gelu_tanh": fc.FC_ACT_GELU_TANH}[MLP_ACTIVATION])
        img_b = np.full(wl.n_req, 64, dtype=np.int32)
        img_e = (wl.seq_lens - 64).astype(np.int32)
        fc.fc_compress_batch_mlp(dw.pool, dw.bt, dw.lens, img_b, img_e)
        torch.cuda.synchronize()

        # pool state against the oracle's bookkeeping (zero-layer pool: no arithmetic)
        st = fo.FreeStack(wl.n_blocks)
        rows = synth.build_block_tables(wl, st.alloc, st.free, lambda ids, ix: ids[ix])
        bt = np.full((wl.n_req, wl.max_blocks), -1, dtype=np.int32)
        for r in range(wl.n_req):
            bt[r, :rows[r].shape[0]] = rows[r]
        bt0 = bt.copy()
        lens = wl.seq_lens.copy()
        skeleton = np.zeros((0, wl.n_blocks, 2, wl.n_heads, wl.block_size, d), np.float16)
        weights = {"w1": [t.cpu().numpy() for t in w1], "b1": [t.cpu().numpy() for t in b1],
                   "w2": [t.cpu().numpy() for t in w2], "b2": [t.cpu().numpy() for t in b2]}
        assert mo.compress_batch_mlp(skeleton, st, bt, lens, img_b, img_e,
                                     np.ones(wl.n_req, np.int32), weights, k,
                                     MLP_ACTIVATION) is None
        stack_g, top_g = fc.fc_pool_export_state(dw.pool)
        assert top_g == st.top and (stack_g[:top_g] == st.stack[:top_g]).all()
        assert (dw.lens == lens).all()
        bt_g = dw.bt.cpu().numpy()
        for r in range(wl.n_req):
            n = fo.blocks_for(int(lens[r]), 16)
            assert (bt_g[r, :n] == bt[r, :n]).all() and (bt_g[r, n:] == -1).all()

        rng = np.random.Generator(np.random.PCG64(404))
        reqs = [int(np.argmax(wl.seq_lens)), int(np.argmin(wl.seq_lens))]
        worst = 0.0
        for i in range(10):
            r = reqs[i] if i < len(reqs) else int(rng.integers(wl.n_req))
            l, h, c = int(rng.integers(wl.n_layers)), int(rng.integers(wl.n_heads)), i % 2
            L = int(wl.seq_lens[r])
            old = torch.from_numpy(bt0[r, :fo.blocks_for(L, 16)].astype(np.int64)).to(dw.dev)
            src = dw.kv[l, old, c, h].cpu().numpy().reshape(-1, d)[:L].astype(np.float64)
            plan = mo.chunk_plan(L, int(img_b[r]), int(img_e[r]), k)
            hid = []
            want = mo.compress_rows(src, plan, weights, k, MLP_ACTIVATION, hid)
            hid = np.array(hid)
            new = torch.from_numpy(bt[r, :fo.blocks_for(len(plan), 16)].astype(np.int64)).to(dw.dev)
            got = dw.kv[l, new, c, h].cpu().numpy().reshape(-1, d)[:len(plan)].astype(np.float64)
            modality = np.array([m for (_, _, m) in plan])
            bound = np.empty_like(want)
            for m in (0, 1):
                sel = modality == m
                if sel.any():
                    bound[sel] = mlp_error_bound(want[sel], hid[sel], weights["w2"][m])
            ratio = np.abs(got - want) / bound
            assert (ratio <= 1.0).all(), (r, l, h, c, float(ratio.max()))
            worst = max(worst, float(ratio.max()))
        print("chunk-MLP full size: worst error %.3f x the derived bound over 10 sampled units"
              % worst, flush=True)
    finally:
        dw.close()


def test_fullsize_decode_attention_config4_after_compression():
    """The decode step's attention over the compressed config-4 batch, as
    bench.py runs it: sampled (request, layer, head) units against the oracle."""
    import torch
    from oracle import decode_oracle as do
    from paper_2503_08461_amd import fastcache as fc
    from paper_2503_08461_amd.device_setup import DeviceWorkload
    wl = synth.make_workload(4)
    _require_room(wl)
    dw = DeviceWorkload(wl)
    try:
        d = wl.head_dim
        dw.compress()
        gen = torch.Generator(device=dw.dev)
        gen.manual_seed(wl.seed + 6000)
        q = torch.randn((wl.n_req, wl.n_layers, wl.n_heads, d), generator=gen, device=dw.dev).half()
        out = fc.fc_decode_attention(dw.pool, dw.bt, dw.lens, q)
        torch.cuda.synchronize()
        bt_g = dw.bt.cpu().numpy()
        rng = np.random.Generator(np.random.PCG64(405))
        for i in range(24):
            r, l, h = int(rng.integers(wl.n_req)), int(rng.integers(wl.n_layers)), \
                int(rng.integers(wl.n_heads))
            L = int(dw.lens[r])
            n = fo.blocks_for(L, 16)
            ids = torch.from_numpy(bt_g[r, :n].astype(np.int64)).to(dw.dev)
            mini = np.zeros((1, n, 2, 1, 16, d), dtype=np.float16)
            mini[0, :, :, 0] = dw.kv[l, ids, :, h].cpu().numpy()
            want = do.decode_attention(mini, np.arange(n)[None, :], np.array([L]),
                                       q[r, l, h].cpu().numpy()[None, None, None, :])[0, 0, 0]
            got = out[r, l, h].cpu().numpy().astype(np.float64)
            err = np.abs(got - want)
            assert (err <= 1e-3 * np.abs(want) + 1e-4).all(), (r, l, h, float(err.max()))
    finally:
        dw.close()
